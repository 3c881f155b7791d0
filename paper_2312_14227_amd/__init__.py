"""MI355X-native elastic selective training step (ElasticTrainer's hot path).

`binding` mirrors the C ABI of include/et.h one to one (argument marshalling only);
`session.Session` owns the device buffers (torch tensors) a context borrows.
The HIP library must have been built (python -m paper_2312_14227_amd.build); importing
`binding` fails loudly if it is missing.  There is no CPU fallback.
"""
