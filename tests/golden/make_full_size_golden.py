"""Writes tests/golden/<config>_seed<seed>.npz: the oracle's results at the full size of a
benchmark workload, sampled so that the file stays small.  Calls only the oracle and the seeded
generators.  Usage:  python tests/golden/make_full_size_golden.py vit_b [seed] [batch]

Stored per tensor k: element indices idx_k (512 drawn uniformly with a fixed seed, plus the 512
elements of largest magnitude, where the mass of the tensor's norm lies), the oracle gradient at
those elements g_k (all tensors selected; by the invariant of selective training these are also the values for
any mask that selects k), the gradient's L2 norm, and Eq. 2's importance with its magnitude sum
for the workload's snapshot.  Also the loss and the logits.  For the convolutional workloads, whose reference
rounds stored tensors to bf16, also per tensor the distance between two bf16-storage evaluations that differ by
summation-order noise (spread), and for the ResNet the same samples of the exact float64 gradient (gx_k).
"""
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import importance as oimp  # noqa: E402
from synth import CONFIGS, make_workload  # noqa: E402

SAMPLES = 512


def sample_indices(k, g, seed):
    numel = g.size
    rng = np.random.default_rng([seed, 900 + k])
    if numel <= 2 * SAMPLES:
        return np.arange(numel, dtype=np.int64)
    uniform = rng.choice(numel, size=SAMPLES, replace=False)
    largest = np.argpartition(np.abs(g.ravel()), numel - SAMPLES)[numel - SAMPLES:]
    return np.unique(np.concatenate([uniform, largest])).astype(np.int64)


def noisy_store(seed):
    """bf16 storage rounding of values that carry relative noise of 3e-7 (what a float32 sum in another order differs
    by from the float64 one): a second, equally correct bf16 evaluation."""
    from oracle import resnet
    rng = np.random.default_rng([seed, 777])
    return lambda a: resnet.round_bf16(a * (1.0 + 3e-7 * rng.standard_normal(a.shape)))


def spread_of(ga, gb):
    return np.array([np.linalg.norm((a - b).ravel()) / max(np.linalg.norm(a.ravel()), 1e-300) for a, b in zip(ga, gb)])


def vgg_in_chunks(cfg, wl, chunk, store=None):
    """The oracle's float64 column matrices of a whole VGG16 batch do not fit this machine's memory.
    No operation of the network mixes samples, so the gradient of the batch-mean loss is the mean of the
    chunks' gradients; the batch size enters only through the factor 1/B of the logit gradient, and a
    ratio of batch sizes that is a power of two commutes with the bf16 storage rounding.  The identity
    is pinned at a small size in tests/test_oracle_vgg.py."""
    from oracle import resnet, vgg
    B = wl.x.shape[0]
    assert B % chunk == 0 and ((B // chunk) & (B // chunk - 1)) == 0
    parts = [vgg.vgg_step(cfg, wl.weights, wl.x[i:i + chunk], wl.y[i:i + chunk], [1] * len(wl.weights),
                          store=store or resnet.round_bf16)
             for i in range(0, B, chunk)]
    n = len(parts)
    return dict(loss=sum(p["loss"] for p in parts) / n,
                grads=[sum(p["grads"][k] for p in parts) / n for k in range(len(wl.weights))],
                logits=np.concatenate([p["logits"] for p in parts], axis=0))


def main():
    name = sys.argv[1]
    seed = int(sys.argv[2]) if len(sys.argv) > 2 else 0
    cfg = CONFIGS[name]
    batch = int(sys.argv[3]) if len(sys.argv) > 3 else cfg.batch
    wl = make_workload(cfg, seed=seed, batch=batch)
    extra = {}
    if cfg.kind == "resnet":
        # a bf16 evaluation of a deep ReLU network is not a rounding of the exact gradient: the stored
        # reference rounds the tensors the bf16 data layout keeps in memory (see oracle/resnet.py)
        from oracle import resnet
        r = resnet.resnet_step(cfg, wl.weights, wl.x, wl.y, [1] * len(wl.weights), store=resnet.round_bf16)
        I = oimp.importance_from_grads(r["grads"], wl.weights, wl.snapshot)
        # How far apart are two correct bf16-storage evaluations of this network?  A second one whose stored values
        # carry relative noise of 3e-7 ahead of the rounding (what a float32 sum in another order differs by from
        # the float64 one) flips a few roundings; behind a flip everything is perturbed at the 2^-9 level, and a
        # ReLU mask bit that changes drops or passes a whole gradient element.  Per tensor the relative L2
        # distance between the two is stored as `spread`; the exact (unrounded) gradient is stored beside both.
        r2 = resnet.resnet_step(cfg, wl.weights, wl.x, wl.y, [1] * len(wl.weights), store=noisy_store(seed))
        extra["spread"] = spread_of(r["grads"], r2["grads"])
        del r2
        rx = resnet.resnet_step(cfg, wl.weights, wl.x, wl.y, [1] * len(wl.weights))
        extra["exact_grads"] = rx["grads"]
        extra["exact_loss"] = np.float64(rx["loss"])
        del rx
    elif cfg.kind == "mobilenet":
        from oracle import mobilenet, resnet
        r = mobilenet.mobilenet_step(cfg, wl.weights, wl.x, wl.y, [1] * len(wl.weights), store=resnet.round_bf16)
        I = oimp.importance_from_grads(r["grads"], wl.weights, wl.snapshot)
        r2 = mobilenet.mobilenet_step(cfg, wl.weights, wl.x, wl.y, [1] * len(wl.weights), store=noisy_store(seed))
        extra["spread"] = spread_of(r["grads"], r2["grads"])
        del r2
    elif cfg.kind == "vgg":
        r = vgg_in_chunks(cfg, wl, 8)
        I = oimp.importance_from_grads(r["grads"], wl.weights, wl.snapshot)
        r2 = vgg_in_chunks(cfg, wl, 8, store=noisy_store(seed))
        extra["spread"] = spread_of(r["grads"], r2["grads"])
        del r2
    else:
        I, r = oimp.importance(cfg, wl.weights, wl.snapshot, wl.x, wl.y)
    A = oimp.abs_importance_from_grads(r["grads"], wl.weights, wl.snapshot)
    out = dict(loss=np.float64(r["loss"]), logits=r["logits"], importance=I, abs_importance=A,
               batch=np.int64(batch), seed=np.int64(seed),
               gnorm=np.array([np.linalg.norm(g.ravel()) for g in r["grads"]]))
    for k, g in enumerate(r["grads"]):
        idx = sample_indices(k, g, seed)
        out["idx_%d" % k] = idx.astype(np.int32)
        out["g_%d" % k] = g.ravel()[idx]
        if "exact_grads" in extra:
            out["gx_%d" % k] = extra["exact_grads"][k].ravel()[idx]
    if "exact_grads" in extra:
        out["exact_gnorm"] = np.array([np.linalg.norm(g.ravel()) for g in extra["exact_grads"]])
        out["exact_loss"] = extra["exact_loss"]
    if "spread" in extra:
        out["spread"] = extra["spread"]
    tag = name if batch == cfg.batch else "%s_b%d" % (name, batch)
    path = os.path.join(ROOT, "tests", "golden", "%s_seed%d.npz" % (tag, seed))
    np.savez_compressed(path, **out)
    print("wrote", path, os.path.getsize(path), "bytes; loss", r["loss"])


if __name__ == "__main__":
    main()
