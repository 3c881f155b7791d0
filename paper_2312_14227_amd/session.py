"""Device-side owner of the buffers a context borrows: weights, optimizer state, gradients and
the workspace live in torch tensors on cuda:0; everything is computed by the library."""
import numpy as np
import torch

from . import binding as et


def desc_from_config(cfg, batch=None):
    B = cfg.batch if batch is None else batch
    if cfg.kind == "mlp":
        return et.make_desc(et.ET_MLP, et.ET_F32, B, dims=cfg.dims)
    if cfg.kind == "resnet":
        return et.make_desc(et.ET_RESNET, et.ET_BF16, B, classes=cfg.classes, image=cfg.image, in_ch=cfg.in_ch,
                            stem=cfg.stem, stage_blocks=cfg.blocks, planes=cfg.planes)
    if cfg.kind == "mobilenet":
        return et.make_desc(et.ET_MOBILENET, et.ET_BF16, B, classes=cfg.classes, image=cfg.image, in_ch=cfg.in_ch,
                            stem=cfg.stem, stage_blocks=[n for (_, _, n, _) in cfg.settings],
                            planes=[c for (_, c, _, _) in cfg.settings], expand=[t for (t, _, _, _) in cfg.settings],
                            strides=[s for (_, _, _, s) in cfg.settings], last=cfg.last)
    if cfg.kind == "vgg":
        return et.make_desc(et.ET_VGG, et.ET_BF16, B, dims=tuple(cfg.fc) + (cfg.classes,), classes=cfg.classes,
                            image=cfg.image, in_ch=cfg.in_ch, stage_blocks=cfg.convs, planes=cfg.widths)
    return et.make_desc(et.ET_VIT, et.ET_BF16, B, tokens=cfg.tokens, patch_dim=cfg.patch_dim, width=cfg.width,
                        heads=cfg.heads, mlp=cfg.mlp, blocks=cfg.blocks, classes=cfg.classes, ln_eps=cfg.ln_eps)


def make_opt(kind, lr=1e-4, beta1=0.9, beta2=0.999, eps=1e-8, momentum=0.9, wd=5e-4, step=1):
    o = et.et_opt()
    o.kind = et.ET_ADAM if kind == "adam" else et.ET_SGDW
    o.lr, o.beta1, o.beta2, o.eps, o.momentum, o.wd, o.step = lr, beta1, beta2, eps, momentum, wd, step
    return o


class Session:
    """One model on one GPU.  `weights` are float32 numpy arrays in chain order (already
    representable in the model's storage type)."""

    def __init__(self, cfg, weights, batch=None, device="cuda:0", with_state=True):
        if not torch.cuda.is_available():
            raise RuntimeError("no GPU: the HIP path has no CPU fallback")
        self.cfg, self.dev = cfg, torch.device(device)
        self.stream = torch.cuda.current_stream(self.dev)
        self.ctx = et.et_create(desc_from_config(cfg, batch), self.stream.cuda_stream)
        self.n = et.et_num_tensors(self.ctx)
        assert self.n == len(weights)
        self.wdtype = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
        self.w, self.grad, self.state = [], [], []
        k = et.et_state_slots(self.ctx)
        for i, w in enumerate(weights):
            numel, _, _ = et.et_tensor_info(self.ctx, i)
            assert numel == w.size
            t = torch.from_numpy(np.ascontiguousarray(w, dtype=np.float32)).to(self.dev)
            self.w.append(t.to(self.wdtype).contiguous())
            self.grad.append(torch.full((numel,), float("nan"), dtype=torch.float32, device=self.dev))
            if with_state:
                slots = []
                for s in range(k):
                    if cfg.dtype == "bf16" and s == 0:
                        slots.append(t.reshape(-1).clone())        # fp32 master weights
                    else:
                        slots.append(torch.zeros(numel, dtype=torch.float32, device=self.dev))
                self.state.append(slots)
        self.ws_bytes = et.et_workspace_bytes(self.ctx)
        self.ws = torch.empty(self.ws_bytes + 256, dtype=torch.uint8, device=self.dev)
        off = (-self.ws.data_ptr()) % 256
        self.ws_ptr = self.ws.data_ptr() + off
        st = [s.data_ptr() for slots in self.state for s in slots] if with_state else None
        et.et_bind(self.ctx, [w.data_ptr() for w in self.w], st, [g.data_ptr() for g in self.grad], self.ws_ptr,
                   self.ws_bytes)

    def close(self):
        if self.ctx is not None:
            torch.cuda.synchronize(self.dev)
            et.et_destroy(self.ctx)
            self.ctx = None

    def put_input(self, x, y):
        xt = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(self.dev).to(self.wdtype).contiguous()
        yt = torch.from_numpy(np.ascontiguousarray(y, dtype=np.int32)).to(self.dev)
        return xt, yt

    def put_snapshot(self, snapshot):
        return [torch.from_numpy(np.ascontiguousarray(s, dtype=np.float32)).to(self.dev).to(self.wdtype).contiguous()
                for s in snapshot]

    def train_step(self, xt, yt, mask, opt=None, want_loss=True):
        return et.et_train_step(self.ctx, xt.data_ptr(), yt.data_ptr(), mask, opt, want_loss)

    def importance(self, xt, yt, snap):
        """snap: list of device tensors in the model's storage type (e.g. clones of self.w)."""
        return et.et_importance(self.ctx, xt.data_ptr(), yt.data_ptr(), [s.data_ptr() for s in snap])

    def importance_master(self, xt, yt, snap_f32):
        """snap_f32: list of float32 device tensors (earlier copies of the master weights)."""
        return et.et_importance_master(self.ctx, xt.data_ptr(), yt.data_ptr(), [s.data_ptr() for s in snap_f32])

    def tensor_metric(self, xt, yt, metric):
        """metric: et.ET_METRIC_WEIGHT_L1 (xt, yt may be None) or et.ET_METRIC_GRAD_L1."""
        return et.et_tensor_metric(self.ctx, xt.data_ptr() if xt is not None else None,
                                   yt.data_ptr() if yt is not None else None, metric, self.n)

    def profile(self, xt, yt, warmup=2, reps=5):
        return et.et_profile(self.ctx, xt.data_ptr(), yt.data_ptr(), warmup, reps)

    def activation(self, name, shape):
        """View (no copy) of a bf16 activation the last forward pass stored in the workspace."""
        ptr, numel = et.et_debug_activation(self.ctx, name)
        assert numel == int(np.prod(shape)), (name, numel, shape)
        if ptr >= self.ws_ptr and ptr + 2 * numel <= self.ws_ptr + self.ws_bytes:
            off = ptr - self.ws.data_ptr()
            return self.ws[off:off + 2 * numel].view(torch.bfloat16).view(*shape)
        return None     # the network input itself: not in the workspace

    def launch_counts(self):
        return et.et_last_launch_counts(self.ctx)

    def grads_host(self, i):
        return self.grad[i].cpu().numpy().astype(np.float64)

    def weights_host(self, i):
        return self.w[i].float().cpu().numpy().astype(np.float64)
