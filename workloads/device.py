"""GPU-side harness helpers: upload seeded tensors as PyTorch device tensors and build a library
context for a workload.  Pure plumbing (no arithmetic of the method)."""
import numpy as np
import torch

from .gen import Weights


def torch_dtype(model):
    return torch.float32 if model.dtype == "fp32" else torch.bfloat16


_MATRICES = ("wq", "wk", "wv", "wo", "wgate", "wup", "wdown")


def _quantized(w, model, device, on_device=False):
    """Narrow weights: (device codes uint8, device scales, dequantised float32 host copy).  "bf16w8": e4m3 codes and
    float32 row scales; "bf16w4": MXFP4 codes (two per byte) and E8M0 block scales.
    on_device: timing runs only -- the same rule evaluated by torch on the GPU (no host copy, nothing to compare)."""
    if model.dtype == "bf16w4":
        if on_device:
            t = torch.from_numpy(np.ascontiguousarray(w)).to(device)
            n, k = t.shape
            blocks = t.view(n, k // 32, 32)
            amax = blocks.abs().amax(dim=2)
            exp = torch.where(amax > 0, torch.floor(torch.log2(amax.clamp_min(1e-38))) - 2.0, torch.zeros_like(amax)).clamp(-126, 127)
            x = (blocks / torch.exp2(exp)[:, :, None]).abs()
            mids = (0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0)
            idx = torch.zeros_like(x, dtype=torch.uint8)
            for i, mid in enumerate(mids):
                idx += ((x > mid) if i % 2 == 0 else (x >= mid)).to(torch.uint8)
            idx |= (blocks < 0).to(torch.uint8) << 3
            flat = idx.view(n, k)
            codes = (flat[:, 0::2] | (flat[:, 1::2] << 4)).contiguous()
            return codes, (exp + 127).to(torch.uint8).contiguous(), None
        from .fp4 import quantize_blocks
        codes, scale, deq = quantize_blocks(w)
        return torch.from_numpy(codes).to(device), torch.from_numpy(scale).to(device), deq
    if on_device:
        t = torch.from_numpy(np.ascontiguousarray(w)).to(device)
        scale = (t.abs().amax(dim=1) / 448.0).clamp_min(1e-30)
        codes = (t / scale[:, None]).clamp(-448.0, 448.0).to(torch.float8_e4m3fn).view(torch.uint8)
        return codes, scale.float(), None
    from .fp8 import quantize_rows
    codes, scale, deq = quantize_rows(w)
    return torch.from_numpy(codes).to(device), torch.from_numpy(scale).to(device), deq


def to_device(arr, model, device="cuda:0"):
    """float32 numpy (already on the model's storage grid) -> device tensor in the model dtype (exact)."""
    t = torch.from_numpy(np.ascontiguousarray(arr))
    return t.to(device=device, dtype=torch_dtype(model), non_blocking=False)


class UploadingWeights:
    """Wraps a Weights generator: every tensor handed out (e.g. to the oracle) is also uploaded once to the
    GPU, so a large model is generated a single time for both sides."""

    def __init__(self, model, seed, device="cuda:0", reuse_buffers=True, device_quantize=False):
        self.device_quantize = device_quantize
        self.inner = Weights(model, seed, reuse_buffers=reuse_buffers)
        self.model = model
        self.device = device
        self.dev = {"layers": [None] * model.n_layers}

    def tok_emb(self):
        a = self.inner.tok_emb()
        self.dev.setdefault("tok_emb", to_device(a, self.model, self.device))
        return a

    def norm_final(self):
        a = self.inner.norm_final()
        self.dev.setdefault("norm_final", to_device(a, self.model, self.device))
        return a

    def lm_head(self):
        a = self.inner.lm_head()
        if self.model.dtype in ("bf16w8", "bf16w4"):
            # (the oracle gets the dequantised values: what the library's codes and scales stand for)
            if "lm_head_deq" not in self.dev:
                self.dev["lm_head"], self.dev["lm_head_scale"], self.dev["lm_head_deq"] = _quantized(a, self.model, self.device, self.device_quantize)
            return self.dev["lm_head_deq"]
        self.dev.setdefault("lm_head", to_device(a, self.model, self.device))
        return a

    def layer(self, l):
        w = self.inner.layer(l)
        if self.model.dtype in ("bf16w8", "bf16w4"):
            out, dev = {}, {}
            for k, v in w.items():
                if k in _MATRICES:
                    dev[k], dev["s" + k[1:]], out[k] = _quantized(v, self.model, self.device, self.device_quantize)
                else:
                    dev[k], out[k] = to_device(v, self.model, self.device), v
            if self.dev["layers"][l] is None:
                self.dev["layers"][l] = dev
            return out
        if self.dev["layers"][l] is None:
            self.dev["layers"][l] = {k: to_device(v, self.model, self.device) for k, v in w.items()}
        return w

    def upload_all(self):
        """Generate and upload whatever has not been requested yet; returns the device weight dict."""
        if "tok_emb" not in self.dev:
            self.tok_emb()
        if "norm_final" not in self.dev:
            self.norm_final()
        if "lm_head" not in self.dev:
            self.lm_head()
        for l in range(self.model.n_layers):
            if self.dev["layers"][l] is None:
                self.layer(l)
        return self.dev


def make_context(model, dev_weights, *, max_branches, max_rows_per_branch, max_shared, max_private,
                 device="cuda:0"):
    from paper_2406_18200_amd import ModelShape, VerifyContext
    shape = ModelShape(model.n_layers, model.d_model, model.n_heads, model.head_dim, model.d_ff, model.vocab,
                       model.dtype, model.rms_eps, model.rope_theta, max_branches, max_rows_per_branch,
                       max_shared, max_private)
    return VerifyContext(shape, dev_weights, device)


def i32(a, device="cuda:0"):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to(device)


def f32(a, device="cuda:0"):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(device)
