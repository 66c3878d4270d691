"""Helpers for the GPU parity tests: upload seeded tensors, run the library, compare with the oracle."""
import numpy as np
import torch

from paper_2112_10065_amd import binding as dp, synth

DEV = torch.device("cuda:0")

# spec tolerances
F32_REL = 1e-5
BF16_REL, BF16_ABS = 2e-2, 5e-2


def bf16_dev(bits):
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to(DEV).view(torch.bfloat16)


def to_np(t):
    return t.float().cpu().numpy() if t.dtype == torch.bfloat16 else t.cpu().numpy()


def errs(got, ref):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    rel = np.linalg.norm(got - ref) / max(np.linalg.norm(ref), 1e-300)
    return rel, float(np.abs(got - ref).max()) if got.size else 0.0


def assert_bf16_close(got, ref, what):
    rel, mx = errs(got, ref)
    assert rel <= BF16_REL and mx <= BF16_ABS, f"{what}: rel_l2={rel:.3e} max_abs={mx:.3e}"


def assert_f32_close(got, ref, what):
    rel, mx = errs(got, ref)
    assert rel <= F32_REL, f"{what}: rel_l2={rel:.3e} max_abs={mx:.3e}"


def workspace(nbytes):
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=DEV)


class ConvCase:
    """Seeded tensors of one conv layer on host (fp32 values, bf16-exact if bf16) and on the device."""

    def __init__(self, tag, n, h, w, c, k, r, s, stride=(1, 1), pad=(0, 0), bf16=True, dist="he_normal",
                 bias=True, relu=True, dx_f32=False):
        self.shape = (n, h, w, c, k, r, s)
        self.stride, self.pad, self.bf16 = stride, pad, bf16
        self.ho = (h + 2 * pad[0] - r) // stride[0] + 1
        self.wo = (w + 2 * pad[1] - s) // stride[1] + 1
        x, wt, b = synth.conv_tensors(tag, n, h, w, c, k, r, s, dist=dist, bias=bias)
        dy = synth.upstream_grad(tag, (n, self.ho, self.wo, k))
        self.b = b
        if bf16:
            xb, wb, dyb = (synth.f32_to_bf16_bits(a) for a in (x, wt, dy))
            self.x, self.w, self.dy = (synth.bf16_bits_to_f32(a) for a in (xb, wb, dyb))
            self.xd, self.wd, self.dyd = bf16_dev(xb), bf16_dev(wb), bf16_dev(dyb)
        else:
            self.x, self.w, self.dy = x, wt, dy
            self.xd, self.wd, self.dyd = (torch.from_numpy(a).to(DEV) for a in (x, wt, dy))
        self.bd = torch.from_numpy(b).to(DEV) if bias else None
        flags = (dp.DP_BIAS if bias else 0) | (dp.DP_RELU if relu else 0) | (dp.DP_DX_F32 if dx_f32 else 0)
        self.relu, self.dx_f32 = relu, dx_f32
        self.desc = dp.conv_desc(n, h, w, c, k, r, s, stride, pad, dp.DP_BF16 if bf16 else dp.DP_F32, flags)
        self.tdt = torch.bfloat16 if bf16 else torch.float32

    def ws(self):
        return workspace(max(dp.dp_conv2d_workspace_bytes(self.desc, p) for p in range(3)))

    def run_fwd(self, ws=None):
        n, h, w, c, k, r, s = self.shape
        y = torch.empty((n, self.ho, self.wo, k), dtype=self.tdt, device=DEV)
        dp.dp_conv2d_fwd(self.desc, self.xd, self.wd, self.bd, y, ws if ws is not None else self.ws())
        return y

    def run_dgrad(self, y_saved, ws=None):
        n, h, w, c, k, r, s = self.shape
        dx = torch.empty((n, h, w, c), dtype=torch.float32 if self.dx_f32 else self.tdt, device=DEV)
        dp.dp_conv2d_bwd_data(self.desc, self.dyd, y_saved, self.wd, dx, ws if ws is not None else self.ws())
        return dx

    def run_dgrad_relu_in(self, y_saved, ws=None):
        """Backward-data with the backward of the ReLU in front of the layer fused in: dx * [x > 0]."""
        n, h, w, c, k, r, s = self.shape
        d = dp.dp_conv_desc.from_buffer_copy(self.desc)
        d.flags |= dp.DP_RELU_IN
        dx = torch.full((n, h, w, c), 3.0, dtype=torch.float32 if self.dx_f32 else self.tdt, device=DEV)
        wsb = workspace(max(dp.dp_conv2d_workspace_bytes(d, p) for p in range(3))) if ws is None else ws
        dp.dp_conv2d_bwd_data_relu(d, self.dyd, y_saved, self.wd, self.xd, dx, wsb)
        return dx

    def run_wgrad(self, y_saved, want_db=True, ws=None):
        n, h, w, c, k, r, s = self.shape
        dw = torch.empty((k, r, s, c), dtype=torch.float32, device=DEV)
        db = torch.empty((k,), dtype=torch.float32, device=DEV) if want_db else None
        dp.dp_conv2d_bwd_filter(self.desc, self.xd, self.dyd, y_saved, dw, db, ws if ws is not None else self.ws())
        return dw, db
