"""Helpers for the GPU parity tests (torch is only the allocator here)."""
import numpy as np
import torch

DEV = "cuda:0"

HP = dict(lr=1e-4, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01)


def dev_f32(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(DEV)


def dev_u16(a: np.ndarray) -> torch.Tensor:
    """uint16 bit patterns -> device int16 tensor holding the same bits."""
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.uint16).view(np.int16)).to(DEV)


def host_f32(t: torch.Tensor) -> np.ndarray:
    return t.detach().cpu().numpy().astype(np.float32, copy=False)


def host_u16(t: torch.Tensor) -> np.ndarray:
    if t.dtype == torch.bfloat16:
        t = t.view(torch.int16)
    return t.detach().cpu().numpy().view(np.uint16)


def ulp_diff(a, b):
    def key(x):
        i = np.ascontiguousarray(x, dtype=np.float32).view(np.int32).astype(np.int64)
        return np.where(i < 0, -(i & 0x7FFFFFFF), i)
    return np.abs(key(a) - key(b))


def bf16_ulp_diff(a, b):
    def key(x):
        i = np.ascontiguousarray(x, dtype=np.uint16).astype(np.int64)
        return np.where(i & 0x8000, -(i & 0x7FFF), i)
    return np.abs(key(a) - key(b))


def assert_state_close(gp, gm, gv, op, om, ov, *, steps=10, tag="", lr=1e-4, p_ulp=None,
                       mv_ulp=None, m_floor=1e-4):
    """The benchmark spec bar |d| <= 1e-6|p| + 1e-7 for p, m, v plus tighter ulp bars derived
    from the arithmetic.

    Per step the kernel rounds sqrt(v) and the quotient m/denominator to fp32 (half an
    ulp of the lr-sized term each, at worst), rounds the scalars lr/bc1 and 1/sqrt(bc2)
    to fp32 in the fp32 mode, and rounds p once; the oracle rounds only p.  So p may
    drift by up to ~3 ulp per step, the ulp taken at max(|p|, lr) because an element
    near zero still carries the rounding of the lr-sized term.  m and v are produced
    by at most three fp32 roundings per step in the fp32 mode (one in the fp64 modes):
    steps + 2 ulp covers both; for m, which is a sum of terms of either sign, the ulp
    is taken at max(|m|, m_floor) with m_floor = (1 - beta1) * typical |g|."""
    if p_ulp is None:
        p_ulp = 3 * steps + 2
    if mv_ulp is None:
        mv_ulp = steps + 2
    for name, g, o in (("p", gp, op), ("m", gm, om), ("v", gv, ov)):
        assert g.shape == o.shape
        bad = np.abs(g.astype(np.float64) - o.astype(np.float64)) > 1e-6 * np.abs(o.astype(np.float64)) + 1e-7
        assert not bad.any(), f"{tag} {name}: {bad.sum()} elements outside 1e-6|x|+1e-7"
        same_nan = np.isnan(g) == np.isnan(o)
        assert same_nan.all(), f"{tag} {name}: NaN pattern differs"
    fin = np.isfinite(op)
    scale = np.spacing(np.maximum(np.abs(op[fin]), np.float32(lr))).astype(np.float64)
    perr = np.abs(gp[fin].astype(np.float64) - op[fin].astype(np.float64)) / scale
    assert perr.max(initial=0) <= p_ulp, f"{tag} p off by {perr.max()} ulp"
    mscale = np.spacing(np.maximum(np.abs(om[fin]), np.float32(m_floor))).astype(np.float64)
    merr = np.abs(gm[fin].astype(np.float64) - om[fin].astype(np.float64)) / mscale
    assert merr.max(initial=0) <= mv_ulp, f"{tag} m off by {merr.max(initial=0)} ulp"
    dv = ulp_diff(gv[fin], ov[fin])
    assert dv.max(initial=0) <= mv_ulp, f"{tag} v ulp {dv.max(initial=0)}"


def sync():
    torch.cuda.synchronize()
