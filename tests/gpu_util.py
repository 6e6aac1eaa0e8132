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


def assert_state_close(gp, gm, gv, op, om, ov, *, p_ulp=16, mv_ulp=8, tag=""):
    """The benchmark spec bar |d| <= 1e-6|p| + 1e-7 for p, m, v plus the tighter ulp bars."""
    for name, g, o in (("p", gp, op), ("m", gm, om), ("v", gv, ov)):
        assert g.shape == o.shape
        bad = np.abs(g.astype(np.float64) - o.astype(np.float64)) > 1e-6 * np.abs(o.astype(np.float64)) + 1e-7
        assert not bad.any(), f"{tag} {name}: {bad.sum()} elements outside 1e-6|x|+1e-7"
        same_nan = np.isnan(g) == np.isnan(o)
        assert same_nan.all(), f"{tag} {name}: NaN pattern differs"
    fin = np.isfinite(op)
    assert ulp_diff(gp[fin], op[fin]).max(initial=0) <= p_ulp, f"{tag} p ulp {ulp_diff(gp[fin], op[fin]).max()}"
    # m crosses zero (cancellation): ulp bar where |m| is not tiny, absolute bar below
    dm = ulp_diff(gm[fin], om[fin])
    big = np.abs(om[fin]) > 1e-7
    assert dm[big].max(initial=0) <= mv_ulp, f"{tag} m ulp {dm[big].max(initial=0)}"
    assert np.abs(gm[fin][~big] - om[fin][~big]).max(initial=0) <= 1e-13, f"{tag} small m"
    dv = ulp_diff(gv[fin], ov[fin])
    assert dv.max(initial=0) <= mv_ulp, f"{tag} v ulp {dv.max(initial=0)}"


def sync():
    torch.cuda.synchronize()
