"""Helpers shared by the GPU parity tests: host<->device marshalling, the
error metric, and conversion between the oracle's contiguous KV arrays and the
library's paged pool.  No stage arithmetic lives here."""
import math

import numpy as np
import torch

from paper_2507_21276_amd import binding as Bd
from paper_2507_21276_amd import synth_inputs as S

TOL = {"f32": 1e-4, "bf16": 2e-2}   # max-abs error relative to the oracle tensor's RMS


def dev(x: np.ndarray, dtype: torch.dtype) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to("cuda").to(dtype).contiguous()


def host(t: torch.Tensor) -> np.ndarray:
    return t.detach().to(torch.float32).cpu().numpy().astype(np.float64)


def rel_err(got: np.ndarray, ref: np.ndarray) -> float:
    rms = math.sqrt(float((ref.astype(np.float64) ** 2).mean()))
    return float(np.abs(got.astype(np.float64) - ref).max()) / max(rms, 1e-30)


def assert_close(got, ref, tol, what="", atol=0.0):
    """max|got - ref| <= tol * RMS(ref) + atol  (atol only for tensors that are exactly zero)."""
    got, ref = np.asarray(got, np.float64), np.asarray(ref, np.float64)
    rms = math.sqrt(float((ref ** 2).mean()))
    worst = float(np.abs(got - ref).max())
    assert worst <= tol * rms + atol, f"{what}: max-abs error {worst:.3e} = {worst / max(rms, 1e-30):.3e} x RMS > {tol:.1e}"
    return worst / max(rms, 1e-30)


def out_rounding_bound(ref, name):
    """Worst-case error of rounding the result itself to a 16-bit output format,
    relative to the tensor RMS: half an ulp of the largest element."""
    ref = np.asarray(ref, np.float64)
    u = {"bf16": 2.0 ** -8, "f16": 2.0 ** -11, "f32": 0.0}[name]
    return u * float(np.abs(ref).max()) / max(math.sqrt(float((ref ** 2).mean())), 1e-30)


def param_slices(cfg):
    return [(n, off, int(np.prod(shape))) for n, off, shape, _ in S.param_layout(cfg)]


def pool_from_oracle_cache(cache, table, n_pages, cfg):
    """Oracle cache[layer][b] = [K, V] ([ctx, h, dh]) -> pools [nL, n_pages, h, P, dh] (float32)."""
    nL, h, dh, P = cfg["n_layers"], cfg["n_heads"], cfg["head_dim"], cfg["page_size"]
    kp = np.zeros((nL, n_pages, h, P, dh), np.float32)
    vp = np.zeros_like(kp)
    for l in range(nL):
        for b, (K, V) in enumerate(cache[l]):
            for j in range(K.shape[0]):
                pg = table[b, j // P]
                kp[l, pg, :, j % P, :] = K[j]
                vp[l, pg, :, j % P, :] = V[j]
    return kp, vp


def gather_rows_from_pool(pool: np.ndarray, table, b, lo, hi):
    """Rows lo..hi-1 of request b from a pool [nL, n_pages, h, P, dh] -> [nL, hi-lo, h, dh]."""
    P = pool.shape[3]
    return np.stack([pool[:, table[b, j // P], :, j % P, :] for j in range(lo, hi)], axis=1)
