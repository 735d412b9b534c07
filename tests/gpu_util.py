"""Helpers shared by the GPU parity tests: move seeded inputs to the GPU, call the C ABI
through the Python binding, and compare with the float64 oracle at the stated tolerances."""
import numpy as np

from paper_2604_12798_amd import workloads as wl

# parity bars (bf16 path vs float64 oracle)
O_MAX_ABS = 2e-2
O_MEAN_ABS = 2e-3
LSE_ABS = 1e-3
MASK_GUARD_NATS = 1e-3   # tiles whose oracle margin is closer to the threshold than this are not compared


def to_gpu(bits: np.ndarray):
    import torch
    return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)


def gpu_inputs(t: dict):
    return to_gpu(t["Q"]), to_gpu(t["K"]), to_gpu(t["V"])


def host_f32(t: dict):
    return tuple(wl.bf16_bits_to_f32(t[k]) for k in "QKV")


def gather_blocks(x, blocks, block_m, N):
    """x: torch tensor [B,H,N,...] on GPU -> numpy float64 [nblk, block_m, ...], NaN-padded rows."""
    import torch
    xs = x.float().cpu().numpy().astype(np.float64)
    out = np.full((len(blocks), block_m) + xs.shape[3:], np.nan)
    for n, (b, h, i) in enumerate(blocks):
        r0, r1 = i * block_m, min(N, (i + 1) * block_m)
        out[n, : r1 - r0] = xs[b, h, r0:r1]
    return out


def check_o_lse(O_gpu, L_gpu, ref_O, ref_L, blocks, block_m, N, what=""):
    got_O = gather_blocks(O_gpu, blocks, block_m, N)
    got_L = gather_blocks(L_gpu, blocks, block_m, N)
    valid = ~np.isnan(ref_L)
    assert not np.isnan(got_O[valid]).any(), what + ": NaN in O"
    err = np.abs(got_O[valid] - ref_O[valid])
    fin = np.isfinite(ref_L) & valid
    lerr = np.abs(got_L[fin] - ref_L[fin]).max() if fin.any() else 0.0
    assert np.array_equal(np.isneginf(got_L[valid]), np.isneginf(ref_L[valid])), what + ": -inf LSE pattern"
    stats = dict(max_abs=float(err.max()), mean_abs=float(err.mean()), lse=float(lerr))
    assert stats["max_abs"] <= O_MAX_ABS and stats["mean_abs"] <= O_MEAN_ABS and stats["lse"] <= LSE_ABS, (what, stats)
    return stats
