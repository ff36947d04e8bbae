"""Helpers for the GPU parity tests: the HIP path on one side, the CPU oracle on the other,
fed the same seeded fp16 bits.  Nothing computed by the HIP path is ever given to the oracle."""
from __future__ import annotations

import numpy as np
import torch

import oracle
import paper_2604_16957_amd as tq
import tq_workloads as wl

MAX_ABS = 2e-3      # attention output: max |gpu - oracle|
REL_L2 = 1e-3       # attention output: |gpu - oracle|_2 / |oracle|_2
# Outputs of magnitude above 1 (sharp softmaxes reproduce single value vectors): the fp16 output's own rounding is
# up to 2^-11 of the value, which the absolute bar cannot absorb beyond |value| = 4; the per-element bar there is
# MAX_ABS + 2^-11 |oracle value| (no slack beyond that representability term), the relative-L2 bar is unchanged.
FP16_HALF_ULP = 2.0 ** -11


def np16(t: torch.Tensor) -> np.ndarray:
    return t.detach().cpu().contiguous().numpy()


def gpu_cache_from(k: torch.Tensor, v: torch.Tensor, capacity=None, pos=0, fill=0xEE, group=32):
    """Quantise fp16 CPU tensors k, v [B,Hkv,S,d] into a fresh device cache with the HIP kernel."""
    B, Hkv, S, d = k.shape
    cache = tq.KVCache(B, Hkv, d, capacity or (pos + S), group_size=group)
    for t in cache.tensors():
        t.view(torch.uint8).fill_(fill)
    tq.tq_quantize_kv(cache, k.cuda(), v.cuda(), pos)
    return cache


def oracle_cache_from(k: torch.Tensor, v: torch.Tensor, group=32):
    kc, ks, kz = oracle.quantize(np16(k), group=group)
    vc, vs, vz = oracle.quantize(np16(v), group=group)
    return kc, ks, kz, vc, vs, vz


def assert_cache_bit_exact(cache, ocache, S, pos=0):
    names = ("k_codes", "k_scale", "k_zero", "v_codes", "v_scale", "v_zero")
    for name, g, o in zip(names, cache.tensors(), ocache):
        g = np16(g)[:, :, pos:pos + S]
        if g.dtype == np.float16:
            g, o = g.view(np.uint16), o.view(np.uint16)
        bad = int((g != o).sum())
        assert bad == 0, f"{name}: {bad} of {g.size} entries differ from the oracle"


def errors(out_gpu: torch.Tensor, ref: np.ndarray):
    got = np16(out_gpu).astype(np.float64)
    assert np.isfinite(got).all(), "non-finite output"
    diff = got - ref
    return float(np.abs(diff).max()), float(np.linalg.norm(diff) / np.linalg.norm(ref))


def assert_close(out_gpu, ref, what=""):
    max_abs, rel = errors(out_gpu, ref)
    assert max_abs <= MAX_ABS and rel <= REL_L2, f"{what}: max-abs {max_abs:.3e}, rel-L2 {rel:.3e}"
    return max_abs, rel


def assert_close_elementwise(out_gpu, ref, what=""):
    """Every element within MAX_ABS + 2^-11 |ref| (the fp16 output's own rounding), and the relative-L2 bar."""
    got = np16(out_gpu).astype(np.float64)
    assert np.isfinite(got).all(), f"{what}: non-finite output"
    diff = np.abs(got - ref)
    over = diff - (MAX_ABS + FP16_HALF_ULP * np.abs(ref))
    rel = float(np.linalg.norm(got - ref) / np.linalg.norm(ref))
    assert over.max() <= 0.0 and rel <= REL_L2, \
        f"{what}: {int((over > 0).sum())} elements over the bar (worst by {over.max():.2e}, max-abs {diff.max():.2e}), rel-L2 {rel:.3e}"
    return float(diff.max()), rel


def oracle_attend_dense_fp16(q: torch.Tensor, ocache, seq_len: int, alpha: float) -> np.ndarray:
    """What the unfused comparator computes by definition: attention (fp64) over K^ and V^ rounded to dense fp16."""
    kd = oracle.dequantize_f16(*[a[:, :, :seq_len] for a in ocache[:3]]).astype(np.float64)
    vd = oracle.dequantize_f16(*[a[:, :, :seq_len] for a in ocache[3:]]).astype(np.float64)
    return oracle.attend_dense(np16(q), kd, vd, alpha)


def assert_comparator_close(out_gpu, q, ocache, seq_len, alpha, what=""):
    """The unfused comparator materialises K^ and V^ as dense fp16 (Sec. 3.1's baseline): that rounding is part of
    what it computes, and it moves the result away from attention over the exact dequantised cache by more than
    the kernels' own error (up to 1.0e-3 relative-L2 on the shapes with outlier key channels, by the oracle's own
    evaluation of both definitions).  It is therefore held, at the same bars as the fused path, to ITS definition:
    the oracle's attention over the oracle's fp16-rounded dense tensors."""
    return assert_close(out_gpu, oracle_attend_dense_fp16(q, ocache, seq_len, alpha), what)


def oracle_attend(q: torch.Tensor, ocache, seq_len: int, alpha: float) -> np.ndarray:
    return oracle.attend_packed(np16(q), *ocache, seq_len=seq_len, alpha=alpha)


def make(w: wl.Workload):
    q, k, v = wl.make_inputs(w, device="cpu")
    return q, k, v
