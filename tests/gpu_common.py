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
# The unfused comparator stores K^ and V^ as dense fp16: every element carries an extra relative
# rounding error of up to 2^-11 (rms ~2.8e-4 of its magnitude).  Through q.k^ over d=128 elements
# (outlier channels of magnitude ~8 included) that is ~5e-4 rms on a score, hence ~5e-4 relative on
# each softmax weight, plus ~3e-4 from V^ itself: about 1e-3 relative L2 on the output.  Its bar is
# therefore wider than the fused path's, which never rounds a dequantised value to fp16.
BASELINE_REL_L2 = 3e-3


def np16(t: torch.Tensor) -> np.ndarray:
    return t.detach().cpu().contiguous().numpy()


def gpu_cache_from(k: torch.Tensor, v: torch.Tensor, capacity=None, pos=0, fill=0xEE):
    """Quantise fp16 CPU tensors k, v [B,Hkv,S,d] into a fresh device cache with the HIP kernel."""
    B, Hkv, S, d = k.shape
    cache = tq.KVCache(B, Hkv, d, capacity or (pos + S))
    for t in cache.tensors():
        t.view(torch.uint8).fill_(fill)
    tq.tq_quantize_kv(cache, k.cuda(), v.cuda(), pos)
    return cache


def oracle_cache_from(k: torch.Tensor, v: torch.Tensor):
    kc, ks, kz = oracle.quantize(np16(k))
    vc, vs, vz = oracle.quantize(np16(v))
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


def assert_close(out_gpu, ref, what="", rel_l2=REL_L2):
    max_abs, rel = errors(out_gpu, ref)
    assert max_abs <= MAX_ABS and rel <= rel_l2, f"{what}: max-abs {max_abs:.3e}, rel-L2 {rel:.3e}"
    return max_abs, rel


def oracle_attend(q: torch.Tensor, ocache, seq_len: int, alpha: float) -> np.ndarray:
    return oracle.attend_packed(np16(q), *ocache, seq_len=seq_len, alpha=alpha)


def make(w: wl.Workload):
    q, k, v = wl.make_inputs(w, device="cpu")
    return q, k, v
