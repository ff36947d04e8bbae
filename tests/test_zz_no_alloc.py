"""The allocation-free entry point, tq_sdpa_int4_decode_static, against tq_sdpa_int4_decode (and the oracle):
several calls in a row on the same static scratch array, each with a smaller input than the one before, so that
every later call finds the earlier one's partial results lying in the array."""
import ctypes

import numpy as np
import pytest
import torch

import paper_2604_16957_amd as tq
import tq_workloads as wl
from paper_2604_16957_amd import binding as B

from gpu_common import MAX_ABS, REL_L2, assert_close, gpu_cache_from, make, np16, oracle_attend, oracle_cache_from

pytestmark = pytest.mark.gpu


def _case(batch, hq, hkv, d, S, seed):
    w = wl.custom(batch=batch, n_q_heads=hq, n_kv_heads=hkv, head_dim=d, seq_len=S, seed=seed, outlier_channels=4)
    q, k, v = make(w)
    return w, q, gpu_cache_from(k, v), oracle_cache_from(k, v)


def test_static_scratch_decode_matches_the_workspace_call_on_calls_in_a_row():
    torch.cuda.set_device(0)
    # 84 MB of cache (two launches: partial kernel + merge kernel), then a sequence short enough for the
    # one-launch route with its in-kernel chunk merge, then a single chunk
    shapes = [(2, 64, 8, 128, 32768, 71), (1, 64, 8, 128, 6000, 72), (1, 16, 2, 128, 700, 73)]
    launches = []
    for batch, hq, hkv, d, S, seed in shapes:
        w, q, cache, ocache = _case(batch, hq, hkv, d, S, seed)
        assert tq.tq_workspace_bytes(batch, hq, d) <= B.TQ_STATIC_SCRATCH_BYTES
        launches.append(tq.tq_decode_launches(cache, hq, S, w.attn_scale))
        qg = q.cuda()
        want = tq.tq_sdpa_int4_decode(cache, qg, S, w.attn_scale)
        got = torch.full_like(want, float("nan"))
        tq.tq_sdpa_int4_decode_static(cache, qg, S, w.attn_scale, got)
        torch.cuda.synchronize()
        diff = (got.double() - want.double()).cpu().numpy()
        ref = np16(want).astype(np.float64)
        assert np.isfinite(diff).all(), f"S={S}: non-finite output"
        assert np.abs(diff).max() <= MAX_ABS and np.linalg.norm(diff) <= REL_L2 * np.linalg.norm(ref), \
            f"S={S}: static-scratch call differs from the workspace call by {np.abs(diff).max():.3e}"
        assert_close(got, oracle_attend(q, ocache, S, w.attn_scale), f"static scratch, S={S}")
    assert launches[0] == 2 and launches[1] == 1 and launches[2] == 1


def test_static_scratch_decode_rejects_what_does_not_fit():
    torch.cuda.set_device(0)
    w, q, cache, _ = _case(1, 16, 2, 128, 64, 74)
    big = B.TqKvCacheStruct.from_buffer_copy(cache.struct)
    big.batch = 64                                   # 64 x 16 heads x 128 chunks x 130 floats: 68 MB of partials
    assert tq.tq_workspace_bytes(64, 16, 128) > B.TQ_STATIC_SCRATCH_BYTES
    out = torch.empty((64, 16, 128), dtype=torch.float16, device="cuda")
    q64 = torch.zeros((64, 16, 128), dtype=torch.float16, device="cuda")
    rc = B.raw().tq_sdpa_int4_decode_static(ctypes.byref(big), q64.data_ptr(), 16, 64, 0.1, out.data_ptr(), None, None)
    assert rc == B.TQ_ERR_WORKSPACE
    rc = B.raw().tq_sdpa_int4_decode_static(ctypes.byref(cache.struct), None, 16, 64, 0.1, out.data_ptr(), None, None)
    assert rc == B.TQ_ERR_NULL


def test_more_workspaces_than_counter_sets_take_the_merge_kernel():
    """(Kept at the very end of the GPU suite: it uses up the library's sets of arrival counters for the rest of the
    process.)  The one-launch decode route gives every workspace a set of arrival counters of its own for the life
    of the process; a workspace that finds them all taken gets the merge kernel (two launches) instead, never a set
    shared with another workspace.  300 distinct workspaces (more than there are sets), in flight 8 at a time: all
    results right."""
    torch.cuda.set_device(0)
    w, q, cache, ocache = _case(2, 24, 3, 128, 5000, 75)
    qg = q.cuda()
    assert tq.tq_decode_launches(cache, 24, 5000, w.attn_scale) == 1
    ref = oracle_attend(q, ocache, 5000, w.attn_scale)
    nbytes = tq.tq_workspace_bytes(2, 24, 128)
    ws = [torch.empty(nbytes, dtype=torch.uint8, device="cuda") for _ in range(300)]
    streams = [torch.cuda.Stream() for _ in range(8)]
    outs = [torch.zeros_like(qg) for _ in ws]
    torch.cuda.synchronize()
    for i, (wsp, o) in enumerate(zip(ws, outs)):
        with torch.cuda.stream(streams[i % len(streams)]):
            tq.tq_sdpa_int4_decode(cache, qg, 5000, w.attn_scale, out=o, workspace=wsp)
    torch.cuda.synchronize()
    for i, o in enumerate(outs):
        assert_close(o, ref, f"workspace {i}")
