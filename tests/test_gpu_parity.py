"""GPU parity: the HIP path (through the C ABI) against the CPU oracle on the same seeded inputs.

Bars: int4 codes, scales and zero-points bit-exact; attention output max-abs <= 2e-3 and
relative L2 <= 1e-3 against the fp64 oracle (fp32 accumulate, fp16 out)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2604_16957_amd as tq
import tq_workloads as wl
from gpu_common import (MAX_ABS, REL_L2, assert_cache_bit_exact, assert_close, assert_close_elementwise, assert_comparator_close,
                        errors, gpu_cache_from, make, np16, oracle_attend,
                        oracle_cache_from)

pytestmark = pytest.mark.gpu

VARIANTS = [1, 2]   # 1 = generic vector-ALU kernel, 2 = matrix-core kernel (skipped where unsupported)


def _decode(cache, q, S, alpha, **kw):
    try:
        out = tq.tq_sdpa_int4_decode(cache, q.cuda(), S, alpha, **kw)
    except tq.TqError as e:
        if e.status == -6 and kw.get("variant") == 2:
            pytest.skip("matrix-core kernel does not cover this shape")
        raise
    torch.cuda.synchronize()
    return out


# ---------------------------------------------------------------- quantise-append (bit-exact)

def _special_values(d=128):
    rng = np.random.default_rng(77)
    rows = []
    rows.append(np.zeros(d))                                   # constant groups
    rows.append(np.full(d, -0.0))
    rows.append(np.full(d, 65504.0))
    rows.append(np.full(d, -65504.0))
    r = np.zeros(d); r[::2] = 65504.0; r[1::2] = -65504.0; rows.append(r)      # widest range
    r = np.zeros(d); r[5] = 2.0 ** -24; rows.append(r)         # range underflows the fp16 scale
    r = rng.integers(-3, 4, d) * 2.0 ** -24; rows.append(r)    # subnormal inputs
    r = 1000.0 + rng.integers(0, 3, d) * 0.5; rows.append(r)   # large |zero-point|
    r = -2000.0 + rng.integers(0, 2, d) * 1.0; rows.append(r)  # |z| > 1024: clamping can fire
    r = rng.integers(0, 16, d) + 0.5; rows.append(r)           # ties everywhere
    r = (rng.integers(0, 16, d) + 0.5) * 0.125 - 1.0; rows.append(r)
    r = rng.standard_normal(d) * 1e-3; rows.append(r)
    r = rng.standard_normal(d) * 300; rows.append(r)
    x = np.stack(rows).astype(np.float16)
    return torch.from_numpy(x).reshape(1, 1, len(rows), d)


def test_quantize_special_values_bit_exact():
    for d in (128, 256):
        x = _special_values(d)
        k, v = x, torch.flip(x, dims=(2,)).contiguous()
        cache = gpu_cache_from(k, v)
        torch.cuda.synchronize()
        assert_cache_bit_exact(cache, oracle_cache_from(k, v), k.shape[2])


@pytest.mark.parametrize("name", ["tiny", "gemma_small", "llama_small"])
def test_quantize_random_bit_exact(name):
    w = {"tiny": wl.WORKLOADS["tiny"],
         "gemma_small": wl.custom(n_q_heads=4, n_kv_heads=2, head_dim=256, seq_len=777, qk_std=0.1, seed=21),
         "llama_small": wl.custom(batch=2, n_q_heads=16, n_kv_heads=2, head_dim=128, seq_len=1500,
                                  outlier_channels=4, seed=22)}[name]
    q, k, v = make(w)
    cache = gpu_cache_from(k, v)
    torch.cuda.synchronize()
    assert_cache_bit_exact(cache, oracle_cache_from(k, v), w.seq_len)


@pytest.mark.parametrize("mode", ["any_bits", "narrow_groups", "full_range", "subnormal", "mixed_exponents", "constant", "ties"])
def test_quantize_adversarial_values_bit_exact(mode):
    """Inputs chosen to sit on the quantiser's edges (Sec. 2.1, Eq. 2-3): arbitrary finite fp16 bit patterns, groups
    of tiny range on a large offset (zero-points in the hundreds), the full fp16 range (scales in the thousands),
    subnormals (the scale underflows to the constant-group rule), exponents mixed inside a group, constant groups with
    single outliers, ramps whose codes land on .5 (round-half-even).  Both quantisers, the append kernel and the one
    inside the merge kernel (the step's new token), against the oracle, bit for bit."""
    modes = ["any_bits", "narrow_groups", "full_range", "subnormal", "mixed_exponents", "constant", "ties"]
    rng = np.random.default_rng(2600 + modes.index(mode))
    for d in (128, 256, 512):
        B, H, S = 2, 2, 65
        n = B * H * S * d
        if mode == "any_bits":
            x = rng.integers(0, 1 << 16, n, dtype=np.uint16)
            x = np.where((x & 0x7C00) == 0x7C00, x & 0x83FF, x).astype(np.uint16).view(np.float16)     # no inf / nan
        elif mode == "narrow_groups":
            base = rng.normal(0, 1, (n // 32, 1)) * rng.choice([1, 100, 1000])
            x = (base + rng.normal(0, 1, (n // 32, 32)) * rng.choice([1e-3, 1e-2, 1])).astype(np.float16).ravel()
        elif mode == "full_range":
            x = (rng.uniform(-1, 1, n) * 65504).astype(np.float16)
        elif mode == "subnormal":
            x = (rng.uniform(-1, 1, n) * rng.choice([1e-4, 6e-5, 1e-6, 6e-8])).astype(np.float16)
        elif mode == "mixed_exponents":
            x = (rng.normal(0, 1, n) * np.exp2(rng.integers(-20, 14, n))).astype(np.float16)
        elif mode == "constant":
            x = np.repeat(rng.normal(0, 10, n // 32).astype(np.float16), 32)
            x[rng.integers(0, n, n // 200)] += np.float16(0.001)
        else:
            k2 = rng.integers(0, 31, n).astype(np.float64) * 0.5
            off = rng.integers(-8, 8, (n // 32, 1)).repeat(32, 1).ravel()
            x = ((k2 + off) * np.exp2(rng.integers(-6, 6, (n // 32, 1)).repeat(32, 1).ravel())).astype(np.float16)
        x = np.where(np.isfinite(x), x, np.float16(0)).astype(np.float16).reshape(B, H, S, d)
        kt, vt = torch.from_numpy(x.copy()), torch.from_numpy(np.ascontiguousarray(x[..., ::-1]))
        ocache = oracle_cache_from(kt, vt)
        cache = gpu_cache_from(kt, vt, capacity=S + 2)
        torch.cuda.synchronize()
        assert_cache_bit_exact(cache, ocache, S)
        step = gpu_cache_from(kt[:, :, :S - 1].contiguous(), vt[:, :, :S - 1].contiguous(), capacity=S + 2)
        tq.tq_sdpa_int4_append_decode(step, kt[:, :, S - 1:].contiguous().cuda(), vt[:, :, S - 1:].contiguous().cuda(),
                                      torch.zeros(B, H, d, dtype=torch.float16, device="cuda"), S, 1.0)
        torch.cuda.synchronize()
        assert_cache_bit_exact(step, ocache, S)


def test_append_writes_only_its_positions():
    w = wl.custom(batch=2, n_q_heads=4, n_kv_heads=2, head_dim=128, seq_len=40, seed=23)
    q, k, v = make(w)
    cap = 64
    cache = gpu_cache_from(k[:, :, :33], v[:, :, :33], capacity=cap, fill=0xEE)      # bulk: tokens 0..32
    for t in range(33, 40):                                                          # then one at a time
        tq.tq_quantize_kv(cache, k[:, :, t:t + 1].contiguous().cuda(), v[:, :, t:t + 1].contiguous().cuda(), t)
    torch.cuda.synchronize()
    assert_cache_bit_exact(cache, oracle_cache_from(k, v), 40)
    for t in cache.tensors():                                                        # the rest is untouched
        assert bool((t.view(torch.uint8)[:, :, 40:] == 0xEE).all())
    with pytest.raises(tq.TqError) as e:
        tq.tq_quantize_kv(cache, k[:, :, :30].contiguous().cuda(), v[:, :, :30].contiguous().cuda(), 40)
    assert e.value.status == -4


# ---------------------------------------------------------------- groups of 64 and 128 elements

@pytest.mark.parametrize("group", [64, 128])
def test_larger_groups_quantise_bit_exact(group):
    """Sec. 2.1 states the scheme for groups of g consecutive elements: with g = 64 / 128 two / four lanes of the
    quantiser share a group (its min and max cross lanes before the scale is worked out).  Special values, edge
    distributions and random data, bulk and token by token, bit for bit against the oracle at the same group size."""
    rng = np.random.default_rng(6400 + group)
    for d in (128, 256, 512):
        x = _special_values(d)
        k, v = x, torch.flip(x, dims=(2,)).contiguous()
        assert_cache_bit_exact(gpu_cache_from(k, v, group=group), oracle_cache_from(k, v, group=group), k.shape[2])
        B, H, S = 2, 3, 67
        n = B * H * S * d
        bits = rng.integers(0, 1 << 16, n, dtype=np.uint16)
        any_bits = np.where((bits & 0x7C00) == 0x7C00, bits & 0x83FF, bits).astype(np.uint16).view(np.float16)
        narrow = (rng.normal(0, 1, (n // group, 1)) * 100 + rng.normal(0, 1, (n // group, group)) * 1e-2).astype(np.float16).ravel()
        ties = ((rng.integers(0, 31, n) * 0.5 + rng.integers(-8, 8, (n // group, 1)).repeat(group, 1).ravel())
                * np.exp2(rng.integers(-6, 6, (n // group, 1)).repeat(group, 1).ravel())).astype(np.float16)
        mixed = (rng.normal(0, 1, n) * np.exp2(rng.integers(-20, 14, n))).astype(np.float16)
        for xs in (any_bits, narrow, ties, mixed):
            xs = np.where(np.isfinite(xs), xs, np.float16(0)).astype(np.float16).reshape(B, H, S, d)
            kt, vt = torch.from_numpy(xs.copy()), torch.from_numpy(np.ascontiguousarray(xs[..., ::-1]))
            ocache = oracle_cache_from(kt, vt, group=group)
            cache = gpu_cache_from(kt, vt, capacity=S + 3, group=group)
            torch.cuda.synchronize()
            assert_cache_bit_exact(cache, ocache, S)
            for t in cache.tensors():
                assert bool((t.view(torch.uint8)[:, :, S:] == 0xEE).all())
            # the step's token through the one-call entry point (append kernel, then the decode)
            step = gpu_cache_from(kt[:, :, :S - 1].contiguous(), vt[:, :, :S - 1].contiguous(), capacity=S + 3, group=group)
            tq.tq_sdpa_int4_append_decode(step, kt[:, :, S - 1:].contiguous().cuda(), vt[:, :, S - 1:].contiguous().cuda(),
                                          torch.zeros(B, 2 * H, d, dtype=torch.float16, device="cuda"), S, 1.0)
            torch.cuda.synchronize()
            assert_cache_bit_exact(step, ocache, S)


@pytest.mark.parametrize("group", [64, 128])
@pytest.mark.parametrize("shape", ["g8_d128_b2_kv3", "g2_d256", "g4_d512"])
def test_larger_groups_decode_matches_oracle(shape, group):
    """Fused decode attention over a cache quantised in groups of 64 / 128 (the matrix-core kernel at d = 128, where
    with groups of 128 the capacity has to be even; the generic vector-ALU kernel elsewhere and as variant 1):
    lengths around tile boundaries, chunk counts, per-sequence lengths, a sliding window, the one-call step, and
    the unfused comparator, each against the oracle at the same group size."""
    shapes = dict(SHAPES, g4_d512=dict(n_q_heads=8, n_kv_heads=2, head_dim=512, v_std=0.5))
    for S in (1, 33, 1000, 4133):
        w = wl.custom(seq_len=S, seed=640 + group + S, **shapes[shape])
        q, k, v = make(w)
        cache = gpu_cache_from(k, v, capacity=S + 7, group=group)
        ocache = oracle_cache_from(k, v, group=group)
        assert_cache_bit_exact(cache, ocache, S)
        ref = oracle_attend(q, ocache, S, w.attn_scale)
        for n_splits in (0, 1, 3, 128):
            out = tq.tq_sdpa_int4_decode(cache, q.cuda(), S, w.attn_scale, n_splits=n_splits)
            torch.cuda.synchronize()
            assert_close(out, ref, f"{shape} g={group} S={S} n_splits={n_splits}")
        assert_close(tq.tq_sdpa_int4_decode(cache, q.cuda(), S, w.attn_scale, variant=1), ref, f"{shape} g={group} variant 1")
        if w.head_dim == 128 and (group == 64 or (S + 7) % 2 == 0):   # the matrix-core kernel takes these (variant 0 too)
            for n_splits in (0, 1, 3):
                out = tq.tq_sdpa_int4_decode(cache, q.cuda(), S, w.attn_scale, variant=2, n_splits=n_splits)
                assert_close(out, ref, f"{shape} g={group} variant 2 n_splits={n_splits}")
        else:                                       # ... and no others: d = 256 / 512, pairs of tokens that straddle rows
            with pytest.raises(tq.TqError) as e:
                tq.tq_sdpa_int4_decode(cache, q.cuda(), S, w.attn_scale, variant=2)
            assert e.value.status == -6
        lens = [max(1, S - 19 * b) for b in range(w.batch)]
        out = tq.tq_sdpa_int4_decode_varlen(cache, q.cuda(), torch.tensor(lens, dtype=torch.int32).cuda(), S, w.attn_scale)
        torch.cuda.synchronize()
        assert_close(out, _oracle_varlen(q, ocache, lens, w.attn_scale), f"{shape} g={group} per-sequence lengths S={S}")
        win = max(1, S // 3)
        out = tq.tq_sdpa_int4_decode(cache, q.cuda(), S, w.attn_scale, window=win)
        torch.cuda.synchronize()
        assert_close(out, _oracle_window(q, ocache, [S] * w.batch, win, w.attn_scale), f"{shape} g={group} window S={S}")
        base = tq.tq_dequant_then_attend(cache, q.cuda(), S, w.attn_scale)
        torch.cuda.synchronize()
        assert_comparator_close(base, q, ocache, S, w.attn_scale, f"{shape} g={group} comparator S={S}")
        if S > 1:                                   # one decode step in one call
            step = gpu_cache_from(k[:, :, :S - 1].contiguous(), v[:, :, :S - 1].contiguous(), capacity=S + 7, group=group)
            out = tq.tq_sdpa_int4_append_decode(step, k[:, :, S - 1:].contiguous().cuda(), v[:, :, S - 1:].contiguous().cuda(),
                                                q.cuda(), S, w.attn_scale)
            torch.cuda.synchronize()
            assert_cache_bit_exact(step, ocache, S)
            assert_close(out, ref, f"{shape} g={group} step S={S}")


@pytest.mark.parametrize("group", [64, 128])
@pytest.mark.parametrize("shape", ["g3_d128", "g8_d128_b2_kv3", "g16_d128", "g24_d128"])
def test_larger_groups_on_the_matrix_cores(shape, group):
    """Groups of 64 / 128 at d = 128 through the matrix-core kernel: the 8-row tile (3 and 8 heads per KV head), the
    16-row tile (16 heads) and two of them per KV head (24 heads); lengths around the 32-token supertile and, at 128,
    around the token pairs that share a metadata dword (odd and even lengths, odd per-sequence lengths); forced chunk
    counts, a sharp softmax, several query tokens, a sliding window (groups of 64: the matrix-core kernel; of 128:
    the generic one), the one-call step."""
    shapes = dict(SHAPES, g24_d128=dict(n_q_heads=24, n_kv_heads=1, head_dim=128))
    for S, n_splits, scale in ((2, 0, None), (31, 0, None), (32, 0, None), (33, 0, None), (34, 0, None), (700, 3, None),
                               (4133, 0, None), (6000, 0, 1.0), (20001, 0, None)):
        kw = dict(attn_scale=scale, v_std=0.5) if scale else {}
        w = wl.custom(seq_len=S, seed=6400 + group + S, **dict(shapes[shape], **kw))
        q, k, v = make(w)
        cap = S + 2 + (S & 1)                       # even: pairs of tokens never straddle rows
        cache = gpu_cache_from(k, v, capacity=cap, group=group)
        ocache = oracle_cache_from(k, v, group=group)
        assert tq.tq_decode_launches(cache, w.n_q_heads, S, w.attn_scale, variant=2) > 0
        ref = oracle_attend(q, ocache, S, w.attn_scale)
        for variant in (0, 2):
            out = tq.tq_sdpa_int4_decode(cache, q.cuda(), S, w.attn_scale, variant=variant, n_splits=n_splits)
            torch.cuda.synchronize()
            assert_close_elementwise(out, ref, f"{shape} g={group} S={S} variant={variant} n_splits={n_splits}")
        lens = [max(1, S - 17 * b) for b in range(w.batch)]
        out = tq.tq_sdpa_int4_decode_varlen(cache, q.cuda(), torch.tensor(lens, dtype=torch.int32).cuda(), S, w.attn_scale,
                                            variant=2)
        torch.cuda.synchronize()
        assert_close_elementwise(out, _oracle_varlen(q, ocache, lens, w.attn_scale), f"{shape} g={group} lengths S={S}")
        if S >= 3:                                  # three query tokens, causal among themselves
            q4 = _queries_for(w, 3)
            out = tq.tq_sdpa_int4_decode(cache, q4.cuda(), S, w.attn_scale, n_splits=n_splits)
            torch.cuda.synchronize()
            assert_close(out, _oracle_causal(q4, ocache, [S] * w.batch, w.attn_scale), f"{shape} g={group} 3 queries S={S}")
        win = max(1, S // 3)
        out = tq.tq_sdpa_int4_decode(cache, q.cuda(), S, w.attn_scale, window=win)
        torch.cuda.synchronize()
        assert_close(out, _oracle_window(q, ocache, [S] * w.batch, win, w.attn_scale), f"{shape} g={group} window S={S}")
        if S > 2:                                   # one decode step in one call
            step = gpu_cache_from(k[:, :, :S - 1].contiguous(), v[:, :, :S - 1].contiguous(), capacity=cap, group=group)
            out = tq.tq_sdpa_int4_append_decode(step, k[:, :, S - 1:].contiguous().cuda(), v[:, :, S - 1:].contiguous().cuda(),
                                                q.cuda(), S, w.attn_scale)
            torch.cuda.synchronize()
            assert_cache_bit_exact(step, ocache, S)
            assert_close_elementwise(out, ref, f"{shape} g={group} step S={S}")


@pytest.mark.parametrize("group", [64, 128])
def test_larger_groups_full_size(group):
    """The headline shape (64 / 8 heads, d = 128, 131072 tokens) quantised in groups of 64 / 128: cache bit-exact,
    every output element against the oracle."""
    w = wl.WORKLOADS["llama128k"]
    q, k, v = make(w)
    cache = gpu_cache_from(k, v, group=group)
    ocache = oracle_cache_from(k, v, group=group)
    del k, v
    assert_cache_bit_exact(cache, ocache, w.seq_len)
    out = tq.tq_sdpa_int4_decode(cache, q.cuda(), w.seq_len, w.attn_scale)
    torch.cuda.synchronize()
    assert_close_elementwise(out, oracle_attend(q, ocache, w.seq_len, w.attn_scale), f"llama128k g={group}")


@pytest.mark.parametrize("group", [64, 128])
def test_larger_groups_over_a_paged_pool(group):
    """Groups of 64 / 128 through the block table: fill, one step per sequence (append + attend in one call) and a
    sliding window, against the oracle at the same group size."""
    lens = [900, 77, 1300, 256]
    PT, max_blocks, n_pages = 256, 6, 30
    w = wl.custom(batch=len(lens), seq_len=max(lens), seed=660 + group, n_q_heads=8, n_kv_heads=2, head_dim=128,
                  outlier_channels=4)
    q, k, v = make(w)
    B, Hkv, d, S = w.batch, w.n_kv_heads, w.head_dim, w.seq_len
    table = np.random.default_rng(6).permutation(n_pages)[:B * max_blocks].reshape(B, max_blocks).astype(np.int32)
    table_dev = torch.from_numpy(table).cuda()
    pool = tq.KVCache(n_pages, Hkv, d, PT, group_size=group)
    for t in pool.tensors():
        t.view(torch.uint8).fill_(0xEE)
    # every sequence's tokens but its last go in by the bulk fill (positions 0), the last by the one-call step
    kz, vz = k.clone(), v.clone()
    tq.tq_quantize_kv_paged(pool, table_dev, kz.cuda(), vz.cuda(), torch.zeros(B, dtype=torch.int32, device="cuda"))
    lens_dev = torch.tensor(lens, dtype=torch.int32, device="cuda")
    kn = torch.stack([k[b, :, lens[b] - 1:lens[b]] for b in range(B)]).contiguous()
    vn = torch.stack([v[b, :, lens[b] - 1:lens[b]] for b in range(B)]).contiguous()
    for t in pool.tensors():                      # wipe each sequence's last token: the step has to write it again
        for b in range(B):
            t.view(torch.uint8)[table[b, (lens[b] - 1) // PT], :, (lens[b] - 1) % PT] = 0xEE
    ocache = oracle_cache_from(k, v, group=group)
    out = tq.tq_sdpa_int4_append_decode_paged(pool, table_dev, kn.cuda(), vn.cuda(), q.cuda(), lens_dev, S, w.attn_scale)
    torch.cuda.synchronize()
    assert_close(out, _oracle_varlen(q, ocache, lens, w.attn_scale), f"paged step g={group}")
    for b in range(B):                            # the stored bits, read back through the table
        for t, o in zip(pool.tensors(), ocache):
            g = np.concatenate([np16(t)[table[b, j]] for j in range((lens[b] + PT - 1) // PT)], axis=1)[:, :lens[b]]
            o = o[b, :, :lens[b]]
            if g.dtype == np.float16:
                g, o = g.view(np.uint16), o.view(np.uint16)
            assert np.array_equal(g, o), f"sequence {b}"
    out = tq.tq_sdpa_int4_decode_paged(pool, table_dev, q.cuda(), lens_dev, S, w.attn_scale, window=100)
    torch.cuda.synchronize()
    assert_close(out, _oracle_window(q, ocache, lens, 100, w.attn_scale), f"paged window g={group}")


# ---------------------------------------------------------------- fused decode attention

SHAPES = {
    "g8_d128": dict(n_q_heads=8, n_kv_heads=1, head_dim=128),
    "g8_d128_b2_kv3": dict(batch=2, n_q_heads=24, n_kv_heads=3, head_dim=128, outlier_channels=4),
    "g2_d256": dict(n_q_heads=4, n_kv_heads=2, head_dim=256, attn_scale=1.0, qk_std=0.1),
    "g1_d128": dict(n_q_heads=2, n_kv_heads=2, head_dim=128),
    "g4_d256": dict(n_q_heads=4, n_kv_heads=1, head_dim=256),
    "g3_d128": dict(n_q_heads=6, n_kv_heads=2, head_dim=128),
    "g16_d128": dict(n_q_heads=16, n_kv_heads=1, head_dim=128),
    # d = 512 rows have four times the elements, and a row that attends one or two tokens IS (nearly) a value vector:
    # with V ~ N(0,1) some outputs then exceed 4, where the fp16 output's own spacing (2^-8) is twice the absolute
    # tolerance.  These shapes serve the masking edge cases, so V gets half the spread.
    "g4_d512_b2_kv2": dict(batch=2, n_q_heads=8, n_kv_heads=2, head_dim=512, attn_scale=1.0, qk_std=0.1, v_std=0.5),
    "g32_d512": dict(n_q_heads=32, n_kv_heads=1, head_dim=512, attn_scale=1.0, qk_std=0.1, v_std=0.5),
    "g6_d512": dict(n_q_heads=6, n_kv_heads=1, head_dim=512, v_std=0.5),
}


@pytest.mark.parametrize("variant", VARIANTS)
@pytest.mark.parametrize("S", [1, 2, 31, 32, 33, 513, 1000, 4133])
@pytest.mark.parametrize("shape", ["g8_d128", "g2_d256", "g8_d128_b2_kv3"])
def test_decode_ragged_lengths(shape, S, variant):
    w = wl.custom(seq_len=S, seed=100 + S, **SHAPES[shape])
    q, k, v = make(w)
    cache = gpu_cache_from(k, v, capacity=S + (3 if S % 2 else 0))
    ocache = oracle_cache_from(k, v)
    assert_cache_bit_exact(cache, ocache, S)
    out = _decode(cache, q, S, w.attn_scale, variant=variant)
    assert_close(out, oracle_attend(q, ocache, S, w.attn_scale), f"{shape} S={S} variant={variant}")


@pytest.mark.parametrize("variant", VARIANTS)
@pytest.mark.parametrize("shape", ["g1_d128", "g4_d256", "g3_d128", "g16_d128"])
def test_decode_other_gqa_ratios(shape, variant):
    w = wl.custom(seq_len=2100, seed=31, **SHAPES[shape])
    q, k, v = make(w)
    cache = gpu_cache_from(k, v)
    ocache = oracle_cache_from(k, v)
    out = _decode(cache, q, w.seq_len, w.attn_scale, variant=variant)
    assert_close(out, oracle_attend(q, ocache, w.seq_len, w.attn_scale), f"{shape} variant={variant}")


@pytest.mark.parametrize("variant", VARIANTS)
def test_result_does_not_depend_on_the_chunking(variant):
    w = wl.custom(seq_len=5000, seed=41, **SHAPES["g8_d128"])
    q, k, v = make(w)
    cache = gpu_cache_from(k, v)
    ref = oracle_attend(q, oracle_cache_from(k, v), w.seq_len, w.attn_scale)
    outs = []
    for n in (0, 1, 2, 7, 64, 128, 1000):
        out = _decode(cache, q, w.seq_len, w.attn_scale, n_splits=n, variant=variant)
        assert_close(out, ref, f"n_splits={n} variant={variant}")
        outs.append(np16(out).astype(np.float64))
    spread = max(np.abs(o - outs[0]).max() for o in outs)
    assert spread <= 5e-4


@pytest.mark.parametrize("variant", VARIANTS)
def test_attends_only_to_seq_len_tokens_of_a_larger_cache(variant):
    w = wl.custom(seq_len=900, seed=42, **SHAPES["g8_d128"])
    q, k, v = make(w)
    cache = gpu_cache_from(k, v, capacity=1024)
    ocache = oracle_cache_from(k[:, :, :517], v[:, :, :517])
    out = _decode(cache, q, 517, w.attn_scale, variant=variant)
    assert_close(out, oracle_attend(q, ocache, 517, w.attn_scale), "prefix of a larger cache")


@pytest.mark.parametrize("variant", VARIANTS)
def test_known_answers(variant):
    # one token -> its dequantised value; identical keys -> mean of the values
    w = wl.custom(seq_len=64, seed=43, **SHAPES["g8_d128"])
    q, k, v = make(w)
    cache = gpu_cache_from(k, v)
    vh = oracle.dequantize(*oracle_cache_from(k, v)[3:])
    out = _decode(cache, q, 1, w.attn_scale, variant=variant)
    assert_close(out, np.broadcast_to(vh[0, 0, 0], (1, 8, vh.shape[-1])), "one token: its dequantised value vector")
    k2 = k.clone(); k2[:] = k[:, :, :1]
    cache2 = gpu_cache_from(k2, v)
    out2 = _decode(cache2, q, 64, w.attn_scale, variant=variant)
    assert_close(out2, np.broadcast_to(vh[0, 0].mean(0), (1, 8, vh.shape[-1])), "identical keys: the mean of the values")


@pytest.mark.parametrize("variant", VARIANTS)
def test_sharp_softmax_large_scores(variant):
    # large attn_scale: the softmax is close to one-hot and scores are far from zero
    w = wl.custom(seq_len=700, seed=44, attn_scale=4.0, **SHAPES["g8_d128"])
    q, k, v = make(w)
    cache = gpu_cache_from(k, v)
    out = _decode(cache, q, w.seq_len, w.attn_scale, variant=variant)
    ref = oracle_attend(q, oracle_cache_from(k, v), w.seq_len, w.attn_scale)
    assert_close_elementwise(out, ref, f"sharp softmax variant={variant}")


@pytest.mark.parametrize("B", [130, 256, 512])
def test_rows_of_their_own_length_are_paired_long_with_short(B):
    """More than a thousand (sequence, KV head) rows of their own lengths, each a single chunk taken by one wave:
    every block orders the sequences by length and gives the two waves of a SIMD the i-th shortest and the i-th
    longest.  Every block has to arrive at the SAME order (equal lengths included), or rows would be computed twice
    and others not at all: every row against the oracle, many equal lengths, and two calls bit for bit alike."""
    Hkv, S = 8, 300
    rng = np.random.default_rng(7000 + B)
    lens = rng.integers(1, S + 1, B).astype(np.int32)
    lens[: B // 4] = rng.choice([33, 64, 65, 200], B // 4)          # many ties
    lens[0] = S
    w = wl.custom(batch=B, n_q_heads=2 * Hkv, n_kv_heads=Hkv, head_dim=128, seq_len=S, seed=7100 + B)
    q, k, v = make(w)
    cache = gpu_cache_from(k, v)
    ocache = oracle_cache_from(k, v)
    assert tq.tq_decode_launches(cache, w.n_q_heads, S, w.attn_scale) == 1
    lens_dev = torch.from_numpy(lens).cuda()
    out = tq.tq_sdpa_int4_decode_varlen(cache, q.cuda(), lens_dev, S, w.attn_scale)
    torch.cuda.synchronize()
    assert_close_elementwise(out, _oracle_varlen(q, ocache, [int(x) for x in lens], w.attn_scale), f"{B} sequences")
    again = tq.tq_sdpa_int4_decode_varlen(cache, q.cuda(), lens_dev, S, w.attn_scale)
    torch.cuda.synchronize()
    assert torch.equal(out, again)


@pytest.mark.parametrize("route", ["packed_rows", "one_block", "planned_chunks"])
def test_sharp_softmax_every_head_keeps_its_own_reference(route):
    """Scores with a spread of tens of log2 units (attn_scale 1 on N(0,1) queries and keys): new maxima keep turning
    up, for one head or another of the group, all along a wave's tokens.  A head's exp2 reference must move only
    when its OWN maximum outgrows it: one that follows every move of a neighbour ends tens of units above the head's
    scores and its weights p * s_v sink into fp16's subnormals (percent-level errors on single rows).  Routes: many
    rows of their own length packed four to a block; one long chunk per block; the device-planned chunks."""
    if route == "packed_rows":
        B, Hkv, S, n_splits = 131, 4, 1025, 0
    elif route == "one_block":
        B, Hkv, S, n_splits = 3, 2, 6000, 1
    else:
        B, Hkv, S, n_splits = 9, 4, 6000, 0
    rng = np.random.default_rng(4052)
    lens = [int(x) for x in rng.integers(S // 2, S + 1, B)]
    w = wl.custom(batch=B, n_q_heads=8 * Hkv, n_kv_heads=Hkv, head_dim=128, seq_len=S, seed=54052, attn_scale=1.0,
                  v_std=0.5)
    q, k, v = make(w)
    cache = gpu_cache_from(k, v)
    ocache = oracle_cache_from(k, v)
    ref = _oracle_varlen(q, ocache, lens, w.attn_scale)
    out = tq.tq_sdpa_int4_decode_varlen(cache, q.cuda(), torch.tensor(lens, dtype=torch.int32, device="cuda"), S,
                                        w.attn_scale, n_splits=n_splits)
    torch.cuda.synchronize()
    assert_close_elementwise(out, ref, route)


@pytest.mark.parametrize("variant", VARIANTS)
def test_bitwise_repeatable(variant):
    w = wl.custom(seq_len=3000, seed=45, **SHAPES["g8_d128_b2_kv3"])
    q, k, v = make(w)
    cache = gpu_cache_from(k, v)
    first = np16(_decode(cache, q, w.seq_len, w.attn_scale, variant=variant)).view(np.uint16)
    for _ in range(5):
        again = np16(_decode(cache, q, w.seq_len, w.attn_scale, variant=variant)).view(np.uint16)
        assert np.array_equal(first, again)


def test_in_kernel_merge_agrees_with_the_two_phase_path():
    """Where decode is one launch (the last block of a KV head merges its chunks in place), the
    result matches partial + reduce: same partials, and the merge differs only in summation order.
    Repeated calls and several chunk counts also check that the arrival counters are left clean."""
    for shape, S in (("g8_d128_b2_kv3", 3000), ("g2_d256", 2100), ("g8_d128", 40)):
        w = wl.custom(seq_len=S, seed=46, **SHAPES[shape])
        q, k, v = make(w)
        cache = gpu_cache_from(k, v)
        ref = oracle_attend(q, oracle_cache_from(k, v), w.seq_len, w.attn_scale)
        assert tq.tq_decode_launches(cache, q.shape[1], S, w.attn_scale) == 1
        ws = torch.empty(tq.tq_workspace_bytes(w.batch, w.n_q_heads, w.head_dim), dtype=torch.uint8, device="cuda")
        for n_splits in (0, 1, 3, 0, 17, 0):
            fused = tq.tq_sdpa_int4_decode(cache, q.cuda(), S, w.attn_scale, workspace=ws, n_splits=n_splits)
            assert_close(fused, ref, f"{shape} in-kernel merge n_splits={n_splits}")
            n = tq.tq_sdpa_int4_partial(cache, q.cuda(), S, w.attn_scale, ws, n_splits=n_splits)
            two = tq.tq_sdpa_int4_reduce(w.batch, w.n_q_heads, w.head_dim, n, ws, torch.empty_like(fused))
            a, b = np16(fused).astype(np.float64), np16(two).astype(np.float64)
            assert np.abs(a - b).max() <= 2.0 ** -10 * max(1.0, np.abs(b).max())    # an fp16 ulp or two


# ---------------------------------------------------------------- unfused comparator

@pytest.mark.parametrize("variant", [0, 1])
def test_dequant_then_attend_matches_oracle(variant):
    """Both attention kernels of the comparator (0: matrix cores where they cover the shape, i.e. d = 128 / 256 and
    up to 16 heads per KV head; 1: the generic vector-ALU kernel) against the comparator's definition, over lengths
    with and without a ragged last supertile, a single token, forced chunk counts, and a group of 20 heads that
    only the generic kernel takes."""
    shapes = dict(SHAPES, g20_d128=dict(n_q_heads=20, n_kv_heads=1, head_dim=128))
    for shape, S, n_splits in (("g8_d128_b2_kv3", 1999, 0), ("g2_d256", 1030, 0), ("g8_d128_b2_kv3", 1, 0),
                               ("g8_d128_b2_kv3", 31, 0), ("g8_d128_b2_kv3", 4096, 3), ("g16_d128", 9001, 0),
                               ("g3_d128", 700, 2), ("g2_d256", 6000, 5), ("g20_d128", 333, 0)):
        w = wl.custom(seq_len=S, seed=51, **shapes[shape])
        q, k, v = make(w)
        cache = gpu_cache_from(k, v, capacity=S + 5)
        ocache = oracle_cache_from(k, v)
        nbytes = tq.tq_dense_scratch_bytes(w.batch, w.n_kv_heads, S, w.head_dim)
        dense = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        out = tq.tq_dequant_then_attend(cache, q.cuda(), S, w.attn_scale, dense_scratch=dense, n_splits=n_splits,
                                        variant=variant)
        torch.cuda.synchronize()
        assert_comparator_close(out, q, ocache, S, w.attn_scale, f"baseline {shape} S={S} variant={variant}")
        # the dense buffers hold fp16((q - z) s) to within one fp16 ulp
        got = np16(dense.view(torch.float16).view(2, w.batch, w.n_kv_heads, S, w.head_dim))
        for i, part in enumerate((ocache[:3], ocache[3:])):
            ref = oracle.dequantize_f16(*part)
            a = got[i].view(np.int16).astype(np.int32)
            b = ref.view(np.int16).astype(np.int32)
            # compare in sign-magnitude order space
            a = np.where(a < 0, -(a & 0x7FFF), a); b = np.where(b < 0, -(b & 0x7FFF), b)
            assert np.abs(a - b).max() <= 1


# ---------------------------------------------------------------- the named workloads, full size,
# in the launch configuration the benchmark times (library defaults)

@pytest.mark.parametrize("name", ["tiny", "llama8k", "gemma32k", "llama128k"])
def test_named_workload_full_size(name):
    w = wl.WORKLOADS[name]
    q, k, v = make(w)
    cache = gpu_cache_from(k, v)
    ocache = oracle_cache_from(k, v)
    assert_cache_bit_exact(cache, ocache, w.seq_len)
    ref = oracle_attend(q, ocache, w.seq_len, w.attn_scale)
    out = _decode(cache, q, w.seq_len, w.attn_scale)
    max_abs, rel = assert_close(out, ref, name)
    print(f"\n{name}: max-abs {max_abs:.2e} rel-L2 {rel:.2e}")
    if name in ("tiny", "llama8k"):
        base = tq.tq_dequant_then_attend(cache, q.cuda(), w.seq_len, w.attn_scale)
        torch.cuda.synchronize()
        assert_comparator_close(base, q, ocache, w.seq_len, w.attn_scale, name + " baseline")


def test_decode_step_append_then_attend():
    # one decode step of the sweep configuration, scaled down: append one token per sequence,
    # then attend over seq_len+1 tokens, for a batch of 4
    w = wl.custom(batch=4, n_q_heads=64, n_kv_heads=8, head_dim=128, seq_len=2048, seed=61, outlier_channels=4)
    q, k, v = make(w)
    S = w.seq_len
    cache = gpu_cache_from(k[:, :, :S - 1], v[:, :, :S - 1], capacity=S)
    tq.tq_quantize_kv(cache, k[:, :, S - 1:].contiguous().cuda(), v[:, :, S - 1:].contiguous().cuda(), S - 1)
    ocache = oracle_cache_from(k, v)
    assert_cache_bit_exact(cache, ocache, S)
    out = _decode(cache, q, S, w.attn_scale)
    assert_close(out, oracle_attend(q, ocache, S, w.attn_scale), "append+attend")


def test_sweep_layers_x_batch4_at_128k_append_then_attend():
    """The full decode-step sweep's launch shape, at full size, on four of its 80 layers: batch 4 of the Llama-70B
    shape at 131072 tokens, every (layer, batch element) pair drawn from its own seed, one step through
    tq_sdpa_int4_append_decode (the new token of every sequence quantised, stored and attended by the call).
    EVERY pair is checked: stored codes, scales and zero-points bit-exact over all 131072 tokens (the appended one
    included), output element by element against the oracle.  The inputs are drawn on the device (fast) and the
    same bits are copied to the host for the oracle."""
    L, B = 4, 4
    base = wl.WORKLOADS["llama128k"]
    S, Hq, Hkv, d = base.seq_len, base.n_q_heads, base.n_kv_heads, base.head_dim
    dev = torch.device("cuda")
    ws = torch.empty(tq.tq_workspace_bytes(B, Hq, d), dtype=torch.uint8, device=dev)
    assert tq.tq_kv_bytes(B, Hkv, S, d) == 4 * base.packed_bytes
    worst_abs = worst_rel = 0.0
    for layer in range(L):
        kb = torch.empty((B, Hkv, S, d), dtype=torch.float16, device=dev)
        vb = torch.empty_like(kb)
        qb = torch.empty((B, Hq, d), dtype=torch.float16, device=dev)
        for b in range(B):
            q, k, v = wl.make_inputs(wl.layer_workload(layer, b), device=dev)
            qb[b], kb[b], vb[b] = q[0], k[0], v[0]
            del q, k, v
        cache = tq.KVCache(B, Hkv, d, S)
        for t in cache.tensors():
            t.view(torch.uint8).fill_(0xEE)
        tq.tq_quantize_kv(cache, kb[:, :, :S - 1].contiguous(), vb[:, :, :S - 1].contiguous(), 0)
        out = tq.tq_sdpa_int4_append_decode(cache, kb[:, :, S - 1:].contiguous(), vb[:, :, S - 1:].contiguous(), qb, S,
                                            base.attn_scale, workspace=ws)
        torch.cuda.synchronize()
        got = [np16(t) for t in cache.tensors()]
        for b in range(B):
            ocache = oracle_cache_from(kb[b:b + 1].cpu(), vb[b:b + 1].cpu())
            for name, g, o in zip(("k_codes", "k_scale", "k_zero", "v_codes", "v_scale", "v_zero"), got, ocache):
                g = g[b:b + 1]
                if g.dtype == np.float16:
                    g, o = g.view(np.uint16), o.view(np.uint16)
                assert np.array_equal(g, o), f"layer {layer} batch element {b}: {name} differs from the oracle"
            ref = oracle_attend(qb[b:b + 1].cpu(), ocache, S, base.attn_scale)
            max_abs, rel = assert_close(out[b:b + 1], ref, f"layer {layer} batch element {b}")
            worst_abs, worst_rel = max(worst_abs, max_abs), max(worst_rel, rel)
        del cache, kb, vb, got
    print(f"\nsweep {L} layers x batch {B} at {S}: worst max-abs {worst_abs:.2e}, worst rel-L2 {worst_rel:.2e}")


# ---------------------------------------------------------------- per-sequence lengths and positions

def _oracle_varlen(q, ocache, lens, alpha):
    """The oracle knows one common length: call it once per sequence with that sequence's own."""
    rows = []
    for b, n in enumerate(lens):
        one = [a[b:b + 1] for a in ocache]
        rows.append(oracle.attend_packed(np16(q[b:b + 1]), *one, seq_len=int(n), alpha=alpha))
    return np.concatenate(rows, axis=0)


@pytest.mark.parametrize("variant", [0, 1, 2])
@pytest.mark.parametrize("shape", ["g8_d128_kv2", "g2_d256"])
def test_decode_with_per_sequence_lengths(shape, variant):
    shapes = dict(SHAPES, g8_d128_kv2=dict(n_q_heads=16, n_kv_heads=2, head_dim=128, outlier_channels=4))
    lens = [1, 33, 1000, 4133, 2048, 31]
    w = wl.custom(batch=len(lens), seq_len=max(lens), seed=71, **shapes[shape])
    q, k, v = make(w)
    cache = gpu_cache_from(k, v, capacity=max(lens) + 11)
    ocache = oracle_cache_from(k, v)
    ref = _oracle_varlen(q, ocache, lens, w.attn_scale)
    lens_dev = torch.tensor(lens, dtype=torch.int32, device="cuda")
    for n_splits in (0, 3):
        try:
            out = tq.tq_sdpa_int4_decode_varlen(cache, q.cuda(), lens_dev, max(lens), w.attn_scale,
                                                n_splits=n_splits, variant=variant)
        except tq.TqError as e:
            if e.status == -6 and variant == 2:
                pytest.skip("matrix-core kernel does not cover this shape")
            raise
        torch.cuda.synchronize()
        assert_close(out, ref, f"{shape} varlen variant={variant} n_splits={n_splits}")
    # lengths outside [1, max_seq_len] are clamped to it; a common length with the same chunk count gives the
    # plain call's bits
    odd = torch.tensor([0, -5, 10 ** 6, 4133, 2048, 31], dtype=torch.int32, device="cuda")
    clamped = [1, 1, max(lens), 4133, 2048, 31]
    out = tq.tq_sdpa_int4_decode_varlen(cache, q.cuda(), odd, max(lens), w.attn_scale, variant=variant)
    assert_close(out, _oracle_varlen(q, ocache, clamped, w.attn_scale), "clamped lengths")
    same = torch.full((len(lens),), 1000, dtype=torch.int32, device="cuda")
    a = tq.tq_sdpa_int4_decode_varlen(cache, q.cuda(), same, 1000, w.attn_scale, variant=variant, n_splits=3)
    b = tq.tq_sdpa_int4_decode(cache, q.cuda(), 1000, w.attn_scale, variant=variant, n_splits=3)
    # same chunking, same partials.  The generic kernel merges both with the merge kernel: same bits.  The plain call of
    # the matrix-core kernel may merge in the kernel instead, in another fp32 summation order: an fp16 ulp apart at most
    if variant == 1:
        assert torch.equal(a, b)
    else:
        fa, fb = a.float(), b.float()
        assert bool(((fa - fb).abs() <= 2.0 ** -10 * fb.abs() + 2.0 ** -24).all())
    c = tq.tq_sdpa_int4_decode_varlen(cache, q.cuda(), same, 1000, w.attn_scale, variant=variant)
    assert_close(c, np16(b).astype(np.float64), "device-planned chunks vs fixed chunks")


def test_append_at_per_sequence_positions():
    w = wl.custom(batch=5, n_q_heads=4, n_kv_heads=2, head_dim=128, seq_len=3, seed=72)
    _, k, v = make(w)
    cap = 40
    cache = tq.KVCache(5, 2, 128, cap)
    for t in cache.tensors():
        t.view(torch.uint8).fill_(0xEE)
    pos = [0, 17, cap - 3, cap - 2, -1]          # the last two do not fit: skipped
    tq.tq_quantize_kv_varlen(cache, k.cuda(), v.cuda(), torch.tensor(pos, dtype=torch.int32, device="cuda"))
    torch.cuda.synchronize()
    ocache = oracle_cache_from(k, v)
    names = ("k_codes", "k_scale", "k_zero", "v_codes", "v_scale", "v_zero")
    for name, g, o in zip(names, cache.tensors(), ocache):
        g = np16(g)
        raw_g = g.view(np.uint8).reshape(5, 2, cap, -1)
        for b, p0 in enumerate(pos):
            fits = 0 <= p0 <= cap - 3
            if fits:
                got, want = g[b, :, p0:p0 + 3], o[b]
                if got.dtype == np.float16:
                    got, want = got.view(np.uint16), want.view(np.uint16)
                assert np.array_equal(got, want), f"{name} sequence {b}"
            keep = np.ones(cap, dtype=bool)
            if fits:
                keep[p0:p0 + 3] = False
            assert (raw_g[b][:, keep] == 0xEE).all(), f"{name} sequence {b}: wrote outside its positions"


# ---------------------------------------------------------------- sliding window

def _oracle_window(q, ocache, lens, window, alpha):
    """Attention over the last `window` tokens of every sequence: the oracle is given exactly those."""
    rows = []
    for b, n in enumerate(lens):
        lo = max(0, n - window)
        one = [a[b:b + 1, :, lo:n] for a in ocache]
        rows.append(oracle.attend_packed(np16(q[b:b + 1]), *one, seq_len=n - lo, alpha=alpha))
    return np.concatenate(rows, axis=0)


@pytest.mark.parametrize("variant", VARIANTS)
@pytest.mark.parametrize("shape", ["g8_d128_b2_kv3", "g2_d256"])
def test_sliding_window(shape, variant):
    S = 3000
    w = wl.custom(seq_len=S, seed=81, **SHAPES[shape])
    q, k, v = make(w)
    cache = gpu_cache_from(k, v, capacity=S + 5)
    ocache = oracle_cache_from(k, v)
    for window in (1, 31, 100, 1024, 2999, 3000, 5000):
        out = _decode(cache, q, S, w.attn_scale, variant=variant, window=window)
        ref = _oracle_window(q, ocache, [S] * w.batch, window, w.attn_scale)
        assert_close(out, ref, f"{shape} window={window} variant={variant}")
    if w.batch > 1:                               # every sequence windows its own length
        lens = [2500, 77][:w.batch]
        lens_dev = torch.tensor(lens, dtype=torch.int32, device="cuda")
        for window, n_splits in ((1024, 0), (1024, 2), (50, 0), (4000, 0)):
            out = tq.tq_sdpa_int4_decode_varlen(cache, q.cuda(), lens_dev, S, w.attn_scale, variant=variant,
                                                window=window, n_splits=n_splits)
            ref = _oracle_window(q, ocache, lens, window, w.attn_scale)
            assert_close(out, ref, f"{shape} varlen window={window} variant={variant}")


# ---------------------------------------------------------------- streams and graphs

def test_concurrent_calls_on_two_streams():
    """Single-launch decodes in flight on two streams at once take different sets of arrival counters."""
    w = wl.custom(seq_len=2500, seed=91, **SHAPES["g8_d128_b2_kv3"])
    q, k, v = make(w)
    cache = gpu_cache_from(k, v)
    ref = oracle_attend(q, oracle_cache_from(k, v), w.seq_len, w.attn_scale)
    qd = q.cuda()
    assert tq.tq_decode_launches(cache, qd.shape[1], w.seq_len, w.attn_scale) == 1
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    ws = [torch.empty(tq.tq_workspace_bytes(w.batch, w.n_q_heads, w.head_dim), dtype=torch.uint8, device="cuda")
          for _ in streams]
    outs = [[torch.empty_like(qd) for _ in range(20)] for _ in streams]
    torch.cuda.synchronize()
    for i in range(20):
        for s, wsp, o in zip(streams, ws, outs):
            with torch.cuda.stream(s):
                tq.tq_sdpa_int4_decode(cache, qd, w.seq_len, w.attn_scale, out=o[i], workspace=wsp)
    torch.cuda.synchronize()
    for si, o in enumerate(outs):                 # (bit for bit per workspace: see the test below)
        assert_close(o[0], ref, f"two streams: stream {si}")
        first = np16(o[0]).view(np.uint16)
        for t in o:
            assert np.array_equal(np16(t).view(np.uint16), first)


def test_single_launch_decodes_on_24_streams_match_the_serial_result():
    """24 decodes of the one-launch route (several chunks per KV head, merged by the block that arrives last) in
    flight at once, each on its own stream with its own workspace: every workspace has its own set of arrival
    counters, so every result equals, bit for bit, the result of the same call made alone WITH THE SAME WORKSPACE.
    (A workspace keeps, for the life of the process, either a set of counters or, if it came when all were taken,
    the merge kernel; the two merges sum in different orders, so results are compared per workspace.)"""
    w = wl.custom(seq_len=8192, seed=93, **SHAPES["g8_d128_b2_kv3"])
    q, k, v = make(w)
    cache = gpu_cache_from(k, v)
    qd = q.cuda()
    assert tq.tq_decode_launches(cache, qd.shape[1], w.seq_len, w.attn_scale) == 1
    assert tq.tq_plan_splits(w.batch, w.n_kv_heads, w.seq_len) > 1
    nbytes = tq.tq_workspace_bytes(w.batch, w.n_q_heads, w.head_dim)
    ref = oracle_attend(q, oracle_cache_from(k, v), w.seq_len, w.attn_scale)
    streams = [torch.cuda.Stream() for _ in range(24)]
    ws = [torch.empty(nbytes, dtype=torch.uint8, device="cuda") for _ in streams]
    want = []
    for si, wsp in enumerate(ws):                 # each call alone, device idle before and after
        alone = tq.tq_sdpa_int4_decode(cache, qd, w.seq_len, w.attn_scale, workspace=wsp)
        torch.cuda.synchronize()
        assert_close(alone, ref, f"alone, workspace {si}")
        want.append(np16(alone).view(np.uint16))
    rounds = 12
    outs = [[torch.zeros_like(qd) for _ in range(rounds)] for _ in streams]
    torch.cuda.synchronize()
    for i in range(rounds):
        for s, wsp, o in zip(streams, ws, outs):
            with torch.cuda.stream(s):
                tq.tq_sdpa_int4_decode(cache, qd, w.seq_len, w.attn_scale, out=o[i], workspace=wsp)
    torch.cuda.synchronize()
    for si, o in enumerate(outs):
        for i, t in enumerate(o):
            assert np.array_equal(np16(t).view(np.uint16), want[si]), f"stream {si}, call {i} differs from the call made alone"


def test_graph_replays_next_to_eager_calls_on_another_stream():
    """A captured one-launch decode keeps the counter set of the workspace it was captured with: replays on one
    stream while eager decodes (another workspace) run on a second stream share nothing, and every replay gives the
    eager result bit for bit."""
    w = wl.custom(seq_len=6000, seed=94, **SHAPES["g8_d128_b2_kv3"])
    q, k, v = make(w)
    cache = gpu_cache_from(k, v)
    qd = q.cuda()
    assert tq.tq_decode_launches(cache, qd.shape[1], w.seq_len, w.attn_scale) == 1
    nbytes = tq.tq_workspace_bytes(w.batch, w.n_q_heads, w.head_dim)
    ws_graph, ws_eager = (torch.empty(nbytes, dtype=torch.uint8, device="cuda") for _ in range(2))
    out_graph = torch.empty_like(qd)
    want = tq.tq_sdpa_int4_decode(cache, qd, w.seq_len, w.attn_scale, workspace=ws_graph).clone()   # (eager first)
    want_eager = tq.tq_sdpa_int4_decode(cache, qd, w.seq_len, w.attn_scale, workspace=ws_eager).clone()
    torch.cuda.synchronize()
    ref = oracle_attend(q, oracle_cache_from(k, v), w.seq_len, w.attn_scale)
    assert_close(want, ref, "eager, the graph's workspace")
    assert_close(want_eager, ref, "eager, the other workspace")   # (bit for bit per workspace, see above)
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        tq.tq_sdpa_int4_decode(cache, qd, w.seq_len, w.attn_scale, out=out_graph, workspace=ws_graph)
    side = torch.cuda.Stream()
    outs_eager = [torch.zeros_like(qd) for _ in range(40)]
    for r in range(5):
        out_graph.zero_()
        torch.cuda.synchronize()
        with torch.cuda.stream(side):             # eager decodes in flight while the graph replays
            for t in outs_eager[r * 8:(r + 1) * 8]:
                tq.tq_sdpa_int4_decode(cache, qd, w.seq_len, w.attn_scale, out=t, workspace=ws_eager)
        g.replay()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(out_graph, want), f"replay round {r}"
    for i, t in enumerate(outs_eager):
        assert torch.equal(t, want_eager), f"eager call {i}"


def test_graph_capture_and_replay():
    """A captured decode step (append + attend, both decode routes) replays to the eager result, with
    eager work and synchronisations between the replays."""
    for shape, S in (("g8_d128_b2_kv3", 1500), ("g2_d256", 700)):
        w = wl.custom(seq_len=S, seed=92, **SHAPES[shape])
        q, k, v = make(w)
        cache = gpu_cache_from(k[:, :, :S - 1], v[:, :, :S - 1], capacity=S)
        kn, vn = k[:, :, S - 1:].contiguous().cuda(), v[:, :, S - 1:].contiguous().cuda()
        qd = q.cuda()
        ws = torch.empty(tq.tq_workspace_bytes(w.batch, w.n_q_heads, w.head_dim), dtype=torch.uint8, device="cuda")
        out1, out2 = torch.empty_like(qd), torch.empty_like(qd)

        def step():
            tq.tq_quantize_kv(cache, kn, vn, S - 1)
            tq.tq_sdpa_int4_decode(cache, qd, S, w.attn_scale, out=out1, workspace=ws)               # one launch
            tq.tq_sdpa_int4_decode(cache, qd, S, w.attn_scale, out=out2, workspace=ws, variant=1)    # two launches

        step()                                    # eager first: also does the one-time kernel attribute set-up
        torch.cuda.synchronize()
        want1, want2 = out1.clone(), out2.clone()
        assert_close(want1, oracle_attend(q, oracle_cache_from(k, v), S, w.attn_scale), "eager step")
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            step()
        for _ in range(4):
            out1.zero_(); out2.zero_()
            cache.k_codes[:, :, S - 1].zero_()    # the replay has to write the appended token again
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            assert torch.equal(out1, want1) and torch.equal(out2, want2)


@pytest.mark.parametrize("route", ["d512", "own_lengths_planned", "own_lengths_rows_as_chunks"])
def test_graph_capture_and_replay_of_the_other_routes(route):
    """The one-call step captured and replayed on the routes the test above does not take: the head_dim 512 kernel
    (its ring is static LDS above 64 KB), per-sequence lengths with device-planned chunks (the plan and the merge
    kernel's appender are redone by every replay), and many rows of their own length (append kernel + decode)."""
    if route == "d512":
        w = wl.custom(seq_len=1500, seed=93, **SHAPES["g32_d512"])
        lens = None
    elif route == "own_lengths_planned":
        w = wl.custom(batch=6, n_q_heads=16, n_kv_heads=2, head_dim=128, seq_len=3000, seed=94)
        lens = [3000, 1, 77, 2049, 1000, 2999]
    else:
        w = wl.custom(batch=70, n_q_heads=32, n_kv_heads=8, head_dim=128, seq_len=600, seed=95)
        lens = [int(x) for x in np.random.default_rng(95).integers(2, 601, 70)]
    S, B = w.seq_len, w.batch
    q, k, v = make(w)
    ocache = oracle_cache_from(k, v)
    cache = gpu_cache_from(k, v, capacity=S)
    own = lens if lens is not None else [S] * B
    kn = torch.stack([k[b, :, own[b] - 1:own[b]] for b in range(B)]).contiguous().cuda()
    vn = torch.stack([v[b, :, own[b] - 1:own[b]] for b in range(B)]).contiguous().cuda()
    qd = q.cuda()
    out = torch.empty_like(qd)
    ws = torch.empty(tq.tq_workspace_bytes(B, w.n_q_heads, w.head_dim), dtype=torch.uint8, device="cuda")
    lens_dev = None if lens is None else torch.tensor(lens, dtype=torch.int32, device="cuda")

    def wipe():                                   # the step has to write every sequence's last token again
        for t in cache.tensors():
            for b in range(B):
                t.view(torch.uint8)[b, :, own[b] - 1] = 0xEE

    def step():
        if lens is None:
            tq.tq_sdpa_int4_append_decode(cache, kn, vn, qd, S, w.attn_scale, out=out, workspace=ws)
        else:
            tq.tq_sdpa_int4_append_decode_varlen(cache, kn, vn, qd, lens_dev, S, w.attn_scale, out=out, workspace=ws)

    wipe()
    step()
    torch.cuda.synchronize()
    want = out.clone()
    ref = oracle_attend(q, ocache, S, w.attn_scale) if lens is None else _oracle_varlen(q, ocache, lens, w.attn_scale)
    assert_close(want, ref, f"{route} eager step")
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        step()
    for _ in range(3):
        out.zero_()
        wipe()
        ws.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, want), f"{route}: a replay differs from the eager step"
        for name, t, o in zip(("k_codes", "k_scale", "k_zero", "v_codes", "v_scale", "v_zero"), cache.tensors(), ocache):
            gt = np16(t)
            if gt.dtype == np.float16:
                gt, o = gt.view(np.uint16), o.view(np.uint16)
            assert np.array_equal(gt[:, :, :S], o[:, :, :S]), f"{route}: {name} after a replay"


# ---------------------------------------------------------------- many small random configurations

def test_random_configurations_against_the_oracle():
    """Seeded sweep over shapes, lengths, chunk counts, windows and per-sequence lengths: every
    combination goes through whichever kernel the library picks and through the generic one."""
    rng = np.random.default_rng(20260416)
    shapes = [(128, 8), (128, 4), (128, 3), (128, 1), (256, 4), (256, 2), (256, 1), (128, 16), (128, 12), (256, 6), (512, 2),
              (512, 20), (512, 32)]
    for case in range(70):
        d, G = shapes[rng.integers(len(shapes))]
        Hkv = int(rng.integers(1, 4))
        B = int(rng.integers(1, 4))
        S = int(rng.choice([1, 7, 32, 63, 64, 65, 255, 256, 257, 1000, 2047, 2049, 3333]))
        cap = S + int(rng.integers(0, 40))
        alpha = float(rng.choice([1.0 / np.sqrt(d), 1.0, 0.02]))
        w = wl.custom(batch=B, n_q_heads=G * Hkv, n_kv_heads=Hkv, head_dim=d, seq_len=S, seed=1000 + case,
                      attn_scale=alpha, qk_std=float(rng.choice([1.0, 0.1])), outlier_channels=int(rng.choice([0, 4])))
        q, k, v = make(w)
        cache = gpu_cache_from(k, v, capacity=cap)
        ocache = oracle_cache_from(k, v)
        n_splits = int(rng.choice([0, 0, 1, 2, 5, 128]))
        window = int(rng.choice([0, 0, 1, 50, 1500]))
        use_lens = bool(rng.integers(2)) and B > 1
        lens = [int(x) for x in rng.integers(1, S + 1, B)] if use_lens else [S] * B
        ref = _oracle_window(q, ocache, lens, window if window > 0 else S, alpha)
        what = f"case {case}: d={d} G={G} Hkv={Hkv} B={B} S={S} n_splits={n_splits} window={window} lens={lens}"
        for variant in (0, 1):
            if use_lens:
                out = tq.tq_sdpa_int4_decode_varlen(cache, q.cuda(), torch.tensor(lens, dtype=torch.int32, device="cuda"),
                                                    S, alpha, n_splits=n_splits, variant=variant, window=window)
            else:
                out = tq.tq_sdpa_int4_decode(cache, q.cuda(), S, alpha, n_splits=n_splits, variant=variant, window=window)
            torch.cuda.synchronize()
            assert_close_elementwise(out, ref, f"{what} variant={variant}")


def test_random_configurations_with_several_query_tokens():
    """The same kind of sweep with 2 ... 8 causal query tokens per sequence (matrix-core kernel only)."""
    rng = np.random.default_rng(20260417)
    shapes = [(128, 8), (128, 4), (128, 3), (128, 1), (256, 2), (256, 1), (128, 16), (256, 3), (512, 2), (512, 5), (512, 8)]
    for case in range(50):
        d, G = shapes[rng.integers(len(shapes))]
        Hkv = int(rng.integers(1, 4))
        B = int(rng.integers(1, 4))
        nq = int(rng.integers(2, 9))
        S = max(nq, int(rng.choice([2, 8, 31, 32, 33, 40, 63, 64, 65, 70, 255, 256, 257, 263, 1000, 2047, 2049, 3333])))
        alpha = float(rng.choice([1.0 / np.sqrt(d), 1.0, 0.02]))
        w = wl.custom(batch=B, n_q_heads=G * Hkv, n_kv_heads=Hkv, head_dim=d, seq_len=S, seed=3000 + case,
                      attn_scale=alpha, qk_std=float(rng.choice([1.0, 0.1])), outlier_channels=int(rng.choice([0, 4])))
        _, k, v = make(w)
        q4 = _queries_for(w, nq)
        cache = gpu_cache_from(k, v, capacity=S + int(rng.integers(0, 40)))
        ocache = oracle_cache_from(k, v)
        n_splits = int(rng.choice([0, 0, 1, 2, 5, 128]))
        use_lens = bool(rng.integers(2)) and B > 1
        lens = [int(x) for x in rng.integers(nq, S + 1, B)] if use_lens else [S] * B
        window = int(rng.choice([0, 0, 1, 9, 50, 1500]))
        ref = _oracle_causal(q4, ocache, lens, alpha, window)
        what = f"case {case}: d={d} G={G} Hkv={Hkv} B={B} S={S} nq={nq} n_splits={n_splits} window={window} lens={lens}"
        if use_lens:
            out = tq.tq_sdpa_int4_decode_varlen(cache, q4.cuda(), torch.tensor(lens, dtype=torch.int32, device="cuda"),
                                                S, alpha, n_splits=n_splits, window=window)
        else:
            out = tq.tq_sdpa_int4_decode(cache, q4.cuda(), S, alpha, n_splits=n_splits, window=window)
        torch.cuda.synchronize()
        assert_close_elementwise(out, ref, what)


def test_random_configurations_of_the_decode_step():
    """The same kind of sweep over the one-call step (append the sequences' last tokens, then attend): common and
    per-sequence lengths, paged pools, 1 ... 4 query tokens, windows, chunk counts, every head dimension; enough
    rows in some cases for the packed-rows routes.  Output against the oracle, and every stored bit of the cache."""
    rng = np.random.default_rng(20260418)
    names = ("k_codes", "k_scale", "k_zero", "v_codes", "v_scale", "v_zero")
    shapes = [(128, 8), (128, 4), (128, 16), (128, 3), (256, 2), (256, 4), (256, 1), (512, 2), (512, 32), (512, 6)]
    for case in range(48):
        kind = str(rng.choice(["common", "own", "own_many", "paged"]))
        d, G = shapes[rng.integers(len(shapes))]
        Hkv, B = int(rng.integers(1, 4)), int(rng.integers(1, 5))
        if kind == "own_many":
            d, G = [(128, 8), (128, 4), (256, 2)][rng.integers(3)]
            Hkv, B = int(rng.choice([4, 8])), int(rng.choice([64, 70, 130]))
            B = max(B, 512 // Hkv + 2)
        nq = int(rng.choice([1, 1, 1, 2, 4])) if kind != "own_many" else 1
        S = max(nq + 1, int(rng.choice([2, 3, 31, 32, 33, 64, 65, 257, 700, 1000, 1025, 2049, 4000])))
        if kind == "own_many":
            S = min(S, 1500)
        alpha = float(rng.choice([1.0 / np.sqrt(d), 1.0, 0.02]))
        window = int(rng.choice([0, 0, 0, 1, 9, 50, 1500]))
        n_splits = int(rng.choice([0, 0, 0, 1, 3, 128])) if kind != "own_many" else 0
        w = wl.custom(batch=B, n_q_heads=G * Hkv, n_kv_heads=Hkv, head_dim=d, seq_len=S, seed=7000 + case, attn_scale=alpha,
                      qk_std=float(rng.choice([1.0, 0.1])), v_std=float(rng.choice([1.0, 0.5])),
                      outlier_channels=int(rng.choice([0, 4])))
        lens = [int(x) for x in rng.integers(nq, S + 1, B)] if kind != "common" else [S] * B
        PT = int(rng.choice([32, 64, 256]))
        what = f"case {case} [{kind}]: d={d} G={G} Hkv={Hkv} B={B} S={S} nq={nq} n_splits={n_splits} window={window} PT={PT}"
        _, k, v = make(w)
        q = _queries_for(w, nq) if nq > 1 else make(w)[0]
        ocache = oracle_cache_from(k, v)
        ref = _oracle_causal(q, ocache, lens, alpha, window) if nq > 1 else \
            _oracle_window(q, ocache, lens, window if window > 0 else S, alpha)
        lens_dev = torch.tensor(lens, dtype=torch.int32, device="cuda")
        # the step's new tokens are each sequence's last nq; the cache holds everything else, 0xEE in their place
        kn = torch.stack([k[b, :, lens[b] - nq:lens[b]] for b in range(B)]).contiguous().cuda()
        vn = torch.stack([v[b, :, lens[b] - nq:lens[b]] for b in range(B)]).contiguous().cuda()
        if kind == "paged":
            max_blocks = (S + PT - 1) // PT
            table = rng.permutation(B * max_blocks + 3)[:B * max_blocks].reshape(B, max_blocks).astype(np.int32)
            table_dev = torch.from_numpy(table).cuda()
            pool = tq.KVCache(B * max_blocks + 3, Hkv, d, PT)
            pad = max_blocks * PT - S
            tq.tq_quantize_kv_paged(pool, table_dev, torch.nn.functional.pad(k, (0, 0, 0, pad)).contiguous().cuda(),
                                    torch.nn.functional.pad(v, (0, 0, 0, pad)).contiguous().cuda(),
                                    torch.zeros(B, dtype=torch.int32, device="cuda"))
            for t in pool.tensors():
                for b in range(B):
                    for pos in range(lens[b] - nq, lens[b]):
                        t.view(torch.uint8)[int(table[b, pos // PT]), :, pos % PT] = 0xEE
            out = tq.tq_sdpa_int4_append_decode_paged(pool, table_dev, kn, vn, q.cuda(), lens_dev, S, alpha,
                                                      n_splits=n_splits, window=window)
            torch.cuda.synchronize()
            stored = [np.stack([np.concatenate([np16(t)[table[b, j]] for j in range(max_blocks)], axis=1)[:, :S]
                                for b in range(B)]) for t in pool.tensors()]
        else:
            cache = gpu_cache_from(k, v, capacity=S + 5)
            for t in cache.tensors():
                for b in range(B):
                    t.view(torch.uint8)[b, :, lens[b] - nq:lens[b]] = 0xEE
            if kind == "common":
                out = tq.tq_sdpa_int4_append_decode(cache, kn, vn, q.cuda(), S, alpha, n_splits=n_splits, window=window)
            else:
                out = tq.tq_sdpa_int4_append_decode_varlen(cache, kn, vn, q.cuda(), lens_dev, S, alpha, n_splits=n_splits,
                                                           window=window)
            torch.cuda.synchronize()
            stored = [np16(t)[:, :, :S] for t in cache.tensors()]
            for t in cache.tensors():
                assert bool((t.view(torch.uint8)[:, :, S:] == 0xEE).all()), f"{what}: wrote past the sequences"
        assert_close_elementwise(out, ref, what)
        for name, g, o in zip(names, stored, ocache):     # (tokens past a sequence's own length: the bulk fill's, untouched)
            o = o[:, :, :S]
            if g.dtype == np.float16:
                g, o = g.view(np.uint16), o.view(np.uint16)
            assert np.array_equal(g, o), f"{what}: {name} differs from the oracle"


# ---------------------------------------------------------------- one call per decode step

@pytest.mark.parametrize("variant", [0, 1])
@pytest.mark.parametrize("shape", ["g8_d128_b2_kv3", "g3_d128", "g2_d256"])
def test_append_decode_in_one_call(shape, variant):
    """tq_sdpa_int4_append_decode = quantise-append of the step's token + attention over all of them:
    the stored bits equal the oracle's and the result matches the oracle over seq_len tokens, whether the
    decode kernel takes the token in itself (matrix-core kernel, d=128) or two kernels are launched."""
    for S, window, n_splits in ((1, 0, 0), (2, 0, 0), (33, 0, 0), (1000, 0, 3), (2500, 0, 0), (2500, 700, 0), (64, 1, 0)):
        w = wl.custom(seq_len=S, seed=95 + S, **SHAPES[shape])
        q, k, v = make(w)
        cache = gpu_cache_from(k[:, :, :S - 1], v[:, :, :S - 1], capacity=S + 3, fill=0xEE) if S > 1 else None
        if cache is None:
            cache = tq.KVCache(w.batch, w.n_kv_heads, w.head_dim, S + 3)
            for t in cache.tensors():
                t.view(torch.uint8).fill_(0xEE)
        kn, vn = k[:, :, S - 1:].contiguous().cuda(), v[:, :, S - 1:].contiguous().cuda()
        out = tq.tq_sdpa_int4_append_decode(cache, kn, vn, q.cuda(), S, w.attn_scale, variant=variant, window=window,
                                            n_splits=n_splits)
        torch.cuda.synchronize()
        ocache = oracle_cache_from(k, v)
        assert_cache_bit_exact(cache, ocache, S)
        for t in cache.tensors():                 # nothing beyond the appended token is touched
            assert bool((t.view(torch.uint8)[:, :, S:] == 0xEE).all())
        ref = _oracle_window(q, ocache, [S] * w.batch, window if window > 0 else S, w.attn_scale)
        assert_close(out, ref, f"{shape} append+decode S={S} window={window} variant={variant}")
        again = tq.tq_sdpa_int4_decode(cache, q.cuda(), S, w.attn_scale, variant=variant, window=window, n_splits=n_splits)
        a, b = np16(out).astype(np.float64), np16(again).astype(np.float64)
        assert np.abs(a - b).max() <= 2.0 ** -9 * max(1.0, np.abs(b).max())   # same step through the two calls


@pytest.mark.parametrize("variant", [0, 2])
@pytest.mark.parametrize("shape", ["g16_d128_b2_kv2", "g12_d128", "g8_d256"])
def test_gqa_groups_larger_than_the_matrix_core_tile(shape, variant):
    """GQA ratios above the 8-row tile (d=128: a tile of 16 rows) or above any tile (d=256: two rows; then several
    blocks stream each KV head, each with its share of the group); plain decode (merged in the kernel or by the
    reduce launch), sliding window, per-sequence lengths and the one-call step all take that path."""
    shapes = dict(g16_d128_b2_kv2=dict(batch=2, n_q_heads=32, n_kv_heads=2, head_dim=128, outlier_channels=4),
                  g12_d128=dict(n_q_heads=12, n_kv_heads=1, head_dim=128),
                  g8_d256=dict(batch=2, n_q_heads=24, n_kv_heads=3, head_dim=256, attn_scale=1.0, qk_std=0.1))
    for S, window, n_splits in ((1, 0, 0), (33, 0, 0), (700, 0, 5), (4133, 0, 0), (4133, 900, 0), (20000, 0, 0)):
        w = wl.custom(seq_len=S, seed=960 + S, **shapes[shape])
        q, k, v = make(w)
        cache = gpu_cache_from(k[:, :, :S - 1], v[:, :, :S - 1], capacity=S + 3) if S > 1 else \
            tq.KVCache(w.batch, w.n_kv_heads, w.head_dim, S + 3)
        kn, vn = k[:, :, S - 1:].contiguous().cuda(), v[:, :, S - 1:].contiguous().cuda()
        out = tq.tq_sdpa_int4_append_decode(cache, kn, vn, q.cuda(), S, w.attn_scale, variant=variant, window=window,
                                            n_splits=n_splits)
        torch.cuda.synchronize()
        ocache = oracle_cache_from(k, v)
        assert_cache_bit_exact(cache, ocache, S)
        ref = _oracle_window(q, ocache, [S] * w.batch, window if window > 0 else S, w.attn_scale)
        assert_close(out, ref, f"{shape} S={S} window={window} variant={variant}")
        lens = [max(1, S - 13 * b) for b in range(w.batch)]
        out = tq.tq_sdpa_int4_decode_varlen(cache, q.cuda(), torch.tensor(lens, dtype=torch.int32).cuda(), S,
                                            w.attn_scale, variant=variant, window=window)
        torch.cuda.synchronize()
        assert_close(out, _oracle_window(q, ocache, lens, window if window > 0 else S, w.attn_scale),
                     f"{shape} per-sequence lengths S={S} window={window} variant={variant}")


@pytest.mark.parametrize("gqa", [9, 10, 16, 24, 40])
def test_sixteen_row_tiles(gqa):
    """d = 128 with 9 or more query rows per KV head: tiles of 16 rows (every column of the tile a row of its own,
    one score accumulator per quantisation group, the P V columns regrouped by group), partly filled (9, 10 of 16),
    full, and several per KV head (24 = 2 x 12, 40 = 4 x 10).  Ragged lengths around the 32-token supertile and
    the chunk boundaries, forced chunk counts, a sliding window, per-sequence lengths, and a sharp softmax where
    every one of the 16 rows keeps moving its own reference."""
    Hkv, B = 2, 2
    for S, window, n_splits, scale in ((1, 0, 0, None), (31, 0, 0, None), (32, 0, 0, None), (33, 0, 0, None),
                                       (1025, 0, 0, None), (2500, 0, 7, None), (4133, 700, 0, None),
                                       (9000, 0, 0, 1.0), (20000, 0, 0, None)):
        kw = dict(attn_scale=scale, v_std=0.5) if scale else {}
        w = wl.custom(batch=B, n_q_heads=gqa * Hkv, n_kv_heads=Hkv, head_dim=128, seq_len=S, seed=1600 + gqa + S,
                      outlier_channels=4, **kw)
        q, k, v = make(w)
        cache = gpu_cache_from(k, v)
        ocache = oracle_cache_from(k, v)
        out = tq.tq_sdpa_int4_decode(cache, q.cuda(), S, w.attn_scale, window=window, n_splits=n_splits)
        torch.cuda.synchronize()
        ref = _oracle_window(q, ocache, [S] * B, window if window > 0 else S, w.attn_scale)
        assert_close_elementwise(out, ref, f"GQA {gqa} S={S} window={window} n_splits={n_splits} scale={scale}")
        lens = [S, max(1, S - 37)]
        out = tq.tq_sdpa_int4_decode_varlen(cache, q.cuda(), torch.tensor(lens, dtype=torch.int32).cuda(), S,
                                            w.attn_scale, window=window)
        torch.cuda.synchronize()
        assert_close_elementwise(out, _oracle_window(q, ocache, lens, window if window > 0 else S, w.attn_scale),
                                 f"GQA {gqa} per-sequence lengths S={S} window={window}")


def test_sixteen_row_tiles_at_128k():
    """16 query heads per KV head over the 128K layer of the headline shape (8 KV heads): one 16-row block per
    chunk and KV head, every output element against the oracle."""
    w = wl.custom(n_q_heads=128, n_kv_heads=8, head_dim=128, seq_len=131072, seed=16128, outlier_channels=4)
    q, k, v = make(w)
    cache = gpu_cache_from(k, v)
    ocache = oracle_cache_from(k, v)
    del k, v
    out = tq.tq_sdpa_int4_decode(cache, q.cuda(), w.seq_len, w.attn_scale)
    torch.cuda.synchronize()
    ref = oracle.attend_packed(np16(q), *ocache, seq_len=w.seq_len, alpha=w.attn_scale)
    assert_close_elementwise(out, ref, "GQA 16 at 128K")


# ---------------------------------------------------------------- several query tokens per sequence

def _queries_for(w, nq):
    """nq query tokens per sequence, [B, nq, H_q, d]: token t is the workload's query drawn with seed + 7 t."""
    import dataclasses
    qs = [make(dataclasses.replace(w, seed=w.seed + 7 * t))[0] for t in range(nq)]
    return torch.stack(qs, dim=1).contiguous()


def _oracle_causal(q4, ocache, lens, alpha, window=0):
    """Query token t of sequence b attends the first lens[b] - (nq - 1 - t) tokens, under a sliding window the
    last `window` of those: the definition, row by row (the oracle is handed exactly the attended slice)."""
    nq = q4.shape[1]
    out = np.empty(tuple(q4.shape), dtype=np.float64)
    for b, n in enumerate(lens):
        for t in range(nq):
            hi = n - (nq - 1 - t)
            lo = max(0, hi - window) if window > 0 else 0
            one = [a[b:b + 1, :, lo:hi] for a in ocache]
            out[b, t] = oracle.attend_packed(np16(q4[b:b + 1, t]), *one, seq_len=hi - lo, alpha=alpha)[0]
    return out


@pytest.mark.parametrize("nq", [2, 3, 4, 8])
@pytest.mark.parametrize("shape", ["g8_d128_b2_kv3", "g2_d256", "g3_d128", "g16_d128", "g4_d256"])
def test_several_query_tokens(shape, nq):
    """n_queries > 1: the sequence's last nq tokens as queries, causal among themselves, against the oracle
    row by row; lengths around the 32-token supertile boundaries put the masked tokens in one supertile, in
    two, and in a chunk of their own."""
    for S, n_splits in ((nq, 0), (31, 0), (33, 0), (63, 0), (64, 0), (65, 0), (66, 0), (71, 0), (1000, 0), (1030, 4),
                        (4133, 0), (20002, 0)):
        if S < nq:
            continue
        w = wl.custom(seq_len=S, seed=1200 + S + nq, **SHAPES[shape])
        _, k, v = make(w)
        q4 = _queries_for(w, nq)
        cache = gpu_cache_from(k, v, capacity=S + 3)
        ocache = oracle_cache_from(k, v)
        out = tq.tq_sdpa_int4_decode(cache, q4.cuda(), S, w.attn_scale, n_splits=n_splits)
        torch.cuda.synchronize()
        assert tuple(out.shape) == tuple(q4.shape)
        ref = _oracle_causal(q4, ocache, [S] * w.batch, w.attn_scale)
        assert_close(out, ref, f"{shape} nq={nq} S={S}")
        # the last query token is the plain decode step over S tokens
        last = tq.tq_sdpa_int4_decode(cache, q4[:, nq - 1].contiguous().cuda(), S, w.attn_scale, n_splits=n_splits)
        a, b = np16(out[:, nq - 1]).astype(np.float64), np16(last).astype(np.float64)
        assert np.abs(a - b).max() <= 2.0 ** -9 * max(1.0, np.abs(b).max())
        # sliding window: every query token attends the last `window` tokens up to its own
        for window in (1, 5, 32, 40, 700):
            out = tq.tq_sdpa_int4_decode(cache, q4.cuda(), S, w.attn_scale, n_splits=n_splits, window=window)
            torch.cuda.synchronize()
            assert_close(out, _oracle_causal(q4, ocache, [S] * w.batch, w.attn_scale, window),
                         f"{shape} nq={nq} S={S} window={window}")


@pytest.mark.parametrize("nq", [2, 5])
@pytest.mark.parametrize("shape", ["g8_d128_b2_kv3", "g2_d256", "g4_d512_b2_kv2"])
def test_several_query_tokens_append_varlen_and_two_phase(shape, nq):
    """The other entry points with n_queries > 1: append the nq tokens and attend in one call (stored bits equal
    the oracle's); per-sequence lengths; phase 1 and phase 2 called separately."""
    for S in (nq, 77, 2500):
        w = wl.custom(seq_len=S, seed=1300 + S + nq, **SHAPES[shape])
        _, k, v = make(w)
        q4 = _queries_for(w, nq)
        ocache = oracle_cache_from(k, v)
        cache = tq.KVCache(w.batch, w.n_kv_heads, w.head_dim, S + 3)
        for t in cache.tensors():
            t.view(torch.uint8).fill_(0xEE)
        if S > nq:
            tq.tq_quantize_kv(cache, k[:, :, :S - nq].contiguous().cuda(), v[:, :, :S - nq].contiguous().cuda(), 0)
        kn, vn = k[:, :, S - nq:].contiguous().cuda(), v[:, :, S - nq:].contiguous().cuda()
        out = tq.tq_sdpa_int4_append_decode(cache, kn, vn, q4.cuda(), S, w.attn_scale)
        torch.cuda.synchronize()
        assert_cache_bit_exact(cache, ocache, S)
        for t in cache.tensors():
            assert bool((t.view(torch.uint8)[:, :, S:] == 0xEE).all())
        assert_close(out, _oracle_causal(q4, ocache, [S] * w.batch, w.attn_scale), f"{shape} append nq={nq} S={S}")
        # per-sequence lengths (each at least nq)
        lens = [max(nq, S - 29 * b) for b in range(w.batch)]
        for window in (0, 3, 50):
            out = tq.tq_sdpa_int4_decode_varlen(cache, q4.cuda(), torch.tensor(lens, dtype=torch.int32).cuda(), S,
                                                w.attn_scale, window=window)
            torch.cuda.synchronize()
            assert_close(out, _oracle_causal(q4, ocache, lens, w.attn_scale, window),
                         f"{shape} varlen nq={nq} S={S} window={window}")
        # the two phases on their own: rows of the workspace and of `out` are (sequence, query token) pairs
        ws = torch.empty(tq.tq_workspace_bytes(w.batch * nq, w.n_q_heads, w.head_dim), dtype=torch.uint8, device="cuda")
        n = tq.tq_sdpa_int4_partial(cache, q4.cuda(), S, w.attn_scale, ws)
        out2 = torch.empty_like(q4, device="cuda")
        tq.tq_sdpa_int4_reduce(w.batch * nq, w.n_q_heads, w.head_dim, n, ws, out2)
        torch.cuda.synchronize()
        assert_close(out2, _oracle_causal(q4, ocache, [S] * w.batch, w.attn_scale), f"{shape} two-phase nq={nq} S={S}")


def test_several_query_tokens_rejections():
    w = wl.custom(seq_len=100, seed=5, **SHAPES["g8_d128"])
    q, k, v = make(w)
    cache = gpu_cache_from(k, v)
    q4 = _queries_for(w, 3).cuda()
    with pytest.raises(tq.TqError) as e:
        tq.tq_sdpa_int4_decode(cache, q4, 100, w.attn_scale, variant=1)
    assert e.value.status == -6
    with pytest.raises(tq.TqError) as e:
        tq.tq_sdpa_int4_decode(cache, q4, 2, w.attn_scale)          # fewer tokens than queries
    assert e.value.status == -3
    with pytest.raises(tq.TqError) as e:
        tq.tq_sdpa_int4_decode(cache, q4, 100, -1.0)                # the generic kernel's case
    assert e.value.status == -6
    q9 = torch.zeros(1, 9, 8, 128, dtype=torch.float16, device="cuda")
    with pytest.raises(tq.TqError) as e:
        tq.tq_sdpa_int4_decode(cache, q9, 100, w.attn_scale)
    assert e.value.status == -6


# ---------------------------------------------------------------- head_dim 512

@pytest.mark.parametrize("shape", ["g4_d512", "g32_d512"])
def test_head_dim_512(shape):
    """d = 512 (the global-attention configuration of the kernel table in the appendix, GQA 32): quantiser bit-exact,
    its own matrix-core kernel (query rows in tiles of 16 or 32) and the generic kernel, every entry point."""
    shapes = dict(g4_d512=dict(batch=2, n_q_heads=8, n_kv_heads=2, head_dim=512, attn_scale=1.0, qk_std=0.1),
                  g32_d512=dict(n_q_heads=32, n_kv_heads=1, head_dim=512, attn_scale=1.0, qk_std=0.1))
    for S in (1, 33, 1000, 4133):
        w = wl.custom(seq_len=S, seed=1400 + S, **shapes[shape])
        q, k, v = make(w)
        ocache = oracle_cache_from(k, v)
        cache = tq.KVCache(w.batch, w.n_kv_heads, w.head_dim, S + 3)
        for t in cache.tensors():
            t.view(torch.uint8).fill_(0xEE)
        if S > 1:
            tq.tq_quantize_kv(cache, k[:, :, :S - 1].contiguous().cuda(), v[:, :, :S - 1].contiguous().cuda(), 0)
        kn, vn = k[:, :, S - 1:].contiguous().cuda(), v[:, :, S - 1:].contiguous().cuda()
        out = tq.tq_sdpa_int4_append_decode(cache, kn, vn, q.cuda(), S, w.attn_scale)
        torch.cuda.synchronize()
        assert_cache_bit_exact(cache, ocache, S)
        for t in cache.tensors():
            assert bool((t.view(torch.uint8)[:, :, S:] == 0xEE).all())
        ref = oracle_attend(q, ocache, S, w.attn_scale)
        assert_close(out, ref, f"{shape} S={S}")
        for n_splits in (1, 3, 128):
            assert_close(tq.tq_sdpa_int4_decode(cache, q.cuda(), S, w.attn_scale, n_splits=n_splits), ref,
                         f"{shape} S={S} n_splits={n_splits}")
        lens = [max(1, S - 17 * b) for b in range(w.batch)]
        out = tq.tq_sdpa_int4_decode_varlen(cache, q.cuda(), torch.tensor(lens, dtype=torch.int32).cuda(), S, w.attn_scale)
        torch.cuda.synchronize()
        assert_close(out, _oracle_varlen(q, ocache, lens, w.attn_scale), f"{shape} per-sequence lengths S={S}")
        win = max(1, S // 3)
        out = tq.tq_sdpa_int4_decode(cache, q.cuda(), S, w.attn_scale, window=win)
        torch.cuda.synchronize()
        assert_close(out, _oracle_window(q, ocache, [S] * w.batch, win, w.attn_scale), f"{shape} window S={S}")
        base = tq.tq_dequant_then_attend(cache, q.cuda(), S, w.attn_scale)
        torch.cuda.synchronize()
        assert_comparator_close(base, q, ocache, S, w.attn_scale, f"{shape} comparator S={S}")
        for variant in (1, 2):                    # the generic kernel, and the head_dim 512 matrix-core kernel by name
            assert_close(tq.tq_sdpa_int4_decode(cache, q.cuda(), S, w.attn_scale, variant=variant), ref,
                         f"{shape} S={S} variant={variant}")


@pytest.mark.parametrize("nq", [2, 3, 8])
@pytest.mark.parametrize("shape", ["g4_d512_b2_kv2", "g32_d512", "g6_d512"])
def test_head_dim_512_several_query_tokens(shape, nq):
    """d = 512 with n_queries > 1: the rows (query token, head) of a KV head fill one tile of 16 or 32 rows or
    several (32 heads x 8 tokens: 256 rows); every row has its own causal end and, under a window, its own start."""
    for S, n_splits in ((nq, 0), (33, 0), (64, 0), (71, 0), (1000, 0), (1030, 4), (2500, 0)):
        if S < nq:
            continue
        w = wl.custom(seq_len=S, seed=1500 + S + nq, **SHAPES[shape])
        _, k, v = make(w)
        q4 = _queries_for(w, nq)
        cache = gpu_cache_from(k, v, capacity=S + 3)
        ocache = oracle_cache_from(k, v)
        out = tq.tq_sdpa_int4_decode(cache, q4.cuda(), S, w.attn_scale, n_splits=n_splits)
        torch.cuda.synchronize()
        assert_close(out, _oracle_causal(q4, ocache, [S] * w.batch, w.attn_scale), f"{shape} nq={nq} S={S}")
        for window in (1, 5, 40, 700):
            out = tq.tq_sdpa_int4_decode(cache, q4.cuda(), S, w.attn_scale, n_splits=n_splits, window=window)
            torch.cuda.synchronize()
            assert_close(out, _oracle_causal(q4, ocache, [S] * w.batch, w.attn_scale, window),
                         f"{shape} nq={nq} S={S} window={window}")
    with pytest.raises(tq.TqError) as e:
        tq.tq_sdpa_int4_decode(cache, q4.cuda(), S, w.attn_scale, variant=1)
    assert e.value.status == -6


# ---------------------------------------------------------------- paged cache

@pytest.mark.parametrize("variant", [0, 1, 2])
@pytest.mark.parametrize("shape", ["g8_d128_kv2", "g2_d256", "g6_d512"])
def test_paged_cache(shape, variant):
    """Sequences scattered page by page over a pool: fill and append through the block table, attend
    with per-sequence lengths; the oracle gets each sequence's tokens gathered back in order."""
    shapes = dict(SHAPES, g8_d128_kv2=dict(n_q_heads=16, n_kv_heads=2, head_dim=128, outlier_channels=4))
    lens = [1000, 77, 2049, 256]
    PT, max_blocks, n_pages = 256, 9, 40
    w = wl.custom(batch=len(lens), seq_len=max(lens) + 1, seed=97, **shapes[shape])
    q, k, v = make(w)                             # token max(lens) is the one appended later
    B, Hkv, d = w.batch, w.n_kv_heads, w.head_dim
    rng = np.random.default_rng(5)
    table = rng.permutation(n_pages)[:B * max_blocks].reshape(B, max_blocks).astype(np.int32)
    table_dev = torch.from_numpy(table).cuda()
    pool = tq.KVCache(n_pages, Hkv, d, PT)
    for t in pool.tensors():
        t.view(torch.uint8).fill_(0xEE)
    S = max(lens)
    zeros = torch.zeros(B, dtype=torch.int32, device="cuda")
    tq.tq_quantize_kv_paged(pool, table_dev, k[:, :, :S].contiguous().cuda(), v[:, :, :S].contiguous().cuda(), zeros)
    torch.cuda.synchronize()
    ocache = oracle_cache_from(k, v)
    names = ("k_codes", "k_scale", "k_zero", "v_codes", "v_scale", "v_zero")

    def gathered(b, n):                           # sequence b's first n tokens, read back through the table
        out = []
        for t in pool.tensors():
            g = np16(t)
            out.append(np.concatenate([g[table[b, j]] for j in range((n + PT - 1) // PT)], axis=1)[:, :n])
        return out

    for b in range(B):
        for name, g, o in zip(names, gathered(b, S), ocache):
            o = o[b, :, :S]
            if g.dtype == np.float16:
                g, o = g.view(np.uint16), o.view(np.uint16)
            assert np.array_equal(g, o), f"{name} sequence {b}"
    used = set(table[:, :(S + PT - 1) // PT].ravel().tolist())
    for t in pool.tensors():                      # pages nobody's tokens reach stay untouched
        raw_t = t.view(torch.uint8).cpu().numpy()
        for page in range(n_pages):
            if page not in used:
                assert (raw_t[page] == 0xEE).all()

    lens_dev = torch.tensor(lens, dtype=torch.int32, device="cuda")
    ref = _oracle_varlen(q, ocache, lens, w.attn_scale)
    if variant != 1:                              # several query tokens per sequence over the paged pool
        q4 = _queries_for(w, 3)
        out = tq.tq_sdpa_int4_decode_paged(pool, table_dev, q4.cuda(), lens_dev, S, w.attn_scale, variant=variant)
        torch.cuda.synchronize()
        assert_close(out, _oracle_causal(q4, ocache, lens, w.attn_scale), f"{shape} paged, 3 query tokens")
    # sliding window over pages: the window's first token need not start a supertile (nor a page)
    for window in (1, 31, 32, 100, 257, 1500, 5000):
        for n_splits in (0, 4):
            try:
                out = tq.tq_sdpa_int4_decode_paged(pool, table_dev, q.cuda(), lens_dev, S, w.attn_scale, variant=variant,
                                                   window=window, n_splits=n_splits)
            except tq.TqError as e:
                if e.status == -6 and variant == 2:
                    pytest.skip("matrix-core kernel does not cover this shape")
                raise
            torch.cuda.synchronize()
            assert_close(out, _oracle_window(q, ocache, lens, window, w.attn_scale),
                         f"{shape} paged window={window} variant={variant} n_splits={n_splits}")
        if variant != 1:
            q4 = _queries_for(w, 3)
            out = tq.tq_sdpa_int4_decode_paged(pool, table_dev, q4.cuda(), lens_dev, S, w.attn_scale, variant=variant,
                                               window=window)
            torch.cuda.synchronize()
            assert_close(out, _oracle_causal(q4, ocache, lens, w.attn_scale, window),
                         f"{shape} paged, 3 query tokens, window={window}")
    for n_splits in (0, 3):
        try:
            out = tq.tq_sdpa_int4_decode_paged(pool, table_dev, q.cuda(), lens_dev, S, w.attn_scale,
                                               n_splits=n_splits, variant=variant)
        except tq.TqError as e:
            if e.status == -6 and variant == 2:
                pytest.skip("matrix-core kernel does not cover this shape")
            raise
        torch.cuda.synchronize()
        assert_close(out, ref, f"{shape} paged variant={variant} n_splits={n_splits}")
    # one decode step: every sequence appends its next token (the one stored at index max(lens) of the source)
    # at its own position, then attends one token more
    kn, vn = k[:, :, S:S + 1].contiguous().cuda(), v[:, :, S:S + 1].contiguous().cuda()
    tq.tq_quantize_kv_paged(pool, table_dev, kn, vn, lens_dev)
    out = tq.tq_sdpa_int4_decode_paged(pool, table_dev, q.cuda(), lens_dev + 1, S + 1, w.attn_scale, variant=variant)
    torch.cuda.synchronize()
    rows = []
    for b, n in enumerate(lens):
        one = [np.concatenate([a[b:b + 1, :, :n], a[b:b + 1, :, S:S + 1]], axis=2) for a in ocache]
        rows.append(oracle.attend_packed(np16(q[b:b + 1]), *one, seq_len=n + 1, alpha=w.attn_scale))
    assert_close(out, np.concatenate(rows, axis=0), f"{shape} paged append+attend variant={variant}")


@pytest.mark.parametrize("shape", ["g8_d128_kv2", "g2_d256", "g6_d512"])
def test_paged_window_whose_rows_start_in_two_supertiles(shape):
    """Paged pool + sliding window + several query tokens: a paged sequence is read from the 32-token boundary before
    its window, and the query rows start one token after another; with the window's first token in the last slots
    of a supertile the later rows start in the NEXT one, which then has to be masked too, in whichever chunk it
    lies.  (A window of 50 on 115 tokens with 4 query tokens: rows start at tokens 62 .. 65.)"""
    shapes = dict(SHAPES, g8_d128_kv2=dict(n_q_heads=16, n_kv_heads=2, head_dim=128, outlier_channels=4))
    PT, window = 64, 50
    for nq in (4, 8):
        # first attended token of the earliest row: len - window - (nq - 1); 29, 30, 31 and 0 modulo 32
        lens = [29 + 32 + window + nq - 1, 30 + 64 + window + nq - 1, 31 + window + nq - 1, 64 + window + nq - 1, window - 7]
        S = max(lens)
        w = wl.custom(batch=len(lens), seq_len=S, seed=2100 + nq, **dict(shapes[shape], attn_scale=1.0))
        _, k, v = make(w)
        q4 = _queries_for(w, nq)
        B, Hkv, d = w.batch, w.n_kv_heads, w.head_dim
        max_blocks = (S + PT - 1) // PT
        rng = np.random.default_rng(nq)
        table = torch.from_numpy(rng.permutation(B * max_blocks + 2)[:B * max_blocks].reshape(B, max_blocks).astype(np.int32)).cuda()
        pool = tq.KVCache(B * max_blocks + 2, Hkv, d, PT)
        pad = max_blocks * PT - S
        tq.tq_quantize_kv_paged(pool, table, torch.nn.functional.pad(k, (0, 0, 0, pad)).contiguous().cuda(),
                                torch.nn.functional.pad(v, (0, 0, 0, pad)).contiguous().cuda(),
                                torch.zeros(B, dtype=torch.int32, device="cuda"))
        ocache = oracle_cache_from(k, v)
        lens_dev = torch.tensor(lens, dtype=torch.int32, device="cuda")
        ref = _oracle_causal(q4, ocache, lens, w.attn_scale, window)
        for n_splits in (0, 1, 3, 4):
            out = tq.tq_sdpa_int4_decode_paged(pool, table, q4.cuda(), lens_dev, S, w.attn_scale, window=window,
                                               n_splits=n_splits)
            torch.cuda.synchronize()
            assert_close_elementwise(out, ref, f"{shape} nq={nq} n_splits={n_splits}")


def test_many_sequences_with_their_own_lengths():
    """More sequences than one round of blocks has chunks for: the device-side plan spreads them over
    several rounds; contiguous rows and pages."""
    B, Hkv, G, d = 40, 4, 8, 128
    rng = np.random.default_rng(11)
    lens = [int(x) for x in rng.integers(1, 700, B)]
    lens[3], lens[17] = 1500, 1
    S = max(lens)
    w = wl.custom(batch=B, n_q_heads=G * Hkv, n_kv_heads=Hkv, head_dim=d, seq_len=S, seed=98, outlier_channels=4)
    q, k, v = make(w)
    ocache = oracle_cache_from(k, v)
    ref = _oracle_varlen(q, ocache, lens, w.attn_scale)
    lens_dev = torch.tensor(lens, dtype=torch.int32, device="cuda")
    cache = gpu_cache_from(k, v)
    for variant in (0, 1):
        out = tq.tq_sdpa_int4_decode_varlen(cache, q.cuda(), lens_dev, S, w.attn_scale, variant=variant)
        torch.cuda.synchronize()
        assert_close(out, ref, f"40 sequences, variant={variant}")
    PT, max_blocks = 64, (S + 63) // 64
    table = torch.from_numpy(rng.permutation(B * max_blocks).astype(np.int32).reshape(B, max_blocks)).cuda()
    pool = tq.KVCache(B * max_blocks, Hkv, d, PT)
    pad = max_blocks * PT - S
    kp = torch.nn.functional.pad(k, (0, 0, 0, pad)).contiguous().cuda()
    vp = torch.nn.functional.pad(v, (0, 0, 0, pad)).contiguous().cuda()
    tq.tq_quantize_kv_paged(pool, table, kp, vp, torch.zeros(B, dtype=torch.int32, device="cuda"))
    out = tq.tq_sdpa_int4_decode_paged(pool, table, q.cuda(), lens_dev, S, w.attn_scale)
    torch.cuda.synchronize()
    assert_close(out, ref, "40 sequences, paged")


def test_many_short_sequences_take_the_single_chunk_route():
    """More (sequence, KV head) rows than the chip has compute units: every sequence is one chunk and the kernel
    writes the output itself, in one launch, also above the size where longer sequences get a merge kernel."""
    w = wl.custom(batch=40, n_q_heads=64, n_kv_heads=8, head_dim=128, seq_len=1500, seed=1500, outlier_channels=4)
    q, k, v = make(w)
    cache = gpu_cache_from(k, v)
    assert tq.tq_kv_bytes(w.batch, w.n_kv_heads, w.seq_len, w.head_dim) > 48 << 20
    assert tq.tq_decode_launches(cache, w.n_q_heads, w.seq_len, w.attn_scale) == 1
    out = tq.tq_sdpa_int4_decode(cache, q.cuda(), w.seq_len, w.attn_scale)
    torch.cuda.synchronize()
    assert_close(out, oracle_attend(q, oracle_cache_from(k, v), w.seq_len, w.attn_scale), "40 sequences of 1500 tokens")


def test_quarter_million_tokens():
    """A context longer than any benchmark shape (the paper's largest fitting context is 236K tokens): the chunk
    cap holds every accumulator to 16K tokens, so the error does not grow with the length."""
    S = 250_007
    w = wl.custom(n_q_heads=8, n_kv_heads=1, head_dim=128, seq_len=S, seed=2500, outlier_channels=4)
    q, k, v = make(w)
    cache = gpu_cache_from(k, v)
    ocache = oracle_cache_from(k, v)
    assert_cache_bit_exact(cache, ocache, S)
    ref = oracle_attend(q, ocache, S, w.attn_scale)
    for variant in (0, 1):
        out = tq.tq_sdpa_int4_decode(cache, q.cuda(), S, w.attn_scale, variant=variant)
        torch.cuda.synchronize()
        max_abs, rel = assert_close(out, ref, f"S={S} variant={variant}")
        print(f"\nS={S} variant={variant}: max-abs {max_abs:.2e} rel-L2 {rel:.2e}")


@pytest.mark.parametrize("variant", [0, 1])
@pytest.mark.parametrize("shape", ["g8_d128_b4_kv2", "g2_d256_b4"])
def test_append_decode_with_per_sequence_lengths(shape, variant):
    """One decode step for a batch whose sequences have their own lengths (each counting its new token), contiguous
    and paged: stored bits equal the oracle's at every sequence's own last position, nothing else is touched, the
    result equals the oracle's over each sequence's tokens; one sequence has no cached token at all."""
    shapes = dict(g8_d128_b4_kv2=dict(batch=4, n_q_heads=16, n_kv_heads=2, head_dim=128, outlier_channels=4),
                  g2_d256_b4=dict(batch=4, n_q_heads=4, n_kv_heads=2, head_dim=256, attn_scale=1.0, qk_std=0.1))
    lens = [1500, 1, 2049, 321]                   # lengths INCLUDING the new token
    S, PT, max_blocks, n_pages = max(lens), 256, 9, 40
    w = wl.custom(seq_len=S, seed=1700, **shapes[shape])
    q, k, v = make(w)
    B, Hkv, d = w.batch, w.n_kv_heads, w.head_dim
    # sequence b's tokens are k[b, :, :lens[b]]; its new token is the last of them
    kn = torch.stack([k[b, :, lens[b] - 1:lens[b]] for b in range(B)]).contiguous()
    vn = torch.stack([v[b, :, lens[b] - 1:lens[b]] for b in range(B)]).contiguous()
    ocache = oracle_cache_from(k, v)
    lens_dev = torch.tensor(lens, dtype=torch.int32, device="cuda")
    cached = torch.tensor([n - 1 for n in lens], dtype=torch.int32, device="cuda")
    names = ("k_codes", "k_scale", "k_zero", "v_codes", "v_scale", "v_zero")
    for window in (0, 1, 2, 300):                 # (a window of one token: the append kernel runs first)
        ref = _oracle_window(q, ocache, lens, window if window > 0 else S, w.attn_scale)
        # ---- contiguous rows
        cache = tq.KVCache(B, Hkv, d, S + 3)
        for t in cache.tensors():
            t.view(torch.uint8).fill_(0xEE)
        tq.tq_quantize_kv(cache, k.cuda(), v.cuda(), 0)       # everything, then the last token of every sequence is
        for t in cache.tensors():                             # wiped again: the call under test has to write it
            for b in range(B):
                t.view(torch.uint8)[b, :, lens[b] - 1:] = 0xEE
        out = tq.tq_sdpa_int4_append_decode_varlen(cache, kn.cuda(), vn.cuda(), q.cuda(), lens_dev, S, w.attn_scale,
                                                   variant=variant, window=window)
        torch.cuda.synchronize()
        for name, g, o in zip(names, cache.tensors(), ocache):
            g = np16(g)
            for b in range(B):
                gb, ob = g[b, :, :lens[b]], o[b, :, :lens[b]]
                if gb.dtype == np.float16:
                    gb, ob = gb.view(np.uint16), ob.view(np.uint16)
                assert np.array_equal(gb, ob), f"{name} sequence {b}"
        for t in cache.tensors():
            for b in range(B):
                assert bool((t.view(torch.uint8)[b, :, lens[b]:] == 0xEE).all())
        assert_close(out, ref, f"{shape} append + decode, own lengths, window={window} variant={variant}")
        # ---- the same over pages in random order
        rng = np.random.default_rng(11)
        table = rng.permutation(n_pages)[:B * max_blocks].reshape(B, max_blocks).astype(np.int32)
        table_dev = torch.from_numpy(table).cuda()
        pool = tq.KVCache(n_pages, Hkv, d, PT)
        for t in pool.tensors():
            t.view(torch.uint8).fill_(0xEE)
        # fill every sequence up to its own cached length: one call per distinct length (positions 0, n_new tokens)
        for b in range(B):
            if lens[b] > 1:
                one = torch.from_numpy(table[b:b + 1]).cuda()
                tq.tq_quantize_kv_paged(pool, one, k[b:b + 1, :, :lens[b] - 1].contiguous().cuda(),
                                        v[b:b + 1, :, :lens[b] - 1].contiguous().cuda(),
                                        torch.zeros(1, dtype=torch.int32, device="cuda"))
        out = tq.tq_sdpa_int4_append_decode_paged(pool, table_dev, kn.cuda(), vn.cuda(), q.cuda(), lens_dev, S, w.attn_scale,
                                                  variant=variant, window=window)
        torch.cuda.synchronize()
        assert_close(out, ref, f"{shape} paged append + decode, window={window} variant={variant}")
        for name, t, o in zip(names, pool.tensors(), ocache):
            g = np16(t)
            for b in range(B):
                n = lens[b]
                got = np.concatenate([g[table[b, j]] for j in range((n + PT - 1) // PT)], axis=1)[:, :n]
                want = o[b, :, :n]
                if got.dtype == np.float16:
                    got, want = got.view(np.uint16), want.view(np.uint16)
                assert np.array_equal(got, want), f"paged {name} sequence {b}"
    del cached
    # two query tokens per sequence (the append kernel runs first): lengths count both new tokens
    if variant == 0:
        lens2 = [1500, 2, 2049, 321]
        q4 = _queries_for(w, 2)
        kn2 = torch.stack([k[b, :, lens2[b] - 2:lens2[b]] for b in range(B)]).contiguous()
        vn2 = torch.stack([v[b, :, lens2[b] - 2:lens2[b]] for b in range(B)]).contiguous()
        cache = tq.KVCache(B, Hkv, d, S + 3)
        tq.tq_quantize_kv(cache, k.cuda(), v.cuda(), 0)
        for t in cache.tensors():
            for b in range(B):
                t.view(torch.uint8)[b, :, lens2[b] - 2:] = 0xEE
        out = tq.tq_sdpa_int4_append_decode_varlen(cache, kn2.cuda(), vn2.cuda(), q4.cuda(),
                                                   torch.tensor(lens2, dtype=torch.int32, device="cuda"), S, w.attn_scale)
        torch.cuda.synchronize()
        assert_close(out, _oracle_causal(q4, ocache, lens2, w.attn_scale), f"{shape} append of two tokens, own lengths")


@pytest.mark.parametrize("shape", ["g8_d128", "g2_d256", "g16_d128", "g3_d128"])
def test_more_rows_than_blocks_are_packed_several_to_a_block(shape):
    """Batches whose (sequence, KV head) rows outnumber the compute units, every row a single chunk: 2, 4 or 8
    rows share a block (4, 2 or 1 waves each).  Lengths cover no full supertile, ragged tails, and more supertiles
    than a row has waves; the row count does not fill the last block; also with a window and several query tokens."""
    shapes = dict(g8_d128=dict(n_q_heads=16, n_kv_heads=2, head_dim=128, outlier_channels=4),
                  g2_d256=dict(n_q_heads=4, n_kv_heads=2, head_dim=256, attn_scale=1.0, qk_std=0.1),
                  g16_d128=dict(n_q_heads=16, n_kv_heads=1, head_dim=128),
                  g3_d128=dict(n_q_heads=6, n_kv_heads=2, head_dim=128))
    for batch in (131, 300, 700):                 # x 2 rows (x 2 parts at GQA 16): 4, 2 and 1 waves per row
        for S in (5, 100, 517):
            w = wl.custom(batch=batch, seq_len=S, seed=1800 + S + batch, **shapes[shape])
            q, k, v = make(w)
            cache = gpu_cache_from(k, v, capacity=S + 2)
            ocache = oracle_cache_from(k, v)
            assert tq.tq_decode_launches(cache, w.n_q_heads, S, w.attn_scale) == 1
            out = tq.tq_sdpa_int4_decode(cache, q.cuda(), S, w.attn_scale)
            torch.cuda.synchronize()
            assert_close(out, oracle_attend(q, ocache, S, w.attn_scale), f"{shape} batch={batch} S={S}")
            win = max(1, S // 2)
            out = tq.tq_sdpa_int4_decode(cache, q.cuda(), S, w.attn_scale, window=win)
            torch.cuda.synchronize()
            assert_close(out, _oracle_window(q, ocache, [S] * batch, win, w.attn_scale), f"{shape} batch={batch} S={S} window")
            if S >= 100 and batch == 300:
                q4 = _queries_for(w, 2)
                out = tq.tq_sdpa_int4_decode(cache, q4.cuda(), S, w.attn_scale)
                torch.cuda.synchronize()
                assert_close(out, _oracle_causal(q4, ocache, [S] * batch, w.attn_scale), f"{shape} batch={batch} S={S}, 2 queries")


@pytest.mark.parametrize("S", [1800, 2600])
def test_eighty_sequences_with_their_own_lengths_and_a_step(S):
    """640 (sequence, KV head) rows with their own lengths.  Up to 2048 tokens every row is one chunk of its own
    length, packed four to a block, and the decode kernel writes the output itself (no chunk plan, no merge kernel;
    the step appends with the append kernel); beyond that the device plans chunks whose slots share blocks and the
    merge kernel takes the step's token in.  Plain decode, a window, and the one-call step, against the oracle."""
    rng = np.random.default_rng(80)
    B = 80
    lens = [int(x) for x in rng.integers(1, S + 1, B)]
    lens[0], lens[1] = S, 1
    w = wl.custom(batch=B, n_q_heads=64, n_kv_heads=8, head_dim=128, seq_len=S, seed=1900, outlier_channels=4)
    q, k, v = make(w)
    cache = gpu_cache_from(k, v)
    ocache = oracle_cache_from(k, v)
    lens_dev = torch.tensor(lens, dtype=torch.int32, device="cuda")
    ref = _oracle_varlen(q, ocache, lens, w.attn_scale)
    out = tq.tq_sdpa_int4_decode_varlen(cache, q.cuda(), lens_dev, S, w.attn_scale)
    torch.cuda.synchronize()
    assert_close(out, ref, "80 sequences, own lengths")
    out = tq.tq_sdpa_int4_decode_varlen(cache, q.cuda(), lens_dev, S, w.attn_scale, window=300)
    torch.cuda.synchronize()
    assert_close(out, _oracle_window(q, ocache, lens, 300, w.attn_scale), "80 sequences, own lengths, window 300")
    # the step: wipe every sequence's last token, hand it over as the new one
    kn = torch.stack([k[b, :, lens[b] - 1:lens[b]] for b in range(B)]).contiguous()
    vn = torch.stack([v[b, :, lens[b] - 1:lens[b]] for b in range(B)]).contiguous()
    for t in cache.tensors():
        for b in range(B):
            t.view(torch.uint8)[b, :, lens[b] - 1] = 0xEE
    out = tq.tq_sdpa_int4_append_decode_varlen(cache, kn.cuda(), vn.cuda(), q.cuda(), lens_dev, S, w.attn_scale)
    torch.cuda.synchronize()
    assert_close(out, ref, "80 sequences, own lengths, append + decode")
    for name, g, o in zip(("k_codes", "k_scale", "k_zero", "v_codes", "v_scale", "v_zero"), cache.tensors(), ocache):
        g = np16(g)
        for b in range(B):
            gb, ob = g[b, :, :lens[b]], o[b, :, :lens[b]]
            if gb.dtype == np.float16:
                gb, ob = gb.view(np.uint16), ob.view(np.uint16)
            assert np.array_equal(gb, ob), f"{name} sequence {b}"


@pytest.mark.parametrize("B,Hq,Hkv", [(128, 32, 8), (172, 24, 4), (86, 48, 4), (32, 128, 8)])
def test_merge_of_thousands_of_outputs_runs_one_block_per_kv_head(B, Hq, Hkv):
    """From 768 (sequence, query head) outputs of 128 elements on (here: thousands), with four or more query heads
    to a KV head, the chunk merge (Eq. 6) folds four heads of a group in one block, 4 or 16 chunks at a time, and
    in a step takes the new token in as the last chunk: groups of 4, 6, 12 and 16 heads, chunk counts from 1 to 7 per sequence, with the
    chunk count asked for and with the device's plan, plain, windowed, two query tokens, and the one-call step."""
    S = 700
    rng = np.random.default_rng(B + Hq)
    lens = [int(x) for x in rng.integers(1, S + 1, B)]
    lens[0], lens[1], lens[2] = S, 1, 101
    w = wl.custom(batch=B, n_q_heads=Hq, n_kv_heads=Hkv, head_dim=128, seq_len=S, seed=2700 + B, outlier_channels=4)
    q, k, v = make(w)
    cache = gpu_cache_from(k, v)
    ocache = oracle_cache_from(k, v)
    lens_dev = torch.tensor(lens, dtype=torch.int32, device="cuda")
    ref = _oracle_varlen(q, ocache, lens, w.attn_scale)
    for n_splits, variant in ((7, 0), (2, 0), (22, 0), (5, 1), (0, 1)):      # (22 chunks: two heads per thread, else four)
        out = tq.tq_sdpa_int4_decode_varlen(cache, q.cuda(), lens_dev, S, w.attn_scale, n_splits=n_splits, variant=variant)
        torch.cuda.synchronize()
        assert_close(out, ref, f"own lengths, {n_splits} chunks, variant {variant}")
    out = tq.tq_sdpa_int4_decode_varlen(cache, q.cuda(), lens_dev, S, w.attn_scale, n_splits=5, window=90)
    torch.cuda.synchronize()
    assert_close(out, _oracle_window(q, ocache, lens, 90, w.attn_scale), "own lengths, 5 chunks, window 90")
    out = tq.tq_sdpa_int4_decode(cache, q.cuda(), S, w.attn_scale, n_splits=3)
    torch.cuda.synchronize()
    assert_close(out, _oracle_varlen(q, ocache, [S] * B, w.attn_scale), "common length, 3 chunks")
    lens2 = [max(2, n) for n in lens]
    q2 = _queries_for(w, 2)
    out = tq.tq_sdpa_int4_decode_varlen(cache, q2.cuda(), torch.tensor(lens2, dtype=torch.int32, device="cuda"), S,
                                        w.attn_scale, n_splits=4)
    torch.cuda.synchronize()
    assert_close(out, _oracle_causal(q2, ocache, lens2, w.attn_scale), "own lengths, 4 chunks, 2 query tokens")
    # the step: wipe every sequence's last token, hand it over as the new one
    kn = torch.stack([k[b, :, lens[b] - 1:lens[b]] for b in range(B)]).contiguous()
    vn = torch.stack([v[b, :, lens[b] - 1:lens[b]] for b in range(B)]).contiguous()
    for t in cache.tensors():
        for b in range(B):
            t.view(torch.uint8)[b, :, lens[b] - 1] = 0xEE
    out = tq.tq_sdpa_int4_append_decode_varlen(cache, kn.cuda(), vn.cuda(), q.cuda(), lens_dev, S, w.attn_scale, n_splits=6)
    torch.cuda.synchronize()
    assert_close(out, ref, "own lengths, 6 chunks, append + decode")
    for name, g, o in zip(("k_codes", "k_scale", "k_zero", "v_codes", "v_scale", "v_zero"), cache.tensors(), ocache):
        g = np16(g)
        for b in range(B):
            gb, ob = g[b, :, :lens[b]], o[b, :, :lens[b]]
            if gb.dtype == np.float16:
                gb, ob = gb.view(np.uint16), ob.view(np.uint16)
            assert np.array_equal(gb, ob), f"{name} sequence {b}"
    # ... and the step at a common length: the last token of every sequence again
    for t in cache.tensors():
        t.view(torch.uint8)[:, :, S - 1] = 0xEE
    out = tq.tq_sdpa_int4_append_decode(cache, k[:, :, S - 1:S].contiguous().cuda(), v[:, :, S - 1:S].contiguous().cuda(),
                                        q.cuda(), S, w.attn_scale, n_splits=3)
    torch.cuda.synchronize()
    assert_close(out, _oracle_varlen(q, ocache, [S] * B, w.attn_scale), "common length, 3 chunks, append + decode")
    assert_cache_bit_exact(cache, ocache, S)


def test_one_long_sequence_among_short_ones():
    """24 sequences, one of 20000 tokens and the others of at most 300: the device's plan gives the long one some
    thirty chunks and the others one each, and the grouped merge kernel (1536 outputs) folds the long one's 16 at
    a time.  Decode and the one-call step, against the oracle."""
    B, S = 24, 20000
    rng = np.random.default_rng(24)
    lens = [int(x) for x in rng.integers(1, 301, B)]
    lens[5] = S
    w = wl.custom(batch=B, n_q_heads=64, n_kv_heads=8, head_dim=128, seq_len=S, seed=2800, outlier_channels=4)
    q, k, v = make(w)
    cache = gpu_cache_from(k, v)
    ocache = oracle_cache_from(k, v)
    lens_dev = torch.tensor(lens, dtype=torch.int32, device="cuda")
    ref = _oracle_varlen(q, ocache, lens, w.attn_scale)
    out = tq.tq_sdpa_int4_decode_varlen(cache, q.cuda(), lens_dev, S, w.attn_scale)
    torch.cuda.synchronize()
    assert_close(out, ref, "one long sequence among short ones")
    kn = torch.stack([k[b, :, lens[b] - 1:lens[b]] for b in range(B)]).contiguous()
    vn = torch.stack([v[b, :, lens[b] - 1:lens[b]] for b in range(B)]).contiguous()
    for t in cache.tensors():
        for b in range(B):
            t.view(torch.uint8)[b, :, lens[b] - 1] = 0xEE
    out = tq.tq_sdpa_int4_append_decode_varlen(cache, kn.cuda(), vn.cuda(), q.cuda(), lens_dev, S, w.attn_scale)
    torch.cuda.synchronize()
    assert_close(out, ref, "one long sequence among short ones, append + decode")
    assert_cache_bit_exact(cache, ocache, S)
