"""Pins for the oracle's attention (CPU only): facts the mathematics fixes, a brute force with
exact rational scores, a library-routine cross-check, and Alg. 1 + Eq. 6 == the definition."""
import math
from fractions import Fraction

import numpy as np
import pytest
from scipy.special import softmax

import oracle


def _rand_case(rng, B=1, Hq=4, Hkv=2, S=37, d=64, std=1.0):
    q = (rng.standard_normal((B, Hq, d)) * std).astype(np.float16)
    k = (rng.standard_normal((B, Hkv, S, d)) * std).astype(np.float16)
    v = rng.standard_normal((B, Hkv, S, d)).astype(np.float16)
    return q, k, v


def _quantize_cache(k, v):
    kc, ks, kz = oracle.quantize(k)
    vc, vs, vz = oracle.quantize(v)
    return kc, ks, kz, vc, vs, vz


def test_single_token_returns_its_dequantised_value():
    rng = np.random.default_rng(0)
    q, k, v = _rand_case(rng, Hq=8, Hkv=2, S=1, d=128)
    cache = _quantize_cache(k, v)
    out = oracle.attend_packed(q, *cache, seq_len=1, alpha=0.3)
    vh = oracle.dequantize(*cache[3:])
    for h in range(8):
        assert np.array_equal(out[0, h], vh[0, h // 4, 0])


def test_identical_keys_and_zero_query_give_mean_of_values():
    rng = np.random.default_rng(1)
    q, k, v = _rand_case(rng, Hq=2, Hkv=1, S=50, d=64)
    k[:] = k[:, :, :1]                                       # all keys equal
    cache = _quantize_cache(k, v)
    vh = oracle.dequantize(*cache[3:])
    out = oracle.attend_packed(q, *cache, seq_len=50, alpha=0.7)
    assert np.allclose(out[0, 0], vh[0, 0].mean(0), rtol=0, atol=1e-13)
    assert np.allclose(out[0, 1], vh[0, 0].mean(0), rtol=0, atol=1e-13)
    _, k2, _ = _rand_case(rng, Hq=2, Hkv=1, S=50, d=64)
    cache2 = _quantize_cache(k2, v)
    out0 = oracle.attend_packed(np.zeros_like(q), *cache2, seq_len=50, alpha=0.7)
    assert np.allclose(out0[0, 0], vh[0, 0].mean(0), rtol=0, atol=1e-13)


def test_seq_len_limits_the_tokens_attended():
    rng = np.random.default_rng(2)
    q, k, v = _rand_case(rng, S=40)
    cache = _quantize_cache(k, v)
    short = tuple(a[:, :, :23] for a in cache)
    a = oracle.attend_packed(q, *cache, seq_len=23, alpha=0.2)       # capacity 40, 23 valid
    b = oracle.attend_packed(q, *short, seq_len=23, alpha=0.2)       # capacity 23
    assert np.array_equal(a, b)


def test_score_shift_invariance():
    rng = np.random.default_rng(3)
    q, k, v = _rand_case(rng)
    K, V = k.astype(np.float64), v.astype(np.float64)
    base = oracle.attend_dense(q, K, V, 0.125)
    for bias in (-40.0, 3.5, 700.0):
        assert np.allclose(oracle.attend_dense(q, K, V, 0.125, score_bias=bias), base, rtol=0, atol=1e-12)
    # the same fact through the keys: adding c*q/|q|^2 to every key adds c to every score of that head
    Hq, Hkv = q.shape[1], k.shape[1]
    q1 = q[:, ::Hq // Hkv]                                   # one head per KV head
    qq = q1.astype(np.float64)
    shift = 5.0 * qq / (qq ** 2).sum(-1, keepdims=True)
    K2 = K + shift[:, :, None, :]
    a = oracle.attend_dense(q1, K, V, 1.0)
    b = oracle.attend_dense(q1, K2, V, 1.0)
    assert np.allclose(a, b, rtol=0, atol=1e-10)


def test_large_scale_selects_argmax_value():
    rng = np.random.default_rng(4)
    q, k, v = _rand_case(rng, Hq=2, Hkv=1, S=64, d=32)
    K, V = k.astype(np.float64), v.astype(np.float64)
    out = oracle.attend_dense(q, K, V, 1e4)
    for h in range(2):
        i = int(np.argmax(K[0, 0] @ q[0, h].astype(np.float64)))
        assert np.allclose(out[0, h], V[0, 0, i], rtol=0, atol=1e-12)


def test_gqa_mapping_and_equal_queries():
    rng = np.random.default_rng(5)
    q, k, v = _rand_case(rng, Hq=6, Hkv=3, S=20, d=32)
    q[0, 1] = q[0, 0]                                        # heads 0,1 share KV head 0
    q[0, 2] = q[0, 0]                                        # head 2 uses KV head 1
    K, V = k.astype(np.float64), v.astype(np.float64)
    out = oracle.attend_dense(q, K, V, 0.2)
    assert np.array_equal(out[0, 0], out[0, 1])
    assert not np.allclose(out[0, 0], out[0, 2])
    # head h must equal a single-head problem on KV head h // G  (G = 2)
    for h in range(6):
        solo = oracle.attend_dense(q[:, h:h + 1], K[:, h // 2:h // 2 + 1], V[:, h // 2:h // 2 + 1], 0.2)
        assert np.array_equal(solo[0, 0], out[0, h])


def test_token_permutation_invariance():
    rng = np.random.default_rng(6)
    q, k, v = _rand_case(rng, S=33)
    cache = _quantize_cache(k, v)
    perm = rng.permutation(33)
    pc = tuple(a[:, :, perm] for a in cache)
    a = oracle.attend_packed(q, *cache, seq_len=33, alpha=0.1)
    b = oracle.attend_packed(q, *pc, seq_len=33, alpha=0.1)
    assert np.allclose(a, b, rtol=0, atol=1e-13)


def test_matches_library_softmax_and_matmul():
    rng = np.random.default_rng(7)
    q, k, v = _rand_case(rng, B=2, Hq=8, Hkv=2, S=129, d=128)
    cache = _quantize_cache(k, v)
    Kh, Vh = oracle.dequantize(*cache[:3]), oracle.dequantize(*cache[3:])
    G = 4
    Kx, Vx = np.repeat(Kh, G, axis=1), np.repeat(Vh, G, axis=1)            # head h -> kv h // G
    scores = 0.0884 * np.einsum("bhd,bhsd->bhs", q.astype(np.float64), Kx)
    ref = np.einsum("bhs,bhsd->bhd", softmax(scores, axis=-1), Vx)
    got = oracle.attend_packed(q, *cache, seq_len=129, alpha=0.0884)
    assert np.allclose(got, ref, rtol=1e-12, atol=1e-13)
    assert np.allclose(oracle.attend_dense(q, Kh, Vh, 0.0884), ref, rtol=1e-12, atol=1e-13)


def _brute_force(q, codes_k, sk, zk, codes_v, sv, zv, alpha, G):
    """Exact rational scores; weights as 1 / sum_j exp(a_j - a_i) (no max subtraction)."""
    def elems(codes, s, z):                                  # -> Fractions, own nibble split
        out = []
        for j in range(2 * len(codes)):
            byte = int(codes[j // 2])
            c = (byte >> 4) if j % 2 else (byte & 15)
            out.append((Fraction(c) - Fraction(float(z[j // 32]))) * Fraction(float(s[j // 32])))
        return out
    B, Hq, d = q.shape
    S = codes_k.shape[2]
    res = np.zeros((B, Hq, d))
    for b in range(B):
        for h in range(Hq):
            kv = h // G
            qf = [Fraction(float(x)) for x in q[b, h]]
            K = [elems(codes_k[b, kv, i], sk[b, kv, i], zk[b, kv, i]) for i in range(S)]
            V = [elems(codes_v[b, kv, i], sv[b, kv, i], zv[b, kv, i]) for i in range(S)]
            a = [float(Fraction(alpha) * sum(x * y for x, y in zip(qf, K[i]))) for i in range(S)]
            w = [1.0 / math.fsum(math.exp(a[j] - a[i]) for j in range(S)) for i in range(S)]
            for j in range(d):
                res[b, h, j] = math.fsum(w[i] * float(V[i][j]) for i in range(S))
    return res


@pytest.mark.parametrize("S,G", [(1, 1), (2, 2), (3, 1), (4, 2)])
def test_brute_force_tiny(S, G):
    rng = np.random.default_rng(10 + S)
    q, k, v = _rand_case(rng, B=1, Hq=2 * G, Hkv=2, S=S, d=32)
    cache = _quantize_cache(k, v)
    got = oracle.attend_packed(q, *cache, seq_len=S, alpha=0.25)
    ref = _brute_force(q, *cache, alpha=0.25, G=G)
    assert np.allclose(got, ref, rtol=1e-13, atol=1e-14)


def test_alg1_plus_eq6_equals_definition():
    rng = np.random.default_rng(8)
    q, k, v = _rand_case(rng, B=2, Hq=4, Hkv=2, S=300, d=64)
    cache = _quantize_cache(k, v)
    Kh, Vh = oracle.dequantize(*cache[:3]), oracle.dequantize(*cache[3:])
    ref = oracle.attend_dense(q, Kh, Vh, 0.125)
    chunkings = [[0, 300], [0, 1, 300], [0, 128, 256, 300], list(range(0, 300, 7)) + [300]]
    for _ in range(4):
        cuts = np.sort(rng.choice(np.arange(1, 300), size=rng.integers(1, 20), replace=False))
        chunkings.append([0] + cuts.tolist() + [300])
    for b in chunkings:
        got = oracle.attend_alg1_eq6(q, Kh, Vh, 0.125, b)
        assert np.max(np.abs(got - ref)) <= 1e-12, b
    # ceil(S/512)-style chunking of Sec. 3.2 on a longer sequence
    q, k, v = _rand_case(rng, B=1, Hq=2, Hkv=1, S=1300, d=32)
    K, V = k.astype(np.float64), v.astype(np.float64)
    b = list(range(0, 1300, 512)) + [1300]
    assert np.max(np.abs(oracle.attend_alg1_eq6(q, K, V, 0.3, b) - oracle.attend_dense(q, K, V, 0.3))) <= 1e-12


def test_quality_level_is_in_the_papers_ballpark():
    # soft sanity only (real-model numbers of Table 1 are not reproducible here):
    # N(0,1) data at int4 g=32 has cosine similarity ~ 1/sqrt(1 + s^2/12) ~ 0.997
    rng = np.random.default_rng(9)
    x = rng.standard_normal((2048, 128)).astype(np.float16)
    xh = oracle.dequantize(*oracle.quantize(x))
    xf = x.astype(np.float64)
    cos = (xf * xh).sum() / math.sqrt((xf ** 2).sum() * (xh ** 2).sum())
    assert 0.994 < cos < 0.9995


@pytest.mark.parametrize("g", [64, 128])
def test_larger_groups_only_change_the_dequantised_values(g):
    """At group size 64 / 128 the packed path reads the scale and zero-point of group j // g for element j and is
    otherwise the same definition: it equals the dense path over numpy's own (code - z) * s with the metadata
    repeated g times (an indexing slip in the packed path would break it), and one cached token returns that
    token's dequantised value vector."""
    rng = np.random.default_rng(40 + g)
    q, k, v = _rand_case(rng, B=2, Hq=6, Hkv=3, S=29, d=256)
    kc, ks, kz = oracle.quantize(k, group=g)
    vc, vs, vz = oracle.quantize(v, group=g)
    assert ks.shape[-1] == 256 // g

    def dense(codes, sc, zp):
        c = np.empty(codes.shape[:-1] + (256,), np.float64)
        c[..., 0::2] = codes & 0xF
        c[..., 1::2] = codes >> 4
        return (c - np.repeat(zp.astype(np.float64), g, -1)) * np.repeat(sc.astype(np.float64), g, -1)

    K, V = dense(kc, ks, kz), dense(vc, vs, vz)
    assert np.array_equal(oracle.dequantize(kc, ks, kz), K) and np.array_equal(oracle.dequantize(vc, vs, vz), V)
    out = oracle.attend_packed(q, kc, ks, kz, vc, vs, vz, seq_len=29, alpha=0.2)
    assert np.allclose(out, oracle.attend_dense(q, K, V, 0.2), rtol=0, atol=1e-13)
    one = oracle.attend_packed(q, kc, ks, kz, vc, vs, vz, seq_len=1, alpha=0.2)
    for h in range(6):
        assert np.array_equal(one[:, h], V[:, h // 2, 0])
