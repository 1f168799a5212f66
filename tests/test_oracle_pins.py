"""Pins for the fp64 CPU oracle: it is checked against things other than itself.

The paper prints no worked numeric example, so the pins are: a hand-derived
example (tests/golden/worked_example.txt), closed forms, invariants of softmax
attention, brute force in exact-sum Python, library routines (scipy softmax /
logsumexp), and the decomposition identity (Eq. 5) at every split point.
Each pin targets a class of mistakes: dropped scale, wrong log base, transposed
or mis-strided operand, wrong GQA head map, wrong block/sequence lookup in a
tree, off-by-one in ragged suffix ranges, a merge with the wrong weights.
"""
import math
import os

import numpy as np
import pytest
import scipy.special

import oracle
from paper_2402_05099_amd import workloads as wl

TOL = 1e-12


def bits(x):
    x = np.asarray(x, dtype=np.float32)
    b = wl.f32_to_bf16_bits(x)
    assert np.array_equal(wl.bf16_bits_to_f32(b), x), "test value not bf16-exact"
    return b.reshape(x.shape)


def grid_values(rng, shape, lo=-16, hi=16, step=0.125):
    """random multiples of `step` (bf16-exact, sums of two stay exact)"""
    return (rng.integers(lo, hi + 1, size=shape) * step).astype(np.float32)


def single(q, K, V, scale, Hkv=1):
    """one shared block, no suffix. q [B,Hq,D], K/V [P,Hkv,D] float arrays (bf16-exact)."""
    B = q.shape[0]
    P = K.shape[0]
    lv = [(bits(K), bits(V), np.array([0, P], np.int32), np.array([0, B], np.int32))]
    return oracle.attention_arrays(bits(q), Hkv, lv, scale=scale)


def parse_golden():
    path = os.path.join(os.path.dirname(__file__), "golden", "worked_example.txt")
    out = {}
    for line in open(path):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        k, *v = line.split()
        out[k] = np.array([float(t) for t in v])
    return out


def test_golden_worked_example_full_parts_and_merge():
    g = parse_golden()
    scale = math.log(g["scale_is_ln"][0])
    q = g["q"].reshape(1, 1, 4)
    K = np.stack([g["k1"], g["k2"], g["k3"]]).reshape(3, 1, 4)
    V = np.stack([g["v1"], g["v2"], g["v3"]]).reshape(3, 1, 4)
    # full attention over prefix(k1,k2) || suffix(k3) stored the way a workload stores them
    lv = [(bits(K[:2]), bits(V[:2]), np.array([0, 2], np.int32), np.array([0, 1], np.int32))]
    O, L = oracle.attention_arrays(bits(q), 1, lv, bits(K[2:]), bits(V[2:]), [0], [1], scale)
    assert np.allclose(O[0, 0], g["O"], rtol=0, atol=TOL)
    assert abs(L[0, 0] - math.log(g["LSE_is_ln"][0])) < TOL
    Op, Lp = oracle.attention_arrays(bits(q), 1, lv, scale=scale)
    Os, Ls = oracle.attention_arrays(bits(q), 1, [], bits(K[2:]), bits(V[2:]), [0], [1], scale)
    assert np.allclose(Op[0, 0], g["O_p"], rtol=0, atol=TOL)
    assert abs(Lp[0, 0] - math.log(g["LSE_p_is_ln"][0])) < TOL
    assert np.allclose(Os[0, 0], g["O_s"], rtol=0, atol=TOL)
    assert abs(Ls[0, 0] - math.log(g["LSE_s_is_ln"][0])) < TOL
    # merge of the hand-derived parts gives the hand-derived whole
    Om, Lm = oracle.merge([g["O_p"][None], g["O_s"][None]],
                          [np.log(g["LSE_p_is_ln"]), np.log(g["LSE_s_is_ln"])])
    assert np.allclose(Om[0], g["O"], rtol=0, atol=TOL)
    assert abs(Lm[0] - math.log(7.0)) < TOL


def test_one_key_returns_its_value_and_score():
    rng = np.random.default_rng(0)
    q = grid_values(rng, (3, 2, 8))
    K = grid_values(rng, (1, 2, 8))
    V = grid_values(rng, (1, 2, 8))
    scale = 0.37
    O, L = single(q, K, V, scale, Hkv=2)
    for b in range(3):
        for h in range(2):
            assert np.array_equal(O[b, h], V[0, h].astype(np.float64))
            s = float(np.dot(q[b, h].astype(np.float64), K[0, h].astype(np.float64))) * scale
            assert abs(L[b, h] - s) <= TOL * max(1.0, abs(s))


def test_two_keys_closed_form_sigmoid():
    rng = np.random.default_rng(1)
    D = 16
    q = grid_values(rng, (1, 1, D), -8, 8)
    K = grid_values(rng, (2, 1, D), -8, 8)
    V = grid_values(rng, (2, 1, D))
    scale = 1.0 / math.sqrt(D)
    O, L = single(q, K, V, scale)
    s = (K[:, 0].astype(np.float64) @ q[0, 0].astype(np.float64)) * scale
    sig = 1.0 / (1.0 + math.exp(-(s[0] - s[1])))
    want = sig * V[0, 0].astype(np.float64) + (1.0 - sig) * V[1, 0].astype(np.float64)
    assert np.allclose(O[0, 0], want, rtol=0, atol=1e-12)
    assert abs(L[0, 0] - (max(s) + math.log1p(math.exp(-abs(s[0] - s[1]))))) < 1e-12


def test_equal_scores_give_mean_of_values():
    rng = np.random.default_rng(2)
    N, D = 37, 8
    V = grid_values(rng, (N, 1, D))
    # (a) zero query: every score is 0
    O, L = single(np.zeros((1, 1, D), np.float32), grid_values(rng, (N, 1, D)), V, 0.5)
    assert np.allclose(O[0, 0], V[:, 0].astype(np.float64).mean(0), rtol=0, atol=TOL)
    assert abs(L[0, 0] - math.log(N)) < TOL
    # (b) identical keys: every score is the same s
    q = grid_values(rng, (1, 1, D), -4, 4)
    k = grid_values(rng, (1, 1, D), -4, 4)
    O, L = single(q, np.repeat(k, N, axis=0), V, 0.25)
    s = float(np.dot(q[0, 0].astype(np.float64), k[0, 0].astype(np.float64))) * 0.25
    assert np.allclose(O[0, 0], V[:, 0].astype(np.float64).mean(0), rtol=0, atol=1e-12)
    assert abs(L[0, 0] - (s + math.log(N))) < 1e-12


def test_constant_values_and_convexity():
    rng = np.random.default_rng(3)
    N, D = 50, 8
    q = grid_values(rng, (2, 1, D), -8, 8)
    K = grid_values(rng, (N, 1, D), -8, 8)
    c = grid_values(rng, (1, 1, D))
    O, _ = single(q, K, np.repeat(c, N, axis=0), 0.3)
    assert np.allclose(O, np.broadcast_to(c.astype(np.float64), O.shape), rtol=0, atol=1e-12)
    V = grid_values(rng, (N, 1, D))
    O, _ = single(q, K, V, 0.3)
    assert np.all(O <= V[:, 0].max(0) + 1e-12) and np.all(O >= V[:, 0].min(0) - 1e-12)


def test_shift_permutation_duplication_invariants():
    rng = np.random.default_rng(4)
    N, D = 41, 8
    scale = 0.125
    q = grid_values(rng, (2, 1, D), -8, 8)
    K = grid_values(rng, (N, 1, D), -8, 8)
    V = grid_values(rng, (N, 1, D))
    O0, L0 = single(q, K, V, scale)
    # shift every key by u: scores move by scale * q.u, O unchanged
    u = grid_values(rng, (1, 1, D), -8, 8)
    O1, L1 = single(q, K + u, V, scale)
    shift = (q[:, 0].astype(np.float64) @ u[0, 0].astype(np.float64)) * scale
    assert np.allclose(O1, O0, rtol=0, atol=1e-11)
    assert np.allclose(L1[:, 0], L0[:, 0] + shift, rtol=0, atol=1e-11)
    # permute (K,V) rows together
    p = rng.permutation(N)
    O2, L2 = single(q, K[p], V[p], scale)
    assert np.allclose(O2, O0, rtol=0, atol=1e-12) and np.allclose(L2, L0, rtol=0, atol=1e-12)
    # duplicate the key/value list
    O3, L3 = single(q, np.concatenate([K, K]), np.concatenate([V, V]), scale)
    assert np.allclose(O3, O0, rtol=0, atol=1e-12)
    assert np.allclose(L3, L0 + math.log(2.0), rtol=0, atol=1e-12)
    # scale acts on scores only: halving scale and doubling q is the same
    O4, L4 = single(2 * q, K, V, scale / 2)
    assert np.allclose(O4, O0, rtol=0, atol=1e-12) and np.allclose(L4, L0, rtol=0, atol=1e-12)


def _widen(a):
    return wl.bf16_bits_to_f32(a).astype(np.float64)


def brute_force(w, b, h):
    """Pure-Python exact-sum attention without max subtraction (tiny inputs only)."""
    G = w.Hq // w.Hkv
    kvh = h // G
    q = _widen(w.Q[b, h]).tolist()
    rows = []
    for li, r0, r1 in w.kv_rows_of(b):
        for r in range(r0, r1):
            rows.append((_widen(w.levels[li].K[r, kvh]).tolist(), _widen(w.levels[li].V[r, kvh]).tolist()))
    for r in range(int(w.offsets[b]), int(w.offsets[b]) + int(w.lengths[b])):
        rows.append((_widen(w.Ks[r, kvh]).tolist(), _widen(w.Vs[r, kvh]).tolist()))
    e = [math.exp(math.fsum(qi * ki for qi, ki in zip(q, k)) * w.scale) for k, _ in rows]
    den = math.fsum(e)
    O = [math.fsum(ei * v[d] for ei, (_, v) in zip(e, rows)) / den for d in range(w.D)]
    return np.array(O), math.log(den)


def test_brute_force_config1():
    w = wl.config(1)
    O, L = oracle.attention(w)
    for b in range(w.B):
        for h in range(w.Hq):
            Ob, Lb = brute_force(w, b, h)
            assert np.allclose(O[b, h], Ob, rtol=0, atol=1e-12)
            assert abs(L[b, h] - Lb) < 1e-12


def test_brute_force_ragged_gqa_tree_tiny():
    w = wl.make_workload("t", 77, 7, 6, 2, 16, [(1, 5, 7), (2, 3, 3)], 0, 4)
    assert w.lengths.min() == 0  # the seed gives at least one empty suffix
    O, L = oracle.attention(w)
    for b in range(w.B):
        for h in range(w.Hq):
            Ob, Lb = brute_force(w, b, h)
            assert np.allclose(O[b, h], Ob, rtol=0, atol=1e-12)
            assert abs(L[b, h] - Lb) < 1e-12


def library_attention(w, b):
    """Textbook softmax(QK^T * scale) V via scipy, on physically concatenated K/V. Returns [Hq,D], [Hq]."""
    G = w.Hq // w.Hkv
    Kc = [_widen(w.levels[li].K[r0:r1]) for li, r0, r1 in w.kv_rows_of(b)]
    Vc = [_widen(w.levels[li].V[r0:r1]) for li, r0, r1 in w.kv_rows_of(b)]
    o, n = int(w.offsets[b]), int(w.lengths[b])
    Kc.append(_widen(w.Ks[o:o + n]))
    Vc.append(_widen(w.Vs[o:o + n]))
    K = np.concatenate(Kc)  # [N,Hkv,D]
    V = np.concatenate(Vc)
    K = np.repeat(K, G, axis=1)  # explicit head repetition -> MHA
    V = np.repeat(V, G, axis=1)
    q = _widen(w.Q[b])  # [Hq,D]
    S = np.einsum("hd,nhd->hn", q, K) * w.scale
    Pm = scipy.special.softmax(S, axis=1)
    return np.einsum("hn,nhd->hd", Pm, V), scipy.special.logsumexp(S, axis=1)


@pytest.mark.parametrize("idx", [1, 2, 3, 4, 5, 6])
def test_library_softmax_on_scaled_down_configs(idx):
    """covers MHA, ragged suffixes, GQA-by-repetition (idx 4) and the tree by physical concatenation (idx 5)"""
    w = wl.scaled_down(idx)
    seqs = sorted(set([0, w.B // 2, w.B - 1, int(np.argmin(w.lengths)), int(np.argmax(w.lengths))]))
    O, L = oracle.attention(w, seqs=seqs)
    for i, b in enumerate(seqs):
        Ob, Lb = library_attention(w, b)
        assert np.allclose(O[i], Ob, rtol=0, atol=1e-12)
        assert np.allclose(L[i], Lb, rtol=0, atol=1e-12)


def test_gqa_equals_mha_with_repeated_kv_heads():
    w = wl.scaled_down(4)
    G = w.G
    lv = w.levels[0]
    rep = [(np.repeat(lv.K, G, axis=1), np.repeat(lv.V, G, axis=1), lv.kv_off, lv.seq_off)]
    O1, L1 = oracle.attention_arrays(w.Q, w.Hq, rep, np.repeat(w.Ks, G, axis=1), np.repeat(w.Vs, G, axis=1),
                                     w.offsets, w.lengths, w.scale)
    O0, L0 = oracle.attention(w)
    assert np.array_equal(O0, O1) and np.array_equal(L0, L1)


def test_seq_subset_matches_full():
    w = wl.scaled_down(5)
    O, L = oracle.attention(w)
    seqs = [5, 0, w.B - 1, 30]
    Os, Ls = oracle.attention(w, seqs=seqs)
    assert np.array_equal(Os, O[seqs]) and np.array_equal(Ls, L[seqs])


def test_decomposition_identity_every_split_point():
    """Eq. 5: merge(part(K1), part(K2)) == full(K1 || K2) for every split, including empty sides."""
    rng = np.random.default_rng(6)
    N, D, B, H = 13, 16, 3, 2
    Q = wl.normal_bf16(6, 0, (B, H, D))
    K = wl.normal_bf16(6, 1, (N, H, D))
    V = wl.normal_bf16(6, 2, (N, H, D))
    scale = 1 / math.sqrt(D)
    whole = [(K, V, np.array([0, N], np.int32), np.array([0, B], np.int32))]
    Of, Lf = oracle.attention_arrays(Q, H, whole, scale=scale)
    for s in range(N + 1):
        a = [(K[:s], V[:s], np.array([0, s], np.int32), np.array([0, B], np.int32))]
        b = [(K[s:], V[s:], np.array([0, N - s], np.int32), np.array([0, B], np.int32))]
        Oa, La = oracle.attention_arrays(Q, H, a, scale=scale)
        Ob, Lb = oracle.attention_arrays(Q, H, b, scale=scale)
        if s == 0:
            assert np.all(Oa == 0) and np.all(np.isneginf(La))
        Om, Lm = oracle.merge([Oa, Ob], [La, Lb])
        assert np.allclose(Om, Of, rtol=0, atol=1e-12), s
        assert np.allclose(Lm, Lf, rtol=0, atol=1e-12), s
    # the same split expressed as shared block + per-sequence suffix (each sequence gets its own copy)
    s = 5
    Ks = np.concatenate([K[s:]] * B)
    Vs = np.concatenate([V[s:]] * B)
    off = np.arange(B, dtype=np.int32) * (N - s)
    ln = np.full(B, N - s, np.int32)
    a = [(K[:s], V[:s], np.array([0, s], np.int32), np.array([0, B], np.int32))]
    O2, L2 = oracle.attention_arrays(Q, H, a, Ks, Vs, off, ln, scale)
    assert np.allclose(O2, Of, rtol=0, atol=1e-12) and np.allclose(L2, Lf, rtol=0, atol=1e-12)


def test_tree_three_way_merge_equals_full():
    w = wl.scaled_down(5)
    Of, Lf = oracle.attention(w)
    parts = [oracle.attention(w, levels=[0], suffix=False),
             oracle.attention(w, levels=[1], suffix=False),
             oracle.attention(w, levels=[], suffix=True)]
    Om, Lm = oracle.merge([p[0] for p in parts], [p[1] for p in parts])
    assert np.allclose(Om, Of, rtol=0, atol=1e-12)
    assert np.allclose(Lm, Lf, rtol=0, atol=1e-12)


def sigmoid_two_way_combine(out1, lse1, out2, lse2):
    """Two parts merged through the logistic function, a form of Eq. 5 derived independently of the oracle's code: the
    weight of part 1 is e^{lse1} / (e^{lse1} + e^{lse2}) = 1 / (1 + e^{lse2 - lse1}), that of part 2 its complement."""
    with np.errstate(over="ignore"):
        w1 = 1.0 / (1.0 + np.exp(lse2 - lse1))
    return out1 * w1[..., None] + out2 * (1.0 - w1)[..., None]


def test_merge_against_two_way_combine_and_nesting():
    rng = np.random.default_rng(7)
    rows, D = 29, 8
    Os = [rng.standard_normal((rows, D)) for _ in range(4)]
    Ls = [rng.standard_normal(rows) * 5 for _ in range(4)]
    O2, L2 = oracle.merge(Os[:2], Ls[:2])
    assert np.allclose(O2, sigmoid_two_way_combine(Os[0], Ls[0], Os[1], Ls[1]), rtol=0, atol=1e-13)
    assert np.allclose(L2, np.logaddexp(Ls[0], Ls[1]), rtol=0, atol=1e-13)
    # Eq. 5 literally (no max subtraction) on moderate LSEs
    w = [np.exp(l) for l in Ls]
    lit = sum(o * wi[:, None] for o, wi in zip(Os, w)) / sum(w)[:, None]
    O4, L4 = oracle.merge(Os, Ls)
    assert np.allclose(O4, lit, rtol=1e-12, atol=1e-12)
    assert np.allclose(L4, scipy.special.logsumexp(np.stack(Ls), axis=0), rtol=0, atol=1e-12)
    # nesting and order independence
    O12, L12 = oracle.merge(Os[:2], Ls[:2])
    O123, L123 = oracle.merge([O12, Os[2]], [L12, Ls[2]])
    On, Ln = oracle.merge([O123, Os[3]], [L123, Ls[3]])
    assert np.allclose(On, O4, rtol=0, atol=1e-12) and np.allclose(Ln, L4, rtol=0, atol=1e-12)
    Op, Lp = oracle.merge(Os[::-1], Ls[::-1])
    assert np.allclose(Op, O4, rtol=0, atol=1e-12) and np.allclose(Lp, L4, rtol=0, atol=1e-12)


def test_merge_empty_parts_and_large_lse():
    D = 4
    O1 = np.arange(8.0).reshape(2, D)
    L1 = np.array([3.0, -np.inf])
    O0 = np.zeros((2, D))
    L0 = np.full(2, -np.inf)
    O, L = oracle.merge([O0, O1], [L0, L1])
    assert np.array_equal(O[0], O1[0]) and L[0] == 3.0
    assert np.all(O[1] == 0) and np.isneginf(L[1])
    # huge LSEs must not overflow
    O, L = oracle.merge([O1[:1], 2 * O1[:1]], [np.array([1000.0]), np.array([1000.0])])
    assert np.allclose(O[0], 1.5 * O1[0]) and abs(L[0] - (1000.0 + math.log(2))) < 1e-9


def test_prefix_length_zero_reduces_to_standard_attention():
    w = wl.make_workload("p0", 9, 5, 4, 2, 32, [(1, 0, 5)], 3, 9)
    O, L = oracle.attention(w)
    for b in range(w.B):
        Ob, Lb = library_attention(w, b)
        assert np.allclose(O[b], Ob, rtol=0, atol=1e-12) and np.allclose(L[b], Lb, rtol=0, atol=1e-12)
    O2, L2 = oracle.attention(w, levels=[], suffix=True)
    assert np.array_equal(O, O2) and np.array_equal(L, L2)


def test_planted_key_dominates():
    w = wl.scaled_down(3, plant="suffix")
    O, L = oracle.attention(w)
    for b in (0, w.B - 1):
        row = int(w.offsets[b]) + int(w.lengths[b]) // 2
        v = _widen(w.Vs[row])  # [Hkv,D]
        assert np.abs(O[b] - v).max() < 1e-2


# ---- several queries per sequence (App. B's num_queries > 1; the causal reading among the new tokens is this build's) ------------------------

def _nq_workload():
    lengths = np.array([0, 1, 2, 3, 4, 9, 5], dtype=np.int32)   # some shorter than nq, one empty
    return wl.make_workload("nq", 91, 7, 4, 2, 16, [(1, 6, 7), (2, 3, 3)], 0, 0, lengths=lengths, nq=3)


def test_several_queries_brute_force_with_explicit_visibility():
    """Pure-Python exact sums; query t of sequence b sees every shared row and suffix rows 0 .. L_b - nq + t."""
    w = _nq_workload()
    assert w.nq == 3 and w.Q.shape == (7, 3, 4, 16)
    O, L = oracle.attention(w)
    assert O.shape == (7, 3, 4, 16) and L.shape == (7, 3, 4)
    G = w.Hq // w.Hkv
    for b in range(w.B):
        for t in range(w.nq):
            for h in range(w.Hq):
                kvh = h // G
                q = _widen(w.Q[b, t, h]).tolist()
                rows = []
                for li, r0, r1 in w.kv_rows_of(b):
                    rows += [(_widen(w.levels[li].K[r, kvh]).tolist(), _widen(w.levels[li].V[r, kvh]).tolist()) for r in range(r0, r1)]
                last_visible = int(w.lengths[b]) - w.nq + t      # index of the query's own suffix row
                for i in range(int(w.lengths[b])):
                    if i <= last_visible:
                        r = int(w.offsets[b]) + i
                        rows.append((_widen(w.Ks[r, kvh]).tolist(), _widen(w.Vs[r, kvh]).tolist()))
                if not rows:
                    assert np.all(O[b, t, h] == 0) and L[b, t, h] == -np.inf
                    continue
                e = [math.exp(math.fsum(qi * ki for qi, ki in zip(q, k)) * w.scale) for k, _ in rows]
                den = math.fsum(e)
                Ob = [math.fsum(ei * v[d] for ei, (_, v) in zip(e, rows)) / den for d in range(w.D)]
                assert np.allclose(O[b, t, h], Ob, rtol=0, atol=1e-12)
                assert abs(L[b, t, h] - math.log(den)) < 1e-12


def test_several_queries_equal_single_query_calls_on_shortened_suffixes():
    """Query t of an nq-query call is the one-query problem whose suffix ends at that token."""
    w = _nq_workload()
    O, L = oracle.attention(w)
    lv = [(l.K, l.V, l.kv_off, l.seq_off) for l in w.levels]
    for t in range(w.nq):
        shortened = np.maximum(w.lengths - (w.nq - 1 - t), 0).astype(np.int32)
        O1, L1 = oracle.attention_arrays(np.ascontiguousarray(w.Q[:, t]), w.Hkv, lv, w.Ks, w.Vs, w.offsets, shortened, w.scale)
        assert np.array_equal(O[:, t], O1) and np.array_equal(L[:, t], L1)
    # the last query is the plain decode query of the paper (num_queries = 1)
    O1, L1 = oracle.attention_arrays(np.ascontiguousarray(w.Q[:, -1]), w.Hkv, lv, w.Ks, w.Vs, w.offsets, w.lengths, w.scale)
    assert np.array_equal(O[:, -1], O1)


def test_several_queries_library_softmax_with_causal_mask():
    """scipy softmax over all rows with the masked scores set to -inf."""
    w = _nq_workload()
    O, L = oracle.attention(w)
    G = w.Hq // w.Hkv
    for b in (2, 4, 5):
        Kc = [_widen(w.levels[li].K[r0:r1]) for li, r0, r1 in w.kv_rows_of(b)]
        Vc = [_widen(w.levels[li].V[r0:r1]) for li, r0, r1 in w.kv_rows_of(b)]
        nshared = sum(k.shape[0] for k in Kc)
        o, n = int(w.offsets[b]), int(w.lengths[b])
        K = np.repeat(np.concatenate(Kc + [_widen(w.Ks[o:o + n])]), G, axis=1)
        V = np.repeat(np.concatenate(Vc + [_widen(w.Vs[o:o + n])]), G, axis=1)
        for t in range(w.nq):
            S = np.einsum("hd,nhd->hn", _widen(w.Q[b, t]), K) * w.scale
            pos = np.arange(n)
            S[:, nshared:][:, pos > n - w.nq + t] = -np.inf
            Pm = scipy.special.softmax(S, axis=1)
            assert np.allclose(O[b, t], np.einsum("hn,nhd->hd", Pm, V), rtol=0, atol=1e-12)
            assert np.allclose(L[b, t], scipy.special.logsumexp(S, axis=1), rtol=0, atol=1e-12)
