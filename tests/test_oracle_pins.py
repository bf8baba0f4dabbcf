"""Pins for the float64 C oracle: brute force, closed forms, invariants, numpy special cases.

The paper prints no worked numeric example, so nothing here is a printed value;
tests/golden/hand_example.txt is a two-key page worked by hand from Eq. 1-3.
Every check compares the oracle with something that is not the oracle.
"""
import math
import os

import numpy as np
import pytest

import oracle
from oracle import OracleCache
from tests import brute


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16 bit patterns (finite inputs)."""
    u = np.ascontiguousarray(x, np.float32).view(np.uint32).astype(np.uint64)
    r = (u + 0x7FFF + ((u >> 16) & 1)) >> 16
    return r.astype(np.uint16)


def bf16_bits_to_f64(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def as_f64(a: np.ndarray) -> np.ndarray:
    return bf16_bits_to_f64(a) if a.dtype == np.uint16 else a.astype(np.float64)


def make_case(seed, B=2, H=4, Hkv=2, D=8, S=4, lens=(13, 7), bf16=False, permute=True, spare_pages=1):
    """Small random cache with a permuted page table, ragged lengths, NaN in never-written slots."""
    rng = np.random.default_rng(seed)
    lens = list(lens)
    caps = [(n + S - 1) // S + spare_pages for n in lens]
    pool = sum(caps) + 2
    ids = rng.permutation(pool) if permute else np.arange(pool)
    pt = np.zeros((B, max(caps)), np.int32)
    off = 0
    for b in range(B):
        pt[b, :caps[b]] = ids[off:off + caps[b]]
        off += caps[b]
    k = np.full((pool, Hkv, S, D), np.nan, np.float32)
    v = np.full((pool, Hkv, S, D), np.nan, np.float32)
    for b in range(B):
        for t in range(lens[b]):
            k[pt[b, t // S], :, t % S, :] = rng.normal(size=(Hkv, D)) + 0.3
            v[pt[b, t // S], :, t % S, :] = rng.normal(size=(Hkv, D))
    q = rng.normal(size=(B, H, D)).astype(np.float32)
    if bf16:
        nan_k, nan_v = np.isnan(k), np.isnan(v)
        kb, vb, q = f32_to_bf16_bits(np.nan_to_num(k)), f32_to_bf16_bits(np.nan_to_num(v)), f32_to_bf16_bits(q)
        kb[nan_k] = 0x7FC0
        vb[nan_v] = 0x7FC0
        k, v = kb, vb
    return OracleCache(k, v, pt, np.array(lens, np.int32), H), q


def logical_keys(c: OracleCache, b, hkv, which="k"):
    cache = as_f64(c.k_cache if which == "k" else c.v_cache)
    N = int(c.seq_lens[b])
    return np.stack([cache[c.page_table[b, t // c.S], hkv, t % c.S] for t in range(N)])


# ---------------------------------------------------------------- stats (Eq. 1, Eq. 2)

@pytest.mark.parametrize("bf16", [False, True])
def test_stats_vs_python_brute_force(bf16):
    c, _ = make_case(1, bf16=bf16)
    kc = as_f64(c.k_cache).tolist()
    for b in range(c.B):
        mean, std = oracle.page_stats(c, b, 1)
        for p in range(c.num_pages(b)):
            rows = brute.key_rows(kc, c.page_table[b].tolist(), c.S, 1, brute.tokens_of(int(c.seq_lens[b]), c.S, [p]))
            m, s = brute.page_mean_std(rows)
            assert np.allclose(mean[p], m, rtol=1e-14, atol=1e-15)
            assert math.isclose(std[p], s, rel_tol=1e-13, abs_tol=1e-15)


def test_stats_hand_example_golden():
    """tests/golden/hand_example.txt: keys (1,0),(3,4); q=(1,1); lambda 0.5."""
    path = os.path.join(os.path.dirname(__file__), "golden", "hand_example.txt")
    vals = {}
    for line in open(path):
        if line.strip() and not line.startswith("#"):
            name, val = line.split("=")
            vals[name.strip()] = [float(x) for x in val.split()]
    k = np.zeros((1, 1, 2, 2), np.float32)
    k[0, 0] = np.array(vals["keys"], np.float32).reshape(2, 2)
    c = OracleCache(k, k.copy(), np.zeros((1, 1), np.int32), np.array([2], np.int32), 1)
    mean, std = oracle.page_stats(c, 0, 0)
    assert np.allclose(mean[0], vals["mean"], rtol=0, atol=1e-15)
    assert math.isclose(std[0], vals["std"][0], rel_tol=1e-15)
    q = np.array(vals["q"], np.float32).reshape(1, 1, 2)
    s = oracle.page_scores(c, q, 0, 0, vals["lambda"][0], mean, std)
    assert math.isclose(s[0], vals["score"][0], rel_tol=1e-15)


def test_stats_closed_forms():
    S, D = 8, 6
    # all keys identical -> mean = key, std = 0
    key = np.arange(1, D + 1, dtype=np.float32) * 0.25
    k = np.tile(key, (1, 1, S, 1)).astype(np.float32)
    c = OracleCache(k, k.copy(), np.zeros((1, 1), np.int32), np.array([S], np.int32), 1)
    mean, std = oracle.page_stats(c, 0, 0)
    assert np.array_equal(mean[0], key.astype(np.float64)) and std[0] == 0.0
    # +-a e_d in equal numbers -> mean 0, per-dim std a on dim d only -> scalar std a
    a, d = 3.0, 2
    k = np.zeros((1, 1, S, D), np.float32)
    k[0, 0, ::2, d] = a
    k[0, 0, 1::2, d] = -a
    c = OracleCache(k, k.copy(), np.zeros((1, 1), np.int32), np.array([S], np.int32), 1)
    mean, std = oracle.page_stats(c, 0, 0)
    assert np.all(mean[0] == 0.0) and math.isclose(std[0], a, rel_tol=1e-15)
    # one valid token -> std 0, mean = that key (partial tail page uses its own count)
    c = OracleCache(k, k.copy(), np.zeros((1, 1), np.int32), np.array([1], np.int32), 1)
    mean, std = oracle.page_stats(c, 0, 0)
    assert np.array_equal(mean[0], k[0, 0, 0].astype(np.float64)) and std[0] == 0.0


@pytest.mark.parametrize("bf16", [False, True])
def test_stats_vs_numpy_and_moment_identity(bf16):
    c, _ = make_case(2, D=16, S=8, lens=(37, 16), bf16=bf16)
    for b in range(c.B):
        for hkv in range(c.Hkv):
            keys = logical_keys(c, b, hkv)
            mean, std = oracle.page_stats(c, b, hkv)
            for p in range(c.num_pages(b)):
                rows = keys[p * c.S:(p + 1) * c.S]
                assert np.allclose(mean[p], rows.mean(0), rtol=1e-13, atol=1e-15)
                assert math.isclose(std[p], np.linalg.norm(rows.std(0, ddof=0)), rel_tol=1e-12, abs_tol=1e-14)
                # std^2 = E||k||^2 - ||mean||^2 (algebraically equal to Eq. 2)
                ident = (rows ** 2).sum(1).mean() - (rows.mean(0) ** 2).sum()
                assert math.isclose(std[p] ** 2, ident, rel_tol=1e-9, abs_tol=1e-12)


def test_stats_permutation_inside_page_and_subrange():
    c, _ = make_case(3, lens=(16, 8), S=8)
    mean0, std0 = oracle.page_stats(c, 0, 0)
    k2 = c.k_cache.copy()
    phys = c.page_table[0, 1]
    k2[phys, 0] = k2[phys, 0][::-1].copy()
    c2 = OracleCache(k2, c.v_cache, c.page_table, c.seq_lens, c.H)
    mean1, std1 = oracle.page_stats(c2, 0, 0)
    assert np.allclose(mean0, mean1, rtol=1e-15, atol=1e-16) and np.allclose(std0, std1, rtol=1e-14)
    # a sub-range returns the matching rows of the full result
    m, s = oracle.page_stats(c, 0, 0, 1, 2)
    assert np.array_equal(m[0], mean0[1]) and s[0] == std0[1]
    with pytest.raises(ValueError):
        oracle.page_stats(c, 0, 0, 0, 3)


def test_bulk_stats_equal_incremental_updates():
    """Refreshing only the pages touched by each appended token ends at the bulk result."""
    c, _ = make_case(4, lens=(13, 7))
    full_lens = c.seq_lens.copy()
    mean_b, std_b = oracle.new_stat_cache(c)
    oracle.update_stats(c, mean_b, std_b)
    mean_i, std_i = oracle.new_stat_cache(c)
    for t in range(int(full_lens.max())):
        cur = np.minimum(full_lens, t + 1).astype(np.int32)
        ci = OracleCache(c.k_cache, c.v_cache, c.page_table, cur, c.H)
        begin = np.where(full_lens > t, t, cur).astype(np.int32)  # sequences already complete: empty range
        oracle.update_stats(ci, mean_i, std_i, begin, cur)
    for b in range(c.B):
        P = c.num_pages(b)
        assert np.array_equal(mean_b[b, :, :P], mean_i[b, :, :P])
        assert np.array_equal(std_b[b, :, :P], std_i[b, :, :P])
    # and the bulk driver equals the per-row function
    m, s = oracle.page_stats(c, 1, 1)
    assert np.array_equal(mean_b[1, 1, :c.num_pages(1)], m) and np.array_equal(std_b[1, 1, :c.num_pages(1)], s)


# ---------------------------------------------------------------- score (Eq. 3, Eq. 6)

@pytest.mark.parametrize("bf16", [False, True])
def test_scores_vs_python_brute_force(bf16):
    c, q = make_case(5, H=6, Hkv=2, bf16=bf16)  # G = 3
    qf = as_f64(q)
    for b in range(c.B):
        for hkv in range(c.Hkv):
            mean, std = oracle.page_stats(c, b, hkv)
            s = oracle.page_scores(c, q, b, hkv, 0.5, mean, std)
            group = [qf[b, hkv * c.G + g].tolist() for g in range(c.G)]
            for p in range(c.num_pages(b)):
                ref = brute.page_score(group, mean[p].tolist(), float(std[p]), 0.5)
                assert math.isclose(s[p], ref, rel_tol=1e-13, abs_tol=1e-14)


def test_score_special_cases():
    c, q = make_case(6, H=4, Hkv=2, D=8)
    b, hkv = 0, 1
    mean, std = oracle.page_stats(c, b, hkv)
    qf = q.astype(np.float64)
    grp = qf[b, hkv * c.G:(hkv + 1) * c.G]
    s = oracle.page_scores(c, q, b, hkv, 0.5, mean, std)
    # numpy form of Eq. 6
    ref = (grp @ mean.T + 0.5 * np.linalg.norm(grp, axis=1)[:, None] * std[None, :]).max(0)
    assert np.allclose(s, ref, rtol=1e-13, atol=1e-14)
    # lambda = 0 -> mean-only ranking (the ablation in Section 4.5)
    s0 = oracle.page_scores(c, q, b, hkv, 0.0, mean, std)
    assert np.allclose(s0, (grp @ mean.T).max(0), rtol=1e-13, atol=1e-14)
    # q = 0 -> all scores 0
    assert np.all(oracle.page_scores(c, np.zeros_like(q), b, hkv, 0.5, mean, std) == 0.0)
    # scaling q by c > 0 scales every score by c (power of two keeps fp32 exact)
    assert np.allclose(oracle.page_scores(c, q * 4.0, b, hkv, 0.5, mean, std), 4.0 * s, rtol=1e-14)
    # duplicating a head inside the group changes nothing; G = 1 is Eq. 3
    qd = q.copy()
    qd[b, hkv * c.G + 1] = qd[b, hkv * c.G]
    sd = oracle.page_scores(c, qd, b, hkv, 0.5, mean, std)
    c1 = OracleCache(c.k_cache, c.v_cache, c.page_table, c.seq_lens, c.Hkv)  # H = Hkv -> G = 1
    q1 = np.ascontiguousarray(q[:, ::c.G, :])
    s1 = oracle.page_scores(c1, q1, b, hkv, 0.5, mean, std)
    g0 = qf[b, hkv * c.G]
    eq3 = mean @ g0 + 0.5 * np.linalg.norm(g0) * std
    assert np.allclose(s1, eq3, rtol=1e-13, atol=1e-14) and np.allclose(sd, eq3, rtol=1e-13, atol=1e-14)


def test_score_bounds_from_cauchy_schwarz():
    """score >= q.mean always (lambda >= 0); with lambda >= sqrt(S) and G = 1, score >= max_j q.k_j."""
    c, q = make_case(7, H=2, Hkv=2, D=8, S=4, lens=(16, 8))
    qf = q.astype(np.float64)
    for b in range(c.B):
        for hkv in range(c.Hkv):
            keys = logical_keys(c, b, hkv)
            mean, std = oracle.page_stats(c, b, hkv)
            s_half = oracle.page_scores(c, q, b, hkv, 0.5, mean, std)
            s_big = oracle.page_scores(c, q, b, hkv, math.sqrt(c.S), mean, std)
            for p in range(c.num_pages(b)):
                dots = keys[p * c.S:(p + 1) * c.S] @ qf[b, hkv]
                assert s_half[p] >= dots.mean() - 1e-12
                assert s_big[p] >= dots.max() - 1e-12


def test_score_orthogonal_invariance():
    """Rotating q and all keys by one orthogonal matrix leaves stats' std and all scores unchanged."""
    rng = np.random.default_rng(8)
    c, q = make_case(8, D=8)
    R, _ = np.linalg.qr(rng.normal(size=(8, 8)))
    # exact float64 rotation cannot be stored in fp32 caches, so compare through float64 stats directly
    for hkv in range(c.Hkv):
        keys = logical_keys(c, 0, hkv)
        mean, std = oracle.page_stats(c, 0, hkv)
        s = oracle.page_scores(c, q, 0, hkv, 0.5, mean, std)
        rk = (keys @ R.T).astype(np.float32)
        k2 = c.k_cache.copy()
        for t in range(int(c.seq_lens[0])):
            k2[c.page_table[0, t // c.S], hkv, t % c.S] = rk[t]
        c2 = OracleCache(k2, c.v_cache, c.page_table, c.seq_lens, c.H)
        q2 = q.copy()
        q2[0] = (q[0].astype(np.float64) @ R.T).astype(np.float32)
        mean2, std2 = oracle.page_stats(c2, 0, hkv)
        s2 = oracle.page_scores(c2, q2, 0, hkv, 0.5, mean2, std2)
        assert np.allclose(std, std2, rtol=1e-5) and np.allclose(s, s2, rtol=1e-4, atol=1e-5)


# ---------------------------------------------------------------- top-k

def test_topk_vs_brute_force_and_properties():
    rng = np.random.default_rng(9)
    for P, k in [(1, 1), (5, 1), (5, 5), (5, 9), (64, 7), (300, 64)]:
        s = np.round(rng.normal(size=P), 1)  # rounding forces ties
        order, kb = oracle.topk(s, k)
        assert kb == min(k, P)
        assert order[:kb].tolist() == brute.topk_set(s.tolist(), k)
        assert sorted(order.tolist()) == list(range(P))  # a permutation: distinct, all < P
        chosen = set(order[:kb].tolist())
        rest = [p for p in range(P) if p not in chosen]
        if rest:
            assert s[list(chosen)].min() >= s[rest].max()


def test_topk_special_cases():
    s = np.array([1.0, 5.0, 5.0, -2.0, 5.0])
    order, kb = oracle.topk(s, 1)
    assert kb == 1 and order[0] == 1                      # argmax, lowest index among ties
    order, kb = oracle.topk(s, 2)
    assert order[:2].tolist() == [1, 2]                   # ties -> lower page index first
    order, kb = oracle.topk(np.full(10, 3.25), 4)
    assert order[:kb].tolist() == [0, 1, 2, 3]            # all equal -> pages 0..k-1, none forced
    order, kb = oracle.topk(s, 5)
    assert kb == 5 and sorted(order.tolist()) == [0, 1, 2, 3, 4]
    assert order.tolist() == np.lexsort((np.arange(5), -s)).tolist()  # numpy's sort as a second opinion


# ---------------------------------------------------------------- attention (Eq. 4, Eq. 5)

@pytest.mark.parametrize("bf16", [False, True])
def test_attention_vs_python_brute_force(bf16):
    c, q = make_case(10, bf16=bf16)
    kc, vc, qf = as_f64(c.k_cache).tolist(), as_f64(c.v_cache).tolist(), as_f64(q)
    scale = 1.0 / math.sqrt(c.D)
    for b, h, pages in [(0, 0, [0, 3]), (0, 3, [1, 2, 3]), (1, 2, [1]), (1, 1, [0, 1])]:
        hkv = h // c.G
        toks = brute.tokens_of(int(c.seq_lens[b]), c.S, pages)
        kr = brute.key_rows(kc, c.page_table[b].tolist(), c.S, hkv, toks)
        vr = brute.key_rows(vc, c.page_table[b].tolist(), c.S, hkv, toks)
        ref_o, ref_lse = brute.softmax_attention(qf[b, h].tolist(), kr, vr, scale)
        o, lse = oracle.attention(c, q, b, h, pages)
        assert np.allclose(o, ref_o, rtol=1e-12, atol=1e-14) and math.isclose(lse, ref_lse, rel_tol=1e-13)
        # explicit scale argument
        o2, lse2 = oracle.attention(c, q, b, h, pages, sm_scale=0.37)
        ref_o2, ref_lse2 = brute.softmax_attention(qf[b, h].tolist(), kr, vr, 0.37)
        assert np.allclose(o2, ref_o2, rtol=1e-12, atol=1e-14) and math.isclose(lse2, ref_lse2, rel_tol=1e-13)


def test_dense_is_softmax_by_definition_and_select_all_equals_dense():
    c, q = make_case(11, D=16)
    qf = q.astype(np.float64)
    for b in range(c.B):
        for h in range(c.H):
            K, V = logical_keys(c, b, h // c.G, "k"), logical_keys(c, b, h // c.G, "v")
            logits = K @ qf[b, h] / math.sqrt(c.D)
            w = np.exp(logits - logits.max())
            ref = (w / w.sum()) @ V
            o, lse = oracle.dense_attention(c, q, b, h)
            assert np.allclose(o, ref, rtol=1e-12, atol=1e-14)
            assert math.isclose(lse, math.log(np.exp(logits).sum()), rel_tol=1e-12)
            o2, lse2 = oracle.attention(c, q, b, h, list(range(c.num_pages(b))))
            assert np.array_equal(o, o2) and lse == lse2
    od, lsed = oracle.dense_decode(c, q)
    o, lse = oracle.dense_attention(c, q, 1, 2)
    assert np.array_equal(od[1, 2], o) and lsed[1, 2] == lse


def test_attention_closed_forms():
    c, q = make_case(12, lens=(13, 1))
    # one page with one token -> o = v, lse = logit
    o, lse = oracle.attention(c, q, 1, 0, [0])
    v0 = c.v_cache[c.page_table[1, 0], 0, 0].astype(np.float64)
    k0 = c.k_cache[c.page_table[1, 0], 0, 0].astype(np.float64)
    assert np.allclose(o, v0, rtol=1e-15) and math.isclose(lse, q[1, 0].astype(np.float64) @ k0 / math.sqrt(c.D), rel_tol=1e-13)
    # q = 0 -> all logits equal -> mean of the V rows; lse = log(#tokens)
    o, lse = oracle.attention(c, np.zeros_like(q), 0, 1, [0, 3])
    V = logical_keys(c, 0, 0, "v")
    rows = np.concatenate([V[0:4], V[12:13]])
    assert np.allclose(o, rows.mean(0), rtol=1e-13, atol=1e-15) and math.isclose(lse, math.log(5), rel_tol=1e-14)
    # V constant -> o is that constant
    v2 = np.where(np.isnan(c.v_cache), np.nan, np.float32(1.5)).astype(np.float32)
    c2 = OracleCache(c.k_cache, v2, c.page_table, c.seq_lens, c.H)
    o, _ = oracle.attention(c2, q, 0, 2, [0, 1, 2])
    assert np.allclose(o, 1.5, rtol=1e-14)
    # heads of one group with identical q give identical o
    qd = q.copy()
    qd[0, 1] = qd[0, 0]
    assert np.array_equal(oracle.attention(c, qd, 0, 0, [1, 2])[0], oracle.attention(c, qd, 0, 1, [1, 2])[0])
    # bad page index is rejected
    with pytest.raises(ValueError):
        oracle.attention(c, q, 0, 0, [4])


def test_attention_key_shift_invariance():
    """Adding one vector to every key shifts all logits by q.c: o unchanged, lse shifted by q.c/sqrt(D)."""
    rng = np.random.default_rng(13)
    c, q = make_case(13, D=8)
    # multiples of 1/8 stay exact in fp32 after the shift
    k = np.where(np.isnan(c.k_cache), np.nan, np.round(np.nan_to_num(c.k_cache) * 8) / 8).astype(np.float32)
    shift = (np.round(rng.normal(size=8) * 8) / 8).astype(np.float32)
    c1 = OracleCache(k, c.v_cache, c.page_table, c.seq_lens, c.H)
    c2 = OracleCache((k + shift).astype(np.float32), c.v_cache, c.page_table, c.seq_lens, c.H)
    o1, l1 = oracle.attention(c1, q, 0, 1, [0, 2, 3])
    o2, l2 = oracle.attention(c2, q, 0, 1, [0, 2, 3])
    assert np.allclose(o1, o2, rtol=1e-12, atol=1e-14)
    assert math.isclose(l2 - l1, q[0, 1].astype(np.float64) @ shift.astype(np.float64) / math.sqrt(8), rel_tol=1e-11)


def test_union_of_page_sets_is_lse_merge():
    """Attention over A u B equals the log-sum-exp weighted combination of attention over A and over B."""
    c, q = make_case(14, lens=(29, 7), S=4, spare_pages=0)
    A, Bset = [0, 5, 7], [1, 2, 6]
    oa, la = oracle.attention(c, q, 0, 3, A)
    ob, lb = oracle.attention(c, q, 0, 3, Bset)
    ou, lu = oracle.attention(c, q, 0, 3, A + Bset)
    m = max(la, lb)
    wa, wb = math.exp(la - m), math.exp(lb - m)
    assert np.allclose(ou, (wa * oa + wb * ob) / (wa + wb), rtol=1e-12, atol=1e-14)
    assert math.isclose(lu, m + math.log(wa + wb), rel_tol=1e-13)
    # order of the page list is irrelevant
    o_rev, l_rev = oracle.attention(c, q, 0, 3, (A + Bset)[::-1])
    assert np.allclose(ou, o_rev, rtol=1e-12, atol=1e-14) and math.isclose(lu, l_rev, rel_tol=1e-14)


# ---------------------------------------------------------------- whole step

@pytest.mark.parametrize("bf16", [False, True])
def test_step_vs_python_brute_force_pipeline(bf16):
    c, q = make_case(15, H=4, Hkv=2, lens=(23, 9), bf16=bf16)
    mean_all, std_all = oracle.new_stat_cache(c)
    oracle.update_stats(c, mean_all, std_all)
    top_k = 3
    r = oracle.sparse_decode_step(c, q, mean_all, std_all, 0.5, top_k)
    kc, vc, qf = as_f64(c.k_cache).tolist(), as_f64(c.v_cache).tolist(), as_f64(q)
    for b in range(c.B):
        N, P = int(c.seq_lens[b]), c.num_pages(b)
        for hkv in range(c.Hkv):
            group = [qf[b, hkv * c.G + g].tolist() for g in range(c.G)]
            scores = []
            for p in range(P):
                rows = brute.key_rows(kc, c.page_table[b].tolist(), c.S, hkv, brute.tokens_of(N, c.S, [p]))
                m, s = brute.page_mean_std(rows)
                scores.append(brute.page_score(group, m, s, 0.5))
            chosen = sorted(brute.topk_set(scores, top_k))
            kb = min(top_k, P)
            assert r["sel_count"][b, hkv] == kb
            assert r["sel"][b, hkv, :kb].tolist() == chosen and np.all(r["sel"][b, hkv, kb:] == -1)
            assert np.allclose(r["scores"][b, hkv, :P], scores, rtol=1e-13, atol=1e-14)
            toks = brute.tokens_of(N, c.S, chosen)
            kr = brute.key_rows(kc, c.page_table[b].tolist(), c.S, hkv, toks)
            vr = brute.key_rows(vc, c.page_table[b].tolist(), c.S, hkv, toks)
            for g in range(c.G):
                h = hkv * c.G + g
                ref_o, ref_lse = brute.softmax_attention(qf[b, h].tolist(), kr, vr, 1 / math.sqrt(c.D))
                assert np.allclose(r["out"][b, h], ref_o, rtol=1e-12, atol=1e-14)
                assert math.isclose(r["lse"][b, h], ref_lse, rel_tol=1e-13)


def test_step_k_at_least_P_equals_dense_and_physical_placement_is_irrelevant():
    c, q = make_case(16, lens=(13, 7), permute=True)
    mean_all, std_all = oracle.new_stat_cache(c)
    oracle.update_stats(c, mean_all, std_all)
    r = oracle.sparse_decode_step(c, q, mean_all, std_all, 0.5, 8)  # k >= P for both sequences
    od, lsed = oracle.dense_decode(c, q)
    assert np.allclose(r["out"], od, rtol=1e-13, atol=1e-15) and np.allclose(r["lse"], lsed, rtol=1e-14)
    assert r["sel_count"].tolist() == [[4, 4], [2, 2]]
    # same logical content placed on different physical pages
    rng = np.random.default_rng(0)
    perm = rng.permutation(c.num_phys_pages)
    inv = np.argsort(perm)
    k2, v2 = c.k_cache[inv].copy(), c.v_cache[inv].copy()  # page that was at i now sits at perm[i]
    pt2 = perm[c.page_table].astype(np.int32)
    c2 = OracleCache(k2, v2, pt2, c.seq_lens, c.H)
    m2, s2 = oracle.new_stat_cache(c2)
    oracle.update_stats(c2, m2, s2)
    r1 = oracle.sparse_decode_step(c, q, mean_all, std_all, 0.5, 2)
    r2 = oracle.sparse_decode_step(c2, q, m2, s2, 0.5, 2)
    assert np.array_equal(r1["sel"], r2["sel"]) and np.array_equal(r1["out"], r2["out"])


def test_batch_entries_are_independent():
    c, q = make_case(17, lens=(13, 7))
    mean_all, std_all = oracle.new_stat_cache(c)
    oracle.update_stats(c, mean_all, std_all)
    r = oracle.sparse_decode_step(c, q, mean_all, std_all, 0.5, 2)
    c1 = OracleCache(c.k_cache, c.v_cache, c.page_table[1:2], c.seq_lens[1:2], c.H)
    m1, s1 = oracle.new_stat_cache(c1)
    oracle.update_stats(c1, m1, s1)
    r1 = oracle.sparse_decode_step(c1, np.ascontiguousarray(q[1:2]), m1, s1, 0.5, 2)
    assert np.array_equal(r["sel"][1], r1["sel"][0]) and np.array_equal(r["out"][1], r1["out"][0])


def test_poisoned_slots_are_never_read():
    """Never-written slots hold NaN in make_case; any read of them would surface as NaN."""
    c, q = make_case(18, lens=(13, 7))
    mean_all, std_all = oracle.new_stat_cache(c)
    oracle.update_stats(c, mean_all, std_all)
    r = oracle.sparse_decode_step(c, q, mean_all, std_all, 0.5, 4)
    assert np.isfinite(r["out"]).all() and np.isfinite(r["lse"]).all()
    for b in range(c.B):
        assert np.isfinite(mean_all[b, :, :c.num_pages(b)]).all()


def test_planted_keys_need_the_std_offset():
    """Config 1's recipe: pages holding one planted key aligned with q rank higher with the std term than without."""
    from paper_2605_27740_amd import workloads as W
    wl = W.config1()
    a = wl.host_arrays()
    c = OracleCache(a["k_cache"], a["v_cache"], a["page_table"], a["seq_lens"], wl.H)
    mean, std = oracle.page_stats(c, 0, 0)
    s_with = oracle.page_scores(c, a["q"], 0, 0, 0.5, mean, std)
    s_without = oracle.page_scores(c, a["q"], 0, 0, 0.0, mean, std)
    # planted pages have the largest std of the row
    planted = np.argsort(-std)[:4]
    rank_with = np.argsort(np.argsort(-s_with))[planted]
    rank_without = np.argsort(np.argsort(-s_without))[planted]
    assert rank_with.sum() <= rank_without.sum()
    assert (rank_with < wl.top_k).all()


def test_topk_forced_recent_pages_invariants():
    """The always-keep option (C ABI; not from the paper, whose method needs no local window -- Section 4.3):
    the set has min(k, P) pages, contains the last min(n, k, P), and among the other pages every selected one
    outranks every unselected one under (score desc, index asc); n = 0 is the plain top-k."""
    rng = np.random.default_rng(5)
    for trial in range(300):
        P = int(rng.integers(1, 40))
        k = int(rng.integers(1, 45))
        n = int(rng.integers(0, 12))
        s = rng.integers(-3, 4, size=P).astype(np.float64) if trial % 2 else rng.normal(size=P)
        got = oracle.topk_forced(s, k, n)
        kb, nf = min(k, P), min(n, k, P)
        assert got.shape == (kb,) and (np.diff(got) > 0).all()
        assert set(range(P - nf, P)) <= set(got.tolist())
        if n == 0:
            order, _ = oracle.topk(s, k)
            assert sorted(order[:kb].tolist()) == got.tolist()
        chosen = [p for p in got.tolist() if p < P - nf]
        others = [p for p in range(P - nf) if p not in chosen]
        for a in chosen:
            for b in others:
                assert (s[a], -a) > (s[b], -b), (trial, a, b)


# ------------------------------------------------------------------ bf16 storage of the means (oracle_round_bf16)

def _all_bf16_values():
    """Every finite bf16 value >= 0 in ascending order with its bit pattern (exhaustive table, 32640 entries)."""
    bits = np.arange(0x0000, 0x7F80, dtype=np.uint16)
    return bf16_bits_to_f64(bits), bits


def _nearest_bf16_brute(x: float) -> int:
    """Nearest bf16 bit pattern of a finite double by exhaustive comparison in exact rational arithmetic;
    ties go to the even fraction (even bit pattern); beyond the largest finite value the midpoint to 2^128 decides."""
    from fractions import Fraction
    vals, bits = _all_bf16_values()
    sign = 0x8000 if math.copysign(1.0, x) < 0 else 0
    a = Fraction(abs(x))
    i = int(np.searchsorted(vals, float(abs(x)), side="right")) - 1      # vals[i] <= |x|
    lo = Fraction(float(vals[i]))
    hi = Fraction(float(vals[i + 1])) if i + 1 < len(vals) else Fraction(2) ** 128
    hi_bits = int(bits[i + 1]) if i + 1 < len(vals) else 0x7F80
    if a - lo < hi - a:
        return sign | int(bits[i])
    if a - lo > hi - a:
        return sign | hi_bits
    return sign | (int(bits[i]) if int(bits[i]) % 2 == 0 else hi_bits)


def test_round_bf16_against_exhaustive_search():
    rng = np.random.default_rng(31)
    x = np.concatenate([
        rng.normal(size=600), rng.normal(size=300) * 1e-3, rng.normal(size=200) * 1e30, rng.normal(size=200) * 1e-39,
        np.ldexp(rng.uniform(1, 2, size=300), rng.integers(-140, 128, size=300)) * rng.choice([-1, 1], size=300),
        [0.0, -0.0, 1.0, -1.0, 3.3895313892515355e38, 3.3961775292304601e38, 3.4e38, -3.4e38, 1e-45, 4.6e-41, 9.2e-41],
    ])
    got = oracle.round_bf16(x)
    want = np.array([_nearest_bf16_brute(float(v)) for v in x], np.uint16)
    assert np.array_equal(got, want), np.nonzero(got != want)[0][:10]


def test_round_bf16_rounds_once_and_ties_to_even():
    """Values that separate one rounding of the double from a rounding through float first, and exact ties."""
    cases = {
        1.0 + 2.0 ** -8 + 2.0 ** -40: 0x3F81,   # just above a tie: up (through float it becomes the tie and goes down)
        1.0 + 2.0 ** -8 - 2.0 ** -40: 0x3F80,
        1.0 + 2.0 ** -8: 0x3F80,                # tie -> even fraction 0000000
        1.0 + 3 * 2.0 ** -8: 0x3F82,            # tie -> even fraction 0000010
        -(1.0 + 3 * 2.0 ** -8): 0xBF82,
        0.5 - 2.0 ** -10: 0x3F00,               # tie just below a power of two (spacing halves there) -> 0.5
        2.0 ** -133: 0x0001, 2.0 ** -134: 0x0000, 3 * 2.0 ** -134: 0x0002,   # subnormals, ties to even
        float("inf"): 0x7F80, float("-inf"): 0xFF80,
    }
    x = np.array(list(cases), np.float64)
    assert oracle.round_bf16(x).tolist() == list(cases.values())
    assert oracle.round_bf16(np.array([float("nan")]))[0] & 0x7FC0 == 0x7FC0
    assert math.copysign(1.0, oracle.bf16_to_double(oracle.round_bf16(np.array([-0.0])))[0]) == -1.0


def test_round_bf16_equals_the_bit_trick_on_float32_inputs():
    """A double that is exactly a float32 rounds like the usual add-0x7fff-plus-lsb integer trick on its bits
    (written independently above), and rounding is idempotent on bf16 values."""
    rng = np.random.default_rng(32)
    x = (rng.normal(size=20000) * np.exp(rng.uniform(-60, 60, size=20000))).astype(np.float32)
    x = x[np.isfinite(x)]
    assert np.array_equal(oracle.round_bf16(x.astype(np.float64)), f32_to_bf16_bits(x))
    vals, bits = _all_bf16_values()
    assert np.array_equal(oracle.round_bf16(vals), bits) and np.array_equal(oracle.bf16_to_double(bits), vals)


# ------------------------------------------------------------------ Eq. 5 over given page lists, whole batch

def test_attention_rows_equals_the_definition_head_by_head():
    c, q = make_case(41, B=3, H=4, Hkv=2, D=8, S=4, lens=(13, 7, 22), spare_pages=0)
    rng = np.random.default_rng(41)
    stride = 5
    sel = np.full((c.B, c.Hkv, stride), -1, np.int32)
    cnt = np.zeros((c.B, c.Hkv), np.int32)
    for b in range(c.B):
        for h in range(c.Hkv):
            n = int(rng.integers(1, min(stride, c.num_pages(b)) + 1))
            sel[b, h, :n] = rng.permutation(c.num_pages(b))[:n]       # any order, distinct
            cnt[b, h] = n
    cnt[1, 0] = 0                                                      # an empty list
    out, lse = oracle.attention_rows(c, q, sel, cnt, 0.3)
    assert (out[1, :c.G] == 0).all() and np.isneginf(lse[1, :c.G]).all()
    kf, vf = as_f64(c.k_cache).tolist(), as_f64(c.v_cache).tolist()
    for b in range(c.B):
        for h in range(c.H):
            hkv = h // c.G
            if cnt[b, hkv] == 0:
                continue
            pages = sel[b, hkv, :cnt[b, hkv]].tolist()
            toks = brute.tokens_of(int(c.seq_lens[b]), c.S, pages)
            o_b, l_b = brute.softmax_attention([float(x) for x in as_f64(q[b, h])],
                                               brute.key_rows(kf, c.page_table[b].tolist(), c.S, hkv, toks),
                                               brute.key_rows(vf, c.page_table[b].tolist(), c.S, hkv, toks), 0.3)
            assert np.allclose(out[b, h], o_b, rtol=1e-12, atol=1e-13) and abs(lse[b, h] - l_b) < 1e-12
    # on the oracle's own selection it reproduces the whole-step driver
    mean_all, std_all = oracle.new_stat_cache(c)
    oracle.update_stats(c, mean_all, std_all)
    r = oracle.sparse_decode_step(c, q, mean_all, std_all, 0.5, 3)
    o2, l2 = oracle.attention_rows(c, q, r["sel"], r["sel_count"])
    assert np.array_equal(o2, r["out"]) and np.array_equal(l2, r["lse"])
