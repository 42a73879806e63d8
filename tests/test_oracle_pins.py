"""Pins of the CPU oracle against what the paper and the mathematics fix.

None of these re-type the oracle's own formulas: each compares it with a closed
form, a brute-force / dense formulation written here in NumPy, an invariant, a
special case that reduces to textbook attention, or a count the paper prints.
"""
import math
import os

import numpy as np
import pytest

HERE = os.path.dirname(os.path.abspath(__file__))


def _rand(rng, n, d, bf16=False):
    x = rng.standard_normal((n, d)).astype(np.float32)
    return x


def _ints(rng, n, d, lo=-4, hi=5):
    return rng.integers(lo, hi, size=(n, d)).astype(np.float32)


# ------------------------------------------------------------------ pyramid

def test_pool_is_mean_closed_form(oracle):
    rng = np.random.default_rng(1)
    for B in (2, 4, 16, 3):
        x = _rand(rng, 64 * B, 24)
        y = oracle.pool(x, B, bf16=False)
        ref = x.astype(np.float64).reshape(64, B, 24).mean(axis=1)
        # fp32 sequential sum of B terms then one division: error below B ulps of the largest partial sum
        bound = (B + 1) * np.finfo(np.float32).eps * np.abs(x).reshape(64, B, 24).sum(axis=1)
        assert np.all(np.abs(y - ref) <= bound + 1e-30)


def test_pool_exact_on_small_integers(oracle):
    rng = np.random.default_rng(2)
    x = _ints(rng, 16 * 16, 8, -100, 100)
    y = oracle.pool(x, 16, bf16=False)
    ref = x.astype(np.int64).reshape(16, 16, 8).sum(axis=1) / 16.0
    assert np.array_equal(y.astype(np.float64), ref)


def test_pool_bf16_rounding_is_nearest_even(oracle):
    # mean of B copies of the same bf16 value is that value; halfway cases go to even
    x = np.array([[1.0, 1.0 + 2.0 ** -7]], np.float32)           # both bf16-exact
    pair = np.concatenate([x, x[:, ::-1]], axis=0)               # rows (a,b),(b,a): mean = 1 + 2^-8 (a tie in bf16)
    y = oracle.pool(pair, 2, bf16=True)
    assert np.array_equal(y, np.array([[1.0, 1.0]], np.float32))  # ties to even mantissa (1.0)
    pair2 = np.array([[1.0 + 2.0 ** -7], [1.0 + 2.0 ** -6]], np.float32)  # mean 1 + 3*2^-8 -> tie -> 1 + 2^-6 (even)
    assert oracle.pool(pair2, 2, bf16=True)[0, 0] == np.float32(1.0 + 2.0 ** -6)
    rng = np.random.default_rng(3)
    z = oracle.to_bf16(_rand(rng, 64, 16))
    out = oracle.pool(z, 4, bf16=True)
    ref = z.astype(np.float64).reshape(16, 4, 16).mean(axis=1)
    ulp = 2.0 ** (np.floor(np.log2(np.maximum(np.abs(ref), 1e-30))) - 7)
    assert np.all(np.abs(out - ref) <= 0.5 * ulp * (1 + 1e-6) + 1e-30)
    assert np.array_equal(oracle.to_bf16(out), out)


def test_pool_twice_matches_direct_mean(oracle):
    rng = np.random.default_rng(4)
    x = _rand(rng, 16 * 16 * 3, 8)
    two = oracle.pool(oracle.pool(x, 16, False), 16, False)
    direct = x.astype(np.float64).reshape(3, 256, 8).mean(axis=1)
    assert np.allclose(two, direct, rtol=0, atol=1e-6)


def test_pyramid_levels_and_shapes(oracle):
    g = oracle.Geometry(256, 32, 4, 2, 3)
    rng = np.random.default_rng(5)
    lv = oracle.pyramid(_rand(rng, 256, 32), g, bf16=False)
    assert [a.shape[0] for a in lv] == [256, 64, 16, 4]
    # recursive: level l is pooled from level l-1, not from level 0 (same thing up to rounding; check exact recursion)
    assert np.array_equal(lv[2], oracle.pool(lv[1], 4, False))


# ---------------------------------------------------------------- selection

def _brute_topk(scores, ids, K):
    """first K of a full sort by (-score, id), returned as an ascending id list"""
    order = np.lexsort((ids, -scores))
    return np.sort(ids[order[:K]])


def test_coarsest_level_topk_is_full_sort(oracle):
    rng = np.random.default_rng(6)
    for n, d, K in ((16, 8, 8), (37, 4, 5), (4, 4, 4)):
        Q, Kk = _ints(rng, n, d), _ints(rng, n, d)         # integers: fp32 scores exact, many ties
        got = oracle.select_level(Q, Kk, 4, None, K)
        S = Q.astype(np.float64) @ Kk.astype(np.float64).T
        for i in range(n):
            assert np.array_equal(got[i], _brute_topk(S[i], np.arange(n), K)), i


def test_sparse_topk_matches_masked_brute_force_with_ties(oracle):
    rng = np.random.default_rng(7)
    B, K = 4, 2
    g = oracle.Geometry(256, 8, B, K, 3)
    Q, Kk = _ints(rng, 256, 8, -2, 3), _ints(rng, 256, 8, -2, 3)
    Qp, Kp = oracle.pyramid(Q, g, False), oracle.pyramid(Kk, g, False)
    I = oracle.select_all(Qp, Kp, g)
    for l in range(g.L, 0, -1):
        S = Qp[l].astype(np.float64) @ Kp[l].astype(np.float64).T      # exact: dyadic rationals
        n_l = g.n(l)
        for i in range(n_l):
            if l == g.L:
                cand = np.arange(n_l)
            else:
                cand = (I[l][i // B][:, None] * B + np.arange(B)[None, :]).reshape(-1)
            assert np.array_equal(I[l - 1][i], _brute_topk(S[i, cand], cand, g.K_l(l - 1))), (l, i)


def test_sparse_topk_gaussian_matches_fp64_outside_near_ties(oracle):
    rng = np.random.default_rng(8)
    g = oracle.Geometry(4096, 16, 16, 4, 2)
    Q, Kk = _rand(rng, 4096, 16), _rand(rng, 4096, 16)
    Qp, Kp = oracle.pyramid(Q, g, False), oracle.pyramid(Kk, g, False)
    I, margins = oracle.select_all(Qp, Kp, g, want_margin=True)
    checked = 0
    for l in (2, 1):
        S = Qp[l].astype(np.float64) @ Kp[l].astype(np.float64).T
        for i in range(g.n(l)):
            cand = np.arange(g.n(l)) if l == g.L else (I[l][i // 16][:, None] * 16 + np.arange(16)).reshape(-1)
            if margins[l - 1][i] > 1e-5:
                assert np.array_equal(I[l - 1][i], _brute_topk(S[i, cand], cand, g.K_l(l - 1)))
                checked += 1
    assert checked > 0.99 * (256 + 16)


def test_every_pick_is_child_of_a_parent_pick(oracle):
    rng = np.random.default_rng(9)
    g = oracle.Geometry(4096, 8, 4, 3, 5)
    Qp, Kp = oracle.pyramid(_rand(rng, 4096, 8), g, False), oracle.pyramid(_rand(rng, 4096, 8), g, False)
    I = oracle.select_all(Qp, Kp, g)
    for l in range(g.L - 1, 0, -1):           # I[l-1] rows are level-l tokens; their parent row is I[l][i // B]
        for i in range(g.n(l)):
            parents = set(I[l][i // g.B].tolist())
            assert all((int(j) // g.B) in parents for j in I[l - 1][i])
    for l in range(g.L):
        assert I[l].shape == (g.n(l + 1), g.K_l(l))
        assert np.all(np.diff(I[l], axis=1) > 0)           # ascending and distinct
        assert I[l].min() >= 0 and I[l].max() < g.n(l + 1)  # key-block ids at level l


def test_selection_invariances(oracle):
    rng = np.random.default_rng(10)
    g = oracle.Geometry(1024, 16, 4, 2, 4)
    Q, Kk = _rand(rng, 1024, 16), _rand(rng, 1024, 16)
    base = oracle.select_all(oracle.pyramid(Q, g, False), oracle.pyramid(Kk, g, False), g)
    # scaling Q by a positive power of two is exact in fp32 and cannot change any ordering
    scaled = oracle.select_all(oracle.pyramid(4.0 * Q, g, False), oracle.pyramid(0.5 * Kk, g, False), g)
    for a, b in zip(base, scaled):
        assert np.array_equal(a, b)
    # swapping the roles of nothing else: V never enters selection (forward() takes it, select_all does not)


def test_single_level_is_textbook_topk(oracle):
    """L = 1: pool, dense scores on pooled tokens, sort (Sec. 3.2)."""
    rng = np.random.default_rng(11)
    B, K, N, d = 4, 3, 64, 8
    g = oracle.Geometry(N, d, B, K, 1)
    Q, Kk = _ints(rng, N, d), _ints(rng, N, d)
    I = oracle.select_all(oracle.pyramid(Q, g, False), oracle.pyramid(Kk, g, False), g)
    Qc = Q.reshape(N // B, B, d).astype(np.float64).mean(1)
    Kc = Kk.reshape(N // B, B, d).astype(np.float64).mean(1)
    S = Qc @ Kc.T
    for i in range(N // B):
        assert np.array_equal(I[0][i], _brute_topk(S[i], np.arange(N // B), K))


def test_teaser_shape_matches_a_by_hand_walk(oracle):
    """N=8, B=2, K=1 (Fig. 1 caption): levels 8/4/2.  Every step written out directly in NumPy: means of pairs,
    arg-max among the allowed candidates, softmax over the six listed tokens with weights 1, 2, 4."""
    rng = np.random.default_rng(12)
    g = oracle.Geometry(8, 4, 2, 1, 2)
    Q, Kk, V = (_rand(rng, 8, 4) for _ in range(3))
    r = oracle.forward(Q, Kk, V, g)
    assert [a.shape for a in r["I"]] == [(4, 1), (2, 1)]
    assert g.list_len(2) == 2 + 2 + 2
    mean2 = lambda x: (x[0::2] + x[1::2]) / np.float32(2)
    Q1, K1, V1 = mean2(Q), mean2(Kk), mean2(V)
    Q2, K2, V2 = mean2(Q1), mean2(K1), mean2(V1)
    I1 = np.array([[int(np.argmax(Q2[i] @ K2.T))] for i in range(2)])           # level-1 key block per level-2 query
    I0 = np.array([[2 * I1[i // 2, 0] + int(np.argmax(Q1[i] @ K1[2 * I1[i // 2, 0]: 2 * I1[i // 2, 0] + 2].T))]
                   for i in range(4)])                                         # level-0 key block per level-1 query
    assert np.array_equal(r["I"][1], I1) and np.array_equal(r["I"][0], I0)
    for q in range(8):
        j0, j1 = I0[q // 2, 0], I1[q // 4, 0]
        keys = np.concatenate([Kk[2 * j0: 2 * j0 + 2], K1[2 * j1: 2 * j1 + 2], K2]).astype(np.float64)
        vals = np.concatenate([V[2 * j0: 2 * j0 + 2], V1[2 * j1: 2 * j1 + 2], V2]).astype(np.float64)
        w = np.array([1, 1, 2, 2, 4, 4], np.float64)
        e = w * np.exp(0.5 * keys @ Q[q].astype(np.float64))
        assert np.allclose(r["O"][q], (e / e.sum()) @ vals, atol=1e-12)
        assert abs(r["LSE"][q] - math.log(e.sum())) < 1e-12


# ------------------------------------------------------------ list building

def test_block_counts_printed_in_the_paper(oracle):
    """Sec. 5.3: K=8 attends 8 + 8 + 128^2/16^3 = 20 blocks at 128x128, and 32 at 256x256 (L=2)."""
    rows = [ln.split() for ln in open(os.path.join(HERE, "golden", "block_counts.txt")) if ln.strip() and ln[0] != "#"]
    for N, B, K, L, blocks in ((int(a), int(b), int(c), int(e), int(f)) for a, b, c, e, f in rows):
        g = oracle.Geometry(N, 8, B, K, L)
        assert g.list_len(L) == blocks * B
        # and the list the attention loop really walks has that many entries, no de-duplication
        idx = np.concatenate([np.tile(np.arange(g.K_l(l), dtype=np.int32), g.n(l + 1)) for l in range(L)])
        lev, tok = oracle.kv_list(idx, g, L, block=5)
        assert len(lev) == blocks * B
        assert np.bincount(lev).tolist() == [g.K_l(l) * B for l in range(L)] + [g.n(L)]


def _dense_mask_forward(Qp0, Kp, Vp, I, g, Le, reweight, scale):
    """Second formulation: a dense weight matrix over the concatenated pyramid."""
    N, B, L = g.N, g.B, g.L
    Kcat = np.concatenate(Kp).astype(np.float64)
    Vcat = np.concatenate(Vp).astype(np.float64)
    W = np.zeros((N, Kcat.shape[0]))
    for l in range(Le + 1):
        off = g.pyr_offset(l)
        w = float(B ** l) if reweight else 1.0
        if l < L:
            for i in range(N // B):
                for j in I[l][i // B ** l]:
                    W[i * B:(i + 1) * B, off + j * B: off + (j + 1) * B] = w
        else:
            W[:, off:off + g.n(L)] = w
    S = scale * (Qp0.astype(np.float64) @ Kcat.T)
    E = W * np.exp(S - S.max(axis=1, keepdims=True))
    den = E.sum(axis=1, keepdims=True)
    return (E / den) @ Vcat, np.log(den[:, 0]) + S.max(axis=1)


@pytest.mark.parametrize("Le,reweight", [(3, 1), (3, 0), (1, 1), (0, 1), (2, 0)])
def test_list_gather_equals_dense_mask_formulation(oracle, Le, reweight):
    rng = np.random.default_rng(13)
    g = oracle.Geometry(256, 32, 4, 2, 3)
    Q, Kk, V = (_rand(rng, 256, 32) for _ in range(3))
    r = oracle.forward(Q, Kk, V, g, Le=Le, reweight=reweight)
    O, LSE = _dense_mask_forward(r["Qp"][0], r["Kp"], r["Vp"], r["I"], g, Le, reweight, 1 / math.sqrt(32))
    assert np.allclose(r["O"], O, rtol=0, atol=1e-12)
    assert np.allclose(r["LSE"], LSE, rtol=0, atol=1e-12)


def test_all_blocks_and_no_enrichment_is_dense_softmax_attention(oracle):
    from scipy.special import logsumexp, softmax
    rng = np.random.default_rng(14)
    N, d, B = 64, 16, 4
    g = oracle.Geometry(N, d, B, N // B, 2)                 # K >= blocks at every level
    Q, Kk, V = (_rand(rng, N, d) for _ in range(3))
    r = oracle.forward(Q, Kk, V, g, Le=0)
    S = (Q.astype(np.float64) @ Kk.astype(np.float64).T) / math.sqrt(d)
    assert np.allclose(r["O"], softmax(S, axis=1) @ V.astype(np.float64), atol=1e-12, rtol=0)
    assert np.allclose(r["LSE"], logsumexp(S, axis=1), atol=1e-12, rtol=0)
    # rows of P sum to one  <=>  O of a constant V is that constant; O is linear in V
    r1 = oracle.forward(Q, Kk, np.ones_like(V), g, Le=0)
    assert np.allclose(r1["O"], 1.0, atol=1e-12)


def test_output_is_linear_in_v_and_rows_sum_to_one_with_enrichment(oracle):
    rng = np.random.default_rng(15)
    g = oracle.Geometry(256, 8, 4, 2, 3)
    Q, Kk, V1, V2 = (_rand(rng, 256, 8) for _ in range(4))
    base = oracle.forward(Q, Kk, V1, g)
    Kp, idx = oracle.cat_pyramid(base["Kp"]), base["idx_cat"]
    pyr = lambda v: np.concatenate([a.astype(np.float64) for a in (  # exact fp64 pyramid
        [v] + [v.reshape(-1, 4 ** l, 8).mean(1) for l in (1, 2, 3)])])
    o1, _ = oracle.attn_fwd(Q, Kp, pyr(V1.astype(np.float64)), idx, g, 3)
    o2, _ = oracle.attn_fwd(Q, Kp, pyr(V2.astype(np.float64)), idx, g, 3)
    o12, _ = oracle.attn_fwd(Q, Kp, pyr(2.0 * V1 - 3.0 * V2.astype(np.float64)), idx, g, 3)
    assert np.allclose(o12, 2 * o1 - 3 * o2, atol=1e-11)
    one, _ = oracle.attn_fwd(Q, Kp, np.ones_like(Kp), idx, g, 3)
    assert np.allclose(one, 1.0, atol=1e-12)


def test_reweighting_is_multiplicity(oracle):
    """If K and V are constant over aligned runs of B^L tokens every coarse token equals its descendants, and a
    level-l token of weight B^l must act exactly like its B^l fine descendants (the paper's nearest-upsample
    argument, Sec. 4.1 'KV Reweighting'): the output equals dense attention with integer multiplicities."""
    rng = np.random.default_rng(16)
    N, d, B, K, L = 256, 8, 4, 2, 3
    g = oracle.Geometry(N, d, B, K, L)
    run = B ** L
    Q = _rand(rng, N, d)
    Kk = np.repeat(oracle.to_bf16(_rand(rng, N // run, d)), run, axis=0)   # short mantissas: pooling is exact
    V = np.repeat(oracle.to_bf16(_rand(rng, N // run, d)), run, axis=0)
    r = oracle.forward(Q, Kk, V, g)
    for l in range(1, L + 1):
        assert np.array_equal(r["Kp"][l], Kk[:: B ** l])
    S = (Q.astype(np.float64) @ Kk.astype(np.float64).T) / math.sqrt(d)
    for blk in (0, 7, 33, 63):
        lev, tok = oracle.kv_list(r["idx_cat"], g, L, blk)
        mult = np.zeros(N)
        for l, t in zip(lev, tok):
            mult[t * B ** l:(t + 1) * B ** l] += 1          # fine descendants of the listed token
        for q in range(blk * B, (blk + 1) * B):
            e = mult * np.exp(S[q] - S[q].max())
            assert np.allclose(r["O"][q], (e / e.sum()) @ V.astype(np.float64), atol=1e-12)
            assert abs(r["LSE"][q] - (math.log(e.sum()) + S[q].max())) < 1e-12
    # without reweighting the identity must fail (the pin is sensitive to the weight)
    r0 = oracle.forward(Q, Kk, V, g, reweight=0)
    assert np.abs(r0["O"] - r["O"]).max() > 1e-3


def test_literal_scaling_reading_is_scaled_keys_and_values(oracle):
    """The switch reweight = 2 is the literal reading of Alg. 1's enrichment loop: level-l keys and values are
    multiplied by B^l before plain (unweighted) attention over the list.  Checked against exactly that, written
    with the dense-mask formulation on pre-scaled pyramids; it is not the default and differs from it."""
    rng = np.random.default_rng(17)
    g = oracle.Geometry(64, 8, 4, 2, 2)
    Q, Kk, V = (_rand(rng, 64, 8) for _ in range(3))
    a = oracle.forward(Q, Kk, V, g, reweight=1)
    b = oracle.forward(Q, Kk, V, g, reweight=2)
    assert np.abs(a["O"] - b["O"]).max() > 1e-2
    Ks = [x.astype(np.float64) * 4.0 ** l for l, x in enumerate(b["Kp"])]
    Vs = [x.astype(np.float64) * 4.0 ** l for l, x in enumerate(b["Vp"])]
    O, LSE = _dense_mask_forward(b["Qp"][0], Ks, Vs, b["I"], g, 2, 0, 1 / math.sqrt(8))
    assert np.allclose(b["O"], O, atol=1e-10) and np.allclose(b["LSE"], LSE, atol=1e-10)


def test_query_sub_range_is_a_slice_of_the_full_call(oracle):
    """attn_fwd(rows=(a, b)) computes exactly rows a..b-1 of the full call (every large-shape parity test relies
    on it), also for ranges that start and end inside a query block."""
    rng = np.random.default_rng(23)
    g = oracle.Geometry(256, 16, 4, 2, 3)
    Q, Kk, V = (_rand(rng, 256, 16) for _ in range(3))
    f = oracle.forward(Q, Kk, V, g)
    Kc, Vc = oracle.cat_pyramid(f["Kp"]), oracle.cat_pyramid(f["Vp"])
    for a, b in ((0, 256), (0, 1), (5, 23), (100, 163), (255, 256)):
        O, LSE = oracle.attn_fwd(Q, Kc, Vc, f["idx_cat"], g, 3, rows=(a, b))
        assert np.array_equal(O[a:b], f["O"][a:b]) and np.array_equal(LSE[a:b], f["LSE"][a:b])
        assert np.isnan(O[:a]).all() and np.isnan(O[b:]).all()


def test_backward_shares_of_a_row_partition_sum_to_the_full_gradients(oracle):
    """attn_bwd(rows=(a, b)) is the share of query rows a..b-1: its dQ has those rows of the full dQ and zeros
    elsewhere, and the dK / dV shares of a partition add up to the full gradients (to fp64 summation order)."""
    rng = np.random.default_rng(24)
    g = oracle.Geometry(256, 16, 4, 2, 3)
    Q, Kk, V = (_rand(rng, 256, 16) for _ in range(3))
    dO = rng.standard_normal((256, 16))
    f = oracle.forward(Q, Kk, V, g)
    Kc, Vc = oracle.cat_pyramid(f["Kp"]), oracle.cat_pyramid(f["Vp"])
    full = oracle.attn_bwd(Q, Kc, Vc, f["idx_cat"], dO, g, 3)
    cuts = [0, 7, 64, 65, 200, 256]
    acc = [np.zeros_like(x) for x in full]
    for a, b in zip(cuts[:-1], cuts[1:]):
        part = oracle.attn_bwd(Q, Kc, Vc, f["idx_cat"], dO, g, 3, rows=(a, b))
        assert np.array_equal(part[0][a:b], full[0][a:b])
        assert not part[0][:a].any() and not part[0][b:].any()
        for s_, p_ in zip(acc, part):
            s_ += p_
    for s_, f_ in zip(acc, full):
        assert np.allclose(s_, f_, rtol=0, atol=1e-12 * max(1.0, np.abs(f_).max()))
    # and a share is not the whole: the pin is sensitive to the range being honoured
    assert np.abs(oracle.attn_bwd(Q, Kc, Vc, f["idx_cat"], dO, g, 3, rows=(0, 64))[1] - full[1]).max() > 1e-3


# ---------------------------------------------------------------- gradients

def _pyr64(x, B, L):
    out = [x]
    for _ in range(L):
        out.append(out[-1].reshape(-1, B, x.shape[1]).mean(axis=1))
    return out


def test_gradients_match_finite_differences(oracle):
    """Config 0 shape; indices frozen; covers the path through the pooled coarse tokens."""
    rng = np.random.default_rng(18)
    N, d, B, K, L = 256, 32, 4, 2, 3
    g = oracle.Geometry(N, d, B, K, L)
    Q, Kk, V = (_rand(rng, N, d) for _ in range(3))
    dO = rng.standard_normal((N, d))
    fwd = oracle.forward(Q, Kk, V, g)
    idx = fwd["idx_cat"]
    x = {"Q": Q.astype(np.float64), "K": Kk.astype(np.float64), "V": V.astype(np.float64)}

    def loss(xs):
        O, _ = oracle.attn_fwd(xs["Q"], np.concatenate(_pyr64(xs["K"], B, L)), np.concatenate(_pyr64(xs["V"], B, L)),
                               idx, g, L)
        return float((O * dO).sum())

    grads = oracle.backward(x["Q"], _pyr64(x["K"], B, L), _pyr64(x["V"], B, L), idx, dO, g)
    eps = 1e-5
    for name, gname in (("Q", "dQ"), ("K", "dK"), ("V", "dV")):
        for _ in range(12):
            t, c = int(rng.integers(N)), int(rng.integers(d))
            xp = {k: v.copy() for k, v in x.items()}
            xm = {k: v.copy() for k, v in x.items()}
            xp[name][t, c] += eps
            xm[name][t, c] -= eps
            fd = (loss(xp) - loss(xm)) / (2 * eps)
            an = grads[gname][t, c]
            assert abs(fd - an) <= 1e-6 * max(1.0, abs(an)), (name, t, c, fd, an)


def test_full_k_gradients_are_dense_attention_gradients(oracle):
    rng = np.random.default_rng(19)
    N, d, B = 64, 16, 4
    g = oracle.Geometry(N, d, B, N // B, 2)
    Q, Kk, V = (rng.standard_normal((N, d)) for _ in range(3))
    dO = rng.standard_normal((N, d))
    idx = np.concatenate([np.tile(np.arange(g.K_l(l), dtype=np.int32), g.n(l + 1)) for l in range(g.L)])
    grads = oracle.backward(Q, _pyr64(Kk, B, 2), _pyr64(V, B, 2), idx, dO, g, Le=0)
    sc = 1 / math.sqrt(d)
    S = sc * Q @ Kk.T
    P = np.exp(S - S.max(1, keepdims=True))
    P /= P.sum(1, keepdims=True)
    dP = dO @ V.T
    dS = P * (dP - (dP * P).sum(1, keepdims=True))
    assert np.allclose(grads["dQ"], sc * dS @ Kk, atol=1e-12)
    assert np.allclose(grads["dK"], sc * dS.T @ Q, atol=1e-12)
    assert np.allclose(grads["dV"], P.T @ dO, atol=1e-12)


def test_gradient_sum_invariants(oracle):
    """sum_t dV[t] = sum_q dO[q] (rows of P sum to one; pooling adjoint preserves sums); sum over keys of dS is 0
    so sum_t dK[t] . x = 0 when all queries are equal to x... checked here in the simpler form sum_c dQ.q = sum dK.k."""
    rng = np.random.default_rng(20)
    g = oracle.Geometry(256, 16, 4, 2, 3)
    Q, Kk, V = (_rand(rng, 256, 16) for _ in range(3))
    dO = rng.standard_normal((256, 16))
    f = oracle.forward(Q, Kk, V, g)
    b = oracle.backward(Q, f["Kp"], f["Vp"], f["idx_cat"], dO, g)
    assert np.allclose(b["dV"].sum(0), dO.sum(0), atol=1e-10)
    # Euler identity: the logits are bilinear in (Q, K-pyramid), so <dQ, Q> = <dKpyr, Kpyr>
    lhs = float((b["dQ"] * Q).sum())
    rhs = float((b["dKpyr"] * oracle.cat_pyramid(f["Kp"])).sum())
    assert abs(lhs - rhs) < 1e-9 * max(1.0, abs(lhs))


# ------------------------------------------------------------ index transpose

def test_transpose_is_exact_and_involutive(oracle):
    rng = np.random.default_rng(21)
    T, K = 97, 5
    I = np.stack([np.sort(rng.choice(T, K, replace=False)) for _ in range(T)]).astype(np.int32)
    Iq, C = oracle.transpose(I, T)
    assert C[0] == 0 and C[-1] == T * K and np.all(np.diff(C) >= 0)
    pairs = set()
    for key in range(T):
        seg = Iq[C[key]:C[key + 1]]
        assert np.all(np.diff(seg) > 0)                     # ascending query rows, each once
        for r in seg:
            assert key in I[r]
            pairs.add((int(r), key))
    assert len(pairs) == T * K
    # brute-force inverse lists
    for key in range(T):
        assert np.array_equal(Iq[C[key]:C[key + 1]], np.nonzero((I == key).any(axis=1))[0])
    # transposing the transposed lists (as ragged CSR) gives back the original rows
    back = [[] for _ in range(T)]
    for key in range(T):
        for r in Iq[C[key]:C[key + 1]]:
            back[r].append(key)
    assert np.array_equal(np.array(back, np.int32), I)


# ------------------------------------------------------------ index reordering (Sec. 5.1)

def test_index_reordering_groups_every_patch_size(oracle):
    """For every i, each aligned run of 4**i tokens is exactly one aligned 2**i x 2**i patch of pixels."""
    W = 32
    order = oracle.nested_order(W)
    assert np.array_equal(np.sort(order), np.arange(W * W))         # a permutation of the pixels
    y, x = order // W, order % W
    for i in range(0, 6):
        side, run = 2 ** i, 4 ** i
        for t0 in range(0, W * W, run):
            ys, xs = y[t0:t0 + run], x[t0:t0 + run]
            assert ys.min() % side == 0 and xs.min() % side == 0
            assert ys.max() - ys.min() == side - 1 and xs.max() - xs.min() == side - 1
            assert len(set(zip(ys.tolist(), xs.tolist()))) == run


def test_index_reordering_is_bit_deinterleaving(oracle):
    """Closed form of the same order: token t's pixel has the even bits of t as x and the odd bits as y."""
    W = 64
    order = oracle.nested_order(W)
    t = np.arange(W * W)
    xs = sum(((t >> (2 * b)) & 1) << b for b in range(6))
    ys = sum(((t >> (2 * b + 1)) & 1) << b for b in range(6))
    assert np.array_equal(order, ys * W + xs)
    # the 4 x 4 case written out by hand
    assert oracle.nested_order(4).tolist() == [0, 1, 4, 5, 2, 3, 6, 7, 8, 9, 12, 13, 10, 11, 14, 15]


def test_index_reordering_round_trip_and_pooling_meaning(oracle):
    rng = np.random.default_rng(23)
    W, d = 16, 8
    x = rng.standard_normal((W * W, d)).astype(np.float32)
    r = oracle.reorder(x)
    assert np.array_equal(oracle.reorder(r, inverse=True), x)
    assert not np.array_equal(r, x)
    # pooling 16 consecutive reordered tokens = the mean over a 4 x 4 pixel patch of the raster image
    pooled = oracle.pool(r, 16, False)
    img = x.reshape(W, W, d).astype(np.float64)
    for py in range(W // 4):
        for px in range(W // 4):
            want = img[4 * py:4 * py + 4, 4 * px:4 * px + 4].reshape(16, d).mean(axis=0)
            t = int(np.nonzero(oracle.nested_order(W) == (4 * py) * W + 4 * px)[0][0]) // 16
            assert np.allclose(pooled[t], want, rtol=0, atol=1e-6)


# ------------------------------------------------------ layer glue: QK-Norm and RoPE (Sec. 5.2, "Training Settings")

def test_qknorm_is_unit_rms_and_scale_invariant(oracle):
    """With unit gain and zero angles every token comes out with root mean square 1 (eps aside), whatever its
    input scale; the gain multiplies channel-wise."""
    rng = np.random.default_rng(31)
    N, d = 64, 32
    x = rng.standard_normal((N, d)) * rng.uniform(0.1, 30.0, (N, 1))
    one, c, s = np.ones(d), np.ones((N, d // 2)), np.zeros((N, d // 2))
    y = oracle.qknorm_rope(x, one, c, s, eps=0.0)
    assert np.allclose(np.sqrt((y * y).mean(1)), 1.0, atol=1e-12)
    assert np.allclose(oracle.qknorm_rope(7.5 * x, one, c, s, eps=0.0), y, atol=1e-12)
    g = rng.uniform(0.5, 2.0, d)
    assert np.allclose(oracle.qknorm_rope(x, g, c, s, eps=0.0), y * g, atol=1e-12)
    # eps sits under the root, added to the mean square: a zero token stays zero, a tiny one is damped
    assert not oracle.qknorm_rope(np.zeros((N, d)), one, c, s, eps=1e-6).any()
    tiny = np.full((1, d), 1e-3)
    assert np.allclose(oracle.qknorm_rope(tiny, one, c[:1], s[:1], eps=1e-6), 1e-3 / math.sqrt(1e-6 + 1e-6), atol=1e-12)


def test_rope_rotates_adjacent_pairs(oracle):
    """Quarter turn: (a, b) -> (-b, a); the rotation keeps every pair's length; it acts on pairs (2i, 2i+1)."""
    rng = np.random.default_rng(32)
    N, d = 16, 8
    x = rng.standard_normal((N, d))
    x /= np.sqrt((x * x).mean(1, keepdims=True))            # already unit RMS: the norm leaves it alone
    one = np.ones(d)
    q = oracle.qknorm_rope(x, one, np.zeros((N, d // 2)), np.ones((N, d // 2)), eps=0.0)
    assert np.allclose(q[:, 0::2], -x[:, 1::2], atol=1e-12) and np.allclose(q[:, 1::2], x[:, 0::2], atol=1e-12)
    ang = rng.uniform(0, 2 * math.pi, (N, d // 2))
    r = oracle.qknorm_rope(x, one, np.cos(ang), np.sin(ang), eps=0.0)
    assert np.allclose(r[:, 0::2] ** 2 + r[:, 1::2] ** 2, x[:, 0::2] ** 2 + x[:, 1::2] ** 2, atol=1e-12)
    z = x[:, 0::2] + 1j * x[:, 1::2]                         # the same rotation as a complex product
    w = z * np.exp(1j * ang)
    assert np.allclose(r[:, 0::2], w.real, atol=1e-12) and np.allclose(r[:, 1::2], w.imag, atol=1e-12)


def test_rope_scores_depend_on_relative_position_only(oracle):
    """The defining property of the rotary embedding: with 1-D position tables, the score of a query at position m
    and a key at position n depends on m - n only (same vectors, shifted positions, same score)."""
    from paper_2512_16615_amd import inputs
    rng = np.random.default_rng(33)
    d, N = 16, 24                                           # 24 is no square: the tables are 1-D
    cos, sin = inputs.rope_tables(N, d)
    qv, kv = rng.standard_normal(d), rng.standard_normal(d)
    Q = np.tile(qv, (N, 1))
    Kk = np.tile(kv, (N, 1))
    one = np.ones(d)
    S = oracle.qknorm_rope(Q, one, cos, sin, 0.0) @ oracle.qknorm_rope(Kk, one, cos, sin, 0.0).T
    for off in (-5, 0, 3):
        diag = np.diagonal(S, offset=off)
        assert np.allclose(diag, diag[0], atol=1e-5)          # fp32 tables
    assert abs(S[0, 5] - S[5, 0]) > 1e-3                     # and it does depend on the sign of the offset


def test_rope_tables_are_axial_on_a_pixel_grid():
    """On a W x W grid the first half of the pairs turns with the row, the second half with the column."""
    from paper_2512_16615_amd import inputs
    W, d = 8, 16
    cos, sin = inputs.rope_tables(W * W, d)
    ang = np.arctan2(sin.astype(np.float64), cos.astype(np.float64)).reshape(W, W, d // 2)
    assert np.allclose(ang[:, 0, : d // 4], ang[:, 5, : d // 4], atol=1e-6)        # row pairs ignore the column
    assert np.allclose(ang[0, :, d // 4:], ang[6, :, d // 4:], atol=1e-6)          # column pairs ignore the row
    assert np.allclose(ang[1, 0, 0], 1.0, atol=1e-6) and np.allclose(ang[0, 1, d // 4], 1.0, atol=1e-6)


def test_glue_then_pool_is_mean_of_the_glued_block(oracle):
    """The fused step is the glue followed by the compression loop's first step: nothing else."""
    from paper_2512_16615_amd import inputs
    rng = np.random.default_rng(34)
    N, d, B = 64, 16, 4
    x = rng.standard_normal((N, d)).astype(np.float32)
    cos, sin = inputs.rope_tables(N, d)
    y = oracle.qknorm_rope(x, np.ones(d), cos, sin).astype(np.float32)
    assert np.allclose(oracle.pool(y, B, False), y.reshape(N // B, B, d).mean(1), atol=1e-6)
