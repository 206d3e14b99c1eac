"""Pins for the CPU oracle: each oracle function is checked against something
other than itself -- closed forms, invariants, library routines, brute force, a
second formulation with dense one-hot matrices, or a figure the paper prints
(tests/golden/paper_constants.txt)."""
import math
import os

import numpy as np
import pytest
import torch

from oracle import kvr_oracle as O

HERE = os.path.dirname(os.path.abspath(__file__))


def golden():
    out = {}
    with open(os.path.join(HERE, "golden", "paper_constants.txt")) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                k, v = line.split("=")
                out[k.strip()] = float(v)
    return out


def rand_params(rng, r):
    return [(int(rng.integers(0, 2 ** 63)) * 2 + 1, int(rng.integers(0, 2 ** 63)),
             int(rng.integers(0, 2 ** 63)) * 2 + 1, int(rng.integers(0, 2 ** 63))) for _ in range(r)]


# ------------------------------------------------------------------ hash / sign
def test_bucket_closed_forms():
    w = 273
    # a = 2^32, b = 0: the high word of a*J is J itself, so h = floor(J*w / 2^32)
    for J in [0, 1, 7, 12345, 2 ** 31 - 1, 2 ** 32 - 1]:
        assert O.bucket_of((1 << 32, 0, 1, 0), J, w) == (J * w) // (1 << 32)
    # a = 1, b = 0: high word is 0 for J < 2^32
    assert O.bucket_of((1, 0, 1, 0), 123456, w) == 0
    # a = 2^63: high word is 2^31 for odd J, 0 for even J
    assert O.bucket_of((1 << 63, 0, 1, 0), 5, w) == w // 2
    assert O.bucket_of((1 << 63, 0, 1, 0), 6, w) == 0
    # b only: h = floor((b >> 32) * w / 2^32); wrap-around of a*J + b is modulo 2^64
    b = 0xFFFFFFFF00000000
    assert O.bucket_of((1, b, 1, 0), 0, w) == w - 1
    assert O.bucket_of((1 << 32, b, 1, 0), 1, w) == 0          # wraps to 0
    # sign: top bit of c*J + d
    assert O.sign_of((1, 0, 1, 0), 5) == 1
    assert O.sign_of((1, 0, 1, 1 << 63), 5) == -1
    assert O.sign_of((1, 0, 1 << 63, 0), 3) == -1
    assert O.sign_of((1, 0, 1 << 63, 0), 4) == 1
    assert O.sign_of((1, 0, 1 << 63, 1 << 63), 3) == 1          # wraps


def test_bucket_range_uniformity_and_sign_balance():
    params = O.hash_params_from_seed(2512, 3)
    w = 37
    n = 37 * 400
    for i in range(3):
        hs = np.array([O.bucket_of(params[i], J, w) for J in range(n)])
        gs = np.array([O.sign_of(params[i], J) for J in range(n)])
        assert hs.min() >= 0 and hs.max() < w
        assert set(np.unique(gs)) == {-1, 1}
        counts = np.bincount(hs, minlength=w)
        chi2 = ((counts - n / w) ** 2 / (n / w)).sum()
        # multiply-shift over consecutive J spreads more evenly than chance; it
        # must in any case not be worse than a random assignment's 99.9% point
        assert chi2 < 70.0
        assert abs(gs.mean()) < 0.05
    # rows are distinct functions
    h0 = [O.bucket_of(params[0], J, w) for J in range(500)]
    h1 = [O.bucket_of(params[1], J, w) for J in range(500)]
    assert h0 != h1


def test_hash_params_lcg():
    rows = O.hash_params_from_seed(0, 2)
    # first LCG state from seed 0 is the increment itself
    assert rows[0][0] == (1442695040888963407 | 1)
    x = 1442695040888963407
    x2 = (x * 6364136223846793005 + 1442695040888963407) % (1 << 64)
    assert rows[0][1] == x2
    for (a, b, c, d) in rows:
        assert a & 1 and c & 1
        assert all(0 <= v < (1 << 64) for v in (a, b, c, d))
    assert O.hash_params_from_seed(5, 3)[:2] == O.hash_params_from_seed(5, 2)
    assert O.hash_params_from_seed(5, 3) != O.hash_params_from_seed(6, 3)


# ------------------------------------------------------------------ storage rounding
def test_to_storage_matches_torch_bf16():
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.standard_normal(20000) * 10 ** rng.uniform(-6, 6, 20000),
                        [0.0, -0.0, 1.0, 1.00390625, 1.01171875, 257.0, 0.1]])
    # float32 path
    got = O.to_storage(x.astype(np.float32), "bf16")
    want = torch.tensor(x.astype(np.float32)).to(torch.bfloat16).double().numpy()
    assert np.array_equal(got, want)
    # float64 path rounds once, from the float64 value: exact ties go to even
    tie = 1.0 + 2.0 ** -8          # halfway between bf16 1.0 and 1.0078125
    assert O.to_storage(np.array([tie]), "bf16")[0] == 1.0
    assert O.to_storage(np.array([tie + 2.0 ** -40]), "bf16")[0] == 1.0078125
    assert O.to_storage(np.array([1.0078125 + 2.0 ** -8]), "bf16")[0] == 1.015625
    # on values that are float32-exact the two paths agree
    x32 = x.astype(np.float32)
    assert np.array_equal(O.to_storage(x32.astype(np.float64), "bf16"), got)
    assert np.array_equal(O.to_storage(x, "f32"), x.astype(np.float32).astype(np.float64))


# ------------------------------------------------------------------ insert
def small_int_tokens(rng, n, D):
    return rng.integers(-8, 9, size=(n, D)).astype(np.float64)


def test_insert_linearity_and_mass():
    rng = np.random.default_rng(1)
    r, w, D = 3, 5, 16
    params = rand_params(rng, r)
    pos = rng.choice(10000, size=40, replace=False)
    K, V = small_int_tokens(rng, 40, D), small_int_tokens(rng, 40, D)
    Z = O.sketch_zeros(r, w, D)
    # sketch(A u B) = sketch(A) + sketch(B)   (integer data: every sum is exact)
    SKa, SVa = O.insert(*Z, params, pos[:25], K[:25], V[:25])
    SKb, SVb = O.insert(*Z, params, pos[25:], K[25:], V[25:])
    SKab, SVab = O.insert(*Z, params, pos, K, V)
    assert np.array_equal(SKab, SKa + SKb) and np.array_equal(SVab, SVa + SVb)
    # inserting B into sketch(A) is the same thing
    SKc, SVc = O.insert(SKa, SVa, params, pos[25:], K[25:], V[25:])
    assert np.array_equal(SKc, SKab) and np.array_equal(SVc, SVab)
    # homogeneity and order independence (exact data)
    SK3, SV3 = O.insert(*Z, params, pos, 3 * K, 3 * V)
    assert np.array_equal(SK3, 3 * SKab) and np.array_equal(SV3, 3 * SVab)
    perm = rng.permutation(40)
    SKp, SVp = O.insert(*Z, params, pos[perm], K[perm], V[perm])
    assert np.array_equal(SKp, SKab) and np.array_equal(SVp, SVab)
    # keys are unsigned: every row holds the whole key mass; values carry g_i(J)
    for i in range(r):
        assert np.array_equal(SKab[i].sum(axis=0), K.sum(axis=0))
        g = np.array([O.sign_of(params[i], int(J)) for J in pos], dtype=np.float64)
        assert np.array_equal(SVab[i].sum(axis=0), (g[:, None] * V).sum(axis=0))
    # zero tokens leave zeros; one token touches exactly r slots per tensor
    SK0, SV0 = O.insert(*Z, params, pos[:5], np.zeros((5, D)), np.zeros((5, D)))
    assert not SK0.any() and not SV0.any()
    SK1, SV1 = O.insert(*Z, params, pos[:1], np.ones((1, D)), np.ones((1, D)))
    assert (np.abs(SK1).sum(axis=2) > 0).sum() == r and (np.abs(SV1).sum(axis=2) > 0).sum() == r
    for i in range(r):
        s = O.bucket_of(params[i], int(pos[0]), w)
        assert np.array_equal(SK1[i, s], np.ones(D))
        assert np.array_equal(SV1[i, s], O.sign_of(params[i], int(pos[0])) * np.ones(D))


def test_insert_sign_mask_variants():
    rng = np.random.default_rng(2)
    r, w, D = 3, 4, 8
    params = rand_params(rng, r)
    pos = np.arange(10)
    K, V = small_int_tokens(rng, 10, D), small_int_tokens(rng, 10, D)
    Z = O.sketch_zeros(r, w, D)
    SK_p, SV_p = O.insert(*Z, params, pos, K, V, sign_mask=2)     # the paper's setting
    SK_b, SV_b = O.insert(*Z, params, pos, K, V, sign_mask=3)
    SK_n, SV_n = O.insert(*Z, params, pos, K, V, sign_mask=0)
    assert np.array_equal(SV_p, SV_b) and np.array_equal(SK_p, SK_n)
    # signing the keys is the same as inserting them as values
    SK_sw, SV_sw = O.insert(*Z, params, pos, V, K, sign_mask=2)
    assert np.array_equal(SK_b, SV_sw)


def test_insert_rounding_once_per_slot_in_list_order():
    # three tokens into one slot (w = 1): stored value = RNE_bf16 of the whole sum,
    # not of partial sums
    params = [(1, 0, 1, 0)]
    Z = O.sketch_zeros(1, 1, 1)
    k = np.array([[1.0], [2.0 ** -8], [2.0 ** -8]])
    SK, _ = O.insert(*Z, params, [0, 1, 2], k, k, storage="bf16")
    assert SK[0, 0, 0] == 1.0078125          # 1 + 2^-7 exactly representable
    # one at a time, each call rounds: 1 + 2^-8 ties to even (1.0) twice
    SKs, SVs = Z
    for j in range(3):
        SKs, SVs = O.insert(SKs, SVs, params, [j], k[j:j + 1], k[j:j + 1], storage="bf16")
    assert SKs[0, 0, 0] == 1.0
    # float32 accumulation follows list order: (2^24 + 1) + 1 in float32 stays 2^24 + 0 -> then +1
    big = np.array([[2.0 ** 24], [1.0], [1.0]])
    A, _ = O.insert(*Z, params, [0, 1, 2], big, big, storage="f32", acc_dtype=np.float32)
    B, _ = O.insert(*Z, params, [1, 2, 0], big[[1, 2, 0]], big[[1, 2, 0]], storage="f32",
                    acc_dtype=np.float32)
    assert A[0, 0, 0] == 2.0 ** 24 and B[0, 0, 0] == 2.0 ** 24 + 2


# ------------------------------------------------------------------ query
def injective_positions(params, w, n, r_needed, limit=200000):
    """Greedy search for n positions such that each is alone in its slot in at
    least r_needed rows (w >= n makes this easy)."""
    r = len(params)
    used = [set() for _ in range(r)]
    out = []
    for J in range(limit):
        hs = [O.bucket_of(params[i], J, w) for i in range(r)]
        if all(hs[i] not in used[i] for i in range(r)):
            out.append(J)
            for i in range(r):
                used[i].add(hs[i])
            if len(out) == n:
                return out
    raise RuntimeError("not found")


@pytest.mark.parametrize("storage", ["f64", "f32", "bf16"])
def test_query_exact_without_collisions(storage):
    rng = np.random.default_rng(3)
    r, w, D, n = 3, 64, 32, 40
    params = O.hash_params_from_seed(99, r)
    pos = injective_positions(params, w, n, r)
    K = O.to_storage(rng.standard_normal((n, D)), storage)
    V = O.to_storage(rng.standard_normal((n, D)), storage)
    SK, SV = O.insert(*O.sketch_zeros(r, w, D), params, pos, K, V, storage=storage)
    Kh, Vh = O.query(SK, SV, params, pos, storage=storage)
    assert np.array_equal(Kh, K) and np.array_equal(Vh, V)


def test_query_exact_when_majority_of_rows_is_clean():
    # add one more token that collides with token 0 in exactly one row: the median
    # of three still returns token 0 exactly
    rng = np.random.default_rng(4)
    r, w, D, n = 3, 64, 8, 10
    params = O.hash_params_from_seed(7, r)
    pos = injective_positions(params, w, n, r)
    h0 = [O.bucket_of(params[i], pos[0], w) for i in range(r)]
    others = [set(O.bucket_of(params[i], p, w) for p in pos[1:]) for i in range(r)]
    extra = None
    for J in range(100000):
        if J in pos:
            continue
        hs = [O.bucket_of(params[i], J, w) for i in range(r)]
        if sum(hs[i] == h0[i] for i in range(r)) == 1 and all(hs[i] not in others[i] for i in range(r)):
            extra = J
            break
    assert extra is not None
    K = rng.standard_normal((n + 1, D))
    V = rng.standard_normal((n + 1, D))
    SK, SV = O.insert(*O.sketch_zeros(r, w, D), params, pos + [extra], K, V)
    Kh, Vh = O.query(SK, SV, params, pos, storage="f64")
    assert np.array_equal(Kh, K[:n]) and np.array_equal(Vh, V[:n])


def test_query_single_row_and_brute_force_median():
    rng = np.random.default_rng(5)
    D = 6
    # r = 1: the (signed) slot itself
    params = rand_params(rng, 1)
    pos = [3, 11, 40]
    K, V = rng.standard_normal((3, D)), rng.standard_normal((3, D))
    SK, SV = O.insert(*O.sketch_zeros(1, 2, D), params, pos, K, V)
    Kh, Vh = O.query(SK, SV, params, pos)
    for t, J in enumerate(pos):
        s = O.bucket_of(params[0], J, 2)
        assert np.array_equal(Kh[t], SK[0, s])
        assert np.array_equal(Vh[t], SV[0, s] * O.sign_of(params[0], J))
    # r = 3, heavy collisions: element-wise sorted()[1]
    params = rand_params(rng, 3)
    pos = list(range(50))
    K, V = rng.standard_normal((50, D)), rng.standard_normal((50, D))
    SK, SV = O.insert(*O.sketch_zeros(3, 4, D), params, pos, K, V)
    Kh, Vh = O.query(SK, SV, params, pos)
    for t in (0, 17, 49):
        J = pos[t]
        for c in range(D):
            ks = sorted(SK[i, O.bucket_of(params[i], J, 4), c] for i in range(3))
            vs = sorted(SV[i, O.bucket_of(params[i], J, 4), c] * O.sign_of(params[i], J) for i in range(3))
            assert Kh[t, c] == ks[1] and Vh[t, c] == vs[1]


def test_median_even_rows():
    res = np.array([[[4.0], [1.0], [3.0], [2.0]]])
    assert O.median_rows(res, "midmean")[0, 0] == 2.5
    assert O.median_rows(res, "lower")[0, 0] == 2.0
    assert O.median_rows(res, "midmean")[0, 0] == np.median(res[0, :, 0])
    # midmean is rounded to storage
    res = np.array([[[1.0], [1.0078125], [0.0], [9.0]]])
    assert O.median_rows(res, "midmean", "bf16")[0, 0] == 1.0     # 1.00390625 ties to even
    r5 = np.random.default_rng(0).standard_normal((7, 5, 3))
    assert np.array_equal(O.median_rows(r5), np.median(r5, axis=1))


def test_query_statistics_match_lemma2_and_unbiasedness():
    """iid N(0,1) data: per-row estimation error has variance (a-1)/w; the median
    of the three rows cuts it by the factor the paper prints in Lemma 2 (0.448;
    exactly 1 - sqrt(3)/pi); the value estimate is unbiased, the key estimate of
    iid zero-mean keys too."""
    g = golden()
    rng = np.random.default_rng(6)
    r, w, D, a = 3, 40, 64, 4000
    ratios, row_vars, v_bias = [], [], []
    for trial in range(3):
        params = O.hash_params_from_seed(1000 + trial, r)
        pos = rng.choice(1 << 20, size=a, replace=False)
        K, V = rng.standard_normal((a, D)), rng.standard_normal((a, D))
        SK, SV = O.insert(*O.sketch_zeros(r, w, D), params, pos, K, V)
        Kh, Vh = O.query(SK, SV, params, pos)
        s0 = np.array([O.bucket_of(params[0], int(J), w) for J in pos])
        g0 = np.array([O.sign_of(params[0], int(J)) for J in pos], dtype=np.float64)
        row_err = SV[0][s0] * g0[:, None] - V
        row_vars.append(row_err.var())
        ratios.append(((Vh - V).var() / row_err.var(), (Kh - K).var() / (SK[0][s0] - K).var()))
        v_bias.append((Vh - V).mean())
    assert abs(np.mean(row_vars) / ((a - 1) / w) - 1) < 0.05
    rv, rk = np.mean([x[0] for x in ratios]), np.mean([x[1] for x in ratios])
    exact = 1 - math.sqrt(3) / math.pi
    assert abs(g["median3_normal_variance_ratio"] - exact) < 1e-3      # the printed figure
    assert abs(rv - exact) < 0.03 and abs(rk - exact) < 0.03
    assert rv < g["median3_variance_upper_ratio"]
    assert abs(np.mean(v_bias)) < 0.05 * math.sqrt((a - 1) / w)


def test_query_tail_bound():
    """Mathematical Analysis: P(Var(median) > a*pi/S * sigma^2) < exp(-a/S), S = r*w."""
    rng = np.random.default_rng(7)
    r, w, D, a = 3, 50, 128, 300
    S = r * w
    params = O.hash_params_from_seed(5, r)
    pos = rng.choice(1 << 20, size=a, replace=False)
    K, V = rng.standard_normal((a, D)), rng.standard_normal((a, D))
    SK, SV = O.insert(*O.sketch_zeros(r, w, D), params, pos, K, V)
    Kh, Vh = O.query(SK, SV, params, pos)
    for est, ref in ((Kh, K), (Vh, V)):
        per_token_var = ((est - ref) ** 2).mean(axis=1)      # D channels share the collisions
        frac = (per_token_var > a * math.pi / S).mean()
        assert frac < math.exp(-a / S)


# ------------------------------------------------------------------ select
def brute_select(scores, ret_pos, n_ctx, n_recent, k):
    pos = np.asarray(ret_pos)
    slots = np.nonzero((pos >= 0) & (pos < n_ctx - n_recent))[0]
    if len(slots) == 0:
        return np.zeros(0, dtype=np.int64)
    sc = np.asarray(scores, dtype=np.float64)[pos[slots]]
    order = np.lexsort((pos[slots], -sc))            # last key is primary
    keep = set(slots[order[:max(k, 0)]].tolist())
    return np.array(sorted(s for s in slots.tolist() if s not in keep), dtype=np.int64)


def test_select_against_lexsort_and_edges():
    rng = np.random.default_rng(8)
    n_ctx, cap = 200, 120
    pos_all = rng.choice(n_ctx, size=100, replace=False)
    ret_pos = np.full(cap, -1, dtype=np.int64)
    ret_pos[rng.choice(cap, size=100, replace=False)] = pos_all
    scores = (rng.integers(0, 12, size=n_ctx) / 8.0).astype(np.float32)    # many ties
    for n_recent, k in [(20, 30), (0, 10), (20, 0), (20, 1000), (500, 5), (20, 79), (20, 80)]:
        es, ep = O.select(scores, ret_pos, n_ctx, n_recent, k)
        want = brute_select(scores, ret_pos, n_ctx, n_recent, k)
        assert np.array_equal(es, want)
        assert np.array_equal(ep, ret_pos[want])
    # tie-break: equal scores -> the earlier position stays
    rp = np.array([5, 3, 9, 1], dtype=np.int64)
    es, ep = O.select(np.ones(10, dtype=np.float32), rp, 10, 0, 2)
    assert ep.tolist() == [5, 9]
    # -0.0 and +0.0 rank equal
    sc = np.zeros(10, dtype=np.float32)
    sc[3] = -0.0
    es, ep = O.select(sc, rp, 10, 0, 2)
    assert ep.tolist() == [5, 9]
    # the set kept is exactly "top k by score"
    sc = rng.standard_normal(10).astype(np.float32)
    es, ep = O.select(sc, rp, 10, 0, 2)
    kept = sorted(set(rp.tolist()) - set(ep.tolist()), key=lambda p: -sc[p])
    assert min(sc[p] for p in kept) >= max(sc[p] for p in ep)


# ------------------------------------------------------------------ attention / revive
def test_attention_matches_library_sdpa():
    rng = np.random.default_rng(9)
    G, n, D = 4, 333, 128
    q, K, V = rng.standard_normal((G, D)), rng.standard_normal((n, D)), rng.standard_normal((n, D))
    scale = 1 / math.sqrt(D)
    o, p = O.attention(q, K, V, scale)
    ref = torch.nn.functional.scaled_dot_product_attention(
        torch.tensor(q)[None], torch.tensor(K)[None], torch.tensor(V)[None], scale=scale)[0].numpy()
    assert np.allclose(o, ref, rtol=1e-12, atol=1e-12)
    assert np.allclose(p.sum(axis=1), 1.0, atol=1e-14)
    # a wrong scale or a transposed operand would not survive this
    ref2 = torch.softmax(torch.tensor(q) @ torch.tensor(K).T * scale, dim=-1).numpy()
    assert np.allclose(p, ref2, rtol=1e-12, atol=1e-15)


def make_state(rng, N=60, D=128, r=3, w=4, n_recent=8, k_cand=9, storage="bf16", G=2, cap_extra=1):
    params = O.hash_params_from_seed(31, r)
    K = O.to_storage(rng.standard_normal((N, D)), storage)
    V = O.to_storage(rng.standard_normal((N, D)), storage)
    q0 = O.to_storage(rng.standard_normal((G, D)), storage)
    st = O.dense_prefill_state(K, V, q0, 1 / math.sqrt(D), r, w, params, storage,
                               n_recent=n_recent, k_candidate=k_cand, n_cap=N + 16)
    return st, K, V


def test_full_budget_equals_dense_attention_and_score_mass():
    rng = np.random.default_rng(10)
    st, K, V = make_state(rng)
    G, D = 2, 128
    q = rng.standard_normal((G, D))
    before = st.scores.copy()
    out, p = st.attend(q, 1 / math.sqrt(D))          # nothing in the sketch yet
    ref = torch.nn.functional.scaled_dot_product_attention(
        torch.tensor(q)[None], torch.tensor(K)[None], torch.tensor(V)[None])[0].numpy()
    assert np.allclose(out, ref, rtol=1e-12, atol=1e-12)
    # every step adds total probability G to the unit's cumulative scores
    assert abs((st.scores.astype(np.float64) - before).sum() - G) < 1e-5


def test_fused_equals_dense_over_reconstruction_and_permutation_invariance():
    rng = np.random.default_rng(11)
    st, K, V = make_state(rng)
    D = 128
    st.compress()
    assert len(st.vague_pos) == 60 - 8 - 9
    st = O.compact(st, 18)
    q = rng.standard_normal((2, D))
    Kh, Vh = O.query(st.SK, st.SV, st.params, st.vague_pos, storage="bf16")
    used = st.ret_pos >= 0
    Kall = np.concatenate([st.K_ret[used], Kh])
    Vall = np.concatenate([st.V_ret[used], Vh])
    ref, _ = O.attention(q, Kall, Vall, 1 / math.sqrt(D))
    out, _, p = O.attend_decode(q, st.K_ret, st.V_ret, st.ret_pos, st.SK, st.SV, st.params,
                                st.vague_pos, st.n_ctx, 1 / math.sqrt(D), storage="bf16")
    assert np.allclose(out, ref, rtol=1e-12, atol=1e-12)
    # order of the index list and of the slots does not matter
    perm = rng.permutation(len(st.vague_pos))
    sp = rng.permutation(18)
    out2, _, _ = O.attend_decode(q, st.K_ret[sp], st.V_ret[sp], st.ret_pos[sp], st.SK, st.SV,
                                 st.params, [st.vague_pos[i] for i in perm], st.n_ctx,
                                 1 / math.sqrt(D), storage="bf16")
    assert np.allclose(out, out2, rtol=1e-12, atol=1e-12)
    # no retained token at all still works
    none = np.full(18, -1, dtype=np.int64)
    out3, _, p3 = O.attend_decode(q, st.K_ret, st.V_ret, none, st.SK, st.SV, st.params,
                                  list(range(st.n_ctx)), st.n_ctx, 1 / math.sqrt(D), storage="bf16")
    assert np.isfinite(out3).all() and np.allclose(p3.sum(axis=1), 1.0)


def test_revive_rejects_overlap_and_gaps():
    rng = np.random.default_rng(12)
    st, _, _ = make_state(rng)
    st.compress()
    with pytest.raises(ValueError):
        O.revive(st.K_ret, st.V_ret, st.ret_pos, st.SK, st.SV, st.params,
                 st.vague_pos + [int(st.ret_pos[st.ret_pos >= 0][0])], st.n_ctx)
    with pytest.raises(ValueError):
        O.revive(st.K_ret, st.V_ret, st.ret_pos, st.SK, st.SV, st.params, st.vague_pos[1:], st.n_ctx)


# ------------------------------------------------------------------ whole step, second formulation
def onehot_step(K, V, q, scale, params, r, w, vague_pos, ret_pos_list, scores, sign=True):
    """Dense-matrix formulation: SK_i = H_i^T K, k_hat = median_i(H_i SK_i) with
    one-hot H_i [n_vague, w]; then textbook attention over all positions."""
    n_ctx, D = K.shape
    vp = list(vague_pos)
    Kv, Vv = K[vp], V[vp]
    est_k, est_v = [], []
    for i in range(r):
        H = np.zeros((len(vp), w))
        gsign = np.ones(len(vp))
        for t, J in enumerate(vp):
            a, b, c, d = params[i]
            H[t, (((a * J + b) % (1 << 64)) >> 32) * w >> 32] = 1.0
            gsign[t] = -1.0 if ((c * J + d) % (1 << 64)) >= (1 << 63) else 1.0
        SKi = H.T @ Kv
        SVi = H.T @ (gsign[:, None] * Vv)
        est_k.append(H @ SKi)
        est_v.append(gsign[:, None] * (H @ SVi))
    Kstar, Vstar = K.copy(), V.copy()
    Kstar[vp] = np.median(np.stack(est_k), axis=0)
    Vstar[vp] = np.median(np.stack(est_v), axis=0)
    lg = (q @ Kstar.T) * scale
    p = np.exp(lg - lg.max(axis=1, keepdims=True))
    p /= p.sum(axis=1, keepdims=True)
    return p @ Vstar, scores + p.sum(axis=0)


def test_whole_step_against_onehot_formulation():
    rng = np.random.default_rng(13)
    N, D, r, w, G = 16, 128, 3, 2, 2
    params = O.hash_params_from_seed(77, r)
    # small-integer data padded with zero channels: every sketch sum is exact
    K = np.zeros((N + 1, D))
    V = np.zeros((N + 1, D))
    K[:, :4] = rng.integers(-3, 4, size=(N + 1, 4))
    V[:, :4] = rng.integers(-3, 4, size=(N + 1, 4))
    q0 = np.zeros((G, D)); q0[:, :4] = rng.integers(-2, 3, size=(G, 4))
    q1 = np.zeros((G, D)); q1[:, :4] = rng.integers(-2, 3, size=(G, 4))
    scale = 1 / math.sqrt(D)
    st = O.dense_prefill_state(K[:N], V[:N], q0, scale, r, w, params, "f64",
                               n_recent=4, k_candidate=3, ret_cap=N + 1, n_cap=N + 1)
    s0 = st.scores.astype(np.float64).copy()
    out, (ev_slots, ev_pos), p = st.decode_step(K[N], V[N], q1, scale)
    # partition sizes: 4 recent + 3 candidates stay, everything else is vague
    assert (st.ret_pos >= 0).sum() == 7 and len(st.vague_pos) == N + 1 - 7
    recent = sorted(st.ret_pos[st.ret_pos >= N + 1 - 4].tolist())
    assert recent == [N - 3, N - 2, N - 1, N]
    # the candidates are the top-3 prefill scores among non-recent positions
    nonrec = np.arange(N + 1 - 4)
    top3 = sorted(nonrec[np.lexsort((nonrec, -s0[nonrec]))[:3]].tolist())
    assert sorted(p_ for p_ in st.ret_pos.tolist() if 0 <= p_ < N + 1 - 4) == top3
    ref_out, ref_scores = onehot_step(K, V, q1, scale, params, r, w, st.vague_pos,
                                      None, s0)
    assert np.allclose(out, ref_out, rtol=1e-12, atol=1e-12)
    assert np.allclose(st.scores, ref_scores, rtol=1e-6, atol=1e-7)


def test_multi_step_bookkeeping_invariants():
    rng = np.random.default_rng(14)
    N, D, r, w = 40, 128, 3, 3
    params = O.hash_params_from_seed(3, r)
    K = O.to_storage(rng.standard_normal((N + 6, D)), "bf16")
    V = O.to_storage(rng.standard_normal((N + 6, D)), "bf16")
    q = O.to_storage(rng.standard_normal((6 + 1, 2, D)), "bf16")
    scale = 1 / math.sqrt(D)
    st = O.dense_prefill_state(K[:N], V[:N], q[0], scale, r, w, params, "bf16",
                               n_recent=5, k_candidate=6, n_cap=N + 6, acc_dtype=np.float32)
    st.compress()
    st = O.compact(st, 12)
    for t in range(6):
        out, (es, ep), p = st.decode_step(K[N + t], V[N + t], q[t + 1], scale)
        assert len(es) == 1                                  # steady state: one in, one out
        assert (st.ret_pos >= 0).sum() == 11 and len(st.free_slots()) == 1
        assert len(st.vague_pos) + 11 == st.n_ctx == N + t + 1
        assert len(set(st.vague_pos)) == len(st.vague_pos)
        assert np.isfinite(out).all()
    # the sketch built incrementally equals one bulk insert of the same tokens in
    # the same order when nothing needs rounding (checked with exact data above);
    # here: it only ever holds bf16-representable values
    assert np.array_equal(st.SK, O.to_storage(st.SK, "bf16"))


# ------------------------------------------------------------------ swap loop (Algorithm 3)
def _injective_positions(params, r, w, n, rng, limit=4000):
    """Positions whose slots are pairwise distinct in every row (no collisions)."""
    chosen, used = [], [set() for _ in range(r)]
    for J in rng.permutation(limit):
        hs = [O.bucket_of(params[i], int(J), w) for i in range(r)]
        if all(hs[i] not in used[i] for i in range(r)):
            chosen.append(int(J))
            for i in range(r):
                used[i].add(hs[i])
            if len(chosen) == n:
                return chosen
    raise AssertionError("no injective set found")


def test_swap_pick_against_brute_force_and_boundaries():
    rng = np.random.default_rng(21)
    for trial in range(200):
        n_ret, n_vague, n_ctx, n_recent = 9, 7, 40, 5
        pos = rng.permutation(n_ctx)
        ret_pos = np.full(n_ret + 2, -1, dtype=np.int64)
        recent = np.arange(n_ctx - n_recent, n_ctx)
        others = np.array([p for p in pos if p < n_ctx - n_recent])
        ret_pos[:n_recent] = recent
        ret_pos[n_recent + 1:n_recent + 1 + 4] = others[:4]            # 4 candidates, with an empty slot between
        vague = [int(p) for p in others[4:4 + n_vague]]
        scores = rng.integers(0, 4, size=n_ctx).astype(np.float32)        # many ties
        rate = float(rng.choice([1.0, 1.1, 1.5]))
        got = O.swap_pick(scores, ret_pos, vague, n_ctx, n_recent, rate)
        # brute force with explicit sorting
        cand = [(float(scores[ret_pos[s]]), -int(ret_pos[s]), s) for s in range(len(ret_pos))
                if 0 <= ret_pos[s] < n_ctx - n_recent]
        cand.sort()
        vg = sorted([(-float(scores[p]), p, i) for i, p in enumerate(vague)])
        cmin, vmax = cand[0], vg[0]
        cond = np.float32(np.float32(cmin[0]) * np.float32(rate)) < np.float32(-vmax[0])
        if cond:
            assert got == (cmin[2], vmax[2])
        else:
            assert got is None
    # strict inequality: equal scores at rate 1.0 do not swap; a Recent token is never the minimum
    scores = np.ones(10, dtype=np.float32)
    ret_pos = np.array([0, 1, 8, 9], dtype=np.int64)
    assert O.swap_pick(scores, ret_pos, [2, 3], 10, 2, 1.0) is None
    scores[3] = 2.0
    assert O.swap_pick(scores, ret_pos, [2, 3], 10, 2, 1.0) == (1, 1)          # tie of candidates 0, 1: later position
    scores[8] = 0.0                                                             # recent token with the lowest score: ignored
    assert O.swap_pick(scores, ret_pos, [2, 3], 10, 2, 1.0) == (1, 1)
    assert O.swap_pick(scores, ret_pos, [], 10, 2, 1.0) is None
    assert O.swap_pick(scores, np.array([8, 9]), [2, 3], 10, 2, 1.0) is None
    # the product is taken in float32: 1.1f * 10f = 11.000000238..., which rounds to 11.0f, so a
    # Vague score of 11 does not exceed it
    scores = np.array([10.0, 11.0, 0, 0], dtype=np.float32)
    assert O.swap_pick(scores, np.array([0, 2, 3]), [1], 4, 2, 1.1) is None
    assert O.swap_pick(scores, np.array([0, 2, 3]), [1], 4, 2, 1.09) == (0, 0)


def test_swap_restores_token_exactly_without_collisions():
    """With no collisions V.Query returns the token itself, so V.Delete removes it
    without a trace: after the swap the sketch equals a sketch built from scratch
    from the new Vague set, and the Candidate slot holds the original token."""
    rng = np.random.default_rng(22)
    r, w, D = 3, 64, 128
    params = rand_params(rng, r)
    pos = _injective_positions(params, r, w, 12, rng)
    vague, cand = pos[:10], pos[10:]
    K = {p: rng.integers(-8, 9, size=D).astype(np.float64) for p in pos}
    V = {p: rng.integers(-8, 9, size=D).astype(np.float64) for p in pos}
    SK, SV = O.sketch_zeros(r, w, D)
    SK, SV = O.insert(SK, SV, params, vague, [K[p] for p in vague], [V[p] for p in vague])
    K_ret = np.stack([K[p] for p in cand]); V_ret = np.stack([V[p] for p in cand])
    ret_pos = np.array(cand, dtype=np.int64)
    vp = list(vague)
    J, pc = vp[3], cand[1]
    SK2, SV2 = O.swap_once(SK, SV, params, K_ret, V_ret, ret_pos, vp, 1, 3)
    new_vague = [p for p in vague if p != J] + [pc]
    SKr, SVr = O.sketch_zeros(r, w, D)
    SKr, SVr = O.insert(SKr, SVr, params, new_vague, [K[p] for p in new_vague], [V[p] for p in new_vague])
    assert np.array_equal(SK2, SKr) and np.array_equal(SV2, SVr)
    assert np.array_equal(K_ret[1], K[J]) and np.array_equal(V_ret[1], V[J])
    assert ret_pos[1] == J and vp[3] == pc and sorted(vp) == sorted(new_vague)
    # every token of the new Vague set is still recovered exactly
    kq, vq = O.query(SK2, SV2, params, vp)
    assert np.array_equal(kq, np.stack([K[p] for p in vp])) and np.array_equal(vq, np.stack([V[p] for p in vp]))


def test_swap_with_collisions_against_onehot_formulation():
    """Delete = subtract the queried estimate from the slots an insert of J adds
    to, with the same signs (dense one-hot formulation, exact integer data)."""
    rng = np.random.default_rng(23)
    r, w, D = 3, 3, 128
    params = rand_params(rng, r)
    vague = [int(p) for p in rng.permutation(60)[:20]]
    cand_pos, cand_slot = 77, 2
    Kt = rng.integers(-4, 5, size=(20, D)).astype(np.float64)
    Vt = rng.integers(-4, 5, size=(20, D)).astype(np.float64)
    SK, SV = O.sketch_zeros(r, w, D)
    SK, SV = O.insert(SK, SV, params, vague, Kt, Vt)
    K_ret = rng.integers(-4, 5, size=(4, D)).astype(np.float64)
    V_ret = rng.integers(-4, 5, size=(4, D)).astype(np.float64)
    kc, vc = K_ret[cand_slot].copy(), V_ret[cand_slot].copy()
    ret_pos = np.array([70, 71, cand_pos, 90], dtype=np.int64)
    i_max = 5
    J = vague[i_max]

    def onehot(Jx):
        H = np.zeros((r, w)); g = np.zeros(r)
        for i in range(r):
            a, b, c, d = params[i]
            H[i, (((a * Jx + b) % (1 << 64)) >> 32) * w >> 32] = 1.0
            g[i] = -1.0 if ((c * Jx + d) % (1 << 64)) >= (1 << 63) else 1.0
        return H, g
    HJ, gJ = onehot(J)
    Hc, gc = onehot(cand_pos)
    k_hat = np.median(np.stack([HJ[i] @ SK[i] for i in range(r)]), axis=0)
    v_hat = np.median(np.stack([gJ[i] * (HJ[i] @ SV[i]) for i in range(r)]), axis=0)
    SK_ref = SK - HJ[:, :, None] * k_hat[None, None, :] + Hc[:, :, None] * kc[None, None, :]
    SV_ref = SV - (gJ[:, None] * HJ)[:, :, None] * v_hat[None, None, :] + (gc[:, None] * Hc)[:, :, None] * vc[None, None, :]
    vp = list(vague)
    SK2, SV2 = O.swap_once(SK, SV, params, K_ret, V_ret, ret_pos, vp, cand_slot, i_max)
    assert np.array_equal(SK2, SK_ref) and np.array_equal(SV2, SV_ref)
    assert np.array_equal(K_ret[cand_slot], k_hat) and np.array_equal(V_ret[cand_slot], v_hat)
    assert ret_pos[cand_slot] == J and vp[i_max] == cand_pos
    # the total key mass of every row changes by exactly (candidate - estimate)
    for i in range(r):
        assert np.array_equal(SK2[i].sum(axis=0) - SK[i].sum(axis=0), kc - k_hat)


def test_swap_rounds_shared_slot_once_delete_then_insert():
    """Delete and insert of one swap are one sketch update: a slot both touch is
    old - estimate + candidate in float32 in that order, rounded to bf16 once."""
    r, w, D = 1, 1, 128                       # one slot: everything collides
    params = [(1, 0, 1, 0)]                   # g = +1 for small J
    SK = np.full((1, 1, D), 256.0); SV = np.full((1, 1, D), 256.0)
    K_ret = np.full((1, D), 1.0); V_ret = np.full((1, D), 1.0)      # candidate adds 1 (half an ulp at 256 in bf16)
    ret_pos = np.array([5], dtype=np.int64)
    vp = [3]
    SK2, SV2 = O.swap_once(SK, SV, params, K_ret, V_ret, ret_pos, vp, 0, 0, storage="bf16",
                           acc_dtype=np.float32)
    # estimate = the slot itself (256): 256 - 256 + 1 = 1 exactly; rounding twice (256 - 256 -> 0, 0 + 1) agrees,
    # but insert-then-delete with a rounding in between (256 + 1 -> 256, - 256 -> 0) would not
    assert np.all(SK2 == 1.0) and np.all(SV2 == 1.0)
    assert np.all(K_ret == 256.0) and ret_pos[0] == 3 and vp == [5]
    # the order inside the float32 sum: (2^24 - 2^24) + 1 = 1, whereas (2^24 + 1) - 2^24 = 0 in float32
    SK = np.full((1, 1, D), 2.0 ** 24); SV = np.full((1, 1, D), 2.0 ** 24)
    K_ret = np.full((1, D), 1.0); V_ret = np.full((1, D), 1.0)
    SK2, SV2 = O.swap_once(SK, SV, params, K_ret, V_ret, np.array([5]), [3], 0, 0, storage="f32",
                           acc_dtype=np.float32)
    assert np.all(SK2 == 1.0) and np.all(SV2 == 1.0)


def test_swap_loop_exit_condition_and_partition():
    rng = np.random.default_rng(24)
    N, D, r, w = 48, 128, 3, 4
    params = O.hash_params_from_seed(5, r)
    K = O.to_storage(rng.standard_normal((N + 4, D)), "bf16")
    V = O.to_storage(rng.standard_normal((N + 4, D)), "bf16")
    q = O.to_storage(rng.standard_normal((5, 2, D)), "bf16")
    scale = 1 / math.sqrt(D)
    st = O.dense_prefill_state(K[:N], V[:N], q[0], scale, r, w, params, "bf16",
                               n_recent=6, k_candidate=8, n_cap=N + 4, acc_dtype=np.float32)
    st.compress()
    st = O.compact(st, 15)
    total_swaps = 0
    for t in range(4):
        n_vague_before = len(st.vague_pos) + 1
        st.decode_step(K[N + t], V[N + t], q[t + 1], scale, replace_rate=1.1, max_swaps=64)
        assert len(st.vague_pos) == n_vague_before                  # swaps keep both parts' sizes
        assert (st.ret_pos >= 0).sum() == 14
        allpos = sorted(st.vague_pos + [int(p) for p in st.ret_pos if p >= 0])
        assert allpos == list(range(st.n_ctx))                       # still a partition of the context
        # after one more unbounded loop nothing is left to swap, and the exit condition holds
        done = st.swap_back(1.1, 1000)
        total_swaps += len(done)
        assert O.swap_pick(st.scores, st.ret_pos, st.vague_pos, st.n_ctx, st.n_recent, 1.1) is None
        cand = [p for p in st.ret_pos if 0 <= p < st.n_ctx - st.n_recent]
        cmin = min(float(st.scores[p]) for p in cand)
        vmax = max(float(st.scores[p]) for p in st.vague_pos)
        assert not (np.float32(np.float32(cmin) * np.float32(1.1)) < np.float32(vmax))
    # max_swaps bounds the loop
    st2 = O.dense_prefill_state(K[:N], V[:N], q[0], scale, r, w, params, "bf16",
                                n_recent=6, k_candidate=8, n_cap=N + 4, acc_dtype=np.float32)
    st2.compress()
    st2.scores[st2.vague_pos] += 10.0          # every Vague token now outranks every Candidate
    assert len(st2.swap_back(1.1, 3)) == 3
    assert len(st2.swap_back(1.1, 0)) == 0


# ------------------------------------------------------------------ Slack (Algorithm 3, first branch)
def _slack_run(slack, steps, seed=41, N=44, n_recent=5, k_cand=7, w=3):
    """A prompt and `steps` decode steps with the given Slack; yields the state and
    what each step evicted."""
    rng = np.random.default_rng(seed)
    D, r = 128, 3
    params = O.hash_params_from_seed(9, r)
    K = O.to_storage(rng.standard_normal((N + steps, D)), "bf16")
    V = O.to_storage(rng.standard_normal((N + steps, D)), "bf16")
    q = O.to_storage(rng.standard_normal((steps + 1, 2, D)), "bf16")
    scale = 1 / math.sqrt(D)
    st = O.dense_prefill_state(K[:N], V[:N], q[0], scale, r, w, params, "bf16", n_recent=n_recent,
                               k_candidate=k_cand, n_cap=N + steps + 2, acc_dtype=np.float32)
    st.compress(slack)
    st = O.compact(st, n_recent + k_cand + slack + 1)
    hist = []
    for t in range(steps):
        scores_before = st.scores.copy()
        ret_before = st.ret_pos.copy()
        out, (es, ep), _ = st.decode_step(K[N + t], V[N + t], q[t + 1], scale, slack=slack)
        hist.append((es.copy(), ep.copy(), scores_before, ret_before, st.r_size, st.n_ctx,
                     st.ret_pos.copy(), list(st.vague_pos), out))
    return st, hist, (K, V, q, params, scale)


def test_slack_zero_is_one_in_one_out_with_a_fixed_recent_window():
    """Slack = 0: the Recent part is always the n_recent newest positions and every step
    evicts exactly the lowest-score candidate (explicit sort, not the oracle's select)."""
    st, hist, _ = _slack_run(0, 9)
    n_recent, k_cand = 5, 7
    for (es, ep, sc, rp, r_size, n_ctx, rp_after, vague, _) in hist:
        assert r_size == n_recent and len(es) == 1
        cand = [int(p) for p in rp if 0 <= p < n_ctx - n_recent]        # rp: before the append (the new token is Recent)
        assert len(cand) == k_cand + 1
        lowest = sorted(cand, key=lambda p: (float(sc[p]), -p))[0]
        assert int(ep[0]) == lowest
        assert sorted(int(p) for p in rp_after if p >= 0)[-n_recent:] == list(range(n_ctx - n_recent, n_ctx))


@pytest.mark.parametrize("slack", [1, 3, 7])
def test_slack_batches_evictions(slack):
    """Slack = s: the Recent queue grows from its budget to budget + s, then s + 1 tokens
    leave it at once and s + 1 tokens (the lowest scores among old Candidates and the
    popped ones) go into the sketch in one insert."""
    n_recent, k_cand, steps = 5, 7, 3 * (slack + 1) + 1
    st, hist, _ = _slack_run(slack, steps)
    for t, (es, ep, sc, rp, r_size, n_ctx, rp_after, vague, _) in enumerate(hist):
        phase = (t + 1) % (slack + 1)
        assert n_recent <= r_size <= n_recent + slack
        if phase == 0:
            assert r_size == n_recent and len(es) == slack + 1
            # Candidates before the pop plus the popped tokens; the slack + 1 lowest leave
            pool = [int(p) for p in rp if 0 <= p < n_ctx - n_recent]
            assert len(pool) == k_cand + slack + 1
            leave = sorted(pool, key=lambda p: (float(sc[p]), -p))[:slack + 1]
            assert sorted(int(p) for p in ep) == sorted(leave)
            assert list(es) == sorted(es)                               # listed in ascending slot order
        else:
            assert r_size == n_recent + phase and len(es) == 0
        kept = sorted(int(p) for p in rp_after if p >= 0)
        assert sorted(kept + vague) == list(range(n_ctx))               # a partition of the context
        assert kept[-r_size:] == list(range(n_ctx - r_size, n_ctx))    # the queue = the newest r_size positions
        assert len(kept) == k_cand + r_size


@pytest.mark.parametrize("slack", [0, 2, 5])
def test_slack_against_a_queue_and_a_heap(slack):
    """Algorithm 3 written out with the paper's own containers -- R a FIFO queue of
    positions, C a min-heap keyed by cumulative score -- driven by the same score
    history; after every step the three parts must be the oracle's."""
    import collections
    import heapq
    n_recent, k_cand, steps = 5, 7, 14
    st, hist, _ = _slack_run(slack, steps, seed=43)
    N = hist[0][5] - 1
    # the prompt: every token pushed into R, then the first branch and the pop loop once
    sc0 = hist[0][2]
    R = collections.deque(range(N))
    C, Vg = [], set()

    def settle(scores):
        if len(R) > n_recent + slack:
            for _ in range(len(R) - n_recent):
                C.append(R.popleft())                                   # oldest first
        heap = [(float(scores[p]), -p, p) for p in C]
        heapq.heapify(heap)                                             # min score on top; ties: the later position
        while len(heap) > k_cand:
            _, _, p = heapq.heappop(heap)
            Vg.add(p)
        C[:] = [p for _, _, p in heap]

    settle(sc0)
    for (es, ep, sc, rp, r_size, n_ctx, rp_after, vague, _) in hist:
        R.append(n_ctx - 1)
        before = set(Vg)
        settle(sc)
        assert sorted(Vg - before) == sorted(int(p) for p in ep)
        assert sorted(Vg) == sorted(vague)
        assert sorted(list(R) + C) == sorted(int(p) for p in rp_after if p >= 0)
        assert len(R) == r_size


def test_slack_shared_slot_is_rounded_once():
    """Several tokens of one bulk pop land in one sketch slot (3 slots per row, 4 tokens):
    the sketch after the step equals one insert call of the popped tokens in ascending
    slot order on the sketch before it, and differs from inserting them one call at a
    time (which would round the shared slot after every token)."""
    slack = 3
    st, hist, (K, V, q, params, scale) = _slack_run(slack, 3)       # state just before the first bulk pop
    SK0, SV0 = st.SK.copy(), st.SV.copy()
    N3 = st.n_ctx
    rng = np.random.default_rng(77)
    kn = O.to_storage(rng.standard_normal(128) * 37.0, "bf16")
    vn = O.to_storage(rng.standard_normal(128) * 37.0, "bf16")
    K_before, V_before = st.K_ret.copy(), st.V_ret.copy()
    out, (es, ep), _ = st.decode_step(kn, vn, q[1], scale, slack=slack)
    assert len(es) == 4
    one_call = O.insert(SK0, SV0, params, ep, K_before[es], V_before[es], storage="bf16", acc_dtype=np.float32)
    assert np.array_equal(st.SK, one_call[0]) and np.array_equal(st.SV, one_call[1])
    sk, sv = SK0, SV0
    for s, p in zip(es, ep):
        sk, sv = O.insert(sk, sv, params, [p], K_before[[s]], V_before[[s]], storage="bf16", acc_dtype=np.float32)
    assert not (np.array_equal(sk, st.SK) and np.array_equal(sv, st.SV))


# ------------------------------------------------------------------ input recipe: per-layer budgets
def test_layer_budgets_preserve_the_total():
    import kvr_synth as S
    wl = S.WORKLOADS["c4"]
    ratios = [1.0 + 0.15 * (2 * l / (wl.layers - 1) - 1) for l in range(wl.layers)]
    per = S.layer_budgets(wl, ratios)
    assert len(per) == wl.layers
    total = sum(p.budget_tokens for p in per)
    assert abs(total - wl.layers * wl.budget_tokens) <= wl.layers          # rounding to whole tokens only
    for p, x in zip(per, ratios):
        assert abs(p.budget - wl.budget * x) < 1e-12                         # mean ratio is 1 here
        assert p.n_retained + p.sketch_slots == p.budget_tokens
        assert p.n_vague0 + p.n_retained == wl.context
    assert per[0].w < wl.w < per[-1].w
    with pytest.raises(ValueError):
        S.layer_budgets(wl, [1.0] * (wl.layers - 1))
    with pytest.raises(ValueError):
        S.layer_budgets(wl, [8.0] + [0.01] * (wl.layers - 1))


# ------------------------------------------------------------------ several queries at once
def _multi_case(rng, N=40, D=128, r=3, w=4, G=2, Tq=4, n_vague=22):
    params = rand_params(rng, r)
    K = O.to_storage(rng.standard_normal((N, D)), "bf16")
    V = O.to_storage(rng.standard_normal((N, D)), "bf16")
    perm = rng.permutation(N - Tq)
    vague = [int(p) for p in perm[:n_vague]]
    ret = [int(p) for p in perm[n_vague:]] + list(range(N - Tq, N))      # the Tq newest tokens are retained raw
    SK, SV = O.sketch_zeros(r, w, D)
    SK, SV = O.insert(SK, SV, params, vague, K[vague], V[vague], storage="bf16", acc_dtype=np.float32)
    slots = rng.permutation(len(ret) + 3)
    ret_pos = np.full(len(ret) + 3, -1, dtype=np.int64)
    K_ret = np.zeros((len(ret) + 3, D)); V_ret = np.zeros((len(ret) + 3, D))
    for s_, p_ in zip(slots, ret):
        ret_pos[s_] = p_; K_ret[s_] = K[p_]; V_ret[s_] = V[p_]
    q = O.to_storage(rng.standard_normal((Tq, G, D)), "bf16")
    q_pos = np.arange(N - Tq, N)
    return params, K_ret, V_ret, ret_pos, SK, SV, vague, q, q_pos, N


def test_attend_multi_against_library_sdpa_with_mask():
    rng = np.random.default_rng(31)
    params, K_ret, V_ret, ret_pos, SK, SV, vague, q, q_pos, N = _multi_case(rng)
    scale = 1 / math.sqrt(128)
    sc0 = rng.random(N).astype(np.float32)
    out, sc1, p = O.attend_multi(q, q_pos, K_ret, V_ret, ret_pos, SK, SV, params, vague, N, scale,
                                 scores=sc0, storage="bf16")
    Kst, Vst = O.revive(K_ret, V_ret, ret_pos, SK, SV, params, vague, N, storage="bf16")
    Tq, G, D = q.shape
    mask = torch.as_tensor(np.arange(N)[None, :] <= q_pos[:, None])                       # [Tq, N]
    qt = torch.as_tensor(q).permute(1, 0, 2).unsqueeze(0)                                  # [1, G, Tq, D]
    kt = torch.as_tensor(Kst).expand(1, G, N, D)
    vt = torch.as_tensor(Vst).expand(1, G, N, D)
    ref = torch.nn.functional.scaled_dot_product_attention(qt, kt, vt, attn_mask=mask, scale=scale)
    assert np.allclose(out, ref[0].permute(1, 0, 2).numpy(), rtol=1e-12, atol=1e-12)
    # a query puts no probability on later positions, all of it on the visible ones
    for t in range(Tq):
        assert np.all(p[t, :, q_pos[t] + 1:] == 0) and np.allclose(p[t].sum(axis=1), 1.0)
    assert abs(float((sc1.astype(np.float64) - sc0).sum()) - Tq * G) < 1e-4
    assert np.allclose(sc1, sc0 + p.sum(axis=(0, 1)), rtol=1e-6, atol=1e-7)


def test_attend_multi_equals_one_query_at_a_time_on_the_truncated_context():
    rng = np.random.default_rng(32)
    params, K_ret, V_ret, ret_pos, SK, SV, vague, q, q_pos, N = _multi_case(rng, Tq=3, G=4)
    scale = 1 / math.sqrt(128)
    out, _, p = O.attend_multi(q, q_pos, K_ret, V_ret, ret_pos, SK, SV, params, vague, N, scale, storage="bf16")
    for t in range(q.shape[0]):
        rp = ret_pos.copy()
        rp[rp > q_pos[t]] = -1                                  # later tokens do not exist yet for this query
        o1, _, p1 = O.attend_decode(q[t], K_ret, V_ret, rp, SK, SV, params, vague, int(q_pos[t]) + 1, scale,
                                    storage="bf16")
        assert np.array_equal(out[t], o1) and np.array_equal(p[t, :, :q_pos[t] + 1], p1)
    # one query at the last position is the decode case
    o_last, sc_last, _ = O.attend_multi(q[-1:], q_pos[-1:], K_ret, V_ret, ret_pos, SK, SV, params, vague, N, scale,
                                        scores=np.zeros(N, dtype=np.float32), storage="bf16")
    o_dec, sc_dec, _ = O.attend_decode(q[-1], K_ret, V_ret, ret_pos, SK, SV, params, vague, N, scale,
                                       scores=np.zeros(N, dtype=np.float32), storage="bf16")
    assert np.array_equal(o_last[0], o_dec) and np.array_equal(sc_last, sc_dec)
    with pytest.raises(ValueError):
        O.attend_multi(q, q_pos + 1, K_ret, V_ret, ret_pos, SK, SV, params, vague, N, scale, storage="bf16")
