"""Pins for the CPU oracle: every function of oracle/ is checked against
something other than itself -- the hand-worked example, closed forms, a
sort-based brute force, the paper's one-hot matrix forms (Eq. 8 / Eq. 9) via
numpy, invariants stated in Sec. 3.1, and numpy's own fp16/fp64 routines."""
import json
import os

import numpy as np
import pytest
from scipy import stats

import oracle
import workloads as wk

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def f16(a):
    return np.asarray(a, dtype=np.float16)


def bits(a):
    return f16(a).view(np.uint16)


def as_f16(b):
    return np.asarray(b, dtype=np.uint16).view(np.float16)


# ------------------------------------------------------------------ example
@pytest.fixture(scope="module")
def ex():
    with open(os.path.join(GOLD, "worked_example.json")) as f:
        e = json.load(f)
    e["A"] = [int(v, 16) for v in e["hash_a"]]
    e["C"] = [int(v, 16) for v in e["hash_c"]]
    return e


def test_worked_example_select(ex):
    for r in range(ex["d"]):
        for a in range(8):
            assert oracle.select(ex["A"][r], ex["C"][r], ex["K"], a) == ex["h"][r][a]
            # the fixture's own t values reduce to the same index
            assert (int(ex["t"][r][a], 16) * ex["K"]) >> 24 == ex["h"][r][a]


def test_worked_example_update_query_linear(ex):
    sk = oracle.update(f16(ex["W"]), ex["tile_in"], ex["tile_out"], ex["d"], ex["A"], ex["C"], [ex["K"]])
    assert as_f16(sk.states).astype(np.float64).reshape(2, 3).tolist() == ex["states"]
    W_hat = oracle.query(sk)
    assert as_f16(W_hat).astype(np.float64).tolist() == ex["W_hat"]
    y = oracle.linear(W_hat, f16([ex["x"]]))
    assert y.tolist() == [ex["y"]]


def test_worked_example_signed_max_query(ex):
    """Query mode 1, Eq. (5) as printed: the hand-derived result on the worked example's states."""
    sk = oracle.update(f16(ex["W"]), ex["tile_in"], ex["tile_out"], ex["d"], ex["A"], ex["C"], [ex["K"]])
    W_hat = oracle.query(sk, oracle.QUERY_SIGNED_MAX)
    assert as_f16(W_hat).astype(np.float64).tolist() == ex["W_hat_signed_max"]
    assert oracle.linear(W_hat, f16([ex["x"]])).tolist() == [ex["y_signed_max"]]


# ------------------------------------------------------------- conversions
def test_half_to_double_all_patterns():
    b = np.arange(65536, dtype=np.uint16)
    ref = b.view(np.float16).astype(np.float64)
    got = oracle.half_to_double(b)
    nan = np.isnan(ref)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], ref[~nan])
    assert np.array_equal(np.signbit(got[~nan]), np.signbit(ref[~nan]))


def test_bf16_generator_roundtrip():
    rng = np.random.default_rng(1)
    a = rng.standard_normal(10000).astype(np.float32)
    b = wk.f32_to_bf16_bits(a)
    back = wk.bf16_bits_to_f32(b)
    assert np.all(np.abs(back - a) <= np.abs(a) * 2.0 ** -8)
    # exact ties go to even: 1 + 2^-8 is halfway between 1 and 1 + 2^-7
    assert wk.f32_to_bf16_bits(np.float32([1.0 + 2.0 ** -8]))[0] == 0x3F80
    assert wk.f32_to_bf16_bits(np.float32([1.0 + 3 * 2.0 ** -8]))[0] == 0x3F82


# ------------------------------------------------------------------ select
def test_select_identity_special_case():
    # K = G = 2^k, A = 2^(24-k), C = 0  =>  h(a) = a
    for k in (3, 8, 12):
        G = 1 << k
        for a in (0, 1, G // 2, G - 1):
            assert oracle.select(1 << (24 - k), 0, G, a) == a


def test_select_range_and_extremes():
    rng = np.random.default_rng(2)
    for K in (1, 2, 3, 42, 83, 1024, 65535):
        for _ in range(200):
            A = int(2 * rng.integers(0, 1 << 23) + 1)
            C = int(rng.integers(0, 1 << 24))
            a = int(rng.integers(0, 1 << 24))
            h = oracle.select(A, C, K, a)
            assert 0 <= h < K
            # independent big-int evaluation
            assert h == (((A * a + C) % (1 << 24)) * K) >> 24
    assert oracle.select(0xFFFFFF, 0xFFFFFF, 65535, 0xFFFFFF) == (((0xFFFFFF * 0xFFFFFF + 0xFFFFFF) % (1 << 24)) * 65535) >> 24


def test_select_spreads_uniformly():
    # chi-square of bucket loads over one 1-D group of 11008 offsets
    wl = wk.cfg3("up")
    A, C = wk.gen_hash_params(wl)
    K = 83
    for r in range(wl.d):
        h = np.array([oracle.select(int(A[r]), int(C[r]), K, a) for a in range(wl.out_features)])
        load = np.bincount(h, minlength=K)
        chi2 = ((load - wl.out_features / K) ** 2 / (wl.out_features / K)).sum()
        # an affine map mod 2^24 is more regular than random: only an upper bound
        assert chi2 < stats.chi2.ppf(0.999, K - 1)
        assert load.min() > 0


# ------------------------------------------------------------------ update
def brute_states(W, tj, to, d, A, C, widths):
    """Sort-based statement of Eq. (4): in each bucket the state is the member
    of smallest magnitude, the earliest such member in stream order."""
    in_f, out_f = W.shape
    out = []
    g = 0
    for jb in range(in_f // tj):
        for ob in range(out_f // to):
            K = int(widths[g]); g += 1
            tile = W[jb * tj:(jb + 1) * tj, ob * to:(ob + 1) * to].reshape(-1)
            mag = np.abs(tile.astype(np.float64))
            for r in range(d):
                h = np.array([(((int(A[r]) * a + int(C[r])) % (1 << 24)) * K) >> 24 for a in range(tile.size)])
                row = np.zeros(K, dtype=np.float16)
                for k in range(K):
                    members = np.nonzero(h == k)[0]
                    if members.size:
                        first_min = members[np.argsort(mag[members], kind="stable")[0]]
                        row[k] = tile[first_min]
                out.append(row)
    return np.concatenate(out)


@pytest.mark.parametrize("shape", [(8, 12, 4, 6, 3), (6, 16, 1, 16, 4), (16, 8, 16, 2, 2), (5, 7, 5, 7, 1)])
def test_update_equals_sort_brute_force(shape):
    in_f, out_f, tj, to, d = shape
    rng = np.random.default_rng(sum(shape))
    # few distinct magnitudes => many ties, both signs, some zeros
    W = (rng.integers(-4, 5, size=(in_f, out_f)) * 0.125).astype(np.float16)
    W[rng.random(W.shape) < 0.1] = np.float16(-0.0)
    n_groups = (in_f // tj) * (out_f // to)
    widths = rng.integers(1, 7, size=n_groups)
    A = 2 * rng.integers(0, 1 << 23, size=d) + 1
    C = rng.integers(0, 1 << 24, size=d)
    sk = oracle.update(W, tj, to, d, A, C, widths)
    ref = brute_states(W, tj, to, d, A, C, widths)
    assert np.array_equal(sk.states, ref.view(np.uint16))


def test_update_matrix_form_eq8():
    """Eq. (8): S[i,j] = min_|.| over k of W_g[i,k] 'times' P[k,j], with the
    one-hot P of Eq. (7) acting as a selector (masked entries are ignored)."""
    rng = np.random.default_rng(8)
    M, G, K = 6, 32, 5            # six 1-D groups of 32 weights
    W = rng.standard_normal((M, G)).astype(np.float16)
    A, C = [0x2B3C4D], [0x123456]
    h = np.array([oracle.select(A[0], C[0], K, a) for a in range(G)])
    P = np.zeros((G, K), dtype=bool)
    P[np.arange(G), h] = True
    S = np.zeros((M, K), dtype=np.float16)
    for i in range(M):
        for j in range(K):
            sel = W[i, P[:, j]]
            if sel.size:
                S[i, j] = sel[np.argmin(np.abs(sel.astype(np.float64)))]
    sk = oracle.update(W, 1, G, 1, A, C, [K] * M)
    assert np.array_equal(as_f16(sk.states).reshape(M, K), S)


# ------------------------------------------------------------------- query
def test_query_matrix_form_eq9_single_row():
    """Eq. (9): W_hat_g = S P^T with one-hot P equals the gather S[i, h(k)]."""
    rng = np.random.default_rng(9)
    M, G, K = 7, 48, 9
    states = rng.standard_normal((M, K)).astype(np.float16)
    A, C = [0x6789AB], [0x0F1E2D]
    h = np.array([oracle.select(A[0], C[0], K, a) for a in range(G)])
    P = np.zeros((G, K))
    P[np.arange(G), h] = 1.0
    ref = states.astype(np.float64) @ P.T
    sk = oracle.Sketch(M, G, 1, G, 1, np.uint32(A), np.uint32(C), np.full(M, K, np.uint32),
                       states.view(np.uint16).ravel())
    got = as_f16(oracle.query(sk)).astype(np.float64)
    assert np.array_equal(got, ref)


def absmax_ref(cands):
    """Magnitude max over axis 0; on equal magnitude the non-negative one."""
    c = cands.astype(np.float64)
    best = c[0].copy()
    for r in range(1, c.shape[0]):
        take = (np.abs(c[r]) > np.abs(best)) | ((np.abs(c[r]) == np.abs(best)) & ~np.signbit(c[r]))
        best = np.where(take, c[r], best)
    return best


@pytest.mark.parametrize("d", [2, 3, 4, 8])
def test_query_multi_row_via_matrix_forms(d):
    """Sec. 3.3: the multi-row case is d independent S and P; Eq. (5) then
    combines the d per-row results."""
    rng = np.random.default_rng(90 + d)
    in_f, out_f, tj, to = 4, 36, 2, 12          # 2 x 3 groups, each with its own width
    n_jb, n_ob = in_f // tj, out_f // to
    widths = np.array([5, 2, 7, 3, 6, 4], dtype=np.uint32)
    A = 2 * rng.integers(0, 1 << 23, size=d) + 1
    C = rng.integers(0, 1 << 24, size=d)
    tables = [(rng.integers(-3, 4, size=(d, int(K))) * 0.25).astype(np.float16) for K in widths]  # many +/- ties
    flat = np.concatenate([t.ravel() for t in tables]).view(np.uint16)
    sk = oracle.Sketch(in_f, out_f, tj, to, d, A, C, widths, flat)
    got = as_f16(oracle.query(sk))
    G = tj * to
    for jb in range(n_jb):
        for ob in range(n_ob):
            g = jb * n_ob + ob
            K = int(widths[g])
            per_row = []
            for r in range(d):
                P = np.zeros((G, K))
                for a in range(G):
                    P[a, (((int(A[r]) * a + int(C[r])) % (1 << 24)) * K) >> 24] = 1.0
                per_row.append(P @ tables[g][r].astype(np.float64))
            ref = absmax_ref(np.stack(per_row)).reshape(tj, to)
            blk = got[jb * tj:(jb + 1) * tj, ob * to:(ob + 1) * to].astype(np.float64)
            assert np.array_equal(blk, ref)
            assert np.array_equal(np.signbit(blk), np.signbit(ref))


@pytest.mark.parametrize("d", [2, 3, 8])
def test_signed_max_query_via_matrix_forms_and_numpy_max(d):
    """Query mode 1: the d per-row results of the one-hot matrix form (Eq. 9) combined by numpy's maximum
    of the signed values; tables drawn from seven values so that equal candidates and sign clashes abound.
    Also: the result is one of the candidates and no candidate exceeds it."""
    rng = np.random.default_rng(190 + d)
    in_f, out_f, tj, to = 4, 36, 2, 12
    n_jb, n_ob = in_f // tj, out_f // to
    widths = np.array([5, 2, 7, 3, 6, 4], dtype=np.uint32)
    A = 2 * rng.integers(0, 1 << 23, size=d) + 1
    C = rng.integers(0, 1 << 24, size=d)
    tables = [(rng.integers(-3, 4, size=(d, int(K))) * 0.25).astype(np.float16) for K in widths]
    for t in tables:
        t[t == 0] = np.float16(0.0)              # +0 only: the sign of a zero result is pinned separately
    flat = np.concatenate([t.ravel() for t in tables]).view(np.uint16)
    sk = oracle.Sketch(in_f, out_f, tj, to, d, A, C, widths, flat)
    got = as_f16(oracle.query(sk, oracle.QUERY_SIGNED_MAX)).astype(np.float64)
    magnitude = as_f16(oracle.query(sk)).astype(np.float64)
    G = tj * to
    differs = 0
    for jb in range(n_jb):
        for ob in range(n_ob):
            g = jb * n_ob + ob
            K = int(widths[g])
            per_row = []
            for r in range(d):
                P = np.zeros((G, K))
                for a in range(G):
                    P[a, (((int(A[r]) * a + int(C[r])) % (1 << 24)) * K) >> 24] = 1.0
                per_row.append(P @ tables[g][r].astype(np.float64))
            cands = np.stack(per_row)
            ref = np.max(cands, axis=0).reshape(tj, to)
            blk = got[jb * tj:(jb + 1) * tj, ob * to:(ob + 1) * to]
            assert np.array_equal(blk, ref)
            assert np.all((cands == ref.reshape(1, G)).any(axis=0))
            differs += int(np.sum(blk != magnitude[jb * tj:(jb + 1) * tj, ob * to:(ob + 1) * to]))
    assert differs > 0                           # the two readings of Eq. (5) are told apart on this data


def test_signed_max_query_zero_tie_and_negative_candidates():
    # +0 and -0 are equal values: the pattern with the clear sign bit wins, whatever the row order
    for order in ([0x0000, 0x8000], [0x8000, 0x0000]):
        sk = oracle.Sketch(1, 1, 1, 1, 2, np.uint32([1, 1]), np.uint32([0, 0]), np.uint32([1]), np.uint16(order))
        assert oracle.query(sk, oracle.QUERY_SIGNED_MAX)[0, 0] == 0x0000
    # all candidates negative: the one of smallest magnitude is the maximum (-0.5 over -2); -0 over -0.5
    for cands, want in (([0xC000, 0xB800], 0xB800), ([0xB800, 0xC000], 0xB800), ([0xB800, 0x8000], 0x8000),
                        ([0x3800, 0xC000], 0x3800)):
        sk = oracle.Sketch(1, 1, 1, 1, 2, np.uint32([1, 1]), np.uint32([0, 0]), np.uint32([1]), np.uint16(cands))
        assert oracle.query(sk, oracle.QUERY_SIGNED_MAX)[0, 0] == want
        assert oracle.query(sk)[0, 0] == max(cands, key=lambda b: (b & 0x7FFF, -(b >> 15)))


def test_query_signed_zero_tie():
    # candidates +0 and -0: the one with the clear sign bit wins, whatever the row order
    for order in ([0x0000, 0x8000], [0x8000, 0x0000]):
        sk = oracle.Sketch(1, 1, 1, 1, 2, np.uint32([1, 1]), np.uint32([0, 0]), np.uint32([1]),
                           np.uint16(order))
        assert oracle.query(sk)[0, 0] == 0x0000


# ----------------------------------------------------- whole reconstruction
def make_sketch(wl, W=None):
    W = wk.gen_weight(wl) if W is None else W
    A, C = wk.gen_hash_params(wl)
    widths = oracle.allocate_widths(wk.gen_importance(wl), wl.budget_states, wl.d)
    return W, oracle.update(W, wl.tile_in, wl.tile_out, wl.d, A, C, widths)


@pytest.mark.parametrize("d", [1, 2, 5])
def test_identity_hash_reproduces_W(d):
    """An injective hash with K >= #weights loses nothing (larger sketch =>
    higher accuracy, Sec. 2.2), for any number of rows."""
    rng = np.random.default_rng(5)
    in_f, out_f, tj, to = 16, 32, 8, 16          # G = 128 = 2^7
    W = rng.standard_normal((in_f, out_f)).astype(np.float16)
    A = [1 << (24 - 7)] * d
    C = [0] * d
    sk = oracle.update(W, tj, to, d, A, C, [128] * 4)
    assert np.array_equal(oracle.query(sk), W.view(np.uint16))


def test_invariants_on_cfg1():
    wl = wk.cfg1()
    W, sk = make_sketch(wl)
    assert sk.states.size == 2048 and list(sk.group_width) == [1024]
    W_hat = as_f16(oracle.query(sk))
    # under-estimate (Sec. 3.1): same value or smaller magnitude
    assert np.all(np.abs(W_hat.astype(np.float64)) <= np.abs(W.astype(np.float64)))
    # membership: each reconstructed weight is one of its d hashed states
    st = as_f16(sk.states).reshape(wl.d, 1024)
    A, C = sk.hash_a, sk.hash_c
    flat = W_hat.reshape(-1)
    rng = np.random.default_rng(0)
    for a in rng.integers(0, flat.size, size=500):
        cands = [st[r, oracle.select(int(A[r]), int(C[r]), 1024, int(a))] for r in range(wl.d)]
        assert flat[a] in cands
    # the min-|.| member of a bucket is preserved exactly in that row, so the
    # share of exactly preserved weights is at least (#non-empty states)/G per row
    exact = np.mean(W_hat.view(np.uint16) == W.view(np.uint16))
    assert exact >= 1024 / 65536 * 0.9


def test_row_order_invariance_and_more_rows_never_hurt():
    wl = wk.small("inv", 32, 64, 8, 32, 4, 2.0, 1)
    W = wk.gen_weight(wl)
    A, C = wk.gen_hash_params(wl)
    widths = oracle.allocate_widths(wk.gen_importance(wl), wl.budget_states, wl.d)
    full = oracle.update(W, 8, 32, 4, A, C, widths)
    ref = oracle.query(full)
    perm = [2, 0, 3, 1]
    swapped = oracle.update(W, 8, 32, 4, A[perm], C[perm], widths)
    assert np.array_equal(oracle.query(swapped), ref)
    prev = None
    for dd in (1, 2, 3, 4):
        sk = oracle.update(W, 8, 32, dd, A[:dd], C[:dd], widths)
        mag = np.abs(as_f16(oracle.query(sk)).astype(np.float64))
        assert np.all(mag <= np.abs(W.astype(np.float64)))
        if prev is not None:
            assert np.all(mag >= prev)
        prev = mag


def test_bucket_minimum_survival_law():
    """Reading of Eq. (6): for a bucket holding n i.i.d. weights the state is
    the minimum magnitude, so P(|s| >= tau) = (1 - F(tau))^n with F the CDF of
    |w|; tau = F^-1(1 - p^(1/n)) then holds with probability exactly p."""
    sigma = 0.02
    wl = wk.small("surv", 64, 4096, 1, 4096, 1, 0.5, 3)
    W, sk = make_sketch(wl)
    K = int(sk.group_width[0])
    A, C = sk.hash_a, sk.hash_c
    h = np.array([oracle.select(int(A[0]), int(C[0]), K, a) for a in range(4096)])
    n_b = np.bincount(h, minlength=K)
    s = np.abs(as_f16(sk.states).astype(np.float64)).reshape(64, K)
    for p in (0.25, 0.5, 0.75):
        n = int(round(n_b.mean()))
        tau = stats.halfnorm.ppf(1 - p ** (1.0 / n), scale=sigma)
        expect = np.mean((1 - stats.halfnorm.cdf(tau, scale=sigma)) ** n_b)
        got = np.mean(s >= tau)
        assert abs(got - expect) < 4 * np.sqrt(expect * (1 - expect) / s.size) + 2e-3
        assert abs(expect - p) < 0.05


# ------------------------------------------------------------------ linear
def test_linear_against_numpy_fp64_and_one_hot():
    rng = np.random.default_rng(11)
    in_f, out_f, batch = 37, 53, 3          # non-square: a transposed operand cannot pass
    W_hat = rng.standard_normal((in_f, out_f)).astype(np.float16)
    x = rng.standard_normal((batch, in_f)).astype(np.float16)
    y = oracle.linear(W_hat, x)
    ref = x.astype(np.float64) @ W_hat.astype(np.float64)
    assert np.allclose(y, ref, rtol=1e-13, atol=1e-15)
    cols = [52, 0, 7]
    assert np.array_equal(oracle.linear(W_hat, x, cols=cols), y[:, cols])
    e = np.zeros((1, in_f), dtype=np.float16); e[0, 5] = 1
    assert np.array_equal(oracle.linear(W_hat, e)[0], W_hat[5].astype(np.float64))
    xb = wk.f32_to_bf16_bits(x.astype(np.float32) * 3.3)
    yb = oracle.linear(W_hat, xb, x_kind="bf16")
    refb = wk.bf16_bits_to_f32(xb).astype(np.float64) @ W_hat.astype(np.float64)
    assert np.allclose(yb, refb, rtol=1e-13, atol=1e-15)


# -------------------------------------------------------- width allocation
def test_allocate_widths_proportional_share():
    # uniform importance: the even split of the budget over rows and groups
    assert list(oracle.allocate_widths(np.ones(1), 2048, 2)) == [1024]
    assert set(oracle.allocate_widths(np.ones(4096), 4096 * 4096 // 32, 3)) == {42}
    wl = wk.cfg3("up")
    imp = wk.gen_importance(wl)
    k = oracle.allocate_widths(imp, wl.budget_states, wl.d)
    assert int(k.sum()) * wl.d <= wl.budget_states
    assert sorted(set(k.tolist())) == [83, 333]
    assert np.sum(k == 333) == 41
    # doubling every importance changes nothing; widths follow the share
    assert np.array_equal(oracle.allocate_widths(imp * 2, wl.budget_states, wl.d), k)
    share = k / k.sum()
    assert np.allclose(share, imp / imp.sum(), rtol=0.02)
    with pytest.raises(ValueError):
        oracle.allocate_widths(np.zeros(3), 10, 1)


def test_row_and_layer_importance_by_hand():
    # Sec. 3.2: I_j = mean over the samples of a_j^2; the layer's value is the mean over its rows
    a = np.array([[1.0, -2.0, 0.0], [3.0, 2.0, 0.5]])
    imp = oracle.row_importance(a)
    assert list(imp) == [5.0, 4.0, 0.125]
    assert oracle.layer_importance(imp) == pytest.approx(9.125 / 3, rel=1e-15)
    assert np.array_equal(oracle.row_importance(-a), imp)            # signs do not matter
    assert np.array_equal(oracle.row_importance(a[::-1]), imp)        # nor the order of the samples
    assert np.allclose(oracle.row_importance(3 * a), 9 * imp)
    # a constant activation vector: its own squares
    assert list(oracle.row_importance(np.tile([[2.0, 0.5]], (7, 1)))) == [4.0, 0.25]
    with pytest.raises(ValueError):
        oracle.row_importance(np.zeros((0, 4)))


def test_layer_budgets_follow_the_importance_share():
    # the paper's formula: share I_l / sum(I) of the total space, whole states
    assert list(oracle.allocate_layer_budgets([1, 1, 2], 4000)) == [1000, 1000, 2000]
    assert list(oracle.allocate_layer_budgets([1, 2, 4], 100)) == [14, 28, 57]          # floors of 100/7 * {1, 2, 4}
    b = oracle.allocate_layer_budgets([0.3, 0.5, 0.2, 1.7], 10 ** 6)
    assert int(b.sum()) <= 10 ** 6 and int(b.sum()) > 10 ** 6 - 4
    assert np.array_equal(oracle.allocate_layer_budgets([3, 5, 2, 17], 10 ** 6), b)     # a common factor changes nothing
    # equal sizes: the size-weighted share is the paper's formula
    assert np.array_equal(oracle.allocate_layer_budgets([1, 2, 4], 100, sizes=[9, 9, 9]), [14, 28, 57])
    # equal importance: every layer gets the same bits per weight
    sizes = np.array([4096 * 4096, 4096 * 11008, 11008 * 4096])
    bud = oracle.allocate_layer_budgets([1, 1, 1], int(sizes.sum()) // 32, sizes=sizes)
    assert np.allclose(16.0 * bud / sizes, 0.5, rtol=1e-6)
    # bits per weight proportional to importance
    bud = oracle.allocate_layer_budgets([1, 3], 10 ** 7, sizes=[10 ** 6, 5 * 10 ** 6])
    assert (bud[1] / 5e6) / (bud[0] / 1e6) == pytest.approx(3.0, rel=1e-5)
    with pytest.raises(ValueError):
        oracle.allocate_layer_budgets([0, 0], 10)
    with pytest.raises(ValueError):
        oracle.allocate_layer_budgets([1, 2], 10, sizes=[1, 2, 3])


def test_configured_geometry_stays_within_budget():
    for wl in (wk.cfg1(), wk.cfg2(), wk.cfg2(True), wk.cfg3("up"), wk.cfg3("down"),
               wk.cfg4(4096, 0.5), wk.cfg4(4096, 0.75), wk.cfg4(11008, 0.5), wk.cfg4(11008, 0.75),
               wk.cfg5_70b()):
        k = oracle.allocate_widths(wk.gen_importance(wl), wl.budget_states, wl.d)
        bpw = 16.0 * wl.d * int(k.sum()) / wl.n_weights
        assert bpw <= wl.bpw + 1e-12 and bpw > 0.97 * wl.bpw, (wl.name, bpw)


# ---------------------------------------------------------- error handling
def test_oracle_rejects_bad_input():
    W = np.ones((4, 4), dtype=np.float16)
    with pytest.raises(ValueError):
        oracle.update(W, 3, 4, 1, [1], [0], [4])            # tile does not divide
    with pytest.raises(ValueError):
        oracle.update(W, 4, 4, 1, [1 << 24], [0], [4])       # A out of range
    Wn = W.copy(); Wn[0, 0] = np.inf
    with pytest.raises(ValueError):
        oracle.update(Wn, 4, 4, 1, [1], [0], [4])
    sk = oracle.Sketch(4, 4, 4, 4, 1, np.uint32([1]), np.uint32([0]), np.uint32([4]), np.uint16([0x7C00] * 4))
    with pytest.raises(ValueError):
        oracle.query(sk)


def test_gate_up_against_a_library_sigmoid_and_closed_forms():
    """Eq. (2) with SiLU: a * sigmoid(a) * b.  Pinned by scipy's logistic function, by SiLU(a) - SiLU(-a) = a,
    by SiLU(0) = 0 and by the large-argument limits."""
    from scipy.special import expit
    rng = np.random.default_rng(12)
    a = rng.standard_normal(1000) * 6
    b = rng.standard_normal(1000)
    got = oracle.gate_up(a, b)
    assert np.allclose(got, a * expit(a) * b, rtol=1e-14, atol=0)
    ones = np.ones_like(a)
    assert np.allclose(oracle.gate_up(a, ones) - oracle.gate_up(-a, ones), a, rtol=1e-13, atol=1e-15)
    assert oracle.gate_up(0.0, 5.0) == 0.0
    assert oracle.gate_up(40.0, 2.0) == pytest.approx(80.0, rel=1e-15)
    assert abs(oracle.gate_up(-40.0, 2.0)) < 1e-15
    assert oracle.gate_up(1.0, 1.0) == pytest.approx(0.7310585786300049, rel=1e-15)     # 1 / (1 + 1/e)
