"""Pins for the CPU oracle: each test ties one oracle function to something
other than itself - a closed form, an invariant, a brute force on tiny inputs,
a value printed in the paper, or a routine of another library."""
import itertools
import math
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

from oracle import zipvl_oracle as oz

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rng(seed):
    return np.random.Generator(np.random.PCG64(seed))


# ------------------------------------------------------------------ scores
def test_mass_sums_to_one_and_is_nonnegative():
    # Row softmax makes every probe row sum to 1, so the accumulated score
    # totals m (Section 4.1, remark under Eq. (7)) and mass totals 1.
    r = _rng(1)
    Hq, Hkv, n, d = 6, 2, 97, 16
    Q, K = r.standard_normal((Hq, n, d)), r.standard_normal((Hkv, n, d))
    probe = np.array([3, 40, 41, 88, 90])
    mass, rank = oz.token_scores(Q, K, probe, 0.25)
    assert np.all(mass >= 0) and np.all(rank >= 0)
    np.testing.assert_allclose(mass.sum(axis=1), 1.0, rtol=0, atol=1e-12)
    # columns after the last probe position are never seen
    assert np.all(mass[:, 91:] == 0) and np.all(rank[:, 91:] == 0)


def test_zero_query_harmonic_closed_form():
    # Q = 0 makes every visible logit equal, so probe row at position P gives
    # 1/(P+1) to each key j <= P.  With probes [n-m, n): a_j = H_n - H_{max(j, n-m)}
    # (harmonic numbers, 0-based j), exact rationals.
    n, m, d = 50, 8, 4
    K = _rng(2).standard_normal((1, n, d))
    Q = np.zeros((1, n, d))
    probe = np.arange(n - m, n)
    mass, rank = oz.token_scores(Q, K, probe, 0.5)
    H = [Fraction(0)]
    for t in range(1, n + 1):
        H.append(H[-1] + Fraction(1, t))
    for j in range(n):
        a = H[n] - H[max(j, n - m)]
        cnt = min(m, n - j)
        assert abs(mass[0, j] - float(a / m)) < 1e-14
        assert abs(rank[0, j] - float(a / cnt)) < 1e-14


def test_structural_count_arbitrary_probes():
    probe = np.array([2, 5, 5 + 4, 20])
    cnt = oz.structural_count(24, probe)
    brute = [sum(1 for p in probe if p >= j) for j in range(24)]
    assert cnt.tolist() == brute
    assert cnt[21] == 0 and cnt[0] == 4


def test_one_hot_scores_select_single_token():
    # One key with a huge logit visible to every probe row takes all the mass.
    r = _rng(3)
    n, d, js = 64, 8, 17
    u = np.zeros(d); u[0] = 1.0
    Q = np.tile(u * 10.0, (1, n, 1))
    K = 0.01 * r.standard_normal((1, n, d))
    K[0, js] = u * 10.0                      # logit 100*scale
    probe = np.arange(n - 16, n)
    mass, rank = oz.token_scores(Q, K, probe, 0.5)
    assert mass[0, js] > 1 - 1e-12
    p, T = oz.select(mass[0].astype(np.float32), rank[0].astype(np.float32), 0.99)
    assert p == 1 and T.tolist() == [js]


def test_all_rows_probe_equals_dense_softmax_column_sums_torch():
    # With every row a probe, Eq. (6)/(8) are the column sums / means of the
    # dense causal attention matrix; that matrix is taken here with torch.
    r = _rng(4)
    n, d = 37, 8
    Q, K = r.standard_normal((1, n, d)), r.standard_normal((1, n, d))
    scale = 1 / math.sqrt(d)
    mass, rank = oz.token_scores(Q, K, np.arange(n), scale)
    S = torch.from_numpy(Q[0]) @ torch.from_numpy(K[0]).T * scale
    S = S.masked_fill(torch.triu(torch.ones(n, n, dtype=torch.bool), diagonal=1), float("-inf"))
    A = torch.softmax(S, dim=1).numpy()
    np.testing.assert_allclose(mass[0] * n, A.sum(0), atol=1e-13)
    np.testing.assert_allclose(rank[0], A.sum(0) / (n - np.arange(n)), atol=1e-13)
    assert oz.structural_count(n, np.arange(n)).tolist() == list(range(n, 0, -1))


def test_scattered_probes_columns_no_probe_sees_get_zero_rank_and_mass_still_sums_to_one():
    # hybrid-style probe list: scattered rows plus a recent span that stops before the end
    r = _rng(55)
    n, d = 120, 8
    Q, K = r.standard_normal((2, n, d)), r.standard_normal((1, n, d))
    probe = np.array([7, 30, 31, 64, 100, 101, 102, 103])
    mass, rank = oz.token_scores(Q, K, probe, 0.3)
    np.testing.assert_allclose(mass.sum(), 1.0, atol=1e-12)
    assert np.all(mass[0, 104:] == 0) and np.all(rank[0, 104:] == 0)
    cnt = oz.structural_count(n, probe)
    assert cnt[0] == 8 and cnt[8] == 7 and cnt[103] == 1 and cnt[104] == 0
    # a column only the last probes see is normalised by that smaller count: rank >= mass * m / cnt
    j = 102
    np.testing.assert_allclose(rank[0, j], mass[0, j] * len(probe) / cnt[j], rtol=1e-12)


def test_group_average_of_query_heads():
    r = _rng(5)
    n, d = 30, 8
    Q, K = r.standard_normal((4, n, d)), r.standard_normal((2, n, d))
    probe = np.arange(n - 5, n)
    mass, rank = oz.token_scores(Q, K, probe, 0.3)
    for g in range(2):
        ms = [oz.token_scores(Q[h:h + 1], K[g:g + 1], probe, 0.3) for h in (2 * g, 2 * g + 1)]
        np.testing.assert_allclose(mass[g], (ms[0][0][0] + ms[1][0][0]) / 2, atol=1e-15)
        np.testing.assert_allclose(rank[g], (ms[0][1][0] + ms[1][1][0]) / 2, atol=1e-15)


def test_transposed_or_unscaled_logits_would_fail():
    # A hand-computed 2-key case: probe at position 1, q=(1,0), k0=(2,0), k1=(0,3).
    Q = np.array([[[9.0, 9.0], [1.0, 0.0]]])
    K = np.array([[[2.0, 0.0], [0.0, 3.0]]])
    mass, _ = oz.token_scores(Q, K, np.array([1]), 0.5)
    e0, e1 = math.exp(1.0), math.exp(0.0)     # logits 2*0.5 and 0
    np.testing.assert_allclose(mass[0], [e0 / (e0 + e1), e1 / (e0 + e1)], atol=1e-15)


# --------------------------------------------------------------- selection
def _brute_min_subset(q, target):
    n = len(q)
    for size in range(1, n + 1):
        for sub in itertools.combinations(range(n), size):
            if sum(q[i] for i in sub) >= target:
                return size
    return n


@pytest.mark.parametrize("seed", range(12))
def test_select_matches_brute_force_subset_enumeration(seed):
    r = _rng(100 + seed)
    n = int(r.integers(2, 11))
    x = r.random(n).astype(np.float32) ** 3
    if seed % 3 == 0:                         # plant ties
        x[r.integers(0, n, 3)] = x[0]
    x = (x / x.sum()).astype(np.float32)
    tau = float(r.choice([0.5, 0.9, 0.95, 0.975, 0.99]))
    q = [int(v) for v in oz.fixed_point(x)]
    target = math.ceil(tau * float(sum(q)))
    p, T = oz.select(x, None, tau)
    assert p == max(1, _brute_min_subset(q, target))
    kept = sum(q[i] for i in T)
    assert kept >= target                                  # kept mass reaches tau
    assert kept - min(q[i] for i in T) < target or p == 1  # minimal: dropping the smallest kept fails
    assert all(x[i] >= x[j] for i in T for j in oz.complement(n, T))
    assert np.all(np.diff(T) > 0)
    assert len(T) + len(oz.complement(n, T)) == n


def test_fixed_point_is_exact_floor():
    x = np.array([0.0, 2.0 ** -41, 2.0 ** -40, 3 * 2.0 ** -40, 1.0, 0.3, 1e-30, 4095.5], dtype=np.float32)
    q = oz.fixed_point(x)
    for xi, qi in zip(x, q):
        assert int(qi) == int(Fraction(float(xi)) * 2 ** 40 // 1)


def test_ties_break_to_lower_index_and_set_is_permutation_invariant():
    x = np.array([0.1, 0.2, 0.2, 0.2, 0.1, 0.2], dtype=np.float32)
    # mass: total 1.0; tau 0.55 needs 3 of the four 0.2's -> lowest three indices
    p, T = oz.select(x, None, 0.55)
    assert p == 3 and T.tolist() == [1, 2, 3]
    # Reorder distinct values: the kept set maps through the permutation.
    r = _rng(7)
    y = (r.random(40) ** 4).astype(np.float32)
    p0, T0 = oz.select(y, None, 0.9)
    perm = r.permutation(40)
    p1, T1 = oz.select(y[perm], None, 0.9)
    assert p0 == p1 and sorted(perm[T1].tolist()) == T0.tolist()


def test_tau_one_keeps_all_and_count_is_monotone_in_tau():
    y = (_rng(8).random(200) ** 6).astype(np.float32)
    assert oz.select(y, None, 1.0)[0] == 200
    ps = [oz.count_important(y, t) for t in (0.1, 0.5, 0.9, 0.95, 0.975, 0.99, 0.999)]
    assert ps == sorted(ps) and ps[0] >= 1


def test_uniform_scores_closed_form():
    # n equal scores of 2^-7 (exact on the grid): p = ceil(tau * n).
    n = 128
    y = np.full(n, 2.0 ** -7, dtype=np.float32)
    for tau in (0.5, 0.9, 0.975, 0.99):
        p, T = oz.select(y, None, tau)
        assert p == math.ceil(tau * n) and T.tolist() == list(range(p))


def test_all_zero_scores_keep_one_token():
    p, T = oz.select(np.zeros(9, dtype=np.float32), None, 0.9)
    assert p == 1 and T.tolist() == [0]


def test_count_by_mass_identify_by_rank():
    mass = np.array([0.5, 0.3, 0.1, 0.1], dtype=np.float32)
    rank = np.array([0.1, 0.2, 0.9, 0.8], dtype=np.float32)
    p, T = oz.select(mass, rank, 0.75)       # 0.5 + 0.3 reaches 0.75 -> p = 2
    assert p == 2 and T.tolist() == [2, 3]   # the two largest by rank


# --------------------------------------------------------------- attention
def test_dense_attention_matches_torch_sdpa():
    r = _rng(9)
    n, d = 70, 16
    Q, K, V = (r.standard_normal((n, d)) for _ in range(3))
    scale = 1 / math.sqrt(d)
    O = oz.dense_causal_attention(Q, K, V, scale, row_block=32)
    t = lambda a: torch.from_numpy(a)[None, None]
    ref = torch.nn.functional.scaled_dot_product_attention(t(Q), t(K), t(V), is_causal=True, scale=scale)
    np.testing.assert_allclose(O, ref[0, 0].numpy(), atol=1e-12)


def test_kept_attention_tau_one_is_dense():
    r = _rng(10)
    n, d = 33, 8
    Q, K, V = (r.standard_normal((n, d)) for _ in range(3))
    O = oz.kept_token_attention(Q, K, V, np.arange(n), 0.4)
    np.testing.assert_allclose(O, oz.dense_causal_attention(Q, K, V, 0.4), atol=0)


def test_kept_attention_equals_key_masked_dense_attention():
    # Independent formulation: instead of gathering, block the dropped keys in
    # the full n x n softmax and read the kept rows.
    r = _rng(11)
    n, d = 41, 8
    Q, K, V = (r.standard_normal((n, d)) for _ in range(3))
    T = np.sort(r.choice(n, 17, replace=False))
    O = oz.kept_token_attention(Q, K, V, T, 0.35)
    keep = np.zeros(n, bool); keep[T] = True
    S = torch.from_numpy(Q @ K.T * 0.35)
    mask = torch.triu(torch.ones(n, n, dtype=torch.bool), 1) | torch.from_numpy(~keep)[None, :]
    A = torch.softmax(S.masked_fill(mask, float("-inf")), 1).numpy()
    full = np.nan_to_num(A) @ V
    np.testing.assert_allclose(O[T], full[T], atol=1e-13)
    assert np.all(O[~keep] == 0)


def test_kept_attention_zero_query_running_mean():
    r = _rng(12)
    n, d = 29, 4
    K, V = r.standard_normal((n, d)), r.standard_normal((n, d))
    T = np.array([0, 3, 4, 11, 28])
    O = oz.kept_token_attention(np.zeros((n, d)), K, V, T, 1.0)
    for i, t in enumerate(T):
        np.testing.assert_allclose(O[t], V[T[: i + 1]].mean(axis=0), atol=1e-14)


def test_kept_attention_rows_equal_the_whole_product_and_the_key_masked_softmax():
    # The row-at-a-time form used for spot checks at sizes where the whole product is slow: it must be
    # (a) the same rows of the gather-then-dense form, (b) the same rows of a full n x n softmax taken with
    # torch in which the dropped keys are blocked, (c) the running mean of V[T] when Q = 0, and it must see
    # the query's own key (row 0 returns V[T_0]) and nothing after it.
    r = _rng(15)
    n, d = 53, 8
    Q, K, V = (r.standard_normal((n, d)) for _ in range(3))
    T = np.sort(r.choice(n, 23, replace=False))
    rows = np.array([0, 1, 7, 21, 22])
    got = oz.kept_token_attention_rows(Q, K, V, T, rows, 0.3)
    np.testing.assert_allclose(got, oz.kept_token_attention(Q, K, V, T, 0.3, compact_out=True)[rows], atol=1e-14)
    keep = np.zeros(n, bool); keep[T] = True
    S = torch.from_numpy(Q @ K.T * 0.3)
    mask = torch.triu(torch.ones(n, n, dtype=torch.bool), 1) | torch.from_numpy(~keep)[None, :]
    A = torch.softmax(S.masked_fill(mask, float("-inf")), 1).numpy()
    np.testing.assert_allclose(got, (A @ V)[T[rows]], atol=1e-13)
    np.testing.assert_array_equal(got[0], V[T[0]])
    zero_q = oz.kept_token_attention_rows(np.zeros((n, d)), K, V, T, rows, 1.0)
    for o, i in zip(zero_q, rows):
        np.testing.assert_allclose(o, V[T[: i + 1]].mean(axis=0), atol=1e-14)
    # a later key must not leak into an earlier row: changing V at T_22 leaves row 21 as it was
    V2 = V.copy(); V2[T[22]] += 100.0
    np.testing.assert_array_equal(oz.kept_token_attention_rows(Q, K, V2, T, rows[:4], 0.3), got[:4])


def test_compaction_and_complement():
    r = _rng(13)
    K, V = r.standard_normal((20, 4)).astype(np.float32), r.standard_normal((20, 4)).astype(np.float32)
    T = np.array([1, 5, 19])
    Kc, Vc, ln = oz.compact_kv(K, V, T)
    assert ln == 3 and Kc.tobytes() == K[[1, 5, 19]].tobytes() and Vc.tobytes() == V[[1, 5, 19]].tobytes()
    assert sorted(oz.complement(20, T).tolist() + T.tolist()) == list(range(20))


def test_decode_is_last_row_of_dense_attention():
    r = _rng(14)
    L, d = 23, 8
    Kc, Vc = r.standard_normal((L + 5, d)), r.standard_normal((L + 5, d))
    q, kn, vn = r.standard_normal(d), r.standard_normal(d), r.standard_normal(d)
    o, Ko, Vo, L1 = oz.decode_step(q, kn, vn, Kc, Vc, L, 0.3)
    assert L1 == L + 1 and np.all(Ko[L] == kn) and np.all(Vo[L] == vn)
    Qfull = np.vstack([r.standard_normal((L, d)), q[None]])
    dense = oz.dense_causal_attention(Qfull, Ko, Vo, 0.3)
    np.testing.assert_allclose(o, dense[-1], atol=1e-14)


def test_layer_is_the_composition_of_its_steps():
    from workloads import make_custom
    w = make_custom(1, 4, 2, 96, 16, "f32", seed=3, m=16, tau=0.9)
    out = oz.zipvl_prefill_layer(w.Q[0], w.K[0], w.V[0], w.probe_pos, 0.9, w.scale)
    assert out["p"].shape == (2,) and all(1 <= p <= 96 for p in out["p"])
    for g in range(2):
        T = out["T"][g]
        assert len(T) == out["p"][g]
        # rows outside T are zero for both query heads of the group
        keep = np.zeros(96, bool); keep[T] = True
        assert np.all(out["O"][2 * g: 2 * g + 2][:, ~keep] == 0)
    full = oz.zipvl_prefill_layer(w.Q[0], w.K[0], w.V[0], w.probe_pos, 1.0, w.scale)
    np.testing.assert_allclose(full["O"][0], oz.dense_causal_attention(w.Q[0, 0], w.K[0, 0], w.V[0, 0], w.scale), atol=1e-13)


def test_shared_scores_are_the_head_mean_and_reduce_to_the_single_head_case():
    from workloads import make_custom
    r = _rng(31)
    x = r.random((5, 200)).astype(np.float32)
    x /= x.sum(axis=1, keepdims=True)
    s = oz.share_scores(x)
    assert s.dtype == np.float32 and s.shape == (200,)
    # the exact mean, to fp32 rounding of 5 additions and one multiplication
    np.testing.assert_allclose(s.astype(np.float64), x.astype(np.float64).mean(axis=0), rtol=6 * 2.0 ** -24)
    assert abs(float(s.astype(np.float64).sum()) - 1.0) < 1e-5          # still a distribution over tokens
    # identical heads: the mean is the head (power-of-two head counts are exact)
    one = x[:1]
    assert oz.share_scores(np.repeat(one, 4, axis=0)).tobytes() == one[0].tobytes()
    assert oz.share_scores(one).tobytes() == one[0].tobytes()
    # a layer with one KV head selects the same set either way
    w = make_custom(1, 2, 1, 96, 16, "f32", seed=4, m=16, tau=0.9)
    a = oz.zipvl_prefill_layer(w.Q[0], w.K[0], w.V[0], w.probe_pos, 0.9, w.scale)
    b = oz.zipvl_prefill_layer(w.Q[0], w.K[0], w.V[0], w.probe_pos, 0.9, w.scale, shared=True)
    assert np.array_equal(a["T"][0], b["T"][0]) and np.array_equal(a["O"], b["O"])


def test_shared_layer_uses_one_set_for_every_head():
    from workloads import make_custom
    w = make_custom(1, 4, 2, 96, 16, "f32", seed=3, m=16, tau=0.9)
    out = oz.zipvl_prefill_layer(w.Q[0], w.K[0], w.V[0], w.probe_pos, 0.9, w.scale, shared=True)
    assert out["p"][0] == out["p"][1] and np.array_equal(out["T"][0], out["T"][1])
    # the set is the selection on the mean of the two heads' fp32 scores
    p, T = oz.select(oz.share_scores(out["mass"]), oz.share_scores(out["rank"]), 0.9)
    assert p == out["p"][0] and np.array_equal(T, out["T"][0])
    # and each head's output is the kept-token attention over that set
    for h in range(4):
        ref = oz.kept_token_attention(w.Q[0, h], w.K[0, h // 2], w.V[0, h // 2], T, w.scale)
        np.testing.assert_array_equal(out["O"][h], ref)


# ------------------------------------------------------- mixed-precision cache
@pytest.mark.parametrize("bits", [2, 4])
def test_row_quantiser_is_nearest_grid_point_with_half_step_error(bits):
    r = _rng(60 + bits)
    X = r.standard_normal((40, 32)).astype(np.float32)
    X[3] = 1.25                                   # constant row: scale 0, every code 0, exact
    codes, scale, zero = oz.quantize_rows(X, bits)
    assert codes.dtype == np.uint8 and codes.max() <= 2 ** bits - 1
    assert scale.dtype == np.float16 and zero.dtype == np.float16
    s, z = scale.astype(np.float64), zero.astype(np.float64)
    assert s[3] == 0 and not codes[3].any() and np.all(oz.dequantize_rows(codes, scale, zero)[3] == 1.25)
    # the row minimum is code 0, the maximum the top code
    live = s > 0
    assert np.all(codes[np.arange(40), X.argmin(axis=1)][live] == 0)
    assert np.all(codes[np.arange(40), X.argmax(axis=1)][live] == 2 ** bits - 1)
    # independent definition: the code is the grid point nearest to x (checked by enumeration of the grid)
    grid = z[:, None, None] + s[:, None, None] * np.arange(2 ** bits)[None, None, :]
    dist = np.abs(X.astype(np.float64)[:, :, None] - grid)
    best = dist.min(axis=2)
    mine = np.abs(X.astype(np.float64) - oz.dequantize_rows(codes, scale, zero))
    assert np.all(mine[live] <= best[live] + 1e-6 * s[live][:, None])
    # hence the half-step bound (the fp16 rounding of the parameters can push the ends out by a little)
    assert np.all(mine[live] <= 0.5 * s[live][:, None] * 1.01 + 2e-3 * np.abs(X[live]).max())


def test_values_on_the_grid_survive_quantisation_exactly():
    z, s = 0.5, 0.125                             # representable in fp16; row spans the whole grid
    for bits in (2, 4):
        q = np.arange(2 ** bits)
        X = (z + s * np.tile(q, 3)).astype(np.float32)[None, :]
        codes, scale, zero = oz.quantize_rows(X, bits)
        assert float(zero[0]) == z and float(scale[0]) == s
        assert np.array_equal(codes[0], np.tile(q, 3))
        assert np.array_equal(oz.dequantize_rows(codes, scale, zero)[0], X[0].astype(np.float64))


def test_mixed_precision_cache_splits_by_T_and_decodes_close_to_the_full_cache():
    r = _rng(64)
    n, d = 96, 32
    K, V = r.standard_normal((n, d)).astype(np.float32), r.standard_normal((n, d)).astype(np.float32)
    T = np.sort(r.choice(n, 30, replace=False))
    qc = oz.quantize_kv(K, V, T)
    assert np.array_equal(qc["U"], np.setdiff1d(np.arange(n), T))
    assert qc["K_hi"][0].shape == (30, d) and qc["K_lo"][0].shape == (66, d)
    assert np.array_equal(qc["K_hi"][0], oz.quantize_rows(K[T], 4)[0])
    assert np.array_equal(qc["V_lo"][0], oz.quantize_rows(V[qc["U"]], 2)[0])
    q = r.standard_normal(d)
    full = oz.decode_attention(q, K, V, n, 0.2)
    # 16-bit codes in both groups: the quantised path must reproduce the full-cache answer
    fine = oz.decode_attention_quantized(q, oz.quantize_kv(K, V, T, 16 - 8, 16 - 8), 0.2)     # 8 bits each
    assert np.abs(fine - full).max() < 2e-2
    coarse = oz.decode_attention_quantized(q, qc, 0.2)
    assert np.abs(coarse - full).max() < 0.6 and np.abs(coarse - full).max() > np.abs(fine - full).max()
    # appended rows take part unquantised: appending the same token twice equals decode over n+2 rows
    kt, vt = r.standard_normal((2, d)), r.standard_normal((2, d))
    a = oz.decode_attention_quantized(q, qc, 0.2, kt, vt)
    Kd = np.concatenate([oz.dequantize_rows(*qc["K_hi"]), oz.dequantize_rows(*qc["K_lo"]), kt])
    Vd = np.concatenate([oz.dequantize_rows(*qc["V_hi"]), oz.dequantize_rows(*qc["V_lo"]), vt])
    np.testing.assert_allclose(a, oz.decode_attention(q, Kd, Vd, n + 2, 0.2), atol=1e-13)


def test_kv_compression_matches_table_3():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "kv_quant_compression.txt")) if l.strip() and not l.startswith("#")]
    assert len(rows) == 2
    for ratio_pct, comp in rows:
        got = oz.kv_quant_compression(float(ratio_pct) / 100.0)
        assert abs(got - float(comp)) / float(comp) < 0.01, (ratio_pct, got, comp)
    # with a pair of parameters per token and KV head (128 elements) the same split compresses less
    assert oz.kv_quant_compression(0.286, elems_per_group=128) < oz.kv_quant_compression(0.286)
    assert abs(oz.kv_quant_compression(1.0, param_bits=0) - 4.0) < 1e-12 and abs(oz.kv_quant_compression(0.0, param_bits=0) - 8.0) < 1e-12


# ------------------------------------------------------- paper's accounting
def test_ratio_accounting_matches_tables_2_and_3():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "ratio_accounting.txt")) if l.strip() and not l.startswith("#")]
    assert len(rows) == 2
    for frames, ratio, flops, kv in rows:
        r = float(ratio) / 100
        assert round(100 * oz.attention_flops_reduction(r), 1) == float(flops)
        assert round(100 * oz.kv_cache_reduction(r), 1) == float(kv)
