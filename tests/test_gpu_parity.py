"""Parity of the HIP path (through the C ABI) against the CPU float64 oracle.

Rules: kept count and kept index set are exact when the oracle's selection is
fed the GPU's own fp32 scores; scores within 1e-9 + 1e-5*value (either input
dtype: the oracle sees the exact device inputs); attention outputs within max-abs 2e-2
(bf16) / 1e-4 (fp32) with the oracle evaluated on the GPU's index set;
compaction bit-exact.
"""
import math
import sys

import numpy as np
import pytest
import torch

import paper_2410_08584_amd as z
from oracle import zipvl_oracle as oz
from workloads import hybrid_probes, make_custom, make_workload

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
ATOL_OUT = {"f32": 1e-4, "bf16": 2e-2}


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def dev(x32: np.ndarray, dtype: str) -> torch.Tensor:
    t = torch.from_numpy(np.ascontiguousarray(x32)).to(DEV)
    return t.to(torch.bfloat16) if dtype == "bf16" else t


def host64(t: torch.Tensor) -> np.ndarray:
    return t.detach().to(torch.float32).cpu().numpy().astype(np.float64)


def score_tol(dtype):
    # The oracle is fed the exact device inputs, so bf16 storage adds nothing: products of bf16 values are
    # exact in fp32 and both dtypes accumulate in fp32.  Relative error of a probability = ln 2 x the absolute
    # error of its log2-domain exponent (about 2e-6 at |logit| <= 30) plus one ulp each for exp2 and log2.
    return (1e-9, 1e-5)


WORST_SCORE_ERR = {"rel": 0.0}       # largest |got - ref| / (1e-9/1e-5 + |ref|) seen in this process, for the log


def assert_scores_close(got, ref, dtype, what):
    a, r = score_tol(dtype)
    err = np.abs(got - ref) - (a + r * np.abs(ref))
    WORST_SCORE_ERR["rel"] = max(WORST_SCORE_ERR["rel"], float((np.abs(got - ref) / (a / r + np.abs(ref))).max()))
    assert err.max() <= 0, f"{what}: worst excess {err.max():.3e} at {np.unravel_index(err.argmax(), err.shape)}"


# ------------------------------------------------------------------ compaction
@pytest.mark.parametrize("dtype,d", [("bf16", 128), ("f32", 64), ("bf16", 64), ("f32", 128)])
def test_compact_kv_bit_exact(dtype, d):
    say(f"compact_kv dtype={dtype} d={d}")
    B, Hkv, n, cap = 2, 3, 333, 300
    r = np.random.Generator(np.random.PCG64(5))
    w = make_custom(B, Hkv, Hkv, n, d, dtype, seed=11)
    # token-major memory order [B,n,H,d] viewed as [B,H,n,d]
    K = dev(w.K, dtype).permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
    V = dev(w.V, dtype)
    ks = [1, 64, 65, 300, 7, 129]
    idx = np.zeros((B * Hkv, n), dtype=np.int32)
    for u, k in enumerate(ks):
        idx[u, :k] = np.sort(r.choice(n, k, replace=False))
    Kc, Vc, ln = z.zipvl_compact_kv(K, V, torch.from_numpy(idx).to(DEV),
                                    torch.tensor(ks, dtype=torch.int32, device=DEV), cap)
    torch.cuda.synchronize()
    assert ln.cpu().tolist() == ks
    Kc_h, Vc_h = Kc.to(torch.float32).cpu().numpy(), Vc.to(torch.float32).cpu().numpy()
    for u, k in enumerate(ks):
        b, g = divmod(u, Hkv)
        ko, vo, _ = oz.compact_kv(w.K[b, g], w.V[b, g], idx[u, :k])
        assert Kc_h[u, :k].tobytes() == ko.tobytes() and Vc_h[u, :k].tobytes() == vo.tobytes()
    # all rows, and a cap smaller than k
    Kc2, Vc2, ln2 = z.zipvl_compact_kv(K, V, None, None, 100)
    torch.cuda.synchronize()
    assert ln2.cpu().tolist() == [100] * (B * Hkv)
    assert Kc2.to(torch.float32).cpu().numpy()[4].tobytes() == w.K[1, 1, :100].tobytes()


# ------------------------------------------------------------------ selection
SELECT_WS = {}


def _select_case(name, mass, rank, tau):
    say(f"select case={name} units={mass.shape[0]} n={mass.shape[1]} tau={tau}")
    mass = np.ascontiguousarray(mass)
    rank = None if rank is None else np.ascontiguousarray(rank)
    m_d = torch.from_numpy(mass).to(DEV)
    r_d = None if rank is None else torch.from_numpy(rank).to(DEV)
    units = mass.shape[0]
    ws = SELECT_WS.setdefault(units, z.select_workspace(units, DEV))      # reused across cases: every call must leave it zero
    ref = [oz.select(mass[u], None if rank is None else rank[u], tau) for u in range(units)]
    for form, w_ in (("one kernel", None), ("two kernels", ws)):
        idx, k = z.zipvl_select(m_d, r_d, tau, ws=w_)
        torch.cuda.synchronize()
        idx, k = idx.cpu().numpy(), k.cpu().numpy()
        for u in range(units):
            p, T = ref[u]
            assert k[u] == p, f"{name} ({form}) unit {u}: k {k[u]} != {p}"
            assert np.array_equal(idx[u, :p], T), f"{name} ({form}) unit {u}: index set differs"
    assert int(ws.view(torch.int32).abs().sum().item()) == 0, f"{name}: the workspace was not left zero"


def test_select_exact_on_synthetic_distributions():
    r = np.random.Generator(np.random.PCG64(21))

    def norm(x):
        return (x / x.sum(axis=1, keepdims=True)).astype(np.float32)

    for n in (1, 2, 63, 64, 65, 577, 1024, 4097, 18432):
        skew = norm(r.random((3, n)) ** 8 + 1e-9)
        rk = (skew * (1 + 0.5 * r.random((3, n)))).astype(np.float32)
        _select_case(f"skew-n{n}", skew, rk, 0.975)
        _select_case(f"skew-single-n{n}", skew, None, 0.9)
    # beyond the LDS-resident key count (27648): keys are re-read from memory on every digit pass
    for n in (27648, 27649, 131072):
        big = norm(r.random((2, n)) ** 6 + 1e-9)
        _select_case(f"long-n{n}", big, (big * (1 + r.random((2, n)))).astype(np.float32), 0.975)
        _select_case(f"long-single-n{n}", big, None, 0.95)
    n = 3000
    ties = norm(np.round(r.random((2, n)) * 6) + 1.0)            # 7 distinct values: many ties
    _select_case("ties", ties, ties[:, ::-1].copy(), 0.7)
    _select_case("ties-single", ties, None, 0.6180339887)
    uni = np.full((2, 1000), 2.0 ** -10, dtype=np.float32)
    for tau in (0.5, 0.975, 0.999, 1.0):
        _select_case("uniform", uni, None, tau)
    _select_case("zeros", np.zeros((2, 500), dtype=np.float32), None, 0.9)
    onehot = np.zeros((2, 700), dtype=np.float32); onehot[0, 699] = 1.0; onehot[1, 0] = 1.0
    _select_case("onehot", onehot, None, 0.99)
    tiny = norm(r.random((2, 2048))) * np.float32(2.0 ** -30)      # most values below the 2^-40 grid step
    _select_case("tiny", tiny.astype(np.float32), None, 0.95)
    wide = norm(np.exp(r.normal(0, 6, (4, 8192))))                # many exponents
    for tau in (0.3, 0.95, 0.975, 0.99, 0.99999):
        _select_case("lognormal", wide, (wide * r.random((4, 8192))).astype(np.float32), tau)
    # softmax-like: a few heavy tokens and a long tail, rank boosts the last 64 columns
    tail = norm(np.concatenate([r.random((2, 40)) * 50, r.random((2, 18392)) * 0.01], axis=1))
    rk = tail.copy(); rk[:, -64:] *= np.linspace(1, 64, 64, dtype=np.float32)
    _select_case("heavy+tail", tail, rk, 0.975)
    # one first-digit bin (a sixteenth of a binade) holding more elements than the gathered list takes, and exactly as many
    for cnt in (2048, 2049, 5000):
        band = (1.0 + r.random((2, cnt)) / 17.0).astype(np.float32)        # all in [1, 1 + 1/16): one bin
        rest = (r.random((2, 3000)) * 0.9).astype(np.float32)
        x = norm(np.concatenate([rest, band], axis=1)[:, r.permutation(3000 + cnt)])
        _select_case(f"crowded-bin-{cnt}", x, (x * (1 + 0.01 * r.random(x.shape))).astype(np.float32), 0.6)
        _select_case(f"crowded-bin-single-{cnt}", x, None, 0.5)
    dup = norm(np.repeat(r.random((2, 40)) ** 3, 100, axis=1)[:, r.permutation(4000)])      # 40 distinct values, 100 copies each
    _select_case("blocks-of-equal-values", dup, dup[:, ::-1].copy(), 0.8)


def test_select_status_word_reports_inputs_outside_the_contract():
    """The optional status word: 0 for valid input, and one bit each for a sign-bit entry, a non-finite entry and a
    mass that sums to 2 or more; both forms of the call; the selection itself still runs (and, for the sign-bit
    case, treats the entry as zero: the result equals the oracle's on the cleaned vector)."""
    say("select status word")
    r = np.random.Generator(np.random.PCG64(23))
    n = 5000
    good = r.random((5, n)).astype(np.float32) ** 4
    good /= good.sum(axis=1, keepdims=True)
    x = np.ascontiguousarray(good.astype(np.float32))
    x[1, 17] = -x[1, 17]                         # negative entry
    x[2, 4000] = np.float32("inf")               # infinity in mass
    x[3] *= np.float32(2.5)                      # sums to 2.5: the integer sum no longer fits its field
    rk = np.ascontiguousarray((good * (1 + r.random((5, n)))).astype(np.float32))
    rk[4, 99] = np.float32("nan")                # NaN in rank only
    ws = z.select_workspace(5, DEV)
    expect = [0, z.SELECT_NEGATIVE, z.SELECT_NONFINITE, z.SELECT_OVERFLOW, z.SELECT_NONFINITE]
    for w_ in (None, ws):
        st = torch.full((5,), -1, dtype=torch.int32, device=DEV)
        idx, k = z.zipvl_select(torch.from_numpy(x).to(DEV), torch.from_numpy(rk).to(DEV), 0.9, ws=w_, status=st)
        torch.cuda.synchronize()
        assert st.cpu().tolist() == expect, st.cpu().tolist()
        for u in (0, 1):                         # valid unit, and the unit whose negative entry counts as zero
            clean = np.where(np.signbit(x[u]), np.float32(0), x[u])
            p, T = oz.select(clean, rk[u], 0.9)
            assert int(k[u]) == p and np.array_equal(idx[u, :p].cpu().numpy(), T)
    # without a status word nothing is written and valid input gives the same result
    idx2, k2 = z.zipvl_select(torch.from_numpy(x[:1]).to(DEV), torch.from_numpy(rk[:1]).to(DEV), 0.9)
    torch.cuda.synchronize()
    assert int(k2[0]) == int(k[0]) and torch.equal(idx2[0, :int(k2[0])], idx[0, :int(k2[0])])


def test_scores_per_query_head_are_the_single_head_scores():
    """ZIPVL_SCORE_PER_QHEAD: one row per query head, nothing averaged (the paper's single-head equations); the group
    mean of those rows is what the default mode returns."""
    say("score per query head")
    B, Hq, Hkv, n, d, dtype = 2, 6, 2, 777, 128, "bf16"
    G = Hq // Hkv
    w = make_custom(B, Hq, Hkv, n, d, dtype, seed=19)
    Q, K = dev(w.Q, dtype), dev(w.K, dtype)
    mass_h, rank_h = z.zipvl_score(Q, K, w.probe_pos, w.scale, flags=z.SCORE_PER_QHEAD)
    mass_g, rank_g = z.zipvl_score(Q, K, w.probe_pos, w.scale)
    torch.cuda.synchronize()
    assert mass_h.shape == (B * Hq, n) and mass_g.shape == (B * Hkv, n)
    mh, rh = host64(mass_h).reshape(B, Hq, n), host64(rank_h).reshape(B, Hq, n)
    for b in range(B):
        for h in range(Hq):
            mo, ro = oz.token_scores(w.Q[b, h:h + 1], w.K[b, h // G:h // G + 1], w.probe_pos, w.scale)    # one head, its own KV head
            assert_scores_close(mh[b, h][None], mo, dtype, "mass")
            assert_scores_close(rh[b, h][None], ro, dtype, "rank")
    np.testing.assert_allclose(mh.reshape(B, Hkv, G, n).mean(axis=2), host64(mass_g).reshape(B, Hkv, n), rtol=2e-6, atol=1e-12)


# ------------------------------------------------------------------ scores
SCORE_CASES = [
    # B, Hq, Hkv, n, d, dtype, m, probe
    (1, 4, 4, 576, 64, "f32", 64, None),
    (2, 4, 2, 700, 128, "bf16", 64, None),
    (1, 6, 2, 333, 64, "bf16", 24, None),
    (1, 2, 1, 1500, 128, "f32", 64, None),
    (1, 7, 1, 2100, 128, "bf16", 64, "scattered"),
    (1, 2, 2, 70, 64, "f32", 64, None),
    (1, 4, 2, 1500, 128, "bf16", 128, "hybrid"),
    (1, 2, 2, 900, 64, "f32", 100, "hybrid"),
    (1, 3, 1, 640, 64, "bf16", 128, "hybrid"),
    (1, 2, 1, 700, 128, "f32", 128, "hybrid"),
]


@pytest.mark.parametrize("case", SCORE_CASES, ids=lambda c: f"B{c[0]}Hq{c[1]}Hkv{c[2]}n{c[3]}d{c[4]}{c[5]}m{c[6]}{c[7] or ''}")
def test_scores_match_oracle(case):
    B, Hq, Hkv, n, d, dtype, m, probe = case
    say(f"score case={case}")
    pp = None
    if probe == "scattered":
        r = np.random.Generator(np.random.PCG64(3))
        pp = np.sort(np.concatenate([r.choice(n - 200, m - 20, replace=False), np.arange(n - 20, n)])).astype(np.int32)
    if probe == "hybrid":
        pp = hybrid_probes(n, seed=n, recent=64, random=m - 64)
    w = make_custom(B, Hq, Hkv, n, d, dtype, seed=100 + n, m=m, probe_pos=pp)
    assert len(w.probe_pos) == m
    Q, K = dev(w.Q, dtype), dev(w.K, dtype)
    mass, rank = z.zipvl_score(Q, K, w.probe_pos, w.scale)
    torch.cuda.synchronize()
    mass, rank = host64(mass).reshape(B, Hkv, n), host64(rank).reshape(B, Hkv, n)
    for b in range(B):
        mo, ro = oz.token_scores(w.Q[b], w.K[b], w.probe_pos, w.scale)
        assert_scores_close(mass[b], mo, dtype, "mass")
        assert_scores_close(rank[b], ro, dtype, "rank")
        np.testing.assert_allclose(mass[b].sum(axis=1), 1.0, atol=2e-5)
    say(f"  worst relative score error so far {WORST_SCORE_ERR['rel']:.2e} (bound 1e-5)")


# ------------------------------------------------------------------ attention
def _attention_case(B, Hq, Hkv, n, d, dtype, ks, seed=0, flags=0, dense=False, reshape_inputs=None):
    G = Hq // Hkv
    w = make_custom(B, Hq, Hkv, n, d, dtype, seed=seed)
    if reshape_inputs is not None:                 # (Q, K) -> (Q', K'), rounded back to the storage type
        q2, k2 = reshape_inputs(w.Q, w.K)
        rnd = (lambda x: torch.from_numpy(x).bfloat16().float().numpy()) if dtype == "bf16" else (lambda x: x.astype(np.float32))
        w.Q, w.K = rnd(np.ascontiguousarray(q2, dtype=np.float32)), rnd(np.ascontiguousarray(k2, dtype=np.float32))
    Q, K, V = dev(w.Q, dtype), dev(w.K, dtype), dev(w.V, dtype)
    units = B * Hkv
    r = np.random.Generator(np.random.PCG64(seed + 1))
    idx = np.zeros((units, n), dtype=np.int32)
    for u in range(units):
        idx[u, :ks[u]] = np.sort(r.choice(n, ks[u], replace=False))
    if dense:
        O = z.zipvl_sparse_prefill(Q, K, V, None, None, w.scale)
    else:
        O = torch.full((B, Hq, n, d), 7.0, dtype=Q.dtype, device=DEV)   # poison: dropped rows must be rewritten
        z.zipvl_sparse_prefill(Q, K, V, torch.from_numpy(idx).to(DEV),
                               torch.tensor(ks, dtype=torch.int32, device=DEV), w.scale, flags, O=O)
    torch.cuda.synchronize()
    Oh = host64(O)
    worst = 0.0
    for b in range(B):
        for h in range(Hq):
            g = h // G
            u = b * Hkv + g
            T = np.arange(n) if dense else idx[u, :ks[u]]
            ref = oz.kept_token_attention(w.Q[b, h], w.K[b, g], w.V[b, g], T, w.scale,
                                          compact_out=bool(flags & z.OUT_COMPACT))
            got = Oh[b, h, :len(T)] if flags & z.OUT_COMPACT else Oh[b, h]
            worst = max(worst, np.abs(got - ref).max())
    say(f"  worst |dO| = {worst:.3e}")
    assert worst <= ATOL_OUT[dtype]


def test_attention_fp32_small_ragged():
    say("attention fp32 d=64 ragged k")
    _attention_case(1, 4, 4, 576, 64, "f32", [576, 1, 130, 67], seed=1)


def test_attention_bf16_gqa_ragged():
    say("attention bf16 d=128 GQA ragged k")
    _attention_case(2, 6, 2, 700, 128, "bf16", [700, 257, 64, 385], seed=2)


def test_attention_kept_count_on_tile_boundaries():
    say("attention bf16 d=128, k = 128, 256, 384 and n (dropped tail must be cleared)")
    _attention_case(2, 4, 2, 640, 128, "bf16", [128, 256, 384, 640], seed=9)
    _attention_case(1, 2, 2, 384, 64, "f32", [384, 128], seed=10)


def test_attention_bf16_d64_and_fp32_d128():
    say("attention bf16 d=64")
    _attention_case(1, 2, 2, 300, 64, "bf16", [300, 129], seed=3)
    say("attention fp32 d=128")
    _attention_case(1, 2, 1, 260, 128, "f32", [200], seed=4)


def test_attention_dense_mode_equals_dense_oracle():
    say("attention dense (idx=k=NULL)")
    _attention_case(1, 4, 2, 450, 128, "bf16", [450, 450], seed=5, dense=True)
    _attention_case(1, 2, 2, 200, 64, "f32", [200, 200], seed=6, dense=True)


def test_attention_logits_far_from_zero():
    """Rows whose logits leave the range in which exponentials need no offset (the kernel's first pass takes
    exp2 of the scaled logits as they are and repeats a workgroup with running maxima when a row sum leaves
    [2^-64, 2^64]): logits of +-150 and more, logits that are all near -100 or near +100, and a mix of ordinary
    and extreme heads in one launch."""
    say("attention with very large / very negative logits")
    for dtype, d, seed, gain in (("bf16", 128, 31, 40.0), ("f32", 64, 32, 16.0)):   # fp32: +-60, within its 1e-4 bound
        ks = [450, 257, 129, 450]
        _attention_case(1, 4, 4, 450, d, dtype, ks, seed=seed, reshape_inputs=lambda q, k: (q * gain, k))
        shift = 3.0 if d == 128 else 4.5
        _attention_case(1, 4, 4, 450, d, dtype, ks, seed=seed + 2, reshape_inputs=lambda q, k: (q - shift, k + shift))
        _attention_case(1, 4, 4, 450, d, dtype, ks, seed=seed + 4, reshape_inputs=lambda q, k: (q + shift, k + shift))
        def mixed(q, k):
            q = q.copy(); q[:, 1] *= gain; q[:, 2] -= shift; k = k.copy(); k[:, 2] += shift
            return q, k
        _attention_case(1, 4, 4, 450, d, dtype, ks, seed=seed + 6, reshape_inputs=mixed)


def test_attention_compact_output_rows():
    say("attention OUT_COMPACT")
    _attention_case(1, 4, 2, 500, 128, "bf16", [333, 128], seed=7, flags=z.OUT_COMPACT)


@pytest.mark.parametrize("n,gain", [(400, 1.0), (448, 1.0), (448, 40.0)])
def test_attention_on_already_compacted_cache(n, gain):
    # n = 448 (whole 64-row tiles, contiguous rows) reads the evicted K cache in place; n = 400 repacks it;
    # gain 40: logits far outside the range the offset-free pass accepts, so every workgroup repeats its keys
    say(f"attention KV_ALREADY_COMPACT n={n} gain={gain}")
    B, Hq, Hkv, d, dtype = 1, 4, 2, 128, "bf16"
    w = make_custom(B, Hq, Hkv, n, d, dtype, seed=8)
    if gain != 1.0:
        w.Q = torch.from_numpy(w.Q * np.float32(gain)).bfloat16().float().numpy()
    Q, K, V = dev(w.Q, dtype), dev(w.K, dtype), dev(w.V, dtype)
    ks = [211, 77]
    r = np.random.Generator(np.random.PCG64(9))
    idx = np.zeros((2, n), dtype=np.int32)
    for u in range(2):
        idx[u, :ks[u]] = np.sort(r.choice(n, ks[u], replace=False))
    idx_d, k_d = torch.from_numpy(idx).to(DEV), torch.tensor(ks, dtype=torch.int32, device=DEV)
    Kc = torch.full((2, n, d), float("nan"), dtype=torch.bfloat16, device=DEV)   # rows beyond k stay NaN
    Vc = torch.full((2, n, d), float("nan"), dtype=torch.bfloat16, device=DEV)
    z.zipvl_compact_kv(K, V, idx_d, k_d, n, Kc=Kc, Vc=Vc)
    O1 = z.zipvl_sparse_prefill(Q, K, V, idx_d, k_d, w.scale)
    O2 = z.zipvl_sparse_prefill(Q, Kc.view(B, Hkv, n, d), Vc.view(B, Hkv, n, d), idx_d, k_d, w.scale,
                                z.KV_ALREADY_COMPACT)
    torch.cuda.synchronize()
    assert not torch.isnan(O2.float()).any()
    assert torch.equal(O1, O2)
    Oh, G = host64(O2), Hq // Hkv
    worst = max(np.abs(Oh[0, h] - oz.kept_token_attention(w.Q[0, h], w.K[0, h // G], w.V[0, h // G], idx[h // G, :ks[h // G]], w.scale)).max()
                for h in range(Hq))
    say(f"  worst |dO| = {worst:.3e}")
    assert worst <= ATOL_OUT[dtype]


# ------------------------------------------------------------------ whole layer
def _edge_rows(p, r, extra):
    """Kept-token rows at the edges of the attention kernel's tiling (128 queries per workgroup, 32 per
    wave, 64 keys per tile): first and last rows of the first, a middle and the last query tile, rows on
    both sides of 64-key tile edges, the last kept row, plus `extra` random rows."""
    last_q, last_k, mid = (p - 1) // 128 * 128, (p - 1) // 64 * 64, (p // 2) // 128 * 128
    cand = [0, 1, 31, 32, 63, 64, 65, 127, 128, 129, mid - 1, mid, mid + 63, mid + 64, mid + 127,
            last_q - 1, last_q, last_k - 1, last_k, p - 2, p - 1]
    cand = [c for c in cand if 0 <= c < p]
    return np.unique(np.concatenate([np.array(cand, dtype=np.int64), r.integers(0, p, extra)]))


def _layer_parity(w, tau, sample_rows=None, heads=None, whole_heads=()):
    """Score, select, compaction and attention of one layer against the oracle.  The attention is run
    twice: on the original K, V (the library gathers K[T], V[T] itself), and exactly as the benchmark's
    step runs it - K and V read in place from the evicted cache (rows past k hold NaN), full-size output
    with the dropped rows cleared by the kernel.  Both outputs meet the oracle on every checked row.
    sample_rows=None: every row of the heads in `heads` (all heads when None).  Otherwise the tile-edge
    rows plus `sample_rows` random ones of those heads, and every row of the heads in `whole_heads`."""
    spec = w.spec
    B, Hq, Hkv, n, d, dtype = w.Q.shape[0], spec.Hq, spec.Hkv, spec.n, spec.d, spec.dtype
    G = Hq // Hkv
    Q, K, V = dev(w.Q, dtype), dev(w.K, dtype), dev(w.V, dtype)
    mass, rank = z.zipvl_score(Q, K, w.probe_pos, w.scale)
    idx, k = z.zipvl_select(mass, rank, tau)
    Kc = torch.full((B * Hkv, n, d), float("nan"), dtype=Q.dtype, device=DEV)
    Vc = torch.full((B * Hkv, n, d), float("nan"), dtype=Q.dtype, device=DEV)
    _, _, ln = z.zipvl_compact_kv(K, V, idx, k, n, Kc=Kc, Vc=Vc)
    outs = {"gathered by the library": z.zipvl_sparse_prefill(Q, K, V, idx, k, w.scale)}
    O2 = torch.full((B, Hq, n, d), 7.0, dtype=Q.dtype, device=DEV)      # poison: every row must be rewritten
    z.zipvl_sparse_prefill(Q, Kc.view(B, Hkv, n, d), Vc.view(B, Hkv, n, d), idx, k, w.scale,
                           z.OUT_FULL | z.KV_ALREADY_COMPACT, O=O2)
    outs["evicted cache read in place (the benchmark's step)"] = O2
    torch.cuda.synchronize()
    mass_h, rank_h = mass.cpu().numpy(), rank.cpu().numpy()
    idx_h, k_h = idx.cpu().numpy(), k.cpu().numpy()
    assert ln.cpu().tolist() == k_h.tolist()
    kept = []
    for b in range(B):
        mo, ro = oz.token_scores(w.Q[b], w.K[b], w.probe_pos, w.scale)
        assert_scores_close(mass_h.reshape(B, Hkv, n)[b].astype(np.float64), mo, dtype, "mass")
        assert_scores_close(rank_h.reshape(B, Hkv, n)[b].astype(np.float64), ro, dtype, "rank")
        for g in range(Hkv):
            u = b * Hkv + g
            p, T = oz.select(mass_h[u], rank_h[u], tau)             # oracle fed the GPU's fp32 scores
            assert k_h[u] == p and np.array_equal(idx_h[u, :p], T), f"unit {u}: selection differs"
            kept.append(p / n)
            ko, vo, _ = oz.compact_kv(w.K[b, g], w.V[b, g], T)
            assert Kc[u, :p].to(torch.float32).cpu().numpy().tobytes() == ko.tobytes()
            assert Vc[u, :p].to(torch.float32).cpu().numpy().tobytes() == vo.tobytes()
    worst = {name: 0.0 for name in outs}
    r = np.random.Generator(np.random.PCG64(77))
    checked_rows = 0
    for b in range(B):
        for h in (range(Hq) if heads is None else sorted(set(heads) | set(whole_heads))):
            g = h // G
            u = b * Hkv + g
            T = idx_h[u, :k_h[u]]
            whole = sample_rows is None or h in whole_heads
            if whole:
                ref = oz.kept_token_attention(w.Q[b, h], w.K[b, g], w.V[b, g], T, w.scale)
                checked_rows += len(T)
            else:
                rows = _edge_rows(len(T), r, sample_rows)
                ref = oz.kept_token_attention_rows(w.Q[b, h], w.K[b, g], w.V[b, g], T, rows, w.scale)
                dropped = np.setdiff1d(np.arange(n), T)
                checked_rows += len(rows)
            for name, O in outs.items():
                Oh = host64(O[b, h])
                assert not np.isnan(Oh).any(), f"{name}: NaN in head {h}"
                if whole:
                    worst[name] = max(worst[name], np.abs(Oh - ref).max())       # dropped rows: ref is 0 there
                else:
                    worst[name] = max(worst[name], np.abs(Oh[T[rows]] - ref).max())
                    assert not Oh[dropped].any(), f"{name}: dropped rows must be zero"
    say(f"  kept {100 * np.mean(kept):.1f}% (min {100 * min(kept):.1f}, max {100 * max(kept):.1f}); {checked_rows} kept rows checked; "
        + "; ".join(f"worst |dO| {name} = {v:.3e}" for name, v in worst.items()))
    for name, v in worst.items():
        assert v <= ATOL_OUT[dtype], name
    return kept


def test_layer_cfg1_full():
    say("layer cfg1 (fp32, n=576)")
    w = make_workload(1)
    _layer_parity(w, w.tau)


def test_layer_with_hybrid_probe_set():
    say("layer with 64 recent + 64 random probes (bf16, GQA 6/2, n=2000)")
    n = 2000
    w = make_custom(1, 6, 2, n, 128, "bf16", seed=21, probe_pos=hybrid_probes(n, seed=5))
    assert len(w.probe_pos) == 128
    _layer_parity(w, 0.975)


# ------------------------------------------------------------------ all-rows (exact) scores
@pytest.mark.parametrize("case", [dict(B=1, Hq=4, Hkv=2, n=333, d=128, dtype="bf16"),
                                  dict(B=2, Hq=2, Hkv=2, n=200, d=64, dtype="f32"),
                                  dict(B=1, Hq=14, Hkv=2, n=700, d=128, dtype="bf16"),
                                  dict(B=1, Hq=2, Hkv=1, n=129, d=128, dtype="f32"),
                                  dict(B=1, Hq=2, Hkv=2, n=64, d=64, dtype="bf16"),
                                  dict(B=1, Hq=1, Hkv=1, n=1, d=128, dtype="bf16")])
def test_all_rows_scores_match_the_oracle(case):
    B, Hq, Hkv, n, d, dtype = (case[key] for key in ("B", "Hq", "Hkv", "n", "d", "dtype"))
    say(f"score_all_rows B={B} Hq={Hq} Hkv={Hkv} n={n} d={d} {dtype}")
    w = make_custom(B, Hq, Hkv, n, d, dtype, seed=71, m=min(64, n))
    Q, K = dev(w.Q, dtype), dev(w.K, dtype)
    mass, rank = z.zipvl_score_all_rows(Q, K, w.scale)
    mass_only, none = z.zipvl_score_all_rows(Q, K, w.scale, want_rank=False)
    torch.cuda.synchronize()
    assert none is None and torch.equal(mass, mass_only)
    mass_h, rank_h = mass.cpu().numpy().astype(np.float64), rank.cpu().numpy().astype(np.float64)
    for b in range(B):
        mo, ro = oz.token_scores(w.Q[b], w.K[b], np.arange(n), w.scale)       # every row is a probe
        assert_scores_close(mass_h.reshape(B, Hkv, n)[b], mo, dtype, "mass")
        assert_scores_close(rank_h.reshape(B, Hkv, n)[b], ro, dtype, "rank")
    assert np.all(np.abs(mass_h.sum(axis=1) - 1.0) < 1e-4)


def test_all_rows_scores_at_cfg2_shape_against_sampled_columns():
    say("score_all_rows at n=3072, 32 heads (sampled heads)")
    w = make_workload(2)
    spec = w.spec
    Q, K = dev(w.Q, spec.dtype), dev(w.K, spec.dtype)
    mass, rank = z.zipvl_score_all_rows(Q, K, w.scale)
    torch.cuda.synchronize()
    n = spec.n
    for u in (0, 13, 31):
        mo, ro = oz.token_scores(w.Q[0, u:u + 1], w.K[0, u:u + 1], np.arange(n), w.scale)
        assert_scores_close(mass[u].cpu().numpy().astype(np.float64)[None], mo, spec.dtype, "mass")
        assert_scores_close(rank[u].cpu().numpy().astype(np.float64)[None], ro, spec.dtype, "rank")


# ------------------------------------------------------------------ one T per layer
def test_share_scores_bit_exact():
    say("share_scores")
    r = np.random.Generator(np.random.PCG64(41))
    for B, Hkv, n in ((1, 4, 18432), (3, 7, 1001), (2, 1, 77)):
        mass = r.random((B * Hkv, n)).astype(np.float32)
        mass /= mass.sum(axis=1, keepdims=True)
        rank = (mass * r.random((B * Hkv, n))).astype(np.float32)
        mb, rb = z.zipvl_share_scores(torch.from_numpy(mass).to(DEV), torch.from_numpy(rank).to(DEV), B)
        mb2, none = z.zipvl_share_scores(torch.from_numpy(mass).to(DEV), None, B)
        torch.cuda.synchronize()
        assert none is None
        for b in range(B):
            ref_m = oz.share_scores(mass[b * Hkv:(b + 1) * Hkv])
            assert mb[b].cpu().numpy().tobytes() == ref_m.tobytes()
            assert mb2[b].cpu().numpy().tobytes() == ref_m.tobytes()
            assert rb[b].cpu().numpy().tobytes() == oz.share_scores(rank[b * Hkv:(b + 1) * Hkv]).tobytes()


@pytest.mark.parametrize("case", [dict(B=2, Hq=8, Hkv=4, n=700, d=128, dtype="bf16", seed=51, full=True),
                                  dict(B=1, Hq=4, Hkv=4, n=333, d=64, dtype="f32", seed=52, full=True),
                                  dict(B=1, Hq=28, Hkv=4, n=4608, d=128, dtype="bf16", seed=53, full=False)])
def test_layer_with_one_important_set_per_batch_element(case):
    B, Hq, Hkv, n, d, dtype = (case[key] for key in ("B", "Hq", "Hkv", "n", "d", "dtype"))
    say(f"layer, one T per batch element: B={B} Hq={Hq} Hkv={Hkv} n={n} d={d} {dtype}")
    G, tau = Hq // Hkv, 0.975
    w = make_custom(B, Hq, Hkv, n, d, dtype, seed=case["seed"])
    Q, K, V = dev(w.Q, dtype), dev(w.K, dtype), dev(w.V, dtype)
    mass, rank = z.zipvl_score(Q, K, w.probe_pos, w.scale)
    mass_b, rank_b = z.zipvl_share_scores(mass, rank, B)
    idx, k = z.zipvl_select(mass_b, rank_b, tau)
    assert idx.shape == (B, n) and k.shape == (B,)
    Kc, Vc, ln = z.zipvl_compact_kv(K, V, idx, k, n, z.T_PER_BATCH)
    O = z.zipvl_sparse_prefill(Q, K, V, idx, k, w.scale, z.T_PER_BATCH)
    # the same attention from the evicted cache, compact output rows (every case: in-place K read and repack)
    Oc = z.zipvl_sparse_prefill(Q, Kc.view(B, Hkv, n, d), Vc.view(B, Hkv, n, d), idx, k, w.scale,
                                z.T_PER_BATCH | z.KV_ALREADY_COMPACT | z.OUT_COMPACT)
    torch.cuda.synchronize()
    mass_h, rank_h = mass.cpu().numpy(), rank.cpu().numpy()
    idx_h, k_h, ln_h = idx.cpu().numpy(), k.cpu().numpy(), ln.cpu().numpy()
    r = np.random.Generator(np.random.PCG64(78))
    worst = 0.0
    for b in range(B):
        # oracle fed the GPU's per-unit fp32 scores: same mean, same selection, exactly
        p, T = oz.select(oz.share_scores(mass_h[b * Hkv:(b + 1) * Hkv]), oz.share_scores(rank_h[b * Hkv:(b + 1) * Hkv]), tau)
        assert k_h[b] == p and np.array_equal(idx_h[b, :p], T), f"batch element {b}: selection differs"
        dropped = np.setdiff1d(np.arange(n), T)
        for g in range(Hkv):
            u = b * Hkv + g
            assert ln_h[u] == p
            ko, vo, _ = oz.compact_kv(w.K[b, g], w.V[b, g], T)
            assert Kc[u, :p].to(torch.float32).cpu().numpy().tobytes() == ko.tobytes()
            assert Vc[u, :p].to(torch.float32).cpu().numpy().tobytes() == vo.tobytes()
        for h in range(Hq):
            g = h // G
            Oh = host64(O[b, h])
            assert not Oh[dropped].any(), "dropped rows must be zero"
            if case["full"]:
                ref = oz.kept_token_attention(w.Q[b, h], w.K[b, g], w.V[b, g], T, w.scale)
                worst = max(worst, np.abs(Oh - ref).max())
                if Oc is not None:
                    worst = max(worst, np.abs(host64(Oc[b, h])[:p] - ref[T]).max())
            else:
                rows = np.unique(np.concatenate([[0, p - 1, min(127, p - 1), min(128, p - 1)], r.integers(0, p, 6)]))
                ref = oz.kept_token_attention_rows(w.Q[b, h], w.K[b, g], w.V[b, g], T, rows, w.scale)
                worst = max(worst, np.abs(Oh[T[rows]] - ref).max())
                worst = max(worst, np.abs(host64(Oc[b, h])[rows] - ref).max())
    say(f"  kept {[int(x) for x in k_h]} of {n}; worst |dO| = {worst:.3e}")
    assert worst <= ATOL_OUT[dtype]


# ------------------------------------------------------------------ mixed-precision cache
def _unpack(codes: np.ndarray, bits: int) -> np.ndarray:
    """[rows, d*bits/8] bytes -> [rows, d] codes (element c in bits [c*bits, c*bits+bits) of the row's bit string)."""
    per = 8 // bits
    out = np.empty((codes.shape[0], codes.shape[1] * per), dtype=np.uint8)
    for e in range(per):
        out[:, e::per] = (codes >> (bits * e)) & ((1 << bits) - 1)
    return out


def _check_qcache_against_oracle(cache, w, dtype, Ts, Hkv):
    """Codes and fp16 parameters of every unit, bit for bit; returns the oracle caches."""
    ref = []
    for u, T in enumerate(Ts):
        b, g = divmod(u, Hkv)
        qc = oz.quantize_kv(w.K[b, g], w.V[b, g], T)
        ref.append(qc)
        nh, nl = len(T), w.K.shape[2] - len(T)
        assert int(cache.len_hi[u]) == nh and int(cache.len_lo[u]) == nl
        for name, t in (("K", cache.K), ("V", cache.V)):
            for grp, bits, rows in (("hi", 4, nh), ("lo", 2, nl)):
                codes, scale, zero = qc[f"{name}_{grp}"]
                got = _unpack(t[f"{grp}_codes"][u, :rows].cpu().numpy(), bits)
                par = t[f"{grp}_params"][u, :rows].cpu().numpy()
                assert par[:, 0].tobytes() == scale.tobytes(), f"unit {u} {name} {grp}: scales differ"
                assert par[:, 1].tobytes() == zero.tobytes(), f"unit {u} {name} {grp}: zeros differ"
                bad = np.argwhere(got != codes)
                assert len(bad) == 0, f"unit {u} {name} {grp}: {len(bad)} codes differ, first at {bad[0]}"
    return ref


@pytest.mark.parametrize("dtype,d", [("bf16", 128), ("f32", 128), ("bf16", 64), ("f32", 64)])
def test_quantize_kv_bit_exact_and_decode_over_it(dtype, d):
    say(f"quantize_kv + decode_attn_q dtype={dtype} d={d}")
    B, Hq, Hkv, n = 2, 6, 3, 333
    G = Hq // Hkv
    w = make_custom(B, Hq, Hkv, n, d, dtype, seed=61)
    K, V = dev(w.K, dtype), dev(w.V, dtype)
    r = np.random.Generator(np.random.PCG64(62))
    ks = [1, 64, 333, 200, 17, 130]                           # k = n: the 2-bit group is empty
    idx = np.zeros((B * Hkv, n), dtype=np.int32)
    for u in range(B * Hkv):
        idx[u, :ks[u]] = np.sort(r.choice(n, ks[u], replace=False))
    idx_d, k_d = torch.from_numpy(idx).to(DEV), torch.tensor(ks, dtype=torch.int32, device=DEV)
    cache = z.zipvl_quantize_kv(K, V, idx_d, k_d, n, n)
    torch.cuda.synchronize()
    ref = _check_qcache_against_oracle(cache, w, dtype, [idx[u, :ks[u]] for u in range(B * Hkv)], Hkv)

    # decode: one query per head over [4-bit rows | 2-bit rows | 3 appended rows]
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    qh = r.standard_normal((B * Hq, d)).astype(np.float32)
    tail_k = r.standard_normal((3, B * Hkv, d)).astype(np.float32)
    tail_v = r.standard_normal((3, B * Hkv, d)).astype(np.float32)
    q = dev(qh, dtype)
    Kt = torch.zeros((B * Hkv, 8, d), dtype=tdt, device=DEV); Vt = torch.zeros_like(Kt)
    lt = torch.zeros((B * Hkv,), dtype=torch.int32, device=DEV)
    o0 = z.zipvl_decode_attn_q(q, cache, w.scale, B=B, Hq=Hq, Hkv=Hkv).float().cpu().numpy().astype(np.float64)
    for step in range(3):
        z.zipvl_kv_append(Kt, Vt, lt, dev(tail_k[step], dtype), dev(tail_v[step], dtype), B=B, Hkv=Hkv)
    o3 = z.zipvl_decode_attn_q(q, cache, w.scale, B=B, Hq=Hq, Hkv=Hkv, K_tail=Kt, V_tail=Vt, len_tail=lt)
    torch.cuda.synchronize()
    o3 = o3.float().cpu().numpy().astype(np.float64)
    q64 = host64(q)
    tk = host64(Kt)[:, :3]; tv = host64(Vt)[:, :3]
    worst = 0.0
    for bh in range(B * Hq):
        b, h = divmod(bh, Hq)
        u = b * Hkv + h // G
        worst = max(worst, np.abs(o0[bh] - oz.decode_attention_quantized(q64[bh], ref[u], w.scale)).max())
        worst = max(worst, np.abs(o3[bh] - oz.decode_attention_quantized(q64[bh], ref[u], w.scale, tk[u], tv[u])).max())
    say(f"  worst |do| = {worst:.3e}")
    assert worst <= ATOL_OUT[dtype]


@pytest.mark.parametrize("Hq,Hkv", [(4, 4), (8, 2), (14, 2)])
def test_decode_over_quantised_cache_for_every_group_size(Hq, Hkv):
    say(f"decode_attn_q Hq={Hq} Hkv={Hkv}")
    B, n, d, dtype = 1, 700, 128, "bf16"
    G = Hq // Hkv
    w = make_custom(B, Hq, Hkv, n, d, dtype, seed=65)
    K, V = dev(w.K, dtype), dev(w.V, dtype)
    r = np.random.Generator(np.random.PCG64(66))
    ks = [r.integers(1, n) for _ in range(Hkv)]
    idx = np.zeros((Hkv, n), dtype=np.int32)
    for u in range(Hkv):
        idx[u, :ks[u]] = np.sort(r.choice(n, ks[u], replace=False))
    cache = z.zipvl_quantize_kv(K, V, torch.from_numpy(idx).to(DEV), torch.tensor(ks, dtype=torch.int32, device=DEV), n, n)
    q = dev(r.standard_normal((Hq, d)).astype(np.float32), dtype)
    o = z.zipvl_decode_attn_q(q, cache, w.scale, B=B, Hq=Hq, Hkv=Hkv)
    torch.cuda.synchronize()
    worst = 0.0
    for h in range(Hq):
        u = h // G
        qc = oz.quantize_kv(w.K[0, u], w.V[0, u], idx[u, :ks[u]])
        worst = max(worst, np.abs(host64(o[h]) - oz.decode_attention_quantized(host64(q[h]), qc, w.scale)).max())
    say(f"  worst |do| = {worst:.3e}")
    assert worst <= 2e-2


def test_quantize_kv_with_one_set_per_batch_element_and_without_T():
    say("quantize_kv T_PER_BATCH / idx=NULL")
    B, Hq, Hkv, n, d, dtype = 2, 4, 4, 1000, 128, "bf16"
    w = make_custom(B, Hq, Hkv, n, d, dtype, seed=63)
    K, V = dev(w.K, dtype), dev(w.V, dtype)
    r = np.random.Generator(np.random.PCG64(64))
    ks = [411, 77]
    idx = np.zeros((B, n), dtype=np.int32)
    for b in range(B):
        idx[b, :ks[b]] = np.sort(r.choice(n, ks[b], replace=False))
    cache = z.zipvl_quantize_kv(K, V, torch.from_numpy(idx).to(DEV), torch.tensor(ks, dtype=torch.int32, device=DEV),
                                n, n, z.T_PER_BATCH)
    torch.cuda.synchronize()
    _check_qcache_against_oracle(cache, w, dtype, [idx[u // Hkv, :ks[u // Hkv]] for u in range(B * Hkv)], Hkv)
    allhi = z.zipvl_quantize_kv(K, V, None, None, n, 8)       # every token important
    torch.cuda.synchronize()
    _check_qcache_against_oracle(allhi, w, dtype, [np.arange(n)] * (B * Hkv), Hkv)


def test_quantised_cache_at_stack_shape_sampled_units():
    say("quantize_kv + decode_attn_q at B4 H32 n8192 (sampled units)")
    from workloads import make_stack_layer_device
    Q, K, V, probe, scale = make_stack_layer_device(7, DEV)
    B, H, n, d = K.shape
    mass, rank = z.zipvl_score(Q, K, probe, scale)
    idx, k = z.zipvl_select(mass, rank, 0.975)
    cache = z.zipvl_quantize_kv(K, V, idx, k, n, n)
    g = torch.Generator(device=DEV); g.manual_seed(5)
    q = torch.randn((B * H, d), generator=g, device=DEV).to(torch.bfloat16)
    o = z.zipvl_decode_attn_q(q, cache, scale, B=B, Hq=H, Hkv=H)
    torch.cuda.synchronize()
    k_h, idx_h = k.cpu().numpy(), idx.cpu().numpy()
    assert cache.len_hi.cpu().tolist() == k_h.tolist() and cache.len_lo.cpu().tolist() == (n - k_h).tolist()
    worst = 0.0
    for u in (0, 37, 127):
        b, h = divmod(u, H)
        Kh, Vh = K[b, h].float().cpu().numpy(), V[b, h].float().cpu().numpy()
        qc = oz.quantize_kv(Kh, Vh, idx_h[u, :k_h[u]])
        for name, t in (("K", cache.K), ("V", cache.V)):
            assert np.array_equal(_unpack(t["hi_codes"][u, :k_h[u]].cpu().numpy(), 4), qc[name + "_hi"][0])
            assert np.array_equal(_unpack(t["lo_codes"][u, :n - k_h[u]].cpu().numpy(), 2), qc[name + "_lo"][0])
        refo = oz.decode_attention_quantized(host64(q[u]), qc, scale)
        worst = max(worst, np.abs(host64(o[u]) - refo).max())
    bits = 8.0 * cache.nbytes() / (2.0 * B * H * n * d)
    say(f"  kept {100 * k_h.mean() / n:.1f}% at 4 bits; {bits:.2f} bits per element incl. parameters "
        f"(compression {16 / bits:.2f}x at full capacity arrays); worst |do| = {worst:.3e}")
    assert worst <= 2e-2


def test_layer_tau_one_is_dense_attention():
    say("layer tau=1")
    w = make_custom(1, 4, 2, 320, 128, "bf16", seed=12)
    Q, K, V = dev(w.Q, "bf16"), dev(w.K, "bf16"), dev(w.V, "bf16")
    mass, rank = z.zipvl_score(Q, K, w.probe_pos, w.scale)
    idx, k = z.zipvl_select(mass, rank, 1.0)
    O = z.zipvl_sparse_prefill(Q, K, V, idx, k, w.scale)
    torch.cuda.synchronize()
    assert k.cpu().tolist() == [320, 320]
    for h in range(4):
        ref = oz.dense_causal_attention(w.Q[0, h], w.K[0, h // 2], w.V[0, h // 2], w.scale)
        assert np.abs(host64(O[0, h]) - ref).max() <= 2e-2


def test_layer_cfg2_sampled():
    say("layer cfg2 (bf16, 32 heads, n=3072), sampled output rows")
    w = make_workload(2)
    _layer_parity(w, w.tau, sample_rows=8, heads=range(32), whole_heads=[0, 13, 31])


def test_layer_cfg3_three_taus_selection_and_sampled_rows():
    say("layer cfg3 (bf16, 40 heads, n=4096)")
    w = make_workload(3)
    ks = []
    for tau in w.spec.taus:
        kept = _layer_parity(w, tau, sample_rows=4, heads=range(0, 40, 3), whole_heads=[7] if tau == w.tau else [])
        ks.append(np.mean(kept))
    assert ks[0] <= ks[1] <= ks[2]


def test_layer_cfg4_headline_shape_sampled():
    say("layer cfg4 (bf16 GQA 28/4, n=18432): one whole query head per KV group, tile-edge rows of all 28 heads")
    w = make_workload(4)
    _layer_parity(w, w.tau, sample_rows=6, heads=range(28), whole_heads=[0, 9, 18, 27])


def test_layer_beyond_the_benchmark_lengths_sampled():
    say("layer at n=40960 (bf16 GQA 2/1): selection keys no longer fit LDS, 320 query tiles per head")
    w = make_custom(1, 2, 1, 40960, 128, "bf16", seed=81, spike_frac=0.05)
    _layer_parity(w, 0.975, sample_rows=10)


def test_layer_cfg5_first_and_last_layer_then_decode_on_evicted_cache():
    say("layer cfg5 (bf16, 32 heads, n=8192), layers 0, 10, 21 and 31 of the ramp, batch slice of 1; then decode on the evicted cache")
    fracs = []
    for layer in (0, 10, 21, 31):
        w = make_workload(5, layer=layer, batch=1)
        kept = _layer_parity(w, w.tau, sample_rows=4, heads=[3, 17, 30], whole_heads=[30] if layer == 31 else [])
        fracs.append(np.mean(kept))
    assert max(fracs) - min(fracs) > 0.05          # the spike ramp makes the kept ratio layer dependent
    # decode: two steps against the evicted cache of the last layer
    spec = w.spec
    Q, K, V = dev(w.Q, "bf16"), dev(w.K, "bf16"), dev(w.V, "bf16")
    mass, rank = z.zipvl_score(Q, K, w.probe_pos, w.scale)
    idx, k = z.zipvl_select(mass, rank, w.tau)
    cap = int(k.max().item()) + 4
    Kc, Vc, ln = z.zipvl_compact_kv(K, V, idx, k, cap)
    r = np.random.Generator(np.random.PCG64(5))
    from workloads import round_to_bf16
    H, d = spec.Hq, spec.d
    idx_h, k_h = idx.cpu().numpy(), k.cpu().numpy()
    Kh = [w.K[0, g][idx_h[g, :k_h[g]]] for g in range(H)]
    Vh = [w.V[0, g][idx_h[g, :k_h[g]]] for g in range(H)]
    for step in range(2):
        q = round_to_bf16(r.standard_normal((H, d)).astype(np.float32))
        kn = round_to_bf16(r.standard_normal((H, d)).astype(np.float32))
        vn = round_to_bf16(r.standard_normal((H, d)).astype(np.float32))
        z.zipvl_kv_append(Kc, Vc, ln, dev(kn, "bf16"), dev(vn, "bf16"), B=1, Hkv=H)
        o = z.zipvl_decode_attn(dev(q, "bf16"), Kc, Vc, ln, w.scale, B=1, Hq=H, Hkv=H)
        torch.cuda.synchronize()
        oh = host64(o)
        for g in (0, 17, 31):
            ref, Kh[g], Vh[g], _ = oz.decode_step(q[g], kn[g], vn[g], Kh[g], Vh[g], len(Kh[g]), w.scale)
            assert np.abs(oh[g] - ref).max() <= 2e-2
        for g in range(H):
            if g not in (0, 17, 31):
                Kh[g] = np.concatenate([Kh[g], kn[g][None]]); Vh[g] = np.concatenate([Vh[g], vn[g][None]])
    assert ln.cpu().tolist() == [int(x) + 2 for x in k_h]


# ------------------------------------------------------------------ decode
@pytest.mark.parametrize("dtype,d,Hq,Hkv", [("bf16", 128, 4, 4), ("bf16", 128, 14, 2), ("f32", 64, 4, 2), ("bf16", 64, 3, 1)])
def test_decode_append_and_attention(dtype, d, Hq, Hkv):
    say(f"decode dtype={dtype} d={d} Hq={Hq} Hkv={Hkv}")
    B, cap = 2, 1300
    G = Hq // Hkv
    units = B * Hkv
    w = make_custom(B, Hq, Hkv, cap, d, dtype, seed=31)
    Kc = dev(w.K, dtype).reshape(units, cap, d).clone()
    Vc = dev(w.V, dtype).reshape(units, cap, d).clone()
    lens = [1, 1299, 640, 17][:units] + [5] * max(0, units - 4)
    ln = torch.tensor(lens, dtype=torch.int32, device=DEV)
    r = np.random.Generator(np.random.PCG64(32))
    from workloads import round_to_bf16
    cast = round_to_bf16 if dtype == "bf16" else (lambda a: a.astype(np.float32))
    q = cast(r.standard_normal((B * Hq, d)).astype(np.float32) * 2)
    kn = cast(r.standard_normal((units, d)).astype(np.float32))
    vn = cast(r.standard_normal((units, d)).astype(np.float32))
    z.zipvl_kv_append(Kc, Vc, ln, dev(kn, dtype), dev(vn, dtype), B=B, Hkv=Hkv)
    o = z.zipvl_decode_attn(dev(q, dtype), Kc, Vc, ln, w.scale, B=B, Hq=Hq, Hkv=Hkv)
    torch.cuda.synchronize()
    assert ln.cpu().tolist() == [x + 1 for x in lens]
    oh = host64(o)
    Kh, Vh = w.K.reshape(units, cap, d), w.V.reshape(units, cap, d)
    worst = 0.0
    for b in range(B):
        for h in range(Hq):
            u = b * Hkv + h // G
            ref, Ko, Vo, L1 = oz.decode_step(q[b * Hq + h], kn[u], vn[u], Kh[u], Vh[u], lens[u], w.scale)
            worst = max(worst, np.abs(oh[b * Hq + h] - ref).max())
            assert Kc[u, lens[u]].to(torch.float32).cpu().numpy().tobytes() == kn[u].tobytes()
    say(f"  worst |do| = {worst:.3e}")
    assert worst <= ATOL_OUT[dtype]


@pytest.mark.parametrize("dtype,d,Hq,Hkv", [("bf16", 128, 4, 4), ("bf16", 128, 14, 2), ("f32", 64, 4, 2), ("bf16", 64, 3, 1),
                                            ("f32", 128, 8, 1), ("bf16", 128, 18, 2)])
def test_decode_step_one_launch_matches_append_then_attention(dtype, d, Hq, Hkv):
    """Three consecutive fused steps (the arrival counters must clear themselves) against the oracle's
    append-then-attend, with an empty unit, a long one and one that is full from the second step on."""
    say(f"decode_step dtype={dtype} d={d} Hq={Hq} Hkv={Hkv}")
    B, cap = 2, 1300
    G = Hq // Hkv
    units = B * Hkv
    w = make_custom(B, Hq, Hkv, cap, d, dtype, seed=33)
    Kc = dev(w.K, dtype).reshape(units, cap, d).clone()
    Vc = dev(w.V, dtype).reshape(units, cap, d).clone()
    lens = [0, 1299, 640, 17][:units] + [5] * max(0, units - 4)
    ln = torch.tensor(lens, dtype=torch.int32, device=DEV)
    r = np.random.Generator(np.random.PCG64(34))
    from workloads import round_to_bf16
    cast = round_to_bf16 if dtype == "bf16" else (lambda a: a.astype(np.float32))
    Kh = [w.K.reshape(units, cap, d)[u].copy() for u in range(units)]
    Vh = [w.V.reshape(units, cap, d)[u].copy() for u in range(units)]
    ws = z.decode_step_workspace(B, Hq, Hkv, cap, d, Kc)
    worst = 0.0
    for step in range(3):
        q = cast(r.standard_normal((B * Hq, d)).astype(np.float32) * 2)
        kn = cast(r.standard_normal((units, d)).astype(np.float32))
        vn = cast(r.standard_normal((units, d)).astype(np.float32))
        o = z.zipvl_decode_step(dev(q, dtype), Kc, Vc, ln, dev(kn, dtype), dev(vn, dtype), w.scale, B=B, Hq=Hq, Hkv=Hkv, ws=ws)
        torch.cuda.synchronize()
        oh = host64(o)
        new_lens = list(lens)
        for u in range(units):
            if lens[u] < cap:
                Kh[u][lens[u]] = kn[u]; Vh[u][lens[u]] = vn[u]
                new_lens[u] = lens[u] + 1
        for b in range(B):
            for h in range(Hq):
                u = b * Hkv + h // G
                ref = oz.decode_attention(q[b * Hq + h], Kh[u], Vh[u], new_lens[u], w.scale)
                worst = max(worst, np.abs(oh[b * Hq + h] - ref).max())
        lens = new_lens
        assert ln.cpu().tolist() == lens
        for u in range(units):                                # the caches hold exactly the oracle's rows
            assert Kc[u, :lens[u]].to(torch.float32).cpu().numpy().tobytes() == Kh[u][:lens[u]].astype(np.float32).tobytes()
            assert Vc[u, :lens[u]].to(torch.float32).cpu().numpy().tobytes() == Vh[u][:lens[u]].astype(np.float32).tobytes()
    assert int(ws[:4 * units].view(torch.int32).abs().sum().item()) == 0      # counters left at zero
    say(f"  worst |do| = {worst:.3e}")
    assert worst <= ATOL_OUT[dtype]


def test_decode_256_fused_steps_bit_identical_to_append_then_attention_at_the_stack_shape():
    """zipvl_decode_step against zipvl_kv_append + zipvl_decode_attn over 256 consecutive steps at the 32-head,
    batch-4 stack shape: outputs, lengths and caches must agree bit for bit at every step (the fused kernel
    takes the new row in its place in the row order, so the arithmetic is the same).  Lengths are ragged,
    cross split boundaries on the way, one unit starts empty and one fills up and must stay unchanged."""
    say("decode_step x256 vs kv_append + decode_attn, B4 H32 d128")
    B, H, d, cap, steps = 4, 32, 128, 2816, 256
    units = B * H
    g = torch.Generator(device=DEV); g.manual_seed(77)
    Ka = torch.randn((units, cap, d), generator=g, device=DEV).to(torch.bfloat16)
    Va = torch.randn((units, cap, d), generator=g, device=DEV).to(torch.bfloat16)
    r = np.random.Generator(np.random.PCG64(78))
    lens = r.integers(1500, 2500, units).astype(np.int32)
    lens[0], lens[1], lens[2], lens[3] = 0, cap - 100, 255, 2559       # empty; fills up after 100 steps; next to split edges
    la = torch.from_numpy(lens).to(DEV)
    Kb, Vb, lb = Ka.clone(), Va.clone(), la.clone()
    ws = z.decode_step_workspace(B, H, H, cap, d, Ka)
    scale = 1.0 / math.sqrt(d)
    oa = torch.empty((units, d), dtype=torch.bfloat16, device=DEV)
    ob = torch.empty_like(oa)
    for step in range(steps):
        q = torch.randn((units, d), generator=g, device=DEV).to(torch.bfloat16)
        kn = torch.randn((units, d), generator=g, device=DEV).to(torch.bfloat16)
        vn = torch.randn((units, d), generator=g, device=DEV).to(torch.bfloat16)
        z.zipvl_decode_step(q, Ka, Va, la, kn, vn, scale, B=B, Hq=H, Hkv=H, ws=ws, o=oa)
        z.zipvl_kv_append(Kb, Vb, lb, kn, vn, B=B, Hkv=H)
        z.zipvl_decode_attn(q, Kb, Vb, lb, scale, B=B, Hq=H, Hkv=H, o=ob)
        torch.cuda.synchronize()
        if not torch.equal(oa, ob):
            bad = (oa != ob).any(dim=1).nonzero().flatten().tolist()
            raise AssertionError(f"step {step}: outputs differ in units {bad[:8]} (lengths {la[bad[:8]].tolist()})")
        assert torch.equal(la, lb), f"step {step}: lengths differ"
    expect = np.minimum(lens.astype(np.int64) + steps, cap)
    assert la.cpu().numpy().tolist() == expect.tolist()
    assert torch.equal(Ka, Kb) and torch.equal(Va, Vb), "caches differ after 256 steps"
    assert int(ws[:4 * units].view(torch.int32).abs().sum().item()) == 0          # counters left at zero
    # and the last step meets the oracle (Eq. (5)) on a few units, the full one included
    oh = host64(oa)
    for u in (0, 1, 2, 3, 77):
        ref = oz.decode_attention(host64(q[u]), host64(Ka[u]), host64(Va[u]), int(expect[u]), scale)
        assert np.abs(oh[u] - ref).max() <= 2e-2
