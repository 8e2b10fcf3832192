"""CPU float64 oracle for the ZipVL prefill path (arXiv 2410.08584).

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain statement of what the
GPU library must compute.  It shares no code with the HIP path and must never
be imported by the product package: only the tests, the smoke check and the
benchmark's CPU-baseline leg may call it.

Everything is numpy float64, one step of the paper at a time, no blocking and
no fusion (dense attention is split over query rows only to bound memory; every
row is still the plain softmax definition).

Readings taken where the paper is silent (each is listed with its reason in
the design notes of the repository):
  * probe rows are causally masked like every other row of Eq. (2);
  * "nnz" of Eq. (8) is the structural count of unmasked entries of a column;
  * the threshold of Eq. (7) is tau times the total of the vector that is
    summed (equal to tau*n for the full matrix, tau*m for m probe rows);
  * the cumulative sum of Eq. (7) is taken over floor(a_j * 2^40) in integers,
    so that its value does not depend on summation order;
  * ties are broken towards the lower token index; T is reported ascending;
  * one selection per (batch, KV head); with grouped-query attention the
    scores of the query heads of a group are averaged;
  * outputs of dropped tokens are zero rows.

Pins (tests/test_oracle_pins.py): row-softmax mass conservation, harmonic-number
closed form for Q=0, one-hot scores, all-rows probes against a dense softmax
taken with another library, brute-force subset enumeration for the selection,
tie/permutation invariance, tau=1, monotonicity in tau, uniform closed form,
masked-dense equivalence and running-mean closed form for the kept-token
attention (whole product and row-at-a-time form alike), head-averaged scores against the float64 mean and the single-head
case, the row quantiser against the nearest-grid-point definition, its
half-step error bound and Table 3's compression ratios, torch SDPA for dense attention, Table 2/3 ratio accounting.
Parity unpinned (our own readings, checked only for self-consistency): the
per-KV-head granularity and group averaging, the zero padding value, the 2^40
grid, the synthetic kept ratios, and the parameter granularity assumed by
kv_quant_compression (a group size fitted to Table 3's two ratios, not a value
the paper states).
Two functions, share_scores and quantize_rows, decide integers (a selection, a
code) from floating point; both take those steps in fp32, the precision the
GPU kernels use, so that the two sides decide alike.  That precision is a
choice made here, not something the paper fixes; the quantiser is pinned
against the float64 nearest-grid-point definition regardless.
"""
from __future__ import annotations

import math
from typing import Optional, Tuple

import numpy as np

FIXED_POINT_BITS = 40


# --------------------------------------------------------------------------
# Step 1: probe attention scores  (supplementary Eq. (A); Algorithm 1, step 2)
# --------------------------------------------------------------------------
def probe_attention(Qh: np.ndarray, Kg: np.ndarray, probe_pos: np.ndarray, scale: float) -> np.ndarray:
    """A' = row-softmax(Q[probe] K^T * scale) with the causal mask of Eq. (2):
    probe row c (token position P_c) sees keys j <= P_c.  Returns [m, n]."""
    Qh = np.asarray(Qh, dtype=np.float64)
    Kg = np.asarray(Kg, dtype=np.float64)
    P = np.asarray(probe_pos, dtype=np.int64)
    n = Kg.shape[0]
    S = (Qh[P] @ Kg.T) * float(scale)
    S = np.where(np.arange(n)[None, :] <= P[:, None], S, -np.inf)
    S = S - S.max(axis=1, keepdims=True)
    E = np.exp(S)
    return E / E.sum(axis=1, keepdims=True)


def structural_count(n: int, probe_pos: np.ndarray) -> np.ndarray:
    """nnz of column j of the masked probe matrix (Eq. (8)): the number of
    probe rows whose position is >= j."""
    P = np.asarray(probe_pos, dtype=np.int64)
    return (P[:, None] >= np.arange(n)[None, :]).sum(axis=0)


def token_scores(Q: np.ndarray, K: np.ndarray, probe_pos: np.ndarray, scale: float
                 ) -> Tuple[np.ndarray, np.ndarray]:
    """Accumulated (Eq. (6)) and normalised (Eq. (8)) score per token from the
    probe rows, for one batch element.

    Q [Hq, n, d], K [Hkv, n, d] -> mass, rank [Hkv, n] float64 where
      a_j    = sum_c A'[c, j]
      mass_j = a_j / m                 (sums to 1 over j for each head)
      rank_j = a_j / nnz_j             (0 where nnz_j = 0)
    averaged over the query heads that share the KV head.
    """
    Hq, n, _ = Q.shape
    Hkv = K.shape[0]
    G = Hq // Hkv
    m = len(probe_pos)
    cnt = structural_count(n, probe_pos).astype(np.float64)
    mass = np.zeros((Hkv, n))
    rank = np.zeros((Hkv, n))
    for g in range(Hkv):
        for h in range(g * G, (g + 1) * G):
            a = probe_attention(Q[h], K[g], probe_pos, scale).sum(axis=0)
            mass[g] += a / m
            rank[g] += np.divide(a, cnt, out=np.zeros(n), where=cnt > 0)
        mass[g] /= G
        rank[g] /= G
    return mass, rank


# --------------------------------------------------------------------------
# Step 2: how many tokens, and which  (Eq. (7), Eq. (9), Eq. (10))
# --------------------------------------------------------------------------
def fixed_point(mass32: np.ndarray) -> np.ndarray:
    """floor(float64(x) * 2^40) as int64, exact for fp32 x in [0, 2^12)."""
    x = np.asarray(mass32, dtype=np.float32).astype(np.float64)
    return np.floor(x * float(2 ** FIXED_POINT_BITS)).astype(np.int64)


def descending_order(x32: np.ndarray) -> np.ndarray:
    """Indices sorted by value descending, equal values by index ascending."""
    x = np.asarray(x32, dtype=np.float32)
    return np.argsort(-x, kind="stable")


def count_important(mass32: np.ndarray, tau: float) -> int:
    """Eq. (7): the smallest p whose top-p accumulated scores reach tau of the
    total; tau >= 1 keeps everything; never less than one token."""
    n = len(mass32)
    if tau >= 1.0:
        return n
    q = fixed_point(mass32)
    C = np.cumsum(q[descending_order(mass32)])
    target = math.ceil(float(tau) * float(int(C[-1])))
    p = int(np.searchsorted(C, target, side="left")) + 1   # first i (1-based) with C_i >= target
    return max(1, min(p, n))


def select(mass32: np.ndarray, rank32: Optional[np.ndarray], tau: float) -> Tuple[int, np.ndarray]:
    """Count by `mass` (Eq. (7)), identify by `rank` (Eq. (9)); `rank32=None`
    uses `mass` for both.  Returns (p, T ascending by position)."""
    p = count_important(mass32, tau)
    r = mass32 if rank32 is None else rank32
    T = np.sort(descending_order(r)[:p])
    return p, T.astype(np.int32)


def share_scores(x32: np.ndarray) -> np.ndarray:
    """One important set for every head of a layer: Algorithm 1 as written
    selects a single T and hands Q[T], K[T], V[T] to one attention call, so
    under that reading the per-head score vectors [U, n] of a batch element
    are averaged into one [n].  The selection that follows is decided by
    these bits, so the precision is fixed: fp32, heads added in ascending
    order, then one multiplication by fp32(1/U)."""
    x32 = np.asarray(x32, dtype=np.float32)
    acc = x32[0].copy()
    for u in range(1, x32.shape[0]):
        acc = (acc + x32[u]).astype(np.float32)
    return (acc * np.float32(1.0 / x32.shape[0])).astype(np.float32)


def complement(n: int, T: np.ndarray) -> np.ndarray:
    """Eq. (10)."""
    keep = np.zeros(n, dtype=bool)
    keep[T] = True
    return np.nonzero(~keep)[0].astype(np.int32)


# --------------------------------------------------------------------------
# Step 3: attention  (Eq. (2); Section 4.2; Algorithm 1 sparse-attention step)
# --------------------------------------------------------------------------
def dense_causal_attention(Qh: np.ndarray, Kg: np.ndarray, Vg: np.ndarray, scale: float,
                           row_block: int = 1024) -> np.ndarray:
    """Eq. (2): O = softmax((Q K^T) * scale + causal mask) V for one head."""
    Qh = np.asarray(Qh, dtype=np.float64)
    Kg = np.asarray(Kg, dtype=np.float64)
    Vg = np.asarray(Vg, dtype=np.float64)
    n = Qh.shape[0]
    O = np.empty((n, Vg.shape[1]))
    for r0 in range(0, n, row_block):          # rows only; memory bound, not a reordering
        r1 = min(n, r0 + row_block)
        S = (Qh[r0:r1] @ Kg[:r1].T) * float(scale)
        S = np.where(np.arange(r1)[None, :] <= np.arange(r0, r1)[:, None], S, -np.inf)
        S = S - S.max(axis=1, keepdims=True)
        E = np.exp(S)
        O[r0:r1] = (E / E.sum(axis=1, keepdims=True)) @ Vg[:r1]
    return O


def kept_token_attention(Qh: np.ndarray, Kg: np.ndarray, Vg: np.ndarray, T: np.ndarray, scale: float,
                         compact_out: bool = False) -> np.ndarray:
    """Attention over the kept tokens only: gather Q[T], K[T], V[T], run causal
    attention on the p gathered rows, and put the outputs back at positions T.
    Rows of dropped tokens are zero ("padded")."""
    T = np.asarray(T, dtype=np.int64)
    Ok = dense_causal_attention(np.asarray(Qh)[T], np.asarray(Kg)[T], np.asarray(Vg)[T], scale)
    if compact_out:
        return Ok
    O = np.zeros((Qh.shape[0], Vg.shape[1]))
    O[T] = Ok
    return O


# --------------------------------------------------------------------------
# Step 4: KV cache  (Section 4.2; Algorithm 1 cache step; Algorithm 2)
# --------------------------------------------------------------------------
def compact_kv(Kg: np.ndarray, Vg: np.ndarray, T: np.ndarray) -> Tuple[np.ndarray, np.ndarray, int]:
    """K <- K[T], V <- V[T] (a copy of the stored values)."""
    T = np.asarray(T, dtype=np.int64)
    return np.array(Kg[T]), np.array(Vg[T]), int(len(T))


def decode_attention(q: np.ndarray, Kc: np.ndarray, Vc: np.ndarray, length: int, scale: float) -> np.ndarray:
    """Eq. (5): one query against the first `length` cached rows."""
    q = np.asarray(q, dtype=np.float64)
    Kc = np.asarray(Kc, dtype=np.float64)[:length]
    Vc = np.asarray(Vc, dtype=np.float64)[:length]
    s = (Kc @ q) * float(scale)
    e = np.exp(s - s.max())
    return (e / e.sum()) @ Vc


def decode_step(q, k_new, v_new, Kc, Vc, length, scale):
    """Algorithm 2: append (k, v) to the cache (Eq. (4)), then attend (Eq. (5)).
    Returns (o, K_out, V_out, length + 1)."""
    Kc = np.concatenate([np.asarray(Kc)[:length], np.asarray(k_new)[None, :]], axis=0)
    Vc = np.concatenate([np.asarray(Vc)[:length], np.asarray(v_new)[None, :]], axis=0)
    return decode_attention(q, Kc, Vc, length + 1, scale), Kc, Vc, length + 1


# --------------------------------------------------------------------------
# Mixed-precision KV cache keyed by T  (Section 5.3.1: important tokens at
# 4 bits, the others at 2 bits; the quantiser itself is not given there)
# --------------------------------------------------------------------------
def quantize_rows(X: np.ndarray, bits: int) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Uniform asymmetric quantisation of every row (one token of one KV head)
    of X [rows, d] to `bits` bits with a per-row (scale, zero) pair kept in
    fp16.  Reading taken here (the paper only names the bit widths):
      zero  = fp16(min_c x_c),  scale = fp16((max_c x_c - min_c x_c) * fp32(1/(2^bits-1)))
      code_c = clamp(rint((x_c - zero) / scale), 0, 2^bits - 1)      (0 when scale = 0)
    all in fp32 with round-half-even, because these steps decide integers and
    the kernel takes them in fp32.  Returns (codes uint8 [rows, d], scale, zero
    float16 [rows])."""
    X = np.asarray(X, dtype=np.float32)
    qmax = np.float32(2 ** bits - 1)
    lo, hi = X.min(axis=1), X.max(axis=1)
    zero = lo.astype(np.float16)
    scale = ((hi - lo) * np.float32(1.0 / float(qmax))).astype(np.float32).astype(np.float16)
    z32, s32 = zero.astype(np.float32)[:, None], scale.astype(np.float32)[:, None]
    with np.errstate(divide="ignore", invalid="ignore"):
        t = ((X - z32).astype(np.float32) / s32).astype(np.float32)
    t = np.where(s32 > 0, t, np.float32(0))
    codes = np.clip(np.rint(t), 0, qmax).astype(np.uint8)
    return codes, scale, zero


def dequantize_rows(codes: np.ndarray, scale: np.ndarray, zero: np.ndarray) -> np.ndarray:
    """x^_c = zero + scale * code_c (float64)."""
    return zero.astype(np.float64)[:, None] + scale.astype(np.float64)[:, None] * codes.astype(np.float64)


def quantize_kv(Kg: np.ndarray, Vg: np.ndarray, T: np.ndarray, hi_bits: int = 4, lo_bits: int = 2):
    """The mixed-precision cache of one KV head: tokens of T (ascending) at
    hi_bits, the others (Eq. (10), ascending) at lo_bits.  Returns a dict with
    the codes / scales / zeros of K and V for both groups."""
    n = np.asarray(Kg).shape[0]
    T = np.asarray(T, dtype=np.int64)
    U = complement(n, T)
    out = {"T": T, "U": U}
    for name, X in (("K", Kg), ("V", Vg)):
        X = np.asarray(X, dtype=np.float32)
        out[name + "_hi"] = quantize_rows(X[T], hi_bits)
        out[name + "_lo"] = quantize_rows(X[U], lo_bits) if len(U) else (np.zeros((0, X.shape[1]), np.uint8), np.zeros(0, np.float16), np.zeros(0, np.float16))
    return out


def decode_attention_quantized(q: np.ndarray, qc: dict, scale: float,
                               K_tail: Optional[np.ndarray] = None, V_tail: Optional[np.ndarray] = None) -> np.ndarray:
    """Eq. (5) over the dequantised cache: every prefill token takes part (the
    important ones from 4-bit codes, the others from 2-bit codes), followed by
    the rows appended during decoding, which are kept as they are."""
    Ks = [dequantize_rows(*qc["K_hi"]), dequantize_rows(*qc["K_lo"])]
    Vs = [dequantize_rows(*qc["V_hi"]), dequantize_rows(*qc["V_lo"])]
    if K_tail is not None and len(K_tail):
        Ks.append(np.asarray(K_tail, dtype=np.float64)); Vs.append(np.asarray(V_tail, dtype=np.float64))
    Kall, Vall = np.concatenate(Ks), np.concatenate(Vs)
    return decode_attention(q, Kall, Vall, len(Kall), scale)


def kv_quant_compression(ratio: float, hi_bits: int = 4, lo_bits: int = 2, elems_per_group: int = 1024,
                         param_bits: int = 32, full_bits: int = 16) -> float:
    """Compression of a 16-bit cache when a fraction `ratio` of the tokens is
    kept at hi_bits and the rest at lo_bits, with one (scale, zero) pair of
    param_bits per group of elems_per_group elements (Section 5.3.1, Table 3;
    a token-wide pair over 8 KV heads of 128 channels is 1024 elements)."""
    return full_bits / (ratio * hi_bits + (1.0 - ratio) * lo_bits + param_bits / elems_per_group)


# --------------------------------------------------------------------------
# Whole layer for one batch element, and the ratio accounting of Tables 2 / 3
# --------------------------------------------------------------------------
def zipvl_prefill_layer(Q, K, V, probe_pos, tau, scale, single_vector: bool = False, shared: bool = False):
    """Algorithm 1 on given Q, K, V states of one batch element.

    Returns dict(mass, rank [Hkv,n] fp32, p [Hkv], T list, O [Hq,n,d],
    Kc, Vc lists).  The fp32 cast of the scores is the precision the selection
    is defined on.  shared=True: one T for the whole layer, selected from the
    head-averaged scores (share_scores); p and T then repeat it per KV head."""
    Hq, n, d = Q.shape
    Hkv = K.shape[0]
    G = Hq // Hkv
    mass, rank = token_scores(Q, K, probe_pos, scale)
    mass32, rank32 = mass.astype(np.float32), rank.astype(np.float32)
    O = np.zeros((Hq, n, V.shape[2]))
    ps, Ts, Kcs, Vcs = [], [], [], []
    if shared:
        p_all, T_all = select(share_scores(mass32), None if single_vector else share_scores(rank32), tau)
    for g in range(Hkv):
        p, T = (p_all, T_all) if shared else select(mass32[g], None if single_vector else rank32[g], tau)
        for h in range(g * G, (g + 1) * G):
            O[h] = kept_token_attention(Q[h], K[g], V[g], T, scale)
        Kc, Vc, _ = compact_kv(K[g], V[g], T)
        ps.append(p), Ts.append(T), Kcs.append(Kc), Vcs.append(Vc)
    return dict(mass=mass32, rank=rank32, p=np.array(ps, dtype=np.int32), T=Ts, O=O, Kc=Kcs, Vc=Vcs)


def attention_flops_reduction(ratio: float) -> float:
    """Attention cost is quadratic in the kept count (Section 3): 1 - r^2."""
    return 1.0 - ratio * ratio


def kv_cache_reduction(ratio: float) -> float:
    """The cache is linear in the kept count (Section 4.2): 1 - r."""
    return 1.0 - ratio


def kept_token_attention_rows(Qh, Kg, Vg, T, rows, scale) -> np.ndarray:
    """Rows `rows` (indices into T) of kept_token_attention's compact output,
    each taken directly from the definition: kept query T_i attends the kept
    keys T_0..T_i.  For spot checks at sizes where the full product is slow."""
    T = np.asarray(T, dtype=np.int64)
    out = np.empty((len(rows), np.asarray(Vg).shape[1]))
    for o, i in enumerate(rows):
        keys = T[: i + 1]
        s = (np.asarray(Kg, dtype=np.float64)[keys] @ np.asarray(Qh, dtype=np.float64)[T[i]]) * float(scale)
        e = np.exp(s - s.max())
        out[o] = (e / e.sum()) @ np.asarray(Vg, dtype=np.float64)[keys]
    return out
