/*
 * zipvl.h - C ABI of the MI355X (gfx950) ZipVL prefill library.
 *
 * The calls follow the paper's statement of the method (arXiv 2410.08584):
 * Algorithm 1 (prefill: probe scores -> adaptive count -> important set ->
 * attention over the kept tokens -> KV-cache eviction) and Algorithm 2
 * (decode against the evicted cache).
 *
 * General rules
 *  - Every pointer marked [device] is GPU memory owned by the caller; the
 *    library borrows it for the duration of the stream-ordered work and never
 *    allocates, frees or synchronises.  Pointers marked [host] are read on the
 *    host before the call returns.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *  - Tensors are addressed as base + b*stride[0] + h*stride[1] + t*stride[2]
 *    + c, strides in ELEMENTS, last dimension (d) contiguous; every row start
 *    must be 16-byte aligned.  Both [B,H,n,d] and [B,n,H,d] memory orders work.
 *  - dtype 0 = IEEE fp32, 1 = bfloat16 (storage); all arithmetic accumulates
 *    in fp32.  d must be 64 or 128.
 *  - A "selection unit" is one (batch, KV head); unit index u = b*Hkv + g.
 *    With grouped-query attention (Hq = G*Hkv) query head h belongs to KV head
 *    h / G.
 *  - Return value: ZIPVL_OK or a negative error code; the text of the last
 *    error of the calling thread is returned by zipvl_last_error().  Invalid
 *    arguments are rejected before any kernel is launched.
 */
#ifndef ZIPVL_H
#define ZIPVL_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ZIPVL_OK             0
#define ZIPVL_EINVAL        -1  /* NULL pointer, negative size, tau outside (0,1], bad probe list */
#define ZIPVL_ESHAPE        -2  /* Hq % Hkv != 0, d not 64/128, n or m beyond the supported maximum */
#define ZIPVL_EALIGN        -3  /* pointer or row stride not 16-byte aligned */
#define ZIPVL_EWORKSPACE    -4  /* workspace missing or too small */
#define ZIPVL_EUNSUPPORTED  -5  /* unknown dtype or flag */
#define ZIPVL_EHIP          -6  /* kernel launch failed */

#define ZIPVL_F32   0
#define ZIPVL_BF16  1

#define ZIPVL_MAX_PROBES 128

/* ops for zipvl_workspace_bytes */
#define ZIPVL_OP_SCORE          1
#define ZIPVL_OP_SELECT         2
#define ZIPVL_OP_SPARSE_PREFILL 3
#define ZIPVL_OP_DECODE         4
#define ZIPVL_OP_QUANTIZE_KV    5
#define ZIPVL_OP_DECODE_Q       6  /* dims->n = cap_hi + cap_lo + cap_tail */
#define ZIPVL_OP_SCORE_ALL_ROWS 7
#define ZIPVL_OP_DECODE_STEP    8  /* dims->n = cap */

/* flags of zipvl_sparse_prefill */
#define ZIPVL_OUT_FULL            0  /* O is [B,Hq,n,d]; rows of dropped tokens are written as zeros */
#define ZIPVL_OUT_COMPACT         1  /* O row i of a head is kept token i (first k rows written) */
#define ZIPVL_KV_ALREADY_COMPACT  2  /* K,V hold the evicted cache: row i is kept token i */
/* flag of zipvl_sparse_prefill and zipvl_compact_kv */
#define ZIPVL_T_PER_BATCH         4  /* idx is [B,n], k is [B]: one important set serves every head of a batch element */

/* flags of zipvl_score */
#define ZIPVL_SCORE_GROUP_MEAN    0  /* one row of scores per (batch, KV head): the mean over the query heads of the group */
#define ZIPVL_SCORE_PER_QHEAD     1  /* one row per (batch, query head): mass, rank are [B*Hq, n], nothing is averaged */

/* bits of the status word of zipvl_select (what its contract excludes, seen in a unit's input) */
#define ZIPVL_SELECT_NEGATIVE     1  /* an entry with the sign bit set: ordered and summed as zero */
#define ZIPVL_SELECT_NONFINITE    2  /* an infinity or NaN: ordered by its bit pattern, summed as zero */
#define ZIPVL_SELECT_OVERFLOW     4  /* mass sums to 2 or more: the integer sum does not fit, k is unreliable */

typedef struct zipvl_dims {
    int32_t B, Hq, Hkv, n, d;
    int32_t dtype;            /* ZIPVL_F32 | ZIPVL_BF16 */
    int64_t q_strides[3];     /* (batch, head, token) strides of Q in elements */
    int64_t k_strides[3];
    int64_t v_strides[3];
} zipvl_dims;

int zipvl_version(void);
const char* zipvl_last_error(void);

/* Bytes of [device] workspace the given op needs for these dims (m = number of
 * probe rows for ZIPVL_OP_SCORE, ignored otherwise).  0 on invalid dims. */
size_t zipvl_workspace_bytes(int op, const zipvl_dims* dims, int m);

/*
 * Token importance from a fixed, small set of probe queries.
 * Paper: supplementary Section A, Eq. (A) (probe attention), Eq. (6)
 * (accumulated score) and Eq. (8) (normalised score); Algorithm 1, steps 2-4.
 *
 *   A'[c,j] = softmax_j( Q[h,P_c] . K[g,j] * softmax_scale ),  keys j > P_c masked
 *   a_j     = sum_c A'[c,j]
 *   mass[u,j] = mean over the G heads of the group of  a_j / m
 *   rank[u,j] = mean over the G heads of the group of  a_j / #{c : P_c >= j}   (0 if none)
 * flags: ZIPVL_SCORE_GROUP_MEAN (default, rows u = b*Hkv + g) or ZIPVL_SCORE_PER_QHEAD (no mean: one row per query
 * head, u = b*Hq + h, mass and rank [B*Hq, n]; the paper writes its equations for a single head).
 *
 * Q [device]          [B,Hq,n,d] by q_strides (only the probe rows are read)
 * K [device]          [B,Hkv,n,d] by k_strides
 * probe_pos [host]    m token positions, strictly ascending, 0 <= P_c < n, 1 <= m <= ZIPVL_MAX_PROBES
 * mass, rank [device] [B*Hkv, n] fp32 contiguous, written for every j (rank may be NULL)
 * ws [device]         zipvl_workspace_bytes(ZIPVL_OP_SCORE, dims, m) bytes, 16-byte aligned
 * A' is never written to memory.  mass of a unit sums to 1 (up to fp32 rounding).
 */
int zipvl_score(const void* Q, const void* K, const zipvl_dims* dims,
                const int32_t* probe_pos, int m, float softmax_scale, int flags,
                float* mass, float* rank, void* ws, size_t ws_bytes, void* stream);

/*
 * The same scores from EVERY row of the attention matrix instead of m probe rows.  Paper: Eq. (6) and
 * Eq. (8) as written in Section 4.1 (the probe rows of the supplementary material approximate these);
 * supplementary Table A, row "all".  A (n x n per head) is never stored; the cost is two passes over the
 * causal half of Q K^T.
 *   A[i,j] = softmax_j( Q[h,i] . K[g,j] * softmax_scale ), keys j > i masked
 *   a_j = sum_{i >= j} A[i,j];  mass[u,j] = group mean of a_j / n;  rank[u,j] = group mean of a_j / (n - j)
 * Q, K, mass, rank as for zipvl_score (rank may be NULL).
 * ws [device]: zipvl_workspace_bytes(ZIPVL_OP_SCORE_ALL_ROWS, dims, 0) bytes, 16-byte aligned.
 */
int zipvl_score_all_rows(const void* Q, const void* K, const zipvl_dims* dims, float softmax_scale,
                         float* mass, float* rank, void* ws, size_t ws_bytes, void* stream);

/*
 * How many tokens to keep and which.  Paper: Eq. (7) (smallest count whose
 * sorted accumulated scores reach tau of the total) and Eq. (9) (that many
 * tokens with the largest normalised score); Algorithm 1, steps 3-5.
 *
 * Per unit u (row u of mass/rank, n entries each, finite and >= 0, mass summing to less than 2 - it
 * sums to 1 when it comes from zipvl_score; an entry with the sign bit set is ordered and summed as 0;
 * n < 2^23):
 *   q_j = floor(mass_j * 2^40)  (exact integers; the sums below are integer sums)
 *   k   = n if tau >= 1, else max(1, min{ i : sum of the i largest q >= ceil(tau * sum of all q) })
 *   T   = the k tokens with the largest rank (equal values: lower index first)
 * idx[u, 0..k-1] receives T in ascending position; idx[u, k..n-1] is left as is.
 *
 * mass [device] [units,n] fp32; rank [device] same shape or NULL (use mass for both steps)
 * tau in (0,1];  idx [device] [units,n] int32;  k [device] [units] int32
 * status [device] [units] int32 or NULL: when given, every unit's inputs are checked on the device against the
 * contract above (one more pass over them) and status[u] receives ZIPVL_SELECT_* bits, 0 if all is well; nothing
 * is read back and the selection runs either way (validation that needs device data cannot be an error code of a
 * call that does not synchronise).
 * ws [device] may be NULL: one kernel, one workgroup per unit.  With a workspace of
 * zipvl_workspace_bytes(ZIPVL_OP_SELECT, dims with B * Hkv = units, 0) bytes (16-byte aligned) the first,
 * widest digit of the search is histogrammed by the whole chip and one workgroup per unit finishes (two
 * kernels; faster for long vectors on few units).  That workspace must be ZERO before the first call that uses
 * it; every call leaves it zero; two calls that overlap on one workspace race.  Same results either way.
 */
int zipvl_select(const float* mass, const float* rank, int units, int n, double tau,
                 int32_t* idx, int32_t* k, int32_t* status, void* ws, size_t ws_bytes, void* stream);

/*
 * One important set per layer instead of one per KV head.  Paper: Algorithm 1 as written selects a
 * single T and hands Q[T], K[T], V[T] to one attention call; this is that reading (the per-head
 * selection is the other one).  The per-unit scores of zipvl_score are averaged over the Hkv units
 * of each batch element, and zipvl_select then runs on B units:
 *   mass_b[b,j] = (mass[b*Hkv+0, j] + mass[b*Hkv+1, j] + ... ) * (1/Hkv)   fp32, units added in ascending order
 * rank_b likewise (rank and rank_b may both be NULL).  mass, rank [device] [B*Hkv, n] fp32;
 * mass_b, rank_b [device] [B, n] fp32 (must not alias the inputs).  Pass the resulting idx [B,n], k [B]
 * to zipvl_sparse_prefill / zipvl_compact_kv with ZIPVL_T_PER_BATCH.
 */
int zipvl_share_scores(const float* mass, const float* rank, int B, int Hkv, int n,
                       float* mass_b, float* rank_b, void* stream);

/*
 * Causal attention over the kept tokens only.  Paper: Section 4.2 and
 * Algorithm 1, sparse-attention step (O = Attention(Q[T], K[T], V[T])), Eq. (2)
 * restricted to T; outputs of dropped tokens are padded (with zeros here).
 *
 * For every query head h of unit u, with T = idx[u, 0..k[u]-1] (ascending):
 *   O[h, T_i] = sum_{j<=i} softmax_j( Q[h,T_i] . K[g,T_j] * softmax_scale ) V[g,T_j]
 * idx, k [device] as written by zipvl_select; both NULL = every token kept (dense).
 * T must hold strictly ascending positions in [0, n) (not checked: the values live on the device).
 * flags: ZIPVL_OUT_FULL (default) | ZIPVL_OUT_COMPACT | ZIPVL_KV_ALREADY_COMPACT | ZIPVL_T_PER_BATCH
 * (with ZIPVL_T_PER_BATCH, T of unit u is idx[b, 0..k[b]-1]).
 * O [device] [B,Hq,n,d] contiguous, dtype as the inputs.
 * ws [device] zipvl_workspace_bytes(ZIPVL_OP_SPARSE_PREFILL, dims, 0) bytes, 256-byte aligned.
 * Numerics: accumulation in fp32; probabilities of a bf16 call are rounded to bf16 before they weigh V and before
 * they are summed.  Logits of any finite magnitude are handled: rows whose scaled logits all lie within about
 * +-44 of zero are exponentiated without an offset, a workgroup with any other row repeats its keys with running
 * maxima (twice the time for that workgroup, the same result up to rounding).  Inputs must be finite.
 */
int zipvl_sparse_prefill(const void* Q, const void* K, const void* V, const zipvl_dims* dims,
                         const int32_t* idx, const int32_t* k, float softmax_scale, int flags,
                         void* O, void* ws, size_t ws_bytes, void* stream);

/*
 * KV-cache eviction.  Paper: Section 4.2, Algorithm 1 cache step (K <- K[T], V <- V[T]).
 * Kc[u, i, :] = K[g, T_i, :], Vc likewise (bit copies), len[u] = k[u].
 * Kc, Vc [device] [B*Hkv, cap, d] contiguous; cap >= max k (rows beyond cap are
 * not written and len is clamped to cap).  idx,k NULL = copy all n rows.
 * flags: 0 or ZIPVL_T_PER_BATCH (idx [B,n], k [B]; len is still written per unit).
 */
int zipvl_compact_kv(const void* K, const void* V, const zipvl_dims* dims,
                     const int32_t* idx, const int32_t* k,
                     void* Kc, void* Vc, int32_t cap, int32_t* len, int flags, void* stream);

/*
 * Decode step, cache side.  Paper: Eq. (4) / Algorithm 2 (K_out = Concat(K_in, k)).
 * Writes k_new[u,:], v_new[u,:] ([B*Hkv, d] contiguous) at row len[u] of each
 * unit's cache and increments len[u]; a full cache (len == cap) is left unchanged.
 * dims->n is ignored; dims->dtype, B, Hkv, d are used.
 */
int zipvl_kv_append(void* Kc, void* Vc, int32_t* len, int32_t cap, const void* k_new,
                    const void* v_new, const zipvl_dims* dims, void* stream);

/*
 * Decode step, attention side.  Paper: Eq. (5) / Algorithm 2:
 *   o[h] = softmax( q[h] . Kc[u, 0..len[u]-1]^T * softmax_scale ) Vc[u, 0..len[u]-1]
 * q, o [device] [B*Hq, d] contiguous; Kc, Vc [device] [B*Hkv, cap, d]; len [device] [B*Hkv].
 * Memory-bound: each cached row is read once per call.  G = Hq/Hkv <= 8.
 * ws [device] zipvl_workspace_bytes(ZIPVL_OP_DECODE, dims (n = cap), 0) bytes.
 */
int zipvl_decode_attn(const void* q, const void* Kc, const void* Vc, const int32_t* len,
                      int32_t cap, const zipvl_dims* dims, float softmax_scale,
                      void* o, void* ws, size_t ws_bytes, void* stream);

/*
 * zipvl_decode_attn for callers that cannot allocate device memory or carry a workspace: code under
 * HIP-graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels
 * and same results as zipvl_decode_attn, without ws / ws_bytes: the partial states of the split-KV kernels
 * live in a fixed array of ZIPVL_STATIC_SCRATCH_BYTES inside the library (one copy per GPU, held until the
 * process ends).  The call allocates and frees nothing.  Dims whose zipvl_workspace_bytes(ZIPVL_OP_DECODE)
 * exceeds ZIPVL_STATIC_SCRATCH_BYTES are rejected with ZIPVL_ESHAPE before anything is launched.
 * Every call on a GPU uses that GPU's one array: calls that overlap in time on one GPU (two streams, two
 * threads) race on it; calls ordered on one stream do not.  The array keeps the last call's contents;
 * nothing in it has to be cleared between calls.
 */
#define ZIPVL_STATIC_SCRATCH_BYTES (8u << 20)
int zipvl_decode_attn_static(const void* q, const void* Kc, const void* Vc, const int32_t* len,
                             int32_t cap, const zipvl_dims* dims, float softmax_scale, void* o, void* stream);

/*
 * One decode step in one launch: zipvl_kv_append followed by zipvl_decode_attn (Eq. (4), Eq. (5) /
 * Algorithm 2), with the same results: the new row is written at row len[u] and takes part in the
 * attention, len[u] is incremented afterwards; a full cache (len == cap) is left unchanged and attended
 * as it is.  Arguments as in those two calls.
 * ws [device]: zipvl_workspace_bytes(ZIPVL_OP_DECODE_STEP, dims (n = cap), 0) bytes, 16-byte aligned.  Its
 * first 4 * B * Hkv bytes are per-unit arrival counters: they must be zero before the first call that
 * uses this workspace, every call leaves them zero, and nothing else may write there between calls
 * (two calls that overlap on one workspace race).  Groups larger than 8 query heads per KV head run the
 * two separate kernels inside this call.
 */
int zipvl_decode_step(const void* q, void* Kc, void* Vc, int32_t* len, int32_t cap, const void* k_new,
                      const void* v_new, const zipvl_dims* dims, float softmax_scale, void* o,
                      void* ws, size_t ws_bytes, void* stream);

/*
 * Mixed-precision KV cache keyed by the important set.  Paper: Section 5.3.1 and Table 3 (important
 * tokens quantised to 4 bits, the other tokens to 2 bits; nothing is evicted).  The quantiser itself is
 * not given there; the one used is uniform, asymmetric, per row (one token of one KV head), in fp32:
 *   zero = fp16(min_c x_c),  scale = fp16((max_c x_c - min_c x_c) * fp32(1/(2^bits - 1))),
 *   code_c = clamp(rint((x_c - zero) / scale), 0, 2^bits - 1)   (all codes 0 when scale = 0),
 *   dequantised value = zero + scale * code_c.
 * One tensor (K or V) of the cache is four [device] arrays:
 */
typedef struct zipvl_qtensor {
    void* hi_codes;   /* [units, cap_hi, d/2] bytes: 4-bit codes, element c in byte c/2, bits 4*(c%2)..4*(c%2)+3 */
    void* hi_params;  /* [units, cap_hi, 2] fp16: (scale, zero) of the row */
    void* lo_codes;   /* [units, cap_lo, d/4] bytes: 2-bit codes, element c in byte c/4, bits 2*(c%4)..2*(c%4)+1 */
    void* lo_params;  /* [units, cap_lo, 2] fp16 */
} zipvl_qtensor;

/*
 * Builds the cache from the prefill K, V [B,Hkv,n,d]: row i of the 4-bit group of unit u is token T_i,
 * row i of the 2-bit group is the i-th token not in T (Eq. (10), ascending position).
 * len_hi[u] = min(k, cap_hi), len_lo[u] = min(n - k, cap_lo) [device, units]; rows beyond a cap are not written.
 * idx, k as written by zipvl_select (NULL = every token important); flags: 0 or ZIPVL_T_PER_BATCH.
 * ws [device]: zipvl_workspace_bytes(ZIPVL_OP_QUANTIZE_KV, dims, 0) bytes, 4-byte aligned.  n <= 262144.
 * All eight arrays 16-byte aligned.
 */
int zipvl_quantize_kv(const void* K, const void* V, const zipvl_dims* dims, const int32_t* idx, const int32_t* k,
                      const zipvl_qtensor* Kq, const zipvl_qtensor* Vq, int32_t cap_hi, int32_t cap_lo,
                      int32_t* len_hi, int32_t* len_lo, int flags, void* ws, size_t ws_bytes, void* stream);

/*
 * Decode attention (Eq. (5) / Algorithm 2) over the mixed-precision cache followed by the rows appended
 * during decoding (K_tail, V_tail [units, cap_tail, d] in the dtype of q, len_tail [units]; all three NULL =
 * no appended rows; zipvl_kv_append maintains them):
 *   o[h] = softmax( q[h] . [K^_hi ; K^_lo ; K_tail]^T * softmax_scale ) [V^_hi ; V^_lo ; V_tail]
 * with K^, V^ the dequantised rows.  q, o [B*Hq, d]; G = Hq/Hkv <= 8.
 * ws [device]: zipvl_workspace_bytes(ZIPVL_OP_DECODE_Q, dims with n = cap_hi + cap_lo + cap_tail, 0) bytes.
 */
int zipvl_decode_attn_q(const void* q, const zipvl_qtensor* Kq, const zipvl_qtensor* Vq,
                        const int32_t* len_hi, const int32_t* len_lo, int32_t cap_hi, int32_t cap_lo,
                        const void* K_tail, const void* V_tail, const int32_t* len_tail, int32_t cap_tail,
                        const zipvl_dims* dims, float softmax_scale, void* o, void* ws, size_t ws_bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* ZIPVL_H */
