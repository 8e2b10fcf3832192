// Attention over the kept tokens (Section 4.2; Algorithm 1, sparse-attention
// step; Eq. (2) restricted to the important set T).
//
// Two kernels:
//   pack   gathers K[T] and V[T] into the workspace, once per KV head, zero-filling
//          the ragged tail.  bf16: both row-major (the P.V operand is fetched from
//          LDS with the transposing read, so an evicted cache with whole tiles is
//          read in place and nothing is packed at all); fp32: V[T] transposed
//          ([d][64 keys] tiles), so that both MFMA operands are contiguous fragments.
//   flash  one workgroup = 128 kept queries of one query head (4 waves x 32
//          rows).  K / V tiles of 64 keys are loaded straight into LDS (double
//          buffered) and shared by the four waves.  S^T = K Q^T and O^T = V^T P^T
//          are taken on 32x32 MFMA tiles, so a lane owns one query column and the
//          softmax statistics are per-lane scalars.  The key loop is a pipeline
//          three tiles deep: a step multiplies P.V for tile t-1, takes the
//          exponentials of tile t and multiplies K Q^T for tile t+1, with the
//          instruction order of the steady state written out (operand reads a few
//          matrix instructions ahead, the vector work and the tile requests spread
//          between them); every tile has a whole step to arrive from memory.
//          The first pass over the keys uses no exponent offset at all (no running
//          maximum, no exchange between lanes, no rescaling): exp2 of the scaled
//          logits as they are.  That is exact as long as the row sums stay far
//          inside the fp32 range, which is checked at the end; a workgroup with a
//          row outside [2^-64, 2^64] repeats its tiles with running maxima.
//          Causality is the plain lower triangle in kept-token coordinates because
//          T is ascending.  Query rows are gathered by idx on load, output rows are
//          scattered by idx on store.  The zero rows of dropped tokens are written
//          by extra workgroups at the end of the same grid (one per head and span
//          of positions), which run in the slots the thinning end of the
//          attention work leaves idle.
// The kept count k lives on the device: the grid covers the worst case (k = n)
// and workgroups beyond a unit's k exit at once; heavy (late) query tiles are
// scheduled first, over all KV heads of a schedule group, because the longest
// workgroup (all k keys) lasts a large part of the whole launch.
#include <algorithm>
#include <atomic>
#include <type_traits>

#include "launch.h"
#include "ldsload.h"

namespace zipvl {

constexpr int kBN = 64;      // keys per tile
// bf16 launch shape: 4 waves x 32 queries.  Measured alternatives: 8 waves per workgroup (half the L2 -> LDS
// traffic per query) is 3 % slower; 64 queries per wave (QB = 2, half the LDS operand reads per MFMA) does
// not fit the register file with the S^T double buffer and spills.
constexpr int kFlashWavesBf16 = 4;
constexpr int kFlashBlocksBf16 = 1;
constexpr int kFillSpan = 512;       // positions per workgroup that clears dropped output rows
constexpr float kLazyLog2 = 8.f;     // slack of the running softmax offset below the running maximum (log2 domain)
constexpr float kSumLow = 0x1p-64f, kSumHigh = 0x1p64f;   // row sums of the offset-free pass that need no second pass
constexpr int kSchedAhead = 3;       // LDS operand reads in flight ahead of the consuming MFMA

// NW = waves per workgroup, QB = 32-query blocks per wave: a workgroup covers 32 QB NW kept queries, its
// K / V^T tiles are fetched from L2 once per that many queries, and every LDS operand fragment a wave
// reads feeds QB matrix instructions.
template <typename T, int D, int NW = 4, int QB = 1>
struct AttnCfg {
    static constexpr int E = Elem<T>::kBytes;
    static constexpr int BM = 32 * QB * NW;                  // queries per workgroup
    static constexpr int NT = 64 * NW;                       // threads per workgroup
    static constexpr int CH = D / Elem<T>::kPerChunk;       // Q/K fragments per row per lane
    static constexpr int ODB = D / 32;                       // 32-row blocks of O^T
    // LDS tiles are unpadded; the 16-byte chunks of a row are XOR-swizzled with the row index instead, so
    // that 16 consecutive rows read at the same logical chunk hit 16 different bank groups.
    static constexpr int KRB = D * E;                        // bytes per K row
    // bf16: V tiles stay row-major ([64 keys][d], like K) and the P.V operand is fetched with the LDS
    // transposing read; fp32 (no such read for 32-bit elements): V^T tiles ([d][64 keys]) packed beforehand.
    static constexpr bool VROWS = E == 2;
    static constexpr int VRB = VROWS ? D * E : kBN * E;      // bytes per row of a V tile
    static constexpr int TILE_BYTES = kBN * D * E;           // one K tile = one V tile
    static constexpr int NLD = TILE_BYTES / 1024 / NW;       // 1-KiB direct-to-LDS loads per wave per tile
    static constexpr int LDS_BYTES = 4 * TILE_BYTES;         // two K and two V buffers
    // bf16, QB = 1: two waves per SIMD (<= 256 registers, accumulators stay in VGPRs); otherwise one
    // wave per SIMD with the whole 512-entry register file
    static constexpr int MIN_WGS = (E == 2 && QB == 1) ? 8 / NW : 1;
};

// ------------------------------------------------------------------ pack
// Key held at element e of 16-byte chunk kc of a V^T tile row (fp32 path): natural order.
__device__ __forceinline__ int vt_key(int kc, int e) { return kc * 4 + e; }

template <typename T, int D>
__global__ __launch_bounds__(256) void pack_kv_kernel(
    const T* __restrict__ K, const T* __restrict__ V,
    int64_t ks0, int64_t ks1, int64_t ks2, int64_t vs0, int64_t vs1, int64_t vs2,
    const int32_t* __restrict__ idx, const int32_t* __restrict__ kcnt,
    T* __restrict__ Kp, T* __restrict__ Vp, int n, int npad, int Hkv, int rows_are_kept, int skip_k, int t_per_batch)
{
    constexpr int EPF = Elem<T>::kPerFrag;
    constexpr int CPR = D / EPF;
    constexpr int LS = D + EPF;                 // padded LDS row (elements)
    constexpr bool VROWS = Elem<T>::kBytes == 2;
    __shared__ __attribute__((aligned(16))) T tile[VROWS ? EPF : kBN * LS];
    const int u = blockIdx.y, b = u / Hkv, g = u - b * Hkv;
    const int t0 = blockIdx.x * kBN;
    const int ut = t_per_batch ? b : u;                   // row of idx / k that holds this unit's T
    int kk = kcnt ? kcnt[ut] : n;
    kk = max(0, min(kk, n));
    if (t0 >= kk) return;
    const T* Kb = K + b * ks0 + g * ks1;
    const T* Vb = V + b * vs0 + g * vs1;
    for (int wi = threadIdx.x; wi < kBN * CPR; wi += 256) {
        const int r = wi / CPR, cc = wi - r * CPR, row = t0 + r;
        uintx4 kv = {0, 0, 0, 0}, vv = {0, 0, 0, 0};
        if (row < kk) {
            const int src = (idx && !rows_are_kept) ? idx[(int64_t)ut * n + row] : row;
            if (!skip_k) kv = load16(Kb + (int64_t)src * ks2 + cc * EPF);
            vv = load16(Vb + (int64_t)src * vs2 + cc * EPF);
        }
        if (!skip_k) store16(Kp + ((int64_t)u * npad + row) * D + cc * EPF, kv);
        if (VROWS) store16(Vp + ((int64_t)u * npad + row) * D + cc * EPF, vv);      // rows past k are zero rows
        else store16(tile + r * LS + cc * EPF, vv);
    }
    if (VROWS) return;
    __syncthreads();
    T* VT = Vp + ((int64_t)u * (npad / kBN) + blockIdx.x) * (D * kBN);
    for (int wi = threadIdx.x; wi < D * (kBN / EPF); wi += 256) {
        const int dd = wi % D, kc = wi / D;
        T v[EPF];
#pragma unroll
        for (int e = 0; e < EPF; ++e) v[e] = tile[vt_key(kc, e) * LS + dd];
        store16(VT + dd * kBN + kc * EPF, *reinterpret_cast<const uintx4*>(v));
    }
}

// ------------------------------------------------------------------ flash
// One tile (TILE_BYTES contiguous in global memory) -> one LDS buffer, without passing through
// registers: every wave issues NLD loads of 1 KiB, lane L of a load writes LDS bytes [16 L, 16 L + 16)
// of that KiB, and picks the global chunk that belongs there under the row swizzle.


// per-lane source offsets for tile_to_lds (rows of RB bytes)
// Row swizzle of a row-major bf16 V tile (rows of RB bytes): the transposing read of a 16-lane group
// touches 4 consecutive keys x 4 consecutive 16-byte chunks, so the key index goes into chunk bits 2..3
// (one bit of it is already an address bit when two rows share a 256-byte bank period).
template <int RB>
__device__ __forceinline__ int v_row_swizzle(int row) { return ((row & 3) >> (RB == 128 ? 1 : 0)) << 2; }

template <int RB, int NW, int NLD, bool VSWZ = false>
__device__ __forceinline__ void lds_fill_offsets(int w, int lane, int (&off)[NLD]) {
#pragma unroll
    for (int q = 0; q < NLD; ++q) {
        const int o = (q * NW + w) * 1024 + lane * 16;
        const int r = o / RB, p = (o % RB) >> 4;
        off[q] = r * RB + ((p ^ (VSWZ ? v_row_swizzle<RB>(r) : k_row_swizzle<RB>(r))) << 4);
    }
}

// Load q of a tile (see tile_to_lds).  When the NW KiB that the waves fetch together cover a whole number of
// swizzle periods (16 rows), a lane's offset inside every such group is the same: one register serves all
// loads and the group's offset goes into the scalar base address.
template <int RB, int NW> constexpr bool kOffsetsRepeat = (NW * 1024 / RB) % 16 == 0;

template <int RB, int NW, int NLD>
__device__ __forceinline__ void tile_load(const char* gtile, int q, const int (&off)[NLD], unsigned lds_dst) {
    if constexpr (kOffsetsRepeat<RB, NW>) load_kib_to_lds(gtile + q * NW * 1024, off[0], lds_dst);
    else load_kib_to_lds(gtile, off[q], lds_dst);
}
template <int RB, int NW, int NLD>
__device__ __forceinline__ void tile_load_pinned(const char* gtile, int q, const int (&off)[NLD], unsigned lds_dst, unsigned& pin) {
    if constexpr (kOffsetsRepeat<RB, NW>) load_kib_to_lds_pinned(gtile + q * NW * 1024, off[0], lds_dst, pin);
    else load_kib_to_lds_pinned(gtile, off[q], lds_dst, pin);
}

template <int RB, int NW, int NLD>
__device__ __forceinline__ void tile_to_lds(const char* gtile, char* lbuf, int w, const int (&off)[NLD]) {
    const unsigned lbase = lds_address(lbuf);
#pragma unroll
    for (int q = 0; q < NLD; ++q) tile_load<RB, NW, NLD>(gtile, q, off, lbase + (q * NW + w) * 1024);
}

// S^T = K Q^T for 32 keys (block blk of the 64-key tile in LDS buffer kb) and the wave's QB query blocks:
// acc[qb][blk][r] = key 32*blk + acc_row(r, h), this lane's query of block qb.  A K fragment is read once for all QB.
template <typename T, int D, int NW, int QB>
__device__ __forceinline__ void qk_block(const char* kb, int blk, int i, int h, int sw,
                                         const uintx4 (&qf)[QB][AttnCfg<T, D, NW, QB>::CH], floatx16 (&acc)[QB][2]) {
    using C = AttnCfg<T, D, NW, QB>;
    floatx16 a[QB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) a[qb] = floatx16{0};
#pragma unroll
    for (int cc = 0; cc < C::CH; ++cc) {
        const uintx4 kf = *reinterpret_cast<const uintx4*>(kb + (blk * 32 + i) * C::KRB + swz_chunk(2 * cc + h, sw));
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) a[qb] = mma_frag<T>(kf, qf[qb][cc], a[qb]);
    }
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) acc[qb][blk] = a[qb];
}

// O^T += V^T P^T for the 32 keys of half HALF: p[qb][HALF] holds the probabilities of S^T block HALF of query block qb.
template <typename T, int D, int NW, int QB> struct PV;

template <int D, int NW, int QB> struct PV<__bf16, D, NW, QB> {
    using C = AttnCfg<__bf16, D, NW, QB>;
    // p[qb][blk][s2]: the probabilities of S^T block blk as P^T operand fragments.  Contraction slot t of
    // this lane <-> key 16*s2 + 8*(t/4) + 4*h + t%4 of the block = accumulator register 8*s2 + t.
    using Probs = uintx4[QB][2][2];
    // The matching V^T operand (lane = channel 32 db + lane % 32, slots = those 8 keys) comes from the
    // row-major V tile through ds_read_b64_tr_b16: in every group of 16 lanes, lane 4e + q supplies the
    // address of 4 consecutive channels of key e, and lane l receives channel l of keys 0..3.  Two reads
    // (keys +0..3 and +8..11 relative to 16 s2 + 4 h) make one operand.  lane_off[db]: this lane's
    // supplier address inside a tile for channel block db (row swizzle included).
    __device__ static __forceinline__ void lane_offsets(int lane, int (&lane_off)[C::ODB]) {
        const int h = lane >> 5, grp = (lane >> 4) & 1, e = (lane >> 2) & 3, q = lane & 3;
        const int row = 4 * h + e;                           // key inside its group of 8 = swizzle of the row
#pragma unroll
        for (int db = 0; db < C::ODB; ++db)
            lane_off[db] = row * C::VRB + swz_chunk(4 * db + 2 * grp + (q >> 1), v_row_swizzle<C::VRB>(row)) + (q & 1) * 8;
    }
    template <int HALF>
    __device__ static __forceinline__ void run(const char* vb, const int (&lane_off)[C::ODB], const Probs& p,
                                               floatx16 (&o)[QB][C::ODB]) {
        typedef short shortx4 __attribute__((ext_vector_type(4)));
        using lds_ptr = __attribute__((address_space(3))) shortx4*;
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) {
#pragma unroll
            for (int db = 0; db < C::ODB; ++db) {
                const char* a0 = vb + lane_off[db] + (32 * HALF + 16 * s2) * C::VRB;
                const uintx2 lo = __builtin_bit_cast(uintx2, __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)a0));
                const uintx2 hi = __builtin_bit_cast(uintx2, __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(a0 + 8 * C::VRB)));
                const uintx4 vf = {lo[0], lo[1], hi[0], hi[1]};
#pragma unroll
                for (int qb = 0; qb < QB; ++qb) o[qb][db] = mma_frag<__bf16>(vf, p[qb][HALF][s2], o[qb][db]);
            }
        }
    }
};

template <int D, int NW, int QB> struct PV<float, D, NW, QB> {
    using C = AttnCfg<float, D, NW, QB>;
    using Probs = floatx16[QB][2];                           // p[qb][blk][r]: as the S^T accumulators
    // lane_off[0] = V^T row of this lane inside a channel block and [1] = its swizzle (i, i & 7)
    __device__ static __forceinline__ void lane_offsets(int lane, int (&lane_off)[C::ODB]) {
        lane_off[0] = lane & 31;
        lane_off[1] = lane >> 5;
    }
    template <int HALF>
    __device__ static __forceinline__ void run(const char* vb, const int (&lane_off)[C::ODB], const Probs& p, floatx16 (&o)[QB][C::ODB]) {
        const int i = lane_off[0], h = lane_off[1], sw = k_row_swizzle<C::VRB>(i);
#pragma unroll
        for (int a = 0; a < 4; ++a) {
            // step (a, t): this lane contributes key 32*HALF + 8*a + 4*h + t
            const int chunk = swz_chunk(8 * HALF + 2 * a + h, sw);
#pragma unroll
            for (int db = 0; db < C::ODB; ++db) {
                const floatx4 v = *reinterpret_cast<const floatx4*>(vb + (db * 32 + i) * C::VRB + chunk);
#pragma unroll
                for (int t = 0; t < 4; ++t)
#pragma unroll
                    for (int qb = 0; qb < QB; ++qb)
                        o[qb][db] = __builtin_amdgcn_mfma_f32_32x32x2f32(v[t], p[qb][HALF][4 * a + t], o[qb][db], 0, 0, 0);
            }
        }
    }
};

// The two half-waves (lanes l and l ^ 32) hold the two halves of each query's keys: combine a per-lane
// value across them with one register swap (no trip through LDS).
__device__ __forceinline__ float xhalf_max(float v) {
    const unsigned u = __float_as_uint(v);
    const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);   // r[0] = lower halves twice, r[1] = upper halves twice
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float xhalf_sum(float v) {
    const unsigned u = __float_as_uint(v);
    const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

template <typename T> __device__ __forceinline__ void store_out4(T* dst, float a, float b, float c, float d);
template <> __device__ __forceinline__ void store_out4<float>(float* dst, float a, float b, float c, float d) {
    *reinterpret_cast<floatx4*>(dst) = floatx4{a, b, c, d};
}
template <> __device__ __forceinline__ void store_out4<__bf16>(__bf16* dst, float a, float b, float c, float d) {
    *reinterpret_cast<uintx2*>(dst) = uintx2{pack_bf16x2(a, b), pack_bf16x2(c, d)};
}

template <typename T, int D, int NW, int QB>
__global__ __launch_bounds__(64 * NW, (AttnCfg<T, D, NW, QB>::MIN_WGS)) void flash_kept_kernel(
    const T* __restrict__ Q, int64_t qs0, int64_t qs1, int64_t qs2,
    const T* __restrict__ Kp, int64_t kp0, int64_t kp1, const T* __restrict__ Vp, int64_t vp0, int64_t vp1,
    const int32_t* __restrict__ idx, const int32_t* __restrict__ kcnt,
    T* __restrict__ O, int n, int npad, int ntq, int ug, int BH, int Hq, int Hkv, float c, int out_compact, int compute_blocks,
    int t_per_batch, int v_in_place)
{
    using C = AttnCfg<T, D, NW, QB>;
    constexpr int kBM = C::BM, kNT = C::NT, kRW = 32 * QB;   // queries per workgroup, threads, queries per wave
    extern __shared__ __attribute__((aligned(16))) char smem[];
    // Workgroup -> (unit group, query tile, unit in group, head of the KV group), in that order of
    // significance; heavy (late) query tiles first inside a group.  A group holds enough KV heads to
    // fill the chip several times over (a few for long GQA sequences, many for short MHA ones): the
    // chip then works through few KV heads at a time, so the caches hold little more than the K / V
    // in use, while the light tail of one group overlaps the heavy start of the next.  The last query
    // tile of a head runs for as long as all its kept keys take; a group must hold many times the
    // chip's resident workgroups for that one not to end alone.
    const int G = Hq / Hkv, NU = BH / G;
    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, i = lane & 31, h = lane >> 5;
    if (blockIdx.x >= (unsigned)compute_blocks) {
        // Outputs of dropped tokens are zero rows.  The workgroups after the last attention workgroup
        // each clear the dropped rows of one head inside one span of kFillSpan positions; they are
        // dispatched last, into the slots that the light end of the attention work leaves idle.
        const int f = blockIdx.x - compute_blocks, s = f / BH, fbh = f - s * BH;
        const int fb = fbh / Hq, fu = fb * Hkv + (fbh - fb * Hq) / G;
        const int32_t* ft = idx + (int64_t)(t_per_batch ? fb : fu) * n;
        const int fk = kcnt ? max(0, min(kcnt[t_per_batch ? fb : fu], n)) : n;
        const int p0 = s * kFillSpan, p1 = min(n, p0 + kFillSpan);
        int* kept = reinterpret_cast<int*>(smem);            // [kFillSpan]
        for (int e = tid; e < kFillSpan; e += kNT) kept[e] = 0;
        int lo = 0, hi = fk;                                 // first kept row at or after p0 (T ascends)
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (ft[mid] < p0) lo = mid + 1; else hi = mid;
        }
        __syncthreads();
        for (int e = lo + tid; e < min(fk, lo + kFillSpan); e += kNT) {
            const int pos = ft[e];
            if (pos >= p0 && pos < p1) kept[pos - p0] = 1;
        }
        __syncthreads();
        constexpr int CPR = D * Elem<T>::kBytes / 16;
        const uintx4 z = {0, 0, 0, 0};
        char* base = reinterpret_cast<char*>(O + ((int64_t)fbh * n + p0) * D);
        for (int q = tid; q < (p1 - p0) * CPR; q += kNT)
            // whole rows, written once and not read again by this path: streaming stores, so that they do not stay
            // behind as dirty lines in the last-level cache, to be written back under the next kernel's reads
            if (!kept[q / CPR]) __builtin_nontemporal_store(z, reinterpret_cast<uintx4*>(base + (int64_t)q * 16));
        return;
    }
    const int full = ug * ntq * G;                           // workgroups of a full group
    const int ngroups = (NU + ug - 1) / ug;
    const int grp = min((int)(blockIdx.x / full), ngroups - 1);
    const int r = blockIdx.x - grp * full;
    const int nu_g = min(ug, NU - grp * ug);
    const int tile_rev = r / (nu_g * G), rr = r - tile_rev * (nu_g * G);
    const int u = grp * ug + rr / G, hg = rr % G;
    const int b = u / Hkv, g = u - b * Hkv, head = g * G + hg, bh = b * Hq + head;
    const int i0 = (ntq - 1 - tile_rev) * kBM;
    const int32_t* tidx = idx ? idx + (int64_t)(t_per_batch ? b : u) * n : nullptr;   // this unit's T
    int kk = kcnt ? kcnt[t_per_batch ? b : u] : n;
    kk = max(0, min(kk, n));
    if (i0 >= kk) return;
    floatx16 o[QB][C::ODB];
    float m_run[QB], l_run[QB];

    const int ntiles = (min(i0 + kBM, kk) + kBN - 1) / kBN;
    const int wave_first_row = i0 + kRW * w, wave_last_row = wave_first_row + kRW - 1;
    const int my_tiles = min(ntiles, wave_last_row / kBN + 1);   // later tiles lie wholly in this wave's future
    const char* kg = reinterpret_cast<const char*>(Kp + b * kp0 + g * kp1);   // row-major kept K rows of this unit
    const char* vg = reinterpret_cast<const char*>(Vp + b * vp0 + g * vp1);   // V tiles of this unit (V^T tiles for fp32)
    char* const Kb0 = smem;
    char* const Vb0 = smem + 2 * C::TILE_BYTES;
    const int sw = k_row_swizzle<C::KRB>(i);
    int koff[C::NLD], voff[C::NLD];
    lds_fill_offsets<C::KRB, NW, C::NLD>(w, lane, koff);
    lds_fill_offsets<C::VRB, NW, C::NLD, C::VROWS>(w, lane, voff);
    int vlane[C::ODB];
    PV<T, D, NW, QB>::lane_offsets(lane, vlane);

    const unsigned klds = lds_address(Kb0) + w * 1024, vlds = lds_address(Vb0) + w * 1024;
    // The first tiles are requested before anything else is loaded: their addresses need only scalars, while the
    // query rows below wait for their positions first (two round trips).
    auto request_first_tiles = [&]() {
        tile_to_lds<C::KRB, NW, C::NLD>(kg, Kb0, w, koff);
        tile_to_lds<C::VRB, NW, C::NLD>(vg, Vb0, w, voff);
        if (ntiles > 1) tile_to_lds<C::KRB, NW, C::NLD>(kg + C::TILE_BYTES, Kb0 + C::TILE_BYTES, w, koff);
    };
    request_first_tiles();
    // kept-token coordinates of this lane's QB queries, their positions, their Q fragments
    int qrow[QB], qpos[QB];
    uintx4 qf[QB][C::CH];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        qrow[qb] = i0 + kRW * w + 32 * qb + i;
        const int qclamp = min(qrow[qb], kk - 1);
        qpos[qb] = tidx ? tidx[qclamp] : qclamp;
        const T* qp = Q + b * qs0 + head * qs1 + (int64_t)qpos[qb] * qs2;
#pragma unroll
        for (int cc = 0; cc < C::CH; ++cc) qf[qb][cc] = load16(qp + cc * Elem<T>::kPerChunk + h * Elem<T>::kPerFrag);
    }
    // One pass over the key tiles.  SAFE = false: the exponent offset stays 0 (softmax is shift invariant, and
    // floating point keeps its relative precision at any magnitude), so there is no running maximum, no
    // exchange between lanes and no rescaling in the loop; valid as long as the row sums stay far inside the
    // fp32 range, which is checked afterwards.  SAFE = true: the offset follows the running maximum.
    auto pass = [&](auto safe_tag) {
    constexpr bool SAFE = decltype(safe_tag)::value;
    using Probs = typename PV<T, D, NW, QB>::Probs;
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        m_run[qb] = -INFINITY;
        l_run[qb] = 0.f;
#pragma unroll
        for (int db = 0; db < C::ODB; ++db) o[qb][db] = floatx16{0};
    }
    // Software pipeline over key tiles, three stages deep.  Step t runs, on the matrix cores, P.V of tile
    // t-1 (first half) and the S^T product of tile t+1 (second half), and on the vector ALU the
    // exponentials of tile t: the three work on different tiles, so nothing inside a step waits for
    // anything else inside it.  K tile t+2 is requested in the first half of step t and first read in the
    // second half of step t+1; V tile t+1 is requested in the second half of step t and first read at the
    // start of step t+2: every tile has a whole step to arrive.  Two barriers per step (middle and end),
    // each preceded by a wait that leaves this wave's two most recent tile requests outstanding.
    if constexpr (SAFE) request_first_tiles();                  // the first pass requested them before the query rows
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    floatx16 sa[QB][2], sb[QB][2];
    Probs pa, pb;
    qk_block<T, D, NW, QB>(Kb0, 0, i, h, sw, qf, sa);       // tile 0 is visible to every row
    qk_block<T, D, NW, QB>(Kb0, 1, i, h, sw, qf, sa);
    __syncthreads();                                         // step 0 overwrites K tile 0

    // wait until at most `pending` of this wave's tile requests (NLD loads each) are outstanding, and for its LDS reads
    auto wait_tiles = [&](int pending) {
        if (pending >= 2) __builtin_amdgcn_s_waitcnt(0x0070 | ((2 * C::NLD) & 15) | (((2 * C::NLD) >> 4) << 14));
        else __builtin_amdgcn_s_waitcnt(0x0070);
    };
    // bf16, one query block per wave: the two halves of a steady-state step with the instruction order written
    // out.  Every matrix instruction is followed by its share of the half's vector work (16 pieces: two
    // products, two exponentials, a pack and a row-sum update per pair of keys) and preceded by the LDS reads
    // of the operand kSchedAhead matrix instructions ahead; nothing moves across the fences between them.
    // HALF 0: P.V of the previous tile (src = its V tile), exponentials of key block 0, requests for a K tile.
    // HALF 1: S^T of the next tile (src = its K tile), exponentials of key block 1, requests for a V tile.
    constexpr bool kExplicit = Elem<T>::kBytes == 2 && QB == 1;
    auto steady_half = [&](auto half_tag, const char* src, floatx16 (&sc)[QB][2], floatx16 (&sn)[QB][2], Probs& pp, Probs& pc,
                           float (&sum)[QB], const char* gt, unsigned lt) {
        if constexpr (kExplicit) {
        constexpr int HALF = decltype(half_tag)::value;
        constexpr int NM = HALF == 0 ? 4 * C::ODB : 2 * C::CH;     // matrix instructions of the half
        constexpr int PPM = 16 / NM;                                // vector pieces per matrix instruction
        typedef short shortx4 __attribute__((ext_vector_type(4)));
        using lds_ptr = __attribute__((address_space(3))) shortx4*;
        uintx4 frag[NM];
        float pe[16];
        auto read = [&](int j) {
            if constexpr (HALF == 0) {
                const int hf = j / (2 * C::ODB), s2 = (j / C::ODB) & 1, db = j % C::ODB;
                const char* a0 = src + vlane[db] + (32 * hf + 16 * s2) * C::VRB;
                const uintx2 lo = __builtin_bit_cast(uintx2, __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)a0));
                const uintx2 hi = __builtin_bit_cast(uintx2, __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(a0 + 8 * C::VRB)));
                frag[j] = uintx4{lo[0], lo[1], hi[0], hi[1]};
            } else {
                const int blk = j & 1, cc = j >> 1;
                frag[j] = *reinterpret_cast<const uintx4*>(src + (blk * 32 + i) * C::KRB + swz_chunk(2 * cc + h, sw));
            }
        };
        auto piece = [&](int q) {                                   // q = 0..15: half a pair of keys
            const int r = 2 * (q >> 1);
            if ((q & 1) == 0) {
                pe[r] = sc[0][HALF][r] * c;
                pe[r + 1] = sc[0][HALF][r + 1] * c;
                pe[r] = fast_exp2(pe[r]);
            } else {
                pe[r + 1] = fast_exp2(pe[r + 1]);
#pragma unroll
                for (int L = 0; L < C::NLD; ++L)
                    if (q == ((2 * L + 1) * 16) / (2 * C::NLD) + 1) {          // request L rides on this piece
                        unsigned pin = __float_as_uint(pe[r + 1]);
                        if constexpr (HALF == 0) tile_load_pinned<C::KRB, NW, C::NLD>(gt, L, koff, lt + L * NW * 1024, pin);
                        else tile_load_pinned<C::VRB, NW, C::NLD>(gt, L, voff, lt + L * NW * 1024, pin);
                        pe[r + 1] = __uint_as_float(pin);
                    }
                const uint32_t pk = pack_bf16x2(pe[r], pe[r + 1]);
                pc[0][HALF][r >> 3][(r & 7) >> 1] = pk;
                sum[0] = add_bf16x2(pk, sum[0]);
            }
        };
#pragma unroll
        for (int j = 0; j < kSchedAhead; ++j) read(j);
#pragma unroll
        for (int j = 0; j < NM; ++j) {
            if (j + kSchedAhead < NM) read(j + kSchedAhead);
            if constexpr (HALF == 0) {
                const int hf = j / (2 * C::ODB), s2 = (j / C::ODB) & 1, db = j % C::ODB;
                o[0][db] = mma_frag<__bf16>(frag[j], pp[0][hf][s2], o[0][db]);
            } else {
                const int blk = j & 1, cc = j >> 1;
                sn[0][blk] = mma_frag<__bf16>(frag[j], qf[0][cc], cc == 0 ? floatx16{0} : sn[0][blk]);
            }
#pragma unroll
            for (int q = 0; q < PPM; ++q) piece(j * PPM + q);
            __builtin_amdgcn_sched_barrier(0);
        }
        }
    };
    auto step = [&](int t, floatx16 (&sc)[QB][2], floatx16 (&sn)[QB][2], Probs& pp, Probs& pc) {
        // requests of this step: K tile t+2 into the buffer tile t has left (first half), V tile t+1 into the
        // one tile t-1 leaves at the middle barrier (second half).  In the steady state they are issued one
        // at a time, each tied to one exponential (a burst of them stalls every wave of the workgroup at the
        // address unit); elsewhere in one go.  Past the last tile the last tile is fetched again, unread.
        const char* kgt = kg + (int64_t)min(t + 2, ntiles - 1) * C::TILE_BYTES;
        const char* vgt = vg + (int64_t)min(t + 1, ntiles - 1) * C::TILE_BYTES;
        const unsigned kl = klds + (t & 1) * C::TILE_BYTES, vl = vlds + ((t + 1) & 1) * C::TILE_BYTES;
        auto fetch_k = [&]() {
#pragma unroll
            for (int q = 0; q < C::NLD; ++q) tile_load<C::KRB, NW, C::NLD>(kgt, q, koff, kl + q * NW * 1024);
        };
        auto fetch_v = [&]() {
#pragma unroll
            for (int q = 0; q < C::NLD; ++q) tile_load<C::VRB, NW, C::NLD>(vgt, q, voff, vl + q * NW * 1024);
        };
        // load L of a half rides on exponential (2L+1) * 16 / (2 NLD) of that half's key block
        auto fetch_after_exp = [&](int blk, int r, float& pinned) {
#pragma unroll
            for (int L = 0; L < C::NLD; ++L)
                if (r == ((2 * L + 1) * 16) / (2 * C::NLD)) {
                    unsigned pin = __float_as_uint(pinned);
                    if (blk == 0) tile_load_pinned<C::KRB, NW, C::NLD>(kgt, L, koff, kl + L * NW * 1024, pin);
                    else tile_load_pinned<C::VRB, NW, C::NLD>(vgt, L, voff, vl + L * NW * 1024, pin);
                    pinned = __uint_as_float(pin);
                }
        };
        const bool has_pv = t >= 1 && t - 1 < my_tiles, has_s = t < my_tiles, has_next = t + 1 < my_tiles;
        const char* kb = Kb0 + ((t + 1) & 1) * C::TILE_BYTES;
        const char* vb = Vb0 + ((t + 1) & 1) * C::TILE_BYTES;          // V tile t-1
        if (C::VROWS && v_in_place && t >= 1 && t * kBN > kk) {
            // A V tile read in place from the evicted cache may hold anything in its rows past k; their
            // probabilities are exact zeros, but 0 * NaN is not: clear those rows in LDS (last tile only).
            char* vt = Vb0 + ((t + 1) & 1) * C::TILE_BYTES;
            const uintx4 z = {0, 0, 0, 0};
            for (int q = tid + (kk - (t - 1) * kBN) * (C::VRB / 16); q < kBN * (C::VRB / 16); q += kNT) store16(vt + q * 16, z);
            __syncthreads();
        }
        float mc[QB], sum[QB];
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) { mc[qb] = 0.f; sum[qb] = 0.f; }
        if (has_s && t * kBN + kBN - 1 > wave_first_row) {       // tile touches the diagonal (wave-uniform)
#pragma unroll
            for (int qb = 0; qb < QB; ++qb)
#pragma unroll
                for (int blk = 0; blk < 2; ++blk)
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        if (t * kBN + 32 * blk + acc_row(r, h) > qrow[qb]) sc[qb][blk][r] = -INFINITY;
        }
        // Probabilities of this tile.  bf16: packed once into P^T operand fragments, and the row sums are
        // taken over the values as rounded to bf16, so that numerator and denominator of the output use
        // the same weights.  fp32: in place.
        auto exps = [&](int blk, bool spread_loads) {
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) {
                if constexpr (Elem<T>::kBytes == 2) {
#pragma unroll
                    for (int r = 0; r < 16; r += 2) {
                        float p0 = fast_exp2(SAFE ? fmaf(sc[qb][blk][r], c, -mc[qb]) : sc[qb][blk][r] * c);
                        float p1 = fast_exp2(SAFE ? fmaf(sc[qb][blk][r + 1], c, -mc[qb]) : sc[qb][blk][r + 1] * c);
                        if (spread_loads && qb == 0) { fetch_after_exp(blk, r, p0); fetch_after_exp(blk, r + 1, p1); }
                        const uint32_t pk = pack_bf16x2(p0, p1);
                        pc[qb][blk][r >> 3][(r & 7) >> 1] = pk;
                        sum[qb] = add_bf16x2(pk, sum[qb]);
                    }
                } else {
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        float p = fast_exp2(SAFE ? fmaf(sc[qb][blk][r], c, -mc[qb]) : sc[qb][blk][r] * c);
                        if (spread_loads && qb == 0) fetch_after_exp(blk, r, p);
                        pc[qb][blk][r] = p;
                        sum[qb] += p;
                    }
                }
            }
        };
        const bool steady = has_pv && has_next && !SAFE;
        // ---- first half: P.V of tile t-1 | exponentials of key block 0 of tile t | requests for K tile t+2
        if (steady) {
            if constexpr (kExplicit) steady_half(std::integral_constant<int, 0>{}, vb, sc, sn, pp, pc, sum, kgt, kl);
            else {
                exps(0, true);
                PV<T, D, NW, QB>::template run<0>(vb, vlane, pp, o);
                PV<T, D, NW, QB>::template run<1>(vb, vlane, pp, o);
            }
        } else {
            fetch_k();
            if (has_pv) {
                PV<T, D, NW, QB>::template run<0>(vb, vlane, pp, o);
                PV<T, D, NW, QB>::template run<1>(vb, vlane, pp, o);
            }
            if (has_s) {
                if constexpr (SAFE) {
                    // raw-logit maxima; the softmax scale (c > 0, log2 domain) is folded into the exponent.  The
                    // offset follows the maximum lazily: it moves only when a logit exceeds it by more than
                    // kLazyLog2 in the log2 domain, so probabilities stay below 2^kLazyLog2 and the accumulators
                    // (which hold every tile up to t-1 by now) are rescaled rarely.  The first tile always moves
                    // it (offset -inf; key 0 is visible to every row, so the maximum is finite).
                    const float lazy = kLazyLog2 / c;
                    float m_new[QB];
                    bool moved = false;
#pragma unroll
                    for (int qb = 0; qb < QB; ++qb) {
                        float mx = -INFINITY;
#pragma unroll
                        for (int blk = 0; blk < 2; ++blk)
#pragma unroll
                            for (int r = 0; r < 16; ++r) mx = fmaxf(mx, sc[qb][blk][r]);
                        mx = xhalf_max(mx);
                        const bool grow = mx > m_run[qb] + lazy;
                        m_new[qb] = grow ? mx : m_run[qb];
                        mc[qb] = m_new[qb] * c;
                        moved |= grow;
                    }
                    if (__any(moved)) {
#pragma unroll
                        for (int qb = 0; qb < QB; ++qb) {
                            const float alpha = fast_exp2(m_run[qb] * c - mc[qb]);   // 1 where the maximum stayed
                            l_run[qb] *= alpha;
#pragma unroll
                            for (int db = 0; db < C::ODB; ++db)
#pragma unroll
                                for (int r = 0; r < 16; ++r) o[qb][db][r] *= alpha;
                            m_run[qb] = m_new[qb];
                        }
                    }
                }
                exps(0, false);
            }
        }
        wait_tiles(2);                                        // K tile t+1 has landed (this wave's part)
        __syncthreads();
        // ---- second half: S^T of tile t+1 | exponentials of key block 1 of tile t | requests for V tile t+1
        if (steady) {
            if constexpr (kExplicit) steady_half(std::integral_constant<int, 1>{}, kb, sc, sn, pp, pc, sum, vgt, vl);
            else {
                exps(1, true);
                qk_block<T, D, NW, QB>(kb, 0, i, h, sw, qf, sn);
                qk_block<T, D, NW, QB>(kb, 1, i, h, sw, qf, sn);
            }
        } else {
            fetch_v();
            if (has_next) {
                qk_block<T, D, NW, QB>(kb, 0, i, h, sw, qf, sn);
                qk_block<T, D, NW, QB>(kb, 1, i, h, sw, qf, sn);
            }
            if (has_s) exps(1, false);
        }
        if (has_s) {
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) l_run[qb] += sum[qb];
        }
        wait_tiles(2);                                        // V tile t has landed (this wave's part)
        __syncthreads();
    };
    // steps 0 .. ntiles: the last one only finishes P.V of the last tile
    for (int t = 0; t <= ntiles; t += 2) {
        step(t, sa, sb, pb, pa);
        if (t + 1 <= ntiles) step(t + 1, sb, sa, pa, pb);
    }
    __builtin_amdgcn_s_waitcnt(0);
    };
    pass(std::false_type{});
    // Output rows.  Everything the stores need is derived again from the thread index here (the empty asm
    // keeps the compiler from carrying row numbers and pointers through the key loop, where registers are
    // scarce); the positions are requested now and arrive during the check below.
    int tid_out = threadIdx.x;
    asm volatile("" : "+v"(tid_out));
    const int w_out = tid_out >> 6, i_out = tid_out & 31, h_out = (tid_out >> 5) & 1;
    int qr_out[QB], orow_out[QB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        qr_out[qb] = i0 + kRW * w_out + 32 * qb + i_out;
        orow_out[qb] = (out_compact || !tidx) ? qr_out[qb] : tidx[min(qr_out[qb], kk - 1)];
    }
    {
        // the offset-free pass stands if every row sum of the workgroup is finite and far from both ends of the
        // fp32 range (no exponential overflowed, the dominant terms did not underflow); otherwise the whole
        // workgroup repeats its tiles with running maxima
        bool bad = false;
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
            const float l_tot = xhalf_sum(l_run[qb]);
            bad |= qrow[qb] < kk && !(l_tot >= kSumLow && l_tot <= kSumHigh);   // rows past k are never stored
        }
        if (__syncthreads_or(bad)) pass(std::true_type{});
    }

#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        const float l_tot = xhalf_sum(l_run[qb]);
        const int qr = qr_out[qb];
        if (qr < kk) {
            const float inv = 1.f / l_tot;
            const int orow = orow_out[qb];
            T* op = O + ((int64_t)bh * n + orow) * D;
#pragma unroll
            for (int db = 0; db < C::ODB; ++db)
#pragma unroll
                for (int a = 0; a < 4; ++a)
                    store_out4<T>(op + 32 * db + 8 * a + 4 * h_out, o[qb][db][4 * a] * inv, o[qb][db][4 * a + 1] * inv,
                                  o[qb][db][4 * a + 2] * inv, o[qb][db][4 * a + 3] * inv);
        }
    }
}

// ------------------------------------------------------------------ host
size_t prefill_workspace_bytes(const zipvl_dims& d) {
    const int e = d.dtype == ZIPVL_BF16 ? 2 : 4;
    const size_t npad = ((size_t)d.n + kBN - 1) / kBN * kBN;
    return 2 * (size_t)d.B * d.Hkv * npad * d.d * e;
}

template <typename T, int D, int NW, int QB>
static int launch_flash(const void* Q, const void* K, const zipvl_dims& d, const int32_t* idx, const int32_t* k,
                        float scale, int out_compact, int t_per_batch, int skip_k, int skip_v, const void* V, const T* Kp, const T* Vp, int npad, void* O, hipStream_t st)
{
    using C = AttnCfg<T, D, NW, QB>;
    static std::atomic<bool> attr_done{false};       // raising the dynamic-LDS cap is idempotent
    if (!attr_done) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(&flash_kept_kernel<T, D, NW, QB>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, C::LDS_BYTES) != hipSuccess)
            return set_error(ZIPVL_EHIP, "sparse_prefill: cannot reserve %d bytes of LDS", C::LDS_BYTES);
        attr_done = true;
    }
    {
        KernelTimer tm(ZIPVL_K_FLASH_KEPT, st);
        const int BH = d.B * d.Hq;
        const int ntq = (d.n + C::BM - 1) / C::BM;
        const int64_t blocks = (int64_t)ntq * BH;
        const int G = d.Hq / d.Hkv;
        // KV heads per scheduling group (see the kernel): about eight waves of workgroups on the chip, so
        // that the longest workgroup (the last query tile) is a small part of a group even when only a
        // fraction of the tiles is kept, but no more K / V than a quarter of the 256 MiB last-level cache
        const int64_t unit_bytes = 2 * (int64_t)npad * D * Elem<T>::kBytes;
        int ug = (int)std::min<int64_t>((16384 / (NW * QB)) / ((int64_t)ntq * G), (64ll << 20) / unit_bytes);
        ug = ug < 1 ? 1 : ug;
        // full-size output of a sparse call: one more workgroup per (head, span of positions) clears dropped rows
        const int64_t fill = (!out_compact && idx) ? (int64_t)BH * ((d.n + kFillSpan - 1) / kFillSpan) : 0;
        if (blocks + fill > 0x7fffffffLL) return set_error(ZIPVL_ESHAPE, "sparse_prefill: %lld workgroups exceed the grid limit", (long long)blocks);
        hipLaunchKernelGGL((flash_kept_kernel<T, D, NW, QB>), dim3((unsigned)(blocks + fill)), dim3(C::NT),
            C::LDS_BYTES, st, (const T*)Q, d.q_strides[0], d.q_strides[1], d.q_strides[2],
            skip_k ? (const T*)K : Kp, skip_k ? d.k_strides[0] : (int64_t)d.Hkv * npad * D,
            skip_k ? d.k_strides[1] : (int64_t)npad * D,
            skip_v ? (const T*)V : Vp, skip_v ? d.v_strides[0] : (int64_t)d.Hkv * npad * D,
            skip_v ? d.v_strides[1] : (int64_t)npad * D, idx, k, (T*)O, d.n, npad, ntq, ug, BH, d.Hq, d.Hkv,
            scale * kLog2e, out_compact, (int)blocks, t_per_batch, skip_v);
    }
    return check_launch("flash_kept");
}

template <typename T, int D>
static int launch_prefill_t(const void* Q, const void* K, const void* V, const zipvl_dims& d,
                            const int32_t* idx, const int32_t* k, float scale, int flags,
                            void* O, void* ws, hipStream_t st)
{
    const int npad = (d.n + kBN - 1) / kBN * kBN;
    const int units = d.B * d.Hkv;
    T* Kp = (T*)ws;
    T* VTp = Kp + (size_t)units * npad * D;
    const int out_compact = (flags & ZIPVL_OUT_COMPACT) ? 1 : 0;
    const int rows_are_kept = (flags & ZIPVL_KV_ALREADY_COMPACT) ? 1 : 0;
    const int t_per_batch = (flags & ZIPVL_T_PER_BATCH) ? 1 : 0;

    // An evicted cache with contiguous rows and whole 64-row tiles is read in place (K always, V when the
    // transposing LDS read applies: then nothing is packed).  Rows between k and the end of the last tile
    // may hold anything: K rows there are masked, V rows there are cleared once they are in LDS.
    const int in_place = (rows_are_kept && d.n % kBN == 0) ? 1 : 0;
    const int skip_k = (in_place && d.k_strides[2] == D) ? 1 : 0;
    const int skip_v = (in_place && Elem<T>::kBytes == 2 && d.v_strides[2] == D) ? 1 : 0;
    if (!(skip_k && skip_v)) {
        KernelTimer tm(ZIPVL_K_PACK_KV, st);
        hipLaunchKernelGGL((pack_kv_kernel<T, D>), dim3(npad / kBN, units), dim3(256), 0, st,
            (const T*)K, (const T*)V, d.k_strides[0], d.k_strides[1], d.k_strides[2],
            d.v_strides[0], d.v_strides[1], d.v_strides[2], idx, k, Kp, VTp, d.n, npad, d.Hkv, rows_are_kept, skip_k, t_per_batch);
        int rc = check_launch("pack_kv");
        if (rc) return rc;
    }

    if constexpr (Elem<T>::kBytes == 2)
        return launch_flash<T, D, kFlashWavesBf16, kFlashBlocksBf16>(Q, K, d, idx, k, scale, out_compact, t_per_batch, skip_k, skip_v, V, Kp, VTp, npad, O, st);
    else
        return launch_flash<T, D, 4, 1>(Q, K, d, idx, k, scale, out_compact, t_per_batch, skip_k, skip_v, V, Kp, VTp, npad, O, st);
}

int launch_sparse_prefill(const void* Q, const void* K, const void* V, const zipvl_dims& d,
                          const int32_t* idx, const int32_t* k, float scale, int flags,
                          void* O, void* ws, hipStream_t st)
{
    if (d.dtype == ZIPVL_BF16) {
        if (d.d == 128) return launch_prefill_t<__bf16, 128>(Q, K, V, d, idx, k, scale, flags, O, ws, st);
        return launch_prefill_t<__bf16, 64>(Q, K, V, d, idx, k, scale, flags, O, ws, st);
    }
    if (d.d == 128) return launch_prefill_t<float, 128>(Q, K, V, d, idx, k, scale, flags, O, ws, st);
    return launch_prefill_t<float, 64>(Q, K, V, d, idx, k, scale, flags, O, ws, st);
}

}  // namespace zipvl
