// Attention over the kept tokens (Section 4.2; Algorithm 1, sparse-attention
// step; Eq. (2) restricted to the important set T).
//
// Two kernels:
//   pack   gathers K[T] row-major and V[T] transposed ([d][64 keys] tiles) into
//          the workspace, once per KV head, zero-filling the ragged tail.  The
//          transposed V is what lets the P.V product read both MFMA operands
//          as contiguous fragments (the contraction runs over keys).
//   flash  one workgroup = 128 kept queries of one query head (4 waves x 32
//          rows).  K / V^T tiles of 64 keys are loaded straight into LDS
//          (double buffered, one barrier per tile) and shared by the four waves;
//          the S^T product of the next tile overlaps the softmax of the current.
//          S^T = K Q^T and O^T = V^T P^T are taken on 32x32 MFMA tiles, so a
//          lane owns one query column: the online-softmax statistics are
//          per-lane scalars and only the running maximum crosses lanes (one
//          exchange between the two half-waves per tile).  Causality is the
//          plain lower triangle in kept-token coordinates because T is
//          ascending.  Query rows are gathered by idx on load, output rows are
//          scattered by idx on store, and the rows of dropped tokens between a
//          workgroup's kept rows are cleared by that workgroup (no separate fill).
// The kept count k lives on the device: the grid covers the worst case (k = n)
// and workgroups beyond a unit's k exit at once; heavy (late) query tiles are
// scheduled first.
#include "launch.h"

namespace zipvl {

constexpr int kBN = 64;      // keys per tile
constexpr int kFlashWavesBf16 = 4;   // 8 (one workgroup per CU) halves the L2 -> LDS traffic but measured no faster
constexpr int kSchedAhead = 3;       // LDS operand reads in flight ahead of the consuming MFMA
constexpr int kSchedValu = 4;        // vector instructions placed between two MFMAs

// NW = waves per workgroup; a wave owns 32 queries, so a workgroup covers 32 NW kept queries and its
// K / V^T tiles are fetched from L2 once per 32 NW queries.
template <typename T, int D, int NW = 4>
struct AttnCfg {
    static constexpr int E = Elem<T>::kBytes;
    static constexpr int BM = 32 * NW;                       // queries per workgroup
    static constexpr int NT = 64 * NW;                       // threads per workgroup
    static constexpr int CH = D / Elem<T>::kPerChunk;       // Q/K fragments per row per lane
    static constexpr int ODB = D / 32;                       // 32-row blocks of O^T
    // LDS tiles are unpadded; the 16-byte chunks of a row are XOR-swizzled with (row & 7) instead, so
    // that any 8 consecutive rows read at the same logical chunk hit 8 different bank groups.
    static constexpr int KRB = D * E;                        // bytes per K row
    static constexpr int VRB = kBN * E;                      // bytes per V^T row
    static constexpr int TILE_BYTES = kBN * D * E;           // one K tile = one V^T tile
    static constexpr int NLD = TILE_BYTES / 1024 / NW;       // 1-KiB direct-to-LDS loads per wave per tile
    static constexpr int LDS_BYTES = 4 * TILE_BYTES;         // two K and two V^T buffers
    static constexpr int NVF = (E == 2 ? 2 : 4) * ODB;       // V^T operand fragments per 32 keys per lane
    static constexpr int MIN_WGS = (E == 2) ? 8 / NW : 1;    // bf16: two waves per SIMD (<= 256 registers, accumulators stay in VGPRs)
};

// ------------------------------------------------------------------ pack
// Key held at element e of 16-byte chunk kc of a V^T tile row.  fp32: natural order.  bf16: inside
// every group of 16 keys the order is [0..3, 8..11 | 4..7, 12..15], which is the order in which the
// two half-waves hold the 8 contraction slots of one P^T fragment, so that a lane's V^T operand is
// one contiguous 16-byte read.
template <typename T> __device__ __forceinline__ int vt_key(int kc, int e);
template <> __device__ __forceinline__ int vt_key<float>(int kc, int e) { return kc * 4 + e; }
template <> __device__ __forceinline__ int vt_key<__bf16>(int kc, int e) {
    return 16 * (kc >> 1) + 8 * (e >> 2) + 4 * (kc & 1) + (e & 3);
}

template <typename T, int D>
__global__ __launch_bounds__(256) void pack_kv_kernel(
    const T* __restrict__ K, const T* __restrict__ V,
    int64_t ks0, int64_t ks1, int64_t ks2, int64_t vs0, int64_t vs1, int64_t vs2,
    const int32_t* __restrict__ idx, const int32_t* __restrict__ kcnt,
    T* __restrict__ Kp, T* __restrict__ VTp, int n, int npad, int Hkv, int rows_are_kept, int skip_k)
{
    constexpr int EPF = Elem<T>::kPerFrag;
    constexpr int CPR = D / EPF;
    constexpr int LS = D + EPF;                 // padded LDS row (elements)
    __shared__ __attribute__((aligned(16))) T tile[kBN * LS];
    const int u = blockIdx.y, b = u / Hkv, g = u - b * Hkv;
    const int t0 = blockIdx.x * kBN;
    int kk = kcnt ? kcnt[u] : n;
    kk = max(0, min(kk, n));
    if (t0 >= kk) return;
    const T* Kb = K + b * ks0 + g * ks1;
    const T* Vb = V + b * vs0 + g * vs1;
    for (int wi = threadIdx.x; wi < kBN * CPR; wi += 256) {
        const int r = wi / CPR, cc = wi - r * CPR, row = t0 + r;
        uintx4 kv = {0, 0, 0, 0}, vv = {0, 0, 0, 0};
        if (row < kk) {
            const int src = (idx && !rows_are_kept) ? idx[(int64_t)u * n + row] : row;
            if (!skip_k) kv = load16(Kb + (int64_t)src * ks2 + cc * EPF);
            vv = load16(Vb + (int64_t)src * vs2 + cc * EPF);
        }
        if (!skip_k) store16(Kp + ((int64_t)u * npad + row) * D + cc * EPF, kv);
        store16(tile + r * LS + cc * EPF, vv);
    }
    __syncthreads();
    T* VT = VTp + ((int64_t)u * (npad / kBN) + blockIdx.x) * (D * kBN);
    for (int wi = threadIdx.x; wi < D * (kBN / EPF); wi += 256) {
        const int dd = wi % D, kc = wi / D;
        T v[EPF];
#pragma unroll
        for (int e = 0; e < EPF; ++e) v[e] = tile[vt_key<T>(kc, e) * LS + dd];
        store16(VT + dd * kBN + kc * EPF, *reinterpret_cast<const uintx4*>(v));
    }
}

// ------------------------------------------------------------------ flash
// byte offset of logical 16-byte chunk `c` in a swizzled LDS row (sw = row & 7)
__device__ __forceinline__ int swz_chunk(int c, int sw) { return (c ^ sw) << 4; }

// One tile (TILE_BYTES contiguous in global memory) -> one LDS buffer, without passing through
// registers: every wave issues NLD loads of 1 KiB, lane L of a load writes LDS bytes [16 L, 16 L + 16)
// of that KiB, and picks the global chunk that belongs there under the row swizzle.
// One 1-KiB direct-to-LDS load of the wave: lane L's 16 bytes at gsrc land at LDS byte lds_base + 16 L.
// global_load_lds_dwordx4 takes the LDS base from M0.  The instruction is written out rather than
// taken from the builtin because the compiler, while such a load is pending, turns every LDS-read
// wait into a wait for ALL outstanding LDS reads, which stalls the matrix pipeline on each operand
// fetch; completion is awaited explicitly (vmcnt) at the end of every pipeline step instead.
__device__ __forceinline__ void load_kib_to_lds(const char* gsrc, unsigned lds_base) {
    const unsigned m0v = __builtin_amdgcn_readfirstlane(lds_base);
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"
                 :: "s"(m0v), "v"(gsrc) : "memory", "m0");
}

__device__ __forceinline__ unsigned lds_address(const char* p) {
    return (unsigned)(uintptr_t)(const __attribute__((address_space(3))) char*)p;
}

template <int NW, int NLD>
__device__ __forceinline__ void tile_to_lds(const char* gtile, char* lbuf, int w, const int (&off)[NLD]) {
    const unsigned lbase = lds_address(lbuf);
#pragma unroll
    for (int q = 0; q < NLD; ++q) load_kib_to_lds(gtile + off[q], lbase + (q * NW + w) * 1024);
}

// per-lane source offsets for tile_to_lds (rows of RB bytes)
template <int RB, int NW, int NLD>
__device__ __forceinline__ void lds_fill_offsets(int w, int lane, int (&off)[NLD]) {
#pragma unroll
    for (int q = 0; q < NLD; ++q) {
        const int o = (q * NW + w) * 1024 + lane * 16;
        const int r = o / RB, p = (o % RB) >> 4;
        off[q] = r * RB + ((p ^ (r & 7)) << 4);
    }
}

// S^T = K Q^T for 32 keys (block blk of the 64-key tile in LDS buffer kb): acc[r] = key 32*blk + acc_row(r, h), this lane's query
template <typename T, int D, int NW>
__device__ __forceinline__ void qk_block(const char* kb, int blk, int i, int h, int sw,
                                         const uintx4 (&qf)[AttnCfg<T, D, NW>::CH], floatx16& acc) {
    using C = AttnCfg<T, D, NW>;
    floatx16 a = {0};
#pragma unroll
    for (int cc = 0; cc < C::CH; ++cc) {
        const uintx4 kf = *reinterpret_cast<const uintx4*>(kb + (blk * 32 + i) * C::KRB + swz_chunk(2 * cc + h, sw));
        a = mma_frag<T>(kf, qf[cc], a);
    }
    acc = a;
}

// O^T += V^T P^T for the 32 keys of half HALF: p[16] holds the probabilities of S^T block HALF.
template <typename T, int D, int NW> struct PV;

template <int D, int NW> struct PV<__bf16, D, NW> {
    using C = AttnCfg<__bf16, D, NW>;
    template <int HALF>
    __device__ static __forceinline__ void run(const char* vb, int i, int h, int sw, const floatx16& p, floatx16 (&o)[C::ODB]) {
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) {
            // contraction slot t of this lane <-> key 16*s2 + 8*(t/4) + 4*h + t%4 of the half = register 8*s2 + t;
            // V^T rows are stored in slot order, so the matching operand is one 16-byte chunk
            uintx4 bfrag;
            bfrag[0] = pack_bf16x2(p[8 * s2 + 0], p[8 * s2 + 1]);
            bfrag[1] = pack_bf16x2(p[8 * s2 + 2], p[8 * s2 + 3]);
            bfrag[2] = pack_bf16x2(p[8 * s2 + 4], p[8 * s2 + 5]);
            bfrag[3] = pack_bf16x2(p[8 * s2 + 6], p[8 * s2 + 7]);
            const int chunk = swz_chunk(2 * (2 * HALF + s2) + h, sw);
#pragma unroll
            for (int db = 0; db < C::ODB; ++db) {
                const uintx4 vf = *reinterpret_cast<const uintx4*>(vb + (db * 32 + i) * C::VRB + chunk);
                o[db] = mma_frag<__bf16>(vf, bfrag, o[db]);
            }
        }
    }
};

template <int D, int NW> struct PV<float, D, NW> {
    using C = AttnCfg<float, D, NW>;
    template <int HALF>
    __device__ static __forceinline__ void run(const char* vb, int i, int h, int sw, const floatx16& p, floatx16 (&o)[C::ODB]) {
#pragma unroll
        for (int a = 0; a < 4; ++a) {
            // step (a, t): this lane contributes key 32*HALF + 8*a + 4*h + t
            const int chunk = swz_chunk(8 * HALF + 2 * a + h, sw);
#pragma unroll
            for (int db = 0; db < C::ODB; ++db) {
                const floatx4 v = *reinterpret_cast<const floatx4*>(vb + (db * 32 + i) * C::VRB + chunk);
#pragma unroll
                for (int t = 0; t < 4; ++t)
                    o[db] = __builtin_amdgcn_mfma_f32_32x32x2f32(v[t], p[4 * a + t], o[db], 0, 0, 0);
            }
        }
    }
};

// Instruction order of the steady-state step (one basic block: S^T of the next tile, exponentials and
// P.V of the current one): LDS operand reads run a few fragments ahead of the matrix instruction that
// consumes them and the vector work is spread evenly between the matrix instructions, so that a wave
// neither waits on LDS latency in front of every MFMA nor bunches its vector work.
template <typename T, int D>
__device__ __forceinline__ void flash_schedule() {
    if constexpr (Elem<T>::kBytes == 2 && D == 128) {
#pragma unroll
        for (int q = 0; q < kSchedAhead; ++q) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   // LDS read
#pragma unroll
        for (int q = 0; q < 32; ++q) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                        // MFMA
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);                        // LDS read
            __builtin_amdgcn_sched_group_barrier(0x002, kSchedValu, 0);         // vector ALU
        }
    }
}

// rows [lo, hi) of head bh of O := 0, spread over `nthreads` threads (16-byte stores)
template <typename T, int D>
__device__ __forceinline__ void zero_rows(T* O, int bh, int n, int lo, int hi, int tid, int nthreads) {
    constexpr int CPR = D * Elem<T>::kBytes / 16;
    const uintx4 z = {0, 0, 0, 0};
    char* base = reinterpret_cast<char*>(O + ((int64_t)bh * n + lo) * D);
    const int64_t chunks = (int64_t)(hi - lo) * CPR;
    for (int64_t q = tid; q < chunks; q += nthreads) store16(base + q * 16, z);
}

template <typename T> __device__ __forceinline__ void store_out4(T* dst, float a, float b, float c, float d);
template <> __device__ __forceinline__ void store_out4<float>(float* dst, float a, float b, float c, float d) {
    *reinterpret_cast<floatx4*>(dst) = floatx4{a, b, c, d};
}
template <> __device__ __forceinline__ void store_out4<__bf16>(__bf16* dst, float a, float b, float c, float d) {
    *reinterpret_cast<uintx2*>(dst) = uintx2{pack_bf16x2(a, b), pack_bf16x2(c, d)};
}

template <typename T, int D, int NW>
__global__ __launch_bounds__(64 * NW, (AttnCfg<T, D, NW>::MIN_WGS)) void flash_kept_kernel(
    const T* __restrict__ Q, int64_t qs0, int64_t qs1, int64_t qs2,
    const T* __restrict__ Kp, int64_t kp0, int64_t kp1, const T* __restrict__ VTp,
    const int32_t* __restrict__ idx, const int32_t* __restrict__ kcnt,
    T* __restrict__ O, int n, int npad, int ntq, int ug, int BH, int Hq, int Hkv, float c, int out_compact, int zero_dropped)
{
    using C = AttnCfg<T, D, NW>;
    constexpr int kBM = C::BM, kNT = C::NT;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    // Workgroup -> (unit group, query tile, unit in group, head of the KV group), in that order of
    // significance; heavy (late) query tiles first inside a group.  A group holds just enough KV heads
    // to fill the chip a few times over (one for long GQA sequences, many for short MHA ones): the
    // chip then works through few KV heads at a time, so every XCD's L2 (workgroups are dealt
    // round-robin to the 8 XCDs) holds little more than the K / V^T it is using, while the light tail
    // of one group overlaps the heavy start of the next.
    const int G = Hq / Hkv, NU = BH / G;
    const int full = ug * ntq * G;                           // workgroups of a full group
    const int ngroups = (NU + ug - 1) / ug;
    const int grp = min((int)(blockIdx.x / full), ngroups - 1);
    const int r = blockIdx.x - grp * full;
    const int nu_g = min(ug, NU - grp * ug);
    const int tile_rev = r / (nu_g * G), rr = r - tile_rev * (nu_g * G);
    const int u = grp * ug + rr / G, hg = rr % G;
    const int b = u / Hkv, g = u - b * Hkv, head = g * G + hg, bh = b * Hq + head;
    const int i0 = (ntq - 1 - tile_rev) * kBM;
    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, i = lane & 31, h = lane >> 5;
    int kk = kcnt ? kcnt[u] : n;
    kk = max(0, min(kk, n));
    if (i0 >= kk) {
        if (zero_dropped && i0 == 0) zero_rows<T, D>(O, bh, n, 0, n, tid, kNT);   // nothing kept at all
        return;
    }
    if (zero_dropped) {
        // Outputs of dropped tokens are zero rows.  This workgroup clears the dropped positions that
        // lie before each of its kept rows; the tile holding the last kept row also clears the tail.
        int* tpos = reinterpret_cast<int*>(smem);            // [kBM + 1], dead before the first tile is staged
        if (tid <= kBM) {
            const int r = i0 - 1 + tid;                      // entry e: position of kept row i0 - 1 + e
            tpos[tid] = r < 0 ? -1 : (r < kk ? idx[(int64_t)u * n + r] : n);
        }
        __syncthreads();
        if (i0 + kBM == kk) zero_rows<T, D>(O, bh, n, tpos[kBM] + 1, n, tid, kNT);   // tail after a full last tile
#pragma unroll
        for (int half = 0; half < kBM / 64; ++half) {
            const int gi = half * 64 + lane;
            unsigned long long open = __ballot(tpos[gi + 1] - tpos[gi] > 1);
            while (open) {                                   // wave-uniform walk over the non-empty gaps
                const int gsel = half * 64 + __builtin_ctzll(open);
                open &= open - 1;
                zero_rows<T, D>(O, bh, n, tpos[gsel] + 1, tpos[gsel + 1], tid, kNT);
            }
        }
        __syncthreads();                                     // tpos is overwritten by the first K tile
    }
    const int qrow = i0 + 32 * w + i;                        // kept-token coordinate of this lane's query
    const int qclamp = min(qrow, kk - 1);
    const int qpos = idx ? idx[(int64_t)u * n + qclamp] : qclamp;

    uintx4 qf[C::CH];
    {
        const T* qp = Q + b * qs0 + head * qs1 + (int64_t)qpos * qs2;
#pragma unroll
        for (int cc = 0; cc < C::CH; ++cc) qf[cc] = load16(qp + cc * Elem<T>::kPerChunk + h * Elem<T>::kPerFrag);
    }
    floatx16 o[C::ODB];
#pragma unroll
    for (int db = 0; db < C::ODB; ++db) o[db] = floatx16{0};
    float m_run = -INFINITY, l_run = 0.f;

    const int ntiles = (min(i0 + kBM, kk) + kBN - 1) / kBN;
    const int wave_first_row = i0 + 32 * w, wave_last_row = wave_first_row + 31;
    const int my_tiles = min(ntiles, wave_last_row / kBN + 1);   // later tiles lie wholly in this wave's future
    const char* kg = reinterpret_cast<const char*>(Kp + b * kp0 + g * kp1);   // row-major kept K rows of this unit
    const char* vg = reinterpret_cast<const char*>(VTp + (int64_t)u * npad * D);
    char* const Kb0 = smem;
    char* const Vb0 = smem + 2 * C::TILE_BYTES;
    const int sw = i & 7;
    int koff[C::NLD], voff[C::NLD];
    lds_fill_offsets<C::KRB, NW, C::NLD>(w, lane, koff);
    lds_fill_offsets<C::VRB, NW, C::NLD>(w, lane, voff);

    // Software pipeline over key tiles.  While tile t is in its softmax (vector ALU) and P.V (matrix)
    // stages, the S^T product of tile t+1 already runs on the matrix cores and the loads of K tile t+2
    // and V^T tile t+1 are in flight straight into LDS.  One barrier per tile.
    tile_to_lds<NW, C::NLD>(kg, Kb0, w, koff);
    tile_to_lds<NW, C::NLD>(vg, Vb0, w, voff);
    if (ntiles > 1) tile_to_lds<NW, C::NLD>(kg + C::TILE_BYTES, Kb0 + C::TILE_BYTES, w, koff);
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    floatx16 sa[2], sb[2];
    qk_block<T, D, NW>(Kb0, 0, i, h, sw, qf, sa[0]);        // tile 0 is visible to every row
    qk_block<T, D, NW>(Kb0, 1, i, h, sw, qf, sa[1]);

    auto step = [&](int t, floatx16 (&sc)[2], floatx16 (&sn)[2]) {
        // this step's loads: K tile t+2 into the buffer tile t has left, V^T tile t+1 into the one tile t-1 has left
        if (t + 2 < ntiles) tile_to_lds<NW, C::NLD>(kg + (int64_t)(t + 2) * C::TILE_BYTES, Kb0 + (t & 1) * C::TILE_BYTES, w, koff);
        if (t + 1 < ntiles) tile_to_lds<NW, C::NLD>(vg + (int64_t)(t + 1) * C::TILE_BYTES, Vb0 + ((t + 1) & 1) * C::TILE_BYTES, w, voff);
        if (t < my_tiles) {
            const int t0 = t * kBN;
            const char* kb = Kb0 + ((t + 1) & 1) * C::TILE_BYTES;
            const char* vb = Vb0 + (t & 1) * C::TILE_BYTES;
            if (t0 + kBN - 1 > wave_first_row) {             // tile touches the diagonal (wave-uniform)
#pragma unroll
                for (int blk = 0; blk < 2; ++blk)
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        if (t0 + 32 * blk + acc_row(r, h) > qrow) sc[blk][r] = -INFINITY;
            }
            float mx = -INFINITY;
#pragma unroll
            for (int blk = 0; blk < 2; ++blk)
#pragma unroll
                for (int r = 0; r < 16; ++r) mx = fmaxf(mx, sc[blk][r]);
            mx = fmaxf(mx, __shfl_xor(mx, 32));
            // raw-logit maximum; the softmax scale (c > 0, log2 domain) is folded into the exponent
            const float m_new = fmaxf(m_run, mx);            // finite: key 0 is visible to every row
            const float mc = m_new * c;
            if (__any(m_new != m_run)) {                     // rescale only when some row's maximum moved
                const float alpha = fast_exp2(m_run * c - mc);
                l_run *= alpha;
#pragma unroll
                for (int db = 0; db < C::ODB; ++db)
#pragma unroll
                    for (int r = 0; r < 16; ++r) o[db][r] *= alpha;
                m_run = m_new;
            }
            float sum = 0.f;
            if (t + 1 < my_tiles) {
                // matrix stream: S^T of tile t+1, then P.V of tile t; vector stream: exponentials of tile t
                qk_block<T, D, NW>(kb, 0, i, h, sw, qf, sn[0]);
                qk_block<T, D, NW>(kb, 1, i, h, sw, qf, sn[1]);
#pragma unroll
                for (int r = 0; r < 16; ++r) { sc[0][r] = fast_exp2(fmaf(sc[0][r], c, -mc)); sum += sc[0][r]; }
                PV<T, D, NW>::template run<0>(vb, i, h, sw, sc[0], o);
#pragma unroll
                for (int r = 0; r < 16; ++r) { sc[1][r] = fast_exp2(fmaf(sc[1][r], c, -mc)); sum += sc[1][r]; }
                PV<T, D, NW>::template run<1>(vb, i, h, sw, sc[1], o);
                flash_schedule<T, D>();
            } else {
#pragma unroll
                for (int r = 0; r < 16; ++r) { sc[0][r] = fast_exp2(fmaf(sc[0][r], c, -mc)); sum += sc[0][r]; }
                PV<T, D, NW>::template run<0>(vb, i, h, sw, sc[0], o);
#pragma unroll
                for (int r = 0; r < 16; ++r) { sc[1][r] = fast_exp2(fmaf(sc[1][r], c, -mc)); sum += sc[1][r]; }
                PV<T, D, NW>::template run<1>(vb, i, h, sw, sc[1], o);
            }
            l_run += sum;
        }
        __builtin_amdgcn_s_waitcnt(0);                       // this wave's direct-to-LDS loads have landed
        __syncthreads();
    };
    for (int t = 0; t < ntiles; t += 2) {
        step(t, sa, sb);
        if (t + 1 < ntiles) step(t + 1, sb, sa);
    }

    const float l_tot = l_run + __shfl_xor(l_run, 32);
    if (qrow < kk) {
        const float inv = 1.f / l_tot;
        const int orow = out_compact ? qrow : qpos;
        T* op = O + ((int64_t)bh * n + orow) * D;
#pragma unroll
        for (int db = 0; db < C::ODB; ++db)
#pragma unroll
            for (int a = 0; a < 4; ++a)
                store_out4<T>(op + 32 * db + 8 * a + 4 * h, o[db][4 * a] * inv, o[db][4 * a + 1] * inv,
                              o[db][4 * a + 2] * inv, o[db][4 * a + 3] * inv);
    }
}

// ------------------------------------------------------------------ host
size_t prefill_workspace_bytes(const zipvl_dims& d) {
    const int e = d.dtype == ZIPVL_BF16 ? 2 : 4;
    const size_t npad = ((size_t)d.n + kBN - 1) / kBN * kBN;
    return 2 * (size_t)d.B * d.Hkv * npad * d.d * e;
}

template <typename T, int D, int NW>
static int launch_flash(const void* Q, const void* K, const zipvl_dims& d, const int32_t* idx, const int32_t* k,
                        float scale, int out_compact, int skip_k, const T* Kp, const T* VTp, int npad, void* O, hipStream_t st)
{
    using C = AttnCfg<T, D, NW>;
    static bool attr_done = false;       // raising the dynamic-LDS cap is idempotent
    if (!attr_done) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(&flash_kept_kernel<T, D, NW>),
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
        int ug = (4096 / NW) / (ntq * G);                   // KV heads per scheduling group (see the kernel)
        ug = ug < 1 ? 1 : ug;
        if (blocks > 0x7fffffffLL) return set_error(ZIPVL_ESHAPE, "sparse_prefill: %lld workgroups exceed the grid limit", (long long)blocks);
        hipLaunchKernelGGL((flash_kept_kernel<T, D, NW>), dim3((unsigned)blocks), dim3(C::NT),
            C::LDS_BYTES, st, (const T*)Q, d.q_strides[0], d.q_strides[1], d.q_strides[2],
            skip_k ? (const T*)K : Kp, skip_k ? d.k_strides[0] : (int64_t)d.Hkv * npad * D,
            skip_k ? d.k_strides[1] : (int64_t)npad * D, VTp, idx, k, (T*)O, d.n, npad, ntq, ug, BH, d.Hq, d.Hkv,
            scale * kLog2e, out_compact, (!out_compact && idx) ? 1 : 0);
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

    // An evicted cache with contiguous rows and whole 64-row tiles is read in place: only V is repacked.
    // (Rows between k and the end of the last tile may hold anything: they are masked, never summed.)
    const int skip_k = (rows_are_kept && d.k_strides[2] == D && d.n % kBN == 0) ? 1 : 0;
    {
        KernelTimer tm(ZIPVL_K_PACK_KV, st);
        hipLaunchKernelGGL((pack_kv_kernel<T, D>), dim3(npad / kBN, units), dim3(256), 0, st,
            (const T*)K, (const T*)V, d.k_strides[0], d.k_strides[1], d.k_strides[2],
            d.v_strides[0], d.v_strides[1], d.v_strides[2], idx, k, Kp, VTp, d.n, npad, d.Hkv, rows_are_kept, skip_k);
    }
    int rc = check_launch("pack_kv");
    if (rc) return rc;

    // bf16: 8 waves share every tile (half the L2 -> LDS traffic per query); fp32 keeps 4 waves
    // (its tiles are twice as large and it runs one wave per SIMD).
    if constexpr (Elem<T>::kBytes == 2)
        return launch_flash<T, D, kFlashWavesBf16>(Q, K, d, idx, k, scale, out_compact, skip_k, Kp, VTp, npad, O, st);
    else
        return launch_flash<T, D, 4>(Q, K, d, idx, k, scale, out_compact, skip_k, Kp, VTp, npad, O, st);
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
