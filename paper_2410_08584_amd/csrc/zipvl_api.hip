// C ABI: argument validation and dispatch.  Nothing here touches device data;
// every check is on the host-visible arguments, and a rejected call launches
// nothing.
#include <cstdarg>
#include <cstdio>
#include <mutex>
#include <vector>
#include "launch.h"

namespace zipvl {

static thread_local char g_err[512] = "";

int set_error(int code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

int check_launch(const char* what) {
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return set_error(ZIPVL_EHIP, "%s: launch failed: %s", what, hipGetErrorString(e));
    return ZIPVL_OK;
}

// ---- optional kernel timing -------------------------------------------------
namespace {
constexpr int kMaxTimed = 8192;
struct TimedLaunch { int id; hipEvent_t start, stop; };
std::mutex g_tmu;
bool g_timing = false;
std::vector<TimedLaunch> g_timed;
std::vector<hipEvent_t> g_pool;       // created once, reused
int g_pool_used = 0;
}  // namespace

KernelTimer::KernelTimer(int kernel_id, hipStream_t s) : slot(-1), st(s) {
    if (!g_timing) return;
    std::lock_guard<std::mutex> lk(g_tmu);
    if ((int)g_timed.size() >= kMaxTimed) return;
    while ((int)g_pool.size() < g_pool_used + 2) {
        hipEvent_t e;
        if (hipEventCreate(&e) != hipSuccess) return;
        g_pool.push_back(e);
    }
    TimedLaunch t{kernel_id, g_pool[g_pool_used], g_pool[g_pool_used + 1]};
    g_pool_used += 2;
    if (hipEventRecord(t.start, st) != hipSuccess) return;
    slot = (int)g_timed.size();
    g_timed.push_back(t);
}

KernelTimer::~KernelTimer() {
    if (slot < 0) return;
    std::lock_guard<std::mutex> lk(g_tmu);
    (void)hipEventRecord(g_timed[slot].stop, st);
}

static bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

static int check_dims(const char* fn, const zipvl_dims* d, bool need_q, bool need_k, bool need_v) {
    if (!d) return set_error(ZIPVL_EINVAL, "%s: dims is NULL", fn);
    if (d->dtype != ZIPVL_F32 && d->dtype != ZIPVL_BF16)
        return set_error(ZIPVL_EUNSUPPORTED, "%s: dtype %d (0 = fp32, 1 = bf16)", fn, d->dtype);
    if (d->B < 1 || d->Hq < 1 || d->Hkv < 1 || d->n < 1)
        return set_error(ZIPVL_EINVAL, "%s: B, Hq, Hkv, n must be positive (got %d %d %d %d)", fn, d->B, d->Hq, d->Hkv, d->n);
    if (d->Hq % d->Hkv != 0) return set_error(ZIPVL_ESHAPE, "%s: Hq=%d is not a multiple of Hkv=%d", fn, d->Hq, d->Hkv);
    if (d->d != 64 && d->d != 128) return set_error(ZIPVL_ESHAPE, "%s: head dim %d (supported: 64, 128)", fn, d->d);
    if ((int64_t)d->B * d->Hq > 65535) return set_error(ZIPVL_ESHAPE, "%s: B*Hq = %lld exceeds 65535", fn, (long long)d->B * d->Hq);
    if (d->n > (1 << 24)) return set_error(ZIPVL_ESHAPE, "%s: n = %d exceeds 2^24", fn, d->n);
    const int per16 = d->dtype == ZIPVL_BF16 ? 8 : 4;
    const int64_t* s[3] = {d->q_strides, d->k_strides, d->v_strides};
    const bool need[3] = {need_q, need_k, need_v};
    const char* nm[3] = {"q", "k", "v"};
    for (int t = 0; t < 3; ++t) {
        if (!need[t]) continue;
        for (int a = 0; a < 3; ++a) {
            if (s[t][a] < 0) return set_error(ZIPVL_EINVAL, "%s: %s_strides[%d] is negative", fn, nm[t], a);
            if (s[t][a] % per16) return set_error(ZIPVL_EALIGN, "%s: %s_strides[%d]=%lld is not a multiple of 16 bytes", fn, nm[t], a, (long long)s[t][a]);
        }
        if (s[t][2] < d->d) return set_error(ZIPVL_EINVAL, "%s: %s token stride %lld is smaller than d", fn, nm[t], (long long)s[t][2]);
    }
    return ZIPVL_OK;
}

#define ZIPVL_REQUIRE_PTR(fn, p)                                                         \
    do {                                                                                 \
        if (!(p)) return set_error(ZIPVL_EINVAL, "%s: %s is NULL", fn, #p);              \
        if (!aligned16(p)) return set_error(ZIPVL_EALIGN, "%s: %s is not 16-byte aligned", fn, #p); \
    } while (0)

}  // namespace zipvl

using namespace zipvl;

extern "C" {

int zipvl_version(void) { return 100; }

const char* zipvl_last_error(void) { return g_err; }

size_t zipvl_workspace_bytes(int op, const zipvl_dims* dims, int m) {
    if (check_dims("zipvl_workspace_bytes", dims, false, false, false)) return 0;
    switch (op) {
        case ZIPVL_OP_SCORE: return score_workspace_bytes(*dims, m);
        case ZIPVL_OP_SELECT: return select_workspace_bytes(dims->B * dims->Hkv);
        case ZIPVL_OP_SPARSE_PREFILL: return prefill_workspace_bytes(*dims);
        case ZIPVL_OP_DECODE: return decode_workspace_bytes(*dims, dims->n);
        case ZIPVL_OP_QUANTIZE_KV: return quantize_workspace_bytes(*dims);
        case ZIPVL_OP_DECODE_Q: return decode_workspace_bytes(*dims, dims->n);
        case ZIPVL_OP_SCORE_ALL_ROWS: return allrows_workspace_bytes(*dims);
        case ZIPVL_OP_DECODE_STEP: return decode_step_workspace_bytes(*dims, dims->n);
        default: set_error(ZIPVL_EUNSUPPORTED, "zipvl_workspace_bytes: unknown op %d", op); return 0;
    }
}

int zipvl_score(const void* Q, const void* K, const zipvl_dims* dims, const int32_t* probe_pos, int m,
                float softmax_scale, int flags, float* mass, float* rank, void* ws, size_t ws_bytes, void* stream)
{
    const char* fn = "zipvl_score";
    int rc = check_dims(fn, dims, true, true, false);
    if (rc) return rc;
    ZIPVL_REQUIRE_PTR(fn, Q);
    ZIPVL_REQUIRE_PTR(fn, K);
    ZIPVL_REQUIRE_PTR(fn, mass);
    if (rank && !aligned16(rank)) return set_error(ZIPVL_EALIGN, "%s: rank is not 16-byte aligned", fn);
    if (!probe_pos) return set_error(ZIPVL_EINVAL, "%s: probe_pos is NULL", fn);
    if (m < 1) return set_error(ZIPVL_EINVAL, "%s: m = %d must be positive", fn, m);
    if (m > ZIPVL_MAX_PROBES) return set_error(ZIPVL_ESHAPE, "%s: m = %d exceeds %d probe rows", fn, m, ZIPVL_MAX_PROBES);
    for (int t = 0; t < m; ++t) {
        if (probe_pos[t] < 0 || probe_pos[t] >= dims->n)
            return set_error(ZIPVL_EINVAL, "%s: probe_pos[%d] = %d is outside [0, %d)", fn, t, probe_pos[t], dims->n);
        if (t && probe_pos[t] <= probe_pos[t - 1])
            return set_error(ZIPVL_EINVAL, "%s: probe_pos must be strictly ascending (entry %d)", fn, t);
    }
    if (!(softmax_scale > 0.f) || !(softmax_scale < 1e30f)) return set_error(ZIPVL_EINVAL, "%s: softmax_scale must be positive and finite", fn);
    if (flags & ~ZIPVL_SCORE_PER_QHEAD) return set_error(ZIPVL_EUNSUPPORTED, "%s: unknown flags 0x%x", fn, flags);
    const size_t need = score_workspace_bytes(*dims, m);
    if (!ws || ws_bytes < need) return set_error(ZIPVL_EWORKSPACE, "%s: workspace of %zu bytes needed, %zu given", fn, need, ws ? ws_bytes : (size_t)0);
    if (!aligned16(ws)) return set_error(ZIPVL_EALIGN, "%s: ws is not 16-byte aligned", fn);
    return launch_score(Q, K, *dims, probe_pos, m, softmax_scale, flags, mass, rank, ws, (hipStream_t)stream);
}

int zipvl_score_all_rows(const void* Q, const void* K, const zipvl_dims* dims, float softmax_scale,
                         float* mass, float* rank, void* ws, size_t ws_bytes, void* stream)
{
    const char* fn = "zipvl_score_all_rows";
    int rc = check_dims(fn, dims, true, true, false);
    if (rc) return rc;
    ZIPVL_REQUIRE_PTR(fn, Q);
    ZIPVL_REQUIRE_PTR(fn, K);
    ZIPVL_REQUIRE_PTR(fn, mass);
    if (rank && !aligned16(rank)) return set_error(ZIPVL_EALIGN, "%s: rank is not 16-byte aligned", fn);
    if (!(softmax_scale > 0.f) || !(softmax_scale < 1e30f)) return set_error(ZIPVL_EINVAL, "%s: softmax_scale must be positive and finite", fn);
    const size_t need = allrows_workspace_bytes(*dims);
    if (!ws || ws_bytes < need) return set_error(ZIPVL_EWORKSPACE, "%s: workspace of %zu bytes needed, %zu given", fn, need, ws ? ws_bytes : (size_t)0);
    if (!aligned16(ws)) return set_error(ZIPVL_EALIGN, "%s: ws is not 16-byte aligned", fn);
    return launch_score_all_rows(Q, K, *dims, softmax_scale, mass, rank, ws, (hipStream_t)stream);
}

int zipvl_select(const float* mass, const float* rank, int units, int n, double tau,
                 int32_t* idx, int32_t* k, int32_t* status, void* ws, size_t ws_bytes, void* stream)
{
    const char* fn = "zipvl_select";
    if (!mass || !idx || !k) return set_error(ZIPVL_EINVAL, "%s: mass, idx and k must not be NULL", fn);
    if (units < 1 || n < 1) return set_error(ZIPVL_EINVAL, "%s: units and n must be positive (got %d, %d)", fn, units, n);
    if (n >= (1 << 23)) return set_error(ZIPVL_ESHAPE, "%s: n = %d must be below 2^23", fn, n);
    if (!(tau > 0.0) || !(tau <= 1.0)) return set_error(ZIPVL_EINVAL, "%s: tau = %g is outside (0, 1]", fn, tau);
    if ((reinterpret_cast<uintptr_t>(mass) | reinterpret_cast<uintptr_t>(rank) |
         reinterpret_cast<uintptr_t>(idx) | reinterpret_cast<uintptr_t>(k) | reinterpret_cast<uintptr_t>(status)) & 3u)
        return set_error(ZIPVL_EALIGN, "%s: pointers must be 4-byte aligned", fn);
    if (ws && (reinterpret_cast<uintptr_t>(ws) & 15u)) return set_error(ZIPVL_EALIGN, "%s: ws is not 16-byte aligned", fn);
    if (ws && ws_bytes < select_workspace_bytes(units))
        return set_error(ZIPVL_EWORKSPACE, "%s: workspace of %zu bytes needed, %zu given (or pass NULL)", fn, select_workspace_bytes(units), ws_bytes);
    return launch_select(mass, rank, units, n, tau, idx, k, status, ws, ws_bytes, (hipStream_t)stream);
}

int zipvl_share_scores(const float* mass, const float* rank, int B, int Hkv, int n,
                       float* mass_b, float* rank_b, void* stream)
{
    const char* fn = "zipvl_share_scores";
    if (!mass || !mass_b) return set_error(ZIPVL_EINVAL, "%s: mass and mass_b must not be NULL", fn);
    if ((rank == nullptr) != (rank_b == nullptr)) return set_error(ZIPVL_EINVAL, "%s: rank and rank_b must both be given or both be NULL", fn);
    if (B < 1 || Hkv < 1 || n < 1) return set_error(ZIPVL_EINVAL, "%s: B, Hkv and n must be positive (got %d, %d, %d)", fn, B, Hkv, n);
    if ((reinterpret_cast<uintptr_t>(mass) | reinterpret_cast<uintptr_t>(rank) |
         reinterpret_cast<uintptr_t>(mass_b) | reinterpret_cast<uintptr_t>(rank_b)) & 3u)
        return set_error(ZIPVL_EALIGN, "%s: pointers must be 4-byte aligned", fn);
    return launch_share_scores(mass, rank, B, Hkv, n, mass_b, rank_b, (hipStream_t)stream);
}

int zipvl_sparse_prefill(const void* Q, const void* K, const void* V, const zipvl_dims* dims,
                         const int32_t* idx, const int32_t* k, float softmax_scale, int flags,
                         void* O, void* ws, size_t ws_bytes, void* stream)
{
    const char* fn = "zipvl_sparse_prefill";
    int rc = check_dims(fn, dims, true, true, true);
    if (rc) return rc;
    ZIPVL_REQUIRE_PTR(fn, Q);
    ZIPVL_REQUIRE_PTR(fn, K);
    ZIPVL_REQUIRE_PTR(fn, V);
    ZIPVL_REQUIRE_PTR(fn, O);
    if ((idx == nullptr) != (k == nullptr)) return set_error(ZIPVL_EINVAL, "%s: idx and k must both be given or both be NULL", fn);
    if (flags & ~(ZIPVL_OUT_COMPACT | ZIPVL_KV_ALREADY_COMPACT | ZIPVL_T_PER_BATCH)) return set_error(ZIPVL_EUNSUPPORTED, "%s: unknown flags 0x%x", fn, flags);
    if (!(softmax_scale > 0.f) || !(softmax_scale < 1e30f)) return set_error(ZIPVL_EINVAL, "%s: softmax_scale must be positive and finite", fn);
    const size_t need = prefill_workspace_bytes(*dims);
    if (!ws || ws_bytes < need) return set_error(ZIPVL_EWORKSPACE, "%s: workspace of %zu bytes needed, %zu given", fn, need, ws ? ws_bytes : (size_t)0);
    if (reinterpret_cast<uintptr_t>(ws) & 255u) return set_error(ZIPVL_EALIGN, "%s: ws is not 256-byte aligned", fn);
    return launch_sparse_prefill(Q, K, V, *dims, idx, k, softmax_scale, flags, O, ws, (hipStream_t)stream);
}

int zipvl_compact_kv(const void* K, const void* V, const zipvl_dims* dims, const int32_t* idx,
                     const int32_t* k, void* Kc, void* Vc, int32_t cap, int32_t* len, int flags, void* stream)
{
    const char* fn = "zipvl_compact_kv";
    int rc = check_dims(fn, dims, false, true, true);
    if (rc) return rc;
    ZIPVL_REQUIRE_PTR(fn, K);
    ZIPVL_REQUIRE_PTR(fn, V);
    ZIPVL_REQUIRE_PTR(fn, Kc);
    ZIPVL_REQUIRE_PTR(fn, Vc);
    if (!len) return set_error(ZIPVL_EINVAL, "%s: len is NULL", fn);
    if ((idx == nullptr) != (k == nullptr)) return set_error(ZIPVL_EINVAL, "%s: idx and k must both be given or both be NULL", fn);
    if (cap < 1) return set_error(ZIPVL_EINVAL, "%s: cap = %d must be positive", fn, cap);
    if (flags & ~ZIPVL_T_PER_BATCH) return set_error(ZIPVL_EUNSUPPORTED, "%s: unknown flags 0x%x", fn, flags);
    return launch_compact_kv(K, V, *dims, idx, k, Kc, Vc, cap, len, flags, (hipStream_t)stream);
}

int zipvl_kv_append(void* Kc, void* Vc, int32_t* len, int32_t cap, const void* k_new,
                    const void* v_new, const zipvl_dims* dims, void* stream)
{
    const char* fn = "zipvl_kv_append";
    int rc = check_dims(fn, dims, false, false, false);
    if (rc) return rc;
    ZIPVL_REQUIRE_PTR(fn, Kc);
    ZIPVL_REQUIRE_PTR(fn, Vc);
    ZIPVL_REQUIRE_PTR(fn, k_new);
    ZIPVL_REQUIRE_PTR(fn, v_new);
    if (!len) return set_error(ZIPVL_EINVAL, "%s: len is NULL", fn);
    if (cap < 1) return set_error(ZIPVL_EINVAL, "%s: cap = %d must be positive", fn, cap);
    return launch_kv_append(Kc, Vc, len, cap, k_new, v_new, *dims, (hipStream_t)stream);
}

int zipvl_decode_attn(const void* q, const void* Kc, const void* Vc, const int32_t* len, int32_t cap,
                      const zipvl_dims* dims, float softmax_scale, void* o, void* ws, size_t ws_bytes,
                      void* stream)
{
    const char* fn = "zipvl_decode_attn";
    int rc = check_dims(fn, dims, false, false, false);
    if (rc) return rc;
    ZIPVL_REQUIRE_PTR(fn, q);
    ZIPVL_REQUIRE_PTR(fn, Kc);
    ZIPVL_REQUIRE_PTR(fn, Vc);
    ZIPVL_REQUIRE_PTR(fn, o);
    if (!len) return set_error(ZIPVL_EINVAL, "%s: len is NULL", fn);
    if (cap < 1) return set_error(ZIPVL_EINVAL, "%s: cap = %d must be positive", fn, cap);
    if (!(softmax_scale > 0.f) || !(softmax_scale < 1e30f)) return set_error(ZIPVL_EINVAL, "%s: softmax_scale must be positive and finite", fn);
    const size_t need = decode_workspace_bytes(*dims, cap);
    if (!ws || ws_bytes < need) return set_error(ZIPVL_EWORKSPACE, "%s: workspace of %zu bytes needed, %zu given", fn, need, ws ? ws_bytes : (size_t)0);
    if (!aligned16(ws)) return set_error(ZIPVL_EALIGN, "%s: ws is not 16-byte aligned", fn);
    return launch_decode_attn(q, Kc, Vc, len, cap, *dims, softmax_scale, o, ws, (hipStream_t)stream);
}

int zipvl_decode_attn_static(const void* q, const void* Kc, const void* Vc, const int32_t* len, int32_t cap,
                             const zipvl_dims* dims, float softmax_scale, void* o, void* stream)
{
    const char* fn = "zipvl_decode_attn_static";
    int rc = check_dims(fn, dims, false, false, false);
    if (rc) return rc;
    ZIPVL_REQUIRE_PTR(fn, q);
    ZIPVL_REQUIRE_PTR(fn, Kc);
    ZIPVL_REQUIRE_PTR(fn, Vc);
    ZIPVL_REQUIRE_PTR(fn, o);
    if (!len) return set_error(ZIPVL_EINVAL, "%s: len is NULL", fn);
    if (cap < 1) return set_error(ZIPVL_EINVAL, "%s: cap = %d must be positive", fn, cap);
    if (!(softmax_scale > 0.f) || !(softmax_scale < 1e30f)) return set_error(ZIPVL_EINVAL, "%s: softmax_scale must be positive and finite", fn);
    return launch_decode_attn_static(q, Kc, Vc, len, cap, *dims, softmax_scale, o, (hipStream_t)stream);
}

int zipvl_decode_step(const void* q, void* Kc, void* Vc, int32_t* len, int32_t cap, const void* k_new,
                      const void* v_new, const zipvl_dims* dims, float softmax_scale, void* o,
                      void* ws, size_t ws_bytes, void* stream)
{
    const char* fn = "zipvl_decode_step";
    int rc = check_dims(fn, dims, false, false, false);
    if (rc) return rc;
    ZIPVL_REQUIRE_PTR(fn, q);
    ZIPVL_REQUIRE_PTR(fn, Kc);
    ZIPVL_REQUIRE_PTR(fn, Vc);
    ZIPVL_REQUIRE_PTR(fn, k_new);
    ZIPVL_REQUIRE_PTR(fn, v_new);
    ZIPVL_REQUIRE_PTR(fn, o);
    if (!len) return set_error(ZIPVL_EINVAL, "%s: len is NULL", fn);
    if (cap < 1) return set_error(ZIPVL_EINVAL, "%s: cap = %d must be positive", fn, cap);
    if (!(softmax_scale > 0.f) || !(softmax_scale < 1e30f)) return set_error(ZIPVL_EINVAL, "%s: softmax_scale must be positive and finite", fn);
    const size_t need = decode_step_workspace_bytes(*dims, cap);
    if (!ws || ws_bytes < need) return set_error(ZIPVL_EWORKSPACE, "%s: workspace of %zu bytes needed, %zu given", fn, need, ws ? ws_bytes : (size_t)0);
    if (!aligned16(ws)) return set_error(ZIPVL_EALIGN, "%s: ws is not 16-byte aligned", fn);
    return launch_decode_step(q, Kc, Vc, len, cap, k_new, v_new, *dims, softmax_scale, o, ws, (hipStream_t)stream);
}

static int check_qtensor(const char* fn, const char* what, const zipvl_qtensor* t) {
    if (!t) return set_error(ZIPVL_EINVAL, "%s: %s is NULL", fn, what);
    const void* ptrs[4] = {t->hi_codes, t->hi_params, t->lo_codes, t->lo_params};
    for (const void* p : ptrs) {
        if (!p) return set_error(ZIPVL_EINVAL, "%s: an array of %s is NULL", fn, what);
        if (!aligned16(p)) return set_error(ZIPVL_EALIGN, "%s: an array of %s is not 16-byte aligned", fn, what);
    }
    return ZIPVL_OK;
}

int zipvl_quantize_kv(const void* K, const void* V, const zipvl_dims* dims, const int32_t* idx, const int32_t* k,
                      const zipvl_qtensor* Kq, const zipvl_qtensor* Vq, int32_t cap_hi, int32_t cap_lo,
                      int32_t* len_hi, int32_t* len_lo, int flags, void* ws, size_t ws_bytes, void* stream)
{
    const char* fn = "zipvl_quantize_kv";
    int rc = check_dims(fn, dims, false, true, true);
    if (rc) return rc;
    ZIPVL_REQUIRE_PTR(fn, K);
    ZIPVL_REQUIRE_PTR(fn, V);
    if ((rc = check_qtensor(fn, "Kq", Kq)) || (rc = check_qtensor(fn, "Vq", Vq))) return rc;
    if (!len_hi || !len_lo) return set_error(ZIPVL_EINVAL, "%s: len_hi / len_lo is NULL", fn);
    if ((idx == nullptr) != (k == nullptr)) return set_error(ZIPVL_EINVAL, "%s: idx and k must both be given or both be NULL", fn);
    if (cap_hi < 1 || cap_lo < 1) return set_error(ZIPVL_EINVAL, "%s: cap_hi = %d and cap_lo = %d must be positive", fn, cap_hi, cap_lo);
    if (flags & ~ZIPVL_T_PER_BATCH) return set_error(ZIPVL_EUNSUPPORTED, "%s: unknown flags 0x%x", fn, flags);
    const size_t need = quantize_workspace_bytes(*dims);
    if (!ws || ws_bytes < need) return set_error(ZIPVL_EWORKSPACE, "%s: workspace of %zu bytes needed, %zu given", fn, need, ws ? ws_bytes : (size_t)0);
    if (reinterpret_cast<uintptr_t>(ws) & 3u) return set_error(ZIPVL_EALIGN, "%s: ws is not 4-byte aligned", fn);
    return launch_quantize_kv(K, V, *dims, idx, k, *Kq, *Vq, cap_hi, cap_lo, len_hi, len_lo, flags, ws, (hipStream_t)stream);
}

int zipvl_decode_attn_q(const void* q, const zipvl_qtensor* Kq, const zipvl_qtensor* Vq,
                        const int32_t* len_hi, const int32_t* len_lo, int32_t cap_hi, int32_t cap_lo,
                        const void* K_tail, const void* V_tail, const int32_t* len_tail, int32_t cap_tail,
                        const zipvl_dims* dims, float softmax_scale, void* o, void* ws, size_t ws_bytes, void* stream)
{
    const char* fn = "zipvl_decode_attn_q";
    int rc = check_dims(fn, dims, false, false, false);
    if (rc) return rc;
    ZIPVL_REQUIRE_PTR(fn, q);
    ZIPVL_REQUIRE_PTR(fn, o);
    if ((rc = check_qtensor(fn, "Kq", Kq)) || (rc = check_qtensor(fn, "Vq", Vq))) return rc;
    if (!len_hi || !len_lo) return set_error(ZIPVL_EINVAL, "%s: len_hi / len_lo is NULL", fn);
    if (cap_hi < 1 || cap_lo < 1) return set_error(ZIPVL_EINVAL, "%s: cap_hi = %d and cap_lo = %d must be positive", fn, cap_hi, cap_lo);
    const bool tail = K_tail || V_tail || len_tail;
    if (tail) {
        if (!K_tail || !V_tail || !len_tail) return set_error(ZIPVL_EINVAL, "%s: K_tail, V_tail and len_tail must all be given or all be NULL", fn);
        if (!aligned16(K_tail) || !aligned16(V_tail)) return set_error(ZIPVL_EALIGN, "%s: K_tail / V_tail is not 16-byte aligned", fn);
        if (cap_tail < 1) return set_error(ZIPVL_EINVAL, "%s: cap_tail = %d must be positive", fn, cap_tail);
    } else {
        cap_tail = 0;
    }
    if (!(softmax_scale > 0.f) || !(softmax_scale < 1e30f)) return set_error(ZIPVL_EINVAL, "%s: softmax_scale must be positive and finite", fn);
    const size_t need = decode_workspace_bytes(*dims, cap_hi + cap_lo + cap_tail);
    if (!ws || ws_bytes < need) return set_error(ZIPVL_EWORKSPACE, "%s: workspace of %zu bytes needed, %zu given", fn, need, ws ? ws_bytes : (size_t)0);
    if (!aligned16(ws)) return set_error(ZIPVL_EALIGN, "%s: ws is not 16-byte aligned", fn);
    return launch_decode_attn_q(q, *Kq, *Vq, len_hi, len_lo, cap_hi, cap_lo, K_tail, V_tail, len_tail, cap_tail,
                                *dims, softmax_scale, o, ws, (hipStream_t)stream);
}

int zipvl_probe_mfma(int iters, int workgroups, float* out, void* stream)
{
    if (iters < 1 || workgroups < 1 || !out) return set_error(ZIPVL_EINVAL, "zipvl_probe_mfma: iters, workgroups must be positive and out given");
    return launch_probe_mfma(iters, workgroups, out, (hipStream_t)stream);
}

int zipvl_probe_stream_read(const void* src, size_t bytes, int workgroups, uint32_t* out, void* stream)
{
    if (!src || !out || workgroups < 1 || bytes < 16 || (bytes & 15)) return set_error(ZIPVL_EINVAL, "zipvl_probe_stream_read: src, out, workgroups >= 1 and bytes a positive multiple of 16 are required");
    if (!aligned16(src)) return set_error(ZIPVL_EALIGN, "zipvl_probe_stream_read: src is not 16-byte aligned");
    return launch_probe_read(src, bytes, workgroups, out, (hipStream_t)stream);
}

int zipvl_timing_enable(int on) {
    std::lock_guard<std::mutex> lk(g_tmu);
    g_timed.clear();
    g_pool_used = 0;
    g_timing = on != 0;
    return ZIPVL_OK;
}

int zipvl_timing_read(int kernel_id, double* total_ms, int* launches) {
    if (!total_ms || !launches) return set_error(ZIPVL_EINVAL, "zipvl_timing_read: NULL output");
    if (kernel_id < 0 || kernel_id >= ZIPVL_K_COUNT) return set_error(ZIPVL_EINVAL, "zipvl_timing_read: kernel id %d", kernel_id);
    std::lock_guard<std::mutex> lk(g_tmu);
    double sum = 0.0;
    int cnt = 0;
    for (const TimedLaunch& t : g_timed) {
        if (t.id != kernel_id) continue;
        if (hipEventSynchronize(t.stop) != hipSuccess) return set_error(ZIPVL_EHIP, "zipvl_timing_read: event wait failed");
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, t.start, t.stop) != hipSuccess) return set_error(ZIPVL_EHIP, "zipvl_timing_read: elapsed time failed");
        sum += ms;
        ++cnt;
    }
    *total_ms = sum;
    *launches = cnt;
    return ZIPVL_OK;
}

}  // extern "C"
