// Host-side launch entry points of each kernel file (internal to the library).
#pragma once
#include "common.h"

namespace zipvl {

// Optional per-kernel timing with HIP events on the launch stream (off by default).
struct KernelTimer {
    KernelTimer(int kernel_id, hipStream_t st);
    ~KernelTimer();
    int slot;
    hipStream_t st;
};

struct ProbeList {            // passed by value in the kernel arguments
    int32_t pos[ZIPVL_MAX_PROBES];
};

size_t score_workspace_bytes(const zipvl_dims& d, int m);
int launch_score(const void* Q, const void* K, const zipvl_dims& d, const int32_t* probe_pos, int m,
                 float scale, int flags, float* mass, float* rank, void* ws, hipStream_t st);

size_t select_workspace_bytes(int units);
int launch_select(const float* mass, const float* rank, int units, int n, double tau,
                  int32_t* idx, int32_t* k, int32_t* status, void* ws, size_t ws_bytes, hipStream_t st);

size_t prefill_workspace_bytes(const zipvl_dims& d);
int launch_sparse_prefill(const void* Q, const void* K, const void* V, const zipvl_dims& d,
                          const int32_t* idx, const int32_t* k, float scale, int flags,
                          void* O, void* ws, hipStream_t st);

int launch_compact_kv(const void* K, const void* V, const zipvl_dims& d, const int32_t* idx,
                      const int32_t* k, void* Kc, void* Vc, int32_t cap, int32_t* len, int flags, hipStream_t st);
int launch_share_scores(const float* mass, const float* rank, int B, int Hkv, int n,
                        float* mass_b, float* rank_b, hipStream_t st);
int launch_kv_append(void* Kc, void* Vc, int32_t* len, int32_t cap, const void* k_new,
                     const void* v_new, const zipvl_dims& d, hipStream_t st);

size_t decode_workspace_bytes(const zipvl_dims& d, int cap);
int launch_decode_attn(const void* q, const void* Kc, const void* Vc, const int32_t* len, int32_t cap,
                       const zipvl_dims& d, float scale, void* o, void* ws, hipStream_t st);

int launch_decode_attn_static(const void* q, const void* Kc, const void* Vc, const int32_t* len, int32_t cap,
                              const zipvl_dims& d, float scale, void* o, hipStream_t st);

size_t decode_step_workspace_bytes(const zipvl_dims& d, int cap);
int launch_decode_step(const void* q, void* Kc, void* Vc, int32_t* len, int32_t cap, const void* k_new,
                       const void* v_new, const zipvl_dims& d, float scale, void* o, void* ws, hipStream_t st);

size_t allrows_workspace_bytes(const zipvl_dims& d);
int launch_score_all_rows(const void* Q, const void* K, const zipvl_dims& d, float scale,
                          float* mass, float* rank, void* ws, hipStream_t st);

size_t quantize_workspace_bytes(const zipvl_dims& d);
int launch_quantize_kv(const void* K, const void* V, const zipvl_dims& d, const int32_t* idx, const int32_t* k,
                       const zipvl_qtensor& Kq, const zipvl_qtensor& Vq, int32_t cap_hi, int32_t cap_lo,
                       int32_t* len_hi, int32_t* len_lo, int flags, void* ws, hipStream_t st);
int launch_decode_attn_q(const void* q, const zipvl_qtensor& Kq, const zipvl_qtensor& Vq, const int32_t* len_hi,
                         const int32_t* len_lo, int32_t cap_hi, int32_t cap_lo, const void* Kt, const void* Vt,
                         const int32_t* len_t, int32_t cap_t, const zipvl_dims& d, float scale, void* o, void* ws, hipStream_t st);

int launch_probe_mfma(int iters, int workgroups, float* out, hipStream_t st);
int launch_probe_read(const void* src, size_t bytes, int workgroups, uint32_t* out, hipStream_t st);

}  // namespace zipvl
