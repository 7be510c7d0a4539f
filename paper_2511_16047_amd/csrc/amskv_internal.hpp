// Internal declarations shared by the host layer and the kernel launchers of libamskv.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "amskv.h"

namespace amskv {

// Resident segments of one layer as the attention kernel walks them: segment i holds
// `len[i]` tokens; in the virtual concatenation K~ of Section 3.1's per-step attention it
// covers rows [virt_start[i], virt_start[i]+len[i]); in the layer's K/V regions it sits at
// token offset phys_off[i].  Passed to kernels by value (lives in scalar registers).
struct SegTable {
  int32_t n;
  int32_t total;  // sum of len = T_kv
  int32_t virt_start[AMSKV_MAX_SCALES];
  int32_t phys_off[AMSKV_MAX_SCALES];
  int32_t len[AMSKV_MAX_SCALES];
};

// Token ranges that slide toward lower offsets when scales are evicted (COMPACT layout),
// in ascending order of offset; dst < src for every entry.
struct MoveList {
  int32_t n;
  int32_t src[AMSKV_MAX_SCALES];
  int32_t dst[AMSKV_MAX_SCALES];
  int32_t len[AMSKV_MAX_SCALES];
};

// ---- kernel launchers (each validates nothing: the host layer has checked shapes) ----
hipError_t launch_attend_bf16(const void* q, void* o, const void* kc, const void* vc, int bh,
                              int t_q, int head_dim, int64_t cap_tokens, const SegTable& seg,
                              float softmax_scale, hipStream_t st);
hipError_t launch_attend_bf16_small(const void* q, void* o, const void* kc, const void* vc, int bh,
                                    int t_q, int head_dim, int64_t cap_tokens, const SegTable& seg,
                                    float softmax_scale, hipStream_t st);
hipError_t launch_attend_f32(const void* q, void* o, const void* kc, const void* vc, int bh,
                             int t_q, int head_dim, int64_t cap_tokens, const SegTable& seg,
                             float softmax_scale, hipStream_t st);
hipError_t launch_append(void* kc, void* vc, const void* k_new, const void* v_new, int bh,
                         int row_bytes, int64_t cap_tokens, const MoveList& mv, int t_new,
                         int dst_new, hipStream_t st);
hipError_t launch_export(const void* kc, const void* vc, void* k_out, void* v_out, int bh,
                         int row_bytes, int64_t cap_tokens, const SegTable& seg, hipStream_t st);
hipError_t launch_similarity(const void* kc, const void* vc, int batch, int heads, int head_dim,
                             int dtype, int64_t cap_tokens, int off_cur, int off_prev, int h_cur,
                             int w_cur, int h_prev, int w_prev, float* partial_ws, float* out_dev,
                             hipStream_t st);

}  // namespace amskv
