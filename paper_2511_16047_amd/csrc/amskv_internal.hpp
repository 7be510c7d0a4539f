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
// A borrowed current scale (read in place from the caller's K/V, never copied) is always the
// last segment: it covers virtual rows [ext_start, total) and its rows come from the external
// pointers handed to the kernel next to the table; ext_start == total when nothing is borrowed.
struct SegTable {
  int32_t n;
  int32_t total;      // sum of len = T_kv
  int32_t ext_start;  // first virtual row of the borrowed segment (== total: none)
  int32_t virt_start[AMSKV_MAX_SCALES];
  int32_t phys_off[AMSKV_MAX_SCALES];
  int32_t len[AMSKV_MAX_SCALES];
};

// Groups of keys of the virtual concatenation, for the attention density: group i covers virtual rows
// [end[i-1], end[i]) (from 0 for the first); end[n-1] == SegTable::total.
struct GroupEnds {
  int32_t n;
  int32_t end[AMSKV_MAX_SCALES];
};

// External (borrowed) K and V of the current scale in the caller's buffers (rows located by
// CallerIo::kv), or null pointers.
// The attention kernel can also write rows it streams into the layer's K/V regions (the append fused into the
// attention of its step; in the token modes a whole iteration of Algorithm 1 -- survivors slide toward offset 0,
// what stays of the new scale lands behind them): row j of the virtual concatenation goes to token offset
// j + wb_delta when j >= wb_from, and to token offset j when ext_start <= j < wb_head_end.  Nothing is written with
// wb_from >= total and wb_head_end <= ext_start (kNoWriteBack, 0).  A destination never lies above its source row,
// and rows are streamed in ascending order by the one workgroup (or wave) that owns the unit, so a row is
// overwritten only after that owner has fetched it; callers ask for cached rows to be moved only for launches
// with one owner per unit (attend_owns_unit).
// When the outcome of the iteration hangs on an Eq. 3 test that is decided on the device just before the launch,
// both outcomes are handed over: alt_if points at the device word the test leaves (non-zero: the layer is
// cache-demanding, the budget grows) and the alt_ triple replaces the wb_ triple when it is set.
constexpr int32_t kNoWriteBack = 0x7fffffff;
struct ExtKV {
  const void* k;
  const void* v;
  int32_t wb_from, wb_delta, wb_head_end;
  const int32_t* alt_if;
  int32_t alt_from, alt_delta, alt_head_end;
};
__host__ __device__ inline bool writes_back(const ExtKV& e, int total, int ext_start) {
  return e.wb_from < total || e.wb_head_end > ext_start;
}
#if defined(__HIPCC__)
// the write-back the launch is to perform, the device's decision applied (uniform over the launch)
__device__ inline ExtKV chosen(ExtKV e) {
  if (e.alt_if != nullptr && *e.alt_if != 0) {
    e.wb_from = e.alt_from;
    e.wb_delta = e.alt_delta;
    e.wb_head_end = e.alt_head_end;
  }
  e.alt_if = nullptr;
  return e;
}
#endif
// token offset row j is written to, or -1
__host__ __device__ inline int write_back_row(const ExtKV& e, int j, int total, int ext_start) {
  if (j >= total) return -1;
  if (j >= e.wb_from) return j + e.wb_delta;
  return j >= ext_start && j < e.wb_head_end ? j : -1;
}

// Where the rows of a tensor owned by the caller sit: row t of unit (b, h) starts, in bytes from
// the tensor's base, at b*batch + h*head + t*tok (the D channels of a row are contiguous).
// Head-major [B][H][T][D] gives {H*T*D, T*D, D} * element size; token-major [B][T][..H*D..] with a
// token stride of `tok` elements gives {T*tok, D, tok} * element size.
struct RowMap {
  int64_t batch, head, tok;
};

// Maps of the tensors one attention call touches besides the cache: Q, O and the current scale's
// own K/V when it is read in place (ExtKV); `heads` splits the unit index bh into (b, h).
struct CallerIo {
  RowMap q, o, kv;
  int32_t heads;
};

// Token ranges that slide toward lower offsets when scales are evicted (COMPACT layout),
// in ascending order of offset; dst < src for every entry.
struct MoveList {
  int32_t n;
  int32_t src[AMSKV_MAX_SCALES];
  int32_t dst[AMSKV_MAX_SCALES];
  int32_t len[AMSKV_MAX_SCALES];
};

// Token ranges of the newest scale that Algorithm 2's trim keeps (its head while the cache is still
// shorter than the condensed part, and its tail): tokens [src_first, src_first + len) go to offset dst.
struct NewRanges {
  int32_t n;
  int32_t src_first[2];
  int32_t dst[2];
  int32_t len[2];
};

#if defined(__HIPCC__)
// Byte offset of row 0 of unit bh = b*heads + h inside a caller tensor.
__device__ __forceinline__ long long unit_offset(const RowMap& m, long long bh, int heads) {
  if (m.batch == m.head * heads) return bh * m.head;  // units back to back (head-major tensors): no division
  const unsigned b = (unsigned)bh / (unsigned)heads;   // bh < 2^24 (checked at create)
  return (long long)b * m.batch + (long long)((unsigned)bh - b * (unsigned)heads) * m.head;
}

// Virtual row j of K~/V~ -> row index inside the layer's cache region of this (b,h), or, for a
// row of the borrowed segment, row index inside the external tensor of this (b,h) (ext = true).
__device__ __forceinline__ int locate_row(const SegTable& seg, int j, bool& ext) {
  ext = j >= seg.ext_start;
  int delta = -seg.ext_start;
  if (!ext) {
    delta = 0;
    for (int g = 0; g < seg.n; ++g)
      if (j >= seg.virt_start[g]) delta = seg.phys_off[g] - seg.virt_start[g];
  }
  return j + delta;
}
#endif

// ---- kernel launchers (each validates nothing: the host layer has checked shapes) ----
// kc/vc are written only when ext.wb_off >= 0 (fused append)
hipError_t launch_attend_bf16(const void* q, void* o, void* kc, void* vc, int bh,
                              int t_q, int head_dim, int64_t cap_tokens, const SegTable& seg,
                              const ExtKV& ext, const CallerIo& io, float softmax_scale, hipStream_t st);
// The attention of a step with the attention density of its queries as a by-product: as launch_attend_bf16, plus
// the per-head masses of the groups in out_dev (heads * AMSKV_MAX_SCALES floats; workspace as for launch_density).
// Exists for t_q above the coarse-scale kernel's range only: attend_density_fused(t_q) tells.
bool attend_density_fused(int t_q);
// launch_attend_bf16 gives every (b,h) to one workgroup (or, on the coarse scales, one wave): the condition for
// asking it to move cached rows (ExtKV)
bool attend_owns_unit(int head_dim, int t_q);
hipError_t launch_attend_density_bf16(const void* q, void* o, void* kc, void* vc, int batch, int heads, int t_q, int head_dim,
                                      int64_t cap_tokens, const SegTable& seg, const ExtKV& ext, const CallerIo& io,
                                      float softmax_scale, const GroupEnds& groups, float* partial_ws, float* out_dev,
                                      hipStream_t st);
hipError_t launch_attend_bf16_small(const void* q, void* o, void* kc, void* vc, int bh,
                                    int t_q, int head_dim, int64_t cap_tokens, const SegTable& seg,
                                    const ExtKV& ext, const CallerIo& io, float softmax_scale, hipStream_t st);
hipError_t launch_attend_f32(const void* q, void* o, void* kc, void* vc, int bh,
                             int t_q, int head_dim, int64_t cap_tokens, const SegTable& seg,
                             const ExtKV& ext, const CallerIo& io, float softmax_scale, hipStream_t st);
// k_new == nullptr: compaction only (the new scale is borrowed, nothing to copy); otherwise tokens
// [src_first, src_first + t_new) of the new scale (rows located by src_map) go to offset dst_new
hipError_t launch_append(void* kc, void* vc, const void* k_new, const void* v_new, int bh,
                         int row_bytes, int64_t cap_tokens, const MoveList& mv, int t_new,
                         int dst_new, int src_first, const RowMap& src_map, int heads, hipStream_t st);
// One iteration of Algorithm 1 at token granularity in one launch: the surviving ranges slide down (mv), then
// the kept ranges of the new scale (rows located by src_map) are copied behind them
hipError_t launch_roll(void* kc, void* vc, const void* k_new, const void* v_new, int bh, int row_bytes,
                       int64_t cap_tokens, const MoveList& mv, const NewRanges& nr, const RowMap& src_map, int heads,
                       hipStream_t st);
// k_out/v_out are head-major [BH][T_kept][row]; ext_map locates the rows of a borrowed scale
hipError_t launch_export(const void* kc, const void* vc, void* k_out, void* v_out, int bh,
                         int row_bytes, int64_t cap_tokens, const SegTable& seg, const ExtKV& ext,
                         const RowMap& ext_map, int heads, hipStream_t st);
// A whole scale, wherever it lives: base pointers of the tensor holding it (the layer's cache
// regions or the caller's K/V), the map of that tensor's rows, and the token offset of the scale
// inside each (b,h) row range; v may be null (keys only)
struct ScaleRef {
  const void* k;
  const void* v;
  RowMap map;
  int32_t off_tokens;
};
hipError_t launch_similarity(const ScaleRef& cur, const ScaleRef& prev, int batch, int heads,
                             int head_dim, int dtype, int h_cur, int w_cur, int h_prev, int w_prev,
                             float* partial_ws, float* out_dev, hipStream_t st);

// the same with the partial sums in the library's static device array instead of partial_ws; batch * heads
// must not exceed AMSKV_STATIC_MAX_UNITS.  Calls no allocating routine.
hipError_t launch_similarity_static(const ScaleRef& cur, const ScaleRef& prev, int batch, int heads,
                                    int head_dim, int dtype, int h_cur, int w_cur, int h_prev, int w_prev,
                                    float* out_dev, hipStream_t st);

// attention density: pieces = one table entry per group of keys (nothing merged); partial_ws holds
// batch*heads*ceil(t_q/32)*AMSKV_MAX_SCALES floats, out_dev heads*AMSKV_MAX_SCALES floats
hipError_t launch_density(const void* q, const void* kc, int batch, int heads, int t_q, int head_dim, int dtype,
                          int64_t cap_tokens, const SegTable& pieces, const ExtKV& ext, const CallerIo& io,
                          float softmax_scale, float* partial_ws, float* out_dev, hipStream_t st);
// Algorithm 1's test decided on the device: *flag_dev = (mean over heads of totals_dev[h*4] / n_tok) < theta
hipError_t launch_theta_flag(const float* totals_dev, int heads, double n_tok, float theta, int32_t* flag_dev,
                             int32_t* flag_host_pinned, hipStream_t st);
// its second stage alone: out[h][p] = mean over the batch of the sum over the query blocks of partial_ws
hipError_t launch_density_total(const float* partial_ws, int batch, int heads, int n_qblk, int n_groups, float* out_dev,
                                hipStream_t st);

}  // namespace amskv
