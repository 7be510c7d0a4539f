// Bandwidth-bound cache kernels: evict + compact + append (Algorithm 1's append and rolling
// step, Algorithm 2's eviction, at scale granularity) and the read-back export.
// All traffic is 16-byte vector loads/stores, consecutive lanes on consecutive chunks.
#include "amskv_internal.hpp"

namespace amskv {
namespace {

constexpr int kThreads = 256;
constexpr int kUnroll = 4;  // 16-byte chunks in flight per thread and pass

__device__ __forceinline__ void wait_all_vector_loads() {
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
}

// Eviction in the COMPACT layout: one workgroup owns one (b,h) row of one tensor (blockIdx.y:
// 0 = K, 1 = V) and slides the surviving segments toward offset 0.  The moved chunks, taken in
// ascending address order, have strictly increasing source and destination addresses with
// dst < src, so a pass that first loads all of its chunks, waits for the data, meets at a
// barrier and only then stores can never overwrite a chunk that a later pass still has to
// read: a store to address X can only alias the source of an EARLIER chunk.
__global__ __launch_bounds__(kThreads) void compact_kernel(char* __restrict__ kc, char* __restrict__ vc,
                                                           int row_bytes, long long cap_tokens, MoveList mv) {
  const int tid = threadIdx.x;
  const long long bh = blockIdx.x;
  char* base = (blockIdx.y ? vc : kc) + bh * cap_tokens * row_bytes;
  const int cpr = row_bytes >> 4;  // chunks per token row

  int total = 0;
  for (int i = 0; i < mv.n; ++i) total += mv.len[i] * cpr;

  for (int c0 = 0; c0 < total; c0 += kThreads * kUnroll) {
    uint4 buf[kUnroll];
    long long dst_byte[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const int c = c0 + u * kThreads + tid;
      dst_byte[u] = -1;
      if (c < total) {
        int rem = c, src_tok = 0, dst_tok = 0;
        for (int i = 0; i < mv.n; ++i) {
          const int n = mv.len[i] * cpr;
          if (rem < n) {
            src_tok = mv.src[i];
            dst_tok = mv.dst[i];
            break;
          }
          rem -= n;
        }
        const long long so = (long long)src_tok * row_bytes + ((long long)rem << 4);
        dst_byte[u] = (long long)dst_tok * row_bytes + ((long long)rem << 4);
        buf[u] = *reinterpret_cast<const uint4*>(base + so);
      }
    }
    wait_all_vector_loads();
    __syncthreads();
#pragma unroll
    for (int u = 0; u < kUnroll; ++u)
      if (dst_byte[u] >= 0) *reinterpret_cast<uint4*>(base + dst_byte[u]) = buf[u];
  }
}

// Token-granular iteration of Algorithm 1 in one launch: the moves of compact_kernel, then -- the workgroup owns the
// row, and behind the last pass's barrier every moved chunk has been read -- the kept ranges of the new scale
// are copied from the caller's tensor to their place behind the survivors (which may overlap where a survivor
// used to be).
__global__ __launch_bounds__(kThreads) void roll_kernel(char* __restrict__ kc, char* __restrict__ vc,
                                                        const char* __restrict__ k_new, const char* __restrict__ v_new,
                                                        int row_bytes, long long cap_tokens, MoveList mv, NewRanges nr,
                                                        RowMap src_map, int heads) {
  const int tid = threadIdx.x;
  const long long bh = blockIdx.x;
  char* base = (blockIdx.y ? vc : kc) + bh * cap_tokens * row_bytes;
  const int cpr = row_bytes >> 4;

  int total = 0;
  for (int i = 0; i < mv.n; ++i) total += mv.len[i] * cpr;
  for (int c0 = 0; c0 < total; c0 += kThreads * kUnroll) {
    uint4 buf[kUnroll];
    long long dst_byte[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const int c = c0 + u * kThreads + tid;
      dst_byte[u] = -1;
      if (c < total) {
        int rem = c, src_tok = 0, dst_tok = 0;
        for (int i = 0; i < mv.n; ++i) {
          const int n = mv.len[i] * cpr;
          if (rem < n) {
            src_tok = mv.src[i];
            dst_tok = mv.dst[i];
            break;
          }
          rem -= n;
        }
        const long long so = (long long)src_tok * row_bytes + ((long long)rem << 4);
        dst_byte[u] = (long long)dst_tok * row_bytes + ((long long)rem << 4);
        buf[u] = *reinterpret_cast<const uint4*>(base + so);
      }
    }
    wait_all_vector_loads();
    __syncthreads();
#pragma unroll
    for (int u = 0; u < kUnroll; ++u)
      if (dst_byte[u] >= 0) *reinterpret_cast<uint4*>(base + dst_byte[u]) = buf[u];
  }
  if (total > 0) __syncthreads();  // the copies below may overwrite sources of the last pass

  const char* src = (blockIdx.y ? v_new : k_new) + unit_offset(src_map, bh, heads);
#pragma unroll
  for (int r = 0; r < 2; ++r) {
    const int n = r < nr.n ? nr.len[r] * cpr : 0;
    const char* from = src + (long long)nr.src_first[r] * src_map.tok;
    char* to = base + (long long)nr.dst[r] * row_bytes;
#pragma unroll 4
    for (int c = tid; c < n; c += kThreads) {
      const int tok = c / cpr;
      *reinterpret_cast<uint4*>(to + ((long long)c << 4)) =
          *reinterpret_cast<const uint4*>(from + (long long)tok * src_map.tok + ((c - tok * cpr) << 4));
    }
  }
}

// Append: copy t_new tokens of the new scale K_s, V_s (the caller's tensors, rows located by
// src_map, starting at token src_first of every (b,h)) into their slot of every (b,h) row of the
// cache.  Flat over all 16-byte chunks of both tensors, so a one-token scale and a 256-token scale
// both run full workgroups; for a whole head-major scale the source side is one contiguous stream.  The token-granular trim of Algorithm 2 keeps a scale in part, hence the range.
// Enqueued after compact_kernel: the slot may overlap the old position of a moved segment.
__global__ __launch_bounds__(kThreads) void append_kernel(char* __restrict__ kc, char* __restrict__ vc,
                                                          const char* __restrict__ k_new,
                                                          const char* __restrict__ v_new, int row_bytes,
                                                          long long cap_tokens, int t_new, int dst_new,
                                                          int src_first, RowMap src_map, int heads,
                                                          long long chunks_per_tensor) {
  const int cpr = row_bytes >> 4;
  const int per_bh = t_new * cpr;  // chunks of one (b,h) row
  const long long first = (long long)blockIdx.x * (kThreads * kUnroll) + threadIdx.x;
  uint4 buf[kUnroll];
  long long dst_off[kUnroll];
  int which[kUnroll];
#pragma unroll
  for (int u = 0; u < kUnroll; ++u) {
    long long c = first + (long long)u * kThreads;
    which[u] = -1;
    if (c < 2 * chunks_per_tensor) {
      which[u] = c >= chunks_per_tensor;
      if (which[u]) c -= chunks_per_tensor;
      const long long bh = c / per_bh;
      const int rem = (int)(c - bh * per_bh);
      dst_off[u] = (bh * cap_tokens + dst_new) * row_bytes + ((long long)rem << 4);
      const int tok = rem / cpr;
      const long long so = unit_offset(src_map, bh, heads) + (src_first + tok) * src_map.tok + ((rem - tok * cpr) << 4);
      buf[u] = *reinterpret_cast<const uint4*>((which[u] ? v_new : k_new) + so);
    }
  }
#pragma unroll
  for (int u = 0; u < kUnroll; ++u)
    if (which[u] >= 0) *reinterpret_cast<uint4*>((which[u] ? vc : kc) + dst_off[u]) = buf[u];
}

// Gather the resident segments, ascending and back to back, into [BH][T_kept][row].
__global__ __launch_bounds__(kThreads) void export_kernel(const char* __restrict__ kc,
                                                          const char* __restrict__ vc, char* __restrict__ k_out,
                                                          char* __restrict__ v_out, int row_bytes,
                                                          long long cap_tokens, SegTable seg, ExtKV ext_kv,
                                                          RowMap ext_map, int heads) {
  const long long bh = blockIdx.x;
  const char* base = (blockIdx.y ? vc : kc) + bh * cap_tokens * row_bytes;
  const char* xbase = (const char*)(blockIdx.y ? ext_kv.v : ext_kv.k) + unit_offset(ext_map, bh, heads);
  char* out = blockIdx.y ? v_out : k_out;
  if (!out) return;
  out += bh * (long long)seg.total * row_bytes;
  const int cpr = row_bytes >> 4;
  const int n = seg.total * cpr;
  for (int c = threadIdx.x; c < n; c += kThreads) {
    const int tok = c / cpr, piece = c - tok * cpr;
    bool ext;
    const long long at = locate_row(seg, tok, ext);
    const char* src = ext ? xbase + at * ext_map.tok : base + at * row_bytes;
    *reinterpret_cast<uint4*>(out + ((long long)c << 4)) = *reinterpret_cast<const uint4*>(src + (piece << 4));
  }
}

}  // namespace

hipError_t launch_append(void* kc, void* vc, const void* k_new, const void* v_new, int bh, int row_bytes,
                         int64_t cap_tokens, const MoveList& mv, int t_new, int dst_new, int src_first,
                         const RowMap& src_map, int heads, hipStream_t st) {
  if (mv.n > 0) {
    hipLaunchKernelGGL(compact_kernel, dim3(bh, 2), dim3(kThreads), 0, st, (char*)kc, (char*)vc, row_bytes,
                       (long long)cap_tokens, mv);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  if (!k_new || t_new <= 0) return hipSuccess;  // borrowed scale: compaction only
  const long long chunks = (long long)bh * t_new * (row_bytes >> 4);
  const long long per_block = (long long)kThreads * kUnroll;
  const unsigned grid = (unsigned)((2 * chunks + per_block - 1) / per_block);
  hipLaunchKernelGGL(append_kernel, dim3(grid), dim3(kThreads), 0, st, (char*)kc, (char*)vc, (const char*)k_new,
                     (const char*)v_new, row_bytes, (long long)cap_tokens, t_new, dst_new, src_first, src_map, heads,
                     chunks);
  return hipGetLastError();
}

hipError_t launch_roll(void* kc, void* vc, const void* k_new, const void* v_new, int bh, int row_bytes,
                       int64_t cap_tokens, const MoveList& mv, const NewRanges& nr, const RowMap& src_map, int heads,
                       hipStream_t st) {
  hipLaunchKernelGGL(roll_kernel, dim3(bh, 2), dim3(kThreads), 0, st, (char*)kc, (char*)vc, (const char*)k_new,
                     (const char*)v_new, row_bytes, (long long)cap_tokens, mv, nr, src_map, heads);
  return hipGetLastError();
}

hipError_t launch_export(const void* kc, const void* vc, void* k_out, void* v_out, int bh, int row_bytes,
                         int64_t cap_tokens, const SegTable& seg, const ExtKV& ext, const RowMap& ext_map, int heads,
                         hipStream_t st) {
  dim3 grid(bh, 2), block(kThreads);
  hipLaunchKernelGGL(export_kernel, grid, block, 0, st, (const char*)kc, (const char*)vc, (char*)k_out,
                     (char*)v_out, row_bytes, (long long)cap_tokens, seg, ext, ext_map, heads);
  return hipGetLastError();
}

}  // namespace amskv
