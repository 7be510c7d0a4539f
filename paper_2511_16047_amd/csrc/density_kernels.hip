// Attention density (Section 4.1): how much of the softmax mass of the queries of the scale being
// generated lands on each group of cached keys (a scale, or the cached part of one), per head.
// An analysis by-product, not part of the generation step: it needs the first product S = Q K~^T
// and the softmax statistics only, never V.
//
// One WAVE owns one unit = (b, h, block of 32 query rows), as in the coarse-scale attention
// kernel: K fragments go straight from memory into the A-operand registers of
// v_mfma_f32_32x32x16_bf16 (S^T = K Q^T, so a lane holds 16 keys of one query column).  The wave
// walks the groups one after the other with one running maximum; at the end of group p it parks
// (sum of exp over the group's keys, maximum at that moment) in LDS, and once the last group is
// done every parked sum is moved to the final maximum, normalised by their total, masked to the
// valid query rows and added up over the 32 query columns.  Everything is reduced in a fixed order:
// per-unit partial sums go to a workspace, a second kernel adds them per head.
#include "amskv_internal.hpp"

namespace amskv {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kWavesPerGroup = 4;

template <int D>
__global__ __launch_bounds__(64 * kWavesPerGroup) void density_partial_kernel(
    const __bf16* __restrict__ q, const char* __restrict__ kc, int t_q, long long cap_tokens, SegTable seg,
    ExtKV ext_kv, CallerIo io, float scale_log2e, int n_qblk, int n_units, float* __restrict__ partial) {
  constexpr int RB = D * 2;
  constexpr int KS = D / 16;
  __shared__ float park_sum[kWavesPerGroup][AMSKV_MAX_SCALES][64];
  __shared__ float park_max[kWavesPerGroup][AMSKV_MAX_SCALES][64];

  const int wave = threadIdx.x >> 6;
  const int lane = threadIdx.x & 63;
  const int unit = blockIdx.x * kWavesPerGroup + wave;
  if (unit >= n_units) return;  // waves are independent: nothing below synchronises across waves
  const int r = lane & 31, h = lane >> 5;
  const long long bh = unit / n_qblk;
  const int q_base = (unit % n_qblk) * 32;
  const char* kb = kc + bh * cap_tokens * RB;
  const char* xk = (const char*)ext_kv.k + unit_offset(io.kv, bh, io.heads);
  const char* q_unit = (const char*)q + unit_offset(io.q, bh, io.heads);

  bf16x8 qf[KS];
  {
    const int row = min(q_base + r, t_q - 1);  // rows past T_q re-read the last row and are masked at the end
#pragma unroll
    for (int t = 0; t < KS; ++t) qf[t] = *reinterpret_cast<const bf16x8*>(q_unit + row * io.q.tok + 32 * t + 16 * h);
  }

  float run_max = -INFINITY;
  for (int p = 0; p < seg.n; ++p) {
    const int len = seg.len[p];
    const int vs = seg.virt_start[p];
    const bool outside = vs >= seg.ext_start;  // the current scale, read in place from the caller's tensor
    const long long tok = outside ? io.kv.tok : (long long)RB;
    const char* base = outside ? xk + (vs - seg.ext_start) * tok : kb + (long long)seg.phys_off[p] * RB;
    float ssum = 0.f;
    for (int j0 = 0; j0 < len; j0 += 32) {
      const char* kp = base + min(j0 + r, len - 1) * tok + 16 * h;
      f32x16 sacc;
#pragma unroll
      for (int v = 0; v < 16; ++v) sacc[v] = 0.f;
#pragma unroll
      for (int t = 0; t < KS; ++t)
        sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<const bf16x8*>(kp + 32 * t), qf[t], sacc, 0, 0, 0);
      float mx = -INFINITY;
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        if (j0 + 8 * (v >> 2) + 4 * h + (v & 3) >= len) sacc[v] = -INFINITY;  // keys past the end of the group
        mx = fmaxf(mx, sacc[v]);
      }
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64));  // key j0 is always valid, so this is finite
      const float new_max = fmaxf(run_max, mx);
      const float mc = new_max * scale_log2e;
      float s = 0.f;
#pragma unroll
      for (int v = 0; v < 16; ++v) s += __builtin_amdgcn_exp2f(fmaf(sacc[v], scale_log2e, -mc));
      ssum = ssum * __builtin_amdgcn_exp2f((run_max - new_max) * scale_log2e) + s;
      run_max = new_max;
    }
    park_sum[wave][p][lane] = ssum;
    park_max[wave][p][lane] = run_max;
  }

  // every parked sum to the final maximum; the two lane halves hold different keys of the same query
  float total = 0.f;
  for (int p = 0; p < seg.n; ++p) {
    float w = park_sum[wave][p][lane] * __builtin_amdgcn_exp2f((park_max[wave][p][lane] - run_max) * scale_log2e);
    w += __shfl_xor(w, 32, 64);
    park_sum[wave][p][lane] = w;
    total += w;
  }
  const float inv = q_base + r < t_q ? 1.0f / total : 0.f;
  for (int p = 0; p < seg.n; ++p) {
    float m = park_sum[wave][p][lane] * inv;
#pragma unroll
    for (int d = 16; d >= 1; d >>= 1) m += __shfl_xor(m, d, 64);  // over the 32 query columns
    if (lane == 0) partial[(long long)unit * AMSKV_MAX_SCALES + p] = m;
  }
}

// The same quantity for fp32 caches, on the vector ALUs (the fp32 path is the reference-precision path, not a
// tuned one): same units, same parking scheme, so workspace and second kernel are shared.  A lane keeps its
// query row in registers and takes every second key of a group (keys j = h mod 2); K rows are read as
// 16-byte chunks that all lanes of a half share.  Each lane runs its own online softmax; the two halves of
// a query meet only at the end.
template <int D>
__global__ __launch_bounds__(64 * kWavesPerGroup) void density_partial_f32_kernel(
    const float* __restrict__ q, const char* __restrict__ kc, int t_q, long long cap_tokens, SegTable seg,
    ExtKV ext_kv, CallerIo io, float scale_log2e, int n_qblk, int n_units, float* __restrict__ partial) {
  constexpr int RB = D * 4;
  __shared__ float park_sum[kWavesPerGroup][AMSKV_MAX_SCALES][64];
  __shared__ float park_max[kWavesPerGroup][AMSKV_MAX_SCALES][64];

  const int wave = threadIdx.x >> 6;
  const int lane = threadIdx.x & 63;
  const int unit = blockIdx.x * kWavesPerGroup + wave;
  if (unit >= n_units) return;
  const int r = lane & 31, h = lane >> 5;
  const long long bh = unit / n_qblk;
  const int q_base = (unit % n_qblk) * 32;
  const char* kb = kc + bh * cap_tokens * RB;
  const char* xk = (const char*)ext_kv.k + unit_offset(io.kv, bh, io.heads);
  const char* q_unit = (const char*)q + unit_offset(io.q, bh, io.heads);

  float4 qr[D / 4];
  {
    const int row = min(q_base + r, t_q - 1);
#pragma unroll
    for (int d = 0; d < D / 4; ++d) qr[d] = *reinterpret_cast<const float4*>(q_unit + row * io.q.tok + 16 * d);
  }

  float run_max = -INFINITY;  // of the keys this lane has seen
  for (int p = 0; p < seg.n; ++p) {
    const int len = seg.len[p];
    const int vs = seg.virt_start[p];
    const bool outside = vs >= seg.ext_start;
    const long long tok = outside ? io.kv.tok : (long long)RB;
    const char* base = outside ? xk + (vs - seg.ext_start) * tok : kb + (long long)seg.phys_off[p] * RB;
    float ssum = 0.f;
    for (int j = h; j < len; j += 2) {
      const float4* kp = reinterpret_cast<const float4*>(base + j * tok);
      float dot = 0.f;
#pragma unroll
      for (int d = 0; d < D / 4; ++d) {
        const float4 kk = kp[d];
        dot = fmaf(qr[d].x, kk.x, dot);
        dot = fmaf(qr[d].y, kk.y, dot);
        dot = fmaf(qr[d].z, kk.z, dot);
        dot = fmaf(qr[d].w, kk.w, dot);
      }
      const float new_max = fmaxf(run_max, dot);
      ssum = ssum * __builtin_amdgcn_exp2f((run_max - new_max) * scale_log2e) +
             __builtin_amdgcn_exp2f((dot - new_max) * scale_log2e);
      run_max = new_max;
    }
    park_sum[wave][p][lane] = ssum;  // 0 with a maximum of -inf while this half has seen no key
    park_max[wave][p][lane] = run_max;
  }

  const float top = fmaxf(run_max, __shfl_xor(run_max, 32, 64));  // finite: key 0 belongs to half 0
  float total = 0.f;
  for (int p = 0; p < seg.n; ++p) {
    float w = park_sum[wave][p][lane] * __builtin_amdgcn_exp2f((park_max[wave][p][lane] - top) * scale_log2e);
    w += __shfl_xor(w, 32, 64);
    park_sum[wave][p][lane] = w;
    total += w;
  }
  const float inv = q_base + r < t_q ? 1.0f / total : 0.f;
  for (int p = 0; p < seg.n; ++p) {
    float m = park_sum[wave][p][lane] * inv;
#pragma unroll
    for (int d = 16; d >= 1; d >>= 1) m += __shfl_xor(m, d, 64);
    if (lane == 0) partial[(long long)unit * AMSKV_MAX_SCALES + p] = m;
  }
}

// out[h][p] = (1/B) * sum over batch and query blocks of partial[(b,h), block][p], fixed order:
// thread = p + 16*part walks every kParts-th unit of the head, four independent sums at a time (the loads are
// what the kernel waits for), then a tree over the parts in LDS.
constexpr int kParts = 64;
__global__ __launch_bounds__(16 * kParts) void density_total_kernel(const float* __restrict__ partial, int batch,
                                                                    int heads, int n_qblk, int n_seg,
                                                                    float* __restrict__ out) {
  __shared__ float red[kParts][16];
  const int hd = blockIdx.x;
  const int p = threadIdx.x & 15, part = threadIdx.x >> 4;
  float acc[4] = {0.f, 0.f, 0.f, 0.f};
  if (p < n_seg) {
    const int per_head = batch * n_qblk;
    auto at = [&](int i) {
      const int b = i / n_qblk, blk = i - b * n_qblk;
      return partial[(((long long)b * heads + hd) * n_qblk + blk) * AMSKV_MAX_SCALES + p];
    };
    int i = part;
    for (; i + 3 * kParts < per_head; i += 4 * kParts) {
      acc[0] += at(i);
      acc[1] += at(i + kParts);
      acc[2] += at(i + 2 * kParts);
      acc[3] += at(i + 3 * kParts);
    }
    for (; i < per_head; i += kParts) acc[0] += at(i);
  }
  red[part][p] = (acc[0] + acc[1]) + (acc[2] + acc[3]);
  __syncthreads();
  for (int m = kParts / 2; m > 0; m >>= 1) {
    if (part < m) red[part][p] += red[part + m][p];
    __syncthreads();
  }
  if (part == 0) out[hd * AMSKV_MAX_SCALES + p] = p < n_seg ? red[0][p] / (float)batch : 0.f;
}

}  // namespace

hipError_t launch_density(const void* q, const void* kc, int batch, int heads, int t_q, int head_dim, int dtype,
                          int64_t cap_tokens, const SegTable& pieces, const ExtKV& ext, const CallerIo& io,
                          float softmax_scale, float* partial_ws, float* out_dev, hipStream_t st) {
  const float c = softmax_scale * 1.4426950408889634f;
  const int n_qblk = (t_q + 31) / 32;
  const long long n_units = (long long)batch * heads * n_qblk;
  dim3 grid((unsigned)((n_units + kWavesPerGroup - 1) / kWavesPerGroup)), block(64 * kWavesPerGroup);
  if (dtype == AMSKV_DTYPE_F32 && head_dim == 64)
    hipLaunchKernelGGL(density_partial_f32_kernel<64>, grid, block, 0, st, (const float*)q, (const char*)kc, t_q,
                       (long long)cap_tokens, pieces, ext, io, c, n_qblk, (int)n_units, partial_ws);
  else if (dtype == AMSKV_DTYPE_F32)
    hipLaunchKernelGGL(density_partial_f32_kernel<128>, grid, block, 0, st, (const float*)q, (const char*)kc, t_q,
                       (long long)cap_tokens, pieces, ext, io, c, n_qblk, (int)n_units, partial_ws);
  else if (head_dim == 64)
    hipLaunchKernelGGL(density_partial_kernel<64>, grid, block, 0, st, (const __bf16*)q, (const char*)kc, t_q,
                       (long long)cap_tokens, pieces, ext, io, c, n_qblk, (int)n_units, partial_ws);
  else
    hipLaunchKernelGGL(density_partial_kernel<128>, grid, block, 0, st, (const __bf16*)q, (const char*)kc, t_q,
                       (long long)cap_tokens, pieces, ext, io, c, n_qblk, (int)n_units, partial_ws);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  return launch_density_total(partial_ws, batch, heads, n_qblk, pieces.n, out_dev, st);
}

hipError_t launch_density_total(const float* partial_ws, int batch, int heads, int n_qblk, int n_groups, float* out_dev,
                                hipStream_t st) {
  hipLaunchKernelGGL(density_total_kernel, dim3(heads), dim3(16 * kParts), 0, st, partial_ws, batch, heads, n_qblk, n_groups,
                     out_dev);
  return hipGetLastError();
}

}  // namespace amskv
