// fp32 per-scale attention over the resident segments (Section 3.1: the queries of scale s
// attend to the cached scales and to their own scale; no mask inside a step).
// Flash-style single pass: K/V tiles staged in LDS, online softmax, everything in fp32 on
// the vector ALUs.  Four lanes share one query row (each owns a quarter of the head dim),
// so a wave covers 16 rows and all LDS reads of a K or V row are 64-byte broadcasts.
#include "amskv_internal.hpp"

namespace amskv {
namespace {

constexpr int kThreads = 256;
constexpr int kRowsPerBlock = kThreads / 4;  // 64 query rows
constexpr int kTileKeys = 32;

template <int D>
__global__ __launch_bounds__(kThreads) void attend_f32_kernel(const float* __restrict__ q,
                                                              float* __restrict__ o,
                                                              float* __restrict__ kc,
                                                              float* __restrict__ vc, int t_q,
                                                              long long cap_tokens, SegTable seg,
                                                              ExtKV ext_kv, CallerIo io, float scale_log2e) {
  constexpr int M = D / 16;  // float4 pieces per lane
  __shared__ __align__(16) float lds_k[kTileKeys * D];
  __shared__ __align__(16) float lds_v[kTileKeys * D];

  const int tid = threadIdx.x;
  const int g = tid & 3;
  const long long bh = blockIdx.x;
  const int row = blockIdx.y * kRowsPerBlock + (tid >> 2);
  const bool row_ok = row < t_q;
  float* kb = kc + bh * cap_tokens * D;
  float* vb = vc + bh * cap_tokens * D;
  const long long x_unit = unit_offset(io.kv, bh, io.heads);  // borrowed current scale, if any
  const char* xk = (const char*)ext_kv.k + x_unit;
  const char* xv = (const char*)ext_kv.v + x_unit;
  const char* q_row = (const char*)q + unit_offset(io.q, bh, io.heads) + (long long)row * io.q.tok;
  char* o_row = (char*)o + unit_offset(io.o, bh, io.heads) + (long long)row * io.o.tok;
  const int t_kv = seg.total;

  float4 qv[M], acc[M];
#pragma unroll
  for (int m = 0; m < M; ++m) {
    qv[m] = row_ok ? *reinterpret_cast<const float4*>(q_row + 4 * (16 * m + 4 * g))
                   : make_float4(0.f, 0.f, 0.f, 0.f);
    acc[m] = make_float4(0.f, 0.f, 0.f, 0.f);
  }
  float run_max = -INFINITY, run_sum = 0.f;

  for (int j0 = 0; j0 < t_kv; j0 += kTileKeys) {
    __syncthreads();
    // stage the tile: virtual row -> physical row through the segment table
    for (int id = tid; id < kTileKeys * (D / 4); id += kThreads) {
      const int r = id / (D / 4), c = id - r * (D / 4);
      const int j = j0 + r;
      float4 kk = make_float4(0.f, 0.f, 0.f, 0.f), vv = kk;
      if (j < t_kv) {
        bool ext;
        const long long at = locate_row(seg, j, ext);
        const long long off = at * D + 4 * c;
        if (ext) {
          kk = *reinterpret_cast<const float4*>(xk + at * io.kv.tok + 16 * c);
          vv = *reinterpret_cast<const float4*>(xv + at * io.kv.tok + 16 * c);
        } else {
          kk = *reinterpret_cast<const float4*>(kb + off);
          vv = *reinterpret_cast<const float4*>(vb + off);
        }
        const int to = write_back_row(ext_kv, j, t_kv, seg.ext_start);
        if (ext && to >= 0 && blockIdx.y == 0) {  // fused append: fill the scale's slot while streaming it
          const long long dst = (long long)to * D + 4 * c;
          *reinterpret_cast<float4*>(kb + dst) = kk;
          *reinterpret_cast<float4*>(vb + dst) = vv;
        }
      }
      *reinterpret_cast<float4*>(lds_k + r * D + 4 * c) = kk;
      *reinterpret_cast<float4*>(lds_v + r * D + 4 * c) = vv;
    }
    __syncthreads();

    float sc[kTileKeys];
    float tile_max = -INFINITY;
#pragma unroll
    for (int jj = 0; jj < kTileKeys; ++jj) {
      float part = 0.f;
#pragma unroll
      for (int m = 0; m < M; ++m) {
        const float4 kk = *reinterpret_cast<const float4*>(lds_k + jj * D + 16 * m + 4 * g);
        part += qv[m].x * kk.x + qv[m].y * kk.y + qv[m].z * kk.z + qv[m].w * kk.w;
      }
      part += __shfl_xor(part, 1, 64);
      part += __shfl_xor(part, 2, 64);
      sc[jj] = (j0 + jj < t_kv) ? part : -INFINITY;
      tile_max = fmaxf(tile_max, sc[jj]);
    }
    const float new_max = fmaxf(run_max, tile_max);
    const float alpha = __builtin_amdgcn_exp2f((run_max - new_max) * scale_log2e);
    const float mc = new_max * scale_log2e;
    float tile_sum = 0.f;
#pragma unroll
    for (int m = 0; m < M; ++m) {
      acc[m].x *= alpha; acc[m].y *= alpha; acc[m].z *= alpha; acc[m].w *= alpha;
    }
#pragma unroll
    for (int jj = 0; jj < kTileKeys; ++jj) {
      const float p = __builtin_amdgcn_exp2f(fmaf(sc[jj], scale_log2e, -mc));
      tile_sum += p;
#pragma unroll
      for (int m = 0; m < M; ++m) {
        const float4 vv = *reinterpret_cast<const float4*>(lds_v + jj * D + 16 * m + 4 * g);
        acc[m].x = fmaf(p, vv.x, acc[m].x);
        acc[m].y = fmaf(p, vv.y, acc[m].y);
        acc[m].z = fmaf(p, vv.z, acc[m].z);
        acc[m].w = fmaf(p, vv.w, acc[m].w);
      }
    }
    run_sum = run_sum * alpha + tile_sum;
    run_max = new_max;
  }

  if (row_ok) {
    const float inv = 1.0f / run_sum;
#pragma unroll
    for (int m = 0; m < M; ++m) {
      float4 r = make_float4(acc[m].x * inv, acc[m].y * inv, acc[m].z * inv, acc[m].w * inv);
      *reinterpret_cast<float4*>(o_row + 4 * (16 * m + 4 * g)) = r;
    }
  }
}

}  // namespace

hipError_t launch_attend_f32(const void* q, void* o, void* kc, void* vc, int bh, int t_q,
                             int head_dim, int64_t cap_tokens, const SegTable& seg, const ExtKV& ext,
                             const CallerIo& io, float softmax_scale, hipStream_t st) {
  const float c = softmax_scale * 1.4426950408889634f;
  dim3 grid(bh, (t_q + kRowsPerBlock - 1) / kRowsPerBlock), block(kThreads);
  if (head_dim == 64)
    hipLaunchKernelGGL(attend_f32_kernel<64>, grid, block, 0, st, (const float*)q, (float*)o, (float*)kc,
                       (float*)vc, t_q, (long long)cap_tokens, seg, ext, io, c);
  else
    hipLaunchKernelGGL(attend_f32_kernel<128>, grid, block, 0, st, (const float*)q, (float*)o, (float*)kc,
                       (float*)vc, t_q, (long long)cap_tokens, seg, ext, io, c);
  return hipGetLastError();
}

}  // namespace amskv
