// Inter-scale similarity (Eq. 3): scale s-1 is resized bilinearly to the grid of scale s on
// the fly (never materialised) and compared with scale s, straight from the cache.
// Bandwidth-bound: each token row is read with 16-byte loads by consecutive lanes.
// Reduction order is fixed (lanes of a token -> xor tree over a wave -> waves in order -> strided lanes and an xor tree over batch), so the
// result is deterministic from run to run.
#include "amskv_internal.hpp"

namespace amskv {
namespace {

constexpr int kThreads = 256;
constexpr int kStaticMaxUnits = AMSKV_STATIC_MAX_UNITS;
constexpr int kMaxDevices = 64;

template <bool BF16>
struct Chunk;  // one 16-byte piece of a token row, widened to fp32

template <>
struct Chunk<true> {
  static constexpr int N = 8;
  float v[8];
  __device__ __forceinline__ void load(const char* p) {
    const uint4 r = *reinterpret_cast<const uint4*>(p);
    const unsigned w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      v[2 * i] = __uint_as_float(w[i] << 16);
      v[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
  }
};

template <>
struct Chunk<false> {
  static constexpr int N = 4;
  float v[4];
  __device__ __forceinline__ void load(const char* p) {
    const float4 r = *reinterpret_cast<const float4*>(p);
    v[0] = r.x; v[1] = r.y; v[2] = r.z; v[3] = r.w;
  }
};

// Source coordinate of the bilinear resize with half-pixel centres, clamped to the grid.
__device__ __forceinline__ void taps(int dst, int n_in, int n_out, int& i0, int& i1, float& lam) {
  float src = ((float)dst + 0.5f) * ((float)n_in / (float)n_out) - 0.5f;
  src = fminf(fmaxf(src, 0.f), (float)(n_in - 1));
  const float f = floorf(src);
  i0 = (int)f;
  i1 = min(i0 + 1, n_in - 1);
  lam = src - f;
}

// grid: (B*H, tensors); one workgroup per (b,h) of one tensor (0 = keys, 1 = values).
// partial[(tensor*BH + bh)*4 + {0,1,2,3}] = sum_t cos_t, sum a.b, sum |a|^2, sum |b|^2.
template <bool BF16>
__global__ __launch_bounds__(kThreads) void similarity_partial_kernel(
    ScaleRef cur_ref, ScaleRef prev_ref, int row_bytes, int heads, int h_cur, int w_cur, int h_prev, int w_prev,
    float* __restrict__ partial) {
  const long long bh = blockIdx.x;
  const char* cur = (const char*)(blockIdx.y ? cur_ref.v : cur_ref.k) + unit_offset(cur_ref.map, bh, heads) +
                    cur_ref.off_tokens * cur_ref.map.tok;
  const char* prev = (const char*)(blockIdx.y ? prev_ref.v : prev_ref.k) + unit_offset(prev_ref.map, bh, heads) +
                     prev_ref.off_tokens * prev_ref.map.tok;
  const long long cur_tok = cur_ref.map.tok, prev_tok = prev_ref.map.tok;
  const int lpt = row_bytes >> 4;          // lanes per token: 8, 16 or 32
  const int sub = threadIdx.x % lpt;       // which 16-byte piece of the row
  const int slot = threadIdx.x / lpt;
  const int tok_per_pass = kThreads / lpt;
  const int t_cur = h_cur * w_cur;

  float acc_cos = 0.f, acc_ab = 0.f, acc_aa = 0.f, acc_bb = 0.f;
  for (int t0 = 0; t0 < t_cur; t0 += tok_per_pass) {
    const int t = t0 + slot;
    float ab = 0.f, aa = 0.f, bb = 0.f;
    if (t < t_cur) {
      const int i = t / w_cur, j = t - i * w_cur;
      int r0, r1, c0, c1;
      float lr, lc;
      taps(i, h_prev, h_cur, r0, r1, lr);
      taps(j, w_prev, w_cur, c0, c1, lc);
      Chunk<BF16> a, p00, p01, p10, p11;
      a.load(cur + t * cur_tok + (sub << 4));
      p00.load(prev + (r0 * w_prev + c0) * prev_tok + (sub << 4));
      p01.load(prev + (r0 * w_prev + c1) * prev_tok + (sub << 4));
      p10.load(prev + (r1 * w_prev + c0) * prev_tok + (sub << 4));
      p11.load(prev + (r1 * w_prev + c1) * prev_tok + (sub << 4));
#pragma unroll
      for (int e = 0; e < Chunk<BF16>::N; ++e) {
        const float left = p00.v[e] * (1.f - lr) + p10.v[e] * lr;    // rows first,
        const float right = p01.v[e] * (1.f - lr) + p11.v[e] * lr;
        const float b = left * (1.f - lc) + right * lc;              // then columns
        ab += a.v[e] * b;
        aa += a.v[e] * a.v[e];
        bb += b * b;
      }
    }
    // sum over the lanes that share a token (lpt is a power of two <= 32)
    for (int m = 1; m < lpt; m <<= 1) {
      ab += __shfl_xor(ab, m, 64);
      aa += __shfl_xor(aa, m, 64);
      bb += __shfl_xor(bb, m, 64);
    }
    if (sub == 0 && t < t_cur) {
      acc_cos += ab / fmaxf(sqrtf(aa) * sqrtf(bb), 1e-12f);
      acc_ab += ab;
      acc_aa += aa;
      acc_bb += bb;
    }
  }

  // workgroup sum in a fixed order: xor tree over the lanes of a wave, then the waves in ascending order
  float acc[4] = {acc_cos, acc_ab, acc_aa, acc_bb};
#pragma unroll
  for (int m = 32; m > 0; m >>= 1)
#pragma unroll
    for (int q = 0; q < 4; ++q) acc[q] += __shfl_xor(acc[q], m, 64);
  __shared__ float red[kThreads / 64][4];
  if ((threadIdx.x & 63) == 0)
    for (int q = 0; q < 4; ++q) red[threadIdx.x >> 6][q] = acc[q];
  __syncthreads();
  if (threadIdx.x < 4) {
    float total = red[0][threadIdx.x];
    for (int w = 1; w < kThreads / 64; ++w) total += red[w][threadIdx.x];
    partial[((long long)blockIdx.y * gridDim.x + bh) * 4 + threadIdx.x] = total;
  }
}

// totals[(tensor*H + h)*4 + q] = sum over b of partial[(tensor*B*H + b*H + h)*4 + q].
// One 64-lane workgroup per (tensor, h): lane i sums batch entries i, i+64, ... in ascending
// order, then a fixed xor tree joins the lanes -- the same order on every run.
__global__ __launch_bounds__(64) void similarity_total_kernel(const float* __restrict__ partial, int batch, int heads,
                                                              float* __restrict__ totals) {
  const int h = blockIdx.x % heads, tn = blockIdx.x / heads;
  float acc[4] = {0.f, 0.f, 0.f, 0.f};
  for (int b = threadIdx.x; b < batch; b += 64) {
    const float4 x = *reinterpret_cast<const float4*>(partial + (((long long)tn * batch + b) * heads + h) * 4);
    acc[0] += x.x; acc[1] += x.y; acc[2] += x.z; acc[3] += x.w;
  }
#pragma unroll
  for (int m = 32; m > 0; m >>= 1)
#pragma unroll
    for (int q = 0; q < 4; ++q) acc[q] += __shfl_xor(acc[q], m, 64);
  if (threadIdx.x == 0)
    *reinterpret_cast<float4*>(totals + ((long long)tn * heads + h) * 4) = make_float4(acc[0], acc[1], acc[2], acc[3]);
}

// Algorithm 1's test on the device: flag = (mean over heads of the mean cosine < theta), from the per-head sums the
// kernel above left (totals[h*4] = sum of the per-token cosines of K).  The arithmetic is spelled out so that the
// host, given the same sums, would decide the same: per head the quotient in double rounded to float, their mean
// in double, compared with theta in double.  One lane.
__global__ __launch_bounds__(64) void theta_flag_kernel(const float* __restrict__ totals, int heads, double n_tok, float theta,
                                                        int32_t* __restrict__ flag, int32_t* __restrict__ flag_host) {
  if (threadIdx.x != 0) return;
  double mean = 0.0;
  for (int h = 0; h < heads; ++h) mean += (double)(float)((double)totals[h * 4] / n_tok);
  mean /= heads;
  const int32_t word = mean < (double)theta ? 1 : 0;
  *flag = word;       // for the launch behind this one
  *flag_host = word;  // pinned host memory: the host reads it behind the event, no transfer
}

// Partial-sum workspace of the entry point that allocates nothing: per (tensor, b, h) four floats, for up to
// kStaticMaxUnits = batch * heads units and both tensors (512 KB).  Every device the library runs on holds its
// own copy for the life of the process.
__device__ __align__(256) float scratch[2 * kStaticMaxUnits * 4];

// Device address of `scratch` on the current device, looked up once per device (the array's name is only a
// host-side handle).
hipError_t scratch_address(float** out) {
  static float* address[kMaxDevices];
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  float* p = __atomic_load_n(&address[dev], __ATOMIC_ACQUIRE);
  if (!p) {
    e = hipGetSymbolAddress((void**)&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    __atomic_store_n(&address[dev], p, __ATOMIC_RELEASE);  // every caller looks up the same value
  }
  *out = p;
  return hipSuccess;
}

}  // namespace

hipError_t launch_similarity_static(const ScaleRef& cur, const ScaleRef& prev, int batch, int heads, int head_dim,
                                    int dtype, int h_cur, int w_cur, int h_prev, int w_prev, float* out_dev,
                                    hipStream_t st) {
  if ((long long)batch * heads > kStaticMaxUnits) return hipErrorInvalidValue;  // the caller checks first
  float* ws = nullptr;
  hipError_t e = scratch_address(&ws);
  if (e != hipSuccess) return e;
  // every partial sum the totals kernel reads is written by the partial kernel of the same call: nothing to clear
  return launch_similarity(cur, prev, batch, heads, head_dim, dtype, h_cur, w_cur, h_prev, w_prev, ws, out_dev, st);
}

hipError_t launch_similarity(const ScaleRef& cur, const ScaleRef& prev, int batch, int heads, int head_dim,
                             int dtype, int h_cur, int w_cur, int h_prev, int w_prev, float* partial_ws,
                             float* out_dev, hipStream_t st) {
  const int tensors = (cur.v && prev.v) ? 2 : 1;
  const int bh = batch * heads;
  dim3 grid(bh, tensors), block(kThreads);
  if (dtype == AMSKV_DTYPE_BF16) {
    hipLaunchKernelGGL(similarity_partial_kernel<true>, grid, block, 0, st, cur, prev, head_dim * 2, heads, h_cur,
                       w_cur, h_prev, w_prev, partial_ws);
  } else {
    hipLaunchKernelGGL(similarity_partial_kernel<false>, grid, block, 0, st, cur, prev, head_dim * 4, heads, h_cur,
                       w_cur, h_prev, w_prev, partial_ws);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(similarity_total_kernel, dim3(tensors * heads), dim3(64), 0, st, (const float*)partial_ws, batch,
                     heads, out_dev);
  return hipGetLastError();
}

hipError_t launch_theta_flag(const float* totals_dev, int heads, double n_tok, float theta, int32_t* flag_dev,
                             int32_t* flag_host_pinned, hipStream_t st) {
  hipLaunchKernelGGL(theta_flag_kernel, dim3(1), dim3(64), 0, st, totals_dev, heads, n_tok, theta, flag_dev, flag_host_pinned);
  return hipGetLastError();
}

}  // namespace amskv
