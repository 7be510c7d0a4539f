// bf16 per-scale attention over the resident segments (Section 3.1: the queries of scale s
// attend to the cached scales and to their own scale; no mask inside a step), written for
// gfx950: 64-lane wavefronts, v_mfma_f32_32x32x16_bf16, LDS-staged K/V tiles, transposing LDS
// reads for the V operand, online softmax with fp32 statistics.
//
// Formulation.  One workgroup of four waves owns all (<= 128*NQ) query rows of a (b,h) tile, so
// K~ and V~ stream from HBM once per tile.  Each wave owns 32*NQ query rows and keeps their Q
// fragments in registers for the whole kernel.  Per 64-key tile it computes the TRANSPOSED
// score block S^T = K Q^T (M = keys, N = queries): in the 32x32 accumulator layout every lane
// then holds 16 keys of ONE query (column = lane%32), so the row max / row sum of the softmax
// are in-lane reductions plus a single exchange between the two lane halves, and the
// probabilities are already in the register layout the second product needs as its B operand:
// O^T += V^T P^T (M = head dim, K = keys, N = queries).  P never touches LDS.
//
// The accumulator row held in slot v of lane l is 8*(v/4) + 4*(l/32) + v%4, so the 8 values a
// lane packs for one K-step of the second product belong to keys base+4h+{0..3} and
// base+8+4h+{0..3} (h = lane/32).  The A operand V^T is fetched to match with two
// ds_read_b64_tr_b16 per K-step: within each group of 16 lanes, lane i supplies the address of
// 4 consecutive head-dim elements of key (i/4) at column group (i%4), and receives the four keys'
// values of column i -- exactly a 4x16 -> 16x4 transpose, so V stays row-major in LDS.
//
// LDS rows are XOR-swizzled at 16-byte granularity (chunk ^= row & 7) so that the 16-byte K
// fragment reads of 32 consecutive rows spread over all banks.
#include "amskv_internal.hpp"

namespace amskv {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kThreads = 256;
constexpr int kWaves = 4;
constexpr int kTileKeys = 64;

#define AMSKV_LDS __attribute__((address_space(3)))

__device__ __forceinline__ bf16x4 lds_read_tr16(const char* p) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4bf16((AMSKV_LDS bf16x4*)(p));
}

template <int D, int NQ>
__global__ __launch_bounds__(kThreads) void attend_bf16_kernel(const __bf16* __restrict__ q,
                                                               __bf16* __restrict__ o,
                                                               const char* __restrict__ kc,
                                                               const char* __restrict__ vc, int t_q,
                                                               long long cap_tokens, SegTable seg,
                                                               float scale_log2e) {
  constexpr int RB = D * 2;       // bytes per token row
  constexpr int CPR = D / 8;      // 16-byte chunks per row
  constexpr int KS = D / 16;      // K-steps of the first product
  constexpr int DB = D / 32;      // 32-row blocks of O^T
  constexpr int BM = kWaves * 32 * NQ;

  __shared__ __align__(16) char lds_k[kTileKeys * RB];
  __shared__ __align__(16) char lds_v[kTileKeys * RB];

  const int tid = threadIdx.x;
  const int wave = tid >> 6;
  const int lane = tid & 63;
  const int r = lane & 31;        // column (query) / row (key or head-dim) index inside a block
  const int h = lane >> 5;        // which half of the K-step this lane feeds
  const long long bh = blockIdx.x;
  const int q_base = blockIdx.y * BM + wave * (32 * NQ);
  const bool wave_active = q_base < t_q;
  const int t_kv = seg.total;
  const char* kb = kc + bh * cap_tokens * RB;
  const char* vb = vc + bh * cap_tokens * RB;

  // Q fragments: B operand of S^T = K Q^T; lane (r,h) holds Q[row r][16t + 8h .. +8)
  bf16x8 qf[NQ][KS];
#pragma unroll
  for (int n = 0; n < NQ; ++n) {
    const int row = q_base + 32 * n + r;
#pragma unroll
    for (int t = 0; t < KS; ++t) {
      if (row < t_q) {
        qf[n][t] = *reinterpret_cast<const bf16x8*>(q + (bh * t_q + row) * D + 16 * t + 8 * h);
      } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) qf[n][t][e] = (__bf16)0.f;
      }
    }
  }

  f32x16 oacc[NQ][DB];
#pragma unroll
  for (int n = 0; n < NQ; ++n)
#pragma unroll
    for (int d = 0; d < DB; ++d)
#pragma unroll
      for (int v = 0; v < 16; ++v) oacc[n][d][v] = 0.f;
  float run_max[NQ], run_sum[NQ];
#pragma unroll
  for (int n = 0; n < NQ; ++n) {
    run_max[n] = -INFINITY;
    run_sum[n] = 0.f;
  }

  // lane-constant pieces of the transposing V read (see header comment)
  const int tr_key = 4 * h + ((lane & 15) >> 2);               // + K-step base (+8 for the second read)
  const int tr_col = 16 * ((lane >> 4) & 1) + 4 * (lane & 3);  // + 32*db

  for (int j0 = 0; j0 < t_kv; j0 += kTileKeys) {
    __syncthreads();
    // stage K and V rows j0 .. j0+63 of the virtual concatenation; rows past the end are zero
#pragma unroll
    for (int id = tid; id < kTileKeys * CPR; id += kThreads) {
      const int row = id / CPR, c = id % CPR;
      const int j = j0 + row;
      uint4 kk = make_uint4(0, 0, 0, 0), vv = kk;
      if (j < t_kv) {
        int delta = 0;
        for (int i = 0; i < seg.n; ++i)
          if (j >= seg.virt_start[i]) delta = seg.phys_off[i] - seg.virt_start[i];
        const long long off = (long long)(j + delta) * RB + 16 * c;
        kk = *reinterpret_cast<const uint4*>(kb + off);
        vv = *reinterpret_cast<const uint4*>(vb + off);
      }
      const int lo = row * RB + 16 * (c ^ (row & 7));
      *reinterpret_cast<uint4*>(lds_k + lo) = kk;
      *reinterpret_cast<uint4*>(lds_v + lo) = vv;
    }
    __syncthreads();
    if (!wave_active) continue;

    // ---- S^T = K Q^T for two 32-key blocks
    f32x16 sacc[NQ][2];
#pragma unroll
    for (int n = 0; n < NQ; ++n)
#pragma unroll
      for (int kbk = 0; kbk < 2; ++kbk)
#pragma unroll
        for (int v = 0; v < 16; ++v) sacc[n][kbk][v] = 0.f;
#pragma unroll
    for (int kbk = 0; kbk < 2; ++kbk) {
      const int row = 32 * kbk + r;
#pragma unroll
      for (int t = 0; t < KS; ++t) {
        const bf16x8 a = *reinterpret_cast<const bf16x8*>(lds_k + row * RB + 16 * ((2 * t + h) ^ (row & 7)));
#pragma unroll
        for (int n = 0; n < NQ; ++n)
          sacc[n][kbk] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[n][t], sacc[n][kbk], 0, 0, 0);
      }
    }
    if (j0 + kTileKeys > t_kv) {  // ragged tail: keys past the end get zero weight
#pragma unroll
      for (int kbk = 0; kbk < 2; ++kbk)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int key = j0 + 32 * kbk + 8 * (v >> 2) + 4 * h + (v & 3);
          if (key >= t_kv) {
#pragma unroll
            for (int n = 0; n < NQ; ++n) sacc[n][kbk][v] = -INFINITY;
          }
        }
    }

    // ---- online softmax; probabilities packed as B operands of the second product
    bf16x8 pf[NQ][2][2];
#pragma unroll
    for (int n = 0; n < NQ; ++n) {
      float mx = -INFINITY;
#pragma unroll
      for (int kbk = 0; kbk < 2; ++kbk)
#pragma unroll
        for (int v = 0; v < 16; ++v) mx = fmaxf(mx, sacc[n][kbk][v]);
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
      const float new_max = fmaxf(run_max[n], mx);
      const float alpha = __builtin_amdgcn_exp2f((run_max[n] - new_max) * scale_log2e);
      const float mc = new_max * scale_log2e;
      float sum = 0.f;
#pragma unroll
      for (int kbk = 0; kbk < 2; ++kbk)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const float p = __builtin_amdgcn_exp2f(fmaf(sacc[n][kbk][v], scale_log2e, -mc));
          sum += p;
          pf[n][kbk][v >> 3][v & 7] = (__bf16)p;
        }
      run_sum[n] = run_sum[n] * alpha + sum;
      run_max[n] = new_max;
#pragma unroll
      for (int d = 0; d < DB; ++d)
#pragma unroll
        for (int v = 0; v < 16; ++v) oacc[n][d][v] *= alpha;
    }

    // ---- O^T += V^T P^T
#pragma unroll
    for (int kbk = 0; kbk < 2; ++kbk)
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const int key0 = 32 * kbk + 16 * u + tr_key;
        const int key1 = key0 + 8;
#pragma unroll
        for (int d = 0; d < DB; ++d) {
          const int col = 32 * d + tr_col;
          const bf16x4 lo = lds_read_tr16(lds_v + key0 * RB + 16 * ((col >> 3) ^ (key0 & 7)) + 2 * (col & 7));
          const bf16x4 hi = lds_read_tr16(lds_v + key1 * RB + 16 * ((col >> 3) ^ (key1 & 7)) + 2 * (col & 7));
          bf16x8 a;
          a[0] = lo[0]; a[1] = lo[1]; a[2] = lo[2]; a[3] = lo[3];
          a[4] = hi[0]; a[5] = hi[1]; a[6] = hi[2]; a[7] = hi[3];
#pragma unroll
          for (int n = 0; n < NQ; ++n)
            oacc[n][d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pf[n][kbk][u], oacc[n][d], 0, 0, 0);
        }
      }
  }

  if (!wave_active) return;
  // ---- O[row][d] = O^T[d][row] / l ; lane (r,h) holds d = 32*db + 8*(v/4) + 4h + v%4 of row r
#pragma unroll
  for (int n = 0; n < NQ; ++n) {
    const float total = run_sum[n] + __shfl_xor(run_sum[n], 32, 64);
    const float inv = 1.0f / total;
    const int row = q_base + 32 * n + r;
    if (row < t_q) {
      __bf16* dst = o + (bh * t_q + row) * D;
#pragma unroll
      for (int d = 0; d < DB; ++d)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          bf16x4 w;
#pragma unroll
          for (int e = 0; e < 4; ++e) w[e] = (__bf16)(oacc[n][d][4 * g + e] * inv);
          *reinterpret_cast<bf16x4*>(dst + 32 * d + 8 * g + 4 * h) = w;
        }
    }
  }
}

template <int D, int NQ>
hipError_t launch(const void* q, void* o, const void* kc, const void* vc, int bh, int t_q, int64_t cap_tokens,
                  const SegTable& seg, float c, hipStream_t st) {
  constexpr int BM = kWaves * 32 * NQ;
  dim3 grid(bh, (t_q + BM - 1) / BM), block(kThreads);
  hipLaunchKernelGGL((attend_bf16_kernel<D, NQ>), grid, block, 0, st, (const __bf16*)q, (__bf16*)o,
                     (const char*)kc, (const char*)vc, t_q, (long long)cap_tokens, seg, c);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_attend_bf16(const void* q, void* o, const void* kc, const void* vc, int bh, int t_q,
                              int head_dim, int64_t cap_tokens, const SegTable& seg, float softmax_scale,
                              hipStream_t st) {
  const float c = softmax_scale * 1.4426950408889634f;
  const bool wide = t_q > 128;  // 256 query rows per workgroup keeps K/V single-pass up to T_q = 256
  if (head_dim == 64)
    return wide ? launch<64, 2>(q, o, kc, vc, bh, t_q, cap_tokens, seg, c, st)
                : launch<64, 1>(q, o, kc, vc, bh, t_q, cap_tokens, seg, c, st);
  return wide ? launch<128, 2>(q, o, kc, vc, bh, t_q, cap_tokens, seg, c, st)
              : launch<128, 1>(q, o, kc, vc, bh, t_q, cap_tokens, seg, c, st);
}

}  // namespace amskv
