// bf16 per-scale attention for the coarse scales (Section 3.1's per-step attention when the
// step has only a handful of query tokens): at T_q of 1..64 a (b,h) unit is a few kilobytes
// of work and the launch is bound by memory latency, not by bandwidth or the matrix cores, so
// the design goal is to have every unit of the launch resident at once.
//
// One WAVE owns one unit = (b, h, block of 32 query rows); the four waves of a workgroup are
// independent (no barrier, no shared data).  K fragments are loaded straight from the cache into
// registers in the A-operand layout of v_mfma_f32_32x32x16_bf16 (lane (r,h) reads 16 bytes of
// key row r), so K never touches LDS; the only LDS use is two 32-key blocks of V per wave, which
// the transposing read ds_read_b64_tr_b16 needs as its source and which direct-to-LDS loads fill
// without passing through registers (that is what lets four waves per SIMD be resident at head
// dim 64).  The loads of block g+1 are issued right after the first product of block g has
// consumed the K registers, so they overlap the softmax and the second product.  Same transposed formulation (S^T = K Q^T, O^T += V^T P^T) and
// the same segment-table walk as the streaming kernel; plain online softmax.
#include "amskv_internal.hpp"

namespace amskv {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
// 16-byte chunk as a native vector: arrays of it stay in registers (HIP's uint4 struct did not)
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int kWavesPerGroup = 4;

#define AMSKV_LDS __attribute__((address_space(3)))

__device__ __forceinline__ bf16x4 lds_read_tr16(const char* p) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4bf16((AMSKV_LDS bf16x4*)(p));
}

// One wave-wide direct-to-LDS load: lane i's 16 bytes at `g` land at lds_wave_base + 16*i (wave-uniform base,
// through M0).  Inline assembly: the compiler does not count it among its outstanding loads, which is safe
// here because every V load is issued BEFORE the K register loads of the same block -- loads complete in
// order, so the wait the compiler places in front of the first use of those K registers covers it.
__device__ __forceinline__ void lds_dma16(const char* g, char* lds_wave_base) {
  const unsigned m0v = (unsigned)(size_t)(AMSKV_LDS char*)lds_wave_base;
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(g), "s"(m0v) : "memory", "m0");
}

__device__ __forceinline__ float max3(float a, float b, float c) {
  float r;
  asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
  return r;
}

// The compiler tracks the wait states a matrix instruction needs before an ordinary vector
// instruction may read its result, but not for a read from inside inline assembly (max3 above).
// Called on the accumulator between the two, this holds the wave for the 11 wait states that an
// 8-pass v_mfma_f32_32x32x16_bf16 requires (one to spare); taking the accumulator as an in/out operand pins
// it after the matrix instructions and before every later use.
__device__ __forceinline__ void settle_mfma(f32x16& acc) { asm volatile("s_nop 11" : "+v"(acc)); }

// Register budget: four waves per SIMD at head dim 64 and two at 128 are the most that fit without spilling;
// every step up in resident waves measured faster on these latency-bound launches.
template <int D>
__global__ __launch_bounds__(64 * kWavesPerGroup, D == 64 ? 4 : 2) void attend_bf16_small_kernel(
    const __bf16* __restrict__ q, __bf16* __restrict__ o, char* __restrict__ kc, char* __restrict__ vc,
    int t_q, long long cap_tokens, SegTable seg, ExtKV ext_in, CallerIo io, float scale_log2e, int n_qblk, int n_units) {
  const ExtKV ext_kv = chosen(ext_in);
  constexpr int RB = D * 2;
  constexpr int CPR = D / 8;
  constexpr int KS = D / 16;
  constexpr int DB = D / 32;
  constexpr int VCH = 32 * CPR / 64;  // 16-byte chunks of a 32-key V block per lane

  __shared__ __align__(1024) char lds_v[kWavesPerGroup][2][32 * RB];  // per wave: the block in use and the one in flight

  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  const int unit = blockIdx.x * kWavesPerGroup + wave;
  if (unit >= n_units) return;  // waves are independent: nothing below synchronises across waves
  const int r = lane & 31, h = lane >> 5;
  const long long bh = unit / n_qblk;
  const int q_base = (unit % n_qblk) * 32;
  const int t_kv = seg.total;
  const int n_blocks = (t_kv + 31) / 32;
  char* kb = kc + bh * cap_tokens * RB;
  char* vb = vc + bh * cap_tokens * RB;
  const long long x_unit = unit_offset(io.kv, bh, io.heads);  // borrowed current scale, if any
  const char* xk = (const char*)ext_kv.k + x_unit;
  const char* xv = (const char*)ext_kv.v + x_unit;
  const long long x_tok = io.kv.tok;
  const char* q_unit = (const char*)q + unit_offset(io.q, bh, io.heads);
  char* o_unit = (char*)o + unit_offset(io.o, bh, io.heads);
  const bool write_back = writes_back(ext_kv, seg.total, seg.ext_start) && q_base == 0;

  bf16x8 qf[KS];
  {
    const int row = min(q_base + r, t_q - 1);
#pragma unroll
    for (int t = 0; t < KS; ++t) qf[t] = *reinterpret_cast<const bf16x8*>(q_unit + row * io.q.tok + 32 * t + 16 * h);
  }

  bf16x8 kf[KS];
  // lane i of V load k fills chunk position i % CPR of row k * (64 / CPR) + i / CPR with the global chunk that the
  // XOR swizzle (same as the streaming kernel's at head dim 64) assigns to that position
  auto load_block = [&](int g) {
    const int j0 = 32 * g;
    char* dst = lds_v[wave][g & 1];
#pragma unroll
    for (int k = 0; k < VCH; ++k) {
      const int row = k * (64 / CPR) + lane / CPR, c = (lane % CPR) ^ (row & 7);
      bool vext;
      const long long vrow = locate_row(seg, min(j0 + row, t_kv - 1), vext);
      lds_dma16((vext ? xv + vrow * x_tok : vb + vrow * RB) + 16 * c, dst + k * 1024);
    }
    bool kext;
    const long long krow = locate_row(seg, min(j0 + r, t_kv - 1), kext);
    const char* kp = kext ? xk + krow * x_tok : kb + krow * RB;
#pragma unroll
    for (int t = 0; t < KS; ++t) kf[t] = *reinterpret_cast<const bf16x8*>(kp + 32 * t + 16 * h);
  };
  load_block(0);

  f32x16 oacc[DB];
#pragma unroll
  for (int d = 0; d < DB; ++d)
#pragma unroll
    for (int v = 0; v < 16; ++v) oacc[d][v] = 0.f;
  float run_max = -INFINITY, run_sum = 0.f;

  const int tr_key = 4 * h + ((lane & 15) >> 2);
  const int tr_col = 16 * ((lane >> 4) & 1) + 4 * (lane & 3);

  for (int g = 0; g < n_blocks; ++g) {
    // every load of block g (the V rows in LDS and the K registers) has landed; an explicit point, because the
    // compiler does not know that the V loads wrote LDS and could otherwise move reads of it above its own wait
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    const char* my_v = lds_v[wave][g & 1];
    f32x16 sacc;
#pragma unroll
    for (int v = 0; v < 16; ++v) sacc[v] = 0.f;
#pragma unroll
    for (int t = 0; t < KS; ++t) sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[t], qf[t], sacc, 0, 0, 0);
    if (write_back) {
      // fused append: this unit also fills the current scale's slot from the registers it just used
      const int j0 = 32 * g;
      const int k_to = write_back_row(ext_kv, j0 + r, t_kv, seg.ext_start);
      if (k_to >= 0) {
        char* dst = kb + (long long)k_to * RB + 16 * h;
#pragma unroll
        for (int t = 0; t < KS; ++t) *reinterpret_cast<bf16x8*>(dst + 32 * t) = kf[t];
      }
#pragma unroll
      for (int k = 0; k < VCH; ++k) {
        const int row = k * (64 / CPR) + lane / CPR, c = (lane % CPR) ^ (row & 7);
        const int v_to = write_back_row(ext_kv, j0 + row, t_kv, seg.ext_start);
        if (v_to >= 0)
          *reinterpret_cast<u32x4*>(vb + (long long)v_to * RB + 16 * c) =
              *reinterpret_cast<const u32x4*>(my_v + k * 1024 + 16 * lane);
      }
    }
    if (g + 1 < n_blocks) load_block(g + 1);  // in flight during the softmax and the second product

    if (g == n_blocks - 1 && (t_kv & 31) != 0) {
      const int valid = t_kv & 31;
#pragma unroll
      for (int v = 0; v < 16; ++v)
        if (8 * (v >> 2) + 4 * h + (v & 3) >= valid) sacc[v] = -INFINITY;
    }
    settle_mfma(sacc);
    float mx = max3(sacc[0], sacc[1], sacc[2]);
#pragma unroll
    for (int v = 3; v < 15; v += 2) mx = max3(mx, sacc[v], sacc[v + 1]);
    const float other = __shfl_xor(max3(mx, sacc[15], sacc[15]), 32, 64);
    mx = max3(mx, sacc[15], other);
    const float new_max = fmaxf(run_max, mx);
    const float alpha = __builtin_amdgcn_exp2f((run_max - new_max) * scale_log2e);
    const float mc = new_max * scale_log2e;
    run_max = new_max;
    const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
    float sum = run_sum * alpha;
    bf16x8 pf[2];
#pragma unroll
    for (int v = 0; v < 16; v += 2) {
      bf16x2 pk;
      pk[0] = (__bf16)__builtin_amdgcn_exp2f(fmaf(sacc[v], scale_log2e, -mc));
      pk[1] = (__bf16)__builtin_amdgcn_exp2f(fmaf(sacc[v + 1], scale_log2e, -mc));
      sum = __builtin_amdgcn_fdot2_f32_bf16(pk, ones, sum, false);
      pf[v >> 3][v & 7] = pk[0];
      pf[v >> 3][(v & 7) + 1] = pk[1];
    }
    run_sum = sum;
#pragma unroll
    for (int d = 0; d < DB; ++d)
#pragma unroll
      for (int v = 0; v < 16; ++v) oacc[d][v] *= alpha;

    __builtin_amdgcn_wave_barrier();  // the V rows written above by all lanes are read below
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
      for (int d = 0; d < DB; ++d) {
        const int key0 = 16 * u + tr_key, key1 = key0 + 8, col = 32 * d + tr_col;
        const bf16x4 lo = lds_read_tr16(my_v + key0 * RB + 16 * ((col >> 3) ^ (key0 & 7)) + 2 * (col & 7));
        const bf16x4 hi = lds_read_tr16(my_v + key1 * RB + 16 * ((col >> 3) ^ (key1 & 7)) + 2 * (col & 7));
        bf16x8 a;
        a[0] = lo[0]; a[1] = lo[1]; a[2] = lo[2]; a[3] = lo[3];
        a[4] = hi[0]; a[5] = hi[1]; a[6] = hi[2]; a[7] = hi[3];
        oacc[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pf[u], oacc[d], 0, 0, 0);
      }
    __builtin_amdgcn_wave_barrier();  // ... and are overwritten by the next iteration
  }

  const float total = run_sum + __shfl_xor(run_sum, 32, 64);
  const float inv = 1.0f / total;
  const int row = q_base + r;
  // The lane halves hold alternate 8-byte pieces of a row (columns 8g + 4h ..); one lane swap per register pairs
  // them up, so that every lane stores 16 bytes and the two lanes of a row 32 contiguous bytes.
  __bf16* dst = reinterpret_cast<__bf16*>(o_unit + min(row, t_q - 1) * io.o.tok);
#pragma unroll
  for (int d = 0; d < DB; ++d)
#pragma unroll
    for (int k = 0; k < 2; ++k) {
      typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
      bf16x4 wa, wb;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        wa[e] = (__bf16)(oacc[d][8 * k + e] * inv);
        wb[e] = (__bf16)(oacc[d][8 * k + 4 + e] * inv);
      }
      const u32x2 a = __builtin_bit_cast(u32x2, wa), b = __builtin_bit_cast(u32x2, wb);
      const auto s0 = __builtin_amdgcn_permlane32_swap(a[0], b[0], false, false);
      const auto s1 = __builtin_amdgcn_permlane32_swap(a[1], b[1], false, false);
      const u32x4 w = {s0[0], s1[0], s0[1], s1[1]};
      if (row < t_q) *reinterpret_cast<u32x4*>(dst + 32 * d + 16 * k + 8 * h) = w;
    }
}

}  // namespace

hipError_t launch_attend_bf16_small(const void* q, void* o, void* kc, void* vc, int bh, int t_q,
                                    int head_dim, int64_t cap_tokens, const SegTable& seg, const ExtKV& ext,
                                    const CallerIo& io, float softmax_scale, hipStream_t st) {
  const float c = softmax_scale * 1.4426950408889634f;
  const int n_qblk = (t_q + 31) / 32;
  const long long n_units = (long long)bh * n_qblk;
  dim3 grid((unsigned)((n_units + kWavesPerGroup - 1) / kWavesPerGroup)), block(64 * kWavesPerGroup);
  if (head_dim == 64)
    hipLaunchKernelGGL(attend_bf16_small_kernel<64>, grid, block, 0, st, (const __bf16*)q, (__bf16*)o, (char*)kc,
                       (char*)vc, t_q, (long long)cap_tokens, seg, ext, io, c, n_qblk, (int)n_units);
  else
    hipLaunchKernelGGL(attend_bf16_small_kernel<128>, grid, block, 0, st, (const __bf16*)q, (__bf16*)o, (char*)kc,
                       (char*)vc, t_q, (long long)cap_tokens, seg, ext, io, c, n_qblk, (int)n_units);
  return hipGetLastError();
}

}  // namespace amskv
