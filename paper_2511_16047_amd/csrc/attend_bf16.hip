// bf16 per-scale attention over the resident segments (Section 3.1: the queries of scale s
// attend to the cached scales and to their own scale; no mask inside a step), written for
// gfx950: 64-lane wavefronts, v_mfma_f32_32x32x16_bf16, K/V tiles streamed HBM -> LDS with
// direct-to-LDS loads through a multi-stage ring, transposing LDS reads for the V operand,
// online softmax with fp32 statistics, and a software pipeline that overlaps the softmax of one
// 32-key block with the second matrix product of the block before it.
//
// Formulation.  One workgroup owns all (<= 32*NQ*kWaves) query rows of a (b,h) tile, so K~ and
// V~ stream from HBM once per tile.  Each wave owns 32*NQ query rows and keeps their Q fragments
// in registers for the whole kernel.  Per 32-key block it computes the TRANSPOSED score block
// S^T = K Q^T (M = keys, N = queries): in the 32x32 accumulator layout every lane then holds 16
// keys of ONE query (column = lane%32), so the row sum (and, when it is needed, the row max) of
// the softmax are in-lane reductions plus a single exchange between the two lane halves, and the
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
// Pipeline.  Block g's softmax runs on the vector ALUs, block g-1's O^T += V^T P^T on the matrix
// cores; they share no data (the probabilities of g-1 were packed one iteration earlier), so
// they sit in one basic block and the scheduler interleaves them.  The softmax reference is lazy:
// the probabilities of a block are formed against the reference the earlier blocks left, and only
// when the sum of a lane's new probabilities shows that some score lay far above it (more than
// 2^kMaxLag times) is the block's maximum taken, the reference moved and the block redone; the
// accumulator rescale this requires is applied one step later.  The common block takes no maximum.  A unit's
// first block, which has no reference and nothing to multiply yet, goes straight to the maximum path.
//
// Density variant (attend_density_bf16_kernel): the same body with one more running sum per lane, over the keys of
// the group of cached keys the stream is in; at the end of a group the per-row sum is parked in LDS, and the
// epilogue turns the parked sums into the softmax mass per group (Section 4.1) next to O.
//
// Memory.  The kernel is HBM-bound at VAR shapes (arithmetic intensity T_q*T_kv/(T_q+T_kv)
// flop/byte, below the chip's ridge), so the tile loop keeps tiles in flight (two at head dim 64):
// global_load_lds_dwordx4 writes 64 lanes x 16 bytes straight into LDS with no register staging,
// and the wave only waits (s_waitcnt vmcnt) for the tile it is about to use.  A direct-to-LDS load
// puts lane i's 16 bytes at base + 16*i, so the XOR swizzle that spreads the fragment reads over the
// banks (chunk ^= swizzle(row)) is applied on the global side: the lane that fills LDS chunk
// position c' of row r fetches global chunk c' ^ swizzle(r).  Rows past the end of K~ re-read the
// last valid row (finite data) and their scores are set to -inf.  A borrowed current scale is the
// tail of the virtual concatenation and its rows are fetched from the caller's K/V instead.
// The ring holds tile t-1 (its last block's V is still being multiplied), t (in use) and the tiles in
// flight: t+1 and t+2 at head dim 64, t+1 alone at head dim 128 (see kAhead).  The query rows take the
// same road once, at the start: direct-to-LDS loads into a piece of the ring no tile has reached yet,
// then one read of the fragments into registers, so that every wait in the kernel is an explicit count.
#include "amskv_internal.hpp"

namespace amskv {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// query-token count up to which the latency-oriented kernel of attend_bf16_small.hip is used
constexpr int kSmallTq = 32;
// the online softmax lets the running max lag by up to this many powers of two before the
// accumulators are rescaled; probabilities then stay below 2^kMaxLag, far inside fp32/bf16 range
constexpr float kMaxLag = 6.0f;
// sum of a lane's 16 new probabilities above which the reference is looked at again: 16 * 2^kMaxLag
constexpr float kTripSum = 1024.0f;

#define AMSKV_LDS __attribute__((address_space(3)))

__device__ __forceinline__ bf16x4 lds_read_tr16(const char* p) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4bf16((AMSKV_LDS bf16x4*)(p));
}

// One wave-wide direct-to-LDS load: lane i's 16 bytes at `g` land at lds_wave_base + 16*i.
// Written as inline assembly on purpose: the ring's reuse distance is enforced by the explicit
// vmcnt waits and barriers in the tile loop, whereas the compiler, seeing an LDS write in
// flight, would drain every outstanding load before each LDS read and serialise the pipeline.
// lds_wave_base must be wave-uniform (it goes through M0).
__device__ __forceinline__ void lds_dma16(const char* g, char* lds_wave_base) {
  const unsigned m0v = (unsigned)(size_t)(AMSKV_LDS char*)lds_wave_base;
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(g), "s"(m0v) : "memory", "m0");
}

// The same load with a wave-uniform 64-bit base in scalar registers and a 32-bit unsigned byte offset per
// lane: the form the tile loop uses whenever all rows of a wave's part of a tile sit in one segment, so
// that the address arithmetic of the common case runs on the scalar unit.
__device__ __forceinline__ void lds_dma16_s(const char* base, unsigned lane_off, char* lds_wave_base) {
  const unsigned m0v = (unsigned)(size_t)(AMSKV_LDS char*)lds_wave_base;
  const unsigned long long b = (unsigned long long)base;
  const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)b), hi = __builtin_amdgcn_readfirstlane((unsigned)(b >> 32));
  const unsigned long long bs = ((unsigned long long)hi << 32) | lo;
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(lane_off), "s"(bs), "s"(m0v) : "memory", "m0");
}

// Compiler-visible use of a register value: the compiler places its own wait for the load that
// produced it here (and not inside the tile loop, where it could not tell the first iteration
// from the rest and would drain every outstanding load on each trip).
__device__ __forceinline__ void settle(const bf16x8& x) { asm volatile("" ::"v"(x)); }

// v_max3_f32 written out: the compiler's fmaxf first canonicalises every operand (one extra
// v_max per element under IEEE rules), which alone costs more than the whole reduction
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

// Maximum of x over the two lane halves (lanes l and l^32), in every lane, without leaving the
// vector ALU: v_permlane32_swap exchanges the upper half of its first operand with the lower half of
// its second, so two copies of x become (lower, lower) and (upper, upper).  x comes out of inline
// assembly, which the compiler's hazard tracking does not see as a vector write, so the wait states a
// lane swap needs after one are spent here explicitly.
__device__ __forceinline__ float half_max(float x) {
  asm volatile("s_nop 1" : "+v"(x));
  const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_int(x), __float_as_int(x), false, false);
  return fmaxf(__int_as_float(sw[0]), __int_as_float(sw[1]));
}

// XOR swizzle of a row's 16-byte chunks in LDS: chunk c of row `row` sits at chunk position c ^ swizzle(row).
// Head dim 64 (8 chunks, two rows per 64 banks): the three low row bits.  Head dim 128 (16 chunks, a row
// spans all banks): a permutation of the four low row bits -- row bits 1..0 move to chunk bits 2..1 and row
// bit 2 to chunk bit 0, so that the four keys one 16-lane group of a transposing V read touches (keys k..k+3,
// two chunks each) land in eight different chunks, and row bit 3 stays in place, which makes the 16 rows of a
// quarter-wave K read hit 16 different chunks.  Measured on the fragment-read patterns of this kernel: the
// (row & 7) form costs 1.15x (K) and 1.37x (V) the time of this one at head dim 128 and nothing at 64.
template <int D>
__device__ __forceinline__ constexpr int swizzle(int row) {
  return D == 64 ? (row & 7) : (((row & 3) << 1) | ((row >> 2) & 1) | (row & 8));
}

template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

template <int D, int kWaves, int kTileKeys>
struct TileLoader {
  static constexpr int RB = D * 2;
  static constexpr int CPR = D / 8;
  static constexpr int kRowsPerLoad = 64 / CPR;                            // rows covered by one wave-wide load
  static constexpr int kLoadsPerWave = kTileKeys / kRowsPerLoad / kWaves;  // per tensor
  static constexpr int kRowsPerWave = kLoadsPerWave * kRowsPerLoad;        // consecutive rows of a tile one wave fetches
  static constexpr int kVmPerTile = 2 * kLoadsPerWave;                     // vector-memory ops per thread and tile
  static_assert(kLoadsPerWave >= 1 && kLoadsPerWave * kRowsPerLoad * kWaves == kTileKeys, "tile/wave split");

  // Where the rows this wave fetches sit.  Everything but `voff` is wave-uniform (scalar registers) and is
  // carried from tile to tile: the wave's rows only move forward, by one tile per fetch, so while they stay
  // inside one segment the next addresses are the last ones plus a constant, and the segment table is looked
  // up again only when the first row passes the segment's end -- a handful of times per launch.
  struct Stream {
    int first;          // first virtual row of the wave's part of the next tile to fetch
    int end;            // first virtual row past the segment that holds `first` (0: nothing looked up yet)
    const char* k;      // address of row `first` (K, V) while first < end
    const char* v;
    long long step;     // bytes from a row to the row kTileKeys further on, in that segment
    bool scalar_ok;     // the scalar-base form of the load can address the segment (32-bit lane offsets)
    unsigned voff[kLoadsPerWave];  // per lane: byte offset of this lane's 16 bytes of load i from row `first`
  };
  // Lane constants of load i, formed again where the rare paths need them (not held in registers): the row inside
  // the wave's part and the byte offset of the swizzled 16-byte chunk this lane fetches.
  // (the lane id goes through an empty asm so that nothing derived from it is kept from the prologue on)
  __device__ static __forceinline__ int fresh(int lane) {
    asm volatile("" : "+v"(lane));
    return lane;
  }
  __device__ static __forceinline__ unsigned lane_row(int i, int lane) { return i * kRowsPerLoad + fresh(lane) / CPR; }
  __device__ static __forceinline__ unsigned lane_chunk(int wave, int i, int lane) {
    lane = fresh(lane);
    const int row = (wave * kLoadsPerWave + i) * kRowsPerLoad + lane / CPR;  // row inside the tile
    return 16u * ((lane % CPR) ^ swizzle<D>(row));
  }

  __device__ static __forceinline__ void init(Stream& s, int wave, int lane) {
    s.first = wave * kRowsPerWave;
    s.end = 0;
    s.k = s.v = nullptr;
    s.step = 0;
    s.scalar_ok = false;
#pragma unroll
    for (int i = 0; i < kLoadsPerWave; ++i) s.voff[i] = 0;
  }

  // Segment that holds virtual row s.first (< total), on the scalar unit.
  __device__ static __forceinline__ void find(Stream& s, const SegTable& seg, const char* kb, const char* vb, const char* xk,
                                              const char* xv, long long x_tok, int wave, int lane) {
    int end = seg.virt_start[0] + seg.len[0], delta = seg.phys_off[0] - seg.virt_start[0];
    for (int g = 1; g < seg.n; ++g)
      if (s.first >= seg.virt_start[g]) {
        end = seg.virt_start[g] + seg.len[g];
        delta = seg.phys_off[g] - seg.virt_start[g];
      }
    const bool ext = s.first >= seg.ext_start;
    if (ext) {
      end = seg.total;
      delta = -seg.ext_start;
    }
    const long long stride = ext ? x_tok : (long long)RB;
    const long long at = (long long)(s.first + delta) * stride;
    s.end = end;
    s.k = (ext ? xk : kb) + at;
    s.v = (ext ? xv : vb) + at;
    s.step = stride * kTileKeys;
    s.scalar_ok = stride < (1ll << 24);
#pragma unroll
    for (int i = 0; i < kLoadsPerWave; ++i) s.voff[i] = lane_row(i, lane) * (unsigned)stride + lane_chunk(wave, i, lane);
  }

  // Fetch the wave's part of the next tile of the virtual concatenation into one ring slot (tiles are
  // fetched in ascending order).  x_tok: byte stride between the rows of the borrowed scale in the caller's
  // tensors.
  __device__ static __forceinline__ void issue(Stream& s, const char* kb, const char* vb, const char* xk, const char* xv,
                                               long long x_tok, char* lds_k, char* lds_v, int t_kv, const SegTable& seg,
                                               int wave, int lane) {
    const int first = s.first;
    if (__builtin_expect(first >= s.end && first < t_kv, 0)) find(s, seg, kb, vb, xk, xv, x_tok, wave, lane);
    s.first = first + kTileKeys;
    if (__builtin_expect(first + kRowsPerWave <= s.end && s.scalar_ok, 1)) {
      // every row of the wave's part lies in one segment: scalar base, lane-constant offsets
#pragma unroll
      for (int i = 0; i < kLoadsPerWave; ++i) {
        const int blk = wave * kLoadsPerWave + i;
        lds_dma16_s(s.k, s.voff[i], lds_k + blk * 1024);
        lds_dma16_s(s.v, s.voff[i], lds_v + blk * 1024);
      }
      s.k += s.step;
      s.v += s.step;
      return;
    }
    // a segment boundary or the end of K~ inside the wave's rows: every lane locates its own row
    const int j0 = first - wave * kRowsPerWave;
#pragma unroll
    for (int i = 0; i < kLoadsPerWave; ++i) {
      const int blk = wave * kLoadsPerWave + i;  // which 1 KB block of the tile
      const int row = blk * kRowsPerLoad + fresh(lane) / CPR;
      bool ext;
      const int row_at = locate_row(seg, min(j0 + row, t_kv - 1), ext);
      const long long off = (long long)row_at * (ext ? x_tok : (long long)RB) + lane_chunk(wave, i, lane);
      lds_dma16((ext ? xk : kb) + off, lds_k + blk * 1024);
      lds_dma16((ext ? xv : vb) + off, lds_v + blk * 1024);
    }
  }

  // Fused append / fused iteration: copy the rows of the landed tile (first row j0) that ExtKV asks for from LDS
  // to their place in the cache (the rows of the current scale into its slot; in the token modes also cached
  // rows that slide toward offset 0).  Each wave stores exactly the 1 KB blocks it fetched,
  // so lane i re-reads its own 16 bytes at block + 16*i and the swizzle of issue() is undone by using the same
  // chunk mapping for the destination.  The stores are ordinary vector-memory operations issued before the
  // next tile's loads; the tile waits of the caller stay valid because a vmcnt wait only counts operations
  // (loads complete in order, and outstanding stores make the wait stricter, not laxer).
  __device__ static __forceinline__ void write_back(const Stream& s, char* kb, char* vb, const char* lds_k, const char* lds_v,
                                                    int j0, int t_kv, const SegTable& seg, const ExtKV& ext, int wave, int lane) {
    const int first = j0 + wave * kRowsPerWave;  // wave-uniform
    if (__builtin_expect(first >= ext.wb_from && first + kRowsPerWave <= t_kv, 1)) {  // all rows of the wave's part move by wb_delta
      const long long at = (long long)(first + ext.wb_delta) * RB;
#pragma unroll
      for (int i = 0; i < kLoadsPerWave; ++i) {
        const int blk = wave * kLoadsPerWave + i;
        const unsigned off = lane_row(i, lane) * RB + lane_chunk(wave, i, lane);
        *reinterpret_cast<uint4*>(kb + at + off) = *reinterpret_cast<const uint4*>(lds_k + blk * 1024 + 16 * lane);
        *reinterpret_cast<uint4*>(vb + at + off) = *reinterpret_cast<const uint4*>(lds_v + blk * 1024 + 16 * lane);
      }
      return;
    }
#pragma unroll
    for (int i = 0; i < kLoadsPerWave; ++i) {
      const int blk = wave * kLoadsPerWave + i;
      const int j = j0 + blk * kRowsPerLoad + fresh(lane) / CPR;
      const int to = write_back_row(ext, j, t_kv, seg.ext_start);
      if (to >= 0) {
        const long long dst = (long long)to * RB + lane_chunk(wave, i, lane);
        *reinterpret_cast<uint4*>(kb + dst) = *reinterpret_cast<const uint4*>(lds_k + blk * 1024 + 16 * lane);
        *reinterpret_cast<uint4*>(vb + dst) = *reinterpret_cast<const uint4*>(lds_v + blk * 1024 + 16 * lane);
      }
    }
  }
};

template <bool B>
struct Flag {
  static constexpr bool value = B;
};

// The work of one workgroup.  kDensity: also leave, per 32-row query block, the softmax mass that lands on each
// group of keys (Section 4.1's attention density as a by-product of the step's own attention; `groups` holds the
// first virtual row past each group, `partial` one float per (b, h, query block, group)).
template <int D, int NQ, int kWaves, int kTileKeys, bool kDensity>
__device__ __forceinline__ void attend_unit(
    const __bf16* __restrict__ q, __bf16* __restrict__ o, char* __restrict__ kc, char* __restrict__ vc,
    int t_q, long long cap_tokens, const SegTable& seg, const ExtKV& ext_kv, const CallerIo& io, float scale_log2e, int n_bh,
    int n_qtiles, const GroupEnds& groups, float* __restrict__ partial) {
  using Loader = TileLoader<D, kWaves, kTileKeys>;
  constexpr int RB = D * 2;   // bytes per token row
  constexpr int KS = D / 16;  // K-steps of the first product
  constexpr int DB = D / 32;  // 32-row blocks of O^T
  constexpr int BM = kWaves * 32 * NQ;
  constexpr int kTileBytes = kTileKeys * RB;
  constexpr int kBlkBytes = 32 * RB;
  constexpr int kBlocksPerTile = kTileKeys / 32;
  // Ring of tiles in LDS: the tile in use, the one before it (the V rows of its last block are still being
  // multiplied) and kAhead tiles in flight.  Head dim 128 is bound by latency at two waves per SIMD: one tile
  // in flight makes the ring 48 KB, so three workgroups fit a CU -- three waves per SIMD, which measured 15 %
  // faster on the 1024x1024 schedule than two waves with two tiles in flight.
  constexpr int kAhead = D == 128 ? 1 : 2;
  constexpr int kStages = kAhead + 2;
  constexpr int kRing = kStages * kTileBytes;
  constexpr int VM = Loader::kVmPerTile;
  // Fetch the K fragments of block g+1 into registers while the softmax of block g runs (16 registers at head
  // dim 64; the head-dim-128 configuration has none to spare, and one-block tiles would need a fifth ring slot).
  // (the density variant keeps the plain loop: one block at a time, the tile barrier in front of a tile's first block)
  constexpr bool kPrefetchK = D == 64 && kBlocksPerTile == 2 && !kDensity;

  __shared__ __align__(1024) char lds_k[kRing];
  __shared__ __align__(1024) char lds_v[kRing];
  // density: per wave and query row, the sum of exp over the keys of each finished group, in the row's current reference
  __shared__ float park[kDensity ? kWaves * NQ : 1][AMSKV_MAX_SCALES][32];

  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lane = tid & 63;
  const int r = lane & 31;  // column (query) / row (key or head-dim) index inside a block
  const int h = lane >> 5;  // which half of the K-step this lane feeds
  // XCD-aware unit mapping: consecutive workgroup ids go round-robin to the 8 XCDs, each with its own L2,
  // so the query tiles of one (b,h) are given ids 8 apart: they land on the same XCD back to back and the
  // second one finds K~/V~ in that L2 instead of fetching them from HBM again.
  int bh_i, q_tile;
  if (n_qtiles == 1) {  // the common case, spelled out: it needs no division
    bh_i = blockIdx.x;
    q_tile = 0;
  } else {
    const unsigned per_group = 8u * n_qtiles, group = blockIdx.x / per_group, within = blockIdx.x - group * per_group;
    bh_i = group * 8 + (within & 7);
    q_tile = within >> 3;
  }
  const long long bh = bh_i;
  if (bh >= n_bh) return;  // whole workgroup leaves together (n_bh not a multiple of 8)
  const int q_base = q_tile * BM + wave * (32 * NQ);
  const bool wave_active = q_base < t_q;
  const int t_kv = seg.total;
  const int n_tiles = (t_kv + kTileKeys - 1) / kTileKeys;
  const int n_blocks = (t_kv + 31) / 32;
  char* kb = kc + bh * cap_tokens * RB;
  char* vb = vc + bh * cap_tokens * RB;
  // the borrowed current scale, if any, in the caller's buffers; Q and O rows of this (b,h)
  const long long x_unit = unit_offset(io.kv, bh, io.heads);
  const char* xk = (const char*)ext_kv.k + x_unit;
  const char* xv = (const char*)ext_kv.v + x_unit;
  const long long x_tok = io.kv.tok;
  // fused append: the workgroup of the first query tile also fills the current scale's slot
  const bool write_back = writes_back(ext_kv, seg.total, seg.ext_start) && q_tile == 0;
  // first row that is written anywhere
  const int wb_first = min(ext_kv.wb_from, ext_kv.wb_head_end > seg.ext_start ? seg.ext_start : kNoWriteBack);

  // ---- prologue.  What the first matrix instruction waits for is kept small: the wave's own Q rows and tile 0.
  // Q goes through LDS like the tiles (direct-to-LDS loads, so every wait below is an explicit count and the
  // first block does not wait for younger tile loads, as it would behind compiler-tracked register loads): each
  // wave fetches its 32*NQ rows into a private piece of the last two ring slots, which the tile stream reaches
  // only after the first barriers, and reads its fragments from there once.  Then kAhead tiles are requested;
  // from the first barrier on the steady rule applies: the barrier of tile `it` frees the slot of tile it-2, and
  // tile it+kAhead is requested into it.
  typename Loader::Stream stream;
  Loader::init(stream, wave, lane);
  // ring positions (byte offsets, the same in the K and the V ring), all wave-uniform
  int fetch_off = 0;  // slot the next tile to fetch goes into
  int sync_off = 0;   // slot of the next tile to become readable
  auto ring_next = [](int off, int by) {
    off += by;
    return off == kRing ? 0 : off;
  };
  constexpr int kQBytes = 32 * NQ * RB;   // Q rows of one wave
  constexpr int kQLoads = kQBytes / 1024;
  constexpr int CPR = Loader::CPR;
  static_assert(kWaves % 2 == 0 && (kWaves / 2) * kQBytes <= 2 * kTileBytes, "Q staging fits the last two slots of each ring");
  char* q_stage = (wave < kWaves / 2 ? lds_k : lds_v) + (kStages - 2) * kTileBytes + (wave % (kWaves / 2)) * kQBytes;
  if (wave_active) {
    // lane i of load j fills chunk position i % CPR of row j * (64 / CPR) + i / CPR; rows past T_q re-read the
    // last row (their results are never stored); same swizzle as the tiles
    const char* q_unit = (const char*)q + unit_offset(io.q, bh, io.heads);
#pragma unroll
    for (int j = 0; j < kQLoads; ++j) {
      const int row = j * (64 / CPR) + lane / CPR;
      const long long at = (long long)min(q_base + row, t_q - 1) * io.q.tok + 16 * ((lane % CPR) ^ swizzle<D>(row));
      lds_dma16(q_unit + at, q_stage + j * 1024);
    }
  }
#pragma unroll
  for (int st = 0; st < kAhead; ++st)
    if (st < n_tiles) {
      Loader::issue(stream, kb, vb, xk, xv, x_tok, lds_k + fetch_off, lds_v + fetch_off, t_kv, seg, wave, lane);
      fetch_off = ring_next(fetch_off, kTileBytes);
    }
  // Q fragments: B operand of S^T = K Q^T; lane (r,h) holds Q[row r][16t + 8h .. +8)
  bf16x8 qf[NQ][KS];
  if (wave_active) {
    // the Q loads are the oldest: once no more than the tile loads are outstanding, Q has landed
    if (kAhead >= 3 && n_tiles >= 3) wait_vmcnt<3 * VM>();
    else if (kAhead >= 2 && n_tiles >= 2) wait_vmcnt<2 * VM>();
    else wait_vmcnt<VM>();
#pragma unroll
    for (int n = 0; n < NQ; ++n)
#pragma unroll
      for (int t = 0; t < KS; ++t) {
        qf[n][t] = *reinterpret_cast<const bf16x8*>(q_stage + (32 * n + r) * RB + 16 * ((2 * t + h) ^ swizzle<D>(32 * n + r)));
        settle(qf[n][t]);  // read before the barrier behind which other waves may request tiles into this piece
      }
  }

  // Tile `it` becomes readable: this wave's loads of it have landed (younger tiles may stay in flight), the
  // barrier extends that to every wave's part, and it also retires the slot of tile it-2, which tile it+kAhead
  // is requested into.  Called for it = 0, 1, ... by every wave of the workgroup.
  // steady: the caller knows that tile it+kAhead exists (nothing to test on the common path).
  auto tile_sync = [&](int it, auto steady) {
    constexpr bool kSteady = decltype(steady)::value;
    if (kSteady) {
      wait_vmcnt<VM*(kAhead - 1)>();
    } else {
      // tiles requested so far beyond `it` may stay in flight: min(n_tiles - it - 1, kAhead - 1) of them
      const int ahead = min(n_tiles - it - 1, kAhead - 1);
      if (kAhead >= 3 && ahead == 2) wait_vmcnt<2 * VM>();
      else if (kAhead >= 2 && ahead == 1) wait_vmcnt<VM>();
      else wait_vmcnt<0>();
    }
    __syncthreads();
    if (write_back && (it + 1) * kTileKeys > wb_first)
      Loader::write_back(stream, kb, vb, lds_k + sync_off, lds_v + sync_off, it * kTileKeys, t_kv, seg, ext_kv, wave, lane);
    sync_off = ring_next(sync_off, kTileBytes);
    if (kSteady || it + kAhead < n_tiles) {
      Loader::issue(stream, kb, vb, xk, xv, x_tok, lds_k + fetch_off, lds_v + fetch_off, t_kv, seg, wave, lane);
      fetch_off = ring_next(fetch_off, kTileBytes);
    }
  };
  constexpr Flag<true> yes;
  constexpr Flag<false> no;
  tile_sync(0, no);
  if (!wave_active) {
    // no query rows (T_q is not a multiple of the workgroup's rows): this wave only fetches its part of every tile
    for (int it = 1; it < n_tiles; ++it) tile_sync(it, no);
    return;
  }

  f32x16 oacc[NQ][DB];
#pragma unroll
  for (int n = 0; n < NQ; ++n)
#pragma unroll
    for (int d = 0; d < DB; ++d)
#pragma unroll
      for (int v = 0; v < 16; ++v) oacc[n][d][v] = 0.f;
  float run_mc[NQ], run_sum[NQ];  // softmax reference times c = softmax scale * log2(e); sum of 2^(s*c - reference)
  // density: this lane's sum over the keys of the group being walked, the group, its end, the block's first row
  float seg_acc[NQ];
  int cur_group = 0, next_end = kDensity ? groups.end[0] : 0, blk_start = 0;
  bf16x8 pf[NQ][2];  // probabilities of the previous block, two K-steps of 16 keys
#pragma unroll
  for (int n = 0; n < NQ; ++n) {
    run_mc[n] = -INFINITY;
    run_sum[n] = 0.f;
    seg_acc[n] = 0.f;
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
      for (int e = 0; e < 8; ++e) pf[n][u][e] = (__bf16)0.f;
  }

  // lane-constant pieces of the fragment addresses
  const int tr_key = 4 * h + ((lane & 15) >> 2);               // + K-step base (+8 for the second read)
  const int tr_col = 16 * ((lane >> 4) & 1) + 4 * (lane & 3);  // + 32*db
  // V^T fragment of K-step u, read x: key = 16u + 8x + tr_key.  The swizzle of that key is the swizzle of tr_key
  // (< 8), plus, at head dim 128, chunk bit 3 flipped when x = 1; u and x therefore enter the address as
  // compile-time offsets: hi_off(d) is what x = 1 adds -- eight rows, and the flip of address bit 7, whose
  // value before the flip is bit 6 of the column, i.e. known from d.
  int v_base[DB];
#pragma unroll
  for (int d = 0; d < DB; ++d) {
    const int col = 32 * d + tr_col;
    v_base[d] = tr_key * RB + 16 * ((col >> 3) ^ swizzle<D>(tr_key)) + 2 * (col & 7);
  }
  auto hi_off = [](int d) { return 8 * RB + (D == 64 ? 0 : (d < 2 ? 128 : -128)); };
  int k_off[KS];  // K fragment byte offsets inside a 32-key block
#pragma unroll
  for (int t = 0; t < KS; ++t) k_off[t] = r * RB + 16 * ((2 * t + h) ^ swizzle<D>(r));

  // ring positions of the blocks a step touches: g-1 (V rows of the second product; first step: block 0
  // itself, multiplied by pf = 0), g, and g+1 (K prefetch)
  int off_prev = 0, off_cur = 0, off_next = kBlkBytes == kRing ? 0 : kBlkBytes;
  float alpha[NQ];
  bool any_rescale = false;  // the rescale decided at block g is applied at the top of block g+1
  bool first_block = true;
#pragma unroll
  for (int n = 0; n < NQ; ++n) alpha[n] = 1.f;

  // K fragments (A operand of S^T = K Q^T) of the block at ring position `off`, LDS -> registers
  bf16x8 kf[KS];
  auto load_k = [&](int off) {
#pragma unroll
    for (int t = 0; t < KS; ++t) kf[t] = *reinterpret_cast<const bf16x8*>(lds_k + off + k_off[t]);
  };
  if (kPrefetchK) load_k(0);
  int next_tile = 1;  // next tile to synchronise on

  // One 32-key block g: S^T, its softmax, and O^T += V^T P^T of block g-1, whose probabilities pf were
  // packed one step earlier and are replaced by those of g as the step goes.
  //   sync_next: (K prefetch only) g is the last block of its tile and another tile follows: the barrier for
  //     that tile sits behind the score products, so that the fragments of the new tile's first block are
  //     fetched while the softmax of g runs.  Every wave has then finished step g-1 (V rows of block g-2 = last
  //     block of the tile two back, which the barrier retires), and what the rest of step g still reads (V rows
  //     of block g-1) lies in the tile one back.  Without K prefetch the caller synchronises in front of the
  //     first block of a tile instead.
  //   has_next: a block g+1 exists (K prefetch)
  //   ragged: g is the last block and t_kv is not a multiple of 32: keys past the end get zero weight
  auto block_step = [&](auto sync_next, auto steady, auto has_next, bool ragged) {
    // ---- (rarely) move the accumulators to the reference chosen in the previous step
    if (__builtin_expect(any_rescale, 0)) {
#pragma unroll
      for (int n = 0; n < NQ; ++n)
#pragma unroll
        for (int d = 0; d < DB; ++d)
#pragma unroll
          for (int v = 0; v < 16; ++v) oacc[n][d][v] *= alpha[n];
    }
    // ---- S^T = K Q^T for this 32-key block
    if (!kPrefetchK) load_k(off_cur);
    f32x16 sacc[NQ];
#pragma unroll
    for (int n = 0; n < NQ; ++n)
#pragma unroll
      for (int v = 0; v < 16; ++v) sacc[n][v] = 0.f;
#pragma unroll
    for (int t = 0; t < KS; ++t)
#pragma unroll
      for (int n = 0; n < NQ; ++n) sacc[n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[t], qf[n][t], sacc[n], 0, 0, 0);
    if (kPrefetchK) {
      if (decltype(sync_next)::value) tile_sync(next_tile++, steady);
      if (decltype(has_next)::value) load_k(off_next);
    }
    if (ragged) {
      const int valid = t_kv & 31;
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int key = 8 * (v >> 2) + 4 * h + (v & 3);
        if (key >= valid) {
#pragma unroll
          for (int n = 0; n < NQ; ++n) sacc[n][v] = -INFINITY;
        }
      }
    }

    // ---- probabilities of this block (vector ALU) next to O^T += V^T P^T of the previous block (matrix
    // cores), one K-step of 16 keys at a time: the matrix instructions of K-step u read the old pf[.][u] when
    // they issue, after which the new probabilities of keys 16u..16u+15 overwrite it.
    // p = 2^(s*c - m*c) in fp32; the row sum is taken over these, the second product uses them rounded to bf16.
    // Lazy reference: m*c (run_mc) is NOT looked for first.  The probabilities are formed against the reference
    // of the blocks before, and the sum of the lane's 16 new ones tells whether that was good enough: while it
    // stays below kTripSum no score exceeded the reference by more than log2(kTripSum) powers of two, which is
    // far inside the range of fp32 and bf16, and the block costs no maximum at all.
    // The first block of a unit has no reference yet and nothing to multiply (pf = 0): it goes straight to the
    // path that takes the maximum.
    float sum[NQ][2];
#pragma unroll
    for (int n = 0; n < NQ; ++n) sum[n][0] = sum[n][1] = 0.f;
    const bool first = first_block;
    first_block = false;
    bool trip = true;
    if (!first) {
#pragma unroll
      for (int u = 0; u < 2; ++u) {
#pragma unroll
        for (int d = 0; d < DB; ++d) {
          const char* vp = lds_v + off_prev + v_base[d];
          const bf16x4 lo = lds_read_tr16(vp + (16 * u) * RB);
          const bf16x4 hi = lds_read_tr16(vp + (16 * u) * RB + hi_off(d));
          bf16x8 a;
          a[0] = lo[0]; a[1] = lo[1]; a[2] = lo[2]; a[3] = lo[3];
          a[4] = hi[0]; a[5] = hi[1]; a[6] = hi[2]; a[7] = hi[3];
#pragma unroll
          for (int n = 0; n < NQ; ++n) oacc[n][d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pf[n][u], oacc[n][d], 0, 0, 0);
        }
#pragma unroll
        for (int n = 0; n < NQ; ++n)
#pragma unroll
          for (int v = 8 * u; v < 8 * u + 8; v += 2) {
            const float p0 = __builtin_amdgcn_exp2f(fmaf(sacc[n][v], scale_log2e, -run_mc[n]));
            const float p1 = __builtin_amdgcn_exp2f(fmaf(sacc[n][v + 1], scale_log2e, -run_mc[n]));
            sum[n][0] += p0;
            sum[n][1] += p1;
            pf[n][u][v & 7] = (__bf16)p0;
            pf[n][u][(v & 7) + 1] = (__bf16)p1;
          }
      }
      // ---- was the reference good enough?  (NaN -- a masked key against the initial reference of -inf -- and
      // +inf -- anything against that reference -- both fail the comparison as written.)
      trip = false;
#pragma unroll
      for (int n = 0; n < NQ; ++n) {
        sum[n][0] += sum[n][1];
        trip |= __builtin_amdgcn_ballot_w64(!(sum[n][0] <= kTripSum)) != 0;
      }
    }
    any_rescale = trip && !first;  // the first block leaves zeros in the accumulators: nothing to rescale
    if (__builtin_expect(trip, 0)) {
      // Some query of the wave needs a new reference (or this is the first block).  Now the maximum of the block
      // is taken, per query over both lane halves; a query moves its reference to it only if it lies more than
      // kMaxLag powers of two above the old one (every lane that tripped does: its largest probability
      // exceeded kTripSum / 16 = 2^kMaxLag).  Then the block's probabilities are formed again.
#pragma unroll
      for (int n = 0; n < NQ; ++n) {
        settle_mfma(sacc[n]);
        const float a0 = max3(sacc[n][0], sacc[n][1], sacc[n][2]), a1 = max3(sacc[n][3], sacc[n][4], sacc[n][5]);
        const float a2 = max3(sacc[n][6], sacc[n][7], sacc[n][8]), a3 = max3(sacc[n][9], sacc[n][10], sacc[n][11]);
        const float a4 = max3(sacc[n][12], sacc[n][13], sacc[n][14]);
        const float b0 = max3(a0, a1, a2), b1 = max3(a3, a4, sacc[n][15]);
        const float full = half_max(max3(b0, b1, b1)) * scale_log2e;  // finite: key 0 of the block is valid for every query
        const float new_mc = full - run_mc[n] > kMaxLag ? full : run_mc[n];
        alpha[n] = __builtin_amdgcn_exp2f(run_mc[n] - new_mc);  // 1 when unchanged, 0 on the first block
        run_sum[n] *= alpha[n];
        if constexpr (kDensity) {  // what was summed against the old reference moves with it
          seg_acc[n] *= alpha[n];
          if (h == 0)
            for (int p = 0; p < cur_group; ++p) park[wave * NQ + n][p][r] *= alpha[n];
        }
        run_mc[n] = new_mc;
        float s0 = 0.f, s1 = 0.f;
#pragma unroll
        for (int v = 0; v < 16; v += 2) {
          const float p0 = __builtin_amdgcn_exp2f(fmaf(sacc[n][v], scale_log2e, -new_mc));
          const float p1 = __builtin_amdgcn_exp2f(fmaf(sacc[n][v + 1], scale_log2e, -new_mc));
          s0 += p0;
          s1 += p1;
          pf[n][v >> 3][v & 7] = (__bf16)p0;
          pf[n][v >> 3][(v & 7) + 1] = (__bf16)p1;
        }
        sum[n][0] = s0 + s1;
      }
    }
    if constexpr (kDensity) {
      // Groups of keys that end inside (or with) this block: the lane's sum over the group = what it gathered in
      // the blocks before + its probabilities of this block up to the cut (formed again, exactly, for the keys
      // below the cut; the whole block's sum when the cut is the block's end) - what earlier cuts of this block took.
      float taken[NQ];
#pragma unroll
      for (int n = 0; n < NQ; ++n) taken[n] = 0.f;
      while (next_end <= blk_start + 32) {
        const int cut = next_end - blk_start;  // 1..32, wave-uniform
#pragma unroll
        for (int n = 0; n < NQ; ++n) {
          float upto = sum[n][0];
          if (cut < 32) {
            upto = 0.f;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
              const int key = 8 * (v >> 2) + 4 * h + (v & 3);
              const float pv = __builtin_amdgcn_exp2f(fmaf(sacc[n][v], scale_log2e, -run_mc[n]));
              upto += key < cut ? pv : 0.f;
            }
          }
          float gsum = seg_acc[n] + (upto - taken[n]);
          gsum += __shfl_xor(gsum, 32, 64);  // the two lane halves hold different keys of the same query
          if (h == 0) park[wave * NQ + n][cur_group][r] = gsum;
          seg_acc[n] = 0.f;
          taken[n] = upto;
        }
        ++cur_group;
        next_end = cur_group < groups.n ? groups.end[cur_group] : 0x7fffffff;
      }
#pragma unroll
      for (int n = 0; n < NQ; ++n) seg_acc[n] += sum[n][0] - taken[n];
      blk_start += 32;
    }
#pragma unroll
    for (int n = 0; n < NQ; ++n) run_sum[n] += sum[n][0];
    off_prev = off_cur;
    off_cur = off_next;
    off_next = ring_next(off_next, kBlkBytes);
  };

  const bool ragged = (t_kv & 31) != 0;
  if (kPrefetchK) {
    // two blocks per tile.  First the tiles whose barrier has nothing to test (the tile it requests exists),
    // then the ones near the end of the stream, then the last tile (1 or 2 blocks).
    int it = 0;
    for (; it + 1 + kAhead < n_tiles; ++it) {
      block_step(no, no, yes, false);
      block_step(yes, yes, yes, false);
    }
    for (; it + 1 < n_tiles; ++it) {
      block_step(no, no, yes, false);
      block_step(yes, no, yes, false);
    }
    if (!(n_blocks & 1)) block_step(no, no, yes, false);
    block_step(no, no, no, ragged);
  } else {
    for (int g = 0; g < n_blocks; ++g) {
      if (g > 0 && g % kBlocksPerTile == 0) tile_sync(next_tile++, no);
      block_step(no, no, no, ragged && g == n_blocks - 1);
    }
  }

  if (any_rescale) {
#pragma unroll
    for (int n = 0; n < NQ; ++n)
#pragma unroll
      for (int d = 0; d < DB; ++d)
#pragma unroll
        for (int v = 0; v < 16; ++v) oacc[n][d][v] *= alpha[n];
  }
  // ---- drain: the last block's O^T += V^T P^T
#pragma unroll
  for (int d = 0; d < DB; ++d) {
    const char* vp = lds_v + off_prev + v_base[d];
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const bf16x4 lo = lds_read_tr16(vp + (16 * u) * RB);
      const bf16x4 hi = lds_read_tr16(vp + (16 * u) * RB + hi_off(d));
      bf16x8 a;
      a[0] = lo[0]; a[1] = lo[1]; a[2] = lo[2]; a[3] = lo[3];
      a[4] = hi[0]; a[5] = hi[1]; a[6] = hi[2]; a[7] = hi[3];
#pragma unroll
      for (int n = 0; n < NQ; ++n) oacc[n][d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pf[n][u], oacc[n][d], 0, 0, 0);
    }
  }

  // ---- O[row][d] = O^T[d][row] / l ; lane (r,h) holds d = 32*db + 8*(v/4) + 4h + v%4 of row r
  char* o_unit = (char*)o + unit_offset(io.o, bh, io.heads);
#pragma unroll
  for (int n = 0; n < NQ; ++n) {
    const float total = run_sum[n] + __shfl_xor(run_sum[n], 32, 64);
    const float inv = 1.0f / total;
    const int row = q_base + 32 * n + r;
    // The lane halves hold alternate 8-byte pieces of a row (columns 8g + 4h ..); one lane swap per register
    // pairs them up, so that every lane stores 16 bytes and the two lanes of a row 32 contiguous bytes (half as
    // many requests to the L2 as 8-byte stores: 2.4 % of the step at the default shape).
    __bf16* dst = reinterpret_cast<__bf16*>(o_unit + min(row, t_q - 1) * io.o.tok);
#pragma unroll
    for (int d = 0; d < DB; ++d)
#pragma unroll
      for (int k = 0; k < 2; ++k) {
        bf16x4 wa, wb;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          wa[e] = (__bf16)(oacc[n][d][8 * k + e] * inv);
          wb[e] = (__bf16)(oacc[n][d][8 * k + 4 + e] * inv);
        }
        const u32x2 a = __builtin_bit_cast(u32x2, wa), b = __builtin_bit_cast(u32x2, wb);
        const auto s0 = __builtin_amdgcn_permlane32_swap(a[0], b[0], false, false);
        const auto s1 = __builtin_amdgcn_permlane32_swap(a[1], b[1], false, false);
        const u32x4 w = {s0[0], s1[0], s0[1], s1[1]};
        if (row < t_q) *reinterpret_cast<u32x4*>(dst + 32 * d + 16 * k + 8 * h) = w;
      }
    if constexpr (kDensity) {
      // mass of the query block on group p = sum over its valid rows of (sum of exp over the group) / (sum over all keys)
      const int n_qblk = (t_q + 31) >> 5;
      const long long qblk = bh * n_qblk + (q_base >> 5) + n;
      for (int p = 0; p < groups.n; ++p) {
        float m = h == 0 && row < t_q ? park[wave * NQ + n][p][r] * inv : 0.f;
#pragma unroll
        for (int d = 16; d >= 1; d >>= 1) m += __shfl_xor(m, d, 64);  // over the 32 query rows (lower lane half)
        if (lane == 0) partial[qblk * AMSKV_MAX_SCALES + p] = m;
      }
    }
  }
}

template <int D, int NQ, int kWaves, int kTileKeys, int kMinWavesPerSimd>
__global__ __launch_bounds__(64 * kWaves, kMinWavesPerSimd) void attend_bf16_kernel(
    const __bf16* __restrict__ q, __bf16* __restrict__ o, char* __restrict__ kc, char* __restrict__ vc,
    int t_q, long long cap_tokens, SegTable seg, ExtKV ext_kv, CallerIo io, float scale_log2e, int n_bh, int n_qtiles) {
  attend_unit<D, NQ, kWaves, kTileKeys, false>(q, o, kc, vc, t_q, cap_tokens, seg, chosen(ext_kv), io, scale_log2e, n_bh,
                                               n_qtiles, GroupEnds{}, nullptr);
}

// The same step with the attention density of its own queries as a by-product (no second pass over Q and K).
template <int D, int NQ, int kWaves, int kTileKeys, int kMinWavesPerSimd>
__global__ __launch_bounds__(64 * kWaves, kMinWavesPerSimd) void attend_density_bf16_kernel(
    const __bf16* __restrict__ q, __bf16* __restrict__ o, char* __restrict__ kc, char* __restrict__ vc,
    int t_q, long long cap_tokens, SegTable seg, ExtKV ext_kv, CallerIo io, float scale_log2e, int n_bh, int n_qtiles,
    GroupEnds groups, float* __restrict__ partial) {
  attend_unit<D, NQ, kWaves, kTileKeys, true>(q, o, kc, vc, t_q, cap_tokens, seg, chosen(ext_kv), io, scale_log2e, n_bh,
                                              n_qtiles, groups, partial);
}

template <int D, int NQ, int kWaves, int kTileKeys, int kMinWavesPerSimd>
hipError_t launch(const void* q, void* o, void* kc, void* vc, int bh, int t_q, int64_t cap_tokens,
                  const SegTable& seg, const ExtKV& ext, const CallerIo& io, float c, hipStream_t st) {
  constexpr int BM = kWaves * 32 * NQ;
  const int n_qtiles = (t_q + BM - 1) / BM;
  dim3 grid((unsigned)(((bh + 7) / 8) * 8 * n_qtiles)), block(64 * kWaves);
  hipLaunchKernelGGL((attend_bf16_kernel<D, NQ, kWaves, kTileKeys, kMinWavesPerSimd>), grid, block, 0, st,
                     (const __bf16*)q, (__bf16*)o, (char*)kc, (char*)vc, t_q, (long long)cap_tokens, seg, ext, io, c,
                     bh, n_qtiles);
  return hipGetLastError();
}

template <int D, int NQ, int kWaves, int kTileKeys, int kMinWavesPerSimd>
hipError_t launch_density_variant(const void* q, void* o, void* kc, void* vc, int bh, int t_q, int64_t cap_tokens,
                                  const SegTable& seg, const ExtKV& ext, const CallerIo& io, float c, const GroupEnds& groups,
                                  float* partial, hipStream_t st) {
  constexpr int BM = kWaves * 32 * NQ;
  const int n_qtiles = (t_q + BM - 1) / BM;
  dim3 grid((unsigned)(((bh + 7) / 8) * 8 * n_qtiles)), block(64 * kWaves);
  hipLaunchKernelGGL((attend_density_bf16_kernel<D, NQ, kWaves, kTileKeys, kMinWavesPerSimd>), grid, block, 0, st,
                     (const __bf16*)q, (__bf16*)o, (char*)kc, (char*)vc, t_q, (long long)cap_tokens, seg, ext, io, c,
                     bh, n_qtiles, groups, partial);
  return hipGetLastError();
}

}  // namespace

bool attend_density_fused(int t_q) { return t_q > kSmallTq; }

bool attend_owns_unit(int head_dim, int t_q) { return t_q <= (head_dim == 64 ? 256 : 128); }

hipError_t launch_attend_density_bf16(const void* q, void* o, void* kc, void* vc, int batch, int heads, int t_q, int head_dim,
                                      int64_t cap_tokens, const SegTable& seg, const ExtKV& ext, const CallerIo& io,
                                      float softmax_scale, const GroupEnds& groups, float* partial_ws, float* out_dev,
                                      hipStream_t st) {
  if (!attend_density_fused(t_q)) return hipErrorInvalidValue;
  const float c = softmax_scale * 1.4426950408889634f;
  const int bh = batch * heads;
  // Four waves of 32 rows and 32-key tiles at either head dim (the ring shares LDS with the per-row group sums,
  // and the block step holds its scores a little longer: three and two waves per SIMD); more than 128 query rows
  // are split over workgroups with ids 8 apart, which re-read K~ and V~ from their XCD's L2.
  hipError_t e;
  if (head_dim == 64)
    e = launch_density_variant<64, 1, 4, 32, 4>(q, o, kc, vc, bh, t_q, cap_tokens, seg, ext, io, c, groups, partial_ws, st);
  else
    e = launch_density_variant<128, 1, 4, 32, 2>(q, o, kc, vc, bh, t_q, cap_tokens, seg, ext, io, c, groups, partial_ws, st);
  if (e != hipSuccess) return e;
  return launch_density_total(partial_ws, batch, heads, (t_q + 31) / 32, groups.n, out_dev, st);
}

hipError_t launch_attend_bf16(const void* q, void* o, void* kc, void* vc, int bh, int t_q,
                              int head_dim, int64_t cap_tokens, const SegTable& seg, const ExtKV& ext, const CallerIo& io,
                              float softmax_scale, hipStream_t st) {
  // coarse scales: latency-bound, one independent wave per 32 query rows
  if (t_q <= kSmallTq) return launch_attend_bf16_small(q, o, kc, vc, bh, t_q, head_dim, cap_tokens, seg, ext, io, softmax_scale, st);
  const float c = softmax_scale * 1.4426950408889634f;
  const bool wide = t_q > 128;  // 256 query rows per workgroup keeps K/V single-pass up to T_q = 256
  if (head_dim == 64)
    // eight waves of 32 rows: ~110 registers per lane, so two workgroups (16 waves) share a CU
    return wide ? launch<64, 1, 8, 64, 4>(q, o, kc, vc, bh, t_q, cap_tokens, seg, ext, io, c, st)
                : launch<64, 1, 4, 32, 4>(q, o, kc, vc, bh, t_q, cap_tokens, seg, ext, io, c, st);
  // head dim 128: 32 query rows per wave (~160 registers) and a three-slot ring give three waves per SIMD,
  // i.e. three workgroups of four waves per CU; 64 rows per wave would halve that
  (void)wide;
  return launch<128, 1, 4, 32, 3>(q, o, kc, vc, bh, t_q, cap_tokens, seg, ext, io, c, st);
}

}  // namespace amskv
