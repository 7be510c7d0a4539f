/* The library used the way a C program would: this file includes include/amskv.h and the HIP runtime API and
 * nothing else -- no torch, no Python, no C++.  It allocates device memory with hipMalloc, drives two layers
 * (one that keeps every scale, one at {condensed 1, window 1}) through amskv_append_scale / amskv_attend for
 * fp32 and bf16 caches, and compares every output with the definition of Section 3.1 (Eq. 2) written out below in
 * double precision over the scales the policy keeps (Section 4.3; the kept sets of this four-scale schedule are
 * listed by hand).  Exit status 0 and the line "abi_check: ok" mean every check held.
 *
 * Test program: built and run by tests/test_gpu_c_abi.py.  Tolerances: 1e-4 (fp32), 2e-2 (bf16), max-abs. */
#include <hip/hip_runtime_api.h>
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "amskv.h"

#define S 4
#define B 2
#define H 2
#define D 64

static const int32_t kSide[S] = {1, 2, 3, 5};
static const int kTok[S] = {1, 4, 9, 25};
/* layer 1, {condensed 1, window 1}: after scale s the layer holds scale 0, scale s-1 and scale s */
static const int kKept1[S][S] = {{0, -1, -1, -1}, {0, 1, -1, -1}, {0, 1, 2, -1}, {0, 2, 3, -1}};

#define HIP(x)                                                                        \
  do {                                                                                \
    hipError_t e_ = (x);                                                              \
    if (e_ != hipSuccess) {                                                           \
      fprintf(stderr, "%s:%d: %s -> %s\n", __FILE__, __LINE__, #x, hipGetErrorString(e_)); \
      exit(1);                                                                        \
    }                                                                                 \
  } while (0)
#define AMS(x)                                                                        \
  do {                                                                                \
    int32_t s_ = (x);                                                                 \
    if (s_ != AMSKV_OK) {                                                             \
      fprintf(stderr, "%s:%d: %s -> %s\n", __FILE__, __LINE__, #x, amskv_status_string(s_)); \
      exit(1);                                                                        \
    }                                                                                 \
  } while (0)

static uint32_t g_state = 2511u;
static float draw(void) { /* uniform in [-1.5, 1.5), a plain linear congruential generator */
  g_state = g_state * 1664525u + 1013904223u;
  return ((float)(g_state >> 8) / 16777216.0f - 0.5f) * 3.0f;
}

static uint16_t to_bf16(float x) { /* round to nearest even */
  uint32_t u;
  memcpy(&u, &x, 4);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}
static float from_bf16(uint16_t h) {
  uint32_t u = (uint32_t)h << 16;
  float x;
  memcpy(&x, &u, 4);
  return x;
}

/* host copies of the per-scale tensors [B][H][T_s][D], as floats holding exactly what the device holds */
static float *q_h[S], *k_h[S], *v_h[S];

static void reference(int bh, int s, const int* kept, double* out /* [T_s][D] */) {
  const double scale = 1.0 / sqrt((double)D);
  for (int i = 0; i < kTok[s]; ++i) {
    const float* qi = q_h[s] + ((size_t)bh * kTok[s] + i) * D;
    double score[1 + 4 + 9 + 25], best = -1e300;
    int n = 0;
    for (int a = 0; a < S && kept[a] >= 0; ++a)
      for (int j = 0; j < kTok[kept[a]]; ++j) {
        const float* kj = k_h[kept[a]] + ((size_t)bh * kTok[kept[a]] + j) * D;
        double dot = 0;
        for (int d = 0; d < D; ++d) dot += (double)qi[d] * kj[d];
        score[n] = dot * scale;
        if (score[n] > best) best = score[n];
        ++n;
      }
    double sum = 0;
    for (int j = 0; j < n; ++j) sum += (score[j] = exp(score[j] - best));
    for (int d = 0; d < D; ++d) out[(size_t)i * D + d] = 0;
    n = 0;
    for (int a = 0; a < S && kept[a] >= 0; ++a)
      for (int j = 0; j < kTok[kept[a]]; ++j, ++n) {
        const float* vj = v_h[kept[a]] + ((size_t)bh * kTok[kept[a]] + j) * D;
        for (int d = 0; d < D; ++d) out[(size_t)i * D + d] += score[n] / sum * vj[d];
      }
  }
}

static int run(int32_t dtype, double tol) {
  const size_t eb = dtype == AMSKV_DTYPE_BF16 ? 2 : 4;
  int failures = 0;
  void *q_d[S], *k_d[S], *v_d[S], *o_d[S];
  for (int s = 0; s < S; ++s) {
    const size_t n = (size_t)B * H * kTok[s] * D;
    q_h[s] = malloc(n * 4), k_h[s] = malloc(n * 4), v_h[s] = malloc(n * 4);
    void* stage = malloc(n * eb);
    float** host[3] = {&q_h[s], &k_h[s], &v_h[s]};
    void** dev[3] = {&q_d[s], &k_d[s], &v_d[s]};
    for (int t = 0; t < 3; ++t) {
      float* h = *host[t];
      for (size_t i = 0; i < n; ++i) {
        h[i] = draw();
        if (eb == 2) {
          ((uint16_t*)stage)[i] = to_bf16(h[i]);
          h[i] = from_bf16(((uint16_t*)stage)[i]);
        } else {
          ((float*)stage)[i] = h[i];
        }
      }
      HIP(hipMalloc(dev[t], n * eb));
      HIP(hipMemcpy(*dev[t], stage, n * eb, hipMemcpyHostToDevice));
    }
    HIP(hipMalloc(&o_d[s], n * eb));
    free(stage);
  }

  const amskv_schedule sched = {S, kSide, kSide, B, dtype};
  const amskv_layer_policy layers[2] = {{0, 0, 1}, {1, 1, 0}};
  amskv_policy pol;
  memset(&pol, 0, sizeof(pol));
  pol.n_layers = 2;
  pol.layer = layers;
  pol.layout = AMSKV_LAYOUT_COMPACT;
  uint64_t need = 0;
  AMS(amskv_cache_required_bytes(2, H, D, &sched, &pol, &need));
  void* arena = NULL;
  HIP(hipMalloc(&arena, need));
  HIP(hipMemset(arena, 0xFF, need));
  amskv_cache* cache = NULL;
  AMS(amskv_cache_create(2, H, D, &sched, &pol, arena, need, &cache));
  hipStream_t stream;
  HIP(hipStreamCreate(&stream));

  double worst = 0;
  double* want = malloc(sizeof(double) * 25 * D);
  void* back = malloc((size_t)B * H * 25 * D * eb);
  for (int s = 0; s < S; ++s)
    for (int layer = 0; layer < 2; ++layer) {
      AMS(amskv_append_scale(cache, layer, s, k_d[s], v_d[s], stream));
      AMS(amskv_attend(cache, layer, s, q_d[s], o_d[s], stream));
      HIP(hipStreamSynchronize(stream));
      const size_t n = (size_t)B * H * kTok[s] * D;
      HIP(hipMemcpy(back, o_d[s], n * eb, hipMemcpyDeviceToHost));
      int kept0[S] = {-1, -1, -1, -1};
      for (int a = 0; a <= s; ++a) kept0[a] = a;
      const int* kept = layer == 0 ? kept0 : kKept1[s];
      /* the library's own report of what the layer holds */
      int32_t n_seg = 0, ids[AMSKV_MAX_SCALES], len[AMSKV_MAX_SCALES];
      int64_t off[AMSKV_MAX_SCALES];
      AMS(amskv_cache_layout(cache, layer, &n_seg, ids, off, len));
      int held = 0, n_kept = 0;
      for (int a = 0; a < S && kept[a] >= 0; ++a) {
        if (a >= n_seg || ids[a] != kept[a] || len[a] != kTok[kept[a]]) {
          fprintf(stderr, "layer %d step %d: kept set differs at entry %d\n", layer, s, a);
          ++failures;
        }
        held += kTok[kept[a]];
        ++n_kept;
      }
      if (n_seg != n_kept || amskv_cache_bytes_held(cache, layer, 1) != (int64_t)(2 * eb * B * H * D) * held) {
        fprintf(stderr, "layer %d step %d: %d segments, %lld bytes held\n", layer, s, (int)n_seg,
                (long long)amskv_cache_bytes_held(cache, layer, 1));
        ++failures;
      }
      for (int bh = 0; bh < B * H; ++bh) {
        reference(bh, s, kept, want);
        for (size_t i = 0; i < (size_t)kTok[s] * D; ++i) {
          const size_t at = (size_t)bh * kTok[s] * D + i;
          const double got = eb == 2 ? from_bf16(((uint16_t*)back)[at]) : ((float*)back)[at];
          const double err = fabs(got - want[i]);
          if (!(err <= tol)) {
            if (failures < 5) fprintf(stderr, "layer %d step %d unit %d element %zu: %g, want %g\n", layer, s, bh, i, got, want[i]);
            ++failures;
          }
          if (err > worst) worst = err;
        }
      }
    }
  printf("abi_check: %s cache, worst max-abs %.3e (bound %.0e)\n", eb == 2 ? "bf16" : "fp32", worst, tol);

  amskv_cache_destroy(cache);
  HIP(hipStreamDestroy(stream));
  HIP(hipFree(arena));
  for (int s = 0; s < S; ++s) {
    HIP(hipFree(q_d[s]));
    HIP(hipFree(k_d[s]));
    HIP(hipFree(v_d[s]));
    HIP(hipFree(o_d[s]));
    free(q_h[s]), free(k_h[s]), free(v_h[s]);
  }
  free(want), free(back);
  return failures;
}

int main(void) {
  int failures = run(AMSKV_DTYPE_F32, 1e-4);
  failures += run(AMSKV_DTYPE_BF16, 2e-2);
  if (failures) {
    fprintf(stderr, "abi_check: %d check(s) failed\n", failures);
    return 1;
  }
  printf("abi_check: ok\n");
  return 0;
}
