"""The CPU oracle under AddressSanitizer and UndefinedBehaviorSanitizer (host code only, no GPU).

A C driver is compiled together with oracle/sagekv_ref.c with -fsanitize=address,undefined and walks
every exported function over both element types, both head modes and the edge shapes (no candidates,
k = 0, k = E, no sink, a window of one token, spare capacity, one-token rows).  Any out-of-bounds
access, use after free, leak, signed overflow or misaligned access aborts the run; the driver also
checks the structural invariants of what comes back (sink and recent kept, ascending order, gathered
rows equal the source rows, probabilities sum to one)."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

DRIVER = r'''
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int sagekv_ref_scores(int dtype, int head_mode, int P, int Hq, int Hkv, int d, int64_t L, const void* q_last,
                      const void* K, float* s_out);
int sagekv_ref_select(int dtype, int head_mode, int P, int Hq, int Hkv, int d, int64_t L, int S, int W, int k, int cap,
                      const void* q_last, const void* K, const void* V, void* Kc, void* Vc, int32_t* kept_idx,
                      float* s_out);
int sagekv_ref_append(int dtype, int P, int Hkv, int d, int cap, int seg, int W, int grow, int32_t* len,
                      const void* k_new, const void* v_new, void* Kc, void* Vc);
int sagekv_ref_decode_attn(int dtype, int head_mode, int P, int Hq, int Hkv, int d, int cap, int S, int k, int W,
                           int len, const void* q, const void* Kc, const void* Vc, float* out);
int sagekv_ref_decode_attn_window_rope(int dtype, int P, int Hq, int Hkv, int d, int cap, int len, const void* q,
                                       const void* Kc, const void* Vc, const double* inv_freq, float* out);
int sagekv_ref_full_attention(int dtype, int G, int d, int64_t L, const void* q, const void* K, const void* V,
                              const int64_t* idx, int64_t n_idx, float* out);
void sagekv_ref_paper_budget(int B, int G, int* sink, int* k, int* recent);

static uint64_t rng = 0x9E3779B97F4A7C15ull;
static double unit(void) { /* uniform in (-1, 1) */
  rng = rng * 6364136223846793005ull + 1442695040888963407ull;
  return (double)(rng >> 11) / 4503599627370496.0 - 1.0;
}
static size_t eb(int dtype) { return dtype == 0 ? 2 : 4; }
static void* random_buf(int dtype, size_t n) {
  void* p = malloc(n * eb(dtype) + 1);
  for (size_t i = 0; i < n; ++i) {
    float f = (float)(2.0 * unit());
    if (dtype == 0) {
      uint32_t b;
      memcpy(&b, &f, 4);
      ((uint16_t*)p)[i] = (uint16_t)(b >> 16);
    } else {
      ((float*)p)[i] = f;
    }
  }
  return p;
}
#define CHECK(c) do { if (!(c)) { fprintf(stderr, "check failed at line %d: %s\n", __LINE__, #c); exit(3); } } while (0)

static void one_case(int dtype, int mode, int P, int Hq, int Hkv, int d, int L, int S, int W, int k, int spare) {
  int G = Hq / Hkv, lists = mode ? G : 1, n_kept = S + lists * k + W, cap = n_kept + spare;
  size_t rb = (size_t)d * eb(dtype);
  void* q = random_buf(dtype, (size_t)P * Hq * d);
  void* K = random_buf(dtype, (size_t)P * Hkv * L * d);
  void* V = random_buf(dtype, (size_t)P * Hkv * L * d);
  void* Kc = random_buf(dtype, (size_t)P * Hkv * cap * d);
  void* Vc = random_buf(dtype, (size_t)P * Hkv * cap * d);
  int32_t* kept = (int32_t*)malloc(sizeof(int32_t) * (size_t)P * Hkv * (n_kept > 0 ? n_kept : 1));
  float* s = (float*)malloc(sizeof(float) * (size_t)P * Hkv * lists * L);
  float* s2 = (float*)malloc(sizeof(float) * (size_t)P * Hkv * lists * L);
  CHECK(sagekv_ref_select(dtype, mode, P, Hq, Hkv, d, L, S, W, k, cap, q, K, V, Kc, Vc, kept, s) == 0);
  CHECK(sagekv_ref_scores(dtype, mode, P, Hq, Hkv, d, L, q, K, s2) == 0);
  CHECK(memcmp(s, s2, sizeof(float) * (size_t)P * Hkv * lists * L) == 0);
  for (int r = 0; r < P * Hkv; ++r) {
    const int32_t* kr = kept + (size_t)r * n_kept;
    for (int t = 0; t < S; ++t) CHECK(kr[t] == t);
    for (int t = 0; t < W; ++t) CHECK(kr[S + lists * k + t] == L - W + t);
    for (int li = 0; li < lists; ++li)
      for (int t = 0; t < k; ++t) {
        int v = kr[S + li * k + t];
        CHECK(v >= S && v < L - W);
        if (t) CHECK(v > kr[S + li * k + t - 1]);
      }
    for (int t = 0; t < n_kept; ++t) {
      CHECK(memcmp((char*)Kc + ((size_t)r * cap + t) * rb, (char*)K + ((size_t)r * L + kr[t]) * rb, rb) == 0);
      CHECK(memcmp((char*)Vc + ((size_t)r * cap + t) * rb, (char*)V + ((size_t)r * L + kr[t]) * rb, rb) == 0);
    }
    for (int li = 0; li < lists; ++li) {
      double tot = 0.0;
      for (int i = 0; i < L; ++i) tot += s[((size_t)r * lists + li) * L + i];
      CHECK(fabs(tot - (mode ? 1.0 : (double)G)) < 1e-4);
    }
  }
  /* decode: FIFO appends across a wrap of the window, then grow mode into the spare capacity */
  float* out = (float*)malloc(sizeof(float) * (size_t)P * Hq * d);
  int32_t len = n_kept;
  for (int t = 0; t < W + 2; ++t) {
    void* kn = random_buf(dtype, (size_t)P * Hkv * d);
    void* vn = random_buf(dtype, (size_t)P * Hkv * d);
    CHECK(sagekv_ref_append(dtype, P, Hkv, d, cap, S + lists * k, W, 0, &len, kn, vn, Kc, Vc) == 0);
    CHECK(len == n_kept);
    CHECK(sagekv_ref_decode_attn(dtype, mode, P, Hq, Hkv, d, cap, S, k, W, n_kept, q, Kc, Vc, out) == 0);
    for (size_t i = 0; i < (size_t)P * Hq * d; ++i) CHECK(out[i] == out[i] && fabsf(out[i]) < 10.f);
    free(kn);
    free(vn);
  }
  if (mode == 0) {
    for (int t = 0; t < spare + 1; ++t) {
      void* kn = random_buf(dtype, (size_t)P * Hkv * d);
      void* vn = random_buf(dtype, (size_t)P * Hkv * d);
      int rc = sagekv_ref_append(dtype, P, Hkv, d, cap, S + k, W, 1, &len, kn, vn, Kc, Vc);
      CHECK(rc == (t < spare ? 0 : 1));  /* the last one does not fit and is refused */
      CHECK(sagekv_ref_decode_attn(dtype, 0, P, Hq, Hkv, d, cap, S, k, W, len, q, Kc, Vc, out) == 0);
      free(kn);
      free(vn);
    }
    CHECK(len == cap);
    /* window-relative rotary attention and the independent full attention (with and without an index list) */
    double* freq = (double*)malloc(sizeof(double) * (d / 2));
    for (int j = 0; j < d / 2; ++j) freq[j] = pow(10000.0, -2.0 * j / d);
    CHECK(sagekv_ref_decode_attn_window_rope(dtype, P, Hq, Hkv, d, cap, len, q, Kc, Vc, freq, out) == 0);
    free(freq);
    float* fo = (float*)malloc(sizeof(float) * (size_t)G * d);
    int64_t* idx = (int64_t*)malloc(sizeof(int64_t) * (size_t)((L + 1) / 2));
    int64_t n_idx = 0;
    for (int i = 0; i < L; i += 2) idx[n_idx++] = i;
    CHECK(sagekv_ref_full_attention(dtype, G, d, L, q, K, V, 0, 0, fo) == 0);
    CHECK(sagekv_ref_full_attention(dtype, G, d, L, q, K, V, idx, n_idx, fo) == 0);
    free(idx);
    free(fo);
  }
  free(out); free(s); free(s2); free(kept); free(q); free(K); free(V); free(Kc); free(Vc);
}

int main(void) {
  for (int dtype = 0; dtype < 2; ++dtype)
    for (int mode = 0; mode < 2; ++mode) {
      one_case(dtype, mode, 2, 4, 2, 8, 50, 3, 5, 7, 2);    /* ordinary */
      one_case(dtype, mode, 1, 6, 2, 4, 40, 0, 1, 10, 0);   /* no sink, the window is the last token only */
      one_case(dtype, mode, 1, 2, 2, 16, 12, 4, 8, 0, 1);   /* E = 0 */
      one_case(dtype, mode, 1, 4, 1, 2, 30, 2, 3, 25, 0);   /* k = E: nothing evicted */
      one_case(dtype, mode, 3, 3, 3, 6, 9, 1, 1, 0, 3);     /* k = 0, G = 1 */
      one_case(dtype, mode, 1, 7, 1, 2, 1, 0, 1, 0, 0);     /* a one-token cache */
    }
  /* invalid arguments are refused without touching memory */
  if (sagekv_ref_select(0, 0, 1, 4, 2, 8, 10, 4, 4, 5, 13, 0, 0, 0, 0, 0, 0, 0) != 1) return 4;
  if (sagekv_ref_select(0, 0, 1, 3, 2, 8, 10, 1, 1, 1, 3, 0, 0, 0, 0, 0, 0, 0) != 1) return 4;
  if (sagekv_ref_decode_attn(0, 0, 1, 4, 2, 8, 10, 1, 1, 1, 11, 0, 0, 0, 0) != 1) return 4;
  int a, b, c;
  sagekv_ref_paper_budget(8192, 4, &a, &b, &c);
  if (a != 2048 || b != 1024 || c != 2048) return 5;
  sagekv_ref_paper_budget(8192, 7, &a, &b, &c);
  if (a != 2048 || b != 512 || c != 2560) return 5;
  puts("oracle clean");
  return 0;
}
'''


def test_oracle_is_clean_under_asan_and_ubsan(tmp_path):
    src = tmp_path / "driver.c"
    src.write_text(DRIVER)
    exe = tmp_path / "driver"
    subprocess.check_call(["gcc", "-std=c99", "-O1", "-g", "-fopenmp", "-fsanitize=address,undefined",
                           "-static-libasan", "-static-libubsan", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer",
                           "-Wall", "-Wextra", "-Werror",
                           str(src), os.path.join(ROOT, "oracle", "sagekv_ref.c"), "-o", str(exe), "-lm"])
    # the sanitizer runtimes are linked statically, so the process environment is passed on as it is
    env = dict(os.environ, OMP_NUM_THREADS="4", UBSAN_OPTIONS="print_stacktrace=1",
               ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0")
    run = subprocess.run([str(exe)], capture_output=True, text=True, env=env, timeout=300)
    assert run.returncode == 0, run.stdout + run.stderr
    assert "oracle clean" in run.stdout
