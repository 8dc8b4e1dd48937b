/* CPU oracle for SAGE-KV's eviction pass and reduced-cache decode attention.
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing in the product path may include, link or
 * call this file; it shares no code with the HIP library.  It is the plain
 * definition of what the method computes, in fp64, one (problem, KV head) row
 * at a time, written from the paper:
 *
 *   Sec. 2, Step 1  four-way partition of the cache (sink | candidates | recent | last token)
 *   Sec. 2, Step 2  attention scores of the last token's query, top-k per head
 *   Sec. 2, Step 3  reduced cache = Concat(sink, top-k, recent, last)
 *   Sec. 2, Step 4  decode over the reduced cache; new tokens enter the recent FIFO
 *   App. A.2        G = Hq / Hkv query heads share a KV head; kept tokens keep their order
 *
 * Readings where the paper is silent (each is restated where it is used):
 *   - indices are 0-based; "recent" here counts the last token (W = R + 1);
 *   - attention score = softmax over the WHOLE row [0, L) of q.k / sqrt(d);
 *   - head mode 0 (group-sum): the G query heads of a KV head add their
 *     probabilities, one top-k per KV head.  Head mode 1 (per-query): every
 *     query head takes its own top-k (the paper's "Hq groups of the top-k");
 *   - ties in the score go to the lower index; selection is on the fp32-rounded score;
 *   - reduced cache is ordered by ascending original position.
 *
 * Pins (tests/test_oracle_*.py): brute-force sort on tiny inputs, closed-form
 * one-hot softmax, row sums, k = E equals full attention, k = 0 keeps exactly
 * sink + recent, q = 0 tie rule, library fp64 softmax/attention cross-check.
 * The choice of the group-sum operator itself is not fixed by the paper:
 * parity unpinned for that choice (every other step is pinned).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { REF_BF16 = 0, REF_F32 = 1 };
enum { REF_GROUP_SUM = 0, REF_PER_QUERY = 1 };

static size_t elem_bytes(int dtype) { return dtype == REF_BF16 ? 2 : 4; }

/* Element `i` of a bf16 / fp32 buffer as a double (both conversions are exact). */
static double load_elem(const void* base, int dtype, int64_t i) {
  if (dtype == REF_BF16) {
    uint32_t bits = (uint32_t)((const uint16_t*)base)[i] << 16;
    float f;
    memcpy(&f, &bits, 4);
    return (double)f;
  }
  return (double)((const float*)base)[i];
}

/* logit[i] = (q . K[i]) / sqrt(d), i in [0, n)  (Step 2; the 1/sqrt(d) scale is the
 * standard attention scale of the model families the paper evaluates). */
static void row_logits(int dtype, int d, int64_t n, const void* q, int64_t q_off, const void* K,
                       int64_t k_off, double* logit) {
  double inv = 1.0 / sqrt((double)d);
  for (int64_t i = 0; i < n; ++i) {
    double acc = 0.0;
    for (int j = 0; j < d; ++j) acc += load_elem(q, dtype, q_off + j) * load_elem(K, dtype, k_off + i * d + j);
    logit[i] = acc * inv;
  }
}

/* In place: logit -> softmax probability over the whole row. */
static void row_softmax(int64_t n, double* x) {
  double m = x[0];
  for (int64_t i = 1; i < n; ++i)
    if (x[i] > m) m = x[i];
  double Z = 0.0;
  for (int64_t i = 0; i < n; ++i) {
    x[i] = exp(x[i] - m);
    Z += x[i];
  }
  for (int64_t i = 0; i < n; ++i) x[i] /= Z;
}

/* Scores of one KV head `c` of problem `p`.
 * group-sum:  s[i] = fl32( sum_{g<G} p[cG+g][i] ), one list (n_lists = 1)
 * per-query:  s[g][i] = fl32( p[cG+g][i] ), G lists                        */
static void head_scores(int dtype, int head_mode, int Hq, int Hkv, int d, int64_t L, const void* q_last,
                        const void* K, int p, int c, float* s /* [n_lists][L] */, double* tmp /* [L] */,
                        double* sum /* [L] */) {
  int G = Hq / Hkv;
  int64_t k_off = ((int64_t)p * Hkv + c) * L * d;
  if (head_mode == REF_GROUP_SUM)
    for (int64_t i = 0; i < L; ++i) sum[i] = 0.0;
  for (int g = 0; g < G; ++g) {
    int h = c * G + g; /* consecutive query heads share a KV head */
    row_logits(dtype, d, L, q_last, ((int64_t)p * Hq + h) * d, K, k_off, tmp);
    row_softmax(L, tmp);
    if (head_mode == REF_GROUP_SUM) {
      for (int64_t i = 0; i < L; ++i) sum[i] += tmp[i];
    } else {
      for (int64_t i = 0; i < L; ++i) s[(int64_t)g * L + i] = (float)tmp[i];
    }
  }
  if (head_mode == REF_GROUP_SUM)
    for (int64_t i = 0; i < L; ++i) s[i] = (float)sum[i];
}

int sagekv_ref_scores(int dtype, int head_mode, int P, int Hq, int Hkv, int d, int64_t L, const void* q_last,
                      const void* K, float* s_out) {
  if (P < 1 || Hkv < 1 || Hq % Hkv || d < 1 || L < 1) return 1;
  int G = Hq / Hkv;
  int n_lists = head_mode == REF_GROUP_SUM ? 1 : G;
  int rows = P * Hkv;
  int err = 0;
#pragma omp parallel for schedule(dynamic)
  for (int r = 0; r < rows; ++r) {
    double* tmp = (double*)malloc(sizeof(double) * L);
    double* sum = (double*)malloc(sizeof(double) * L);
    if (!tmp || !sum) {
#pragma omp atomic write
      err = 2;
    } else {
      head_scores(dtype, head_mode, Hq, Hkv, d, L, q_last, K, r / Hkv, r % Hkv, s_out + (int64_t)r * n_lists * L, tmp,
                  sum);
    }
    free(tmp);
    free(sum);
  }
  return err;
}

/* Order for the top-k: larger score first, equal scores by lower index. */
typedef struct {
  float s;
  int32_t i;
} cand_t;

static int cand_before(const void* a, const void* b) {
  const cand_t* x = (const cand_t*)a;
  const cand_t* y = (const cand_t*)b;
  if (x->s > y->s) return -1;
  if (x->s < y->s) return 1;
  return (x->i > y->i) - (x->i < y->i);
}

static int int_ascending(const void* a, const void* b) {
  int32_t x = *(const int32_t*)a, y = *(const int32_t*)b;
  return (x > y) - (x < y);
}

/* Step 2's top-k over the candidates [S, L-W): the k best by (score desc, index asc),
 * returned in ascending position (App. A.2: kept tokens keep their order). */
static void topk_candidates(const float* s, int64_t L, int S, int W, int k, cand_t* scratch, int32_t* sel) {
  int64_t E = L - S - W;
  for (int64_t j = 0; j < E; ++j) {
    scratch[j].s = s[S + j];
    scratch[j].i = (int32_t)(S + j);
  }
  qsort(scratch, (size_t)E, sizeof(cand_t), cand_before);
  for (int j = 0; j < k; ++j) sel[j] = scratch[j].i;
  qsort(sel, (size_t)k, sizeof(int32_t), int_ascending);
}

/* Eviction pass (Steps 1-3).
 *   q_last [P,Hq,d], K,V [P,Hkv,L,d] (contiguous), element type `dtype`.
 *   n_kept = S + n_lists*k + W with n_lists = 1 (group-sum) or G (per-query).
 *   kept_idx [P,Hkv,n_kept]: [0,S) ++ sel(list 0) ++ ... ++ sel(list n_lists-1) ++ [L-W,L)
 *   Kc,Vc [P,Hkv,cap,d]: rows [0,n_kept) are copies of K,V at kept_idx; the rest untouched.
 *   s_out (nullable) [P,Hkv,n_lists,L] fp32 scores.                                     */
int sagekv_ref_select(int dtype, int head_mode, int P, int Hq, int Hkv, int d, int64_t L, int S, int W, int k,
                      int cap, const void* q_last, const void* K, const void* V, void* Kc, void* Vc,
                      int32_t* kept_idx, float* s_out) {
  if (P < 1 || Hkv < 1 || Hq % Hkv || d < 1 || L < 1) return 1;
  if (S < 0 || W < 1 || k < 0 || (int64_t)S + W + k > L) return 1;
  int G = Hq / Hkv;
  int n_lists = head_mode == REF_GROUP_SUM ? 1 : G;
  int n_kept = S + n_lists * k + W;
  if (cap < n_kept) return 1;
  size_t eb = elem_bytes(dtype);
  int rows = P * Hkv;
  int err = 0;
#pragma omp parallel for schedule(dynamic)
  for (int r = 0; r < rows; ++r) {
    float* s = (float*)malloc(sizeof(float) * L * n_lists);
    double* tmp = (double*)malloc(sizeof(double) * L);
    double* sum = (double*)malloc(sizeof(double) * L);
    cand_t* scratch = (cand_t*)malloc(sizeof(cand_t) * (size_t)(L > 0 ? L : 1));
    if (!s || !tmp || !sum || !scratch) {
#pragma omp atomic write
      err = 2;
    } else {
      head_scores(dtype, head_mode, Hq, Hkv, d, L, q_last, K, r / Hkv, r % Hkv, s, tmp, sum);
      if (s_out) memcpy(s_out + (int64_t)r * n_lists * L, s, sizeof(float) * L * n_lists);
      int32_t* kept = kept_idx + (int64_t)r * n_kept;
      for (int t = 0; t < S; ++t) kept[t] = t;                                      /* sink            */
      for (int g = 0; g < n_lists; ++g)                                            /* top-k per list  */
        topk_candidates(s + (int64_t)g * L, L, S, W, k, scratch, kept + S + g * k);
      for (int t = 0; t < W; ++t) kept[S + n_lists * k + t] = (int32_t)(L - W + t); /* recent + last   */
      const char* Kr = (const char*)K + (size_t)r * L * d * eb;
      const char* Vr = (const char*)V + (size_t)r * L * d * eb;
      char* Kcr = (char*)Kc + (size_t)r * cap * d * eb;
      char* Vcr = (char*)Vc + (size_t)r * cap * d * eb;
      for (int t = 0; t < n_kept; ++t) {
        memcpy(Kcr + (size_t)t * d * eb, Kr + (size_t)kept[t] * d * eb, d * eb);
        memcpy(Vcr + (size_t)t * d * eb, Vr + (size_t)kept[t] * d * eb, d * eb);
      }
    }
    free(s);
    free(tmp);
    free(sum);
    free(scratch);
  }
  return err;
}

/* Step 4's cache update.  The recent window is the segment [seg, seg+W) of every
 * reduced row.  fifo: drop its oldest entry (the first), shift, put the new token last.
 * grow (not in the paper; keeps everything): write the new token at *len and add one. */
int sagekv_ref_append(int dtype, int P, int Hkv, int d, int cap, int seg, int W, int grow, int32_t* len,
                      const void* k_new /* [P,Hkv,d] */, const void* v_new, void* Kc, void* Vc) {
  size_t rb = (size_t)d * elem_bytes(dtype);
  if (grow && *len >= cap) return 1;
  if (!grow && (W < 1 || seg + W > cap)) return 1;
  for (int r = 0; r < P * Hkv; ++r) {
    char* Kcr = (char*)Kc + (size_t)r * cap * rb;
    char* Vcr = (char*)Vc + (size_t)r * cap * rb;
    int slot;
    if (grow) {
      slot = *len;
    } else {
      memmove(Kcr + (size_t)seg * rb, Kcr + (size_t)(seg + 1) * rb, (size_t)(W - 1) * rb);
      memmove(Vcr + (size_t)seg * rb, Vcr + (size_t)(seg + 1) * rb, (size_t)(W - 1) * rb);
      slot = seg + W - 1;
    }
    memcpy(Kcr + (size_t)slot * rb, (const char*)k_new + (size_t)r * rb, rb);
    memcpy(Vcr + (size_t)slot * rb, (const char*)v_new + (size_t)r * rb, rb);
  }
  if (grow) *len += 1;
  return 0;
}

/* out[j] = sum_t softmax_t(q.Kc[t]/sqrt(d)) Vc[t][j] over the listed positions t. */
static void attend(int dtype, int d, const void* q, int64_t q_off, const void* Kc, const void* Vc, int64_t kv_off,
                   const int32_t* pos, int n, double* w, float* out) {
  double inv = 1.0 / sqrt((double)d);
  for (int t = 0; t < n; ++t) {
    double acc = 0.0;
    for (int j = 0; j < d; ++j)
      acc += load_elem(q, dtype, q_off + j) * load_elem(Kc, dtype, kv_off + (int64_t)pos[t] * d + j);
    w[t] = acc * inv;
  }
  row_softmax(n, w);
  for (int j = 0; j < d; ++j) {
    double acc = 0.0;
    for (int t = 0; t < n; ++t) acc += w[t] * load_elem(Vc, dtype, kv_off + (int64_t)pos[t] * d + j);
    out[j] = (float)acc;
  }
}

/* Decode attention over the reduced cache (Step 4).
 *   q [P,Hq,d]; Kc,Vc [P,Hkv,cap,d]; out [P,Hq,d] fp32.
 *   group-sum: every head of the group attends positions [0, len).
 *   per-query: head g attends sink [0,S), its own list [S+g*k, S+(g+1)*k) and the
 *              recent window [S+G*k, S+G*k+W)  (len is ignored).                   */
int sagekv_ref_decode_attn(int dtype, int head_mode, int P, int Hq, int Hkv, int d, int cap, int S, int k, int W,
                           int len, const void* q, const void* Kc, const void* Vc, float* out) {
  if (P < 1 || Hkv < 1 || Hq % Hkv || d < 1) return 1;
  int G = Hq / Hkv;
  int n = head_mode == REF_GROUP_SUM ? len : S + k + W;
  if (n < 1 || (head_mode == REF_GROUP_SUM ? len : S + G * k + W) > cap) return 1;
  int err = 0;
#pragma omp parallel for schedule(dynamic)
  for (int ph = 0; ph < P * Hq; ++ph) {
    int p = ph / Hq, h = ph % Hq, c = h / G, g = h % G;
    int32_t* pos = (int32_t*)malloc(sizeof(int32_t) * n);
    double* w = (double*)malloc(sizeof(double) * n);
    if (!pos || !w) {
#pragma omp atomic write
      err = 2;
    } else {
      if (head_mode == REF_GROUP_SUM) {
        for (int t = 0; t < n; ++t) pos[t] = t;
      } else {
        int t = 0;
        for (int i = 0; i < S; ++i) pos[t++] = i;
        for (int i = 0; i < k; ++i) pos[t++] = S + g * k + i;
        for (int i = 0; i < W; ++i) pos[t++] = S + G * k + i;
      }
      attend(dtype, d, q, (int64_t)ph * d, Kc, Vc, ((int64_t)p * Hkv + c) * cap * d, pos, n, w, out + (int64_t)ph * d);
    }
    free(pos);
    free(w);
  }
  return err;
}

/* StreamLLM_R decode attention (Sec. 3.1 baselines (3a); App. A.1): the cache holds keys WITHOUT
 * rotary embedding and positions are those inside the window, not those of the original
 * sequence: the cache entry at window index i gets position i, the query (the newest entry, at
 * index len-1) gets position len-1, so positions stay in [0, len) however long the text grows.
 *   Rotary embedding at position p (RoFormer), pairs (j, j + d/2), angle p * inv_freq[j]:
 *     x'[j]       = x[j] cos - x[j + d/2] sin
 *     x'[j + d/2] = x[j + d/2] cos + x[j] sin
 *   q [P,Hq,d] and Kc [P,Hkv,cap,d] un-rotated, Kc/Vc rows in window order (sink first, then the
 *   recent tokens oldest to newest); inv_freq [d/2] fp64; out [P,Hq,d] fp32.
 * Everything in fp64 on the stored element values; one rounding to fp32 at the end.  The paper
 * does not print the pairing or the frequencies: the pairing is that of the Hugging Face
 * Llama/Qwen code the paper integrates with, the frequencies are an input.              */
int sagekv_ref_decode_attn_window_rope(int dtype, int P, int Hq, int Hkv, int d, int cap, int len, const void* q,
                                       const void* Kc, const void* Vc, const double* inv_freq, float* out) {
  if (P < 1 || Hkv < 1 || Hq % Hkv || d < 2 || d % 2 || len < 1 || len > cap) return 1;
  int G = Hq / Hkv, half = d / 2;
  int err = 0;
#pragma omp parallel for schedule(dynamic)
  for (int ph = 0; ph < P * Hq; ++ph) {
    int p = ph / Hq, h = ph % Hq, c = h / G;
    int64_t kv_off = ((int64_t)p * Hkv + c) * cap * d;
    double* qr = (double*)malloc(sizeof(double) * d);
    double* w = (double*)malloc(sizeof(double) * len);
    if (!qr || !w) {
#pragma omp atomic write
      err = 2;
    } else {
      double pq = (double)(len - 1);
      for (int j = 0; j < half; ++j) {
        double a = load_elem(q, dtype, (int64_t)ph * d + j), b = load_elem(q, dtype, (int64_t)ph * d + j + half);
        double cs = cos(pq * inv_freq[j]), sn = sin(pq * inv_freq[j]);
        qr[j] = a * cs - b * sn;
        qr[j + half] = b * cs + a * sn;
      }
      double best = -INFINITY;
      for (int i = 0; i < len; ++i) {
        double dot = 0.0;
        for (int j = 0; j < half; ++j) {
          double a = load_elem(Kc, dtype, kv_off + (int64_t)i * d + j);
          double b = load_elem(Kc, dtype, kv_off + (int64_t)i * d + j + half);
          double cs = cos((double)i * inv_freq[j]), sn = sin((double)i * inv_freq[j]);
          dot += qr[j] * (a * cs - b * sn) + qr[j + half] * (b * cs + a * sn);
        }
        w[i] = dot / sqrt((double)d);
        if (w[i] > best) best = w[i];
      }
      double denom = 0.0;
      for (int i = 0; i < len; ++i) {
        w[i] = exp(w[i] - best);
        denom += w[i];
      }
      for (int j = 0; j < d; ++j) {
        double num = 0.0;
        for (int i = 0; i < len; ++i) num += w[i] * load_elem(Vc, dtype, kv_off + (int64_t)i * d + j);
        out[(int64_t)ph * d + j] = (float)(num / denom);
      }
    }
    free(qr);
    free(w);
  }
  return err;
}

/* Independent plain attention of G query heads over one KV row, used to check the
 * "nothing evicted equals full attention" invariant.  Deliberately a different code
 * path from attend(): three explicit passes, positions given by an optional list.
 *   q [G,d], K,V [L,d], idx (nullable: all of [0,L)) [n_idx], out [G,d] fp32.       */
int sagekv_ref_full_attention(int dtype, int G, int d, int64_t L, const void* q, const void* K, const void* V,
                              const int64_t* idx, int64_t n_idx, float* out) {
  int64_t n = idx ? n_idx : L;
  if (n < 1) return 1;
  double* e = (double*)malloc(sizeof(double) * n);
  if (!e) return 2;
  for (int g = 0; g < G; ++g) {
    double best = -INFINITY;
    for (int64_t t = 0; t < n; ++t) {
      int64_t i = idx ? idx[t] : t;
      double dot = 0.0;
      for (int j = 0; j < d; ++j) dot += load_elem(K, dtype, i * d + j) * load_elem(q, dtype, (int64_t)g * d + j);
      e[t] = dot / sqrt((double)d);
      if (e[t] > best) best = e[t];
    }
    double denom = 0.0;
    for (int64_t t = 0; t < n; ++t) {
      e[t] = exp(e[t] - best);
      denom += e[t];
    }
    for (int j = 0; j < d; ++j) {
      double num = 0.0;
      for (int64_t t = 0; t < n; ++t) {
        int64_t i = idx ? idx[t] : t;
        num += e[t] * load_elem(V, dtype, i * d + j);
      }
      out[(int64_t)g * d + j] = (float)(num / denom);
    }
  }
  free(e);
  return 0;
}

/* Paper's budget rule (App. A.2): sink = B/4, k = B/(2G) per query head, recent = what is
 * left of B.  The appendix prints k = 512 for G = 7, B = 8192 although 8192/14 = 585; both
 * printed cases (G = 4 -> 1024, G = 7 -> 512) agree with "B/(2G) rounded down to a power of
 * two", which is the reading taken here. */
void sagekv_ref_paper_budget(int B, int G, int* sink, int* k, int* recent) {
  int kk = 1;
  while (2 * kk <= B / (2 * G)) kk *= 2;
  *sink = B / 4;
  *k = kk;
  *recent = B - *sink - G * kk;
}

#ifdef _OPENMP
#include <omp.h>
int sagekv_ref_threads(void) { return omp_get_max_threads(); }
#else
int sagekv_ref_threads(void) { return 1; }
#endif
