/*
 * saap_ref.c -- CPU oracle of the SAAP decode hot path (arXiv 2502.08246).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * GPU library is checked against.  It shares no code with the GPU path and the
 * product never calls it: only the tests, the smoke check and the benchmark's
 * cpu_baseline leg load it.
 *
 * Every function works on host arrays.  Floating-point inputs are `float`
 * arrays (bf16 inputs are widened to float by the caller, which is exact);
 * all arithmetic is double precision, written as the definition reads:
 * no blocking, no partial results, no merge.  Given the bucket ids and the
 * selected buckets the method computes exactly softmax attention restricted to
 * a subset of the keys (Section 4, "Beyond top-k"), so the oracle for attention
 * is that restricted softmax written out; Algorithms 1 and 2 of Appendix F are
 * one way of evaluating it and are deliberately NOT followed here.
 *
 * Parity pins (tests/test_oracle_*.py): numpy brute force on tiny inputs, the FP8 code table
 * against the format and its encoder against a nearest-value search,
 * closed forms (equal keys -> mean of values, one key -> its value), nprobe = B
 * equals dense attention, library softmax/matmul/argsort, CSR invariants, the
 * balanced-selectivity column of the paper's Table "nprobe_selectivity"; the prefill-time
 * attention reduces to causal softmax attention (every bucket listed) and, for one token, to the
 * decode-time windowed attention.
 * Every function has at least one such pin.  The paper prints no numeric
 * attention output, score or index, so there is no worked example of those to
 * store: the pins come from the mathematics, the number format and the one
 * table of the paper that is a closed form.
 *
 * Build: gcc -O2 -fopenmp -ffp-contract=off -shared -fPIC saap_ref.c -lm
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static int g_threads = 1;

/* Number of host threads the loops over independent rows / (sequence, head) pairs may use. */
void ref_set_threads(int n) { g_threads = n > 0 ? n : 1; }
int ref_get_threads(void) { return g_threads; }

/* Inner product as the definition of saap_assign_keys states it: exact products
 * (a float times a float is exact in double), summed in index order. */
static double dot_in_order(const float* a, const float* b, int d) {
  double t = 0.0;
  for (int j = 0; j < d; ++j) t += (double)a[j] * (double)b[j];
  return t;
}

/* Section 2 (indexing step) / Section 4: each key goes to the bucket of its
 * nearest centroid.  argmax_b <x, c_b> + bias_b, lowest b on exact ties. */
void ref_assign_keys(const float* x, const float* cent, const float* bias, int32_t* ids,
                     int S, int Hkv, int N, int B, int d) {
  for (int s = 0; s < S; ++s)
    for (int h = 0; h < Hkv; ++h)
#pragma omp parallel for num_threads(g_threads) schedule(static)
      for (int n = 0; n < N; ++n) {
        const float* xr = x + (((size_t)s * Hkv + h) * N + n) * d;
        int best = 0;
        double best_t = 0.0;
        for (int b = 0; b < B; ++b) {
          double t = dot_in_order(xr, cent + ((size_t)h * B + b) * d, d);
          if (bias) t += (double)bias[(size_t)h * B + b];
          if (b == 0 || t > best_t) { best_t = t; best = b; }
        }
        ids[((size_t)s * Hkv + h) * N + n] = best;
      }
}

/* Appendix F: Off and Idx group the keys of a bucket together; bucket c holds
 * Idx[Off[c] : Off[c] + len[c]].  Members are listed in ascending position.
 * `slack` free slots follow every bucket (0 reproduces the paper's tensors).
 * Slack slots: idx = -1, Ks/Vs rows untouched. */
void ref_build_bucket_index(const int32_t* ids, const float* K, const float* V,
                            int32_t* off, int32_t* len, int32_t* idx, float* Ks, float* Vs,
                            int S, int Hkv, int N, int Ncap, int B, int d, int slack) {
  for (int u = 0; u < S * Hkv; ++u) {
    const int32_t* id = ids + (size_t)u * N;
    int32_t* o = off + (size_t)u * (B + 1);
    int32_t* l = len + (size_t)u * B;
    int32_t* ix = idx + (size_t)u * Ncap;
    for (int b = 0; b < B; ++b) l[b] = 0;
    for (int n = 0; n < N; ++n)
      if (id[n] >= 0 && id[n] < B) l[id[n]] += 1;
    o[0] = 0;
    for (int b = 0; b < B; ++b) o[b + 1] = o[b] + l[b] + slack;
    for (int j = 0; j < Ncap; ++j) ix[j] = -1;
    int32_t* fill = (int32_t*)calloc((size_t)B, sizeof(int32_t));
    for (int n = 0; n < N; ++n) {
      int b = id[n];
      if (b < 0 || b >= B) continue;
      int j = o[b] + fill[b]++;
      ix[j] = n;
      if (K && Ks) memcpy(Ks + ((size_t)u * Ncap + j) * d, K + ((size_t)u * N + n) * d, sizeof(float) * d);
      if (V && Vs) memcpy(Vs + ((size_t)u * Ncap + j) * d, V + ((size_t)u * N + n) * d, sizeof(float) * d);
    }
    free(fill);
  }
}

/* One new key per (sequence, KV head): assign as above, store it in the first
 * free slot of its bucket.  A full bucket leaves everything unchanged for that
 * key and raises the returned flag. */
int ref_append_keys(const float* x_new, const float* k_new, const float* v_new,
                    const int32_t* pos_new, const float* cent, const float* bias,
                    const int32_t* off, int32_t* len, int32_t* idx, float* Ks, float* Vs,
                    int32_t* new_ids, int S, int Hkv, int Ncap, int B, int d) {
  int overflow = 0;
  for (int s = 0; s < S; ++s)
    for (int h = 0; h < Hkv; ++h) {
      int u = s * Hkv + h;
      int32_t b;
      ref_assign_keys(x_new + (size_t)u * d, cent + (size_t)h * B * d, bias ? bias + (size_t)h * B : NULL,
                      &b, 1, 1, 1, B, d);
      new_ids[u] = b;
      const int32_t* o = off + (size_t)u * (B + 1);
      int32_t* l = len + (size_t)u * B;
      if (o[b] + l[b] >= o[b + 1]) { overflow = 1; continue; }
      int j = o[b] + l[b];
      idx[(size_t)u * Ncap + j] = pos_new ? pos_new[s] : -2;
      memcpy(Ks + ((size_t)u * Ncap + j) * d, k_new + (size_t)u * d, sizeof(float) * d);
      memcpy(Vs + ((size_t)u * Ncap + j) * d, v_new + (size_t)u * d, sizeof(float) * d);
      l[b] += 1;
    }
  return overflow;
}

/* Which of the Hw weight sets serves query head hq. */
static int weight_set(int hq, int Hq, int Hkv, int Hw) {
  if (Hw == Hq) return hq;
  if (Hw == Hkv) return hq / (Hq / Hkv);
  return 0;
}

/* Section 4 / Section 6.1: f_q is a two-layer perceptron with a ReLU; its
 * output is a distribution over the buckets (softmax of the logits).
 * hidden == 0 is the one-layer model z = W2 x + b2 with W2 [Hw,B,d]: with the
 * key centroids as W2 it is the symmetric "K-means" routing baseline of
 * Section 6.1 (queries are assigned like keys). */
void ref_classify_queries(const float* xq, const float* W1, const float* b1, const float* W2,
                          const float* b2, int Hw, float* scores, int S, int Hq, int Hkv, int d,
                          int hidden, int B, int output_kind) {
  double* hbuf = (double*)malloc(sizeof(double) * (hidden > 0 ? hidden : 1));
  double* z = (double*)malloc(sizeof(double) * B);
  for (int s = 0; s < S; ++s)
    for (int hq = 0; hq < Hq; ++hq) {
      int w = weight_set(hq, Hq, Hkv, Hw);
      const float* x = xq + ((size_t)s * Hq + hq) * d;
      for (int i = 0; i < hidden; ++i) {
        const float* wr = W1 + ((size_t)w * hidden + i) * d;
        double t = 0.0;
        for (int j = 0; j < d; ++j) t += (double)wr[j] * (double)x[j];
        if (b1) t += (double)b1[(size_t)w * hidden + i];
        hbuf[i] = t > 0.0 ? t : 0.0;
      }
      double zmax = -INFINITY;
      for (int b = 0; b < B; ++b) {
        double t = 0.0;
        if (hidden > 0) {
          const float* wr = W2 + ((size_t)w * B + b) * hidden;
          for (int i = 0; i < hidden; ++i) t += (double)wr[i] * hbuf[i];
        } else {
          const float* wr = W2 + ((size_t)w * B + b) * d;
          for (int j = 0; j < d; ++j) t += (double)wr[j] * (double)x[j];
        }
        if (b2) t += (double)b2[(size_t)w * B + b];
        z[b] = t;
        if (t > zmax) zmax = t;
      }
      float* out = scores + ((size_t)s * Hq + hq) * B;
      if (output_kind == 1) {
        for (int b = 0; b < B; ++b) out[b] = (float)z[b];
      } else {
        double sum = 0.0;
        for (int b = 0; b < B; ++b) sum += exp(z[b] - zmax);
        for (int b = 0; b < B; ++b) out[b] = (float)(exp(z[b] - zmax) / sum);
      }
    }
  free(hbuf);
  free(z);
}

typedef struct { float g; int32_t id; } scored;

static int by_score_then_id(const void* a, const void* b) {
  const scored* x = (const scored*)a;
  const scored* y = (const scored*)b;
  if (x->g > y->g) return -1;
  if (x->g < y->g) return 1;
  return (x->id > y->id) - (x->id < y->id);
}

/* Section 5 "Batched queries": sum f_q over the heads that share a KV head and
 * take the nprobe largest entries.  The sum is taken in single precision in
 * head order (this is the one place where the precision is part of the
 * definition: it decides integers).  mode 1 ranks each query head alone. */
void ref_select_buckets(const float* scores, int32_t* selected, int S, int Hq, int Hkv, int B,
                        int nprobe, int mode) {
  int G = Hq / Hkv;
  int lists = mode == 1 ? Hq : Hkv;
  int heads = mode == 1 ? 1 : G;
  scored* arr = (scored*)malloc(sizeof(scored) * (size_t)B);
  for (int s = 0; s < S; ++s)
    for (int l = 0; l < lists; ++l) {
      for (int b = 0; b < B; ++b) {
        volatile float g = scores[((size_t)s * Hq + (size_t)l * heads) * B + b];
        for (int i = 1; i < heads; ++i) g = g + scores[((size_t)s * Hq + (size_t)l * heads + i) * B + b];
        arr[b].g = g;
        arr[b].id = b;
      }
      qsort(arr, (size_t)B, sizeof(scored), by_score_then_id);
      for (int j = 0; j < nprobe; ++j) selected[((size_t)s * lists + l) * nprobe + j] = arr[j].id;
    }
  free(arr);
}

/* Softmax attention of one query over the keys whose positions are listed in
 * `members` (count entries): a_n = scale <q,k_n>; out = sum softmax(a)_n v_n;
 * lse = log sum exp a_n.  Empty list: out = 0, lse = -inf. */
static void attend_list(const float* q, const float* K, const float* V, const int32_t* members,
                        long count, double scale, int d, double* out, double* lse) {
  for (int e = 0; e < d; ++e) out[e] = 0.0;
  if (count == 0) { if (lse) *lse = -INFINITY; return; }
  double* a = (double*)malloc(sizeof(double) * (size_t)count);
  double amax = -INFINITY;
  for (long i = 0; i < count; ++i) {
    long n = members ? members[i] : i;
    const float* k = K + (size_t)n * d;
    double t = 0.0;
    for (int e = 0; e < d; ++e) t += (double)q[e] * (double)k[e];
    a[i] = t * scale;
    if (a[i] > amax) amax = a[i];
  }
  double sum = 0.0;
  for (long i = 0; i < count; ++i) {
    long n = members ? members[i] : i;
    double w = exp(a[i] - amax);
    sum += w;
    const float* v = V + (size_t)n * d;
    for (int e = 0; e < d; ++e) out[e] += w * (double)v[e];
  }
  for (int e = 0; e < d; ++e) out[e] /= sum;
  if (lse) *lse = amax + log(sum);
  free(a);
}

/* Section 4 "Beyond top-k": every key of the visited buckets enters the softmax.
 * K,V are in POSITION order [S,Hkv,Nrows,d]; the visited keys are found through
 * the index, idx[off[b] : off[b]+len[b]], as in Appendix F.  Positions of keys
 * appended after the build must be < Nrows. */
void ref_sparse_decode_attention(const float* q, const float* K, const float* V,
                                 const int32_t* off, const int32_t* len, const int32_t* idx,
                                 const int32_t* selected, int nprobe, int mode, float scale,
                                 double* out, double* lse, int S, int Hq, int Hkv, int Nrows,
                                 int Ncap, int B, int d) {
  int G = Hq / Hkv;
  int units = S * Hq;
#pragma omp parallel for num_threads(g_threads) schedule(dynamic)
  for (int t = 0; t < units; ++t) {
    int s = t / Hq, hq = t % Hq, h = hq / G;
    size_t u = (size_t)s * Hkv + h;
    const int32_t* sel = mode == 1 ? selected + (size_t)t * nprobe : selected + u * nprobe;
    long count = 0;
    for (int j = 0; j < nprobe; ++j) count += len[u * B + sel[j]];
    int32_t* members = (int32_t*)malloc(sizeof(int32_t) * (size_t)(count > 0 ? count : 1));
    long c = 0;
    for (int j = 0; j < nprobe; ++j) {
      int b = sel[j];
      for (int r = 0; r < len[u * B + b]; ++r) members[c++] = idx[u * Ncap + off[u * (B + 1) + b] + r];
    }
    attend_list(q + (size_t)t * d, K + u * Nrows * d, V + u * Nrows * d, members, count,
                (double)scale, d, out + (size_t)t * d, lse ? lse + t : NULL);
    free(members);
  }
}

/* Full softmax attention over the N keys of the head (Section 6.2 baseline). */
void ref_dense_decode_attention(const float* q, const float* K, const float* V, float scale,
                                double* out, double* lse, int S, int Hq, int Hkv, int N, int d) {
  int G = Hq / Hkv;
  int units = S * Hq;
#pragma omp parallel for num_threads(g_threads) schedule(dynamic)
  for (int t = 0; t < units; ++t) {
    int s = t / Hq, hq = t % Hq, h = hq / G;
    size_t u = (size_t)s * Hkv + h;
    attend_list(q + (size_t)t * d, K + u * N * d, V + u * N * d, NULL, N, (double)scale, d,
                out + (size_t)t * d, lse ? lse + t : NULL);
  }
}

/* Section 4 "Learning the query assignment", Eq. 1: the query model is trained towards the row of
 * A * H_k, i.e. the attention mass that falls into each bucket.  For a decode query:
 *   mass[b] = sum over the keys n with ids[n] = b of softmax_n(scale * <q, k_n>)   (softmax over all N keys)
 * Written on POSITION-ordered K [S,Hkv,N,d] and ids [S,Hkv,N]; mass [S,Hq,B] sums to 1 per row. */
void ref_bucket_attention_mass(const float* q, const float* K, const int32_t* ids, float scale, double* mass,
                               int S, int Hq, int Hkv, int N, int B, int d) {
  int G = Hq / Hkv;
  int units = S * Hq;
#pragma omp parallel for num_threads(g_threads) schedule(dynamic)
  for (int t = 0; t < units; ++t) {
    int s = t / Hq, hq = t % Hq, h = hq / G;
    size_t u = (size_t)s * Hkv + h;
    const float* qq = q + (size_t)t * d;
    double* a = (double*)malloc(sizeof(double) * (size_t)N);
    double amax = -INFINITY;
    for (int n = 0; n < N; ++n) {
      const float* k = K + (u * N + n) * d;
      double x = 0.0;
      for (int e = 0; e < d; ++e) x += (double)qq[e] * (double)k[e];
      a[n] = x * (double)scale;
      if (a[n] > amax) amax = a[n];
    }
    double sum = 0.0;
    double* m = mass + (size_t)t * B;
    for (int b = 0; b < B; ++b) m[b] = 0.0;
    for (int n = 0; n < N; ++n) {
      double w = exp(a[n] - amax);
      sum += w;
      m[ids[u * N + n]] += w;
    }
    for (int b = 0; b < B; ++b) m[b] /= sum;
    free(a);
  }
}

/* Section 3 "Per-head attention span" + Appendix F: the first n_sink keys (attention
 * sink) and the n_recent most recent keys are always attended; every other key takes
 * part only if its bucket is visited.  Written on POSITION-ordered tensors, no index:
 * K,V [S,Hkv,Nt,d], ids [S,Hkv,Nt] (bucket of every key), selected [S,Hkv,nprobe]
 * (mode 1: [S,Hq,nprobe]).  U = { n : n < n_sink  or  n >= Nt - n_recent  or
 * ids[n] in selected }. */
void ref_windowed_decode_attention(const float* q, const float* K, const float* V, const int32_t* ids,
                                   const int32_t* selected, int nprobe, int mode, int n_sink,
                                   int n_recent, float scale, double* out, double* lse, int S, int Hq,
                                   int Hkv, int Nt, int B, int d) {
  int G = Hq / Hkv;
  int units = S * Hq;
#pragma omp parallel for num_threads(g_threads) schedule(dynamic)
  for (int t = 0; t < units; ++t) {
    int s = t / Hq, hq = t % Hq, h = hq / G;
    size_t u = (size_t)s * Hkv + h;
    const int32_t* sel = mode == 1 ? selected + (size_t)t * nprobe : selected + u * nprobe;
    char* visit = (char*)calloc((size_t)B, 1);
    for (int j = 0; j < nprobe; ++j) visit[sel[j]] = 1;
    int32_t* members = (int32_t*)malloc(sizeof(int32_t) * (size_t)(Nt > 0 ? Nt : 1));
    long c = 0;
    for (int n = 0; n < Nt; ++n) {
      int b = ids[u * Nt + n];
      if (n < n_sink || n >= Nt - n_recent || (b >= 0 && b < B && visit[b])) members[c++] = n;
    }
    attend_list(q + (size_t)t * d, K + u * Nt * d, V + u * Nt * d, members, c, (double)scale, d,
                out + (size_t)t * d, lse ? lse + t : NULL);
    free(members);
    free(visit);
  }
}

/* Prefill-time sparse attention.  The paper's Conclusion names it as the next step and defines
 * nothing; the reading used here carries the decode-time rule (Section 3 "Per-head attention span",
 * Section 4 "Beyond top-k", Section 5 "Batched queries") over to a block of Tq consecutive prompt
 * tokens.  The query of token t of sequence s stands at position p = pos0[s] + t and sees, of the keys
 * at positions n <= p (causal, its own key included), with L = p + 1 keys so far:
 *     n < n_sink,  or  n >= L - n_recent,  or  ids[n] in the token's list selected[s,h,t,:],
 * one list per token and KV head, shared by the G heads of the group.  Position-ordered tensors, no index:
 * q [S,Tq,Hq,d], K,V [S,Hkv,Nt,d], ids [S,Hkv,Nt], selected [S,Hkv,Tq,nprobe], pos0 [S] with
 * pos0 + Tq <= Nt; out [S,Tq,Hq,d], lse [S,Tq,Hq]. */
void ref_prefill_sparse_attention(const float* q, const float* K, const float* V, const int32_t* ids,
                                  const int32_t* selected, const int32_t* pos0, int nprobe, int n_sink,
                                  int n_recent, float scale, double* out, double* lse, int S, int Hq,
                                  int Hkv, int Tq, int Nt, int B, int d) {
  int G = Hq / Hkv;
  long rows = (long)S * Tq * Hq;
#pragma omp parallel for num_threads(g_threads) schedule(dynamic)
  for (long r = 0; r < rows; ++r) {
    int hq = (int)(r % Hq), t = (int)((r / Hq) % Tq), s = (int)(r / ((long)Hq * Tq)), h = hq / G;
    size_t u = (size_t)s * Hkv + h;
    int L = pos0[s] + t + 1;                       /* keys the token can see at all */
    const int32_t* sel = selected + (u * Tq + t) * nprobe;
    char* visit = (char*)calloc((size_t)B, 1);
    for (int j = 0; j < nprobe; ++j) visit[sel[j]] = 1;
    int32_t* members = (int32_t*)malloc(sizeof(int32_t) * (size_t)(L > 0 ? L : 1));
    long c = 0;
    for (int n = 0; n < L; ++n) {
      int b = ids[u * Nt + n];
      if (n < n_sink || n >= L - n_recent || (b >= 0 && b < B && visit[b])) members[c++] = n;
    }
    attend_list(q + (size_t)r * d, K + u * Nt * d, V + u * Nt * d, members, c, (double)scale, d,
                out + (size_t)r * d, lse ? lse + r : NULL);
    free(members);
    free(visit);
  }
}

/* ---- index with a resident block ------------------------------------------------------
 * The paper keeps the sink + recent keys in dense tensors (K_l, V_l of Appendix F) and
 * says nothing of how a key moves from there into its bucket as generation goes on.
 * Layout used here (a reading; both sides follow it so that the state can be compared
 * bit for bit): the index has B regular buckets and one more run, number B, of exactly
 * W = n_sink + n_recent slots, the resident block.  Key at position p is resident while
 * p < n_sink or p >= Nt - n_recent, and then sits in slot
 *     r(p) = p                                   if p < n_sink
 *            n_sink + (p - n_sink) mod n_recent  otherwise,
 * so the recent part is a ring: the key entering at position p takes the slot of the key
 * at p - n_recent, which moves to the first free slot of its own bucket.
 * off [.,B+2], len [.,B+1], idx [.,Ncap], res_ids [.,W] = bucket id of each resident key
 * (-1 for an empty slot), Ncap = max(N - W, 0) + B*slack + W. */
static int resident_slot(int p, int n_sink, int n_recent) {
  return p < n_sink ? p : n_sink + (p - n_sink) % n_recent;
}

void ref_build_windowed_index(const int32_t* ids, const float* K, const float* V, int32_t* off,
                              int32_t* len, int32_t* idx, float* Ks, float* Vs, int32_t* res_ids,
                              int S, int Hkv, int N, int Ncap, int B, int d, int slack, int n_sink,
                              int n_recent) {
  int W = n_sink + n_recent;
  for (int u = 0; u < S * Hkv; ++u) {
    const int32_t* id = ids + (size_t)u * N;
    int32_t* o = off + (size_t)u * (B + 2);
    int32_t* l = len + (size_t)u * (B + 1);
    int32_t* ix = idx + (size_t)u * Ncap;
    int32_t* rid = res_ids + (size_t)u * W;
    for (int b = 0; b <= B; ++b) l[b] = 0;
    for (int j = 0; j < W; ++j) rid[j] = -1;
    for (int n = 0; n < N; ++n) {
      int resident = n < n_sink || n >= N - n_recent;
      if (resident) l[B] += 1;
      else if (id[n] >= 0 && id[n] < B) l[id[n]] += 1;
    }
    o[0] = 0;
    for (int b = 0; b < B; ++b) o[b + 1] = o[b] + l[b] + slack;
    o[B + 1] = o[B] + W;
    for (int j = 0; j < Ncap; ++j) ix[j] = -1;
    int32_t* fill = (int32_t*)calloc((size_t)B, sizeof(int32_t));
    for (int n = 0; n < N; ++n) {
      int resident = n < n_sink || n >= N - n_recent;
      int j;
      if (resident) {
        int r = resident_slot(n, n_sink, n_recent);
        j = o[B] + r;
        rid[r] = id[n];
      } else {
        int b = id[n];
        if (b < 0 || b >= B) continue;
        j = o[b] + fill[b]++;
      }
      ix[j] = n;
      memcpy(Ks + ((size_t)u * Ncap + j) * d, K + ((size_t)u * N + n) * d, sizeof(float) * d);
      memcpy(Vs + ((size_t)u * Ncap + j) * d, V + ((size_t)u * N + n) * d, sizeof(float) * d);
    }
    free(fill);
  }
}

/* One new key per (sequence, KV head) at position pos_new[s] (= the number of keys the
 * sequence held before).  The key's bucket is found as in ref_assign_keys.  It becomes
 * resident; the key it displaces (position pos - n_recent) is appended to its bucket.
 * If that bucket has no free slot nothing at all changes for this (sequence, head) and
 * the returned flag is set.  With n_recent = 0 the new key goes straight to its bucket. */
int ref_window_push(const float* x_new, const float* k_new, const float* v_new, const int32_t* pos_new,
                    const float* cent, const float* bias, const int32_t* off, int32_t* len,
                    int32_t* idx, float* Ks, float* Vs, int32_t* res_ids, int32_t* new_ids, int S,
                    int Hkv, int Ncap, int B, int d, int n_sink, int n_recent) {
  int overflow = 0;
  int W = n_sink + n_recent;
  for (int s = 0; s < S; ++s)
    for (int h = 0; h < Hkv; ++h) {
      int u = s * Hkv + h;
      int pos = pos_new[s];
      int32_t b;
      ref_assign_keys(x_new + (size_t)u * d, cent + (size_t)h * B * d, bias ? bias + (size_t)h * B : NULL,
                      &b, 1, 1, 1, B, d);
      new_ids[u] = b;
      const int32_t* o = off + (size_t)u * (B + 2);
      int32_t* l = len + (size_t)u * (B + 1);
      int32_t* ix = idx + (size_t)u * Ncap;
      float* Ku = Ks + (size_t)u * Ncap * d;
      float* Vu = Vs + (size_t)u * Ncap * d;
      int j;                      /* slot that receives the new key */
      if (pos < W) {              /* the resident block is not full yet */
        j = o[B] + resident_slot(pos, n_sink, n_recent);
        l[B] += 1;
      } else if (n_recent == 0) { /* no ring: straight into the bucket */
        if (o[b] + l[b] >= o[b + 1]) { overflow = 1; continue; }
        j = o[b] + l[b];
        l[b] += 1;
      } else {
        int r = resident_slot(pos, n_sink, n_recent);
        int e = res_ids[(size_t)u * W + r];
        j = o[B] + r;
        if (o[e] + l[e] >= o[e + 1]) { overflow = 1; continue; }
        int dst = o[e] + l[e];
        ix[dst] = ix[j];
        memcpy(Ku + (size_t)dst * d, Ku + (size_t)j * d, sizeof(float) * d);
        memcpy(Vu + (size_t)dst * d, Vu + (size_t)j * d, sizeof(float) * d);
        l[e] += 1;
      }
      if (j >= o[B]) res_ids[(size_t)u * W + (j - o[B])] = b;
      ix[j] = pos;
      memcpy(Ku + (size_t)j * d, k_new + (size_t)u * d, sizeof(float) * d);
      memcpy(Vu + (size_t)j * d, v_new + (size_t)u * d, sizeof(float) * d);
    }
  return overflow;
}

/* Fresh slack behind every bucket, nothing assigned again: members keep their bucket and
 * their order.  runs = B, or B + 1 with a resident run that keeps its slot count.
 * Returns 1 (and moves nothing) if Ncap_new is too small for some (sequence, head). */
int ref_recompact_index(const int32_t* off, const int32_t* len, const int32_t* idx, const float* Ks,
                        const float* Vs, int32_t* off_new, int32_t* idx_new, float* Kn, float* Vn,
                        int S, int Hkv, int Ncap, int Ncap_new, int B, int resident, int d, int slack_new) {
  int runs = B + resident;
  for (int u = 0; u < S * Hkv; ++u) {
    const int32_t* o = off + (size_t)u * (runs + 1);
    const int32_t* l = len + (size_t)u * runs;
    int32_t* on = off_new + (size_t)u * (runs + 1);
    on[0] = 0;
    for (int b = 0; b < B; ++b) on[b + 1] = on[b] + l[b] + slack_new;
    if (resident) on[B + 1] = on[B] + (o[B + 1] - o[B]);
    if (on[runs] > Ncap_new) return 1;
  }
  for (int u = 0; u < S * Hkv; ++u) {
    const int32_t* o = off + (size_t)u * (runs + 1);
    const int32_t* l = len + (size_t)u * runs;
    const int32_t* on = off_new + (size_t)u * (runs + 1);
    for (int j = 0; j < Ncap_new; ++j) idx_new[(size_t)u * Ncap_new + j] = -1;
    for (int b = 0; b < runs; ++b)
      for (int r = 0; r < l[b]; ++r) {
        size_t src = (size_t)u * Ncap + o[b] + r, dst = (size_t)u * Ncap_new + on[b] + r;
        idx_new[dst] = idx[src];
        memcpy(Kn + dst * d, Ks + src * d, sizeof(float) * d);
        memcpy(Vn + dst * d, Vs + src * d, sizeof(float) * d);
      }
  }
  return 0;
}

/* Centroid step of k-means (Section 4; spherical variant of Section 3): on
 * POSITION-ordered features x [S,Hkv,N,d] with their bucket ids.  c_b = mean of the
 * members of b over all sequences, divided by its norm if normalize; a bucket without
 * members keeps cent_old[b].  Output in double, not rounded. */
void ref_update_centroids(const float* x, const int32_t* ids, const float* cent_old, double* cent_new,
                          int S, int Hkv, int N, int B, int d, int normalize) {
  for (int h = 0; h < Hkv; ++h)
    for (int b = 0; b < B; ++b) {
      double* c = cent_new + ((size_t)h * B + b) * d;
      for (int e = 0; e < d; ++e) c[e] = 0.0;
      long count = 0;
      for (int s = 0; s < S; ++s)
        for (int n = 0; n < N; ++n)
          if (ids[((size_t)s * Hkv + h) * N + n] == b) {
            const float* xr = x + (((size_t)s * Hkv + h) * N + n) * d;
            for (int e = 0; e < d; ++e) c[e] += (double)xr[e];
            count += 1;
          }
      if (count == 0) {
        for (int e = 0; e < d; ++e) c[e] = (double)cent_old[((size_t)h * B + b) * d + e];
        continue;
      }
      double sq = 0.0;
      for (int e = 0; e < d; ++e) { c[e] /= (double)count; sq += c[e] * c[e]; }
      if (normalize && sq > 0.0) {
        double nrm = sqrt(sq);
        for (int e = 0; e < d; ++e) c[e] /= nrm;
      }
    }
}

/*
 * 8-bit storage of the bucket-sorted K/V (the paper calls compression of the cached vectors
 * complementary to the partition, Section 2 "Vector search based on partitions" / related work;
 * it fixes no format, so this is a reading: OCP FP8 E4M3 -- 1 sign, 4 exponent bits with
 * bias 7, 3 mantissa bits, subnormals, no infinities, largest finite value 448, codes 0x7f and
 * 0xff are NaN -- with one power-of-two scale per (sequence, KV head) and tensor:
 *   scale = 2^e, e the smallest integer with max|x| <= 448 * 2^e  (scale = 1 for an all-zero unit)
 *   code  = round-to-nearest-even of x / scale on the E4M3 grid
 * Attention on such a cache is attention on the decoded values scale * value(code), which are
 * exact in float, so the attention oracle above applies to them unchanged.
 */
float ref_fp8_e4m3_decode(uint8_t code) {
  const int sign = code >> 7, e = (code >> 3) & 15, m = code & 7;
  double v;
  if (e == 15 && m == 7) return NAN;
  if (e == 0) v = ldexp((double)m, -9);                 /* subnormal: m * 2^-6 / 8 */
  else v = ldexp(1.0 + (double)m / 8.0, e - 7);
  return (float)(sign ? -v : v);
}

uint8_t ref_fp8_e4m3_encode(float x) {
  const uint8_t sign = signbit(x) ? 0x80 : 0x00;
  double a = fabs((double)x);
  if (isnan(x)) return 0x7f;
  if (a >= 448.0) return sign | 0x7e;                   /* saturate (never reached below: |x| <= 448) */
  if (a < ldexp(1.0, -6)) {                             /* subnormal grid: multiples of 2^-9 */
    const int q = (int)nearbyint(ldexp(a, 9));          /* ties to even; q = 8 is the smallest normal */
    return sign | (uint8_t)q;
  }
  int ex;
  const double f = frexp(a, &ex);                       /* a = f * 2^ex, f in [0.5, 1) */
  int e = ex - 1;                                       /* a = (2f) * 2^e, 2f in [1, 2) */
  int q = (int)nearbyint((2.0 * f - 1.0) * 8.0);        /* ties to even */
  if (q == 8) {
    q = 0;
    e += 1;
  }
  return sign | (uint8_t)(((e + 7) << 3) | q);
}

/* scale of one unit: 2^e with the smallest e such that amax <= 448 * 2^e; 448 = 0.875 * 2^9 */
static float fp8_unit_scale(float amax) {
  if (!(amax > 0.f)) return 1.f;
  int ex;
  const float f = frexpf(amax, &ex);                    /* amax = f * 2^ex, f in [0.5, 1) */
  int e = f <= 0.875f ? ex - 9 : ex - 8;
  if (e < -100) e = -100;
  if (e > 100) e = 100;
  return ldexpf(1.f, e);
}

/* x [units, rows, d] -> codes [units, rows, d], scale [units] */
void ref_quantize_fp8(const float* x, uint8_t* codes, float* scale, long long units, long long rows, int d) {
  for (long long u = 0; u < units; ++u) {
    const float* xu = x + (size_t)u * rows * d;
    float amax = 0.f;
    for (long long i = 0; i < rows * d; ++i)
      if (fabsf(xu[i]) > amax) amax = fabsf(xu[i]);
    const float sc = fp8_unit_scale(amax);
    scale[u] = sc;
    for (long long i = 0; i < rows * d; ++i) codes[(size_t)u * rows * d + i] = ref_fp8_e4m3_encode(xu[i] / sc);
  }
}

/* Rows that join a cache whose scales are already fixed: x [units, rows, d], scale [units] ->
 * codes of x / scale, values beyond the format's range taking the largest finite code (+-448). */
void ref_quantize_fp8_scaled(const float* x, const float* scale, uint8_t* codes, long long units, long long rows,
                             int d) {
  for (long long u = 0; u < units; ++u)
    for (long long i = 0; i < rows * d; ++i) {
      float y = x[(size_t)u * rows * d + i] / scale[u];
      if (y > 448.f) y = 448.f;
      if (y < -448.f) y = -448.f;
      codes[(size_t)u * rows * d + i] = ref_fp8_e4m3_encode(y);
    }
}

/* codes [units, rows, d], scale [units] -> x [units, rows, d] = scale * value(code) (exact in float) */
void ref_dequantize_fp8(const uint8_t* codes, const float* scale, float* x, long long units, long long rows, int d) {
  for (long long u = 0; u < units; ++u)
    for (long long i = 0; i < rows * d; ++i)
      x[(size_t)u * rows * d + i] = scale[u] * ref_fp8_e4m3_decode(codes[(size_t)u * rows * d + i]);
}

/* Selectivity (Section 6.1): the fraction of keys that take part in the
 * computation, averaged over the lists (heads).  n_keys = keys per head. */
double ref_selectivity(const int32_t* len, const int32_t* selected, int lists, int B, int nprobe,
                       long n_keys) {
  double acc = 0.0;
  for (int l = 0; l < lists; ++l) {
    long c = 0;
    for (int j = 0; j < nprobe; ++j) c += len[(size_t)l * B + selected[(size_t)l * nprobe + j]];
    acc += (double)c / (double)n_keys;
  }
  return acc / lists;
}
