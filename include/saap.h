/*
 * saap.h -- C ABI of the SAAP decode hot path for AMD MI355X (gfx950).
 *
 * SAAP ("self-attention with asymmetric partitions", arXiv 2502.08246) keeps a
 * long-context KV cache in buckets.  Keys are assigned to buckets at prefill
 * (nearest centroid of a pre-trained k-means, Section 4); at decode a small
 * query classifier scores the buckets (Section 4, "Asymmetric assignment"),
 * the nprobe best buckets are taken jointly for the query heads that share a
 * KV head (Section 5, "Batched queries"), and exact softmax attention runs
 * over every key of the visited buckets (Section 4, "Beyond top-k";
 * Appendix F, Algorithms 1 and 2).
 *
 * Conventions shared by every call
 *   - All data pointers are DEVICE pointers unless a comment says "host".
 *     The caller owns every buffer.  The library allocates no device memory,
 *     never synchronises and never copies to the host: all work is enqueued
 *     on `stream` (a hipStream_t passed as void*, NULL = the null stream).
 *   - Data pointers must be 16-byte aligned.
 *   - Tensors are dense, row-major, innermost dimension last.
 *   - Indices are int32, 0-based (the paper's bucket ids are 1-based).
 *   - dtype: SAAP_F32 (0) or SAAP_BF16 (1).  bf16 is the upper 16 bits of
 *     the IEEE fp32 pattern.
 *   - Shapes: S sequences, Hq query heads, Hkv KV heads, G = Hq/Hkv query
 *     heads per KV head (1, 2, 4 or 8), d = 128 features per head, N keys
 *     per KV head, B buckets per KV head (the paper's C), nprobe visited
 *     buckets (the paper's l).
 *   - Return value: SAAP_OK or a negative status.  Argument checks happen
 *     on the host before anything is enqueued; a failing call enqueues
 *     nothing.  A status is also what a call returns when run on a machine
 *     without a usable GPU (SAAP_HIP_ERROR).
 *   - Workspace.  `ws` is caller-provided device scratch of at least
 *     saap_workspace_bytes(op, ...) bytes.  Its first SAAP_WS_HEADER_BYTES
 *     bytes hold arrival counters: they must be zero before the first call
 *     that uses the buffer (saap_workspace_reset does that) and every call
 *     leaves them zero again when its kernels have finished.  The rest is
 *     scratch without meaning between calls.  Two calls that run
 *     concurrently must not share a workspace.
 */
#ifndef SAAP_H
#define SAAP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  SAAP_OK = 0,
  SAAP_INVALID_ARG = -1,         /* null/misaligned pointer, bad shape, nprobe > B ... */
  SAAP_UNSUPPORTED = -2,         /* dtype / d / G / size outside what the kernels cover */
  SAAP_WORKSPACE_TOO_SMALL = -3,
  SAAP_BUCKET_FULL = -4,         /* reserved: reported through overflow_flag on the device */
  SAAP_HIP_ERROR = -5            /* a HIP runtime call failed (no GPU, launch error) */
};

enum { SAAP_F32 = 0, SAAP_BF16 = 1 };

/* select_buckets / sparse_decode_attention routing modes */
enum {
  SAAP_GROUP_SUM = 0,   /* one bucket list per KV head from the summed scores of its G heads */
  SAAP_INDEPENDENT = 1  /* one bucket list per query head */
};

/* classify_queries output kinds */
enum { SAAP_PROBS = 0, SAAP_LOGITS = 1 };

/* operation ids for saap_workspace_bytes */
enum {
  SAAP_OP_ASSIGN_KEYS = 0,
  SAAP_OP_BUILD_BUCKET_INDEX = 1,
  SAAP_OP_CLASSIFY_QUERIES = 2,
  SAAP_OP_SELECT_BUCKETS = 3,
  SAAP_OP_SPARSE_DECODE_ATTENTION = 4,
  SAAP_OP_DENSE_DECODE_ATTENTION = 5,
  SAAP_OP_APPEND_KEYS = 6,
  SAAP_OP_WINDOW_PUSH = 7,
  SAAP_OP_BUCKET_ATTENTION_MASS = 8,
  SAAP_OP_QUERY_MODEL_LOSS_GRADS = 9,  /* shape: Hkv = weight sets, N = rows per set, d, hidden, B */
  SAAP_OP_BUCKET_ATTENTION_MASS_BATCH = 10,  /* shape: S, Hkv, N = queries per KV head, B */
  SAAP_OP_PLANNED_DECODE_ATTENTION = 11,     /* shape: S, Hq, Hkv, mode */
  SAAP_OP_PREFILL_SPARSE_ATTENTION = 12      /* shape: S, Hq, Hkv, N = query tokens per sequence (Tq), nprobe */
};

#define SAAP_WS_HEADER_BYTES 65536u
#define SAAP_STATIC_SCRATCH_BYTES (8u << 20)   /* scratch built into the library for saap_sparse_decode_attention_noalloc */
#define SAAP_MAX_BUCKETS 8192      /* B and nprobe limit of select / sparse attention */
#define SAAP_HEAD_DIM 128

/* Shape record used only by saap_workspace_bytes; unused fields may be 0. */
typedef struct {
  int32_t S, Hq, Hkv, N, B, nprobe, d, hidden, dtype, mode;
} saap_shape;

/* Bytes of workspace `op` needs for `shape` (header included); 0 if the op or
 * shape is invalid.  Pure host arithmetic. */
size_t saap_workspace_bytes(int32_t op, const saap_shape* shape /* host */);

/* Enqueue a fill kernel that zeroes the workspace header. */
int32_t saap_workspace_reset(void* ws, size_t ws_bytes, void* stream);

/* Human-readable name of a status code (host string, never NULL). */
const char* saap_status_string(int32_t status);

/* Number of compute units of the current device (host query; <= 0 on error). */
int32_t saap_device_compute_units(void);

/* Measurement aid, not part of the method: reads `bytes` of device memory once with 16-byte
 * loads that carry the non-temporal hint (as the attention kernels read K and V) and folds
 * them into `sink` (device, >= 4 * 4 * compute units bytes).  Its
 * bandwidth is the streaming-read ceiling that the attention kernels are reported against
 * beside the published HBM peak. */
int32_t saap_stream_read_probe(const void* src, size_t bytes, void* sink, size_t sink_bytes, void* stream);

/* Measurement aid, not part of the method: every wave of `wgs_per_cu` (1..8) four-wave workgroups per
 * compute unit runs `iters` rounds of eight independent v_mfma_f32_32x32x16_bf16 (the instruction of
 * assign_keys) on operands it reads once from `operands` (device, bf16 values, `bytes` >= 64, 16-byte
 * aligned; lanes wrap around the buffer), with no other memory traffic.  `*flop_out` (host, may be
 * NULL) receives the floating-point operations of the launch; the caller times it.  `sink` (device,
 * >= 4 bytes) is written practically never.  The rate depends on the operand VALUES (the device
 * lowers its clock under the switching activity of random data), which is what this call shows. */
int32_t saap_mfma_rate_probe(const void* operands, size_t bytes, int32_t iters, int32_t wgs_per_cu, void* sink,
                             double* flop_out /* host */, void* stream);

/*
 * assign_keys -- prefill-time assignment of keys to buckets.
 * Section 2 ("Vector search based on partitions", indexing step) and Section 4:
 * a key goes to exactly one bucket, that of its nearest centroid.
 *   bucket_ids[s,h,n] = argmax_b ( <x[s,h,n,:], centroids[h,b,:]> + bias[h,b] )
 * with the inner product taken as the sum, in index order, of the exact
 * products in double precision, and the lowest b winning exact ties.  bias ==
 * NULL is maximum inner product (spherical k-means with unit centroids);
 * bias[b] = -|c_b|^2/2 is the Euclidean nearest centroid.  The features x are
 * what the clustering was trained on (keys before RoPE, Section 4
 * "Assigning with(out) RoPE"), not necessarily the cached keys.
 *   x          [S,Hkv,N,d]  dtype
 *   centroids  [Hkv,B,d]    dtype
 *   bias       [Hkv,B]      fp32 or NULL
 *   bucket_ids [S,Hkv,N]    int32, out
 * bf16 inputs run on the matrix cores with fp32 accumulation; rows whose best
 * two scores are closer than the accumulation error bound are re-scored in
 * double precision, so the result is the argmax defined above bit for bit.
 */
int32_t saap_assign_keys(const void* x, const void* centroids, const float* bias,
                         int32_t* bucket_ids,
                         int32_t S, int32_t Hkv, int32_t N, int32_t B, int32_t d, int32_t dtype,
                         void* ws, size_t ws_bytes, void* stream);

/*
 * build_bucket_index -- the CSR index of Appendix F (tensors Off and Idx) plus
 * a bucket-sorted copy of K and V, so that a bucket is one contiguous run
 * (Section 2 notes that an inverted file ideally stores a bucket contiguously).
 *   len[s,h,b]   = number of keys n with bucket_ids[s,h,n] == b
 *   off[s,h,0]   = 0,  off[s,h,b+1] = off[s,h,b] + len[s,h,b] + slack
 *   idx[s,h,off[b]+r] = position of the r-th member of b, members in
 *                  ascending position (stable); slack slots hold -1
 *   Ksorted[s,h,j,:] = K[s,h,idx[j],:] (likewise V) for member slots;
 *                  slack slots are left untouched
 * The paper's Off has no slack (slack = 0 gives off[B] = N).  slack > 0
 * reserves free slots behind every bucket for saap_append_keys.
 * Ncap must equal N + B*slack.
 *   bucket_ids [S,Hkv,N] int32; K,V [S,Hkv,N,d] dtype
 *   off [S,Hkv,B+1], len [S,Hkv,B], idx [S,Hkv,Ncap] int32, out
 *   Ksorted,Vsorted [S,Hkv,Ncap,d] dtype, out
 * Ids outside [0,B) are a caller error; such keys are dropped from the index.
 */
int32_t saap_build_bucket_index(const int32_t* bucket_ids, const void* K, const void* V,
                                int32_t* off, int32_t* len, int32_t* idx,
                                void* Ksorted, void* Vsorted,
                                int32_t S, int32_t Hkv, int32_t N, int32_t Ncap, int32_t B,
                                int32_t d, int32_t dtype, int32_t slack,
                                void* ws, size_t ws_bytes, void* stream);

/*
 * append_keys -- one decode step's new key per (sequence, KV head): assign it
 * as in saap_assign_keys and store it in the first free slot of its bucket.
 * The paper needs the index to absorb keys during generation (Section 1) and
 * gives no mechanism; this layout uses the slack slots of build_bucket_index.
 *   x_new [S,Hkv,d] features; k_new, v_new [S,Hkv,d] cache rows (dtype)
 *   pos_new [S] int32 (>= 0) or NULL: position recorded in idx (NULL records -2)
 *   new_bucket_ids [S,Hkv] int32, out
 *   overflow_flag  device int32: set to 1 if some bucket had no free slot;
 *                  that key is not stored (len unchanged), others are.
 * Workspace: SAAP_OP_APPEND_KEYS (S, Hkv, B): the centroids are scored by ceil(B/64)
 * workgroups per (sequence, head), which meet through it.
 */
int32_t saap_append_keys(const void* x_new, const void* k_new, const void* v_new,
                         const int32_t* pos_new,
                         const void* centroids, const float* bias,
                         const int32_t* off, int32_t* len, int32_t* idx,
                         void* Ksorted, void* Vsorted,
                         int32_t* new_bucket_ids, int32_t* overflow_flag,
                         int32_t S, int32_t Hkv, int32_t Ncap, int32_t B, int32_t d, int32_t dtype,
                         void* ws, size_t ws_bytes, void* stream);

/*
 * classify_queries -- the query assignment model f_q of Section 4 (a two-layer
 * perceptron with ReLU, Section 6.1; batch-norm folded into W1,b1 by the caller):
 *   h = max(0, W1 x + b1);  z = W2 h + b2;  scores = softmax(z)  (or z itself)
 *   xq [S,Hq,d] dtype (query features, before RoPE)
 *   W1 [Hw,hidden,d], W2 [Hw,B,hidden] dtype; b1 [Hw,hidden], b2 [Hw,B] fp32 or NULL
 *   Hw weight sets: 1 (shared), Hkv (one per KV head) or Hq (one per query head)
 *   scores [S,Hq,B] fp32, out
 * hidden must be a multiple of 32 and B a multiple of 16.
 * hidden = 0 selects the one-layer model z = W2 x + b2 with W2 [Hw,B,d] (W1, b1 unused, may
 * be NULL): with the key centroids as W2 and Hw = Hkv it is the symmetric "K-means" routing
 * of Section 6.1, where a query goes to the buckets of its nearest centroids as a key does.
 */
int32_t saap_classify_queries(const void* xq, const void* W1, const float* b1,
                              const void* W2, const float* b2, int32_t Hw,
                              float* scores,
                              int32_t S, int32_t Hq, int32_t Hkv, int32_t d, int32_t hidden, int32_t B,
                              int32_t dtype, int32_t output_kind,
                              void* ws, size_t ws_bytes, void* stream);

/*
 * select_buckets -- the nprobe most promising buckets (Section 4; Section 5
 * "Batched queries": the scores of the G heads sharing a KV head are summed and
 * one list is taken for the group).
 *   GROUP_SUM:   g[s,h,b] = ((p_0 + p_1) + p_2) + ... over the group's heads in
 *                head order, in fp32; selected [S,Hkv,nprobe]
 *   INDEPENDENT: g = the head's own scores; selected [S,Hq,nprobe]
 * The list holds the nprobe largest g, ordered by (g descending, id
 * ascending); equal scores resolve to the lower id.  Scores must be finite.
 * 0 <= nprobe <= B <= SAAP_MAX_BUCKETS.
 */
int32_t saap_select_buckets(const float* scores, int32_t* selected,
                            int32_t S, int32_t Hq, int32_t Hkv, int32_t B, int32_t nprobe,
                            int32_t mode, void* ws, size_t ws_bytes, void* stream);

/*
 * select_buckets_from_logits -- saap_select_buckets with the last step of the query
 * classifier folded in (Section 4 "Asymmetric assignment": f_q ends in a distribution over
 * the buckets; Section 5 "Batched queries": the distributions of a group are summed), one
 * launch less per decode step:
 *   p[s,hq,:] = softmax(logits[s,hq,:]) in fp32,  then select as saap_select_buckets does on p.
 *   logits [S,Hq,B] fp32 as written by saap_classify_queries with SAAP_LOGITS
 *   probs  [S,Hq,B] fp32 out, or NULL: the probabilities the selection was made from
 *          (written when nprobe > 0)
 * Covers nprobe up to half of B rounded up to a power of two (the range served by the radix
 * selection) and G in {1, 2, 4, 8}; otherwise SAAP_UNSUPPORTED, and the caller uses SAAP_PROBS +
 * saap_select_buckets.
 */
int32_t saap_select_buckets_from_logits(const float* logits, float* probs, int32_t* selected,
                                        int32_t S, int32_t Hq, int32_t Hkv, int32_t B, int32_t nprobe,
                                        int32_t mode, void* ws, size_t ws_bytes, void* stream);

/*
 * classify_select -- the routing of a decode step in one call: saap_classify_queries with SAAP_LOGITS
 * followed by saap_select_buckets_from_logits (or, with `plan` != NULL, saap_select_buckets_planned)
 * in SAAP_GROUP_SUM mode: f_q of Section 4 for every query head, its distributions summed over the
 * heads of a group and the nprobe best buckets taken (Section 5 "Batched queries").  The results are
 * those of the separate calls, bit for bit.
 *   logits [S,Hq,B] fp32, out; probs [S,Hq,B] fp32 out or NULL; selected [S,Hkv,nprobe] int32, out
 *   plan: NULL, or the visit plan of the lists (then off, len and resident_run as in
 *   saap_select_buckets_planned); the remaining arguments as in saap_classify_queries.
 * At batch 1 with one weight set per KV head (S = 1, Hw = Hkv, bf16, B <= 4096) the selection runs inside
 * the classifier's output launch: the last workgroup of a weight set to finish selects its list, so the
 * step has one launch less.  Every other shape takes the separate launches.
 * Workspace: SAAP_OP_CLASSIFY_QUERIES.
 */
int32_t saap_classify_select(const void* xq, const void* W1, const float* b1,
                             const void* W2, const float* b2, int32_t Hw,
                             float* logits, float* probs, int32_t* selected,
                             const int32_t* off, const int32_t* len, int32_t resident_run, int32_t* plan,
                             int32_t S, int32_t Hq, int32_t Hkv, int32_t d, int32_t hidden, int32_t B,
                             int32_t nprobe, int32_t dtype,
                             void* ws, size_t ws_bytes, void* stream);

/*
 * sparse_decode_attention -- exact softmax attention over the union of the
 * selected buckets (Section 4 "Beyond top-k"; Appendix F Algorithms 1 and 2:
 * partial attention with a running maximum, then a log-sum-exp merge):
 *   U = all member slots of the selected buckets
 *   a_n = scale * <q, k_n>,  out = sum_n softmax(a)_n v_n,  lse = log sum_n exp(a_n)
 *   q [S,Hq,d] dtype (after RoPE); Ksorted,Vsorted [S,Hkv,Ncap,d] dtype
 *   off [S,Hkv,B+1], len [S,Hkv,B]; selected as written by saap_select_buckets
 *   out [S,Hq,d] of out_dtype; lse [S,Hq] fp32 or NULL
 * All G heads of a group are computed together from one read of K and V
 * (GROUP_SUM).  With INDEPENDENT lists (selected [S,Hq,nprobe]) the union of the
 * G lists of a group is read once and every head attends only the keys of its own
 * list (B <= 8192; beyond that every head reads its list separately).
 * An empty selection gives out = 0, lse = -inf.
 * Bucket ids in `selected` must be distinct and inside [0,B).
 * Arithmetic: scores, softmax weights, sums and the merge in fp32.  On bf16 caches the weighted sum
 * of the values runs on the matrix cores, where a weight enters with 16 significant bits (two bf16
 * parts) and a bf16 value exactly; fp32 caches use fp32 throughout.
 */
int32_t saap_sparse_decode_attention(const void* q, const void* Ksorted, const void* Vsorted,
                                     const int32_t* off, const int32_t* len,
                                     const int32_t* selected, int32_t nprobe, int32_t mode,
                                     float scale, void* out, int32_t out_dtype, float* lse,
                                     int32_t S, int32_t Hq, int32_t Hkv, int32_t Ncap, int32_t B,
                                     int32_t d, int32_t dtype,
                                     void* ws, size_t ws_bytes, void* stream);

/*
 * select_attend -- saap_select_buckets_from_logits and saap_sparse_decode_attention in one call:
 * the nprobe best buckets of every KV head's group (Section 5 "Batched queries": the classifier
 * outputs of the G heads, here their softmax over the logits, are summed and the top nprobe taken,
 * ordered by score descending, id ascending), then exact attention over those buckets (Section 4
 * "Beyond top-k", Appendix F Algorithms 1 and 2).
 *   logits [S,Hq,B] fp32 (saap_classify_queries with SAAP_LOGITS); selected [S,Hkv,nprobe] int32 is
 *   an OUTPUT (the lists attended, identical to what saap_select_buckets_from_logits returns);
 *   every other argument as in saap_sparse_decode_attention with mode SAAP_GROUP_SUM.
 * For bf16 and 8-bit caches, 64 <= B <= 4096 and lists shorter than half of B (rounded up to powers
 * of two) it is ONE launch: every workgroup of a (sequence, KV head) derives the list itself from
 * the logits and goes on to attend, which saves a launch and a dependent memory round trip per
 * decode step.  Other shapes run as the two calls; the results are the same either way.
 * Workspace: SAAP_OP_SPARSE_DECODE_ATTENTION.
 */
int32_t saap_select_attend(const float* logits, const void* q, const void* Ksorted, const void* Vsorted,
                           const int32_t* off, const int32_t* len, int32_t nprobe, float scale,
                           int32_t* selected, void* out, int32_t out_dtype, float* lse,
                           int32_t S, int32_t Hq, int32_t Hkv, int32_t Ncap, int32_t B, int32_t d,
                           int32_t dtype, void* ws, size_t ws_bytes, void* stream);

/* The same over an index with a resident run (saap_build_windowed_index): the attention sink and the recent
 * keys (Section 3 "Per-head attention span") are visited after the selected buckets, as by
 * saap_windowed_decode_attention.  B counts the buckets (the columns of `logits`); resident_run is B,
 * or -1 for an index without such a run (then this is saap_select_attend). */
int32_t saap_select_attend_windowed(const float* logits, const void* q, const void* Ksorted, const void* Vsorted,
                                    const int32_t* off, const int32_t* len, int32_t nprobe, int32_t resident_run,
                                    float scale, int32_t* selected, void* out, int32_t out_dtype, float* lse,
                                    int32_t S, int32_t Hq, int32_t Hkv, int32_t Ncap, int32_t B, int32_t d,
                                    int32_t dtype, void* ws, size_t ws_bytes, void* stream);

/* The same on an 8-bit cache written by saap_quantize_kv (q bf16). */
int32_t saap_select_attend_fp8(const float* logits, const void* q, const uint8_t* K8, const uint8_t* V8,
                               const float* kscale, const float* vscale, const int32_t* off,
                               const int32_t* len, int32_t nprobe, float scale, int32_t* selected,
                               void* out, int32_t out_dtype, float* lse,
                               int32_t S, int32_t Hq, int32_t Hkv, int32_t Ncap, int32_t B, int32_t d,
                               void* ws, size_t ws_bytes, void* stream);

/*
 * sparse_decode_attention_noalloc -- saap_sparse_decode_attention for callers that cannot allocate or
 * pass device scratch: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  The arguments, the result and the limits are those of saap_sparse_decode_attention
 * without `ws` / `ws_bytes`: the partial results and arrival counters live in a device array built
 * into the library (SAAP_STATIC_SCRATCH_BYTES = 8 MiB per GPU, held from the first call on that
 * GPU until the process ends).  The call allocates nothing and frees nothing; it enqueues a small
 * fill kernel that clears the array's counters and then the attention kernel, both on `stream`.
 *   Shapes whose scratch would exceed the array (about S*Hkv*(Hq/Hkv) > 120 heads in one call, or
 *   more than 512 lists) return SAAP_WORKSPACE_TOO_SMALL before anything is enqueued; so do invalid
 *   arguments (the codes of saap_sparse_decode_attention), checked before the device is touched.
 *   Every call on a GPU shares that GPU's array: calls that overlap in time on one GPU (two
 *   streams, two threads) race and must be serialised by the caller.
 */
int32_t saap_sparse_decode_attention_noalloc(const void* q, const void* Ksorted, const void* Vsorted,
                                             const int32_t* off, const int32_t* len,
                                             const int32_t* selected, int32_t nprobe, int32_t mode,
                                             float scale, void* out, int32_t out_dtype, float* lse,
                                             int32_t S, int32_t Hq, int32_t Hkv, int32_t Ncap, int32_t B,
                                             int32_t d, int32_t dtype, void* stream);

/*
 * dense_decode_attention -- softmax attention over every key (the full-attention
 * baseline of Section 6.2), as a uniform split of the keys over workgroups with
 * the same merge (the Flash-Decoding scheme Section 5 refers to).
 *   off == NULL: K,V are packed [S,Hkv,N,d].
 *   off != NULL: K,V are a bucket-sorted cache [S,Hkv,N,d] with N = Ncap; only
 *                member slots (off[b] .. off[b]+len[b]) are attended; B buckets.
 */
int32_t saap_dense_decode_attention(const void* q, const void* K, const void* V,
                                    const int32_t* off, const int32_t* len, int32_t B,
                                    float scale, void* out, int32_t out_dtype, float* lse,
                                    int32_t S, int32_t Hq, int32_t Hkv, int32_t N, int32_t d,
                                    int32_t dtype,
                                    void* ws, size_t ws_bytes, void* stream);

/*
 * ---- attention sink and recent keys (Section 3 "Per-head attention span"; Appendix F) ----
 * The paper attends the first key(s) of the sequence and the most recent ones exhaustively
 * ("1+2047") and searches only the remaining keys through the buckets; Algorithm 2 of
 * Appendix F gives those dense keys one more block of the partial-attention launch.  The
 * paper keeps them in separate tensors and does not say how a key moves into its bucket
 * when it leaves the window.  Layout used here: the sorted cache has B regular buckets and
 * one more run, number B, of exactly W = n_sink + n_recent slots, the resident block.
 * The key at position p is resident while p < n_sink or p >= (keys so far) - n_recent and
 * then sits in slot  r(p) = p  for p < n_sink,  n_sink + (p - n_sink) mod n_recent
 * otherwise: the recent part is a ring.
 *
 * build_windowed_index -- saap_build_bucket_index with the resident keys kept out of the
 * buckets.
 *   off [S,Hkv,B+2]: off[b+1] = off[b] + len[b] + slack for b < B, off[B+1] = off[B] + W
 *   len [S,Hkv,B+1]: len[B] = number of resident keys (min(N, W) after the build)
 *   idx [S,Hkv,Ncap], Ksorted, Vsorted [S,Hkv,Ncap,d]; free slots hold idx = -1
 *   resident_ids [S,Hkv,W] int32, out: bucket id of the key in each resident slot (-1: empty)
 *   Ncap must equal max(N - W, 0) + B*slack + W.  n_sink, n_recent >= 0.
 * Workspace: as SAAP_OP_BUILD_BUCKET_INDEX for the same S, Hkv, N, B.
 */
int32_t saap_build_windowed_index(const int32_t* bucket_ids, const void* K, const void* V,
                                  int32_t* off, int32_t* len, int32_t* idx,
                                  void* Ksorted, void* Vsorted, int32_t* resident_ids,
                                  int32_t S, int32_t Hkv, int32_t N, int32_t Ncap, int32_t B,
                                  int32_t d, int32_t dtype, int32_t slack,
                                  int32_t n_sink, int32_t n_recent,
                                  void* ws, size_t ws_bytes, void* stream);

/*
 * window_push -- one decode step's new key per (sequence, KV head) enters the resident
 * block; the key it displaces (position pos - n_recent) is appended to the first free slot
 * of its own bucket (its id was kept in resident_ids).  The new key's bucket is found as in
 * saap_assign_keys (double precision, lowest id on ties) and stored for its later move.
 *   x_new, k_new, v_new [S,Hkv,d] dtype; pos_new [S] int32: position of the new key
 *   (= number of keys the sequence held before; pushes must come in position order);
 *   centroids [Hkv,B,d], bias [Hkv,B] or NULL; off, len, idx, Ksorted, Vsorted,
 *   resident_ids as written by saap_build_windowed_index (updated in place);
 *   new_bucket_ids [S,Hkv] int32, out; overflow_flag: one device int32.
 * While the block is not full (pos < W) the key takes slot r(pos) and nothing moves.  With
 * n_recent = 0 the new key goes straight into its bucket.  If the bucket that must take a
 * key has no free slot, nothing changes for that (sequence, head), *overflow_flag is set
 * to 1 and the caller rebuilds the index; the flag is never cleared by the library.
 * Workspace: SAAP_OP_WINDOW_PUSH (S, Hkv, B): the centroids are scored by ceil(B/64)
 * workgroups per (sequence, head), which meet through it.
 */
int32_t saap_window_push(const void* x_new, const void* k_new, const void* v_new,
                         const int32_t* pos_new, const void* centroids, const float* bias,
                         const int32_t* off, int32_t* len, int32_t* idx,
                         void* Ksorted, void* Vsorted, int32_t* resident_ids,
                         int32_t* new_bucket_ids, int32_t* overflow_flag,
                         int32_t S, int32_t Hkv, int32_t Ncap, int32_t B, int32_t d, int32_t dtype,
                         int32_t n_sink, int32_t n_recent,
                         void* ws, size_t ws_bytes, void* stream);

/*
 * windowed_decode_attention -- saap_sparse_decode_attention over the selected buckets
 * AND one run that is always visited (Algorithm 2 of Appendix F: block 0 handles the dense
 * keys, blocks 1..nprobe the buckets; here it is one more run of the same launch).
 *   runs            number of runs per (sequence, head) in `len` (B + 1 for an index made
 *                   by saap_build_windowed_index); off [S,Hkv,runs+1], len [S,Hkv,runs]
 *   resident_run    the run that is always visited (B for such an index), or -1 for none
 *   selected        [S,Hkv,nprobe] (or [S,Hq,nprobe]); must not contain resident_run
 * nprobe = 0 attends the resident block alone (sink + recent keys only).
 * Workspace: as SAAP_OP_SPARSE_DECODE_ATTENTION.
 */
int32_t saap_windowed_decode_attention(const void* q, const void* Ksorted, const void* Vsorted,
                                       const int32_t* off, const int32_t* len,
                                       const int32_t* selected, int32_t nprobe, int32_t mode,
                                       int32_t resident_run,
                                       float scale, void* out, int32_t out_dtype, float* lse,
                                       int32_t S, int32_t Hq, int32_t Hkv, int32_t Ncap, int32_t runs,
                                       int32_t d, int32_t dtype,
                                       void* ws, size_t ws_bytes, void* stream);

/*
 * recompact_index -- index maintenance during long generations: when a bucket's slack has
 * run out (overflow flag of saap_append_keys / saap_window_push) the cache is laid out afresh
 * with `slack_new` free slots behind every bucket, WITHOUT assigning any key again: every
 * member keeps its bucket and its order, only the offsets change.  (The paper needs the index
 * to take new keys during generation, Section 1, and gives no mechanism.)
 *   off, len, idx, Ksorted, Vsorted: the current index ([.,runs+1], [.,runs], [.,Ncap], [.,Ncap,d])
 *   resident: 1 if the index has a resident run behind its B buckets (it keeps its slot count)
 *   off_new [S,Hkv,runs+1], idx_new [S,Hkv,Ncap_new], Ksorted_new, Vsorted_new [S,Hkv,Ncap_new,d]: out;
 *   they must not alias the inputs.  len is valid for both layouts.  resident_ids stays valid.
 *   Ncap_new must hold sum(len) + B*slack_new (+ the resident slots) of every (sequence, head);
 *   if it does not, *overflow_flag (device int32, zeroed by the caller) is set and nothing is moved.
 */
int32_t saap_recompact_index(const int32_t* off, const int32_t* len, const int32_t* idx,
                             const void* Ksorted, const void* Vsorted,
                             int32_t* off_new, int32_t* idx_new, void* Ksorted_new, void* Vsorted_new,
                             int32_t* overflow_flag,
                             int32_t S, int32_t Hkv, int32_t Ncap, int32_t Ncap_new, int32_t B,
                             int32_t resident, int32_t d, int32_t dtype, int32_t slack_new, void* stream);

/*
 * update_centroids -- the centroid step of the k-means that defines the buckets (Section 4
 * "Learning the key assignment"; the spherical variant is the one Section 3 uses; Appendix A):
 *   c_b <- mean of the member features of bucket b over all sequences, divided by its norm if
 *   normalize != 0; a bucket without members keeps centroids_old[b].
 * saap_assign_keys (assignment), saap_build_bucket_index applied to the FEATURES (grouping) and
 * this call make one Lloyd iteration on the device.
 *   x_sorted [S,Hkv,Ncap,d] dtype: features grouped by bucket; off [S,Hkv,B+1], len [S,Hkv,B]
 *   centroids_old, centroids_new [Hkv,B,d] dtype (may be the same buffer)
 * Sums are taken in fp32 in a fixed order (reproducible); the result is rounded to dtype.
 */
int32_t saap_update_centroids(const void* x_sorted, const int32_t* off, const int32_t* len,
                              const void* centroids_old, void* centroids_new,
                              int32_t S, int32_t Hkv, int32_t Ncap, int32_t B, int32_t d, int32_t dtype,
                              int32_t normalize, void* stream);

/*
 * bucket_attention_mass -- the share of a query's softmax attention that falls into each
 * bucket: the row of A * H_k that the query model is trained towards (Section 4 "Learning the
 * query assignment", Eq. 1: KL divergence between f_q(q) and that row), and, summed over a
 * selection, the attention mass the selection captures:
 *   mass[s,hq,b] = sum over the member slots n of bucket b of softmax_n(scale * <q, k_n>),
 *   the softmax taken over all member slots of the (sequence, KV head).
 *   q [S,Hq,d] dtype; Ksorted [S,Hkv,Ncap,d] dtype; off [S,Hkv,B+1], len [S,Hkv,B]
 *   mass [S,Hq,B] fp32, out (rows sum to 1; all zero for a head without keys)
 *   lse  [S,Hq] fp32 or NULL, out: log sum_n exp(scale * <q, k_n>) over all member slots
 * Workspace: SAAP_OP_BUCKET_ATTENTION_MASS (S, Hq, Hkv, B).
 */
int32_t saap_bucket_attention_mass(const void* q, const void* Ksorted,
                                   const int32_t* off, const int32_t* len,
                                   float scale, float* mass, float* lse,
                                   int32_t S, int32_t Hq, int32_t Hkv, int32_t Ncap, int32_t B,
                                   int32_t d, int32_t dtype,
                                   void* ws, size_t ws_bytes, void* stream);

/*
 * bucket_attention_mass_batch -- saap_bucket_attention_mass for a training batch: R queries per
 * (sequence, KV head) instead of the G heads of a decode step (Section 4 "Query assignment
 * function": the rows of A * H_k for the sampled queries of a prompt).  The scores run on the
 * matrix cores, so the keys are read once per 128 queries.
 *   q [S,Hkv,R,d] bf16; Ksorted [S,Hkv,Ncap,d] bf16; off [S,Hkv,B+1], len [S,Hkv,B]
 *   mass [S,Hkv,R,B] fp32, out; lse [S,Hkv,R] fp32 or NULL, out
 * Workspace: SAAP_OP_BUCKET_ATTENTION_MASS_BATCH (S, Hkv, N = R, B): 8 bytes per (query, bucket).
 */
int32_t saap_bucket_attention_mass_batch(const void* q, const void* Ksorted,
                                         const int32_t* off, const int32_t* len,
                                         float scale, float* mass, float* lse,
                                         int32_t S, int32_t Hkv, int32_t R, int32_t Ncap, int32_t B,
                                         int32_t d, int32_t dtype,
                                         void* ws, size_t ws_bytes, void* stream);

/*
 * ---- training of the query model (Section 4 "Query assignment function", Eq. 1) ----
 * The two-layer model of saap_classify_queries in fp32:
 *   z = W2 relu(W1 x + b1) + b2,  f_q(x) = softmax(z)
 *   W1 [Hw,hidden,d], b1 [Hw,hidden], W2 [Hw,B,hidden], b2 [Hw,B]   (device, fp32; Hw weight sets)
 */
typedef struct {
  float* W1;
  float* b1;
  float* W2;
  float* b2;
} saap_mlp_f32;   /* host struct of device pointers */

/*
 * query_model_loss_grads -- loss of Eq. 1 and its gradients for one batch per weight set:
 *   L[w] = 1/R sum_r sum_b T[w,r,b] (log T[w,r,b] - log f_q(x[w,r])[b]),   0 log 0 = 0
 * the Kullback-Leibler divergence between the target rows T (rows of A * H_k: the bucket
 * attention mass of saap_bucket_attention_mass) and the model's distributions, averaged over
 * the batch.  The derivative of relu at 0 is 0.
 *   x [Hw,R,d] x_dtype; target [Hw,R,B] fp32 (>= 0); params: the model; grads: out, same shapes
 *   loss [Hw] fp32, out.  params and grads are host structs.
 * Sums run in a fixed order: the same inputs give the same bits.
 * Workspace: SAAP_OP_QUERY_MODEL_LOSS_GRADS.
 */
int32_t saap_query_model_loss_grads(const void* x, const float* target,
                                    const saap_mlp_f32* params /* host */,
                                    const saap_mlp_f32* grads /* host */, float* loss,
                                    int32_t Hw, int32_t R, int32_t d, int32_t hidden, int32_t B,
                                    int32_t x_dtype, void* ws, size_t ws_bytes, void* stream);

/*
 * query_model_bn_loss_grads -- the same loss and gradients for the model WITH batch
 * normalisation of the hidden layer (Section 6.1: two layers, batch normalisation, ReLU):
 *   a = W1 x + b1;  h = relu(gamma * (a - mean_r a) / sqrt(var_r a + eps) + beta);  z = W2 h + b2
 * with the statistics of the batch per weight set and hidden unit (variance with divisor R).
 * The paper gives no constants: eps and momentum are the caller's (1e-5 and 0.1 are usual).
 *   bn (host struct of device pointers): gamma, beta [Hw,hidden] fp32; grad_gamma, grad_beta out;
 *   running_mean, running_var [Hw,hidden] fp32 or both NULL: updated in place as
 *   run = (1 - momentum) run + momentum * batch, the variance entering with divisor R - 1.
 * R >= 2.  Everything else as saap_query_model_loss_grads; same workspace.
 */
typedef struct {
  float* gamma;
  float* beta;
  float* grad_gamma;
  float* grad_beta;
  float* running_mean;
  float* running_var;
  float momentum;
  float eps;
} saap_batch_norm_f32;

int32_t saap_query_model_bn_loss_grads(const void* x, const float* target,
                                       const saap_mlp_f32* params /* host */,
                                       const saap_mlp_f32* grads /* host */,
                                       const saap_batch_norm_f32* bn /* host */, float* loss,
                                       int32_t Hw, int32_t R, int32_t d, int32_t hidden, int32_t B,
                                       int32_t x_dtype, void* ws, size_t ws_bytes, void* stream);

/*
 * fold_batch_norm -- the inference form of a model trained with saap_query_model_bn_loss_grads:
 * with fixed statistics the normalisation is an affine map, so
 *   s = gamma / sqrt(running_var + eps);  W1' = s * W1 (row-wise);  b1' = (b1 - running_mean) s + beta
 * and saap_classify_queries on (W1', b1', W2, b2) is the normalised model.
 *   W1 [Hw,hidden,d], b1, gamma, beta, running_mean, running_var [Hw,hidden] fp32 (device)
 *   W1_out [Hw,hidden,d] out_dtype (SAAP_F32 or SAAP_BF16, rounded to nearest even); b1_out fp32
 */
int32_t saap_fold_batch_norm(const float* W1, const float* b1, const float* gamma, const float* beta,
                             const float* running_mean, const float* running_var, float eps,
                             void* W1_out, float* b1_out, int32_t Hw, int32_t hidden, int32_t d,
                             int32_t out_dtype, void* stream);

/*
 * adam_update -- one step of Adam (the optimiser named in the paper's training details) on one
 * tensor of n fp32 elements, in place:
 *   m = beta1 m + (1 - beta1) g;  v = beta2 v + (1 - beta2) g^2
 *   p -= lr * (m / (1 - beta1^step)) / (sqrt(v / (1 - beta2^step)) + eps),   step >= 1
 * A training step of the query model is saap_query_model_loss_grads followed by this call on
 * W1, b1, W2 and b2.
 */
int32_t saap_adam_update(float* param, const float* grad, float* m, float* v, size_t n,
                         int32_t step, float lr, float beta1, float beta2, float eps, void* stream);

/*
 * quantize_kv -- 8-bit copy of a bucket-sorted K/V cache.  Section 2 (related work) calls
 * compression of the cached vectors complementary to the partition and fixes no format; here:
 * OCP FP8 E4M3 (1 sign, 4 exponent bits with bias 7, 3 mantissa bits, subnormals, no
 * infinities, largest finite value 448) with one power-of-two scale per (sequence, KV head)
 * and tensor.  It halves the bytes the decode attention reads per key (256 instead of 512).
 *   scale = 2^e, e the smallest integer with max|x| <= 448 * 2^e (1 for an all-zero unit);
 *   code  = x / scale rounded to the nearest E4M3 value, ties to even.
 *   Ksorted, Vsorted [S,Hkv,Ncap,d] dtype (device, finite values; free slots count as data)
 *   K8, V8 [S,Hkv,Ncap,d] uint8, out;  kscale, vscale [S,Hkv] fp32, out
 * off, len, idx of the index stay valid for the 8-bit copy.
 * Workspace: SAAP_WS_HEADER_BYTES suffice.
 */
int32_t saap_quantize_kv(const void* Ksorted, const void* Vsorted, uint8_t* K8, uint8_t* V8,
                         float* kscale, float* vscale,
                         int32_t S, int32_t Hkv, int32_t Ncap, int32_t d, int32_t dtype,
                         void* ws, size_t ws_bytes, void* stream);

/*
 * sparse_decode_attention_fp8 / windowed_decode_attention_fp8 / dense_decode_attention_fp8 --
 * saap_sparse_decode_attention, saap_windowed_decode_attention and saap_dense_decode_attention on a cache written by saap_quantize_kv: the attention is that of
 * the decoded values kscale * value(K8), vscale * value(V8) (exact softmax over the visited
 * keys, fp32 accumulation), K and V are read as one byte per feature.
 *   q [S,Hq,d] bf16; K8, V8 [S,Hkv,Ncap,d] uint8; kscale, vscale [S,Hkv] fp32
 *   the remaining arguments as in the 16-bit calls (mode: SAAP_GROUP_SUM lists [S,Hkv,nprobe]
 *   or SAAP_INDEPENDENT lists [S,Hq,nprobe])
 *   dense: off != NULL as in saap_dense_decode_attention (a bucket-sorted cache), B buckets
 * Workspace: as SAAP_OP_SPARSE_DECODE_ATTENTION / SAAP_OP_DENSE_DECODE_ATTENTION.
 */
int32_t saap_sparse_decode_attention_fp8(const void* q, const uint8_t* K8, const uint8_t* V8,
                                         const float* kscale, const float* vscale,
                                         const int32_t* off, const int32_t* len,
                                         const int32_t* selected, int32_t nprobe, int32_t mode,
                                         float scale, void* out, int32_t out_dtype, float* lse,
                                         int32_t S, int32_t Hq, int32_t Hkv, int32_t Ncap, int32_t B,
                                         int32_t d,
                                         void* ws, size_t ws_bytes, void* stream);

/* saap_windowed_decode_attention on an 8-bit cache (saap_quantize_kv applied to the cache of
 * saap_build_windowed_index): the resident run is visited besides the selected buckets. */
int32_t saap_windowed_decode_attention_fp8(const void* q, const uint8_t* K8, const uint8_t* V8,
                                           const float* kscale, const float* vscale,
                                           const int32_t* off, const int32_t* len,
                                           const int32_t* selected, int32_t nprobe, int32_t mode,
                                           int32_t resident_run,
                                           float scale, void* out, int32_t out_dtype, float* lse,
                                           int32_t S, int32_t Hq, int32_t Hkv, int32_t Ncap, int32_t runs,
                                           int32_t d,
                                           void* ws, size_t ws_bytes, void* stream);

int32_t saap_dense_decode_attention_fp8(const void* q, const uint8_t* K8, const uint8_t* V8,
                                        const float* kscale, const float* vscale,
                                        const int32_t* off, const int32_t* len, int32_t B,
                                        float scale, void* out, int32_t out_dtype, float* lse,
                                        int32_t S, int32_t Hq, int32_t Hkv, int32_t N, int32_t d,
                                        void* ws, size_t ws_bytes, void* stream);

/*
 * ---- visit plans: routing hands the attention its work list ready-made ----
 * Section 5 ("On GPU") observes that with one block per visited bucket the largest bucket sets the
 * run time, and Appendix F (Algorithm 2) merges one partial result per block.  Here the selection
 * step writes, per list, a VISIT PLAN: the runs of the sorted cache to attend, as first rows and an
 * exclusive prefix of their lengths, and their total.  saap_planned_decode_attention concatenates
 * the key ranges of ALL lists and deals that global range to the workgroups in equal shares, so
 * that neither a large bucket nor a large list makes one workgroup finish late; a list is merged
 * (Algorithm 2) from as many partial results as workgroups held a piece of it.
 *
 * Plan layout, int32, per list (units = S*Hkv lists for SAAP_GROUP_SUM, S*Hq for SAAP_INDEPENDENT),
 * stride = 2*nruns + 2 rounded up to a multiple of 4:
 *   [0] total keys | [1 .. nruns+1] pre[0..nruns] (pre[0] = 0, pre[j+1] = pre[j] + len of run j) |
 *   [nruns+2 .. 2*nruns+1] first row of run j in the (sequence, KV head)'s sorted cache
 * nruns = nprobe (+ 1 if a resident run is always visited; it comes last).
 *
 * saap_visit_plan_bytes: size of the plan buffer (host arithmetic; 0 for invalid arguments).
 */
size_t saap_visit_plan_bytes(int32_t S, int32_t Hq, int32_t Hkv, int32_t nruns, int32_t mode);

/*
 * build_visit_plan -- the plan of given lists (any caller-made `selected`, as
 * saap_sparse_decode_attention takes it), one small launch.
 *   selected [S,Hkv,nprobe] or [S,Hq,nprobe] int32 (ids outside [0,runs) are clamped);
 *   off [S,Hkv,runs+1], len [S,Hkv,runs]; resident_run: a run visited by every list, or -1
 *   plan: out, saap_visit_plan_bytes(S, Hq, Hkv, nprobe + (resident_run >= 0), mode) bytes
 */
int32_t saap_build_visit_plan(const int32_t* selected, const int32_t* off, const int32_t* len,
                              int32_t nprobe, int32_t mode, int32_t resident_run, int32_t* plan,
                              int32_t S, int32_t Hq, int32_t Hkv, int32_t runs, void* stream);

/*
 * select_buckets_planned -- saap_select_buckets (input_kind SAAP_PROBS) or
 * saap_select_buckets_from_logits (SAAP_LOGITS) that also writes the visit plan of its lists in the
 * same launch: the lengths and first rows of the selected buckets are read while the scores are.
 *   off [S,Hkv,runs+1], len [S,Hkv,runs] with runs = B, or B + 1 when resident_run = B (the index of
 *   saap_build_windowed_index); selected, probs, the order of the list and the limits as in those calls;
 *   plan: out, nruns = nprobe + (resident_run >= 0).
 */
int32_t saap_select_buckets_planned(const float* scores, int32_t input_kind, float* probs,
                                    const int32_t* off, const int32_t* len, int32_t resident_run,
                                    int32_t* selected, int32_t* plan,
                                    int32_t S, int32_t Hq, int32_t Hkv, int32_t B, int32_t nprobe,
                                    int32_t mode, void* ws, size_t ws_bytes, void* stream);

/*
 * planned_decode_attention -- saap_sparse_decode_attention / saap_windowed_decode_attention driven by
 * a visit plan (same result: exact softmax attention over the listed runs, Section 4 "Beyond top-k",
 * Algorithms 1 and 2 of Appendix F; a list without keys gives out = 0, lse = -inf).
 *   q [S,Hq,d] dtype; Ksorted, Vsorted [S,Hkv,Ncap,d] dtype; plan as above with nruns runs per list
 *   mode SAAP_GROUP_SUM: a list serves the G heads of its KV head; SAAP_INDEPENDENT: one list per
 *   query head, every head reads its list on its own.
 * Limits: S*lists <= 4096, nruns <= 8191, S*Hkv*Ncap < 2^31; otherwise SAAP_UNSUPPORTED.
 * Workspace: SAAP_OP_PLANNED_DECODE_ATTENTION.  The _fp8 form reads a cache written by saap_quantize_kv.
 */
int32_t saap_planned_decode_attention(const void* q, const void* Ksorted, const void* Vsorted,
                                      const int32_t* plan, int32_t nruns, int32_t mode, float scale,
                                      void* out, int32_t out_dtype, float* lse,
                                      int32_t S, int32_t Hq, int32_t Hkv, int32_t Ncap, int32_t d, int32_t dtype,
                                      void* ws, size_t ws_bytes, void* stream);

int32_t saap_planned_decode_attention_fp8(const void* q, const uint8_t* K8, const uint8_t* V8,
                                          const float* kscale, const float* vscale,
                                          const int32_t* plan, int32_t nruns, int32_t mode, float scale,
                                          void* out, int32_t out_dtype, float* lse,
                                          int32_t S, int32_t Hq, int32_t Hkv, int32_t Ncap, int32_t d,
                                          void* ws, size_t ws_bytes, void* stream);

/*
 * prefill_sparse_attention -- sparse attention for a block of prompt tokens.  The paper's Conclusion
 * names prefill-time sparse attention as the next step and defines nothing; this call carries the
 * decode-time rule (Section 3 "Per-head attention span": attention sink and recent keys are always
 * attended; Section 4 "Beyond top-k": every key of the listed buckets; Section 5 "Batched queries":
 * one list for the G heads of a group) over to every token of the block:
 *   the query of token t of sequence s stands at position p = pos0[s] + t and attends, of the
 *   L = p + 1 keys at positions n <= p (causal, its own key included), those with
 *       n < n_sink,  or  n >= L - n_recent,  or  bucket(n) in selected[s,h,t,:].
 *   q [S,Tq,Hq,d] dtype (after RoPE), token-major as activations are
 *   K, V [S,Hkv,Nt,d] dtype: the prompt's keys and values in position order (pos0 + Tq <= Nt)
 *   Ksorted, Vsorted [S,Hkv,Ncap,d], off, len, idx: the bucket index over those Nt keys (or over
 *     more of the prompt: members at positions > p are not attended), as saap_build_bucket_index wrote it
 *   selected [S,Hkv,Tq,nprobe] int32: one list per token and KV head (distinct ids inside [0,B))
 *   pos0 [S] int32, device;  out [S,Tq,Hq,d] of out_dtype;  lse [S,Tq,Hq] fp32 or NULL
 * Sink and recent keys are read from K, V; of a listed bucket only the members between them are
 * read from the sorted cache (they form one stretch of the bucket's rows, the members being
 * stored in ascending position).  Every (token, KV head) pair gets a visit plan and the keys of all
 * pairs are dealt to the workgroups in equal shares, as saap_planned_decode_attention does: the
 * tokens of a block see very different numbers of keys.
 * Limits: S*Tq*Hkv <= 4096 per call (longer blocks are split by the caller); the limits of
 * saap_planned_decode_attention with nruns = nprobe + 2.
 * Workspace: SAAP_OP_PREFILL_SPARSE_ATTENTION (S, Hq, Hkv, N = Tq, nprobe).
 */
int32_t saap_prefill_sparse_attention(const void* q, const void* K, const void* V,
                                      const void* Ksorted, const void* Vsorted,
                                      const int32_t* off, const int32_t* len, const int32_t* idx,
                                      const int32_t* selected, const int32_t* pos0,
                                      int32_t nprobe, int32_t n_sink, int32_t n_recent, float scale,
                                      void* out, int32_t out_dtype, float* lse,
                                      int32_t S, int32_t Hq, int32_t Hkv, int32_t Tq, int32_t Nt, int32_t Ncap,
                                      int32_t B, int32_t d, int32_t dtype,
                                      void* ws, size_t ws_bytes, void* stream);

/*
 * append_keys_fp8 / window_push_fp8 -- saap_append_keys and saap_window_push on an 8-bit cache:
 * keys generated after prefill (Section 3: the key of each new token is assigned to a bucket
 * like the prefill keys) join a cache whose scales saap_quantize_kv has fixed.
 *   x_new, k_new, v_new [S,Hkv,d] bf16; centroids [Hkv,B,d] bf16, bias [Hkv,B] or NULL
 *   K8, V8 [S,Hkv,Ncap,d] uint8 and kscale, vscale [S,Hkv] fp32 as written by saap_quantize_kv
 *   every other argument, the bucket choice, the slot taken, the overflow behaviour and the
 *   workspace as in the 16-bit call of the same name
 * The stored row is code(x / scale) of its (sequence, head), ties to even; a feature beyond
 * 448 * scale takes the largest finite code of its sign (the scales stay as they are: a
 * caller that expects growing magnitudes quantises again from a 16-bit copy).  A key that a
 * push displaces moves inside the cache as bytes.
 */
int32_t saap_append_keys_fp8(const void* x_new, const void* k_new, const void* v_new,
                             const int32_t* pos_new, const void* centroids, const float* bias,
                             const int32_t* off, int32_t* len, int32_t* idx,
                             uint8_t* K8, uint8_t* V8, const float* kscale, const float* vscale,
                             int32_t* new_bucket_ids, int32_t* overflow_flag,
                             int32_t S, int32_t Hkv, int32_t Ncap, int32_t B, int32_t d,
                             void* ws, size_t ws_bytes, void* stream);

int32_t saap_window_push_fp8(const void* x_new, const void* k_new, const void* v_new,
                             const int32_t* pos_new, const void* centroids, const float* bias,
                             const int32_t* off, int32_t* len, int32_t* idx,
                             uint8_t* K8, uint8_t* V8, const float* kscale, const float* vscale,
                             int32_t* resident_ids, int32_t* new_bucket_ids, int32_t* overflow_flag,
                             int32_t S, int32_t Hkv, int32_t Ncap, int32_t B, int32_t d,
                             int32_t n_sink, int32_t n_recent,
                             void* ws, size_t ws_bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* SAAP_H */
