// Decode attention kernels: sparse attention over the visited buckets of a bucket-sorted
// KV cache, and dense attention over all keys (Section 4 "Beyond top-k", Section 5 "On GPU",
// Appendix F Algorithms 1 and 2 of arXiv 2502.08246).
//
// Design for gfx950 (not the paper's one-block-per-bucket scheme):
//   * A "unit" is one (sequence, KV head) with its G query heads.  The visited buckets of
//     a unit are contiguous runs of the sorted cache; concatenated they form a virtual key
//     range [0,T), cut into chunks of 128 keys that are dealt round-robin to the unit's P
//     workgroups, so the load is balanced whatever the bucket sizes are and neighbouring
//     workgroups stream neighbouring memory.  One more run can be visited always (the
//     attention sink + recent keys of Section 3), and with independent routing the union of
//     the heads' lists is visited once with a head mask per run.
//   * Inside a wavefront, 16 lanes read one 256-byte bf16 row with one 16-byte load each
//     (four rows per wave instruction, whole cache lines).  Each 16-lane group is a "key
//     processor" with its own running maximum, sum and output accumulator for all G heads
//     (Algorithm 1), so K and V are read once for the whole group of heads.
//   * Dot products are reduced over the 16 lanes with DPP lane exchanges; the four key
//     processors of a wave, the waves of a workgroup (through LDS) and the P workgroups of a
//     unit (through the workspace) are combined with the log-sum-exp merge of Algorithm 2.
//     The last workgroup of a unit to arrive (atomic counter) performs the final merge, so
//     partial attention and merge are one launch.
//   * On bf16 and 8-bit caches the value product P V runs on the matrix cores, the keys a
//     lane holds being the sum index of v_mfma_f32_16x16x16_bf16; the running maximum is then
//     one per head and wave.  On an 8-bit cache with four heads per KV head the scores run
//     there as well.
#include "select_body.h"

#include <mutex>

namespace saap {
namespace {

constexpr int kMaxP = 128;         // workgroups per unit (workspace is sized for this)

struct AttnParams {
  const void* q;          // [S,Hq,d]
  const void* K;          // [kv units, rows, d]
  const void* V;
  const int32_t* off;     // [kv units, B+1] or null
  const int32_t* len;     // [kv units, B]   or null
  const int32_t* selected;  // [units, nseg] or null (identity list)
  void* out;              // [S,Hq,d]
  float* lse;             // [S,Hq] or null
  float* part_o;          // [units, P, G, d]
  float* part_ml;         // [units, P, G, 2]
  unsigned long long* counters;   // [units * cstride] arrivals, eight 8-bit fields (one per XCD); zero on entry and on exit
  int cstride;            // 8-byte words between the counters of two units (16: a cache line each, so that the arrivals
                          // of different units do not queue at one line)
  long long rows;         // rows per kv unit
  int nseg;               // runs visited per unit (selected buckets + the always-visited run); list mode only
  int nsel;               // entries per unit in `selected` (the first nsel runs of the list)
  int resident;           // run visited after the selected ones (list entry nsel), or -1
  int max_chunks;         // upper bound on the chunks one workgroup processes (sizes the LDS tables)
  int B;
  int n_units;
  int P;
  int Hq, Hkv;
  int independent;        // unit = (sequence, query head) instead of (sequence, KV head)
  int masked_lists;       // MASKED kernels: lists per unit in `selected` (one per head), nsel entries each
  int use_table;          // list mode: build the per-chunk run table (pays off from a few chunks per workgroup)
  int stage;              // list mode: copy the unit's len/off arrays to LDS (needs nseg <= 2*NT, B <= 8*NT)
  int out_bf16;
  int n_dense;            // keys per unit in dense mode
  float scale_log2;       // scale * log2(e)
  const float* kscale;    // 8-bit cache: [kv units] scale of the K codes, else null
  const float* vscale;    // 8-bit cache: [kv units] scale of the V codes, else null
  // selection in the same launch (kernels with SEL != 0): the classifier's logits; `selected` is then an output
  const float* logits;    // [S,Hq,B]
  int32_t* selected_out;  // [units, nsel], written by the first workgroup of every unit
  int sel_B;              // buckets the logits cover (p.B counts the runs of the index: one more with a resident run)
  int sel_n_sort, sel_cap;       // geometry of the selection (select_geometry)
  unsigned sel_plan_off;  // byte offset of its staging area in LDS
  unsigned sel_lds;       // bytes of LDS the selection uses; the run tables of the attention follow
};
constexpr int kDtypeFp8 = 2;   // internal dtype code of an 8-bit cache (queries are bf16)

// Partial results cross workgroups inside one launch.  The writer stores them write-through to
// the device-coherent level and counts its arrival once the stores are acknowledged; the last
// workgroup to arrive invalidates its non-coherent cache lines once (acquire fence) and then
// reads the partials with ordinary loads.  A release fence per writer is avoided on purpose: it
// writes back the whole L2 and costs more than the attention itself when hundreds of
// workgroups do it.
__device__ __forceinline__ void coherent_store(float* p, float v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// Wait until every outstanding store of this wave has been acknowledged.
__device__ __forceinline__ void wait_stores() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// Merge `n` partial results (m_i, l_i, o_i[e]) for one (head, feature) pair:
// M = max m_i; o = sum 2^(m_i-M) o_i; l = sum 2^(m_i-M) l_i   (Algorithm 2, symmetric form).
template <typename FM, typename FL, typename FO>
__device__ __forceinline__ void lse_merge(int n, FM get_m, FL get_l, FO get_o, float& M, float& l, float& o) {
  M = kNegBig;
#pragma unroll
  for (int i = 0; i < n; ++i) M = fmaxf(M, get_m(i));
  l = 0.f;
  o = 0.f;
#pragma unroll
  for (int i = 0; i < n; ++i) {
    float w = fast_exp2(get_m(i) - M);
    l = fmaf(w, get_l(i), l);
    o = fmaf(w, get_o(i), o);
  }
}

__device__ __forceinline__ void store_out(const AttnParams& p, int qrow, int e, float M, float l, float o, float vs) {
  float r = l > 0.f ? vs * (o / l) : 0.f;
  if (p.out_bf16) reinterpret_cast<bf16_t*>(p.out)[(size_t)qrow * kD + e] = (bf16_t)f32_to_bf16_bits(r);
  else reinterpret_cast<float*>(p.out)[(size_t)qrow * kD + e] = r;
  if (e == 0 && p.lse) p.lse[qrow] = l > 0.f ? (M + __log2f(l)) * kLn2 : -INFINITY;
}

// bf16 and 8-bit caches use the matrix cores (see consume_batch).
// Values, O += P V: for every group size.  The sum runs over the keys, and the four keys a lane holds of a
// row piece are the four k-values a lane contributes to v_mfma_f32_16x16x16_bf16, so the loads keep their layout
// (16 lanes per row, whole cache lines).
// Scores, S = K Q^T: for 8-bit caches and groups of four heads only.  The sum runs over the features, so the operand wants lane (m, kg) to
// hold a piece of row m: 16 different rows in 16 neighbouring lanes, a load that touches 16 cache lines per 16
// lanes.  On 8-bit rows this still pays (v_mfma_f32_16x16x32_fp8_fp8 takes the codes as they are, where the
// vector ALUs convert every code before they multiply it with four heads: 29 against 32 us at 8 x 128k); on
// bf16 rows it does not (48 against 43 us there), v_dot2_f32_bf16 on whole cache lines is faster.
template <typename T, int G>
constexpr bool kMatrixScores = sizeof(T) == 1 && G == 4;
template <typename T, int G>
constexpr bool kMatrixValues = sizeof(T) <= 2;

// One batch of a key processor: KB rows of K and V, and which of them are real keys.
// MM (matrix-core scores): the wave's 16 keys form the A operand instead, lane (m, kg) = (lane % 16, lane / 16)
// holding bytes [kg*16, kg*16+16) of both 64-byte halves of the row of key m = 4*processor + slot.
template <typename T, int KB, bool MM>
struct BatchKeys {
  Vec8<T> k[KB];
};
template <typename T, int KB>
struct BatchKeys<T, KB, true> {
  uint4 ka[2];                // the two 64-byte halves of a row of codes
};
template <typename T, int KB, bool MM = false>
struct Batch : BatchKeys<T, KB, MM> {
  Vec8<T> v[KB];
  unsigned valid;   // bit i: slot i holds a key of the range
  unsigned heads;   // MASKED kernels: bits 8i .. 8i+7 = heads that attend the key in slot i
};

// The query rows of a unit as the dot products want them.  Vector path: 8 features of each head per lane.
template <typename T, int G, bool MM = kMatrixScores<T, G>>
struct Queries {
  typedef typename DotType<T>::type TQ;
  Vec8<TQ> v[G];
  // `scale_log2` is the factor that turns the lane's dot products into base-2 logits; the matrix path folds the
  // scaling of its operand into it
  __device__ __forceinline__ void load(const void* q, int qrow0, int sub, int /*grp*/, float& /*scale_log2*/) {
#pragma unroll
    for (int g = 0; g < G; ++g) v[g].load(reinterpret_cast<const TQ*>(q) + (size_t)(qrow0 + g) * kD + sub * 8);
  }
};
// Matrix path: the B operand.  Lane (n, kg) holds, for head n % 4, the features the A operand's lane (m, kg)
// holds of its key: [kg*16, kg*16+16) of both halves of the row, as E4M3 codes.  A bf16 query has 8 significant
// bits and a code 4, so the row is scaled by a power of two (largest element into [128, 256)) and split into
// two rows of codes, hi = the nearest code and lo = the rest, which is a code exactly unless it falls below the
// smallest one (2^-9 against a largest element >= 128: an error of 2^-17 of it at most).
template <>
struct Queries<fp8_t, 4, true> {
  long hi[4], lo[4];          // [half * 2 + piece]: 8 codes each
  __device__ __forceinline__ void load(const void* q, int qrow0, int sub, int grp, float& scale_log2) {
    typedef float f32x2_t __attribute__((ext_vector_type(2)));
    const bf16_t* row = reinterpret_cast<const bf16_t*>(q) + (size_t)(qrow0 + (sub & 3)) * kD + grp * 16;
    uint4 raw[4];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      raw[2 * h] = *reinterpret_cast<const uint4*>(row + h * 64);
      raw[2 * h + 1] = *reinterpret_cast<const uint4*>(row + h * 64 + 8);
    }
    float x[32];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      Vec8<bf16_t> w;
      w.r = raw[i];
      w.to_float(x + 8 * i);
    }
    float big = 0.f;
#pragma unroll
    for (int i = 0; i < 32; ++i) big = fmaxf(big, fabsf(x[i]));
    big = max_rows(big);                                  // the head's largest element, in all its lanes
    const unsigned eb = (__float_as_uint(big) >> 23) & 0xffu;
    const bool scaled = eb >= 8u && eb < 255u;
    const float up = scaled ? __uint_as_float((261u - eb) << 23) : 1.f;     // 2^(7 - floor(log2 big))
    const float down = scaled ? __uint_as_float((eb - 7u) << 23) : 1.f;     // its inverse
    scale_log2 *= down;
#pragma unroll
    for (int o = 0; o < 4; ++o) {                        // operand o: 8 codes from x[8o .. 8o+8)
      int h32[2] = {0, 0}, l32[2] = {0, 0};
#pragma unroll
      for (int wd = 0; wd < 2; ++wd) {                   // word wd: codes of x[8o + 4wd .. 8o + 4wd + 4)
        const float a = x[8 * o + 4 * wd] * up, b = x[8 * o + 4 * wd + 1] * up;
        const float c = x[8 * o + 4 * wd + 2] * up, d = x[8 * o + 4 * wd + 3] * up;
        h32[wd] = __builtin_amdgcn_cvt_pk_fp8_f32(a, b, h32[wd], false);
        h32[wd] = __builtin_amdgcn_cvt_pk_fp8_f32(c, d, h32[wd], true);
        const f32x2_t b0 = __builtin_amdgcn_cvt_pk_f32_fp8(h32[wd], false), b1 = __builtin_amdgcn_cvt_pk_f32_fp8(h32[wd], true);
        l32[wd] = __builtin_amdgcn_cvt_pk_fp8_f32(a - b0[0], b - b0[1], l32[wd], false);
        l32[wd] = __builtin_amdgcn_cvt_pk_fp8_f32(c - b1[0], d - b1[1], l32[wd], true);
      }
      hi[o] = (long)(((unsigned long long)(unsigned)h32[1] << 32) | (unsigned)h32[0]);
      lo[o] = (long)(((unsigned long long)(unsigned)l32[1] << 32) | (unsigned)l32[0]);
    }
  }
};

// One stage of the reduction of N partial sums over a 16-lane group.  The lane keeps the half
// of the values selected by `bit` (its partner under the lane exchange CTRL keeps the other
// half) and adds the partner's contribution: v[0 .. N/2) afterwards.
template <int N, int CTRL>
__device__ __forceinline__ void scatter_stage(float* v, bool bit) {
#pragma unroll
  for (int j = 0; j < N / 2; ++j) {
    const float keep = bit ? v[N / 2 + j] : v[j];
    const float give = bit ? v[j] : v[N / 2 + j];
    v[j] = keep + dpp_mov<CTRL>(give);
  }
}
template <int N, int CTRL>
__device__ __forceinline__ void allreduce_stage(float* v) {
#pragma unroll
  for (int j = 0; j < N; ++j) v[j] += dpp_mov<CTRL>(v[j]);
}
// Sums each of C (4, 8 or 16) values over the 16 lanes of a group; lane s returns the total of
// value (s & (C-1)).  45 instructions for C = 16 against 64 for an all-reduce of every value.
template <int C>
__device__ __forceinline__ float reduce_scatter16(float* v, int sub) {
  if constexpr (C == 16) scatter_stage<16, kDppMirror>(v, sub & 8); else allreduce_stage<C, kDppMirror>(v);
  if constexpr (C >= 8) scatter_stage<(C >= 16 ? 8 : C), kDppHalfMirror>(v, sub & 4); else allreduce_stage<C, kDppHalfMirror>(v);
  scatter_stage<4, kDppXor2>(v, sub & 2);
  scatter_stage<2, kDppXor1>(v, sub & 1);
  return v[0];
}
// max / sum over the lanes s, s+ST, s+2ST, ... of a 16-lane group that hold the same head.
template <int ST, int END>
__device__ __forceinline__ float ror_max(float x) {
  if constexpr (ST < END) {
    x = fmaxf(x, dpp_mov<0x120 + ST>(x));
    return ror_max<ST * 2, END>(x);
  } else {
    return x;
  }
}
template <int ST, int END>
__device__ __forceinline__ float ror_sum(float x) {
  if constexpr (ST < END) {
    x += dpp_mov<0x120 + ST>(x);
    return ror_sum<ST * 2, END>(x);
  } else {
    return x;
  }
}
// value of lane L of the 16-lane group, in every lane of the group
template <int L>
__device__ __forceinline__ float group_bcast(float x) { return dpp_mov<0x150 + L>(x); }
// the same for an integer and a lane number i < N that the unrolled caller knows at compile time (a register move
// where a shuffle would go through the LDS crossbar)
template <int N>
__device__ __forceinline__ unsigned row_lane(int x, int i) {
  static_assert(N <= 4, "lanes 0..3 of the group");
  switch (i) {
    case 0: return dpp_u32<0x150>((unsigned)x);
    case 1: return dpp_u32<0x151>((unsigned)x);
    case 2: return dpp_u32<0x152>((unsigned)x);
    default: return dpp_u32<0x153>((unsigned)x);
  }
}

// The unnormalised outputs a lane accumulates: 8 features of each of the G heads.  Matrix path: one
// accumulator of the matrix instruction per feature, whose four registers are the four heads.
template <int G, bool MM>
struct Accum {
  float O[G][8];
  __device__ __forceinline__ void zero() {
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
      for (int e = 0; e < 8; ++e) O[g][e] = 0.f;
  }
  __device__ __forceinline__ void rows(float (&out)[G][8]) const {
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
      for (int e = 0; e < 8; ++e) out[g][e] = O[g][e];
  }
};
// Rows 0..3 of the product (heads 0..3) are the registers of the lanes of row 0; with eight heads, rows 4..7 are
// those of the lanes of row 1.
template <int G>
struct Accum<G, true> {
  f32x4_t c[8];
  __device__ __forceinline__ void zero() {
#pragma unroll
    for (int e = 0; e < 8; ++e) c[e] = f32x4_t{0.f, 0.f, 0.f, 0.f};
  }
  // out[g][e] in the lanes of row 0 (what the combination across waves reads)
  __device__ __forceinline__ void rows(float (&out)[G][8]) const {
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        if (g < 4) out[g][e] = c[e][g];
        else out[g][e] = __shfl_down(c[e][g - 4], 16);
      }
  }
};

// Scores of a wave batch on the matrix cores (8-bit cache, four heads): S^T = K Q^T, 16 keys x 128 features
// against 4 heads (each in four columns), the hi and the lo codes of the queries on an accumulator each.  The
// result's lane (n, row) holds the scores of head n % 4 for the four slots of processor `row`; lane n keeps slot
// n / 4, the (slot, head) combination it owns in the softmax below.
template <typename T>
__device__ __forceinline__ float matrix_scores(const Batch<T, 4, true>& bt, const Queries<T, 4, true>& qv, int sub) {
  f32x4_t acc_h = {0.f, 0.f, 0.f, 0.f}, acc_l = acc_h;
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const long a0 = (long)(((unsigned long long)bt.ka[h].y << 32) | bt.ka[h].x);
    const long a1 = (long)(((unsigned long long)bt.ka[h].w << 32) | bt.ka[h].z);
    acc_h = __builtin_amdgcn_mfma_f32_16x16x32_fp8_fp8(a0, qv.hi[2 * h], acc_h, 0, 0, 0);
    acc_l = __builtin_amdgcn_mfma_f32_16x16x32_fp8_fp8(a0, qv.lo[2 * h], acc_l, 0, 0, 0);
    acc_h = __builtin_amdgcn_mfma_f32_16x16x32_fp8_fp8(a1, qv.hi[2 * h + 1], acc_h, 0, 0, 0);
    acc_l = __builtin_amdgcn_mfma_f32_16x16x32_fp8_fp8(a1, qv.lo[2 * h + 1], acc_l, 0, 0, 0);
  }
  const f32x4_t acc = acc_h + acc_l;
  const int slot = sub >> 2;
  return slot == 0 ? acc[0] : slot == 1 ? acc[1] : slot == 2 ? acc[2] : acc[3];
}

// The B operands of the value product: for each of the lane's eight features e, that feature of the KB keys
// (slots) whose row pieces the lane holds, as bf16; with two slots the other two k-values are zero.
typedef __bf16 bf16x2v_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x4v_t __attribute__((ext_vector_type(4)));
template <int KB>
__device__ __forceinline__ void values_by_feature(const Vec8<bf16_t> (&v)[KB], bf16x4v_t (&vb)[8]) {
  // word w of a row piece holds features 2w and 2w+1: the low (high) halves of the slots' words are feature
  // 2w (2w+1) of the keys
#pragma unroll
  for (int w = 0; w < 4; ++w) {
    auto word = [&](int i) { return w == 0 ? v[i].r.x : w == 1 ? v[i].r.y : w == 2 ? v[i].r.z : v[i].r.w; };
    const unsigned s0 = word(0), s1 = word(1);
    uint2 even = make_uint2(__builtin_amdgcn_perm(s1, s0, 0x05040100u), 0u);
    uint2 odd = make_uint2(__builtin_amdgcn_perm(s1, s0, 0x07060302u), 0u);
    if constexpr (KB == 4) {
      const unsigned s2 = word(2), s3 = word(3);
      even.y = __builtin_amdgcn_perm(s3, s2, 0x05040100u);
      odd.y = __builtin_amdgcn_perm(s3, s2, 0x07060302u);
    }
    vb[2 * w] = __builtin_bit_cast(bf16x4v_t, even);
    vb[2 * w + 1] = __builtin_bit_cast(bf16x4v_t, odd);
  }
}
template <int KB>
__device__ __forceinline__ void values_by_feature(const Vec8<fp8_t> (&v)[KB], bf16x4v_t (&vb)[8]) {
#pragma unroll
  for (int w = 0; w < 2; ++w) {                          // word w of a row piece: the codes of features 4w .. 4w+3
    const unsigned s0 = w ? v[0].r.y : v[0].r.x, s1 = w ? v[1].r.y : v[1].r.x;
    unsigned s2 = 0u, s3 = 0u;                           // code 0 is the value 0
    if constexpr (KB == 4) {
      s2 = w ? v[2].r.y : v[2].r.x;
      s3 = w ? v[3].r.y : v[3].r.x;
    }
    // bytes of two slots interleaved, then pairs of those: (slot 0, 1, 2, 3) of one feature per word
    const unsigned t01l = __builtin_amdgcn_perm(s1, s0, 0x05010400u), t01h = __builtin_amdgcn_perm(s1, s0, 0x07030602u);
    const unsigned t23l = __builtin_amdgcn_perm(s3, s2, 0x05010400u), t23h = __builtin_amdgcn_perm(s3, s2, 0x07030602u);
    const unsigned f[4] = {__builtin_amdgcn_perm(t23l, t01l, 0x05040100u), __builtin_amdgcn_perm(t23l, t01l, 0x07060302u),
                           __builtin_amdgcn_perm(t23h, t01h, 0x05040100u), __builtin_amdgcn_perm(t23h, t01h, 0x07060302u)};
#pragma unroll
    for (int x = 0; x < 4; ++x) {                        // E4M3 -> bf16 is exact
      const bf16x2v_t b01 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8((int)f[x], 1.0f, false);
      const bf16x2v_t b23 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8((int)f[x], 1.0f, true);
      vb[4 * w + x] = bf16x4v_t{b01[0], b01[1], b23[0], b23[1]};
    }
  }
}

// O += P V of a wave batch on the matrix cores, two v_mfma_f32_16x16x16_bf16 per feature e of the lane's eight:
// the sum runs over the wave's keys, k = 4 * processor + slot (two slots with eight heads: k-values 2 and 3 of
// every processor are zero).
// A (weights): lane (m, row) holds head m's weights of the slots of processor `row`; they sit in lanes m, m+G,
// m+2G, ... of the row (`pw` is the weight of the lane's own (slot, head)) and come by row rotation; lanes from G
// on collect other combinations, rows of the product that nobody reads.  A weight goes in as two bf16 numbers,
// its upper 16 bits and the rest rounded (16 significant bits together), one product each.
// B: values_by_feature.  The result's rows 0..G-1 are the heads (Accum), summed over all four processors; what
// the other rows accumulate is never read.
template <typename T, int G>
__device__ __forceinline__ void matrix_value_update(const Vec8<T> (&v)[G == 8 ? 2 : 4], float pw, Accum<G, true>& acc_o) {
  constexpr int KB = G == 8 ? 2 : 4;
  typedef float f32x2_t __attribute__((ext_vector_type(2)));
  const unsigned p_hi = __float_as_uint(pw) & 0xffff0000u;
  const float p_rest = pw - __uint_as_float(p_hi);
  const f32x2_t rest2 = {p_rest, p_rest};
  const unsigned w0 = p_hi | (__builtin_bit_cast(unsigned, __builtin_convertvector(rest2, bf16x2v_t)) & 0xffffu);
  // slot j: lane i <- lane i + j*G (mod 16), a rotation by 16 - j*G
  const unsigned w1 = dpp_u32<0x120 + ((16 - G) & 15)>(w0);
  unsigned w2 = 0u, w3 = 0u;
  if constexpr (KB == 4) {
    w2 = dpp_u32<0x120 + ((16 - 2 * G) & 15)>(w0);
    w3 = dpp_u32<0x120 + ((16 - 3 * G) & 15)>(w0);
  }
  const uint2 a_hi2 = make_uint2(__builtin_amdgcn_perm(w1, w0, 0x07060302u), __builtin_amdgcn_perm(w3, w2, 0x07060302u));
  const uint2 a_lo2 = make_uint2(__builtin_amdgcn_perm(w1, w0, 0x05040100u), __builtin_amdgcn_perm(w3, w2, 0x05040100u));
  const bf16x4v_t a_hi = __builtin_bit_cast(bf16x4v_t, a_hi2), a_lo = __builtin_bit_cast(bf16x4v_t, a_lo2);
  bf16x4v_t vb[8];
  values_by_feature<KB>(v, vb);
  // the eight accumulators in turn, twice: no product waits for the one before it
#pragma unroll
  for (int e = 0; e < 8; ++e) acc_o.c[e] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(a_hi, vb[e], acc_o.c[e], 0, 0, 0);
#pragma unroll
  for (int e = 0; e < 8; ++e) acc_o.c[e] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(a_lo, vb[e], acc_o.c[e], 0, 0, 0);
}

// One batch of Algorithm 1 for a key processor: scores of the batch's KB keys against the G heads, running
// maximum / sum / output update.  `m` is the running maximum of the head the lane owns, `l` the sum of the
// lane's own (key slot, head) weights, acc_o the output slices of all G heads.
template <typename T, int G, bool MASKED>
__device__ __forceinline__ void consume_batch(const Batch<T, (G == 8 ? 2 : 4), kMatrixScores<T, G>>& bt,
                                              const Queries<T, G>& qv, float scale_log2, int sub,
                                              float& m, float& l, Accum<G, kMatrixValues<T, G>>& acc_o) {
  constexpr int KB = G == 8 ? 2 : 4;
  constexpr int C = KB * G;
  typedef typename DotType<T>::type TQ;
  const int c_own = sub & (C - 1);              // the combination this lane owns after the reduction
  const int i_own = c_own / G;                  // ... its key slot
  float dot;
  if constexpr (kMatrixScores<T, G>) {
    dot = matrix_scores<T>(bt, qv, sub);
  } else {
    // partial dot products of the lane's 8 features, all (key slot, head) combinations ...
    float d[C];
#pragma unroll
    for (int i = 0; i < KB; ++i) {
      const Vec8<TQ> kw = dot_operand(bt.k[i]);
#pragma unroll
      for (int g = 0; g < G; ++g) d[i * G + g] = kw.dot(qv.v[g]);
    }
    // ... reduced over the 16 lanes so that each lane ends up with ONE complete score
    dot = reduce_scatter16<C>(d, sub);
  }
  bool live = (bt.valid >> i_own) & 1u;
  if constexpr (MASKED) live = live && ((bt.heads >> (8 * i_own + c_own % G)) & 1u);
  const float t = live ? dot * scale_log2 : -INFINITY;
  // Algorithm 1, one step per batch: the head's running maximum lives in the lanes that own it
  float bm = ror_max<G, C>(t);
  // matrix path: the value product sums over the 16 keys of the wave, so its four processors keep ONE running
  // maximum per head
  if constexpr (kMatrixValues<T, G>) bm = max_rows(bm);
  const float mn = fmaxf(m, bm);
  if (__builtin_amdgcn_ballot_w64(mn > m) != 0ull) {      // some maximum moved: rescale (wave-uniform branch)
    const float alpha = fast_exp2(m - mn);
    l *= alpha;
    if constexpr (kMatrixValues<T, G>) {
      // register i of an accumulator is head i in the lanes of row 0 (head 4 + i in those of row 1 with eight
      // heads); lane h of every row owns head h's factor
      f32x4_t ag = {group_bcast<0>(alpha), group_bcast<1>(alpha), group_bcast<2>(alpha), group_bcast<3>(alpha)};
      if constexpr (G == 8) {
        const f32x4_t ag1 = {group_bcast<4>(alpha), group_bcast<5>(alpha), group_bcast<6>(alpha), group_bcast<7>(alpha)};
        if ((threadIdx.x >> 4) & 1) ag = ag1;
      }
#pragma unroll
      for (int e = 0; e < 8; ++e) acc_o.c[e] *= ag;
    } else {
#pragma unroll
      for (int g = 0; g < G; ++g) {
        float ag;
        if constexpr (G == 1) ag = alpha; else ag = g == 0 ? group_bcast<0>(alpha) : g == 1 ? group_bcast<1>(alpha) : g == 2 ? group_bcast<2>(alpha) : g == 3 ? group_bcast<3>(alpha) : g == 4 ? group_bcast<4>(alpha) : g == 5 ? group_bcast<5>(alpha) : g == 6 ? group_bcast<6>(alpha) : group_bcast<7>(alpha);
#pragma unroll
        for (int e = 0; e < 8; ++e) acc_o.O[g][e] *= ag;
      }
    }
    m = mn;
  }
  const float pw = fast_exp2(t - m);          // weight of the lane's own (key slot, head)
  l += pw;
  if constexpr (kMatrixValues<T, G>) {
    matrix_value_update<T, G>(bt.v, pw, acc_o);
  } else {
    // every lane needs every weight of its group for the value update: broadcast from the owner
    float pb[C];
    pb[0] = group_bcast<0>(pw); pb[1] = group_bcast<1>(pw); pb[2] = group_bcast<2>(pw); pb[3] = group_bcast<3>(pw);
    if constexpr (C >= 8) { pb[4] = group_bcast<4>(pw); pb[5] = group_bcast<5>(pw); pb[6] = group_bcast<6>(pw); pb[7] = group_bcast<7>(pw); }
    if constexpr (C == 16) {
      pb[8] = group_bcast<8>(pw); pb[9] = group_bcast<9>(pw); pb[10] = group_bcast<10>(pw); pb[11] = group_bcast<11>(pw);
      pb[12] = group_bcast<12>(pw); pb[13] = group_bcast<13>(pw); pb[14] = group_bcast<14>(pw); pb[15] = group_bcast<15>(pw);
    }
#pragma unroll
    for (int i = 0; i < KB; ++i) {
      float vf[8];
      bt.v[i].to_float(vf);
#pragma unroll
      for (int g = 0; g < G; ++g)
#pragma unroll
        for (int e = 0; e < 8; ++e) acc_o.O[g][e] = fmaf(pb[i * G + g], vf[e], acc_o.O[g][e]);
    }
  }
}

// End of a key range: the head's sum of weights is added up over the key slots, then the four key
// processors of the wave are combined (Algorithm 2 on registers): common maximum per head, rescale, add
// up across the four 16-lane rows.
template <int G, bool MM = false>
__device__ __forceinline__ void wave_combine(float& m, float& l, const Accum<G, MM>& acc_o, float (&O)[G][8]) {
  constexpr int C = (G == 8 ? 2 : 4) * G;
  l = ror_sum<G, C>(l);
  acc_o.rows(O);
  if constexpr (MM) {
    // matrix path: one running maximum for the wave, and the outputs (row 0) already hold the sum over its processors
    l = sum_rows(l);
    return;
  }
  const float mw = max_rows(m);
  const float a = fast_exp2(m - mw);          // scale of this processor's sums for the lane's own head
  m = mw;
  l = sum_rows(l * a);
#pragma unroll
  for (int g = 0; g < G; ++g) {
    float ag;
    if constexpr (G == 1) ag = a; else ag = g == 0 ? group_bcast<0>(a) : g == 1 ? group_bcast<1>(a) : g == 2 ? group_bcast<2>(a) : g == 3 ? group_bcast<3>(a) : g == 4 ? group_bcast<4>(a) : g == 5 ? group_bcast<5>(a) : g == 6 ? group_bcast<6>(a) : group_bcast<7>(a);
#pragma unroll
    for (int e = 0; e < 8; ++e) O[g][e] = sum_rows(O[g][e] * ag);
  }
}

// The waves of a workgroup combine their results through LDS (`scratch`: nw * G * (d + 2) floats, free
// for use once every wave has passed the barrier at the top): Algorithm 2 over the nw partial results,
// one (head, feature) per thread; every thread derives the weights 2^(m_j - M) of its head itself (nw
// exponentials) rather than waiting for a shared table.  emit(g, e, M, L, O) receives the merged values.
template <int G, int NT, typename F>
__device__ __forceinline__ void workgroup_combine(float* scratch, float m, float l, const float (&O)[G][8], F emit) {
  constexpr int nw = NT / 64;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, sub = lane & 15, grp = lane >> 4;
  SAAP_TRACE_WAVE(10);                                    // (debug builds) the last wave to get here stamps last
  __syncthreads();
  SAAP_TRACE(11);
  float* w_o = scratch;                                   // [nw][G][d] unnormalised outputs
  float* w_m = w_o + nw * G * kD;                         // [nw][G] maxima
  float* w_l = w_m + nw * G;                              // [nw][G] sums of weights
  if (grp == 0) {
#pragma unroll
    for (int g = 0; g < G; ++g) {
      float4* dst = reinterpret_cast<float4*>(w_o + (wave * G + g) * kD + sub * 8);
      dst[0] = make_float4(O[g][0], O[g][1], O[g][2], O[g][3]);
      dst[1] = make_float4(O[g][4], O[g][5], O[g][6], O[g][7]);
    }
    if (sub < G) {            // lane `sub` owns head `sub` (key slot 0)
      w_m[wave * G + sub] = m;
      w_l[wave * G + sub] = l;
    }
  }
  __syncthreads();
  SAAP_TRACE(13);
  for (int x = tid; x < G * kD; x += NT) {
    const int g = x / kD, e = x % kD;
    // every LDS read goes out before the first use: read, wait and use per wave would be eight round trips
    float mj[nw], lj[nw], oj[nw];
#pragma unroll
    for (int j = 0; j < nw; ++j) {
      mj[j] = w_m[j * G + g];
      lj[j] = w_l[j * G + g];
      oj[j] = w_o[(j * G + g) * kD + e];
    }
    __builtin_amdgcn_sched_barrier(0);
    float M = kNegBig;
#pragma unroll
    for (int j = 0; j < nw; ++j) M = fmaxf(M, mj[j]);
    float L = 0.f, Ov = 0.f;
#pragma unroll
    for (int j = 0; j < nw; ++j) {
      const float w = fast_exp2(mj[j] - M);
      L = fmaf(w, lj[j], L);
      Ov = fmaf(w, oj[j], Ov);
    }
    emit(g, e, M, L, Ov);
  }
}

// Final merge of a unit by its last workgroup (Algorithm 2): P partial results, stored from slot
// `slot0` on, become out / lse of the unit's G heads.  One partial is kCols = G*d/4 float4 columns; the
// workgroup's threads form NT/kCols groups that take the partials round-robin, eight loads in flight
// each, while one wave per head turns the partial maxima into weights.  `scratch` holds
// P*G + 2G + 4 floats and NT float4.
// Loads of partial results that other XCDs may have written: with COHERENT they are agent-scope atomic
// loads (two 8-byte loads per float4), which look past this XCD's L2, where a line of the workspace may
// survive from an earlier launch.  Without it the caller has made its caches safe to read.
template <bool COHERENT>
__device__ __forceinline__ float2 merge_load2(const float2* p) {
  if constexpr (COHERENT) {
    const unsigned long long u = __hip_atomic_load(reinterpret_cast<const unsigned long long*>(p), __ATOMIC_RELAXED,
                                                   __HIP_MEMORY_SCOPE_AGENT);
    return make_float2(__uint_as_float((unsigned)u), __uint_as_float((unsigned)(u >> 32)));
  } else {
    return *p;
  }
}
typedef float f32x4_asm __attribute__((ext_vector_type(4)));
// Eight 16-byte loads at agent scope (sc1: past this XCD's L2), issued back to back; entries with on[k]
// false load the first address and are zeroed.  The loads are written in assembly because the compiler
// offers atomic loads of at most 8 bytes; the wait that follows them names every destination, so no use
// of the values can move before it.
template <bool COHERENT>
__device__ __forceinline__ void merge_load4x8(const float4* const (&ptr)[8], const bool (&on)[8], float4 (&v)[8]) {
  if constexpr (COHERENT) {
    f32x4_asm r[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) asm volatile("global_load_dwordx4 %0, %1, off sc1" : "=v"(r[k]) : "v"(ptr[k]) : "memory");
    asm volatile("s_waitcnt vmcnt(0)"
                 : "+v"(r[0]), "+v"(r[1]), "+v"(r[2]), "+v"(r[3]), "+v"(r[4]), "+v"(r[5]), "+v"(r[6]), "+v"(r[7])
                 :
                 : "memory");
#pragma unroll
    for (int k = 0; k < 8; ++k) v[k] = on[k] ? make_float4(r[k].x, r[k].y, r[k].z, r[k].w) : make_float4(0.f, 0.f, 0.f, 0.f);
  } else {
    // every load is issued, on a valid address, before any value is looked at: as loads under the `on` branches
    // they waited for one another (one memory round trip per partial result instead of one in all)
    float4 r[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      r[k] = *ptr[k];
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      v[k].x = on[k] ? r[k].x : 0.f;
      v[k].y = on[k] ? r[k].y : 0.f;
      v[k].z = on[k] ? r[k].z : 0.f;
      v[k].w = on[k] ? r[k].w : 0.f;
    }
  }
}

template <int G, int NT, bool COHERENT = false>
__device__ __forceinline__ void final_merge(const float* part_o, const float* part_ml, size_t slot0, int P, int qrow0,
                                            float vs, void* out, int out_bf16, float* lse, float* scratch) {
  constexpr int nw = NT / 64;
  constexpr int kCols = G * kD / 4;
  constexpr int kInFlight = 8;
  constexpr int n_groups = NT / kCols;                // >= 1: NT >= 256 >= kCols
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int colx = tid % kCols, pgrp = tid / kCols;
  const int g_col = colx / (kD / 4);
  const float4* po = reinterpret_cast<const float4*>(part_o) + slot0 * kCols + colx;
  const float2* pml = reinterpret_cast<const float2*>(part_ml) + slot0 * G;
  float* s_w = scratch;                                // [P*G] weights 2^(m_i - M)
  float* s_M = s_w + P * G;                            // [G]
  float* s_L = s_M + G;                                // [G]
  float4* s_acc = reinterpret_cast<float4*>(s_L + G + ((4 - (P * G + 2 * G) % 4) % 4));   // [n_groups][kCols]

  // every load of the first round goes out before anything waits: the (max, sum) pairs first,
  // they are needed first
  float2 ml[2];
  const int g_w = wave < G ? wave : 0;               // wave w weighs head w (and w+nw, ... below)
#pragma unroll
  for (int k = 0; k < 2; ++k) {
    const int pi = lane + 64 * k;
    ml[k] = pi < P ? merge_load2<COHERENT>(pml + (size_t)pi * G + g_w) : make_float2(kNegBig, 0.f);
  }
  float4 v[kInFlight];
  auto load_round = [&](int first) {
    const float4* ptr[kInFlight];
    bool on[kInFlight];
#pragma unroll
    for (int k = 0; k < kInFlight; ++k) {
      const int pi = first + k * n_groups;
      on[k] = pi < P;
      ptr[k] = po + (size_t)(on[k] ? pi : 0) * kCols;
    }
    merge_load4x8<COHERENT>(ptr, on, v);
  };
  if constexpr (!COHERENT) load_round(pgrp);     // in flight while the weights are made (the assembly loads wait at once)
  for (int g = wave; g < G; g += nw) {
    if (g != g_w) {
#pragma unroll
      for (int k = 0; k < 2; ++k) {
        const int pi = lane + 64 * k;
        ml[k] = pi < P ? merge_load2<COHERENT>(pml + (size_t)pi * G + g) : make_float2(kNegBig, 0.f);
      }
    }
    float mx = fmaxf(ml[0].x, ml[1].x);
    for (int pi = lane + 128; pi < P; pi += 64) mx = fmaxf(mx, merge_load2<COHERENT>(pml + (size_t)pi * G + g).x);   // more than 128 partials
    mx = wave_max(mx);
    float lsum = 0.f;
#pragma unroll
    for (int k = 0; k < 2; ++k) {
      const int pi = lane + 64 * k;
      const float w = fast_exp2(ml[k].x - mx);
      if (pi < P) s_w[pi * G + g] = w;
      lsum = fmaf(w, ml[k].y, lsum);
    }
    for (int pi = lane + 128; pi < P; pi += 64) {
      const float2 t = merge_load2<COHERENT>(pml + (size_t)pi * G + g);
      const float w = fast_exp2(t.x - mx);
      s_w[pi * G + g] = w;
      lsum = fmaf(w, t.y, lsum);
    }
    lsum = wave_sum(lsum);
    if (lane == 0) {
      s_M[g] = mx;
      s_L[g] = lsum;
    }
  }
  if constexpr (COHERENT) load_round(pgrp);
  __syncthreads();
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int p0 = pgrp;; p0 += n_groups * kInFlight) {
    // the weights of the round first, all reads in flight together (a partial past the end was loaded as zeros
    // and takes the last partial's weight)
    float wv[kInFlight];
#pragma unroll
    for (int k = 0; k < kInFlight; ++k) wv[k] = s_w[min(p0 + k * n_groups, P - 1) * G + g_col];
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int k = 0; k < kInFlight; ++k) {
      acc.x = fmaf(wv[k], v[k].x, acc.x);
      acc.y = fmaf(wv[k], v[k].y, acc.y);
      acc.z = fmaf(wv[k], v[k].z, acc.z);
      acc.w = fmaf(wv[k], v[k].w, acc.w);
    }
    const int nxt = p0 + n_groups * kInFlight;
    if (nxt - pgrp >= P) break;     // uniform over the workgroup: depends on P and n_groups only
    load_round(nxt);
  }
  if (pgrp < n_groups) s_acc[pgrp * kCols + colx] = acc;
  __syncthreads();
  if (tid < kCols) {
    float4 r = s_acc[tid];
    for (int gi = 1; gi < n_groups; ++gi) {
      const float4 a = s_acc[gi * kCols + tid];
      r.x += a.x; r.y += a.y; r.z += a.z; r.w += a.w;
    }
    const float L = s_L[g_col], M = s_M[g_col];
    const float inv = L > 0.f ? vs * (1.0f / L) : 0.f;   // vs: scale of an 8-bit cache's V codes, else 1
    r.x *= inv; r.y *= inv; r.z *= inv; r.w *= inv;
    const int qrow = qrow0 + g_col, e0 = (colx % (kD / 4)) * 4;
    if (out_bf16) {
      uint2 pk;
      pk.x = f32_to_bf16_bits(r.x) | (f32_to_bf16_bits(r.y) << 16);
      pk.y = f32_to_bf16_bits(r.z) | (f32_to_bf16_bits(r.w) << 16);
      *reinterpret_cast<uint2*>(reinterpret_cast<bf16_t*>(out) + (size_t)qrow * kD + e0) = pk;
    } else {
      *reinterpret_cast<float4*>(reinterpret_cast<float*>(out) + (size_t)qrow * kD + e0) = r;
    }
    if (e0 == 0 && lse) lse[qrow] = L > 0.f ? (M + __log2f(L)) * kLn2 : -INFINITY;
  }
}

// MASKED (with LIST): every head of the group brings its own list of runs (independent routing).
// The union of the lists is visited once; a key takes part only for the heads whose list holds
// its run (the others see a score of -inf for it).
// SEL != 0 (with LIST, 512 threads): the launch also selects.  Every workgroup of a unit runs the selection of
// the unit's list from the classifier's logits itself (SEL buckets per thread), all of them arriving at the same
// list, and goes on with it: one launch and one dependent memory round trip less per decode step than a
// selection kernel in front, and no hand-over between workgroups.
template <typename T, int G, bool LIST, int NT, bool MASKED = false, int SEL = 0>
__global__ void __launch_bounds__(NT) attn_kernel(AttnParams p) {
  extern __shared__ __align__(16) unsigned char smem[];
  __shared__ int s_wsum[16];
  __shared__ int s_last;

  constexpr int nw = NT / 64;
  constexpr int KB = G == 8 ? 2 : 4;            // keys a key processor has in flight per batch
  constexpr int C = KB * G;                     // (key, head) combinations per batch: 4, 8 or 16
  constexpr bool kPrefetch = sizeof(T) <= 2;    // fp32 rows are too wide to double-buffer
  constexpr bool kFp8 = sizeof(T) == 1;
  typedef typename DotType<T>::type TQ;         // queries of an 8-bit cache are bf16
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int sub = lane & 15, grp = lane >> 4;
  SAAP_TRACE(0);
  const int unit = blockIdx.x % p.n_units;
  const int wg = blockIdx.x / p.n_units;

  // unit -> kv unit and first query row
  int kvu, qrow0;
  if (p.independent) {
    const int s = unit / p.Hq, hq = unit % p.Hq;
    kvu = s * p.Hkv + hq / (p.Hq / p.Hkv);
    qrow0 = unit;
  } else {
    kvu = unit;
    qrow0 = unit * G;   // (s*Hkv + h) * G == s*Hq + h*G
  }
  const T* Kb = reinterpret_cast<const T*>(p.K) + (size_t)kvu * p.rows * kD + sub * 8;
  const T* Vb = reinterpret_cast<const T*>(p.V) + (size_t)kvu * p.rows * kD + sub * 8;

  // 8-bit cache: the codes' scales fold into the score scale and into the final division
  float scale_log2 = p.scale_log2, vs = 1.f;
  if constexpr (kFp8) {
    scale_log2 *= p.kscale[kvu];
    vs = p.vscale[kvu];
  }
  // the query rows of the G heads
  constexpr bool MM = kMatrixScores<T, G>, MV = kMatrixValues<T, G>;
  Queries<T, G> qv;
  qv.load(p.q, qrow0, sub, grp, scale_log2);
  const T* Kmm = reinterpret_cast<const T*>(p.K) + (size_t)kvu * p.rows * kD + grp * 16;   // matrix path: the lane's 16 bytes of a 64-byte piece

  constexpr int NG = nw * 4;            // key processors in the workgroup
  constexpr int chunk = NG * KB;        // keys the workgroup consumes per batch
  const int kp = wave * 4 + grp;

  // with the selection in the launch its LDS comes first and the tables form a visit plan row: total, pre, rowoff
  int* tables = reinterpret_cast<int*>(smem + (SEL != 0 ? p.sel_lds : 0u));
  int* pre = tables + (SEL != 0 ? 1 : 0);           // [nseg+1] exclusive prefix of run lengths
  int* rowoff = pre + (p.nseg + 1);                 // [nseg]   first row of each run
  int* seglo = rowoff + p.nseg;                     // [max_chunks] run holding the first key of my k-th chunk
  int* seghi = seglo + p.max_chunks;                // [max_chunks] run holding its last key
  int* segm = seghi + p.max_chunks;                 // MASKED: [nseg] heads that attend each run
  int T_total;
  int nseg = p.nseg;                                // MASKED: p.nseg is the capacity, the union may be shorter
  if constexpr (LIST && MASKED) {
    // Union of the G lists in ascending bucket order.  Every thread owns B/NT consecutive buckets:
    // their len/off loads go out first and are in flight while the head masks are collected.
    int* hm = segm + p.nseg;                        // [B] heads that selected each bucket
    const int32_t* lenu = p.len + (size_t)kvu * p.B;
    const int32_t* offu = p.off + (size_t)kvu * (p.B + 1);
    const int perb = (p.B + NT - 1) / NT;           // <= 16: B <= SAAP_MAX_BUCKETS + 1, NT >= 512 checked on the host
    const int bb0 = tid * perb;
    int lv[16], ov[16];
#pragma unroll
    for (int k = 0; k < 16; ++k) {
      const int b = min(bb0 + k, p.B - 1);
      lv[k] = lenu[b];
      ov[k] = offu[b];
    }
    const int n_entries = p.masked_lists * p.nsel;
    const int32_t* selu = p.selected + (size_t)unit * n_entries;
    int sv[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) sv[k] = n_entries > 0 ? selu[min(tid + k * NT, n_entries - 1)] : 0;
    for (int b = tid; b < p.B; b += NT) hm[b] = 0;
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const int j = tid + k * NT;
      if (j < n_entries) atomicOr(&hm[min(max(sv[k], 0), p.B - 1)], 1 << (j / p.nsel));
    }
    for (int j = tid + 4 * NT; j < n_entries; j += NT)
      atomicOr(&hm[min(max(selu[j], 0), p.B - 1)], 1 << (j / p.nsel));
    if (tid == 0 && p.resident >= 0) atomicOr(&hm[p.resident], (1 << G) - 1);
    __syncthreads();
    int cnt = 0, mine = 0;
#pragma unroll
    for (int k = 0; k < 16; ++k)
      if (k < perb && bb0 + k < p.B && hm[bb0 + k] != 0) {
        ++cnt;
        mine += lv[k];
      }
    const unsigned incl_c = wave_prefix_sum((unsigned)cnt), incl_k = wave_prefix_sum((unsigned)mine);
    __shared__ int s_csum[16];
    if (lane == 63) {
      s_csum[wave] = (int)incl_c;
      s_wsum[wave] = (int)incl_k;
    }
    __syncthreads();
    int j = (int)incl_c - cnt, run = (int)incl_k - mine, total_c = 0;
    for (int w = 0; w < nw; ++w) {
      if (w < wave) {
        j += s_csum[w];
        run += s_wsum[w];
      }
      total_c += s_csum[w];
    }
    nseg = total_c;
    if (tid == 0) pre[0] = 0;
#pragma unroll
    for (int k = 0; k < 16; ++k)
      if (k < perb && bb0 + k < p.B && hm[bb0 + k] != 0) {
        run += lv[k];
        pre[j + 1] = run;
        rowoff[j] = ov[k];
        segm[j] = hm[bb0 + k];
        ++j;
      }
    __syncthreads();
    T_total = pre[nseg];
  } else if constexpr (LIST && SEL != 0) {
    PlanOut po{};
    po.off = p.off;
    po.len = p.len;
    po.plan = tables;                               // the plan row goes to LDS (stride 0: this unit's row only)
    po.runs = p.B;
    po.resident = p.resident;                       // the always-visited run, if any, closes the plan
    po.ps = 0;
    po.lds_off = p.sel_plan_off;
    select_radix_body<SEL, true, false>(smem, unit, p.logits, nullptr, wg == 0 ? p.selected_out : nullptr, p.Hq,
                                        p.Hkv, p.sel_B, p.nsel, 0, p.sel_n_sort, p.sel_cap, po);
    __syncthreads();
    T_total = tables[0];
  } else if (LIST) {
    const int per = (nseg + NT - 1) / NT;
    const int j0 = tid * per, j1 = min(j0 + per, nseg);
    const int32_t* lenu = p.len + (size_t)kvu * p.B;
    const int32_t* offu = p.off + (size_t)kvu * (p.B + 1);
    const int32_t* sel = p.selected ? p.selected + (size_t)unit * p.nsel : nullptr;
    int mine = 0;
    if (p.stage) {
      // One memory round trip instead of two: the selected list and the unit's whole len/off
      // arrays are fetched together into LDS, the gather by bucket id then reads LDS.
      int* s_len = seghi + p.max_chunks;                // [B]
      int* s_off = s_len + p.B;                         // [B]
      int sv[2], lv[8], ov[8];
#pragma unroll
      for (int k = 0; k < 2; ++k) {
        const int j = tid + k * NT;
        sv[k] = j < p.nsel ? sel[j] : p.resident;      // entry nsel (if any) is the always-visited run
      }
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        const int b = tid + k * NT;
        if (b < p.B) {
          lv[k] = lenu[b];
          ov[k] = offu[b];
        }
      }
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        const int b = tid + k * NT;
        if (b < p.B) {
          s_len[b] = lv[k];
          s_off[b] = ov[k];
        }
      }
      int bsel[2];                                       // per <= 2 in this mode
      if (per == 1) {
        // thread j already holds entry j of the list
        bsel[0] = sv[0];
        __syncthreads();
      } else {
#pragma unroll
        for (int k = 0; k < 2; ++k) {
          const int j = tid + k * NT;
          if (j < nseg) pre[j + 1] = sv[k];             // bucket id for now
        }
        __syncthreads();
        for (int j = j0; j < j1; ++j) bsel[j - j0] = pre[j + 1];
        __syncthreads();
      }
      for (int j = j0; j < j1; ++j) {
        const int b = bsel[j - j0];
        const int ln = s_len[b];
        pre[j + 1] = ln;
        rowoff[j] = s_off[b];
        mine += ln;
      }
    } else {
      for (int j = j0; j < j1; ++j) {
        const int b = j < p.nsel ? (sel ? sel[j] : j) : p.resident;
        const int ln = lenu[b];
        pre[j + 1] = ln;            // temporarily the length; turned into a prefix below
        rowoff[j] = offu[b];
        mine += ln;
      }
    }
    const int incl = (int)wave_prefix_sum((unsigned)mine);
    if (lane == 63) s_wsum[wave] = incl;
    __syncthreads();
    int base = 0;
    for (int w = 0; w < wave; ++w) base += s_wsum[w];
    int run = base + incl - mine;
    for (int j = j0; j < j1; ++j) {
      const int ln = pre[j + 1];
      if (j == 0) pre[0] = 0;
      run += ln;
      pre[j + 1] = run;
    }
    if (nseg == 0 && tid == 0) pre[0] = 0;
    __syncthreads();
    T_total = pre[nseg];
  } else {
    T_total = p.n_dense;
  }
  if (LIST) {
    // runs that hold the first and the last key of each of this workgroup's chunks, so that the
    // per-key lookups in the loop search a handful of runs instead of all of them
    for (int k = tid; p.use_table; k += NT) {
      const long long first = ((long long)wg + (long long)k * p.P) * chunk;
      if (first >= T_total || k >= p.max_chunks) break;
      const int v0 = (int)first;
      const int v1 = (int)min((long long)T_total, first + chunk) - 1;
      int a0 = 0, b0 = nseg, a1 = 0, b1 = nseg;
      while (b0 - a0 > 1 || b1 - a1 > 1) {
        const int m0 = (a0 + b0) >> 1, m1 = (a1 + b1) >> 1;
        if (b0 - a0 > 1) { if (pre[m0] <= v0) a0 = m0; else b0 = m0; }
        if (b1 - a1 > 1) { if (pre[m1] <= v1) a1 = m1; else b1 = m1; }
      }
      seglo[k] = a0;
      seghi[k] = a1;
    }
    if (p.use_table) __syncthreads();
  }
  SAAP_TRACE(1);

  // per lane: running maximum of its head, sum of its own (key slot, head) weights, and the
  // output slices of all G heads
  float m = kNegBig, l = 0.f;
  Accum<G, MV> acc_o;
  acc_o.zero();

  // The virtual key range [0,T) is cut into chunks of NG*KB keys; chunk c belongs to
  // workgroup c % P, so neighbouring workgroups stream neighbouring memory at any moment.
  // Virtual key of (this processor, slot i) of the chunk at `base` is base + i*NG + kp.
  const long long stride = (long long)chunk * p.P;

  auto load_batch = [&](long long base, int k, Batch<T, KB, MM>& bt) {
    int row, hmask = 0;
    {
      long long vl = base + (sub & (KB - 1)) * NG + kp;   // lane `sub` resolves slot sub % KB
      int v = (int)(vl < T_total ? vl : T_total - 1);
      if (LIST) {
        const bool tab = p.use_table && k < p.max_chunks;
        int a = tab ? seglo[k] : 0, b = tab ? seghi[k] + 1 : nseg;
        while (b - a > 1) {
          const int mid = (a + b) >> 1;
          if (pre[mid] <= v) a = mid; else b = mid;
        }
        row = rowoff[a] + (v - pre[a]);
        // a list that breaks the contract (repeated or overlapping runs, a damaged index) must
        // not turn into a read outside the cache
        row = min(max(row, 0), (int)p.rows - 1);
        if constexpr (MASKED) hmask = segm[a];
      } else {
        row = v;
      }
    }
    bt.valid = 0u;
    bt.heads = 0u;
    if constexpr (MM) {
      // operand row m = lane % 16 is the key of (processor m / 4, slot m % 4), resolved by lane m % 4 of that processor
      const int rk = __shfl(row, (sub >> 2) * 16 + (sub & 3));
#pragma unroll
      for (int c = 0; c < 2; ++c) bt.ka[c] = stream_load16(Kmm + (size_t)rk * kD + c * 64);
    }
#pragma unroll
    for (int i = 0; i < KB; ++i) {
      const int r = (int)row_lane<KB>(row, i);      // the row resolved by lane i of this 16-lane group
      if constexpr (MASKED) bt.heads |= row_lane<KB>(hmask, i) << (8 * i);
      if (base + i * NG + kp < T_total) bt.valid |= 1u << i;
      if constexpr (!MM) bt.k[i].load_stream(Kb + (size_t)r * kD);
      bt.v[i].load_stream(Vb + (size_t)r * kD);
    }
  };

  auto consume = [&](const Batch<T, KB, MM>& bt) { consume_batch<T, G, MASKED>(bt, qv, scale_log2, sub, m, l, acc_o); };

  {
    long long base = (long long)wg * chunk;
    int k = 0;
    if (base < T_total) {
      Batch<T, KB, MM> cur;
      load_batch(base, k, cur);
      if constexpr (kPrefetch) {
        for (base += stride, ++k; base < T_total; base += stride, ++k) {
          Batch<T, KB, MM> nxt;
          load_batch(base, k, nxt);     // in flight while the current batch is consumed
          // keep it that way: without the fence the scheduler starts on the current batch (and its
          // wait for memory) before the next batch's loads have been issued
          __builtin_amdgcn_sched_barrier(0);
          consume(cur);
          cur = nxt;
        }
        consume(cur);
      } else {
        consume(cur);
        for (base += stride, ++k; base < T_total; base += stride, ++k) {
          load_batch(base, k, cur);
          consume(cur);
        }
      }
    }
  }

  SAAP_TRACE(3);
  float O[G][8];
  wave_combine<G, MV>(m, l, acc_o, O);

  // waves -> LDS (the index arrays are dead once every wave has passed the barrier inside)
  SAAP_TRACE(9);
  workgroup_combine<G, NT>(reinterpret_cast<float*>(smem), m, l, O, [&](int g, int e, float M, float L, float Ov) {
    if (p.P == 1) {
      store_out(p, qrow0 + g, e, M, L, Ov, vs);
    } else {
      const size_t slot = ((size_t)unit * p.P + wg) * G + g;
      coherent_store(&p.part_o[slot * kD + e], Ov);
      if (e == 0) {
        coherent_store(&p.part_ml[slot * 2 + 0], M);
        coherent_store(&p.part_ml[slot * 2 + 1], L);
      }
    }
  });
  if (p.P == 1) return;

  // The last workgroup of the unit to arrive merges the P partial results (Algorithm 2).
  // The partials were stored write-through; once every store of the workgroup is acknowledged
  // the arrival is counted.
  SAAP_TRACE(4);
  wait_stores();
  SAAP_TRACE(5);
  __syncthreads();
  if (tid == 0) {
    // The arrival counter has one 8-bit field per XCD (P <= 128 fits): besides "am I last" it
    // tells the last workgroup whether every partial was written through its own XCD's L2.
    const unsigned xcc = (unsigned)__builtin_amdgcn_s_getreg(20 | (3 << 11)) & 7u;   // HW_REG_XCC_ID[3:0]
    const unsigned long long old = __hip_atomic_fetch_add(&p.counters[(size_t)unit * p.cstride], 1ull << (8 * xcc), __ATOMIC_RELAXED,
                                                          __HIP_MEMORY_SCOPE_AGENT);
    unsigned total = 0;
#pragma unroll
    for (int x = 0; x < 8; ++x) total += (unsigned)(old >> (8 * x)) & 0xffu;
    const unsigned mine = (unsigned)(old >> (8 * xcc)) & 0xffu;
    s_last = total == (unsigned)(p.P - 1) ? (mine == total ? 2 : 1) : 0;
  }
  __syncthreads();
  if (!s_last) return;
  if (s_last == 2) {
    // all partials went through this XCD's L2, which is coherent for its compute units: dropping
    // this compute unit's L1 lines is enough
    asm volatile("buffer_inv sc0" ::: "memory");
    SAAP_TRACE(12);
  } else {
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
  }
  SAAP_TRACE(6);

  final_merge<G, NT>(p.part_o, p.part_ml, (size_t)unit * p.P, p.P, qrow0, vs, p.out, p.out_bf16, p.lse,
                     reinterpret_cast<float*>(smem));
  SAAP_TRACE(8);
  if (tid == 0) __hip_atomic_store(&p.counters[(size_t)unit * p.cstride], 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}


// ------------------------------------------------------------------------------------------------
// Attention from a visit plan: the work of ALL units dealt to the workgroups in equal shares.
//
// A visit plan lists, per unit, the runs of the sorted cache to attend (first row and an exclusive
// prefix of the run lengths) and their total T_u.  The units' key ranges are concatenated into one
// global range of sum T_u keys and workgroup w takes keys [w*Q, (w+1)*Q) of it, Q = ceil(sum / W):
// every workgroup streams the same number of keys whatever the sizes of the visited buckets and of
// the units are (Section 5 "On GPU" notes that one block per bucket makes the largest bucket set the
// run time; with one team of workgroups per unit the largest unit does).  A workgroup whose share
// crosses a unit boundary finishes one unit (partial result, Algorithm 2) and goes on with the next;
// a unit is merged by the last of the workgroups that hold a piece of it.  Inside a workgroup the waves
// take batches of keys from the piece's counter, so a wave that memory serves late takes fewer.
//
// Plan layout per unit (stride ps = 2*nseg + 2 rounded up to a multiple of 4 ints):
//   [0] T_u | [1 .. nseg+1] pre[0..nseg], pre[0] = 0, pre[j+1] = pre[j] + length of run j | [nseg+2 ..] first row of run j
struct PlanParams {
  const void* q;          // [S,Hq,d]
  const void* K;          // [kv units, rows, d]
  const void* V;
  const int32_t* plan;    // [units, ps]
  void* out;              // [S,Hq,d]
  float* lse;             // [S,Hq] or null
  float* part_o;          // [slots, G, d]
  float* part_ml;         // [slots, G, 2]
  unsigned long long* counters;   // [units * cstride] arrivals; zero on entry and on exit
  int cstride;            // 8-byte words between the counters of two units
  long long rows;         // rows per kv unit
  const void* K2;         // second pair of tensors [kv units, rows2, d] or null: plan rows from `rows` on mean row - rows of
  const void* V2;         // these (prefill: the position-ordered keys beside the bucket-sorted ones)
  long long rows2;
  int tq;                 // units of one sequence that share a kv unit (query tokens per sequence; 1 at decode)
  int nseg;               // runs per unit in the plan
  int ps;                 // ints per unit in the plan
  int n_units;
  int Hq, Hkv;
  int independent;        // unit = (sequence, query head) instead of (sequence, KV head)
  int out_bf16;
  int all_tables;         // every unit's table is copied to LDS at the start (one memory round trip)
  int q_min;              // least number of keys per workgroup
  int piece_cost;         // what starting a piece of a unit costs a workgroup, in keys it could have streamed instead
  float scale_log2;       // scale * log2(e)
  const float* kscale;    // 8-bit cache: [kv units] scale of the K codes, else null
  const float* vscale;
};
constexpr int kPlanMaxWgs = 1024;       // workgroups of a planned launch (sizes the partial results)
constexpr int kPlanMaxUnits = 4096;
constexpr int kPlanTableInts = 16384;   // all units' tables fit LDS up to this many ints

__host__ __device__ constexpr int plan_stride(int nseg) { return (2 * nseg + 2 + 3) & ~3; }

// Pins a loaded value in its registers at this point of the program, so that the load is issued here
// and not moved into the branch that consumes it (where each load would wait for the one before).
__device__ __forceinline__ void issue_here(int4& v) { asm volatile("" : "+v"(v.x), "+v"(v.y), "+v"(v.z), "+v"(v.w)); }

// largest j in [0, n) with a[j] <= v  (a non-decreasing, a[0] <= v), found by the whole wave at once: every
// lane looks at one entry (every step-th one while more than 64 are left) and a ballot counts the entries
// not above v, which form a prefix.  One or two LDS round trips where a binary search takes six to thirteen.
// All lanes must call it with the same arguments.
__device__ __forceinline__ int wave_last_not_above(const int* a, int n, int v, int lane) {
  int lo = 0, len = n;
  while (len > 64) {
    const int step = (len + 63) >> 6;
    const int idx = lo + lane * step;
    const bool le = idx < lo + len && a[idx] <= v;
    const int k = __popcll(__ballot(le)) - 1;
    lo += k * step;
    len = min(step, len - k * step);
  }
  const bool le = lane < len && a[lo + lane] <= v;
  return lo + __popcll(__ballot(le)) - 1;
}

// largest j in [lo, hi) with a[j] <= v  (a non-decreasing, a[lo] <= v)
__device__ __forceinline__ int last_not_above(const int* a, int lo, int hi, int v) {
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (a[mid] <= v) lo = mid; else hi = mid;
  }
  return lo;
}

constexpr int kPieceSlots = 2;          // pieces of one workgroup that may be open at the same time

// The waves of a workgroup deposit the result of their keys of a piece in LDS; the last one to do so
// combines them (Algorithm 2 over the nw partial results, two outputs per lane and head: features `lane`
// and `lane + 64`).  emit(g, e, M, L, O) receives the merged values.  Called by one wave.
template <int G, int nw, typename F>
__device__ __forceinline__ void combine_deposits(const float* area, int lane, F emit) {
  const float* w_o = area;                                // [nw][G][d] unnormalised outputs
  const float* w_m = w_o + nw * G * kD;                   // [nw][G] maxima
  const float* w_l = w_m + nw * G;                        // [nw][G] sums of weights
#pragma unroll
  for (int g = 0; g < G; ++g) {
    // the head's LDS reads all go out before the first use
    float wj[nw], lj[nw], a0[nw], a1[nw];
#pragma unroll
    for (int j = 0; j < nw; ++j) {
      wj[j] = w_m[j * G + g];
      lj[j] = w_l[j * G + g];
      a0[j] = w_o[(j * G + g) * kD + lane];
      a1[j] = w_o[(j * G + g) * kD + 64 + lane];
    }
    __builtin_amdgcn_sched_barrier(0);
    float M = kNegBig;
#pragma unroll
    for (int j = 0; j < nw; ++j) M = fmaxf(M, wj[j]);
    float L = 0.f, o0 = 0.f, o1 = 0.f;
#pragma unroll
    for (int j = 0; j < nw; ++j) {
      const float w = fast_exp2(wj[j] - M);
      L = fmaf(w, lj[j], L);
      o0 = fmaf(w, a0[j], o0);
      o1 = fmaf(w, a1[j], o1);
    }
    emit(g, lane, M, L, o0);
    emit(g, lane + 64, M, L, o1);
  }
}

template <typename T, int G, int NT>
__global__ void __launch_bounds__(NT) attn_plan_kernel(PlanParams p) {
  extern __shared__ __align__(16) unsigned char smem[];
  __shared__ int s_wsum[2][16];
  __shared__ int s_next[kPieceSlots];     // next wave batch of the piece in the slot
  __shared__ int s_done[kPieceSlots];     // waves that have deposited their result of it
  __shared__ int s_gen[kPieceSlots];      // pieces the slot has served
  __shared__ int s_npend;
  __shared__ int s_pend[2][4];            // units this workgroup merges at the end: unit, first slot, partials, kind

  constexpr int nw = NT / 64;
  constexpr int KB = G == 8 ? 2 : 4;            // keys a key processor has in flight per batch
  constexpr int WB = 4 * KB;                    // keys of a wave batch: KB consecutive keys for each of its 4 processors
  constexpr bool kPrefetch = sizeof(T) <= 2;    // fp32 rows are too wide to double-buffer
  constexpr bool kFp8 = sizeof(T) == 1;
  constexpr int kDepositFloats = nw * G * (kD + 2);
  typedef typename DotType<T>::type TQ;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int sub = lane & 15, grp = lane >> 4;
  const int U = p.n_units, W = (int)gridDim.x;
  // Neighbouring shares go to one XCD (workgroups are handed to the XCDs in turn), so that most units are
  // merged from partial results that never left that XCD's L2.  Only speed depends on it.
  const int w = (W & 7) == 0 ? (int)(blockIdx.x & 7) * (W >> 3) + (int)(blockIdx.x >> 3) : (int)blockIdx.x;
  // The global range counts, before the keys of every unit, `F` positions that nobody reads: what a piece
  // costs its workgroup besides streaming.  A workgroup whose share crosses into another unit therefore
  // streams fewer keys than one that stays inside a unit, and both finish together.
  const int F = p.piece_cost;
  SAAP_TRACE(0);

  int* s_ustart = reinterpret_cast<int*>(smem);           // [U+1] start of each unit in the global range
  int* s_urank = s_ustart + (U + 1);                      // [U+1] units with keys before each unit
  int* s_tab = s_urank + (U + 1) + ((4 - (2 * (U + 1)) % 4) % 4);   // [U*ps] or [ps] plan tables (16-byte aligned)
  float* scratch = reinterpret_cast<float*>(s_tab + (p.all_tables ? U * p.ps : p.ps));   // deposits; merge scratch at the end

  if (tid < kPieceSlots) {
    s_next[tid] = 0;
    s_done[tid] = 0;
    s_gen[tid] = 0;
  }
  if (tid == 0) s_npend = 0;

  // ---- totals of all units -> ranges of the units in the global range
  if (p.all_tables) {
    // every load of a round goes out before the first store waits for one: unconditional, the index clamped
    const int n4 = U * p.ps / 4;
    const int4* src = reinterpret_cast<const int4*>(p.plan);
    for (int i0 = 0; i0 < n4; i0 += 8 * NT) {
      int4 r[8];
#pragma unroll
      for (int k = 0; k < 8; ++k) r[k] = src[min(i0 + tid + k * NT, n4 - 1)];
#pragma unroll
      for (int k = 0; k < 8; ++k) issue_here(r[k]);
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        const int i = i0 + tid + k * NT;
        if (i < n4) reinterpret_cast<int4*>(s_tab)[i] = r[k];
      }
    }
    __syncthreads();
  }
  {
    const int per = (U + NT - 1) / NT;                    // <= kPlanMaxUnits / NT
    const int u0 = tid * per;
    int tv[kPlanMaxUnits / NT];
#pragma unroll
    for (int k = 0; k < kPlanMaxUnits / NT; ++k) {
      const int u = u0 + k;
      const int uc = min(u, U - 1);
      tv[k] = p.all_tables ? s_tab[uc * p.ps] : p.plan[(size_t)uc * p.ps];
      if (k >= per || u >= U) tv[k] = 0;
    }
    int mine = 0, cnt = 0;
#pragma unroll
    for (int k = 0; k < kPlanMaxUnits / NT; ++k) {
      tv[k] = tv[k] > 0 ? tv[k] + F : 0;                  // extent in the global range
      mine += tv[k];
      cnt += tv[k] > 0 ? 1 : 0;
    }
    const int incl_k = (int)wave_prefix_sum((unsigned)mine), incl_c = (int)wave_prefix_sum((unsigned)cnt);
    if (lane == 63) {
      s_wsum[0][wave] = incl_k;
      s_wsum[1][wave] = incl_c;
    }
    __syncthreads();
    int run = incl_k - mine, rank = incl_c - cnt, tot_k = 0, tot_c = 0;
#pragma unroll
    for (int x = 0; x < nw; ++x) {
      if (x < wave) {
        run += s_wsum[0][x];
        rank += s_wsum[1][x];
      }
      tot_k += s_wsum[0][x];
      tot_c += s_wsum[1][x];
    }
#pragma unroll
    for (int k = 0; k < kPlanMaxUnits / NT; ++k) {
      const int u = u0 + k;
      if (k < per && u < U) {
        s_ustart[u] = run;
        s_urank[u] = rank;
        run += tv[k];
        rank += tv[k] > 0 ? 1 : 0;
      }
    }
    if (tid == 0) {
      s_ustart[U] = tot_k;
      s_urank[U] = tot_c;
    }
    __syncthreads();
  }
  const int t_all = s_ustart[U];
  const int Q = max((t_all + W - 1) / W, p.q_min);        // share of a workgroup
  const long long k0 = (long long)w * Q;
  const int k1 = (int)min((long long)t_all, k0 + Q);

  // a unit without keys has no workgroup: out = 0, lse = -inf written by workgroup u mod W
  for (int u = w; u < U; u += W) {
    if (s_ustart[u + 1] != s_ustart[u]) continue;
    const int qr = p.independent ? u : u * G;
    for (int x = tid; x < G * kD; x += NT) {
      if (p.out_bf16) reinterpret_cast<bf16_t*>(p.out)[(size_t)qr * kD + x] = (bf16_t)0;
      else reinterpret_cast<float*>(p.out)[(size_t)qr * kD + x] = 0.f;
    }
    if (tid < G && p.lse) p.lse[qr + tid] = -INFINITY;
  }
  if (k0 >= t_all) return;
  SAAP_TRACE(1);

  // ---- the pieces of my share, one unit after the other.  The waves go through them on their own:
  // inside a piece every wave takes the next batch of WB keys from the piece's counter until none is left
  // (a wave that was held up simply takes fewer), deposits its result in the slot's LDS area and moves on;
  // whoever deposits last combines the deposits and sends the piece's result off.  No workgroup barrier.
  int piece = 0;
  int u = wave_last_not_above(s_ustart, U, (int)k0, lane);   // the unit that holds position k0 (it has keys)
  for (int ks = (int)k0; ks < k1; ++u) {
    const int us = s_ustart[u], ue = s_ustart[u + 1];
    if (ue == us) continue;
    const int rs = us + F;                                // the unit's keys follow its F unread positions
    const int a = max(ks, rs) - rs, b = min(k1, ue) - rs; // my piece of unit u: its keys [a, b)
    ks = ue;
    if (b <= a) continue;                                 // my share ends before the unit's first key
    const int slot = piece % kPieceSlots, use = piece / kPieceSlots;
    ++piece;
    int kvu, qrow0;
    if (p.independent) {
      const int s = u / p.Hq, hq = u % p.Hq;
      kvu = s * p.Hkv + hq / (p.Hq / p.Hkv);
      qrow0 = u;
    } else {
      kvu = p.tq == 1 ? u : (u / (p.Hkv * p.tq)) * p.Hkv + u % p.Hkv;   // units are (sequence, token, KV head)
      qrow0 = u * G;
    }
    const T* Kb = reinterpret_cast<const T*>(p.K) + (size_t)kvu * p.rows * kD + sub * 8;
    const T* Vb = reinterpret_cast<const T*>(p.V) + (size_t)kvu * p.rows * kD + sub * 8;
    // rows of the second pair of tensors, addressed so that plan row r >= p.rows lands on its row r - p.rows
    const T* Kb2 = reinterpret_cast<const T*>(p.K2) + ((size_t)kvu * p.rows2 - (size_t)p.rows) * kD + sub * 8;
    const T* Vb2 = reinterpret_cast<const T*>(p.V2) + ((size_t)kvu * p.rows2 - (size_t)p.rows) * kD + sub * 8;
    const int row_end = (int)(p.rows + p.rows2);
    float scale_log2 = p.scale_log2, vs = 1.f;
    if constexpr (kFp8) {
      scale_log2 *= p.kscale[kvu];
      vs = p.vscale[kvu];
    }
    constexpr bool MM = kMatrixScores<T, G>, MV = kMatrixValues<T, G>;
    Queries<T, G> qv;
    qv.load(p.q, qrow0, sub, grp, scale_log2);
    // matrix path: the lane's piece of a row, in either pair of tensors
    const T* Kmm = reinterpret_cast<const T*>(p.K) + (size_t)kvu * p.rows * kD + grp * 16;
    const T* Kmm2 = reinterpret_cast<const T*>(p.K2) + ((size_t)kvu * p.rows2 - (size_t)p.rows) * kD + grp * 16;
    SAAP_TRACE(12);
    const int* tab = s_tab + u * p.ps;
    if (!p.all_tables) {
      // the tables do not fit LDS together: one unit's table at a time, the workgroup in step
      tab = s_tab;
      __syncthreads();                                    // the table of the piece before is dead
      const int n4 = p.ps / 4;
      const int4* src = reinterpret_cast<const int4*>(p.plan + (size_t)u * p.ps);
      for (int i0 = 0; i0 < n4; i0 += 8 * NT) {
        int4 r[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) r[k] = src[min(i0 + tid + k * NT, n4 - 1)];
#pragma unroll
        for (int k = 0; k < 8; ++k) issue_here(r[k]);
#pragma unroll
        for (int k = 0; k < 8; ++k) {
          const int i = i0 + tid + k * NT;
          if (i < n4) reinterpret_cast<int4*>(s_tab)[i] = r[k];
        }
      }
      __syncthreads();
    }
    const int* pre = tab + 1;                             // [nseg+1]
    const int* rowoff = tab + p.nseg + 2;                 // [nseg]
    // runs that hold the first and the last key of the piece
    const int ra = wave_last_not_above(pre, p.nseg, a, lane), rb = wave_last_not_above(pre, p.nseg, b - 1, lane);

    SAAP_TRACE(13);
    // The slot is free once the piece that used it before has been sent off.  The flags live in LDS, which
    // serves a wave's operations in order; relaxed accesses are enough there, and an acquire would also
    // wait for the query loads in flight.
    while (__hip_atomic_load(&s_gen[slot], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP) != use)
      __builtin_amdgcn_s_sleep(1);
    asm volatile("" ::: "memory");
    SAAP_TRACE(14);
    auto grab = [&]() {                                   // first key of the wave's next batch
      int g = 0;
      if (lane == 0) g = __hip_atomic_fetch_add(&s_next[slot], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
      return a + __builtin_amdgcn_readfirstlane(g) * WB;
    };

    float m = kNegBig, l = 0.f;
    Accum<G, MV> acc_o;
    acc_o.zero();

    // Keys of (processor grp, slot i) of the wave batch at `base`: base + i*4 + grp, so one load instruction of
    // the wave reads four neighbouring rows.  The lane's keys only move forward through the piece: its run is
    // found by stepping on from the run of its key in the batch before.
    int j = ra;
    auto load_batch = [&](int base, Batch<T, KB, MM>& bt) {
      int row;
      {
        const int v = min(base + (sub & (KB - 1)) * 4 + grp, b - 1);   // lane `sub` resolves slot sub % KB
        while (j < rb && pre[j + 1] <= v) ++j;
        row = rowoff[j] + (v - pre[j]);
        // a plan that breaks the contract (overlapping runs, a damaged index) must not turn into a
        // read outside the cache
        row = min(max(row, 0), row_end - 1);
      }
      bt.valid = 0u;
      bt.heads = 0u;
      if constexpr (MM) {
        // operand row m = lane % 16 is the key of (processor m / 4, slot m % 4), resolved by lane m % 4 of that processor
        const int rk = __shfl(row, (sub >> 2) * 16 + (sub & 3));
        const T* src = (rk >= (int)p.rows ? Kmm2 : Kmm) + (size_t)rk * kD;
#pragma unroll
        for (int c = 0; c < 2; ++c) bt.ka[c] = stream_load16(src + c * 64);
      }
#pragma unroll
      for (int i = 0; i < KB; ++i) {
        const int r = (int)row_lane<KB>(row, i);
        // slots past the end of the piece read its last key again (and score -inf): loads under a
        // branch would make the number of loads in flight unknown to the wait counters, and every wait
        // would then drain them all
        if (base + i * 4 + grp < b) bt.valid |= 1u << i;
        const bool second = r >= (int)p.rows;
        if constexpr (!MM) bt.k[i].load_stream((second ? Kb2 : Kb) + (size_t)r * kD);
        bt.v[i].load_stream((second ? Vb2 : Vb) + (size_t)r * kD);
      }
    };
    auto consume = [&](const Batch<T, KB, MM>& bt) { consume_batch<T, G, false>(bt, qv, scale_log2, sub, m, l, acc_o); };
    {
      // two batches at once to begin with; from then on one batch ahead, its LDS round trip off the path
      int base;
      {
        int g = 0;
        if (lane == 0) g = __hip_atomic_fetch_add(&s_next[slot], 2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        base = a + __builtin_amdgcn_readfirstlane(g) * WB;
      }
      if (base < b) {
        int next = base + WB;
        SAAP_TRACE(15);
        Batch<T, KB, MM> cur;
        load_batch(base, cur);
        SAAP_TRACE(2);
        if constexpr (kPrefetch) {
          while (next < b) {
            const int after = grab();
            Batch<T, KB, MM> nxt;
            load_batch(next, nxt);      // in flight while the current batch is consumed
            __builtin_amdgcn_sched_barrier(0);
            consume(cur);
            cur = nxt;
            next = after;
          }
          consume(cur);
        } else {
          consume(cur);
          while (next < b) {
            const int after = grab();
            load_batch(next, cur);
            consume(cur);
            next = after;
          }
        }
      }
    }

    // ---- end of the piece
    float O[G][8];
    wave_combine<G, MV>(m, l, acc_o, O);
    const int w_first = rs / Q, w_last = (ue - 1) / Q;    // the workgroups that hold the unit's first and last key
    const int P = w_last - w_first + 1;
    // partial results are numbered along the global range: (workgroup, unit) pairs in order differ by at
    // least one in w + rank(u), so a unit's partial results are consecutive
    const size_t pslot = (size_t)w + s_urank[u];
    float* area = scratch + slot * kDepositFloats;
    auto emit = [&](int g, int e, float M, float L, float Ov) {
      if (P == 1) {
        const float r = L > 0.f ? vs * (Ov / L) : 0.f;
        if (p.out_bf16) reinterpret_cast<bf16_t*>(p.out)[(size_t)(qrow0 + g) * kD + e] = (bf16_t)f32_to_bf16_bits(r);
        else reinterpret_cast<float*>(p.out)[(size_t)(qrow0 + g) * kD + e] = r;
        if (e == 0 && p.lse) p.lse[qrow0 + g] = L > 0.f ? (M + __log2f(L)) * kLn2 : -INFINITY;
      } else {
        coherent_store(&p.part_o[(pslot * G + g) * kD + e], Ov);
        if (e == 0) {
          coherent_store(&p.part_ml[(pslot * G + g) * 2 + 0], M);
          coherent_store(&p.part_ml[(pslot * G + g) * 2 + 1], L);
        }
      }
    };
    // Arrival at the unit's counter (one lane): count in bits 0-15, sum of the arrivals' XCD numbers in
    // bits 16-31, sum of their squares in bits 32-47.  sum = n*x and squares = n*x*x hold only if every
    // arrival came from XCD x: then all partial results went through this XCD's L2.  The workgroup whose
    // arrival completes the unit merges it when all its own pieces are done (at most two of its units are
    // shared with other workgroups: the first and the last of its share).
    auto arrive = [&]() {
      const unsigned long long xcc = (unsigned long long)((unsigned)__builtin_amdgcn_s_getreg(20 | (3 << 11)) & 7u);
      const unsigned long long old = __hip_atomic_fetch_add(&p.counters[(size_t)u * p.cstride], 1ull | (xcc << 16) | ((xcc * xcc) << 32),
                                                            __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      const unsigned long long n = old & 0xffffull, sx = (old >> 16) & 0xffffull, sxx = (old >> 32) & 0xffffull;
      if (n == (unsigned long long)(P - 1)) {
        const int at = __hip_atomic_fetch_add(&s_npend, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        s_pend[at][0] = u;
        s_pend[at][1] = w_first + s_urank[u];
        s_pend[at][2] = P;
        s_pend[at][3] = (sx == n * xcc && sxx == n * xcc * xcc) ? 2 : 1;
      }
    };
    if (ue + F >= k1) {
      // The last piece of my share: the waves have nothing to go on with, so they combine their results
      // together (every thread one output) rather than leave it to one of them.
      workgroup_combine<G, NT>(area, m, l, O, emit);
      SAAP_TRACE(4);
      if (P > 1) {
        wait_stores();
        __syncthreads();
        if (tid == 0) arrive();
      }
      break;
    }
    // Any other piece: deposit and go on with the next piece; the last wave to deposit combines the
    // deposits and sends the piece's result off while the others stream already.
    {
      float* w_o = area;
      float* w_m = w_o + nw * G * kD;
      float* w_l = w_m + nw * G;
      if (grp == 0) {
#pragma unroll
        for (int g = 0; g < G; ++g) {
          float4* dst = reinterpret_cast<float4*>(w_o + (wave * G + g) * kD + sub * 8);
          dst[0] = make_float4(O[g][0], O[g][1], O[g][2], O[g][3]);
          dst[1] = make_float4(O[g][4], O[g][5], O[g][6], O[g][7]);
        }
        if (sub < G) {            // lane `sub` owns head `sub` (key slot 0)
          w_m[wave * G + sub] = m;
          w_l[wave * G + sub] = l;
        }
      }
    }
    int arrived = 0;
    if (lane == 0) arrived = __hip_atomic_fetch_add(&s_done[slot], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    if (__builtin_amdgcn_readfirstlane(arrived) != nw - 1) continue;
    asm volatile("" ::: "memory");
    SAAP_TRACE_WAVE(9);
    combine_deposits<G, nw>(area, lane, emit);
    if (P > 1) {
      wait_stores();
      SAAP_TRACE_WAVE(10);
      if (lane == 0) arrive();
    }
    SAAP_TRACE_WAVE(11);
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");     // the deposits have been read
    if (lane == 0) {
      s_next[slot] = 0;
      s_done[slot] = 0;
      __hip_atomic_store(&s_gen[slot], use + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    }
  }
  SAAP_TRACE(3);

  // ---- units that were completed by this workgroup's arrival: Algorithm 2 over their partial results
  __syncthreads();
  SAAP_TRACE(5);
  const int npend = s_npend;
  for (int i = 0; i < npend; ++i) {
    const int mu = s_pend[i][0], slot0 = s_pend[i][1], P = s_pend[i][2], kind = s_pend[i][3];
    const int kvu = p.independent ? (mu / p.Hq) * p.Hkv + (mu % p.Hq) / (p.Hq / p.Hkv)
                                  : p.tq == 1 ? mu : (mu / (p.Hkv * p.tq)) * p.Hkv + mu % p.Hkv;
    const int qrow0 = p.independent ? mu : mu * G;
    float vs = 1.f;
    if constexpr (kFp8) vs = p.vscale[kvu];
    if (kind == 2) {
      // this XCD's L2 is coherent for its compute units: dropping this compute unit's L1 lines is enough
      asm volatile("buffer_inv sc0" ::: "memory");
      final_merge<G, NT, false>(p.part_o, p.part_ml, (size_t)slot0, P, qrow0, vs, p.out, p.out_bf16, p.lse, scratch);
    } else {
      // partial results from several XCDs: read them past this XCD's L2 (an acquire fence at agent scope would
      // instead drop that whole L2, the classifier's weights included)
      final_merge<G, NT, true>(p.part_o, p.part_ml, (size_t)slot0, P, qrow0, vs, p.out, p.out_bf16, p.lse, scratch);
    }
    if (tid == 0) __hip_atomic_store(&p.counters[(size_t)mu * p.cstride], 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();                                      // the merge scratch is used again
  }
  SAAP_TRACE(8);
}

// Visit plan of every unit from its list of runs: one workgroup per unit.
__global__ void __launch_bounds__(256) visit_plan_kernel(const int32_t* __restrict__ selected, const int32_t* __restrict__ off,
                                                        const int32_t* __restrict__ len, int32_t* __restrict__ plan,
                                                        int nsel, int resident, int runs, int ps, int Hq, int Hkv,
                                                        int independent) {
  __shared__ int s_wsum[4];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int unit = blockIdx.x;
  const int kvu = independent ? (unit / Hq) * Hkv + (unit % Hq) / (Hq / Hkv) : unit;
  const int nseg = nsel + (resident >= 0 ? 1 : 0);
  const int32_t* lenu = len + (size_t)kvu * runs;
  const int32_t* offu = off + (size_t)kvu * (runs + 1);
  const int32_t* sel = selected ? selected + (size_t)unit * nsel : nullptr;
  int32_t* pl = plan + (size_t)unit * ps;
  const int per = (nseg + 255) / 256;
  const int j0 = tid * per, j1 = min(j0 + per, nseg);
  int mine = 0;
  for (int j = j0; j < j1; ++j) {
    const int b = j < nsel ? min(max(sel[j], 0), runs - 1) : resident;
    mine += max(lenu[b], 0);
  }
  const int incl = (int)wave_prefix_sum((unsigned)mine);
  if (lane == 63) s_wsum[wave] = incl;
  __syncthreads();
  int run = incl - mine, total = 0;
  for (int x = 0; x < 4; ++x) {
    if (x < wave) run += s_wsum[x];
    total += s_wsum[x];
  }
  for (int j = j0; j < j1; ++j) {
    const int b = j < nsel ? min(max(sel[j], 0), runs - 1) : resident;
    run += max(lenu[b], 0);
    pl[2 + j] = run;
    pl[nseg + 2 + j] = offu[b];
  }
  if (tid == 0) {
    pl[0] = total;
    pl[1] = 0;
  }
}

// Visit plans of a block of prompt tokens: one workgroup per (sequence, token, KV head).  The token at
// position p sees, of the L = p + 1 keys so far, the first n_sink, the last n_recent and the members of its
// listed buckets.  Runs of its plan: [0] the sink keys and [1] the recent keys, read from the position-ordered
// tensors (plan rows from Ncap on), then one run per listed bucket: those members of the bucket that lie
// between the sink and the recent keys.  The members of a bucket are stored in ascending position, so that
// part is one stretch of the bucket's rows, found by two binary searches in `idx`.
__global__ void __launch_bounds__(256) prefill_plan_kernel(const int32_t* __restrict__ selected, const int32_t* __restrict__ off,
                                                          const int32_t* __restrict__ len, const int32_t* __restrict__ idx,
                                                          const int32_t* __restrict__ pos0, int32_t* __restrict__ plan,
                                                          int nprobe, int n_sink, int n_recent, int B, int Ncap, int Nt,
                                                          int Tq, int Hkv, int ps) {
  __shared__ int s_wsum[4];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int unit = blockIdx.x;                            // (s * Tq + t) * Hkv + h
  const int h = unit % Hkv, t = (unit / Hkv) % Tq, s = unit / (Hkv * Tq);
  const int kvu = s * Hkv + h;
  const int L = min(max(pos0[s] + t + 1, 0), Nt);         // keys the token can see at all
  const int sink_end = min(n_sink, L);                    // positions [0, sink_end) are the sink
  const int recent_begin = max(sink_end, L - n_recent);   // positions [recent_begin, L) the recent keys
  const int nseg = nprobe + 2;
  const int32_t* lenu = len + (size_t)kvu * B;
  const int32_t* offu = off + (size_t)kvu * (B + 1);
  const int32_t* idxu = idx + (size_t)kvu * Ncap;
  const int32_t* sel = selected + ((size_t)kvu * Tq + t) * nprobe;
  int32_t* pl = plan + (size_t)unit * ps;
  // first member of the run at `first` (n members, ascending positions) whose position is not below `bound`
  auto lower = [&](int first, int n, int bound) {
    int lo = 0, hi = n;
    while (lo < hi) {
      const int mid = (lo + hi) >> 1;
      if (idxu[first + mid] < bound) lo = mid + 1; else hi = mid;
    }
    return lo;
  };
  const int per = (nseg + 255) / 256;
  const int j0 = tid * per, j1 = min(j0 + per, nseg);
  int mine = 0;
  for (int j = j0; j < j1; ++j) {
    int first, n;
    if (j == 0) {
      first = Ncap;
      n = sink_end;
    } else if (j == 1) {
      first = Ncap + recent_begin;
      n = L - recent_begin;
    } else {
      const int b = min(max(sel[j - 2], 0), B - 1);
      const int o = offu[b], m = max(lenu[b], 0);
      const int lo = lower(o, m, sink_end), hi = lower(o, m, recent_begin);
      first = o + lo;
      n = max(hi - lo, 0);
    }
    pl[nseg + 2 + j] = first;
    pl[2 + j] = n;                                        // its length for now; the prefix below
    mine += n;
  }
  const int incl = (int)wave_prefix_sum((unsigned)mine);
  if (lane == 63) s_wsum[wave] = incl;
  __syncthreads();
  int run = incl - mine, total = 0;
  for (int x = 0; x < 4; ++x) {
    if (x < wave) run += s_wsum[x];
    total += s_wsum[x];
  }
  for (int j = j0; j < j1; ++j) {
    run += pl[2 + j];
    pl[2 + j] = run;
  }
  if (tid == 0) {
    pl[0] = total;
    pl[1] = 0;
  }
}

// bytes of one key's K row and V row
static int key_bytes(int dtype) { return dtype == kDtypeFp8 ? 2 * kD : dtype == SAAP_BF16 ? 4 * kD : 8 * kD; }

struct LaunchPlan {
  int P, threads, stage, max_chunks;
  size_t lds;
};

// Workgroups per unit for a launch shape: the device filled once, no more than the work gives.
static long long plan_p(int n_units, long long est_keys_per_unit, int threads, int wgs_per_cu, int kb) {
  const long long chunk = (long long)(threads / 16) * kb;   // keys per workgroup batch
  long long P = (long long)device_cus() * wgs_per_cu / n_units;
  const long long by_work = (est_keys_per_unit + chunk - 1) / chunk;
  if (P > by_work) P = by_work;
  if (P > kMaxP) P = kMaxP;
  return P < 1 ? 1 : P;
}

// Two launch shapes: one workgroup of 512 threads per compute unit, or two of 256.  Over one
// contiguous range (dense attention) the second streams up to 8 % faster (measured: 660 -> 605 us over
// 4.3 GB, 7.1 TB/s) but doubles the partial results that the merging workgroup of a unit reads, which
// costs about 0.02 us per extra partial and head; it is taken when the first outweighs the second.
// Over a list of buckets the two shapes measured alike within 1 % at 0.2 and 0.9 GB per launch and the
// first is better below that, so a launch with a selection always takes the first.
static bool narrow_shape_pays(int n_units, long long est_keys_per_unit, int G, int key_bytes, int kb) {
  const double stream_us = (double)est_keys_per_unit * n_units * key_bytes / 6.0e6;   // at 6 TB/s
  const long long p_wide = plan_p(n_units, est_keys_per_unit, 512, 1, kb);
  const long long p_narrow = plan_p(n_units, est_keys_per_unit, 256, 2, kb);
  const double merge_us = 0.02 * G * (double)(p_narrow > p_wide ? p_narrow - p_wide : 0) + 0.5;
  return 0.08 * stream_us > merge_us;
}

LaunchPlan plan_launch(int n_units, long long est_keys_per_unit, long long max_keys_per_unit, int G, int nseg,
                       bool list, int B, bool has_selection, int key_bytes, bool masked = false) {
  const int kb = G == 8 ? 2 : 4;
  int threads = env_int("SAAP_ATTN_THREADS", 0);
  if (threads != 256 && threads != 512)
    threads = !masked && !has_selection && narrow_shape_pays(n_units, est_keys_per_unit, G, key_bytes, kb) ? 256 : 512;
  if (masked) threads = 512;
  const int wgs_per_cu = env_int("SAAP_ATTN_WGS_PER_CU", threads == 256 ? 2 : 1);
  const long long chunk = (long long)(threads / 16) * kb;   // keys per workgroup batch
  long long P = plan_p(n_units, est_keys_per_unit, threads, wgs_per_cu, kb);
  const int force_p = env_int("SAAP_ATTN_P", 0);
  if (force_p > 0 && force_p <= kMaxP) P = force_p;
  LaunchPlan lp;
  lp.P = (int)P;
  lp.threads = threads;
  lp.max_chunks = (int)(((max_keys_per_unit + chunk - 1) / chunk + P - 1) / P + 1);
  size_t a = list ? (size_t)(2 * nseg + 1 + 2 * lp.max_chunks) * sizeof(int) : 0;
  lp.stage = !masked && list && has_selection && nseg <= 2 * threads && B <= 8 * threads && env_int("SAAP_ATTN_STAGE", 1);
  if (lp.stage) a += (size_t)2 * B * sizeof(int);
  if (masked) a += (size_t)(nseg + B) * sizeof(int);     // heads per run, heads per bucket
  const size_t b = (size_t)(threads / 64) * G * (kD + 2) * sizeof(float) + G * sizeof(float);
  const size_t c = (size_t)(P * G + 2 * G + 4) * sizeof(float) + (size_t)threads * sizeof(float4);
  lp.lds = a > b ? a : b;
  if (c > lp.lds) lp.lds = c;
  return lp;
}

template <typename T, int G, bool LIST, int NT, bool MASKED = false, int SEL = 0>
int32_t launch_nt(const AttnParams& p, const LaunchPlan& lp, hipStream_t stream) {
  auto kern = attn_kernel<T, G, LIST, NT, MASKED, SEL>;
  if (lp.lds > 48 * 1024) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                            (int)lp.lds) != hipSuccess)
      return SAAP_HIP_ERROR;
  }
  saap_trace_arm();
  hipLaunchKernelGGL(kern, dim3((unsigned)(p.n_units * p.P)), dim3((unsigned)lp.threads), lp.lds, stream, p);
  return launch_status();
}

template <typename T, int G, bool LIST>
int32_t launch_one(const AttnParams& p, const LaunchPlan& lp, hipStream_t stream) {
  return lp.threads == 256 ? launch_nt<T, G, LIST, 256>(p, lp, stream) : launch_nt<T, G, LIST, 512>(p, lp, stream);
}

// Independent routing with G > 1 heads per KV head: the masked kernels, 512 threads only.
int32_t launch_masked(const AttnParams& p, const LaunchPlan& lp, int G, int dtype, hipStream_t stream) {
#define SAAP_CASE(TT, GG) return launch_nt<TT, GG, true, 512, true>(p, lp, stream)
  if (dtype == kDtypeFp8) {
    switch (G) {
      case 2: SAAP_CASE(fp8_t, 2);
      case 4: SAAP_CASE(fp8_t, 4);
      case 8: SAAP_CASE(fp8_t, 8);
    }
  } else if (dtype == SAAP_BF16) {
    switch (G) {
      case 2: SAAP_CASE(bf16_t, 2);
      case 4: SAAP_CASE(bf16_t, 4);
      case 8: SAAP_CASE(bf16_t, 8);
    }
  } else {
    switch (G) {
      case 2: SAAP_CASE(float, 2);
      case 4: SAAP_CASE(float, 4);
      case 8: SAAP_CASE(float, 8);
    }
  }
#undef SAAP_CASE
  return SAAP_UNSUPPORTED;
}

template <bool LIST>
int32_t launch_attn(const AttnParams& p, const LaunchPlan& lp, int G, int dtype, hipStream_t stream) {
#define SAAP_CASE(TT, GG) return launch_one<TT, GG, LIST>(p, lp, stream)
  if (dtype == kDtypeFp8) {
    switch (G) {
      case 1: SAAP_CASE(fp8_t, 1);
      case 2: SAAP_CASE(fp8_t, 2);
      case 4: SAAP_CASE(fp8_t, 4);
      case 8: SAAP_CASE(fp8_t, 8);
    }
  } else if (dtype == SAAP_BF16) {
    switch (G) {
      case 1: SAAP_CASE(bf16_t, 1);
      case 2: SAAP_CASE(bf16_t, 2);
      case 4: SAAP_CASE(bf16_t, 4);
      case 8: SAAP_CASE(bf16_t, 8);
    }
  } else {
    switch (G) {
      case 1: SAAP_CASE(float, 1);
      case 2: SAAP_CASE(float, 2);
      case 4: SAAP_CASE(float, 4);
      case 8: SAAP_CASE(float, 8);
    }
  }
#undef SAAP_CASE
  return SAAP_UNSUPPORTED;
}

}  // namespace

// Workspace bytes of the attention calls for `units` units of G heads.
size_t attn_workspace_bytes(long long units, int G) {
  return (size_t)SAAP_WS_HEADER_BYTES + (size_t)units * kMaxP * G * (kD + 2) * sizeof(float);
}
size_t prefill_workspace_bytes(long long S, int Tq, int Hq, int Hkv, int nprobe);
// ... of the planned attention: one partial result per (workgroup, unit) pair that meets
size_t planned_workspace_bytes(long long units, int G) {
  return (size_t)SAAP_WS_HEADER_BYTES + (size_t)(kPlanMaxWgs + units) * G * (kD + 2) * sizeof(float);
}

}  // namespace saap

using namespace saap;

static int32_t check_common(const void* q, const void* K, const void* V, void* out, int S, int Hq, int Hkv,
                            int d, int dtype, int out_dtype, const void* ws) {
  if (!q || !K || !V || !out || !ws) return SAAP_INVALID_ARG;
  if (!aligned16(q) || !aligned16(K) || !aligned16(V) || !aligned16(out) || !aligned16(ws)) return SAAP_INVALID_ARG;
  if (S <= 0 || Hq <= 0 || Hkv <= 0 || Hq % Hkv != 0) return SAAP_INVALID_ARG;
  if ((dtype != SAAP_F32 && dtype != SAAP_BF16 && dtype != kDtypeFp8) || (out_dtype != SAAP_F32 && out_dtype != SAAP_BF16))
    return SAAP_INVALID_ARG;
  if (d != kD) return SAAP_UNSUPPORTED;
  const int G = Hq / Hkv;
  if (G != 1 && G != 2 && G != 4 && G != 8) return SAAP_UNSUPPORTED;
  return SAAP_OK;
}

// The index and the bucket lists of the list-driven attention calls.
static int32_t check_lists(const int32_t* off, const int32_t* len, const int32_t* selected, int nprobe, int mode,
                           int resident_run, int Ncap, int B) {
  if (!off || !len || (nprobe > 0 && !selected)) return SAAP_INVALID_ARG;
  if (mode != SAAP_GROUP_SUM && mode != SAAP_INDEPENDENT) return SAAP_INVALID_ARG;
  if (B <= 0 || Ncap <= 0 || nprobe < 0 || resident_run < -1 || resident_run >= B) return SAAP_INVALID_ARG;
  const int nseg = nprobe + (resident_run >= 0 ? 1 : 0);
  if (nseg > B) return SAAP_INVALID_ARG;
  if (nseg > SAAP_MAX_BUCKETS) return SAAP_UNSUPPORTED;
  return SAAP_OK;
}

// ---- visit plans and the attention that follows them ---------------------------------------------

static long long plan_units(int S, int Hq, int Hkv, int mode) { return mode == SAAP_INDEPENDENT ? (long long)S * Hq : (long long)S * Hkv; }

extern "C" size_t saap_visit_plan_bytes(int32_t S, int32_t Hq, int32_t Hkv, int32_t nruns, int32_t mode) {
  if (S <= 0 || Hq <= 0 || Hkv <= 0 || Hq % Hkv != 0 || nruns < 0 || nruns > SAAP_MAX_BUCKETS) return 0;
  if (mode != SAAP_GROUP_SUM && mode != SAAP_INDEPENDENT) return 0;
  return (size_t)plan_units(S, Hq, Hkv, mode) * plan_stride(nruns) * sizeof(int32_t);
}

extern "C" int32_t saap_build_visit_plan(const int32_t* selected, const int32_t* off, const int32_t* len,
                                         int32_t nprobe, int32_t mode, int32_t resident_run, int32_t* plan,
                                         int32_t S, int32_t Hq, int32_t Hkv, int32_t runs, void* stream) {
  begin_call();
  if (!off || !len || !plan || !aligned16(plan) || (nprobe > 0 && !selected)) return SAAP_INVALID_ARG;
  if (S <= 0 || Hq <= 0 || Hkv <= 0 || Hq % Hkv != 0 || runs <= 0) return SAAP_INVALID_ARG;
  if (mode != SAAP_GROUP_SUM && mode != SAAP_INDEPENDENT) return SAAP_INVALID_ARG;
  if (nprobe < 0 || resident_run < -1 || resident_run >= runs) return SAAP_INVALID_ARG;
  const int nseg = nprobe + (resident_run >= 0 ? 1 : 0);
  if (nseg > runs) return SAAP_INVALID_ARG;
  if (nseg > SAAP_MAX_BUCKETS) return SAAP_UNSUPPORTED;
  const long long units = plan_units(S, Hq, Hkv, mode);
  hipLaunchKernelGGL(visit_plan_kernel, dim3((unsigned)units), dim3(256), 0, static_cast<hipStream_t>(stream), selected,
                     off, len, plan, nprobe, resident_run, runs, plan_stride(nseg), Hq, Hkv,
                     mode == SAAP_INDEPENDENT ? 1 : 0);
  return launch_status();
}

template <typename T>
static int32_t launch_planned(const PlanParams& p, int G, unsigned grid, size_t lds, hipStream_t stream) {
#define SAAP_CASE(GG)                                                                                     \
  case GG: {                                                                                              \
    auto kern = attn_plan_kernel<T, GG, 512>;                                                             \
    if (lds > 48 * 1024 && hipFuncSetAttribute(reinterpret_cast<const void*>(kern),                      \
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess) \
      return SAAP_HIP_ERROR;                                                                              \
    saap_trace_arm();                                                                                     \
    hipLaunchKernelGGL(kern, dim3(grid), dim3(512), lds, stream, p);                                      \
    return launch_status();                                                                               \
  }
  switch (G) {
    SAAP_CASE(1)
    SAAP_CASE(2)
    SAAP_CASE(4)
    SAAP_CASE(8)
  }
#undef SAAP_CASE
  return SAAP_UNSUPPORTED;
}

// K2, V2 (or null) with rows2 rows per (sequence, KV head): plan rows from Ncap on.  tq > 1: S counts
// (sequence, token) pairs of which tq consecutive ones share the (sequence, KV head) tensors.
static int32_t planned_attention(const void* q, const void* Ksorted, const void* Vsorted, const float* kscale,
                                 const float* vscale, const int32_t* plan, int32_t nruns, int32_t mode, float scale,
                                 void* out, int32_t out_dtype, float* lse, int32_t S, int32_t Hq, int32_t Hkv,
                                 int32_t Ncap, int32_t d, int32_t dtype, void* ws, size_t ws_bytes, void* stream,
                                 const void* K2 = nullptr, const void* V2 = nullptr, int32_t rows2 = 0, int32_t tq = 1) {
  int32_t st = check_common(q, Ksorted, Vsorted, out, S, Hq, Hkv, d, dtype, out_dtype, ws);
  if (st != SAAP_OK) return st;
  if (!plan || !aligned16(plan)) return SAAP_INVALID_ARG;
  if (mode != SAAP_GROUP_SUM && mode != SAAP_INDEPENDENT) return SAAP_INVALID_ARG;
  if (nruns < 0 || Ncap <= 0) return SAAP_INVALID_ARG;
  if (dtype == kDtypeFp8 && (!kscale || !vscale)) return SAAP_INVALID_ARG;
  const bool indep = mode == SAAP_INDEPENDENT;
  const int G = indep ? 1 : Hq / Hkv;
  const long long units = plan_units(S, Hq, Hkv, mode);
  const int ps = plan_stride(nruns);
  // every unit's keys are numbered in one 32-bit range
  if (units > kPlanMaxUnits || ps > kPlanTableInts || units * ((long long)Ncap + rows2 + 65536) >= (1ll << 31))
    return SAAP_UNSUPPORTED;
  if (K2 && (!V2 || !aligned16(K2) || !aligned16(V2) || rows2 <= 0 || tq < 1 || S % tq != 0 || mode != SAAP_GROUP_SUM))
    return SAAP_INVALID_ARG;
  if (ws_bytes < planned_workspace_bytes(units, G)) return SAAP_WORKSPACE_TOO_SMALL;

  long long W = device_cus();
  if (W > units * kMaxP) W = units * kMaxP;
  if (W > kPlanMaxWgs) W = kPlanMaxWgs;
  W = env_int("SAAP_PLAN_WGS", (int)W);
  if (W < 1 || W > kPlanMaxWgs) return SAAP_INVALID_ARG;
  constexpr int NT = 512;
  PlanParams p{};
  p.q = q; p.K = Ksorted; p.V = Vsorted; p.plan = plan; p.out = out; p.lse = lse;
  p.counters = reinterpret_cast<unsigned long long*>(ws);
  p.cstride = units * 128 <= (long long)SAAP_WS_HEADER_BYTES ? 16 : 1;
  p.part_ml = reinterpret_cast<float*>(static_cast<char*>(ws) + SAAP_WS_HEADER_BYTES);
  p.part_o = p.part_ml + (size_t)(kPlanMaxWgs + units) * G * 2;
  p.rows = Ncap; p.nseg = nruns; p.ps = ps; p.n_units = (int)units; p.Hq = Hq; p.Hkv = Hkv;
  p.K2 = K2 ? K2 : Ksorted; p.V2 = K2 ? V2 : Vsorted; p.rows2 = K2 ? rows2 : 0; p.tq = tq;
  p.independent = indep ? 1 : 0; p.out_bf16 = out_dtype == SAAP_BF16;
  p.q_min = env_int("SAAP_PLAN_QMIN", (NT / 16) * (G == 8 ? 2 : 4));     // one batch of every wave
  p.piece_cost = env_int("SAAP_PLAN_PIECE_COST", 128);
  if (p.piece_cost < 0 || p.piece_cost > 65536 || p.q_min < 1) return SAAP_INVALID_ARG;
  p.scale_log2 = scale * kLog2e; p.kscale = kscale; p.vscale = vscale;
  // LDS: unit ranges and ranks | plan tables | deposits of the open pieces, reused as merge scratch
  const size_t f_deposits = (size_t)kPieceSlots * (NT / 64) * G * (kD + 2);
  const size_t f_merge = (size_t)W * G + 2 * G + 8 + (size_t)NT * 4;
  const size_t fixed = ((size_t)2 * (units + 1) + 3) * sizeof(int) + (f_deposits > f_merge ? f_deposits : f_merge) * sizeof(float);
  const size_t lds_max = 160 * 1024 - 1024;               // a compute unit's LDS less the kernel's static arrays
  p.all_tables = fixed + (size_t)units * ps * sizeof(int) <= lds_max ? 1 : 0;
  const size_t lds = fixed + (p.all_tables ? (size_t)units * ps : (size_t)ps) * sizeof(int);
  if (lds > lds_max) return SAAP_UNSUPPORTED;
  hipStream_t hs = static_cast<hipStream_t>(stream);
  if (dtype == kDtypeFp8) return launch_planned<fp8_t>(p, G, (unsigned)W, lds, hs);
  if (dtype == SAAP_BF16) return launch_planned<bf16_t>(p, G, (unsigned)W, lds, hs);
  return launch_planned<float>(p, G, (unsigned)W, lds, hs);
}

extern "C" int32_t saap_planned_decode_attention(const void* q, const void* Ksorted, const void* Vsorted,
                                                 const int32_t* plan, int32_t nruns, int32_t mode, float scale,
                                                 void* out, int32_t out_dtype, float* lse, int32_t S, int32_t Hq,
                                                 int32_t Hkv, int32_t Ncap, int32_t d, int32_t dtype, void* ws,
                                                 size_t ws_bytes, void* stream) {
  begin_call();
  if (dtype != SAAP_F32 && dtype != SAAP_BF16) return SAAP_INVALID_ARG;
  return planned_attention(q, Ksorted, Vsorted, nullptr, nullptr, plan, nruns, mode, scale, out, out_dtype, lse, S, Hq,
                           Hkv, Ncap, d, dtype, ws, ws_bytes, stream);
}

extern "C" int32_t saap_planned_decode_attention_fp8(const void* q, const uint8_t* K8, const uint8_t* V8,
                                                     const float* kscale, const float* vscale, const int32_t* plan,
                                                     int32_t nruns, int32_t mode, float scale, void* out,
                                                     int32_t out_dtype, float* lse, int32_t S, int32_t Hq, int32_t Hkv,
                                                     int32_t Ncap, int32_t d, void* ws, size_t ws_bytes, void* stream) {
  begin_call();
  if (!kscale || !vscale) return SAAP_INVALID_ARG;
  return planned_attention(q, K8, V8, kscale, vscale, plan, nruns, mode, scale, out, out_dtype, lse, S, Hq, Hkv, Ncap,
                           d, kDtypeFp8, ws, ws_bytes, stream);
}

// Attention over the selected runs plus, if resident_run >= 0, one run that is always visited.
// B = runs per unit in `len`.
// dtype kDtypeFp8: Ksorted, Vsorted hold E4M3 codes with the per-unit scales kscale, vscale; q is bf16.
static int32_t sparse_attention(const void* q, const void* Ksorted, const void* Vsorted, const float* kscale,
                                const float* vscale, const int32_t* off,
                                const int32_t* len, const int32_t* selected, int32_t nprobe, int32_t mode,
                                int32_t resident_run, float scale, void* out, int32_t out_dtype, float* lse,
                                int32_t S, int32_t Hq, int32_t Hkv, int32_t Ncap, int32_t B, int32_t d,
                                int32_t dtype, void* ws, size_t ws_bytes, void* stream) {
  int32_t st = check_common(q, Ksorted, Vsorted, out, S, Hq, Hkv, d, dtype, out_dtype, ws);
  if (st != SAAP_OK) return st;
  st = check_lists(off, len, selected, nprobe, mode, resident_run, Ncap, B);
  if (st != SAAP_OK) return st;
  int nseg = nprobe + (resident_run >= 0 ? 1 : 0);
  const bool indep = mode == SAAP_INDEPENDENT;
  // Independent routing of G > 1 heads that share a KV head: one unit per KV head visits the union
  // of the heads' lists once, each head attending only its own runs (masked kernels).  They hold
  // 16 buckets per thread at most; beyond that every head is a unit of its own.
  const int heads = Hq / Hkv;
  const bool masked = indep && heads > 1 && B <= 16 * 512;
  if (dtype == kDtypeFp8 && (!kscale || !vscale)) return SAAP_INVALID_ARG;
  const int G = masked ? heads : indep ? 1 : heads;
  const long long units = indep && !masked ? (long long)S * Hq : (long long)S * Hkv;
  if (masked) {
    const long long cap = (long long)heads * nprobe + (resident_run >= 0 ? 1 : 0);
    nseg = (int)(cap < B ? cap : B);
  }
  if (units * sizeof(unsigned long long) > SAAP_WS_HEADER_BYTES) return SAAP_UNSUPPORTED;
  if (ws_bytes < attn_workspace_bytes(units, G)) return SAAP_WORKSPACE_TOO_SMALL;

  AttnParams p{};
  p.q = q; p.K = Ksorted; p.V = Vsorted; p.off = off; p.len = len; p.selected = selected;
  p.out = out; p.lse = lse;
  p.counters = reinterpret_cast<unsigned long long*>(ws);
  p.cstride = units * 128 <= (long long)SAAP_WS_HEADER_BYTES ? 16 : 1;
  p.part_ml = reinterpret_cast<float*>(static_cast<char*>(ws) + SAAP_WS_HEADER_BYTES);
  p.part_o = p.part_ml + (size_t)units * kMaxP * G * 2;
  p.rows = Ncap; p.nsel = nprobe; p.resident = resident_run; p.nseg = nseg; p.B = B; p.n_units = (int)units;
  p.Hq = Hq; p.Hkv = Hkv; p.independent = indep && !masked ? 1 : 0; p.masked_lists = masked ? heads : 0;
  p.out_bf16 = out_dtype == SAAP_BF16;
  p.n_dense = 0; p.scale_log2 = scale * kLog2e; p.kscale = kscale; p.vscale = vscale;
  // expected keys per unit: balanced buckets, plus the paper's default window for the resident run
  const long long est = (long long)Ncap * (masked ? nseg : nprobe) / B + (resident_run >= 0 ? 2048 : 0);
  LaunchPlan lp = plan_launch((int)units, est, Ncap, G, nseg, true, B, nseg > 0, key_bytes(dtype), masked);
  p.P = lp.P;
  p.stage = lp.stage;
  p.max_chunks = lp.max_chunks;
  p.use_table = (est + (long long)lp.P * (lp.threads / 16 * (G == 8 ? 2 : 4)) - 1) / ((long long)lp.P * (lp.threads / 16 * (G == 8 ? 2 : 4))) > 2;
  if (masked) return launch_masked(p, lp, G, dtype, static_cast<hipStream_t>(stream));
  return launch_attn<true>(p, lp, G, dtype, static_cast<hipStream_t>(stream));
}

extern "C" int32_t saap_sparse_decode_attention(const void* q, const void* Ksorted, const void* Vsorted,
                                                const int32_t* off, const int32_t* len,
                                                const int32_t* selected, int32_t nprobe, int32_t mode,
                                                float scale, void* out, int32_t out_dtype, float* lse,
                                                int32_t S, int32_t Hq, int32_t Hkv, int32_t Ncap, int32_t B,
                                                int32_t d, int32_t dtype, void* ws, size_t ws_bytes,
                                                void* stream) {
  begin_call();
  return sparse_attention(q, Ksorted, Vsorted, nullptr, nullptr, off, len, selected, nprobe, mode, -1, scale, out,
                          out_dtype, lse, S, Hq, Hkv, Ncap, B, d, dtype, ws, ws_bytes, stream);
}

extern "C" int32_t saap_windowed_decode_attention(const void* q, const void* Ksorted, const void* Vsorted,
                                                  const int32_t* off, const int32_t* len,
                                                  const int32_t* selected, int32_t nprobe, int32_t mode,
                                                  int32_t resident_run, float scale, void* out,
                                                  int32_t out_dtype, float* lse, int32_t S, int32_t Hq,
                                                  int32_t Hkv, int32_t Ncap, int32_t runs, int32_t d,
                                                  int32_t dtype, void* ws, size_t ws_bytes, void* stream) {
  begin_call();
  return sparse_attention(q, Ksorted, Vsorted, nullptr, nullptr, off, len, selected, nprobe, mode, resident_run, scale,
                          out, out_dtype, lse, S, Hq, Hkv, Ncap, runs, d, dtype, ws, ws_bytes, stream);
}

static int32_t dense_attention(const void* q, const void* K, const void* V, const float* kscale, const float* vscale,
                               const int32_t* off, const int32_t* len, int32_t B, float scale, void* out,
                               int32_t out_dtype, float* lse, int32_t S, int32_t Hq, int32_t Hkv, int32_t N, int32_t d,
                               int32_t dtype, void* ws, size_t ws_bytes, void* stream) {
  int32_t st = check_common(q, K, V, out, S, Hq, Hkv, d, dtype, out_dtype, ws);
  if (st == SAAP_OK && dtype == kDtypeFp8 && (!kscale || !vscale)) st = SAAP_INVALID_ARG;
  if (st != SAAP_OK) return st;
  if (N <= 0) return SAAP_INVALID_ARG;
  if ((off == nullptr) != (len == nullptr)) return SAAP_INVALID_ARG;
  if (off && (B <= 0 || B > SAAP_MAX_BUCKETS)) return B <= 0 ? SAAP_INVALID_ARG : SAAP_UNSUPPORTED;
  const int G = Hq / Hkv;
  const long long units = (long long)S * Hkv;
  if (units * sizeof(unsigned long long) > SAAP_WS_HEADER_BYTES) return SAAP_UNSUPPORTED;
  if (ws_bytes < attn_workspace_bytes(units, G)) return SAAP_WORKSPACE_TOO_SMALL;

  AttnParams p{};
  p.q = q; p.K = K; p.V = V; p.off = off; p.len = len; p.selected = nullptr;
  p.out = out; p.lse = lse;
  p.counters = reinterpret_cast<unsigned long long*>(ws);
  p.cstride = units * 128 <= (long long)SAAP_WS_HEADER_BYTES ? 16 : 1;
  p.part_ml = reinterpret_cast<float*>(static_cast<char*>(ws) + SAAP_WS_HEADER_BYTES);
  p.part_o = p.part_ml + (size_t)units * kMaxP * G * 2;
  p.rows = N; p.nseg = off ? B : 0; p.nsel = p.nseg; p.resident = -1; p.B = B; p.n_units = (int)units;
  p.Hq = Hq; p.Hkv = Hkv; p.independent = 0; p.out_bf16 = out_dtype == SAAP_BF16;
  p.n_dense = N; p.scale_log2 = scale * kLog2e; p.kscale = kscale; p.vscale = vscale;
  LaunchPlan lp = plan_launch((int)units, N, N, G, p.nseg, off != nullptr, B, false, key_bytes(dtype));
  p.P = lp.P;
  p.stage = 0;
  p.max_chunks = lp.max_chunks;
  p.use_table = 1;
  hipStream_t hs = static_cast<hipStream_t>(stream);
  return off ? launch_attn<true>(p, lp, G, dtype, hs) : launch_attn<false>(p, lp, G, dtype, hs);
}

extern "C" int32_t saap_dense_decode_attention(const void* q, const void* K, const void* V,
                                               const int32_t* off, const int32_t* len, int32_t B,
                                               float scale, void* out, int32_t out_dtype, float* lse,
                                               int32_t S, int32_t Hq, int32_t Hkv, int32_t N, int32_t d,
                                               int32_t dtype, void* ws, size_t ws_bytes, void* stream) {
  begin_call();
  if (dtype != SAAP_F32 && dtype != SAAP_BF16) return SAAP_INVALID_ARG;
  return dense_attention(q, K, V, nullptr, nullptr, off, len, B, scale, out, out_dtype, lse, S, Hq, Hkv, N, d, dtype,
                         ws, ws_bytes, stream);
}

extern "C" int32_t saap_sparse_decode_attention_fp8(const void* q, const uint8_t* K8, const uint8_t* V8,
                                                    const float* kscale, const float* vscale,
                                                    const int32_t* off, const int32_t* len,
                                                    const int32_t* selected, int32_t nprobe, int32_t mode,
                                                    float scale, void* out, int32_t out_dtype, float* lse,
                                                    int32_t S, int32_t Hq, int32_t Hkv, int32_t Ncap, int32_t B,
                                                    int32_t d, void* ws, size_t ws_bytes, void* stream) {
  begin_call();
  if (!kscale || !vscale) return SAAP_INVALID_ARG;
  return sparse_attention(q, K8, V8, kscale, vscale, off, len, selected, nprobe, mode, -1, scale, out, out_dtype, lse,
                          S, Hq, Hkv, Ncap, B, d, kDtypeFp8, ws, ws_bytes, stream);
}

extern "C" int32_t saap_windowed_decode_attention_fp8(const void* q, const uint8_t* K8, const uint8_t* V8,
                                                      const float* kscale, const float* vscale,
                                                      const int32_t* off, const int32_t* len,
                                                      const int32_t* selected, int32_t nprobe, int32_t mode,
                                                      int32_t resident_run, float scale, void* out,
                                                      int32_t out_dtype, float* lse, int32_t S, int32_t Hq,
                                                      int32_t Hkv, int32_t Ncap, int32_t runs, int32_t d, void* ws,
                                                      size_t ws_bytes, void* stream) {
  begin_call();
  if (!kscale || !vscale) return SAAP_INVALID_ARG;
  return sparse_attention(q, K8, V8, kscale, vscale, off, len, selected, nprobe, mode, resident_run, scale, out,
                          out_dtype, lse, S, Hq, Hkv, Ncap, runs, d, kDtypeFp8, ws, ws_bytes, stream);
}

extern "C" int32_t saap_dense_decode_attention_fp8(const void* q, const uint8_t* K8, const uint8_t* V8,
                                                   const float* kscale, const float* vscale,
                                                   const int32_t* off, const int32_t* len, int32_t B,
                                                   float scale, void* out, int32_t out_dtype, float* lse,
                                                   int32_t S, int32_t Hq, int32_t Hkv, int32_t N, int32_t d,
                                                   void* ws, size_t ws_bytes, void* stream) {
  begin_call();
  if (!kscale || !vscale) return SAAP_INVALID_ARG;
  return dense_attention(q, K8, V8, kscale, vscale, off, len, B, scale, out, out_dtype, lse, S, Hq, Hkv, N, d,
                         kDtypeFp8, ws, ws_bytes, stream);
}

// ---- selection and attention in one launch -------------------------------------------------------------
namespace saap {
namespace {
template <typename T, int G>
int32_t launch_selecting(const AttnParams& p, const LaunchPlan& lp, int ept, hipStream_t stream) {
  switch (ept) {
    case 2: return launch_nt<T, G, true, 512, false, 2>(p, lp, stream);
    case 4: return launch_nt<T, G, true, 512, false, 4>(p, lp, stream);
    default: return launch_nt<T, G, true, 512, false, 8>(p, lp, stream);
  }
}
}  // namespace
}  // namespace saap

// Shapes the selecting kernels take: group lists, 1024-4096 buckets handled by 512 threads, a list short enough
// for the radix selection, bf16 or 8-bit cache.  Anything else runs as the two calls.
static int32_t select_attend(const float* logits, const void* q, const void* Ksorted, const void* Vsorted,
                             const float* kscale, const float* vscale, const int32_t* off, const int32_t* len,
                             int32_t nprobe, int32_t resident_run, float scale, int32_t* selected, void* out,
                             int32_t out_dtype, float* lse, int32_t S, int32_t Hq, int32_t Hkv, int32_t Ncap, int32_t B,
                             int32_t d, int32_t dtype, void* ws, size_t ws_bytes, void* stream) {
  // B: buckets (columns of the logits); the index has one run more when a resident run is visited (its number is B)
  int32_t st = check_common(q, Ksorted, Vsorted, out, S, Hq, Hkv, d, dtype, out_dtype, ws);
  if (st != SAAP_OK) return st;
  if (!logits || !aligned16(logits) || !off || !len || B <= 0 || Ncap <= 0 || nprobe < 0 || nprobe > B) return SAAP_INVALID_ARG;
  if (resident_run != -1 && resident_run != B) return SAAP_INVALID_ARG;
  const int runs = B + (resident_run >= 0 ? 1 : 0);
  const int nseg = nprobe + (resident_run >= 0 ? 1 : 0);
  if (nprobe > 0 && (!selected || !aligned16(selected))) return SAAP_INVALID_ARG;
  if (dtype == kDtypeFp8 && (!kscale || !vscale)) return SAAP_INVALID_ARG;
  const int G = Hq / Hkv;
  const long long units = (long long)S * Hkv;
  int n_pow2 = 2, n_sort = 2;
  while (n_pow2 < B) n_pow2 <<= 1;
  while (n_sort < nprobe) n_sort <<= 1;
  const int ept = B <= 1024 ? 2 : B <= 2048 ? 4 : 8;
  const SelectGeometry geo = select_geometry(B, nprobe, true, runs);
  // a workgroup has 64 KB of LDS: the selection's area and the run tables behind it must fit with room for the
  // kernels' static arrays
  const bool lds_fits = ((geo.lds + 15) & ~(size_t)15) + (size_t)(2 * nseg + 2) * sizeof(int) <= 48 * 1024;
  const bool one_launch = nprobe > 0 && (dtype == SAAP_BF16 || dtype == kDtypeFp8) && B >= 64 && B <= 4096 && n_sort < n_pow2 &&
                          lds_fits && units * sizeof(unsigned long long) <= SAAP_WS_HEADER_BYTES &&
                          env_int("SAAP_SELECT_ATTEND_FUSED", 1) != 0;
  auto two_calls = [&]() -> int32_t {
    const int32_t s1 = saap_select_buckets_from_logits(logits, nullptr, selected, S, Hq, Hkv, B, nprobe, SAAP_GROUP_SUM, nullptr, 0, stream);
    if (s1 != SAAP_OK) return s1;
    return sparse_attention(q, Ksorted, Vsorted, kscale, vscale, off, len, selected, nprobe, SAAP_GROUP_SUM, resident_run,
                            scale, out, out_dtype, lse, S, Hq, Hkv, Ncap, runs, d, dtype, ws, ws_bytes, stream);
  };
  if (!one_launch) return two_calls();
  if (ws_bytes < attn_workspace_bytes(units, G)) return SAAP_WORKSPACE_TOO_SMALL;
  AttnParams p{};
  p.q = q; p.K = Ksorted; p.V = Vsorted; p.off = off; p.len = len; p.selected = nullptr;
  p.logits = logits; p.selected_out = selected;
  p.out = out; p.lse = lse;
  p.counters = reinterpret_cast<unsigned long long*>(ws);
  p.cstride = units * 128 <= (long long)SAAP_WS_HEADER_BYTES ? 16 : 1;
  p.part_ml = reinterpret_cast<float*>(static_cast<char*>(ws) + SAAP_WS_HEADER_BYTES);
  p.part_o = p.part_ml + (size_t)units * kMaxP * G * 2;
  p.rows = Ncap; p.nsel = nprobe; p.resident = resident_run; p.nseg = nseg; p.B = runs; p.sel_B = B; p.n_units = (int)units;
  p.Hq = Hq; p.Hkv = Hkv; p.independent = 0; p.masked_lists = 0;
  p.out_bf16 = out_dtype == SAAP_BF16;
  p.n_dense = 0; p.scale_log2 = scale * kLog2e; p.kscale = kscale; p.vscale = vscale;
  // expected keys per unit as in sparse_attention: balanced buckets, plus the paper's default window for the resident run
  const long long est = (long long)Ncap * nprobe / runs + (resident_run >= 0 ? 2048 : 0);
  LaunchPlan lp = plan_launch((int)units, est, Ncap, G, nseg, true, runs, true, key_bytes(dtype));
  if (lp.threads != 512) return two_calls();               // only a tuning override asks for another shape
  p.P = lp.P;
  p.stage = 0;
  p.max_chunks = lp.max_chunks;
  p.use_table = (est + (long long)lp.P * (lp.threads / 16 * (G == 8 ? 2 : 4)) - 1) / ((long long)lp.P * (lp.threads / 16 * (G == 8 ? 2 : 4))) > 2;
  p.sel_n_sort = geo.n_sort;
  p.sel_cap = geo.cap;
  p.sel_plan_off = geo.plan_off;
  p.sel_lds = (unsigned)((geo.lds + 15) & ~(size_t)15);
  // selection area, then the plan row (total, pre, rowoff) and the per-chunk tables; the combination and merge
  // scratch of plan_launch overlays them later
  const size_t need = (size_t)p.sel_lds + (size_t)(2 * nseg + 2 + 2 * lp.max_chunks) * sizeof(int);
  if (need > 60 * 1024) return two_calls();                // very long units on few workgroups: the chunk tables alone fill the LDS
  if (need > lp.lds) lp.lds = need;
  hipStream_t hs = static_cast<hipStream_t>(stream);
#define SAAP_CASE(TT, GG) return launch_selecting<TT, GG>(p, lp, ept, hs)
  if (dtype == kDtypeFp8) {
    switch (G) {
      case 1: SAAP_CASE(fp8_t, 1);
      case 2: SAAP_CASE(fp8_t, 2);
      case 4: SAAP_CASE(fp8_t, 4);
      case 8: SAAP_CASE(fp8_t, 8);
    }
  } else {
    switch (G) {
      case 1: SAAP_CASE(bf16_t, 1);
      case 2: SAAP_CASE(bf16_t, 2);
      case 4: SAAP_CASE(bf16_t, 4);
      case 8: SAAP_CASE(bf16_t, 8);
    }
  }
#undef SAAP_CASE
  return SAAP_UNSUPPORTED;
}

extern "C" int32_t saap_select_attend(const float* logits, const void* q, const void* Ksorted, const void* Vsorted,
                                      const int32_t* off, const int32_t* len, int32_t nprobe, float scale,
                                      int32_t* selected, void* out, int32_t out_dtype, float* lse, int32_t S,
                                      int32_t Hq, int32_t Hkv, int32_t Ncap, int32_t B, int32_t d, int32_t dtype,
                                      void* ws, size_t ws_bytes, void* stream) {
  begin_call();
  if (dtype != SAAP_BF16 && dtype != SAAP_F32) return SAAP_UNSUPPORTED;
  return select_attend(logits, q, Ksorted, Vsorted, nullptr, nullptr, off, len, nprobe, -1, scale, selected, out, out_dtype,
                       lse, S, Hq, Hkv, Ncap, B, d, dtype, ws, ws_bytes, stream);
}

extern "C" int32_t saap_select_attend_windowed(const float* logits, const void* q, const void* Ksorted,
                                               const void* Vsorted, const int32_t* off, const int32_t* len,
                                               int32_t nprobe, int32_t resident_run, float scale, int32_t* selected,
                                               void* out, int32_t out_dtype, float* lse, int32_t S, int32_t Hq,
                                               int32_t Hkv, int32_t Ncap, int32_t B, int32_t d, int32_t dtype, void* ws,
                                               size_t ws_bytes, void* stream) {
  begin_call();
  if (dtype != SAAP_BF16 && dtype != SAAP_F32) return SAAP_UNSUPPORTED;
  return select_attend(logits, q, Ksorted, Vsorted, nullptr, nullptr, off, len, nprobe, resident_run, scale, selected, out,
                       out_dtype, lse, S, Hq, Hkv, Ncap, B, d, dtype, ws, ws_bytes, stream);
}

extern "C" int32_t saap_select_attend_fp8(const float* logits, const void* q, const uint8_t* K8, const uint8_t* V8,
                                          const float* kscale, const float* vscale, const int32_t* off,
                                          const int32_t* len, int32_t nprobe, float scale, int32_t* selected,
                                          void* out, int32_t out_dtype, float* lse, int32_t S, int32_t Hq,
                                          int32_t Hkv, int32_t Ncap, int32_t B, int32_t d, void* ws, size_t ws_bytes,
                                          void* stream) {
  begin_call();
  return select_attend(logits, q, K8, V8, kscale, vscale, off, len, nprobe, -1, scale, selected, out, out_dtype, lse, S, Hq,
                       Hkv, Ncap, B, d, kDtypeFp8, ws, ws_bytes, stream);
}

// ---- attention for callers that cannot allocate ---------------------------------------------------
// The workspace of this entry point is a device array that is part of the library's image: every GPU
// the library runs on holds SAAP_STATIC_SCRATCH_BYTES of it from the first call until the process ends.
namespace {
static __device__ __align__(256) unsigned char scratch[SAAP_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices];   // per device: that device's copy of `scratch` (the array's name is no device address)

// Address of the current device's copy of `scratch`; looked up once per device, with that device current.
int32_t static_scratch(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return SAAP_HIP_ERROR;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return SAAP_HIP_ERROR;
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return SAAP_OK;
}
}  // namespace

extern "C" int32_t saap_sparse_decode_attention_noalloc(const void* q, const void* Ksorted, const void* Vsorted,
                                                        const int32_t* off, const int32_t* len,
                                                        const int32_t* selected, int32_t nprobe, int32_t mode,
                                                        float scale, void* out, int32_t out_dtype, float* lse,
                                                        int32_t S, int32_t Hq, int32_t Hkv, int32_t Ncap, int32_t B,
                                                        int32_t d, int32_t dtype, void* stream) {
  begin_call();
  if (dtype != SAAP_F32 && dtype != SAAP_BF16) return SAAP_INVALID_ARG;
  // every argument is checked before the device is touched (the scratch is the one pointer that is not the caller's)
  int32_t st = check_common(q, Ksorted, Vsorted, out, S, Hq, Hkv, d, dtype, out_dtype, /*ws=*/q);
  if (st != SAAP_OK) return st;
  st = check_lists(off, len, selected, nprobe, mode, -1, Ncap, B);
  if (st != SAAP_OK) return st;
  // the shape decides the scratch it needs; more than the array holds is refused before anything is enqueued
  const int heads = Hq / Hkv;
  const bool indep = mode == SAAP_INDEPENDENT;
  const bool masked = indep && heads > 1 && B <= 16 * 512;
  const long long units = indep && !masked ? (long long)S * Hq : (long long)S * Hkv;
  const int G = masked ? heads : indep ? 1 : heads;
  if (units * 128 > (long long)SAAP_WS_HEADER_BYTES || attn_workspace_bytes(units, G) > (size_t)SAAP_STATIC_SCRATCH_BYTES)
    return SAAP_WORKSPACE_TOO_SMALL;
  void* ws = nullptr;
  st = static_scratch(&ws);
  if (st != SAAP_OK) return st;
  // The array keeps what the last call left.  Its arrival counters must be zero when the kernel starts: a
  // fill kernel clears them on the caller's stream (a call that was abandoned midway may have left some set).
  st = saap_workspace_reset(ws, SAAP_STATIC_SCRATCH_BYTES, stream);
  if (st != SAAP_OK) return st;
  return sparse_attention(q, Ksorted, Vsorted, nullptr, nullptr, off, len, selected, nprobe, mode, -1, scale, out,
                          out_dtype, lse, S, Hq, Hkv, Ncap, B, d, dtype, ws, SAAP_STATIC_SCRATCH_BYTES, stream);
}

// ---- prefill-time sparse attention: per-token visit plans, then the planned attention ----------------
size_t saap::prefill_workspace_bytes(long long S, int Tq, int Hq, int Hkv, int nprobe) {
  const long long units = S * Tq * Hkv;
  return planned_workspace_bytes(units, Hq / Hkv) + (size_t)units * plan_stride(nprobe + 2) * sizeof(int32_t);
}

extern "C" int32_t saap_prefill_sparse_attention(const void* q, const void* K, const void* V, const void* Ksorted,
                                                 const void* Vsorted, const int32_t* off, const int32_t* len,
                                                 const int32_t* idx, const int32_t* selected, const int32_t* pos0,
                                                 int32_t nprobe, int32_t n_sink, int32_t n_recent, float scale,
                                                 void* out, int32_t out_dtype, float* lse, int32_t S, int32_t Hq,
                                                 int32_t Hkv, int32_t Tq, int32_t Nt, int32_t Ncap, int32_t B,
                                                 int32_t d, int32_t dtype, void* ws, size_t ws_bytes, void* stream) {
  begin_call();
  if (dtype != SAAP_F32 && dtype != SAAP_BF16) return SAAP_INVALID_ARG;
  int32_t st = check_common(q, Ksorted, Vsorted, out, S, Hq, Hkv, d, dtype, out_dtype, ws);
  if (st != SAAP_OK) return st;
  if (!K || !V || !off || !len || !idx || !pos0 || (nprobe > 0 && !selected) || !aligned16(K) || !aligned16(V))
    return SAAP_INVALID_ARG;
  if (Tq <= 0 || Nt <= 0 || Ncap <= 0 || B <= 0 || nprobe < 0 || nprobe > B || n_sink < 0 || n_recent < 0)
    return SAAP_INVALID_ARG;
  if (nprobe + 2 > SAAP_MAX_BUCKETS) return SAAP_UNSUPPORTED;
  const long long units = (long long)S * Tq * Hkv;
  if (units > kPlanMaxUnits) return SAAP_UNSUPPORTED;
  if (ws_bytes < prefill_workspace_bytes(S, Tq, Hq, Hkv, nprobe)) return SAAP_WORKSPACE_TOO_SMALL;
  const int ps = plan_stride(nprobe + 2);
  const size_t att_bytes = planned_workspace_bytes(units, Hq / Hkv);
  int32_t* plan = reinterpret_cast<int32_t*>(static_cast<char*>(ws) + att_bytes);
  hipLaunchKernelGGL(prefill_plan_kernel, dim3((unsigned)units), dim3(256), 0, static_cast<hipStream_t>(stream), selected,
                     off, len, idx, pos0, plan, nprobe, n_sink, n_recent, B, Ncap, Nt, Tq, Hkv, ps);
  st = launch_status();
  if (st != SAAP_OK) return st;
  return planned_attention(q, Ksorted, Vsorted, nullptr, nullptr, plan, nprobe + 2, SAAP_GROUP_SUM, scale, out, out_dtype,
                           lse, S * Tq, Hq, Hkv, Ncap, d, dtype, ws, att_bytes, stream, K, V, Nt, Tq);
}
