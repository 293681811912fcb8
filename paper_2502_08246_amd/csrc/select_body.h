// The selection of one bucket list by one workgroup, shared by the selection kernels (select.hip) and by the
// classifier's output kernel, whose last workgroup per list can run it in the same launch (classify.hip).
// Section 4 and Section 5 ("Batched queries") of arXiv 2502.08246: the classifier outputs of the G heads that share
// a KV head are summed and the nprobe best buckets taken, ordered by (score descending, id ascending).
#pragma once

#include "common.h"

namespace saap {
namespace {


constexpr int kRankSortMax = 1024;   // selected lists up to this length are ordered by counting larger keys
constexpr int kBucketRankMin = 384;  // ... candidate lists longer than this by bucketing first (measured break-even)

// Words of the tie bitmap in LDS: one bit per bucket, at least 256 words (the region doubles as the
// bucket offsets of the bucketed ranking) and an even count (what follows holds 8-byte entries).
__host__ __device__ constexpr int bitmap_words(int B) {
  const int w = B / 32 + 1 < 256 ? 256 : B / 32 + 1;
  return (w + 1) & ~1;
}

// Sum of the heads' scores of bucket b, in fp32 in head order.  All loads go out before the
// first add (heads <= 8).
__device__ __forceinline__ float group_score(const float* sc, int heads, int B, int b) {
  float v[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) v[i] = i < heads ? sc[(size_t)i * B + b] : 0.f;
  float g = v[0];
#pragma unroll
  for (int i = 1; i < 8; ++i)
    if (i < heads) g = g + v[i];
  return g + 0.0f;                                                // -0 -> +0
}

// What the selection hands to the attention besides the ids: the visit plan of the list (total keys,
// exclusive prefix of the run lengths, first rows; layout in saap.h).  `sel` holds the nsel ordered ids,
// `lens` / `offs` the lengths and first rows of the unit's runs; the always-visited run, if any, comes
// last.  Called by the whole workgroup after a barrier that made `sel` visible.
struct PlanOut {
  const int32_t* off;   // [kv units, runs+1] or null: no plan wanted
  const int32_t* len;   // [kv units, runs]
  int32_t* plan;        // [units, ps]
  int runs, resident, ps;
  unsigned lds_off;     // byte offset of the plan staging area in dynamic LDS: len [runs] | off [runs] | sel [nprobe]
};

__device__ __forceinline__ void emit_plan(const int* sel, const int* lens, const int* offs, int nsel, int resident,
                                          int32_t* pl) {
  __shared__ int s_psum[16];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, nt = blockDim.x, nw = nt >> 6;
  const int nseg = nsel + (resident >= 0 ? 1 : 0);
  if (nseg <= 64) {
    // one wave holds the whole list: its prefix sum needs no exchange between waves
    if (wave == 0) {
      const int b = lane < nseg ? (lane < nsel ? sel[lane] : resident) : 0;
      const int mine = lane < nseg ? max(lens[b], 0) : 0;
      const int incl = (int)wave_prefix_sum((unsigned)mine);
      if (lane < nseg) {
        pl[2 + lane] = incl;
        pl[nseg + 2 + lane] = offs[b];
      }
      if (lane == 63) {
        pl[0] = incl;
        pl[1] = 0;
      }
    }
    return;
  }
  const int per = (nseg + nt - 1) / nt;
  const int j0 = tid * per, j1 = min(j0 + per, nseg);
  int mine = 0;
  for (int j = j0; j < j1; ++j) mine += max(lens[j < nsel ? sel[j] : resident], 0);
  const int incl = (int)wave_prefix_sum((unsigned)mine);
  if (lane == 63) s_psum[wave] = incl;
  __syncthreads();
  int run = incl - mine, total = 0;
  for (int x = 0; x < nw; ++x) {
    if (x < wave) run += s_psum[x];
    total += s_psum[x];
  }
  for (int j = j0; j < j1; ++j) {
    const int b = j < nsel ? sel[j] : resident;
    run += max(lens[b], 0);
    pl[2 + j] = run;
    pl[nseg + 2 + j] = offs[b];
  }
  if (tid == 0) {
    pl[0] = total;
    pl[1] = 0;
  }
}

__device__ __forceinline__ float wave_max_f32(float x) {
  x = fmaxf(x, dpp_mov<kDppXor1>(x));
  x = fmaxf(x, dpp_mov<kDppXor2>(x));
  x = fmaxf(x, dpp_mov<kDppHalfMirror>(x));
  x = fmaxf(x, dpp_mov<kDppMirror>(x));
  return max_rows(x);
}
__device__ __forceinline__ float wave_sum_f32(float x) { return sum_rows(sum16(x)); }

// Softmax of the list's HEADS rows of logits, held EPT per thread, and their sum over the heads:
// p = exp(z - max z) / sum exp(z - max z) per row in fp32, g = ((p_0 + p_1) + p_2) + ... in head
// order.  The probabilities are also written to `p_rows` if it is not null, so that what was
// selected from can be checked.  Called by the whole workgroup.
// COHERENT: the logits were written by other workgroups of the SAME launch (write-through stores): they are read with
// agent-scope loads, past this XCD's L2.
template <int EPT, int HEADS, bool COHERENT>
__device__ __forceinline__ void softmax_group_scores(const float* __restrict__ z_rows, float* __restrict__ p_rows,
                                                     int B, float* gs) {
  __shared__ float s_red[2][16][HEADS];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, nt = blockDim.x, nw = nt >> 6;
  float z[EPT][HEADS];
  // every load is unconditional (clamped index) so that all of them are in flight together;
  // what lies outside the row becomes -inf afterwards
#pragma unroll
  for (int e = 0; e < EPT; ++e) {
    const int b = min(tid + e * nt, B - 1);
#pragma unroll
    for (int i = 0; i < HEADS; ++i) {
      if constexpr (COHERENT) z[e][i] = __hip_atomic_load(&z_rows[(size_t)i * B + b], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      else z[e][i] = z_rows[(size_t)i * B + b];
    }
  }
  float red[HEADS];
#pragma unroll
  for (int i = 0; i < HEADS; ++i) {
    float m = -INFINITY;
#pragma unroll
    for (int e = 0; e < EPT; ++e) {
      if (tid + e * nt >= B) z[e][i] = -INFINITY;
      m = fmaxf(m, z[e][i]);
    }
    red[i] = wave_max_f32(m);
  }
  if (lane == 0) {
#pragma unroll
    for (int i = 0; i < HEADS; ++i) s_red[0][wave][i] = red[i];
  }
  __syncthreads();
#pragma unroll
  for (int i = 0; i < HEADS; ++i) {
    // the waves' partial results, one per lane, reduced again inside every wave
    const float m = wave_max_f32(lane < nw ? s_red[0][lane][i] : -INFINITY);
    float sum = 0.f;
#pragma unroll
    for (int e = 0; e < EPT; ++e) {
      z[e][i] = __expf(z[e][i] - m);      // exp(-inf) = 0 for the padding
      sum += z[e][i];
    }
    red[i] = wave_sum_f32(sum);
  }
  if (lane == 0) {
#pragma unroll
    for (int i = 0; i < HEADS; ++i) s_red[1][wave][i] = red[i];
  }
  __syncthreads();
#pragma unroll
  for (int i = 0; i < HEADS; ++i) {
    red[i] = 1.0f / wave_sum_f32(lane < nw ? s_red[1][lane][i] : 0.f);
  }
#pragma unroll
  for (int e = 0; e < EPT; ++e) {
    const int b = tid + e * nt;
    float g = 0.f;
#pragma unroll
    for (int i = 0; i < HEADS; ++i) {
      const float pr = z[e][i] * red[i];
      if (p_rows && b < B) p_rows[(size_t)i * B + b] = pr;
      g = i == 0 ? pr : g + pr;
    }
    gs[e] = g + 0.0f;
  }
}

// The selection of one list by one workgroup (any number of threads nt with EPT * nt >= B): `smem` is the workgroup's
// dynamic LDS, laid out as select_geometry() says.  Called by every thread of the workgroup.
template <int EPT, bool LOGITS, bool COHERENT>
__device__ __forceinline__ void select_radix_body(unsigned char* smem, int unit, const float* __restrict__ scores,
                                                  float* __restrict__ probs, int32_t* __restrict__ selected, int Hq,
                                                  int Hkv, int B, int nprobe, int independent, int n_sort, int cap,
                                                  PlanOut po) {
  unsigned long long* sortbuf = reinterpret_cast<unsigned long long*>(smem);   // [cap] candidates, cap >= n_sort
  unsigned* eqbits = reinterpret_cast<unsigned*>(sortbuf + cap);               // [B/32 + 1]
  __shared__ unsigned s_hist[2][256];
  __shared__ unsigned s_digit, s_krem, s_bin, s_cnt, s_neq, s_and, s_or;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, nt = blockDim.x;
  const int G = Hq / Hkv;
  const int heads = independent ? 1 : G;
  const size_t row0 = independent ? (size_t)unit : (size_t)unit * G;
  const float* sc = scores + row0 * B;

  SAAP_TRACE(0);
  // visit plan: the unit's run lengths and first rows are fetched in the same memory round trip as the
  // scores and parked in LDS until the ordered list exists
  int* s_len = reinterpret_cast<int*>(smem + po.lds_off);       // [runs]
  int* s_off = s_len + po.runs;                                 // [runs]
  int* s_sel = s_off + po.runs;                                 // [nprobe]
  int lv[EPT + 1], ov[EPT + 1];
  if (po.off) {
    const int kvu = independent ? (unit / Hq) * Hkv + (unit % Hq) / G : unit;
    const int32_t* lenu = po.len + (size_t)kvu * po.runs;
    const int32_t* offu = po.off + (size_t)kvu * (po.runs + 1);
#pragma unroll
    for (int e = 0; e <= EPT; ++e) {
      const int b = min(tid + e * nt, po.runs - 1);
      lv[e] = lenu[b];
      ov[e] = offu[b];
    }
  }
  // the selection's counters and buffers start at zero; with logits the two barriers of the softmax below put
  // this ahead of their first use, otherwise a barrier of its own does
  if (tid == 0) { s_cnt = 0u; s_neq = 0u; s_and = 0xFFFFFFFFu; s_or = 0u; }
  for (int i = tid; i < cap; i += nt) sortbuf[i] = 0ull;
  for (int i = tid; i <= B / 32; i += nt) eqbits[i] = 0u;
  for (int i = tid; i < 256; i += nt) s_hist[0][i] = 0u;
  unsigned key[EPT];
  {
    float gs[EPT];
    if constexpr (LOGITS) {
      float* pr = probs ? probs + row0 * B : nullptr;
      switch (heads) {
        case 1: softmax_group_scores<EPT, 1, COHERENT>(sc, pr, B, gs); break;
        case 2: softmax_group_scores<EPT, 2, COHERENT>(sc, pr, B, gs); break;
        case 4: softmax_group_scores<EPT, 4, COHERENT>(sc, pr, B, gs); break;
        default: softmax_group_scores<EPT, 8, COHERENT>(sc, pr, B, gs); break;
      }
      SAAP_TRACE(5);
    } else {
#pragma unroll
      for (int e = 0; e < EPT; ++e) {
        const int b = tid + e * nt;
        gs[e] = group_score(sc, heads, B, b < B ? b : 0);
      }
    }
#pragma unroll
    for (int e = 0; e < EPT; ++e) key[e] = tid + e * nt < B ? float_order_key(gs[e]) : 0u;   // 0 sorts below every finite score
  }
  if (po.off) {
#pragma unroll
    for (int e = 0; e <= EPT; ++e) {
      const int b = tid + e * nt;
      if (b < po.runs) {
        s_len[b] = lv[e];
        s_off[b] = ov[e];
      }
    }
  }
  if constexpr (!LOGITS) __syncthreads();   // (the plan's staging area is read after several more barriers)

  // Bits shared by every score image need no pass (softmax outputs share most exponent bits,
  // which would otherwise pile all buckets into two or three histogram bins).
  {
    unsigned a = 0xFFFFFFFFu, o = 0u;
#pragma unroll
    for (int e = 0; e < EPT; ++e)
      if (tid + e * nt < B) { a &= key[e]; o |= key[e]; }
    a = wave_and(a);
    o = wave_or(o);
    if (lane == 0) { atomicAnd(&s_and, a); atomicOr(&s_or, o); }
  }
  __syncthreads();
  SAAP_TRACE(1);
  const unsigned diff = s_and ^ s_or;
  int rem = diff ? 32 - __clz(diff) : 0;                 // undetermined low bits
  unsigned mask = rem >= 32 ? 0u : ~((1u << rem) - 1u);
  unsigned prefix = s_and & mask, k_rem = (unsigned)nprobe;

  // most-significant-digit radix select: after all digits `prefix` is the score image of the
  // nprobe-th largest bucket and k_rem the number of buckets equal to it that are taken.  The
  // passes stop early once the buckets above the bin that holds the nprobe-th one, plus that
  // bin, fit the candidate buffer: ordering the candidates settles the rest (the usual case after
  // one or two digits).
  int pass = 0;
  bool early = false;
  while (rem > 0) {
    const int width = rem < 8 ? rem : 8;
    const int shift = rem - width;
    const unsigned dmask = (1u << width) - 1u;
    unsigned* hist = s_hist[pass & 1];
    unsigned* hist_next = s_hist[(pass + 1) & 1];
    for (int i = tid; i < 256; i += nt) hist_next[i] = 0u;
#pragma unroll
    for (int e = 0; e < EPT; ++e)
      if (tid + e * nt < B && (key[e] & mask) == prefix) atomicAdd(&hist[(key[e] >> shift) & dmask], 1u);
    __syncthreads();
    if (wave == 0) {
      // lane i looks at bins 255-4i .. 252-4i, so a prefix sum over the lanes counts the
      // buckets in higher bins
      const int top = 255 - 4 * lane;
      const unsigned c[4] = {hist[top], hist[top - 1], hist[top - 2], hist[top - 3]};
      const unsigned tot = c[0] + c[1] + c[2] + c[3];
      unsigned cum = wave_prefix_sum(tot) - tot;
#pragma unroll
      for (int b = 0; b < 4; ++b) {
        if (cum < k_rem && cum + c[b] >= k_rem) {
          s_digit = (unsigned)(top - b);
          s_krem = k_rem - cum;
          s_bin = c[b];
        }
        cum += c[b];
      }
    }
    __syncthreads();
    prefix |= s_digit << shift;
    mask |= dmask << shift;
    k_rem = s_krem;
    rem = shift;
    ++pass;
    if (rem > 0 && (unsigned)nprobe - k_rem + s_bin <= (unsigned)cap) {
      early = true;
      break;
    }
  }
  SAAP_TRACE(2);
  int n_cand = nprobe;                 // entries of sortbuf to put in order; the first nprobe are the result
  if (early) {
    // candidates: every bucket whose determined digits are at or above the threshold bin
    n_cand = (int)((unsigned)nprobe - k_rem + s_bin);
#pragma unroll
    for (int e = 0; e < EPT; ++e) {
      const int b = tid + e * nt;
      if (b < B && (key[e] & mask) >= prefix) {
        const unsigned long long takers = __ballot(1);
        unsigned base = 0u;
        if (lane == __ffsll((long long)takers) - 1) base = atomicAdd(&s_cnt, (unsigned)__popcll(takers));
        base = (unsigned)__builtin_amdgcn_readfirstlane((int)base);
        const unsigned pos = base + (unsigned)__popcll(takers & ((1ull << lane) - 1ull));
        sortbuf[pos] = ((unsigned long long)key[e] << 32) | (unsigned long long)(0xFFFFFFFFu - (unsigned)b);
      }
    }
    __syncthreads();
  } else {
    // buckets scoring exactly `prefix`: k_rem of them are taken, lowest ids first
#pragma unroll
    for (int e = 0; e < EPT; ++e) {
      const int b = tid + e * nt;
      if (b < B && key[e] == prefix) {
        atomicAdd(&s_neq, 1u);
        atomicOr(&eqbits[b >> 5], 1u << (b & 31));
      }
    }
    __syncthreads();
    const bool all_equal_taken = s_neq == k_rem;
#pragma unroll
    for (int e = 0; e < EPT; ++e) {
      const int b = tid + e * nt;
      if (b >= B) continue;
      bool take = key[e] > prefix;
      if (key[e] == prefix) {
        if (all_equal_taken) {
          take = true;
        } else {
          unsigned rank = __popc(eqbits[b >> 5] & ((1u << (b & 31)) - 1u));
          for (int w = 0; w < (b >> 5); ++w) rank += __popc(eqbits[w]);
          take = rank < k_rem;
        }
      }
      if (take) {
        // one LDS atomic per wave: the first taking lane reserves slots for all of them
        const unsigned long long takers = __ballot(1);
        unsigned base = 0u;
        if (lane == __ffsll((long long)takers) - 1) base = atomicAdd(&s_cnt, (unsigned)__popcll(takers));
        base = (unsigned)__builtin_amdgcn_readfirstlane((int)base);
        const unsigned pos = base + (unsigned)__popcll(takers & ((1ull << lane) - 1ull));
        sortbuf[pos] = ((unsigned long long)key[e] << 32) | (unsigned long long)(0xFFFFFFFFu - (unsigned)b);
      }
    }
    __syncthreads();
  }
  SAAP_TRACE(3);
  int32_t* out = selected ? selected + (size_t)unit * nprobe : nullptr;   // null: the list is wanted in LDS only
  auto put = [&](unsigned place, int32_t id) {
    if (out) out[place] = id;
    if (po.off) s_sel[place] = id;
  };
  auto finish = [&]() {
    if (!po.off) return;
    __syncthreads();
    emit_plan(s_sel, s_len, s_off, nprobe, po.resident, po.plan + (size_t)unit * po.ps);
  };
  if (n_sort <= kRankSortMax && n_cand > kBucketRankMin) {
    // Long candidate lists: counting every larger key costs n^2 comparisons on one compute unit.
    // Instead the candidates are dealt into 256 buckets by the leading bits of (score image - lowest
    // image), largest first; the place of a key is the number of keys in earlier buckets plus the
    // number of larger keys in its own bucket (a handful).
    unsigned long long* tmp = reinterpret_cast<unsigned long long*>(eqbits + bitmap_words(B) + cap);   // [cap]
    unsigned* cnt = s_hist[0];
    unsigned* fill = s_hist[1];
    if (tid == 0) { s_and = 0xFFFFFFFFu; s_or = 0u; }            // lowest / highest score image
    for (int i = tid; i < 256; i += nt) { cnt[i] = 0u; fill[i] = 0u; }
    __syncthreads();
    {
      unsigned lo = 0xFFFFFFFFu, hi = 0u;
      for (int i = tid; i < n_cand; i += nt) {
        const unsigned k32 = (unsigned)(sortbuf[i] >> 32);
        lo = min(lo, k32);
        hi = max(hi, k32);
      }
      if (lo <= hi) { atomicMin(&s_and, lo); atomicMax(&s_or, hi); }
    }
    __syncthreads();
    const unsigned lo32 = s_and, span = s_or - s_and;
    const int bshift = span < 256u ? 0 : (32 - __clz(span)) - 8;
    auto bucket_of = [&](unsigned long long key) { return 255 - (int)(((unsigned)(key >> 32) - lo32) >> bshift); };
    for (int i = tid; i < n_cand; i += nt) atomicAdd(&cnt[bucket_of(sortbuf[i])], 1u);
    __syncthreads();
    unsigned* bbase = eqbits;                                    // [256] first place of each bucket (the bitmap is dead)
    if (wave == 0) {
      const unsigned c[4] = {cnt[4 * lane], cnt[4 * lane + 1], cnt[4 * lane + 2], cnt[4 * lane + 3]};
      const unsigned tot = c[0] + c[1] + c[2] + c[3];
      unsigned cum = wave_prefix_sum(tot) - tot;
#pragma unroll
      for (int b = 0; b < 4; ++b) {
        bbase[4 * lane + b] = cum;
        cum += c[b];
      }
    }
    __syncthreads();
    for (int i = tid; i < n_cand; i += nt) {
      const unsigned long long cand = sortbuf[i];
      const int bk = bucket_of(cand);
      tmp[bbase[bk] + atomicAdd(&fill[bk], 1u)] = cand;
    }
    __syncthreads();
    for (int i = tid; i < n_cand; i += nt) {
      const unsigned long long mine = tmp[i];
      const int bk = bucket_of(mine);
      const unsigned first = bbase[bk], n = cnt[bk];
      unsigned place = first;
      for (unsigned j = first; j < first + n; ++j) place += tmp[j] > mine ? 1u : 0u;
      if (place < (unsigned)nprobe) put(place, (int32_t)(0xFFFFFFFFu - (unsigned)(mine & 0xFFFFFFFFull)));
    }
    SAAP_TRACE(4);
    finish();
    return;
  }
  if (n_sort <= kRankSortMax) {
    // keys are distinct: the place of a key is the number of larger keys.  The comparisons of one key are
    // split over `parts` neighbouring lanes (a power of two, so they share a wave): each counts the larger
    // keys in its slice, the counts are added up over those lanes, and the first of them places the key.
    if (tid == 0) SAAP_TRACE_VALUE(6, n_cand);
    int parts = 1;
    while (parts < 64 && 2 * parts * n_cand <= nt) parts *= 2;
    const int slice = (n_cand + parts - 1) / parts;
    const int items = n_cand * parts;
    for (int w0 = 0; w0 < items; w0 += nt) {             // uniform trip count: every lane takes part in the exchanges
      const int w = w0 + tid;
      const int i = w / parts, part = w % parts;
      const bool real = w < items;
      const int j0 = part * slice, j1 = real ? min(j0 + slice, n_cand) : j0;
      const unsigned long long mine = sortbuf[real ? i : 0];
      unsigned cnt = 0u;
#pragma unroll 8
      for (int j = j0; j < j1; ++j) cnt += sortbuf[j] > mine ? 1u : 0u;
      for (int o = 1; o < parts; o <<= 1) cnt += (unsigned)__shfl_xor((int)cnt, o);
      if (real && part == 0 && cnt < (unsigned)nprobe) put(cnt, (int32_t)(0xFFFFFFFFu - (unsigned)(mine & 0xFFFFFFFFull)));
    }
    SAAP_TRACE(4);
    finish();
    return;
  }
  for (int k = 2; k <= n_sort; k <<= 1) {
    for (int j = k >> 1; j > 0; j >>= 1) {
      for (int i = tid; i < n_sort; i += nt) {
        const int x = i ^ j;
        if (x > i) {
          const unsigned long long a = sortbuf[i], c = sortbuf[x];
          const bool descending = (i & k) == 0;
          if (descending ? (a < c) : (a > c)) {
            sortbuf[i] = c;
            sortbuf[x] = a;
          }
        }
      }
      __syncthreads();
    }
  }
  for (int j = tid; j < nprobe; j += nt) put((unsigned)j, (int32_t)(0xFFFFFFFFu - (unsigned)(sortbuf[j] & 0xFFFFFFFFull)));
  finish();
}


// Launch geometry of the radix selection for B buckets and lists of nprobe: padded list length, candidate
// buffer, bytes of dynamic LDS and where the visit plan's staging area begins in it.
struct SelectGeometry {
  int n_pow2, n_sort, cap;
  size_t lds;
  unsigned plan_off;
};
inline SelectGeometry select_geometry(int B, int nprobe, bool with_plan, int runs) {
  SelectGeometry g{};
  g.n_pow2 = 2;
  while (g.n_pow2 < B) g.n_pow2 <<= 1;
  g.n_sort = 2;
  while (g.n_sort < nprobe) g.n_sort <<= 1;
  // candidate buffer: the padded list plus some room (the counting that orders the candidates
  // grows with the square of their number, another radix pass costs less than that for long
  // lists), the padded list itself where a bitonic network does the ordering
  g.cap = g.n_sort <= kRankSortMax ? (g.n_sort <= 128 ? 2 * g.n_sort : g.n_sort + 128) : g.n_sort;
  // sortbuf [cap] | bitmap [B/32 + 1, padded to 256 words and to an even count] | spare words [cap] | bucketed copy [cap]
  g.lds = (size_t)g.cap * sizeof(unsigned long long) + (size_t)bitmap_words(B) * sizeof(unsigned) +
          (g.n_sort <= kRankSortMax ? (size_t)g.cap * (sizeof(unsigned) + sizeof(unsigned long long)) : 0);
  if (with_plan) {
    g.lds = (g.lds + 15) & ~(size_t)15;
    g.plan_off = (unsigned)g.lds;
    g.lds += (size_t)(2 * runs + nprobe) * sizeof(int);
  }
  return g;
}

}  // namespace
}  // namespace saap
