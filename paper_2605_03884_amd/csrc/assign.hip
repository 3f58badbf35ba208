// assign.hip — bit-width assignment from per-token scores (paper Sec. 3.3: the combined
// score S(t) decides b(t) under a memory budget), the planning of a card from the same scores
// (Sec. 4.2.1: bit-width vector, slots, header), and the histogram of a bits vector.
//
// Ranking rule: tokens ordered by (score descending, index ascending), scores compared in
// the IEEE total order.  The first cut[0] tokens get 16 bits, up to cut[1] 8 bits, up to
// cut[2] 4 bits, the rest 2.  No sort is needed: for each cut a 4-pass radix select over the
// 32-bit order keys finds the key of the token at that rank and how many tokens lie strictly
// before it; tokens whose key equals the cut key are then admitted by increasing index until
// the cut is full (a stable block-wide prefix count).  One workgroup of 1024 threads does the
// selection; thread i owns the consecutive tokens [i * per, (i + 1) * per).
//
// What this kernel costs is set by two things, neither of them memory: it runs once per launch,
// so every line of its code is fetched cold, and its sixteen waves share the issue slots of one
// compute unit.  Hence: a thread keeps its keys in registers, and the kernel is instantiated per
// number of keys per thread (1, 2, 4, ... 32, chosen from the token count), so that a launch
// touches only the code of its own size; the passes after the first are one rolled loop; the
// first pass's histogram is kept in 16 copies against same-word atomics (real scores share sign
// and exponent); later passes test a key against all three cut prefixes and skip the counting
// code for waves that hold no match; cuts whose prefixes still coincide share one histogram; a
// wave without ties needs three comparisons per key for the widths.  Beyond 32768 tokens an
// older form takes over that re-reads the scores (they stay in cache) instead of holding keys.
//
// Planning variant (PLAN): once the cut keys are known every thread knows the widths of its own
// tokens, so a block-wide prefix count of the classes gives the stable slots, order[] and the
// bits copy, and the header follows - scores to a planned card in one launch instead of three
// (allocator, classification, and the gaps between them).  The launch has several workgroups:
// each repeats the whole selection by itself (no workgroup talks to another) and then writes the
// tables of its own share of at most 2048 consecutive tokens.  A share's entries of order[] are
// four contiguous runs, one per class; they, the slots and the widths are put together in LDS and
// leave as whole lines.
#include "qkv_common.h"
#include "qkv_plan.h"

namespace qkv {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kThreads = 1024;
constexpr int kWaves = kThreads / kWaveSize;
constexpr int kCopies = 16;                  // of the first pass's histogram
constexpr uint32_t kRankedMax = 32768;       // tokens the ranked kernels take: at most 32 per thread
constexpr uint32_t kShareTokens = 2048;      // tokens whose tables one workgroup writes

// What the planning variant needs beyond the allocator's arguments.
struct PlanArgs {
  CardGeom g;                  // built on the host from the budget's class counts
  qkv_card_header_t header;    // as the host filled it (status 0)
  PadTable pads;
  uint8_t* card;
  uint32_t share_waves;        // workgroup b writes the tables of the tokens of waves [b * share_waves, (b + 1) * share_waves)
};

// Key that grows as the rank grows: smaller key = better score.  -0 ranks below +0.
__device__ inline uint32_t rank_key(float score) {
  const uint32_t x = __float_as_uint(score);
  const uint32_t up = (x & 0x80000000u) ? ~x : (x | 0x80000000u);   // ascending in the score
  return ~up;
}

__device__ inline uint32_t uniform(uint32_t v) { return (uint32_t)__builtin_amdgcn_readfirstlane((int)v); }

// Prefix over the waves of a workgroup.  tot[0 .. kWaves) are wave totals in LDS (written before the last
// barrier); the result holds, in lanes 0 .. 15 of every wave, the inclusive running sum.  One LDS read and
// four DPP steps: a loop of dependent LDS reads would cost a full LDS latency per wave.
__device__ inline uint32_t scan_wave_totals(const uint32_t* tot, uint32_t lane) {
  uint32_t v = tot[lane & (kWaves - 1u)];
  v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x111, 0xF, 0xF, true);    // row_shr:1
  v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x112, 0xF, 0xF, true);    // row_shr:2
  v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x114, 0xF, 0xF, true);    // row_shr:4
  v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x118, 0xF, 0xF, true);    // row_shr:8
  return v;
}
// Sum of the totals of waves [0, w) from that running sum; w must be the same in every lane.
__device__ inline uint32_t waves_below(uint32_t running, uint32_t w) {
  const uint32_t at = uniform(w);
  return at == 0u ? 0u : (uint32_t)__builtin_amdgcn_readlane((int)running, (int)(at - 1u));
}

// T <= KPT * 1024: thread tid owns the tokens [tid * KPT, tid * KPT + KPT) and keeps their keys in registers.
// PLAN: also write slot[], order[], the bits copy, header and pads of plan->card; `bits` may then be null.
template <int KPT, bool PLAN>
__device__ __forceinline__ void ranked_body(const float* __restrict__ scores, uint32_t T, uint32_t cut0, uint32_t cut1,
                                            uint32_t cut2, uint8_t* __restrict__ bits, bool aligned, const PlanArgs* plan) {
  __shared__ u32x4 wide4[256 * kCopies / 4];            // first pass: bucket d, copy c at word [d * 16 + c]; later the stage
  __shared__ uint32_t hist2[2][3][256];                 // two sets, so that one is cleared while the other is searched; later the stage of the widths
  __shared__ uint32_t sel_prefix[3];                    // key bits fixed so far
  __shared__ uint32_t sel_left[3];                      // rank still to descend inside the current bucket
  __shared__ uint32_t sel_same[3];                      // keys equal to the cut key
  __shared__ __attribute__((aligned(16))) uint32_t wave_tot[3][kWaves];
  __shared__ __attribute__((aligned(16))) uint32_t wave_cls[3][kWaves];
  uint32_t* wide = reinterpret_cast<uint32_t*>(wide4);
  const uint32_t tid = threadIdx.x;
  const uint32_t lane = tid & 63u, wave = tid >> 6;
  const uint32_t cut[3] = {cut0, cut1, cut2};
  // A cut equal to T has no token at that rank: every token lies before it, handled without a key.
  // Cuts do not decrease, so live[2] implies live[1] implies live[0].
  const bool live[3] = {cut0 < T, cut1 < T, cut2 < T};

  const uint32_t t0 = min(tid * (uint32_t)KPT, T);
  const uint32_t n_own = min(t0 + (uint32_t)KPT, T) - t0;
  uint32_t keys[KPT];
  if (KPT % 4 == 0 && aligned && n_own == (uint32_t)KPT) {          // 128-bit loads
#pragma unroll
    for (int i = 0; i < KPT; i += 4) {
      const float4 f = *reinterpret_cast<const float4*>(scores + t0 + i);
      keys[i] = rank_key(f.x); keys[i + 1] = rank_key(f.y); keys[i + 2] = rank_key(f.z); keys[i + 3] = rank_key(f.w);
    }
  } else {
#pragma unroll
    for (int i = 0; i < KPT; ++i) keys[i] = ((uint32_t)i < n_own) ? rank_key(scores[t0 + i]) : 0u;
  }

  // ---- pass 0: one histogram of the top byte, shared by the three cuts
  wide4[tid] = (u32x4)(0u);                             // 256 * 16 words = 1024 x 16 bytes
  __syncthreads();
#pragma unroll
  for (int i = 0; i < KPT; ++i)
    if ((uint32_t)i < n_own) atomicAdd(&wide[(keys[i] >> 24) * kCopies + (lane & (kCopies - 1u))], 1u);
  __syncthreads();
  if (tid < 256) {
    uint32_t s = 0;
#pragma unroll
    for (int i = 0; i < kCopies; ++i) s += wide[tid * kCopies + ((i + tid) & (kCopies - 1u))];
    hist2[0][0][tid] = s;
  } else if (tid < 4 * 256) {
    hist2[1][(tid >> 8) - 1u][tid & 255u] = 0;          // the set the next pass counts into
  }
  __syncthreads();
  if (wave < 3 && live[wave]) {
    uint32_t left = cut[wave], same;
    const uint32_t d = find_bucket(hist2[0][0], lane, left, same);
    if (lane == 0) { sel_prefix[wave] = d << 24; sel_left[wave] = left; }
  }
  __syncthreads();

  // ---- passes 1..3: per cut, only the keys inside its bucket so far.  Cuts whose prefixes are still the
  // same count the same keys: they share the histogram of the first of them (rep).
#pragma unroll 1
  for (int pass = 1; pass < 4; ++pass) {
    const uint32_t shift = 24u - 8u * (uint32_t)pass;
    const uint32_t pre0 = uniform(sel_prefix[0]), pre1 = uniform(sel_prefix[1]), pre2 = uniform(sel_prefix[2]);
    const uint32_t rep1 = (live[0] && pre1 == pre0) ? 0u : 1u;
    const uint32_t rep2 = (live[0] && pre2 == pre0) ? 0u : (live[1] && pre2 == pre1) ? 1u : 2u;
    const bool count0 = live[0], count1 = live[1] && rep1 == 1u, count2 = live[2] && rep2 == 2u;
    uint32_t (*hist)[256] = hist2[pass & 1];            // cleared during the previous search
    const uint32_t high_mask = 0xFFFFFFFFu << (shift + 8u);
#pragma unroll
    for (int i = 0; i < KPT; ++i) {
      const uint32_t key = keys[i];
      const bool own = (uint32_t)i < n_own;
      const bool h0 = own && count0 && ((key ^ pre0) & high_mask) == 0u;
      const bool h1 = own && count1 && ((key ^ pre1) & high_mask) == 0u;
      const bool h2 = own && count2 && ((key ^ pre2) & high_mask) == 0u;
      if (__builtin_amdgcn_ballot_w64(h0 || h1 || h2) != 0ull) {       // many waves hold no key of any bucket
        const uint32_t d = (key >> shift) & 255u;
        if (h0) atomicAdd(&hist[0][d], 1u);
        if (h1) atomicAdd(&hist[1][d], 1u);
        if (h2) atomicAdd(&hist[2][d], 1u);
      }
    }
    __syncthreads();
    if (wave < 3) {
      if (live[wave]) {
        const uint32_t from = wave == 0 ? 0u : wave == 1 ? rep1 : rep2;
        uint32_t left = sel_left[wave], same;
        const uint32_t d = find_bucket(hist[from], lane, left, same);
        if (lane == 0) { sel_prefix[wave] |= d << shift; sel_left[wave] = left; sel_same[wave] = same; }
      }
    } else if (wave < 15) {                             // meanwhile the other set is cleared for the next pass
      const uint32_t i = tid - 3u * kWaveSize;          // 0 .. 767
      hist2[(pass & 1) ^ 1][i >> 8][i & 255u] = 0;
    }
    __syncthreads();
  }

  // Now sel_prefix[c] is the key at rank cut[c], sel_same[c] the number of tokens with exactly that key and
  // sel_left[c] how many of those still belong before the cut.
  uint32_t keyc[3], quota[3];
  bool unique = true;               // every cut key occurs once: then it is the cut token's own, and no tie rule is needed
#pragma unroll
  for (int c = 0; c < 3; ++c) {
    keyc[c] = uniform(sel_prefix[c]); quota[c] = uniform(sel_left[c]);
    unique = unique && (!live[c] || uniform(sel_same[c]) == 1u);
  }
  uint32_t run[3] = {0, 0, 0};
  bool no_ties = true;
  if (!unique) {
    uint32_t eq[3] = {0, 0, 0};
#pragma unroll
    for (int i = 0; i < KPT; ++i) {
#pragma unroll
      for (int c = 0; c < 3; ++c) eq[c] += ((uint32_t)i < n_own && live[c] && keys[i] == keyc[c]);
    }
#pragma unroll
    for (int c = 0; c < 3; ++c) {
      const uint32_t inc = wave_inclusive_scan(eq[c]);
      run[c] = inc - eq[c];
      if (lane == 63) wave_tot[c][wave] = inc;
    }
    __syncthreads();
#pragma unroll
    for (int c = 0; c < 3; ++c) run[c] += waves_below(scan_wave_totals(wave_tot[c], lane), wave);
    // A wave none of whose keys equals a cut key needs no tie rule either.
    no_ties = __builtin_amdgcn_ballot_w64((eq[0] | eq[1] | eq[2]) != 0u) == 0ull;
  }
  // Class of a key: how many of the three cuts it lies before (0..3 for 2, 4, 8, 16 bits).  The cut keys do not
  // decrease and a token admitted at one cut is admitted at the later ones, so the three answers just add up.
  auto class_of_key = [&](uint32_t key) -> uint32_t {
    uint32_t c = 0;
    if (no_ties) {                  // three comparisons per key
#pragma unroll
      for (int k = 0; k < 3; ++k) c += (!live[k] || key < keyc[k]);
    } else {
#pragma unroll
      for (int k = 0; k < 3; ++k) {
        if (!live[k]) { ++c; continue; }
        const bool is_eq = key == keyc[k];
        c += (key < keyc[k] || (is_eq && run[k] < quota[k]));
        run[k] += is_eq;
      }
    }
    return c;
  };
  auto width_of = [&](uint32_t key) -> uint32_t { return 2u << class_of_key(key); };

  if constexpr (!PLAN) {
    if (KPT % 8 == 0 && aligned && n_own == (uint32_t)KPT) {       // 8 widths per 64-bit store
#pragma unroll
      for (int i = 0; i < KPT; i += 8) {
        uint64_t w = 0;
#pragma unroll
        for (int j = 0; j < 8; ++j) w |= (uint64_t)width_of(keys[i + j]) << (8 * j);
        *reinterpret_cast<uint64_t*>(bits + t0 + i) = w;
      }
    } else {
#pragma unroll
      for (int i = 0; i < KPT; ++i)
        if ((uint32_t)i < n_own) bits[t0 + i] = (uint8_t)width_of(keys[i]);
    }
  } else {
    // ---- the card's front matter.  Thread tid owns the consecutive tokens [t0, t0 + n_own), so exactly t0
    // tokens lie before them, and the classes among those follow from a block-wide prefix count.
    const CardGeom& g = plan->g;
    uint8_t* card = plan->card;
    uint8_t* bits_card = card + g.off_bits;
    uint32_t* slot_out = reinterpret_cast<uint32_t*>(card + g.off_slot);
    uint32_t* order_out = reinterpret_cast<uint32_t*>(card + g.off_order);
    const uint32_t w0 = blockIdx.x * plan->share_waves, w1 = min(w0 + plan->share_waves, (uint32_t)kWaves);
    const bool mine = wave >= w0 && wave < w1;            // whole waves
    uint32_t cls[(KPT + 15) / 16] = {};                   // the classes of the own tokens, 2 bits each
    uint32_t at_least[3] = {0, 0, 0};                     // own tokens of class >= 1, 2, 3
#pragma unroll
    for (int i = 0; i < KPT; ++i) {
      if ((uint32_t)i < n_own) {
        const uint32_t c = class_of_key(keys[i]);
        cls[i / 16] |= c << (2 * (i % 16));
        at_least[0] += (c >= 1u); at_least[1] += (c >= 2u); at_least[2] += (c >= 3u);
      }
    }
    const uint32_t own[3] = {at_least[0] - at_least[1], at_least[1] - at_least[2], at_least[2]};   // of 4, 8, 16 bits
    uint32_t before[3];
#pragma unroll
    for (int c = 0; c < 3; ++c) {
      const uint32_t inc = wave_inclusive_scan(own[c]);
      before[c] = inc - own[c];
      if (lane == 63) wave_cls[c][wave] = inc;
    }
    __syncthreads();
    // class runs of this workgroup's share inside order[]: first slot and length (classes 1..3 counted, class 0 the rest)
    uint32_t first[4], len[4];
#pragma unroll
    for (int c = 0; c < 3; ++c) {
      const uint32_t running = scan_wave_totals(wave_cls[c], lane);
      before[c] += waves_below(running, wave);
      first[c + 1] = waves_below(running, w0);
      len[c + 1] = waves_below(running, w1) - first[c + 1];
    }
    const uint32_t share_t0 = min(w0 * (uint32_t)(kWaveSize * KPT), T), share_t1 = min(w1 * (uint32_t)(kWaveSize * KPT), T);
    const uint32_t share_n = share_t1 - share_t0;         // <= kShareTokens
    first[0] = share_t0 - first[1] - first[2] - first[3];
    len[0] = share_n - len[1] - len[2] - len[3];
    const uint32_t at[4] = {0u, len[0], len[0] + len[1], len[0] + len[1] + len[2]};      // run starts inside the stage
    uint32_t* stage_order = wide;                         // kShareTokens entries each
    uint32_t* stage_slot = wide + kShareTokens;
    uint8_t* stage_bits = reinterpret_cast<uint8_t*>(&hist2[0][0][0]);
    if (mine) {
      // next free slot of every class for this thread's tokens; class 0 is what remains of the t0 tokens before
      uint32_t next[4] = {t0 - before[0] - before[1] - before[2], before[0], before[1], before[2]};
      const uint32_t lt0 = t0 - share_t0;
#pragma unroll
      for (int i = 0; i < KPT; ++i) {
        if ((uint32_t)i < n_own) {
          const uint32_t c = (cls[i / 16] >> (2 * (i % 16))) & 3u;
          const uint32_t s = (c == 0) ? next[0] : (c == 1) ? next[1] : (c == 2) ? next[2] : next[3];
          next[0] += (c == 0); next[1] += (c == 1); next[2] += (c == 2); next[3] += (c == 3);
          const uint32_t li = s + ((c == 0) ? at[0] - first[0] : (c == 1) ? at[1] - first[1] : (c == 2) ? at[2] - first[2]
                                                                                                     : at[3] - first[3]);
          stage_order[li] = t0 + i;
          stage_slot[lt0 + i] = s;
          stage_bits[lt0 + i] = (uint8_t)width_of_class((int)c);
        }
      }
    }
    __syncthreads();
    for (uint32_t i = tid; i < share_n; i += kThreads) slot_out[share_t0 + i] = stage_slot[i];
#pragma unroll
    for (int c = 0; c < 4; ++c)
      for (uint32_t i = tid; i < len[c]; i += kThreads) order_out[g.base[c] + first[c] + i] = stage_order[at[c] + i];
    // widths: share_t0 is a multiple of 64, so the card's copy goes out in words; the caller's pointer may be odd
    const uint32_t* stage_words = reinterpret_cast<const uint32_t*>(stage_bits);
    const bool words_ok = bits == nullptr || (reinterpret_cast<uintptr_t>(bits) & 3u) == 0u;
    for (uint32_t i = tid; i < share_n / 4u; i += kThreads) {
      reinterpret_cast<uint32_t*>(bits_card + share_t0)[i] = stage_words[i];
      if (bits && words_ok) reinterpret_cast<uint32_t*>(bits + share_t0)[i] = stage_words[i];
    }
    for (uint32_t i = (share_n & ~3u) + tid; i < share_n; i += kThreads) {
      bits_card[share_t0 + i] = stage_bits[i];
      if (bits && words_ok) bits[share_t0 + i] = stage_bits[i];
    }
    if (bits && !words_ok)
      for (uint32_t i = tid; i < share_n; i += kThreads) bits[share_t0 + i] = stage_bits[i];
    // widths come from the allocator and the counts from the same cuts: nothing for the status word to report
    if (blockIdx.x == 0) write_header_and_pads(card, plan->header, plan->pads, 0u, tid);
  }
}

template <int KPT>
__global__ __launch_bounds__(kThreads) void ranked_assign_kernel(const float* __restrict__ scores, uint32_t T, uint32_t cut0,
                                                                 uint32_t cut1, uint32_t cut2, uint8_t* __restrict__ bits,
                                                                 bool aligned) {
  ranked_body<KPT, false>(scores, T, cut0, cut1, cut2, bits, aligned, nullptr);
}

template <int KPT>
__global__ __launch_bounds__(kThreads) void assign_plan_kernel(const float* __restrict__ scores, uint32_t cut0, uint32_t cut1,
                                                               uint32_t cut2, uint8_t* __restrict__ bits, bool aligned,
                                                               PlanArgs plan) {
  ranked_body<KPT, true>(scores, plan.g.tokens, cut0, cut1, cut2, bits, aligned, &plan);
}

// Any T: the same selection with every sweep a loop over the scores and a first-pass histogram in 32 copies.
__global__ __launch_bounds__(kThreads) void long_assign_kernel(const float* __restrict__ scores, uint32_t T, uint32_t cut0,
                                                               uint32_t cut1, uint32_t cut2, uint8_t* __restrict__ bits) {
  constexpr int kWide = 32;
  __shared__ uint32_t wide[256 * kWide];     // first pass: bucket d, copy c at [d * 32 + c]
  __shared__ uint32_t hist[3][256];
  __shared__ uint32_t sel_prefix[3];
  __shared__ uint32_t sel_left[3];
  __shared__ uint32_t wave_tot[3][kWaves];
  const uint32_t tid = threadIdx.x;
  const uint32_t lane = tid & 63u, wave = tid >> 6;
  const uint32_t cut[3] = {cut0, cut1, cut2};
  const uint32_t per = (T + kThreads - 1) / kThreads;
  const uint32_t t0 = min(tid * per, T);
  const uint32_t t1 = min(t0 + per, T);
  auto for_each_key = [&](auto&& f) {
#pragma unroll 4
    for (uint32_t t = t0; t < t1; ++t) f(rank_key(scores[t]), t);
  };
  for (uint32_t i = tid; i < 256 * kWide; i += kThreads) wide[i] = 0;
  __syncthreads();
  for_each_key([&](uint32_t key, uint32_t) { atomicAdd(&wide[(key >> 24) * kWide + (lane & 31u)], 1u); });
  __syncthreads();
  if (tid < 256) {
    uint32_t s = 0;
#pragma unroll 8
    for (int i = 0; i < kWide; ++i) s += wide[tid * kWide + ((i + tid) & 31u)];
    hist[0][tid] = s;
  }
  __syncthreads();
  if (wave < 3 && cut[wave] < T) {
    uint32_t left = cut[wave];
    const uint32_t d = find_bucket(hist[0], lane, left);
    if (lane == 0) { sel_prefix[wave] = d << 24; sel_left[wave] = left; }
  }
  __syncthreads();
#pragma unroll 1
  for (int pass = 1; pass < 4; ++pass) {
    const int shift = 24 - 8 * pass;
    if (tid < 3 * 256) hist[tid >> 8][tid & 255u] = 0;
    uint32_t pre[3];
#pragma unroll
    for (int c = 0; c < 3; ++c) pre[c] = sel_prefix[c];
    __syncthreads();
    const uint32_t high_mask = 0xFFFFFFFFu << (shift + 8);
    for_each_key([&](uint32_t key, uint32_t) {
#pragma unroll
      for (int c = 0; c < 3; ++c) {
        if (cut[c] < T && ((key ^ pre[c]) & high_mask) == 0) atomicAdd(&hist[c][(key >> shift) & 255u], 1u);
      }
    });
    __syncthreads();
    if (wave < 3 && cut[wave] < T) {
      uint32_t left = sel_left[wave];
      const uint32_t d = find_bucket(hist[wave], lane, left);
      if (lane == 0) { sel_prefix[wave] |= d << shift; sel_left[wave] = left; }
    }
    __syncthreads();
  }
  uint32_t keyc[3], quota[3];
#pragma unroll
  for (int c = 0; c < 3; ++c) { keyc[c] = sel_prefix[c]; quota[c] = sel_left[c]; }
  uint32_t eq[3] = {0, 0, 0};
  for_each_key([&](uint32_t key, uint32_t) {
#pragma unroll
    for (int c = 0; c < 3; ++c) eq[c] += (key == keyc[c]);
  });
  uint32_t run[3];
#pragma unroll
  for (int c = 0; c < 3; ++c) {
    const uint32_t inc = wave_inclusive_scan(eq[c]);
    run[c] = inc - eq[c];
    if (lane == 63) wave_tot[c][wave] = inc;
  }
  __syncthreads();
#pragma unroll
  for (int c = 0; c < 3; ++c) {
    uint32_t before = 0;
    for (uint32_t w = 0; w < wave; ++w) before += wave_tot[c][w];
    run[c] += before;
  }
  for_each_key([&](uint32_t key, uint32_t t) {
    bool before[3];
#pragma unroll
    for (int c = 0; c < 3; ++c) {
      if (cut[c] >= T) { before[c] = true; continue; }
      const bool is_eq = key == keyc[c];
      before[c] = key < keyc[c] || (is_eq && run[c] < quota[c]);
      run[c] += is_eq;
    }
    bits[t] = (uint8_t)(before[0] ? 16u : before[1] ? 8u : before[2] ? 4u : 2u);
  });
}

__global__ __launch_bounds__(256) void count_kernel(const uint8_t* __restrict__ bits, uint64_t T,
                                                    unsigned long long* __restrict__ counts4) {
  __shared__ uint32_t part[4];
  if (threadIdx.x < 4) part[threadIdx.x] = 0;
  __syncthreads();
  uint32_t cnt[4] = {0, 0, 0, 0};
  const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
  for (uint64_t t = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; t < T; t += stride) {
    const uint32_t b = bits[t];
    cnt[0] += (b == 2); cnt[1] += (b == 4); cnt[2] += (b == 8); cnt[3] += (b == 16);
  }
#pragma unroll
  for (int c = 0; c < 4; ++c) if (cnt[c]) atomicAdd(&part[c], cnt[c]);
  __syncthreads();
  if (threadIdx.x < 4 && part[threadIdx.x]) atomicAdd(&counts4[threadIdx.x], (unsigned long long)part[threadIdx.x]);
}

__global__ void zero4_kernel(unsigned long long* p) {
  if (threadIdx.x < 4) p[threadIdx.x] = 0;
}

}  // namespace

uint32_t assign_plan_max_tokens() { return kRankedMax; }

namespace {
// Keys per thread of the ranked kernels: the smallest of 1, 2, 4, 8, 16, 32 that covers `tokens` with 1024 threads.
uint32_t keys_per_thread(uint32_t tokens) {
  uint32_t kpt = 1;
  while (kpt * kThreads < tokens) kpt *= 2;
  return kpt;
}
}  // namespace

hipError_t launch_assign(const float* scores, uint32_t tokens, const uint32_t cuts[3], uint8_t* bits,
                         hipStream_t stream) {
  const dim3 grid(1), block(kThreads);
  const bool aligned = reinterpret_cast<uintptr_t>(scores) % 16 == 0 && reinterpret_cast<uintptr_t>(bits) % 8 == 0;
#define QKV_LAUNCH_ASSIGN(K) \
  hipLaunchKernelGGL(ranked_assign_kernel<K>, grid, block, 0, stream, scores, tokens, cuts[0], cuts[1], cuts[2], bits, aligned)
  if (tokens > kRankedMax) {
    hipLaunchKernelGGL(long_assign_kernel, grid, block, 0, stream, scores, tokens, cuts[0], cuts[1], cuts[2], bits);
  } else {
    switch (keys_per_thread(tokens)) {
      case 1: QKV_LAUNCH_ASSIGN(1); break;
      case 2: QKV_LAUNCH_ASSIGN(2); break;
      case 4: QKV_LAUNCH_ASSIGN(4); break;
      case 8: QKV_LAUNCH_ASSIGN(8); break;
      case 16: QKV_LAUNCH_ASSIGN(16); break;
      default: QKV_LAUNCH_ASSIGN(32); break;
    }
  }
#undef QKV_LAUNCH_ASSIGN
  return hipGetLastError();
}

// tokens <= assign_plan_max_tokens()
hipError_t launch_assign_plan(const float* scores, const uint32_t cuts[3], uint8_t* bits, const CardGeom& geom,
                              const qkv_card_header_t& header, uint8_t* card, hipStream_t stream) {
  PlanArgs plan;
  plan.g = geom;
  plan.header = header;
  plan.pads = make_pad_table(geom);
  plan.card = card;
  const uint32_t tokens = geom.tokens;
  if (tokens > kRankedMax) return hipErrorInvalidValue;
  const bool aligned = reinterpret_cast<uintptr_t>(scores) % 16 == 0;
  // a share is whole waves and at most kShareTokens tokens
  const uint32_t kpt = keys_per_thread(tokens);
  uint32_t share_waves = kShareTokens / (kpt * kWaveSize);             // >= 1 since kpt <= 32
  if (share_waves > (uint32_t)kWaves) share_waves = kWaves;
  const uint32_t used_waves = ((tokens + kpt - 1) / kpt + kWaveSize - 1) / kWaveSize;
  plan.share_waves = share_waves;
  const dim3 grid((used_waves + share_waves - 1) / share_waves), block(kThreads);
#define QKV_LAUNCH_PLAN(K) \
  hipLaunchKernelGGL(assign_plan_kernel<K>, grid, block, 0, stream, scores, cuts[0], cuts[1], cuts[2], bits, aligned, plan)
  switch (kpt) {
    case 1: QKV_LAUNCH_PLAN(1); break;
    case 2: QKV_LAUNCH_PLAN(2); break;
    case 4: QKV_LAUNCH_PLAN(4); break;
    case 8: QKV_LAUNCH_PLAN(8); break;
    case 16: QKV_LAUNCH_PLAN(16); break;
    default: QKV_LAUNCH_PLAN(32); break;
  }
#undef QKV_LAUNCH_PLAN
  return hipGetLastError();
}

hipError_t launch_count(const uint8_t* bits, uint64_t tokens, unsigned long long* counts4, hipStream_t stream) {
  hipLaunchKernelGGL(zero4_kernel, dim3(1), dim3(64), 0, stream, counts4);
  uint64_t blocks = (tokens + 256 * 16 - 1) / (256 * 16);
  if (blocks < 1) blocks = 1;
  if (blocks > 1024) blocks = 1024;
  hipLaunchKernelGGL(count_kernel, dim3((uint32_t)blocks), dim3(256), 0, stream, bits, tokens, counts4);
  return hipGetLastError();
}

}  // namespace qkv
