// classify.hip — token classification and stable compaction (first step of card creation,
// paper Sec. 4.2.1: the card carries the token-level bit-width vector; tokens are bucketed
// by width so that every width owns one contiguous segment of the card).
//
// Workgroup b of 256 threads owns the 2048 tokens [2048 b, 2048 b + 2048), 8 consecutive
// tokens (one 64-bit word of widths) per thread.  No workgroup talks to another: each one
// first counts the classes over the whole bits vector by itself (a few words per thread,
// byte-parallel arithmetic), which yields both the class totals - where each class starts
// inside order[] - and the counts in front of its own tokens.  A packed DPP scan over the
// per-thread counters then gives every token its slot, so the bucketing is stable
// (increasing token index inside a class).  The work is bound by instruction issue, not by
// memory, which is why it is spread over several compute units instead of one.
// Workgroup 0 also writes the header and zeroes the pad bytes of every section.
#include "qkv_common.h"
#include "qkv_plan.h"

namespace qkv {
namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / kWaveSize;
constexpr uint32_t kPerThread = 8;
constexpr uint32_t kPerBlock = kThreads * kPerThread;

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// Number of bytes of w equal to the byte replicated in `pattern` (exact, no carries between bytes).
__device__ inline uint32_t count_bytes_equal(uint64_t w, uint64_t pattern) {
  const uint64_t low7 = 0x7F7F7F7F7F7F7F7Full;
  const uint64_t x = w ^ pattern;
  const uint64_t zero = ~(((x & low7) + low7) | x | low7);      // 0x80 in every byte of x that is 0
  return (uint32_t)__builtin_popcountll(zero);
}

// The widths of tokens t0 .. t0+7 as the 8 bytes of a word (first token lowest); tokens at or
// past T read as 0 (no class pattern, so they are never counted).
__device__ inline uint64_t load_widths(const uint8_t* __restrict__ bits, uint32_t t0, uint32_t T, bool aligned) {
  if (t0 >= T) return 0;
  if (aligned && t0 + kPerThread <= T) return *reinterpret_cast<const uint64_t*>(bits + t0);
  uint64_t w = 0;
#pragma unroll
  for (uint32_t i = 0; i < kPerThread; ++i)
    if (t0 + i < T) w |= (uint64_t)bits[t0 + i] << (8 * i);
  return w;
}

// Sums of N values over the workgroup with one barrier.  `slots` is LDS scratch.
template <int N>
__device__ inline void block_sums(uint32_t (&v)[N], uint32_t lane, uint32_t wave, uint32_t (*slots)[kWaves]) {
#pragma unroll
  for (int n = 0; n < N; ++n) {
    const uint32_t inc = wave_inclusive_scan(v[n]);
    if (lane == 63) slots[n][wave] = inc;
  }
  __syncthreads();
#pragma unroll
  for (int n = 0; n < N; ++n) {
    uint32_t s = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) s += slots[n][w];
    v[n] = s;
  }
}

__global__ __launch_bounds__(kThreads) void classify_kernel(const uint8_t* __restrict__ bits, CardGeom g,
                                                           qkv_card_header_t header, PadTable pads,
                                                           uint8_t* __restrict__ card, bool aligned) {
  __shared__ uint32_t sum_slots[7][kWaves];
  __shared__ uint32_t slots[kWaves];
  const uint32_t tid = threadIdx.x;
  const uint32_t lane = tid & 63u, wave = tid >> 6;
  const uint32_t T = g.tokens;
  const uint32_t block_t0 = blockIdx.x * kPerBlock;       // < T for every launched workgroup
  const uint32_t t0 = block_t0 + tid * kPerThread;

  // ---- counts over the whole vector: totals, and what lies in front of this workgroup.
  // Thread tid visits the words tid, tid + 256, ...: its own word is one of them.
  const uint64_t p2 = 0x0202020202020202ull, p4 = p2 << 1, p8 = p2 << 2, p16 = p2 << 3;
  uint32_t tot1 = 0, tot2 = 0, tot3 = 0, valid = 0;       // classes 1..3, and all four valid widths
  uint32_t pre1 = 0, pre2 = 0, pre3 = 0;                  // classes 1..3 among the tokens below block_t0
  uint64_t mine = 0;
  const uint32_t n_words = (T + kPerThread - 1) / kPerThread;
  for (uint32_t i = tid; i < n_words; i += kThreads) {
    const uint64_t w = load_widths(bits, i * kPerThread, T, aligned);
    const uint32_t c1 = count_bytes_equal(w, p4), c2 = count_bytes_equal(w, p8), c3 = count_bytes_equal(w, p16);
    tot1 += c1; tot2 += c2; tot3 += c3;
    valid += c1 + c2 + c3 + count_bytes_equal(w, p2);
    const bool before = i * kPerThread < block_t0;
    pre1 += before ? c1 : 0u; pre2 += before ? c2 : 0u; pre3 += before ? c3 : 0u;
    if (i * kPerThread == t0) mine = w;
  }
  {
    uint32_t v[7] = {tot1, tot2, tot3, valid, pre1, pre2, pre3};
    block_sums<7>(v, lane, wave, sum_slots);
    tot1 = v[0]; tot2 = v[1]; tot3 = v[2]; valid = v[3]; pre1 = v[4]; pre2 = v[5]; pre3 = v[6];
  }
  const uint32_t tot0 = T - tot1 - tot2 - tot3;
  const uint32_t pre0 = block_t0 - pre1 - pre2 - pre3;
  // class bases from the histogram the device saw: order[] is then a permutation of 0..T-1
  // whatever the host passed as counts
  const uint32_t base1 = tot0, base2 = base1 + tot1, base3 = base2 + tot2;

  // ---- slots of this workgroup's tokens: a scan of the per-thread counts of classes 1..3,
  // 10 bits each in one word (a wave holds at most 512 tokens); class 0 is what remains
  uint32_t cls[kPerThread];
  uint32_t packed = 0;
  uint32_t n_mine = 0;
#pragma unroll
  for (uint32_t i = 0; i < kPerThread; ++i) {
    cls[i] = class_of((uint32_t)(mine >> (8 * i)) & 0xFFu);
    if (t0 + i < T) {
      ++n_mine;
      packed += (cls[i] == 1) ? 1u : (cls[i] == 2) ? (1u << 10) : (cls[i] == 3) ? (1u << 20) : 0u;
    }
  }
  const uint32_t inc = wave_inclusive_scan(packed);
  const uint32_t inc_n = wave_inclusive_scan(n_mine);
  if (lane == 63) slots[wave] = inc;
  __syncthreads();
  uint32_t w1 = 0, w2 = 0, w3 = 0;                        // classes 1..3 in the lower waves of this workgroup
#pragma unroll
  for (int w = 0; w < kWaves; ++w) {
    const uint32_t x = ((uint32_t)w < wave) ? slots[w] : 0u;
    w1 += x & 1023u; w2 += (x >> 10) & 1023u; w3 += x >> 20;
  }
  const uint32_t ex = inc - packed;                       // lower lanes of this wave
  const uint32_t e1 = ex & 1023u, e2 = (ex >> 10) & 1023u, e3 = ex >> 20;
  const uint32_t tokens_below = wave * (kWaveSize * kPerThread) + (inc_n - n_mine);   // inside the workgroup
  uint32_t run1 = pre1 + w1 + e1, run2 = pre2 + w2 + e2, run3 = pre3 + w3 + e3;
  uint32_t run0 = pre0 + tokens_below - (w1 + e1) - (w2 + e2) - (w3 + e3);

  uint8_t* bits_out = card + g.off_bits;
  uint32_t* slot_out = reinterpret_cast<uint32_t*>(card + g.off_slot);
  uint32_t* order_out = reinterpret_cast<uint32_t*>(card + g.off_order);
  uint32_t slot[kPerThread];
#pragma unroll
  for (uint32_t i = 0; i < kPerThread; ++i) {
    const uint32_t c = cls[i];
    const uint32_t s = (c == 0) ? run0 : (c == 1) ? run1 : (c == 2) ? run2 : run3;
    run0 += (c == 0); run1 += (c == 1); run2 += (c == 2); run3 += (c == 3);
    slot[i] = s;
    if (t0 + i < T) order_out[((c == 0) ? 0u : (c == 1) ? base1 : (c == 2) ? base2 : base3) + s] = t0 + i;
  }
  if (t0 + kPerThread <= T) {
    *reinterpret_cast<u32x4*>(slot_out + t0) = (u32x4){slot[0], slot[1], slot[2], slot[3]};
    *reinterpret_cast<u32x4*>(slot_out + t0 + 4) = (u32x4){slot[4], slot[5], slot[6], slot[7]};
    *reinterpret_cast<uint64_t*>(bits_out + t0) = mine;
  } else {
#pragma unroll
    for (uint32_t i = 0; i < kPerThread; ++i) {
      if (t0 + i < T) { slot_out[t0 + i] = slot[i]; bits_out[t0 + i] = (uint8_t)(mine >> (8 * i)); }
    }
  }

  if (blockIdx.x != 0) return;

  // header (the status word filled in from what the device saw) and the pad bytes behind every section
  uint32_t status = (valid != T) ? QKV_STATUS_BAD_BITS : 0u;
  if (tot0 != g.n[0] || tot1 != g.n[1] || tot2 != g.n[2] || tot3 != g.n[3]) status |= QKV_STATUS_BAD_COUNTS;
  write_header_and_pads(card, header, pads, status, tid);
}

}  // namespace

hipError_t launch_classify(const uint8_t* bits, const CardGeom& geom, const qkv_card_header_t& header,
                           uint8_t* card, hipStream_t stream) {
  const bool aligned = reinterpret_cast<uintptr_t>(bits) % 8 == 0;
  const uint32_t blocks = (geom.tokens + kPerBlock - 1) / kPerBlock;
  hipLaunchKernelGGL(classify_kernel, dim3(blocks), dim3(kThreads), 0, stream, bits, geom, header, make_pad_table(geom), card, aligned);
  return hipGetLastError();
}

}  // namespace qkv
