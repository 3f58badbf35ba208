// classify.hip — token classification and stable compaction (first step of card creation,
// paper Sec. 4.2.1: the card carries the token-level bit-width vector; tokens are bucketed
// by width so that every width owns one contiguous segment of the card).
//
// One workgroup of 1024 threads walks the tokens in chunks of 8192: thread i owns the 8
// consecutive tokens 8 i .. 8 i + 7 of the chunk.  A first sweep counts the four classes
// over all tokens (that fixes where each class starts inside order[]).  The second sweep
// takes a block-wide exclusive scan of the per-thread class counters per chunk, which gives
// every token its slot: the bucketing is stable (increasing token index inside a class).
// slot[] and the copy of bits[] leave as 128- and 64-bit stores; the chunk's piece of
// order[] is scattered into LDS first and leaves as coalesced stores, one contiguous range
// per class.  The same kernel writes the header and zeroes the pad bytes of every section.
#include "qkv_common.h"

namespace qkv {
namespace {

constexpr int kThreads = 1024;
constexpr int kWaves = kThreads / kWaveSize;
constexpr uint32_t kPerThread = 8;
constexpr uint32_t kChunk = kThreads * kPerThread;

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// class of a width; anything else is flagged and treated as 2-bit so that order[] stays a permutation
__device__ inline uint32_t class_of(uint32_t b, uint32_t& bad) {
  const uint32_t c = (b == 4) ? 1u : (b == 8) ? 2u : (b == 16) ? 3u : 0u;
  bad |= (c == 0 && b != 2);
  return c;
}

// The widths of tokens t0 .. t0+7 as the 8 bytes of a word (first token lowest); tokens at or
// past T read as 0.
__device__ inline uint64_t load_widths(const uint8_t* __restrict__ bits, uint32_t t0, uint32_t T, bool aligned) {
  if (aligned && t0 + kPerThread <= T) return *reinterpret_cast<const uint64_t*>(bits + t0);
  uint64_t w = 0;
#pragma unroll
  for (uint32_t i = 0; i < kPerThread; ++i)
    if (t0 + i < T) w |= (uint64_t)bits[t0 + i] << (8 * i);
  return w;
}

struct BlockScan {
  uint32_t before[4];   // tokens of each class owned by lower threads
  uint32_t total[4];    // tokens of each class in the whole block
};

// Exclusive block-wide scan of four per-thread counters.  Two barriers; wave_tot is scratch.
__device__ inline BlockScan block_scan4(const uint32_t (&cnt)[4], uint32_t lane, uint32_t wave,
                                        uint32_t (*wave_tot)[kWaves]) {
  BlockScan r;
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    const uint32_t inc = wave_inclusive_scan(cnt[c]);
    r.before[c] = inc - cnt[c];
    if (lane == 63) wave_tot[c][wave] = inc;
  }
  __syncthreads();
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    uint32_t before = 0, all = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
      const uint32_t x = wave_tot[c][w];
      before += ((uint32_t)w < wave) ? x : 0u;
      all += x;
    }
    r.before[c] += before;
    r.total[c] = all;
  }
  __syncthreads();
  return r;
}

__device__ inline uint32_t pick4(uint32_t c, uint32_t a0, uint32_t a1, uint32_t a2, uint32_t a3) {
  return (c == 0) ? a0 : (c == 1) ? a1 : (c == 2) ? a2 : a3;
}

__global__ __launch_bounds__(kThreads) void classify_kernel(const uint8_t* __restrict__ bits, CardGeom g,
                                                           qkv_card_header_t header, uint8_t* __restrict__ card,
                                                           bool aligned) {
  __shared__ uint32_t order_lds[kChunk];
  __shared__ uint32_t wave_tot[4][kWaves];
  __shared__ uint32_t bad_any;
  const uint32_t tid = threadIdx.x;
  const uint32_t lane = tid & 63u, wave = tid >> 6;
  const uint32_t T = g.tokens;
  const uint32_t n_chunks = (T + kChunk - 1) / kChunk;
  if (tid == 0) bad_any = 0;

  // ---- sweep 1: class totals over all tokens
  uint32_t cnt[4] = {0, 0, 0, 0};
  uint32_t bad = 0;
  uint64_t first_widths = 0;
  for (uint32_t k = 0; k < n_chunks; ++k) {
    const uint32_t t0 = k * kChunk + tid * kPerThread;
    const uint64_t w = load_widths(bits, min(t0, T), T, aligned);
    if (k == 0) first_widths = w;
#pragma unroll
    for (uint32_t i = 0; i < kPerThread; ++i) {
      if (t0 + i < T) {
        const uint32_t c = class_of((uint32_t)(w >> (8 * i)) & 0xFFu, bad);
        cnt[0] += (c == 0); cnt[1] += (c == 1); cnt[2] += (c == 2); cnt[3] += (c == 3);
      }
    }
  }
  const BlockScan all = block_scan4(cnt, lane, wave, wave_tot);
  if (bad) atomicOr(&bad_any, 1u);
  // class bases from the histogram the device saw: order[] is then a permutation of 0..T-1
  // whatever the host passed as counts
  const uint32_t base1 = all.total[0], base2 = base1 + all.total[1], base3 = base2 + all.total[2];

  uint8_t* bits_out = card + g.off_bits;
  uint32_t* slot_out = reinterpret_cast<uint32_t*>(card + g.off_slot);
  uint32_t* order_out = reinterpret_cast<uint32_t*>(card + g.off_order);

  // ---- sweep 2: slots, chunk by chunk
  uint32_t carry[4] = {0, 0, 0, 0};            // tokens of each class in the chunks already done
  for (uint32_t k = 0; k < n_chunks; ++k) {
    const uint32_t t0 = k * kChunk + tid * kPerThread;
    const uint64_t w = (k == 0) ? first_widths : load_widths(bits, min(t0, T), T, aligned);
    uint32_t cls[kPerThread];
    uint32_t mine[4] = {0, 0, 0, 0};
    uint32_t ignore = 0;
#pragma unroll
    for (uint32_t i = 0; i < kPerThread; ++i) {
      cls[i] = class_of((uint32_t)(w >> (8 * i)) & 0xFFu, ignore);
      if (t0 + i < T) { mine[0] += (cls[i] == 0); mine[1] += (cls[i] == 1); mine[2] += (cls[i] == 2); mine[3] += (cls[i] == 3); }
    }
    const BlockScan sc = block_scan4(mine, lane, wave, wave_tot);
    // where each class's run of this chunk starts inside the LDS staging array
    const uint32_t reg1 = sc.total[0], reg2 = reg1 + sc.total[1], reg3 = reg2 + sc.total[2];
    uint32_t run0 = sc.before[0], run1 = sc.before[1], run2 = sc.before[2], run3 = sc.before[3];
    uint32_t slot[kPerThread];
#pragma unroll
    for (uint32_t i = 0; i < kPerThread; ++i) {
      const uint32_t c = cls[i];
      const uint32_t in_chunk = pick4(c, run0, run1, run2, run3);
      run0 += (c == 0); run1 += (c == 1); run2 += (c == 2); run3 += (c == 3);
      slot[i] = pick4(c, carry[0], carry[1], carry[2], carry[3]) + in_chunk;
      if (t0 + i < T) order_lds[pick4(c, 0u, reg1, reg2, reg3) + in_chunk] = t0 + i;
    }
    if (t0 + kPerThread <= T) {
      *reinterpret_cast<u32x4*>(slot_out + t0) = (u32x4){slot[0], slot[1], slot[2], slot[3]};
      *reinterpret_cast<u32x4*>(slot_out + t0 + 4) = (u32x4){slot[4], slot[5], slot[6], slot[7]};
      *reinterpret_cast<uint64_t*>(bits_out + t0) = w;
    } else {
#pragma unroll
      for (uint32_t i = 0; i < kPerThread; ++i) {
        if (t0 + i < T) { slot_out[t0 + i] = slot[i]; bits_out[t0 + i] = (uint8_t)(w >> (8 * i)); }
      }
    }
    __syncthreads();
    const uint32_t chunk_n = min(kChunk, T - k * kChunk);
    for (uint32_t p = tid; p < chunk_n; p += kThreads) {
      const uint32_t c = (p >= reg3) ? 3u : (p >= reg2) ? 2u : (p >= reg1) ? 1u : 0u;
      const uint32_t dst = pick4(c, 0u, base1, base2, base3) + pick4(c, carry[0], carry[1], carry[2], carry[3]) +
                           (p - pick4(c, 0u, reg1, reg2, reg3));
      order_out[dst] = order_lds[p];
    }
#pragma unroll
    for (int c = 0; c < 4; ++c) carry[c] += sc.total[c];
    __syncthreads();
  }

  // header: 64 dwords, the status word (dword 48) filled in from what the device saw
  if (tid < 64) {
    uint32_t status = bad_any ? QKV_STATUS_BAD_BITS : 0u;
    if (all.total[0] != g.n[0] || all.total[1] != g.n[1] || all.total[2] != g.n[2] || all.total[3] != g.n[3])
      status |= QKV_STATUS_BAD_COUNTS;
    const uint32_t* h = reinterpret_cast<const uint32_t*>(&header);
    uint32_t v = h[tid];
    if (tid == 48) v = status;
    reinterpret_cast<uint32_t*>(card)[tid] = v;
  }

  // pad bytes behind every section (each less than 256 bytes)
  if (tid >= 256 && tid < 512) {
    const uint32_t i = tid - 256;
    const uint64_t P = g.planes, D = g.head_dim, M = (uint64_t)(g.head_dim / g.group_size) * 4;
    uint64_t start[10], used[10];
    start[0] = g.off_bits;  used[0] = T;
    start[1] = g.off_slot;  used[1] = 4ull * T;
    start[2] = g.off_order; used[2] = 4ull * T;
#pragma unroll
    for (int c = 0; c < 3; ++c) {
      start[3 + 2 * c] = g.off_codes[c]; used[3 + 2 * c] = P * g.n[c] * (D * width_of_class(c) / 8);
      start[4 + 2 * c] = g.off_meta[c];  used[4 + 2 * c] = P * g.n[c] * M;
    }
    start[9] = g.off_fp16; used[9] = P * g.n[3] * D * 2;
#pragma unroll
    for (int s = 0; s < 10; ++s) {
      const uint64_t pad = align256(used[s]) - used[s];
      if (i < pad) card[start[s] + used[s] + i] = 0;
    }
  }
}

}  // namespace

hipError_t launch_classify(const uint8_t* bits, const CardGeom& geom, const qkv_card_header_t& header,
                           uint8_t* card, hipStream_t stream) {
  const bool aligned = reinterpret_cast<uintptr_t>(bits) % 8 == 0;
  hipLaunchKernelGGL(classify_kernel, dim3(1), dim3(kThreads), 0, stream, bits, geom, header, card, aligned);
  return hipGetLastError();
}

}  // namespace qkv
