// classify.hip — token classification and stable compaction (first step of card creation,
// paper Sec. 4.2.1: the card carries the token-level bit-width vector; tokens are bucketed
// by width so that every width owns one contiguous segment of the card).
//
// One workgroup of 1024 threads.  Thread i owns a contiguous run of tokens; a block-wide
// exclusive scan of the four per-class counters gives each run its first slot, so the
// bucketing is stable (increasing token index inside a class).  The same kernel copies the
// bits vector into the card, writes the header and zeroes the pad bytes of every section.
#include "qkv_common.h"

namespace qkv {
namespace {

constexpr int kThreads = 1024;
constexpr int kWaves = kThreads / kWaveSize;

__device__ inline uint32_t wave_inclusive_scan(uint32_t v, uint32_t lane) {
#pragma unroll
  for (int d = 1; d < kWaveSize; d <<= 1) {
    const uint32_t o = __shfl_up(v, d, kWaveSize);
    if (lane >= (uint32_t)d) v += o;
  }
  return v;
}

__device__ inline int class_of(uint32_t b, uint32_t& bad) {
  switch (b) {
    case 2: return 0;
    case 4: return 1;
    case 8: return 2;
    case 16: return 3;
    default: bad = 1; return 0;    // flagged in the header; treated as 2-bit so order[] stays a permutation
  }
}

// KPT > 0: each thread keeps the widths of its KPT consecutive tokens in registers (needs
// T <= KPT * kThreads); KPT == 0: any T, widths read twice.
template <int KPT>
__global__ __launch_bounds__(kThreads) void classify_kernel(const uint8_t* __restrict__ bits, CardGeom g,
                                                           qkv_card_header_t header, uint8_t* __restrict__ card) {
  __shared__ uint32_t wave_tot[4][kWaves];
  __shared__ uint32_t bad_any;
  const uint32_t tid = threadIdx.x;
  const uint32_t lane = tid & 63u, wave = tid >> 6;
  const uint32_t T = g.tokens;
  const uint32_t per = KPT > 0 ? (uint32_t)KPT : (T + kThreads - 1) / kThreads;
  const uint32_t t0 = min(tid * per, T);      // tid * per < 2^32: per <= T / 1024 + 1
  const uint32_t t1 = min(t0 + per, T);
  if (tid == 0) bad_any = 0;

  uint32_t held[KPT > 0 ? KPT : 1];
  if (KPT > 0) {
#pragma unroll
    for (int i = 0; i < KPT; ++i) held[i] = (t0 + i < t1) ? bits[t0 + i] : 2u;
  }
  auto for_each_token = [&](auto&& f) {
    if (KPT > 0) {
#pragma unroll
      for (int i = 0; i < KPT; ++i) if (t0 + i < t1) f(held[i], t0 + i);
    } else {
#pragma unroll 4
      for (uint32_t t = t0; t < t1; ++t) f((uint32_t)bits[t], t);
    }
  };

  uint32_t cnt[4] = {0, 0, 0, 0};
  uint32_t bad = 0;
  for_each_token([&](uint32_t b, uint32_t) {
    const int c = class_of(b, bad);
    cnt[0] += (c == 0); cnt[1] += (c == 1); cnt[2] += (c == 2); cnt[3] += (c == 3);
  });

  uint32_t run[4];
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    const uint32_t inc = wave_inclusive_scan(cnt[c], lane);
    run[c] = inc - cnt[c];
    if (lane == 63) wave_tot[c][wave] = inc;
  }
  __syncthreads();
  if (bad) atomicOr(&bad_any, 1u);
  uint32_t tot[4];
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    uint32_t before = 0, all = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
      const uint32_t x = wave_tot[c][w];
      if ((uint32_t)w < wave) before += x;
      all += x;
    }
    run[c] += before;
    tot[c] = all;
  }
  // class bases from the histogram the device saw: order[] is then a permutation of 0..T-1
  // whatever the host passed as counts
  uint32_t base[4];
  base[0] = 0; base[1] = tot[0]; base[2] = tot[0] + tot[1]; base[3] = tot[0] + tot[1] + tot[2];

  uint8_t* bits_out = card + g.off_bits;
  uint32_t* slot_out = reinterpret_cast<uint32_t*>(card + g.off_slot);
  uint32_t* order_out = reinterpret_cast<uint32_t*>(card + g.off_order);
  for_each_token([&](uint32_t b, uint32_t t) {
    uint32_t dummy = 0;
    const int c = class_of(b, dummy);
    const uint32_t s = (c == 0) ? run[0]++ : (c == 1) ? run[1]++ : (c == 2) ? run[2]++ : run[3]++;
    bits_out[t] = (uint8_t)b;
    slot_out[t] = s;
    order_out[base[c] + s] = t;
  });
  __syncthreads();

  // header: 64 dwords, the status word (dword 48) filled in from what the device saw
  if (tid < 64) {
    uint32_t status = bad_any ? QKV_STATUS_BAD_BITS : 0u;
    if (tot[0] != g.n[0] || tot[1] != g.n[1] || tot[2] != g.n[2] || tot[3] != g.n[3]) status |= QKV_STATUS_BAD_COUNTS;
    const uint32_t* h = reinterpret_cast<const uint32_t*>(&header);
    uint32_t v = h[tid];
    if (tid == 48) v = status;
    reinterpret_cast<uint32_t*>(card)[tid] = v;
  }

  // pad bytes behind every section (each less than 256 bytes)
  if (tid < 256) {
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
      if (tid < pad) card[start[s] + used[s] + tid] = 0;
    }
  }
}

}  // namespace

hipError_t launch_classify(const uint8_t* bits, const CardGeom& geom, const qkv_card_header_t& header,
                           uint8_t* card, hipStream_t stream) {
  const dim3 grid(1), block(kThreads);
  if (geom.tokens <= 8u * kThreads)
    hipLaunchKernelGGL(classify_kernel<8>, grid, block, 0, stream, bits, geom, header, card);
  else if (geom.tokens <= 32u * kThreads)
    hipLaunchKernelGGL(classify_kernel<32>, grid, block, 0, stream, bits, geom, header, card);
  else
    hipLaunchKernelGGL(classify_kernel<0>, grid, block, 0, stream, bits, geom, header, card);
  return hipGetLastError();
}

}  // namespace qkv
