// assign.hip — bit-width assignment from per-token scores (paper Sec. 3.3: the combined
// score S(t) decides b(t) under a memory budget) and the histogram of a bits vector.
//
// Ranking rule: tokens ordered by (score descending, index ascending), scores compared in
// the IEEE total order.  The first cut[0] tokens get 16 bits, up to cut[1] 8 bits, up to
// cut[2] 4 bits, the rest 2.  No sort is needed: for each cut a 4-pass radix select over the
// 32-bit order keys finds the key of the token at that rank and how many tokens lie strictly
// before it; tokens whose key equals the cut key are then admitted by increasing index until
// the cut is full (a stable block-wide prefix count).  One workgroup does it all: the scores
// are a few tens of KiB and stay in cache over the five sweeps.
//
// The first pass sees every key and real scores share their top byte (sign and exponent), so
// its histogram is kept in 32 copies, one per lane modulo 32: lanes of one instruction never
// add to the same word.  The later passes only count keys that match a cut's prefix.
#include "qkv_common.h"

namespace qkv {
namespace {

constexpr int kThreads = 1024;
constexpr int kWaves = kThreads / kWaveSize;
constexpr int kCopies = 32;

// Key that grows as the rank grows: smaller key = better score.  -0 ranks below +0.
__device__ inline uint32_t rank_key(float score) {
  const uint32_t x = __float_as_uint(score);
  const uint32_t up = (x & 0x80000000u) ? ~x : (x | 0x80000000u);   // ascending in the score
  return ~up;
}

// KPT > 0: each thread keeps the keys of its KPT consecutive tokens in registers (needs
// T <= KPT * kThreads); KPT == 0: any T, keys re-read from the scores on every sweep.
template <int KPT>
__global__ __launch_bounds__(kThreads) void assign_kernel(const float* __restrict__ scores, uint32_t T, uint32_t cut0,
                                                          uint32_t cut1, uint32_t cut2, uint8_t* __restrict__ bits,
                                                          bool aligned) {
  __shared__ uint32_t wide[256 * kCopies];   // first pass: bucket d, copy c at [d * 32 + c]
  __shared__ uint32_t hist[3][256];
  __shared__ uint32_t sel_prefix[3];         // key bits fixed so far
  __shared__ uint32_t sel_left[3];           // rank still to descend inside the current bucket
  __shared__ uint32_t wave_tot[3][kWaves];
  const uint32_t tid = threadIdx.x;
  const uint32_t lane = tid & 63u, wave = tid >> 6;
  const uint32_t cut[3] = {cut0, cut1, cut2};

  // thread tid owns the tokens [t0, t1)
  const uint32_t per = KPT > 0 ? (uint32_t)KPT : (T + kThreads - 1) / kThreads;
  const uint32_t t0 = min(tid * per, T);
  const uint32_t t1 = min(t0 + per, T);
  uint32_t keys[KPT > 0 ? KPT : 1];
  if (KPT > 0) {
    if (aligned && t0 + KPT <= T) {      // 128-bit loads
#pragma unroll
      for (int i = 0; i < KPT; i += 4) {
        const float4 f = *reinterpret_cast<const float4*>(scores + t0 + i);
        keys[i] = rank_key(f.x); keys[i + 1] = rank_key(f.y); keys[i + 2] = rank_key(f.z); keys[i + 3] = rank_key(f.w);
      }
    } else {
#pragma unroll
      for (int i = 0; i < KPT; ++i) keys[i] = (t0 + i < t1) ? rank_key(scores[t0 + i]) : 0u;
    }
  }
  // visits every owned token's key
  auto for_each_key = [&](auto&& f) {
    if (KPT > 0) {
#pragma unroll
      for (int i = 0; i < KPT; ++i) if (t0 + i < t1) f(keys[i], t0 + i);
    } else {
#pragma unroll 4
      for (uint32_t t = t0; t < t1; ++t) f(rank_key(scores[t]), t);
    }
  };

  // ---- pass 0: one histogram of the top byte, shared by the three cuts
  for (uint32_t i = tid; i < 256 * kCopies; i += kThreads) wide[i] = 0;
  __syncthreads();
  for_each_key([&](uint32_t key, uint32_t) { atomicAdd(&wide[(key >> 24) * kCopies + (lane & 31u)], 1u); });
  __syncthreads();
  if (tid < 256) {
    uint32_t s = 0;
#pragma unroll 8
    for (int i = 0; i < kCopies; ++i) s += wide[tid * kCopies + ((i + tid) & 31u)];
    hist[0][tid] = s;
  }
  __syncthreads();
  // A cut equal to T has no token at that rank: every token lies before it, handled below
  // without a key.
  if (wave < 3 && cut[wave] < T) {
    uint32_t left = cut[wave];
    const uint32_t d = find_bucket(hist[0], lane, left);
    if (lane == 0) { sel_prefix[wave] = d << 24; sel_left[wave] = left; }
  }
  __syncthreads();

  // ---- passes 1..3: per cut, only the keys inside its bucket so far
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

  // Now sel_prefix[c] is the key at rank cut[c] and sel_left[c] the number of tokens with
  // exactly that key that still belong before the cut.
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
  auto width_of = [&](uint32_t key) -> uint32_t {
    bool before[3];
#pragma unroll
    for (int c = 0; c < 3; ++c) {
      if (cut[c] >= T) { before[c] = true; continue; }
      const bool is_eq = key == keyc[c];
      before[c] = key < keyc[c] || (is_eq && run[c] < quota[c]);
      run[c] += is_eq;
    }
    return before[0] ? 16u : before[1] ? 8u : before[2] ? 4u : 2u;
  };
  if (KPT > 0 && aligned && t0 + KPT <= T) {       // 8 widths per 64-bit store
#pragma unroll
    for (int i = 0; i < KPT; i += 8) {
      uint64_t w = 0;
#pragma unroll
      for (int j = 0; j < 8; ++j) w |= (uint64_t)width_of(keys[i + j]) << (8 * j);
      *reinterpret_cast<uint64_t*>(bits + t0 + i) = w;
    }
  } else {
    for_each_key([&](uint32_t key, uint32_t t) { bits[t] = (uint8_t)width_of(key); });
  }
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

hipError_t launch_assign(const float* scores, uint32_t tokens, const uint32_t cuts[3], uint8_t* bits,
                         hipStream_t stream) {
  const dim3 grid(1), block(kThreads);
  const bool aligned = reinterpret_cast<uintptr_t>(scores) % 16 == 0 && reinterpret_cast<uintptr_t>(bits) % 8 == 0;
  if (tokens <= 8u * kThreads)
    hipLaunchKernelGGL(assign_kernel<8>, grid, block, 0, stream, scores, tokens, cuts[0], cuts[1], cuts[2], bits, aligned);
  else if (tokens <= 32u * kThreads)
    hipLaunchKernelGGL(assign_kernel<32>, grid, block, 0, stream, scores, tokens, cuts[0], cuts[1], cuts[2], bits, aligned);
  else
    hipLaunchKernelGGL(assign_kernel<0>, grid, block, 0, stream, scores, tokens, cuts[0], cuts[1], cuts[2], bits, aligned);
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
