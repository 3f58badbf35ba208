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
#include "qkv_common.h"

namespace qkv {
namespace {

constexpr int kThreads = 1024;
constexpr int kWaves = kThreads / kWaveSize;

// Key that grows as the rank grows: smaller key = better score.  -0 ranks below +0.
__device__ inline uint32_t rank_key(float score) {
  const uint32_t x = __float_as_uint(score);
  const uint32_t up = (x & 0x80000000u) ? ~x : (x | 0x80000000u);   // ascending in the score
  return ~up;
}

__device__ inline uint32_t wave_inclusive_scan(uint32_t v, uint32_t lane) {
#pragma unroll
  for (int d = 1; d < kWaveSize; d <<= 1) {
    const uint32_t o = __shfl_up(v, d, kWaveSize);
    if (lane >= (uint32_t)d) v += o;
  }
  return v;
}

__global__ __launch_bounds__(kThreads) void assign_kernel(const float* __restrict__ scores, uint32_t T, uint32_t cut0,
                                                          uint32_t cut1, uint32_t cut2, uint8_t* __restrict__ bits) {
  __shared__ uint32_t hist[3][256];
  __shared__ uint32_t sel_prefix[3];     // key bits fixed so far
  __shared__ uint32_t sel_left[3];       // rank still to descend inside the current bucket
  __shared__ uint32_t wave_tot[3][kWaves];
  const uint32_t tid = threadIdx.x;
  const uint32_t lane = tid & 63u, wave = tid >> 6;
  const uint32_t cut[3] = {cut0, cut1, cut2};

  if (tid < 3) { sel_prefix[tid] = 0; sel_left[tid] = cut[tid]; }

  // radix select, most significant byte first.  A cut equal to T has no token at that rank:
  // every token lies before it, handled below without a key.
  for (int pass = 0; pass < 4; ++pass) {
    const int shift = 24 - 8 * pass;
    for (uint32_t i = tid; i < 3 * 256; i += kThreads) hist[i >> 8][i & 255u] = 0;
    __syncthreads();
    uint32_t pre[3];
#pragma unroll
    for (int c = 0; c < 3; ++c) pre[c] = sel_prefix[c];
    const uint32_t high_mask = pass == 0 ? 0u : (0xFFFFFFFFu << (shift + 8));
    for (uint32_t t = tid; t < T; t += kThreads) {
      const uint32_t key = rank_key(scores[t]);
#pragma unroll
      for (int c = 0; c < 3; ++c) {
        if (cut[c] < T && ((key ^ pre[c]) & high_mask) == 0) atomicAdd(&hist[c][(key >> shift) & 255u], 1u);
      }
    }
    __syncthreads();
    if (tid < 3 && cut[tid] < T) {
      uint32_t left = sel_left[tid];
      uint32_t d = 0;
      // the bucket that holds rank `left`: first d with cumulative count > left
      for (; d < 255; ++d) {
        const uint32_t h = hist[tid][d];
        if (left < h) break;
        left -= h;
      }
      sel_prefix[tid] |= d << shift;
      sel_left[tid] = left;
    }
    __syncthreads();
  }

  // Now sel_prefix[c] is the key at rank cut[c] and sel_left[c] the number of tokens with
  // exactly that key that still belong before the cut.
  uint32_t keyc[3], quota[3];
#pragma unroll
  for (int c = 0; c < 3; ++c) { keyc[c] = sel_prefix[c]; quota[c] = sel_left[c]; }

  const uint32_t per = (T + kThreads - 1) / kThreads;
  const uint32_t t0 = min(tid * per, T);
  const uint32_t t1 = min(t0 + per, T);
  uint32_t eq[3] = {0, 0, 0};
  for (uint32_t t = t0; t < t1; ++t) {
    const uint32_t key = rank_key(scores[t]);
#pragma unroll
    for (int c = 0; c < 3; ++c) eq[c] += (key == keyc[c]);
  }
  uint32_t run[3];
#pragma unroll
  for (int c = 0; c < 3; ++c) {
    const uint32_t inc = wave_inclusive_scan(eq[c], lane);
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
  for (uint32_t t = t0; t < t1; ++t) {
    const uint32_t key = rank_key(scores[t]);
    bool before[3];
#pragma unroll
    for (int c = 0; c < 3; ++c) {
      if (cut[c] >= T) { before[c] = true; continue; }
      const bool is_eq = key == keyc[c];
      before[c] = key < keyc[c] || (is_eq && run[c] < quota[c]);
      run[c] += is_eq;
    }
    bits[t] = before[0] ? 16 : before[1] ? 8 : before[2] ? 4 : 2;
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
  hipLaunchKernelGGL(assign_kernel, dim3(1), dim3(kThreads), 0, stream, scores, tokens, cuts[0], cuts[1], cuts[2],
                     bits);
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
