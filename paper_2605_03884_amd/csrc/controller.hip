// controller.hip — the bit-width controller on the device: the network that scores tokens
// (paper Sec. 4.1.2) and the allocator that follows the budgeted objective of Sec. 3.3
// literally.
//
// Network: 6 features per token -> 64 hidden units (ReLU) -> one score, 512 parameters (no
// output bias: it cannot change a ranking).  One token per thread; the parameters arrive as
// a kernel argument, so every lane reads them through uniform loads.  fp32 in a fixed order:
// a hidden unit starts at its bias and takes one fused multiply-add per feature in feature
// order; the score starts at +0 and takes one fused multiply-add per hidden unit in unit
// order.
//
// Allocator: every token starts at 2 bits; the upgrades 2->4, 4->8, 8->16 cost 2, 4, 8 bits
// and, with the error model eps(b) = 1 / (2^b - 1), gain S * 2/15, S * 4/255, S * 32/65535
// per bit.  All 3T upgrades are ranked by (gain per bit descending, level ascending, token
// ascending) and the longest prefix that fits the budget is taken.  No sort: a radix select
// over the 32-bit gain keys, with histograms weighted by cost, finds the key at which the
// budget runs out and what is left of the budget there; the upgrades with exactly that key
// are then admitted level by level, by increasing token index, until one does not fit.
#include "qkv_common.h"

namespace qkv {
namespace {

constexpr int kFeatures = 6, kHidden = 64;

__global__ __launch_bounds__(256) void controller_kernel(const float* __restrict__ features, uint32_t T,
                                                         qkv_controller_t p, float* __restrict__ scores) {
  const uint32_t t = blockIdx.x * 256u + threadIdx.x;
  if (t >= T) return;
  const float2* row = reinterpret_cast<const float2*>(features + (uint64_t)t * kFeatures);   // 24-byte rows
  const float2 x01 = row[0], x23 = row[1], x45 = row[2];
  const float x[kFeatures] = {x01.x, x01.y, x23.x, x23.y, x45.x, x45.y};
  float s = 0.0f;
#pragma unroll
  for (int j = 0; j < kHidden; ++j) {
    float a = p.b1[j];
#pragma unroll
    for (int i = 0; i < kFeatures; ++i) a = __builtin_fmaf(x[i], p.w1[j][i], a);
    const float h = a > 0.0f ? a : 0.0f;       // NaN -> 0
    s = __builtin_fmaf(h, p.w2[j], s);
  }
  scores[t] = s;
}

// ---------------------------------------------------------------------------------------------

constexpr int kThreads = 1024;
constexpr int kWaves = kThreads / kWaveSize;
constexpr int kCopies = 32;

// Key of an upgrade: grows as the gain per bit falls.  The gain is +0 or positive, so its bit
// pattern orders like its value.
__device__ inline uint32_t gain_key(float score, float per_bit) {
  const float s = score > 0.0f ? score : 0.0f;     // negative and NaN scores count as 0
  return ~__float_as_uint(s * per_bit);
}

// KPT > 0: each thread keeps the scores of its KPT consecutive tokens in registers (needs T <= KPT * kThreads);
// KPT == 0: any T, scores re-read on every sweep.
template <int KPT>
__global__ __launch_bounds__(kThreads) void greedy_kernel(const float* __restrict__ scores, uint32_t T,
                                                          uint32_t spare, uint8_t* __restrict__ bits,
                                                          unsigned long long* __restrict__ counts4) {
  __shared__ uint32_t wide[256 * kCopies];   // first pass: bucket d, copy c at [d * 32 + c]
  __shared__ uint32_t hist[256];
  __shared__ uint32_t sel_prefix, sel_left;
  __shared__ uint32_t wave_tot[3][kWaves];
  __shared__ uint32_t class_tot[4];
  const uint32_t tid = threadIdx.x;
  const uint32_t lane = tid & 63u, wave = tid >> 6;
  const float per_bit[3] = {(float)(2.0 / 15.0), (float)(4.0 / 255.0), (float)(32.0 / 65535.0)};

  const uint32_t per = KPT > 0 ? (uint32_t)KPT : (T + kThreads - 1) / kThreads;   // thread tid owns the tokens [t0, t1)
  const uint32_t t0 = min(tid * per, T);
  const uint32_t t1 = min(t0 + per, T);
  float mine[KPT > 0 ? KPT : 1];
  if (KPT > 0) {
#pragma unroll
    for (int i = 0; i < KPT; ++i) mine[i] = (t0 + i < t1) ? scores[t0 + i] : 0.0f;
  }
  // visits every owned token's score
  auto for_each_score = [&](auto&& f) {
    if (KPT > 0) {
#pragma unroll
      for (int i = 0; i < KPT; ++i) if (t0 + i < t1) f(mine[i], t0 + i);
    } else {
      for (uint32_t t = t0; t < t1; ++t) f(scores[t], t);
    }
  };
  // `spare` counts units of 2 bits; the upgrades weigh 1, 2, 4.  If all 7T fit, nothing is selected.
  const bool everything = spare >= 7u * T;

  uint32_t kstar = 0, left = 0;
  if (!everything) {
    // ---- pass 0: weighted histogram of the top key byte over all upgrades
    for (uint32_t i = tid; i < 256 * kCopies; i += kThreads) wide[i] = 0;
    if (tid < 4) class_tot[tid] = 0;
    __syncthreads();
    for_each_score([&](float s, uint32_t) {
#pragma unroll
      for (int l = 0; l < 3; ++l) atomicAdd(&wide[(gain_key(s, per_bit[l]) >> 24) * kCopies + (lane & 31u)], 1u << l);
    });
    __syncthreads();
    if (tid < 256) {
      uint32_t sum = 0;
#pragma unroll 8
      for (int i = 0; i < kCopies; ++i) sum += wide[tid * kCopies + ((i + tid) & 31u)];
      hist[tid] = sum;
    }
    __syncthreads();
    if (wave == 0) {      // the histogram's total, 7T, exceeds spare
      uint32_t l = spare;
      const uint32_t d = find_bucket(hist, lane, l);
      if (lane == 0) { sel_prefix = d << 24; sel_left = l; }
    }
    __syncthreads();
    // ---- passes 1..3: only the upgrades inside the bucket chosen so far
    for (int pass = 1; pass < 4; ++pass) {
      const int shift = 24 - 8 * pass;
      const uint32_t pre = sel_prefix;
      if (tid < 256) hist[tid] = 0;
      __syncthreads();
      const uint32_t high_mask = 0xFFFFFFFFu << (shift + 8);
      for_each_score([&](float s, uint32_t) {
#pragma unroll
        for (int l = 0; l < 3; ++l) {
          const uint32_t key = gain_key(s, per_bit[l]);
          if (((key ^ pre) & high_mask) == 0) atomicAdd(&hist[(key >> shift) & 255u], 1u << l);
        }
      });
      __syncthreads();
      if (wave == 0) {
        uint32_t l = sel_left;
        const uint32_t d = find_bucket(hist, lane, l);
        if (lane == 0) { sel_prefix = pre | (d << shift); sel_left = l; }
      }
      __syncthreads();
    }
    kstar = sel_prefix;     // the key at which the budget runs out
    left = sel_left;        // units still free for the upgrades with exactly that key
  } else {
    if (tid < 4) class_tot[tid] = 0;
    __syncthreads();
  }

  // ---- upgrades with key == kstar: per level, how many lie at lower token indices
  uint32_t run[3] = {0, 0, 0}, quota[3] = {0, 0, 0};
  if (!everything) {
    uint32_t eq[3] = {0, 0, 0};
    for_each_score([&](float s, uint32_t) {
#pragma unroll
      for (int l = 0; l < 3; ++l) eq[l] += (gain_key(s, per_bit[l]) == kstar);
    });
#pragma unroll
    for (int l = 0; l < 3; ++l) {
      const uint32_t inc = wave_inclusive_scan(eq[l]);
      run[l] = inc - eq[l];
      if (lane == 63) wave_tot[l][wave] = inc;
    }
    __syncthreads();
    uint32_t n[3];
#pragma unroll
    for (int l = 0; l < 3; ++l) {
      uint32_t before = 0, all = 0;
      for (uint32_t w = 0; w < (uint32_t)kWaves; ++w) {
        const uint32_t x = wave_tot[l][w];
        before += (w < wave) ? x : 0u;
        all += x;
      }
      run[l] += before;
      n[l] = all;
    }
    // admitted level by level until one upgrade does not fit; nothing after it is taken
    uint32_t free_units = left;
    quota[0] = min(n[0], free_units);
    bool full = quota[0] == n[0];
    free_units -= quota[0];
    quota[1] = full ? min(n[1], free_units / 2u) : 0u;
    full = full && quota[1] == n[1];
    free_units -= 2u * quota[1];
    quota[2] = full ? min(n[2], free_units / 4u) : 0u;
  }

  uint32_t cnt[4] = {0, 0, 0, 0};
  for_each_score([&](float s, uint32_t t) {
    bool taken[3];
#pragma unroll
    for (int l = 0; l < 3; ++l) {
      const uint32_t key = gain_key(s, per_bit[l]);
      const bool is_eq = key == kstar;
      taken[l] = everything || key < kstar || (is_eq && run[l] < quota[l]);
      run[l] += is_eq;
    }
    const uint32_t c = taken[0] ? (taken[1] ? (taken[2] ? 3u : 2u) : 1u) : 0u;
    bits[t] = (uint8_t)(2u << c);
    cnt[0] += (c == 0); cnt[1] += (c == 1); cnt[2] += (c == 2); cnt[3] += (c == 3);
  });
  if (counts4 != nullptr) {
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const uint32_t inc = wave_inclusive_scan(cnt[c]);
      if (lane == 63 && inc) atomicAdd(&class_tot[c], inc);
    }
    __syncthreads();
    if (tid < 4) counts4[tid] = class_tot[tid];
  }
}

}  // namespace

hipError_t launch_controller(const float* features, uint32_t tokens, const qkv_controller_t& params, float* scores,
                             hipStream_t stream) {
  hipLaunchKernelGGL(controller_kernel, dim3((tokens + 255u) / 256u), dim3(256), 0, stream, features, tokens, params,
                     scores);
  return hipGetLastError();
}

hipError_t launch_greedy(const float* scores, uint32_t tokens, uint32_t spare_units, uint8_t* bits,
                         unsigned long long* counts4, hipStream_t stream) {
  if (tokens <= 8u * kThreads)
    hipLaunchKernelGGL(greedy_kernel<8>, dim3(1), dim3(kThreads), 0, stream, scores, tokens, spare_units, bits, counts4);
  else if (tokens <= 32u * kThreads)
    hipLaunchKernelGGL(greedy_kernel<32>, dim3(1), dim3(kThreads), 0, stream, scores, tokens, spare_units, bits, counts4);
  else
    hipLaunchKernelGGL(greedy_kernel<0>, dim3(1), dim3(kThreads), 0, stream, scores, tokens, spare_units, bits, counts4);
  return hipGetLastError();
}

}  // namespace qkv
