// attend.hip — decode-step attention of one new query token directly over a card (paper
// Sec. 4.3: consuming a foreign quantized cache inside attention instead of rebuilding the
// dense fp16 cache first, which the paper leaves as future work).
//
// For every layer l and query head hq (kv head h = hq / R, R = query heads per kv head):
//     s_t = scale * <q[l,hq], K^[l,h,t]>,   o = softmax(s) . V^[l,h,:],   lse = log sum exp s
// with K^, V^ the dequantized fp16 values, exactly those the injection kernel would write.
// A softmax sum does not care about the order of its terms, so the card's segments are used
// as they lie: no order[] lookup, no gather.
//
// Work decomposition.  A wave takes one task: up to `chunk` consecutive rows of one width's
// segment for one (layer, kv head), for all R query heads, and leaves an unnormalised
// partial (running maximum m, sum l, sum of p.V^) in a workspace; a second kernel merges the
// partials of each (layer, query head).  Inside a task, in rounds of 16 tokens:
//   scores   lane (n, kq) = (token n of the round, quarter kq of the head dimension) reads its
//            span of 32 codes and its pair, decodes it to 8 MFMA B operands, and eight
//            v_mfma_f32_16x16x16_f16 accumulate q.K^ for 16 tokens x up to 16 query heads
//            (the k index of the MFMA is a fixed permutation of the head dimension, applied to
//            q and K^ alike).  Scores go to LDS.
//   softmax  one maximum per head over the task's tokens, p = exp2(s - m) back into LDS.
//   values   the lane decodes its span of V^ and accumulates p.V^ for 4 query heads in 128
//            fp32 registers (fp16 operand read in place by v_fma_mix_f32); at the end the 16
//            token lanes of each quarter are summed with DPP moves.
#include "qkv_common.h"
#include "qkv_decode.h"

namespace qkv {
namespace {

typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kRoundTokens = 16;
#ifndef QKV_ATTEND_HEADS_PER_PASS
#define QKV_ATTEND_HEADS_PER_PASS 2
#endif
constexpr int kHeadsPerPass = QKV_ATTEND_HEADS_PER_PASS;   // 1, 2 or 4
// Rounds whose loads are in flight ahead of the arithmetic: as many as the registers allow
// (a fetched span is 3 / 5 / 9 / 16 registers at 2 / 4 / 8 / 16 bits).
template <int W> struct Prefetch { static constexpr int kRounds = (W == 2) ? 4 : (W == 4) ? 3 : (W == 8) ? 2 : 1; };
constexpr int kLdsFloatsPerWave = 2048;      // scores of one task: chunk tokens x padded query heads

struct AttendArgs {
  const uint8_t* card;
  uint64_t card_bytes;
  uint32_t layers, kv_heads, head_dim, group_size;
  uint64_t tokens;
  const uint16_t* q;       // fp16 [L][Hq][D]
  uint32_t q_heads;        // Hq
  uint32_t rep;            // R = Hq / H, 1 .. 16
  float scale_log2;        // softmax scale times log2(e)
  float* part_o;           // [L*H][max_tasks][R][D] unnormalised sums of p.V^
  float* part_ml;          // [L*H][max_tasks][R][2]  (m in log2 units, l); l = 0 marks an empty task
  uint32_t max_tasks;      // tasks per (layer, kv head) the workspace was sized for
  uint32_t chunk;          // tokens per task
  float* out;              // fp32 [L][Hq][D]
  float* lse;              // fp32 [L][Hq] or null
  uint32_t* status;        // or null
};

template <int CTRL>
__device__ inline float dpp_f(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, false));
}

// acc += f32(low / high half of w) * p
__device__ inline void fma_lo(float& acc, uint32_t w, float p) {
  asm("v_fma_mix_f32 %0, %1, %2, %0 op_sel:[0,0,0] op_sel_hi:[1,0,0]" : "+v"(acc) : "v"(w), "v"(p));
}
__device__ inline void fma_hi(float& acc, uint32_t w, float p) {
  asm("v_fma_mix_f32 %0, %1, %2, %0 op_sel:[1,0,0] op_sel_hi:[1,0,0]" : "+v"(acc) : "v"(w), "v"(p));
}

__device__ inline float wave_max(float v) {
#pragma unroll
  for (int d = 1; d < kWaveSize; d <<= 1) v = fmaxf(v, __shfl_xor(v, d, kWaveSize));
  return v;
}
__device__ inline float wave_sum(float v) {
#pragma unroll
  for (int d = 1; d < kWaveSize; d <<= 1) v += __shfl_xor(v, d, kWaveSize);
  return v;
}

template <int W, int G>
struct SpanData {
  uint32_t cw[W == 16 ? 16 : W];
  uint32_t pair;
};

// Issues the loads of one span; nothing is decoded yet.
template <int W, int G>
__device__ inline SpanData<W, G> fetch_span(const uint8_t* card, const CardGeom& g, int c, uint64_t row, uint32_t kq,
                                            bool valid) {
  constexpr int GS = G / 32;
  constexpr int NW = (W == 16) ? 16 : W;
  SpanData<W, G> d;
#pragma unroll
  for (int i = 0; i < NW; ++i) d.cw[i] = 0;
  d.pair = 0;
  if (valid) {
    const uint64_t gsp = row * 4 + kq;
    if (W == 16) {
      const u32x4* src = reinterpret_cast<const u32x4*>(card + g.off_fp16 + gsp * 64u);
#pragma unroll
      for (int h = 0; h < 4; ++h) {
        const u32x4 t = src[h];
        d.cw[4 * h] = t.x; d.cw[4 * h + 1] = t.y; d.cw[4 * h + 2] = t.z; d.cw[4 * h + 3] = t.w;
      }
    } else {
      const uint8_t* src = card + g.off_codes[c] + gsp * (4u * W);
      if (W == 2) {
        const u32x2 t = *reinterpret_cast<const u32x2*>(src);
        d.cw[0] = t.x; d.cw[1] = t.y;
      } else {
#pragma unroll
        for (int h = 0; h < NW / 4; ++h) {
          const u32x4 t = *reinterpret_cast<const u32x4*>(src + 16 * h);
          d.cw[4 * h] = t.x; d.cw[4 * h + 1] = t.y; d.cw[4 * h + 2] = t.z; d.cw[4 * h + 3] = t.w;
        }
      }
      d.pair = reinterpret_cast<const uint32_t*>(card + g.off_meta[c])[gsp / GS];
    }
  }
  return d;
}

// The 32 values of a fetched span as 16 packed fp16 pairs.
template <int W, int G>
__device__ inline void decode_fetched(const SpanData<W, G>& d, uint32_t (&out)[16]) {
  if constexpr (W == 16) {
#pragma unroll
    for (int i = 0; i < 16; ++i) out[i] = d.cw[i];
  } else {
    const float s = half_bits_to_float(d.pair & 0xFFFFu);
    const float z = half_bits_to_float(d.pair >> 16);
    decode_span<W>(d.cw, s, z, out);
  }
}

// One task: rows [j0, j1) of class c for the pair (layer, kv head) = pair.
template <int W, int G>
__device__ inline void attend_task(const AttendArgs& a, const CardGeom& g, int c, uint32_t pair, uint32_t j0, uint32_t j1,
                                   uint32_t lane, float* lds, uint64_t part) {
  const uint32_t n = lane & 15u, kq = lane >> 4;
  const uint32_t R = a.rep, R4 = (R + 3u) & ~3u;
  const uint32_t lh = g.planes >> 1;
  const uint32_t n_c = g.n[c];
  const uint64_t k_row0 = (uint64_t)pair * n_c;            // K plane p = pair, V plane p = L*H + pair
  const uint64_t v_row0 = (uint64_t)(lh + pair) * n_c;
  const uint32_t cnt = j1 - j0;
  const uint32_t rounds = (cnt + kRoundTokens - 1) / kRoundTokens;
  constexpr int kPrefetch = Prefetch<W>::kRounds;

  // ---- q as MFMA A operands: row m = lane % 16 is query head m of this kv head, the lane holds
  // q[m][32 kq .. 32 kq + 31]; operand j is q[m][32 kq + 4 j .. + 3]
  f16x4 qa[8];
  {
    u32x4 raw[4];
#pragma unroll
    for (int h = 0; h < 4; ++h) raw[h] = (u32x4)(0u);
    if (n < R) {
      const uint32_t l = pair / g.kv_heads, hh = pair - l * g.kv_heads;
      const u32x4* src = reinterpret_cast<const u32x4*>(a.q + ((uint64_t)(l * a.q_heads + hh * R + n) * 128u + 32u * kq));
#pragma unroll
      for (int h = 0; h < 4; ++h) raw[h] = src[h];
    }
#pragma unroll
    for (int h = 0; h < 4; ++h) {
      qa[2 * h] = __builtin_bit_cast(f16x4, (u32x2){raw[h].x, raw[h].y});
      qa[2 * h + 1] = __builtin_bit_cast(f16x4, (u32x2){raw[h].z, raw[h].w});
    }
  }

  // ---- scores: lds[token * R4 + head] in log2 units, -inf for tokens past the task's end.
  // The loads of the next kPrefetch rounds are always in flight.
  {
    SpanData<W, G> buf[kPrefetch];
#pragma unroll
    for (int u = 0; u < kPrefetch; ++u) {
      const uint32_t t = u * kRoundTokens + n;
      buf[u] = fetch_span<W, G>(a.card, g, c, k_row0 + j0 + t, kq, t < cnt);
    }
    for (uint32_t rd0 = 0; rd0 < rounds; rd0 += kPrefetch) {
#pragma unroll
      for (int u = 0; u < kPrefetch; ++u) {
        const uint32_t rd = rd0 + u;
        if (rd < rounds) {                         // uniform over the wave
          uint32_t kb[16];
          decode_fetched<W, G>(buf[u], kb);
          const uint32_t tn = (rd + kPrefetch) * kRoundTokens + n;
          buf[u] = fetch_span<W, G>(a.card, g, c, k_row0 + j0 + tn, kq, tn < cnt);
          f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int j = 0; j < 8; ++j)
            acc = __builtin_amdgcn_mfma_f32_16x16x16f16(qa[j], __builtin_bit_cast(f16x4, (u32x2){kb[2 * j], kb[2 * j + 1]}),
                                                        acc, 0, 0, 0);
          // the lane holds heads 4 kq .. 4 kq + 3 of token n
          const uint32_t t = rd * kRoundTokens + n;
          if (4u * kq < R4) {
            const bool live = t < cnt;
            f32x4 sc;
            sc.x = live ? acc.x * a.scale_log2 : -INFINITY;
            sc.y = live ? acc.y * a.scale_log2 : -INFINITY;
            sc.z = live ? acc.z * a.scale_log2 : -INFINITY;
            sc.w = live ? acc.w * a.scale_log2 : -INFINITY;
            *reinterpret_cast<f32x4*>(lds + t * R4 + 4u * kq) = sc;
          }
        }
      }
    }
  }

  // ---- softmax over the task's tokens, head by head (the wave's own LDS writes are in order)
  const uint32_t slots = rounds * kRoundTokens;
  for (uint32_t r = 0; r < R; ++r) {
    float m = -INFINITY;
    for (uint32_t t = lane; t < slots; t += kWaveSize) m = fmaxf(m, lds[t * R4 + r]);
    m = wave_max(m);
    float l = 0.f;
    for (uint32_t t = lane; t < slots; t += kWaveSize) {
      const float p = __builtin_amdgcn_exp2f(lds[t * R4 + r] - m);
      lds[t * R4 + r] = p;
      l += p;
    }
    l = wave_sum(l);
    if (lane == 0) {
      a.part_ml[(part * R + r) * 2] = m;
      a.part_ml[(part * R + r) * 2 + 1] = l;
    }
  }

  // ---- values: kHeadsPerPass query heads at a time (their 32 x kHeadsPerPass accumulators
  // are what limits the number of waves per SIMD)
  for (uint32_t hg = 0; hg < R; hg += kHeadsPerPass) {
    float acc[kHeadsPerPass][32];
#pragma unroll
    for (int r = 0; r < kHeadsPerPass; ++r)
#pragma unroll
      for (int i = 0; i < 32; ++i) acc[r][i] = 0.f;
    SpanData<W, G> buf[kPrefetch];
#pragma unroll
    for (int u = 0; u < kPrefetch; ++u) {
      const uint32_t t = u * kRoundTokens + n;
      buf[u] = fetch_span<W, G>(a.card, g, c, v_row0 + j0 + t, kq, t < cnt);
    }
    for (uint32_t rd0 = 0; rd0 < rounds; rd0 += kPrefetch) {
#pragma unroll
      for (int u = 0; u < kPrefetch; ++u) {
        const uint32_t rd = rd0 + u;
        if (rd < rounds) {
          uint32_t vb[16];
          decode_fetched<W, G>(buf[u], vb);
          const uint32_t tn = (rd + kPrefetch) * kRoundTokens + n;
          buf[u] = fetch_span<W, G>(a.card, g, c, v_row0 + j0 + tn, kq, tn < cnt);
          float pr[kHeadsPerPass];
#pragma unroll
          for (int r = 0; r < kHeadsPerPass; ++r) pr[r] = lds[(rd * kRoundTokens + n) * R4 + hg + r];   // hg + r < R4
#pragma unroll
          for (int r = 0; r < kHeadsPerPass; ++r) {
#pragma unroll
            for (int i = 0; i < 16; ++i) {
              fma_lo(acc[r][2 * i], vb[i], pr[r]);
              fma_hi(acc[r][2 * i + 1], vb[i], pr[r]);
            }
          }
        }
      }
    }
    // sum over the 16 token lanes of each quarter, then lane n = 0 of the quarter writes 32 dims
#pragma unroll
    for (int r = 0; r < kHeadsPerPass; ++r) {
#pragma unroll
      for (int i = 0; i < 32; ++i) {
        float v = acc[r][i];
        v += dpp_f<0xB1>(v);      // quad_perm [1,0,3,2]
        v += dpp_f<0x4E>(v);      // quad_perm [2,3,0,1]
        v += dpp_f<0x141>(v);     // row_half_mirror
        v += dpp_f<0x140>(v);     // row_mirror
        acc[r][i] = v;
      }
    }
    if (n == 0) {
#pragma unroll
      for (int r = 0; r < kHeadsPerPass; ++r) {
        if (hg + r < R) {
          f32x4* dst = reinterpret_cast<f32x4*>(a.part_o + (part * R + hg + r) * 128u + 32u * kq);
#pragma unroll
          for (int i = 0; i < 8; ++i) dst[i] = (f32x4){acc[r][4 * i], acc[r][4 * i + 1], acc[r][4 * i + 2], acc[r][4 * i + 3]};
        }
      }
    }
  }
}

template <int G>
__global__ __launch_bounds__(kBlockThreads) __attribute__((amdgpu_waves_per_eu(2)))
void attend_kernel(AttendArgs a) {
  __shared__ __attribute__((aligned(16))) float lds[kWavesPerBlock][kLdsFloatsPerWave];
  CardGeom g;
  if (!card_geometry_from_header(a.card, a.card_bytes, a.layers, a.kv_heads, a.head_dim, a.group_size, a.tokens, g))
    return;                                   // uniform over the grid
  const uint32_t lane = threadIdx.x & 63u;
  const uint32_t wave = threadIdx.x >> 6;
  const uint32_t gw = blockIdx.x * kWavesPerBlock + wave;
  const uint32_t pairs = g.planes >> 1;
  const uint32_t pair = gw / a.max_tasks;
  if (pair >= pairs) return;
  uint32_t tau = gw - pair * a.max_tasks;
  const uint64_t part = (uint64_t)pair * a.max_tasks + tau;

  // which class and which rows this task covers
  int cls = -1;
  uint32_t j0 = 0, j1 = 0;
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    const uint32_t chunks = (g.n[c] + a.chunk - 1) / a.chunk;
    if (cls < 0) {
      if (tau < chunks) {
        cls = c;
        j0 = tau * a.chunk;
        j1 = min(g.n[c], j0 + a.chunk);
      } else {
        tau -= chunks;
      }
    }
  }
  if (cls < 0) {                               // spare task: an empty partial
    for (uint32_t r = lane; r < a.rep; r += kWaveSize) {
      a.part_ml[(part * a.rep + r) * 2] = -INFINITY;
      a.part_ml[(part * a.rep + r) * 2 + 1] = 0.f;
    }
    return;
  }
  float* my_lds = lds[wave];
  if (cls == 0) attend_task<2, G>(a, g, 0, pair, j0, j1, lane, my_lds, part);
  if (cls == 1) attend_task<4, G>(a, g, 1, pair, j0, j1, lane, my_lds, part);
  if (cls == 2) attend_task<8, G>(a, g, 2, pair, j0, j1, lane, my_lds, part);
  if (cls == 3) attend_task<16, G>(a, g, 3, pair, j0, j1, lane, my_lds, part);
}

// Merges the partials of one (layer, query head): thread d owns output dimension d.
__global__ __launch_bounds__(128) void attend_merge_kernel(AttendArgs a) {
  CardGeom g;
  if (!card_geometry_from_header(a.card, a.card_bytes, a.layers, a.kv_heads, a.head_dim, a.group_size, a.tokens, g))
    return;
  const uint32_t d = threadIdx.x;
  const uint32_t lq = blockIdx.x;                      // l * Hq + hq
  const uint32_t l = lq / a.q_heads, hq = lq - l * a.q_heads;
  const uint32_t h = hq / a.rep, r = hq - h * a.rep;
  const uint64_t part0 = (uint64_t)(l * a.kv_heads + h) * a.max_tasks;
  float M = -INFINITY;
  for (uint32_t t = 0; t < a.max_tasks; ++t) {
    const float* ml = a.part_ml + ((part0 + t) * a.rep + r) * 2;
    if (ml[1] > 0.f) M = fmaxf(M, ml[0]);
  }
  float den = 0.f, num = 0.f;
  for (uint32_t t = 0; t < a.max_tasks; ++t) {
    const float* ml = a.part_ml + ((part0 + t) * a.rep + r) * 2;
    if (ml[1] > 0.f) {
      const float w = __builtin_amdgcn_exp2f(ml[0] - M);
      den += w * ml[1];
      num += w * a.part_o[((part0 + t) * a.rep + r) * 128u + d];
    }
  }
  a.out[(uint64_t)lq * 128u + d] = num / den;
  if (d == 0 && a.lse) a.lse[lq] = (M + __builtin_log2f(den)) * 0.69314718055994530942f;
}

__global__ void attend_status_kernel(AttendArgs a) {
  CardGeom g;
  const bool ok = card_geometry_from_header(a.card, a.card_bytes, a.layers, a.kv_heads, a.head_dim, a.group_size,
                                            a.tokens, g);
  if (threadIdx.x == 0 && blockIdx.x == 0) *a.status = ok ? 0u : QKV_STATUS_BAD_HEADER;
}

}  // namespace

// Tokens per task and tasks per (layer, kv head) for a given shape: the scores of one task
// (chunk tokens x query heads padded to a multiple of 4) fill 8 KiB of LDS.
void attend_plan(uint64_t tokens, uint32_t rep, uint32_t* chunk, uint32_t* max_tasks) {
  const uint32_t r4 = (rep + 3u) & ~3u;
  *chunk = (kLdsFloatsPerWave / r4) & ~15u;      // whole rounds of 16 tokens
  *max_tasks = (uint32_t)((tokens + *chunk - 1) / *chunk) + 3u;   // every class may end with a partly filled task
}

hipError_t launch_attend(const uint8_t* card, uint64_t card_bytes, const CardGeom& expect, const void* q,
                         uint32_t q_heads, float softmax_scale, float* out, float* lse, float* workspace,
                         uint32_t* status, hipStream_t stream) {
  AttendArgs a;
  a.card = card;
  a.card_bytes = card_bytes;
  a.layers = expect.layers; a.kv_heads = expect.kv_heads; a.head_dim = expect.head_dim; a.group_size = expect.group_size;
  a.tokens = expect.tokens;
  a.q = static_cast<const uint16_t*>(q);
  a.q_heads = q_heads;
  a.rep = q_heads / expect.kv_heads;
  a.scale_log2 = softmax_scale * 1.44269504088896340736f;
  attend_plan(expect.tokens, a.rep, &a.chunk, &a.max_tasks);
  const uint64_t pairs = (uint64_t)expect.layers * expect.kv_heads;
  a.part_o = workspace;
  a.part_ml = workspace + pairs * a.max_tasks * a.rep * 128u;
  a.out = out;
  a.lse = lse;
  a.status = status;
  if (status) {
    hipLaunchKernelGGL(attend_status_kernel, dim3(1), dim3(kWaveSize), 0, stream, a);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  const uint64_t waves = pairs * a.max_tasks;
  const dim3 grid((uint32_t)((waves + kWavesPerBlock - 1) / kWavesPerBlock)), block(kBlockThreads);
  switch (expect.group_size) {
    case 32: hipLaunchKernelGGL(attend_kernel<32>, grid, block, 0, stream, a); break;
    case 64: hipLaunchKernelGGL(attend_kernel<64>, grid, block, 0, stream, a); break;
    default: hipLaunchKernelGGL(attend_kernel<128>, grid, block, 0, stream, a); break;
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(attend_merge_kernel, dim3(expect.layers * q_heads), dim3(128), 0, stream, a);
  return hipGetLastError();
}

}  // namespace qkv
