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
//   scores   lane (n, kq) = (token n of the round, quarter kq of a slab of 128 dimensions) reads
//            its span of 32 codes and its pair, decodes it to 8 MFMA operands of 4 dimensions,
//            and eight MFMAs accumulate q.K^ for the round's tokens and the kv head's query
//            heads (the k index of the MFMA is a fixed permutation of the head dimension,
//            applied to q and K^ alike).  Scores go to LDS.
//   softmax  one maximum per head over the task's tokens, p = exp2(s - m) back into LDS.
//   values   the round's packed V rows are regrouped through LDS (still packed) so that a lane
//            holds 4 consecutive tokens x 8 dimensions, decodes them into 8 MFMA operands,
//            and 2 x 8 MFMAs (softmax weights as an fp16 high part and the fp16 remainder, into
//            the same accumulators) add p.V^.
// Which MFMA: v_mfma_f32_4x4x4_16b_f16 for up to 4 query heads per kv head, the 16 x 16 x 16
// form for 5 .. 16 (see attend_task).  head_dim 256 is two slabs, head_dim 64 half a one.
// 2-bit spans, most of a card at low budgets, are not decoded by arithmetic: a group has only
// four decoded values, which are computed once, and a selector table in LDS indexed by a byte of
// four codes drives v_perm_b32 to pick them.  Rounds are taken in whole groups of 4 / 3 / 2 /
// 1 (at 2 / 4 / 8 / 16 bits) without a branch in between; rounds past a task's end see zeros and
// count as -inf.  About 106 registers (head_dim 256: up to 128) and 10 KiB of LDS per wave: four
// waves per SIMD.

#include <atomic>

#include "qkv_common.h"
#include "qkv_decode.h"

namespace qkv {
namespace {

typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kRoundTokens = 16;
constexpr int kAttendWaves = 1;              // waves per workgroup (they would not interact): one keeps every LDS address an immediate
// Rounds whose loads are in flight ahead of the arithmetic: as many as the registers allow
// (a fetched span is 3 / 5 / 9 / 16 registers at 2 / 4 / 8 / 16 bits).
template <int W> struct Prefetch { static constexpr int kRounds = (W == 2) ? 4 : (W == 4) ? 3 : (W == 8) ? 2 : 1; };
constexpr int kLdsFloatsPerWave = 1536;      // scores of one task: chunk tokens x padded query heads (6 KiB)

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
  uint32_t* valid;         // one word of the workspace: 1 when the header was accepted
};

template <int W, int G>
struct SpanData {
  uint32_t cw[W == 16 ? 16 : W];
  uint32_t pair;
};

// Where lane (n, kq) finds its span in round 0 of a task; every round is 16 rows further.
struct LanePtrs {
  const uint8_t* codes;    // packed codes (or the raw fp16 span)
  const uint8_t* pair;     // the group's (scale, zero)
};

// DS = spans of 32 values per token (head_dim / 32); sq = which of them, 0 .. DS - 1.
template <int W, int G, int DS>
__device__ inline LanePtrs lane_pointers(const uint8_t* card, const CardGeom& g, int c, uint64_t row0, uint32_t n,
                                         uint32_t sq) {
  constexpr int GS = G / 32;
  const uint64_t gsp = (row0 + n) * DS + sq;
  LanePtrs p;
  if (W == 16) {
    p.codes = card + g.off_fp16 + gsp * 64u;
    p.pair = nullptr;
  } else {
    p.codes = card + g.off_codes[c] + gsp * (4u * W);
    p.pair = card + g.off_meta[c] + (gsp / GS) * 4u;
  }
  return p;
}

// Issues the loads of the lane's span in round rd; nothing is decoded yet.  Zeros when !valid.
template <int W, int G, int DS>
__device__ inline SpanData<W, G> fetch_span(const LanePtrs& p, uint32_t rd, bool valid) {
  constexpr int GS = G / 32;
  constexpr int NW = (W == 16) ? 16 : W;
  SpanData<W, G> d;
#pragma unroll
  for (int i = 0; i < NW; ++i) d.cw[i] = 0;
  d.pair = 0;
  if (valid) {
    const uint8_t* src = p.codes + (uint64_t)rd * (kRoundTokens * DS * 4u * W);    // 16 rows of DS spans of 4 W bytes
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
    if (W != 16) d.pair = *reinterpret_cast<const uint32_t*>(p.pair + (uint64_t)rd * (kRoundTokens * DS * 4u / GS));
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

template <int G>
__device__ inline void decode_fetched_select(const SpanData<2, G>& d, const uint8_t* table, uint32_t (&out)[16]) {
  decode_span2_select(d.cw, half_bits_to_float(d.pair & 0xFFFFu), half_bits_to_float(d.pair >> 16), table, out);
}

// ---- value pass helpers -----------------------------------------------------------------------
//
// For the weighted sum the MFMA contracts over tokens, so a lane must hold, for one output
// dimension, the values of four consecutive tokens.  The round's 16 rows are therefore loaded
// as they lie (lane (n, kq) = token n, quarter kq), dropped into LDS still packed, and picked
// up again by lane (a, kt) as the pieces "token 4 kt + i, dimensions 8 a .. 8 a + 7", i = 0..3.
// Operand e of the round is then B_e[token][a] = V^[token][8 a + e], and eight MFMAs give
// out[head][8 a + e] for 16 heads at once.  Only packed codes cross LDS, never decoded values.

template <int W> struct Piece { uint32_t w[W == 16 ? 4 : (W == 8 ? 2 : 1)]; };

// float values of the 8 codes of pieces i0 and i0+1 (W = 2: two 16-bit pieces share the masks)
template <int W>
__device__ inline void piece_codes(const Piece<W>& p0, const Piece<W>& p1, float (&c0)[8], float (&c1)[8]) {
  if constexpr (W == 2) {
    const uint32_t both = (p0.w[0] & 0xFFFFu) | (p1.w[0] << 16);
#pragma unroll
    for (int k = 0; k < 4; ++k) {                       // byte layout of m: [p0 code k, p0 code 4+k, p1 code k, p1 code 4+k]
      const uint32_t m = (both >> (2 * k)) & 0x03030303u;
      c0[k] = byte_to_float(m, 0); c0[4 + k] = byte_to_float(m, 1);
      c1[k] = byte_to_float(m, 2); c1[4 + k] = byte_to_float(m, 3);
    }
  } else if constexpr (W == 4) {
    const uint32_t e0 = p0.w[0] & 0x0F0F0F0Fu, o0 = (p0.w[0] >> 4) & 0x0F0F0F0Fu;
    const uint32_t e1 = p1.w[0] & 0x0F0F0F0Fu, o1 = (p1.w[0] >> 4) & 0x0F0F0F0Fu;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      c0[2 * j] = byte_to_float(e0, j); c0[2 * j + 1] = byte_to_float(o0, j);
      c1[2 * j] = byte_to_float(e1, j); c1[2 * j + 1] = byte_to_float(o1, j);
    }
  } else {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      c0[j] = byte_to_float(p0.w[0], j); c0[4 + j] = byte_to_float(p0.w[1], j);
      c1[j] = byte_to_float(p1.w[0], j); c1[4 + j] = byte_to_float(p1.w[1], j);
    }
  }
}

// fp16(fma(c0, s0, z0)) | fp16(fma(c1, s1, z1)) << 16: the two roundings of the decoder, two tokens at once
__device__ inline uint32_t decode_two_tokens(float c0, float s0, float z0, float c1, float s1, float z1) {
  float x = __builtin_fmaf(c0, s0, z0);
  float y = __builtin_fmaf(c1, s1, z1);
  asm("" : "+v"(x));
  asm("" : "+v"(y));
  const f32x2 v = {x, y};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, f16x2));
}

// ---- the LDS tile of a round: 16 packed rows, regrouped ------------------------------------------
//
// Used for the value rows of every card and for the key rows of cards grouped per channel.  In both
// cases the MFMA contracts over the tile's rows, so a lane must hold four consecutive rows of one
// column; the loader lane (n, kq) holds row n, columns 32 kq .. 32 kq + 31.

// one row's pitch in the tile; rows of 32 / 64 bytes get a pitch of 40 / 80 so that the four rows a read
// instruction touches (4 apart) fall on different banks.  Behind the rows, as [quarter][row]: the
// 4 x 16 pairs (2-bit rows: 4 x 16 four-value tables), and at 2 bits the 2 KiB selector table.
template <int W> struct TileGeo {
  static constexpr uint32_t kRowBytes = (W == 2) ? 40u : (W == 4) ? 80u : 16u * W;
  static constexpr uint32_t kPairsAt = (W == 16) ? 0u : 16u * kRowBytes;
};

// Loader side: lane (n, kq) drops its fetched span and the span's pair into the tile.
template <int W, int G>
__device__ inline void stage_span(const SpanData<W, G>& d, uint8_t* tile, uint32_t n, uint32_t kq) {
  uint32_t* pairs_lds = reinterpret_cast<uint32_t*>(tile + TileGeo<W>::kPairsAt);
  uint8_t* dst = tile + n * TileGeo<W>::kRowBytes + kq * (4u * W);
  if constexpr (W == 2) {
    *reinterpret_cast<u32x2*>(dst) = (u32x2){d.cw[0], d.cw[1]};
  } else {
#pragma unroll
    for (int h = 0; h < (W == 16 ? 16 : W) / 4; ++h)
      reinterpret_cast<u32x4*>(dst)[h] = (u32x4){d.cw[4 * h], d.cw[4 * h + 1], d.cw[4 * h + 2], d.cw[4 * h + 3]};
  }
  if constexpr (W == 2) {
    // the span's four decoded values instead of its (scale, zero): x_k = fp16(fma(k, scale, zero))
    const float s = half_bits_to_float(d.pair & 0xFFFFu);
    const float z = half_bits_to_float(d.pair >> 16);
    reinterpret_cast<u32x2*>(pairs_lds)[kq * 16u + n] = (u32x2){decode_pair(0.0f, 1.0f, s, z), decode_pair(2.0f, 3.0f, s, z)};
  } else if constexpr (W != 16) {
    pairs_lds[kq * 16u + n] = d.pair;
  }
}

// Reader side: lane (a, kt) picks up the pieces "rows 4 kt + i, columns 8 a .. 8 a + 7", i = 0 .. 3, and decodes
// them into the eight operands b[e] = {X[4kt][8a+e], X[4kt+1][8a+e], X[4kt+2][8a+e], X[4kt+3][8a+e]}.
template <int W>
__device__ inline void operands_from_tile(const uint8_t* tile, const uint8_t* table, uint32_t a, uint32_t kt, u32x2 (&b)[8]) {
  constexpr uint32_t kRowBytes = TileGeo<W>::kRowBytes;
  const uint32_t* pairs_lds = reinterpret_cast<const uint32_t*>(tile + TileGeo<W>::kPairsAt);
  if constexpr (W == 2) {
    // by selection: the piece's two code bytes index the selector table, the selectors pick the
    // values out of the row's four; then pairs of columns are turned into pairs of rows
    uint32_t tv[4][4];                     // row i, column pair m: {X[8a+2m], X[8a+2m+1]}
    const u32x4* xs = reinterpret_cast<const u32x4*>(pairs_lds) + ((a >> 2) * 16u + 4u * kt) / 2u;
    const u32x4 x01 = xs[0], x23 = xs[1];  // the four-value tables of rows 4 kt .. 4 kt + 3 for this lane's columns
    const uint32_t xl[4] = {x01.x, x01.z, x23.x, x23.z}, xh[4] = {x01.y, x01.w, x23.y, x23.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const uint32_t piece = *reinterpret_cast<const uint16_t*>(tile + (4u * kt + i) * kRowBytes + a * 2u);
      const u32x2 s0 = *reinterpret_cast<const u32x2*>(table + byte_times8<0>(piece));
      const u32x2 s1 = *reinterpret_cast<const u32x2*>(table + byte_times8<1>(piece));
      tv[i][0] = __builtin_amdgcn_perm(xh[i], xl[i], s0.x);
      tv[i][1] = __builtin_amdgcn_perm(xh[i], xl[i], s0.y);
      tv[i][2] = __builtin_amdgcn_perm(xh[i], xl[i], s1.x);
      tv[i][3] = __builtin_amdgcn_perm(xh[i], xl[i], s1.y);
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const uint32_t sel = (e & 1) ? 0x07060302u : 0x05040100u;      // high or low halves of two words
      b[e].x = __builtin_amdgcn_perm(tv[1][e >> 1], tv[0][e >> 1], sel);
      b[e].y = __builtin_amdgcn_perm(tv[3][e >> 1], tv[2][e >> 1], sel);
    }
  } else {
    Piece<W> pc[4];
    uint32_t pr[4] = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const uint8_t* src = tile + (4u * kt + i) * kRowBytes + a * W;
      if constexpr (W == 2) pc[i].w[0] = *reinterpret_cast<const uint16_t*>(src);
      else if constexpr (W == 4) pc[i].w[0] = *reinterpret_cast<const uint32_t*>(src);
      else if constexpr (W == 8) { const u32x2 t = *reinterpret_cast<const u32x2*>(src); pc[i].w[0] = t.x; pc[i].w[1] = t.y; }
      else { const u32x4 t = *reinterpret_cast<const u32x4*>(src); pc[i].w[0] = t.x; pc[i].w[1] = t.y; pc[i].w[2] = t.z; pc[i].w[3] = t.w; }
    }
    if constexpr (W != 16) {
      const u32x4 t = *reinterpret_cast<const u32x4*>(pairs_lds + (a >> 2) * 16u + 4u * kt);
      pr[0] = t.x; pr[1] = t.y; pr[2] = t.z; pr[3] = t.w;
    }
    if constexpr (W == 16) {
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const uint32_t sel = (e & 1) ? 0x07060302u : 0x05040100u;      // high or low halves of two words
        b[e].x = __builtin_amdgcn_perm(pc[1].w[e >> 1], pc[0].w[e >> 1], sel);
        b[e].y = __builtin_amdgcn_perm(pc[3].w[e >> 1], pc[2].w[e >> 1], sel);
      }
    } else {
      float c0[8], c1[8], c2[8], c3[8];
      piece_codes<W>(pc[0], pc[1], c0, c1);
      piece_codes<W>(pc[2], pc[3], c2, c3);
      const float s0 = half_bits_to_float(pr[0] & 0xFFFFu), z0 = half_bits_to_float(pr[0] >> 16);
      const float s1 = half_bits_to_float(pr[1] & 0xFFFFu), z1 = half_bits_to_float(pr[1] >> 16);
      const float s2 = half_bits_to_float(pr[2] & 0xFFFFu), z2 = half_bits_to_float(pr[2] >> 16);
      const float s3 = half_bits_to_float(pr[3] & 0xFFFFu), z3 = half_bits_to_float(pr[3] >> 16);
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        b[e].x = decode_two_tokens(c0[e], s0, z0, c1[e], s1, z1);
        b[e].y = decode_two_tokens(c2[e], s2, z2, c3[e], s3, z3);
      }
    }
  }
}

// ---- cross-lane helpers ------------------------------------------------------------------------

template <int CTRL>
__device__ inline float dpp_move(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, false));
}
// maximum / sum over the 16 lanes of a row, left in every lane of the row (row_ror: 8, 4, 2, 1)
__device__ inline float row_max16(float v) {
  v = fmaxf(v, dpp_move<0x128>(v));
  v = fmaxf(v, dpp_move<0x124>(v));
  v = fmaxf(v, dpp_move<0x122>(v));
  return fmaxf(v, dpp_move<0x121>(v));
}
__device__ inline float row_sum16(float v) {
  v += dpp_move<0x128>(v);
  v += dpp_move<0x124>(v);
  v += dpp_move<0x122>(v);
  return v + dpp_move<0x121>(v);
}

// Lane (n, kq) holds four partial sums a_r, one per head r, each to be added up over the four
// lanes (n, 0 .. 3); returns in lane (n, kq) the total of head kq.  v_permlane32_swap hands the
// lower half of the wave its partner's first operand and the upper half its partner's second
// one; v_permlane16_swap does the same between neighbouring rows of 16.
__device__ inline float sum_over_quarters(float a0, float a1, float a2, float a3) {
  const auto s02 = __builtin_amdgcn_permlane32_swap(__builtin_bit_cast(uint32_t, a0), __builtin_bit_cast(uint32_t, a2), false, false);
  const uint32_t s02x = s02[0], s02y = s02[1];
  const float u0 = __builtin_bit_cast(float, s02x) + __builtin_bit_cast(float, s02y);      // heads 0 | 2
  const auto s13 = __builtin_amdgcn_permlane32_swap(__builtin_bit_cast(uint32_t, a1), __builtin_bit_cast(uint32_t, a3), false, false);
  const uint32_t s13x = s13[0], s13y = s13[1];
  const float u1 = __builtin_bit_cast(float, s13x) + __builtin_bit_cast(float, s13y);      // heads 1 | 3
  const auto sr = __builtin_amdgcn_permlane16_swap(__builtin_bit_cast(uint32_t, u0), __builtin_bit_cast(uint32_t, u1), false, false);
  const uint32_t srx = sr[0], sry = sr[1];
  return __builtin_bit_cast(float, srx) + __builtin_bit_cast(float, sry);
}

// ---- score pass over key planes grouped per channel ---------------------------------------------
//
// Uniform cards with group size 32 whose key spans hold the 32 tokens of one token block for ONE
// channel (section layout [plane][token block][channel][32 codes]).  The contraction over the head
// dimension then runs over the card's rows, exactly as the value pass contracts over tokens, and the
// same tile does the regrouping: a round is 16 channels x 4 token blocks (a super-block of 128
// tokens); loader lane (n, kq) fetches channel 16 r + n of token block kq, reader lane (a, kt) gets
// "channels 16 r + 4 kt .. + 3, tokens 8 a .. 8 a + 7 of the super-block" as eight operands, and
// the other MFMA operand is q[head][16 r + 4 kt .. + 3], exact in fp16 (one MFMA per operand).
// After head_dim / 16 rounds the lane holds the scores of its eight tokens: summed over its own
// channels only when NARROW (sum_over_quarters adds the four kt and leaves head kt), complete
// otherwise (the 16 x 16 x 16 product adds the four kt itself; the lane holds heads 4 kt .. + 3).
template <int W, bool NARROW, int DS>
__device__ inline void score_pass_kc(const AttendArgs& a, const CardGeom& g, int c, uint32_t pair, uint32_t j0, uint32_t cnt,
                                     uint32_t slots, uint32_t lane, float* lds, uint32_t pitch, uint32_t R4, uint8_t* tile,
                                     const uint8_t* table) {
  static_assert(W == 2 || W == 4 || W == 8, "per-channel key groups exist at 2, 4 and 8 bits");
  constexpr uint32_t D = 32u * DS;
  constexpr int kRounds = (int)D / 16;                      // rounds per super-block
  constexpr int kAhead = (W == 2) ? 4 : 2;                  // rounds whose loads are in flight; divides kRounds
  const uint32_t n = lane & 15u, kq = lane >> 4;
  const uint32_t R = a.rep;
  const uint32_t head = NARROW ? (n & 3u) : n;
  f16x4 qa[kRounds];
  {
    const uint32_t l = pair / g.kv_heads, hh = pair - l * g.kv_heads;
    const uint16_t* src = a.q + ((uint64_t)(l * a.q_heads + hh * R + (head < R ? head : 0u)) * D + 4u * kq);
#pragma unroll
    for (int r = 0; r < kRounds; ++r) {
      u32x2 raw = (u32x2)(0u);
      if (head < R) raw = *reinterpret_cast<const u32x2*>(src + 16 * r);
      qa[r] = __builtin_bit_cast(f16x4, raw);
    }
  }
  // first group (token block, channel 0) of the task's key plane: blocks of 32 tokens, head_dim groups each
  const uint64_t grp0 = ((uint64_t)pair * (g.tokens / 32u) + j0 / 32u) * D;
  const uint8_t* codes0 = a.card + g.off_codes[c];
  const uint8_t* pairs0 = a.card + g.off_meta[c];
  const auto fetch = [&](uint32_t sb, uint32_t r) {
    SpanData<W, 32> d;
#pragma unroll
    for (int i = 0; i < W; ++i) d.cw[i] = 0;
    d.pair = 0;
    const uint32_t tb = 4u * sb + kq;                        // token block inside the task
    if (32u * tb < cnt) {
      const uint64_t grp = grp0 + (uint64_t)tb * D + 16u * r + n;
      const uint8_t* src = codes0 + grp * (4u * W);
      if constexpr (W == 2) {
        const u32x2 t = *reinterpret_cast<const u32x2*>(src);
        d.cw[0] = t.x; d.cw[1] = t.y;
      } else {
#pragma unroll
        for (int h = 0; h < W / 4; ++h) {
          const u32x4 t = *reinterpret_cast<const u32x4*>(src + 16 * h);
          d.cw[4 * h] = t.x; d.cw[4 * h + 1] = t.y; d.cw[4 * h + 2] = t.z; d.cw[4 * h + 3] = t.w;
        }
      }
      d.pair = *reinterpret_cast<const uint32_t*>(pairs0 + grp * 4u);
    }
    return d;
  };
  SpanData<W, 32> buf[kAhead];
#pragma unroll
  for (int u = 0; u < kAhead; ++u) buf[u] = fetch(0u, (uint32_t)u);
  // every slot the softmax will read gets a value: `slots` is the task's token count rounded up to the softmax's
  // own granularity (at most the pitch), which can reach into a super-block that holds no token
  const uint32_t superblocks = (slots + 127u) / 128u;
  for (uint32_t sb = 0; sb < superblocks; ++sb) {
    f32x4 acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int r = 0; r < kRounds; ++r) {
      stage_span<W, 32>(buf[r % kAhead], tile, n, kq);
      buf[r % kAhead] = (r + kAhead < kRounds) ? fetch(sb, (uint32_t)(r + kAhead)) : fetch(sb + 1u, (uint32_t)(r + kAhead - kRounds));
      u32x2 b[8];
      operands_from_tile<W>(tile, table, n, kq, b);
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const f16x4 be = __builtin_bit_cast(f16x4, b[e]);
        if constexpr (NARROW) acc[e] = __builtin_amdgcn_mfma_f32_4x4x4f16(qa[r], be, acc[e], 0, 0, 0);
        else acc[e] = __builtin_amdgcn_mfma_f32_16x16x16f16(qa[r], be, acc[e], 0, 0, 0);
      }
    }
    // tokens 128 sb + 8 a + e, e = 0 .. 7, of this lane
    const uint32_t t0 = 128u * sb + 8u * n;
    if constexpr (NARROW) {
      float sc[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float v = sum_over_quarters(acc[e].x, acc[e].y, acc[e].z, acc[e].w);      // head kq
        sc[e] = (t0 + e < cnt) ? v * a.scale_log2 : -INFINITY;
      }
      float* dst = lds + kq * pitch + t0;
      if (t0 < pitch) *reinterpret_cast<f32x4*>(dst) = (f32x4){sc[0], sc[1], sc[2], sc[3]};
      if (t0 + 4u < pitch) *reinterpret_cast<f32x4*>(dst + 4) = (f32x4){sc[4], sc[5], sc[6], sc[7]};
    } else {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const uint32_t r = 4u * kq + i;                      // the lane holds heads 4 kq .. 4 kq + 3
        if (r < R4) {
          float sc[8];
#pragma unroll
          for (int e = 0; e < 8; ++e) sc[e] = (t0 + e < cnt) ? acc[e][i] * a.scale_log2 : -INFINITY;
          float* dst = lds + r * pitch + t0;
          if (t0 < pitch) *reinterpret_cast<f32x4*>(dst) = (f32x4){sc[0], sc[1], sc[2], sc[3]};
          if (t0 + 4u < pitch) *reinterpret_cast<f32x4*>(dst + 4) = (f32x4){sc[4], sc[5], sc[6], sc[7]};
        }
      }
    }
  }
}

// One task: rows [j0, j1) of class c for the pair (layer, kv head) = pair.
// lds: scores / weights as [head][chunk] floats (R4 * chunk <= kLdsFloatsPerWave);
// tile: the round's packed rows (16 tokens x up to 256 bytes) followed by the rows' pairs.
//
// NARROW (at most 4 query heads per kv head, the grouped-query case): the contractions run on
// v_mfma_f32_4x4x4_16b_f16, sixteen independent 4 x 4 x 4 products per instruction, at half the
// cycles of the 16 x 16 x 16 form, whose rows 4 .. 15 would be idle.  Block b = lanes 4 b .. 4 b + 3;
// a lane gives row (lane % 4) of A and column (lane % 4) of B, and gets column (lane % 4) of the
// block's product, one row per register.
//   scores   A = q[head n % 4][4 dimensions], B = K^[token n][the same 4 dimensions]: the lane gets
//            the scores of its token n against the four heads, summed over its quarter kq of the
//            head dimension only; sum_over_quarters finishes the sum and leaves lane (n, kq)
//            with head kq, which it stores.
//   values   A = weights[head a % 4][tokens 4 kt .. + 3], B = V^[those tokens][dimension 8 a + e]:
//            the lane accumulates, over its own four tokens of every round, out[4 heads][8 a + e];
//            the four kt are added up once, at the end of the task.
// Otherwise (5 .. 16 query heads per kv head) the 16 x 16 x 16 form is used with the tokens as rows
// of the score product, so that a lane ends up with four consecutive tokens of one head.
//
// DS = head_dim / 32 spans per token.  The lane mapping covers a slab of 128 dimensions (4 spans);
// head_dim 256 is two slabs (the score of a round adds both up before it is stored, the value
// pass sweeps the task once per slab), head_dim 64 half a slab (quarters 2 and 3 see zeros).
template <int W, int G, bool NARROW, int DS, bool KC>
__device__ inline void attend_task(const AttendArgs& a, const CardGeom& g, int c, uint32_t pair, uint32_t j0, uint32_t j1,
                                   uint32_t lane, float* lds, uint8_t* tile, const uint8_t* table, uint64_t part) {
  const uint32_t n = lane & 15u, kq = lane >> 4;          // also (a, kt) of the value pass
  const uint32_t R = a.rep, R4 = NARROW ? 4u : ((R + 3u) & ~3u);
  const uint32_t chunk = a.chunk % 192u == 0u ? a.chunk : 96u;      // LDS pitch of a head's scores: the task size, padded
  const uint32_t lh = g.planes >> 1;
  const uint32_t n_c = g.n[c];
  const uint64_t k_row0 = (uint64_t)pair * n_c;            // K plane p = pair, V plane p = L*H + pair
  const uint64_t v_row0 = (uint64_t)(lh + pair) * n_c;
  const uint32_t cnt = j1 - j0;
  const uint32_t rounds = (cnt + kRoundTokens - 1) / kRoundTokens;
  constexpr int kPrefetch = (DS > 4 && W >= 8) ? 1 : Prefetch<W>::kRounds;     // two slabs in flight cost twice the registers
  constexpr int S = (DS + 3) / 4;                          // slabs of 128 dimensions
  constexpr uint32_t D = 32u * DS;
  const bool lane_has_span = DS >= 4 || kq < (uint32_t)DS; // head_dim 64: quarters 2 and 3 hold nothing
  // Rounds are processed in whole groups of kPrefetch; the task size is a multiple of such a group, so the padded
  // rounds stay inside the task's share of LDS.  The softmax covers `slots` tokens, those past the task's end at -inf.
  const uint32_t slots = (rounds + kPrefetch - 1) / kPrefetch * kPrefetch * kRoundTokens;
  if constexpr (KC) {
    if constexpr (W != 16 && G == 32 && DS <= 4)
      score_pass_kc<W, NARROW, DS>(a, g, c, pair, j0, cnt, slots, lane, lds, chunk, R4, tile, table);
  } else {
    LanePtrs kp[S];
#pragma unroll
    for (int sl = 0; sl < S; ++sl) kp[sl] = lane_pointers<W, G, DS>(a.card, g, c, k_row0 + j0, n, lane_has_span ? 4u * sl + kq : 0u);

    // ---- q as MFMA operands: the lane holds q[head][128 sl + 32 kq .. + 31] of head n (head n % 4 when
    // NARROW); operand j of slab sl is q[head][128 sl + 32 kq + 4 j .. + 3]
    f16x4 qa[S][8];
#pragma unroll
    for (int sl = 0; sl < S; ++sl) {
      u32x4 raw[4];
#pragma unroll
      for (int h = 0; h < 4; ++h) raw[h] = (u32x4)(0u);
      const uint32_t head = NARROW ? (n & 3u) : n;
      if (head < R && lane_has_span) {
        const uint32_t l = pair / g.kv_heads, hh = pair - l * g.kv_heads;
        const u32x4* src = reinterpret_cast<const u32x4*>(a.q + ((uint64_t)(l * a.q_heads + hh * R + head) * D + 128u * sl + 32u * kq));
#pragma unroll
        for (int h = 0; h < 4; ++h) raw[h] = src[h];
      }
#pragma unroll
      for (int h = 0; h < 4; ++h) {
        qa[sl][2 * h] = __builtin_bit_cast(f16x4, (u32x2){raw[h].x, raw[h].y});
        qa[sl][2 * h + 1] = __builtin_bit_cast(f16x4, (u32x2){raw[h].z, raw[h].w});
      }
    }

    // ---- scores: lds[head * chunk + token] in log2 units, -inf for tokens past the task's end.
    // The loads of the next kPrefetch rounds are always in flight.
    {
      SpanData<W, G> buf[kPrefetch][S];
#pragma unroll
      for (int u = 0; u < kPrefetch; ++u) {
        const uint32_t t = u * kRoundTokens + n;
#pragma unroll
        for (int sl = 0; sl < S; ++sl) buf[u][sl] = fetch_span<W, G, DS>(kp[sl], u, t < cnt && lane_has_span);
      }
      for (uint32_t rd0 = 0; rd0 < rounds; rd0 += kPrefetch) {
#pragma unroll
        for (int u = 0; u < kPrefetch; ++u) {
          const uint32_t rd = rd0 + u;
          {                                          // rounds past the task's end see zeros and store -inf
            f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int sl = 0; sl < S; ++sl) {
              uint32_t kb[16];
              if constexpr (W == 2) decode_fetched_select<G>(buf[u][sl], table, kb);
              else decode_fetched<W, G>(buf[u][sl], kb);
              const uint32_t tn = (rd + kPrefetch) * kRoundTokens + n;
              buf[u][sl] = fetch_span<W, G, DS>(kp[sl], rd + kPrefetch, tn < cnt && lane_has_span);
#pragma unroll
              for (int j = 0; j < 8; ++j) {
                const f16x4 kj = __builtin_bit_cast(f16x4, (u32x2){kb[2 * j], kb[2 * j + 1]});
                if constexpr (NARROW) acc = __builtin_amdgcn_mfma_f32_4x4x4f16(qa[sl][j], kj, acc, 0, 0, 0);
                else acc = __builtin_amdgcn_mfma_f32_16x16x16f16(kj, qa[sl][j], acc, 0, 0, 0);
              }
            }
            if constexpr (NARROW) {
              // head kq of token n
              const float sc = sum_over_quarters(acc.x, acc.y, acc.z, acc.w);
              const uint32_t t = rd * kRoundTokens + n;
              lds[kq * chunk + t] = (t < cnt) ? sc * a.scale_log2 : -INFINITY;
            } else {
              // tokens 4 kq .. 4 kq + 3 of head n
              const uint32_t t = rd * kRoundTokens + 4u * kq;
              if (n < R4) {
                f32x4 sc;
                sc.x = (t < cnt) ? acc.x * a.scale_log2 : -INFINITY;
                sc.y = (t + 1u < cnt) ? acc.y * a.scale_log2 : -INFINITY;
                sc.z = (t + 2u < cnt) ? acc.z * a.scale_log2 : -INFINITY;
                sc.w = (t + 3u < cnt) ? acc.w * a.scale_log2 : -INFINITY;
                *reinterpret_cast<f32x4*>(lds + n * chunk + t) = sc;
              }
            }
          }
        }
      }
    }

  }   // per-token key groups

  // ---- softmax over the task's tokens, four heads at a time: row kq of the wave takes head
  // 4 hg + kq, its lane n the tokens 64 i + 4 n .. + 3 (the wave's own LDS accesses are in order).
  // the first value rows are requested now, so that they arrive while the softmax runs
  LanePtrs vp = lane_pointers<W, G, DS>(a.card, g, c, v_row0 + j0, n, lane_has_span ? kq : 0u);
  SpanData<W, G> vbuf[kPrefetch];
#pragma unroll
  for (int u = 0; u < kPrefetch; ++u) {
    const uint32_t t = u * kRoundTokens + n;
    vbuf[u] = fetch_span<W, G, DS>(vp, u, t < cnt && lane_has_span);
  }
  for (uint32_t hg = 0; hg < R4; hg += 4u) {
    const uint32_t r = hg + kq;
    float* row = lds + r * chunk;
    float m = -INFINITY;
    for (uint32_t t = 4u * n; t < slots; t += 64u) {
      const f32x4 sv = *reinterpret_cast<const f32x4*>(row + t);
      m = fmaxf(fmaxf(m, fmaxf(sv.x, sv.y)), fmaxf(sv.z, sv.w));
    }
    m = row_max16(m);
    float l = 0.f;
    for (uint32_t t = 4u * n; t < slots; t += 64u) {
      const f32x4 sv = *reinterpret_cast<const f32x4*>(row + t);
      u32x4 packed;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float p = __builtin_amdgcn_exp2f(sv[i] - m);
        l += p;
        // what the value pass feeds the MFMA: p * 2^14 as an fp16 high part plus the fp16 remainder (both go
        // into the same accumulator; the remainder is a normal number for any p that matters), packed into
        // the score's slot
        const float ps = p * 16384.0f;
        const _Float16 hi = (_Float16)ps;
        const _Float16 lo = (_Float16)(ps - (float)hi);
        packed[i] = (uint32_t)__builtin_bit_cast(uint16_t, hi) | ((uint32_t)__builtin_bit_cast(uint16_t, lo) << 16);
      }
      *reinterpret_cast<u32x4*>(row + t) = packed;
    }
    l = row_sum16(l);
    if (n == 0 && r < R) {
      a.part_ml[(part * R + r) * 2] = m;
      a.part_ml[(part * R + r) * 2 + 1] = l;
    }
  }

  // ---- values
  const uint32_t w_head = NARROW ? (n & 3u) : n;            // the head whose weights this lane feeds the MFMA
  // one sweep over the task's rows per slab of 128 output dimensions (the weights stay in LDS)
#pragma unroll 1
  for (int sl = 0; sl < S; ++sl) {
    if (sl > 0) {
      vp = lane_pointers<W, G, DS>(a.card, g, c, v_row0 + j0, n, 4u * sl + kq);
#pragma unroll
      for (int u = 0; u < kPrefetch; ++u) {
        const uint32_t t = u * kRoundTokens + n;
        vbuf[u] = fetch_span<W, G, DS>(vp, u, t < cnt);
      }
    }
    f32x4 acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = (f32x4){0.f, 0.f, 0.f, 0.f};
    {
      SpanData<W, G> (&buf)[kPrefetch] = vbuf;
      for (uint32_t rd0 = 0; rd0 < rounds; rd0 += kPrefetch) {
#pragma unroll
        for (int u = 0; u < kPrefetch; ++u) {
          const uint32_t rd = rd0 + u;
          {                                          // rounds past the task's end add zero weights times zeros
            // rows into LDS as they were loaded: token n, quarter kq
            stage_span<W, G>(buf[u], tile, n, kq);
            const uint32_t tn = (rd + kPrefetch) * kRoundTokens + n;
            buf[u] = fetch_span<W, G, DS>(vp, rd + kPrefetch, tn < cnt && lane_has_span);

            // lane (a, kt) = (n, kq): b[e] = {V^[4kt][8a+e], V^[4kt+1][8a+e], V^[4kt+2][8a+e], V^[4kt+3][8a+e]}
            u32x2 b[8];
            operands_from_tile<W>(tile, table, n, kq, b);
            // A operands: the weights of head w_head for tokens 4 kt .. 4 kt + 3, high parts and low parts
            u32x4 pw = (u32x4)(0u);
            if (w_head < R4) pw = *reinterpret_cast<const u32x4*>(lds + w_head * chunk + rd * kRoundTokens + 4u * kq);
            const f16x4 a_hi = __builtin_bit_cast(f16x4, (u32x2){__builtin_amdgcn_perm(pw.y, pw.x, 0x05040100u),
                                                                 __builtin_amdgcn_perm(pw.w, pw.z, 0x05040100u)});
            const f16x4 a_lo = __builtin_bit_cast(f16x4, (u32x2){__builtin_amdgcn_perm(pw.y, pw.x, 0x07060302u),
                                                                 __builtin_amdgcn_perm(pw.w, pw.z, 0x07060302u)});
#pragma unroll
            for (int e = 0; e < 8; ++e) {
              const f16x4 be = __builtin_bit_cast(f16x4, b[e]);
              if constexpr (NARROW) {
                acc[e] = __builtin_amdgcn_mfma_f32_4x4x4f16(a_hi, be, acc[e], 0, 0, 0);
                acc[e] = __builtin_amdgcn_mfma_f32_4x4x4f16(a_lo, be, acc[e], 0, 0, 0);
              } else {
                acc[e] = __builtin_amdgcn_mfma_f32_16x16x16f16(a_hi, be, acc[e], 0, 0, 0);
                acc[e] = __builtin_amdgcn_mfma_f32_16x16x16f16(a_lo, be, acc[e], 0, 0, 0);
              }
            }
          }
        }
      }
    }
    if constexpr (NARROW) {
      // the lane holds, for its own tokens only, out[heads 0 .. 3][dimensions 8 n .. 8 n + 7]: add up the four kt;
      // lane (n, kq) is left with head kq
      // (every lane takes part in the sums; only the stores are conditional)
      float o[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) o[e] = sum_over_quarters(acc[e].x, acc[e].y, acc[e].z, acc[e].w) * (1.0f / 16384.0f);
      if (kq < R && (DS >= 4 || n < 8u)) {          // head_dim 64: lanes n >= 8 stand for dimensions that do not exist
        f32x4* dst = reinterpret_cast<f32x4*>(a.part_o + (part * R + kq) * D + 128u * sl + 8u * n);
        dst[0] = (f32x4){o[0], o[1], o[2], o[3]};
        dst[1] = (f32x4){o[4], o[5], o[6], o[7]};
      }
    } else {
      // the lane holds out[heads 4 kq .. 4 kq + 3][dimensions 8 n .. 8 n + 7]
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const uint32_t r = 4u * kq + i;
        if (r < R && (DS >= 4 || n < 8u)) {
          float o[8];
#pragma unroll
          for (int e = 0; e < 8; ++e) o[e] = acc[e][i] * (1.0f / 16384.0f);
          f32x4* dst = reinterpret_cast<f32x4*>(a.part_o + (part * R + r) * D + 128u * sl + 8u * n);
          dst[0] = (f32x4){o[0], o[1], o[2], o[3]};
          dst[1] = (f32x4){o[4], o[5], o[6], o[7]};
        }
      }
    }
  }
}

// KC: the card's key planes are grouped per channel (a uniform card at 2, 4 or 8 bits, group size 32).
template <int G, bool NARROW, int DS, bool KC>
__global__ __launch_bounds__(kAttendWaves * kWaveSize) __attribute__((amdgpu_waves_per_eu(2)))
void attend_kernel(AttendArgs a) {
  __shared__ __attribute__((aligned(16))) float lds[kAttendWaves][kLdsFloatsPerWave];
  // the value pass's LDS, 4 KiB: 16 packed rows (640 / 1280 / 2048 / 4096 bytes at 2 / 4 / 8 / 16 bits), then the
  // rows' pairs (256 bytes; 512 bytes of four-value tables at 2 bits), then at 2 bits the 2 KiB selector table
  __shared__ __attribute__((aligned(16))) uint8_t tiles[kAttendWaves][16 * 256];
  CardGeom g;
  bool ok = card_geometry_from_header(a.card, a.card_bytes, a.layers, a.kv_heads, a.head_dim, a.group_size,
                                      a.tokens, g, KC ? QKV_FLAG_KEYS_PER_CHANNEL : 0u);
  if (KC && ok) {                              // the shapes the per-channel score pass is written for
    const bool uniform = g.n[0] == g.tokens || g.n[1] == g.tokens || g.n[2] == g.tokens;
    ok = uniform && g.group_size == 32u && g.head_dim <= 128u && g.tokens % (g.head_dim == 64u ? 64u : 32u) == 0u;
  }
  // the header's verdict, for the merging kernel that follows on the stream and for the caller
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    *a.valid = ok ? 1u : 0u;
    if (a.status) *a.status = ok ? 0u : QKV_STATUS_BAD_HEADER;
  }
  if (!ok) return;                            // uniform over the grid
  const uint32_t lane = threadIdx.x & 63u;
  const uint32_t wave = (kAttendWaves == 1) ? 0u : threadIdx.x >> 6;     // a constant keeps every LDS address an immediate
  const uint32_t gw = blockIdx.x * kAttendWaves + wave;
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
  uint8_t* my_tile = tiles[wave];
  uint8_t* my_table = my_tile + 16 * 40 + 512;
  if (cls == 0) {
    build_select_table(reinterpret_cast<u32x2*>(my_table), lane);
    attend_task<2, G, NARROW, DS, KC>(a, g, 0, pair, j0, j1, lane, my_lds, my_tile, my_table, part);
  }
  if (cls == 1) attend_task<4, G, NARROW, DS, KC>(a, g, 1, pair, j0, j1, lane, my_lds, my_tile, my_table, part);
  if (cls == 2) attend_task<8, G, NARROW, DS, KC>(a, g, 2, pair, j0, j1, lane, my_lds, my_tile, my_table, part);
  if constexpr (!KC) {                         // a card grouped per channel has no raw rows
    if (cls == 3) attend_task<16, G, NARROW, DS, false>(a, g, 3, pair, j0, j1, lane, my_lds, my_tile, my_table, part);
  }
}

// Merges the partials of one (layer, query head): thread d owns output dimension d.  The
// (m, l) pairs of all tasks are first gathered into LDS by parallel loads, so that the
// weights cost no chain of dependent global loads.
constexpr int kMergeBatch = 256;             // tasks whose (m, l) are held in LDS at a time

__global__ __launch_bounds__(256) void attend_merge_kernel(AttendArgs a) {
  __shared__ float ml_m[kMergeBatch], ml_l[kMergeBatch];
  if (*a.valid == 0) return;                           // header refused: outputs stay untouched
  const uint32_t d = threadIdx.x, D = a.head_dim;      // one thread per output dimension
  const uint32_t lq = blockIdx.x;                      // l * Hq + hq
  const uint32_t l = lq / a.q_heads, hq = lq - l * a.q_heads;
  const uint32_t h = hq / a.rep, r = hq - h * a.rep;
  const uint64_t part0 = (uint64_t)(l * a.kv_heads + h) * a.max_tasks;
  float M = -INFINITY, den = 0.f, num = 0.f;           // running maximum, and sums relative to it
  for (uint32_t t0 = 0; t0 < a.max_tasks; t0 += kMergeBatch) {
    const uint32_t nb = min((uint32_t)kMergeBatch, a.max_tasks - t0);
    __syncthreads();
    for (uint32_t t = d; t < nb; t += D) {
      const float* ml = a.part_ml + ((part0 + t0 + t) * a.rep + r) * 2;
      ml_m[t] = ml[0];
      ml_l[t] = ml[1];
    }
    __syncthreads();
    float Mb = M;
    for (uint32_t t = 0; t < nb; ++t) if (ml_l[t] > 0.f) Mb = fmaxf(Mb, ml_m[t]);
    if (Mb == -INFINITY) continue;                     // nothing but empty tasks so far (uniform over the block)
    const float rescale = __builtin_amdgcn_exp2f(M - Mb);   // 0 when M is still -inf
    den *= rescale;
    num *= rescale;
    M = Mb;
    // loads first, unconditionally (an empty task's slot holds anything: it is read but not used)
#pragma unroll 8
    for (uint32_t t = 0; t < nb; ++t) {
      const float v = a.part_o[((part0 + t0 + t) * a.rep + r) * D + d];
      const float lt = ml_l[t];
      const float w = __builtin_amdgcn_exp2f(ml_m[t] - M);
      den += (lt > 0.f) ? w * lt : 0.f;
      num += (lt > 0.f) ? w * v : 0.f;
    }
  }
  a.out[(uint64_t)lq * D + d] = num / den;
  if (d == 0 && a.lse) a.lse[lq] = (M + __builtin_log2f(den)) * 0.69314718055994530942f;
}

}  // namespace

// Tokens per task and tasks per (layer, kv head) for a given shape.  The scores of one task (tokens x
// query heads padded to a multiple of 4) must fit the wave's 6 KiB of LDS.  Tasks are processed in groups
// of 4, 3, 2 or 1 rounds of 16 tokens, depending on the width, and a task size that all of these divide
// keeps the padded rounds inside the task's LDS: multiples of 192 tokens, or 64 tokens when fewer than
// 192 fit (a 64-token task pads to 96 at most).  The larger size means fewer partials and less per-task
// work (90 us against 96 us at 8K tokens x 256 pairs); the smaller one is taken when the larger would
// not even fill the chip's wave slots once (one wave per task, four waves per SIMD, 256 compute units).
void attend_plan(uint64_t tokens, uint32_t rep, uint64_t pairs, uint32_t* chunk, uint32_t* max_tasks) {
  const uint32_t r4 = (rep + 3u) & ~3u;
  const uint32_t room = kLdsFloatsPerWave / r4;                 // tokens whose scores fit, 96 at least
  const uint32_t limit = room >= 192u ? room / 192u * 192u : 64u;
  const uint64_t slots = 256u * 4u * 4u;
  uint32_t c = limit;
  while (c > 192u && pairs * ((tokens + c - 1) / c + 2u) < slots) c -= 192u;
  *chunk = c;
  *max_tasks = (uint32_t)((tokens + *chunk - 1) / *chunk) + 3u;   // every class may end with a partly filled task
}

// ---- scratch for callers that cannot allocate -------------------------------------------------
//
// qkv_card_attend_static keeps the partials in this array instead of a caller's workspace.  Every
// GPU the library runs on holds its own copy, at its own address, until the process ends.  In host
// code the array's name is only a handle for the runtime: the device address comes from
// hipGetSymbolAddress, once per device, and that address is what kernels and copies are given.
namespace {
constexpr uint64_t kStaticScratchBytes = QKV_ATTEND_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) float scratch[kStaticScratchBytes / sizeof(float)];
std::atomic<float*> g_scratch_at[64];        // per device ordinal, null = not looked up yet
}  // namespace

// The current device's copy of the scratch array.  Looks the address up on the first call per device.
hipError_t attend_static_scratch(float** ptr) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
  float* p = g_scratch_at[dev].load(std::memory_order_acquire);
  if (p == nullptr) {
    void* at = nullptr;
    e = hipGetSymbolAddress(&at, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (at == nullptr) return hipErrorInvalidSymbol;
    p = static_cast<float*>(at);
    g_scratch_at[dev].store(p, std::memory_order_release);
  }
  *ptr = p;
  return hipSuccess;
}

hipError_t launch_attend(const uint8_t* card, uint64_t card_bytes, const CardGeom& expect, const void* q,
                         uint32_t q_heads, float softmax_scale, float* out, float* lse, float* workspace,
                         uint32_t* status, bool keys_per_channel, hipStream_t stream) {
  AttendArgs a;
  a.card = card;
  a.card_bytes = card_bytes;
  a.layers = expect.layers; a.kv_heads = expect.kv_heads; a.head_dim = expect.head_dim; a.group_size = expect.group_size;
  a.tokens = expect.tokens;
  a.q = static_cast<const uint16_t*>(q);
  a.q_heads = q_heads;
  a.rep = q_heads / expect.kv_heads;
  a.scale_log2 = softmax_scale * 1.44269504088896340736f;
  attend_plan(expect.tokens, a.rep, (uint64_t)expect.layers * expect.kv_heads, &a.chunk, &a.max_tasks);
  const uint64_t pairs = (uint64_t)expect.layers * expect.kv_heads;
  const uint32_t D = expect.head_dim;
  a.part_o = workspace;
  a.part_ml = workspace + pairs * a.max_tasks * a.rep * D;
  a.valid = reinterpret_cast<uint32_t*>(workspace + pairs * a.max_tasks * a.rep * (D + 2u));
  a.out = out;
  a.lse = lse;
  a.status = status;
  const uint64_t waves = pairs * a.max_tasks;
  const dim3 grid((uint32_t)((waves + kAttendWaves - 1) / kAttendWaves)), block(kAttendWaves * kWaveSize);
  const bool narrow = a.rep <= 4u;             // grouped-query shapes: the 4 x 4 x 4 contraction
  const uint32_t G = expect.group_size;
#define QKV_LAUNCH_ATTEND(GG, DSS)                                                                     \
  do {                                                                                                 \
    if (narrow) hipLaunchKernelGGL((attend_kernel<GG, true, DSS, false>), grid, block, 0, stream, a);  \
    else hipLaunchKernelGGL((attend_kernel<GG, false, DSS, false>), grid, block, 0, stream, a);        \
  } while (0)
  if (keys_per_channel) {                      // the host has checked: group size 32, head_dim 64 or 128
    if (D == 64u) {
      if (narrow) hipLaunchKernelGGL((attend_kernel<32, true, 2, true>), grid, block, 0, stream, a);
      else hipLaunchKernelGGL((attend_kernel<32, false, 2, true>), grid, block, 0, stream, a);
    } else {
      if (narrow) hipLaunchKernelGGL((attend_kernel<32, true, 4, true>), grid, block, 0, stream, a);
      else hipLaunchKernelGGL((attend_kernel<32, false, 4, true>), grid, block, 0, stream, a);
    }
  } else if (D == 64u) {
    if (G == 32u) QKV_LAUNCH_ATTEND(32, 2); else QKV_LAUNCH_ATTEND(64, 2);
  } else if (D == 128u) {
    if (G == 32u) QKV_LAUNCH_ATTEND(32, 4); else if (G == 64u) QKV_LAUNCH_ATTEND(64, 4); else QKV_LAUNCH_ATTEND(128, 4);
  } else {
    if (G == 32u) QKV_LAUNCH_ATTEND(32, 8); else if (G == 64u) QKV_LAUNCH_ATTEND(64, 8); else QKV_LAUNCH_ATTEND(128, 8);
  }
#undef QKV_LAUNCH_ATTEND
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(attend_merge_kernel, dim3(expect.layers * q_heads), dim3(D), 0, stream, a);
  return hipGetLastError();
}

}  // namespace qkv
