// unpack.hip — receiver-side injection (paper Sec. 4.2.2): the card's quantized groups are
// unpacked and dequantized into a dense fp16 K/V cache, 16-bit rows are copied back.
//
// Mirror image of the packing kernel.  A wave takes a tile of 512 sixteen-byte output
// chunks (32 rows at head_dim 128) of one width's segment.  Each lane owns one span of 32
// consecutive values per round (two rounds per tile): it reads its span's packed codes
// (8 / 16 / 32 bytes, contiguous with its neighbours') and its group's (scale, zero) pair
// straight from the card, decodes 32 values, and writes the 64 bytes into LDS.  The tile is
// then read back row-major (chunk index XOR-swizzled so that both directions touch every
// bank once per pass) and stored with 128-bit writes to the rows that order[] names: every
// store instruction of a wave writes whole 256-byte rows.
//
// The card is untrusted input: the kernel rebuilds the section offsets from the header's
// class counts, checks them against the buffer size and the caller's shape, and bounds
// every order[] entry, so no access can leave the card or the output tensors.
#include "qkv_common.h"
#include "qkv_decode.h"

namespace qkv {
namespace {

struct UnpackArgs {
  const uint8_t* card;
  uint64_t card_bytes;
  uint32_t flags;                                    // the grouping the caller expects (header flags word)
  uint32_t layers, kv_heads, head_dim, group_size;   // the shape the outputs were sized for
  uint64_t tokens;
  uint8_t* k_out;
  uint8_t* v_out;
  uint32_t* status;                                  // may be null
};

// Injection into per-layer caches: the same tiles, but only the planes of a layer range,
// rows addressed through per-layer base pointers and strides, and - optionally - every key
// row rotated to a shifted position on its way out (rotary embedding, half-split pairing).
struct InjectArgs {
  const uint8_t* card;
  uint64_t card_bytes;
  uint32_t layers, kv_heads, head_dim, group_size;
  uint64_t tokens;
  uint32_t layer_begin, layer_count;
  uint64_t head_stride, token_stride;                // bytes
  uint32_t rope;                                     // 1: rotate the keys with cs[]
  uint32_t* status;                                  // may be null
  uint64_t k_layer[QKV_INJECT_MAX_LAYERS];           // where token 0 of head 0 of layer layer_begin + i goes
  uint64_t v_layer[QKV_INJECT_MAX_LAYERS];
  float cs[128][2];                                  // (cos, sin) of the shift for pair index i < head_dim / 2
};

// What a lane needs to rotate its 16-byte chunk of a key row: the (cos, sin) of its 8 elements,
// the sign of the partner term and where the partner chunk sits.
struct RopeLane {
  float c[8], s[8];
  uint32_t flip;          // 0x80000000 for the first half of a row (x c - y s), 0 for the second (x c + y s)
  uint32_t partner;       // lane distance (XOR) to the chunk holding the partner elements
};

typedef __attribute__((address_space(1))) u32x4 global_u32x4;

// LDS position (in 16-byte units) of output chunk q of a tile.
__device__ inline uint32_t swizzle(uint32_t q) { return q ^ ((q >> 3) & 3u); }

// The card's three tables must tell one story: entry j of class c's part of order[] names token t only if
// bits[t] is that class's width and slot[t] is j.  Then no token is named twice, so every output row is
// written exactly once; an entry that fails is skipped and reported like one that names no token at all.
// (t < tokens has been checked; the two look-ups hit tables of a few KiB that stay in cache.)
__device__ inline bool tables_agree(const uint8_t* card, const CardGeom& g, int c, uint32_t j, uint32_t t) {
  const uint32_t width = card[g.off_bits + t];
  const uint32_t slot = reinterpret_cast<const uint32_t*>(card + g.off_slot)[t];
  return width == width_of_class(c) && slot == j;
}

// Address of the output row that row `lane` of the tile starting at segment row r0 goes to;
// 0 for rows past the segment's end and for corrupt order[] entries.
__device__ inline uint64_t tile_row_address(const UnpackArgs& a, const CardGeom& g, int c, uint32_t r0, uint32_t n_rows,
                                            uint32_t lane, uint32_t tile_rows, uint32_t& bad) {
  uint64_t addr = 0;
  const uint32_t r = r0 + lane;
  if (lane < tile_rows && r < n_rows) {
    const uint32_t n = g.n[c];
    const uint32_t p = r / n;
    const uint32_t j = r - p * n;
    const uint32_t t = reinterpret_cast<const uint32_t*>(a.card + g.off_order)[g.base[c] + j];
    const uint32_t lh = g.planes >> 1;
    const uint32_t row_bytes = g.head_dim * 2u;
    if (t < g.tokens && tables_agree(a.card, g, c, j, t)) {
      addr = (p < lh) ? reinterpret_cast<uint64_t>(a.k_out) + ((uint64_t)p * g.tokens + t) * row_bytes
                      : reinterpret_cast<uint64_t>(a.v_out) + ((uint64_t)(p - lh) * g.tokens + t) * row_bytes;
    } else {
      bad = 1;
    }
  }
  return addr;
}

// Two elements x of a key row and their partners y: fp16( fma(x, cos, -+ fl32(y * sin)) ).  The fp32 result
// and the conversion are kept apart (see decode_pair).
__device__ inline uint32_t rotate_pair(uint32_t xd, uint32_t yd, float c0, float s0, float c1, float s1, uint32_t flip) {
  const f16x2 xh = __builtin_bit_cast(f16x2, xd), yh = __builtin_bit_cast(f16x2, yd);
  const float t0 = __uint_as_float(__float_as_uint((float)yh.x * s0) ^ flip);
  const float t1 = __uint_as_float(__float_as_uint((float)yh.y * s1) ^ flip);
  float r0 = __builtin_fmaf((float)xh.x, c0, t0);
  float r1 = __builtin_fmaf((float)xh.y, c1, t1);
  asm("" : "+v"(r0));
  asm("" : "+v"(r1));
  const f32x2 v = {r0, r1};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, f16x2));
}

__device__ inline u32x4 rotate_chunk(u32x4 x, u32x4 y, const RopeLane& r) {
  u32x4 o;
  o.x = rotate_pair(x.x, y.x, r.c[0], r.s[0], r.c[1], r.s[1], r.flip);
  o.y = rotate_pair(x.y, y.y, r.c[2], r.s[2], r.c[3], r.s[3], r.flip);
  o.z = rotate_pair(x.z, y.z, r.c[4], r.s[4], r.c[5], r.s[5], r.flip);
  o.w = rotate_pair(x.w, y.w, r.c[6], r.s[6], r.c[7], r.s[7], r.flip);
  return o;
}

// Stores the tile: chunk 64 k + lane goes to its row, rows without an address are skipped.
__device__ inline void store_tile(uint64_t my_row_addr, uint32_t lane, uint32_t lpr_shift, const u32x4 (&data)[kTileIters]) {
  const uint32_t in_row = (lane & ((1u << lpr_shift) - 1u)) * 16u;
#pragma unroll
  for (int k = 0; k < kTileIters; ++k) {
    const uint32_t src_lane = (k * kWaveSize + lane) >> lpr_shift;
    const uint32_t lo = __shfl((uint32_t)my_row_addr, src_lane, kWaveSize);
    const uint32_t hi = __shfl((uint32_t)(my_row_addr >> 32), src_lane, kWaveSize);
    const uint64_t row = ((uint64_t)hi << 32) | lo;
    if (row != 0) __builtin_nontemporal_store(data[k], reinterpret_cast<global_u32x4*>(row + in_row));
  }
}

// Decodes the tile of class c that starts at segment row r0 (rows at or past n_rows are skipped) and stores
// it to the row addresses in my_row (lane i: row r0 + i).  ROPE: rotate every row with `rope`.
template <int W, int G, bool KEEP, bool ROPE>
__device__ inline void unpack_tile(const uint8_t* card, const CardGeom& g, int c, uint32_t r0, uint32_t n_rows,
                                   uint64_t my_row, uint32_t lane, u32x4* lds, const RopeLane& rope) {
  constexpr int GS = G / 32;                     // spans (lanes) per group
  const uint32_t lpr_shift = g.lpr_shift;
  const uint32_t spr_shift = lpr_shift - 2;      // log2(spans per row)

  const uint8_t* codes_seg = card + g.off_codes[c];
  const uint32_t* meta_seg = reinterpret_cast<const uint32_t*>(card + g.off_meta[c]);
  const uint64_t span0 = (uint64_t)r0 << spr_shift;
  const uint64_t seg_spans = (uint64_t)n_rows << spr_shift;

  // both rounds' codes and pairs first, so the loads overlap
  uint32_t cw[kTileRounds][W];
  uint32_t pair[kTileRounds];
#pragma unroll
  for (int round = 0; round < kTileRounds; ++round) {
    const uint64_t gsp = span0 + round * kWaveSize + lane;
#pragma unroll
    for (int i = 0; i < W; ++i) cw[round][i] = 0;
    pair[round] = 0;
    if (gsp < seg_spans) {
      const uint8_t* src = codes_seg + gsp * (4u * W);
      if (W == 2) {
        const u32x2 t = card_load<KEEP>(reinterpret_cast<const u32x2*>(src));
        cw[round][0] = t.x; cw[round][1] = t.y;
      } else {
#pragma unroll
        for (int h = 0; h < W / 4; ++h) {
          const u32x4 t = card_load<KEEP>(reinterpret_cast<const u32x4*>(src + 16 * h));
          cw[round][4 * h] = t.x; cw[round][4 * h + 1] = t.y; cw[round][4 * h + 2] = t.z; cw[round][4 * h + 3] = t.w;
        }
      }
      pair[round] = card_load<KEEP>(meta_seg + gsp / GS);
    }
  }

  const uint32_t x = (lane >> 1) & 3u;           // swizzle term of this lane's spans
#pragma unroll
  for (int round = 0; round < kTileRounds; ++round) {
    const uint32_t sp = round * kWaveSize + lane;
    const float s = half_bits_to_float(pair[round] & 0xFFFFu);
    const float z = half_bits_to_float(pair[round] >> 16);
    uint32_t out[16];
    decode_span<W>(cw[round], s, z, out);
#pragma unroll
    for (int j = 0; j < 4; ++j) lds[4 * sp + (j ^ x)] = (u32x4){out[4 * j], out[4 * j + 1], out[4 * j + 2], out[4 * j + 3]};
  }

  u32x4 data[kTileIters];
  const uint32_t rslot = swizzle(lane);
#pragma unroll
  for (int k = 0; k < kTileIters; ++k) data[k] = lds[k * kWaveSize + rslot];
  if (ROPE) {                                    // the partner chunk of the same row, straight from LDS
    const uint32_t pslot = swizzle(lane ^ rope.partner);
#pragma unroll
    for (int k = 0; k < kTileIters; ++k) data[k] = rotate_chunk(data[k], lds[k * kWaveSize + pslot], rope);
  }
  store_tile(my_row, lane, lpr_shift, data);
}

// A tile of key rows of a uniform card with groups per channel: a lane decodes the 32 tokens of two
// neighbouring channels of one token block (their codes and pairs lie side by side in the card), turns
// "two tokens of one channel" into "two channels of one token" and drops the tile into LDS row by row:
// each of its 32 stores covers a whole row of the tile across the wave.  The tile then leaves like any
// other.  Mirror image of the packing kernel's pack_tile_kc.
template <int W, bool KEEP, bool ROPE>
__device__ inline void unpack_tile_kc(const uint8_t* card, const CardGeom& g, int c, uint32_t r0, uint32_t key_rows,
                                      uint64_t my_row, uint32_t lane, u32x4* lds, const RopeLane& rope) {
  const uint32_t lpr_shift = g.lpr_shift;
  const uint32_t D = g.head_dim;
  const uint32_t cp = lane & ((D >> 1) - 1u);               // channel pair: channels 2 cp, 2 cp + 1
  const uint32_t tbl = lane >> (lpr_shift + 2u);            // token block inside the tile (head_dim 64: two)
  const uint32_t blk = r0 / 32u + tbl;
  uint32_t cw[2][W];
  u32x2 pairs = (u32x2)(0u);
#pragma unroll
  for (int i = 0; i < W; ++i) { cw[0][i] = 0; cw[1][i] = 0; }
  if (32u * blk < key_rows) {
    const uint64_t grp = (uint64_t)blk * D + 2u * cp;       // and grp + 1
    const u32x4* src = reinterpret_cast<const u32x4*>(card + g.off_codes[c] + grp * (4u * W));
    uint32_t flat[2 * W];
#pragma unroll
    for (int h = 0; h < W / 2; ++h) {
      const u32x4 t = card_load<KEEP>(src + h);
      flat[4 * h] = t.x; flat[4 * h + 1] = t.y; flat[4 * h + 2] = t.z; flat[4 * h + 3] = t.w;
    }
#pragma unroll
    for (int i = 0; i < W; ++i) { cw[0][i] = flat[i]; cw[1][i] = flat[W + i]; }
    pairs = card_load<KEEP>(reinterpret_cast<const u32x2*>(card + g.off_meta[c]) + (grp >> 1));
  }
  uint32_t xa[16], xb[16];                                  // x[j] = tokens 2j, 2j+1 of the block, channel 2 cp / 2 cp + 1
  decode_span<W>(cw[0], half_bits_to_float(pairs.x & 0xFFFFu), half_bits_to_float(pairs.x >> 16), xa);
  decode_span<W>(cw[1], half_bits_to_float(pairs.y & 0xFFFFu), half_bits_to_float(pairs.y >> 16), xb);
  uint32_t* lds32 = reinterpret_cast<uint32_t*>(lds);
#pragma unroll
  for (int j = 0; j < 16; ++j) {
    const uint32_t qa = ((32u * tbl + 2u * j) << lpr_shift) + (cp >> 2);      // chunk of (token 2j, channels 2 cp, 2 cp + 1)
    const uint32_t qb = qa + (1u << lpr_shift);
    lds32[swizzle(qa) * 4u + (cp & 3u)] = __builtin_amdgcn_perm(xb[j], xa[j], 0x05040100u);
    lds32[swizzle(qb) * 4u + (cp & 3u)] = __builtin_amdgcn_perm(xb[j], xa[j], 0x07060302u);
  }
  u32x4 data[kTileIters];
  const uint32_t rslot = swizzle(lane);
#pragma unroll
  for (int k = 0; k < kTileIters; ++k) data[k] = lds[k * kWaveSize + rslot];
  if (ROPE) {
    const uint32_t pslot = swizzle(lane ^ rope.partner);
#pragma unroll
    for (int k = 0; k < kTileIters; ++k) data[k] = rotate_chunk(data[k], lds[k * kWaveSize + pslot], rope);
  }
  store_tile(my_row, lane, lpr_shift, data);
}

template <bool KEEP, bool ROPE>
__device__ inline void copy_tile(const uint8_t* card, const CardGeom& g, uint32_t r0, uint32_t n_rows, uint64_t my_row,
                                 uint32_t lane, const RopeLane& rope) {
  const uint32_t lpr_shift = g.lpr_shift;
  const uint32_t row_bytes = g.head_dim * 2u;
  const uint8_t* src = card + g.off_fp16 + (uint64_t)r0 * row_bytes;
  const uint64_t seg_left = ((uint64_t)n_rows - r0) * row_bytes;   // bytes from the tile start to the segment end
  u32x4 data[kTileIters];
#pragma unroll
  for (int k = 0; k < kTileIters; ++k) {
    const uint64_t off = (uint64_t)(k * kWaveSize + lane) * 16u;
    data[k] = (u32x4)(0u);
    if (off < seg_left) data[k] = card_load<KEEP>(reinterpret_cast<const u32x4*>(src + off));
  }
  if (ROPE) {
#pragma unroll
    for (int k = 0; k < kTileIters; ++k) {
      u32x4 y;
      y.x = __shfl_xor(data[k].x, rope.partner, kWaveSize); y.y = __shfl_xor(data[k].y, rope.partner, kWaveSize);
      y.z = __shfl_xor(data[k].z, rope.partner, kWaveSize); y.w = __shfl_xor(data[k].w, rope.partner, kWaveSize);
      data[k] = rotate_chunk(data[k], y, rope);
    }
  }
  store_tile(my_row, lane, lpr_shift, data);
}

// Writes the header verdict; runs before the unpacking grid on the same stream.
__global__ void unpack_status_kernel(UnpackArgs a) {
  CardGeom g;
  const bool ok = card_geometry_from_header(a.card, a.card_bytes, a.layers, a.kv_heads, a.head_dim, a.group_size, a.tokens, g,
                                            a.flags);
  if (threadIdx.x == 0 && blockIdx.x == 0) *a.status = ok ? 0u : QKV_STATUS_BAD_HEADER;
}

// The tiles of width class C, dealt to the waves round-robin from the segment's end, continuing where
// the previous class stopped.
template <int C, int G, bool KEEP, bool KC>
__device__ inline void unpack_class(const UnpackArgs& a, const CardGeom& g, uint32_t gw, uint32_t n_waves, uint32_t lane,
                                    u32x4* lds, uint32_t& cum, uint32_t& bad) {
  const uint32_t n_rows = g.planes * g.n[C];
  if (n_rows == 0) return;
  const uint32_t tile_rows = kTileChunks >> g.lpr_shift;
  const uint32_t tiles = (n_rows + tile_rows - 1) / tile_rows;
  const uint32_t first = (gw + n_waves - cum) % n_waves;
  const RopeLane no_rope = {};
  for (uint32_t i = first; i < tiles; i += n_waves) {
    const uint32_t r0 = (tiles - 1 - i) * tile_rows;
    const uint64_t my_row = tile_row_address(a, g, C, r0, n_rows, lane, tile_rows, bad);
    if constexpr (C == 3) {
      copy_tile<KEEP, false>(a.card, g, r0, n_rows, my_row, lane, no_rope);
    } else {
      constexpr int W = C == 0 ? 2 : C == 1 ? 4 : 8;
      if (KC && r0 < (n_rows >> 1)) unpack_tile_kc<W, KEEP, false>(a.card, g, C, r0, n_rows >> 1, my_row, lane, lds, no_rope);   // key rows
      else unpack_tile<W, G, KEEP, false>(a.card, g, C, r0, n_rows, my_row, lane, lds, no_rope);
    }
  }
  cum = (cum + tiles) % n_waves;
}

// KC: a uniform card whose key planes (the first half of every segment) are grouped per channel.
template <int G, bool KEEP, bool KC>
__global__ __launch_bounds__(kBlockThreads) void unpack_kernel(UnpackArgs a) {
  __shared__ u32x4 lds[kWavesPerBlock][kTileChunks];
  CardGeom g;
  if (!card_geometry_from_header(a.card, a.card_bytes, a.layers, a.kv_heads, a.head_dim, a.group_size, a.tokens, g,
                                 KC ? QKV_FLAG_KEYS_PER_CHANNEL : 0u)) return;          // uniform over the grid: every wave leaves
  if (KC) {                                      // the shapes the per-channel tiles are written for
    const bool uniform = g.n[0] == g.tokens || g.n[1] == g.tokens || g.n[2] == g.tokens;
    const uint32_t tile_tokens = kTileChunks >> g.lpr_shift;
    if (!uniform || g.group_size != 32u || g.head_dim > 128u || g.tokens % max(32u, tile_tokens) != 0u) return;
  }
  const uint32_t lane = threadIdx.x & 63u;
  const uint32_t wave = threadIdx.x >> 6;
  const uint32_t gw = blockIdx.x * kWavesPerBlock + wave;
  const uint32_t n_waves = gridDim.x * kWavesPerBlock;
  u32x4* my_lds = lds[wave];

  uint32_t bad = 0;
  if (!KC) {
    // Plane by plane, from the last plane to the first; inside a plane the raw rows' tiles first, the 2-bit rows'
    // last, each width from its last tile down - the card is still walked from its end, which is what the memory-
    // side cache holds of a card a little larger than itself (a 302 MB card: 212 us this way, 264 us front to back).
    // A tile never straddles planes; each (plane, width) ends in a partial tile.  Width by width over the whole
    // card, as the card itself is laid out, a plane's rows of the rarer widths were written into DRAM pages that
    // nobody else touched at that time; plane by plane, all rows of one stretch of a plane (2 MiB at 8K tokens, some
    // twenty planes in flight) leave within microseconds of each other.  32K tokens, four hops at budgets 6 / 4 / 3 / 2:
    // 1163 / 1031 / 963 / 851 us width by width, 1060 / 996 / 950 / 860 us plane by plane.  (The packing kernel keeps
    // the card's own order: there the scattered side is the smaller one and plane by plane cost 3 %.)
    const uint32_t tile_rows = kTileChunks >> g.lpr_shift;
    const uint32_t tp0 = (g.n[0] + tile_rows - 1) / tile_rows, tp1 = (g.n[1] + tile_rows - 1) / tile_rows,
                   tp2 = (g.n[2] + tile_rows - 1) / tile_rows, tp3 = (g.n[3] + tile_rows - 1) / tile_rows;
    const uint32_t per_plane = tp0 + tp1 + tp2 + tp3;
    const uint32_t s = (uint32_t)__builtin_amdgcn_readfirstlane((int)gw);
    const uint32_t pr = s / per_plane;
    if (pr >= g.planes) return;
    const uint32_t p = g.planes - 1u - pr;
    uint32_t k = s - pr * per_plane;
    const RopeLane no_rope = {};
    if (k < tp3) {
      const uint32_t r0 = p * g.n[3] + (tp3 - 1u - k) * tile_rows, end = (p + 1u) * g.n[3];
      const uint64_t my_row = tile_row_address(a, g, 3, r0, end, lane, tile_rows, bad);
      copy_tile<KEEP, false>(a.card, g, r0, end, my_row, lane, no_rope);
    } else if ((k -= tp3) < tp2) {
      const uint32_t r0 = p * g.n[2] + (tp2 - 1u - k) * tile_rows, end = (p + 1u) * g.n[2];
      const uint64_t my_row = tile_row_address(a, g, 2, r0, end, lane, tile_rows, bad);
      unpack_tile<8, G, KEEP, false>(a.card, g, 2, r0, end, my_row, lane, my_lds, no_rope);
    } else if ((k -= tp2) < tp1) {
      const uint32_t r0 = p * g.n[1] + (tp1 - 1u - k) * tile_rows, end = (p + 1u) * g.n[1];
      const uint64_t my_row = tile_row_address(a, g, 1, r0, end, lane, tile_rows, bad);
      unpack_tile<4, G, KEEP, false>(a.card, g, 1, r0, end, my_row, lane, my_lds, no_rope);
    } else {
      k -= tp1;
      const uint32_t r0 = p * g.n[0] + (tp0 - 1u - k) * tile_rows, end = (p + 1u) * g.n[0];
      const uint64_t my_row = tile_row_address(a, g, 0, r0, end, lane, tile_rows, bad);
      unpack_tile<2, G, KEEP, false>(a.card, g, 0, r0, end, my_row, lane, my_lds, no_rope);
    }
    if (bad && a.status) atomicOr(a.status, QKV_STATUS_BAD_ORDER);
    return;
  }
  // The card is walked from its end to its start: right after packing, its tail is what the
  // 256 MB memory-side cache still holds (a card of 302 MB unpacks in 212 us this way, 264 us
  // front to back; cards that fit, or that are several times larger, are indifferent).
  uint32_t cum = 0;
  unpack_class<3, G, KEEP, KC>(a, g, gw, n_waves, lane, my_lds, cum, bad);
  unpack_class<2, G, KEEP, KC>(a, g, gw, n_waves, lane, my_lds, cum, bad);
  unpack_class<1, G, KEEP, KC>(a, g, gw, n_waves, lane, my_lds, cum, bad);
  unpack_class<0, G, KEEP, KC>(a, g, gw, n_waves, lane, my_lds, cum, bad);
  if (bad && a.status) atomicOr(a.status, QKV_STATUS_BAD_ORDER);
}

// Row address for injection: plane p of the card -> (K or V, layer, head) -> the caller's
// per-layer tensor.  Only planes of the layer range are ever asked for.
__device__ inline uint64_t inject_row_address(const InjectArgs& a, const CardGeom& g, int c, uint32_t kv, uint32_t r0,
                                              uint32_t seg_hi, uint32_t lane, uint32_t tile_rows, uint32_t& bad) {
  uint64_t addr = 0;
  const uint32_t r = r0 + lane;
  if (lane < tile_rows && r < seg_hi) {
    const uint32_t n = g.n[c];
    const uint32_t p = r / n;
    const uint32_t j = r - p * n;
    const uint32_t t = reinterpret_cast<const uint32_t*>(a.card + g.off_order)[g.base[c] + j];
    const uint32_t pl = p - kv * (g.planes >> 1);
    const uint32_t layer = pl / a.kv_heads;
    const uint32_t head = pl - layer * a.kv_heads;
    const uint32_t li = min(layer - a.layer_begin, a.layer_count - 1u);
    if (t < g.tokens && tables_agree(a.card, g, c, j, t)) {
      addr = (kv ? a.v_layer[li] : a.k_layer[li]) + head * a.head_stride + t * a.token_stride;
    } else {
      bad = 1;
    }
  }
  return addr;
}

// One (class, K or V) range of the card's rows for the layer range: its tiles are dealt to the
// waves round-robin, continuing where the previous range stopped.  (K and V as separate
// instances of this code measure faster than one instance looping over both.)
template <int C, int KV, int G, bool KEEP, bool ROPE, bool KC>
__device__ inline void inject_range(const InjectArgs& a, const CardGeom& g, const RopeLane& rope, uint32_t gw,
                                    uint32_t n_waves, uint32_t lane, u32x4* lds, uint32_t& cum, uint32_t& bad) {
  const uint32_t n = g.n[C];
  if (n == 0) return;
  const uint32_t tile_rows = kTileChunks >> g.lpr_shift;
  const uint32_t seg_lo = ((uint32_t)KV * (g.planes >> 1) + a.layer_begin * a.kv_heads) * n;
  const uint32_t seg_rows = a.layer_count * a.kv_heads * n;
  const uint32_t seg_hi = seg_lo + seg_rows;
  const uint32_t tiles = (seg_rows + tile_rows - 1) / tile_rows;
  constexpr bool rot = KV == 0 && ROPE;            // only keys depend on the position
  const uint32_t first = (gw + n_waves - cum) % n_waves;
  for (uint32_t i = first; i < tiles; i += n_waves) {
    const uint32_t r0 = seg_lo + (tiles - 1 - i) * tile_rows;
    const uint64_t my_row = inject_row_address(a, g, C, (uint32_t)KV, r0, seg_hi, lane, tile_rows, bad);
    if (C == 3) {
      copy_tile<KEEP, rot>(a.card, g, r0, seg_hi, my_row, lane, rope);
    } else {
      constexpr int W = C == 0 ? 2 : C == 1 ? 4 : 8;
      if (KC && KV == 0) unpack_tile_kc<W, KEEP, rot>(a.card, g, C, r0, (g.planes >> 1) * n, my_row, lane, lds, rope);
      else unpack_tile<W, G, KEEP, rot>(a.card, g, C, r0, seg_hi, my_row, lane, lds, rope);
    }
  }
  cum = (cum + tiles) % n_waves;
}

template <int G, bool KEEP, bool ROPE, bool KC>
__global__ __launch_bounds__(kBlockThreads) void inject_kernel(InjectArgs a) {
  __shared__ u32x4 lds[kWavesPerBlock][kTileChunks];
  CardGeom g;
  if (!card_geometry_from_header(a.card, a.card_bytes, a.layers, a.kv_heads, a.head_dim, a.group_size, a.tokens, g,
                                 KC ? QKV_FLAG_KEYS_PER_CHANNEL : 0u)) return;
  if (KC) {                                      // the shapes the per-channel tiles are written for
    const bool uniform = g.n[0] == g.tokens || g.n[1] == g.tokens || g.n[2] == g.tokens;
    const uint32_t tile_tokens = kTileChunks >> g.lpr_shift;
    if (!uniform || g.group_size != 32u || g.head_dim > 128u || g.tokens % max(32u, tile_tokens) != 0u) return;
  }
  const uint32_t lane = threadIdx.x & 63u;
  const uint32_t wave = threadIdx.x >> 6;
  const uint32_t gw = blockIdx.x * kWavesPerBlock + wave;
  const uint32_t n_waves = gridDim.x * kWavesPerBlock;
  u32x4* my_lds = lds[wave];

  // chunk 64 k + lane of a tile is chunk (lane mod chunks-per-row) of its row, whatever k
  RopeLane rope = {};
  if (ROPE) {
    const uint32_t half = (1u << g.lpr_shift) >> 1;             // chunks in half a row
    const uint32_t qc = lane & (2u * half - 1u);
    rope.partner = half;
    rope.flip = qc < half ? 0x80000000u : 0u;
    const uint32_t i0 = 8u * (qc & (half - 1u));
#pragma unroll
    for (int e = 0; e < 8; ++e) { rope.c[e] = a.cs[i0 + e][0]; rope.s[e] = a.cs[i0 + e][1]; }
  }

  // from the card's end to its start, as the dense kernel does
  uint32_t bad = 0, cum = 0;
  inject_range<3, 1, G, KEEP, ROPE, KC>(a, g, rope, gw, n_waves, lane, my_lds, cum, bad);
  inject_range<3, 0, G, KEEP, ROPE, KC>(a, g, rope, gw, n_waves, lane, my_lds, cum, bad);
  inject_range<2, 1, G, KEEP, ROPE, KC>(a, g, rope, gw, n_waves, lane, my_lds, cum, bad);
  inject_range<2, 0, G, KEEP, ROPE, KC>(a, g, rope, gw, n_waves, lane, my_lds, cum, bad);
  inject_range<1, 1, G, KEEP, ROPE, KC>(a, g, rope, gw, n_waves, lane, my_lds, cum, bad);
  inject_range<1, 0, G, KEEP, ROPE, KC>(a, g, rope, gw, n_waves, lane, my_lds, cum, bad);
  inject_range<0, 1, G, KEEP, ROPE, KC>(a, g, rope, gw, n_waves, lane, my_lds, cum, bad);
  inject_range<0, 0, G, KEEP, ROPE, KC>(a, g, rope, gw, n_waves, lane, my_lds, cum, bad);
  if (bad && a.status) atomicOr(a.status, QKV_STATUS_BAD_ORDER);
}

}  // namespace

hipError_t launch_unpack(const uint8_t* card, uint64_t card_bytes, const CardGeom& expect, void* k_out, void* v_out,
                         uint32_t* status, bool keys_per_channel, hipStream_t stream) {
  UnpackArgs a;
  a.card = card;
  a.card_bytes = card_bytes;
  a.flags = keys_per_channel ? QKV_FLAG_KEYS_PER_CHANNEL : 0u;
  a.layers = expect.layers; a.kv_heads = expect.kv_heads; a.head_dim = expect.head_dim; a.group_size = expect.group_size;
  a.tokens = expect.tokens;
  a.k_out = static_cast<uint8_t*>(k_out);
  a.v_out = static_cast<uint8_t*>(v_out);
  a.status = status;
  if (status) {
    hipLaunchKernelGGL(unpack_status_kernel, dim3(1), dim3(kWaveSize), 0, stream, a);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  // the class counts are only known on the device: size the grid for the worst split
  const uint32_t tile_rows = kTileChunks >> expect.lpr_shift;
  const uint64_t rows = (uint64_t)expect.planes * expect.tokens;
  const uint64_t tiles = keys_per_channel ? (rows + tile_rows - 1) / tile_rows + 3
                                          : (uint64_t)expect.planes * ((expect.tokens + tile_rows - 1) / tile_rows + 3);
  const dim3 grid(grid_blocks(tiles)), block(kBlockThreads);
  const bool keep = card_bytes <= kCacheResidentCardBytes;
  if (keys_per_channel) {                        // group size 32 only (checked by the caller)
    if (keep) hipLaunchKernelGGL((unpack_kernel<32, true, true>), grid, block, 0, stream, a);
    else hipLaunchKernelGGL((unpack_kernel<32, false, true>), grid, block, 0, stream, a);
    return hipGetLastError();
  }
  switch (expect.group_size * 2 + (keep ? 1 : 0)) {
    case 65: hipLaunchKernelGGL((unpack_kernel<32, true, false>), grid, block, 0, stream, a); break;
    case 64: hipLaunchKernelGGL((unpack_kernel<32, false, false>), grid, block, 0, stream, a); break;
    case 129: hipLaunchKernelGGL((unpack_kernel<64, true, false>), grid, block, 0, stream, a); break;
    case 128: hipLaunchKernelGGL((unpack_kernel<64, false, false>), grid, block, 0, stream, a); break;
    case 257: hipLaunchKernelGGL((unpack_kernel<128, true, false>), grid, block, 0, stream, a); break;
    default: hipLaunchKernelGGL((unpack_kernel<128, false, false>), grid, block, 0, stream, a); break;
  }
  return hipGetLastError();
}

hipError_t launch_inject(const uint8_t* card, uint64_t card_bytes, const CardGeom& expect, uint32_t layer_begin,
                         uint32_t layer_count, void* const* k_layers, void* const* v_layers, uint64_t head_stride_bytes,
                         uint64_t token_stride_bytes, const float (*cos_sin)[2], bool keys_per_channel, uint32_t* status,
                         hipStream_t stream) {
  InjectArgs a;
  a.card = card;
  a.card_bytes = card_bytes;
  a.layers = expect.layers; a.kv_heads = expect.kv_heads; a.head_dim = expect.head_dim; a.group_size = expect.group_size;
  a.tokens = expect.tokens;
  a.layer_begin = layer_begin;
  a.layer_count = layer_count;
  a.head_stride = head_stride_bytes;
  a.token_stride = token_stride_bytes;
  a.rope = cos_sin != nullptr;
  a.status = status;
  for (uint32_t i = 0; i < QKV_INJECT_MAX_LAYERS; ++i) {
    a.k_layer[i] = i < layer_count ? reinterpret_cast<uint64_t>(k_layers[i]) : 0;
    a.v_layer[i] = i < layer_count ? reinterpret_cast<uint64_t>(v_layers[i]) : 0;
  }
  for (uint32_t i = 0; i < 128; ++i) {
    const bool used = cos_sin != nullptr && i < expect.head_dim / 2;
    a.cs[i][0] = used ? cos_sin[i][0] : 1.0f;
    a.cs[i][1] = used ? cos_sin[i][1] : 0.0f;
  }
  if (status) {
    UnpackArgs u;
    u.card = card; u.card_bytes = card_bytes; u.flags = keys_per_channel ? QKV_FLAG_KEYS_PER_CHANNEL : 0u;
    u.layers = expect.layers; u.kv_heads = expect.kv_heads; u.head_dim = expect.head_dim; u.group_size = expect.group_size;
    u.tokens = expect.tokens;
    u.k_out = nullptr; u.v_out = nullptr; u.status = status;
    hipLaunchKernelGGL(unpack_status_kernel, dim3(1), dim3(kWaveSize), 0, stream, u);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  // worst split of the tokens over the classes; every (class, K or V) range may end in a partial tile
  const uint32_t tile_rows = kTileChunks >> expect.lpr_shift;
  const uint64_t rows = 2ull * layer_count * expect.kv_heads * expect.tokens;
  const uint64_t tiles = (rows + tile_rows - 1) / tile_rows + 8;
  const dim3 grid(grid_blocks(tiles)), block(kBlockThreads);
  const bool keep = card_bytes <= kCacheResidentCardBytes;
  if (keys_per_channel) {                        // group size 32 only (checked by the caller)
    switch ((keep ? 2 : 0) + (a.rope ? 1 : 0)) {
      case 3: hipLaunchKernelGGL((inject_kernel<32, true, true, true>), grid, block, 0, stream, a); break;
      case 2: hipLaunchKernelGGL((inject_kernel<32, true, false, true>), grid, block, 0, stream, a); break;
      case 1: hipLaunchKernelGGL((inject_kernel<32, false, true, true>), grid, block, 0, stream, a); break;
      default: hipLaunchKernelGGL((inject_kernel<32, false, false, true>), grid, block, 0, stream, a); break;
    }
    return hipGetLastError();
  }
  const int variant = (int)expect.group_size * 4 + (keep ? 2 : 0) + (a.rope ? 1 : 0);
  switch (variant) {
    case 131: hipLaunchKernelGGL((inject_kernel<32, true, true, false>), grid, block, 0, stream, a); break;
    case 130: hipLaunchKernelGGL((inject_kernel<32, true, false, false>), grid, block, 0, stream, a); break;
    case 129: hipLaunchKernelGGL((inject_kernel<32, false, true, false>), grid, block, 0, stream, a); break;
    case 128: hipLaunchKernelGGL((inject_kernel<32, false, false, false>), grid, block, 0, stream, a); break;
    case 259: hipLaunchKernelGGL((inject_kernel<64, true, true, false>), grid, block, 0, stream, a); break;
    case 258: hipLaunchKernelGGL((inject_kernel<64, true, false, false>), grid, block, 0, stream, a); break;
    case 257: hipLaunchKernelGGL((inject_kernel<64, false, true, false>), grid, block, 0, stream, a); break;
    case 256: hipLaunchKernelGGL((inject_kernel<64, false, false, false>), grid, block, 0, stream, a); break;
    case 515: hipLaunchKernelGGL((inject_kernel<128, true, true, false>), grid, block, 0, stream, a); break;
    case 514: hipLaunchKernelGGL((inject_kernel<128, true, false, false>), grid, block, 0, stream, a); break;
    case 513: hipLaunchKernelGGL((inject_kernel<128, false, true, false>), grid, block, 0, stream, a); break;
    default: hipLaunchKernelGGL((inject_kernel<128, false, false, false>), grid, block, 0, stream, a); break;
  }
  return hipGetLastError();
}

}  // namespace qkv
