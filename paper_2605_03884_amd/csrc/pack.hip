// pack.hip — quantize + bit-pack + segment store (card creation, paper Sec. 4.2.1:
// keys and values packed into quantized groups, one bit width per token).
//
// Work decomposition.  Inside the card every width owns a segment that is a flat array of
// N_c = P * n_c rows (plane-major, then slot).  A wave takes "tiles" of 512 sixteen-byte
// input chunks (4096 fp16 values = 32 rows at head_dim 128); tile i of a segment covers flat
// rows [i*R, (i+1)*R), so the tile's code bytes and its (scale, zero) pairs are each one
// contiguous, 128-byte aligned run of the card.  Wave w handles the global tiles
// w, w + W, w + 2W, ... over the four segments in turn.
//
// Inside a tile.
//   1. Rows are gathered through order[]: whole 256-byte rows, 128-bit loads, 1 KiB per
//      load instruction (lane l of load k holds chunk 64 k + l).
//   2. The 8 KiB tile is turned through LDS so that each lane then owns one "span" of 32
//      consecutive values (64 bytes) - a whole quantization group at group size 32.  The
//      chunk index is XOR-swizzled so that both the row-major writes and the span-major
//      reads touch every LDS bank once per pass.
//   3. Per span: min / max with packed 3-input fp16 instructions and no cross-lane traffic
//      (one or two DPP steps at group size 64 / 128), scale and reciprocal once per span,
//      three VALU operations per value (subtract, multiply-round, shift-insert).
//   4. A lane's packed codes (8 / 16 / 32 bytes) and pair (4 bytes) are contiguous with its
//      neighbours', so they go straight to the card with coalesced stores.
// The hardware min / max order -0 below +0 and keep subnormals, so the group extrema do not
// depend on the reduction order.
#include "qkv_common.h"
#include "qkv_encode.h"

namespace qkv {
namespace {

typedef __attribute__((address_space(1))) const u32x4 global_u32x4;

struct PackArgs {
  CardGeom g;
  const uint8_t* k;
  const uint8_t* v;
  uint8_t* card;
};

// LDS position (in 16-byte units) of input chunk q of a tile.
__device__ inline uint32_t swizzle(uint32_t q) { return q ^ ((q >> 3) & 3u); }

// ---- rows of a tile -------------------------------------------------------------------------

// Address of the fp16 row that row `lane` of the tile is made from; 0 past the segment's end and
// for an order[] entry that names no token (the row then reads as zeros and `bad` is raised): the
// table lives in the caller's card buffer, so it is bounded like any other untrusted input.
__device__ inline uint64_t tile_row_address(const PackArgs& a, int c, uint32_t r0, uint32_t n_rows, uint32_t lane,
                                            uint32_t tile_rows, uint32_t& bad) {
  const CardGeom& g = a.g;
  uint64_t addr = 0;
  const uint32_t r = r0 + lane;
  if (lane < tile_rows && r < n_rows) {
    const uint32_t n = g.n[c];
    const uint32_t p = r / n;
    const uint32_t j = r - p * n;
    const uint32_t t = reinterpret_cast<const uint32_t*>(a.card + g.off_order)[g.base[c] + j];
    const uint32_t lh = g.planes >> 1;
    const uint32_t row_bytes = g.head_dim * 2u;
    // V rows continue the plane numbering after K's; each address stays inside its own tensor
    if (t < g.tokens) {
      addr = (p < lh) ? reinterpret_cast<uint64_t>(a.k) + ((uint64_t)p * g.tokens + t) * row_bytes
                      : reinterpret_cast<uint64_t>(a.v) + ((uint64_t)(p - lh) * g.tokens + t) * row_bytes;
    } else {
      bad = 1;
    }
  }
  return addr;
}

// Loads the tile: data[k] = chunk 64 k + lane, zero where the row does not exist.
__device__ inline void load_tile(uint64_t my_row_addr, uint32_t lane, uint32_t lpr_shift, u32x4 (&data)[kTileIters]) {
  const uint32_t in_row = (lane & ((1u << lpr_shift) - 1u)) * 16u;
#pragma unroll
  for (int k = 0; k < kTileIters; ++k) {
    const uint32_t src_lane = (k * kWaveSize + lane) >> lpr_shift;
    const uint32_t lo = __shfl((uint32_t)my_row_addr, src_lane, kWaveSize);
    const uint32_t hi = __shfl((uint32_t)(my_row_addr >> 32), src_lane, kWaveSize);
    const uint64_t row = ((uint64_t)hi << 32) | lo;
    data[k] = (u32x4)(0u);
    if (row != 0) data[k] = __builtin_nontemporal_load(reinterpret_cast<global_u32x4*>(row + in_row));
  }
}

// ---- one span of 32 values --------------------------------------------------------------------

template <int W, int G, bool KEEP>
__device__ inline void pack_tile(const PackArgs& a, int c, uint32_t r0, uint32_t n_rows, uint32_t lane, u32x4* lds,
                                 uint32_t& bad) {
  constexpr int GS = G / 32;                     // spans (lanes) per group
  const CardGeom& g = a.g;
  const uint32_t lpr_shift = g.lpr_shift;
  const uint32_t tile_rows = kTileChunks >> lpr_shift;
  const uint32_t spr_shift = lpr_shift - 2;      // log2(spans per row)

  const uint64_t my_row = tile_row_address(a, c, r0, n_rows, lane, tile_rows, bad);
  u32x4 data[kTileIters];
  load_tile(my_row, lane, lpr_shift, data);
  const uint32_t wslot = swizzle(lane);
#pragma unroll
  for (int k = 0; k < kTileIters; ++k) lds[k * kWaveSize + wslot] = data[k];

  const uint32_t x = (lane >> 1) & 3u;           // swizzle term of this lane's spans
  uint8_t* codes_seg = a.card + g.off_codes[c];
  uint32_t* meta_seg = reinterpret_cast<uint32_t*>(a.card + g.off_meta[c]);
  const uint64_t span0 = (uint64_t)r0 << spr_shift;                   // first span of the tile inside the segment
  const uint64_t seg_spans = (uint64_t)n_rows << spr_shift;

#pragma unroll 1
  for (int round = 0; round < kTileRounds; ++round) {
    const uint32_t sp = round * kWaveSize + lane;
    uint32_t w[16];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const u32x4 t = lds[4 * sp + (j ^ x)];
      w[4 * j + 0] = t.x; w[4 * j + 1] = t.y; w[4 * j + 2] = t.z; w[4 * j + 3] = t.w;
    }
    uint32_t out[W];
    const uint32_t pair = quantize_span<W, GS>(w, out);

    const uint64_t gsp = span0 + sp;
    if (gsp < seg_spans) {
      uint8_t* dst = codes_seg + gsp * (4u * W);
      if (W == 2) card_store<KEEP>(reinterpret_cast<u32x2*>(dst), (u32x2){out[0], out[1]});
      if (W >= 4) card_store<KEEP>(reinterpret_cast<u32x4*>(dst), (u32x4){out[0], out[1], out[2], out[3]});
      if (W == 8) card_store<KEEP>(reinterpret_cast<u32x4*>(dst + 16), (u32x4){out[4], out[5], out[6], out[7]});
      if ((sp & (GS - 1)) == 0) card_store<KEEP>(&meta_seg[gsp / GS], pair);
    }
  }
}

// ---- one tile of the fp16 segment: rows copied bit for bit ---------------------------------

// A tile of key rows of a uniform card with groups per channel: the tile is gathered into LDS as usual,
// but a lane then takes, per round, the 32 tokens of one token block for one channel (a column of the
// tile; 64 lanes read 64 neighbouring channels of a row at a time), quantizes them as one group, and
// stores codes and pair at [token block][channel].  Head dimensions 64 and 128 only: a tile must hold
// whole blocks of 32 tokens.
template <int W, bool KEEP>
__device__ inline void pack_tile_kc(const PackArgs& a, int c, uint32_t r0, uint32_t n_rows, uint32_t key_rows,
                                    uint32_t lane, u32x4* lds, uint32_t& bad) {
  const CardGeom& g = a.g;
  const uint32_t lpr_shift = g.lpr_shift;
  const uint32_t tile_rows = kTileChunks >> lpr_shift;
  const uint64_t my_row = tile_row_address(a, c, r0, n_rows, lane, tile_rows, bad);
  u32x4 data[kTileIters];
  load_tile(my_row, lane, lpr_shift, data);
  const uint32_t wslot = swizzle(lane);
#pragma unroll
  for (int k = 0; k < kTileIters; ++k) lds[k * kWaveSize + wslot] = data[k];

  const uint16_t* lds16 = reinterpret_cast<const uint16_t*>(lds);
  uint8_t* codes_seg = a.card + g.off_codes[c];
  uint32_t* meta_seg = reinterpret_cast<uint32_t*>(a.card + g.off_meta[c]);
  const uint32_t D = g.head_dim;
#pragma unroll 1
  for (int round = 0; round < kTileRounds; ++round) {
    const uint32_t sp = round * kWaveSize + lane;
    const uint32_t d = sp & (D - 1u);                       // channel
    const uint32_t tbl = sp >> (lpr_shift + 3u);            // token block inside the tile (head_dim 64: two)
    uint32_t w[16];
#pragma unroll
    for (int j = 0; j < 16; ++j) {
      const uint32_t qa = ((32u * tbl + 2u * j) << lpr_shift) + (d >> 3);      // chunk of (token 2j, channel d)
      const uint32_t qb = qa + (1u << lpr_shift);
      const uint32_t xa = lds16[swizzle(qa) * 8u + (d & 7u)];
      const uint32_t xb = lds16[swizzle(qb) * 8u + (d & 7u)];
      w[j] = xa | (xb << 16);
    }
    uint32_t out[W];
    const uint32_t pair = quantize_span<W, 1>(w, out);
    const uint32_t blk = r0 / 32u + tbl;                    // token block inside the segment: planes follow each other
    if (32u * blk < key_rows) {
      const uint64_t grp = (uint64_t)blk * D + d;
      uint8_t* dst = codes_seg + grp * (4u * W);
      if (W == 2) card_store<KEEP>(reinterpret_cast<u32x2*>(dst), (u32x2){out[0], out[1]});
      if (W >= 4) card_store<KEEP>(reinterpret_cast<u32x4*>(dst), (u32x4){out[0], out[1], out[2], out[3]});
      if (W == 8) card_store<KEEP>(reinterpret_cast<u32x4*>(dst + 16), (u32x4){out[4], out[5], out[6], out[7]});
      card_store<KEEP>(&meta_seg[grp], pair);
    }
  }
}

template <bool KEEP>
__device__ inline void copy_tile(const PackArgs& a, uint32_t r0, uint32_t n_rows, uint32_t lane, uint32_t& bad) {
  const CardGeom& g = a.g;
  const uint32_t lpr_shift = g.lpr_shift;
  const uint32_t tile_rows = kTileChunks >> lpr_shift;
  const uint32_t row_bytes = g.head_dim * 2u;
  const uint64_t my_row = tile_row_address(a, 3, r0, n_rows, lane, tile_rows, bad);
  u32x4 data[kTileIters];
  load_tile(my_row, lane, lpr_shift, data);
  uint8_t* dst = a.card + g.off_fp16 + (uint64_t)r0 * row_bytes;
  const uint64_t left = ((uint64_t)n_rows - r0) * row_bytes;     // bytes from the tile start to the segment end
#pragma unroll
  for (int k = 0; k < kTileIters; ++k) {
    const uint64_t off = (uint64_t)(k * kWaveSize + lane) * 16u;
    if (off < left) card_store<KEEP>(reinterpret_cast<u32x4*>(dst + off), data[k]);
  }
}

// ---- grid ----------------------------------------------------------------------------------------

// KC: the card is uniform and its key planes (the first half of every segment) are grouped per channel.
template <int G, bool KEEP, bool KC>
__global__ __launch_bounds__(kBlockThreads) void pack_kernel(PackArgs a) {
  __shared__ u32x4 lds[kWavesPerBlock][kTileChunks];
  const uint32_t lane = threadIdx.x & 63u;
  const uint32_t wave = threadIdx.x >> 6;
  const uint32_t gw = blockIdx.x * kWavesPerBlock + wave;
  const uint32_t n_waves = gridDim.x * kWavesPerBlock;
  const uint32_t tile_rows = kTileChunks >> a.g.lpr_shift;
  u32x4* my_lds = lds[wave];

  uint32_t bad = 0;   // an order[] entry past the last token was met
  uint32_t cum = 0;   // tiles of the classes already done, modulo n_waves
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    const uint32_t n_rows = a.g.planes * a.g.n[c];
    if (n_rows == 0) continue;
    const uint32_t tiles = (n_rows + tile_rows - 1) / tile_rows;
    const uint32_t first = (gw + n_waves - cum) % n_waves;
    for (uint32_t i = first; i < tiles; i += n_waves) {
      const uint32_t r0 = i * tile_rows;
      if (KC && c < 3 && r0 < (n_rows >> 1)) {                 // key rows: the host made sure no tile straddles the halves
        if (c == 0) pack_tile_kc<2, KEEP>(a, 0, r0, n_rows, n_rows >> 1, lane, my_lds, bad);
        if (c == 1) pack_tile_kc<4, KEEP>(a, 1, r0, n_rows, n_rows >> 1, lane, my_lds, bad);
        if (c == 2) pack_tile_kc<8, KEEP>(a, 2, r0, n_rows, n_rows >> 1, lane, my_lds, bad);
        continue;
      }
      if (c == 0) pack_tile<2, G, KEEP>(a, 0, r0, n_rows, lane, my_lds, bad);
      if (c == 1) pack_tile<4, G, KEEP>(a, 1, r0, n_rows, lane, my_lds, bad);
      if (c == 2) pack_tile<8, G, KEEP>(a, 2, r0, n_rows, lane, my_lds, bad);
      if (c == 3) copy_tile<KEEP>(a, r0, n_rows, lane, bad);
    }
    cum = (cum + tiles) % n_waves;
  }
  // the header's status word (byte 192); the planning kernel wrote it earlier on the same stream
  if (bad) atomicOr(reinterpret_cast<uint32_t*>(a.card + 192), QKV_STATUS_BAD_ORDER);
}

}  // namespace

hipError_t launch_pack(const CardGeom& geom, const void* k, const void* v, uint8_t* card, bool keys_per_channel,
                       hipStream_t stream) {
  PackArgs a;
  a.g = geom;
  a.k = static_cast<const uint8_t*>(k);
  a.v = static_cast<const uint8_t*>(v);
  a.card = card;
  const uint32_t tile_rows = kTileChunks >> geom.lpr_shift;
  uint64_t tiles = 0;
  for (int c = 0; c < 4; ++c) {
    const uint64_t rows = (uint64_t)geom.planes * geom.n[c];
    tiles += (rows + tile_rows - 1) / tile_rows;
  }
  if (tiles == 0) return hipSuccess;
  const dim3 grid(grid_blocks(tiles)), block(kBlockThreads);
  const bool keep = geom.total <= kCacheResidentCardBytes;
  if (keys_per_channel) {                        // group size 32 only (checked by the caller)
    if (keep) hipLaunchKernelGGL((pack_kernel<32, true, true>), grid, block, 0, stream, a);
    else hipLaunchKernelGGL((pack_kernel<32, false, true>), grid, block, 0, stream, a);
    return hipGetLastError();
  }
  switch (geom.group_size * 2 + (keep ? 1 : 0)) {
    case 65: hipLaunchKernelGGL((pack_kernel<32, true, false>), grid, block, 0, stream, a); break;
    case 64: hipLaunchKernelGGL((pack_kernel<32, false, false>), grid, block, 0, stream, a); break;
    case 129: hipLaunchKernelGGL((pack_kernel<64, true, false>), grid, block, 0, stream, a); break;
    case 128: hipLaunchKernelGGL((pack_kernel<64, false, false>), grid, block, 0, stream, a); break;
    case 257: hipLaunchKernelGGL((pack_kernel<128, true, false>), grid, block, 0, stream, a); break;
    default: hipLaunchKernelGGL((pack_kernel<128, false, false>), grid, block, 0, stream, a); break;
  }
  return hipGetLastError();
}

}  // namespace qkv
