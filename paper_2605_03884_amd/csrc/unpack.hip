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
  uint32_t layers, kv_heads, head_dim, group_size;   // the shape the outputs were sized for
  uint64_t tokens;
  uint8_t* k_out;
  uint8_t* v_out;
  uint32_t* status;                                  // may be null
};

typedef __attribute__((address_space(1))) u32x4 global_u32x4;

// LDS position (in 16-byte units) of output chunk q of a tile.
__device__ inline uint32_t swizzle(uint32_t q) { return q ^ ((q >> 3) & 3u); }

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
    if (t < g.tokens) {
      addr = (p < lh) ? reinterpret_cast<uint64_t>(a.k_out) + ((uint64_t)p * g.tokens + t) * row_bytes
                      : reinterpret_cast<uint64_t>(a.v_out) + ((uint64_t)(p - lh) * g.tokens + t) * row_bytes;
    } else {
      bad = 1;
    }
  }
  return addr;
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

template <int W, int G, bool KEEP>
__device__ inline void unpack_tile(const UnpackArgs& a, const CardGeom& g, int c, uint32_t r0, uint32_t n_rows,
                                   uint32_t lane, u32x4* lds, uint32_t& bad) {
  constexpr int GS = G / 32;                     // spans (lanes) per group
  const uint32_t lpr_shift = g.lpr_shift;
  const uint32_t tile_rows = kTileChunks >> lpr_shift;
  const uint32_t spr_shift = lpr_shift - 2;      // log2(spans per row)
  const uint64_t my_row = tile_row_address(a, g, c, r0, n_rows, lane, tile_rows, bad);

  const uint8_t* codes_seg = a.card + g.off_codes[c];
  const uint32_t* meta_seg = reinterpret_cast<const uint32_t*>(a.card + g.off_meta[c]);
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
  store_tile(my_row, lane, lpr_shift, data);
}

template <bool KEEP>
__device__ inline void copy_tile(const UnpackArgs& a, const CardGeom& g, uint32_t r0, uint32_t n_rows, uint32_t lane,
                                 uint32_t& bad) {
  const uint32_t lpr_shift = g.lpr_shift;
  const uint32_t tile_rows = kTileChunks >> lpr_shift;
  const uint32_t row_bytes = g.head_dim * 2u;
  const uint64_t my_row = tile_row_address(a, g, 3, r0, n_rows, lane, tile_rows, bad);
  const uint8_t* src = a.card + g.off_fp16 + (uint64_t)r0 * row_bytes;
  const uint64_t seg_left = ((uint64_t)n_rows - r0) * row_bytes;   // bytes from the tile start to the segment end
  u32x4 data[kTileIters];
#pragma unroll
  for (int k = 0; k < kTileIters; ++k) {
    const uint64_t off = (uint64_t)(k * kWaveSize + lane) * 16u;
    data[k] = (u32x4)(0u);
    if (off < seg_left) data[k] = card_load<KEEP>(reinterpret_cast<const u32x4*>(src + off));
  }
  store_tile(my_row, lane, lpr_shift, data);
}

// Writes the header verdict; runs before the unpacking grid on the same stream.
__global__ void unpack_status_kernel(UnpackArgs a) {
  CardGeom g;
  const bool ok = card_geometry_from_header(a.card, a.card_bytes, a.layers, a.kv_heads, a.head_dim, a.group_size, a.tokens, g);
  if (threadIdx.x == 0 && blockIdx.x == 0) *a.status = ok ? 0u : QKV_STATUS_BAD_HEADER;
}

template <int G, bool KEEP>
__global__ __launch_bounds__(kBlockThreads) void unpack_kernel(UnpackArgs a) {
  __shared__ u32x4 lds[kWavesPerBlock][kTileChunks];
  CardGeom g;
  if (!card_geometry_from_header(a.card, a.card_bytes, a.layers, a.kv_heads, a.head_dim, a.group_size, a.tokens, g)) return;          // uniform over the grid: every wave leaves
  const uint32_t lane = threadIdx.x & 63u;
  const uint32_t wave = threadIdx.x >> 6;
  const uint32_t gw = blockIdx.x * kWavesPerBlock + wave;
  const uint32_t n_waves = gridDim.x * kWavesPerBlock;
  const uint32_t tile_rows = kTileChunks >> g.lpr_shift;
  u32x4* my_lds = lds[wave];

  // The card is walked from its end to its start: right after packing, its tail is what the
  // 256 MB memory-side cache still holds (a card of 302 MB unpacks in 212 us this way, 264 us
  // front to back; cards that fit, or that are several times larger, are indifferent).
  uint32_t bad = 0;
  uint32_t cum = 0;
#pragma unroll
  for (int c = 3; c >= 0; --c) {
    const uint32_t n_rows = g.planes * g.n[c];
    if (n_rows == 0) continue;
    const uint32_t tiles = (n_rows + tile_rows - 1) / tile_rows;
    const uint32_t first = (gw + n_waves - cum) % n_waves;
    for (uint32_t i = first; i < tiles; i += n_waves) {
      const uint32_t r0 = (tiles - 1 - i) * tile_rows;
      if (c == 0) unpack_tile<2, G, KEEP>(a, g, 0, r0, n_rows, lane, my_lds, bad);
      if (c == 1) unpack_tile<4, G, KEEP>(a, g, 1, r0, n_rows, lane, my_lds, bad);
      if (c == 2) unpack_tile<8, G, KEEP>(a, g, 2, r0, n_rows, lane, my_lds, bad);
      if (c == 3) copy_tile<KEEP>(a, g, r0, n_rows, lane, bad);
    }
    cum = (cum + tiles) % n_waves;
  }
  if (bad && a.status) atomicOr(a.status, QKV_STATUS_BAD_ORDER);
}

}  // namespace

hipError_t launch_unpack(const uint8_t* card, uint64_t card_bytes, const CardGeom& expect, void* k_out, void* v_out,
                         uint32_t* status, hipStream_t stream) {
  UnpackArgs a;
  a.card = card;
  a.card_bytes = card_bytes;
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
  const uint64_t tiles = (rows + tile_rows - 1) / tile_rows + 3;
  const dim3 grid(grid_blocks(tiles)), block(kBlockThreads);
  const bool keep = card_bytes <= kCacheResidentCardBytes;
  switch (expect.group_size * 2 + (keep ? 1 : 0)) {
    case 65: hipLaunchKernelGGL((unpack_kernel<32, true>), grid, block, 0, stream, a); break;
    case 64: hipLaunchKernelGGL((unpack_kernel<32, false>), grid, block, 0, stream, a); break;
    case 129: hipLaunchKernelGGL((unpack_kernel<64, true>), grid, block, 0, stream, a); break;
    case 128: hipLaunchKernelGGL((unpack_kernel<64, false>), grid, block, 0, stream, a); break;
    case 257: hipLaunchKernelGGL((unpack_kernel<128, true>), grid, block, 0, stream, a); break;
    default: hipLaunchKernelGGL((unpack_kernel<128, false>), grid, block, 0, stream, a); break;
  }
  return hipGetLastError();
}

}  // namespace qkv
