// pack.hip — quantize + bit-pack + segment store (card creation, paper Sec. 4.2.1:
// keys and values packed into quantized groups, one bit width per token).
//
// Work decomposition.  Inside the card every width owns a segment that is a flat array of
// N_c = P * n_c rows (plane-major, then slot).  A wave takes "tiles" of 512 sixteen-byte
// input chunks (4096 fp16 values = 32 rows at head_dim 128); tile i of a segment covers flat
// rows [i*R, (i+1)*R), so every tile's code bytes and (scale, zero) pairs are one contiguous,
// 128-byte aligned run of the card.  The grid is persistent: wave w handles the global tiles
// w, w + W, w + 2W, ... over the four segments in turn.
//
// Inside a tile, lane l of iteration k holds chunk q = 64 k + l: 8 consecutive values of row
// q / (D/8).  A quantization group of G values is G/8 neighbouring lanes, reduced with DPP.
// Rows are gathered through order[] (256-byte aligned full rows), codes are staged through
// LDS so the card is written with 128-bit stores.
#include "qkv_common.h"

namespace qkv {
namespace {

struct PackArgs {
  CardGeom g;
  const uint8_t* k;
  const uint8_t* v;
  uint8_t* card;
};

// ---- cross-lane and packed-half helpers -------------------------------------------------

template <int CTRL>
__device__ inline uint32_t dpp(uint32_t v) {
  return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xF, 0xF, false);
}

// min of two packed fp16 pairs.  The hardware instruction orders -0 below +0 and keeps
// subnormals, so the result does not depend on the reduction order.
__device__ inline uint32_t pk_min(uint32_t a, uint32_t b) {
  uint32_t r;
  asm("v_pk_min_f16 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
  return r;
}
// min(-a, -b) on both halves
__device__ inline uint32_t pk_min_neg(uint32_t a, uint32_t b) {
  uint32_t r;
  asm("v_pk_min_f16 %0, %1, %2 neg_lo:[1,1] neg_hi:[1,1]" : "=v"(r) : "v"(a), "v"(b));
  return r;
}

constexpr int kQuadXor1 = 0xB1;        // quad_perm:[1,0,3,2]
constexpr int kQuadXor2 = 0x4E;        // quad_perm:[2,3,0,1]
constexpr int kRowHalfMirror = 0x141;  // lane i <-> 7 - i inside 8 lanes
constexpr int kRowMirror = 0x140;      // lane i <-> 15 - i inside 16 lanes

// v holds (min, -max) of a lane's 8 values; returns the same pair over the GL lanes of a group.
template <int GL>
__device__ inline uint32_t group_reduce(uint32_t v) {
  v = pk_min(v, dpp<kQuadXor1>(v));
  v = pk_min(v, dpp<kQuadXor2>(v));
  if (GL >= 8) v = pk_min(v, dpp<kRowHalfMirror>(v));
  if (GL >= 16) v = pk_min(v, dpp<kRowMirror>(v));
  return v;
}

__device__ inline float half_bits_to_float(uint32_t h) {
  return (float)__builtin_bit_cast(_Float16, (uint16_t)h);
}
__device__ inline uint32_t float_to_half_bits(float f) {
  return (uint32_t)__builtin_bit_cast(uint16_t, (_Float16)f);   // round to nearest even
}

constexpr float kMagic = 12582912.0f;       // 2^23 + 2^22: adding it rounds to an integer, ties to even
constexpr uint32_t kMagicBits = 0x4B400000u;

// Sum of kMagicBits << (i*W) over the codes that share one 32-bit accumulator.
template <int W>
__host__ __device__ constexpr uint32_t magic_carry() {
  uint32_t s = 0;
  const int n = (W == 8) ? 4 : 8;
  for (int i = 0; i < n; ++i) s += kMagicBits << (i * W);
  return s;
}

// Row id (plane * T + token) that lane `lane` of the wave looks up for row `lane` of a tile.
// 0xFFFFFFFF marks rows past the end of the segment.
__device__ inline uint32_t tile_row_lookup(const CardGeom& g, const uint32_t* __restrict__ order, int c, uint32_t r0,
                                           uint32_t n_rows, uint32_t lane, uint32_t tile_rows) {
  uint32_t rowid = 0xFFFFFFFFu;
  const uint32_t r = r0 + lane;
  if (lane < tile_rows && r < n_rows) {
    const uint32_t n = g.n[c];
    const uint32_t p = r / n;
    const uint32_t j = r - p * n;
    const uint32_t t = order[g.base[c] + j];
    rowid = p * g.tokens + t;
  }
  return rowid;
}

__device__ inline const uint8_t* row_address(const PackArgs& a, uint32_t rowid, uint32_t row_bytes) {
  // V rows continue the numbering after K's; integer arithmetic, so no pointer ever leaves its buffer
  const uint64_t k_bytes = (uint64_t)a.g.k_rows * row_bytes;
  const uint64_t off = (uint64_t)rowid * row_bytes;
  const uint64_t addr = (rowid < a.g.k_rows) ? reinterpret_cast<uint64_t>(a.k) + off
                                             : reinterpret_cast<uint64_t>(a.v) + (off - k_bytes);
  return reinterpret_cast<const uint8_t*>(addr);
}

// ---- one tile of a quantized segment ------------------------------------------------------

template <int W, int G>
__device__ inline void pack_tile(const PackArgs& a, int c, uint32_t r0, uint32_t n_rows, uint32_t lane,
                                 uint8_t* lds_codes, uint32_t* lds_meta) {
  constexpr int GL = G / 8;                       // lanes per group
  constexpr uint32_t QMAX = (1u << W) - 1u;
  const CardGeom& g = a.g;
  const uint32_t lpr_shift = g.lpr_shift;
  const uint32_t tile_rows = kTileChunks >> lpr_shift;
  const uint32_t row_bytes = g.head_dim * 2u;
  const uint32_t* order = reinterpret_cast<const uint32_t*>(a.card + g.off_order);

  const uint32_t my_row = tile_row_lookup(g, order, c, r0, n_rows, lane, tile_rows);

  uint4 data[kTileIters];
#pragma unroll
  for (int k = 0; k < kTileIters; ++k) {
    const uint32_t q = k * kWaveSize + lane;
    const uint32_t rowid = __shfl(my_row, q >> lpr_shift, kWaveSize);
    data[k] = make_uint4(0, 0, 0, 0);
    if (rowid != 0xFFFFFFFFu) {
      const uint8_t* src = row_address(a, rowid, row_bytes) + (q & ((1u << lpr_shift) - 1u)) * 16u;
      data[k] = *reinterpret_cast<const uint4*>(src);
    }
  }

#pragma unroll
  for (int k = 0; k < kTileIters; ++k) {
    const uint32_t q = k * kWaveSize + lane;
    const uint32_t w0 = data[k].x, w1 = data[k].y, w2 = data[k].z, w3 = data[k].w;
    // (min, -max) over the lane's 8 values, then over the group's lanes
    const uint32_t mn2 = pk_min(pk_min(w0, w1), pk_min(w2, w3));
    const uint32_t ng2 = pk_min(pk_min_neg(w0, w1), pk_min_neg(w2, w3));
    const uint32_t lo = __builtin_amdgcn_perm(ng2, mn2, 0x05040100u);   // (mn2.lo, ng2.lo)
    const uint32_t hi = __builtin_amdgcn_perm(ng2, mn2, 0x07060302u);   // (mn2.hi, ng2.hi)
    const uint32_t red = group_reduce<GL>(pk_min(lo, hi));
    const uint32_t mn_h = red & 0xFFFFu;
    const uint32_t mx_h = (red >> 16) ^ 0x8000u;

    // scale and reciprocal: fp32, this order, IEEE division
    const float fmn = half_bits_to_float(mn_h);
    const float fmx = half_bits_to_float(mx_h);
    const float range = fmx - fmn;
    const float s32 = range / (float)QMAX;
    const uint32_t s_h = float_to_half_bits(s32);
    const float s = half_bits_to_float(s_h);
    const float inv = (s > 0.0f) ? 1.0f / s : 0.0f;

    // codes: RNE of the exact product through the magic-number fma, clamped to QMAX
    const uint32_t words[4] = {w0, w1, w2, w3};
    uint32_t acc0 = 0, acc1 = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const uint32_t hbits = (i & 1) ? (words[i >> 1] >> 16) : (words[i >> 1] & 0xFFFFu);
      const float d = half_bits_to_float(hbits) - fmn;
      const float r = __builtin_fmaf(d, inv, kMagic);
      const uint32_t u = min(__float_as_uint(r), kMagicBits + QMAX);
      if (W == 8) {
        if (i < 4) acc0 = (u << (8 * i)) + acc0; else acc1 = (u << (8 * (i - 4))) + acc1;
      } else {
        acc0 = (u << (W * i)) + acc0;
      }
    }
    acc0 -= magic_carry<W>();
    if (W == 8) acc1 -= magic_carry<W>();

    if (W == 2) reinterpret_cast<uint16_t*>(lds_codes)[q] = (uint16_t)acc0;
    if (W == 4) reinterpret_cast<uint32_t*>(lds_codes)[q] = acc0;
    if (W == 8) reinterpret_cast<uint2*>(lds_codes)[q] = make_uint2(acc0, acc1);
    if ((lane & (GL - 1)) == 0) lds_meta[q / GL] = s_h | (mn_h << 16);   // fp16 scale first, then fp16 zero
  }
  __builtin_amdgcn_wave_barrier();

  // codes: tile = 512*W bytes, 16 bytes per lane per store
  {
    const uint64_t seg_bytes = (uint64_t)n_rows * (g.head_dim * W / 8);
    const uint64_t tile_off = (uint64_t)r0 * (g.head_dim * W / 8);
    uint8_t* dst = a.card + g.off_codes[c];
#pragma unroll
    for (int m = 0; m < W / 2; ++m) {
      const uint32_t idx = m * kWaveSize + lane;
      const uint4 o = reinterpret_cast<const uint4*>(lds_codes)[idx];
      const uint64_t off = tile_off + (uint64_t)idx * 16u;
      if (off < seg_bytes) *reinterpret_cast<uint4*>(dst + off) = o;
    }
  }
  // (scale, zero) pairs: 512/GL dwords per tile
  {
    constexpr int kDwords = kTileChunks / GL;
    const uint64_t seg_dwords = (uint64_t)n_rows * (g.head_dim / G);
    const uint64_t tile_dw = (uint64_t)r0 * (g.head_dim / G);
    uint32_t* dst = reinterpret_cast<uint32_t*>(a.card + g.off_meta[c]);
#pragma unroll
    for (int m = 0; m < (kDwords + kWaveSize - 1) / kWaveSize; ++m) {
      const uint32_t idx = m * kWaveSize + lane;
      if (idx < (uint32_t)kDwords && tile_dw + idx < seg_dwords) dst[tile_dw + idx] = lds_meta[idx];
    }
  }
  __builtin_amdgcn_wave_barrier();
}

// ---- one tile of the fp16 segment: rows copied bit for bit ---------------------------------

__device__ inline void copy_tile(const PackArgs& a, uint32_t r0, uint32_t n_rows, uint32_t lane) {
  const CardGeom& g = a.g;
  const uint32_t lpr_shift = g.lpr_shift;
  const uint32_t tile_rows = kTileChunks >> lpr_shift;
  const uint32_t row_bytes = g.head_dim * 2u;
  const uint32_t* order = reinterpret_cast<const uint32_t*>(a.card + g.off_order);
  const uint32_t my_row = tile_row_lookup(g, order, 3, r0, n_rows, lane, tile_rows);
  uint4 data[kTileIters];
  bool valid[kTileIters];
#pragma unroll
  for (int k = 0; k < kTileIters; ++k) {
    const uint32_t q = k * kWaveSize + lane;
    const uint32_t rowid = __shfl(my_row, q >> lpr_shift, kWaveSize);
    valid[k] = rowid != 0xFFFFFFFFu;
    data[k] = make_uint4(0, 0, 0, 0);
    if (valid[k]) {
      const uint8_t* src = row_address(a, rowid, row_bytes) + (q & ((1u << lpr_shift) - 1u)) * 16u;
      data[k] = *reinterpret_cast<const uint4*>(src);
    }
  }
  uint8_t* dst = a.card + g.off_fp16 + (uint64_t)r0 * row_bytes;
#pragma unroll
  for (int k = 0; k < kTileIters; ++k) {
    const uint32_t q = k * kWaveSize + lane;
    if (valid[k]) *reinterpret_cast<uint4*>(dst + (uint64_t)q * 16u) = data[k];
  }
}

// ---- persistent kernel ------------------------------------------------------------------------

template <int G>
__global__ __launch_bounds__(kBlockThreads) void pack_kernel(PackArgs a) {
  __shared__ __attribute__((aligned(16))) uint8_t lds_codes[kWavesPerBlock][kTileChunks * 8];
  __shared__ uint32_t lds_meta[kWavesPerBlock][kTileChunks / 4];
  const uint32_t lane = threadIdx.x & 63u;
  const uint32_t wave = threadIdx.x >> 6;
  const uint32_t gw = blockIdx.x * kWavesPerBlock + wave;
  const uint32_t n_waves = gridDim.x * kWavesPerBlock;
  const uint32_t tile_rows = kTileChunks >> a.g.lpr_shift;
  uint8_t* my_codes = lds_codes[wave];
  uint32_t* my_meta = lds_meta[wave];

  uint32_t cum = 0;   // tiles of the classes already done, modulo n_waves
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    const uint32_t n_rows = a.g.planes * a.g.n[c];
    if (n_rows == 0) continue;
    const uint32_t tiles = (n_rows + tile_rows - 1) / tile_rows;
    const uint32_t first = (gw + n_waves - cum) % n_waves;
    for (uint32_t i = first; i < tiles; i += n_waves) {
      const uint32_t r0 = i * tile_rows;
      if (c == 0) pack_tile<2, G>(a, 0, r0, n_rows, lane, my_codes, my_meta);
      if (c == 1) pack_tile<4, G>(a, 1, r0, n_rows, lane, my_codes, my_meta);
      if (c == 2) pack_tile<8, G>(a, 2, r0, n_rows, lane, my_codes, my_meta);
      if (c == 3) copy_tile(a, r0, n_rows, lane);
    }
    cum = (cum + tiles) % n_waves;
  }
}

}  // namespace

hipError_t launch_pack(const CardGeom& geom, const void* k, const void* v, uint8_t* card, hipStream_t stream) {
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
  const dim3 grid(persistent_blocks(tiles)), block(kBlockThreads);
  switch (geom.group_size) {
    case 32: hipLaunchKernelGGL(pack_kernel<32>, grid, block, 0, stream, a); break;
    case 64: hipLaunchKernelGGL(pack_kernel<64>, grid, block, 0, stream, a); break;
    default: hipLaunchKernelGGL(pack_kernel<128>, grid, block, 0, stream, a); break;
  }
  return hipGetLastError();
}

}  // namespace qkv
