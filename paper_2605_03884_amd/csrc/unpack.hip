// unpack.hip — receiver-side injection (paper Sec. 4.2.2): the card's quantized groups are
// unpacked and dequantized into a dense fp16 K/V cache, 16-bit rows are copied back.
//
// Mirror image of the packing kernel.  A wave takes a tile of 512 sixteen-byte output
// chunks (32 rows at head_dim 128) of one width's segment: the tile's code bytes and
// (scale, zero) pairs are one contiguous run of the card, loaded with 128-bit reads and
// staged in LDS; lane l of iteration k then owns output chunk q = 64 k + l, picks its 8
// codes and its group's pair out of LDS, and stores 8 fp16 values with one 128-bit write
// to the row that order[] names.  Every store instruction of a wave therefore writes whole
// 256-byte rows.
//
// The card is untrusted input: the kernel rebuilds the section offsets from the header's
// class counts, checks them against the buffer size and the caller's shape, and bounds
// every order[] entry, so no access can leave the card or the output tensors.
#include "qkv_common.h"

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

__device__ inline float half_bits_to_float(uint32_t h) {
  return (float)__builtin_bit_cast(_Float16, (uint16_t)h);
}

// True when the header describes a layout-v1 card of the expected shape that fits in
// card_bytes; fills `g` from the header's class counts.  Uniform over the grid.
__device__ inline bool load_geometry(const UnpackArgs& a, CardGeom& g) {
  const qkv_card_header_t* h = reinterpret_cast<const qkv_card_header_t*>(a.card);
  const uint32_t* w = reinterpret_cast<const uint32_t*>(a.card);
  bool ok = w[0] == 0x43564B51u && w[1] == 0x00445241u;          // "QKVC" "ARD\0"
  ok = ok && h->version == QKV_CARD_VERSION && h->header_bytes == QKV_CARD_HEADER_BYTES;
  ok = ok && h->layers == a.layers && h->kv_heads == a.kv_heads && h->head_dim == a.head_dim &&
       h->group_size == a.group_size && h->tokens == a.tokens;
  uint64_t counts[4];
  uint64_t sum = 0;
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    counts[c] = h->count[c];
    ok = ok && counts[c] <= a.tokens;
    sum += ok ? counts[c] : 0;
  }
  ok = ok && sum == a.tokens;
  if (!ok) return false;
  build_geom(g, a.layers, a.kv_heads, a.head_dim, a.group_size, a.tokens, counts);
  ok = g.total <= a.card_bytes && h->total_bytes == g.total;
  ok = ok && h->off_bits == g.off_bits && h->off_slot == g.off_slot && h->off_order == g.off_order &&
       h->off_fp16 == g.off_fp16;
#pragma unroll
  for (int c = 0; c < 3; ++c) ok = ok && h->off_codes[c] == g.off_codes[c] && h->off_meta[c] == g.off_meta[c];
  return ok;
}

// Row id (plane * T + token) of row `lane` of the tile starting at segment row r0, or
// 0xFFFFFFFF for rows past the segment's end and for corrupt order[] entries.
__device__ inline uint32_t tile_row_lookup(const CardGeom& g, const uint32_t* __restrict__ order, int c, uint32_t r0,
                                           uint32_t n_rows, uint32_t lane, uint32_t tile_rows, uint32_t& bad) {
  uint32_t rowid = 0xFFFFFFFFu;
  const uint32_t r = r0 + lane;
  if (lane < tile_rows && r < n_rows) {
    const uint32_t n = g.n[c];
    const uint32_t p = r / n;
    const uint32_t j = r - p * n;
    const uint32_t t = order[g.base[c] + j];
    if (t < g.tokens) rowid = p * g.tokens + t; else bad = 1;
  }
  return rowid;
}

__device__ inline uint8_t* row_address(const UnpackArgs& a, const CardGeom& g, uint32_t rowid, uint32_t row_bytes) {
  const uint64_t k_bytes = (uint64_t)g.k_rows * row_bytes;
  const uint64_t off = (uint64_t)rowid * row_bytes;
  const uint64_t addr = (rowid < g.k_rows) ? reinterpret_cast<uint64_t>(a.k_out) + off
                                           : reinterpret_cast<uint64_t>(a.v_out) + (off - k_bytes);
  return reinterpret_cast<uint8_t*>(addr);
}

typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

// decode = fp16( fma(code, scale, zero) ): an fp32 fma rounded to fp32, then rounded to
// fp16, both to nearest even.  The two steps are kept apart on purpose: the fused
// fma-and-convert instruction rounds the exact sum once, straight to fp16, which gives a
// different value whenever the fp32 result lands on an fp16 midpoint.
__device__ inline uint32_t decode_pair(uint32_t q0, uint32_t q1, float s, float z) {
  float a = __builtin_fmaf((float)q0, s, z);
  float b = __builtin_fmaf((float)q1, s, z);
  asm("" : "+v"(a));
  asm("" : "+v"(b));
  const f32x2 v = {a, b};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, f16x2));
}

template <int W, int G>
__device__ inline void unpack_tile(const UnpackArgs& a, const CardGeom& g, int c, uint32_t r0, uint32_t n_rows,
                                   uint32_t lane, uint8_t* lds_codes, uint32_t* lds_meta, uint32_t& bad) {
  constexpr int GL = G / 8;
  constexpr uint32_t MASK = (1u << W) - 1u;
  const uint32_t lpr_shift = g.lpr_shift;
  const uint32_t tile_rows = kTileChunks >> lpr_shift;
  const uint32_t row_bytes = g.head_dim * 2u;
  const uint32_t* order = reinterpret_cast<const uint32_t*>(a.card + g.off_order);
  const uint32_t my_row = tile_row_lookup(g, order, c, r0, n_rows, lane, tile_rows, bad);

  // stage the tile's codes and pairs
  {
    const uint64_t seg_bytes = (uint64_t)n_rows * (g.head_dim * W / 8);
    const uint64_t tile_off = (uint64_t)r0 * (g.head_dim * W / 8);
    const uint8_t* src = a.card + g.off_codes[c];
#pragma unroll
    for (int m = 0; m < W / 2; ++m) {
      const uint32_t idx = m * kWaveSize + lane;
      const uint64_t off = tile_off + (uint64_t)idx * 16u;
      uint4 v = make_uint4(0, 0, 0, 0);
      if (off < seg_bytes) v = *reinterpret_cast<const uint4*>(src + off);
      reinterpret_cast<uint4*>(lds_codes)[idx] = v;
    }
    constexpr int kDwords = kTileChunks / GL;
    const uint64_t seg_dwords = (uint64_t)n_rows * (g.head_dim / G);
    const uint64_t tile_dw = (uint64_t)r0 * (g.head_dim / G);
    const uint32_t* msrc = reinterpret_cast<const uint32_t*>(a.card + g.off_meta[c]);
#pragma unroll
    for (int m = 0; m < (kDwords + kWaveSize - 1) / kWaveSize; ++m) {
      const uint32_t idx = m * kWaveSize + lane;
      if (idx < (uint32_t)kDwords) lds_meta[idx] = (tile_dw + idx < seg_dwords) ? msrc[tile_dw + idx] : 0u;
    }
  }
  __builtin_amdgcn_wave_barrier();

#pragma unroll
  for (int k = 0; k < kTileIters; ++k) {
    const uint32_t q = k * kWaveSize + lane;
    const uint32_t rowid = __shfl(my_row, q >> lpr_shift, kWaveSize);
    const uint32_t pair = lds_meta[q / GL];
    const float s = half_bits_to_float(pair & 0xFFFFu);
    const float z = half_bits_to_float(pair >> 16);
    uint32_t lo = 0, hi = 0;      // the chunk's 8 codes, W bits each, little end first
    if (W == 2) lo = reinterpret_cast<const uint16_t*>(lds_codes)[q];
    if (W == 4) lo = reinterpret_cast<const uint32_t*>(lds_codes)[q];
    if (W == 8) { const uint2 t = reinterpret_cast<const uint2*>(lds_codes)[q]; lo = t.x; hi = t.y; }
    uint32_t code[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      if (W == 8) code[i] = ((i < 4 ? lo : hi) >> (8 * (i & 3))) & MASK;
      else code[i] = (lo >> (W * i)) & MASK;
    }
    uint4 out;
    out.x = decode_pair(code[0], code[1], s, z);
    out.y = decode_pair(code[2], code[3], s, z);
    out.z = decode_pair(code[4], code[5], s, z);
    out.w = decode_pair(code[6], code[7], s, z);
    if (rowid != 0xFFFFFFFFu) {
      uint8_t* dst = row_address(a, g, rowid, row_bytes) + (q & ((1u << lpr_shift) - 1u)) * 16u;
      *reinterpret_cast<uint4*>(dst) = out;
    }
  }
  __builtin_amdgcn_wave_barrier();
}

__device__ inline void copy_tile(const UnpackArgs& a, const CardGeom& g, uint32_t r0, uint32_t n_rows, uint32_t lane,
                                 uint32_t& bad) {
  const uint32_t lpr_shift = g.lpr_shift;
  const uint32_t tile_rows = kTileChunks >> lpr_shift;
  const uint32_t row_bytes = g.head_dim * 2u;
  const uint32_t* order = reinterpret_cast<const uint32_t*>(a.card + g.off_order);
  const uint32_t my_row = tile_row_lookup(g, order, 3, r0, n_rows, lane, tile_rows, bad);
  const uint8_t* src = a.card + g.off_fp16 + (uint64_t)r0 * row_bytes;
  const uint64_t seg_left = ((uint64_t)n_rows - r0) * row_bytes;   // bytes from the tile start to the segment end
  uint4 data[kTileIters];
#pragma unroll
  for (int k = 0; k < kTileIters; ++k) {
    const uint32_t q = k * kWaveSize + lane;
    data[k] = make_uint4(0, 0, 0, 0);
    if ((uint64_t)q * 16u < seg_left) data[k] = *reinterpret_cast<const uint4*>(src + (uint64_t)q * 16u);
  }
#pragma unroll
  for (int k = 0; k < kTileIters; ++k) {
    const uint32_t q = k * kWaveSize + lane;
    const uint32_t rowid = __shfl(my_row, q >> lpr_shift, kWaveSize);
    if (rowid != 0xFFFFFFFFu) {
      uint8_t* dst = row_address(a, g, rowid, row_bytes) + (q & ((1u << lpr_shift) - 1u)) * 16u;
      *reinterpret_cast<uint4*>(dst) = data[k];
    }
  }
}

// Writes the header verdict; runs before the unpacking grid on the same stream.
__global__ void unpack_status_kernel(UnpackArgs a) {
  CardGeom g;
  const bool ok = load_geometry(a, g);
  if (threadIdx.x == 0 && blockIdx.x == 0) *a.status = ok ? 0u : QKV_STATUS_BAD_HEADER;
}

template <int G>
__global__ __launch_bounds__(kBlockThreads) void unpack_kernel(UnpackArgs a) {
  __shared__ __attribute__((aligned(16))) uint8_t lds_codes[kWavesPerBlock][kTileChunks * 8];
  __shared__ uint32_t lds_meta[kWavesPerBlock][kTileChunks / 4];
  CardGeom g;
  if (!load_geometry(a, g)) return;          // uniform over the grid: every wave leaves
  const uint32_t lane = threadIdx.x & 63u;
  const uint32_t wave = threadIdx.x >> 6;
  const uint32_t gw = blockIdx.x * kWavesPerBlock + wave;
  const uint32_t n_waves = gridDim.x * kWavesPerBlock;
  const uint32_t tile_rows = kTileChunks >> g.lpr_shift;
  uint8_t* my_codes = lds_codes[wave];
  uint32_t* my_meta = lds_meta[wave];

  uint32_t bad = 0;
  uint32_t cum = 0;
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    const uint32_t n_rows = g.planes * g.n[c];
    if (n_rows == 0) continue;
    const uint32_t tiles = (n_rows + tile_rows - 1) / tile_rows;
    const uint32_t first = (gw + n_waves - cum) % n_waves;
    for (uint32_t i = first; i < tiles; i += n_waves) {
      const uint32_t r0 = i * tile_rows;
      if (c == 0) unpack_tile<2, G>(a, g, 0, r0, n_rows, lane, my_codes, my_meta, bad);
      if (c == 1) unpack_tile<4, G>(a, g, 1, r0, n_rows, lane, my_codes, my_meta, bad);
      if (c == 2) unpack_tile<8, G>(a, g, 2, r0, n_rows, lane, my_codes, my_meta, bad);
      if (c == 3) copy_tile(a, g, r0, n_rows, lane, bad);
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
  const dim3 grid(persistent_blocks(tiles)), block(kBlockThreads);
  switch (expect.group_size) {
    case 32: hipLaunchKernelGGL(unpack_kernel<32>, grid, block, 0, stream, a); break;
    case 64: hipLaunchKernelGGL(unpack_kernel<64>, grid, block, 0, stream, a); break;
    default: hipLaunchKernelGGL(unpack_kernel<128>, grid, block, 0, stream, a); break;
  }
  return hipGetLastError();
}

}  // namespace qkv
