// qkv_common.h — geometry of a card and small device helpers shared by the HIP kernels.
// Internal to the GPU library (not part of the C ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/qkvcard.h"

namespace qkv {

constexpr int kWaveSize = 64;
#ifndef QKV_TILE_CHUNKS
#define QKV_TILE_CHUNKS 512
#endif
constexpr int kTileChunks = QKV_TILE_CHUNKS;   // 16-byte fp16 chunks one wave handles per tile (8 per lane)
constexpr int kTileIters = kTileChunks / kWaveSize;
constexpr int kTileRounds = kTileChunks / (4 * kWaveSize);   // spans of 32 values per lane and tile
static_assert(kTileChunks % (4 * kWaveSize) == 0 && kTileChunks >= 256 && kTileChunks <= 512,
              "a tile is a whole number of 64-span rounds and at most 64 rows at head_dim 64");
#ifndef QKV_BLOCK_THREADS
#define QKV_BLOCK_THREADS 256
#endif
constexpr int kBlockThreads = QKV_BLOCK_THREADS;      // independent waves, 4 per workgroup
constexpr int kWavesPerBlock = kBlockThreads / kWaveSize;

// Cards up to this size are written and read with plain accesses so that they stay in the
// 256 MB memory-side cache between packing and unpacking; larger ones are streamed past it
// (measured: 267 and 302 MB cards are faster kept, a 1.8 GB card 4 % faster streamed).
constexpr uint64_t kCacheResidentCardBytes = 512ull << 20;

// Everything a kernel needs to find its way around a card.  Built on the host for the
// packing kernels (counts are an argument there) and rebuilt on the device from the header
// for unpacking.
struct CardGeom {
  uint32_t layers, kv_heads, head_dim, group_size;
  uint32_t tokens;          // T
  uint32_t planes;          // P = 2 * L * H
  uint32_t k_rows;          // L * H * T: rows (plane, token) below this belong to K
  uint32_t lpr_shift;       // log2(lanes per row) = log2(head_dim / 8)
  uint32_t n[4];            // tokens per class (widths 2, 4, 8, 16)
  uint32_t base[4];         // first index of each class inside order[]
  uint64_t off_bits, off_slot, off_order;
  uint64_t off_codes[3], off_meta[3];
  uint64_t off_fp16;
  uint64_t total;
};

__host__ __device__ inline uint64_t align256(uint64_t x) { return (x + 255u) & ~(uint64_t)255u; }

__host__ __device__ inline uint32_t width_of_class(int c) { return 2u << c; }   // 2, 4, 8, 16

// Fills every field from (L, H, D, G, T) and the four class counts.  Shape must have been
// validated by the caller.
__host__ __device__ inline void build_geom(CardGeom& g, uint32_t L, uint32_t H, uint32_t D, uint32_t G,
                                           uint64_t T, const uint64_t counts[4]) {
  g.layers = L; g.kv_heads = H; g.head_dim = D; g.group_size = G;
  g.tokens = (uint32_t)T;
  g.planes = 2u * L * H;
  g.k_rows = L * H * (uint32_t)T;
  g.lpr_shift = (D == 64) ? 3u : (D == 128) ? 4u : 5u;
  uint32_t b = 0;
  for (int c = 0; c < 4; ++c) { g.n[c] = (uint32_t)counts[c]; g.base[c] = b; b += g.n[c]; }
  const uint64_t P = g.planes;
  uint64_t off = QKV_CARD_HEADER_BYTES;
  g.off_bits = off;  off += align256(T);
  g.off_slot = off;  off += align256(4 * T);
  g.off_order = off; off += align256(4 * T);
  for (int c = 0; c < 3; ++c) {
    const uint64_t row_bytes = (uint64_t)D * width_of_class(c) / 8;
    g.off_codes[c] = off; off += align256(P * counts[c] * row_bytes);
    g.off_meta[c] = off;  off += align256(P * counts[c] * (uint64_t)(D / G) * 4);
  }
  g.off_fp16 = off; off += align256(P * counts[3] * (uint64_t)D * 2);
  g.total = off;
}

// Host-side checks of the supported shape domain; returns QKV_OK or an error code.
inline int check_shape(int32_t L, int32_t H, int32_t D, int32_t G, int64_t T) {
  if (L < 1 || H < 1 || T < 1) return QKV_ERR_SHAPE;
  if (D != 64 && D != 128 && D != 256) return QKV_ERR_SHAPE;
  if (G != 32 && G != 64 && G != 128) return QKV_ERR_GROUP;
  if (G > D || D % G != 0) return QKV_ERR_GROUP;
  if ((int64_t)L * H > (1 << 24)) return QKV_ERR_SHAPE;
  const uint64_t rows = 2ull * (uint64_t)L * (uint64_t)H * (uint64_t)T;
  if (rows >= (1ull << 32)) return QKV_ERR_SHAPE;
  return QKV_OK;
}

inline int check_counts(int64_t T, const int64_t counts[4]) {
  int64_t sum = 0;
  for (int c = 0; c < 4; ++c) {
    if (counts[c] < 0 || counts[c] > T) return QKV_ERR_COUNTS;
    sum += counts[c];
  }
  return sum == T ? QKV_OK : QKV_ERR_COUNTS;
}

// Inclusive prefix sum over the 64 lanes of a wave, in data-parallel-primitive moves only:
// shifts by 1, 2, 4, 8 inside each row of 16 lanes, then the last lane of row 0 / 2 is added
// to row 1 / 3 and the last lane of row 1 to rows 2 and 3.
__device__ inline uint32_t wave_inclusive_scan(uint32_t v) {
  v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x111, 0xF, 0xF, true);    // row_shr:1
  v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x112, 0xF, 0xF, true);    // row_shr:2
  v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x114, 0xF, 0xF, true);    // row_shr:4
  v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x118, 0xF, 0xF, true);    // row_shr:8
  v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x142, 0xA, 0xF, false);   // row_bcast:15 -> rows 1, 3
  v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x143, 0xC, 0xF, false);   // row_bcast:31 -> rows 2, 3
  return v;
}

// One wave finds the bucket that holds rank `left` in a 256-bucket histogram: the first d
// whose cumulative count exceeds `left`.  Returns d, lowers `left` by the count before it and
// gives that bucket's own count in `in_bucket`.  The histogram's total must exceed `left`.
__device__ inline uint32_t find_bucket(const uint32_t* hist, uint32_t lane, uint32_t& left, uint32_t& in_bucket) {
  const uint32_t h0 = hist[4 * lane], h1 = hist[4 * lane + 1], h2 = hist[4 * lane + 2], h3 = hist[4 * lane + 3];
  const uint32_t inc = wave_inclusive_scan(h0 + h1 + h2 + h3);
  const uint64_t over = __builtin_amdgcn_ballot_w64(inc > left);
  const int owner = (int)__builtin_ctzll(over | (1ull << 63));        // the same in every lane: plain lane reads
  const uint32_t before = (uint32_t)__builtin_amdgcn_readlane((int)(inc - (h0 + h1 + h2 + h3)), owner);
  const uint32_t a0 = (uint32_t)__builtin_amdgcn_readlane((int)h0, owner), a1 = (uint32_t)__builtin_amdgcn_readlane((int)h1, owner),
                 a2 = (uint32_t)__builtin_amdgcn_readlane((int)h2, owner), a3 = (uint32_t)__builtin_amdgcn_readlane((int)h3, owner);
  uint32_t rest = left - before;
  uint32_t d = 4u * (uint32_t)owner;
  in_bucket = a0;
  if (rest >= a0) {
    rest -= a0; ++d; in_bucket = a1;
    if (rest >= a1) {
      rest -= a1; ++d; in_bucket = a2;
      if (rest >= a2) { rest -= a2; ++d; in_bucket = a3; }
    }
  }
  left = rest;
  return d;
}
__device__ inline uint32_t find_bucket(const uint32_t* hist, uint32_t lane, uint32_t& left) {
  uint32_t in_bucket;
  return find_bucket(hist, lane, left, in_bucket);
}

// Number of workgroups for a streaming kernel with `tiles` wave-tiles of work.
int grid_blocks(uint64_t tiles);

// Kernel launchers (one per source file).  All enqueue on `stream` and return a hipError_t.
hipError_t launch_classify(const uint8_t* bits, const CardGeom& geom, const qkv_card_header_t& header,
                           uint8_t* card, hipStream_t stream);
hipError_t launch_pack(const CardGeom& geom, const void* k, const void* v, uint8_t* card, bool keys_per_channel,
                       hipStream_t stream);
hipError_t launch_unpack(const uint8_t* card, uint64_t card_bytes, const CardGeom& expect, void* k_out, void* v_out,
                         uint32_t* status, bool keys_per_channel, hipStream_t stream);
hipError_t launch_inject(const uint8_t* card, uint64_t card_bytes, const CardGeom& expect, uint32_t layer_begin,
                         uint32_t layer_count, void* const* k_layers, void* const* v_layers, uint64_t head_stride_bytes,
                         uint64_t token_stride_bytes, const float (*cos_sin)[2], bool keys_per_channel, uint32_t* status,
                         hipStream_t stream);
hipError_t launch_requant(const uint8_t* card_in, uint64_t card_in_bytes, const CardGeom& out, uint8_t* card_out,
                          uint32_t* status, hipStream_t stream);
hipError_t launch_assign(const float* scores, uint32_t tokens, const uint32_t cuts[3], uint8_t* bits,
                         hipStream_t stream);
uint32_t assign_plan_max_tokens();      // longest sequence launch_assign_plan takes
hipError_t launch_assign_plan(const float* scores, const uint32_t cuts[3], uint8_t* bits, const CardGeom& geom,
                              const qkv_card_header_t& header, uint8_t* card, hipStream_t stream);
void attend_plan(uint64_t tokens, uint32_t rep, uint64_t pairs, uint32_t* chunk, uint32_t* max_tasks);
hipError_t launch_attend(const uint8_t* card, uint64_t card_bytes, const CardGeom& expect, const void* q,
                         uint32_t q_heads, float softmax_scale, float* out, float* lse, float* workspace,
                         uint32_t* status, bool keys_per_channel, hipStream_t stream);
hipError_t attend_static_scratch(float** ptr);     // the current device's copy of the static scratch array
hipError_t launch_count(const uint8_t* bits, uint64_t tokens, unsigned long long* counts4, hipStream_t stream);
hipError_t launch_controller(const float* features, uint32_t tokens, const qkv_controller_t& params, float* scores,
                             hipStream_t stream);
hipError_t launch_greedy(const float* scores, uint32_t tokens, uint32_t spare_units, uint8_t* bits,
                         unsigned long long* counts4, hipStream_t stream);

}  // namespace qkv
