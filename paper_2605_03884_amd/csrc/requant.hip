// requant.hip — one hop of a multi-hop chain without the dense cache in between (paper Sec. 3.2,
// challenge 3: a cache is forwarded from agent to agent; Sec. 4.2: a card is what travels).
//
// An agent that forwards a card at new bit widths would otherwise rebuild the dense fp16 cache
// (injection) and build the next card from it (card creation): 2 x (dense + card) bytes of traffic.
// Here every span of 32 values is read from the incoming card, decoded with the injection kernel's
// decoder, quantized with the card-creation kernel's quantizer and stored into the outgoing card; the
// dense values only ever exist in registers.  The result is, byte for byte, the card that creation
// would build from the injected cache.
//
// Work decomposition: the outgoing card's segments are walked as in card creation, a wave taking 64 rows
// at a time, one per lane.  A lane finds its row's token through the outgoing card's order[] (written
// by the classification kernel just before, on the same stream) and the token's old width and slot
// through the incoming card's tables.  Neighbouring rows of an outgoing segment had different old
// widths, and the decoders of different widths can only run one after the other under lane masks, so
// the 64 rows are first sorted by old width (ballots and one cross-lane permutation); the rounds that
// follow then see one width each, except where two widths meet.  The work is bound by instruction
// issue, not by memory.  The only LDS is the selector table of the 2-bit decoder.
//
// The incoming card is untrusted: header and offsets are rebuilt and checked on the device, table
// entries are bounded before they are used.
#include "qkv_common.h"
#include "qkv_encode.h"

namespace qkv {
namespace {

// The rows of a turn leave in sorted order, their pieces a few rounds apart: plain stores let the L2 put whole
// lines together whatever the card's size (nontemporal ones cost 14 - 50 % on 1 - 2 GB cards).
constexpr bool kMergeStores = true;

struct RequantArgs {
  const uint8_t* card_in;
  uint64_t card_in_bytes;
  uint32_t layers, kv_heads, head_dim, group_size;
  uint64_t tokens;
  CardGeom out;                 // the outgoing card's geometry (host-known counts)
  uint8_t* card_out;
  uint32_t* status;             // may be null
};

__global__ void requant_status_kernel(RequantArgs a) {
  CardGeom g;
  const bool ok = card_geometry_from_header(a.card_in, a.card_in_bytes, a.layers, a.kv_heads, a.head_dim, a.group_size,
                                            a.tokens, g);
  if (threadIdx.x == 0 && blockIdx.x == 0) *a.status = ok ? 0u : QKV_STATUS_BAD_HEADER;
}

// The 32 values (16 packed pairs) of span q of the row (plane p, slot) of old class CO of the incoming card.
// One instance per old class, so that every geometry field is picked at compile time.
template <int CO, int G, bool KEEP>
__device__ __forceinline__ void decode_old_class(const uint8_t* card, const CardGeom& in, uint32_t p, uint32_t slot,
                                                 uint32_t q, uint32_t spr_shift, const u32x2* table, uint32_t (&w)[16],
                                                 uint32_t& bad) {
  constexpr int GS = G / 32;
  const uint32_t n_old = in.n[CO];
  if (slot >= n_old) { bad = 1; return; }
  const uint64_t gsp = (((uint64_t)p * n_old + slot) << spr_shift) + q;
  if constexpr (CO == 3) {
    const u32x4* src = reinterpret_cast<const u32x4*>(card + in.off_fp16 + gsp * 64u);
#pragma unroll
    for (int h = 0; h < 4; ++h) {
      const u32x4 v = card_load<KEEP>(src + h);
      w[4 * h] = v.x; w[4 * h + 1] = v.y; w[4 * h + 2] = v.z; w[4 * h + 3] = v.w;
    }
  } else {
    constexpr int W = CO == 0 ? 2 : CO == 1 ? 4 : 8;
    const uint32_t pair = card_load<KEEP>(reinterpret_cast<const uint32_t*>(card + in.off_meta[CO]) + gsp / GS);
    const float s = half_bits_to_float(pair & 0xFFFFu);
    const float z = half_bits_to_float(pair >> 16);
    const uint8_t* src = card + in.off_codes[CO] + gsp * (4u * W);
    uint32_t cw[W];
    if constexpr (W == 2) {
      const u32x2 v = card_load<KEEP>(reinterpret_cast<const u32x2*>(src));
      cw[0] = v.x; cw[1] = v.y;
    } else {
#pragma unroll
      for (int h = 0; h < W / 4; ++h) {
        const u32x4 v = card_load<KEEP>(reinterpret_cast<const u32x4*>(src) + h);
        cw[4 * h] = v.x; cw[4 * h + 1] = v.y; cw[4 * h + 2] = v.z; cw[4 * h + 3] = v.w;
      }
    }
    if constexpr (W == 2) decode_span2_select(cw, s, z, reinterpret_cast<const uint8_t*>(table), w);      // most spans at low budgets: by selection
    else decode_span<W>(cw, s, z, w);
  }
}

// What a lane knows about one row of a turn: where its values lie in the incoming card.
struct RowDesc {
  uint32_t cls;     // old class 0..3; 4: the tables point outside the incoming card (the row becomes zeros); 5: no row
  uint32_t slot;    // the token's slot in its old segment
  uint32_t plane;
};

// The rows of outgoing class C, 64 per wave and turn (one per lane), dealt round-robin and continuing
// where the previous class stopped.  A turn first looks its 64 rows up (token through the outgoing
// order[], old width and slot through the incoming tables), then sorts them by old class with six
// ballots, so that the 64 spans of a round mostly share one decoder, and works through them in
// head_dim / 32 rounds; lane l of round k takes span (k * 64 + l) mod (spans per row) of sorted row
// (k * 64 + l) / (spans per row).  The next turn's look-ups are in flight meanwhile.
template <int C, int G, bool KEEP>
__device__ __forceinline__ void requant_class(const RequantArgs& a, const CardGeom& in, uint32_t gw, uint32_t n_waves, uint32_t lane,
                                     const u32x2* table, uint32_t& cum, uint32_t& bad) {
  constexpr int GS = G / 32;
  const CardGeom& out = a.out;
  const uint32_t n_new = out.n[C];
  if (n_new == 0) return;
  const uint32_t spr_shift = out.lpr_shift - 2u;                       // log2(spans per row)
  const uint32_t rounds = 1u << spr_shift;
  const uint32_t n_rows = out.planes * n_new;                          // below 2^32 by the shape rules
  const uint32_t tiles = (uint32_t)(((uint64_t)n_rows + kWaveSize - 1u) / kWaveSize);
  const uint32_t* order_out = reinterpret_cast<const uint32_t*>(a.card_out + out.off_order) + out.base[C];
  const uint32_t first = (gw + n_waves - cum) % n_waves;

  auto look_up = [&](uint32_t i) -> RowDesc {
    RowDesc d = {5u, 0u, 0u};
    const uint64_t r64 = (uint64_t)i * kWaveSize + lane;
    if (i < tiles && r64 < n_rows) {
      const uint32_t r = (uint32_t)r64;
      // plane without a division per lane: one for the turn's first row (the same in every lane), then at most
      // one plane boundary inside the turn's 64 rows when the class has that many tokens
      const uint32_t row_first = i * kWaveSize;
      const uint32_t plane_first = row_first / n_new;
      const uint32_t p = (n_new < (uint32_t)kWaveSize) ? r / n_new
                                                       : plane_first + (r - plane_first * n_new >= n_new ? 1u : 0u);
      d.plane = p;
      d.cls = 4u;
      const uint32_t t = order_out[r - p * n_new];
      if (t < out.tokens) {
        const uint32_t width = a.card_in[in.off_bits + t];
        const uint32_t sl = reinterpret_cast<const uint32_t*>(a.card_in + in.off_slot)[t];
        const bool ok = (width == 2 && sl < in.n[0]) || (width == 4 && sl < in.n[1]) || (width == 8 && sl < in.n[2]) ||
                        (width == 16 && sl < in.n[3]);
        if (ok) { d.cls = (width == 2) ? 0u : (width == 4) ? 1u : (width == 8) ? 2u : 3u; d.slot = sl; }
      }
    }
    return d;
  };

  RowDesc next = look_up(first);
  for (uint32_t i = first; i < tiles; i += n_waves) {
    const RowDesc mine = next;
    next = look_up(i + n_waves);                       // in flight while this turn is worked through
    if (mine.cls == 4u) bad = 1;

    // stable sort of the turn's rows by class: rank = rows of lower classes + rows of my class in lower lanes
    uint32_t rank = 0, below = 0;
#pragma unroll
    for (uint32_t k = 0; k < 6u; ++k) {
      const uint64_t m = __builtin_amdgcn_ballot_w64(mine.cls == k);
      const uint32_t before = __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
      if (mine.cls == k) rank = below + before;
      below += (uint32_t)__builtin_popcountll(m);
    }
    // lane s receives the row of rank s
    const int to = (int)(rank * 4u);
    const uint32_t s_id = (uint32_t)__builtin_amdgcn_ds_permute(to, (int)(lane | (mine.cls << 8)));
    const uint32_t s_slot = (uint32_t)__builtin_amdgcn_ds_permute(to, (int)mine.slot);
    const uint32_t s_plane = (uint32_t)__builtin_amdgcn_ds_permute(to, (int)mine.plane);

#pragma unroll 1
    for (uint32_t k = 0; k < rounds; ++k) {
      const uint32_t x = k * kWaveSize + lane;
      const int from = (int)((x >> spr_shift) * 4u);
      const uint32_t q = x & (rounds - 1u);
      const uint32_t id = (uint32_t)__builtin_amdgcn_ds_bpermute(from, (int)s_id);
      const uint32_t slot = (uint32_t)__builtin_amdgcn_ds_bpermute(from, (int)s_slot);
      const uint32_t p = (uint32_t)__builtin_amdgcn_ds_bpermute(from, (int)s_plane);
      const uint32_t cls = id >> 8;
      if (__builtin_amdgcn_ballot_w64(cls < 5u) == 0) break;            // rows that do not exist sort last
      const bool live = cls < 5u;
      uint32_t w[16];
#pragma unroll
      for (int j = 0; j < 16; ++j) w[j] = 0;
      if (cls == 0u) decode_old_class<0, G, KEEP>(a.card_in, in, p, slot, q, spr_shift, table, w, bad);
      else if (cls == 1u) decode_old_class<1, G, KEEP>(a.card_in, in, p, slot, q, spr_shift, table, w, bad);
      else if (cls == 2u) decode_old_class<2, G, KEEP>(a.card_in, in, p, slot, q, spr_shift, table, w, bad);
      else if (cls == 3u) decode_old_class<3, G, KEEP>(a.card_in, in, p, slot, q, spr_shift, table, w, bad);
      const uint64_t gsp = ((((uint64_t)i * kWaveSize) + (id & 63u)) << spr_shift) + q;    // the span's place in the outgoing segment
      if constexpr (C == 3) {
        if (live) {
          u32x4* dst = reinterpret_cast<u32x4*>(a.card_out + out.off_fp16 + gsp * 64u);
#pragma unroll
          for (int h = 0; h < 4; ++h) card_store<kMergeStores>(dst + h, (u32x4){w[4 * h], w[4 * h + 1], w[4 * h + 2], w[4 * h + 3]});
        }
      } else {
        constexpr int W = C == 0 ? 2 : C == 1 ? 4 : 8;
        uint32_t codes[W];
        const uint32_t pair = quantize_span<W, GS>(w, codes);        // every lane takes part: groups span lanes
        if (live) {
          uint8_t* dst = a.card_out + out.off_codes[C] + gsp * (4u * W);
          if (W == 2) card_store<kMergeStores>(reinterpret_cast<u32x2*>(dst), (u32x2){codes[0], codes[1]});
          if (W >= 4) card_store<kMergeStores>(reinterpret_cast<u32x4*>(dst), (u32x4){codes[0], codes[1], codes[2], codes[3]});
          if (W == 8) card_store<kMergeStores>(reinterpret_cast<u32x4*>(dst + 16), (u32x4){codes[4], codes[5], codes[6], codes[7]});
          if ((gsp & (GS - 1)) == 0)
            card_store<kMergeStores>(reinterpret_cast<uint32_t*>(a.card_out + out.off_meta[C]) + gsp / GS, pair);
        }
      }
    }
  }
  cum = (cum + tiles) % n_waves;
}

template <int G, bool KEEP>
__global__ __launch_bounds__(kBlockThreads) void requant_kernel(RequantArgs a) {
  __shared__ u32x2 tables[kWavesPerBlock][256];      // selector tables of the 2-bit decoder
  CardGeom in;
  if (!card_geometry_from_header(a.card_in, a.card_in_bytes, a.layers, a.kv_heads, a.head_dim, a.group_size, a.tokens, in))
    return;                                   // uniform over the grid
  const uint32_t lane = threadIdx.x & 63u;
  const uint32_t wave = threadIdx.x >> 6;
  const uint32_t gw = blockIdx.x * kWavesPerBlock + wave;
  const uint32_t n_waves = gridDim.x * kWavesPerBlock;
  build_select_table(tables[wave], lane);      // each wave its own copy: no barrier, fewer bank conflicts
  const u32x2* table = tables[wave];
  uint32_t bad = 0, cum = 0;
  requant_class<0, G, KEEP>(a, in, gw, n_waves, lane, table, cum, bad);
  requant_class<1, G, KEEP>(a, in, gw, n_waves, lane, table, cum, bad);
  requant_class<2, G, KEEP>(a, in, gw, n_waves, lane, table, cum, bad);
  requant_class<3, G, KEEP>(a, in, gw, n_waves, lane, table, cum, bad);
  if (bad && a.status) atomicOr(a.status, QKV_STATUS_BAD_ORDER);
}

}  // namespace

hipError_t launch_requant(const uint8_t* card_in, uint64_t card_in_bytes, const CardGeom& out, uint8_t* card_out,
                          uint32_t* status, hipStream_t stream) {
  RequantArgs a;
  a.card_in = card_in;
  a.card_in_bytes = card_in_bytes;
  a.layers = out.layers; a.kv_heads = out.kv_heads; a.head_dim = out.head_dim; a.group_size = out.group_size;
  a.tokens = out.tokens;
  a.out = out;
  a.card_out = card_out;
  a.status = status;
  if (status) {
    hipLaunchKernelGGL(requant_status_kernel, dim3(1), dim3(kWaveSize), 0, stream, a);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  uint64_t tiles = 0;                           // turns: 64 rows each
  for (int c = 0; c < 4; ++c) tiles += ((uint64_t)out.planes * out.n[c] + kWaveSize - 1u) / kWaveSize;
  if (tiles == 0) return hipSuccess;
  // A wave's start-up (header checks, selector table) costs about as much as 128 spans, and the kernel is bound
  // by instruction issue: several turns per wave once there are enough waves to fill the chip several times over
  // (measured at 8K tokens: 261 us against 280 us with 128 spans per wave).
  const uint64_t fill = 8192;
  const uint64_t per_wave = out.head_dim >= 256u ? 1u : out.head_dim == 128u ? 2u : 4u;      // 512 spans
  uint64_t waves = (tiles + per_wave - 1) / per_wave;
  if (waves < fill) waves = tiles < fill ? tiles : fill;
  const dim3 grid(grid_blocks(waves)), block(kBlockThreads);
  const bool keep = out.total <= kCacheResidentCardBytes && card_in_bytes <= kCacheResidentCardBytes;
  switch (out.group_size * 2 + (keep ? 1 : 0)) {
    case 65: hipLaunchKernelGGL((requant_kernel<32, true>), grid, block, 0, stream, a); break;
    case 64: hipLaunchKernelGGL((requant_kernel<32, false>), grid, block, 0, stream, a); break;
    case 129: hipLaunchKernelGGL((requant_kernel<64, true>), grid, block, 0, stream, a); break;
    case 128: hipLaunchKernelGGL((requant_kernel<64, false>), grid, block, 0, stream, a); break;
    case 257: hipLaunchKernelGGL((requant_kernel<128, true>), grid, block, 0, stream, a); break;
    default: hipLaunchKernelGGL((requant_kernel<128, false>), grid, block, 0, stream, a); break;
  }
  return hipGetLastError();
}

}  // namespace qkv
