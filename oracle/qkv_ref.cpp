// qkv_ref.cpp — CPU oracle for CacheCard creation and receiver-side dequantization.
//
// TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, single-threaded statement of
// what the GPU library must compute.  Nothing in the product path may call it; only the
// tests, the smoke check and the benchmark's CPU-baseline leg do.  It shares no code,
// header or table with the GPU library: every constant below is written out again from
// the layout description, on purpose.
//
// What it follows.  The paper (Sec. 3.1, 3.3, 4.2.1, 4.2.2) says what a card holds and
// that the receiver rebuilds fp16 K/V from it; it gives no numeric detail of the
// quantizer and no byte layout.  The readings taken here (group axis, asymmetric
// min-max, fp32 arithmetic order, fp16 scale/zero, little-endian code packing, segment
// layout, rank-quantile allocator) are listed in the repository's design notes; each
// function names the one it implements.
//
// Pins (tests marked "not gpu"): closed-form card size; fp16 rows passing through
// bit-for-bit; exact round trip of values already on the quantization grid; error
// bound scale/2 (+ output rounding); min -> code 0, max -> code qmax; brute-force
// nearest-code search in exact rational arithmetic on tiny inputs; numpy float16/float32
// re-computation of scale, codes and decode for uniform cards; exhaustive fp16<->fp32
// conversion against numpy; hand-written packed bytes; permutation properties of
// slot/order; closed-form counts, monotonicity, tie rule and permutation equivariance
// of the allocator.
// Parity unpinned: how well these codes preserve model accuracy (needs the paper's
// model weights and evaluation set, which are not available).

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <vector>

namespace {

// ---------------------------------------------------------------------------------
// IEEE binary16 <-> binary32, written out (no compiler half type, no F16C).
// ---------------------------------------------------------------------------------

float half_to_float(uint16_t h) {
  const uint32_t sign = (uint32_t)(h >> 15) << 31;
  const uint32_t exp = (h >> 10) & 0x1f;
  const uint32_t man = h & 0x3ff;
  uint32_t out;
  if (exp == 0) {
    if (man == 0) {
      out = sign;                                   // signed zero
    } else {
      // subnormal: value = man * 2^-24, exact in binary32
      float f = std::ldexp((float)man, -24);
      std::memcpy(&out, &f, 4);
      out |= sign;
    }
  } else if (exp == 31) {
    out = sign | 0x7f800000u | (man << 13);         // inf / NaN, payload kept
  } else {
    out = sign | ((exp + 112) << 23) | (man << 13); // rebias 15 -> 127
  }
  float f;
  std::memcpy(&f, &out, 4);
  return f;
}

// Round-to-nearest-even conversion of a binary32 to binary16 bits.
uint16_t float_to_half_rne(float f) {
  uint32_t x;
  std::memcpy(&x, &f, 4);
  const uint16_t sign = (uint16_t)((x >> 16) & 0x8000);
  const uint32_t absx = x & 0x7fffffffu;
  if (absx >= 0x7f800000u) {                        // inf or NaN
    if (absx == 0x7f800000u) return sign | 0x7c00;
    uint16_t payload = (uint16_t)((absx >> 13) & 0x3ff);
    if (payload == 0) payload = 0x200;              // keep it a NaN
    return sign | 0x7c00 | payload;
  }
  // Work on the magnitude in units of the target's last place.
  // value = m * 2^(e-23) with m in [2^23, 2^24) for normal binary32 inputs.
  int e = (int)(absx >> 23);
  uint32_t m = absx & 0x7fffffu;
  if (e == 0) {
    // binary32 subnormal: far below half of the smallest binary16 subnormal (2^-25)
    return sign;
  }
  m |= 0x800000u;
  e -= 127;                                         // unbiased exponent of the leading bit
  if (e > 15) return sign | 0x7c00;                 // beyond the largest finite half even before rounding
  int shift;                                        // how many low bits of m are dropped
  int he;                                           // biased half exponent field before rounding carry
  if (e >= -14) {                                   // normal half range
    shift = 13;
    he = e + 15;
  } else {                                          // subnormal half: last place is 2^-24
    shift = 13 + (-14 - e);
    he = 0;
    if (shift > 25) return sign;                    // below 2^-26: rounds to zero
  }
  uint32_t kept = m >> shift;
  const uint32_t rem = m & ((1u << shift) - 1u);
  const uint32_t half = 1u << (shift - 1);
  if (rem > half || (rem == half && (kept & 1u))) kept += 1;
  uint32_t bits;
  if (he == 0) {
    bits = kept;                                    // may carry into exponent field 1: correct
  } else {
    bits = ((uint32_t)he << 10) + (kept - 0x400u);  // kept has the hidden bit at 2^10; carry moves up
  }
  if (bits >= 0x7c00u) return sign | 0x7c00;        // rounded up to infinity
  return sign | (uint16_t)bits;
}

// Key that orders binary16 bit patterns like the IEEE total order on non-NaN values
// (-0 below +0).  Larger key = larger value.
inline uint16_t half_order_key(uint16_t h) {
  return (h & 0x8000) ? (uint16_t)~h : (uint16_t)(h | 0x8000);
}

// Same for binary32 bit patterns.
inline uint32_t float_order_key(uint32_t x) {
  return (x & 0x80000000u) ? ~x : (x | 0x80000000u);
}

// ---------------------------------------------------------------------------------
// Card geometry
// ---------------------------------------------------------------------------------

struct RefDesc {            // same fields, same order as the library's descriptor
  int32_t layers, kv_heads, head_dim, group_size;
  int64_t tokens;
  uint64_t model_id, sender_id;
  int64_t position_offset;
};

struct Layout {
  uint64_t planes;
  uint64_t off_bits, off_slot, off_order;
  uint64_t off_codes[3], off_meta[3];
  uint64_t off_fp16;
  uint64_t total;
  uint64_t row_bytes[3];    // bytes of one packed row for widths 2, 4, 8
  uint64_t meta_bytes;      // bytes of one row's (scale, zero) pairs
};

const int kWidth[4] = {2, 4, 8, 16};

inline uint64_t round_up_256(uint64_t x) { return (x + 255u) / 256u * 256u; }

enum {
  kOk = 0, kErrNull = -1, kErrShape = -2, kErrGroup = -3, kErrBudget = -4,
  kErrCapacity = -5, kErrAlign = -6, kErrCounts = -7, kErrFormat = -9, kErrBits = -10
};

int check_desc(const RefDesc* d) {
  if (!d) return kErrNull;
  if (d->layers < 1 || d->kv_heads < 1 || d->tokens < 1 || d->head_dim < 4) return kErrShape;
  if (d->group_size < 4 || d->group_size % 4 != 0) return kErrGroup;
  if (d->head_dim % d->group_size != 0) return kErrGroup;
  return kOk;
}

int check_counts(const RefDesc* d, const int64_t counts[4]) {
  if (!counts) return kErrNull;
  int64_t sum = 0;
  for (int c = 0; c < 4; ++c) {
    if (counts[c] < 0) return kErrCounts;
    sum += counts[c];
  }
  return sum == d->tokens ? kOk : kErrCounts;
}

// Section offsets of the card: header, bits, slot, order, then for each of the widths
// 2, 4, 8 the code rows followed by the (scale, zero) pairs, then the raw fp16 rows.
Layout make_layout(const RefDesc& d, const int64_t counts[4]) {
  Layout lay{};
  const uint64_t T = (uint64_t)d.tokens, D = (uint64_t)d.head_dim, G = (uint64_t)d.group_size;
  lay.planes = 2ull * (uint64_t)d.layers * (uint64_t)d.kv_heads;
  lay.meta_bytes = (D / G) * 4;
  uint64_t off = 256;
  lay.off_bits = off;  off += round_up_256(T);
  lay.off_slot = off;  off += round_up_256(4 * T);
  lay.off_order = off; off += round_up_256(4 * T);
  for (int c = 0; c < 3; ++c) {
    lay.row_bytes[c] = D * (uint64_t)kWidth[c] / 8;
    lay.off_codes[c] = off; off += round_up_256(lay.planes * (uint64_t)counts[c] * lay.row_bytes[c]);
    lay.off_meta[c] = off;  off += round_up_256(lay.planes * (uint64_t)counts[c] * lay.meta_bytes);
  }
  lay.off_fp16 = off; off += round_up_256(lay.planes * (uint64_t)counts[3] * D * 2);
  lay.total = off;
  return lay;
}

void put_u32(uint8_t* p, uint32_t v) { for (int i = 0; i < 4; ++i) p[i] = (uint8_t)(v >> (8 * i)); }
void put_u64(uint8_t* p, uint64_t v) { for (int i = 0; i < 8; ++i) p[i] = (uint8_t)(v >> (8 * i)); }
uint32_t get_u32(const uint8_t* p) { uint32_t v = 0; for (int i = 0; i < 4; ++i) v |= (uint32_t)p[i] << (8 * i); return v; }
uint64_t get_u64(const uint8_t* p) { uint64_t v = 0; for (int i = 0; i < 8; ++i) v |= (uint64_t)p[i] << (8 * i); return v; }

int class_of_width(uint8_t b) {
  switch (b) { case 2: return 0; case 4: return 1; case 8: return 2; case 16: return 3; default: return -1; }
}

// ---------------------------------------------------------------------------------
// Quantizer for one group
// ---------------------------------------------------------------------------------

// Asymmetric min-max quantization of n fp16 values at `width` bits.  fp32 arithmetic in
// this exact order; scale is stored rounded to fp16 and that stored value is what both
// sides use; the zero point is the group minimum itself.
void quantize_group(const uint16_t* x, int n, int width, uint16_t* scale_h, uint16_t* zero_h, uint8_t* codes) {
  uint16_t mn = x[0], mx = x[0];
  for (int i = 1; i < n; ++i) {
    if (half_order_key(x[i]) < half_order_key(mn)) mn = x[i];
    if (half_order_key(x[i]) > half_order_key(mx)) mx = x[i];
  }
  const int qmax = (1 << width) - 1;
  const float fmn = half_to_float(mn);
  const float fmx = half_to_float(mx);
  const volatile float range = fmx - fmn;            // volatile: one fp32 rounding per step
  const volatile float s32 = range / (float)qmax;
  const uint16_t sh = float_to_half_rne(s32);
  const float s = half_to_float(sh);
  volatile float inv = 0.0f;
  if (s > 0.0f) inv = 1.0f / s;
  for (int i = 0; i < n; ++i) {
    const volatile float d = half_to_float(x[i]) - fmn;
    // 24-bit x 24-bit product is exact in binary64; one rounding, ties to even
    const double r = std::nearbyint((double)d * (double)inv);
    int q = (int)r;
    if (q > qmax) q = qmax;
    codes[i] = (uint8_t)q;
  }
  *scale_h = sh;
  *zero_h = mn;
}

// decode = fp16( fma(code, scale, zero) ), the fma in fp32 with a single rounding.
uint16_t dequantize_one(uint8_t code, uint16_t scale_h, uint16_t zero_h) {
  const float r = std::fmaf((float)code, half_to_float(scale_h), half_to_float(zero_h));
  return float_to_half_rne(r);
}

// Code i of a row occupies bits [(i*w) mod 8, +w) of byte floor(i*w/8).
void pack_codes(const uint8_t* codes, int n, int width, uint8_t* out) {
  const int nbytes = n * width / 8;
  for (int i = 0; i < nbytes; ++i) out[i] = 0;
  for (int i = 0; i < n; ++i) {
    const int bit = i * width;
    out[bit / 8] |= (uint8_t)(codes[i] << (bit % 8));
  }
}

void unpack_codes(const uint8_t* in, int n, int width, uint8_t* codes) {
  const int mask = (1 << width) - 1;
  for (int i = 0; i < n; ++i) {
    const int bit = i * width;
    codes[i] = (uint8_t)((in[bit / 8] >> (bit % 8)) & mask);
  }
}

// ---------------------------------------------------------------------------------
// Budget -> class counts, scores -> bits
// ---------------------------------------------------------------------------------

// Piecewise-linear mix between all-2-bit (budget 2), 30/40/25/5 % of 2/4/8/16 bit
// (budget 5) and all-fp16 (budget 16), in integers on budget*1000, floors everywhere.
int budget_counts(int64_t T, double budget, int64_t counts[4]) {
  if (!(budget >= 2.0 && budget <= 16.0)) return kErrBudget;   // also rejects NaN
  if (T < 1) return kErrShape;
  const long long bm = std::llrint(budget * 1000.0);
  if (bm < 2000 || bm > 16000) return kErrBudget;
  __int128 n16, n8, n4;
  if (bm <= 5000) {
    const __int128 e = bm - 2000;
    n16 = (__int128)5 * e * T / 300000;
    n8 = (__int128)25 * e * T / 300000;
    n4 = (__int128)40 * e * T / 300000;
  } else {
    const __int128 e = bm - 5000;
    n16 = (__int128)T * (5 * (11000 - e) + 100 * e) / 1100000;
    n8 = (__int128)T * 25 * (11000 - e) / 1100000;
    n4 = (__int128)T * 40 * (11000 - e) / 1100000;
  }
  counts[3] = (int64_t)n16;
  counts[2] = (int64_t)n8;
  counts[1] = (int64_t)n4;
  counts[0] = T - counts[3] - counts[2] - counts[1];
  return kOk;
}

}  // namespace

// ===================================================================================
// C entry points (host pointers everywhere)
// ===================================================================================
extern "C" {

float qkv_ref_half_to_float(uint16_t h) { return half_to_float(h); }
uint16_t qkv_ref_float_to_half(float f) { return float_to_half_rne(f); }

// Closed-form card size (layout description; leading term is the paper's size model, Sec. 3.1).
int qkv_ref_card_bytes(const RefDesc* desc, const int64_t counts[4], uint64_t* bytes_out) {
  if (!bytes_out) return kErrNull;
  int rc = check_desc(desc);
  if (rc) return rc;
  rc = check_counts(desc, counts);
  if (rc) return rc;
  *bytes_out = make_layout(*desc, counts).total;
  return kOk;
}

// All section offsets, for tests: out[0..10] = bits, slot, order, codes2, meta2, codes4,
// meta4, codes8, meta8, fp16, total.
int qkv_ref_card_offsets(const RefDesc* desc, const int64_t counts[4], uint64_t out[11]) {
  if (!out) return kErrNull;
  int rc = check_desc(desc);
  if (rc) return rc;
  rc = check_counts(desc, counts);
  if (rc) return rc;
  const Layout lay = make_layout(*desc, counts);
  out[0] = lay.off_bits; out[1] = lay.off_slot; out[2] = lay.off_order;
  for (int c = 0; c < 3; ++c) { out[3 + 2 * c] = lay.off_codes[c]; out[4 + 2 * c] = lay.off_meta[c]; }
  out[9] = lay.off_fp16; out[10] = lay.total;
  return kOk;
}

int qkv_ref_budget_counts(int64_t tokens, double budget, int64_t counts_out[4]) {
  if (!counts_out) return kErrNull;
  return budget_counts(tokens, budget, counts_out);
}

// Rank tokens by (score descending, index ascending) in the IEEE total order and hand
// out widths 16, 8, 4, 2 to consecutive rank ranges (paper Sec. 3.3: the score decides
// the width under a budget).
int qkv_ref_assign_bits(const float* scores, int64_t tokens, double budget, uint8_t* bits, int64_t counts_out[4]) {
  if (!scores || !bits || !counts_out) return kErrNull;
  int64_t counts[4];
  const int rc = budget_counts(tokens, budget, counts);
  if (rc) return rc;
  std::vector<int64_t> idx((size_t)tokens);
  for (int64_t t = 0; t < tokens; ++t) idx[(size_t)t] = t;
  std::stable_sort(idx.begin(), idx.end(), [&](int64_t a, int64_t b) {
    uint32_t xa, xb;
    std::memcpy(&xa, &scores[a], 4);
    std::memcpy(&xb, &scores[b], 4);
    return float_order_key(xa) > float_order_key(xb);   // stable: equal scores keep index order
  });
  int64_t r = 0;
  for (int64_t i = 0; i < counts[3]; ++i) bits[idx[(size_t)r++]] = 16;
  for (int64_t i = 0; i < counts[2]; ++i) bits[idx[(size_t)r++]] = 8;
  for (int64_t i = 0; i < counts[1]; ++i) bits[idx[(size_t)r++]] = 4;
  for (int64_t i = 0; i < counts[0]; ++i) bits[idx[(size_t)r++]] = 2;
  for (int c = 0; c < 4; ++c) counts_out[c] = counts[c];
  return kOk;
}

int qkv_ref_count_bits(const uint8_t* bits, int64_t tokens, int64_t counts_out[4]) {
  if (!bits || !counts_out) return kErrNull;
  for (int c = 0; c < 4; ++c) counts_out[c] = 0;
  for (int64_t t = 0; t < tokens; ++t) {
    const int c = class_of_width(bits[t]);
    if (c >= 0) counts_out[c] += 1;
  }
  return kOk;
}

// Stable bucketing by width: slot[t] = number of earlier tokens of the same width;
// order = tokens listed class by class (2, 4, 8, 16), increasing t inside a class.
int qkv_ref_compact(const uint8_t* bits, int64_t tokens, uint32_t* slot, uint32_t* order, int64_t counts_out[4]) {
  if (!bits || !slot || !order || !counts_out) return kErrNull;
  int64_t counts[4] = {0, 0, 0, 0};
  for (int64_t t = 0; t < tokens; ++t) {
    const int c = class_of_width(bits[t]);
    if (c < 0) return kErrBits;
    slot[t] = (uint32_t)counts[c];
    counts[c] += 1;
  }
  int64_t base[4];
  base[0] = 0;
  for (int c = 1; c < 4; ++c) base[c] = base[c - 1] + counts[c - 1];
  for (int64_t t = 0; t < tokens; ++t) {
    const int c = class_of_width(bits[t]);
    order[base[c] + slot[t]] = (uint32_t)t;
  }
  for (int c = 0; c < 4; ++c) counts_out[c] = counts[c];
  return kOk;
}

// One group, exposed so the tests can pin the quantizer by itself.
int qkv_ref_quantize_group(const uint16_t* x, int n, int width, uint16_t* scale_h, uint16_t* zero_h, uint8_t* codes) {
  if (!x || !scale_h || !zero_h || !codes) return kErrNull;
  if (n < 1 || (width != 2 && width != 4 && width != 8)) return kErrShape;
  quantize_group(x, n, width, scale_h, zero_h, codes);
  return kOk;
}

int qkv_ref_dequantize_group(const uint8_t* codes, int n, uint16_t scale_h, uint16_t zero_h, uint16_t* out) {
  if (!codes || !out) return kErrNull;
  for (int i = 0; i < n; ++i) out[i] = dequantize_one(codes[i], scale_h, zero_h);
  return kOk;
}

int qkv_ref_pack_codes(const uint8_t* codes, int n, int width, uint8_t* out) {
  if (!codes || !out) return kErrNull;
  if ((width != 2 && width != 4 && width != 8) || n * width % 8 != 0) return kErrShape;
  pack_codes(codes, n, width, out);
  return kOk;
}

int qkv_ref_unpack_codes(const uint8_t* in, int n, int width, uint8_t* codes) {
  if (!in || !codes) return kErrNull;
  if ((width != 2 && width != 4 && width != 8) || n * width % 8 != 0) return kErrShape;
  unpack_codes(in, n, width, codes);
  return kOk;
}

// CacheCard creation (paper Sec. 4.2.1).  k, v: fp16 bits [L][H][T][D]; card: capacity bytes.
int qkv_ref_quantize_pack(const RefDesc* desc, const uint16_t* k, const uint16_t* v, const uint8_t* bits,
                          const int64_t counts[4], uint8_t* card, uint64_t capacity) {
  if (!k || !v || !bits || !card) return kErrNull;
  int rc = check_desc(desc);
  if (rc) return rc;
  rc = check_counts(desc, counts);
  if (rc) return rc;
  const Layout lay = make_layout(*desc, counts);
  if (capacity < lay.total) return kErrCapacity;

  const int64_t T = desc->tokens;
  const int D = desc->head_dim, G = desc->group_size;
  const uint64_t planes_per_tensor = (uint64_t)desc->layers * (uint64_t)desc->kv_heads;

  // check the bits vector against the counts before touching the card
  int64_t have[4];
  qkv_ref_count_bits(bits, T, have);
  if (have[0] + have[1] + have[2] + have[3] != T) return kErrBits;
  for (int c = 0; c < 4; ++c) if (have[c] != counts[c]) return kErrCounts;

  std::memset(card, 0, (size_t)lay.total);

  // header
  std::memcpy(card + 0, "QKVCARD\0", 8);
  put_u32(card + 8, 1);
  put_u32(card + 12, 256);
  put_u32(card + 16, (uint32_t)desc->layers);
  put_u32(card + 20, (uint32_t)desc->kv_heads);
  put_u32(card + 24, (uint32_t)D);
  put_u32(card + 28, (uint32_t)G);
  put_u64(card + 32, (uint64_t)T);
  for (int c = 0; c < 4; ++c) put_u64(card + 40 + 8 * c, (uint64_t)counts[c]);
  put_u64(card + 72, lay.total);
  put_u64(card + 80, lay.off_bits);
  put_u64(card + 88, lay.off_slot);
  put_u64(card + 96, lay.off_order);
  for (int c = 0; c < 3; ++c) put_u64(card + 104 + 8 * c, lay.off_codes[c]);
  for (int c = 0; c < 3; ++c) put_u64(card + 128 + 8 * c, lay.off_meta[c]);
  put_u64(card + 152, lay.off_fp16);
  put_u64(card + 160, desc->model_id);
  put_u64(card + 168, desc->sender_id);
  put_u64(card + 176, (uint64_t)desc->position_offset);
  {
    // achieved average bit width (paper Sec. 4.2.1, "average-bit statistics")
    const double total_bits = 2.0 * (double)counts[0] + 4.0 * (double)counts[1] + 8.0 * (double)counts[2] + 16.0 * (double)counts[3];
    const float avg = (float)(total_bits / (double)T);
    uint32_t u;
    std::memcpy(&u, &avg, 4);
    put_u32(card + 184, u);
  }
  put_u32(card + 188, 0);   // flags
  put_u32(card + 192, 0);   // status

  // bits, slot, order
  std::memcpy(card + lay.off_bits, bits, (size_t)T);
  std::vector<uint32_t> slot((size_t)T), order((size_t)T);
  int64_t cnt2[4];
  rc = qkv_ref_compact(bits, T, slot.data(), order.data(), cnt2);
  if (rc) return rc;
  for (int64_t t = 0; t < T; ++t) {
    put_u32(card + lay.off_slot + 4 * (uint64_t)t, slot[(size_t)t]);
    put_u32(card + lay.off_order + 4 * (uint64_t)t, order[(size_t)t]);
  }

  // rows
  std::vector<uint8_t> codes((size_t)D);
  for (uint64_t p = 0; p < lay.planes; ++p) {
    const uint16_t* src_plane = (p < planes_per_tensor) ? k + p * (uint64_t)T * D
                                                        : v + (p - planes_per_tensor) * (uint64_t)T * D;
    for (int64_t t = 0; t < T; ++t) {
      const uint16_t* row = src_plane + (uint64_t)t * D;
      const int c = class_of_width(bits[t]);
      const uint64_t j = slot[(size_t)t];
      if (c == 3) {
        uint8_t* dst = card + lay.off_fp16 + (p * (uint64_t)counts[3] + j) * (uint64_t)D * 2;
        for (int i = 0; i < D; ++i) { dst[2 * i] = (uint8_t)(row[i] & 0xff); dst[2 * i + 1] = (uint8_t)(row[i] >> 8); }
        continue;
      }
      const int w = kWidth[c];
      uint8_t* dst_codes = card + lay.off_codes[c] + (p * (uint64_t)counts[c] + j) * lay.row_bytes[c];
      uint8_t* dst_meta = card + lay.off_meta[c] + (p * (uint64_t)counts[c] + j) * lay.meta_bytes;
      for (int g = 0; g < D / G; ++g) {
        uint16_t sh, zh;
        quantize_group(row + g * G, G, w, &sh, &zh, codes.data() + g * G);
        dst_meta[4 * g + 0] = (uint8_t)(sh & 0xff);
        dst_meta[4 * g + 1] = (uint8_t)(sh >> 8);
        dst_meta[4 * g + 2] = (uint8_t)(zh & 0xff);
        dst_meta[4 * g + 3] = (uint8_t)(zh >> 8);
      }
      pack_codes(codes.data(), D, w, dst_codes);
    }
  }
  return kOk;
}

// Header check shared by peek and unpack: returns kOk and fills desc/counts, or kErrFormat.
static int parse_header(const uint8_t* card, uint64_t card_bytes, RefDesc* d, int64_t counts[4], Layout* lay_out) {
  if (card_bytes < 256) return kErrFormat;
  if (std::memcmp(card, "QKVCARD\0", 8) != 0) return kErrFormat;
  if (get_u32(card + 8) != 1 || get_u32(card + 12) != 256) return kErrFormat;
  d->layers = (int32_t)get_u32(card + 16);
  d->kv_heads = (int32_t)get_u32(card + 20);
  d->head_dim = (int32_t)get_u32(card + 24);
  d->group_size = (int32_t)get_u32(card + 28);
  d->tokens = (int64_t)get_u64(card + 32);
  d->model_id = get_u64(card + 160);
  d->sender_id = get_u64(card + 168);
  d->position_offset = (int64_t)get_u64(card + 176);
  if (check_desc(d) != kOk) return kErrFormat;
  for (int c = 0; c < 4; ++c) counts[c] = (int64_t)get_u64(card + 40 + 8 * c);
  if (check_counts(d, counts) != kOk) return kErrFormat;
  const Layout lay = make_layout(*d, counts);
  if (get_u64(card + 72) != lay.total || lay.total > card_bytes) return kErrFormat;
  if (get_u64(card + 80) != lay.off_bits || get_u64(card + 88) != lay.off_slot || get_u64(card + 96) != lay.off_order) return kErrFormat;
  for (int c = 0; c < 3; ++c) {
    if (get_u64(card + 104 + 8 * c) != lay.off_codes[c]) return kErrFormat;
    if (get_u64(card + 128 + 8 * c) != lay.off_meta[c]) return kErrFormat;
  }
  if (get_u64(card + 152) != lay.off_fp16) return kErrFormat;
  *lay_out = lay;
  return kOk;
}

int qkv_ref_card_peek(const uint8_t* card, uint64_t card_bytes, RefDesc* desc_out, int64_t counts_out[4],
                      float* avg_bits_out, uint32_t* status_out) {
  if (!card) return kErrNull;
  RefDesc d{};
  int64_t counts[4];
  Layout lay;
  const int rc = parse_header(card, card_bytes, &d, counts, &lay);
  if (rc) return rc;
  if (desc_out) *desc_out = d;
  if (counts_out) for (int c = 0; c < 4; ++c) counts_out[c] = counts[c];
  if (avg_bits_out) { uint32_t u = get_u32(card + 184); std::memcpy(avg_bits_out, &u, 4); }
  if (status_out) *status_out = get_u32(card + 192);
  return kOk;
}

// The planes [p_begin, p_end) of a card with per-token groups, decoded into k_out / v_out.
static void unpack_per_token(const uint8_t* card, const Layout& lay, const RefDesc& d, const int64_t counts[4],
                             uint64_t p_begin, uint64_t p_end, uint16_t* k_out, uint16_t* v_out) {
  const int64_t T = d.tokens;
  const int D = d.head_dim, G = d.group_size;
  const uint64_t planes_per_tensor = (uint64_t)d.layers * (uint64_t)d.kv_heads;
  const uint8_t* bits = card + lay.off_bits;
  std::vector<uint8_t> codes((size_t)D);
  for (uint64_t p = p_begin; p < p_end; ++p) {
    uint16_t* dst_plane = (p < planes_per_tensor) ? k_out + p * (uint64_t)T * D
                                                  : v_out + (p - planes_per_tensor) * (uint64_t)T * D;
    for (int64_t t = 0; t < T; ++t) {
      uint16_t* row = dst_plane + (uint64_t)t * D;
      const int c = class_of_width(bits[t]);
      const uint64_t j = get_u32(card + lay.off_slot + 4 * (uint64_t)t);
      if (c == 3) {
        const uint8_t* src = card + lay.off_fp16 + (p * (uint64_t)counts[3] + j) * (uint64_t)D * 2;
        for (int i = 0; i < D; ++i) row[i] = (uint16_t)(src[2 * i] | (src[2 * i + 1] << 8));
        continue;
      }
      const int w = kWidth[c];
      const uint8_t* src_codes = card + lay.off_codes[c] + (p * (uint64_t)counts[c] + j) * lay.row_bytes[c];
      const uint8_t* src_meta = card + lay.off_meta[c] + (p * (uint64_t)counts[c] + j) * lay.meta_bytes;
      unpack_codes(src_codes, D, w, codes.data());
      for (int g = 0; g < D / G; ++g) {
        const uint16_t sh = (uint16_t)(src_meta[4 * g] | (src_meta[4 * g + 1] << 8));
        const uint16_t zh = (uint16_t)(src_meta[4 * g + 2] | (src_meta[4 * g + 3] << 8));
        for (int i = 0; i < G; ++i) row[g * G + i] = dequantize_one(codes[(size_t)(g * G + i)], sh, zh);
      }
    }
  }
}

// Checks the three tables of a parsed card before they are used as indices: every width valid, slot[t] the
// rank of t among the tokens of its width, the class counts those of the header, and order[] the inverse of
// slot[] (entry base_c + slot[t] names t).  A card whose tables disagree anywhere is refused as a whole.
static int validate_tables(const uint8_t* card, const Layout& lay, const RefDesc& d, const int64_t counts[4]) {
  const uint8_t* bits = card + lay.off_bits;
  int64_t base[4];
  base[0] = 0;
  for (int c = 1; c < 4; ++c) base[c] = base[c - 1] + counts[c - 1];
  int64_t seen[4] = {0, 0, 0, 0};
  for (int64_t t = 0; t < d.tokens; ++t) {
    const int c = class_of_width(bits[t]);
    if (c < 0) return kErrFormat;
    if ((int64_t)get_u32(card + lay.off_slot + 4 * (uint64_t)t) != seen[c]) return kErrFormat;
    if (seen[c] >= counts[c]) return kErrFormat;
    if ((int64_t)get_u32(card + lay.off_order + 4 * (uint64_t)(base[c] + seen[c])) != t) return kErrFormat;
    seen[c] += 1;
  }
  for (int c = 0; c < 4; ++c) if (seen[c] != counts[c]) return kErrFormat;
  return kOk;
}

// Receiver-side injection (paper Sec. 4.2.2): dense fp16 K/V from a card.  Token t's row
// is found through the card's own bits and slot tables.
int qkv_ref_unpack_dequant(const uint8_t* card, uint64_t card_bytes, const RefDesc* expect,
                           uint16_t* k_out, uint16_t* v_out) {
  if (!card || !expect || !k_out || !v_out) return kErrNull;
  RefDesc d{};
  int64_t counts[4];
  Layout lay;
  int rc = parse_header(card, card_bytes, &d, counts, &lay);
  if (rc) return rc;
  if (d.layers != expect->layers || d.kv_heads != expect->kv_heads || d.head_dim != expect->head_dim ||
      d.group_size != expect->group_size || d.tokens != expect->tokens) return kErrFormat;
  if (get_u32(card + 188) != 0) return kErrFormat;      // a card with another grouping needs its own call
  rc = validate_tables(card, lay, d, counts);
  if (rc) return rc;
  unpack_per_token(card, lay, d, counts, 0, lay.planes, k_out, v_out);
  return kOk;
}

// ---- keys grouped per channel -------------------------------------------------------------------
//
// Variant for uniform cards (every token at the same width 2, 4 or 8), after the per-channel key /
// per-token value scheme the paper cites as related work (Sec. 2, KIVI): key outliers sit in a few
// channels, so a key group runs along the tokens of one channel instead of along the channels of one
// token.  Values keep their per-token groups.  Reading taken here: group size 32 both ways, tokens a
// multiple of 32; key group (plane p, token block tb, channel d) holds tokens 32 tb .. 32 tb + 31 of
// channel d; the same quantizer as everywhere else.  The card keeps its layout and sizes - a key
// plane's code section is [token block][channel][32 codes], its pair section [token block][channel] -
// and says so in bit 0 of the header's flags word.

static int uniform_class(const RefDesc* desc, const int64_t counts[4]) {
  if (desc->group_size != 32 || desc->tokens % 32 != 0) return -1;
  for (int c = 0; c < 3; ++c) if (counts[c] == desc->tokens) return c;
  return -1;
}

int qkv_ref_quantize_pack_kc(const RefDesc* desc, const uint16_t* k, const uint16_t* v, const uint8_t* bits,
                             const int64_t counts[4], uint8_t* card, uint64_t capacity) {
  if (!k || !v || !bits || !card) return kErrNull;
  int rc = check_desc(desc);
  if (rc) return rc;
  rc = check_counts(desc, counts);
  if (rc) return rc;
  const int c = uniform_class(desc, counts);
  if (c < 0) return kErrShape;
  rc = qkv_ref_quantize_pack(desc, k, v, bits, counts, card, capacity);      // header, tables, value planes
  if (rc) return rc;
  put_u32(card + 188, 1);                                                    // flags: keys per channel
  const Layout lay = make_layout(*desc, counts);
  const int64_t T = desc->tokens;
  const int D = desc->head_dim, w = kWidth[c];
  const uint64_t key_planes = (uint64_t)desc->layers * (uint64_t)desc->kv_heads;
  const uint64_t group_bytes = 32u * (uint64_t)w / 8u;
  uint16_t x[32];
  uint8_t codes[32];
  for (uint64_t p = 0; p < key_planes; ++p) {
    const uint16_t* plane = k + p * (uint64_t)T * D;
    for (int64_t tb = 0; tb < T / 32; ++tb) {
      for (int d = 0; d < D; ++d) {
        for (int i = 0; i < 32; ++i) x[i] = plane[(uint64_t)(32 * tb + i) * D + d];
        uint16_t sh, zh;
        quantize_group(x, 32, w, &sh, &zh, codes);
        const uint64_t g = (p * (uint64_t)(T / 32) + (uint64_t)tb) * (uint64_t)D + (uint64_t)d;
        pack_codes(codes, 32, w, card + lay.off_codes[c] + g * group_bytes);
        uint8_t* m = card + lay.off_meta[c] + g * 4;
        m[0] = (uint8_t)(sh & 0xff); m[1] = (uint8_t)(sh >> 8); m[2] = (uint8_t)(zh & 0xff); m[3] = (uint8_t)(zh >> 8);
      }
    }
  }
  return kOk;
}

int qkv_ref_unpack_dequant_kc(const uint8_t* card, uint64_t card_bytes, const RefDesc* expect,
                              uint16_t* k_out, uint16_t* v_out) {
  if (!card || !expect || !k_out || !v_out) return kErrNull;
  RefDesc d{};
  int64_t counts[4];
  Layout lay;
  int rc = parse_header(card, card_bytes, &d, counts, &lay);
  if (rc) return rc;
  if (d.layers != expect->layers || d.kv_heads != expect->kv_heads || d.head_dim != expect->head_dim ||
      d.group_size != expect->group_size || d.tokens != expect->tokens) return kErrFormat;
  if (get_u32(card + 188) != 1) return kErrFormat;
  const int c = uniform_class(&d, counts);
  if (c < 0) return kErrFormat;
  rc = validate_tables(card, lay, d, counts);
  if (rc) return rc;
  const int64_t T = d.tokens;
  const int D = d.head_dim, w = kWidth[c];
  const uint64_t key_planes = (uint64_t)d.layers * (uint64_t)d.kv_heads;
  unpack_per_token(card, lay, d, counts, key_planes, lay.planes, k_out, v_out);       // values
  const uint64_t group_bytes = 32u * (uint64_t)w / 8u;
  uint8_t codes[32];
  for (uint64_t p = 0; p < key_planes; ++p) {
    uint16_t* plane = k_out + p * (uint64_t)T * D;
    for (int64_t tb = 0; tb < T / 32; ++tb) {
      for (int dd = 0; dd < D; ++dd) {
        const uint64_t g = (p * (uint64_t)(T / 32) + (uint64_t)tb) * (uint64_t)D + (uint64_t)dd;
        unpack_codes(card + lay.off_codes[c] + g * group_bytes, 32, w, codes);
        const uint8_t* m = card + lay.off_meta[c] + g * 4;
        const uint16_t sh = (uint16_t)(m[0] | (m[1] << 8)), zh = (uint16_t)(m[2] | (m[3] << 8));
        for (int i = 0; i < 32; ++i) plane[(uint64_t)(32 * tb + i) * D + dd] = dequantize_one(codes[i], sh, zh);
      }
    }
  }
  return kOk;
}

}  // extern "C"
