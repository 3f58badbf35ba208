// Drives the CPU oracle's C entry points under AddressSanitizer and UndefinedBehaviorSanitizer (host only; built and
// run by tests/test_oracle_sanitizers.py).  Every buffer is a heap allocation of exactly the size the entry point is
// told, so any access past an end is reported; cards are also handed over truncated and with damaged bytes, which
// must end in an error code, never in a report.
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <memory>
#include <random>
#include <vector>

struct RefDesc {
  int32_t layers, kv_heads, head_dim, group_size;
  int64_t tokens;
  uint64_t model_id, sender_id;
  int64_t position_offset;
};

extern "C" {
float qkv_ref_half_to_float(uint16_t h);
uint16_t qkv_ref_float_to_half(float f);
int qkv_ref_card_bytes(const RefDesc*, const int64_t counts[4], uint64_t* bytes_out);
int qkv_ref_card_offsets(const RefDesc*, const int64_t counts[4], uint64_t out[11]);
int qkv_ref_budget_counts(int64_t tokens, double budget, int64_t counts_out[4]);
int qkv_ref_assign_bits(const float* scores, int64_t tokens, double budget, uint8_t* bits, int64_t counts_out[4]);
int qkv_ref_count_bits(const uint8_t* bits, int64_t tokens, int64_t counts_out[4]);
int qkv_ref_compact(const uint8_t* bits, int64_t tokens, uint32_t* slot, uint32_t* order, int64_t counts_out[4]);
int qkv_ref_quantize_group(const uint16_t* x, int n, int width, uint16_t* scale_h, uint16_t* zero_h, uint8_t* codes);
int qkv_ref_dequantize_group(const uint8_t* codes, int n, uint16_t scale_h, uint16_t zero_h, uint16_t* out);
int qkv_ref_pack_codes(const uint8_t* codes, int n, int width, uint8_t* out);
int qkv_ref_unpack_codes(const uint8_t* in, int n, int width, uint8_t* codes);
int qkv_ref_quantize_pack(const RefDesc*, const uint16_t* k, const uint16_t* v, const uint8_t* bits, const int64_t counts[4],
                          uint8_t* card, uint64_t capacity);
int qkv_ref_card_peek(const uint8_t* card, uint64_t card_bytes, RefDesc* desc_out, int64_t counts_out[4], float* avg_bits,
                      uint32_t* status);
int qkv_ref_unpack_dequant(const uint8_t* card, uint64_t card_bytes, const RefDesc* expect, uint16_t* k_out, uint16_t* v_out);
int qkv_ref_quantize_pack_kc(const RefDesc*, const uint16_t* k, const uint16_t* v, const uint8_t* bits, const int64_t counts[4],
                             uint8_t* card, uint64_t capacity);
int qkv_ref_unpack_dequant_kc(const uint8_t* card, uint64_t card_bytes, const RefDesc* expect, uint16_t* k_out, uint16_t* v_out);
int qkv_ref_controller_scores(const float* features, int64_t tokens, const float* w1, const float* b1, const float* w2,
                              float* scores);
int qkv_ref_assign_bits_greedy(const float* scores, int64_t tokens, double budget, uint8_t* bits, int64_t counts_out[4]);
int qkv_ref_rope_table(int32_t head_dim, double base, int64_t delta, float* cos_out, float* sin_out);
int qkv_ref_rope_rotate(uint16_t* rows, int64_t n_rows, int32_t head_dim, const float* cos_t, const float* sin_t);
}

namespace {

// A heap block of exactly n elements (never a vector with spare capacity behind it).
template <typename T>
struct Exact {
  std::unique_ptr<T[]> p;
  size_t n;
  explicit Exact(size_t count) : p(new T[count ? count : 1]), n(count) {}
  T* data() { return p.get(); }
};

#define REQUIRE(cond)                                                          \
  do {                                                                         \
    if (!(cond)) { std::printf("line %d: %s\n", __LINE__, #cond); return 1; } \
  } while (0)

int groups(std::mt19937& rng) {
  std::uniform_real_distribution<float> span(-70000.f, 70000.f);      // beyond the fp16 range on purpose: conversions saturate
  for (int width : {2, 4, 8}) {
    for (int n : {32, 64, 128}) {
      for (int it = 0; it < 200; ++it) {
        Exact<uint16_t> x(n), back(n);
        const int kind = it % 4;
        for (int i = 0; i < n; ++i) {
          float f = kind == 0 ? span(rng) * 1e-3f : kind == 1 ? 1.0f : kind == 2 ? (float)(i % 7) * 6.1e-5f : span(rng) * 0.9f;
          uint16_t h = qkv_ref_float_to_half(f);
          if ((h & 0x7C00u) == 0x7C00u) h = 0x7BFFu;                   // quantized values must be finite
          x.data()[i] = h;
        }
        uint16_t s = 0, z = 0;
        Exact<uint8_t> codes(n), packed(n * width / 8), again(n);
        REQUIRE(qkv_ref_quantize_group(x.data(), n, width, &s, &z, codes.data()) == 0);
        REQUIRE(qkv_ref_pack_codes(codes.data(), n, width, packed.data()) == 0);
        REQUIRE(qkv_ref_unpack_codes(packed.data(), n, width, again.data()) == 0);
        REQUIRE(std::memcmp(codes.data(), again.data(), n) == 0);
        REQUIRE(qkv_ref_dequantize_group(codes.data(), n, s, z, back.data()) == 0);
      }
    }
  }
  return 0;
}

int cards(std::mt19937& rng, int* n_cards, int* n_damaged) {
  std::normal_distribution<float> normal;
  const uint8_t widths[4] = {2, 4, 8, 16};
  for (int it = 0; it < 120; ++it) {
    const int D = 64 << (rng() % 3);
    int G = 32 << (rng() % 3);
    if (G > D) G = D;
    const int L = 1 + rng() % 3, H = 1 + rng() % 3;
    const bool per_channel = it % 4 == 0 && G == 32 && D <= 128;
    int64_t T = 1 + rng() % 200;
    if (per_channel) T = (D == 64 ? 64 : 32) * (1 + rng() % 3);
    RefDesc d{L, H, D, G, T, 11, 22, -33};
    Exact<uint8_t> bits(T);
    const uint8_t uniform = widths[rng() % 3];
    for (int64_t t = 0; t < T; ++t) bits.data()[t] = per_channel ? uniform : widths[rng() % 4];
    int64_t counts[4], c2[4];
    REQUIRE(qkv_ref_count_bits(bits.data(), T, counts) == 0);
    Exact<uint32_t> slot(T), order(T);
    REQUIRE(qkv_ref_compact(bits.data(), T, slot.data(), order.data(), c2) == 0);
    uint64_t total = 0, off[11];
    REQUIRE(qkv_ref_card_bytes(&d, counts, &total) == 0);
    REQUIRE(qkv_ref_card_offsets(&d, counts, off) == 0 && off[10] == total);
    const size_t elems = (size_t)L * H * T * D;
    Exact<uint16_t> k(elems), v(elems), ko(elems), vo(elems);
    for (size_t i = 0; i < elems; ++i) {
      k.data()[i] = qkv_ref_float_to_half(normal(rng) * 3.f);
      v.data()[i] = qkv_ref_float_to_half(normal(rng));
    }
    Exact<uint8_t> card(total);
    auto pack = per_channel ? qkv_ref_quantize_pack_kc : qkv_ref_quantize_pack;
    auto unpack = per_channel ? qkv_ref_unpack_dequant_kc : qkv_ref_unpack_dequant;
    auto other = per_channel ? qkv_ref_unpack_dequant : qkv_ref_unpack_dequant_kc;
    REQUIRE(pack(&d, k.data(), v.data(), bits.data(), counts, card.data(), total) == 0);
    if (total > 0) REQUIRE(pack(&d, k.data(), v.data(), bits.data(), counts, card.data(), total - 1) != 0);   // one byte short
    REQUIRE(unpack(card.data(), total, &d, ko.data(), vo.data()) == 0);
    REQUIRE(other(card.data(), total, &d, ko.data(), vo.data()) != 0);                                          // the other grouping refuses
    RefDesc seen{};
    float avg = 0;
    uint32_t status = 1;
    REQUIRE(qkv_ref_card_peek(card.data(), total, &seen, c2, &avg, &status) == 0 && seen.tokens == T && status == 0);
    ++*n_cards;
    // truncated at every section start, one byte before it and one after, and at a few random lengths
    for (int s = 0; s < 11; ++s) {
      for (int64_t delta = -1; delta <= 1; ++delta) {
        const int64_t len = (int64_t)off[s] + delta;
        if (len < 0 || (uint64_t)len >= total) continue;
        Exact<uint8_t> cut((size_t)len);
        std::memcpy(cut.data(), card.data(), (size_t)len);
        REQUIRE(unpack(cut.data(), (uint64_t)len, &d, ko.data(), vo.data()) != 0);
        qkv_ref_card_peek(cut.data(), (uint64_t)len, &seen, c2, &avg, &status);
      }
    }
    // damaged bytes in the header and the three tables: any return code, no report
    const uint64_t tables_end = off[3];
    for (int hit = 0; hit < 60; ++hit) {
      Exact<uint8_t> bad(total);
      std::memcpy(bad.data(), card.data(), total);
      const int n_bytes = 1 + rng() % 4;
      for (int b = 0; b < n_bytes; ++b) bad.data()[rng() % tables_end] = (uint8_t)rng();
      unpack(bad.data(), total, &d, ko.data(), vo.data());
      qkv_ref_card_peek(bad.data(), total, &seen, c2, &avg, &status);
      ++*n_damaged;
    }
    // the allocators, the controller and the realignment on the same sizes
    Exact<float> scores(T), features(T * 6), w1(64 * 6), b1(64), w2(64);
    for (int64_t t = 0; t < T; ++t) scores.data()[t] = normal(rng);
    for (int64_t i = 0; i < T * 6; ++i) features.data()[i] = normal(rng);
    for (int i = 0; i < 64 * 6; ++i) w1.data()[i] = normal(rng);
    for (int i = 0; i < 64; ++i) { b1.data()[i] = normal(rng); w2.data()[i] = normal(rng); }
    const double budget = 2.0 + (double)(rng() % 14001) / 1000.0;
    REQUIRE(qkv_ref_assign_bits(scores.data(), T, budget, bits.data(), c2) == 0);
    REQUIRE(qkv_ref_budget_counts(T, budget, counts) == 0 && std::memcmp(counts, c2, sizeof(c2)) == 0);
    REQUIRE(qkv_ref_controller_scores(features.data(), T, w1.data(), b1.data(), w2.data(), scores.data()) == 0);
    REQUIRE(qkv_ref_assign_bits_greedy(scores.data(), T, budget, bits.data(), c2) == 0);
    Exact<float> cos_t(D / 2), sin_t(D / 2);
    REQUIRE(qkv_ref_rope_table(D, 500000.0, (int64_t)(rng() % 200000) - 100000, cos_t.data(), sin_t.data()) == 0);
    REQUIRE(qkv_ref_rope_rotate(ko.data(), (int64_t)L * H * T, D, cos_t.data(), sin_t.data()) == 0);
  }
  return 0;
}

}  // namespace

int main() {
  std::mt19937 rng(20260503u);
  int n_cards = 0, n_damaged = 0;
  if (groups(rng)) return 1;
  if (cards(rng, &n_cards, &n_damaged)) return 2;
  std::printf("sanitizer drive ok: %d cards, %d damaged copies\n", n_cards, n_damaged);
  return 0;
}
