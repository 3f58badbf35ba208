// controller_ref.cpp — CPU oracle for the bit-width controller.  TEST INFRASTRUCTURE ONLY:
// used by tests/, the smoke check and the benchmark's CPU-baseline leg; the product library
// shares no code with it.  Plain, slow, single-threaded.
//
// Two pieces:
//
//  * The extended controller's network (paper Sec. 4.1.2): a 6-dimensional feature vector
//    per token [frequency, quality, attention variance, entropy, downstream demand, segment
//    type] goes through a 2-layer MLP with 512 parameters.  The paper fixes neither the hidden
//    width, the activation nor what the output is.  Reading taken here: 64 hidden units with
//    ReLU and one linear output without bias, 6*64 + 64 + 64 = 512 parameters exactly; the
//    output is the combined score S(t) of Sec. 3.3, and an output bias would not change any
//    ranking.  Arithmetic is fp32 in a fixed order: hidden unit j starts from its bias and
//    takes one fused multiply-add per feature, features in order; the score starts from +0
//    and takes one fused multiply-add per hidden unit, units in order.
//
//  * The allocator that follows the objective of Sec. 3.3 literally: minimise
//    sum_t eps(b(t)) * S(t) under sum_t b(t) <= budget * T, with the error model
//    eps(b) = 1 / (2^b - 1) (the step of a b-bit min-max quantizer relative to its range).
//    Every token starts at 2 bits.  The upgrades 2->4, 4->8, 8->16 cost 2, 4, 8 bits and gain
//    S * (eps(lo) - eps(hi)); per bit that is S * 2/15, S * 4/255, S * 32/65535.  Greedy rule:
//    list all 3T upgrades by (gain per bit descending, upgrade level ascending, token index
//    ascending) and take the longest prefix of that list that fits the budget.  The gain per
//    bit is one fp32 product of max(S, 0) with the constant rounded to fp32; a NaN score
//    counts as 0.  Gains per bit of one token never increase with the level, so a prefix
//    never holds an upgrade without the one below it.
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <vector>

namespace {

constexpr int kOk = 0, kErrNull = -1, kErrShape = -2, kErrBudget = -4;
constexpr int kFeatures = 6, kHidden = 64;

struct Upgrade {
  float gain_per_bit;
  int level;        // 0: 2->4, 1: 4->8, 2: 8->16
  int64_t token;
};

}  // namespace

extern "C" {

// features [T][6], w1 [64][6], b1 [64], w2 [64]  ->  scores [T]
int qkv_ref_controller_scores(const float* features, int64_t tokens, const float* w1, const float* b1,
                              const float* w2, float* scores) {
  if (!features || !w1 || !b1 || !w2 || !scores) return kErrNull;
  if (tokens < 1) return kErrShape;
  for (int64_t t = 0; t < tokens; ++t) {
    const float* x = features + t * kFeatures;
    float s = 0.0f;
    for (int j = 0; j < kHidden; ++j) {
      float a = b1[j];
      for (int i = 0; i < kFeatures; ++i) a = std::fmaf(x[i], w1[j * kFeatures + i], a);
      const float h = a > 0.0f ? a : 0.0f;      // ReLU; NaN -> 0
      s = std::fmaf(h, w2[j], s);
    }
    scores[t] = s;
  }
  return kOk;
}

int qkv_ref_assign_bits_greedy(const float* scores, int64_t tokens, double budget, uint8_t* bits,
                               int64_t counts_out[4]) {
  if (!scores || !bits || !counts_out) return kErrNull;
  if (!(budget >= 2.0 && budget <= 16.0)) return kErrBudget;
  if (tokens < 1) return kErrShape;
  const long long bm = std::llrint(budget * 1000.0);
  if (bm < 2000 || bm > 16000) return kErrBudget;
  const __int128 budget_bits = (__int128)bm * tokens / 1000;      // floor(budget * T)
  __int128 spare = budget_bits - (__int128)2 * tokens;              // what the upgrades may spend

  const float per_bit[3] = {(float)(2.0 / 15.0), (float)(4.0 / 255.0), (float)(32.0 / 65535.0)};
  const int cost[3] = {2, 4, 8};
  std::vector<Upgrade> list;
  list.reserve((size_t)tokens * 3);
  for (int level = 0; level < 3; ++level)            // level-major, then token: the tie order
    for (int64_t t = 0; t < tokens; ++t) {
      const float s = scores[t] > 0.0f ? scores[t] : 0.0f;
      list.push_back({s * per_bit[level], level, t});
    }
  std::stable_sort(list.begin(), list.end(),
                   [](const Upgrade& a, const Upgrade& b) { return a.gain_per_bit > b.gain_per_bit; });

  std::vector<int> level_reached((size_t)tokens, 0);
  for (const Upgrade& u : list) {
    if (cost[u.level] > spare) break;                // the prefix ends at the first upgrade that does not fit
    spare -= cost[u.level];
    level_reached[(size_t)u.token] += 1;
  }
  for (int c = 0; c < 4; ++c) counts_out[c] = 0;
  for (int64_t t = 0; t < tokens; ++t) {
    const int c = level_reached[(size_t)t];
    bits[t] = (uint8_t)(2 << c);
    counts_out[c] += 1;
  }
  return kOk;
}

}  // extern "C"
