// api.hip — the C ABI of the CacheCard library: argument checks, card geometry, launch
// planning.  Every operation's arithmetic runs in the HIP kernels of this directory; there
// is no host fallback.
#include <cmath>
#include <cstdlib>
#include <cstring>

#include "qkv_common.h"

namespace qkv {

// Grid size for the streaming kernels: one wave per tile, four waves per workgroup (measured faster than a
// persistent grid whose waves stride over the tiles: 216 vs 226 us packing, 191 vs 206 us unpacking at 8K tokens).
int grid_blocks(uint64_t tiles) {
  uint64_t n = (tiles + kWavesPerBlock - 1) / kWavesPerBlock;
  if (n > 0x7FFFFFFFull) n = 0x7FFFFFFFull;
  return n < 1 ? 1 : (int)n;
}

namespace {

int check_desc(const qkv_desc_t* d) {
  if (!d) return QKV_ERR_NULL;
  return check_shape(d->layers, d->kv_heads, d->head_dim, d->group_size, d->tokens);
}

// Class counts bought by a budget: linear blend between the all-2-bit mix at 2.0, the
// 30/40/25/5 % mix at 5.0 and the all-fp16 mix at 16.0, in thousandths of a bit, with floors
// so that the code bits never exceed budget * T.
int counts_for_budget(int64_t T, double budget, int64_t out[4]) {
  if (T < 1) return QKV_ERR_SHAPE;
  if (!std::isfinite(budget) || budget < 2.0 || budget > 16.0) return QKV_ERR_BUDGET;
  const long long milli = std::llrint(budget * 1000.0);
  if (milli < 2000 || milli > 16000) return QKV_ERR_BUDGET;
  // shares of the 16-, 8- and 4-bit classes as numerator / denominator of T
  unsigned __int128 num16, num8, num4, den;
  if (milli <= 5000) {
    const unsigned long long up = (unsigned long long)(milli - 2000);   // 0 .. 3000
    num16 = 5ull * up; num8 = 25ull * up; num4 = 40ull * up;
    den = 100ull * 3000ull;
  } else {
    const unsigned long long up = (unsigned long long)(milli - 5000);   // 0 .. 11000
    const unsigned long long down = 11000ull - up;
    num16 = 5ull * down + 100ull * up; num8 = 25ull * down; num4 = 40ull * down;
    den = 100ull * 11000ull;
  }
  const unsigned __int128 t = (unsigned __int128)(uint64_t)T;
  out[3] = (int64_t)(uint64_t)(num16 * t / den);
  out[2] = (int64_t)(uint64_t)(num8 * t / den);
  out[1] = (int64_t)(uint64_t)(num4 * t / den);
  out[0] = T - out[3] - out[2] - out[1];
  return QKV_OK;
}

void to_u64(const int64_t in[4], uint64_t out[4]) {
  for (int c = 0; c < 4; ++c) out[c] = (uint64_t)in[c];
}

// Host-side validation of a header read back from a card.
bool header_valid(const qkv_card_header_t& h, uint64_t card_bytes, CardGeom& g) {
  static const uint8_t magic[8] = {'Q', 'K', 'V', 'C', 'A', 'R', 'D', 0};
  if (std::memcmp(h.magic, magic, 8) != 0) return false;
  if (h.version != QKV_CARD_VERSION || h.header_bytes != QKV_CARD_HEADER_BYTES) return false;
  if (h.layers > 0x7FFFFFFFu || h.kv_heads > 0x7FFFFFFFu || h.head_dim > 0x7FFFFFFFu || h.group_size > 0x7FFFFFFFu ||
      h.tokens > 0x7FFFFFFFFFFFFFFFull)
    return false;
  if (check_shape((int32_t)h.layers, (int32_t)h.kv_heads, (int32_t)h.head_dim, (int32_t)h.group_size,
                  (int64_t)h.tokens) != QKV_OK)
    return false;
  uint64_t sum = 0;
  for (int c = 0; c < 4; ++c) {
    if (h.count[c] > h.tokens) return false;
    sum += h.count[c];
  }
  if (sum != h.tokens) return false;
  if (h.flags != 0u) {   // the one flag there is: keys grouped per channel, uniform cards of certain shapes only
    if (h.flags != QKV_FLAG_KEYS_PER_CHANNEL) return false;
    if (h.group_size != 32 || (h.head_dim != 64 && h.head_dim != 128) || h.tokens % (h.head_dim == 64 ? 64 : 32) != 0)
      return false;
    if (h.count[0] != h.tokens && h.count[1] != h.tokens && h.count[2] != h.tokens) return false;
  }
  build_geom(g, h.layers, h.kv_heads, h.head_dim, h.group_size, h.tokens, h.count);
  if (h.total_bytes != g.total || g.total > card_bytes) return false;
  if (h.off_bits != g.off_bits || h.off_slot != g.off_slot || h.off_order != g.off_order || h.off_fp16 != g.off_fp16)
    return false;
  for (int c = 0; c < 3; ++c)
    if (h.off_codes[c] != g.off_codes[c] || h.off_meta[c] != g.off_meta[c]) return false;
  return true;
}

}  // namespace
}  // namespace qkv

using namespace qkv;

extern "C" {

int qkv_version(void) { return 100; }   // 0.1.0

const char* qkv_error_string(int code) {
  switch (code) {
    case QKV_OK: return "ok";
    case QKV_ERR_NULL: return "a required pointer is null";
    case QKV_ERR_SHAPE: return "unsupported layers / kv_heads / tokens / head_dim";
    case QKV_ERR_GROUP: return "unsupported group_size";
    case QKV_ERR_BUDGET: return "average-bit budget outside [2, 16]";
    case QKV_ERR_CAPACITY: return "card buffer too small";
    case QKV_ERR_ALIGN: return "device pointer not aligned as required";
    case QKV_ERR_COUNTS: return "class counts negative or not summing to tokens";
    case QKV_ERR_HIP: return "a HIP runtime call failed";
    case QKV_ERR_FORMAT: return "not a valid layout-v1 card header";
    case QKV_ERR_OVERLAP: return "input and output buffers overlap";
    default: return "unknown error code";
  }
}

int qkv_card_bytes(const qkv_desc_t* desc, const int64_t counts[4], uint64_t* bytes_out) {
  if (!desc || !counts || !bytes_out) return QKV_ERR_NULL;
  int rc = check_desc(desc);
  if (rc) return rc;
  rc = check_counts(desc->tokens, counts);
  if (rc) return rc;
  uint64_t n[4];
  to_u64(counts, n);
  CardGeom g;
  build_geom(g, desc->layers, desc->kv_heads, desc->head_dim, desc->group_size, desc->tokens, n);
  *bytes_out = g.total;
  return QKV_OK;
}

int qkv_budget_counts(int64_t tokens, double avg_bits_budget, int64_t counts_out[4]) {
  if (!counts_out) return QKV_ERR_NULL;
  int64_t tmp[4];
  const int rc = counts_for_budget(tokens, avg_bits_budget, tmp);
  if (rc) return rc;
  std::memcpy(counts_out, tmp, sizeof(tmp));
  return QKV_OK;
}

int qkv_assign_bits(const float* scores_dev, int64_t tokens, double avg_bits_budget, uint8_t* bits_dev,
                    int64_t counts_out[4], void* stream) {
  if (!scores_dev || !bits_dev || !counts_out) return QKV_ERR_NULL;
  if (tokens < 1 || tokens >= (1ll << 31)) return QKV_ERR_SHAPE;
  if (reinterpret_cast<uintptr_t>(scores_dev) % 4 != 0) return QKV_ERR_ALIGN;
  int64_t counts[4];
  const int rc = counts_for_budget(tokens, avg_bits_budget, counts);
  if (rc) return rc;
  const uint32_t cuts[3] = {(uint32_t)counts[3], (uint32_t)(counts[3] + counts[2]),
                            (uint32_t)(counts[3] + counts[2] + counts[1])};
  if (launch_assign(scores_dev, (uint32_t)tokens, cuts, bits_dev, static_cast<hipStream_t>(stream)) != hipSuccess)
    return QKV_ERR_HIP;
  std::memcpy(counts_out, counts, sizeof(counts));
  return QKV_OK;
}

int qkv_controller_scores(const float* features_dev, int64_t tokens, const qkv_controller_t* params,
                          float* scores_dev, void* stream) {
  if (!features_dev || !params || !scores_dev) return QKV_ERR_NULL;
  if (tokens < 1 || tokens >= (1ll << 31)) return QKV_ERR_SHAPE;
  if (reinterpret_cast<uintptr_t>(features_dev) % 8 != 0 || reinterpret_cast<uintptr_t>(scores_dev) % 4 != 0)
    return QKV_ERR_ALIGN;
  return launch_controller(features_dev, (uint32_t)tokens, *params, scores_dev, static_cast<hipStream_t>(stream)) ==
                 hipSuccess ? QKV_OK : QKV_ERR_HIP;
}

int qkv_assign_bits_greedy(const float* scores_dev, int64_t tokens, double avg_bits_budget, uint8_t* bits_dev,
                           uint64_t* counts_dev, void* stream) {
  if (!scores_dev || !bits_dev) return QKV_ERR_NULL;
  if (tokens < 1 || tokens >= (1ll << 28)) return QKV_ERR_SHAPE;
  if (!(avg_bits_budget >= 2.0 && avg_bits_budget <= 16.0)) return QKV_ERR_BUDGET;
  const long long bm = std::llrint(avg_bits_budget * 1000.0);
  if (bm < 2000 || bm > 16000) return QKV_ERR_BUDGET;
  if (reinterpret_cast<uintptr_t>(scores_dev) % 4 != 0 || reinterpret_cast<uintptr_t>(counts_dev) % 8 != 0)
    return QKV_ERR_ALIGN;
  const int64_t budget_bits = (int64_t)(((__int128)bm * tokens) / 1000);
  const uint32_t spare_units = (uint32_t)((budget_bits - 2 * tokens) / 2);      // upgrades cost 1, 2, 4 units of 2 bits
  return launch_greedy(scores_dev, (uint32_t)tokens, spare_units, bits_dev,
                       reinterpret_cast<unsigned long long*>(counts_dev), static_cast<hipStream_t>(stream)) == hipSuccess
             ? QKV_OK : QKV_ERR_HIP;
}

int qkv_count_bits(const uint8_t* bits_dev, int64_t tokens, int64_t counts_out[4], void* stream) {
  if (!bits_dev || !counts_out) return QKV_ERR_NULL;
  if (tokens < 1) return QKV_ERR_SHAPE;
  hipStream_t s = static_cast<hipStream_t>(stream);
  unsigned long long* dev = nullptr;
  if (hipMalloc(reinterpret_cast<void**>(&dev), 4 * sizeof(unsigned long long)) != hipSuccess) return QKV_ERR_HIP;
  unsigned long long host[4] = {0, 0, 0, 0};
  bool ok = launch_count(bits_dev, (uint64_t)tokens, dev, s) == hipSuccess;
  ok = ok && hipMemcpyAsync(host, dev, sizeof(host), hipMemcpyDeviceToHost, s) == hipSuccess;
  ok = (hipStreamSynchronize(s) == hipSuccess) && ok;
  ok = (hipFree(dev) == hipSuccess) && ok;
  if (!ok) return QKV_ERR_HIP;
  for (int c = 0; c < 4; ++c) counts_out[c] = (int64_t)host[c];
  return QKV_OK;
}

namespace {

// Checks shared by the card-building calls; fills the geometry.
static int prepare_card(const qkv_desc_t* desc, const int64_t counts[4], const void* card_dev, uint64_t card_capacity,
                 CardGeom& g, uint64_t n[4]) {
  int rc = check_desc(desc);
  if (rc) return rc;
  rc = check_counts(desc->tokens, counts);
  if (rc) return rc;
  if (reinterpret_cast<uintptr_t>(card_dev) % QKV_CARD_ALIGN != 0) return QKV_ERR_ALIGN;
  to_u64(counts, n);
  build_geom(g, desc->layers, desc->kv_heads, desc->head_dim, desc->group_size, desc->tokens, n);
  if (card_capacity < g.total) return QKV_ERR_CAPACITY;
  return QKV_OK;
}

// The header the host knows before the device has looked at anything (status 0).
static qkv_card_header_t make_header(const qkv_desc_t* desc, const CardGeom& g, const uint64_t n[4], uint32_t flags) {
  qkv_card_header_t h;
  std::memset(&h, 0, sizeof(h));
  static const uint8_t magic[8] = {'Q', 'K', 'V', 'C', 'A', 'R', 'D', 0};
  std::memcpy(h.magic, magic, 8);
  h.version = QKV_CARD_VERSION;
  h.header_bytes = QKV_CARD_HEADER_BYTES;
  h.layers = (uint32_t)desc->layers;
  h.kv_heads = (uint32_t)desc->kv_heads;
  h.head_dim = (uint32_t)desc->head_dim;
  h.group_size = (uint32_t)desc->group_size;
  h.tokens = (uint64_t)desc->tokens;
  uint64_t code_bits = 0;
  for (int c = 0; c < 4; ++c) { h.count[c] = n[c]; code_bits += n[c] * width_of_class(c); }
  h.total_bytes = g.total;
  h.off_bits = g.off_bits; h.off_slot = g.off_slot; h.off_order = g.off_order;
  for (int c = 0; c < 3; ++c) { h.off_codes[c] = g.off_codes[c]; h.off_meta[c] = g.off_meta[c]; }
  h.off_fp16 = g.off_fp16;
  h.model_id = desc->model_id;
  h.sender_id = desc->sender_id;
  h.position_offset = desc->position_offset;
  h.avg_bits = (float)((double)code_bits / (double)h.tokens);   // achieved average bit width (Sec. 4.2.1)
  h.flags = flags;
  h.status = 0;
  return h;
}

static int plan_card(const qkv_desc_t* desc, const uint8_t* bits_dev, const CardGeom& g, const uint64_t n[4], uint8_t* card,
              hipStream_t s, uint32_t flags = 0) {
  const qkv_card_header_t h = make_header(desc, g, n, flags);
  return launch_classify(bits_dev, g, h, card, s) == hipSuccess ? QKV_OK : QKV_ERR_HIP;
}

// Scores and a budget to widths and a planned card, one launch.  `counts_out` gets the budget's class counts.
static int assign_and_plan(const qkv_desc_t* desc, const float* scores_dev, double avg_bits_budget, uint8_t* bits_dev,
                    int64_t counts_out[4], void* card_dev, uint64_t card_capacity, CardGeom& g, hipStream_t s) {
  int rc = check_desc(desc);
  if (rc) return rc;
  if (desc->tokens >= (1ll << 31)) return QKV_ERR_SHAPE;
  int64_t counts[4];
  rc = counts_for_budget(desc->tokens, avg_bits_budget, counts);
  if (rc) return rc;
  if (reinterpret_cast<uintptr_t>(scores_dev) % 4 != 0) return QKV_ERR_ALIGN;
  uint64_t n[4];
  rc = prepare_card(desc, counts, card_dev, card_capacity, g, n);
  if (rc) return rc;
  const uint32_t cuts[3] = {(uint32_t)counts[3], (uint32_t)(counts[3] + counts[2]),
                            (uint32_t)(counts[3] + counts[2] + counts[1])};
  const qkv_card_header_t h = make_header(desc, g, n, 0u);
  uint8_t* card = static_cast<uint8_t*>(card_dev);
  if ((uint64_t)desc->tokens <= assign_plan_max_tokens()) {
    if (launch_assign_plan(scores_dev, cuts, bits_dev, g, h, card, s) != hipSuccess) return QKV_ERR_HIP;
  } else {
    // Sequences beyond the one-launch kernel's reach: the allocator and the classification one after the
    // other, same bytes.  Without a buffer from the caller the widths go straight to their place in the
    // card, where the classification rewrites every byte with the value it read there.
    uint8_t* widths = bits_dev ? bits_dev : card + g.off_bits;
    if (launch_assign(scores_dev, (uint32_t)desc->tokens, cuts, widths, s) != hipSuccess) return QKV_ERR_HIP;
    if (launch_classify(widths, g, h, card, s) != hipSuccess) return QKV_ERR_HIP;
  }
  std::memcpy(counts_out, counts, sizeof(counts));
  return QKV_OK;
}

}  // namespace

int qkv_card_plan(const qkv_desc_t* desc, const uint8_t* bits_dev, const int64_t counts[4], void* card_dev,
                  uint64_t card_capacity, void* stream) {
  if (!desc || !bits_dev || !counts || !card_dev) return QKV_ERR_NULL;
  CardGeom g;
  uint64_t n[4];
  const int rc = prepare_card(desc, counts, card_dev, card_capacity, g, n);
  if (rc) return rc;
  return plan_card(desc, bits_dev, g, n, static_cast<uint8_t*>(card_dev), static_cast<hipStream_t>(stream));
}

int qkv_assign_plan(const qkv_desc_t* desc, const float* scores_dev, double avg_bits_budget, uint8_t* bits_dev,
                    int64_t counts_out[4], void* card_dev, uint64_t card_capacity, void* stream) {
  if (!desc || !scores_dev || !counts_out || !card_dev) return QKV_ERR_NULL;
  CardGeom g;
  return assign_and_plan(desc, scores_dev, avg_bits_budget, bits_dev, counts_out, card_dev, card_capacity, g,
                         static_cast<hipStream_t>(stream));
}

int qkv_assign_quantize_pack(const qkv_desc_t* desc, const void* k_dev, const void* v_dev, const float* scores_dev,
                             double avg_bits_budget, uint8_t* bits_dev, int64_t counts_out[4], void* card_dev,
                             uint64_t card_capacity, void* stream) {
  if (!desc || !k_dev || !v_dev || !scores_dev || !counts_out || !card_dev) return QKV_ERR_NULL;
  if (reinterpret_cast<uintptr_t>(k_dev) % 16 != 0 || reinterpret_cast<uintptr_t>(v_dev) % 16 != 0) return QKV_ERR_ALIGN;
  CardGeom g;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int rc = assign_and_plan(desc, scores_dev, avg_bits_budget, bits_dev, counts_out, card_dev, card_capacity, g, s);
  if (rc) return rc;
  return launch_pack(g, k_dev, v_dev, static_cast<uint8_t*>(card_dev), false, s) == hipSuccess ? QKV_OK : QKV_ERR_HIP;
}

int qkv_card_fill(const qkv_desc_t* desc, const void* k_dev, const void* v_dev, const int64_t counts[4],
                  void* card_dev, uint64_t card_capacity, void* stream) {
  if (!desc || !k_dev || !v_dev || !counts || !card_dev) return QKV_ERR_NULL;
  CardGeom g;
  uint64_t n[4];
  const int rc = prepare_card(desc, counts, card_dev, card_capacity, g, n);
  if (rc) return rc;
  if (reinterpret_cast<uintptr_t>(k_dev) % 16 != 0 || reinterpret_cast<uintptr_t>(v_dev) % 16 != 0) return QKV_ERR_ALIGN;
  return launch_pack(g, k_dev, v_dev, static_cast<uint8_t*>(card_dev), false, static_cast<hipStream_t>(stream)) == hipSuccess
             ? QKV_OK : QKV_ERR_HIP;
}

int qkv_quantize_pack(const qkv_desc_t* desc, const void* k_dev, const void* v_dev, const uint8_t* bits_dev,
                      const int64_t counts[4], void* card_dev, uint64_t card_capacity, void* stream) {
  if (!desc || !k_dev || !v_dev || !bits_dev || !counts || !card_dev) return QKV_ERR_NULL;
  CardGeom g;
  uint64_t n[4];
  int rc = prepare_card(desc, counts, card_dev, card_capacity, g, n);
  if (rc) return rc;
  if (reinterpret_cast<uintptr_t>(k_dev) % 16 != 0 || reinterpret_cast<uintptr_t>(v_dev) % 16 != 0) return QKV_ERR_ALIGN;
  hipStream_t s = static_cast<hipStream_t>(stream);
  uint8_t* card = static_cast<uint8_t*>(card_dev);
  rc = plan_card(desc, bits_dev, g, n, card, s);
  if (rc) return rc;
  if (launch_pack(g, k_dev, v_dev, card, false, s) != hipSuccess) return QKV_ERR_HIP;
  return QKV_OK;
}

int qkv_requantize(const void* card_in_dev, uint64_t card_in_bytes, const qkv_desc_t* desc, const uint8_t* bits_dev,
                   const int64_t counts[4], void* card_out_dev, uint64_t card_out_capacity, uint32_t* status_dev,
                   void* stream) {
  if (!card_in_dev || !desc || !bits_dev || !counts || !card_out_dev) return QKV_ERR_NULL;
  CardGeom g;
  uint64_t n[4];
  int rc = prepare_card(desc, counts, card_out_dev, card_out_capacity, g, n);
  if (rc) return rc;
  if (card_in_bytes < QKV_CARD_HEADER_BYTES) return QKV_ERR_CAPACITY;
  if (reinterpret_cast<uintptr_t>(card_in_dev) % QKV_CARD_ALIGN != 0 || reinterpret_cast<uintptr_t>(status_dev) % 4 != 0)
    return QKV_ERR_ALIGN;
  {   // rows of the new card are written while rows of the old one are still being read
    const uintptr_t in0 = reinterpret_cast<uintptr_t>(card_in_dev), out0 = reinterpret_cast<uintptr_t>(card_out_dev);
    if (in0 < out0 + g.total && out0 < in0 + card_in_bytes) return QKV_ERR_OVERLAP;
  }
  hipStream_t s = static_cast<hipStream_t>(stream);
  uint8_t* card = static_cast<uint8_t*>(card_out_dev);
  rc = plan_card(desc, bits_dev, g, n, card, s);
  if (rc) return rc;
  if (launch_requant(static_cast<const uint8_t*>(card_in_dev), card_in_bytes, g, card, status_dev, s) != hipSuccess)
    return QKV_ERR_HIP;
  return QKV_OK;
}

namespace {
// Shapes the per-channel key tiles are written for.
static int check_keys_per_channel(const qkv_desc_t* d) {
  if (d->group_size != 32 || (d->head_dim != 64 && d->head_dim != 128)) return QKV_ERR_SHAPE;
  if (d->tokens % (d->head_dim == 64 ? 64 : 32) != 0) return QKV_ERR_SHAPE;
  return QKV_OK;
}
}  // namespace

int qkv_quantize_pack_kc(const qkv_desc_t* desc, const void* k_dev, const void* v_dev, const uint8_t* bits_dev,
                         const int64_t counts[4], void* card_dev, uint64_t card_capacity, void* stream) {
  if (!desc || !k_dev || !v_dev || !bits_dev || !counts || !card_dev) return QKV_ERR_NULL;
  CardGeom g;
  uint64_t n[4];
  int rc = prepare_card(desc, counts, card_dev, card_capacity, g, n);
  if (rc) return rc;
  rc = check_keys_per_channel(desc);
  if (rc) return rc;
  if (counts[0] != desc->tokens && counts[1] != desc->tokens && counts[2] != desc->tokens) return QKV_ERR_COUNTS;
  if (reinterpret_cast<uintptr_t>(k_dev) % 16 != 0 || reinterpret_cast<uintptr_t>(v_dev) % 16 != 0) return QKV_ERR_ALIGN;
  hipStream_t s = static_cast<hipStream_t>(stream);
  uint8_t* card = static_cast<uint8_t*>(card_dev);
  rc = plan_card(desc, bits_dev, g, n, card, s, QKV_FLAG_KEYS_PER_CHANNEL);
  if (rc) return rc;
  if (launch_pack(g, k_dev, v_dev, card, true, s) != hipSuccess) return QKV_ERR_HIP;
  return QKV_OK;
}

namespace {
static int unpack_any(const void* card_dev, uint64_t card_bytes, const qkv_desc_t* expect, void* k_out_dev, void* v_out_dev,
               uint32_t* status_dev, bool keys_per_channel, void* stream) {
  if (!card_dev || !expect || !k_out_dev || !v_out_dev) return QKV_ERR_NULL;
  int rc = check_desc(expect);
  if (rc) return rc;
  if (keys_per_channel) {
    rc = check_keys_per_channel(expect);
    if (rc) return rc;
  }
  if (card_bytes < QKV_CARD_HEADER_BYTES) return QKV_ERR_CAPACITY;
  if (reinterpret_cast<uintptr_t>(k_out_dev) % 16 != 0 || reinterpret_cast<uintptr_t>(v_out_dev) % 16 != 0 ||
      reinterpret_cast<uintptr_t>(card_dev) % QKV_CARD_ALIGN != 0 || reinterpret_cast<uintptr_t>(status_dev) % 4 != 0)
    return QKV_ERR_ALIGN;
  const uint64_t zero[4] = {0, 0, 0, (uint64_t)expect->tokens};
  CardGeom g;
  build_geom(g, expect->layers, expect->kv_heads, expect->head_dim, expect->group_size, expect->tokens, zero);
  if (launch_unpack(static_cast<const uint8_t*>(card_dev), card_bytes, g, k_out_dev, v_out_dev, status_dev,
                    keys_per_channel, static_cast<hipStream_t>(stream)) != hipSuccess)
    return QKV_ERR_HIP;
  return QKV_OK;
}
}  // namespace

int qkv_unpack_dequant(const void* card_dev, uint64_t card_bytes, const qkv_desc_t* expect, void* k_out_dev,
                       void* v_out_dev, uint32_t* status_dev, void* stream) {
  return unpack_any(card_dev, card_bytes, expect, k_out_dev, v_out_dev, status_dev, false, stream);
}

int qkv_unpack_dequant_kc(const void* card_dev, uint64_t card_bytes, const qkv_desc_t* expect, void* k_out_dev,
                          void* v_out_dev, uint32_t* status_dev, void* stream) {
  return unpack_any(card_dev, card_bytes, expect, k_out_dev, v_out_dev, status_dev, true, stream);
}

int qkv_inject_layers(const void* card_dev, uint64_t card_bytes, const qkv_desc_t* expect, const qkv_inject_t* where,
                      uint32_t* status_dev, void* stream) {
  if (!card_dev || !expect || !where || !where->k_layers || !where->v_layers) return QKV_ERR_NULL;
  const int rc = check_desc(expect);
  if (rc) return rc;
  if (where->layer_count < 1 || where->layer_count > QKV_INJECT_MAX_LAYERS || where->layer_begin < 0 ||
      where->layer_begin > expect->layers - where->layer_count)
    return QKV_ERR_SHAPE;
  if (where->token_stride < expect->head_dim || where->token_stride % 8 != 0 || where->head_stride < 0 ||
      where->head_stride % 8 != 0 || where->token_stride >= (1ll << 40) || where->head_stride >= (1ll << 40))
    return QKV_ERR_SHAPE;
  // the farthest element a row address can reach must stay far inside 64-bit byte arithmetic
  if ((__int128)where->token_stride * expect->tokens >= ((__int128)1 << 46) ||
      (__int128)where->head_stride * expect->kv_heads >= ((__int128)1 << 46))
    return QKV_ERR_SHAPE;
  if (!(where->rope_base >= 0.0) || !std::isfinite(where->rope_base) || where->rope_delta <= -(1ll << 31) ||
      where->rope_delta >= (1ll << 31))
    return QKV_ERR_SHAPE;
  if (where->keys_per_channel != 0) {
    if (where->keys_per_channel != 1) return QKV_ERR_SHAPE;
    const int rk = check_keys_per_channel(expect);
    if (rk) return rk;
  }
  if (card_bytes < QKV_CARD_HEADER_BYTES) return QKV_ERR_CAPACITY;
  if (reinterpret_cast<uintptr_t>(card_dev) % QKV_CARD_ALIGN != 0 || reinterpret_cast<uintptr_t>(status_dev) % 4 != 0)
    return QKV_ERR_ALIGN;
  for (int i = 0; i < where->layer_count; ++i) {
    if (!where->k_layers[i] || !where->v_layers[i]) return QKV_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(where->k_layers[i]) % 16 != 0 || reinterpret_cast<uintptr_t>(where->v_layers[i]) % 16 != 0)
      return QKV_ERR_ALIGN;
  }
  // the rotation of the shift, one (cos, sin) per element pair (Sec. 3.2, challenge 2)
  float cos_sin[128][2];
  const bool rope = where->rope_base > 0.0;
  if (rope) {
    const int D = expect->head_dim;
    for (int i = 0; i < D / 2; ++i) {
      const double theta = std::pow(where->rope_base, -2.0 * i / D);
      const double angle = (double)where->rope_delta * theta;
      cos_sin[i][0] = (float)std::cos(angle);
      cos_sin[i][1] = (float)std::sin(angle);
    }
  }
  const uint64_t zero[4] = {0, 0, 0, (uint64_t)expect->tokens};
  CardGeom g;
  build_geom(g, expect->layers, expect->kv_heads, expect->head_dim, expect->group_size, expect->tokens, zero);
  if (launch_inject(static_cast<const uint8_t*>(card_dev), card_bytes, g, (uint32_t)where->layer_begin,
                    (uint32_t)where->layer_count, where->k_layers, where->v_layers, (uint64_t)where->head_stride * 2u,
                    (uint64_t)where->token_stride * 2u, rope ? cos_sin : nullptr, where->keys_per_channel == 1, status_dev,
                    static_cast<hipStream_t>(stream)) != hipSuccess)
    return QKV_ERR_HIP;
  return QKV_OK;
}

namespace {
// Shape rules of the fused attention path and the floats of workspace it needs.
static int attend_workspace_floats(const qkv_desc_t* expect, int32_t q_heads, uint64_t* floats) {
  const int rc = check_desc(expect);
  if (rc) return rc;
  if (q_heads < expect->kv_heads || q_heads % expect->kv_heads != 0 || q_heads / expect->kv_heads > 16)
    return QKV_ERR_SHAPE;
  const uint32_t rep = (uint32_t)(q_heads / expect->kv_heads);
  uint32_t chunk = 0, max_tasks = 0;
  attend_plan((uint64_t)expect->tokens, rep, (uint64_t)expect->layers * (uint64_t)expect->kv_heads, &chunk, &max_tasks);
  *floats = (uint64_t)expect->layers * (uint64_t)expect->kv_heads * max_tasks * rep * ((uint32_t)expect->head_dim + 2u) + 4u;   // + verdict word
  return QKV_OK;
}
}  // namespace

int qkv_card_attend_workspace(const qkv_desc_t* expect, int32_t q_heads, uint64_t* bytes_out) {
  if (!expect || !bytes_out) return QKV_ERR_NULL;
  uint64_t floats = 0;
  const int rc = attend_workspace_floats(expect, q_heads, &floats);
  if (rc) return rc;
  *bytes_out = floats * sizeof(float);
  return QKV_OK;
}

namespace {
// Checks of both attention entry points; fills the geometry the kernels validate the header against and
// the floats of scratch the launch needs.
static int prepare_attend(const void* card_dev, uint64_t card_bytes, const qkv_desc_t* expect, const void* q_dev, int32_t q_heads,
                   float softmax_scale, const float* out_dev, const float* lse_dev, const uint32_t* status_dev, CardGeom& g,
                   uint64_t& floats, bool keys_per_channel = false) {
  if (!card_dev || !expect || !q_dev || !out_dev) return QKV_ERR_NULL;
  const int rc = attend_workspace_floats(expect, q_heads, &floats);
  if (rc) return rc;
  if (keys_per_channel) {                      // the shape rules of qkv_quantize_pack_kc
    if (expect->group_size != 32) return QKV_ERR_GROUP;
    if (expect->head_dim > 128 || expect->tokens % (expect->head_dim == 64 ? 64 : 32) != 0) return QKV_ERR_SHAPE;
  }
  if (!std::isfinite(softmax_scale)) return QKV_ERR_SHAPE;
  if (card_bytes < QKV_CARD_HEADER_BYTES) return QKV_ERR_CAPACITY;
  if (reinterpret_cast<uintptr_t>(card_dev) % QKV_CARD_ALIGN != 0 || reinterpret_cast<uintptr_t>(q_dev) % 16 != 0 ||
      reinterpret_cast<uintptr_t>(out_dev) % 16 != 0 || reinterpret_cast<uintptr_t>(lse_dev) % 4 != 0 ||
      reinterpret_cast<uintptr_t>(status_dev) % 4 != 0)
    return QKV_ERR_ALIGN;
  const uint64_t zero[4] = {0, 0, 0, (uint64_t)expect->tokens};
  build_geom(g, expect->layers, expect->kv_heads, expect->head_dim, expect->group_size, expect->tokens, zero);
  return QKV_OK;
}
}  // namespace

int qkv_card_attend(const void* card_dev, uint64_t card_bytes, const qkv_desc_t* expect, const void* q_dev,
                    int32_t q_heads, float softmax_scale, float* out_dev, float* lse_dev, void* workspace_dev,
                    uint64_t workspace_bytes, uint32_t* status_dev, void* stream) {
  if (!workspace_dev) return QKV_ERR_NULL;
  CardGeom g;
  uint64_t floats = 0;
  const int rc = prepare_attend(card_dev, card_bytes, expect, q_dev, q_heads, softmax_scale, out_dev, lse_dev, status_dev, g, floats);
  if (rc) return rc;
  if (workspace_bytes < floats * sizeof(float)) return QKV_ERR_CAPACITY;
  if (reinterpret_cast<uintptr_t>(workspace_dev) % 16 != 0) return QKV_ERR_ALIGN;
  if (launch_attend(static_cast<const uint8_t*>(card_dev), card_bytes, g, q_dev, (uint32_t)q_heads, softmax_scale,
                    out_dev, lse_dev, static_cast<float*>(workspace_dev), status_dev, false,
                    static_cast<hipStream_t>(stream)) != hipSuccess)
    return QKV_ERR_HIP;
  return QKV_OK;
}

int qkv_card_attend_kc(const void* card_dev, uint64_t card_bytes, const qkv_desc_t* expect, const void* q_dev,
                       int32_t q_heads, float softmax_scale, float* out_dev, float* lse_dev, void* workspace_dev,
                       uint64_t workspace_bytes, uint32_t* status_dev, void* stream) {
  if (!workspace_dev) return QKV_ERR_NULL;
  CardGeom g;
  uint64_t floats = 0;
  const int rc = prepare_attend(card_dev, card_bytes, expect, q_dev, q_heads, softmax_scale, out_dev, lse_dev, status_dev, g, floats,
                                true);
  if (rc) return rc;
  if (workspace_bytes < floats * sizeof(float)) return QKV_ERR_CAPACITY;
  if (reinterpret_cast<uintptr_t>(workspace_dev) % 16 != 0) return QKV_ERR_ALIGN;
  if (launch_attend(static_cast<const uint8_t*>(card_dev), card_bytes, g, q_dev, (uint32_t)q_heads, softmax_scale,
                    out_dev, lse_dev, static_cast<float*>(workspace_dev), status_dev, true,
                    static_cast<hipStream_t>(stream)) != hipSuccess)
    return QKV_ERR_HIP;
  return QKV_OK;
}

int qkv_card_attend_static(const void* card_dev, uint64_t card_bytes, const qkv_desc_t* expect, const void* q_dev,
                           int32_t q_heads, float softmax_scale, float* out_dev, float* lse_dev, uint32_t* status_dev,
                           void* stream) {
  CardGeom g;
  uint64_t floats = 0;
  const int rc = prepare_attend(card_dev, card_bytes, expect, q_dev, q_heads, softmax_scale, out_dev, lse_dev, status_dev, g, floats);
  if (rc) return rc;
  if (floats * sizeof(float) > (uint64_t)QKV_ATTEND_STATIC_SCRATCH_BYTES) return QKV_ERR_CAPACITY;   // shape beyond the fixed scratch
  float* scratch_at = nullptr;
  if (attend_static_scratch(&scratch_at) != hipSuccess) return QKV_ERR_HIP;
  if (launch_attend(static_cast<const uint8_t*>(card_dev), card_bytes, g, q_dev, (uint32_t)q_heads, softmax_scale,
                    out_dev, lse_dev, scratch_at, status_dev, false, static_cast<hipStream_t>(stream)) != hipSuccess)
    return QKV_ERR_HIP;
  return QKV_OK;
}

namespace {
// Copies a card's header to the host (synchronising the stream) and validates it.
static int fetch_header(const void* card_dev, uint64_t card_bytes, void* stream, qkv_card_header_t& h) {
  if (!card_dev) return QKV_ERR_NULL;
  if (card_bytes < QKV_CARD_HEADER_BYTES) return QKV_ERR_FORMAT;
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (hipMemcpyAsync(&h, card_dev, sizeof(h), hipMemcpyDeviceToHost, s) != hipSuccess) return QKV_ERR_HIP;
  if (hipStreamSynchronize(s) != hipSuccess) return QKV_ERR_HIP;
  CardGeom g;
  return header_valid(h, card_bytes, g) ? QKV_OK : QKV_ERR_FORMAT;
}
}  // namespace

int qkv_card_flags(const void* card_dev, uint64_t card_bytes, uint32_t* flags_out, void* stream) {
  if (!flags_out) return QKV_ERR_NULL;
  qkv_card_header_t h;
  const int rc = fetch_header(card_dev, card_bytes, stream, h);
  if (rc) return rc;
  *flags_out = h.flags;
  return QKV_OK;
}

int qkv_card_peek(const void* card_dev, uint64_t card_bytes, qkv_desc_t* desc_out, int64_t counts_out[4],
                  float* avg_bits_out, uint32_t* status_out, void* stream) {
  qkv_card_header_t h;
  const int rc = fetch_header(card_dev, card_bytes, stream, h);
  if (rc) return rc;
  if (desc_out) {
    desc_out->layers = (int32_t)h.layers;
    desc_out->kv_heads = (int32_t)h.kv_heads;
    desc_out->head_dim = (int32_t)h.head_dim;
    desc_out->group_size = (int32_t)h.group_size;
    desc_out->tokens = (int64_t)h.tokens;
    desc_out->model_id = h.model_id;
    desc_out->sender_id = h.sender_id;
    desc_out->position_offset = h.position_offset;
  }
  if (counts_out) for (int c = 0; c < 4; ++c) counts_out[c] = (int64_t)h.count[c];
  if (avg_bits_out) *avg_bits_out = h.avg_bits;
  if (status_out) *status_out = h.status;
  return QKV_OK;
}

}  // extern "C"
