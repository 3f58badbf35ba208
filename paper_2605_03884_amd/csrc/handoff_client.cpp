// handoff_client.cpp — one handoff through the C ABI from a plain HIP host program (no Python, no torch):
// scores -> qkv_assign_bits -> qkv_quantize_pack -> qkv_unpack_dequant, buffers from hipMalloc.
//
//   handoff_client <in> <out>
//   in : int32 layers, kv_heads, head_dim, group_size; int64 tokens; double budget;
//        float scores[T]; uint16 K[L][H][T][D]; uint16 V[L][H][T][D]          (fp16 bit patterns)
//   out: int64 counts[4]; uint64 card_bytes; uint32 status; uint32 zero; uint8 bits[T]; uint8 card[card_bytes];
//        uint16 K_out[...]; uint16 V_out[...]
// Exit status 0 on success; every failing call is reported on stderr.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "qkvcard.h"

#define HIP_OK(call)                                                                          \
  do {                                                                                        \
    hipError_t e_ = (call);                                                                   \
    if (e_ != hipSuccess) { std::fprintf(stderr, "%s: %s\n", #call, hipGetErrorString(e_)); return 2; } \
  } while (0)
#define QKV_DO(call)                                                                          \
  do {                                                                                        \
    int rc_ = (call);                                                                         \
    if (rc_ != QKV_OK) { std::fprintf(stderr, "%s: %s\n", #call, qkv_error_string(rc_)); return 3; } \
  } while (0)

static bool read_all(std::FILE* f, void* p, size_t n) { return std::fread(p, 1, n, f) == n; }
static bool write_all(std::FILE* f, const void* p, size_t n) { return std::fwrite(p, 1, n, f) == n; }

int main(int argc, char** argv) {
  if (argc != 3) { std::fprintf(stderr, "usage: %s <in> <out>\n", argv[0]); return 1; }
  std::FILE* in = std::fopen(argv[1], "rb");
  if (!in) { std::perror(argv[1]); return 1; }
  int32_t shape[4];
  int64_t tokens;
  double budget;
  if (!read_all(in, shape, sizeof shape) || !read_all(in, &tokens, 8) || !read_all(in, &budget, 8)) return 1;
  qkv_desc_t desc = {};
  desc.layers = shape[0]; desc.kv_heads = shape[1]; desc.head_dim = shape[2]; desc.group_size = shape[3];
  desc.tokens = tokens; desc.model_id = 8; desc.sender_id = 1; desc.position_offset = 0;
  const size_t elems = (size_t)shape[0] * shape[1] * (size_t)tokens * shape[2];
  std::vector<float> scores((size_t)tokens);
  std::vector<uint16_t> k(elems), v(elems);
  if (!read_all(in, scores.data(), scores.size() * 4) || !read_all(in, k.data(), elems * 2) || !read_all(in, v.data(), elems * 2)) {
    std::fprintf(stderr, "short input file\n");
    return 1;
  }
  std::fclose(in);

  hipStream_t stream;
  HIP_OK(hipStreamCreate(&stream));
  float* d_scores; uint8_t* d_bits; void *d_k, *d_v, *d_ko, *d_vo; uint32_t* d_status;
  HIP_OK(hipMalloc((void**)&d_scores, scores.size() * 4));
  HIP_OK(hipMalloc((void**)&d_bits, (size_t)tokens));
  HIP_OK(hipMalloc(&d_k, elems * 2)); HIP_OK(hipMalloc(&d_v, elems * 2));
  HIP_OK(hipMalloc(&d_ko, elems * 2)); HIP_OK(hipMalloc(&d_vo, elems * 2));
  HIP_OK(hipMalloc((void**)&d_status, 4));
  HIP_OK(hipMemcpyAsync(d_scores, scores.data(), scores.size() * 4, hipMemcpyHostToDevice, stream));
  HIP_OK(hipMemcpyAsync(d_k, k.data(), elems * 2, hipMemcpyHostToDevice, stream));
  HIP_OK(hipMemcpyAsync(d_v, v.data(), elems * 2, hipMemcpyHostToDevice, stream));

  int64_t counts[4];
  QKV_DO(qkv_assign_bits(d_scores, tokens, budget, d_bits, counts, stream));      // counts: closed form, no sync needed
  uint64_t card_bytes = 0;
  QKV_DO(qkv_card_bytes(&desc, counts, &card_bytes));
  void* d_card;
  HIP_OK(hipMalloc(&d_card, card_bytes));                                          // hipMalloc returns 256-byte aligned memory
  QKV_DO(qkv_quantize_pack(&desc, d_k, d_v, d_bits, counts, d_card, card_bytes, stream));
  QKV_DO(qkv_unpack_dequant(d_card, card_bytes, &desc, d_ko, d_vo, d_status, stream));

  std::vector<uint8_t> bits((size_t)tokens), card(card_bytes);
  std::vector<uint16_t> ko(elems), vo(elems);
  uint32_t status[2] = {0xFFFFFFFFu, 0};
  HIP_OK(hipMemcpyAsync(bits.data(), d_bits, bits.size(), hipMemcpyDeviceToHost, stream));
  HIP_OK(hipMemcpyAsync(card.data(), d_card, card_bytes, hipMemcpyDeviceToHost, stream));
  HIP_OK(hipMemcpyAsync(ko.data(), d_ko, elems * 2, hipMemcpyDeviceToHost, stream));
  HIP_OK(hipMemcpyAsync(vo.data(), d_vo, elems * 2, hipMemcpyDeviceToHost, stream));
  HIP_OK(hipMemcpyAsync(status, d_status, 4, hipMemcpyDeviceToHost, stream));
  HIP_OK(hipStreamSynchronize(stream));

  std::FILE* out = std::fopen(argv[2], "wb");
  if (!out) { std::perror(argv[2]); return 1; }
  const bool ok = write_all(out, counts, sizeof counts) && write_all(out, &card_bytes, 8) && write_all(out, status, 8) &&
                  write_all(out, bits.data(), bits.size()) && write_all(out, card.data(), card.size()) &&
                  write_all(out, ko.data(), elems * 2) && write_all(out, vo.data(), elems * 2);
  std::fclose(out);
  void* all[] = {d_scores, d_bits, d_k, d_v, d_ko, d_vo, d_card, d_status};
  for (void* p : all) (void)hipFree(p);
  (void)hipStreamDestroy(stream);
  return ok ? 0 : 1;
}
