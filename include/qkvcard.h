/*
 * qkvcard.h — C ABI of the CacheCard library for MI355X (gfx950).
 *
 * A CacheCard is the artifact one agent hands to the next (paper Sec. 4.2.1):
 * the sender's K/V cache as quantized groups, the token-level bit-width vector,
 * sequence length, model / sender identifiers, a position-offset placeholder and
 * the achieved average bit width.  The receiver rebuilds a dense fp16 K/V cache
 * from it before its next forward pass (paper Sec. 4.2.2).
 *
 * The paper fixes what a card carries, not its bytes; this header fixes the
 * bytes ("card layout v1").  All multi-byte fields are little-endian.
 *
 * Tensors.  K and V are fp16, contiguous [layers][kv_heads][tokens][head_dim]
 * (paper Sec. 3.1: K^(l,h), V^(l,h) in R^{n x d}).  A "plane" is one (kv, l, h)
 * matrix; planes are numbered p = kv*L*H + l*H + h with kv = 0 for K, 1 for V,
 * P = 2*L*H planes in all.  A "row" is the head_dim values of one token in one
 * plane.
 *
 * Bit widths.  Every token t has one width b(t) in {2, 4, 8, 16} shared by all
 * planes (paper Sec. 3.3); 16 means the fp16 row is carried unchanged.  Classes
 * are numbered 0..3 for widths 2, 4, 8, 16.
 *
 * Quantizer (per row, per group of G consecutive head_dim values, b < 16):
 *   mn, mx   = min / max of the group under the fp16 total order (-0 < +0)
 *   scale_h  = fp16_rne( (f32(mx) - f32(mn)) / (2^b - 1) )     fp32, IEEE division
 *   zero_h   = mn
 *   inv      = scale_h > 0 ? 1.0f / f32(scale_h) : 0           fp32, IEEE division
 *   code_i   = min(2^b - 1, rne_int( (f32(x_i) - f32(mn)) * inv ))
 *              (difference rounded to fp32, product exact, rounded once)
 *   decode   = fp16_rne( fma(f32(code_i), f32(scale_h), f32(zero_h)) )   fp32 fma
 * Code i of a row sits in bits [(i*b) mod 8, +b) of row byte floor(i*b/8).
 *
 * Card layout v1.  al(x) = x rounded up to a multiple of 256.  Sections, in order,
 * each starting 256-byte aligned, pad bytes zero:
 *   header            256 bytes, see qkv_card_header_t
 *   bits              u8 [T]           al(T)      the token-level bit-width vector
 *   slot              u32[T]           al(4T)     rank of t among tokens of its width
 *   order             u32[T]           al(4T)     tokens sorted by (class, t)
 *   codes_2, meta_2   [P][n2][D*2/8] bytes, then [P][n2][D/G]{fp16 scale, fp16 zero}
 *   codes_4, meta_4   likewise for the 4-bit tokens
 *   codes_8, meta_8   likewise for the 8-bit tokens
 *   fp16              [P][n16][D] raw fp16
 * Row j of a segment belongs to token order[base_c + j], base_c = number of tokens
 * in lower classes.  The card holds byte offsets only, so it can be copied, saved
 * and reloaded freely.
 *
 * Conventions for every entry point.
 *   - Return value: QKV_OK (0) or a negative QKV_ERR_* code.  Nothing is thrown or
 *     aborted across this boundary.  When an error is returned no output buffer has
 *     been written and no GPU work has been enqueued.
 *   - "device" pointers are HIP device memory of the current device; "host"
 *     pointers are ordinary process memory.  The caller owns every buffer; the
 *     library keeps no pointer to caller memory after a call returns and reads no
 *     environment variable.  Its only state between calls is the fixed scratch
 *     array of qkv_card_attend_static (one per GPU, its address looked up once).
 *   - No call allocates device memory except qkv_count_bits (32 bytes, freed before
 *     it returns).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  GPU
 *     work is enqueued there and the call returns without waiting, except where
 *     a function says it synchronises.
 *   - Supported shapes: head_dim in {64, 128, 256}; group_size in {32, 64, 128},
 *     group_size <= head_dim; layers, kv_heads, tokens >= 1; P * tokens < 2^32.
 */
#ifndef QKVCARD_H
#define QKVCARD_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define QKV_OK             0
#define QKV_ERR_NULL      -1  /* a required pointer is NULL                                  */
#define QKV_ERR_SHAPE     -2  /* layers / kv_heads / tokens / head_dim outside the supported set */
#define QKV_ERR_GROUP     -3  /* group_size unsupported or not dividing head_dim              */
#define QKV_ERR_BUDGET    -4  /* average-bit budget outside [2, 16] or not finite             */
#define QKV_ERR_CAPACITY  -5  /* card buffer smaller than the card                            */
#define QKV_ERR_ALIGN     -6  /* a device pointer is not aligned as required                  */
#define QKV_ERR_COUNTS    -7  /* class counts negative or not summing to tokens               */
#define QKV_ERR_HIP       -8  /* a HIP runtime call failed                                    */
#define QKV_ERR_FORMAT    -9  /* card header is not a valid layout-v1 header (peek, flags)    */
#define QKV_ERR_OVERLAP   -10 /* an output buffer overlaps an input that is read meanwhile    */

#define QKV_CARD_VERSION        1u
#define QKV_CARD_HEADER_BYTES   256u
#define QKV_CARD_ALIGN          256u

/* bits in the status words written by the kernels */
/* Header flags. */
#define QKV_FLAG_KEYS_PER_CHANNEL 1u   /* uniform card whose key groups run along the tokens of a channel */

#define QKV_STATUS_BAD_BITS     0x1u  /* a bits[] value was not 2, 4, 8 or 16 (treated as 2)   */
#define QKV_STATUS_BAD_COUNTS   0x2u  /* counts[] passed by the host differ from the histogram */
#define QKV_STATUS_BAD_HEADER   0x4u  /* unpack: magic / version / shape / sizes do not match  */
#define QKV_STATUS_BAD_ORDER    0x8u  /* an order[] entry was >= tokens (row skipped / zeros)  */

/* Problem description, host memory, caller-owned (paper Sec. 3.1 shape, Sec. 4.2.1 metadata). */
typedef struct qkv_desc {
  int32_t  layers;          /* L                                                   */
  int32_t  kv_heads;        /* H: heads the cache stores (8 for Llama-3.1-8B)      */
  int32_t  head_dim;        /* D                                                   */
  int32_t  group_size;      /* G: consecutive head_dim values sharing scale / zero */
  int64_t  tokens;          /* T: sequence length                                  */
  uint64_t model_id;        /* opaque, copied into the header                      */
  uint64_t sender_id;       /* opaque, copied into the header                      */
  int64_t  position_offset; /* placeholder, stored, not interpreted                */
} qkv_desc_t;

/* The first 256 bytes of a card (paper Sec. 4.2.1: metadata and average-bit statistics). */
typedef struct qkv_card_header {
  uint8_t  magic[8];        /*   0  "QKVCARD\0"                                 */
  uint32_t version;         /*   8  QKV_CARD_VERSION                            */
  uint32_t header_bytes;    /*  12  256                                         */
  uint32_t layers;          /*  16                                              */
  uint32_t kv_heads;        /*  20                                              */
  uint32_t head_dim;        /*  24                                              */
  uint32_t group_size;      /*  28                                              */
  uint64_t tokens;          /*  32                                              */
  uint64_t count[4];        /*  40  tokens of width 2, 4, 8, 16                 */
  uint64_t total_bytes;     /*  72  size of the whole card                      */
  uint64_t off_bits;        /*  80  byte offsets of the sections from card start */
  uint64_t off_slot;        /*  88                                              */
  uint64_t off_order;       /*  96                                              */
  uint64_t off_codes[3];    /* 104  widths 2, 4, 8                              */
  uint64_t off_meta[3];     /* 128  widths 2, 4, 8                              */
  uint64_t off_fp16;        /* 152                                              */
  uint64_t model_id;        /* 160                                              */
  uint64_t sender_id;       /* 168                                              */
  int64_t  position_offset; /* 176                                              */
  float    avg_bits;        /* 184  (float)((double)sum of b(t) / (double)T)    */
  uint32_t flags;           /* 188  0, or QKV_FLAG_KEYS_PER_CHANNEL             */
  uint32_t status;          /* 192  QKV_STATUS_* bits set by the packing kernels */
  uint8_t  reserved[60];    /* 196  zero                                        */
} qkv_card_header_t;

/* Library version as major*10000 + minor*100 + patch.  Host only.  (A utility of the boundary; no passage of the
 * paper stands behind it.  The same holds for qkv_error_string.) */
int qkv_version(void);

/* Static, NUL-terminated text for a return code.  Host only; never NULL. */
const char* qkv_error_string(int code);

/*
 * Exact size in bytes of the card for `desc` and class counts {n2, n4, n8, n16}
 * (closed form of the layout above; the paper's size model, Sec. 3.1, is its
 * leading term).  Pure host integer arithmetic, no GPU call.
 *   desc, counts, bytes_out: host.  counts must be >= 0 and sum to desc->tokens.
 */
int qkv_card_bytes(const qkv_desc_t* desc, const int64_t counts[4], uint64_t* bytes_out);

/*
 * Class counts {n2, n4, n8, n16} that an average code-bit budget buys for T tokens
 * (paper Sec. 3.3: sum of b(t) stays within the budget).  Piecewise-linear between
 * three anchor mixes: all 2-bit at 2.0; 30 % / 40 % / 25 % / 5 % (2/4/8/16 bit) at
 * 5.0; all fp16 at 16.0.  Integer arithmetic on round(budget*1000), floors, so
 * sum b(t) <= budget*T.  Pure host arithmetic, no GPU call.
 */
int qkv_budget_counts(int64_t tokens, double avg_bits_budget, int64_t counts_out[4]);

/*
 * Bit-width assignment from per-token scores and a budget (paper Sec. 3.3: S(t)
 * decides b(t) under a memory budget).  Tokens are ranked by (score descending,
 * index ascending), scores compared in the IEEE total order (-0 < +0; NaN is a
 * precondition violation); the first n16 get 16, the next n8 get 8, the next n4
 * get 4, the rest 2, with the counts of qkv_budget_counts.
 *   scores_dev: device, float[T].   bits_dev: device, uint8_t[T], written.
 *   counts_out: host, int64_t[4], filled before return without a device sync.
 * Asynchronous on `stream`.
 */
int qkv_assign_bits(const float* scores_dev, int64_t tokens, double avg_bits_budget,
                    uint8_t* bits_dev, int64_t counts_out[4], void* stream);

/*
 * Histogram of a caller-made bits vector (uniform cards as in the paper's latency experiment, Sec. 5.3, or any
 * explicit mix): a utility that yields the class counts the card-building calls need; it restates no formula of
 * the paper.
 *   bits_dev: device, uint8_t[T].  counts_out: host, int64_t[4] for widths 2,4,8,16.
 * Values other than 2/4/8/16 are not counted (the sum then falls short of T).
 * Allocates and frees a small device scratch buffer and SYNCHRONISES `stream`.
 */
int qkv_count_bits(const uint8_t* bits_dev, int64_t tokens, int64_t counts_out[4], void* stream);

/*
 * Parameters of the extended controller's network (paper Sec. 4.1.2): a 2-layer MLP with 512
 * parameters over the 6 per-token features [frequency, quality, attention variance, entropy,
 * downstream demand, segment type].  The paper fixes neither hidden width, activation nor
 * output; here: 64 hidden units with ReLU and one linear output without bias
 * (6*64 + 64 + 64 = 512), the output being the combined score S(t) of Sec. 3.3.
 */
typedef struct qkv_controller {
  float w1[64][6];   /* hidden unit j, feature i */
  float b1[64];
  float w2[64];
} qkv_controller_t;

/*
 * Scores of the controller network for every token (paper Sec. 4.1.2).
 *   features_dev: device, float[T][6], row-major, 8-byte aligned.  Caller-owned, read only.
 *   params:       host; copied into the launch, may be freed on return.
 *   scores_dev:   device, float[T], written.
 * fp32 in a fixed order: hidden unit j = relu(fma chain over the features in order, starting
 * from b1[j]); score = fma chain over the hidden units in order, starting from +0.  A hidden
 * pre-activation that is NaN counts as 0.  Asynchronous on `stream`.
 * Errors: QKV_ERR_NULL, QKV_ERR_SHAPE (T < 1 or T >= 2^31), QKV_ERR_ALIGN, QKV_ERR_HIP.
 */
int qkv_controller_scores(const float* features_dev, int64_t tokens, const qkv_controller_t* params,
                          float* scores_dev, void* stream);

/*
 * Bit widths that follow the budgeted objective of paper Sec. 3.3 literally: minimise
 * sum_t eps(b(t)) * S(t) under sum_t b(t) <= avg_bits_budget * T, with the error model
 * eps(b) = 1 / (2^b - 1).  Every token starts at 2 bits; the upgrades 2->4, 4->8, 8->16 cost
 * 2, 4, 8 bits and gain max(S, 0) * {2/15, 4/255, 32/65535} per bit (one fp32 product with the
 * constant rounded to fp32; NaN scores count as 0).  All upgrades are ranked by (gain per bit
 * descending, level ascending, token index ascending) and the longest prefix whose cost fits
 * floor(budget * T) - 2T bits is taken; the budget is read as in qkv_assign_bits (rounded to
 * 1/1000 bit).  The class counts depend on the scores, so they are produced on the device:
 *   scores_dev: device, float[T], 4-byte aligned.   bits_dev: device, uint8_t[T], written.
 *   counts_dev: device, uint64_t[4] for widths 2,4,8,16, 8-byte aligned, written; may be NULL.
 * Asynchronous on `stream`; allocates nothing.
 * Errors: QKV_ERR_NULL, QKV_ERR_SHAPE (T < 1 or T >= 2^28), QKV_ERR_BUDGET, QKV_ERR_ALIGN, QKV_ERR_HIP.
 */
int qkv_assign_bits_greedy(const float* scores_dev, int64_t tokens, double avg_bits_budget,
                           uint8_t* bits_dev, uint64_t* counts_dev, void* stream);

/*
 * CacheCard creation (paper Sec. 4.2.1): classify tokens by width and compact them
 * stably into per-width segments (slot, order), quantize and bit-pack K and V rows
 * at their token's width, copy 16-bit rows unchanged, write header and metadata.
 *   desc:     host.
 *   k_dev, v_dev: device, fp16 [L][H][T][D], 16-byte aligned, read only.  Values of
 *             tokens with b < 16 must be finite; 16-bit tokens may hold anything.
 *   bits_dev: device, uint8_t[T], values in {2,4,8,16}.
 *   counts:   host, {n2,n4,n8,n16}, must equal the histogram of bits_dev (it fixes
 *             the segment sizes before the device has looked at bits_dev).
 *   card_dev: device, 256-byte aligned, card_capacity >= qkv_card_bytes(desc, counts).
 *             Exactly qkv_card_bytes bytes are written, none beyond.
 * Faults only the device can see set header.status: QKV_STATUS_BAD_BITS,
 * QKV_STATUS_BAD_COUNTS.  The card is then unusable but every access stayed in bounds.
 * Asynchronous on `stream`.
 */
int qkv_quantize_pack(const qkv_desc_t* desc, const void* k_dev, const void* v_dev,
                      const uint8_t* bits_dev, const int64_t counts[4],
                      void* card_dev, uint64_t card_capacity, void* stream);

/*
 * The two halves of qkv_quantize_pack, for a sender that knows the widths before its K/V
 * are final (paper Sec. 4.2.1: the card's metadata - bit-width vector, sequence length,
 * identifiers, average-bit statistic - does not depend on the cache contents):
 *   qkv_card_plan  writes the header, the bits / slot / order tables and the section pads;
 *   qkv_card_fill  quantizes, packs and copies the K/V rows into a card planned with the
 *                  same desc and counts (it reads the card's order table, not bits_dev).
 * Arguments, alignment rules, error codes and status bits are those of qkv_quantize_pack;
 * plan followed by fill on one stream produces the same bytes.  Both are asynchronous.
 * qkv_card_fill trusts nothing it reads from the card: an order[] entry that names no token
 * (a card that was never planned, or was overwritten since) yields a row of zeros and sets
 * QKV_STATUS_BAD_ORDER in the status word at byte 192 of the card; no access leaves K, V or
 * the first qkv_card_bytes bytes of the card.
 */
int qkv_card_plan(const qkv_desc_t* desc, const uint8_t* bits_dev, const int64_t counts[4],
                  void* card_dev, uint64_t card_capacity, void* stream);
int qkv_card_fill(const qkv_desc_t* desc, const void* k_dev, const void* v_dev, const int64_t counts[4],
                  void* card_dev, uint64_t card_capacity, void* stream);

/*
 * Scores to a planned card in one launch (paper Sec. 3.3: the score decides the width under the
 * budget; Sec. 4.2.1: the card's bit-width vector, sequence length, identifiers and average-bit
 * statistic).  Does what qkv_assign_bits followed by qkv_card_plan does - same widths, same
 * header, tables and pads, byte for byte - but in a single kernel: the workgroup that ranks the
 * scores already holds every token's width, so slots, order[] and the header follow at once.
 *   desc:       host.  tokens < 2^31.
 *   scores_dev: device, float[T], 4-byte aligned (NaN is a precondition violation).
 *   bits_dev:   device, uint8_t[T], written; may be NULL (the widths are in the card anyway).
 *   counts_out: host, int64_t[4]: the budget's class counts (= qkv_budget_counts), filled before
 *               return without a device sync; pass them on to qkv_card_fill.
 *   card_dev:   device, 256-byte aligned, card_capacity >= qkv_card_bytes(desc, counts_out).
 * qkv_card_fill on the same stream completes the card.  qkv_assign_quantize_pack is the two in
 * one call: scores, budget and K/V in, widths and the whole card out (k_dev, v_dev as for
 * qkv_quantize_pack).  Asynchronous on `stream`; allocate nothing.
 * Errors: QKV_ERR_NULL, QKV_ERR_SHAPE, QKV_ERR_GROUP, QKV_ERR_BUDGET, QKV_ERR_ALIGN,
 * QKV_ERR_CAPACITY, QKV_ERR_HIP.
 */
int qkv_assign_plan(const qkv_desc_t* desc, const float* scores_dev, double avg_bits_budget,
                    uint8_t* bits_dev, int64_t counts_out[4], void* card_dev, uint64_t card_capacity,
                    void* stream);
int qkv_assign_quantize_pack(const qkv_desc_t* desc, const void* k_dev, const void* v_dev,
                             const float* scores_dev, double avg_bits_budget, uint8_t* bits_dev,
                             int64_t counts_out[4], void* card_dev, uint64_t card_capacity, void* stream);

/*
 * Receiver-side injection (paper Sec. 4.2.2): unpack and dequantize a card into a
 * dense fp16 K/V cache.
 *   card_dev:   device, 256-byte aligned, card_bytes readable bytes.
 *   expect:     host; layers, kv_heads, head_dim, group_size, tokens the caller's
 *               output buffers were sized for (ids and position_offset ignored).
 *   k_out_dev, v_out_dev: device, fp16 [L][H][T][D], 16-byte aligned, written in full
 *               when the card is valid.
 *   status_dev: device uint32_t, may be NULL.  Set to 0 when the header matches
 *               `expect` and fits in card_bytes, else to QKV_STATUS_BAD_HEADER and
 *               the outputs are left untouched; QKV_STATUS_BAD_ORDER is or-ed in if
 *               a corrupt order[] entry was skipped.
 * The kernels read the class counts from the header on the device, so no host copy
 * of the card is needed.  Asynchronous on `stream`.
 */
int qkv_unpack_dequant(const void* card_dev, uint64_t card_bytes, const qkv_desc_t* expect,
                       void* k_out_dev, void* v_out_dev, uint32_t* status_dev, void* stream);

/*
 * Variant for uniform cards (every token at the same width 2, 4 or 8) with the keys grouped per
 * channel, after the per-channel key / per-token value scheme the paper cites as related work
 * (Sec. 2): key outliers live in a few channels, so a key group holds the 32 tokens
 * 32 tb .. 32 tb + 31 of ONE channel instead of 32 channels of one token; values keep per-token
 * groups.  Same quantizer, same card layout and sizes; in the key planes a code section reads
 * [plane][token block][channel][32 codes] and a pair section [plane][token block][channel]; the
 * header's flags word holds QKV_FLAG_KEYS_PER_CHANNEL.
 *
 * qkv_quantize_pack_kc / qkv_unpack_dequant_kc take the arguments of qkv_quantize_pack /
 * qkv_unpack_dequant and behave like them, with these extra conditions (QKV_ERR_SHAPE otherwise):
 * group_size 32, head_dim 64 or 128, tokens a multiple of 32 (of 64 at head_dim 64); and
 * (QKV_ERR_COUNTS) counts naming exactly one of the widths 2, 4, 8 for all tokens.  A card of
 * one grouping handed to the other grouping's call is refused on the device (QKV_STATUS_BAD_HEADER,
 * nothing written); qkv_inject_layers takes either grouping (its keys_per_channel field says
 * which), and qkv_card_attend_kc is qkv_card_attend for this grouping.
 */
int qkv_quantize_pack_kc(const qkv_desc_t* desc, const void* k_dev, const void* v_dev, const uint8_t* bits_dev,
                         const int64_t counts[4], void* card_dev, uint64_t card_capacity, void* stream);
int qkv_unpack_dequant_kc(const void* card_dev, uint64_t card_bytes, const qkv_desc_t* expect,
                          void* k_out_dev, void* v_out_dev, uint32_t* status_dev, void* stream);

/*
 * Receiver-side injection into per-layer caches (paper Sec. 4.2.2: the receiver rebuilds fp16
 * past_key_values, which frameworks keep as one key tensor and one value tensor per layer), for a
 * range of layers, so that injection can run layer by layer ahead of the receiver's forward
 * pass; optionally with the keys realigned to a shifted position (Sec. 3.2, challenge 2; the
 * card's position-offset field of Sec. 4.2.1 exists for this).
 *
 * Layer layer_begin + i of the card goes to k_layers[i] / v_layers[i]: device pointers to where
 * token 0 of head 0 lands; token t of head h lands h * head_stride + t * token_stride elements
 * further, as one contiguous row of head_dim fp16 values.  A cache of shape
 * [kv_heads][capacity][head_dim] that already holds a prefix of P tokens takes
 * head_stride = capacity * head_dim, token_stride = head_dim and pointers advanced by P rows.
 * Pointers 16-byte aligned, strides multiples of 8 elements, token_stride >= head_dim.  Any
 * other layout in which rows do not overlap works too (the library checks alignment and
 * token_stride only; it cannot see the tensors' extents).  The pointer arrays are host memory,
 * read before the call returns.
 *
 * Realignment (rope_base > 0): cached keys are assumed to carry rotary position embedding in the
 * half-split pairing (element i with i + head_dim/2, angle position * rope_base^(-2i/head_dim)).
 * Moving a key by rope_delta positions is one more rotation:
 *   theta_i = pow(rope_base, -2 i / head_dim)                      (double)
 *   c_i = (float)cos(rope_delta * theta_i), s_i = (float)sin(...)   (double, rounded to fp32)
 *   x'[i]     = fp16( fma(x[i],     c_i, -fl32(x[i+D/2] * s_i)) )
 *   x'[i+D/2] = fp16( fma(x[i+D/2], c_i, +fl32(x[i]     * s_i)) )
 * applied to the dequantized fp16 key values (and to 16-bit key rows, which must then be finite);
 * values are never rotated.  rope_base == 0 copies the keys as qkv_unpack_dequant does.
 *
 * Validation, status_dev and asynchrony as for qkv_unpack_dequant.  Allocates nothing.
 * Errors: QKV_ERR_NULL, QKV_ERR_SHAPE (layer range outside the card, layer_count < 1 or
 * > QKV_INJECT_MAX_LAYERS, bad strides - negative, not multiples of 8, token_stride < head_dim,
 * token_stride * tokens or head_stride * kv_heads >= 2^46 -, rope_base < 0 or not finite, |rope_delta| >= 2^31),
 * QKV_ERR_GROUP, QKV_ERR_CAPACITY, QKV_ERR_ALIGN, QKV_ERR_HIP.
 */
#define QKV_INJECT_MAX_LAYERS 64

typedef struct qkv_inject {
  int32_t layer_begin, layer_count;
  void* const* k_layers;            /* host array [layer_count] of device pointers */
  void* const* v_layers;
  int64_t head_stride, token_stride;  /* in fp16 elements */
  double rope_base;                 /* 0: no realignment */
  int64_t rope_delta;               /* positions to move the keys by */
  int32_t keys_per_channel;         /* 1: the card was made by qkv_quantize_pack_kc (its shape rules apply), else 0 */
  int32_t reserved;                 /* 0 */
} qkv_inject_t;

int qkv_inject_layers(const void* card_dev, uint64_t card_bytes, const qkv_desc_t* expect,
                      const qkv_inject_t* where, uint32_t* status_dev, void* stream);

/*
 * One hop of a multi-hop chain without the dense cache in between (paper Sec. 3.2, challenge 3:
 * error accumulates as a cache is forwarded from agent to agent; Sec. 4.2: the card is what
 * travels).  Builds, from an incoming card and new bit widths, exactly the card that
 * qkv_quantize_pack would build from the cache qkv_unpack_dequant rebuilds - byte for byte -
 * but moves only the two cards' bytes: every span is decoded and quantized again in registers.
 *   card_in_dev, card_in_bytes: the incoming card (device, 256-byte aligned, per-token groups);
 *               validated on the device like qkv_unpack_dequant does.
 *   desc:       host; shape of both cards (must match the incoming header) and the identifiers
 *               and position offset that go into the outgoing header.
 *   bits_dev, counts: the new widths, as for qkv_quantize_pack.
 *   card_out_dev, card_out_capacity: as for qkv_quantize_pack; must not overlap the incoming card.
 *   status_dev: device uint32_t, may be NULL.  0, or QKV_STATUS_BAD_HEADER when the incoming
 *               card was refused (the outgoing card then holds header and tables but no rows),
 *               QKV_STATUS_BAD_ORDER or-ed in when a corrupt table entry of the incoming card was
 *               skipped (its rows are then zeros).
 * Asynchronous on `stream`; allocates nothing.
 * Errors: as qkv_quantize_pack; QKV_ERR_OVERLAP when the two cards' byte ranges intersect.
 */
int qkv_requantize(const void* card_in_dev, uint64_t card_in_bytes, const qkv_desc_t* desc,
                   const uint8_t* bits_dev, const int64_t counts[4], void* card_out_dev,
                   uint64_t card_out_capacity, uint32_t* status_dev, void* stream);

/*
 * Decode-step attention of one new query token directly over a card, without rebuilding
 * the dense cache (paper Sec. 4.3: consuming a foreign quantized cache inside attention,
 * which the paper names as its long-term goal).  For every layer l and query head hq, with
 * kv head h = hq / (q_heads / kv_heads):
 *     s_t = softmax_scale * <q[l][hq], K^[l][h][t]>,   t = 0 .. T-1
 *     out[l][hq] = sum_t softmax(s)_t * V^[l][h][t],   lse[l][hq] = log sum_t exp(s_t)
 * where K^, V^ are the dequantized fp16 values, exactly those qkv_unpack_dequant would
 * write (raw 16-bit rows as they are).  Scores are accumulated in fp32 from fp16 products,
 * the softmax and the weighted sum run in fp32; against the float64 definition a score is off
 * by at most head_dim * 2^-24 * softmax_scale * sum_i |q_i K^_ti| (summation order only), which
 * for caches of ordinary magnitude leaves out within a few units in 1e-6 of max|V^|.
 *   card_dev, card_bytes, expect, status_dev: as for qkv_unpack_dequant; head_dim 64, 128 or 256
 *             (the kernel is laid out for 128: at 64 half of its lanes idle, at 256 it takes the
 *             head dimension in two halves), keys grouped per token.
 *   q_dev:    device, fp16 [layers][q_heads][head_dim], 16-byte aligned.  q_heads is a multiple
 *             of kv_heads, at most 16 query heads per kv head.
 *   out_dev:  device, float [layers][q_heads][head_dim], 16-byte aligned, written in full.
 *   lse_dev:  device, float [layers][q_heads], may be NULL.  With (out, lse) the caller can
 *             merge this result with attention over its own tokens.
 *   workspace_dev: device scratch of at least qkv_card_attend_workspace() bytes, 16-byte
 *             aligned; contents on entry and exit are unspecified.
 * When the header does not match, out / lse are left untouched (status_dev says so).
 * Asynchronous on `stream`.
 *
 * Several new tokens at once (a speculative window, a short suffix): every card token precedes
 * all of them, so no mask is needed and a "query head" may just as well be a (token, head) pair.
 * With S tokens and R = query heads per kv head, S * R <= 16, lay q out as
 * [layers][kv_heads][S][R][head_dim] and pass q_heads = kv_heads * S * R; out and lse come back in
 * the same order.  The card is then read once for all S tokens.
 */
int qkv_card_attend_workspace(const qkv_desc_t* expect, int32_t q_heads, uint64_t* bytes_out);
int qkv_card_attend(const void* card_dev, uint64_t card_bytes, const qkv_desc_t* expect,
                    const void* q_dev, int32_t q_heads, float softmax_scale,
                    float* out_dev, float* lse_dev, void* workspace_dev, uint64_t workspace_bytes,
                    uint32_t* status_dev, void* stream);

/*
 * qkv_card_attend for cards whose keys are grouped per channel (those of qkv_quantize_pack_kc; paper
 * Sec. 2 names the scheme, Sec. 4.3 the goal).  Same arguments, same results to the same bound, under
 * the shape rules of qkv_quantize_pack_kc (group_size 32: QKV_ERR_GROUP otherwise; head_dim 64 or 128,
 * tokens a multiple of 32, of 64 at head_dim 64: QKV_ERR_SHAPE otherwise).  There a key group holds 32
 * tokens of one channel, so the scores contract over the card's rows, the way the weighted sum of the
 * values does.  A card of the other grouping is refused on the device (QKV_STATUS_BAD_HEADER, nothing
 * written), and so does qkv_card_attend refuse a card of this one; qkv_card_flags says which a card is.
 */
int qkv_card_attend_kc(const void* card_dev, uint64_t card_bytes, const qkv_desc_t* expect,
                       const void* q_dev, int32_t q_heads, float softmax_scale,
                       float* out_dev, float* lse_dev, void* workspace_dev, uint64_t workspace_bytes,
                       uint32_t* status_dev, void* stream);

/*
 * qkv_card_attend for callers that cannot allocate device memory - code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc: the same kernels, the same results bit for
 * bit, with the partials kept in a fixed array inside the library instead of a caller's workspace.
 * Arguments as for qkv_card_attend, without the workspace.  The call allocates and frees nothing.
 *   - The array holds QKV_ATTEND_STATIC_SCRATCH_BYTES per GPU the library runs on, from the first
 *     call on that GPU until the process ends.  A shape whose qkv_card_attend_workspace() exceeds it
 *     is refused with QKV_ERR_CAPACITY (the Llama-3.1-8B shape at 8192 tokens with 32 query heads
 *     needs 13.3 MB; at 32768 tokens use qkv_card_attend with a workspace).
 *   - All calls on one GPU share the array: two calls that overlap in time on the same GPU (on
 *     different streams, or from different threads) race and give wrong results.  Calls on one
 *     stream are ordered by the stream.  Nothing in the array needs clearing between calls: every
 *     partial a call reads it has written itself.
 *   - The first call on a GPU looks the array's device address up with the runtime; make that
 *     first call outside a graph capture.
 */
#define QKV_ATTEND_STATIC_SCRATCH_BYTES (16u << 20)
int qkv_card_attend_static(const void* card_dev, uint64_t card_bytes, const qkv_desc_t* expect,
                           const void* q_dev, int32_t q_heads, float softmax_scale,
                           float* out_dev, float* lse_dev, uint32_t* status_dev, void* stream);

/*
 * Read a card's header back to the host (paper Sec. 4.2.1: the card is self-describing - sequence length, identifiers,
 * position offset, achieved average bit width) and validate it (magic, version, shape
 * domain, counts summing to tokens, section offsets equal to the closed form,
 * total_bytes <= card_bytes).  Any out pointer may be NULL.  SYNCHRONISES `stream`.
 * Returns QKV_ERR_FORMAT for an invalid header (out values are then not written).
 */
int qkv_card_peek(const void* card_dev, uint64_t card_bytes, qkv_desc_t* desc_out,
                  int64_t counts_out[4], float* avg_bits_out, uint32_t* status_out,
                  void* stream);

/*
 * The flags word of a card's header: 0, or QKV_FLAG_KEYS_PER_CHANNEL for a card whose keys are
 * grouped per channel.  It tells a receiver which of qkv_unpack_dequant / qkv_unpack_dequant_kc
 * (and which keys_per_channel value of qkv_inject_layers) the card is for - the card is
 * self-describing (paper Sec. 4.2.1).  Validates the header like qkv_card_peek, and also that a
 * flagged card has a shape and widths that grouping allows; flags_out (host) is written only on
 * QKV_OK.  SYNCHRONISES `stream`.
 * Errors: QKV_ERR_NULL, QKV_ERR_FORMAT, QKV_ERR_HIP.
 */
int qkv_card_flags(const void* card_dev, uint64_t card_bytes, uint32_t* flags_out, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* QKVCARD_H */
