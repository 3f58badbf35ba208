// inject_ref.cpp — CPU oracle for the position realignment of injected keys.  TEST
// INFRASTRUCTURE ONLY; the product library shares no code with it.
//
// The paper names the problem (Sec. 3.2, challenge 2: positional encodings must be realigned
// when the receiver has a different prefix) and reserves a position-offset field in the card
// for it (Sec. 4.2.1); it gives no procedure.  Reading taken here, for caches that hold keys
// after rotary position embedding in the half-split pairing (element i pairs with i + D/2,
// angle position * base^(-2i/D)): rotations compose, so a key cached at position m becomes the
// key of position m + delta by one more rotation by delta * base^(-2i/D).
//
//   theta_i = pow(base, -2 i / D)              in double
//   c_i = (float)cos(delta * theta_i),  s_i = (float)sin(delta * theta_i)     double libm, rounded to fp32
//   a = x[i], b = x[i + D/2]                   fp16 values of the dequantized cache, widened to fp32
//   x'[i]       = fp16( fma(a, c_i, -fl32(b * s_i)) )
//   x'[i + D/2] = fp16( fma(b, c_i, +fl32(a * s_i)) )
// fp32 product rounded once, one fp32 fma, then round-to-nearest-even to fp16.
#include <cmath>
#include <cstdint>

extern "C" float qkv_ref_half_to_float(uint16_t h);       // the oracle's own software conversions
extern "C" uint16_t qkv_ref_float_to_half(float f);

extern "C" {

// cos_out, sin_out: float[head_dim / 2]
int qkv_ref_rope_table(int32_t head_dim, double base, int64_t delta, float* cos_out, float* sin_out) {
  if (!cos_out || !sin_out) return -1;
  if (head_dim < 2 || head_dim % 2 != 0 || !(base > 0.0)) return -2;
  for (int i = 0; i < head_dim / 2; ++i) {
    const double theta = std::pow(base, -2.0 * i / head_dim);
    const double angle = (double)delta * theta;
    cos_out[i] = (float)std::cos(angle);
    sin_out[i] = (float)std::sin(angle);
  }
  return 0;
}

// rows: uint16_t[n_rows][head_dim] fp16 bit patterns, rotated in place.
int qkv_ref_rope_rotate(uint16_t* rows, int64_t n_rows, int32_t head_dim, const float* cos_t, const float* sin_t) {
  if (!rows || !cos_t || !sin_t) return -1;
  if (head_dim < 2 || head_dim % 2 != 0 || n_rows < 0) return -2;
  const int half = head_dim / 2;
  for (int64_t r = 0; r < n_rows; ++r) {
    uint16_t* x = rows + r * head_dim;
    for (int i = 0; i < half; ++i) {
      const float a = qkv_ref_half_to_float(x[i]);
      const float b = qkv_ref_half_to_float(x[i + half]);
      const float bs = b * sin_t[i];
      const float as = a * sin_t[i];
      x[i] = qkv_ref_float_to_half(std::fmaf(a, cos_t[i], -bs));
      x[i + half] = qkv_ref_float_to_half(std::fmaf(b, cos_t[i], as));
    }
  }
  return 0;
}

}  // extern "C"
