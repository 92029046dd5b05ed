/* CPU oracle in plain C with OpenMP: a second, independent statement of what the hot path
 * computes, used to cross-check the numpy oracle and to time the definitions on all host cores.
 * TEST INFRASTRUCTURE ONLY - the product never links or calls this.
 *
 * Same definitions as the numpy oracle, written separately:
 *   ragged_pack     DB = +0 everywhere, then DB[l_t .. l_t + e_t) = tensor t   (Section 5, DBuffer:
 *                   the fused group copy + zero)
 *   shard_reduce    out[i] = (sum over the W partials of P[w][i], in double, w ascending) / W, rounded
 *                   once to float, on the payload segments; 0 elsewhere   (Section 2.3)
 *   block quantise  per bh x bw block (edge blocks partial): amax = max |x|; scale = amax / 448 in
 *                   float; code = E4M3 (OCP "fn": bias 7, no inf, max 448) of x / scale clamped to
 *                   +-448, round to nearest, ties to even, sign kept; amax == 0: scale 0, codes 0
 *   dequantise      bf16( value(code) * scale ), nearest even
 * bf16 values travel as uint16 bit patterns.  No fast-math, no fused multiply-add: every operation is
 * a single IEEE float or double operation.
 */
#include <math.h>
#include <stdint.h>
#include <string.h>

static float bf16_to_f32(uint16_t b) {
  uint32_t u = (uint32_t)b << 16;
  float f;
  memcpy(&f, &u, 4);
  return f;
}

static uint16_t f32_to_bf16(float f) {
  uint32_t u;
  memcpy(&u, &f, 4);
  u += 0x7FFFu + ((u >> 16) & 1u);   /* nearest, ties to even (finite inputs) */
  return (uint16_t)(u >> 16);
}

/* value of an E4M3 code */
static float e4m3_value(uint8_t c) {
  const int s = c >> 7, e = (c >> 3) & 15, m = c & 7;
  const float mag = e == 0 ? ldexpf((float)m, -9) : ldexpf((float)(8 + m), e - 10);
  return s ? -mag : mag;
}

/* nearest E4M3 code of y, |y| <= 448: the exponent by frexp, the mantissa by nearbyintf (the
 * default rounding mode rounds ties to even), a carry out of the mantissa moves to the next
 * exponent; below 2^-6 the grid is the fixed step 2^-9 */
static uint8_t e4m3_encode(float y) {
  const uint8_t sign = signbit(y) ? 0x80 : 0;
  const float a = fabsf(y);
  int code;
  if (a < 0.015625f) {                       /* subnormal range, and its upper edge 2^-6 = code 8 */
    code = (int)nearbyintf(ldexpf(a, 9));
  } else {
    int ex;
    const float fr = frexpf(a, &ex);          /* a = fr * 2^ex, fr in [0.5, 1) */
    int m = (int)nearbyintf(ldexpf(fr, 4)) - 8;   /* fr * 16 in [8, 16): 1.mmm * 8 */
    int e = ex - 1 + 7;
    if (m == 8) {
      m = 0;
      ++e;
    }
    code = (e << 3) | m;
    if (code > 0x7E) code = 0x7E;
  }
  return (uint8_t)(sign | code);
}

int oc_num_threads(void);

void oc_ragged_pack(const uint16_t* const* srcs, const int64_t* offsets, const int64_t* sizes, int n,
                    uint16_t* db, int64_t total) {
  int64_t i;
  int t;
#pragma omp parallel for schedule(static)
  for (i = 0; i < total; ++i) db[i] = 0;
  for (t = 0; t < n; ++t) {
    const uint16_t* src = srcs[t];
    uint16_t* dst = db + offsets[t];
    const int64_t e = sizes[t];
#pragma omp parallel for schedule(static)
    for (i = 0; i < e; ++i) dst[i] = src[i];
  }
}

void oc_shard_reduce(const uint16_t* partials, int W, int64_t S, const int64_t* seg_off,
                     const int64_t* seg_len, int nseg, float* out) {
  int64_t i;
  int s;
#pragma omp parallel for schedule(static)
  for (i = 0; i < S; ++i) out[i] = 0.0f;
  for (s = 0; s < nseg; ++s) {
    const int64_t d = seg_off[s], len = seg_len[s];
#pragma omp parallel for schedule(static)
    for (i = 0; i < len; ++i) {
      double acc = 0.0;
      int w;
      for (w = 0; w < W; ++w) acc += (double)bf16_to_f32(partials[(int64_t)w * S + d + i]);
      out[d + i] = (float)(acc / (double)W);
    }
  }
}

/* sum over the W partials of |P[w][i]| in double: the scale of shard_reduce's accepted error */
void oc_shard_abs_sum(const uint16_t* partials, int W, int64_t S, double* out) {
  int64_t i;
#pragma omp parallel for schedule(static)
  for (i = 0; i < S; ++i) {
    double acc = 0.0;
    int w;
    for (w = 0; w < W; ++w) acc += fabs((double)bf16_to_f32(partials[(int64_t)w * S + i]));
    out[i] = acc;
  }
}

/* The mean in float, in the one stated order that makes the reduction reproducible bit for bit (a
 * reading: the paper fixes no order): partial w is added, w ascending, to running sum number
 * w mod 8, all eight starting from +0; the sums combine as ((a0+a1)+(a2+a3))+((a4+a5)+(a6+a7));
 * the result is multiplied by the float value of 1/W.  Every operation is one rounded float
 * operation (volatile keeps the compiler from re-associating or widening). */
void oc_shard_reduce_f32_ordered(const uint16_t* partials, int W, int64_t S, const int64_t* seg_off,
                                 const int64_t* seg_len, int nseg, float* out) {
  int64_t i;
  int s;
  const float inv = 1.0f / (float)W;
#pragma omp parallel for schedule(static)
  for (i = 0; i < S; ++i) out[i] = 0.0f;
  for (s = 0; s < nseg; ++s) {
    const int64_t d = seg_off[s], len = seg_len[s];
#pragma omp parallel for schedule(static)
    for (i = 0; i < len; ++i) {
      volatile float a[8] = {0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f};
      volatile float s01, s23, s45, s67, lo, hi, total;
      int w;
      for (w = 0; w < W; ++w) a[w & 7] = a[w & 7] + bf16_to_f32(partials[(int64_t)w * S + d + i]);
      s01 = a[0] + a[1];
      s23 = a[2] + a[3];
      s45 = a[4] + a[5];
      s67 = a[6] + a[7];
      lo = s01 + s23;
      hi = s45 + s67;
      total = lo + hi;
      out[d + i] = total * inv;
    }
  }
}

void oc_quantise_matrix(const uint16_t* x, int64_t R, int64_t C, int bh, int bw, uint8_t* codes,
                        float* scales) {
  const int64_t nbr = (R + bh - 1) / bh, nbc = (C + bw - 1) / bw;
  int64_t b;
#pragma omp parallel for schedule(dynamic, 4)
  for (b = 0; b < nbr * nbc; ++b) {
    const int64_t br = b / nbc, bc = b % nbc;
    const int64_t r1 = (br + 1) * bh < R ? (br + 1) * bh : R;
    const int64_t c1 = (bc + 1) * bw < C ? (bc + 1) * bw : C;
    int64_t r, c;
    float amax = 0.0f, scale;
    for (r = br * bh; r < r1; ++r)
      for (c = bc * bw; c < c1; ++c) {
        const float a = fabsf(bf16_to_f32(x[r * C + c]));
        if (a > amax) amax = a;
      }
    scale = amax / 448.0f;
    scales[b] = amax > 0.0f ? scale : 0.0f;
    for (r = br * bh; r < r1; ++r)
      for (c = bc * bw; c < c1; ++c) {
        if (amax > 0.0f) {
          float y = bf16_to_f32(x[r * C + c]) / scale;
          if (y > 448.0f) y = 448.0f;
          if (y < -448.0f) y = -448.0f;
          codes[r * C + c] = e4m3_encode(y);
        } else {
          codes[r * C + c] = 0;
        }
      }
  }
}

void oc_dequantise_matrix(const uint8_t* codes, const float* scales, int64_t R, int64_t C, int bh,
                          int bw, uint16_t* out) {
  const int64_t nbc = (C + bw - 1) / bw;
  int64_t r;
#pragma omp parallel for schedule(static)
  for (r = 0; r < R; ++r) {
    int64_t c;
    for (c = 0; c < C; ++c) {
      const float v = e4m3_value(codes[r * C + c]) * scales[(r / bh) * nbc + c / bw];
      out[r * C + c] = f32_to_bf16(v);
    }
  }
}

/* single values, for the pins */
uint8_t oc_e4m3_encode(float y) { return e4m3_encode(y); }
float oc_e4m3_value(uint8_t c) { return e4m3_value(c); }
uint16_t oc_f32_to_bf16(float f) { return f32_to_bf16(f); }

#ifdef _OPENMP
#include <omp.h>
int oc_num_threads(void) { return omp_get_max_threads(); }
void oc_set_num_threads(int n) { omp_set_num_threads(n); }
#else
int oc_num_threads(void) { return 1; }
void oc_set_num_threads(int n) { (void)n; }
#endif
