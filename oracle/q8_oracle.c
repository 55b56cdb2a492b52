/*
 * CPU oracle for low-rank Adam with 8-bit block-wise moments ("8-bit GaLore", Sec. 4.3 of
 * arXiv 2403.03507: the low-rank moments M, V are kept by an 8-bit optimizer).
 *
 * TEST INFRASTRUCTURE ONLY.  Called by the tests, never by the product path; shares no code with
 * the HIP library.
 *
 * PARITY UNPINNED BY THE PAPER: the paper names 8-bit Adam but prints neither a number format nor
 * a quantisation rule.  The format below is this build's own definition; the pins in
 * tests/test_oracle_q8.py check the oracle against that definition stated in closed form
 * (tables from exact rationals, brute-force nearest neighbour, idempotence, error bounds), not
 * against the paper.
 *
 * Definition (stated in real arithmetic; evaluated here in fp64, see oracle_adam_q8_def).
 *   Block     256 consecutive elements of the row-major moment matrix (the last block may be short).
 *   Scale     one fp32 number per block: max |m| (first moment), max v (second moment), rounded to
 *             fp32 (nearest even) because it is stored as fp32.
 *   M code    1 sign bit (set whenever m < 0, also beside the magnitude 0), 4 exponent bits e, 3 mantissa bits f:
 *               e > 0: magnitude (1 + f/8) 2^(e-15);   e = 0: magnitude (f/8) 2^-14.
 *               Largest magnitude used: e = 15, f = 0, i.e. 1.
 *   V code    5 exponent bits e, 3 mantissa bits f (no sign):
 *               e > 0: (1 + f/8) 2^(e-31);   e = 0: (f/8) 2^-30.   Largest used: e = 31, f = 0, i.e. 1.
 *   Decode    value = magnitude * scale.
 *   Encode    y = |x| / scale (0 when scale = 0); the code is the table entry NEAREST to y (an y
 *             above 1, possible only through the rounding of the scale, gets the entry 1); of two
 *             equally near entries the one with the even mantissa field wins.
 *             Written here as a search over the table, not as bit manipulation.
 *   Step      the update block of Algorithm 2 on the decoded old moments:
 *               m = beta1 m_old + (1-beta1) g ;  v = beta2 v_old + (1-beta2) g^2
 *               n = (m / (1-beta1^k)) / (sqrt(v / (1-beta2^k)) + eps)
 *             then the block's new scales are taken over the new m, v and the new codes are
 *             encoded against them.  n uses the unquantised new moments.
 *
 * Two routines implement it.
 *   oracle_adam_q8_def   THE DEFINITION: every quantity above in fp64 (decode products are exact in
 *                        fp64, the recurrence and the quotient y are rounded at 2^-53).  A code of an
 *                        fp32 implementation may differ from it only where y lies within fp32 rounding
 *                        distance of the midpoint between two table entries; the GPU stage test counts
 *                        and bounds those entries.
 *   oracle_adam_q8       SECOND CHECKER in the kernel's precision: the same step as one stated fp32
 *                        operation sequence (below), against which an fp32 kernel that follows the
 *                        sequence is bit-identical.  It says nothing the definition does not say; it
 *                        lets a test tell a wrong code from a rounding-distance code.
 *                          y = min(|x| * (1 / scale), 1): one fp32 division per block, one fp32
 *                              multiplication per element
 *                          m = fma(beta1, m_old, (1-beta1) * g)
 *                          v = fma(beta2, v_old, ((1-beta2) * g) * g)
 *                          n = (m * inv_c1) / (sqrt(v * inv_c2) + eps)
 *                        each operation rounded once; (1-beta) and inv_c are fp32 inputs.
 */
#pragma STDC FP_CONTRACT OFF
#include <math.h>
#include <stdint.h>
#include <stdlib.h>

#define Q8_BLOCK 256

/* magnitude of an M code without its sign (code & 0x7f) or of a V code, exactly, as double */
static double q8_magnitude(int code, int ebits) {
  const int f = code & 7;
  const int e = code >> 3;
  const int bias = (1 << ebits) - 1; /* 15 or 31 */
  if (e == 0) return ldexp((double)f / 8.0, 1 - bias);
  return ldexp(1.0 + (double)f / 8.0, e - bias);
}

/* number of magnitudes in use: codes 0 .. top, where top = (bias << 3) decodes to 1 */
static int q8_top(int ebits) { return ((1 << ebits) - 1) << 3; }

void oracle_q8_decode_table(int is_v, double* out /* 128 (M) or 256 (V) entries; unused codes get -1 */) {
  const int ebits = is_v ? 5 : 4;
  const int n = is_v ? 256 : 128;
  for (int c = 0; c < n; ++c) out[c] = c <= q8_top(ebits) ? q8_magnitude(c, ebits) : -1.0;
}

/* nearest table entry to y in [0, 1]; ties to the even mantissa field */
static int q8_nearest(double y, int ebits) {
  const int top = q8_top(ebits);
  int best = 0;
  double best_d = fabs(q8_magnitude(0, ebits) - y);
  for (int c = 1; c <= top; ++c) {
    const double d = fabs(q8_magnitude(c, ebits) - y); /* exact: both are short dyadic numbers / an fp32 value */
    if (d < best_d || (d == best_d && (c & 1) == 0 && (best & 1) == 1)) { best = c; best_d = d; }
  }
  return best;
}

uint8_t oracle_q8_encode_m(float x, float scale) {
  if (scale == 0.0f || x == 0.0f) return 0;
  const float inv = 1.0f / scale;   /* one fp32 division (the same for every element of a block) */
  float y = fabsf(x) * inv;         /* one fp32 multiplication */
  if (y > 1.0f) y = 1.0f;           /* |x| <= scale, but the rounded reciprocal can overshoot by an ulp */
  const int mag = q8_nearest((double)y, 4);
  return (uint8_t)((x < 0.0f ? 0x80 : 0) | mag);
}

uint8_t oracle_q8_encode_v(float x, float scale) {
  if (scale == 0.0f || x <= 0.0f) return 0;
  const float inv = 1.0f / scale;
  float y = x * inv;
  if (y > 1.0f) y = 1.0f;
  return (uint8_t)q8_nearest((double)y, 5);
}

float oracle_q8_decode_m(uint8_t code, float scale) {
  const float mag = (float)q8_magnitude(code & 0x7f, 4); /* exact */
  const float v = mag * scale;                            /* one fp32 multiplication */
  return (code & 0x80) ? -v : v;
}

float oracle_q8_decode_v(uint8_t code, float scale) { return (float)q8_magnitude(code, 5) * scale; }

/* One Adam step on `count` elements with 8-bit moments.  R: projected gradient; Mc, Vc: codes
 * (in/out); Ms, Vs: block scales (in/out, ceil(count/256) entries); N: normalised update (out). */
void oracle_adam_q8(const float* R, uint8_t* Mc, uint8_t* Vc, float* Ms, float* Vs, float* N, int64_t count,
                    float beta1, float beta2, float one_minus_beta1, float one_minus_beta2, float eps,
                    float inv_c1, float inv_c2) {
  float m[Q8_BLOCK], v[Q8_BLOCK];
  for (int64_t b0 = 0; b0 < count; b0 += Q8_BLOCK) {
    const int len = count - b0 < Q8_BLOCK ? (int)(count - b0) : Q8_BLOCK;
    const int64_t blk = b0 / Q8_BLOCK;
    float smax = 0.0f, vmax = 0.0f;
    for (int i = 0; i < len; ++i) {
      const float g = R[b0 + i];
      const float m_old = oracle_q8_decode_m(Mc[b0 + i], Ms[blk]);
      const float v_old = oracle_q8_decode_v(Vc[b0 + i], Vs[blk]);
      const float gm = one_minus_beta1 * g;
      m[i] = fmaf(beta1, m_old, gm);
      float gv = one_minus_beta2 * g;
      gv = gv * g;
      v[i] = fmaf(beta2, v_old, gv);
      const float mh = m[i] * inv_c1;
      const float vh = v[i] * inv_c2;
      const float den = sqrtf(vh) + eps;
      N[b0 + i] = mh / den;
      if (fabsf(m[i]) > smax) smax = fabsf(m[i]);
      if (v[i] > vmax) vmax = v[i];
    }
    Ms[blk] = smax;
    Vs[blk] = vmax;
    for (int i = 0; i < len; ++i) {
      Mc[b0 + i] = oracle_q8_encode_m(m[i], smax);
      Vc[b0 + i] = oracle_q8_encode_v(v[i], vmax);
    }
  }
}

/* THE DEFINITION, in fp64.  One Adam step on `count` elements with 8-bit moments.
 * R: projected gradient (fp32 values); Mc, Vc: codes (in/out); Ms, Vs: block scales (in/out, fp32,
 * ceil(count/256) entries); N: normalised update (out, fp64); Ym, Yv: the quotients |m| / scale and
 * v / scale the codes were chosen from (out, fp64; lets a test measure how far a quotient lies from
 * the midpoint between two table entries).  beta1, beta2, eps are the numbers the caller uses (for
 * an fp32 interface: the fp32-representable values); k >= 1 is the step of the bias correction. */
void oracle_adam_q8_def(const float* R, uint8_t* Mc, uint8_t* Vc, float* Ms, float* Vs, double* N, double* Ym,
                        double* Yv, int64_t count, double beta1, double beta2, double eps, int64_t k) {
  const double c1 = 1.0 - pow(beta1, (double)k);
  const double c2 = 1.0 - pow(beta2, (double)k);
  double m[Q8_BLOCK], v[Q8_BLOCK];
  for (int64_t b0 = 0; b0 < count; b0 += Q8_BLOCK) {
    const int len = count - b0 < Q8_BLOCK ? (int)(count - b0) : Q8_BLOCK;
    const int64_t blk = b0 / Q8_BLOCK;
    double mmax = 0.0, vmax = 0.0;
    for (int i = 0; i < len; ++i) {
      const double g = (double)R[b0 + i];
      const int mc = Mc[b0 + i];
      double m_old = q8_magnitude(mc & 0x7f, 4) * (double)Ms[blk]; /* exact: 4 x 24 significant bits */
      if (mc & 0x80) m_old = -m_old;
      const double v_old = q8_magnitude(Vc[b0 + i], 5) * (double)Vs[blk];
      m[i] = beta1 * m_old + (1.0 - beta1) * g;
      v[i] = beta2 * v_old + (1.0 - beta2) * g * g;
      N[b0 + i] = (m[i] / c1) / (sqrt(v[i] / c2) + eps);
      if (fabs(m[i]) > mmax) mmax = fabs(m[i]);
      if (v[i] > vmax) vmax = v[i];
    }
    const float ms = (float)mmax, vs = (float)vmax; /* stored as fp32: nearest even */
    Ms[blk] = ms;
    Vs[blk] = vs;
    for (int i = 0; i < len; ++i) {
      const double ym = ms == 0.0f ? 0.0 : fabs(m[i]) / (double)ms;
      const double yv = vs == 0.0f || v[i] <= 0.0 ? 0.0 : v[i] / (double)vs;
      Ym[b0 + i] = ym;
      Yv[b0 + i] = yv;
      const int mag = q8_nearest(ym, 4); /* an y above 1 is nearest to the top entry, 1 */
      Mc[b0 + i] = (uint8_t)((m[i] < 0.0 ? 0x80 : 0) | mag);
      Vc[b0 + i] = (uint8_t)q8_nearest(yv, 5);
    }
  }
}

/* array forms for the tests */
void oracle_q8_encode_m_array(const float* x, const float* scale, uint8_t* out, int64_t n) {
  for (int64_t i = 0; i < n; ++i) out[i] = oracle_q8_encode_m(x[i], scale[i]);
}
void oracle_q8_encode_v_array(const float* x, const float* scale, uint8_t* out, int64_t n) {
  for (int64_t i = 0; i < n; ++i) out[i] = oracle_q8_encode_v(x[i], scale[i]);
}
void oracle_q8_decode_m_array(const uint8_t* c, const float* scale, float* out, int64_t n) {
  for (int64_t i = 0; i < n; ++i) out[i] = oracle_q8_decode_m(c[i], scale[i]);
}
void oracle_q8_decode_v_array(const uint8_t* c, const float* scale, float* out, int64_t n) {
  for (int64_t i = 0; i < n; ++i) out[i] = oracle_q8_decode_v(c[i], scale[i]);
}
