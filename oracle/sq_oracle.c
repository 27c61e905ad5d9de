/*
 * CPU oracle for the SQ-format linear layer.   *** TEST INFRASTRUCTURE ***
 *
 * A plain, slow, step-by-step statement of what the layer computes, used only to
 * check the GPU library and as the timed CPU baseline.  It shares no code with the
 * GPU library, is never called from it, and is never a fallback for it.
 *
 * What it follows (paper: "SQ-format: A Unified Sparse-Quantized Hardware-friendly
 * Data Format for LLMs"):
 *   - Section 3.1, Eq. (1): a matrix is cut into banks of b contiguous elements; in
 *     every bank a fixed fraction (1-s) of the elements is kept in the high precision
 *     and the rest in the low precision; a mask says which is which; only one operand
 *     of the product is in SQ-format, the other is a plain uniform format.
 *   - Section 3.2.1: symmetric quantisation.
 *   - Section 3.2.2 and Section 4.3: on activations the dynamic rule picks, per bank
 *     and per token, the elements of largest absolute value.
 *   - Section 3.2.2 and Algorithm 2: the static rule fixes the high-precision
 *     channels of each bank ahead of time from I_j = |mean_t|A_tj| * sum_i W'_ij|.
 *   - Section 3.3: the product is the sum of a high-precision and a low-precision
 *     product, split by the mask.
 * Where the paper is silent the reading taken is stated at the function.
 *
 * Pins (tests/test_oracle_*.py): brute-force k-pass arg-max selection, hand-built
 * rows with power-of-two scales and exact half-way cases, the 2:4 special case
 * (Section 3.1), numpy int64 matmul of the unpacked operands, one-hot weights,
 * k = b (plain W4A8) and emptied-hi (plain W4A4) reductions, fp64 epilogue,
 * hand-computed bf16 half-way patterns for the output rounding,
 * a hand-computed static-importance bank, and the equivalent-bit values printed in
 * the paper's Table 3.
 * Parity unpinned: nothing in the paper prints a worked encoding or product, so
 * agreement with the authors' own implementation cannot be checked; only agreement
 * with the definitions above can.
 *
 * Conventions: M tokens (rows), K input channels, N output channels, b bank size,
 * k = (1-s)*b high-precision elements per bank, G = K/b banks per row.
 * bf16 values travel as their 16-bit patterns.  Inputs must be finite.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define SQO_OK 0
#define SQO_ERR_ARG (-1)
#define SQO_ERR_MASK (-2)     /* a bank of the static mask does not hold exactly k bits */
#define SQO_ERR_OVERFLOW (-3) /* an accumulator left the int32 range */

static float bf16_value(uint16_t bits) {
  uint32_t u = (uint32_t)bits << 16;
  float f;
  memcpy(&f, &u, sizeof f);
  return f;
}

static uint16_t bf16_round(float f) { /* round-half-even to bf16, finite inputs */
  uint32_t u;
  memcpy(&u, &f, sizeof u);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

static int magnitude_key(uint16_t bits) { return bits & 0x7FFF; } /* |x| order == integer order for finite bf16; +0 and -0 tie */

int sqo_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/*
 * Selection inside one bank (Section 3.1: fixed count per bank; Section 3.2.2 /
 * Section 4.3: by absolute activation).  Reading where the paper is silent: ties in
 * |x| go to the lower channel index.  The bank's channels are ordered by
 * (|x| descending, index ascending) with a stable insertion sort and the first k
 * are taken.
 */
static void select_bank_dynamic(const uint16_t *xb, int b, int k, uint8_t *is_hi) {
  int order[1024];
  for (int i = 0; i < b; ++i) {
    int key = magnitude_key(xb[i]);
    int p = i;
    while (p > 0 && magnitude_key(xb[order[p - 1]]) < key) { /* strict: equal keys keep index order */
      order[p] = order[p - 1];
      --p;
    }
    order[p] = i;
  }
  memset(is_hi, 0, (size_t)b);
  for (int t = 0; t < k; ++t) is_hi[order[t]] = 1;
}

/* Row-level selection, exported so that tests can pin it on its own. */
int sqo_select_dynamic(const uint16_t *x_row, int K, int b, int k, uint8_t *is_hi /* [K] */) {
  if (!x_row || !is_hi || b <= 0 || b > 1024 || k < 1 || k > b || K <= 0 || K % b) return SQO_ERR_ARG;
  for (int g = 0; g < K / b; ++g) select_bank_dynamic(x_row + (size_t)g * b, b, k, is_hi + (size_t)g * b);
  return SQO_OK;
}

static int mask_bit(const uint32_t *mask, int j) { return (mask[j >> 5] >> (j & 31)) & 1u; }

/*
 * Encode X [M, K] (row stride ldx elements) into the SQ-format of Eq. (1):
 *   d_lo     [M, K/2]  low-precision codes, INT4 two's complement, element 2i in bits 0-3 and
 *                      2i+1 in bits 4-7 of byte i; 0 at high-precision positions
 *   hi_val   [M, G, k] high-precision INT8 codes, ascending channel order inside the bank
 *   mask_out [M, K/32] (dynamic only; may be NULL in static mode) bit j%32 of word j/32 set <=> channel j is high
 *   s_lo, s_hi [M]     per-token scales
 * mode 0 = dynamic (per token top-k by |x|), 1 = static (channel mask shared by all tokens, [K/32]).
 *
 * Readings where the paper is silent:
 *   - both scales are per token: s_hi = amax_hi/127, s_lo = amax_lo/7, where amax_hi / amax_lo
 *     are the row maxima of |x| over the selected / the remaining channels;
 *   - codes are round-half-even of the fp32 product x * (Q/amax), with Q/amax one fp32 division
 *     per row, clamped to [-Q, Q] (symmetric, Section 3.2.1): -128 and -8 never occur;
 *   - an all-zero part has scale 1 and codes 0.
 */
int sqo_encode(const uint16_t *x, int64_t M, int K, int64_t ldx, int b, int k, int mode,
               const uint32_t *static_mask, uint8_t *d_lo, int8_t *hi_val, uint32_t *mask_out,
               float *s_lo, float *s_hi) {
  if (!x || !d_lo || !hi_val || !s_lo || !s_hi) return SQO_ERR_ARG;
  if (M < 0 || K <= 0 || b <= 0 || b > 1024 || k < 1 || k > b || K % b || K % 32 || ldx < K) return SQO_ERR_ARG;
  if (mode != 0 && mode != 1) return SQO_ERR_ARG;
  if (mode == 1 && !static_mask) return SQO_ERR_ARG;
  if (mode == 0 && !mask_out) return SQO_ERR_ARG;
  const int G = K / b;
  if (mode == 1) {
    for (int g = 0; g < G; ++g) {
      int c = 0;
      for (int i = 0; i < b; ++i) c += mask_bit(static_mask, g * b + i);
      if (c != k) return SQO_ERR_MASK;
    }
  }
#pragma omp parallel
  {
    uint8_t *is_hi = (uint8_t *)malloc((size_t)K);
    int *code_lo = (int *)malloc(sizeof(int) * (size_t)K);
#pragma omp for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
      const uint16_t *xr = x + m * ldx;
      /* 1. which channels are high precision */
      if (mode == 0) {
        for (int g = 0; g < G; ++g) select_bank_dynamic(xr + (size_t)g * b, b, k, is_hi + (size_t)g * b);
      } else {
        for (int j = 0; j < K; ++j) is_hi[j] = (uint8_t)mask_bit(static_mask, j);
      }
      /* 2. per-token scales */
      float amax_hi = 0.0f, amax_lo = 0.0f;
      for (int j = 0; j < K; ++j) {
        float a = fabsf(bf16_value(xr[j]));
        if (is_hi[j]) { if (a > amax_hi) amax_hi = a; }
        else          { if (a > amax_lo) amax_lo = a; }
      }
      float sc_hi = 1.0f, inv_hi = 0.0f, sc_lo = 1.0f, inv_lo = 0.0f;
      if (amax_hi != 0.0f) { sc_hi = amax_hi / 127.0f; inv_hi = 127.0f / amax_hi; }
      if (amax_lo != 0.0f) { sc_lo = amax_lo / 7.0f;   inv_lo = 7.0f / amax_lo; }
      s_hi[m] = sc_hi;
      s_lo[m] = sc_lo;
      /* 3. symmetric quantisation, round-half-even */
      int8_t *hv = hi_val + m * (int64_t)G * k;
      int nh = 0;
      for (int j = 0; j < K; ++j) {
        float v = bf16_value(xr[j]);
        if (is_hi[j]) {
          volatile float p = v * inv_hi; /* one fp32 multiply, rounded to fp32 before rounding to integer */
          float r = nearbyintf(p);
          if (r > 127.0f) r = 127.0f;
          if (r < -127.0f) r = -127.0f;
          hv[nh++] = (int8_t)(int)r; /* channels are visited in ascending order */
          code_lo[j] = 0;
        } else {
          volatile float p = v * inv_lo;
          float r = nearbyintf(p);
          if (r > 7.0f) r = 7.0f;
          if (r < -7.0f) r = -7.0f;
          code_lo[j] = (int)r;
        }
      }
      /* 4. pack */
      uint8_t *dl = d_lo + m * (int64_t)(K / 2);
      for (int i = 0; i < K / 2; ++i)
        dl[i] = (uint8_t)((code_lo[2 * i] & 0xF) | ((code_lo[2 * i + 1] & 0xF) << 4));
      if (mode == 0) {
        uint32_t *mo = mask_out + m * (int64_t)(K / 32);
        for (int wd = 0; wd < K / 32; ++wd) {
          uint32_t bits = 0;
          for (int t = 0; t < 32; ++t) bits |= (uint32_t)is_hi[wd * 32 + t] << t;
          mo[wd] = bits;
        }
      }
    }
    free(is_hi);
    free(code_lo);
  }
  return SQO_OK;
}

static int nibble_value(const uint8_t *packed, int64_t j) { /* sign-extended INT4 code j of a packed row */
  int v = (packed[j >> 1] >> ((j & 1) * 4)) & 0xF;
  return v >= 8 ? v - 16 : v;
}

/*
 * The two integer products and the dequantising epilogue (Section 3.3: the product is
 * split by the mask into a high- and a low-precision part; Eq. (1) gives each part its
 * own scale, so each has its own accumulator):
 *   acc_lo[m,n] = sum_j       D_lo[m,j] * Wq[n,j]
 *   acc_hi[m,n] = sum_{j hi}  S_hi[m,j] * Wq[n,j]
 *   y[m,n]      = (acc_lo*s_lo[m] + acc_hi*s_hi[m]) * s_w[n]
 * evaluated in fp32 as  t = (float)acc_lo * s_lo;  t = fma((float)acc_hi, s_hi, t);  y = t * s_w,
 * and again in fp64 (y64) without intermediate rounding for the tolerance test.
 * mask: mask_stride = K/32 for a dynamic encoding, 0 for a static one (one mask for every row).
 * Weights: [N, K/2] packed INT4 in [-8, 7], per-output-channel fp32 scales.
 * Any of acc_lo / acc_hi / y32 / ybf16 / y64 may be NULL.
 */
int sqo_gemm(int64_t M, int K, int64_t N, int b, int k, const uint8_t *d_lo, const int8_t *hi_val,
             const uint32_t *mask, int64_t mask_stride, const float *s_lo, const float *s_hi,
             const uint8_t *wq, const float *s_w, int32_t *acc_lo, int32_t *acc_hi, float *y32,
             uint16_t *ybf16, double *y64) {
  if (!d_lo || !hi_val || !mask || !s_lo || !s_hi || !wq || !s_w) return SQO_ERR_ARG;
  if (M < 0 || N < 0 || K <= 0 || b <= 0 || k < 1 || k > b || K % b || K % 32) return SQO_ERR_ARG;
  const int G = K / b;
  const int nhi = G * k;
  int overflow = 0;
  /* plain [N, K] copy of the weight codes */
  int8_t *w = (int8_t *)malloc((size_t)N * (size_t)K + 1);
  for (int64_t n = 0; n < N; ++n)
    for (int j = 0; j < K; ++j) w[n * K + j] = (int8_t)nibble_value(wq + n * (K / 2), j);
#pragma omp parallel reduction(| : overflow)
  {
    int8_t *d = (int8_t *)malloc((size_t)K);
    int *pos = (int *)malloc(sizeof(int) * (size_t)nhi);
#pragma omp for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
      const uint32_t *mk = mask + m * mask_stride;
      for (int j = 0; j < K; ++j) d[j] = (int8_t)nibble_value(d_lo + m * (K / 2), j);
      int c = 0;
      for (int j = 0; j < K && c < nhi; ++j)
        if (mask_bit(mk, j)) pos[c++] = j;
      for (; c < nhi; ++c) pos[c] = 0, overflow |= 2; /* malformed mask */
      const int8_t *h = hi_val + m * (int64_t)nhi;
      for (int64_t n = 0; n < N; ++n) {
        const int8_t *wr = w + n * K;
        int64_t a_lo = 0, a_hi = 0;
        for (int j = 0; j < K; ++j) a_lo += (int64_t)d[j] * (int64_t)wr[j];
        for (int t = 0; t < nhi; ++t) a_hi += (int64_t)h[t] * (int64_t)wr[pos[t]];
        if (a_lo > INT32_MAX || a_lo < INT32_MIN || a_hi > INT32_MAX || a_hi < INT32_MIN) overflow |= 1;
        if (acc_lo) acc_lo[m * N + n] = (int32_t)a_lo;
        if (acc_hi) acc_hi[m * N + n] = (int32_t)a_hi;
        volatile float t0 = (float)(int32_t)a_lo * s_lo[m];
        float t1 = fmaf((float)(int32_t)a_hi, s_hi[m], t0);
        volatile float y = t1 * s_w[n];
        if (y32) y32[m * N + n] = y;
        if (ybf16) ybf16[m * N + n] = bf16_round(y);
        if (y64)
          y64[m * N + n] = ((double)a_lo * (double)s_lo[m] + (double)a_hi * (double)s_hi[m]) * (double)s_w[n];
      }
    }
    free(d);
    free(pos);
  }
  free(w);
  if (overflow & 2) return SQO_ERR_MASK;
  if (overflow & 1) return SQO_ERR_OVERFLOW;
  return SQO_OK;
}

/*
 * Static mask from a calibration batch (Section 3.2.2, Algorithm 2):
 *   Abar_j = mean over calibration tokens of |A_tj|          (reading: mean of magnitudes)
 *   I_j    = | Abar_j * sum_n W'_nj |,  W'_nj = s_w[n]*Wq[n,j] (the dequantised weights)
 * and in every bank the k channels of largest I_j are high precision (ties to the lower index).
 * All in fp64.  importance_out [K] may be NULL.
 */
int sqo_static_mask(const uint16_t *calib, int64_t T, int K, const uint8_t *wq, const float *s_w,
                    int64_t N, int b, int k, uint32_t *mask_out /* [K/32] */, double *importance_out) {
  if (!calib || !wq || !s_w || !mask_out) return SQO_ERR_ARG;
  if (T <= 0 || N <= 0 || K <= 0 || b <= 0 || b > 1024 || k < 1 || k > b || K % b || K % 32) return SQO_ERR_ARG;
  double *imp = (double *)malloc(sizeof(double) * (size_t)K);
  for (int j = 0; j < K; ++j) {
    double a = 0.0;
    for (int64_t t = 0; t < T; ++t) a += fabs((double)bf16_value(calib[t * K + j]));
    a /= (double)T;
    double cs = 0.0;
    for (int64_t n = 0; n < N; ++n) cs += (double)s_w[n] * (double)nibble_value(wq + n * (K / 2), j);
    imp[j] = fabs(a * cs);
  }
  memset(mask_out, 0, sizeof(uint32_t) * (size_t)(K / 32));
  for (int g = 0; g < K / b; ++g) {
    int order[1024];
    for (int i = 0; i < b; ++i) {
      int p = i;
      while (p > 0 && imp[g * b + order[p - 1]] < imp[g * b + i]) {
        order[p] = order[p - 1];
        --p;
      }
      order[p] = i;
    }
    for (int t = 0; t < k; ++t) {
      int j = g * b + order[t];
      mask_out[j >> 5] |= 1u << (j & 31);
    }
  }
  if (importance_out) memcpy(importance_out, imp, sizeof(double) * (size_t)K);
  free(imp);
  return SQO_OK;
}

/* out[i] = fmaf(a[i], b[i], c[i]): the correctly rounded fused multiply-add of the C library, for the numpy
 * oracles of the layer's variants (numpy has no fused multiply-add). */
void sqo_fma32(int64_t n, const float *a, const float *b, const float *c, float *out) {
  for (int64_t i = 0; i < n; ++i) out[i] = fmaf(a[i], b[i], c[i]);
}
