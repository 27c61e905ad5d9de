/*
 * libsq — SQ-format linear layer on one AMD MI355X (gfx950).  C ABI.
 *
 * The layer (paper "SQ-format: A Unified Sparse-Quantized Hardware-friendly Data Format
 * for LLMs"): an activation matrix X [M, K] (bf16) is put into SQ-format (Section 3.1,
 * Eq. (1)): every row is cut into banks of `bank` contiguous channels; in each bank
 * `topk` channels are kept as INT8 ("high") and the others as INT4 ("low"); a mask records
 * which.  The high channels are either the per-token largest magnitudes of the bank (dynamic,
 * Sections 3.2.2 and 4.3) or fixed for all tokens by a calibrated channel mask (static,
 * Algorithm 2).  The other operand is a plain INT4 weight matrix with one scale per output
 * channel (Section 3.1: only one operand is in SQ-format).  The product is evaluated as two
 * integer products split by the mask (Section 3.3) and dequantised:
 *
 *     acc_lo[m,n] = sum_j      D_lo[m,j] * Wq[n,j]          (INT4 x INT4 -> INT32)
 *     acc_hi[m,n] = sum_{j hi} S_hi[m,j] * Wq[n,j]          (INT8 x INT4 -> INT32)
 *     Y[m,n]      = (acc_lo * s_lo[m] + acc_hi * s_hi[m]) * s_w[n]
 *
 * General rules
 *   - Every data pointer is a DEVICE pointer owned by the caller unless it says "host".
 *     The library never allocates, frees or synchronises: each call checks its arguments,
 *     enqueues kernels on `stream` (a hipStream_t passed as void*; NULL = default stream)
 *     and returns.  Structs are read on the host during the call only.
 *   - Return value: SQ_OK (0) or a negative sq_status.  Invalid arguments never launch anything.
 *   - Data pointers must be 16-byte aligned (the workspace of sq_linear: 256-byte).  ldx must keep the rows of X
 *     16-byte aligned; any ldy >= N is accepted (rows of Y that are 16-byte aligned are stored with vector stores).
 *   - Activations must be finite; NaN/Inf give unspecified codes.  A row part whose largest
 *     magnitude is subnormal gives unspecified codes.
 *   - No environment variables.  The only process-wide state is one "initialised" flag per device: the first
 *     launching call on a device (or sq_init) raises the dynamic-LDS limit of every kernel there
 *     (hipFuncSetAttribute), under a mutex; afterwards the launch path reads that flag and nothing else.
 *     Calls on different streams are independent as long as their buffers (workspace included) are distinct.
 *   - The calls may be captured into a HIP graph once the device is initialised: call sq_init() (or any
 *     launching entry point) on the device before starting a capture.
 */
#ifndef SQ_H_
#define SQ_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  SQ_OK = 0,
  SQ_ERR_NULL = -1,        /* a required pointer is NULL */
  SQ_ERR_SHAPE = -2,       /* M, K, N <= 0; K % bank; K % 64; leading dimension too small; K too large */
  SQ_ERR_UNSUPPORTED = -3, /* bank / topk / mode / out_dtype outside the supported set; static mode without a mask */
  SQ_ERR_ALIGN = -4,       /* pointer or leading dimension breaks the alignment rule */
  SQ_ERR_LAUNCH = -5,      /* the HIP runtime refused a launch */
  SQ_ERR_MASK = -6,        /* (prepack, host check) a bank of the static mask does not hold exactly topk bits */
  SQ_ERR_WORKSPACE = -7,   /* workspace NULL or smaller than sq_workspace_bytes() */
  SQ_ERR_SCRATCH = -8      /* sq_linear_noalloc: the problem needs more than SQ_NOALLOC_SCRATCH_BYTES of workspace */
} sq_status;

/* SQ_DYNAMIC_TIED: the dynamic rule with the two scales of a token tied, s_lo = 16 * s_hi (a variant for
 * hardware whose low- and high-precision products cost the same, cf. Sections 3.3 and 5.2): an INT4 low code d
 * stands for the INT8 value 16*d, the row is one INT8 operand, the layer one product with one accumulator:
 *     A = max(amax_hi, amax_lo * 127/112)   s_hi = A / 127   s_lo = 16 * s_hi
 *     acc[m,n] = sum_j c[m,j] * Wq[n,j],  c = high code at high channels, 16 * low code elsewhere
 *     Y[m,n]   = (acc * s_hi[m]) * s_w[n]
 * The stored format (d_lo, hi_val, mask, scales) is the same; sq_act::hi_dense then holds c for every channel.
 * Needs K / bank to be a power of two (at most 256, at most 128 for bank 128). */
enum { SQ_DYNAMIC = 0, SQ_STATIC = 1, SQ_DYNAMIC_TIED = 2 };
enum { SQ_OUT_F32 = 0, SQ_OUT_BF16 = 1 };

/* Problem description.  Section 4.1 writes a setting as B-(h_high/h_low)-s: here B = bank,
 * h_high/h_low = 8/4, s = 1 - topk/bank. */
typedef struct {
  int32_t M, K, N;   /* tokens, input channels, output channels.  K % bank == 0, K % 64 == 0, K <= 131072,
                        K / bank <= 512 */
  int32_t bank;      /* 32, 64 or 128 */
  int32_t topk;      /* high-precision channels per bank: a power of two, <= 32 and <= bank/2; dynamic mode also
                        >= bank/16 (the sparsities 1/2 ... 15/16 of Section 4.1); static mode: (K/bank)*topk % 32 == 0 */
  int32_t mode;      /* SQ_DYNAMIC, SQ_STATIC or SQ_DYNAMIC_TIED */
  int32_t out_dtype; /* SQ_OUT_F32 or SQ_OUT_BF16 */
  int32_t h_high;    /* bits of the high-precision codes: 8 or 4; 0 = 8 */
  int32_t h_low;     /* bits of the low-precision codes: 4, 3 or 2; 0 = 4.  Supported pairs (Section 4.1, Table 3):
                        8/4, 8/3, 8/2, 4/2.  The codes are symmetric, |code| <= 2^(bits-1) - 1, and travel in the
                        same containers whatever the pair (INT8 bytes in hi_val, 4-bit nibbles in d_lo), so the
                        products are the same kernels; sq_pack_storage writes them at their true widths.
                        SQ_DYNAMIC_TIED takes 8/4 only. */
} sq_params;

/* An activation matrix in SQ-format: ([X_quant], [S_quant], [m]) of Eq. (1). */
typedef struct {
  uint8_t *d_lo;    /* [M, K/2]  low part: INT4 two's complement in [-7, 7], channel 2i in bits 0-3 and
                       2i+1 in bits 4-7 of byte i; 0 at high positions */
  int8_t *hi_val;   /* [M, K/bank, topk]  high part: INT8 in [-127, 127], ascending channel order inside the bank */
  uint32_t *mask;   /* dynamic: [M, K/32] written by sq_encode; static: [K/32], the caller's channel mask (read only).
                       bit (j % 32) of word j/32 set <=> channel j is high precision */
  float *scale_lo;  /* [M] per-token scale of the low part  (largest low magnitude / 7) */
  float *scale_hi;  /* [M] per-token scale of the high part (largest high magnitude / 127) */
  int8_t *hi_dense; /* optional (may be NULL), dynamic modes only: [M, K] matrix-core-ready image of the high part,
                       a pure function of (hi_val, mask): the INT8 codes at their channels, 0 elsewhere, the 8
                       channels of every group stored even channels first, then odd channels (channel 8q+e sits
                       at byte 8q + 4*(e%2) + e/2).  sq_encode writes
                       it when the pointer is set; sq_gemm uses it when set and otherwise builds it in its
                       workspace.  Not part of the format: a cache that saves sq_gemm one pass.
                       SQ_DYNAMIC_TIED: the same array holds the layer's single INT8 operand instead: the high
                       codes at their channels and 16 * (low code) at the others, in the same byte order. */
  uint8_t *lo_compact; /* optional (may be NULL), static mode only: [M, K_lo/2], K_lo = K - (K/bank)*topk: the low
                       codes of the low channels only, ascending channel order, two per byte -- the activations
                       "selected and gathered" by the mask (Section 3.3), the operand that goes with the reordered
                       weights of sq_weight_prepack.  A pure function of (d_lo, mask).  sq_encode writes it when the
                       pointer is set (K <= 65535 and K <= about 37000 so that a row fits in LDS; otherwise
                       SQ_ERR_UNSUPPORTED); then d_lo may be NULL.  sq_gemm multiplies it when set (the low
                       product then runs over K_lo channels) and d_lo otherwise (over K). */
} sq_act;

/* Plain INT4 weights with one fp32 scale per output channel. */
typedef struct {
  const uint8_t *wq;      /* [N, K/2]  same nibble order as d_lo, values in [-8, 7] */
  const float *scale;     /* [N] */
  const void *prepacked;  /* static mode: output of sq_weight_prepack (required); dynamic modes: ignored, may be NULL */
} sq_weight;

/*
 * The format at its equivalent bit width (Section 4.1: y = (1-s)*h_high + s*h_low bits per element): per token
 * row a bit stream of K*y/8 bytes = the high codes of the high channels at h_high bits each, then the low codes
 * of the LOW channels only at h_low bits each, ascending channel order; code t of a section occupies its bits
 * [t*h, (t+1)*h), bit i of a section is bit i%8 of its byte i/8, two's complement.  The mask and the scales of
 * the sq_act are stored beside it, unchanged.
 *   sq_storage_row_bytes: K*y/8 (0 for invalid parameters)
 *   sq_pack_storage:   a (d_lo, hi_val, mask as in sq_gemm)  ->  packed device [M, sq_storage_row_bytes(p)]
 *   sq_unpack_storage: packed, a->mask  ->  a->d_lo, a->hi_val   (the exact inverse)
 * Storage conversions, not part of the layer's hot path; they only enqueue work on `stream`.
 */
size_t sq_storage_row_bytes(const sq_params *p);
int sq_pack_storage(const sq_params *p, const sq_act *a, uint8_t *packed, void *stream);
int sq_unpack_storage(const sq_params *p, const uint8_t *packed, const sq_act *a, void *stream);
/* The implicit-mask form (Section 3.1: the mask "represented implicitly by low-precision parts"; Section 3.2.1: the
 * code the symmetric low format leaves unused marks a high-precision element): the low section covers ALL K
 * channels and holds v_mask = -2^(h_low-1) at the high channels; no mask is stored, sq_unpack_storage_sentinel
 * writes it to a->mask (dynamic layout [M, K/32]) together with d_lo and hi_val.  K*x/8 bytes per row,
 * x = (1-s)*h_high + h_low (Section 4.1).  Dynamic modes only (SQ_ERR_UNSUPPORTED in static mode). */
size_t sq_storage_row_bytes_sentinel(const sq_params *p);
int sq_pack_storage_sentinel(const sq_params *p, const sq_act *a, uint8_t *packed, void *stream);
int sq_unpack_storage_sentinel(const sq_params *p, const uint8_t *packed, const sq_act *a, void *stream);

/* Per-device initialisation for the current device (idempotent, thread-safe): raises the kernels' dynamic-LDS
 * limits.  Every launching entry point does this on its first call on a device; call it explicitly before a
 * stream capture.  Also looks up the address of sq_linear_noalloc's scratch array.  SQ_OK or SQ_ERR_LAUNCH. */
int sq_init(void);

/* Byte sizes of the four arrays of an sq_act for these parameters (scales: M floats each).
 * Returns the total; any out pointer may be NULL.  Returns 0 if the parameters are invalid. */
size_t sq_act_bytes(const sq_params *p, size_t *d_lo, size_t *hi_val, size_t *mask, size_t *scale);

/* Bytes of device workspace sq_gemm needs when a->hi_dense is NULL (dynamic: the image of the
 * high part, M*K bytes; static: none -> returns 16 so that a valid pointer can always be passed, except for
 * M <= 32 with K % 128 == 0, where a workspace of M*K bytes lets sq_gemm run the weight-streaming decode kernel
 * on the dense low part and an image of the high part; without it the generic tile runs). */
size_t sq_gemm_workspace_bytes(const sq_params *p);

/* Bytes of device workspace sq_linear needs: the encoded activations in the form sq_gemm multiplies
 * (dynamic modes: an sq_act with hi_dense; static mode: lo_compact, hi_val and the scales). */
size_t sq_linear_workspace_bytes(const sq_params *p);

/* Bytes of sq_act::lo_compact for these parameters (static mode; 0 otherwise). */
size_t sq_lo_compact_bytes(const sq_params *p);

/* Bytes of the reordered weight image for the static mode, N*K/2 (0 in the dynamic modes). */
size_t sq_weight_prepack_bytes(const sq_params *p);

/*
 * Static mode only (Algorithm 2, last step: the weights are reordered by the mask so that the
 * kernels only select and gather on the activation side, Section 3.3): the weight columns are
 * reordered so that the high channels are contiguous and the low channels are contiguous:
 *   out = [ N x K_hi/2 bytes: columns of the high channels | N x K_lo/2 bytes: columns of the low channels ],
 * K_hi = (K/bank)*topk, K_lo = K - K_hi, ascending channel order in both (the orders of hi_val and lo_compact).
 *   wq               device [N, K/2]
 *   static_mask_host HOST   [K/32], or NULL.  When given it is checked here: every bank must hold exactly
 *                    topk bits (SQ_ERR_MASK, nothing is launched)
 *   static_mask      device [K/32] (same content as the host copy when there is one): everything on the
 *                    device is done from this one, so a mask produced by sq_calibrate_static needs no host copy
 *   out              device, sq_weight_prepack_bytes(p) bytes
 *   bad_banks        device int32, or NULL: receives the number of banks of static_mask that do not hold
 *                    exactly topk bits (0 for a valid mask); an image built from a malformed mask is unusable
 */
int sq_weight_prepack(const sq_params *p, const uint8_t *wq, const uint32_t *static_mask_host,
                      const uint32_t *static_mask, void *out, int32_t *bad_banks, void *stream);

/*
 * X -> SQ-format (Eq. (1); selection rule of Sections 3.2.2 / 4.3 or Algorithm 2's mask).
 *   x_bf16       device [M, ldx] bf16 bit patterns, ldx >= K (elements)
 *   static_mask  device [K/32] in static mode (also stored by the caller in out->mask), NULL in dynamic mode
 *   out          arrays sized by sq_act_bytes; in static mode out->mask is not written, and out->d_lo may be NULL
 *                when out->lo_compact is set
 * Ties in magnitude go to the lower channel; codes are round-half-even of x * (Q / amax).
 */
int sq_encode(const sq_params *p, const uint16_t *x_bf16, int64_t ldx, const uint32_t *static_mask,
              const sq_act *out, void *stream);

/*
 * The two integer products of Section 3.3 and the dequantising epilogue.
 *   a           encoded activations (static mode: a->mask is the [K/32] channel mask)
 *   w           weights
 *   y           device [M, ldy] fp32 or bf16 (p->out_dtype), ldy >= N (elements)
 *   acc_lo_dbg  optional device [M, N] int32: the exact low-part accumulators (SQ_DYNAMIC_TIED: zeros)
 *   acc_hi_dbg  optional device [M, N] int32: the exact high-part accumulators (SQ_DYNAMIC_TIED: the single
 *               accumulator of the combined operand)
 *   workspace   device, sq_gemm_workspace_bytes(p) bytes, contents destroyed; may be NULL (size 0) when
 *               a->hi_dense is set or in static mode
 */
int sq_gemm(const sq_params *p, const sq_act *a, const sq_weight *w, void *y, int64_t ldy,
            int32_t *acc_lo_dbg, int32_t *acc_hi_dbg, void *workspace, size_t workspace_bytes, void *stream);

/* Which of its kernels sq_gemm / sq_linear run for these parameters (static storage, never NULL):
 * "tile256x256" (SQ_DYNAMIC_TIED on shapes with at least 512 tiles of 256 x 256), "tile128x256" (workgroup tile of 128 tokens x 256 output channels; shapes with more than 128 such tiles),
 * "tile128x128" (fewer tiles), "tile64x64" (M <= 64), "tile64x128" (33 <= M <= 64 and N >= 25473), "stream32" (dynamic mode, M <= 32, K % 128 == 0: the
 * weight-streaming decode kernel), or "invalid".  Informational: tests use it to state which kernel a case covers. */
const char *sq_gemm_variant(const sq_params *p);

/* sq_encode into the workspace followed by sq_gemm: Y = SQ(X) . W^T, everything on `stream`.
 * workspace: device, 256-byte aligned, sq_linear_workspace_bytes(p) bytes, contents destroyed. */
int sq_linear(const sq_params *p, const uint16_t *x_bf16, int64_t ldx, const uint32_t *static_mask,
              const sq_weight *w, void *y, int64_t ldy, void *workspace, size_t workspace_bytes, void *stream);

/*
 * sq_linear for callers that cannot allocate device memory: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Same arguments and result as sq_linear, without the workspace:
 * the encoded activations between sq_encode and sq_gemm are kept in a fixed device array inside the
 * library (SQ_NOALLOC_SCRATCH_BYTES per GPU the library runs on, held until the process ends).  The call
 * allocates and frees nothing.  Limit: sq_linear_workspace_bytes(p) <= SQ_NOALLOC_SCRATCH_BYTES (decode and
 * small prefill batches, e.g. 512 tokens x 8192 channels), otherwise SQ_ERR_SCRATCH and nothing is launched.
 * All calls on one GPU share that GPU's array, whatever their stream: calls that overlap in time on one GPU
 * race, so order them (one stream, or events).  The array keeps the previous call's contents; nothing in it
 * has to start at zero, every byte that is read was written earlier in the same call.
 * The array's address is looked up on the first launching call on a device or by sq_init: do one of them
 * before a capture starts.
 */
#define SQ_NOALLOC_SCRATCH_BYTES (8u << 20)
int sq_linear_noalloc(const sq_params *p, const uint16_t *x_bf16, int64_t ldx, const uint32_t *static_mask,
                      const sq_weight *w, void *y, int64_t ldy, void *stream);

/*
 * SQ-format on WEIGHTS at run time: the W(SQx)Ay linear layer (Section 3.2.1, Algorithm 1, Figure 1's caption;
 * Section 3.3; Section 4.1).  Every bank of `bank` input channels of every output channel is a quantisation group:
 * its `topk` most important weights, I = w^2 / diag(H^-1)^2, are h_high-bit codes with one scale, the others
 * h_low-bit codes with another; the low part keeps its shape and carries v_mask = -2^(h_low-1) at the high
 * positions, the high part is compact (ascending channel order).  The activations are plain per-token symmetric
 * INT8 or INT4 codes.  Per bank g the two integer products are exact; they are dequantised and added bank by bank:
 *     f = 0;  for g:  t = fl(float(acc_lo_g) * s_lo[n,g]);  t = fma(float(acc_hi_g), s_hi[n,g], t);  f = fl(f + t)
 *     Y[m,n] = fl(f * s_a[m])
 * `p`: M, K, N, bank (64 or 128), topk (1 ... bank), h_high / h_low (a pair as above), out_dtype; mode is not read.
 * Per-group low scales below 2^-122 are outside the supported range (the compute image stores them divided by 16).
 * The per-bank scales make the layer bound by vector arithmetic (five instructions per accumulator register and
 * bank), not by the matrix cores.
 */
typedef struct {
  uint8_t *lo;      /* [N, K/2]  low codes in 4-bit containers (sign-extended), v_mask at the high positions */
  int8_t *hi_val;   /* [N, K/bank, topk] */
  float *scale_lo;  /* [N, K/bank] */
  float *scale_hi;  /* [N, K/bank] */
} sq_wsq;

/* Byte sizes of the arrays of an sq_wsq (scale: each of the two); returns the total, 0 for invalid parameters. */
size_t sq_wsq_bytes(const sq_params *p, size_t *lo, size_t *hi_val, size_t *scale);
/* Offline: w_bf16 device [N, ldw] (ldw >= K) -> SQ-format.  hinv_diag: device [K] positive floats, diag(H^-1) of
 * Algorithm 1, or NULL for 1 (ranking by |w|); ties in importance go to the lower channel. */
int sq_wsq_encode(const sq_params *p, const uint16_t *w_bf16, int64_t ldw, const float *hinv_diag, const sq_wsq *out,
                  void *stream);
/* Offline: the compute-ready image of the weights, sq_wsq_prepack_bytes(p) bytes (low part with zeros at the high
 * positions; the high part as a zero-padded INT8 matrix in the byte order of sq_act::hi_dense; the two scale arrays
 * transposed to [K/bank, N rounded up to 128]). */
size_t sq_wsq_prepack_bytes(const sq_params *p);
int sq_wsq_prepack(const sq_params *p, const sq_wsq *w, void *out, void *stream);
/* Plain per-token symmetric quantisation of X [M, ldx] (bf16) to `bits` = 8 or 4: a8 device [M, K] codes (stored per 8
 * channels as even channels, then odd channels: the byte order of the weight images), a_scale device [M]. */
int sq_quantize_act(const sq_params *p, const uint16_t *x_bf16, int64_t ldx, int bits, int8_t *a8, float *a_scale,
                    void *stream);
/* The layer's products and fp32 accumulation.  prepacked: output of sq_wsq_prepack.  y device [M, ldy].
 * acc_lo_dbg / acc_hi_dbg: optional device [M, N, K/bank] int32, the exact per-bank products. */
int sq_wsq_gemm(const sq_params *p, const int8_t *a8, const float *a_scale, const sq_wsq *w, const void *prepacked, void *y,
                int64_t ldy, int32_t *acc_lo_dbg, int32_t *acc_hi_dbg, void *stream);
/* sq_quantize_act into the workspace followed by sq_wsq_gemm. */
size_t sq_wsq_linear_workspace_bytes(const sq_params *p);
int sq_wsq_linear(const sq_params *p, const uint16_t *x_bf16, int64_t ldx, int act_bits, const sq_wsq *w,
                  const void *prepacked, void *y, int64_t ldy, void *workspace, size_t workspace_bytes, void *stream);

/* Reference point for the benchmark: a plain per-token W4A8 layer (no SQ split) on the same
 * INT8 matrix-core kernel, which is what Section 4.2 says W4A8 falls back to on GPUs.
 * sq_dense_w4a8_prepack reorders the nibbles of wq [N, K/2] into `out` (N*K/2 bytes) for it; the
 * result goes into w->prepacked.  a_i8 device [M, K] INT8 codes, a_scale device [M];
 * Y = (A.Wq^T) * a_scale[m] * s_w[n].  Only M, K, N and out_dtype of `p` are read. */
int sq_dense_w4a8_prepack(const sq_params *p, const uint8_t *wq, void *out, void *stream);
int sq_dense_w4a8_gemm(const sq_params *p, const int8_t *a_i8, const float *a_scale, const sq_weight *w,
                       void *y, int64_t ldy, void *stream);

/* Static-mask calibration on the device (Algorithm 2 up to the mask; Section 3.2.2):
 *   Abar_j = mean over the T calibration tokens of |x_calib[t, j]|,
 *   I_j    = | Abar_j * sum_n scale[n] * wq[n, j] |   (the dequantised weights of the layer),
 * and in every bank the topk channels of largest I_j are the high-precision ones, ties to the lower
 * channel.  All arithmetic is fp64; the sums are formed as partial sums over fixed chunks of rows,
 * added in chunk order, so a call gives the same bits every time.
 * p: K, N, bank, topk are read, mode must be SQ_STATIC.  x_calib device bf16 [T, ldx] (ldx >= K,
 * multiple of 8, 16-byte aligned), w->wq / w->scale as for sq_gemm (w->prepacked is not read).
 * mask_out device [K/32] uint32 (bit j%32 of word j/32 set <=> channel j is high): the static_mask
 * argument of sq_encode / sq_linear and, copied to the host, of sq_weight_prepack.
 * importance_out device [K] doubles, or NULL.  workspace device, 16-byte aligned,
 * sq_calibrate_workspace_bytes(p, T) bytes (0 for invalid arguments); the caller owns everything.
 * Errors: SQ_ERR_NULL, SQ_ERR_SHAPE (T <= 0 or > 2^24, ldx < K), SQ_ERR_UNSUPPORTED (dynamic mode),
 * SQ_ERR_ALIGN, SQ_ERR_WORKSPACE, SQ_ERR_LAUNCH.  Only enqueues work on `stream`. */
size_t sq_calibrate_workspace_bytes(const sq_params *p, int64_t T);
int sq_calibrate_static(const sq_params *p, const uint16_t *x_calib, int64_t ldx, int64_t T, const sq_weight *w,
                        uint32_t *mask_out, double *importance_out, void *workspace, size_t workspace_bytes,
                        void *stream);

/* Measurement probes (used by the benchmark only; nothing on the layer's path calls them).
 * sq_probe_mfma_i8: `blocks` workgroups of 4 waves, each wave issuing iters x 8 independent
 *   v_mfma_i32_32x32x32_i8 (the instruction both products of Section 3.3 run on here) on register
 *   operands: 2 * 32768 * 8 * iters * 4 * blocks operations per launch.  random_operands != 0: the operands
 *   are pseudo-random widened INT4 codes that change from instruction to instruction (what real data looks
 *   like to the multipliers); 0: small constants (fewest bits toggling, highest clock).  `sink` device,
 *   blocks * 256 int32, receives one word per thread.  1 <= blocks <= 65536, iters >= 8 and a multiple of 8.
 * sq_probe_stream: reads read_bytes from `src` and writes write_bytes to `dst` (device, 16-byte
 *   aligned, sizes multiples of 16, either may be 0 but not both), coalesced: what a plain streaming
 *   kernel with the encoder's mix of bytes read and written sustains.
 * Both only enqueue work on `stream`; errors as for the other calls. */
int sq_probe_mfma_i8(int blocks, int iters, int random_operands, int32_t *sink, void *stream);
/* The same rate probe for the two other matrix paths of the chip that could carry a part of the layer (Section 3.3:
 * the split pays when the low-precision path is faster): kind 0 = v_mfma_scale_f32_32x32x64_f8f6f4 on FP6 E3M2
 * operands (E3M2 holds every INT4 code exactly), kind 1 = v_smfmac_i32_32x32x64_i8 (2:4 structured-sparse INT8);
 * 2 * 65536 * 8 * iters * 4 * blocks (dense-equivalent) operations per launch.  Arguments as sq_probe_mfma_i8.
 * sq_probe_fp6_tile: one wave accumulates `reps` products of a 32x64 by 64x32 tile of E3M2 codes on top of c0:
 *   a, b device, 64 lanes x 32 bytes: lane l holds row (a) / column (b) l % 32, K slots 32*(l/32) ... +31, slot t
 *   in bits [6t, 6t+6) of the lane's first 24 bytes; c device, 64 lanes x 16 floats: register r of lane l is
 *   row 8*(r/4) + 4*(l/32) + r%4, column l%32.  32-byte aligned pointers, 1 <= reps <= 2^20.
 * Used by tests/test_gpu_probes.py to show that integer products are exact on that path while sums stay below 2^24. */
int sq_probe_mfma_alt(int kind, int blocks, int iters, int32_t *sink, void *stream);
int sq_probe_fp6_tile(const void *a, const void *b, float *c, float c0, int reps, void *stream);
int sq_probe_stream(const void *src, size_t read_bytes, void *dst, size_t write_bytes, void *stream);

/* Human-readable name of a status code (static storage, never NULL). */
const char *sq_status_string(int status);

/* Library version, "major.minor". */
const char *sq_version(void);

#ifdef __cplusplus
}
#endif
#endif /* SQ_H_ */
