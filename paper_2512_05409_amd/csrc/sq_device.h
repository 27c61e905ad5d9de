// Shared declarations of the libsq kernels (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "sq.h"

namespace sq {

// Largest code magnitude of a symmetric integer format of `bits` bits (0: the default width), Section 3.2.1.
inline float code_max(int bits, int default_bits) {
  return static_cast<float>((1 << ((bits ? bits : default_bits) - 1)) - 1);
}

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

// ---- per-device initialisation (sq_api.cpp): raises the dynamic-LDS limits of the kernels and looks up
// the address of the no-allocation scratch array, once per device; every launching entry point calls it. ----
int ensure_device_ready();
int device_compute_units();  // of the current device (recorded by ensure_device_ready)
int init_gemm_kernels();     // sq_gemm.hip
int init_encode_kernels();   // sq_encode.hip
int init_scratch(int dev);   // sq_noalloc.hip

// ---- launchers (defined in the .hip files, called by the C ABI in sq_api.cpp) ----

// X -> SQ-format, dynamic rule (per-token top-k by magnitude inside each bank).
int launch_encode_dynamic(const sq_params& p, const uint16_t* x, int64_t ldx, const sq_act& out, hipStream_t st);
// The streaming kernel of the dynamic rule (sq_encode_dyn.hip): which shapes it takes, its one-time
// initialisation, and its launcher.  image: hi_dense (two scales) or the combined INT8 operand (tied), or null.
bool encode_stream_supports(const sq_params& p);
int init_encode_stream_kernels();
int launch_encode_stream(const sq_params& p, const uint16_t* x, int64_t ldx, const sq_act& out, int8_t* image, bool tied,
                         float q_hi, float q_lo, hipStream_t st);
// Row-staged static encoder (sq_encode_static.hip): shapes it takes, one-time initialisation, launcher.
bool encode_static_gather_supports(const sq_params& p);
int init_encode_static_kernels();
int launch_encode_static_gather(const sq_params& p, const uint16_t* x, int64_t ldx, const uint32_t* mask,
                                const sq_act& out, hipStream_t st);
// Static mode: the low channels' weight columns made contiguous; number of malformed banks of a mask -> *bad.
int launch_weight_prepack_lo(int N, int K, int bank, int topk, const uint8_t* wq, const uint32_t* mask, uint8_t* out,
                             hipStream_t st);
int launch_mask_check(int K, int bank, int topk, const uint32_t* mask, int32_t* bad, hipStream_t st);
// X -> SQ-format, static rule (channel mask shared by all tokens).
int launch_encode_static(const sq_params& p, const uint16_t* x, int64_t ldx, const uint32_t* mask, const sq_act& out,
                         hipStream_t st);
// (hi_val, mask) -> zero-padded INT8 image [M, K] of the high part, in the K order the GEMM kernel consumes.
int launch_expand_hi(const sq_params& p, const sq_act& a, int8_t* s_hi_dense, hipStream_t st);
// Gather of the high channels' weight columns for the static mode.
int launch_weight_prepack(int N, int K, int bank, int topk, int k_hi_padded, const uint8_t* wq, const uint32_t* mask,
                          uint8_t* out, hipStream_t st);

// Static-mask calibration (Algorithm 2): how the rows are chunked, and the four kernels.
// partial_a: [chunks_a, K] doubles, partial_w: [chunks_w, K] doubles, importance: [K] doubles.
void calibrate_chunks(int64_t T, int N, int* chunks_a, int* rows_a, int* chunks_w, int* rows_w);
int launch_calibrate_static(const sq_params& p, const uint16_t* x, int64_t ldx, int64_t T, const uint8_t* wq,
                            const float* s_w, uint32_t* mask, double* importance, double* partial_a, double* partial_w,
                            hipStream_t st);

// Pack / unpack the bit-packed storage stream (sq_storage.hip).
int launch_storage(const sq_params& p, const sq_act& act, uint8_t* packed, bool pack, bool sentinel, hipStream_t st);

// SQ-format on weights (sq_wsq.hip).
int launch_wsq_encode(const sq_params& p, const uint16_t* w, int64_t ldw, const float* hinv, const sq_wsq& out, hipStream_t st);
int init_wsq_kernels();
int launch_wsq_prepack(const sq_params& p, const sq_wsq& w, uint8_t* lo_clean, int8_t* hi_dense, float* s_lo_t, float* s_hi_t,
                       hipStream_t st);
int launch_quantize_act(const sq_params& p, const uint16_t* x, int64_t ldx, int bits, int8_t* a8, float* a_scale, hipStream_t st);
int launch_wsq_gemm(const sq_params& p, const int8_t* a8, const float* a_scale, const sq_wsq& w, const uint8_t* lo_clean,
                    const int8_t* hi_dense, const float* s_lo_t, const float* s_hi_t, void* y, int64_t ldy,
                    int32_t* acc_lo_dbg, int32_t* acc_hi_dbg, hipStream_t st);

struct GemmArgs {
  int M, N, K;          // K of the layer
  int K_lo;             // channels of the low pass: K, or K - K_hi when both operands are the reordered ones
  int K_hi;             // channels of the compact high pass (static / dense-W4A8), multiple of 32
  const uint8_t* a_lo;  // [M, K_lo/2] packed INT4 (nullptr: no low pass)
  const uint8_t* w_lo;  // [N, K_lo/2] weights of the low pass (wq, or the reordered low columns)
  const int8_t* a_hi_dense;  // dynamic: [M, K] zero-padded INT8 in consumer order (nullptr otherwise)
  const int8_t* a_hi_compact;  // static: [M, K_hi] INT8 natural order (nullptr otherwise)
  int64_t lda_hi_compact;      // row stride of a_hi_compact in bytes
  const uint8_t* wq;           // [N, K/2]
  const uint8_t* w_hi;         // static: [N, K_hi/2] gathered, half-split nibble order
  const float* s_lo;           // [M] (nullptr -> treated as 0 contribution)
  const float* s_hi;           // [M]
  const float* s_w;            // [N]
  void* y;
  int64_t ldy;
  int out_bf16;
  int32_t* acc_lo_dbg;
  int32_t* acc_hi_dbg;
};
int launch_gemm(const GemmArgs& g, hipStream_t st);
// Name of the kernel variant launch_gemm picks for a shape ("tile256x256", "tile128x256", "tile128x128",
// "tile64x64", "stream32").  dynamic: two products in one loop; single: one product (tied scales, plain W4A8).
const char* gemm_variant_name(int M, int N, int K, bool dynamic, bool single);

}  // namespace sq
