// Two measurement probes behind the C ABI (sq_probe_mfma_i8, sq_probe_stream): what this chip sustains
// on the matrix instruction the products use and on a plain streaming kernel with a chosen mix of
// bytes read and written.  The benchmark prints them beside the vendor peaks; nothing on the layer's
// path calls them.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "sq.h"

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef unsigned int v4u __attribute__((ext_vector_type(4)));

// Every wave issues iters x 8 independent v_mfma_i32_32x32x32_i8 on register operands.  RANDOM: the operands
// are pseudo-random bytes that differ from instruction to instruction (eight operand pairs in rotation), which
// is what the products of real data look like to the multipliers; with constant operands the instruction
// stream is the same but far fewer bits toggle, and the chip holds a higher clock.
template <bool RANDOM>
__global__ __launch_bounds__(256) void mfma_rate_kernel(int iters, int32_t* __restrict__ sink) {
  v4i a[8], b[8];
  unsigned x = 0x9E3779B9u * (blockIdx.x * 256 + threadIdx.x + 1);
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      x = x * 1664525u + 1013904223u;
      a[i][q] = RANDOM ? static_cast<int>(x & 0xF0F0F0F0u) : (q + 1);  // widened INT4 codes: low nibbles zero
      x = x * 1664525u + 1013904223u;
      b[i][q] = RANDOM ? static_cast<int>(x & 0xF0F0F0F0u) : (q + 4);
    }
  v16i acc[8];
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[i][r] = 0;
  for (int it = 0; it < iters; it += 8) {  // iters is rounded up to a multiple of 8 by the caller
#pragma unroll
    for (int u = 0; u < 8; ++u)
#pragma unroll
      for (int i = 0; i < 8; ++i) acc[i] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[i], b[(i + u) & 7], acc[i], 0, 0, 0);
  }
  int s = 0;
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) s += acc[i][r];
  sink[blockIdx.x * 256 + threadIdx.x] = s;
}

typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));

// The two other matrix paths of CDNA4 that could carry a part of the layer, on register operands, as rate probes:
//  KIND 0: v_mfma_scale_f32_32x32x64_f8f6f4 with FP6 E3M2 operands and unit block scales (E3M2 holds every integer
//          of [-8, 8], so INT4 x INT4 products and their fp32 sums below 2^24 are exact): 2*32*32*64 operations each;
//  KIND 1: v_smfmac_i32_32x32x64_i8, the 2:4 structured-sparse INT8 instruction (A holds 2 of every 4 K slots):
//          counted as the 2*32*32*64 operations of the dense product it stands for.
// Eight independent accumulators per wave; the operands are arbitrary bit patterns (rates only).
template <int KIND>
__global__ __launch_bounds__(256) void alt_rate_kernel(int iters, int32_t* __restrict__ sink) {
  unsigned x = 0x9E3779B9u * (blockIdx.x * 256 + threadIdx.x + 1);
  v8i a[8], b[8];
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      x = x * 1664525u + 1013904223u;
      a[i][q] = static_cast<int>(x & 0x1F7DF7DFu);  // FP6: exponent fields kept below the maximum (finite values)
      x = x * 1664525u + 1013904223u;
      b[i][q] = static_cast<int>(x & 0x1F7DF7DFu);
    }
  int s = 0;
  if constexpr (KIND == 0) {
    v16f acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][r] = 0.0f;
    for (int it = 0; it < iters; it += 8) {
#pragma unroll
      for (int u = 0; u < 8; ++u)
#pragma unroll
        for (int i = 0; i < 8; ++i)
          acc[i] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a[i], b[(i + u) & 7], acc[i], 3, 3, 0, 0x7F7F7F7F, 0, 0x7F7F7F7F);
    }
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) s += static_cast<int>(acc[i][r] != 0.0f);
  } else {
    v16i acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][r] = 0;
    for (int it = 0; it < iters; it += 8) {
#pragma unroll
      for (int u = 0; u < 8; ++u)
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const v4i as = {a[i][0], a[i][1], a[i][2], a[i][3]};
          acc[i] = __builtin_amdgcn_smfmac_i32_32x32x64_i8(as, b[(i + u) & 7], acc[i], 0x44444444, 0, 0);
        }
    }
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) s += acc[i][r];
  }
  sink[blockIdx.x * 256 + threadIdx.x] = s;
}

// One 32x32x64 product on the FP6 path, for checking its exactness on integer operands: lane l holds row (A) /
// column (B) l % 32 and the 32 K slots 32*(l/32) ... +31 as 6-bit E3M2 codes, slot t in bits [6t, 6t+6) of its
// eight dwords; accumulator register r of lane l is row 8*(r/4) + 4*(l/32) + r%4, column l%32.  reps products are
// accumulated on top of c0.
__global__ __launch_bounds__(64) void fp6_tile_kernel(const v8i* __restrict__ a, const v8i* __restrict__ b,
                                                      v16f* __restrict__ c, float c0, int reps) {
  v16f acc;
#pragma unroll
  for (int r = 0; r < 16; ++r) acc[r] = c0;
  const v8i av = a[threadIdx.x], bv = b[threadIdx.x];
  for (int i = 0; i < reps; ++i)
    acc = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(av, bv, acc, 3, 3, 0, 0x7F7F7F7F, 0, 0x7F7F7F7F);
  c[threadIdx.x] = acc;
}

// Reads n_read 16-byte chunks and writes n_write chunks, both coalesced, grid-stride.
__global__ __launch_bounds__(256) void stream_kernel(const v4u* __restrict__ src, int64_t n_read, v4u* __restrict__ dst,
                                                     int64_t n_write) {
  const int64_t stride = static_cast<int64_t>(gridDim.x) * blockDim.x;
  const int64_t t = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  v4u acc = {0u, 0u, 0u, 0u};
  for (int64_t i = t; i < n_read; i += stride) acc ^= src[i];
  for (int64_t i = t; i < n_write; i += stride) dst[i] = acc;
}

}  // namespace

extern "C" int sq_probe_mfma_i8(int blocks, int iters, int random_operands, int32_t* sink, void* stream) {
  if (!sink) return SQ_ERR_NULL;
  if (blocks <= 0 || blocks > 65536 || iters <= 0 || iters % 8) return SQ_ERR_SHAPE;
  if (random_operands)
    hipLaunchKernelGGL(mfma_rate_kernel<true>, dim3(blocks), dim3(256), 0, static_cast<hipStream_t>(stream), iters, sink);
  else
    hipLaunchKernelGGL(mfma_rate_kernel<false>, dim3(blocks), dim3(256), 0, static_cast<hipStream_t>(stream), iters, sink);
  return hipGetLastError() == hipSuccess ? SQ_OK : SQ_ERR_LAUNCH;
}

extern "C" int sq_probe_mfma_alt(int kind, int blocks, int iters, int32_t* sink, void* stream) {
  if (!sink) return SQ_ERR_NULL;
  if (blocks <= 0 || blocks > 65536 || iters <= 0 || iters % 8) return SQ_ERR_SHAPE;
  if (kind == 0)
    hipLaunchKernelGGL(alt_rate_kernel<0>, dim3(blocks), dim3(256), 0, static_cast<hipStream_t>(stream), iters, sink);
  else if (kind == 1)
    hipLaunchKernelGGL(alt_rate_kernel<1>, dim3(blocks), dim3(256), 0, static_cast<hipStream_t>(stream), iters, sink);
  else
    return SQ_ERR_UNSUPPORTED;
  return hipGetLastError() == hipSuccess ? SQ_OK : SQ_ERR_LAUNCH;
}

extern "C" int sq_probe_fp6_tile(const void* a, const void* b, float* c, float c0, int reps, void* stream) {
  if (!a || !b || !c) return SQ_ERR_NULL;
  if (reps <= 0 || reps > (1 << 20)) return SQ_ERR_SHAPE;
  if ((reinterpret_cast<uintptr_t>(a) | reinterpret_cast<uintptr_t>(b) | reinterpret_cast<uintptr_t>(c)) & 31) return SQ_ERR_ALIGN;
  hipLaunchKernelGGL(fp6_tile_kernel, dim3(1), dim3(64), 0, static_cast<hipStream_t>(stream), static_cast<const v8i*>(a),
                     static_cast<const v8i*>(b), reinterpret_cast<v16f*>(c), c0, reps);
  return hipGetLastError() == hipSuccess ? SQ_OK : SQ_ERR_LAUNCH;
}

extern "C" int sq_probe_stream(const void* src, size_t read_bytes, void* dst, size_t write_bytes, void* stream) {
  if ((read_bytes && !src) || (write_bytes && !dst)) return SQ_ERR_NULL;
  if ((read_bytes | write_bytes) & 15) return SQ_ERR_SHAPE;
  if (read_bytes + write_bytes == 0) return SQ_ERR_SHAPE;
  if ((reinterpret_cast<uintptr_t>(src) | reinterpret_cast<uintptr_t>(dst)) & 15) return SQ_ERR_ALIGN;
  const int64_t n_read = static_cast<int64_t>(read_bytes / 16), n_write = static_cast<int64_t>(write_bytes / 16);
  const int64_t most = n_read > n_write ? n_read : n_write;
  int64_t blocks = (most + 255) / 256;
  if (blocks > 256 * 32) blocks = 256 * 32;  // a few chunks per thread at the benchmark's sizes
  hipLaunchKernelGGL(stream_kernel, dim3(static_cast<unsigned>(blocks)), dim3(256), 0, static_cast<hipStream_t>(stream),
                     static_cast<const v4u*>(src), n_read, static_cast<v4u*>(dst), n_write);
  return hipGetLastError() == hipSuccess ? SQ_OK : SQ_ERR_LAUNCH;
}
