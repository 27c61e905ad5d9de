// Static-mask calibration on the device (Algorithm 2; Section 3.2.2): from a batch of calibration
// activations and the quantised weights of the layer,
//   Abar_j = mean over the calibration tokens of |A_tj|
//   I_j    = | Abar_j * sum_n s_w[n] * Wq[n, j] |
// and in every bank the k channels of largest I_j become the high-precision channels (ties to the
// lower channel).  Everything is fp64.  The two sums are formed as per-chunk partial sums (a chunk of
// rows per workgroup, its rows dealt to four waves whose sums are added in wave order) that a second
// kernel adds up in chunk order, so the result does not depend on scheduling.  Terms and partial sums of both sums are exactly representable in fp64
// whenever the summands span fewer than 53 bits between the largest sum and the smallest set bit
// (bf16 magnitudes, fp32 scale times a 4-bit integer); then the sums equal the sequential ones bit
// for bit, whatever the chunking.
#include "sq_device.h"

namespace sq {
namespace {

// Both column-sum kernels: a workgroup is 4 waves over the same channels; wave w takes rows
// r0 + w, r0 + w + 4, ... of the workgroup's chunk of rows, and the four sums are added in wave order
// through LDS.  blockIdx.y = row chunk.

// |X| column sums: lane = 8 consecutive channels (one 16-byte load per row).
__global__ __launch_bounds__(256) void calib_abs_sum_kernel(const uint16_t* __restrict__ x, int64_t ldx, int64_t T, int K,
                                                            int rows_per_chunk, double* __restrict__ partial) {
  __shared__ double red[3][64][8];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int c8 = blockIdx.x * 64 + lane;  // group of 8 channels
  const bool live = c8 * 8 < K;
  const int64_t t0 = static_cast<int64_t>(blockIdx.y) * rows_per_chunk;
  const int64_t t1 = min(T, t0 + rows_per_chunk);
  double acc[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) acc[i] = 0.0;
  if (live) {
#pragma unroll 4
    for (int64_t t = t0 + wave; t < t1; t += 4) {
      const uint4 v = *reinterpret_cast<const uint4*>(x + t * ldx + c8 * 8);
      const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        acc[2 * i] += static_cast<double>(__uint_as_float((w[i] & 0x7FFFu) << 16));
        acc[2 * i + 1] += static_cast<double>(__uint_as_float(w[i] & 0x7FFF0000u));
      }
    }
  }
  if (wave > 0) {
#pragma unroll
    for (int i = 0; i < 8; ++i) red[wave - 1][lane][i] = acc[i];
  }
  __syncthreads();
  if (wave == 0 && live) {
    double* dst = partial + static_cast<int64_t>(blockIdx.y) * K + c8 * 8;
#pragma unroll
    for (int i = 0; i < 8; ++i) dst[i] = ((acc[i] + red[0][lane][i]) + red[1][lane][i]) + red[2][lane][i];
  }
}

// Column sums of the dequantised weights: lane = 16 consecutive channels (one 8-byte load per weight row).
__global__ __launch_bounds__(256) void calib_weight_sum_kernel(const uint8_t* __restrict__ wq, const float* __restrict__ s_w,
                                                               int N, int K, int rows_per_chunk,
                                                               double* __restrict__ partial) {
  __shared__ double red[3][64][16];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int c16 = blockIdx.x * 64 + lane;  // group of 16 channels
  const bool live = c16 * 16 < K;
  const int n0 = blockIdx.y * rows_per_chunk;
  const int n1 = min(N, n0 + rows_per_chunk);
  double acc[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) acc[i] = 0.0;
  if (live) {
#pragma unroll 4
    for (int n = n0 + wave; n < n1; n += 4) {
      const uint2 v = *reinterpret_cast<const uint2*>(wq + static_cast<int64_t>(n) * (K / 2) + c16 * 8);
      const double s = static_cast<double>(s_w[n]);
      const uint32_t w[2] = {v.x, v.y};
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int code = static_cast<int>(w[i >> 3] << (28 - 4 * (i & 7))) >> 28;  // sign-extended nibble
        acc[i] = __fma_rn(s, static_cast<double>(code), acc[i]);  // the product is exact: same as multiply, then add
      }
    }
  }
  if (wave > 0) {
#pragma unroll
    for (int i = 0; i < 16; ++i) red[wave - 1][lane][i] = acc[i];
  }
  __syncthreads();
  if (wave == 0 && live) {
    double* dst = partial + static_cast<int64_t>(blockIdx.y) * K + c16 * 16;
#pragma unroll
    for (int i = 0; i < 16; ++i) dst[i] = ((acc[i] + red[0][lane][i]) + red[1][lane][i]) + red[2][lane][i];
  }
}

// I_j from the partial sums (added in chunk order), one thread per channel.
__global__ __launch_bounds__(64) void calib_importance_kernel(const double* __restrict__ pa, int chunks_a,
                                                               const double* __restrict__ pw, int chunks_w, int64_t T,
                                                               int K, double* __restrict__ importance) {
  const int j = blockIdx.x * 64 + threadIdx.x;
  if (j >= K) return;
  double a = 0.0, cs = 0.0;
  // unrolled so that the loads of several chunks are in flight together; the additions stay in chunk order
#pragma unroll 16
  for (int c = 0; c < chunks_a; ++c) a += pa[static_cast<int64_t>(c) * K + j];
#pragma unroll 16
  for (int c = 0; c < chunks_w; ++c) cs += pw[static_cast<int64_t>(c) * K + j];
  a /= static_cast<double>(T);
  importance[j] = fabs(a * cs);
}

// Per bank: the k channels of largest importance, ties to the lower channel.  One wave per bank (bank <=
// 128): lane l holds channels l and l + 64; k rounds of a wave-wide arg-max over the channels not yet
// taken (larger score wins, equal scores: lower channel), whose owner then marks its channel.
__global__ __launch_bounds__(64) void calib_select_kernel(const double* __restrict__ importance, int K, int bank, int topk,
                                                          uint32_t* __restrict__ mask) {
  const int g = blockIdx.x, lane = threadIdx.x;
  const double* imp = importance + static_cast<int64_t>(g) * bank;
  const bool has0 = lane < bank, has1 = lane + 64 < bank;
  const double v0 = has0 ? imp[lane] : 0.0, v1 = has1 ? imp[lane + 64] : 0.0;
  bool free0 = has0, free1 = has1;
  for (int t = 0; t < topk; ++t) {
    // this lane's candidate: channel `lane` is below `lane + 64`, so it also wins an equal score
    int idx = 1 << 30;
    double v = 0.0;
    if (free0) {
      idx = lane;
      v = v0;
    }
    if (free1 && (idx == (1 << 30) || v1 > v)) {
      idx = lane + 64;
      v = v1;
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
      const double ov = __shfl_xor(v, off);
      const int oi = __shfl_xor(idx, off);
      const bool mine_valid = idx != (1 << 30), other_valid = oi != (1 << 30);
      const bool take = other_valid && (!mine_valid || ov > v || (ov == v && oi < idx));
      if (take) {
        v = ov;
        idx = oi;
      }
    }
    if (idx == lane) free0 = false;
    if (idx == lane + 64) free1 = false;
  }
  const unsigned long long b0 = __ballot(has0 && !free0), b1 = __ballot(has1 && !free1);
  if (lane == 0) {
    uint32_t* dst = mask + static_cast<int64_t>(g) * (bank / 32);
    dst[0] = static_cast<uint32_t>(b0);
    if (bank >= 64) dst[1] = static_cast<uint32_t>(b0 >> 32);
    if (bank == 128) {
      dst[2] = static_cast<uint32_t>(b1);
      dst[3] = static_cast<uint32_t>(b1 >> 32);
    }
  }
}

}  // namespace

void calibrate_chunks(int64_t T, int N, int* chunks_a, int* rows_a, int* chunks_w, int* rows_w) {
  // enough row chunks to spread the work over the chip, rows per chunk not below 8 / 64
  int ra = static_cast<int>((T + 63) / 64);
  if (ra < 8) ra = 8;
  *rows_a = ra;
  *chunks_a = static_cast<int>((T + ra - 1) / ra);
  int rw = (N + 63) / 64;
  if (rw < 64) rw = 64;
  *rows_w = rw;
  *chunks_w = (N + rw - 1) / rw;
}

int launch_calibrate_static(const sq_params& p, const uint16_t* x, int64_t ldx, int64_t T, const uint8_t* wq,
                            const float* s_w, uint32_t* mask, double* importance, double* partial_a, double* partial_w,
                            hipStream_t st) {
  int ca, ra, cw, rw;
  calibrate_chunks(T, p.N, &ca, &ra, &cw, &rw);
  hipLaunchKernelGGL(calib_abs_sum_kernel, dim3((p.K / 8 + 63) / 64, ca), dim3(256), 0, st, x, ldx, T, p.K, ra,
                     partial_a);
  hipLaunchKernelGGL(calib_weight_sum_kernel, dim3((p.K / 16 + 63) / 64, cw), dim3(256), 0, st, wq, s_w, p.N, p.K, rw,
                     partial_w);
  hipLaunchKernelGGL(calib_importance_kernel, dim3((p.K + 63) / 64), dim3(64), 0, st, partial_a, ca, partial_w, cw, T,
                     p.K, importance);
  const int banks = p.K / p.bank;
  hipLaunchKernelGGL(calib_select_kernel, dim3(banks), dim3(64), 0, st, importance, p.K, p.bank, p.topk, mask);
  return hipGetLastError() == hipSuccess ? SQ_OK : SQ_ERR_LAUNCH;
}

}  // namespace sq
