// SQ-format on WEIGHTS at run time (Section 3.2.1, Algorithm 1, Figure 1's caption; Section 3.3): the W(SQ)A8 /
// W(SQ)A4 linear layer, gfx950.  Every bank of b input channels of every output channel is a quantisation group
// of its own: its k most important weights (I = w^2 / diag(H^-1)^2) are INT8 with one scale, the others INT4 with
// another, and the low part carries the unused code v_mask at the high positions.  The activations are plain
// per-token INT8 (or INT4) codes.
//     Y[m,n] = s_a[m] * sum_g ( acc_lo[m,n,g] * s_lo[n,g] + acc_hi[m,n,g] * s_hi[n,g] )
// The scales change from bank to bank along K, so integer accumulators of different banks cannot be added: each
// bank's two products (exact, on v_mfma_i32_32x32x32_i8) are converted and folded into an fp32 accumulator in a
// fixed order.  That is 5 vector instructions per accumulator register per bank against 4 matrix instructions
// per bank of 64 channels: this layer is bound by vector arithmetic, not by the matrix cores.
// The kernels here are written for correctness against the oracle (single-buffered LDS tiles, 64 x 64 outputs per
// workgroup), not tuned: this file is the first working form of the second workload, not its final one.
#include "sq_device.h"

namespace sq {
namespace {

typedef unsigned int v4u __attribute__((ext_vector_type(4)));
constexpr float kMagic = 12582912.0f;  // 1.5 * 2^23: adding it leaves rne(x) in the low mantissa bits

__device__ __forceinline__ int rne_code(float x, float inv) {
  // the mantissa field of 1.5 * 2^23 + n is 0x400000 + n
  return static_cast<int>(__float_as_uint(__fadd_rn(__fmul_rn(x, inv), kMagic)) & 0x7FFFFFu) - 0x400000;
}
__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __uint_as_float(static_cast<uint32_t>(b) << 16); }
__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f) { return __builtin_bit_cast(uint16_t, static_cast<__bf16>(f)); }

// ---- offline: weights -> SQ-format.  One thread per (output channel, bank) group. ----
template <int B>
__global__ __launch_bounds__(64) void wsq_encode_kernel(const uint16_t* __restrict__ w, int64_t ldw, int N, int K, int kt,
                                                        const float* __restrict__ hinv, float q_hi, float q_lo, int v_mask,
                                                        uint8_t* __restrict__ lo, int8_t* __restrict__ hi_val,
                                                        float* __restrict__ s_lo, float* __restrict__ s_hi) {
  const int G = K / B;
  const int64_t idx = static_cast<int64_t>(blockIdx.x) * 64 + threadIdx.x;
  if (idx >= static_cast<int64_t>(N) * G) return;
  const int64_t n = idx / G;
  const int g = static_cast<int>(idx - n * G);
  const uint16_t* src = w + n * ldw + static_cast<int64_t>(g) * B;
  float wv[B], imp[B];
  for (int i = 0; i < B; ++i) {
    wv[i] = bf16_to_f32(src[i]);
    const float d = hinv ? hinv[g * B + i] : 1.0f;
    imp[i] = __fdiv_rn(__fmul_rn(wv[i], wv[i]), __fmul_rn(d, d));
  }
  uint32_t flag[B / 32];
  for (int q = 0; q < B / 32; ++q) flag[q] = 0;
  for (int t = 0; t < kt; ++t) {  // k passes of "largest importance not yet taken, lowest channel on ties"
    int best = -1;
    float bv = -1.0f;
    for (int i = 0; i < B; ++i) {
      const bool taken = (flag[i >> 5] >> (i & 31)) & 1u;
      if (!taken && imp[i] > bv) {
        bv = imp[i];
        best = i;
      }
    }
    if (best >= 0) flag[best >> 5] |= 1u << (best & 31);
  }
  float a_hi = 0.0f, a_lo = 0.0f;
  for (int i = 0; i < B; ++i) {
    const float a = fabsf(wv[i]);
    if ((flag[i >> 5] >> (i & 31)) & 1u) a_hi = fmaxf(a_hi, a);
    else a_lo = fmaxf(a_lo, a);
  }
  const float inv_hi = a_hi != 0.0f ? __fdiv_rn(q_hi, a_hi) : 0.0f;
  const float inv_lo = a_lo != 0.0f ? __fdiv_rn(q_lo, a_lo) : 0.0f;
  s_hi[idx] = a_hi != 0.0f ? __fdiv_rn(a_hi, q_hi) : 1.0f;
  s_lo[idx] = a_lo != 0.0f ? __fdiv_rn(a_lo, q_lo) : 1.0f;
  uint8_t* ldst = lo + n * (K / 2) + static_cast<int64_t>(g) * (B / 2);
  int8_t* hdst = hi_val + idx * kt;
  int nh = 0;
  const int iq_hi = static_cast<int>(q_hi), iq_lo = static_cast<int>(q_lo);
  for (int i = 0; i < B; i += 2) {
    uint32_t byte = 0;
    for (int e = 0; e < 2; ++e) {
      int code;
      if ((flag[(i + e) >> 5] >> ((i + e) & 31)) & 1u) {
        const int c = min(max(rne_code(wv[i + e], inv_hi), -iq_hi), iq_hi);
        if (nh < kt) hdst[nh] = static_cast<int8_t>(c);
        ++nh;
        code = v_mask;
      } else {
        code = min(max(rne_code(wv[i + e], inv_lo), -iq_lo), iq_lo);
      }
      byte |= static_cast<uint32_t>(code & 0xF) << (4 * e);
    }
    ldst[i / 2] = static_cast<uint8_t>(byte);
  }
}

// ---- offline: compute-ready image of the weights: the low part with zeros at the high positions, and the high
// part as a zero-padded INT8 matrix in the byte order the widened low part unfolds to (per 8 channels: the even
// channels, then the odd ones).  One thread per 32 channels. ----
__global__ __launch_bounds__(256) void wsq_prepack_kernel(int N, int K, int B, int kt, int vm_nibble,
                                                          const uint8_t* __restrict__ lo, const int8_t* __restrict__ hi_val,
                                                          uint8_t* __restrict__ lo_clean, int8_t* __restrict__ hi_dense) {
  const int wpr = K / 32;
  const int64_t idx = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
  if (idx >= static_cast<int64_t>(N) * wpr) return;
  const int64_t n = idx / wpr;
  const int wg = static_cast<int>(idx - n * wpr);
  const int bank = wg / (B / 32);
  const uint8_t* row = lo + n * (K / 2);
  int rank = 0;  // high weights of the bank before this word
  for (int ch = bank * B; ch < wg * 32; ++ch) rank += ((row[ch >> 1] >> ((ch & 1) * 4)) & 0xF) == vm_nibble;
  const int8_t* hv = hi_val + (n * (K / B) + bank) * kt;
  uint32_t clean[4] = {0, 0, 0, 0};
  int8_t dense[32];
  for (int i = 0; i < 32; ++i) dense[i] = 0;
  for (int i = 0; i < 32; ++i) {
    const int ch = wg * 32 + i;
    const int nib = (row[ch >> 1] >> ((ch & 1) * 4)) & 0xF;
    if (nib == vm_nibble) {
      const int pos = (i & ~7) | ((i & 1) << 2) | ((i & 7) >> 1);
      dense[pos] = rank < kt ? hv[rank] : 0;
      ++rank;
    } else {
      clean[i >> 3] |= static_cast<uint32_t>(nib) << (4 * (i & 7));
    }
  }
  *reinterpret_cast<uint4*>(lo_clean + n * (K / 2) + static_cast<int64_t>(wg) * 16) = make_uint4(clean[0], clean[1], clean[2], clean[3]);
  int8_t* hd = hi_dense + n * K + static_cast<int64_t>(wg) * 32;
  for (int i = 0; i < 32; ++i) hd[i] = dense[i];
}

// ---- run time: plain per-token symmetric quantisation of the activations (Section 4.1: the operand that is not
// in SQ-format is plain INTy), codes written in the byte order of the weight images.  One workgroup per row. ----
__global__ __launch_bounds__(256) void quantize_act_kernel(const uint16_t* __restrict__ x, int64_t ldx, int K, float q,
                                                           int8_t* __restrict__ a8, float* __restrict__ a_scale) {
  __shared__ uint32_t amax_sh;
  if (threadIdx.x == 0) amax_sh = 0;
  __syncthreads();
  const int64_t m = blockIdx.x;
  const uint16_t* row = x + m * ldx;
  uint32_t mx = 0;
  for (int c = threadIdx.x; c < K / 8; c += 256) {
    const uint4 v = *reinterpret_cast<const uint4*>(row + c * 8);
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
    for (int e = 0; e < 4; ++e) mx = max(mx, max(w[e] & 0x7FFFu, (w[e] >> 16) & 0x7FFFu));
  }
  atomicMax(&amax_sh, mx);
  __syncthreads();
  const uint32_t am = amax_sh;
  const float amax = __uint_as_float(am << 16);
  const float inv = am ? __fdiv_rn(q, amax) : 0.0f;
  if (threadIdx.x == 0) a_scale[m] = am ? __fdiv_rn(amax, q) : 1.0f;
  const int iq = static_cast<int>(q);
  for (int c = threadIdx.x; c < K / 8; c += 256) {
    const uint4 v = *reinterpret_cast<const uint4*>(row + c * 8);
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
    uint32_t ev = 0, od = 0;  // codes of the even / odd channels of the group
    for (int e = 0; e < 4; ++e) {
      const int c0 = min(max(rne_code(__uint_as_float(w[e] << 16), inv), -iq), iq);
      const int c1 = min(max(rne_code(__uint_as_float(w[e] & 0xFFFF0000u), inv), -iq), iq);
      ev |= static_cast<uint32_t>(c0 & 0xFF) << (8 * e);
      od |= static_cast<uint32_t>(c1 & 0xFF) << (8 * e);
    }
    *reinterpret_cast<uint2*>(a8 + m * K + c * 8) = make_uint2(ev, od);
  }
}

__device__ __forceinline__ v4i widen_half(const v4u p, int s) {
  const unsigned a = p[2 * s], b = p[2 * s + 1];
  return v4i{static_cast<int>((a << 4) & 0xF0F0F0F0u), static_cast<int>(a & 0xF0F0F0F0u),
             static_cast<int>((b << 4) & 0xF0F0F0F0u), static_cast<int>(b & 0xF0F0F0F0u)};
}

struct WsqGemmArgs {
  int M, N, K, G;
  const int8_t* a8;        // [M, K] activation codes
  const float* a_scale;    // [M]
  const uint8_t* lo_clean; // [N, K/2]
  const int8_t* hi_dense;  // [N, K]
  const float* s_lo;       // [N, G]
  const float* s_hi;
  void* y;
  int64_t ldy;
  int out_bf16;
  int32_t* acc_lo_dbg;     // optional [M, N, G]
  int32_t* acc_hi_dbg;
};

// 64 tokens x 64 output channels per workgroup, four waves of 32 x 32; one bank per trip.
template <int B>
__global__ __launch_bounds__(256) void wsq_gemm_kernel(WsqGemmArgs g) {
  __shared__ __attribute__((aligned(16))) char s_a[64 * B];       // activation codes of the bank
  __shared__ __attribute__((aligned(16))) char s_wl[64 * (B / 2)];  // packed low weights
  __shared__ __attribute__((aligned(16))) char s_wh[64 * B];      // INT8 high weights
  __shared__ float s_sl[64], s_sh[64];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int r = lane & 31, h = lane >> 5;
  const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
  float f[16];
#pragma unroll
  for (int q = 0; q < 16; ++q) f[q] = 0.0f;

  for (int bank = 0; bank < g.G; ++bank) {
    // ---- stage the bank's operands (rows past the edge re-read the last row; never stored) ----
    for (int c = tid; c < 64 * B / 16; c += 256) {
      const int row = c / (B / 16), ch = c % (B / 16);
      *reinterpret_cast<v4u*>(s_a + row * B + ch * 16) =
          *reinterpret_cast<const v4u*>(g.a8 + static_cast<int64_t>(min(m0 + row, g.M - 1)) * g.K + bank * B + ch * 16);
      *reinterpret_cast<v4u*>(s_wh + row * B + ch * 16) =
          *reinterpret_cast<const v4u*>(g.hi_dense + static_cast<int64_t>(min(n0 + row, g.N - 1)) * g.K + bank * B + ch * 16);
    }
    for (int c = tid; c < 64 * B / 32; c += 256) {
      const int row = c / (B / 32), ch = c % (B / 32);
      *reinterpret_cast<v4u*>(s_wl + row * (B / 2) + ch * 16) =
          *reinterpret_cast<const v4u*>(g.lo_clean + static_cast<int64_t>(min(n0 + row, g.N - 1)) * (g.K / 2) + bank * (B / 2) + ch * 16);
    }
    if (tid < 64) {
      const int64_t n = min(n0 + tid, g.N - 1);
      s_sl[tid] = g.s_lo[n * g.G + bank];
      s_sh[tid] = g.s_hi[n * g.G + bank];
    }
    __syncthreads();

    // ---- the bank's two integer products (exact) ----
    v16i acc_lo, acc_hi;
#pragma unroll
    for (int q = 0; q < 16; ++q) {
      acc_lo[q] = 0;
      acc_hi[q] = 0;
    }
#pragma unroll
    for (int kb = 0; kb < B / 64; ++kb) {
      const v4u wl = *reinterpret_cast<const v4u*>(s_wl + (32 * wn + r) * (B / 2) + kb * 32 + h * 16);
#pragma unroll
      for (int s = 0; s < 2; ++s) {
        const v4i a16 = *reinterpret_cast<const v4i*>(s_a + (32 * wm + r) * B + kb * 64 + (2 * h + s) * 16);
        const v4i wh = *reinterpret_cast<const v4i*>(s_wh + (32 * wn + r) * B + kb * 64 + (2 * h + s) * 16);
        acc_lo = __builtin_amdgcn_mfma_i32_32x32x32_i8(a16, widen_half(wl, s), acc_lo, 0, 0, 0);
        acc_hi = __builtin_amdgcn_mfma_i32_32x32x32_i8(a16, wh, acc_hi, 0, 0, 0);
      }
    }
    // ---- fold into the fp32 accumulator, in the layer's fixed order ----
    const float sl = s_sl[32 * wn + r], sh = s_sh[32 * wn + r];
#pragma unroll
    for (int q = 0; q < 16; ++q) {
      const int alo = acc_lo[q] >> 4;  // the widened low weights carry a factor 16
      float t = __fmul_rn(static_cast<float>(alo), sl);
      t = __fmaf_rn(static_cast<float>(acc_hi[q]), sh, t);
      f[q] = __fadd_rn(f[q], t);
      if (g.acc_lo_dbg || g.acc_hi_dbg) {
        const int m = m0 + 32 * wm + 8 * (q >> 2) + 4 * h + (q & 3), n = n0 + 32 * wn + r;
        if (m < g.M && n < g.N) {
          const int64_t o = (static_cast<int64_t>(m) * g.N + n) * g.G + bank;
          if (g.acc_lo_dbg) g.acc_lo_dbg[o] = alo;
          if (g.acc_hi_dbg) g.acc_hi_dbg[o] = acc_hi[q];
        }
      }
    }
    __syncthreads();  // the tiles are overwritten by the next bank
  }
  // ---- epilogue ----
  const int n = n0 + 32 * wn + r;
#pragma unroll
  for (int q = 0; q < 16; ++q) {
    const int m = m0 + 32 * wm + 8 * (q >> 2) + 4 * h + (q & 3);
    if (m < g.M && n < g.N) {
      const float y = __fmul_rn(f[q], g.a_scale[m]);
      const int64_t o = static_cast<int64_t>(m) * g.ldy + n;
      if (g.out_bf16) reinterpret_cast<uint16_t*>(g.y)[o] = f32_to_bf16_rne(y);
      else reinterpret_cast<float*>(g.y)[o] = y;
    }
  }
}

// ---- the throughput kernel ----
// 128 tokens x 128 output channels per workgroup, four waves of 64 x 64 (2 x 2 tiles of 32 x 32: 64 fp32 and 128
// integer accumulator registers per lane).  A K step is 64 channels; its operands (8 KB of activation codes, 8 KB of
// INT8 high weights, 4 KB of packed low weights, 1 KB of the bank's scales) are copied into one of three LDS stages
// by LDS-direct loads two steps ahead, rows XOR-swizzled as in the activation-SQ kernel.  After the last step of a
// bank the two integer tiles are folded into the fp32 accumulators (5 vector instructions per register): that fold,
// not the matrix instructions, is what bounds the kernel; with two workgroups per compute unit one wave's fold
// overlaps the other's matrix instructions.
typedef __attribute__((address_space(3))) void* lds_ptr_t;
constexpr int W2_A = 0, W2_WH = 8192, W2_WL = 16384, W2_SC = 20480, W2_STAGE = 21504, W2_NS = 3;

__device__ __forceinline__ int w2_off4(int row, int c) { return (row << 6) + (((c ^ (row >> 2)) & 3) << 4); }  // 64-byte rows
__device__ __forceinline__ int w2_off2(int row, int c) { return (row << 5) + (((c ^ (row >> 3)) & 1) << 4); }  // 32-byte rows

template <int N>
__device__ __forceinline__ void w2_wait() {  // at most N vector-memory operations outstanding, LDS reads drained, barrier
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_waitcnt((N & 15) | (7 << 4) | (0 << 8) | ((N >> 4) << 14));
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

struct Wsq2Args {
  int M, N, K, G, Npad, bpb;  // bpb: 64-channel steps per bank (1 or 2)
  const int8_t* a8;
  const float* a_scale;
  const uint8_t* lo_clean;
  const int8_t* hi_dense;
  const float* s_lo_t;  // [G, Npad]
  const float* s_hi_t;
  void* y;
  int64_t ldy;
  int out_bf16;
};

__global__ __launch_bounds__(256, 2) void wsq_gemm2_kernel(Wsq2Args g) {
  extern __shared__ __attribute__((aligned(16))) char lds[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;
  const int r = lane & 31, h = lane >> 5;
  const int m0 = blockIdx.y * 128, n0 = blockIdx.x * 128;
  const int steps = g.K / 64;

  // per-lane sources of the copies of one step (at k = 0)
  const char* pa[2];
  const char* pwh[2];
  const char* pwl;
  for (int i = 0; i < 2; ++i) {
    const int idx = tid + 256 * i, row = idx >> 2, c = ((idx & 3) ^ (row >> 2)) & 3;
    pa[i] = reinterpret_cast<const char*>(g.a8) + static_cast<int64_t>(min(m0 + row, g.M - 1)) * g.K + c * 16;
    pwh[i] = reinterpret_cast<const char*>(g.hi_dense) + static_cast<int64_t>(min(n0 + row, g.N - 1)) * g.K + c * 16;
  }
  {
    const int row = tid >> 1, c = ((tid & 1) ^ (row >> 3)) & 1;
    pwl = reinterpret_cast<const char*>(g.lo_clean) + static_cast<int64_t>(min(n0 + row, g.N - 1)) * (g.K / 2) + c * 16;
  }
  // scales of a bank for the workgroup's 128 channels: lanes 0-31 of wave 0 the low ones, lanes 32-63 the high ones
  const char* psc = reinterpret_cast<const char*>(lane < 32 ? g.s_lo_t : g.s_hi_t) + (static_cast<int64_t>(n0) + (lane & 31) * 4) * 4;

  auto issue = [&](int step) {
    char* st = lds + (step % W2_NS) * W2_STAGE;
    for (int i = 0; i < 2; ++i) {
      const char* src = pa[i] + step * 64;
      __builtin_amdgcn_global_load_lds(src, (lds_ptr_t)(st + W2_A + (256 * i + 64 * wave) * 16), 16, 0, 0);
    }
    for (int i = 0; i < 2; ++i) {
      const char* src = pwh[i] + step * 64;
      __builtin_amdgcn_global_load_lds(src, (lds_ptr_t)(st + W2_WH + (256 * i + 64 * wave) * 16), 16, 0, 0);
    }
    {
      const char* src = pwl + step * 32;
      __builtin_amdgcn_global_load_lds(src, (lds_ptr_t)(st + W2_WL + 64 * wave * 16), 16, 0, 0);
    }
    if (wave == 0) {
      const char* src = psc + static_cast<int64_t>(step / g.bpb) * g.Npad * 4;
      __builtin_amdgcn_global_load_lds(src, (lds_ptr_t)(st + W2_SC), 16, 0, 0);
    }
  };

  issue(0);
  if (steps > 1) issue(1);

  float f[2][2][16];
  v16i acc_lo[2][2], acc_hi[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int q = 0; q < 16; ++q) f[i][j][q] = 0.0f;
  const v16i zero = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};

  for (int kt = 0; kt < steps; ++kt) {
    // step kt has landed when at most the copies of step kt+1 are outstanding (wave 0 issues one more per step)
    if (kt + 1 < steps) {
      if (wave == 0) w2_wait<6>();
      else w2_wait<5>();
    } else {
      w2_wait<0>();
    }
    // the stage of step kt-1 is free now (every wave has passed its fold / its last read of it before this barrier)
    if (kt + 2 < steps) issue(kt + 2);
    const char* st = lds + (kt % W2_NS) * W2_STAGE;
    v4i a[2][2], wh[2][2];
    v4u wl[2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int s2 = 0; s2 < 2; ++s2) a[i][s2] = *reinterpret_cast<const v4i*>(st + W2_A + w2_off4(64 * wm + 32 * i + r, 2 * h + s2));
#pragma unroll
    for (int j = 0; j < 2; ++j) {
#pragma unroll
      for (int s2 = 0; s2 < 2; ++s2) wh[j][s2] = *reinterpret_cast<const v4i*>(st + W2_WH + w2_off4(64 * wn + 32 * j + r, 2 * h + s2));
      wl[j] = *reinterpret_cast<const v4u*>(st + W2_WL + w2_off2(64 * wn + 32 * j + r, h));
    }
    const bool first = kt % g.bpb == 0;  // first step of a bank: its products start from zero (no registers to clear)
#pragma unroll
    for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const v4i wlo = widen_half(wl[j], s2);
#pragma unroll
        for (int i = 0; i < 2; ++i) {
          if (s2 == 0 && first) {
            acc_lo[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[i][s2], wlo, zero, 0, 0, 0);
            acc_hi[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[i][s2], wh[j][s2], zero, 0, 0, 0);
          } else {
            acc_lo[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[i][s2], wlo, acc_lo[i][j], 0, 0, 0);
            acc_hi[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[i][s2], wh[j][s2], acc_hi[i][j], 0, 0, 0);
          }
        }
      }
    if ((kt + 1) % g.bpb == 0) {  // last step of a bank: fold its two integer tiles into the fp32 accumulators
      const float* sc = reinterpret_cast<const float*>(st + W2_SC);
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const float sl = sc[64 * wn + 32 * j + r], sh = sc[128 + 64 * wn + 32 * j + r];
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
          for (int q = 0; q < 16; ++q) {
            // the widened low weights carry a factor 16, which the transposed low scales carry inverted (sl is
            // s_lo / 16: float(16 a) * (s / 16) is float(a) * s bit for bit while s / 16 is a normal number)
            float t = __fmul_rn(static_cast<float>(acc_lo[i][j][q]), sl);
            t = __fmaf_rn(static_cast<float>(acc_hi[i][j][q]), sh, t);
            f[i][j][q] = __fadd_rn(f[i][j][q], t);
          }
      }
    }
  }

  // ---- epilogue: y = f * s_a[m] ----
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int q = 0; q < 16; ++q) {
      const int m = m0 + 64 * wm + 32 * i + 8 * (q >> 2) + 4 * h + (q & 3);
      if (m < g.M) {
        const float sa = g.a_scale[m];
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          const int n = n0 + 64 * wn + 32 * j + r;
          if (n < g.N) {
            const float y = __fmul_rn(f[i][j][q], sa);
            const int64_t o = static_cast<int64_t>(m) * g.ldy + n;
            if (g.out_bf16) reinterpret_cast<uint16_t*>(g.y)[o] = f32_to_bf16_rne(y);
            else reinterpret_cast<float*>(g.y)[o] = y;
          }
        }
      }
    }
}

// scales [N, G] -> [G, Npad] (zero beyond N), so that a bank's scales of 128 consecutive channels are contiguous;
// the low scales are stored divided by 16 (exact for every scale above 2^-122)
__global__ __launch_bounds__(256) void wsq_scales_t_kernel(int N, int G, int Npad, const float* __restrict__ s_lo,
                                                           const float* __restrict__ s_hi, float* __restrict__ lo_t,
                                                           float* __restrict__ hi_t) {
  const int64_t idx = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
  if (idx >= static_cast<int64_t>(G) * Npad) return;
  const int gq = static_cast<int>(idx / Npad), n = static_cast<int>(idx - static_cast<int64_t>(gq) * Npad);
  lo_t[idx] = n < N ? s_lo[static_cast<int64_t>(n) * G + gq] * 0.0625f : 0.0f;  // / 16: see the fold of wsq_gemm2_kernel
  hi_t[idx] = n < N ? s_hi[static_cast<int64_t>(n) * G + gq] : 0.0f;
}

}  // namespace

int init_wsq_kernels() {
  return hipFuncSetAttribute(reinterpret_cast<const void*>(wsq_gemm2_kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                             W2_NS * W2_STAGE) == hipSuccess
             ? SQ_OK
             : SQ_ERR_LAUNCH;
}

int launch_wsq_encode(const sq_params& p, const uint16_t* w, int64_t ldw, const float* hinv, const sq_wsq& out, hipStream_t st) {
  const int G = p.K / p.bank;
  const int64_t groups = static_cast<int64_t>(p.N) * G;
  const unsigned blocks = static_cast<unsigned>((groups + 63) / 64);
  const float q_hi = code_max(p.h_high, 8), q_lo = code_max(p.h_low, 4);
  const int v_mask = -(1 << ((p.h_low ? p.h_low : 4) - 1));
  if (p.bank == 64)
    hipLaunchKernelGGL(wsq_encode_kernel<64>, dim3(blocks), dim3(64), 0, st, w, ldw, p.N, p.K, p.topk, hinv, q_hi, q_lo, v_mask,
                       out.lo, out.hi_val, out.scale_lo, out.scale_hi);
  else
    hipLaunchKernelGGL(wsq_encode_kernel<128>, dim3(blocks), dim3(64), 0, st, w, ldw, p.N, p.K, p.topk, hinv, q_hi, q_lo, v_mask,
                       out.lo, out.hi_val, out.scale_lo, out.scale_hi);
  return hipGetLastError() == hipSuccess ? SQ_OK : SQ_ERR_LAUNCH;
}

int launch_wsq_prepack(const sq_params& p, const sq_wsq& w, uint8_t* lo_clean, int8_t* hi_dense, float* s_lo_t, float* s_hi_t,
                       hipStream_t st) {
  const int64_t total = static_cast<int64_t>(p.N) * (p.K / 32);
  const int vm = (-(1 << ((p.h_low ? p.h_low : 4) - 1))) & 0xF;
  hipLaunchKernelGGL(wsq_prepack_kernel, dim3(static_cast<unsigned>((total + 255) / 256)), dim3(256), 0, st, p.N, p.K, p.bank,
                     p.topk, vm, w.lo, w.hi_val, lo_clean, hi_dense);
  if (hipGetLastError() != hipSuccess) return SQ_ERR_LAUNCH;
  const int G = p.K / p.bank, Npad = (p.N + 127) / 128 * 128;
  const int64_t n_sc = static_cast<int64_t>(G) * Npad;
  hipLaunchKernelGGL(wsq_scales_t_kernel, dim3(static_cast<unsigned>((n_sc + 255) / 256)), dim3(256), 0, st, p.N, G, Npad,
                     w.scale_lo, w.scale_hi, s_lo_t, s_hi_t);
  return hipGetLastError() == hipSuccess ? SQ_OK : SQ_ERR_LAUNCH;
}

int launch_quantize_act(const sq_params& p, const uint16_t* x, int64_t ldx, int bits, int8_t* a8, float* a_scale, hipStream_t st) {
  hipLaunchKernelGGL(quantize_act_kernel, dim3(p.M), dim3(256), 0, st, x, ldx, p.K, code_max(bits, 8), a8, a_scale);
  return hipGetLastError() == hipSuccess ? SQ_OK : SQ_ERR_LAUNCH;
}

int launch_wsq_gemm(const sq_params& p, const int8_t* a8, const float* a_scale, const sq_wsq& w, const uint8_t* lo_clean,
                    const int8_t* hi_dense, const float* s_lo_t, const float* s_hi_t, void* y, int64_t ldy,
                    int32_t* acc_lo_dbg, int32_t* acc_hi_dbg, hipStream_t st) {
  if (!acc_lo_dbg && !acc_hi_dbg && p.M > 64) {  // the throughput kernel (the small kernel below also dumps the per-bank products)
    Wsq2Args a;
    a.M = p.M;
    a.N = p.N;
    a.K = p.K;
    a.G = p.K / p.bank;
    a.Npad = (p.N + 127) / 128 * 128;
    a.bpb = p.bank / 64;
    a.a8 = a8;
    a.a_scale = a_scale;
    a.lo_clean = lo_clean;
    a.hi_dense = hi_dense;
    a.s_lo_t = s_lo_t;
    a.s_hi_t = s_hi_t;
    a.y = y;
    a.ldy = ldy;
    a.out_bf16 = p.out_dtype == SQ_OUT_BF16;
    hipLaunchKernelGGL(wsq_gemm2_kernel, dim3((p.N + 127) / 128, (p.M + 127) / 128), dim3(256), W2_NS * W2_STAGE, st, a);
    return hipGetLastError() == hipSuccess ? SQ_OK : SQ_ERR_LAUNCH;
  }
  WsqGemmArgs g;
  g.M = p.M;
  g.N = p.N;
  g.K = p.K;
  g.G = p.K / p.bank;
  g.a8 = a8;
  g.a_scale = a_scale;
  g.lo_clean = lo_clean;
  g.hi_dense = hi_dense;
  g.s_lo = w.scale_lo;
  g.s_hi = w.scale_hi;
  g.y = y;
  g.ldy = ldy;
  g.out_bf16 = p.out_dtype == SQ_OUT_BF16;
  g.acc_lo_dbg = acc_lo_dbg;
  g.acc_hi_dbg = acc_hi_dbg;
  const dim3 grid((p.N + 63) / 64, (p.M + 63) / 64);
  if (p.bank == 64) hipLaunchKernelGGL(wsq_gemm_kernel<64>, grid, dim3(256), 0, st, g);
  else hipLaunchKernelGGL(wsq_gemm_kernel<128>, grid, dim3(256), 0, st, g);
  return hipGetLastError() == hipSuccess ? SQ_OK : SQ_ERR_LAUNCH;
}

}  // namespace sq
