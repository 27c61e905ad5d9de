// sq_gemm: the two integer products of the SQ-format linear layer (Section 3.3) on the INT8
// matrix cores of gfx950, with the dequantising epilogue fused.
//
// CDNA4 has no INT4 matrix instruction, so both products run on v_mfma_i32_32x32x32_i8.
// INT4 codes are widened on the way into LDS without sign extension: a nibble placed in the
// HIGH four bits of a byte is the signed byte 16*code, so
//     lo_bytes = (dword << 4) & 0xF0F0F0F0      (codes 0,2,4,6 of the 8 in a dword)
//     hi_bytes =  dword       & 0xF0F0F0F0      (codes 1,3,5,7)
// and the accumulators come out as exact multiples (256x when both operands are widened this
// way, 16x when only the weights are), shifted back in the epilogue.  Integer addition is
// order-independent, so the products are bit-exact whatever the K order; both operands simply
// use the same one: inside a group of 32 channels, the 16 even channels then the 16 odd ones.
//
// LDS holds operands in matrix-instruction order: for every (32-row block, 32-channel group) a
// 1 KB block whose 16-byte chunk c belongs to lane c of the wave that will issue the MFMA
// (lane = row % 32 + 32 * half).  A wave's operand read is then one contiguous 1 KB ds_read_b128.
#include "sq_device.h"

namespace sq {
namespace {

constexpr int BM = 128;   // tokens per workgroup tile
constexpr int BN = 128;   // output channels per workgroup tile
constexpr int KS = 128;   // channels per K step
constexpr int NT = 256;   // threads: 4 waves as 2 (M) x 2 (N), each 64 tokens x 64 channels
constexpr int KG = KS / 32;
constexpr int ROT = 4;    // per-group rotation of the chunks inside a 1 KB block (spreads the writers over banks)
constexpr int OPER_BYTES = (BM / 32) * KG * 1024;  // one operand tile of one stage: 16 KB
constexpr int STAGE_BYTES = 3 * OPER_BYTES;        // A_lo | A_hi | B
constexpr int LDS_BYTES = 2 * STAGE_BYTES;
static_assert(BM == BN, "operand tiles share one size");

__device__ __forceinline__ int frag_offset(int row, int kg, int half) {
  return (((row >> 5) * KG + kg) << 10) + ((((row & 31) + 32 * half + ROT * kg) & 63) << 4);
}

typedef unsigned int v4u __attribute__((ext_vector_type(4)));

struct Staging {
  v4u a_lo[2];
  v4u a_hi[4];
  v4u b[2];
};

// Operand sources of one K loop.  Row pointers are already clamped to valid rows.
template <bool LO, bool HI>
struct Loader {
  const uint8_t* a_lo;   // + row * lda_lo
  int64_t lda_lo;
  const int8_t* a_hi;
  int64_t lda_hi;
  const uint8_t* b;
  int64_t ldb;
  int kext;              // channels in this loop (multiple of 32)
  int m0, n0, M, N;

  // Loads are unconditional from an address clamped into the operand (rows past the edge repeat the
  // last row and are never stored; channel groups past kext read the last group and are zeroed).
  __device__ __forceinline__ void load(Staging& s, int k0) const {
    const int tid = threadIdx.x;
    const v4u zero = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int c = tid + NT * i;
      const int row = c >> 2, kg = c & 3;
      const int k = k0 + kg * 32;
      const bool ok = k < kext;
      const int kc = ok ? k : kext - 32;
      if (LO) {
        const int m = min(m0 + row, M - 1);
        const v4u v = *reinterpret_cast<const v4u*>(a_lo + m * lda_lo + (kc >> 1));
        s.a_lo[i] = ok ? v : zero;
      }
      const int n = min(n0 + row, N - 1);
      const v4u v = *reinterpret_cast<const v4u*>(b + n * ldb + (kc >> 1));
      s.b[i] = ok ? v : zero;
    }
    if (HI) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int c = tid + NT * i;
        const int row = c >> 3, ch = c & 7;
        const int k = k0 + ch * 16;
        const bool ok = k < kext;
        const int kc = ok ? k : kext - 16;
        const int m = min(m0 + row, M - 1);
        const v4u v = *reinterpret_cast<const v4u*>(a_hi + m * lda_hi + kc);
        s.a_hi[i] = ok ? v : zero;
      }
    }
  }

  __device__ __forceinline__ void store(const Staging& s, char* stage) const {
    const int tid = threadIdx.x;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int c = tid + NT * i;
      const int row = c >> 2, kg = c & 3;
      if (LO) {
        const v4u v = s.a_lo[i];
        *reinterpret_cast<v4u*>(stage + frag_offset(row, kg, 0)) = (v << 4) & 0xF0F0F0F0u;
        *reinterpret_cast<v4u*>(stage + frag_offset(row, kg, 1)) = v & 0xF0F0F0F0u;
      }
      const v4u v = s.b[i];
      *reinterpret_cast<v4u*>(stage + 2 * OPER_BYTES + frag_offset(row, kg, 0)) = (v << 4) & 0xF0F0F0F0u;
      *reinterpret_cast<v4u*>(stage + 2 * OPER_BYTES + frag_offset(row, kg, 1)) = v & 0xF0F0F0F0u;
    }
    if (HI) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int c = tid + NT * i;
        const int row = c >> 3, ch = c & 7;
        *reinterpret_cast<v4u*>(stage + OPER_BYTES + frag_offset(row, ch >> 1, ch & 1)) = s.a_hi[i];
      }
    }
  }
};

template <bool LO, bool HI>
__device__ __forceinline__ void compute_stage(const char* stage, int wm, int wn, int lane, v16i (&acc_lo)[2][2],
                                              v16i (&acc_hi)[2][2]) {
#pragma unroll
  for (int kg = 0; kg < KG; ++kg) {
    const int chunk = ((lane + ROT * kg) & 63) << 4;
    v4i bf[2], alo[2], ahi[2];
#pragma unroll
    for (int j = 0; j < 2; ++j)
      bf[j] = *reinterpret_cast<const v4i*>(stage + 2 * OPER_BYTES + (((wn * 2 + j) * KG + kg) << 10) + chunk);
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      if (LO) alo[i] = *reinterpret_cast<const v4i*>(stage + (((wm * 2 + i) * KG + kg) << 10) + chunk);
      if (HI) ahi[i] = *reinterpret_cast<const v4i*>(stage + OPER_BYTES + (((wm * 2 + i) * KG + kg) << 10) + chunk);
    }
#pragma unroll
    for (int i = 0; i < 2; ++i) {
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        if (LO) acc_lo[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(alo[i], bf[j], acc_lo[i][j], 0, 0, 0);
        if (HI) acc_hi[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(ahi[i], bf[j], acc_hi[i][j], 0, 0, 0);
      }
    }
  }
}

template <bool LO, bool HI>
__device__ __forceinline__ void k_loop(const Loader<LO, HI>& ld, char* lds, int wm, int wn, int lane,
                                       v16i (&acc_lo)[2][2], v16i (&acc_hi)[2][2]) {
  const int steps = (ld.kext + KS - 1) / KS;
  Staging s;
  ld.load(s, 0);
  ld.store(s, lds);
  __syncthreads();
  for (int kt = 0; kt < steps; ++kt) {
    char* cur = lds + (kt & 1) * STAGE_BYTES;
    char* nxt = lds + ((kt + 1) & 1) * STAGE_BYTES;
    const bool more = (kt + 1) < steps;
    if (more) ld.load(s, (kt + 1) * KS);
    compute_stage<LO, HI>(cur, wm, wn, lane, acc_lo, acc_hi);
    if (more) ld.store(s, nxt);
    __syncthreads();
  }
}

__device__ __forceinline__ uint16_t bf16_rne(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return static_cast<uint16_t>(u >> 16);
}

// MODE 0: dynamic (low + zero-padded high in one K loop); 1: static (low loop over K, then the
// compact high loop over K_hi); 2: high loop only (plain W4A8 reference).
template <int MODE>
__global__ __launch_bounds__(NT) void gemm_kernel(GemmArgs g) {
  extern __shared__ __attribute__((aligned(16))) char lds[];
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;

  v16i acc_lo[2][2], acc_hi[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        acc_lo[i][j][r] = 0;
        acc_hi[i][j][r] = 0;
      }

  if (MODE == 0) {
    Loader<true, true> ld{g.a_lo, g.K / 2, g.a_hi_dense, g.K, g.wq, g.K / 2, g.K, m0, n0, g.M, g.N};
    k_loop<true, true>(ld, lds, wm, wn, lane, acc_lo, acc_hi);
  } else if (MODE == 1) {
    Loader<true, false> l1{g.a_lo, g.K / 2, nullptr, 0, g.wq, g.K / 2, g.K, m0, n0, g.M, g.N};
    k_loop<true, false>(l1, lds, wm, wn, lane, acc_lo, acc_hi);
    Loader<false, true> l2{nullptr, 0, g.a_hi_compact, g.lda_hi_compact, g.w_hi, g.K_hi / 2, g.K_hi, m0, n0, g.M, g.N};
    k_loop<false, true>(l2, lds, wm, wn, lane, acc_lo, acc_hi);
  } else {
    Loader<false, true> l2{nullptr, 0, g.a_hi_compact, g.lda_hi_compact, g.w_hi, g.K_hi / 2, g.K_hi, m0, n0, g.M, g.N};
    k_loop<false, true>(l2, lds, wm, wn, lane, acc_lo, acc_hi);
  }

  // Epilogue: Y = (acc_lo * s_lo[m] + acc_hi * s_hi[m]) * s_w[n], in this order, in fp32.
  // Accumulator register r of lane l of a 32x32 tile is row 8*(r/4) + 4*(l/32) + r%4, column l%32.
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int n = n0 + wn * 64 + j * 32 + (lane & 31);
    const bool n_ok = n < g.N;
    const float sw = n_ok ? g.s_w[n] : 0.0f;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int m = m0 + wm * 64 + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
        if (n_ok && m < g.M) {
          const int lo = acc_lo[i][j][r] >> 8;  // exact: both operands carried a factor 16
          const int hi = acc_hi[i][j][r] >> 4;  // exact: the weights carried a factor 16
          float t = g.s_lo ? __fmul_rn(static_cast<float>(lo), g.s_lo[m]) : 0.0f;
          t = __fmaf_rn(static_cast<float>(hi), g.s_hi[m], t);
          const float y = __fmul_rn(t, sw);
          const int64_t o = static_cast<int64_t>(m) * g.ldy + n;
          if (g.out_bf16) reinterpret_cast<uint16_t*>(g.y)[o] = bf16_rne(y);
          else reinterpret_cast<float*>(g.y)[o] = y;
          if (g.acc_lo_dbg) g.acc_lo_dbg[static_cast<int64_t>(m) * g.N + n] = lo;
          if (g.acc_hi_dbg) g.acc_hi_dbg[static_cast<int64_t>(m) * g.N + n] = hi;
        }
      }
    }
  }
}

template <int MODE>
int launch_mode(const GemmArgs& g, hipStream_t st) {
  // The kernel needs more dynamic LDS than the default limit; raising it is per device and
  // idempotent, so a race between threads only repeats the call.
  static bool attr_done[64] = {};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return SQ_ERR_LAUNCH;
  if (!attr_done[dev]) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(gemm_kernel<MODE>), hipFuncAttributeMaxDynamicSharedMemorySize,
                            LDS_BYTES) != hipSuccess)
      return SQ_ERR_LAUNCH;
    attr_done[dev] = true;
  }
  dim3 grid((g.N + BN - 1) / BN, (g.M + BM - 1) / BM);
  hipLaunchKernelGGL(gemm_kernel<MODE>, grid, dim3(NT), LDS_BYTES, st, g);
  return hipGetLastError() == hipSuccess ? SQ_OK : SQ_ERR_LAUNCH;
}

}  // namespace

int launch_gemm(const GemmArgs& g, hipStream_t st) {
  if (g.a_lo && g.a_hi_dense) return launch_mode<0>(g, st);
  if (g.a_lo && g.a_hi_compact) return launch_mode<1>(g, st);
  if (!g.a_lo && g.a_hi_compact) return launch_mode<2>(g, st);
  return SQ_ERR_UNSUPPORTED;
}

}  // namespace sq
