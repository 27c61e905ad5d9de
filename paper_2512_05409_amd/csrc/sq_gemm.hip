// sq_gemm: the two integer products of the SQ-format linear layer (Section 3.3) on the INT8
// matrix cores of gfx950, with the dequantising epilogue fused.
//
// CDNA4 has no INT4 matrix instruction, so both products run on v_mfma_i32_32x32x32_i8.
// INT4 codes stay packed (two per byte) from HBM through LDS and are widened in registers just
// before the matrix instruction, without sign extension: a nibble placed in the HIGH four bits
// of a byte is the signed byte 16*code, so for a dword p of eight codes
//     (p << 4) & 0xF0F0F0F0   are codes 0,2,4,6 (times 16)      p & 0xF0F0F0F0   are codes 1,3,5,7
// and the accumulators come out as exact multiples (256x when both operands are widened this
// way, 16x when only the weights are), shifted back in the epilogue.  Integer addition is
// order-independent, so the products are bit-exact whatever the K order, as long as both operands
// use the same one.  The order used: a 16-byte chunk of packed codes (32 channels) feeds two
// consecutive matrix instructions; instruction s (0/1) takes dwords 2s, 2s+1 of the chunk as
// [evens of dword 2s | odds of dword 2s | evens of dword 2s+1 | odds of dword 2s+1].  The INT8
// image of the high part is stored in exactly that byte order (see sq_act::hi_dense).
//
// Work split: a workgroup of 4 waves computes 128 tokens x 256 output channels; a wave computes
// 64 tokens x 128 channels for BOTH products (2 x 2x4 tiles of 32x32, 256 accumulator registers).
// A K step of 128 channels is staged through LDS, double buffered.  LDS rows are row-major with
// the 16-byte chunk index XOR-swizzled by the row, which keeps both the staging stores (4 or 8
// consecutive lanes per row) and the operand reads (32 consecutive rows per half wave) conflict-free.
#include "sq_device.h"

namespace sq {
namespace {

typedef unsigned int v4u __attribute__((ext_vector_type(4)));

constexpr int KS = 128;  // channels per K step
constexpr int NT = 256;  // threads per workgroup

template <int BM_, int BN_>
struct Tile {
  static constexpr int BM = BM_;              // tokens per workgroup
  static constexpr int BN = BN_;              // output channels per workgroup
  static constexpr int WM = BM / 2;           // tokens per wave (waves are 2 x 2)
  static constexpr int WN = BN / 2;           // channels per wave
  static constexpr int TI = WM / 32;          // 32-row tiles per wave along M
  static constexpr int TJ = WN / 32;          // along N
  static constexpr int A_LO = 0;              // [BM][64 B]   packed INT4
  static constexpr int A_HI = BM * 64;        // [BM][128 B]  INT8
  static constexpr int B_OFF = A_HI + BM * 128;  // [BN][64 B] packed INT4
  static constexpr int STAGE = B_OFF + BN * 64;
  static constexpr int LDS_BYTES = 2 * STAGE;
};

// Byte offset of 16-byte chunk c of a row inside an operand tile.
__device__ __forceinline__ int off4(int row, int c) { return (row << 6) + (((c ^ (row >> 2)) & 3) << 4); }   // 4 chunks / row
__device__ __forceinline__ int off8(int row, int c) { return (row << 7) + (((c ^ (row >> 1)) & 7) << 4); }   // 8 chunks / row

template <typename T>
struct Staging {
  v4u a_lo[T::BM * 4 / NT];
  v4u a_hi[T::BM * 8 / NT];
  v4u b[T::BN * 4 / NT];
};

// Operand sources of one K loop.  LO: the packed low part is an operand; HI: an INT8 operand
// (the zero-padded image of the high part, or the compact high codes) is.
template <typename T, bool LO, bool HI>
struct Loader {
  const uint8_t* a_lo;
  int64_t lda_lo;
  const int8_t* a_hi;
  int64_t lda_hi;
  const uint8_t* b;
  int64_t ldb;
  int kext;  // channels in this loop (multiple of 32)
  int m0, n0, M, N;

  // Loads are unconditional from an address clamped into the operand: rows past the edge repeat the
  // last row and are never stored; chunks past kext (only possible in the last, partial K step) read
  // the last chunk and are zeroed when they are written to LDS.
  __device__ __forceinline__ void load(Staging<T>& s, int k0) const {
    const int tid = threadIdx.x;
    if (LO) {
#pragma unroll
      for (int i = 0; i < T::BM * 4 / NT; ++i) {
        const int idx = tid + NT * i, row = idx >> 2, c = idx & 3;
        const int k = min(k0 + c * 32, kext - 32);
        const int m = min(m0 + row, M - 1);
        s.a_lo[i] = *reinterpret_cast<const v4u*>(a_lo + m * lda_lo + (k >> 1));
      }
    }
    if (HI) {
#pragma unroll
      for (int i = 0; i < T::BM * 8 / NT; ++i) {
        const int idx = tid + NT * i, row = idx >> 3, c = idx & 7;
        const int k = min(k0 + c * 16, kext - 16);
        const int m = min(m0 + row, M - 1);
        s.a_hi[i] = *reinterpret_cast<const v4u*>(a_hi + m * lda_hi + k);
      }
    }
#pragma unroll
    for (int i = 0; i < T::BN * 4 / NT; ++i) {
      const int idx = tid + NT * i, row = idx >> 2, c = idx & 3;
      const int k = min(k0 + c * 32, kext - 32);
      const int n = min(n0 + row, N - 1);
      s.b[i] = *reinterpret_cast<const v4u*>(b + n * ldb + (k >> 1));
    }
  }

  __device__ __forceinline__ void store(Staging<T>& s, char* stage, int k0) const {
    const int tid = threadIdx.x;
    if (k0 + KS > kext) {  // partial K step (uniform branch): zero what lies past the end
      const v4u zero = {0u, 0u, 0u, 0u};
#pragma unroll
      for (int i = 0; i < T::BM * 4 / NT; ++i)
        if (LO && k0 + ((tid + NT * i) & 3) * 32 >= kext) s.a_lo[i] = zero;
#pragma unroll
      for (int i = 0; i < T::BM * 8 / NT; ++i)
        if (HI && k0 + ((tid + NT * i) & 7) * 16 >= kext) s.a_hi[i] = zero;
#pragma unroll
      for (int i = 0; i < T::BN * 4 / NT; ++i)
        if (k0 + ((tid + NT * i) & 3) * 32 >= kext) s.b[i] = zero;
    }
    if (LO) {
#pragma unroll
      for (int i = 0; i < T::BM * 4 / NT; ++i) {
        const int idx = tid + NT * i;
        *reinterpret_cast<v4u*>(stage + T::A_LO + off4(idx >> 2, idx & 3)) = s.a_lo[i];
      }
    }
    if (HI) {
#pragma unroll
      for (int i = 0; i < T::BM * 8 / NT; ++i) {
        const int idx = tid + NT * i;
        *reinterpret_cast<v4u*>(stage + T::A_HI + off8(idx >> 3, idx & 7)) = s.a_hi[i];
      }
    }
#pragma unroll
    for (int i = 0; i < T::BN * 4 / NT; ++i) {
      const int idx = tid + NT * i;
      *reinterpret_cast<v4u*>(stage + T::B_OFF + off4(idx >> 2, idx & 3)) = s.b[i];
    }
  }
};

// One packed chunk (32 INT4 codes) -> the INT8 operands of two consecutive matrix instructions.
__device__ __forceinline__ void widen(const v4u p, v4i& s0, v4i& s1) {
  const v4u e = (p << 4) & 0xF0F0F0F0u;
  const v4u o = p & 0xF0F0F0F0u;
  s0 = v4i{static_cast<int>(e[0]), static_cast<int>(o[0]), static_cast<int>(e[1]), static_cast<int>(o[1])};
  s1 = v4i{static_cast<int>(e[2]), static_cast<int>(o[2]), static_cast<int>(e[3]), static_cast<int>(o[3])};
}

template <typename T, bool LO, bool HI>
__device__ __forceinline__ void compute_stage(const char* stage, int wm, int wn, int lane, v16i (&acc_lo)[T::TI][T::TJ],
                                              v16i (&acc_hi)[T::TI][T::TJ]) {
  const int r = lane & 31, h = lane >> 5;
#pragma unroll
  for (int g = 0; g < KS / 64; ++g) {
    v4i bw[T::TJ][2], alo[T::TI][2], ahi[T::TI][2];
#pragma unroll
    for (int j = 0; j < T::TJ; ++j) {
      const v4u p = *reinterpret_cast<const v4u*>(stage + T::B_OFF + off4(wn * T::WN + j * 32 + r, 2 * g + h));
      widen(p, bw[j][0], bw[j][1]);
    }
#pragma unroll
    for (int i = 0; i < T::TI; ++i) {
      const int row = wm * T::WM + i * 32 + r;
      if (LO) {
        const v4u p = *reinterpret_cast<const v4u*>(stage + T::A_LO + off4(row, 2 * g + h));
        widen(p, alo[i][0], alo[i][1]);
      }
      if (HI) {
        ahi[i][0] = *reinterpret_cast<const v4i*>(stage + T::A_HI + off8(row, 4 * g + 2 * h));
        ahi[i][1] = *reinterpret_cast<const v4i*>(stage + T::A_HI + off8(row, 4 * g + 2 * h + 1));
      }
    }
#pragma unroll
    for (int s = 0; s < 2; ++s) {
#pragma unroll
      for (int i = 0; i < T::TI; ++i) {
#pragma unroll
        for (int j = 0; j < T::TJ; ++j) {
          if (LO) acc_lo[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(alo[i][s], bw[j][s], acc_lo[i][j], 0, 0, 0);
          if (HI) acc_hi[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(ahi[i][s], bw[j][s], acc_hi[i][j], 0, 0, 0);
        }
      }
    }
  }
}

template <typename T, bool LO, bool HI>
__device__ __forceinline__ void k_loop(const Loader<T, LO, HI>& ld, char* lds, int wm, int wn, int lane,
                                       v16i (&acc_lo)[T::TI][T::TJ], v16i (&acc_hi)[T::TI][T::TJ]) {
  const int steps = (ld.kext + KS - 1) / KS;
  Staging<T> s;
  ld.load(s, 0);
  ld.store(s, lds, 0);
  __syncthreads();
  for (int kt = 0; kt < steps; ++kt) {
    char* cur = lds + (kt & 1) * T::STAGE;
    char* nxt = lds + ((kt + 1) & 1) * T::STAGE;
    const bool more = (kt + 1) < steps;
    if (more) ld.load(s, (kt + 1) * KS);
    compute_stage<T, LO, HI>(cur, wm, wn, lane, acc_lo, acc_hi);
    if (more) ld.store(s, nxt, (kt + 1) * KS);
    __syncthreads();
  }
}

__device__ __forceinline__ uint16_t bf16_rne(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return static_cast<uint16_t>(u >> 16);
}

// Maps the linear workgroup id to a tile so that (a) the workgroups resident on one XCD at a time
// (ids congruent mod 8 go to the same XCD) cover a compact 4 x 8 patch of tiles and share operand
// tiles in that XCD's L2, and (b) every XCD walks its own contiguous range of the tile order.
__device__ __forceinline__ void tile_of_block(int tiles_m, int tiles_n, int& tm, int& tn) {
  const int total = tiles_m * tiles_n;
  const int id = blockIdx.x;
  const int per_xcd = (total + 7) / 8;
  const int lin = (id & 7) * per_xcd + (id >> 3);  // position in the tile order
  if (lin >= total) {  // the grid is rounded up to a multiple of 8: the overhang does nothing
    tm = -1;
    tn = -1;
    return;
  }
  constexpr int BAND = 4;  // tile rows walked together
  const int band = lin / (BAND * tiles_n);
  const int within = lin - band * (BAND * tiles_n);
  const int rows_here = min(BAND, tiles_m - band * BAND);
  tn = within / rows_here;
  tm = band * BAND + within - tn * rows_here;
}

// Epilogue: Y = (acc_lo * s_lo[m] + acc_hi * s_hi[m]) * s_w[n], in this order, in fp32.
// Accumulator register r of lane l of a 32x32 tile is row 8*(r/4) + 4*(l/32) + r%4, column l%32, so a
// lane holds single elements of many rows.  The per-token scales of the workgroup's rows and the
// finished outputs go through LDS (free after the K loops): every wave transposes 32 rows x WN columns
// at a time and then stores 16 bytes per lane, whole row segments at once.
template <typename T, typename OutT>
__device__ __forceinline__ void epilogue_typed(const GemmArgs& g, char* lds, v16i (&acc_lo)[T::TI][T::TJ],
                                               v16i (&acc_hi)[T::TI][T::TJ], int m0, int n0, int wm, int wn, int wave,
                                               int lane) {
  constexpr int ESZ = sizeof(OutT);
  constexpr int ROW = T::WN * ESZ + 16;   // padded row of the transposition buffer (bytes)
  constexpr int PER16 = 16 / ESZ;         // outputs per 16-byte store
  constexpr int CHUNKS = T::WN / PER16;   // 16-byte chunks per row
  constexpr int ROWS_PER_PASS = 64 / CHUNKS;
  static_assert(1024 + 4 * 32 * ROW <= T::LDS_BYTES, "transposition buffers must fit in the stage memory");
  const int tid = threadIdx.x;
  float* sc = reinterpret_cast<float*>(lds);  // [0, BM): s_lo, [BM, 2 BM): s_hi   (BM <= 128)
  char* tb = lds + 1024 + wave * (32 * ROW);
  if (tid < T::BM) {
    const int m = min(m0 + tid, g.M - 1);
    sc[tid] = g.s_lo ? g.s_lo[m] : 0.0f;
    sc[T::BM + tid] = g.s_hi[m];
  }
  __syncthreads();
  float sw[T::TJ];
#pragma unroll
  for (int j = 0; j < T::TJ; ++j) {
    const int n = n0 + wn * T::WN + j * 32 + (lane & 31);
    sw[j] = n < g.N ? g.s_w[n] : 0.0f;
  }
  const bool vec_ok = (g.ldy % PER16) == 0;  // rows of Y stay 16-byte aligned
  OutT* yout = reinterpret_cast<OutT*>(g.y);
#pragma unroll
  for (int i = 0; i < T::TI; ++i) {
#pragma unroll
    for (int rq = 0; rq < 4; ++rq) {
      const int rl0 = 8 * rq + 4 * (lane >> 5);  // 4 consecutive rows of the 32: registers 4 rq + e
      const float4 slo4 = *reinterpret_cast<const float4*>(sc + wm * T::WM + i * 32 + rl0);
      const float4 shi4 = *reinterpret_cast<const float4*>(sc + T::BM + wm * T::WM + i * 32 + rl0);
      const float slo[4] = {slo4.x, slo4.y, slo4.z, slo4.w};
      const float shi[4] = {shi4.x, shi4.y, shi4.z, shi4.w};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
#pragma unroll
        for (int j = 0; j < T::TJ; ++j) {
          const int lo = acc_lo[i][j][4 * rq + e] >> 8;  // exact: both operands carried a factor 16
          const int hi = acc_hi[i][j][4 * rq + e] >> 4;  // exact: the weights carried a factor 16
          float t = __fmul_rn(static_cast<float>(lo), slo[e]);
          t = __fmaf_rn(static_cast<float>(hi), shi[e], t);
          const float y = __fmul_rn(t, sw[j]);
          OutT* dst = reinterpret_cast<OutT*>(tb + (rl0 + e) * ROW) + j * 32 + (lane & 31);
          if constexpr (ESZ == 2) *dst = bf16_rne(y);
          else *dst = y;
        }
      }
    }
    __syncthreads();
#pragma unroll
    for (int pass = 0; pass < 32 / ROWS_PER_PASS; ++pass) {
      const int rl = pass * ROWS_PER_PASS + lane / CHUNKS, ch = lane % CHUNKS;
      const int m = m0 + wm * T::WM + i * 32 + rl;
      const int n = n0 + wn * T::WN + ch * PER16;
      if (m < g.M && n < g.N) {
        OutT* dst = yout + static_cast<int64_t>(m) * g.ldy + n;
        if (vec_ok && n + PER16 <= g.N) {
          *reinterpret_cast<uint4*>(dst) = *reinterpret_cast<const uint4*>(tb + rl * ROW + ch * 16);
        } else {  // ragged right edge or unaligned rows: element by element, straight from LDS
          const OutT* src = reinterpret_cast<const OutT*>(tb + rl * ROW + ch * 16);
          for (int q = 0; q < PER16 && n + q < g.N; ++q) dst[q] = src[q];
        }
      }
    }
    __syncthreads();
  }
  if (g.acc_lo_dbg || g.acc_hi_dbg) {  // test hook: the exact accumulators, written element by element
#pragma unroll
    for (int i = 0; i < T::TI; ++i)
#pragma unroll
      for (int j = 0; j < T::TJ; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int m = m0 + wm * T::WM + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
          const int n = n0 + wn * T::WN + j * 32 + (lane & 31);
          if (m < g.M && n < g.N) {
            if (g.acc_lo_dbg) g.acc_lo_dbg[static_cast<int64_t>(m) * g.N + n] = acc_lo[i][j][r] >> 8;
            if (g.acc_hi_dbg) g.acc_hi_dbg[static_cast<int64_t>(m) * g.N + n] = acc_hi[i][j][r] >> 4;
          }
        }
  }
}

template <typename T>
__device__ __forceinline__ void epilogue(const GemmArgs& g, char* lds, v16i (&acc_lo)[T::TI][T::TJ],
                                         v16i (&acc_hi)[T::TI][T::TJ], int m0, int n0, int wm, int wn, int wave, int lane) {
  if (g.out_bf16) epilogue_typed<T, uint16_t>(g, lds, acc_lo, acc_hi, m0, n0, wm, wn, wave, lane);
  else epilogue_typed<T, float>(g, lds, acc_lo, acc_hi, m0, n0, wm, wn, wave, lane);
}

// MODE 0: dynamic (low + zero-padded high in one K loop); 1: static (low loop over K, then the
// compact high loop over K_hi); 2: high loop only (plain W4A8 reference).
template <typename T, int MODE>
__global__ __launch_bounds__(NT) void gemm_kernel(GemmArgs g) {
  extern __shared__ __attribute__((aligned(16))) char lds[];
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  int tm, tn;
  tile_of_block((g.M + T::BM - 1) / T::BM, (g.N + T::BN - 1) / T::BN, tm, tn);
  if (tm < 0) return;
  const int m0 = tm * T::BM, n0 = tn * T::BN;

  v16i acc_lo[T::TI][T::TJ], acc_hi[T::TI][T::TJ];
#pragma unroll
  for (int i = 0; i < T::TI; ++i)
#pragma unroll
    for (int j = 0; j < T::TJ; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        acc_lo[i][j][r] = 0;
        acc_hi[i][j][r] = 0;
      }

  if (MODE == 0) {
    Loader<T, true, true> ld{g.a_lo, g.K / 2, g.a_hi_dense, g.K, g.wq, g.K / 2, g.K, m0, n0, g.M, g.N};
    k_loop<T, true, true>(ld, lds, wm, wn, lane, acc_lo, acc_hi);
  } else if (MODE == 1) {
    Loader<T, true, false> l1{g.a_lo, g.K / 2, nullptr, 0, g.wq, g.K / 2, g.K, m0, n0, g.M, g.N};
    k_loop<T, true, false>(l1, lds, wm, wn, lane, acc_lo, acc_hi);
    Loader<T, false, true> l2{nullptr, 0, g.a_hi_compact, g.lda_hi_compact, g.w_hi, g.K_hi / 2, g.K_hi, m0, n0, g.M, g.N};
    k_loop<T, false, true>(l2, lds, wm, wn, lane, acc_lo, acc_hi);
  } else {
    Loader<T, false, true> l2{nullptr, 0, g.a_hi_compact, g.lda_hi_compact, g.w_hi, g.K_hi / 2, g.K_hi, m0, n0, g.M, g.N};
    k_loop<T, false, true>(l2, lds, wm, wn, lane, acc_lo, acc_hi);
  }

  epilogue<T>(g, lds, acc_lo, acc_hi, m0, n0, wm, wn, wave, lane);
}

template <typename T, int MODE>
int launch_mode(const GemmArgs& g, hipStream_t st) {
  // The kernel needs more dynamic LDS than the default limit; raising it is per device and
  // idempotent, so a race between threads only repeats the call.
  static bool attr_done[64] = {};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return SQ_ERR_LAUNCH;
  if (!attr_done[dev]) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(gemm_kernel<T, MODE>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, T::LDS_BYTES) != hipSuccess)
      return SQ_ERR_LAUNCH;
    attr_done[dev] = true;
  }
  const int tiles = ((g.N + T::BN - 1) / T::BN) * ((g.M + T::BM - 1) / T::BM);
  const int blocks = (tiles + 7) / 8 * 8;
  hipLaunchKernelGGL((gemm_kernel<T, MODE>), dim3(blocks), dim3(NT), T::LDS_BYTES, st, g);
  return hipGetLastError() == hipSuccess ? SQ_OK : SQ_ERR_LAUNCH;
}

}  // namespace

int launch_gemm(const GemmArgs& g, hipStream_t st) {
  typedef Tile<128, 256> Big;
  if (g.a_lo && g.a_hi_dense) return launch_mode<Big, 0>(g, st);
  if (g.a_lo && g.a_hi_compact) return launch_mode<Big, 1>(g, st);
  if (!g.a_lo && g.a_hi_compact) return launch_mode<Big, 2>(g, st);
  return SQ_ERR_UNSUPPORTED;
}

}  // namespace sq
