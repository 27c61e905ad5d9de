// sq_encode, static rule (Algorithm 2: the high-precision channels of every bank are fixed for all tokens by
// a calibrated channel mask), row-staged kernel for gfx950.
//
// With a static mask the selection costs nothing and the work is a gather: the paper's GPU path (Section 3.3)
// reorders the weights by the mask ahead of time so that at run time "only selection and gathering" is left on
// the activation side.  This kernel therefore writes, besides the format's own arrays, the activations in that
// reordered form: `lo_compact`, the low codes of the low channels only (K_lo = K - K_hi of them, ascending
// channel order), next to `hi_val`, the high codes of the high channels only -- the two operands of the two
// products, each contiguous, so that the low product runs over K_lo channels instead of K.
//
// A workgroup walks over token rows.  Per workgroup, once: two index tables in LDS, built from the mask:
// the channel of every compact low position and of every compact high position.  Per row: the row is copied
// from HBM into LDS by coalesced LDS-direct loads; the work is output-centric: every thread owns whole dwords
// of the outputs (8 low codes, 4 high codes, or 8 dense low codes), gathers their source values from the staged
// row through the tables into registers (taking the row maxima of both parts on the way), and once the scales
// are known quantises from the registers, so every store is coalesced and the staged row is free early: the
// next row's copy runs under the reduction, the quantisation and the stores of this one.
#include "sq_encode_common.h"

namespace sq {
namespace {

using namespace enc;

typedef __attribute__((address_space(3))) void* lds_ptr_t;
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef unsigned short u16x8 __attribute__((ext_vector_type(8)));
typedef unsigned short u16x4 __attribute__((ext_vector_type(4)));
typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));

// max of two pairs of 16-bit magnitudes, both halves in one instruction (v_pk_max_u16)
__device__ __forceinline__ uint32_t pk_max_u16(uint32_t a, uint32_t b) {
  return __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(u16x2, a), __builtin_bit_cast(u16x2, b)));
}

constexpr int NT = 256;

struct GatherArgs {
  const uint16_t* x;
  int64_t ldx;
  int M, K, B, kt, G;
  int K_hi, K_lo;
  const uint32_t* mask;   // [K/32]
  uint8_t* d_lo;          // [M, K/2] dense low codes, or null
  uint8_t* lo_compact;    // [M, K_lo/2], or null
  int8_t* hi_val;         // [M, K_hi]
  float* s_lo;
  float* s_hi;
  int row_bytes_padded;   // LDS bytes of the staged row (K * 2 rounded up to 4096)
  float q_hi, q_lo;       // largest code magnitudes of the two parts (127 and 7 for the 8/4 pair)
};

// MAXI: output dwords of each kind a thread owns at most (K / 8 / 256 rounded up).
template <int MAXI>
__global__ __launch_bounds__(NT) void encode_static_gather_kernel(GatherArgs a) {
  extern __shared__ __attribute__((aligned(16))) char lds[];
  __shared__ uint32_t amax_sh[2][2];
  char* row = lds;                                                                  // staged bf16 row
  uint16_t* src_lo = reinterpret_cast<uint16_t*>(lds + a.row_bytes_padded);         // [K_lo] channel of compact low position
  uint16_t* src_hi = src_lo + ((a.K_lo + 7) & ~7);                                  // [K_hi]
  uint32_t* mask_sh = reinterpret_cast<uint32_t*>(src_hi + ((a.K_hi + 7) & ~7));    // [K/32] the channel mask
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);

  // ---- once per workgroup: the mask and the two index tables ----
  for (int w = tid; w < a.K / 32; w += NT) mask_sh[w] = a.mask[w];
  if (tid < 4) amax_sh[tid >> 1][tid & 1] = 0;
  const int nlo = a.B - a.kt;
  for (int g = tid; g < a.G; g += NT) {
    int cl = 0, ch = 0;
    for (int i = 0; i < a.B; ++i) {
      const int j = g * a.B + i;
      const bool hi = (a.mask[j >> 5] >> (j & 31)) & 1u;
      if (hi) {
        if (ch < a.kt) src_hi[g * a.kt + ch] = static_cast<uint16_t>(j);  // a malformed mask cannot write out of range
        ++ch;
      } else {
        if (cl < nlo) src_lo[g * nlo + cl] = static_cast<uint16_t>(j);
        ++cl;
      }
    }
    for (; ch < a.kt; ++ch) src_hi[g * a.kt + ch] = static_cast<uint16_t>(g * a.B);
    for (; cl < nlo; ++cl) src_lo[g * nlo + cl] = static_cast<uint16_t>(g * a.B);
  }

  const int chunks = a.K / 8;                 // 16-byte pieces of a row
  const int n_copy = (chunks + NT - 1) / NT;  // copy instructions per thread and row
  const int n_lo = a.lo_compact ? a.K_lo / 8 : 0, n_hi = a.K_hi / 4, n_dense = a.d_lo ? chunks : 0;

  // thread t copies pieces t, t + 256, ... (1 KB of consecutive memory per wave instruction)
  auto stage_row = [&](int64_t m) {
    const char* xrow = reinterpret_cast<const char*>(a.x + m * a.ldx);
    for (int i = 0; i < n_copy; ++i) {
      int c = i * NT + tid;
      c = c < chunks ? c : chunks - 1;  // the tail re-reads the last piece (it lands in the padding)
      const char* src = xrow + c * 16;
      __builtin_amdgcn_global_load_lds(src, (lds_ptr_t)(row + (i * NT + wave * 64) * 16), 16, 0, 0);
    }
  };

  if (blockIdx.x < a.M) stage_row(blockIdx.x);
  int par = 0;
  for (int64_t m = blockIdx.x; m < a.M; m += gridDim.x, par ^= 1) {
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_waitcnt((0 & 15) | (7 << 4) | (15 << 8) | (0 << 14));  // vmcnt(0): the copy has landed
    __syncthreads();                                                           // barrier A
    if (tid < 2) amax_sh[par ^ 1][tid] = 0;  // the next row's maxima (last read before barrier A)

    // ---- gather: every thread fetches the source values of the output dwords it owns, packed two bf16 per
    // register, and takes the maxima of their magnitudes on the way ----
    // (Threads whose dword index is past the end gather the last dword again instead of being masked off:
    // without branches all the gathers of a thread are in flight together and it waits once.)
    uint32_t vlo[MAXI][4], vhi[MAXI][2], vde[MAXI][4];
    uint32_t mx_hi = 0, mx_lo = 0;  // packed: two 15-bit magnitudes per register
    const int it_lo = (n_lo + NT - 1) / NT, it_hi = (n_hi + NT - 1) / NT, it_de = (n_dense + NT - 1) / NT;  // uniform
    {
#pragma unroll
      for (int i = 0; i < MAXI; ++i) {
        if (i >= it_lo) break;
        const int j = min(i * NT + tid, n_lo - 1);
        const u16x8 idx = *reinterpret_cast<const u16x8*>(src_lo + 8 * j);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const uint32_t x0 = *reinterpret_cast<const uint16_t*>(row + 2 * idx[2 * q]);
          const uint32_t x1 = *reinterpret_cast<const uint16_t*>(row + 2 * idx[2 * q + 1]);
          vlo[i][q] = x0 | (x1 << 16);
          mx_lo = pk_max_u16(mx_lo, vlo[i][q] & 0x7FFF7FFFu);
        }
      }
    }
#pragma unroll
    for (int i = 0; i < MAXI; ++i) {
      if (i >= it_hi) break;
      const int j = min(i * NT + tid, n_hi - 1);
      const u16x4 idx = *reinterpret_cast<const u16x4*>(src_hi + 4 * j);
#pragma unroll
      for (int q = 0; q < 2; ++q) {
        const uint32_t x0 = *reinterpret_cast<const uint16_t*>(row + 2 * idx[2 * q]);
        const uint32_t x1 = *reinterpret_cast<const uint16_t*>(row + 2 * idx[2 * q + 1]);
        vhi[i][q] = x0 | (x1 << 16);
        mx_hi = pk_max_u16(mx_hi, vhi[i][q] & 0x7FFF7FFFu);
      }
    }
    {
#pragma unroll
      for (int i = 0; i < MAXI; ++i) {
        if (i >= it_de) break;
        const int j = min(i * NT + tid, n_dense - 1);
        const u32x4 v = *reinterpret_cast<const u32x4*>(row + j * 16);
#pragma unroll
        for (int q = 0; q < 4; ++q) vde[i][q] = v[q];
      }
    }
    // without lo_compact the low maximum comes from the dense pieces
    if (!a.lo_compact) {
#pragma unroll
      for (int i = 0; i < MAXI; ++i) {
        const int j = i * NT + tid;
        if (j < n_dense) {
          const uint32_t mb = (mask_sh[j >> 2] >> (8 * (j & 3))) & 0xFFu;
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            const uint32_t w = vde[i][e >> 1];
            const uint32_t mag = (e & 1) ? ((w >> 16) & 0x7FFFu) : (w & 0x7FFFu);
            mx_lo = umax(mx_lo, ((mb >> e) & 1u) ? 0u : mag);
          }
        }
      }
    }
    __syncthreads();  // barrier B: the staged row has been read for the last time
    if (m + gridDim.x < a.M) stage_row(m + gridDim.x);  // the next row streams in under the rest of this one

    mx_hi = umax(mx_hi & 0xFFFFu, mx_hi >> 16);
    mx_lo = umax(mx_lo & 0xFFFFu, mx_lo >> 16);
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      mx_hi = umax(mx_hi, static_cast<uint32_t>(__shfl_xor(static_cast<int>(mx_hi), off, 64)));
      mx_lo = umax(mx_lo, static_cast<uint32_t>(__shfl_xor(static_cast<int>(mx_lo), off, 64)));
    }
    if (lane == 0) {
      atomicMax(&amax_sh[par][0], mx_hi);
      atomicMax(&amax_sh[par][1], mx_lo);
    }
    __syncthreads();  // barrier C
    const uint32_t ah = amax_sh[par][0], al = amax_sh[par][1];
    const float amax_hi = __uint_as_float(ah << 16), amax_lo = __uint_as_float(al << 16);
    const float inv_hi = ah ? a.q_hi / amax_hi : 0.0f;
    const float inv_lo = al ? a.q_lo / amax_lo : 0.0f;
    if (tid == 0) {
      a.s_hi[m] = ah ? amax_hi / a.q_hi : 1.0f;
      a.s_lo[m] = al ? amax_lo / a.q_lo : 1.0f;
    }

    // ---- quantise from the registers: whole output dwords per thread, coalesced stores ----
    uint32_t* dst_lo = reinterpret_cast<uint32_t*>(a.lo_compact + m * (a.K_lo / 2));
    uint32_t* dst_hi = reinterpret_cast<uint32_t*>(a.hi_val + m * a.K_hi);
    uint32_t* dst_de = reinterpret_cast<uint32_t*>(a.d_lo + m * (a.K / 2));
#pragma unroll
    for (int i = 0; i < MAXI; ++i) {
      const int j = i * NT + tid;
      if (j < n_lo) dst_lo[j] = quant_lo8(vlo[i], inv_lo);
      if (j < n_hi) {
        uint32_t acc = 0;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const uint32_t w = vhi[i][e >> 1];
          const float xf = __uint_as_float((e & 1) ? (w & 0xFFFF0000u) : (w << 16));
          const float r = __fadd_rn(__fmul_rn(xf, inv_hi), kRoundMagic);
          acc = __builtin_amdgcn_alignbit(__float_as_uint(r), acc, 8);
        }
        dst_hi[j] = acc;
      }
      if (j < n_dense) {
        const uint32_t mb = (mask_sh[j >> 2] >> (8 * (j & 3))) & 0xFFu;
        dst_de[j] = quant_lo8(vde[i], inv_lo) & ~spread_bits_to_nibbles(mb);
      }
    }
  }
}

}  // namespace

// Rows up to 65535 channels (16-bit table entries) whose stage and tables fit in LDS.
bool encode_static_gather_supports(const sq_params& p) {
  if (p.K > 20 * NT * 8) return false;  // 40960: output dwords per thread; also keeps the tables' entries in 16 bits
  const size_t row = (static_cast<size_t>(p.K) * 2 + 4095) / 4096 * 4096;
  return row + static_cast<size_t>(p.K) * 2 + p.K / 8 + 64 <= 150 * 1024;
}

static size_t gather_lds_bytes(int K) {
  const size_t row = (static_cast<size_t>(K) * 2 + 4095) / 4096 * 4096;
  return row + static_cast<size_t>(K) * 2 + K / 8 + 64;  // staged row, two 16-bit tables, the mask
}

int init_encode_static_kernels() {
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(encode_static_gather_kernel<8>),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, 150 * 1024 + 64);
  if (e == hipSuccess)
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(encode_static_gather_kernel<20>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, 150 * 1024 + 64);
  return e == hipSuccess ? SQ_OK : SQ_ERR_LAUNCH;
}

int launch_encode_static_gather(const sq_params& p, const uint16_t* x, int64_t ldx, const uint32_t* mask,
                                const sq_act& out, hipStream_t st) {
  GatherArgs a;
  a.x = x;
  a.ldx = ldx;
  a.M = p.M;
  a.K = p.K;
  a.B = p.bank;
  a.kt = p.topk;
  a.G = p.K / p.bank;
  a.K_hi = a.G * p.topk;
  a.K_lo = p.K - a.K_hi;
  a.mask = mask;
  a.d_lo = out.d_lo;
  a.lo_compact = out.lo_compact;
  a.hi_val = out.hi_val;
  a.s_lo = out.scale_lo;
  a.s_hi = out.scale_hi;
  a.q_hi = code_max(p.h_high, 8);
  a.q_lo = code_max(p.h_low, 4);
  a.row_bytes_padded = static_cast<int>((static_cast<size_t>(p.K) * 2 + 4095) / 4096 * 4096);
  const size_t lds = gather_lds_bytes(p.K);
  const int cus = device_compute_units();
  int per_cu = static_cast<int>(160 * 1024 / (lds + 256));
  if (per_cu < 1) per_cu = 1;
  if (per_cu > 4) per_cu = 4;
  const int64_t cap = static_cast<int64_t>(cus) * per_cu;
  const int blocks = static_cast<int>(p.M < cap ? p.M : cap);
  if (p.K <= 8 * NT * 8) hipLaunchKernelGGL(encode_static_gather_kernel<8>, dim3(blocks), dim3(NT), lds, st, a);
  else hipLaunchKernelGGL(encode_static_gather_kernel<20>, dim3(blocks), dim3(NT), lds, st, a);
  return hipGetLastError() == hipSuccess ? SQ_OK : SQ_ERR_LAUNCH;
}

}  // namespace sq
