// sq_encode, dynamic rule, streaming kernel (gfx950): bf16 activations -> SQ-format (Section 3.1, Eq. (1);
// per-token top-k of every bank by magnitude, Sections 3.2.2 / 4.3).
//
// A wave works on "units" of 64 consecutive banks (one bank per lane) and walks over several of them.
// The activations of a unit are copied from HBM straight into LDS by LDS-direct loads, fully coalesced
// (every wave instruction moves 1 KB of consecutive memory), one unit ahead of the arithmetic: the copies
// occupy no registers, so the fetch of unit u+1 runs under the selection network of unit u.  A lane then
// reads its own bank from LDS; the 16-byte chunks of a bank row are XOR-swizzled (on the global side of
// the copy) so that the 64 lanes, each reading chunk c of its own row, hit distinct LDS banks.
// The waits for the copies are explicit (s_waitcnt with a count).  The LDS reads use clang vector types: the
// compiler orders an LDS read after every outstanding LDS-direct load it thinks may alias (a full vmcnt(0)
// wait, which would serialise fetch and arithmetic), and it does think so for HIP's uint4 struct type.
// Selection, scales, quantisation and packing are the register-only steps of sq_encode_common.h.  The row
// maxima are combined with wave shuffles (and through LDS when a row spans several waves).  The
// matrix-core-ready image (sq_act::hi_dense) is put together in the lane's own LDS row, which is free once
// the low part has been quantised.
//
// TIED (tied-scale variant of the format): both parts share one scale step, s_lo = 16 * s_hi, so that the
// layer needs a single INT8 operand and one accumulator; the image then holds 16 * (low code) at the low
// channels and the high code at the high channels.
#include "sq_encode_common.h"

namespace sq {
namespace {

using namespace enc;

typedef __attribute__((address_space(3))) void* lds_ptr_t;

template <int B>
struct StreamCfg {
  static constexpr int NCH = B / 8;                        // 16-byte chunks per bank row
  static constexpr int ROWB = 2 * B;                       // bytes per bank row
  static constexpr int SH = B == 32 ? 2 : (B == 64 ? 1 : 0);  // swizzle: chunk index ^ (row >> SH)
  static constexpr int RPI = 64 / NCH;                     // bank rows per copy instruction (1 KB)
  static constexpr int STAGE = 64 * ROWB;                  // bytes per wave and stage
  static constexpr int NW = B == 128 ? 2 : 4;              // waves per workgroup
  static constexpr int LDS_BYTES = NW * 2 * STAGE;
};

template <int B>
__device__ __forceinline__ int bank_off(int row, int c) {
  typedef StreamCfg<B> C;
  return row * C::ROWB + (((c ^ (row >> C::SH)) & (C::NCH - 1)) << 4);
}

struct StreamArgs {
  const uint16_t* x;
  int64_t ldx;       // elements
  int M, K, G;       // G = K / bank, a power of two here
  int lgG;           // log2(G)
  int lg;            // log2(min(G, 64)): lanes of a wave that belong to one row
  int wpr;           // waves per row (G / 64 when G > 64, else 1)
  int64_t units;     // ceil(M * G / 64)
  uint8_t* d_lo;
  int8_t* hi_val;
  uint32_t* mask;
  float* s_lo;
  float* s_hi;
  int8_t* image;     // hi_dense (two scales) or the combined INT8 operand (TIED); may be null
  float q_hi, q_lo;  // largest code magnitudes of the two parts (127 and 7 for the 8/4 pair)
};

// at most n vector-memory operations outstanding (gfx9 s_waitcnt encoding), LDS counters untouched
constexpr int waitcnt_vm(int n) { return (n & 15) | (7 << 4) | (15 << 8) | ((n >> 4) << 14); }

// Vector-memory operations of a wave retire in order, and stores count like loads.  The wait for the copy of
// the next unit must not also wait for the stores of the unit just finished, which are younger than that
// copy: it waits until "at most as many operations as were issued after the copy" are outstanding.  That
// number has to be exact, so the stores of a unit's results are single instructions written out here (the
// compiler can neither merge nor split them); kStores<B, KT> counts them.
// The wide stores carry the sc1 bit: the L2 then writes the lines through instead of keeping all of a launch's
// output dirty until the write-back at the end of the kernel, where nothing is left to overlap it with.
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ void store16(void* p, u32x4 v) {
  // A store of more than 8 bytes must not be followed directly by an instruction that overwrites its data
  // registers (the compiler's hazard handling does not look inside asm statements): two idle slots follow.
  asm volatile("global_store_dwordx4 %0, %1, off sc1\n\ts_nop 1" ::"v"(p), "v"(v) : "memory");
}
__device__ __forceinline__ void store8(void* p, u32x2 v) {
  asm volatile("global_store_dwordx2 %0, %1, off sc1" ::"v"(p), "v"(v) : "memory");
}
__device__ __forceinline__ void store4(void* p, unsigned v) {
  asm volatile("global_store_dword %0, %1, off" ::"v"(p), "v"(v) : "memory");
}
__device__ __forceinline__ void store2(void* p, unsigned v) {
  asm volatile("global_store_short %0, %1, off" ::"v"(p), "v"(v) : "memory");
}
// N bytes (a power of two from 2 to 32) held in dwords
template <int N>
__device__ __forceinline__ void store_n(void* p, const uint32_t* w) {
  if constexpr (N >= 16) {
#pragma unroll
    for (int i = 0; i < N / 16; ++i)
      store16(static_cast<char*>(p) + 16 * i, u32x4{w[4 * i], w[4 * i + 1], w[4 * i + 2], w[4 * i + 3]});
  } else if constexpr (N == 8) {
    store8(p, u32x2{w[0], w[1]});
  } else if constexpr (N == 4) {
    store4(p, w[0]);
  } else {
    static_assert(N == 2, "size");
    store2(p, w[0]);
  }
}
// A wave's results that are more than 8 bytes per bank (the packed low codes, the matrix-core image) leave
// through LDS: written by the owning lanes into a [64 banks][R bytes] array, read back in memory order, so
// that every store instruction writes 1 KB of consecutive memory.  (Stored straight from the owning lanes, a
// 64-byte transaction to L2 would carry 16 or 32 useful bytes, and the L2's transaction rate, not HBM, would
// bound the kernel.)  The 16-byte chunks of a bank's R bytes are XOR-swizzled so that the owners' writes are
// free of LDS bank conflicts; the read-back covers whole 256-byte spans whatever the swizzle.
template <int R>
__device__ __forceinline__ int out_off(int bank, int c) {
  constexpr int NC = R / 16;
  if constexpr (NC == 1) return bank * R;
  constexpr int SHIFT = NC == 8 ? 1 : (NC == 4 ? 2 : 3);  // log2(16 / NC): banks per 256 bytes
  return bank * R + (((c ^ (bank >> SHIFT)) & (NC - 1)) << 4);
}

struct UnitPos {
  int64_t row0;  // row of the unit's first bank
  int g0;        // its bank index inside the row
  int lg;        // log2(banks of one row inside a unit)
  int M;
};

// out: start of the [M][row_bytes] array, R bytes per bank; region: the LDS array written with out_off<R>.
template <int R>
__device__ __forceinline__ void store_unit(char* out, int64_t row_bytes, const UnitPos& u, const char* region, int lane) {
  constexpr int NC = R / 16;
#pragma unroll
  for (int j = 0; j < NC; ++j) {
    const int q = j * 64 + lane;  // 16-byte chunk of the unit, in memory order
    const int bank = q / NC, c = q % NC;
    const u32x4 v = *reinterpret_cast<const u32x4*>(region + out_off<R>(bank, c));
    if (u.lg == 6) {  // the unit lies inside one row: one run of 64 * R bytes
      store16(out + u.row0 * row_bytes + static_cast<int64_t>(u.g0) * R + q * 16, v);
    } else {
      const int64_t row = u.row0 + (bank >> u.lg);
      const int g = bank & ((1 << u.lg) - 1);
      if (row < u.M) store16(out + row * row_bytes + g * R + c * 16, v);
    }
  }
}

constexpr int n_store_instr(int bytes) { return bytes >= 16 ? bytes / 16 : 1; }
template <int B, int KT>
constexpr int kStores(bool image) {
  return n_store_instr(B / 2) + n_store_instr(KT) + n_store_instr(B / 8) + (image ? B / 16 : 0);
}

template <int B>
__device__ __forceinline__ void issue_unit(const StreamArgs& a, int64_t u, char* stage, int lane) {
  typedef StreamCfg<B> C;
  const int64_t bi0 = u * 64;
  const int64_t row0 = bi0 >> a.lgG;
  const int g0 = static_cast<int>(bi0 & (a.G - 1));
  if (a.lg == 6) {
    // the unit lies inside one row: 64 * ROWB consecutive bytes
    const char* base = reinterpret_cast<const char*>(a.x) + (row0 * a.ldx + static_cast<int64_t>(g0) * B) * 2;
#pragma unroll
    for (int i = 0; i < C::NCH; ++i) {
      const int rr = i * C::RPI + lane / C::NCH;  // bank row of the unit this lane's 16 bytes land in
      const int c = ((lane % C::NCH) ^ (rr >> C::SH)) & (C::NCH - 1);
      const char* src = base + rr * C::ROWB + c * 16;
      __builtin_amdgcn_global_load_lds(src, (lds_ptr_t)(stage + i * 1024), 16, 0, 0);
    }
  } else {
    const int gw_mask = (1 << a.lg) - 1;
#pragma unroll
    for (int i = 0; i < C::NCH; ++i) {
      const int rr = i * C::RPI + lane / C::NCH;
      const int c = ((lane % C::NCH) ^ (rr >> C::SH)) & (C::NCH - 1);
      int64_t row = row0 + (rr >> a.lg);
      row = row < a.M ? row : a.M - 1;  // the last unit may reach past the last row: fetch valid memory
      const char* src = reinterpret_cast<const char*>(a.x) + (row * a.ldx + static_cast<int64_t>(rr & gw_mask) * B) * 2 + c * 16;
      __builtin_amdgcn_global_load_lds(src, (lds_ptr_t)(stage + i * 1024), 16, 0, 0);
    }
  }
}

template <int B, int KT, bool TIED>
__global__ __launch_bounds__(64 * StreamCfg<B>::NW) void encode_stream_kernel(StreamArgs a) {
  typedef StreamCfg<B> C;
  static_assert(B % 32 == 0 && KT >= 1 && KT <= 32 && (KT & (KT - 1)) == 0 && B % KT == 0 && B / KT >= 2, "shape");
  extern __shared__ __attribute__((aligned(16))) char lds[];
  __shared__ uint32_t cross[2][C::NW][2];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  char* my = lds + wave * 2 * C::STAGE;
  const int gw = 1 << a.lg;
  // Position of this lane's bank relative to the first bank of a unit: lrow rows further down (0 when a row
  // spans the whole wave), lg banks further right.  The addresses of a unit's results are a wave-uniform base
  // (scalar arithmetic) plus these per-lane byte offsets, which never change.
  const int lrow = lane >> a.lg;
  const int lgb = lane & (gw - 1);
  const uint32_t off_mask = static_cast<uint32_t>(lrow) * (a.K / 8) + lgb * (B / 8);

  // Order of a wave's vector-memory operations: copy(0), copy(1), then per unit u: [wait for copy(u)],
  // scale stores (u), result stores (u), copy(u + 2).  When unit u is waited for, the operations issued after
  // copy(u) are the result stores of unit u-1 and copy(u + 1).
  const int64_t stride = static_cast<int64_t>(gridDim.x) * C::NW;
  int64_t ub = blockIdx.x;
  {
    const int64_t u0 = ub * C::NW + wave;
    if (u0 < a.units) issue_unit<B>(a, u0, my, lane);
    if (u0 + stride < a.units) issue_unit<B>(a, u0 + stride, my + C::STAGE, lane);
  }
  for (int it = 0; ub * C::NW < a.units; ub += gridDim.x, ++it) {
    const int64_t u = ub * C::NW + wave;
    const bool wave_active = u < a.units;
    const bool has_next = u + stride < a.units;  // copy(u + 1 in this wave's sequence) is in flight
    char* stage = my + (it & 1) * C::STAGE;
    asm volatile("" ::: "memory");
    {
      constexpr int S0 = kStores<B, KT>(false), S1 = kStores<B, KT>(true);
      if (it == 0) {
        if (has_next) __builtin_amdgcn_s_waitcnt(waitcnt_vm(C::NCH));
        else __builtin_amdgcn_s_waitcnt(waitcnt_vm(0));
      } else if (a.image) {
        if (has_next) __builtin_amdgcn_s_waitcnt(waitcnt_vm(S1 + C::NCH));
        else __builtin_amdgcn_s_waitcnt(waitcnt_vm(S1));
      } else {
        if (has_next) __builtin_amdgcn_s_waitcnt(waitcnt_vm(S0 + C::NCH));
        else __builtin_amdgcn_s_waitcnt(waitcnt_vm(S0));
      }
    }
    asm volatile("" ::: "memory");

    const int64_t bi0 = u * 64;                              // first bank of the unit (wave-uniform)
    const int64_t row0 = bi0 >> a.lgG;                       // its row
    const int g0 = static_cast<int>(bi0 & (a.G - 1));        // and its bank index inside the row
    const int64_t row = row0 + lrow;
    const int g = g0 + lgb;
    const bool active = wave_active && row < a.M;

    // ---- selection ----
    uint32_t top[KT];
    uint32_t mag_hi = 0, mag_lo = 0;  // this bank's largest high / low magnitude (bf16 bits)
    if (wave_active) {
      uint32_t key[B];
#pragma unroll
      for (int i = 0; i < C::NCH; ++i) {
        const u32x4 v = *reinterpret_cast<const u32x4*>(stage + bank_off<B>(lane, i));
        const uint32_t w[4] = {v[0], v[1], v[2], v[3]};
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          key[8 * i + 2 * q] = make_key(__builtin_amdgcn_alignbit(w[q], w[q], 15), 8 * i + 2 * q);
          key[8 * i + 2 * q + 1] = make_key(__builtin_amdgcn_alignbit(w[q], w[q], 31), 8 * i + 2 * q + 1);
        }
      }
#pragma unroll
      for (int g0 = 0; g0 < B; g0 += KT) sort_desc<KT>(key + g0);
      uint32_t dropped[KT];
#pragma unroll
      for (int i = 0; i < KT; ++i) dropped[i] = 0;
#pragma unroll
      for (int width = KT; width < B; width <<= 1) {
#pragma unroll
        for (int base = 0; base < B; base += 2 * width) {
          uint32_t* p = key + base;
          uint32_t* q = key + base + width;
#pragma unroll
          for (int i = 0; i < KT; ++i) {
            const uint32_t ai = p[i], bj = q[KT - 1 - i];
            p[i] = umax(ai, bj);
            dropped[i] = umax(dropped[i], umin(ai, bj));
          }
          if (2 * width < B) bitonic_merge_desc<KT>(p);  // the last merge only needs the set
        }
      }
      uint32_t dmax = dropped[0], tmax = key[0];
#pragma unroll
      for (int i = 1; i < KT; ++i) {
        dmax = umax(dmax, dropped[i]);
        tmax = umax(tmax, key[i]);
      }
#pragma unroll
      for (int i = 0; i < KT; ++i) top[i] = key[i];
      mag_hi = key_magnitude(tmax);
      mag_lo = key_magnitude(dmax);
    }

    // ---- row maxima: the gw lanes of a row inside this wave, then the waves of a row ----
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      if (off < gw) {
        mag_hi = umax(mag_hi, static_cast<uint32_t>(__shfl_xor(static_cast<int>(mag_hi), off, 64)));
        mag_lo = umax(mag_lo, static_cast<uint32_t>(__shfl_xor(static_cast<int>(mag_lo), off, 64)));
      }
    }
    if (a.wpr > 1) {  // uniform over the workgroup
      if (lane == 0) {
        cross[it & 1][wave][0] = mag_hi;
        cross[it & 1][wave][1] = mag_lo;
      }
      __syncthreads();
      const int w0 = wave - wave % a.wpr;
      for (int w = w0; w < w0 + a.wpr; ++w) {
        mag_hi = umax(mag_hi, cross[it & 1][w][0]);
        mag_lo = umax(mag_lo, cross[it & 1][w][1]);
      }
    }
    if (active) {
    // ---- per-token scales ----
    const float amax_hi = __uint_as_float(mag_hi << 16), amax_lo = __uint_as_float(mag_lo << 16);
    float inv_hi, inv_lo, sc_hi, sc_lo;
    if constexpr (TIED) {
      // one scale step for both parts: s_hi = A / 127 with A = max(amax_hi, amax_lo * 127/112), s_lo = 16 * s_hi
      const float A = fmaxf(amax_hi, __fmul_rn(amax_lo, 127.0f / 112.0f));
      const bool nz = A != 0.0f;
      inv_hi = nz ? 127.0f / A : 0.0f;
      sc_hi = nz ? A / 127.0f : 1.0f;
      inv_lo = __fmul_rn(inv_hi, 0.0625f);
      sc_lo = __fmul_rn(sc_hi, 16.0f);
    } else {
      inv_hi = mag_hi ? a.q_hi / amax_hi : 0.0f;
      inv_lo = mag_lo ? a.q_lo / amax_lo : 0.0f;
      sc_hi = mag_hi ? amax_hi / a.q_hi : 1.0f;
      sc_lo = mag_lo ? amax_lo / a.q_lo : 1.0f;
    }
    if (g == 0) {
      a.s_hi[row] = sc_hi;
      a.s_lo[row] = sc_lo;
    }

    // ---- high part: quantise the k selected values, order them by channel, emit codes and mask ----
    uint32_t ent[KT];  // channel << 8 | code byte
    uint32_t mw[B / 32];
#pragma unroll
    for (int w = 0; w < B / 32; ++w) mw[w] = 0;
#pragma unroll
    for (int t = 0; t < KT; ++t) {
      const uint32_t ch = key_channel(top[t]);
      const float r = __fadd_rn(__fmul_rn(key_value(top[t]), inv_hi), kRoundMagic);
      ent[t] = (ch << 8) | (__float_as_uint(r) & 0xFFu);
      if constexpr (B == 32) {
        mw[0] |= 1u << ch;
      } else if constexpr (B == 64) {
        const uint64_t bit = 1ull << ch;
        mw[0] |= static_cast<uint32_t>(bit);
        mw[1] |= static_cast<uint32_t>(bit >> 32);
      } else {
#pragma unroll
        for (int w = 0; w < B / 32; ++w) mw[w] |= ((ch >> 5) == static_cast<uint32_t>(w)) ? (1u << (ch & 31u)) : 0u;
      }
    }
    uint32_t scat[KT];  // image byte offset << 8 | code byte
#pragma unroll
    for (int t = 0; t < KT; ++t) {
      const uint32_t ch = ent[t] >> 8;
      scat[t] = ((((ch & ~7u) | ((ch & 1u) << 2) | ((ch & 7u) >> 1))) << 8) | (ent[t] & 0xFFu);
    }
    sort_desc<KT>(ent);  // descending channel; read back reversed
    uint32_t hv[(KT + 3) / 4];
#pragma unroll
    for (int i = 0; i < (KT + 3) / 4; ++i) hv[i] = 0;
#pragma unroll
    for (int t = 0; t < KT; ++t) hv[t / 4] |= (ent[KT - 1 - t] & 0xFFu) << (8 * (t % 4));
    store_n<KT>(a.hi_val + bi0 * KT + lane * KT, hv);
    store_n<B / 8>(reinterpret_cast<char*>(a.mask) + row0 * (a.K / 8) + g0 * (B / 8) + off_mask, mw);

    // ---- low part: every channel quantised (the bank is read from LDS again, which keeps it out of the
    // registers during the selection), the selected ones cleared ----
    asm volatile("" ::: "memory");
    uint32_t dl[B / 8];
#pragma unroll
    for (int i = 0; i < C::NCH; ++i) {
      const u32x4 v = *reinterpret_cast<const u32x4*>(stage + bank_off<B>(lane, i));
      const uint32_t w[4] = {v[0], v[1], v[2], v[3]};
      const uint32_t q = quant_lo8(w, inv_lo);
      const uint32_t clear = spread_bits_to_nibbles(mw[i / 4] >> (8 * (i % 4)));
      dl[i] = q & ~clear;
    }
    // the bank's row in LDS has been read for the last time: the stage now takes the outgoing arrays
    constexpr int D_OFF = 0, I_OFF = 64 * (B / 2);
    static_assert(I_OFF + 64 * B <= C::STAGE, "outgoing arrays must fit in a stage");
#pragma unroll
    for (int i = 0; i < B / 32; ++i)
      *reinterpret_cast<u32x4*>(stage + D_OFF + out_off<B / 2>(lane, i)) = u32x4{dl[4 * i], dl[4 * i + 1], dl[4 * i + 2], dl[4 * i + 3]};

    // ---- matrix-core-ready image of the bank, B bytes: inside every group of 8 channels the even channels
    // first, then the odd ones: the base bytes (zeros, or 16 x the low codes in the tied variant -- a nibble
    // moved to the high half of a byte is 16 x its value), then the k high codes scattered to their channels
    // (a lane can address LDS bytes dynamically, not registers). ----
    if (a.image) {
#pragma unroll
      for (int i = 0; i < B / 16; ++i) {
        u32x4 v = {0u, 0u, 0u, 0u};
        if constexpr (TIED) {
          v = u32x4{(dl[2 * i] << 4) & 0xF0F0F0F0u, dl[2 * i] & 0xF0F0F0F0u, (dl[2 * i + 1] << 4) & 0xF0F0F0F0u,
                    dl[2 * i + 1] & 0xF0F0F0F0u};
        }
        *reinterpret_cast<u32x4*>(stage + I_OFF + out_off<B>(lane, i)) = v;
      }
#pragma unroll
      for (int t = 0; t < KT; ++t) {
        const uint32_t off = scat[t] >> 8;
        stage[I_OFF + out_off<B>(lane, off >> 4) + (off & 15u)] = static_cast<char>(scat[t] & 0xFFu);
      }
    }
    }  // active

    if (wave_active) {
      const UnitPos up = {row0, g0, a.lg, a.M};
      store_unit<B / 2>(reinterpret_cast<char*>(a.d_lo), a.K / 2, up, stage + 0, lane);
      if (a.image) store_unit<B>(reinterpret_cast<char*>(a.image), a.K, up, stage + 64 * (B / 2), lane);
    }

    // the stage of this unit is free now: enqueue the copy of the unit after next into it
    asm volatile("" ::: "memory");
    if (u + 2 * stride < a.units) issue_unit<B>(a, u + 2 * stride, stage, lane);
  }
}

template <int B, int KT, bool TIED>
int launch_stream_t(const StreamArgs& a, hipStream_t st) {
  typedef StreamCfg<B> C;
  const int64_t groups = (a.units + C::NW - 1) / C::NW;
  const int cus = device_compute_units();
  const int resident = 160 * 1024 / C::LDS_BYTES;  // workgroups a compute unit holds at once
  const int64_t cap = static_cast<int64_t>(cus) * resident;
  const int blocks = static_cast<int>(groups < cap ? groups : cap);
  hipLaunchKernelGGL((encode_stream_kernel<B, KT, TIED>), dim3(blocks), dim3(64 * C::NW), C::LDS_BYTES, st, a);
  return hipGetLastError() == hipSuccess ? SQ_OK : SQ_ERR_LAUNCH;
}

template <int B, int KT, bool TIED>
hipError_t raise_stream_lds_limit() {
  return hipFuncSetAttribute(reinterpret_cast<const void*>(encode_stream_kernel<B, KT, TIED>),
                             hipFuncAttributeMaxDynamicSharedMemorySize, StreamCfg<B>::LDS_BYTES);
}

#define SQ_STREAM_CASES(X)                                                                        \
  X(32, 2) X(32, 4) X(32, 8) X(32, 16) X(64, 4) X(64, 8) X(64, 16) X(64, 32) X(128, 8) X(128, 16) X(128, 32)

}  // namespace

bool encode_stream_supports(const sq_params& p) {
  const int G = p.K / p.bank;
  const int nw = p.bank == 128 ? 2 : 4;
  if ((G & (G - 1)) != 0) return false;  // rows of 1, 2, 4, ... banks
  return G <= 64 * nw;                   // a row spans at most the waves of one workgroup
}

int init_encode_stream_kernels() {
  hipError_t e = hipSuccess;
#define X(B, KT)                                                          \
  if (e == hipSuccess) e = raise_stream_lds_limit<B, KT, false>();        \
  if (e == hipSuccess) e = raise_stream_lds_limit<B, KT, true>();
  SQ_STREAM_CASES(X)
#undef X
  return e == hipSuccess ? SQ_OK : SQ_ERR_LAUNCH;
}

int launch_encode_stream(const sq_params& p, const uint16_t* x, int64_t ldx, const sq_act& out, int8_t* image,
                         bool tied, float q_hi, float q_lo, hipStream_t st) {
  StreamArgs a;
  a.x = x;
  a.ldx = ldx;
  a.M = p.M;
  a.K = p.K;
  a.G = p.K / p.bank;
  const int gw = a.G < 64 ? a.G : 64;
  a.lg = 0;
  while ((1 << a.lg) < gw) ++a.lg;
  a.lgG = 0;
  while ((1 << a.lgG) < a.G) ++a.lgG;
  a.wpr = a.G > 64 ? a.G / 64 : 1;
  a.units = (static_cast<int64_t>(p.M) * a.G + 63) / 64;
  a.d_lo = out.d_lo;
  a.hi_val = out.hi_val;
  a.mask = out.mask;
  a.s_lo = out.scale_lo;
  a.s_hi = out.scale_hi;
  a.image = image;
  a.q_hi = q_hi;
  a.q_lo = q_lo;
#define X(B, KT)                                                                                        \
  if (p.bank == B && p.topk == KT)                                                                      \
    return tied ? launch_stream_t<B, KT, true>(a, st) : launch_stream_t<B, KT, false>(a, st);
  SQ_STREAM_CASES(X)
#undef X
  return SQ_ERR_UNSUPPORTED;
}

}  // namespace sq
