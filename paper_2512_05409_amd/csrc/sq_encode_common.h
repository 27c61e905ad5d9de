// Device helpers shared by the SQ-format encoders (gfx950): the comparator networks of the per-bank
// top-k selection, the selection keys, and the quantise-and-pack step of the low part.
#pragma once
#include "sq_device.h"

namespace sq {
namespace enc {

constexpr float kRoundMagic = 12582912.0f;  // 1.5 * 2^23

__device__ __forceinline__ uint32_t umax(uint32_t a, uint32_t b) { return a > b ? a : b; }
__device__ __forceinline__ uint32_t umin(uint32_t a, uint32_t b) { return a < b ? a : b; }

// Sorts v[0..N) descending (N a power of two); every index is a compile-time constant.
template <int N>
__device__ __forceinline__ void bitonic_sort_desc(uint32_t* v) {
#pragma unroll
  for (int k = 2; k <= N; k <<= 1) {
#pragma unroll
    for (int j = k >> 1; j > 0; j >>= 1) {
#pragma unroll
      for (int i = 0; i < N; ++i) {
        const int l = i ^ j;
        if (l > i) {
          const uint32_t a = v[i], b = v[l];
          const uint32_t mx = umax(a, b), mn = umin(a, b);
          const bool desc = (i & k) == 0;
          v[i] = desc ? mx : mn;
          v[l] = desc ? mn : mx;
        }
      }
    }
  }
}

__device__ __forceinline__ void cex_desc(uint32_t* v, int i, int j) {  // larger value to the lower index
  const uint32_t a = v[i], b = v[j];
  v[i] = umax(a, b);
  v[j] = umin(a, b);
}

// Sorts v[0..N) descending with the smallest known comparator networks for N = 2, 4, 8 (1, 5, 19
// exchanges instead of the bitonic 1, 6, 24); larger N fall back to the bitonic network.
template <int N>
__device__ __forceinline__ void sort_desc(uint32_t* v) {
  if constexpr (N == 2) {
    cex_desc(v, 0, 1);
  } else if constexpr (N == 4) {
    cex_desc(v, 0, 1); cex_desc(v, 2, 3);
    cex_desc(v, 0, 2); cex_desc(v, 1, 3);
    cex_desc(v, 1, 2);
  } else if constexpr (N == 8) {
    cex_desc(v, 0, 1); cex_desc(v, 2, 3); cex_desc(v, 4, 5); cex_desc(v, 6, 7);
    cex_desc(v, 0, 2); cex_desc(v, 1, 3); cex_desc(v, 4, 6); cex_desc(v, 5, 7);
    cex_desc(v, 1, 2); cex_desc(v, 5, 6); cex_desc(v, 0, 4); cex_desc(v, 3, 7);
    cex_desc(v, 1, 5); cex_desc(v, 2, 6);
    cex_desc(v, 1, 4); cex_desc(v, 3, 6);
    cex_desc(v, 2, 4); cex_desc(v, 3, 5);
    cex_desc(v, 3, 4);
  } else {
    bitonic_sort_desc<N>(v);
  }
}

// v[0..N) is bitonic; sorts it descending.
template <int N>
__device__ __forceinline__ void bitonic_merge_desc(uint32_t* v) {
#pragma unroll
  for (int j = N >> 1; j > 0; j >>= 1) {
#pragma unroll
    for (int i = 0; i < N; ++i) {
      const int l = i ^ j;
      if (l > i) {
        const uint32_t a = v[i], b = v[l];
        v[i] = umax(a, b);
        v[l] = umin(a, b);
      }
    }
  }
}

// 8 mask bits -> 8 nibbles of all-ones / all-zeros.
__device__ __forceinline__ uint32_t spread_bits_to_nibbles(uint32_t b8) {
  uint32_t t = b8 & 0xFFu;
  t = (t | (t << 12)) & 0x000F000Fu;
  t = (t | (t << 6)) & 0x03030303u;
  t = (t | (t << 3)) & 0x11111111u;
  t |= t << 1;  // each 1 -> 0xF (two shift-or steps; a multiplication by 15 would be a quarter-rate instruction)
  t |= t << 2;
  return t;
}

// Low-part codes of 8 consecutive channels (4 packed bf16 pairs) as one dword of nibbles.  The channels
// of the high part come through here too, with quotients far outside [-7, 7]: only the low four bits
// of each rounded value are kept, and the caller clears those nibbles.
__device__ __forceinline__ uint32_t quant_lo8(const uint32_t* pairs, float inv_lo) {
  uint32_t acc = 0;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const uint32_t w = pairs[e >> 1];
    const float xf = __uint_as_float((e & 1) ? (w & 0xFFFF0000u) : (w << 16));
    const float r = __fadd_rn(__fmul_rn(xf, inv_lo), kRoundMagic);
    // shift the nibbles gathered so far down by four bits and enter the low four bits of r at the top: after
    // eight elements the first one sits in bits 0-3 (one funnel shift per element, no masking)
    acc = __builtin_amdgcn_alignbit(__float_as_uint(r), acc, 4);
  }
  return acc;
}

template <int N>
__device__ __forceinline__ void store_bytes(int8_t* dst, const uint32_t* words) {
  // N bytes (N a power of two <= 32) held in ceil(N/4) dwords; dst is N-byte aligned.
  if constexpr (N >= 16) {
#pragma unroll
    for (int i = 0; i < N / 16; ++i)
      reinterpret_cast<uint4*>(dst)[i] = make_uint4(words[4 * i], words[4 * i + 1], words[4 * i + 2], words[4 * i + 3]);
  } else if constexpr (N == 8) {
    *reinterpret_cast<uint2*>(dst) = make_uint2(words[0], words[1]);
  } else if constexpr (N == 4) {
    *reinterpret_cast<uint32_t*>(dst) = words[0];
  } else if constexpr (N == 2) {
    *reinterpret_cast<uint16_t*>(dst) = static_cast<uint16_t>(words[0]);
  } else {
    *dst = static_cast<int8_t>(words[0]);
  }
}

// Selection key of one element: magnitude (15 bits of the bf16) in bits 31..17, 255 - channel in bits
// 8..1, the sign in bit 0.  Keys of one bank are distinct, larger magnitude sorts first and among equal
// magnitudes the lower channel does (Section 3.1, the top-k rule with ties to the lower index).
// `rot` is the bf16 pair rotated so that the wanted element's magnitude sits in bits 31..17 and its
// sign in bit 0.
__device__ __forceinline__ uint32_t make_key(uint32_t rot, uint32_t ch) {
  return (rot & 0xFFFE0001u) | ((255u - ch) << 1);
}
__device__ __forceinline__ uint32_t key_channel(uint32_t key) { return 255u - ((key >> 1) & 255u); }
__device__ __forceinline__ uint32_t key_magnitude(uint32_t key) { return key >> 17; }
__device__ __forceinline__ float key_value(uint32_t key) {  // the element as fp32
  return __uint_as_float(__builtin_amdgcn_alignbit(key, key, 1) & 0xFFFF0000u);
}

}  // namespace enc
}  // namespace sq
