// The SQ-format at its equivalent bit width (Section 4.1: y = (1-s)*h_high + s*h_low bits per element):
// conversion between the compute containers of an sq_act (INT8 high codes, 4-bit low codes dense over K)
// and the packed stream -- per token row the high codes of the high channels at h_high bits each, then the low
// codes of the low channels only at h_low bits each, ascending channel order, least significant bit first.
// Storage conversions, off the layer's hot path: one thread per output byte (pack) or per 32 channels (unpack).
#include "sq_device.h"

namespace sq {
namespace {

struct StoreArgs {
  int M, K, B, kt, G, hh, hl;
  int K_hi, K_lo;
  int row_bytes, hi_bytes;
  int64_t mask_stride;  // words between the masks of consecutive rows (0: one mask for all rows)
  const uint32_t* mask;
  uint32_t* mask_out;   // sentinel form, unpack: the mask recovered from the sentinels
  int sentinel;         // 1: the low section covers all K channels and carries v_mask = -2^(hl-1) at the high ones
  uint8_t* d_lo;
  int8_t* hi_val;
  uint8_t* packed;
};

__device__ __forceinline__ int nibble_at(const uint8_t* d_lo_row, int ch) {
  return (d_lo_row[ch >> 1] >> ((ch & 1) * 4)) & 0xF;
}

// channel (inside the row) of the r-th low channel of bank `bank`
__device__ int low_channel(const uint32_t* mrow, int bank, int B, int r) {
  for (int w = 0; w < B / 32; ++w) {
    uint32_t zeros = ~mrow[bank * (B / 32) + w];
    const int c = __popc(zeros);
    if (r < c) {
      for (; r > 0; --r) zeros &= zeros - 1;
      return bank * B + w * 32 + __ffs(static_cast<int>(zeros)) - 1;
    }
    r -= c;
  }
  return bank * B;  // malformed mask: stay in range
}

__global__ __launch_bounds__(256) void pack_storage_kernel(StoreArgs a) {
  const int64_t idx = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
  if (idx >= static_cast<int64_t>(a.M) * a.row_bytes) return;
  const int64_t m = idx / a.row_bytes;
  const int b = static_cast<int>(idx - m * a.row_bytes);
  uint32_t out = 0;
  if (b < a.hi_bytes) {
    const int8_t* h = a.hi_val + m * a.K_hi;
    out = a.hh == 8 ? static_cast<uint8_t>(h[b]) : ((h[2 * b] & 0xF) | ((h[2 * b + 1] & 0xF) << 4));
  } else {
    const uint32_t* mrow = a.mask + m * a.mask_stride;
    const uint8_t* drow = a.d_lo + m * (a.K / 2);
    const int bit0 = (b - a.hi_bytes) * 8;  // first bit of this byte inside the low section
    const int nlo = a.B - a.kt;
    const uint32_t cmask = (1u << a.hl) - 1u;
    const int n_codes = a.sentinel ? a.K : a.K_lo;
    for (int t = bit0 / a.hl; t * a.hl < bit0 + 8 && t < n_codes; ++t) {
      uint32_t code;
      if (a.sentinel) {  // code t belongs to channel t; the high channels carry the unused most negative code
        const bool hi = (mrow[t >> 5] >> (t & 31)) & 1u;
        code = hi ? (1u << (a.hl - 1)) : (static_cast<uint32_t>(nibble_at(drow, t)) & cmask);
      } else {
        const int ch = low_channel(mrow, t / nlo, a.B, t % nlo);
        code = static_cast<uint32_t>(nibble_at(drow, ch)) & cmask;
      }
      const int sh = t * a.hl - bit0;
      out |= sh >= 0 ? code << sh : code >> (-sh);
    }
  }
  a.packed[idx] = static_cast<uint8_t>(out);
}

// h bits at bit offset `o` of a section of `n` bytes, sign-extended
__device__ __forceinline__ int bits_at(const uint8_t* sec, int n, int o, int h) {
  const int by = o >> 3;
  uint32_t v = sec[by];
  if (by + 1 < n) v |= static_cast<uint32_t>(sec[by + 1]) << 8;
  v = (v >> (o & 7)) & ((1u << h) - 1u);
  return (v & (1u << (h - 1))) ? static_cast<int>(v) - (1 << h) : static_cast<int>(v);
}

// Sentinel form: the mask is not stored; a low code equal to v_mask marks a high channel.
__global__ __launch_bounds__(256) void unpack_sentinel_kernel(StoreArgs a) {
  const int64_t idx = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
  const int wpr = a.K / 32;
  if (idx >= static_cast<int64_t>(a.M) * wpr) return;
  const int64_t m = idx / wpr;
  const int wg = static_cast<int>(idx - m * wpr);
  const int wpb = a.B / 32;
  const int bank = wg / wpb;
  const uint8_t* hsec = a.packed + m * a.row_bytes;
  const uint8_t* lsec = hsec + a.hi_bytes;
  const int lbytes = a.row_bytes - a.hi_bytes;
  const int v_mask = -(1 << (a.hl - 1));
  int nh = 0;  // high channels of the bank before this word
  for (int ch = bank * a.B; ch < wg * 32; ++ch) nh += bits_at(lsec, lbytes, ch * a.hl, a.hl) == v_mask;
  int8_t* hv = a.hi_val + m * a.K_hi + bank * a.kt;
  uint32_t dl[4] = {0, 0, 0, 0};
  uint32_t word = 0;
  for (int i = 0; i < 32; ++i) {
    const int code = bits_at(lsec, lbytes, (wg * 32 + i) * a.hl, a.hl);
    if (code == v_mask) {
      word |= 1u << i;
      if (nh < a.kt) hv[nh] = static_cast<int8_t>(bits_at(hsec, a.hi_bytes, (bank * a.kt + nh) * a.hh, a.hh));
      ++nh;
    } else {
      dl[i >> 3] |= static_cast<uint32_t>(code & 0xF) << (4 * (i & 7));
    }
  }
  a.mask_out[m * wpr + wg] = word;
  *reinterpret_cast<uint4*>(a.d_lo + m * (a.K / 2) + static_cast<int64_t>(wg) * 16) = make_uint4(dl[0], dl[1], dl[2], dl[3]);
}

__global__ __launch_bounds__(256) void unpack_storage_kernel(StoreArgs a) {
  const int64_t idx = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
  const int wpr = a.K / 32;
  if (idx >= static_cast<int64_t>(a.M) * wpr) return;
  const int64_t m = idx / wpr;
  const int wg = static_cast<int>(idx - m * wpr);
  const uint32_t* mrow = a.mask + m * a.mask_stride;
  const int wpb = a.B / 32;
  const int bank = wg / wpb;
  int hi_before = 0;  // high channels of the bank in the words before this one
  for (int w = bank * wpb; w < wg; ++w) hi_before += __popc(mrow[w]);
  const uint32_t word = mrow[wg];
  const uint8_t* hsec = a.packed + m * a.row_bytes;
  const uint8_t* lsec = hsec + a.hi_bytes;
  const int in_bank0 = (wg - bank * wpb) * 32;  // channel index inside the bank of this word's first channel
  int8_t* hv = a.hi_val + m * a.K_hi + bank * a.kt;
  uint32_t dl[4] = {0, 0, 0, 0};
  int nh = hi_before;
  for (int i = 0; i < 32; ++i) {
    if ((word >> i) & 1u) {
      if (nh < a.kt) hv[nh] = static_cast<int8_t>(bits_at(hsec, a.hi_bytes, (bank * a.kt + nh) * a.hh, a.hh));
      ++nh;
    } else {
      const int t = bank * (a.B - a.kt) + (in_bank0 + i - nh);
      if (t < a.K_lo) {
        const int code = bits_at(lsec, a.row_bytes - a.hi_bytes, t * a.hl, a.hl);
        dl[i >> 3] |= static_cast<uint32_t>(code & 0xF) << (4 * (i & 7));
      }
    }
  }
  *reinterpret_cast<uint4*>(a.d_lo + m * (a.K / 2) + static_cast<int64_t>(wg) * 16) = make_uint4(dl[0], dl[1], dl[2], dl[3]);
}

}  // namespace

int launch_storage(const sq_params& p, const sq_act& act, uint8_t* packed, bool pack, bool sentinel, hipStream_t st) {
  StoreArgs a;
  a.M = p.M;
  a.K = p.K;
  a.B = p.bank;
  a.kt = p.topk;
  a.G = p.K / p.bank;
  a.hh = p.h_high ? p.h_high : 8;
  a.hl = p.h_low ? p.h_low : 4;
  a.K_hi = a.G * p.topk;
  a.K_lo = p.K - a.K_hi;
  a.hi_bytes = a.K_hi * a.hh / 8;
  a.row_bytes = a.hi_bytes + (sentinel ? p.K : a.K_lo) * a.hl / 8;
  a.sentinel = sentinel ? 1 : 0;
  a.mask_out = act.mask;
  a.mask_stride = p.mode == SQ_STATIC ? 0 : p.K / 32;
  a.mask = act.mask;
  a.d_lo = act.d_lo;
  a.hi_val = act.hi_val;
  a.packed = packed;
  const int64_t total = pack ? static_cast<int64_t>(p.M) * a.row_bytes : static_cast<int64_t>(p.M) * (p.K / 32);
  const unsigned blocks = static_cast<unsigned>((total + 255) / 256);
  if (pack) hipLaunchKernelGGL(pack_storage_kernel, dim3(blocks), dim3(256), 0, st, a);
  else if (sentinel) hipLaunchKernelGGL(unpack_sentinel_kernel, dim3(blocks), dim3(256), 0, st, a);
  else hipLaunchKernelGGL(unpack_storage_kernel, dim3(blocks), dim3(256), 0, st, a);
  return hipGetLastError() == hipSuccess ? SQ_OK : SQ_ERR_LAUNCH;
}

}  // namespace sq
