// sq_encode: bf16 activations -> SQ-format (Section 3.1, Eq. (1)); gfx950.
//
// One lane owns one bank of one token row and keeps it in registers.  The per-token
// top-k of the dynamic rule (Sections 3.2.2 / 4.3) is a register-only selection network
// on keys that are unique inside the bank, so that ties in magnitude resolve to the lower
// channel without any extra pass:
//     key = |x| bits (15) << 9  |  (255 - channel_in_bank) << 1  |  sign
// Groups of k keys are sorted, then merged pairwise keeping only the k largest of each
// pair; the largest key ever dropped gives the bank's largest low-precision magnitude.
// The per-token scales need the row maxima of both parts, which the lanes of a row
// combine through LDS integer atomics (bf16 magnitudes order like integers).
// The codes are round-half-even of the fp32 product x * (Q/amax): the rounding is done by
// adding 1.5*2^23, which leaves the two's complement integer in the low mantissa bits.
#include "sq_encode_common.h"

namespace sq {
namespace {

using namespace enc;

// Thread layout shared by both encoders: a block covers R consecutive rows, lane t owns bank
// (t % G) of row (t / G); G = K / bank.  amax_sh[2r], amax_sh[2r+1] = row maxima (bf16 magnitude
// bits) of the high / low part.
struct BankCoord {
  int r_local, g;
  int64_t row;
  bool active;
};
__device__ __forceinline__ BankCoord bank_coord(int G, int R, int M) {
  BankCoord c;
  c.r_local = static_cast<int>(threadIdx.x) / G;
  c.g = static_cast<int>(threadIdx.x) - c.r_local * G;
  c.row = static_cast<int64_t>(blockIdx.x) * R + c.r_local;
  c.active = (c.r_local < R) && (c.row < M);
  return c;
}

template <int B>
__device__ __forceinline__ void load_bank(const uint16_t* __restrict__ x, int64_t ldx, int64_t row, int g, uint32_t* xr) {
  const uint4* src = reinterpret_cast<const uint4*>(x + row * ldx + static_cast<int64_t>(g) * B);
#pragma unroll
  for (int i = 0; i < B / 8; ++i) {
    const uint4 v = src[i];
    xr[4 * i + 0] = v.x;
    xr[4 * i + 1] = v.y;
    xr[4 * i + 2] = v.z;
    xr[4 * i + 3] = v.w;
  }
}

// Dynamic rule (Section 3.1, Eq. (1) with the per-bank top-k mask).  More blocks than the chip holds at
// once are launched for the large shapes, so that the fetches and stores of one block overlap the
// arithmetic of another; a variant in which a block walked over several row groups and fetched the next
// one ahead was slower at every size.
template <int B, int KT, int MAXT>
__global__ __launch_bounds__(MAXT) void encode_dynamic_kernel(const uint16_t* __restrict__ x, int64_t ldx, int M, int K,
                                                              int G, int R, uint8_t* __restrict__ d_lo,
                                                              int8_t* __restrict__ hi_val, uint32_t* __restrict__ mask,
                                                              float* __restrict__ s_lo, float* __restrict__ s_hi,
                                                              int8_t* __restrict__ hi_dense, float q_hi, float q_lo) {
  extern __shared__ __attribute__((aligned(16))) char dense_stage[];  // blockDim * B bytes when hi_dense is set
  static_assert(B % 32 == 0 && KT >= 1 && KT <= 32 && (KT & (KT - 1)) == 0 && B % KT == 0 && B / KT >= 2, "shape");
  __shared__ uint32_t amax_sh[64];
  if (threadIdx.x < 64) amax_sh[threadIdx.x] = 0;
  __syncthreads();
  const BankCoord c = bank_coord(G, R, M);

  uint32_t xr[B / 2];  // the bank: bf16 pairs, channel 2i in the low half of xr[i]
  uint32_t top[KT];    // the k largest keys (unordered)
  if (c.active) {
    load_bank<B>(x, ldx, c.row, c.g, xr);
    uint32_t key[B];
#pragma unroll
    for (int i = 0; i < B / 2; ++i) {
      const uint32_t w = xr[i];
      key[2 * i] = make_key(__builtin_amdgcn_alignbit(w, w, 15), 2 * i);
      key[2 * i + 1] = make_key(__builtin_amdgcn_alignbit(w, w, 31), 2 * i + 1);
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
        uint32_t* a = key + base;
        uint32_t* b = key + base + width;
#pragma unroll
        for (int i = 0; i < KT; ++i) {
          const uint32_t ai = a[i], bj = b[KT - 1 - i];
          a[i] = umax(ai, bj);
          dropped[i] = umax(dropped[i], umin(ai, bj));
        }
        // the survivors form a bitonic sequence; the next merge needs them sorted, the last one only
        // needs the set (the high codes are re-ordered by channel anyway)
        if (2 * width < B) bitonic_merge_desc<KT>(a);
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
    atomicMax(&amax_sh[2 * c.r_local], key_magnitude(tmax));
    atomicMax(&amax_sh[2 * c.r_local + 1], key_magnitude(dmax));
  }
  __syncthreads();
  if (!c.active) return;

  const uint32_t ah = amax_sh[2 * c.r_local], al = amax_sh[2 * c.r_local + 1];
  const float amax_hi = __uint_as_float(ah << 16), amax_lo = __uint_as_float(al << 16);
  const float inv_hi = ah ? q_hi / amax_hi : 0.0f;
  const float inv_lo = al ? q_lo / amax_lo : 0.0f;
  if (c.g == 0) {
    s_hi[c.row] = ah ? amax_hi / q_hi : 1.0f;
    s_lo[c.row] = al ? amax_lo / q_lo : 1.0f;
  }

  // ---- high part: quantise the k selected values, order them by channel, emit codes and mask ----
  uint32_t ent[KT];  // channel << 8 | code byte
  uint32_t mw[B / 32];
#pragma unroll
  for (int w = 0; w < B / 32; ++w) mw[w] = 0;
#pragma unroll
  for (int t = 0; t < KT; ++t) {
    const uint32_t ch = key_channel(top[t]);
    const float v = __fmul_rn(key_value(top[t]), inv_hi);
    const float r = __fadd_rn(v, kRoundMagic);
    ent[t] = (ch << 8) | (__float_as_uint(r) & 0xFFu);
#pragma unroll
    for (int w = 0; w < B / 32; ++w) mw[w] |= ((ch >> 5) == static_cast<uint32_t>(w)) ? (1u << (ch & 31u)) : 0u;
  }
  if (hi_dense) {
    // Matrix-core-ready image of the bank's high part: zeros, then the k codes scattered to their
    // channels (inside every group of 8 channels: the even ones, then the odd ones).  The scatter goes
    // through LDS, where a lane can address bytes dynamically; chunk c of lane t sits at
    // (c * blockDim + t) * 16, an area no other lane touches.
    const int nt = blockDim.x, t = threadIdx.x;
#pragma unroll
    for (int ch16 = 0; ch16 < B / 16; ++ch16)
      *reinterpret_cast<uint4*>(dense_stage + (ch16 * nt + t) * 16) = make_uint4(0, 0, 0, 0);
#pragma unroll
    for (int i = 0; i < KT; ++i) {
      const uint32_t ch = ent[i] >> 8;
      const uint32_t off = (ch & ~7u) | ((ch & 1u) << 2) | ((ch & 7u) >> 1);
      dense_stage[((off >> 4) * nt + t) * 16 + (off & 15u)] = static_cast<char>(ent[i] & 0xFFu);
    }
    uint4* hd = reinterpret_cast<uint4*>(hi_dense + c.row * K + static_cast<int64_t>(c.g) * B);
#pragma unroll
    for (int ch16 = 0; ch16 < B / 16; ++ch16) hd[ch16] = *reinterpret_cast<const uint4*>(dense_stage + (ch16 * nt + t) * 16);
  }
  sort_desc<KT>(ent);  // descending channel; read back reversed
  uint32_t hv[(KT + 3) / 4];
#pragma unroll
  for (int i = 0; i < (KT + 3) / 4; ++i) hv[i] = 0;
#pragma unroll
  for (int t = 0; t < KT; ++t) hv[t / 4] |= (ent[KT - 1 - t] & 0xFFu) << (8 * (t % 4));
  store_bytes<KT>(hi_val + (c.row * G + c.g) * KT, hv);
  uint32_t* mdst = mask + c.row * (K / 32) + static_cast<int64_t>(c.g) * (B / 32);
#pragma unroll
  for (int w = 0; w < B / 32; ++w) mdst[w] = mw[w];

  // ---- low part: every channel quantised, the selected ones cleared ----
  uint32_t dl[B / 8];
#pragma unroll
  for (int j = 0; j < B / 8; ++j) {
    const uint32_t q = quant_lo8(xr + 4 * j, inv_lo);
    const uint32_t clear = spread_bits_to_nibbles(mw[j / 4] >> (8 * (j % 4)));
    dl[j] = q & ~clear;
  }
  uint4* ddst = reinterpret_cast<uint4*>(d_lo + c.row * (K / 2) + static_cast<int64_t>(c.g) * (B / 2));
#pragma unroll
  for (int i = 0; i < B / 32; ++i) ddst[i] = make_uint4(dl[4 * i], dl[4 * i + 1], dl[4 * i + 2], dl[4 * i + 3]);
}

// Static rule (Algorithm 2): the high channels of a bank are the set bits of a channel mask shared by
// all tokens.  kt = bits per bank (validated by the caller of the library when the mask is prepacked).
template <int B, int MAXT>
__global__ __launch_bounds__(MAXT) void encode_static_kernel(const uint16_t* __restrict__ x, int64_t ldx, int M, int K,
                                                             int G, int R, int kt, const uint32_t* __restrict__ cmask,
                                                             uint8_t* __restrict__ d_lo, int8_t* __restrict__ hi_val,
                                                             float* __restrict__ s_lo, float* __restrict__ s_hi,
                                                             float q_hi, float q_lo) {
  __shared__ uint32_t amax_sh[64];
  __shared__ int8_t stage[MAXT * 32];  // per lane: up to 32 high codes in channel order
  if (threadIdx.x < 64) amax_sh[threadIdx.x] = 0;
  __syncthreads();
  const BankCoord c = bank_coord(G, R, M);
  uint32_t xr[B / 2];
  uint32_t mw[B / 32];
  if (c.active) {
    const uint4* src = reinterpret_cast<const uint4*>(x + c.row * ldx + static_cast<int64_t>(c.g) * B);
#pragma unroll
    for (int i = 0; i < B / 8; ++i) {
      const uint4 v = src[i];
      xr[4 * i + 0] = v.x;
      xr[4 * i + 1] = v.y;
      xr[4 * i + 2] = v.z;
      xr[4 * i + 3] = v.w;
    }
#pragma unroll
    for (int w = 0; w < B / 32; ++w) mw[w] = cmask[c.g * (B / 32) + w];
    uint32_t bank_hi = 0, bank_lo = 0;
#pragma unroll
    for (int i = 0; i < B; ++i) {
      const uint32_t w = xr[i / 2];
      const uint32_t mag = (i & 1) ? ((w >> 16) & 0x7FFFu) : (w & 0x7FFFu);
      const bool hi = (mw[i / 32] >> (i % 32)) & 1u;
      bank_hi = umax(bank_hi, hi ? mag : 0u);
      bank_lo = umax(bank_lo, hi ? 0u : mag);
    }
    atomicMax(&amax_sh[2 * c.r_local], bank_hi);
    atomicMax(&amax_sh[2 * c.r_local + 1], bank_lo);
  }
  __syncthreads();
  if (!c.active) return;

  const uint32_t ah = amax_sh[2 * c.r_local], al = amax_sh[2 * c.r_local + 1];
  const float amax_hi = __uint_as_float(ah << 16), amax_lo = __uint_as_float(al << 16);
  const float inv_hi = ah ? q_hi / amax_hi : 0.0f;
  const float inv_lo = al ? q_lo / amax_lo : 0.0f;
  if (c.g == 0) {
    s_hi[c.row] = ah ? amax_hi / q_hi : 1.0f;
    s_lo[c.row] = al ? amax_lo / q_lo : 1.0f;
  }

  int8_t* my = stage + threadIdx.x * 32;
  int cnt = 0;
#pragma unroll
  for (int i = 0; i < B; ++i) {
    const bool hi = (mw[i / 32] >> (i % 32)) & 1u;
    if (hi && cnt < 32) {
      const uint32_t w = xr[i / 2];
      const float xf = __uint_as_float((i & 1) ? (w & 0xFFFF0000u) : (w << 16));
      const float r = __fadd_rn(__fmul_rn(xf, inv_hi), kRoundMagic);
      my[cnt] = static_cast<int8_t>(__float_as_uint(r) & 0xFFu);
      ++cnt;
    }
  }
  int8_t* hdst = hi_val + (c.row * G + c.g) * kt;
  for (int t = 0; t < kt; ++t) hdst[t] = my[t];

  uint32_t dl[B / 8];
#pragma unroll
  for (int j = 0; j < B / 8; ++j) {
    const uint32_t q = quant_lo8(xr + 4 * j, inv_lo);
    const uint32_t clear = spread_bits_to_nibbles(mw[j / 4] >> (8 * (j % 4)));
    dl[j] = q & ~clear;
  }
  uint4* ddst = reinterpret_cast<uint4*>(d_lo + c.row * (K / 2) + static_cast<int64_t>(c.g) * (B / 2));
#pragma unroll
  for (int i = 0; i < B / 32; ++i) ddst[i] = make_uint4(dl[4 * i], dl[4 * i + 1], dl[4 * i + 2], dl[4 * i + 3]);
}

// (hi_val, mask) -> zero-padded INT8 image of the high part.  Inside every group of 8 channels the
// bytes are stored even channels first, then odd channels: the order in which the GEMM kernel's
// nibble widening delivers a weight row.
// d_lo != nullptr (tied scales): the other bytes hold 16 x the low codes instead of zeros.
__global__ __launch_bounds__(256) void expand_hi_kernel(const int8_t* __restrict__ hi_val,
                                                        const uint32_t* __restrict__ mask,
                                                        const uint8_t* __restrict__ d_lo, int64_t total, int K,
                                                        int B, int KT, int mask_rows, int8_t* __restrict__ out) {
  __shared__ uint4 stage[256 * 2];
  const int64_t idx = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
  if (idx >= total) return;
  const int wpr = K / 32;
  const int64_t row = idx / wpr;
  const int wg = static_cast<int>(idx - row * wpr);
  const int wpb = B / 32;
  const int bank = wg / wpb;
  const uint32_t* mrow = mask + (mask_rows ? row * wpr : 0);  // mask_rows == 0: one channel mask for all rows (static)
  int rank = 0;
  for (int w = bank * wpb; w < wg; ++w) rank += __popc(mrow[w]);
  uint32_t word = mrow[wg];
  const int8_t* src = hi_val + (row * (K / B) + bank) * KT + rank;
  uint4* my = stage + threadIdx.x * 2;
  my[0] = make_uint4(0, 0, 0, 0);
  my[1] = make_uint4(0, 0, 0, 0);
  if (d_lo) {  // a nibble moved to the high half of its byte is 16 x the code
    const uint4 d = *reinterpret_cast<const uint4*>(d_lo + row * (K / 2) + static_cast<int64_t>(wg) * 16);
    my[0] = make_uint4((d.x << 4) & 0xF0F0F0F0u, d.x & 0xF0F0F0F0u, (d.y << 4) & 0xF0F0F0F0u, d.y & 0xF0F0F0F0u);
    my[1] = make_uint4((d.z << 4) & 0xF0F0F0F0u, d.z & 0xF0F0F0F0u, (d.w << 4) & 0xF0F0F0F0u, d.w & 0xF0F0F0F0u);
  }
  int8_t* myb = reinterpret_cast<int8_t*>(my);
  int left = KT - rank;  // never read past the bank's codes, whatever the mask holds
  while (word && left > 0) {
    const int e = __ffs(static_cast<int>(word)) - 1;
    word &= word - 1;
    myb[(e & ~7) | ((e & 1) << 2) | ((e & 7) >> 1)] = *src++;
    --left;
  }
  uint4* dst = reinterpret_cast<uint4*>(out + row * K + static_cast<int64_t>(wg) * 32);
  dst[0] = my[0];
  dst[1] = my[1];
}

// Static mode, low part of the reordered weights (Algorithm 2, last step): the columns of the low channels,
// ascending channel order, made contiguous: out [N, K_lo/2], plain nibble order (code 2i in the low nibble of
// byte i) -- the order of sq_act::lo_compact.
__global__ __launch_bounds__(256) void weight_prepack_lo_kernel(int N, int K, int B, int KT,
                                                                const uint8_t* __restrict__ wq,
                                                                const uint32_t* __restrict__ mask,
                                                                uint8_t* __restrict__ out) {
  const int nlo = B - KT;
  const int bytes_per_row = (K / B) * nlo / 2;
  const int64_t idx = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
  if (idx >= static_cast<int64_t>(N) * bytes_per_row) return;
  const int64_t n = idx / bytes_per_row;
  const int byte = static_cast<int>(idx - n * bytes_per_row);
  uint32_t res = 0;
  for (int h = 0; h < 2; ++h) {
    const int t = 2 * byte + h;  // compact low position
    const int bank = t / nlo;
    int r = t % nlo;
    int ch = -1;
    for (int i = 0; i < B; ++i) {
      const int cc = bank * B + i;
      if (!((mask[cc >> 5] >> (cc & 31)) & 1u)) {
        if (r == 0) { ch = cc; break; }
        --r;
      }
    }
    uint32_t code = 0;
    if (ch >= 0) code = (wq[n * (K / 2) + (ch >> 1)] >> ((ch & 1) * 4)) & 0xFu;
    res |= code << (4 * h);
  }
  out[idx] = static_cast<uint8_t>(res);
}

// Number of banks of a channel mask that do not hold exactly KT bits -> *bad (one workgroup).
__global__ __launch_bounds__(256) void mask_check_kernel(int G, int B, int KT, const uint32_t* __restrict__ mask,
                                                         int32_t* __restrict__ bad) {
  __shared__ int total;
  if (threadIdx.x == 0) total = 0;
  __syncthreads();
  int mine = 0;
  for (int g = threadIdx.x; g < G; g += 256) {
    int c = 0;
    for (int w = 0; w < B / 32; ++w) c += __popc(mask[g * (B / 32) + w]);
    mine += c != KT;
  }
  if (mine) atomicAdd(&total, mine);
  __syncthreads();
  if (threadIdx.x == 0) *bad = total;
}

// Static mode: compact copy of the high channels' weight columns.  Output row n holds k_hi_padded
// codes (zero beyond (K/B)*KT); byte j of every group of 8 codes (4 bytes) carries code j in its low and
// code j+4 in its high nibble, so that the GEMM kernel's nibble widening yields the codes in natural order.
__global__ __launch_bounds__(256) void weight_prepack_kernel(int N, int K, int B, int KT, int k_hi_padded,
                                                             const uint8_t* __restrict__ wq,
                                                             const uint32_t* __restrict__ mask,
                                                             uint8_t* __restrict__ out) {
  const int64_t idx = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
  const int bytes_per_row = k_hi_padded / 2;
  if (idx >= static_cast<int64_t>(N) * bytes_per_row) return;
  const int64_t n = idx / bytes_per_row;
  const int byte = static_cast<int>(idx - n * bytes_per_row);
  const int grp = byte / 4, j = byte % 4;
  const int k_hi = mask ? (K / B) * KT : K;
  uint32_t res = 0;
  for (int h = 0; h < 2; ++h) {
    const int t = grp * 8 + j + 4 * h;  // index into the compact list of high channels
    uint32_t code = 0;
    if (!mask) {  // every channel, in order (plain W4A8 reference)
      code = (wq[n * (K / 2) + (t >> 1)] >> ((t & 1) * 4)) & 0xFu;
    } else if (t < k_hi) {
      const int bank = t / KT;
      int r = t % KT;
      int ch = -1;
      for (int i = 0; i < B; ++i) {
        const int cc = bank * B + i;
        if ((mask[cc >> 5] >> (cc & 31)) & 1u) {
          if (r == 0) { ch = cc; break; }
          --r;
        }
      }
      if (ch >= 0) code = (wq[n * (K / 2) + (ch >> 1)] >> ((ch & 1) * 4)) & 0xFu;
    }
    res |= code << (4 * h);
  }
  out[idx] = static_cast<uint8_t>(res);
}

template <int B, int KT, int MAXT>
int launch_dyn_t(const sq_params& p, const uint16_t* x, int64_t ldx, const sq_act& o, hipStream_t st, int G, int R,
                 int threads, int blocks) {
  // up to MAXT * B bytes; the limit of every instantiation was raised by init_encode_kernels
  const size_t lds = o.hi_dense ? static_cast<size_t>(threads) * B : 0;
  hipLaunchKernelGGL((encode_dynamic_kernel<B, KT, MAXT>), dim3(blocks), dim3(threads), lds, st, x, ldx, p.M, p.K, G, R,
                     o.d_lo, o.hi_val, o.mask, o.scale_lo, o.scale_hi, o.hi_dense, code_max(p.h_high, 8), code_max(p.h_low, 4));
  return hipGetLastError() == hipSuccess ? SQ_OK : SQ_ERR_LAUNCH;
}

template <int B, int KT>
int launch_dyn(const sq_params& p, const uint16_t* x, int64_t ldx, const sq_act& o, hipStream_t st) {
  const int G = p.K / B;
  int R = 256 / G;
  if (R < 1) R = 1;
  if (R > 32) R = 32;
  const int threads = ((R * G + 63) / 64) * 64;
  const int blocks = (p.M + R - 1) / R;
  if (threads <= 256) return launch_dyn_t<B, KT, 256>(p, x, ldx, o, st, G, R, threads, blocks);
  return launch_dyn_t<B, KT, 512>(p, x, ldx, o, st, G, R, threads, blocks);
}

template <int B>
int launch_stat(const sq_params& p, const uint16_t* x, int64_t ldx, const uint32_t* mask, const sq_act& o,
                hipStream_t st) {
  const int G = p.K / B;
  int R = 256 / G;
  if (R < 1) R = 1;
  if (R > 32) R = 32;
  const int threads = ((R * G + 63) / 64) * 64;
  const int blocks = (p.M + R - 1) / R;
  if (threads <= 256) {
    hipLaunchKernelGGL((encode_static_kernel<B, 256>), dim3(blocks), dim3(threads), 0, st, x, ldx, p.M, p.K, G, R,
                       p.topk, mask, o.d_lo, o.hi_val, o.scale_lo, o.scale_hi, code_max(p.h_high, 8), code_max(p.h_low, 4));
  } else {
    hipLaunchKernelGGL((encode_static_kernel<B, 512>), dim3(blocks), dim3(threads), 0, st, x, ldx, p.M, p.K, G, R,
                       p.topk, mask, o.d_lo, o.hi_val, o.scale_lo, o.scale_hi, code_max(p.h_high, 8), code_max(p.h_low, 4));
  }
  return hipGetLastError() == hipSuccess ? SQ_OK : SQ_ERR_LAUNCH;
}

template <int B, int KT, int MAXT>
hipError_t raise_encode_lds_limit() {
  return hipFuncSetAttribute(reinterpret_cast<const void*>(encode_dynamic_kernel<B, KT, MAXT>),
                             hipFuncAttributeMaxDynamicSharedMemorySize, MAXT * B);
}

}  // namespace

// Long rows with bank 128 need more dynamic LDS for the hi_dense staging than the default limit: raised here
// for every instantiation, once per device (library initialisation, never on the launch path).
int init_encode_kernels() {
  hipError_t e = hipSuccess;
#define SQ_CASE(B, KT)                                                        \
  if (e == hipSuccess) e = raise_encode_lds_limit<B, KT, 256>();              \
  if (e == hipSuccess) e = raise_encode_lds_limit<B, KT, 512>();
  SQ_CASE(32, 2) SQ_CASE(32, 4) SQ_CASE(32, 8) SQ_CASE(32, 16)
  SQ_CASE(64, 4) SQ_CASE(64, 8) SQ_CASE(64, 16) SQ_CASE(64, 32)
  SQ_CASE(128, 8) SQ_CASE(128, 16) SQ_CASE(128, 32)
#undef SQ_CASE
  if (e != hipSuccess) return SQ_ERR_LAUNCH;
  const int rc = init_encode_stream_kernels();
  return rc != SQ_OK ? rc : init_encode_static_kernels();
}

int launch_encode_dynamic(const sq_params& p, const uint16_t* x, int64_t ldx, const sq_act& out, hipStream_t st) {
  // Rows whose bank count is a power of two up to 64, or 64 / 128 / 256, take the streaming kernel; the
  // kernel below covers every other K / bank <= 512 (checked by the caller).
  if (encode_stream_supports(p))
    return launch_encode_stream(p, x, ldx, out, out.hi_dense, false, code_max(p.h_high, 8), code_max(p.h_low, 4), st);
#define SQ_CASE(B, KT) \
  if (p.bank == B && p.topk == KT) return launch_dyn<B, KT>(p, x, ldx, out, st);
  SQ_CASE(32, 2) SQ_CASE(32, 4) SQ_CASE(32, 8) SQ_CASE(32, 16)
  SQ_CASE(64, 4) SQ_CASE(64, 8) SQ_CASE(64, 16) SQ_CASE(64, 32)
  SQ_CASE(128, 8) SQ_CASE(128, 16) SQ_CASE(128, 32)
#undef SQ_CASE
  return SQ_ERR_UNSUPPORTED;
}

int launch_encode_static(const sq_params& p, const uint16_t* x, int64_t ldx, const uint32_t* mask, const sq_act& out,
                         hipStream_t st) {
  // rows that fit in LDS take the row-staged kernel (which can also write the reordered low part); the kernel
  // below covers the longer ones (dense low part only: the caller has checked that no lo_compact is asked for)
  if (encode_static_gather_supports(p)) return launch_encode_static_gather(p, x, ldx, mask, out, st);
  if (p.bank == 32) return launch_stat<32>(p, x, ldx, mask, out, st);
  if (p.bank == 64) return launch_stat<64>(p, x, ldx, mask, out, st);
  if (p.bank == 128) return launch_stat<128>(p, x, ldx, mask, out, st);
  return SQ_ERR_UNSUPPORTED;
}

int launch_expand_hi(const sq_params& p, const sq_act& a, int8_t* s_hi_dense, hipStream_t st) {
  const int64_t total = static_cast<int64_t>(p.M) * (p.K / 32);
  const int64_t blocks = (total + 255) / 256;
  hipLaunchKernelGGL(expand_hi_kernel, dim3(static_cast<unsigned>(blocks)), dim3(256), 0, st, a.hi_val, a.mask,
                     p.mode == SQ_DYNAMIC_TIED ? a.d_lo : nullptr, total, p.K, p.bank, p.topk, p.mode == SQ_STATIC ? 0 : 1,
                     s_hi_dense);
  return hipGetLastError() == hipSuccess ? SQ_OK : SQ_ERR_LAUNCH;
}

int launch_weight_prepack(int N, int K, int bank, int topk, int k_hi_padded, const uint8_t* wq, const uint32_t* mask,
                          uint8_t* out, hipStream_t st) {
  const int64_t total = static_cast<int64_t>(N) * (k_hi_padded / 2);
  const int64_t blocks = (total + 255) / 256;
  hipLaunchKernelGGL(weight_prepack_kernel, dim3(static_cast<unsigned>(blocks)), dim3(256), 0, st, N, K, bank, topk,
                     k_hi_padded, wq, mask, out);
  return hipGetLastError() == hipSuccess ? SQ_OK : SQ_ERR_LAUNCH;
}

int launch_weight_prepack_lo(int N, int K, int bank, int topk, const uint8_t* wq, const uint32_t* mask, uint8_t* out,
                             hipStream_t st) {
  const int64_t total = static_cast<int64_t>(N) * ((K / bank) * (bank - topk) / 2);
  const int64_t blocks = (total + 255) / 256;
  hipLaunchKernelGGL(weight_prepack_lo_kernel, dim3(static_cast<unsigned>(blocks)), dim3(256), 0, st, N, K, bank, topk,
                     wq, mask, out);
  return hipGetLastError() == hipSuccess ? SQ_OK : SQ_ERR_LAUNCH;
}

int launch_mask_check(int K, int bank, int topk, const uint32_t* mask, int32_t* bad, hipStream_t st) {
  hipLaunchKernelGGL(mask_check_kernel, dim3(1), dim3(256), 0, st, K / bank, bank, topk, mask, bad);
  return hipGetLastError() == hipSuccess ? SQ_OK : SQ_ERR_LAUNCH;
}

}  // namespace sq
