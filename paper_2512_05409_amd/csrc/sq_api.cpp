// C ABI of libsq: argument checks, workspace carving and kernel dispatch.  No allocation, no
// synchronisation; every entry point only enqueues work on the caller's stream.
#include <string.h>

#include <atomic>
#include <mutex>

#include "sq_device.h"

namespace sq {

// The only process-wide state of the library: one flag per device saying that the kernels' dynamic-LDS
// limits have been raised and the scratch array of sq_linear_noalloc has been located there (and, with it,
// the device's number of compute units, which the encoders size their grids by).
static int g_compute_units[64];  // written once per device under the mutex below, read after the acquire load

int device_compute_units() {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64 || g_compute_units[dev] <= 0) return 256;
  return g_compute_units[dev];
}

int ensure_device_ready() {
  static std::atomic<int> ready[64];
  static std::mutex mu;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return SQ_ERR_LAUNCH;
  if (ready[dev].load(std::memory_order_acquire)) return SQ_OK;
  std::lock_guard<std::mutex> lock(mu);
  if (ready[dev].load(std::memory_order_relaxed)) return SQ_OK;
  int cus = 0;
  if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && cus > 0) g_compute_units[dev] = cus;
  int rc = init_gemm_kernels();
  if (rc == SQ_OK) rc = init_encode_kernels();
  if (rc == SQ_OK) rc = init_scratch(dev);
  if (rc == SQ_OK) rc = init_wsq_kernels();
  if (rc == SQ_OK) ready[dev].store(1, std::memory_order_release);
  return rc;
}

}  // namespace sq

namespace {

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline bool pow2(int v) { return v > 0 && (v & (v - 1)) == 0; }

int check_params(const sq_params* p) {
  if (!p) return SQ_ERR_NULL;
  if (p->M <= 0 || p->K <= 0 || p->N <= 0) return SQ_ERR_SHAPE;
  if (p->bank != 32 && p->bank != 64 && p->bank != 128) return SQ_ERR_UNSUPPORTED;
  if (p->K % p->bank || p->K % 64 || p->K > 131072) return SQ_ERR_SHAPE;
  if (p->K / p->bank > 512) return SQ_ERR_SHAPE;
  if (p->M > (1 << 22) || p->N > (1 << 24)) return SQ_ERR_SHAPE;
  if (p->mode != SQ_DYNAMIC && p->mode != SQ_STATIC && p->mode != SQ_DYNAMIC_TIED) return SQ_ERR_UNSUPPORTED;
  if (p->out_dtype != SQ_OUT_F32 && p->out_dtype != SQ_OUT_BF16) return SQ_ERR_UNSUPPORTED;
  if (!pow2(p->topk) || p->topk > 32 || p->topk * 2 > p->bank) return SQ_ERR_UNSUPPORTED;
  if (p->mode != SQ_STATIC && p->topk * 16 < p->bank) return SQ_ERR_UNSUPPORTED;  // s in {1/2,3/4,7/8,15/16}
  if (p->mode == SQ_DYNAMIC_TIED && !sq::encode_stream_supports(*p)) return SQ_ERR_UNSUPPORTED;
  if (p->mode == SQ_STATIC && ((p->K / p->bank) * p->topk) % 32) return SQ_ERR_UNSUPPORTED;
  {  // precision pair (Section 4.1): 0/0 = 8/4, or one of 8/4, 8/3, 8/2, 4/2
    const int hh = p->h_high ? p->h_high : 8, hl = p->h_low ? p->h_low : 4;
    const bool ok = (hh == 8 && (hl == 4 || hl == 3 || hl == 2)) || (hh == 4 && hl == 2);
    if (!ok) return SQ_ERR_UNSUPPORTED;
    if (p->mode == SQ_DYNAMIC_TIED && !(hh == 8 && hl == 4)) return SQ_ERR_UNSUPPORTED;
  }
  return SQ_OK;
}

inline int k_hi_of(const sq_params* p) { return (p->K / p->bank) * p->topk; }
// Static mode with a handful of tokens: the layer is bound by streaming the weights once, which the
// weight-streaming decode kernel does about twice as fast as the generic small tile; it takes the dense low part
// and a zero-padded image of the high part (built from hi_val and the channel mask), i.e. the dynamic operands.
inline bool static_decode(const sq_params* p) { return p->mode == SQ_STATIC && p->M <= 32 && p->K % 128 == 0; }
inline size_t lo_compact_bytes(const sq_params* p) { return static_cast<size_t>(p->M) * ((p->K - k_hi_of(p)) / 2); }

struct ActLayout {
  size_t d_lo, hi_val, mask, scale, total;
};
ActLayout act_layout(const sq_params* p) {
  ActLayout l;
  l.d_lo = static_cast<size_t>(p->M) * (p->K / 2);
  l.hi_val = static_cast<size_t>(p->M) * k_hi_of(p);
  l.mask = p->mode != SQ_STATIC ? static_cast<size_t>(p->M) * (p->K / 32) * 4 : static_cast<size_t>(p->K / 32) * 4;
  l.scale = static_cast<size_t>(p->M) * 4;
  l.total = l.d_lo + l.hi_val + l.mask + 2 * l.scale;
  return l;
}

int check_act(const sq_params* p, const sq_act* a) {
  if (!a || !a->hi_val || !a->mask || !a->scale_lo || !a->scale_hi) return SQ_ERR_NULL;
  if (!a->d_lo && !(p->mode == SQ_STATIC && a->lo_compact)) return SQ_ERR_NULL;
  if (!aligned16(a->d_lo) || !aligned16(a->hi_val) || !aligned16(a->mask) || !aligned16(a->scale_lo) ||
      !aligned16(a->scale_hi) || !aligned16(a->hi_dense) || !aligned16(a->lo_compact))
    return SQ_ERR_ALIGN;
  return SQ_OK;
}

int check_weight(const sq_params* p, const sq_weight* w) {
  if (!w || !w->wq || !w->scale) return SQ_ERR_NULL;
  if (p->mode == SQ_STATIC && !w->prepacked) return SQ_ERR_NULL;
  if (!aligned16(w->wq) || !aligned16(w->scale) || (w->prepacked && !aligned16(w->prepacked))) return SQ_ERR_ALIGN;
  return SQ_OK;
}

int check_y(const sq_params* p, const void* y, int64_t ldy) {
  if (!y) return SQ_ERR_NULL;
  if (ldy < p->N) return SQ_ERR_SHAPE;
  if (!aligned16(y)) return SQ_ERR_ALIGN;
  return SQ_OK;
}

}  // namespace

extern "C" {

int sq_init(void) { return sq::ensure_device_ready(); }

const char* sq_gemm_variant(const sq_params* p) {
  if (check_params(p) != SQ_OK) return "invalid";
  return sq::gemm_variant_name(p->M, p->N, p->K, p->mode == SQ_DYNAMIC, p->mode == SQ_DYNAMIC_TIED);
}

size_t sq_act_bytes(const sq_params* p, size_t* d_lo, size_t* hi_val, size_t* mask, size_t* scale) {
  if (check_params(p) != SQ_OK) return 0;
  const ActLayout l = act_layout(p);
  if (d_lo) *d_lo = l.d_lo;
  if (hi_val) *hi_val = l.hi_val;
  if (mask) *mask = l.mask;
  if (scale) *scale = l.scale;
  return l.total;
}

size_t sq_gemm_workspace_bytes(const sq_params* p) {
  if (check_params(p) != SQ_OK) return 0;
  if (p->mode != SQ_STATIC || static_decode(p)) return align_up(static_cast<size_t>(p->M) * p->K, 256);
  return 16;
}

size_t sq_lo_compact_bytes(const sq_params* p) {
  if (check_params(p) != SQ_OK || p->mode != SQ_STATIC) return 0;
  return lo_compact_bytes(p);
}

size_t sq_linear_workspace_bytes(const sq_params* p) {
  if (check_params(p) != SQ_OK) return 0;
  const ActLayout l = act_layout(p);
  const bool compact = p->mode == SQ_STATIC && sq::encode_static_gather_supports(*p) && !static_decode(p);
  size_t t = align_up(compact ? lo_compact_bytes(p) : l.d_lo, 256) + align_up(l.hi_val, 256) + 2 * align_up(l.scale, 256);
  if (static_decode(p)) t += align_up(static_cast<size_t>(p->M) * p->K, 256);
  if (p->mode != SQ_STATIC) t += align_up(l.mask, 256) + align_up(static_cast<size_t>(p->M) * p->K, 256);
  return t;
}

size_t sq_weight_prepack_bytes(const sq_params* p) {
  if (check_params(p) != SQ_OK || p->mode != SQ_STATIC) return 0;
  return static_cast<size_t>(p->N) * (p->K / 2);
}

int sq_weight_prepack(const sq_params* p, const uint8_t* wq, const uint32_t* static_mask_host,
                      const uint32_t* static_mask, void* out, int32_t* bad_banks, void* stream) {
  int rc = check_params(p);
  if (rc != SQ_OK) return rc;
  if (p->mode != SQ_STATIC) return SQ_ERR_UNSUPPORTED;
  if (!wq || !static_mask || !out) return SQ_ERR_NULL;
  if (!aligned16(wq) || !aligned16(out) || !aligned16(static_mask)) return SQ_ERR_ALIGN;
  for (int g = 0; static_mask_host && g < p->K / p->bank; ++g) {
    int c = 0;
    for (int i = 0; i < p->bank; ++i) {
      const int j = g * p->bank + i;
      c += (static_mask_host[j >> 5] >> (j & 31)) & 1u;
    }
    if (c != p->topk) return SQ_ERR_MASK;
  }
  if ((rc = sq::ensure_device_ready()) != SQ_OK) return rc;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (bad_banks && (rc = sq::launch_mask_check(p->K, p->bank, p->topk, static_mask, bad_banks, st)) != SQ_OK) return rc;
  uint8_t* o = static_cast<uint8_t*>(out);
  rc = sq::launch_weight_prepack(p->N, p->K, p->bank, p->topk, k_hi_of(p), wq, static_mask, o, st);
  if (rc != SQ_OK) return rc;
  return sq::launch_weight_prepack_lo(p->N, p->K, p->bank, p->topk, wq, static_mask,
                                      o + static_cast<size_t>(p->N) * (k_hi_of(p) / 2), st);
}

size_t sq_calibrate_workspace_bytes(const sq_params* p, int64_t T) {
  if (check_params(p) != SQ_OK || p->mode != SQ_STATIC || T <= 0 || T > (1 << 24)) return 0;
  int ca, ra, cw, rw;
  sq::calibrate_chunks(T, p->N, &ca, &ra, &cw, &rw);
  return (static_cast<size_t>(ca) + cw + 1) * p->K * sizeof(double);
}

int sq_calibrate_static(const sq_params* p, const uint16_t* x_calib, int64_t ldx, int64_t T, const sq_weight* w,
                        uint32_t* mask_out, double* importance_out, void* workspace, size_t workspace_bytes,
                        void* stream) {
  int rc = check_params(p);
  if (rc != SQ_OK) return rc;
  if (p->mode != SQ_STATIC) return SQ_ERR_UNSUPPORTED;
  if (!x_calib || !w || !w->wq || !w->scale || !mask_out) return SQ_ERR_NULL;
  if (T <= 0 || T > (1 << 24) || ldx < p->K) return SQ_ERR_SHAPE;
  if (!aligned16(x_calib) || (ldx % 8) || !aligned16(w->wq) || !aligned16(w->scale) || !aligned16(mask_out) ||
      !aligned16(importance_out))
    return SQ_ERR_ALIGN;
  const size_t need = sq_calibrate_workspace_bytes(p, T);
  if (!workspace || workspace_bytes < need) return SQ_ERR_WORKSPACE;
  if (!aligned16(workspace)) return SQ_ERR_ALIGN;
  if ((rc = sq::ensure_device_ready()) != SQ_OK) return rc;
  int ca, ra, cw, rw;
  sq::calibrate_chunks(T, p->N, &ca, &ra, &cw, &rw);
  double* pa = static_cast<double*>(workspace);
  double* pw = pa + static_cast<size_t>(ca) * p->K;
  double* imp = importance_out ? importance_out : pw + static_cast<size_t>(cw) * p->K;
  return sq::launch_calibrate_static(*p, x_calib, ldx, T, w->wq, w->scale, mask_out, imp, pa, pw,
                                     static_cast<hipStream_t>(stream));
}

int sq_encode(const sq_params* p, const uint16_t* x_bf16, int64_t ldx, const uint32_t* static_mask, const sq_act* out,
              void* stream) {
  int rc = check_params(p);
  if (rc != SQ_OK) return rc;
  if (!x_bf16) return SQ_ERR_NULL;
  if (ldx < p->K) return SQ_ERR_SHAPE;
  if (!aligned16(x_bf16) || (ldx % 8)) return SQ_ERR_ALIGN;
  if (p->mode == SQ_STATIC) {
    if (!static_mask) return SQ_ERR_UNSUPPORTED;
    if (!out || (!out->d_lo && !out->lo_compact) || !out->hi_val || !out->scale_lo || !out->scale_hi) return SQ_ERR_NULL;
    if (!aligned16(out->d_lo) || !aligned16(out->hi_val) || !aligned16(static_mask) || !aligned16(out->lo_compact))
      return SQ_ERR_ALIGN;
    if (out->lo_compact && !sq::encode_static_gather_supports(*p)) return SQ_ERR_UNSUPPORTED;
    if ((rc = sq::ensure_device_ready()) != SQ_OK) return rc;
    return sq::launch_encode_static(*p, x_bf16, ldx, static_mask, *out, static_cast<hipStream_t>(stream));
  }
  rc = check_act(p, out);
  if (rc != SQ_OK) return rc;
  if ((rc = sq::ensure_device_ready()) != SQ_OK) return rc;
  if (p->mode == SQ_DYNAMIC_TIED)
    return sq::launch_encode_stream(*p, x_bf16, ldx, *out, out->hi_dense, true, 127.0f, 7.0f, static_cast<hipStream_t>(stream));  // (8/4) only
  return sq::launch_encode_dynamic(*p, x_bf16, ldx, *out, static_cast<hipStream_t>(stream));
}

int sq_gemm(const sq_params* p, const sq_act* a, const sq_weight* w, void* y, int64_t ldy, int32_t* acc_lo_dbg,
            int32_t* acc_hi_dbg, void* workspace, size_t workspace_bytes, void* stream) {
  int rc = check_params(p);
  if (rc != SQ_OK) return rc;
  if ((rc = check_act(p, a)) != SQ_OK) return rc;
  if ((rc = check_weight(p, w)) != SQ_OK) return rc;
  if ((rc = check_y(p, y, ldy)) != SQ_OK) return rc;
  const bool need_ws = p->mode != SQ_STATIC && !a->hi_dense;
  if (need_ws && (!workspace || workspace_bytes < sq_gemm_workspace_bytes(p))) return SQ_ERR_WORKSPACE;
  if (need_ws && !aligned16(workspace)) return SQ_ERR_ALIGN;
  if ((rc = sq::ensure_device_ready()) != SQ_OK) return rc;
  hipStream_t st = static_cast<hipStream_t>(stream);

  sq::GemmArgs g;
  memset(&g, 0, sizeof g);
  g.M = p->M;
  g.N = p->N;
  g.K = p->K;
  g.a_lo = a->d_lo;
  g.K_lo = p->K;
  g.wq = w->wq;
  g.w_lo = w->wq;
  g.s_lo = a->scale_lo;
  g.s_hi = a->scale_hi;
  g.s_w = w->scale;
  g.y = y;
  g.ldy = ldy;
  g.out_bf16 = p->out_dtype == SQ_OUT_BF16;
  g.acc_lo_dbg = acc_lo_dbg;
  g.acc_hi_dbg = acc_hi_dbg;
  if (p->mode != SQ_STATIC) {
    const int8_t* image = a->hi_dense;
    if (!image) {
      rc = sq::launch_expand_hi(*p, *a, static_cast<int8_t*>(workspace), st);
      if (rc != SQ_OK) return rc;
      image = static_cast<const int8_t*>(workspace);
    }
    if (p->mode == SQ_DYNAMIC) {
      g.a_hi_dense = image;
    } else {
      // tied scales: one product of the combined INT8 operand (stored in the order the plain weight rows
      // unfold to) with the weights as they are, scaled by s_hi
      g.a_lo = nullptr;
      g.s_lo = nullptr;
      g.K_hi = p->K;
      g.a_hi_compact = image;
      g.lda_hi_compact = p->K;
      g.w_hi = w->wq;
    }
  } else if (static_decode(p) && a->d_lo && workspace && workspace_bytes >= sq_gemm_workspace_bytes(p) && aligned16(workspace)) {
    // few tokens: the dynamic operands (see static_decode); optional -- without a workspace the generic tile runs
    rc = sq::launch_expand_hi(*p, *a, static_cast<int8_t*>(workspace), st);
    if (rc != SQ_OK) return rc;
    g.a_hi_dense = static_cast<const int8_t*>(workspace);
  } else {
    g.K_hi = k_hi_of(p);
    g.a_hi_compact = a->hi_val;
    g.lda_hi_compact = g.K_hi;
    g.w_hi = static_cast<const uint8_t*>(w->prepacked);
    if (a->lo_compact) {  // both operands reordered by the mask: the low product skips the high channels
      g.a_lo = a->lo_compact;
      g.K_lo = p->K - g.K_hi;
      g.w_lo = g.w_hi + static_cast<size_t>(p->N) * (g.K_hi / 2);
    }
  }
  return sq::launch_gemm(g, st);
}

int sq_linear(const sq_params* p, const uint16_t* x_bf16, int64_t ldx, const uint32_t* static_mask, const sq_weight* w,
              void* y, int64_t ldy, void* workspace, size_t workspace_bytes, void* stream) {
  int rc = check_params(p);
  if (rc != SQ_OK) return rc;
  if (!workspace || workspace_bytes < sq_linear_workspace_bytes(p)) return SQ_ERR_WORKSPACE;
  if (reinterpret_cast<uintptr_t>(workspace) & 255u) return SQ_ERR_ALIGN;
  if (p->mode == SQ_STATIC && !static_mask) return SQ_ERR_UNSUPPORTED;
  // checked here so that a bad weight / output argument cannot leave a half-done call behind
  if ((rc = check_weight(p, w)) != SQ_OK) return rc;
  if ((rc = check_y(p, y, ldy)) != SQ_OK) return rc;
  const ActLayout l = act_layout(p);
  char* ws = static_cast<char*>(workspace);
  sq_act a;
  memset(&a, 0, sizeof a);
  if (p->mode == SQ_STATIC && sq::encode_static_gather_supports(*p) && !static_decode(p)) {
    a.lo_compact = reinterpret_cast<uint8_t*>(ws);
    ws += align_up(lo_compact_bytes(p), 256);
  } else {
    a.d_lo = reinterpret_cast<uint8_t*>(ws);
    ws += align_up(l.d_lo, 256);
  }
  a.hi_val = reinterpret_cast<int8_t*>(ws);
  ws += align_up(l.hi_val, 256);
  a.scale_lo = reinterpret_cast<float*>(ws);
  ws += align_up(l.scale, 256);
  a.scale_hi = reinterpret_cast<float*>(ws);
  ws += align_up(l.scale, 256);
  a.hi_dense = nullptr;
  if (p->mode != SQ_STATIC) {
    a.mask = reinterpret_cast<uint32_t*>(ws);
    ws += align_up(l.mask, 256);
    a.hi_dense = reinterpret_cast<int8_t*>(ws);
    ws += align_up(static_cast<size_t>(p->M) * p->K, 256);
  } else {
    a.mask = const_cast<uint32_t*>(static_mask);
  }
  void* gemm_ws = nullptr;
  size_t gemm_ws_bytes = 0;
  if (static_decode(p)) {
    gemm_ws = ws;
    gemm_ws_bytes = align_up(static_cast<size_t>(p->M) * p->K, 256);
  }
  rc = sq_encode(p, x_bf16, ldx, static_mask, &a, stream);
  if (rc != SQ_OK) return rc;
  return sq_gemm(p, &a, w, y, ldy, nullptr, nullptr, gemm_ws, gemm_ws_bytes, stream);
}

size_t sq_storage_row_bytes(const sq_params* p) {
  if (check_params(p) != SQ_OK) return 0;
  const int hh = p->h_high ? p->h_high : 8, hl = p->h_low ? p->h_low : 4;
  return static_cast<size_t>(k_hi_of(p)) * hh / 8 + static_cast<size_t>(p->K - k_hi_of(p)) * hl / 8;
}

size_t sq_storage_row_bytes_sentinel(const sq_params* p) {
  if (check_params(p) != SQ_OK || p->mode == SQ_STATIC) return 0;
  const int hh = p->h_high ? p->h_high : 8, hl = p->h_low ? p->h_low : 4;
  return static_cast<size_t>(k_hi_of(p)) * hh / 8 + static_cast<size_t>(p->K) * hl / 8;
}

static int storage_call(const sq_params* p, const sq_act* a, uint8_t* packed, bool pack, bool sentinel, void* stream) {
  int rc = check_params(p);
  if (rc != SQ_OK) return rc;
  if (sentinel && p->mode == SQ_STATIC) return SQ_ERR_UNSUPPORTED;  // a shared channel mask needs no sentinels
  if (!a || !a->d_lo || !a->hi_val || !a->mask || !packed) return SQ_ERR_NULL;
  if (!aligned16(a->d_lo) || !aligned16(a->hi_val) || !aligned16(a->mask)) return SQ_ERR_ALIGN;
  if ((rc = sq::ensure_device_ready()) != SQ_OK) return rc;
  return sq::launch_storage(*p, *a, packed, pack, sentinel, static_cast<hipStream_t>(stream));
}

int sq_pack_storage(const sq_params* p, const sq_act* a, uint8_t* packed, void* stream) {
  return storage_call(p, a, packed, true, false, stream);
}

int sq_unpack_storage(const sq_params* p, const uint8_t* packed, const sq_act* a, void* stream) {
  return storage_call(p, a, const_cast<uint8_t*>(packed), false, false, stream);
}

int sq_pack_storage_sentinel(const sq_params* p, const sq_act* a, uint8_t* packed, void* stream) {
  return storage_call(p, a, packed, true, true, stream);
}

int sq_unpack_storage_sentinel(const sq_params* p, const uint8_t* packed, const sq_act* a, void* stream) {
  return storage_call(p, a, const_cast<uint8_t*>(packed), false, true, stream);
}

// ---- SQ-format on weights ----
static int check_wsq_params(const sq_params* p) {
  if (!p) return SQ_ERR_NULL;
  if (p->M <= 0 || p->K <= 0 || p->N <= 0) return SQ_ERR_SHAPE;
  if (p->bank != 64 && p->bank != 128) return SQ_ERR_UNSUPPORTED;
  if (p->K % p->bank || p->K > 131072 || p->M > (1 << 22) || p->N > (1 << 24)) return SQ_ERR_SHAPE;
  if (p->topk < 1 || p->topk > p->bank) return SQ_ERR_UNSUPPORTED;
  if (p->out_dtype != SQ_OUT_F32 && p->out_dtype != SQ_OUT_BF16) return SQ_ERR_UNSUPPORTED;
  const int hh = p->h_high ? p->h_high : 8, hl = p->h_low ? p->h_low : 4;
  if (!((hh == 8 && (hl == 4 || hl == 3 || hl == 2)) || (hh == 4 && hl == 2))) return SQ_ERR_UNSUPPORTED;
  return SQ_OK;
}

static int check_wsq(const sq_wsq* w) {
  if (!w || !w->lo || !w->hi_val || !w->scale_lo || !w->scale_hi) return SQ_ERR_NULL;
  if (!aligned16(w->lo) || !aligned16(w->hi_val) || !aligned16(w->scale_lo) || !aligned16(w->scale_hi)) return SQ_ERR_ALIGN;
  return SQ_OK;
}

size_t sq_wsq_bytes(const sq_params* p, size_t* lo, size_t* hi_val, size_t* scale) {
  if (check_wsq_params(p) != SQ_OK) return 0;
  const size_t G = p->K / p->bank;
  const size_t l = static_cast<size_t>(p->N) * (p->K / 2), h = static_cast<size_t>(p->N) * G * p->topk, s = static_cast<size_t>(p->N) * G * 4;
  if (lo) *lo = l;
  if (hi_val) *hi_val = h;
  if (scale) *scale = s;
  return l + h + 2 * s;
}

int sq_wsq_encode(const sq_params* p, const uint16_t* w_bf16, int64_t ldw, const float* hinv_diag, const sq_wsq* out,
                  void* stream) {
  int rc = check_wsq_params(p);
  if (rc != SQ_OK) return rc;
  if (!w_bf16) return SQ_ERR_NULL;
  if ((rc = check_wsq(out)) != SQ_OK) return rc;
  if (ldw < p->K) return SQ_ERR_SHAPE;
  if ((rc = sq::ensure_device_ready()) != SQ_OK) return rc;
  return sq::launch_wsq_encode(*p, w_bf16, ldw, hinv_diag, *out, static_cast<hipStream_t>(stream));
}

static size_t wsq_scales_t_bytes(const sq_params* p) {  // one transposed, padded scale array
  return static_cast<size_t>(p->K / p->bank) * ((p->N + 127) / 128 * 128) * 4;
}

size_t sq_wsq_prepack_bytes(const sq_params* p) {
  if (check_wsq_params(p) != SQ_OK) return 0;
  return static_cast<size_t>(p->N) * (p->K / 2) + static_cast<size_t>(p->N) * p->K + 2 * wsq_scales_t_bytes(p);
}

int sq_wsq_prepack(const sq_params* p, const sq_wsq* w, void* out, void* stream) {
  int rc = check_wsq_params(p);
  if (rc != SQ_OK) return rc;
  if ((rc = check_wsq(w)) != SQ_OK) return rc;
  if (!out) return SQ_ERR_NULL;
  if (!aligned16(out)) return SQ_ERR_ALIGN;
  if ((rc = sq::ensure_device_ready()) != SQ_OK) return rc;
  uint8_t* o = static_cast<uint8_t*>(out);
  uint8_t* hd = o + static_cast<size_t>(p->N) * (p->K / 2);
  uint8_t* sl = hd + static_cast<size_t>(p->N) * p->K;
  return sq::launch_wsq_prepack(*p, *w, o, reinterpret_cast<int8_t*>(hd), reinterpret_cast<float*>(sl),
                                reinterpret_cast<float*>(sl + wsq_scales_t_bytes(p)), static_cast<hipStream_t>(stream));
}

int sq_quantize_act(const sq_params* p, const uint16_t* x_bf16, int64_t ldx, int bits, int8_t* a8, float* a_scale,
                    void* stream) {
  if (!p || !x_bf16 || !a8 || !a_scale) return SQ_ERR_NULL;
  if (p->M <= 0 || p->K <= 0 || p->K % 64 || p->K > 131072 || ldx < p->K) return SQ_ERR_SHAPE;
  if (bits != 8 && bits != 4) return SQ_ERR_UNSUPPORTED;
  if (!aligned16(x_bf16) || (ldx % 8) || !aligned16(a8)) return SQ_ERR_ALIGN;
  int rc = sq::ensure_device_ready();
  if (rc != SQ_OK) return rc;
  return sq::launch_quantize_act(*p, x_bf16, ldx, bits, a8, a_scale, static_cast<hipStream_t>(stream));
}

int sq_wsq_gemm(const sq_params* p, const int8_t* a8, const float* a_scale, const sq_wsq* w, const void* prepacked, void* y,
                int64_t ldy, int32_t* acc_lo_dbg, int32_t* acc_hi_dbg, void* stream) {
  int rc = check_wsq_params(p);
  if (rc != SQ_OK) return rc;
  if (!a8 || !a_scale || !prepacked) return SQ_ERR_NULL;
  if ((rc = check_wsq(w)) != SQ_OK) return rc;
  if ((rc = check_y(p, y, ldy)) != SQ_OK) return rc;
  if (!aligned16(a8) || !aligned16(prepacked)) return SQ_ERR_ALIGN;
  if ((rc = sq::ensure_device_ready()) != SQ_OK) return rc;
  const uint8_t* o = static_cast<const uint8_t*>(prepacked);
  const uint8_t* hd = o + static_cast<size_t>(p->N) * (p->K / 2);
  const uint8_t* sl = hd + static_cast<size_t>(p->N) * p->K;
  return sq::launch_wsq_gemm(*p, a8, a_scale, *w, o, reinterpret_cast<const int8_t*>(hd), reinterpret_cast<const float*>(sl),
                             reinterpret_cast<const float*>(sl + wsq_scales_t_bytes(p)), y, ldy, acc_lo_dbg, acc_hi_dbg,
                             static_cast<hipStream_t>(stream));
}

size_t sq_wsq_linear_workspace_bytes(const sq_params* p) {
  if (check_wsq_params(p) != SQ_OK) return 0;
  return align_up(static_cast<size_t>(p->M) * p->K, 256) + align_up(static_cast<size_t>(p->M) * 4, 256);
}

int sq_wsq_linear(const sq_params* p, const uint16_t* x_bf16, int64_t ldx, int act_bits, const sq_wsq* w,
                  const void* prepacked, void* y, int64_t ldy, void* workspace, size_t workspace_bytes, void* stream) {
  int rc = check_wsq_params(p);
  if (rc != SQ_OK) return rc;
  if (!workspace || workspace_bytes < sq_wsq_linear_workspace_bytes(p)) return SQ_ERR_WORKSPACE;
  if (reinterpret_cast<uintptr_t>(workspace) & 255u) return SQ_ERR_ALIGN;
  if ((rc = check_wsq(w)) != SQ_OK) return rc;
  if (!prepacked) return SQ_ERR_NULL;
  if ((rc = check_y(p, y, ldy)) != SQ_OK) return rc;
  int8_t* a8 = static_cast<int8_t*>(workspace);
  float* sa = reinterpret_cast<float*>(static_cast<char*>(workspace) + align_up(static_cast<size_t>(p->M) * p->K, 256));
  if ((rc = sq_quantize_act(p, x_bf16, ldx, act_bits, a8, sa, stream)) != SQ_OK) return rc;
  return sq_wsq_gemm(p, a8, sa, w, prepacked, y, ldy, nullptr, nullptr, stream);
}

int sq_dense_w4a8_prepack(const sq_params* p, const uint8_t* wq, void* out, void* stream) {
  if (!p || !wq || !out) return SQ_ERR_NULL;
  if (p->K <= 0 || p->N <= 0 || p->K % 64 || p->K > 131072) return SQ_ERR_SHAPE;
  if (!aligned16(wq) || !aligned16(out)) return SQ_ERR_ALIGN;
  return sq::launch_weight_prepack(p->N, p->K, 0, 0, p->K, wq, nullptr, static_cast<uint8_t*>(out),
                                   static_cast<hipStream_t>(stream));
}

int sq_dense_w4a8_gemm(const sq_params* p, const int8_t* a_i8, const float* a_scale, const sq_weight* w, void* y,
                       int64_t ldy, void* stream) {
  if (!p) return SQ_ERR_NULL;
  if (p->M <= 0 || p->K <= 0 || p->N <= 0 || p->K % 64 || p->K > 131072) return SQ_ERR_SHAPE;
  if (p->out_dtype != SQ_OUT_F32 && p->out_dtype != SQ_OUT_BF16) return SQ_ERR_UNSUPPORTED;
  if (!a_i8 || !a_scale || !w || !w->scale || !w->prepacked) return SQ_ERR_NULL;
  int rc = check_y(p, y, ldy);
  if (rc != SQ_OK) return rc;
  if (!aligned16(a_i8) || !aligned16(w->prepacked)) return SQ_ERR_ALIGN;
  if ((rc = sq::ensure_device_ready()) != SQ_OK) return rc;
  sq::GemmArgs g;
  memset(&g, 0, sizeof g);
  g.M = p->M;
  g.N = p->N;
  g.K = p->K;
  g.K_hi = p->K;
  g.a_hi_compact = a_i8;
  g.lda_hi_compact = p->K;
  g.w_hi = static_cast<const uint8_t*>(w->prepacked);
  g.s_hi = a_scale;
  g.s_w = w->scale;
  g.y = y;
  g.ldy = ldy;
  g.out_bf16 = p->out_dtype == SQ_OUT_BF16;
  return sq::launch_gemm(g, static_cast<hipStream_t>(stream));
}

const char* sq_status_string(int status) {
  switch (status) {
    case SQ_OK: return "SQ_OK";
    case SQ_ERR_NULL: return "SQ_ERR_NULL: a required pointer is NULL";
    case SQ_ERR_SHAPE: return "SQ_ERR_SHAPE: bad M/K/N, K not a multiple of bank and 64, or leading dimension too small";
    case SQ_ERR_UNSUPPORTED: return "SQ_ERR_UNSUPPORTED: bank/topk/mode/out_dtype outside the supported set";
    case SQ_ERR_ALIGN: return "SQ_ERR_ALIGN: pointer or leading dimension not 16-byte aligned";
    case SQ_ERR_LAUNCH: return "SQ_ERR_LAUNCH: the HIP runtime refused a launch";
    case SQ_ERR_MASK: return "SQ_ERR_MASK: a bank of the static mask does not hold exactly topk bits";
    case SQ_ERR_WORKSPACE: return "SQ_ERR_WORKSPACE: workspace missing or too small";
    case SQ_ERR_SCRATCH: return "SQ_ERR_SCRATCH: the problem needs more than the built-in scratch of sq_linear_noalloc";
    default: return "unknown sq_status";
  }
}

const char* sq_version(void) { return "0.1"; }

}  // extern "C"
