// sq_linear_noalloc: sq_linear for callers that cannot allocate device memory (code under HIP graph
// capture, tight serving loops, harnesses that forbid hipMalloc).  The workspace sq_linear takes from its
// caller -- the encoded activations between sq_encode and sq_gemm -- lives here in a file-scope device array
// of fixed size instead.  Host code never uses the array's name as an address: every device holds its own
// copy at its own address, looked up once per device with hipGetSymbolAddress and kept in a table.
#include "sq_device.h"

namespace {

__device__ __align__(256) unsigned char scratch[SQ_NOALLOC_SCRATCH_BYTES];

void* g_scratch_of_device[64];  // written under ensure_device_ready's mutex, read after its acquire load

}  // namespace

namespace sq {

int init_scratch(int dev) {
  void* ptr = nullptr;
  if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return SQ_ERR_LAUNCH;
  g_scratch_of_device[dev] = ptr;
  return SQ_OK;
}

}  // namespace sq

extern "C" int sq_linear_noalloc(const sq_params* p, const uint16_t* x_bf16, int64_t ldx, const uint32_t* static_mask,
                                 const sq_weight* w, void* y, int64_t ldy, void* stream) {
  const size_t need = sq_linear_workspace_bytes(p);
  // invalid parameters: let sq_linear name the error (it checks them before it looks at the workspace)
  if (need == 0) return sq_linear(p, x_bf16, ldx, static_mask, w, y, ldy, nullptr, 0, stream);
  if (need > SQ_NOALLOC_SCRATCH_BYTES) return SQ_ERR_SCRATCH;
  int rc = sq::ensure_device_ready();
  if (rc != SQ_OK) return rc;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64 || !g_scratch_of_device[dev]) return SQ_ERR_LAUNCH;
  // Everything sq_gemm reads from the workspace is written by sq_encode of the same call (all M rows of
  // d_lo, hi_val, mask, both scales and hi_dense), so nothing has to start at zero.
  return sq_linear(p, x_bf16, ldx, static_mask, w, y, ldy, g_scratch_of_device[dev], SQ_NOALLOC_SCRATCH_BYTES, stream);
}
