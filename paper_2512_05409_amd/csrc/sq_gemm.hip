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
// A K step of 128 channels is copied into one of three LDS stages by LDS-direct loads, two steps
// ahead of its use.  LDS rows are row-major with the 16-byte chunk index XOR-swizzled by the row,
// which keeps the operand reads (32 consecutive rows per half wave) free of bank conflicts.
#include "sq_device.h"

namespace sq {
namespace {

typedef unsigned int v4u __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int KS = 128;  // channels per K step
#ifndef SQ_HUGE_MIN_TILES
#define SQ_HUGE_MIN_TILES 512
#endif
constexpr int kHugeMinTiles = SQ_HUGE_MIN_TILES;
  // 256x256 tiles a single-product shape needs to use them
constexpr int NT = 256;  // threads per workgroup

// WITH_LO = false: a tile for loops without a packed low operand (the single-product modes), whose stage
// holds no room for one; that is what lets 256 tokens x 256 channels fit three stages into LDS.
// NS: LDS stages of the K loop.  The copy of step kt + NS - 1 is enqueued while step kt is multiplied, so a copy
// has NS - 2 whole K steps to land before anything waits for it.
template <int BM_, int BN_, bool WITH_LO = true, int NS_ = 3>
struct Tile {
  static constexpr int NS = NS_;
  static constexpr int BM = BM_;              // tokens per workgroup
  static constexpr int BN = BN_;              // output channels per workgroup
  static constexpr int WM = BM / 2;           // tokens per wave (waves are 2 x 2)
  static constexpr int WN = BN / 2;           // channels per wave
  static constexpr int TI = WM / 32;          // 32-row tiles per wave along M
  static constexpr int TJ = WN / 32;          // along N
  static constexpr int A_LO = 0;              // [BM][64 B]   packed INT4
  static constexpr int A_HI = WITH_LO ? BM * 64 : 0;  // [BM][128 B]  INT8
  static constexpr int B_OFF = A_HI + BM * 128;  // [BN][64 B] packed INT4
  static constexpr int STAGE = B_OFF + BN * 64;
  static constexpr int LDS_BYTES = NS * STAGE;
  static_assert(NS >= 3 && LDS_BYTES <= 160 * 1024, "stages must fit in the 160 KB of LDS");
};

// Byte offset of 16-byte chunk c of a row inside an operand tile.
__device__ __forceinline__ int off4(int row, int c) { return (row << 6) + (((c ^ (row >> 2)) & 3) << 4); }   // 4 chunks / row
__device__ __forceinline__ int off8(int row, int c) { return (row << 7) + (((c ^ (row >> 1)) & 7) << 4); }   // 8 chunks / row

// 16 zero bytes in device memory: the source of operand chunks that lie past the end of K.
__device__ __attribute__((aligned(16))) const unsigned int kZeroChunk[4] = {0u, 0u, 0u, 0u};

typedef __attribute__((address_space(3))) void* lds_ptr_t;

// s_waitcnt immediate (gfx9 encoding: vmcnt[3:0] | expcnt[6:4] | lgkmcnt[11:8] | vmcnt_hi[15:14]):
// at most n vector-memory operations (here: LDS-direct loads) outstanding, and no LDS operation.
constexpr int waitcnt_vm_lgkm0(int n) { return (n & 15) | (7 << 4) | (0 << 8) | ((n >> 4) << 14); }

// Workgroup barrier for the K loop.  __syncthreads() would also wait for every outstanding
// LDS-direct load (its release fence drains vmcnt), i.e. for the copy that was enqueued a moment
// ago for two steps ahead.  Here the wave waits only until at most `pending` of its loads are in
// flight (loads retire in order, so the older step is complete) and until its own LDS reads have
// returned, then joins the barrier.  The empty asm statements stop the compiler from moving
// memory accesses across it.
template <int PENDING>
__device__ __forceinline__ void pipeline_barrier() {
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(PENDING));
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

// Operand sources of one K loop and the asynchronous copy of one K step into an LDS stage.
// LO: the packed low part is an operand; HI: an INT8 operand (the zero-padded image of the high
// part, or the compact high codes) is.  The copy uses LDS-direct loads (global_load_lds_dwordx4):
// each wave instruction moves 64 x 16 bytes into 1 KB of LDS, lane l landing at byte 16*l, so the
// XOR swizzle is applied on the global side: the lane that lands in position p of a row fetches
// chunk p ^ swizzle(row).  Four (or eight) consecutive lanes still read 64 (128) contiguous bytes.
template <typename T, bool LO, bool HI>
struct Pipe {
  static constexpr int N_LO = LO ? T::BM * 4 / NT : 0;
  static constexpr int N_HI = HI ? T::BM * 8 / NT : 0;
  static constexpr int N_B = T::BN * 4 / NT;
  static constexpr int NLOAD = N_LO + N_HI + N_B;  // loads per wave per K step

  const char* p_lo[N_LO > 0 ? N_LO : 1];  // per-lane source of each load at k = 0
  const char* p_hi[N_HI > 0 ? N_HI : 1];
  const char* p_b[N_B];
  int kc_lo, kc_hi;  // first channel of this lane's chunk inside a K step (packed operands / INT8 operand)
  int kext;          // channels in this loop (multiple of 32)
  int wave;          // uniform

  __device__ __forceinline__ void init(const uint8_t* a_lo, int64_t lda_lo, const int8_t* a_hi, int64_t lda_hi,
                                       const uint8_t* b, int64_t ldb, int kext_, int m0, int n0, int M, int N) {
    const int tid = threadIdx.x;
    kext = kext_;
    wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    {
      const int row = tid >> 2;  // rows of later loads differ by a multiple of 64: same swizzle
      kc_lo = (((tid & 3) ^ (row >> 2)) & 3) * 32;
    }
    {
      const int row = tid >> 3;  // rows of later loads differ by a multiple of 32
      kc_hi = (((tid & 7) ^ (row >> 1)) & 7) * 16;
    }
#pragma unroll
    for (int i = 0; i < N_LO; ++i) {
      const int m = min(m0 + ((tid + NT * i) >> 2), M - 1);
      p_lo[i] = reinterpret_cast<const char*>(a_lo) + m * lda_lo + (kc_lo >> 1);
    }
#pragma unroll
    for (int i = 0; i < N_HI; ++i) {
      const int m = min(m0 + ((tid + NT * i) >> 3), M - 1);
      p_hi[i] = reinterpret_cast<const char*>(a_hi) + m * lda_hi + kc_hi;
    }
#pragma unroll
    for (int i = 0; i < N_B; ++i) {
      const int n = min(n0 + ((tid + NT * i) >> 2), N - 1);
      p_b[i] = reinterpret_cast<const char*>(b) + n * ldb + (kc_lo >> 1);
    }
  }

  // Enqueue the copy of K step `step` into `stage`.  TAIL: the step may reach past kext (only the last
  // step of a loop can); its chunks past the end come from kZeroChunk.
  template <bool TAIL>
  __device__ __forceinline__ void issue(char* stage, int step) const {
    const int k0 = step * KS;
    const char* zero = reinterpret_cast<const char*>(kZeroChunk);
    const bool lo_ok = !TAIL || (k0 + kc_lo < kext);
    const bool hi_ok = !TAIL || (k0 + kc_hi < kext);
#pragma unroll
    for (int i = 0; i < N_LO; ++i) {
      const char* src = lo_ok ? p_lo[i] + (k0 >> 1) : zero;
      __builtin_amdgcn_global_load_lds(src, (lds_ptr_t)(stage + T::A_LO + (NT * i + 64 * wave) * 16), 16, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < N_HI; ++i) {
      const char* src = hi_ok ? p_hi[i] + k0 : zero;
      __builtin_amdgcn_global_load_lds(src, (lds_ptr_t)(stage + T::A_HI + (NT * i + 64 * wave) * 16), 16, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < N_B; ++i) {
      const char* src = lo_ok ? p_b[i] + (k0 >> 1) : zero;
      __builtin_amdgcn_global_load_lds(src, (lds_ptr_t)(stage + T::B_OFF + (NT * i + 64 * wave) * 16), 16, 0, 0);
    }
  }
};

// The operands one wave needs for 64 channels (two matrix instructions deep) of its tile.
template <typename T>
struct Frags {
  v4u alo[T::TI];     // packed low codes: 32 channels per row tile
  v4u bw[T::TJ];      // packed weight codes
  v4i ahi[T::TI][2];  // INT8 high codes, one 16-byte operand per matrix instruction
};

template <typename T, bool LO, bool HI>
__device__ __forceinline__ void read_frags(Frags<T>& f, const char* stage, int g, int wm, int wn, int lane) {
  const int r = lane & 31, h = lane >> 5;
#pragma unroll
  for (int j = 0; j < T::TJ; ++j)
    f.bw[j] = *reinterpret_cast<const v4u*>(stage + T::B_OFF + off4(wn * T::WN + j * 32 + r, 2 * g + h));
#pragma unroll
  for (int i = 0; i < T::TI; ++i) {
    const int row = wm * T::WM + i * 32 + r;
    if (LO) f.alo[i] = *reinterpret_cast<const v4u*>(stage + T::A_LO + off4(row, 2 * g + h));
    if (HI) {
      f.ahi[i][0] = *reinterpret_cast<const v4i*>(stage + T::A_HI + off8(row, 4 * g + 2 * h));
      f.ahi[i][1] = *reinterpret_cast<const v4i*>(stage + T::A_HI + off8(row, 4 * g + 2 * h + 1));
    }
  }
}

// Half s (0/1) of a packed chunk (16 of its 32 INT4 codes) -> the INT8 operand of matrix instruction s.
__device__ __forceinline__ v4i widen(const v4u p, int s) {
  const unsigned a = p[2 * s], b = p[2 * s + 1];
  return v4i{static_cast<int>((a << 4) & 0xF0F0F0F0u), static_cast<int>(a & 0xF0F0F0F0u),
             static_cast<int>((b << 4) & 0xF0F0F0F0u), static_cast<int>(b & 0xF0F0F0F0u)};
}

// Widened operands of one 32-channel slice of the fragments.
template <typename T>
struct Wide {
  v4i bw[T::TJ];
  v4i alo[T::TI];
};

template <typename T, bool LO>
__device__ __forceinline__ void widen_slice(Wide<T>& w, const Frags<T>& f, int s) {
#pragma unroll
  for (int j = 0; j < T::TJ; ++j) w.bw[j] = widen(f.bw[j], s);
  if (LO) {
#pragma unroll
    for (int i = 0; i < T::TI; ++i) w.alo[i] = widen(f.alo[i], s);
  }
}

// The matrix instructions of one 32-channel slice (s = 0/1): 2 * TI * TJ of them, all independent.
template <typename T, bool LO, bool HI>
__device__ __forceinline__ void mma_slice(const Wide<T>& w, const Frags<T>& f, int s, v16i (&acc_lo)[T::TI][T::TJ],
                                          v16i (&acc_hi)[T::TI][T::TJ]) {
#pragma unroll
  for (int i = 0; i < T::TI; ++i) {
#pragma unroll
    for (int j = 0; j < T::TJ; ++j) {
      if (LO) acc_lo[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(w.alo[i], w.bw[j], acc_lo[i][j], 0, 0, 0);
      if (HI) acc_hi[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(f.ahi[i][s], w.bw[j], acc_hi[i][j], 0, 0, 0);
    }
  }
}

// Scheduling recipe for one slice: every matrix instruction is followed by a few of the other
// instructions of the region (a wave issues in order, so whatever is not tucked behind a matrix
// instruction leaves the matrix pipeline idle).  VMEM / DS: how many of the first slots also take
// one LDS-direct load / one LDS read.
template <int NMFMA, int VALU, int SALU, int VMEM, int DS>
__device__ __forceinline__ void interleave() {
#pragma unroll
  for (int k = 0; k < NMFMA; ++k) {
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
    if (VALU) __builtin_amdgcn_sched_group_barrier(0x002, VALU, 0);
    if (SALU) __builtin_amdgcn_sched_group_barrier(0x004, SALU, 0);
    if (k < VMEM) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
    if (k < DS) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
  }
}

// One iteration of the K loop (see k_loop): four slices of 32 channels.  While the matrix
// instructions of a slice run, the operands of the following slice are widened, and the packed
// operands of the slice after that are fetched from LDS, so nothing a matrix instruction needs was
// requested less than a slice (about 500 cycles) earlier.
//   on entry: f0 = fragments of (step kt, channels 0-63), w0 = its slice 0, widened
//   slice A: multiply w0     | fetch f1 = (step kt, channels 64-127), widen f0 slice 1 -> w1
//   slice B: multiply w1     | enqueue the copy of step kt+2, widen f1 slice 0 -> w0
//   barrier (step kt+1 is complete in LDS, step kt's stage may be overwritten)
//   slice C: multiply w0     | fetch f0 = (step kt+1, channels 0-63), widen f1 slice 1 -> w1
//   slice D: multiply w1     | widen f0 slice 0 -> w0
// FILL: 0 = nothing to copy, 1 = the copy of step kt + NS - 1 is enqueued, 2 = the same and that step may be
// partial; ALLOW: K steps whose copies may still be in flight at the barrier (those after step kt+1);
// NEXT: step kt+1 exists.
template <typename T, bool LO, bool HI, int FILL, int ALLOW, bool NEXT>
__device__ __forceinline__ void k_iteration(const Pipe<T, LO, HI>& pipe, char* lds, int kt, int st_cur, int wm, int wn,
                                            int lane, Frags<T>& f0, Frags<T>& f1, Wide<T>& w0, Wide<T>& w1,
                                            v16i (&acc_lo)[T::TI][T::TJ], v16i (&acc_hi)[T::TI][T::TJ]) {
  constexpr int NL = Pipe<T, LO, HI>::NLOAD;
  constexpr int NM = (LO ? 1 : 0) * T::TI * T::TJ + (HI ? 1 : 0) * T::TI * T::TJ;  // matrix instructions per slice
  constexpr int NR = T::TJ + (LO ? T::TI : 0) + (HI ? 2 * T::TI : 0);               // LDS reads per fragment set
  const int st_next = st_cur == T::NS - 1 ? 0 : st_cur + 1;
  const int st_fill = st_cur == 0 ? T::NS - 1 : st_cur - 1;  // the stage of step kt - 1, read for the last time before the previous barrier
  // slice A
  read_frags<T, LO, HI>(f1, lds + st_cur * T::STAGE, 1, wm, wn, lane);
  widen_slice<T, LO>(w1, f0, 1);
  mma_slice<T, LO, HI>(w0, f0, 0, acc_lo, acc_hi);
  interleave<NM, 4, 0, 0, NR>();
  __builtin_amdgcn_sched_barrier(0);
  // slice B
  if (FILL == 1) pipe.template issue<false>(lds + st_fill * T::STAGE, kt + T::NS - 1);
  if (FILL == 2) pipe.template issue<true>(lds + st_fill * T::STAGE, kt + T::NS - 1);
  widen_slice<T, LO>(w0, f1, 0);
  mma_slice<T, LO, HI>(w1, f0, 1, acc_lo, acc_hi);
  interleave<NM, 6, 3, FILL ? NL : 0, 0>();
  __builtin_amdgcn_sched_barrier(0);
  pipeline_barrier<ALLOW * NL>();
  // slice C
  if (NEXT) read_frags<T, LO, HI>(f0, lds + st_next * T::STAGE, 0, wm, wn, lane);
  widen_slice<T, LO>(w1, f1, 1);
  mma_slice<T, LO, HI>(w0, f1, 0, acc_lo, acc_hi);
  interleave<NM, 4, 0, 0, NEXT ? NR : 0>();
  __builtin_amdgcn_sched_barrier(0);
  // slice D
  if (NEXT) widen_slice<T, LO>(w0, f0, 0);
  mma_slice<T, LO, HI>(w1, f1, 1, acc_lo, acc_hi);
  interleave<NM, 3, 0, 0, 0>();
  __builtin_amdgcn_sched_barrier(0);
}

// K loop over NS LDS stages: the copy of step kt + NS - 1 is enqueued while step kt is multiplied; every wave
// waits for its own copy of step kt+1 in the middle of iteration kt (younger copies stay in flight), the
// workgroup meets at a barrier, and the matrix pipeline has operands in registers on both sides of it (see
// k_iteration).  The last NS iterations are peeled so that the steady-state body has no branches.
// Safety: the stage overwritten by the copy of step kt + NS - 1 held step kt-1, last read before the
// barrier of iteration kt-1, and every wave drains its LDS reads (lgkmcnt 0) before that barrier.
// k_loop_start enqueues the first NS - 1 steps; k_loop expects them enqueued (whatever independent work the
// caller has goes between the two calls, under the latency of those first copies).
template <typename T, bool LO, bool HI>
__device__ __forceinline__ void k_loop_start(const Pipe<T, LO, HI>& pipe, char* lds, int st0 = 0) {
  pipe.template issue<true>(lds + st0 * T::STAGE, 0);
#pragma unroll
  for (int s0 = 1; s0 < T::NS - 1; ++s0)
    if (pipe.kext > s0 * KS) pipe.template issue<true>(lds + ((st0 + s0) % T::NS) * T::STAGE, s0);
}

// The last iterations of a K loop, peeled: with R steps left after the current one, the iteration that still
// enqueues a copy (R == NS - 1: the last step, which may be partial), then the ones that only drain.
template <typename T, bool LO, bool HI, int R>
__device__ __forceinline__ void k_loop_tail(const Pipe<T, LO, HI>& pipe, char* lds, int steps, int& kt, int& st, int wm, int wn,
                                            int lane, Frags<T>& f0, Frags<T>& f1, Wide<T>& w0, Wide<T>& w1,
                                            v16i (&acc_lo)[T::TI][T::TJ], v16i (&acc_hi)[T::TI][T::TJ]) {
  constexpr int D = T::NS - 1;
  if (steps - 1 - kt == R) {
    constexpr int FILL = R == D ? 2 : 0;
    constexpr int ALLOW = R == D ? D - 1 : (R > 0 ? R - 1 : 0);
    k_iteration<T, LO, HI, FILL, ALLOW, (R > 0)>(pipe, lds, kt, st, wm, wn, lane, f0, f1, w0, w1, acc_lo, acc_hi);
    st = st == T::NS - 1 ? 0 : st + 1;
    ++kt;
  }
  if constexpr (R > 0) k_loop_tail<T, LO, HI, R - 1>(pipe, lds, steps, kt, st, wm, wn, lane, f0, f1, w0, w1, acc_lo, acc_hi);
}

template <int N, int NL>
__device__ __forceinline__ void first_barrier(int in_flight) {  // in_flight steps enqueued, step 0 must have landed
  if constexpr (N > 1) {
    if (in_flight >= N) {
      pipeline_barrier<(N - 1) * NL>();
      return;
    }
    first_barrier<N - 1, NL>(in_flight);
  } else {
    pipeline_barrier<0>();
  }
}

template <typename T, bool LO, bool HI>
__device__ __forceinline__ void k_loop(const Pipe<T, LO, HI>& pipe, char* lds, int wm, int wn, int lane,
                                       v16i (&acc_lo)[T::TI][T::TJ], v16i (&acc_hi)[T::TI][T::TJ], int st0 = 0) {
  constexpr int NL = Pipe<T, LO, HI>::NLOAD;
  constexpr int D = T::NS - 1;
  const int steps = (pipe.kext + KS - 1) / KS;
  first_barrier<D, NL>(steps < D ? steps : D);
  Frags<T> f0, f1;
  Wide<T> w0, w1;
  read_frags<T, LO, HI>(f0, lds + st0 * T::STAGE, 0, wm, wn, lane);
  widen_slice<T, LO>(w0, f0, 0);
  int st = st0, kt = 0;
  for (; kt + D + 1 < steps; ++kt) {  // steady state: copies of full steps only, D - 1 steps in flight at the barrier
    k_iteration<T, LO, HI, 1, D - 1, true>(pipe, lds, kt, st, wm, wn, lane, f0, f1, w0, w1, acc_lo, acc_hi);
    st = st == T::NS - 1 ? 0 : st + 1;
  }
  k_loop_tail<T, LO, HI, D>(pipe, lds, steps, kt, st, wm, wn, lane, f0, f1, w0, w1, acc_lo, acc_hi);
  __syncthreads();  // the stages are reused by the next loop / the epilogue
}

// fp32 -> bf16, round to nearest even (v_cvt_pk_bf16_f32).
__device__ __forceinline__ uint16_t bf16_rne(float f) { return __builtin_bit_cast(uint16_t, static_cast<__bf16>(f)); }

// Orders this wave's LDS writes before its later LDS reads of other lanes' data (compiler barrier +
// wait for the wave's outstanding LDS operations); no other wave is involved.
__device__ __forceinline__ void wave_lds_fence() {
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_waitcnt((15) | (7 << 4) | (0 << 8) | (3 << 14));  // lgkmcnt(0)
  asm volatile("" ::: "memory");
}

// Maps the linear workgroup id to a tile so that (a) the workgroups resident on one XCD at a time
// (ids congruent mod 8 go to the same XCD) cover a compact 4 x 8 patch of tiles and share operand
// tiles in that XCD's L2, and (b) every XCD walks its own contiguous range of the tile order.
__device__ __forceinline__ void tile_of_block(int id, int tiles_m, int tiles_n, int& tm, int& tn) {
  const int total = tiles_m * tiles_n;
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
// The scales a thread contributes to the epilogue, fetched at the start of the kernel so that their
// latency hides under the K loop.
template <typename T>
struct EpiScales {
  float slo, shi;    // thread t < BM: s_lo and s_hi of row m0 + t
  float sw[T::TJ];   // s_w of this lane's column in each of the wave's 32-column tiles
};

template <typename T>
__device__ __forceinline__ void load_epi_scales(EpiScales<T>& e, const GemmArgs& g, int m0, int n0, int wn, int lane) {
  const int tid = threadIdx.x;
  const int m = min(m0 + (tid < T::BM ? tid : 0), g.M - 1);
  e.slo = g.s_lo ? g.s_lo[m] : 0.0f;
  e.shi = g.s_hi[m];
#pragma unroll
  for (int j = 0; j < T::TJ; ++j) {
    const int n = n0 + wn * T::WN + j * 32 + (lane & 31);
    e.sw[j] = g.s_w[min(n, g.N - 1)];
  }
}

template <typename T, typename OutT>
__device__ __forceinline__ void epilogue_typed(const GemmArgs& g, const EpiScales<T>& es, char* lds,
                                               v16i (&acc_lo)[T::TI][T::TJ], v16i (&acc_hi)[T::TI][T::TJ], int m0, int n0,
                                               int wm, int wn, int wave, int lane) {
  constexpr int ESZ = sizeof(OutT);
  constexpr int ROW = T::WN * ESZ + 16;   // padded row of the transposition buffer (bytes)
  constexpr int PER16 = 16 / ESZ;         // outputs per 16-byte store
  constexpr int CHUNKS = T::WN / PER16;   // 16-byte chunks per row
  constexpr int ROWS_PER_PASS = 64 / CHUNKS;
  constexpr int SC_BYTES = 2 * T::BM * 4;  // [0, BM): s_lo, [BM, 2 BM): s_hi
  static_assert(SC_BYTES + 4 * 32 * ROW <= T::LDS_BYTES, "transposition buffers must fit in the stage memory");
  const int tid = threadIdx.x;
  float* sc = reinterpret_cast<float*>(lds);
  char* tb = lds + SC_BYTES + wave * (32 * ROW);
  if (tid < T::BM) {
    sc[tid] = es.slo;
    sc[T::BM + tid] = es.shi;
  }
  // workgroup barrier without the memory fence of __syncthreads(): only LDS traffic has to be ordered here
  pipeline_barrier<63>();
  const bool vec_ok = (g.ldy % PER16) == 0;  // rows of Y stay 16-byte aligned
  OutT* yout = reinterpret_cast<OutT*>(g.y);
#pragma unroll
  for (int i = 0; i < T::TI; ++i) {
#pragma unroll
    for (int rq = 0; rq < 4; ++rq) {
      const int rl0 = 8 * rq + 4 * (lane >> 5);  // 4 consecutive rows of the 32: registers 4 rq + e
      // (clang vector types, not HIP's float4: the compiler orders reads of the latter after every LDS-direct
      // load in flight with a full vmcnt(0) wait)
      const f32x4 slo4 = *reinterpret_cast<const f32x4*>(sc + wm * T::WM + i * 32 + rl0);
      const f32x4 shi4 = *reinterpret_cast<const f32x4*>(sc + T::BM + wm * T::WM + i * 32 + rl0);
      const float slo[4] = {slo4[0], slo4[1], slo4[2], slo4[3]};
      const float shi[4] = {shi4[0], shi4[1], shi4[2], shi4[3]};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
#pragma unroll
        for (int j = 0; j < T::TJ; ++j) {
          // the accumulators carry the widening factors 256 and 16: shifted out exactly, as integers
          float t = __fmul_rn(static_cast<float>(acc_lo[i][j][4 * rq + e] >> 8), slo[e]);
          t = __fmaf_rn(static_cast<float>(acc_hi[i][j][4 * rq + e] >> 4), shi[e], t);
          const float y = __fmul_rn(t, es.sw[j]);
          OutT* dst = reinterpret_cast<OutT*>(tb + (rl0 + e) * ROW) + j * 32 + (lane & 31);
          if constexpr (ESZ == 2) *dst = bf16_rne(y);
          else *dst = y;
        }
      }
    }
    wave_lds_fence();  // the buffer is private to the wave: its LDS operations execute in order
#pragma unroll
    for (int pass = 0; pass < 32 / ROWS_PER_PASS; ++pass) {
      const int rl = pass * ROWS_PER_PASS + lane / CHUNKS, ch = lane % CHUNKS;
      const int m = m0 + wm * T::WM + i * 32 + rl;
      const int n = n0 + wn * T::WN + ch * PER16;
      if (m < g.M && n < g.N) {
        OutT* dst = yout + static_cast<int64_t>(m) * g.ldy + n;
        if (vec_ok && n + PER16 <= g.N) {
          // streaming store (nt): Y is written once and not read by this kernel; measured 2 % on the
          // single-product kernel, neutral on the two-product one.  Written as asm, so the two idle slots a
          // wide store needs before its data registers may be overwritten are added by hand.
          const v4u vv = *reinterpret_cast<const v4u*>(tb + rl * ROW + ch * 16);
          asm volatile("global_store_dwordx4 %0, %1, off nt\n\ts_nop 1" ::"v"(dst), "v"(vv) : "memory");
        } else {  // ragged right edge or unaligned rows: element by element, straight from LDS
          const OutT* src = reinterpret_cast<const OutT*>(tb + rl * ROW + ch * 16);
          for (int q = 0; q < PER16 && n + q < g.N; ++q) dst[q] = src[q];
        }
      }
    }
    wave_lds_fence();
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
__device__ __forceinline__ void epilogue(const GemmArgs& g, const EpiScales<T>& es, char* lds,
                                         v16i (&acc_lo)[T::TI][T::TJ], v16i (&acc_hi)[T::TI][T::TJ], int m0, int n0, int wm,
                                         int wn, int wave, int lane) {
  if (g.out_bf16) epilogue_typed<T, uint16_t>(g, es, lds, acc_lo, acc_hi, m0, n0, wm, wn, wave, lane);
  else epilogue_typed<T, float>(g, es, lds, acc_lo, acc_hi, m0, n0, wm, wn, wave, lane);
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
  tile_of_block(blockIdx.x, (g.M + T::BM - 1) / T::BM, (g.N + T::BN - 1) / T::BN, tm, tn);
  if (tm < 0) return;
  const int m0 = tm * T::BM, n0 = tn * T::BN;

  // Order: scales first (they are the oldest vector-memory operations, so no later wait is held up by
  // them), then the first copies of the K loop, then the accumulators are cleared under their latency.
  EpiScales<T> es;
  load_epi_scales<T>(es, g, m0, n0, wn, lane);
  constexpr bool HI1 = MODE == 0;  // the first loop also carries the INT8 operand (dynamic mode)
  Pipe<T, true, HI1> p1;           // MODE 0: low + zero-padded high; MODE 1: low only; MODE 2: unused
  Pipe<T, false, true> p2;         // MODE 1, 2: the compact high loop
  if constexpr (MODE == 0) {
    p1.init(g.a_lo, g.K / 2, g.a_hi_dense, g.K, g.wq, g.K / 2, g.K, m0, n0, g.M, g.N);
    k_loop_start<T, true, HI1>(p1, lds);
  } else if constexpr (MODE == 1) {
    p1.init(g.a_lo, g.K_lo / 2, nullptr, 0, g.w_lo, g.K_lo / 2, g.K_lo, m0, n0, g.M, g.N);
    k_loop_start<T, true, HI1>(p1, lds);
  } else {
    p2.init(nullptr, 0, g.a_hi_compact, g.lda_hi_compact, g.w_hi, g.K_hi / 2, g.K_hi, m0, n0, g.M, g.N);
    k_loop_start<T, false, true>(p2, lds);
  }

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

  if constexpr (MODE == 0) {
    k_loop<T, true, HI1>(p1, lds, wm, wn, lane, acc_lo, acc_hi);
  } else {
    if constexpr (MODE == 1) {
      k_loop<T, true, HI1>(p1, lds, wm, wn, lane, acc_lo, acc_hi);
      p2.init(nullptr, 0, g.a_hi_compact, g.lda_hi_compact, g.w_hi, g.K_hi / 2, g.K_hi, m0, n0, g.M, g.N);
      k_loop_start<T, false, true>(p2, lds);
    }
    k_loop<T, false, true>(p2, lds, wm, wn, lane, acc_lo, acc_hi);
  }

  epilogue<T>(g, es, lds, acc_lo, acc_hi, m0, n0, wm, wn, wave, lane);
}

template <typename T, int MODE>
int launch_mode(const GemmArgs& g, hipStream_t st) {
  const int tiles = ((g.N + T::BN - 1) / T::BN) * ((g.M + T::BM - 1) / T::BM);
  const int blocks = (tiles + 7) / 8 * 8;
  hipLaunchKernelGGL((gemm_kernel<T, MODE>), dim3(blocks), dim3(NT), T::LDS_BYTES, st, g);
  return hipGetLastError() == hipSuccess ? SQ_OK : SQ_ERR_LAUNCH;
}


// ---------------------------------------------------------------------------------------------
// Decode shapes (M <= 64, dynamic mode): the layer is bound by streaming the INT4 weights once from
// HBM, not by the matrix cores, and HBM needs tens of kilobytes in flight per compute unit.
// Vector-memory operations of a wave retire in order, so one wave cannot keep a deep queue of weight
// loads and, at the same time, wait for the shallow queue of (L2-resident) activation loads.  The
// workgroup is therefore specialised: waves 0 and 1 multiply (32 output channels each, all tokens)
// and copy the activation tiles six K steps ahead (ring of eight stages); wave 2 only copies weights,
// seven K steps ahead, into its own ring of eight LDS stages.  Each wave waits on its own counter; one workgroup barrier
// per K step publishes both copies.  Both copies are published one step earlier than they are
// multiplied, so that a consumer fetches the operands of step kt+1 from LDS while the matrix
// instructions of step kt run: the per-step chain "barrier -> LDS read -> multiply -> barrier", which
// otherwise bounds the streaming rate at N * 64 bytes per chain time, shrinks to the multiply.
// A workgroup covers 64 output channels, so N/64 workgroups (two per compute unit) stream disjoint rows.
// TI = number of 32-token blocks (1: M <= 32, 2: M <= 64).  Requires K % 128 == 0.  Only TI = 1 is dispatched: with
// two token blocks (12 KB of activations per stage, one workgroup per compute unit, or shallower activation rings to
// fit two) the kernel was slower than the generic 64 x 64 tile at every ring depth tried (67-70 us against 54 us at
// 64 tokens on the 70B shape).
template <int TI, int TJ>
struct SkinnyCfg {
  static constexpr int BM = 32 * TI;
  static constexpr int BN = 64 * TJ;           // TJ = 32-channel tiles per consumer wave (1 or 2)
  static constexpr int A_LO = 0;
  static constexpr int A_HI = BM * 64;
  static constexpr int A_STAGE = BM * 192;
  static constexpr int A_STAGES = 8;
  static constexpr int A_DIST = 6;  // the activation copy of step kt + A_DIST is enqueued during step kt
  static constexpr int W_OFF = A_STAGES * A_STAGE;
  static constexpr int W_STAGE = BN * 64;
  static constexpr int W_STAGES = 8;
  static constexpr int W_AHEAD = W_STAGES - 1;
  static constexpr int LDS_BYTES = W_OFF + W_STAGES * W_STAGE;
  static constexpr int N_LO = BM * 4 / 128;   // activation copies per consumer wave and K step
  static constexpr int N_HI = BM * 8 / 128;
  static constexpr int NA = N_LO + N_HI;
  static constexpr int THREADS = 192;
};

// Weight loader wave: the four wave copies (64 rows x 64 bytes) of K step `step` into its ring stage.
template <int TI, int TJ>
__device__ __forceinline__ void skinny_issue_w(const char* const (&src)[4 * TJ], char* lds, int step) {
  typedef SkinnyCfg<TI, TJ> C;
  char* dst = lds + C::W_OFF + (step % C::W_STAGES) * C::W_STAGE;
#pragma unroll
  for (int q = 0; q < 4 * TJ; ++q)
    __builtin_amdgcn_global_load_lds(src[q] + step * 64, (lds_ptr_t)(dst + q * 1024), 16, 0, 0);
}

// Consumer waves: this wave's share of the activation tiles of K step `step`.
template <int TI, int TJ>
__device__ __forceinline__ void skinny_issue_a(const char* const (&p_lo)[SkinnyCfg<TI, TJ>::N_LO],
                                               const char* const (&p_hi)[SkinnyCfg<TI, TJ>::N_HI], char* lds, int step,
                                               int wave) {
  typedef SkinnyCfg<TI, TJ> C;
  char* dst = lds + (step % C::A_STAGES) * C::A_STAGE;
#pragma unroll
  for (int i = 0; i < C::N_LO; ++i)
    __builtin_amdgcn_global_load_lds(p_lo[i] + step * 64, (lds_ptr_t)(dst + C::A_LO + (128 * i + 64 * wave) * 16), 16, 0, 0);
#pragma unroll
  for (int i = 0; i < C::N_HI; ++i)
    __builtin_amdgcn_global_load_lds(p_hi[i] + step * 128, (lds_ptr_t)(dst + C::A_HI + (128 * i + 64 * wave) * 16), 16, 0, 0);
}

// Operands of one K step of a consumer wave: packed weights of its 32 channels, packed low codes and
// INT8 high codes of the tokens (two 64-channel halves each).
template <int TI, int TJ>
struct SkinnyOps {
  v4u fw[TJ][2];
  v4u fa[TI][2];
  v4i fh[TI][4];
};

// sa_idx / sw_idx: ring stages of the step's activation and weight tiles (compile-time constants in the
// steady state, so that the reads differ only in their immediate offsets).
template <int TI, int TJ>
__device__ __forceinline__ void skinny_fetch_at(SkinnyOps<TI, TJ>& o, const char* lds, int sa_idx, int sw_idx, int wave,
                                                int r, int h) {
  typedef SkinnyCfg<TI, TJ> C;
  const char* sa = lds + sa_idx * C::A_STAGE;
  const char* sw = lds + C::W_OFF + sw_idx * C::W_STAGE;
#pragma unroll
  for (int gq = 0; gq < 2; ++gq) {
#pragma unroll
    for (int j = 0; j < TJ; ++j) o.fw[j][gq] = *reinterpret_cast<const v4u*>(sw + off4((wave * TJ + j) * 32 + r, 2 * gq + h));
#pragma unroll
    for (int i = 0; i < TI; ++i) {
      o.fa[i][gq] = *reinterpret_cast<const v4u*>(sa + C::A_LO + off4(i * 32 + r, 2 * gq + h));
      o.fh[i][2 * gq] = *reinterpret_cast<const v4i*>(sa + C::A_HI + off8(i * 32 + r, 4 * gq + 2 * h));
      o.fh[i][2 * gq + 1] = *reinterpret_cast<const v4i*>(sa + C::A_HI + off8(i * 32 + r, 4 * gq + 2 * h + 1));
    }
  }
}

template <int TI, int TJ>
__device__ __forceinline__ void skinny_fetch(SkinnyOps<TI, TJ>& o, const char* lds, int step, int wave, int r, int h) {
  skinny_fetch_at<TI, TJ>(o, lds, step % SkinnyCfg<TI, TJ>::A_STAGES, step % SkinnyCfg<TI, TJ>::W_STAGES, wave, r, h);
}

template <int TI, int TJ>
__device__ __forceinline__ void skinny_mma(const SkinnyOps<TI, TJ>& o, v16i (&acc_lo)[TI][TJ], v16i (&acc_hi)[TI][TJ]) {
#pragma unroll
  for (int gq = 0; gq < 2; ++gq)
#pragma unroll
    for (int s2 = 0; s2 < 2; ++s2) {
      v4i bw[TJ];
#pragma unroll
      for (int j = 0; j < TJ; ++j) bw[j] = widen(o.fw[j][gq], s2);
#pragma unroll
      for (int i = 0; i < TI; ++i) {
        const v4i alo = widen(o.fa[i][gq], s2);
#pragma unroll
        for (int j = 0; j < TJ; ++j) {
          acc_lo[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(alo, bw[j], acc_lo[i][j], 0, 0, 0);
          acc_hi[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(o.fh[i][2 * gq + s2], bw[j], acc_hi[i][j], 0, 0, 0);
        }
      }
    }
}

// Multiply one step, then join the step's barrier; `copied`: this step enqueued an activation copy, so
// A_DIST - 2 younger ones may stay in flight, otherwise everything outstanding is waited for.
template <int TI, int TJ>
__device__ __forceinline__ void pipeline_barrier_after(const SkinnyOps<TI, TJ>& cur, v16i (&acc_lo)[TI][TJ], v16i (&acc_hi)[TI][TJ],
                                                       bool copied) {
  typedef SkinnyCfg<TI, TJ> C;
  skinny_mma<TI, TJ>(cur, acc_lo, acc_hi);
  if (copied) pipeline_barrier<(C::A_DIST - 2) * C::NA>();
  else pipeline_barrier<0>();
}

// Step kt + U of a trip of eight steps that starts at a multiple of eight (the ring sizes divide eight, so
// every stage index is a compile-time constant).  The sources of the activation copies of step kt + U + A_DIST
// are a wave-uniform base (scalar registers, advanced by scalar additions) plus a per-lane 32-bit offset
// that never changes.  (The instruction's immediate offset is no use here: for a copy into LDS it is added
// to the LDS address as well.)
// LAST: the trip is the last one of the K loop (it ends at the last step): only its first steps still have a
// copy to enqueue, its last step has no successor to fetch, and the barrier's allowance shrinks with the
// copies that remain outstanding.
template <int TI, int TJ, int U, bool LAST = false>
__device__ __forceinline__ void skinny_steady_step(const SkinnyOps<TI, TJ>& cur, SkinnyOps<TI, TJ>& nxt, const char* ub_lo,
                                                   const char* ub_hi, const unsigned (&l_lo)[SkinnyCfg<TI, TJ>::N_LO],
                                                   const unsigned (&l_hi)[SkinnyCfg<TI, TJ>::N_HI], char* lds, int wave,
                                                   int r, int h, v16i (&acc_lo)[TI][TJ], v16i (&acc_hi)[TI][TJ]) {
  typedef SkinnyCfg<TI, TJ> C;
  static_assert(8 % C::A_STAGES == 0 && 8 % C::W_STAGES == 0, "ring sizes must divide the trip length");
  constexpr bool FETCH = !LAST || U + 1 < 8;
  constexpr bool COPY = !LAST || U + C::A_DIST < 8;
  // copies still outstanding at the barrier may be those of steps kt+U+3 ... : A_DIST-2 steps' worth in the
  // steady state, in the last trip only up to its last step (step kt+7)
  constexpr int YOUNGER = LAST ? (7 - (U + 2) > 0 ? 7 - (U + 2) : 0) : C::A_DIST - 2;
  constexpr int PENDING = (YOUNGER < C::A_DIST - 2 ? YOUNGER : C::A_DIST - 2) * C::NA;
  if (FETCH) skinny_fetch_at<TI, TJ>(nxt, lds, (U + 1) % C::A_STAGES, (U + 1) % C::W_STAGES, wave, r, h);
  if (COPY) {
    char* dst = lds + ((U + C::A_DIST) % C::A_STAGES) * C::A_STAGE;
    const char* s_lo = ub_lo + (U + C::A_DIST) * 64;
    const char* s_hi = ub_hi + (U + C::A_DIST) * 128;
#pragma unroll
    for (int i = 0; i < C::N_LO; ++i)
      __builtin_amdgcn_global_load_lds(s_lo + l_lo[i], (lds_ptr_t)(dst + C::A_LO + (128 * i + 64 * wave) * 16), 16, 0, 0);
#pragma unroll
    for (int i = 0; i < C::N_HI; ++i)
      __builtin_amdgcn_global_load_lds(s_hi + l_hi[i], (lds_ptr_t)(dst + C::A_HI + (128 * i + 64 * wave) * 16), 16, 0, 0);
  }
  skinny_mma<TI, TJ>(cur, acc_lo, acc_hi);
  pipeline_barrier<PENDING>();  // the copies of steps <= kt + U + 2 have landed
}

template <int TI, int TJ>
__global__ __launch_bounds__(192) void gemm_skinny_kernel(GemmArgs g) {
  typedef SkinnyCfg<TI, TJ> C;
  extern __shared__ __attribute__((aligned(16))) char lds[];
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n0 = blockIdx.x * C::BN;
  const int steps = g.K / KS;
  constexpr int W_AHEAD = C::W_AHEAD;

  if (wave == 2) {
    // ---- weight loader: 4 wave copies (64 rows x 64 bytes) per K step, W_AHEAD steps ahead ----
    const char* src[4 * TJ];
#pragma unroll
    for (int q = 0; q < 4 * TJ; ++q) {
      const int row = 16 * q + (lane >> 2);
      const int c = ((lane & 3) ^ (row >> 2)) & 3;
      src[q] = reinterpret_cast<const char*>(g.wq) + static_cast<int64_t>(min(n0 + row, g.N - 1)) * (g.K / 2) + c * 16;
    }
    // at barrier kt (the prologue barrier is kt = -1) the copies of steps <= kt+2 have landed
    const int pre = min(C::W_AHEAD, steps);
    for (int s2 = 0; s2 < pre; ++s2) skinny_issue_w<TI, TJ>(src, lds, s2);
    if (pre == C::W_AHEAD) pipeline_barrier<4 * TJ * (C::W_AHEAD - 2)>();
    else pipeline_barrier<0>();
    for (int kt = 0; kt < steps; ++kt) {
      if (kt + C::W_AHEAD < steps) {
        const int ahead = kt + W_AHEAD;
        skinny_issue_w<TI, TJ>(src, lds, ahead);
        pipeline_barrier<4 * TJ * (C::W_AHEAD - 2)>();  // five younger steps stay in flight
      } else {
        pipeline_barrier<0>();
      }
    }
    return;
  }

  // ---- consumers ----
  const int r = lane & 31, h = lane >> 5;
  const char* p_lo[C::N_LO];
  const char* p_hi[C::N_HI];
#pragma unroll
  for (int i = 0; i < C::N_LO; ++i) {
    const int idx = tid + 128 * i, row = idx >> 2;
    const int c = ((idx & 3) ^ (row >> 2)) & 3;
    p_lo[i] = reinterpret_cast<const char*>(g.a_lo) + static_cast<int64_t>(min(row, g.M - 1)) * (g.K / 2) + c * 16;
  }
#pragma unroll
  for (int i = 0; i < C::N_HI; ++i) {
    const int idx = tid + 128 * i, row = idx >> 3;
    const int c = ((idx & 7) ^ (row >> 1)) & 7;
    p_hi[i] = reinterpret_cast<const char*>(g.a_hi_dense) + static_cast<int64_t>(min(row, g.M - 1)) * g.K + c * 16;
  }

  // per-token scales of the rows this lane's accumulator registers hold
  float slo[TI][16], shi[TI][16];
#pragma unroll
  for (int i = 0; i < TI; ++i)
#pragma unroll
    for (int q = 0; q < 16; ++q) {
      const int m = min(i * 32 + 8 * (q >> 2) + 4 * h + (q & 3), g.M - 1);
      slo[i][q] = g.s_lo[m];
      shi[i][q] = g.s_hi[m];
    }
  float sw[TJ];
#pragma unroll
  for (int j = 0; j < TJ; ++j) sw[j] = g.s_w[min(n0 + (wave * TJ + j) * 32 + r, g.N - 1)];

  v16i acc_lo[TI][TJ], acc_hi[TI][TJ];
#pragma unroll
  for (int i = 0; i < TI; ++i)
#pragma unroll
  for (int j = 0; j < TJ; ++j)
#pragma unroll
    for (int q = 0; q < 16; ++q) {
      acc_lo[i][q] = 0;
      acc_hi[i][q] = 0;
    }

  // At barrier kt (prologue: kt = -1) this wave's activation copies of steps <= kt+2 have landed.  A copy
  // is enqueued A_DIST steps before it is multiplied and has A_DIST - 2 steps to arrive: with one step
  // (a few hundred nanoseconds here) the wait for it was half of every step.
  constexpr int D = C::A_DIST;
#pragma unroll
  for (int s0 = 0; s0 < D; ++s0)
    if (s0 < steps) skinny_issue_a<TI, TJ>(p_lo, p_hi, lds, s0, wave);
  if (steps >= D) pipeline_barrier<(D - 2) * C::NA>();
  else pipeline_barrier<0>();
  // Operands of one K step are fetched from LDS one step ahead of the matrix instructions that use them.
  // The steady state has no branches (the compiler then keeps the accumulators where they are and waits
  // for the LDS reads of step kt+1 only after the matrix instructions of step kt have been issued) and no
  // address arithmetic: with few tokens a step is a handful of matrix instructions, so every other
  // instruction in it counts.
  SkinnyOps<TI, TJ> o0, o1;
  skinny_fetch<TI, TJ>(o0, lds, 0, wave, r, h);
  int kt = 0;
  {
    // steady state: trips of eight steps with compile-time stage indices
    unsigned l_lo[C::N_LO], l_hi[C::N_HI];  // per-lane byte offsets of the copies' sources (below 2^32: M <= 64 rows)
#pragma unroll
    for (int i = 0; i < C::N_LO; ++i) l_lo[i] = static_cast<unsigned>(p_lo[i] - reinterpret_cast<const char*>(g.a_lo));
#pragma unroll
    for (int i = 0; i < C::N_HI; ++i) l_hi[i] = static_cast<unsigned>(p_hi[i] - reinterpret_cast<const char*>(g.a_hi_dense));
    const char* ub_lo = reinterpret_cast<const char*>(g.a_lo);
    const char* ub_hi = reinterpret_cast<const char*>(g.a_hi_dense);
    for (; kt + 8 + D <= steps; kt += 8) {  // the copy of step kt + 7 + A_DIST is the last one a trip enqueues
      skinny_steady_step<TI, TJ, 0>(o0, o1, ub_lo, ub_hi, l_lo, l_hi, lds, wave, r, h, acc_lo, acc_hi);
      skinny_steady_step<TI, TJ, 1>(o1, o0, ub_lo, ub_hi, l_lo, l_hi, lds, wave, r, h, acc_lo, acc_hi);
      skinny_steady_step<TI, TJ, 2>(o0, o1, ub_lo, ub_hi, l_lo, l_hi, lds, wave, r, h, acc_lo, acc_hi);
      skinny_steady_step<TI, TJ, 3>(o1, o0, ub_lo, ub_hi, l_lo, l_hi, lds, wave, r, h, acc_lo, acc_hi);
      skinny_steady_step<TI, TJ, 4>(o0, o1, ub_lo, ub_hi, l_lo, l_hi, lds, wave, r, h, acc_lo, acc_hi);
      skinny_steady_step<TI, TJ, 5>(o1, o0, ub_lo, ub_hi, l_lo, l_hi, lds, wave, r, h, acc_lo, acc_hi);
      skinny_steady_step<TI, TJ, 6>(o0, o1, ub_lo, ub_hi, l_lo, l_hi, lds, wave, r, h, acc_lo, acc_hi);
      skinny_steady_step<TI, TJ, 7>(o1, o0, ub_lo, ub_hi, l_lo, l_hi, lds, wave, r, h, acc_lo, acc_hi);
      ub_lo += 8 * 64;
      ub_hi += 8 * 128;
    }
    if (steps - kt == 8) {  // exactly one trip left (K a multiple of 1024): the same code, winding down
      skinny_steady_step<TI, TJ, 0, true>(o0, o1, ub_lo, ub_hi, l_lo, l_hi, lds, wave, r, h, acc_lo, acc_hi);
      skinny_steady_step<TI, TJ, 1, true>(o1, o0, ub_lo, ub_hi, l_lo, l_hi, lds, wave, r, h, acc_lo, acc_hi);
      skinny_steady_step<TI, TJ, 2, true>(o0, o1, ub_lo, ub_hi, l_lo, l_hi, lds, wave, r, h, acc_lo, acc_hi);
      skinny_steady_step<TI, TJ, 3, true>(o1, o0, ub_lo, ub_hi, l_lo, l_hi, lds, wave, r, h, acc_lo, acc_hi);
      skinny_steady_step<TI, TJ, 4, true>(o0, o1, ub_lo, ub_hi, l_lo, l_hi, lds, wave, r, h, acc_lo, acc_hi);
      skinny_steady_step<TI, TJ, 5, true>(o1, o0, ub_lo, ub_hi, l_lo, l_hi, lds, wave, r, h, acc_lo, acc_hi);
      skinny_steady_step<TI, TJ, 6, true>(o0, o1, ub_lo, ub_hi, l_lo, l_hi, lds, wave, r, h, acc_lo, acc_hi);
      skinny_steady_step<TI, TJ, 7, true>(o1, o0, ub_lo, ub_hi, l_lo, l_hi, lds, wave, r, h, acc_lo, acc_hi);
      kt += 8;
    }
  }
  // the remaining steps (fewer than 8 + A_DIST): stage indices and addresses computed at run time
  while (kt < steps) {
    if (kt + 1 < steps) skinny_fetch<TI, TJ>(o1, lds, kt + 1, wave, r, h);
    if (kt + D < steps) {
      skinny_issue_a<TI, TJ>(p_lo, p_hi, lds, kt + D, wave);
      pipeline_barrier_after<TI, TJ>(o0, acc_lo, acc_hi, true);
    } else {
      pipeline_barrier_after<TI, TJ>(o0, acc_lo, acc_hi, false);
    }
    if (++kt >= steps) break;
    if (kt + 1 < steps) skinny_fetch<TI, TJ>(o0, lds, kt + 1, wave, r, h);
    if (kt + D < steps) {
      skinny_issue_a<TI, TJ>(p_lo, p_hi, lds, kt + D, wave);
      pipeline_barrier_after<TI, TJ>(o1, acc_lo, acc_hi, true);
    } else {
      pipeline_barrier_after<TI, TJ>(o1, acc_lo, acc_hi, false);
    }
    ++kt;
  }

  // epilogue: the outputs are few (M <= 64 rows); plain stores
  if (n < g.N) {
#pragma unroll
    for (int i = 0; i < TI; ++i)
#pragma unroll
      for (int q = 0; q < 16; ++q) {
        const int m = i * 32 + 8 * (q >> 2) + 4 * h + (q & 3);
        if (m < g.M) {
          float t = __fmul_rn(static_cast<float>(acc_lo[i][q] >> 8), slo[i][q]);
          t = __fmaf_rn(static_cast<float>(acc_hi[i][q] >> 4), shi[i][q], t);
          const float y = __fmul_rn(t, sw);
          const int64_t o = static_cast<int64_t>(m) * g.ldy + n;
          if (g.out_bf16) reinterpret_cast<uint16_t*>(g.y)[o] = bf16_rne(y);
          else reinterpret_cast<float*>(g.y)[o] = y;
          if (g.acc_lo_dbg) g.acc_lo_dbg[static_cast<int64_t>(m) * g.N + n] = acc_lo[i][q] >> 8;
          if (g.acc_hi_dbg) g.acc_hi_dbg[static_cast<int64_t>(m) * g.N + n] = acc_hi[i][q] >> 4;
        }
      }
  }
}

template <int TI, int TJ>
int launch_skinny(const GemmArgs& g, hipStream_t st) {
  typedef SkinnyCfg<TI, TJ> C;
  hipLaunchKernelGGL((gemm_skinny_kernel<TI, TJ>), dim3((g.N + C::BN - 1) / C::BN), dim3(C::THREADS), C::LDS_BYTES, st, g);
  return hipGetLastError() == hipSuccess ? SQ_OK : SQ_ERR_LAUNCH;
}

// Three stages everywhere: a fourth stage for the 128x256 tile (exactly the 160 KB of LDS) and four or six for
// the 64x64 tile were timed and change nothing (c3: 680 us either way on dense random operands; 64 tokens:
// 55.7 / 60.4 us against 56.8 us) -- the copies are not what the loop waits for.
typedef Tile<128, 256> Big;   // matrix-core bound shapes
typedef Tile<64, 64> Skinny;  // M <= 64 (decode): bound by streaming the INT4 weights once from HBM, so the
                              // tile is narrow in N to spread the weight rows over every compute unit
                              // (several small workgroups per unit keep enough loads in flight)
typedef Tile<64, 128> SkinnyWide;  // the same for very wide layers: every workgroup re-reads the activation tile from
                                   // L2 on each K step, and at 64 tokens that traffic (three times the weight
                                   // stream) is what bounds the 64-wide tile; twice the channels per workgroup
                                   // halves it (52 us against 55.5 us on the 70B shape) as long as the wider
                                   // tiles still cover most compute units
typedef Tile<128, 128> Mid;   // shapes with too few 128x256 tiles to occupy every compute unit
typedef Tile<256, 256, false> Huge;  // single-product modes on large shapes: with one accumulator set a wave
                                     // holds 128 x 128 outputs, which halves the operand traffic and the
                                     // widening arithmetic per matrix instruction and doubles the matrix
                                     // instructions between two barriers to 64, as in the two-product loop

enum Variant { V_BIG, V_MID, V_SMALL, V_STREAM, V_HUGE, V_SMALL_WIDE };

// Which kernel a shape runs on.  dynamic: the call has the low operand and the zero-padded high image;
// single: one product only (tied scales, plain W4A8).
Variant pick_variant(int M, int N, int K, bool dynamic, bool single) {
  if (M <= 64) {
    if (dynamic && M <= 32 && K % KS == 0) return V_STREAM;
    return (M > 32 && (N + 127) / 128 >= 200) ? V_SMALL_WIDE : V_SMALL;
  }
  const int64_t huge_tiles = static_cast<int64_t>((M + 255) / 256) * ((N + 255) / 256);
  if (single && huge_tiles >= kHugeMinTiles) return V_HUGE;
  const int64_t big_tiles = static_cast<int64_t>((M + 127) / 128) * ((N + 255) / 256);
  return big_tiles <= 128 ? V_MID : V_BIG;  // then twice as many half-size tiles still run in one round
}

template <typename T, int MODE>
hipError_t raise_lds_limit() {
  return hipFuncSetAttribute(reinterpret_cast<const void*>(gemm_kernel<T, MODE>),
                             hipFuncAttributeMaxDynamicSharedMemorySize, T::LDS_BYTES);
}

template <int MODE>
int launch_for_mode(const GemmArgs& g, hipStream_t st, Variant v) {
  if constexpr (MODE == 2) {
    if (v == V_HUGE) return launch_mode<Huge, 2>(g, st);
  }
  if (v == V_BIG) return launch_mode<Big, MODE>(g, st);
  if (v == V_MID) return launch_mode<Mid, MODE>(g, st);
  if (v == V_SMALL_WIDE) return launch_mode<SkinnyWide, MODE>(g, st);
  return launch_mode<Skinny, MODE>(g, st);
}

}  // namespace

// The GEMM kernels use more dynamic LDS than the default limit; the limit of every instantiation is raised
// here, once per device (called by the library's per-device initialisation, never on the launch path).
int init_gemm_kernels() {
  hipError_t e = hipSuccess;
#define SQ_RAISE(T)                                          \
  if (e == hipSuccess) e = raise_lds_limit<T, 0>();          \
  if (e == hipSuccess) e = raise_lds_limit<T, 1>();          \
  if (e == hipSuccess) e = raise_lds_limit<T, 2>();
  SQ_RAISE(Big) SQ_RAISE(Mid) SQ_RAISE(Skinny) SQ_RAISE(SkinnyWide)
#undef SQ_RAISE
  if (e == hipSuccess) e = raise_lds_limit<Huge, 2>();
  if (e == hipSuccess)
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(gemm_skinny_kernel<1>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, SkinnyCfg<1>::LDS_BYTES);
  return e == hipSuccess ? SQ_OK : SQ_ERR_LAUNCH;
}

const char* gemm_variant_name(int M, int N, int K, bool dynamic, bool single) {
  switch (pick_variant(M, N, K, dynamic, single)) {
    case V_HUGE: return "tile256x256";
    case V_BIG: return "tile128x256";
    case V_MID: return "tile128x128";
    case V_SMALL: return "tile64x64";
    case V_SMALL_WIDE: return "tile64x128";
    default: return "stream32";
  }
}

int launch_gemm(const GemmArgs& g, hipStream_t st) {
  const bool dynamic = g.a_lo && g.a_hi_dense;
  const Variant v = pick_variant(g.M, g.N, g.K, dynamic, !g.a_lo);
  if (dynamic) {
    if (v == V_STREAM) return launch_skinny<1>(g, st);
    return launch_for_mode<0>(g, st, v);
  }
  if (g.a_lo && g.a_hi_compact) return launch_for_mode<1>(g, st, v);
  if (!g.a_lo && g.a_hi_compact) return launch_for_mode<2>(g, st, v);
  return SQ_ERR_UNSUPPORTED;
}

}  // namespace sq
