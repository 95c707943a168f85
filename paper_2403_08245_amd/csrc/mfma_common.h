// Device helpers shared by the bf16 matrix-core grouped GEMM kernels (gfx950): vector types,
// direct-to-LDS loads with hand-placed waits, the two swizzled LDS tile layouts and the
// tile search over the expert offsets.
#pragma once
#include "common.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int HK = 32;            // contraction elements per LDS stage (one half-step)
constexpr int NSTAGE = 4;
constexpr int NTHREADS = 256;
constexpr int TB = 256;           // tile edge (rows and columns of the output tile)
constexpr int TILE_BYTES = TB * HK * 2;       // one operand tile of one stage: 16 KB
constexpr int STAGE_BYTES = 2 * TILE_BYTES;   // A tile then B tile
constexpr int NLD = TB / 64;      // load instructions per wavefront per operand tile (4)
constexpr int FR = TB / 64;       // 32x32 fragments per wavefront along each tile edge (4)

#define LDS_AS __attribute__((address_space(3)))

// 16 (or 4) bytes per lane, global -> LDS without passing through registers.  The LDS
// destination (a byte address in M0) is wave-uniform; lane L's data lands at lds_addr +
// 16 * L (4 * L).  Written as inline assembly so that the waits are placed by hand: several
// stages stay in flight while another one is read, ordered only by `wait_loads` + barrier.
__device__ __forceinline__ void load16_to_lds(const void *gsrc, uint32_t lds_addr) {
  __asm__ volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_addr), "v"(gsrc) : "memory", "m0");
}
// Same with the address split into a wave-uniform 64-bit base (scalar registers) and a 32-bit
// per-lane byte offset: half the address registers go to the memory pipeline per instruction,
// which shortens the issue of the load inside a matrix-instruction stream.
__device__ __forceinline__ void load16_to_lds(const void *base, uint32_t byte_off, uint32_t lds_addr) {
  __asm__ volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_addr), "v"(byte_off), "s"(base)
                   : "memory", "m0");
}
// Range-checked form: a raw buffer descriptor (base address, byte count) in four scalar registers and a
// 32-bit lane offset; a lane whose bytes lie past the byte count lands zeros in LDS instead of loading.
// Used where rows past the end of a segment have to contribute nothing to a sum.
typedef int int32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ int32x4 buffer_window(const void *base, uint32_t bytes) {
  const unsigned long long p = (unsigned long long)base;
  int32x4 r;
  r[0] = __builtin_amdgcn_readfirstlane((int)(uint32_t)p);
  r[1] = __builtin_amdgcn_readfirstlane((int)(uint32_t)((p >> 32) & 0xffffu));   // stride 0: a raw buffer
  r[2] = __builtin_amdgcn_readfirstlane((int)bytes);
  r[3] = 0x00020000;                                                            // 32-bit raw data format
  return r;
}
__device__ __forceinline__ void load16_to_lds_checked(int32x4 window, uint32_t byte_off, uint32_t lds_addr) {
  __asm__ volatile("s_mov_b32 m0, %0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds" ::"s"(lds_addr), "v"(byte_off), "s"(window)
                   : "memory", "m0");
}
__device__ __forceinline__ void load4_to_lds(const void *gsrc, uint32_t lds_addr) {
  __asm__ volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dword %1, off" ::"s"(lds_addr), "v"(gsrc) : "memory", "m0");
}
// Waits until at most N of this wavefront's global loads are outstanding (they finish in order).
template <int N> __device__ __forceinline__ void wait_loads() {
  __asm__ volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}
__device__ __forceinline__ uint32_t lds_address(const char *p) { return (uint32_t)(size_t)(LDS_AS const char *)p; }
__device__ __forceinline__ void sched_fence() { __builtin_amdgcn_sched_barrier(0); }

__device__ __align__(16) const uint32_t g_zero16[4] = {0u, 0u, 0u, 0u};
// Landing zone for the epilogue's masked-out lanes: they store here instead of branching
// around the store (the contents are never read).
__device__ __align__(16) uint32_t g_trash[64 * 4];

// ---------------------------------------------------------------- KC tile (256 rows x 32, k contiguous)
__device__ __forceinline__ int kc_swz(int row) { return (row >> 2) & 3; }
// Load instruction `inst` (0..3) of a wavefront covers 16 rows; lane -> (tile row, source chunk).
__device__ __forceinline__ void kc_lane_slot(int wave, int lane, int inst, int &row, int &chunk) {
  row = (wave * NLD + inst) * 16 + (lane >> 2);
  chunk = (lane & 3) ^ kc_swz(row);
}
// fragment for v_mfma_32x32x16: lane holds row (rbase + lane%32), k = kk*16 + 8*(lane/32) + 0..7
__device__ __forceinline__ bf16x8 kc_frag(const char *tile, int rbase, int kk, int lane) {
  int row = rbase + (lane & 31);
  int chunk = (kk * 2 + (lane >> 5)) ^ kc_swz(row);
  return *reinterpret_cast<const bf16x8 *>(tile + row * 64 + chunk * 16);
}

// ---------------------------------------------------------------- TR tile (32 x 256, columns contiguous)
__device__ __forceinline__ int tr_swz(int row) { return (row & 3) << 2; }
// Load instruction `inst` (0..3) of a wavefront covers 2 contraction rows of 512 B.
__device__ __forceinline__ void tr_lane_slot(int wave, int lane, int inst, int &row, int &chunk) {
  row = (wave * NLD + inst) * 2 + (lane >> 5);
  chunk = (lane & 31) ^ tr_swz(row);
}
// fragment: lane holds column (cbase + lane%32), contraction rows kk*16 + 8*(lane/32) + 0..7
__device__ __forceinline__ bf16x8 tr_frag(const char *tile, int cbase, int kk, int lane) {
  int col = cbase + 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
  int row0 = kk * 16 + 8 * (lane >> 5) + ((lane & 15) >> 2);
  union { bf16x8 v; s16x4 h[2]; } u;
#pragma unroll
  for (int t = 0; t < 2; ++t) {
    int row = row0 + 4 * t;
    int off = row * (TB * 2) + ((((col >> 3) ^ tr_swz(row))) << 4) + ((col & 7) << 1);
    u.h[t] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS s16x4 *)(tile + off));
  }
  return u.v;
}
// byte offset inside an operand tile of a wavefront's load instruction (both layouts: 1 KB each)
__device__ __forceinline__ int inst_off(int wave, int inst) { return (wave * NLD + inst) * 1024; }

// Finds expert and first row of M-tile `tile` when each expert's segment is cut into tiles of
// ROWS rows.  Every wavefront runs the search on its own: lane x looks at expert c0 + x, a wave
// prefix sum counts the tiles before it, a ballot picks the expert that owns `tile`.
template <int ROWS>
__device__ __forceinline__ bool locate_rows(const int32_t *offsets, int E, int tile, int lane, int &e, int &row0,
                                            int &row_end) {
  int base = 0;
  for (int c0 = 0; c0 < E; c0 += 64) {
    int x = c0 + lane;
    int lo = 0, hi = 0;
    if (x < E) { lo = offsets[x]; hi = offsets[x + 1]; }
    int nt = (hi - lo + ROWS - 1) / ROWS;
    int incl = nt;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
      int up = __shfl_up(incl, d, 64);
      if (lane >= d) incl += up;
    }
    // wave-uniform values are moved to scalar registers by hand so that the callers' control
    // flow (tile bookkeeping of the persistent kernels) stays scalar as well
    int total = __builtin_amdgcn_readfirstlane(__shfl(incl, 63, 64));
    if (tile < base + total) {
      unsigned long long owns = __ballot(base + incl > tile);
      int first = __ffsll((long long)owns) - 1;
      int before = __builtin_amdgcn_readfirstlane(__shfl(incl - nt, first, 64));
      e = c0 + first;
      row0 = __builtin_amdgcn_readfirstlane(__shfl(lo, first, 64)) + (tile - base - before) * ROWS;
      row_end = __builtin_amdgcn_readfirstlane(__shfl(hi, first, 64));
      return true;
    }
    base += total;
  }
  return false;
}
__device__ __forceinline__ bool locate_tile(const int32_t *offsets, int E, int tile, int lane, int &e, int &row0,
                                            int &row_end) {
  return locate_rows<TB>(offsets, E, tile, lane, e, row0, row_end);
}

// Blocks are dealt round-robin to the 8 XCDs; give each XCD a contiguous run of tile ids so
// that tiles sharing operand panels meet in the same L2.
__device__ __forceinline__ int xcd_contiguous_id(int pid, int grid) {
  int per = grid >> 3;  // grid is a multiple of 8
  return (pid & 7) * per + (pid >> 3);
}

}  // namespace
