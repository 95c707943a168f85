// bf16 matrix-core grouped GEMMs for gfx950 (MI355X):
//   * scatter2scatter (Sec. 3.2): rows gathered through the order indices, multiplied by the
//     row's expert matrix W[e] (forward) or W[e]^T (input gradient, Sec. 3.2.1), rows written
//     grouped or scattered.  The grouped copy of the input never exists in HBM: the gather
//     happens in the global->LDS load, the "padded tile" of Sec. 3.1 lives only in LDS.
//   * groupXTY (Sec. 3.2.1): dW[e] = Xbar_e^T dYbar_e over the expert's variable-length row
//     segment, the token rows again gathered on the fly.
//
// Shape of every kernel: 256 threads = 4 wavefronts in a 2x2 grid over a BM x BN output
// tile, v_mfma_f32_32x32x16_bf16 with fp32 accumulators, contraction step 64, two LDS
// stages filled by direct-to-LDS 16-byte global loads (each lane supplies its own gathered
// address), one barrier per step.
//
// Two LDS tile layouts, both XOR-swizzled at 16-byte granularity so that the fragment reads
// are bank-conflict free:
//   KC tile: rows x 64 contraction elements, contraction contiguous (128 B per row); a lane's
//            8 consecutive-k fragment comes from one ds_read_b128.
//   TR tile: 64 contraction rows x C columns, columns contiguous; fragments come from two
//            ds_read_b64_tr_b16 (the transposing LDS read), which hand each lane 4
//            consecutive contraction elements of one column.
// Forward uses KC for X and TR for W; the input gradient uses KC for both (W^T is already
// contraction-contiguous); groupXTY uses TR for both operands.
#include "common.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int BK = 64;            // contraction elements per step
constexpr int NTHREADS = 256;
constexpr int NWAVES = 4;

#define LDS_AS __attribute__((address_space(3)))
#define GLB_AS __attribute__((address_space(1)))

// 16 bytes per lane, global -> LDS without passing through registers.  The LDS destination
// (a byte address in M0) is wave-uniform; lane L's data lands at lds_addr + 16 * L.  Written
// as inline assembly so that the waits are placed by hand: the loads of the next stage stay in
// flight while the current stage is read, and only `wait_all_loads` + the barrier order them.
__device__ __forceinline__ void load16_to_lds(const void *gsrc, uint32_t lds_addr) {
  __asm__ volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_addr), "v"(gsrc) : "memory", "m0");
}
__device__ __forceinline__ void wait_all_loads() { __asm__ volatile("s_waitcnt vmcnt(0)" ::: "memory"); }
__device__ __forceinline__ uint32_t lds_address(const char *p) { return (uint32_t)(size_t)(LDS_AS const char *)p; }

__device__ __align__(16) const uint32_t g_zero16[4] = {0u, 0u, 0u, 0u};

// ---------------------------------------------------------------- KC tile (rows x 64, k contiguous)
__device__ __forceinline__ int kc_swz(int row) { return (row >> 1) & 7; }
// lane's source chunk for load instruction `inst` of a ROWS-row tile: returns the tile row and
// the logical 16-byte chunk (0..7) this lane must fetch so that LDS ends up swizzled.
template <int ROWS>
__device__ __forceinline__ void kc_lane_slot(int wave, int lane, int inst, int &row, int &chunk) {
  row = (wave * (ROWS / 32) + inst) * 8 + (lane >> 3);
  chunk = (lane & 7) ^ kc_swz(row);
}
template <int ROWS> __device__ __forceinline__ int kc_inst_off(int wave, int inst) {
  return (wave * (ROWS / 32) + inst) * 1024;
}
// fragment for v_mfma_32x32x16: lane holds row (rbase + lane%32), k = kk*16 + 8*(lane/32) + 0..7
__device__ __forceinline__ bf16x8 kc_frag(const char *tile, int rbase, int kk, int lane) {
  int row = rbase + (lane & 31);
  int chunk = (kk * 2 + (lane >> 5)) ^ kc_swz(row);
  return *reinterpret_cast<const bf16x8 *>(tile + row * 128 + chunk * 16);
}

// ---------------------------------------------------------------- TR tile (64 x C, columns contiguous)
__device__ __forceinline__ int tr_swz(int row) { return (row & 3) << 2; }
template <int C>
__device__ __forceinline__ void tr_lane_slot(int wave, int lane, int inst, int &row, int &chunk) {
  constexpr int CPR = C / 8;          // 16-byte chunks per row
  constexpr int RPI = 64 / CPR;       // rows per load instruction
  row = (wave * (C / 32) + inst) * RPI + lane / CPR;
  chunk = (lane % CPR) ^ tr_swz(row);
}
template <int C> __device__ __forceinline__ int tr_inst_off(int wave, int inst) {
  return (wave * (C / 32) + inst) * 1024;
}
// fragment: lane holds column (cbase + lane%32), contraction rows kk*16 + 8*(lane/32) + 0..7
template <int C> __device__ __forceinline__ bf16x8 tr_frag(const char *tile, int cbase, int kk, int lane) {
  int col = cbase + 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
  int row0 = kk * 16 + 8 * (lane >> 5) + ((lane & 15) >> 2);
  union { bf16x8 v; s16x4 h[2]; } u;
#pragma unroll
  for (int t = 0; t < 2; ++t) {
    int row = row0 + 4 * t;
    int off = row * (C * 2) + ((((col >> 3) ^ tr_swz(row))) << 4) + ((col & 7) << 1);
    u.h[t] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS s16x4 *)(tile + off));
  }
  return u.v;
}


// Pins the instruction order of one contraction sub-step: every matrix instruction is
// followed by one LDS read of the next sub-step's fragments, so the reads complete under the
// shadow of the MFMA pipe instead of after it (one wavefront per SIMD has nothing else to
// hide them behind).
template <int N_MFMA, int N_DSREAD> __device__ __forceinline__ void interleave_mfma_dsread() {
#pragma unroll
  for (int i = 0; i < N_DSREAD; ++i) {
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // 1 MFMA
    __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);  // 1 DS read
  }
  if (N_MFMA > N_DSREAD) __builtin_amdgcn_sched_group_barrier(0x008, N_MFMA - N_DSREAD, 0);
}

// Finds expert and first row of M-tile `tile` when each expert's segment is cut into BM-row tiles.
__device__ __forceinline__ bool locate_tile(const int32_t *offsets, int E, int bm, int tile, int &e, int &row0,
                                            int &row_end) {
  int acc = 0;
  for (int x = 0; x < E; ++x) {
    int lo = offsets[x], hi = offsets[x + 1];
    int nt = (hi - lo + bm - 1) / bm;
    if (tile < acc + nt) {
      e = x;
      row0 = lo + (tile - acc) * bm;
      row_end = hi;
      return true;
    }
    acc += nt;
  }
  return false;
}

// Blocks are dealt round-robin to the 8 XCDs; give each XCD a contiguous run of tile ids so
// that tiles sharing operand panels meet in the same L2.
__device__ __forceinline__ int xcd_contiguous_id(int pid, int grid) {
  int per = grid >> 3;  // grid is a multiple of 8
  return (pid & 7) * per + (pid >> 3);
}

template <int BM, int BN, int FM, int FN>
__device__ __forceinline__ void store_tile_rows(const f32x16 (&acc)[FM][FN], bf16_t *C, int ldc, const RowMap &cmap,
                                                int row0, int row_end, int col0, int ncols, int wm, int wn, int lane) {
#pragma unroll
  for (int fm = 0; fm < FM; ++fm) {
    int i = row0 + wm * (BM / 2) + fm * 32 + (lane & 31);
    if (i >= row_end) continue;
    bf16_t *crow = C + (size_t)map_row(cmap, i) * ldc;
#pragma unroll
    for (int fn = 0; fn < FN; ++fn) {
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        int n = col0 + wn * (BN / 2) + fn * 32 + 8 * g + 4 * (lane >> 5);
        if (n < ncols) {
          bf16x4 v;
#pragma unroll
          for (int q = 0; q < 4; ++q) v[q] = (bf16_t)acc[fm][fn][g * 4 + q];
          *reinterpret_cast<bf16x4 *>(crow + n) = v;
        }
      }
    }
  }
}

// ======================================================================================
// scatter2scatter: C[cmap(i), n0:n0+BN] = A[amap(i), :] * op(W[e])[:, n0:n0+BN]
// ======================================================================================
template <bool TRANS_W, int BM, int BN>
__global__ void __launch_bounds__(NTHREADS, 1) s2s_mfma_kernel(S2SArgs a, int tiles_n, int group_m) {
  constexpr int FM = BM / 64, FN = BN / 64;              // 32x32 fragments per wave
  constexpr int A_BYTES = BM * BK * 2, B_BYTES = BN * BK * 2, STAGE = A_BYTES + B_BYTES;
  extern __shared__ __attribute__((aligned(1024))) char smem[];

  // ---- which tile
  const int vid = xcd_contiguous_id(blockIdx.x, gridDim.x);
  const int tiles_per_group = group_m * tiles_n;
  const int grp = vid / tiles_per_group, in_grp = vid % tiles_per_group;
  const int mt = grp * group_m + in_grp % group_m;
  const int nt = in_grp / group_m;
  int e, row0, row_end;
  if (nt >= tiles_n || !locate_tile(a.offsets, a.E, BM, mt, e, row0, row_end)) return;
  const int n0 = nt * BN;

  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int wm = wave >> 1, wn = wave & 1;
  const bf16_t *A = (const bf16_t *)a.A;
  const bf16_t *W = (const bf16_t *)a.W + (size_t)e * a.w_stride;

  // ---- per-lane source pointers (contraction offset 0); rows past the segment re-read its last row
  const bf16_t *pa[BM / 32];
#pragma unroll
  for (int I = 0; I < BM / 32; ++I) {
    int r, c;
    kc_lane_slot<BM>(wave, lane, I, r, c);
    int i = min(row0 + r, row_end - 1);
    pa[I] = A + (size_t)map_row(a.a_map, i) * a.K + c * 8;
  }
  const bf16_t *pb[BN / 32];
#pragma unroll
  for (int I = 0; I < BN / 32; ++I) {
    int r, c;
    if (TRANS_W) {  // KC tile over rows n of W (row stride ldw), contraction along the row
      kc_lane_slot<BN>(wave, lane, I, r, c);
      int n = min(n0 + r, a.N - 1);
      pb[I] = W + (size_t)n * a.ldw + c * 8;
    } else {        // TR tile: contraction rows of W, BN columns
      tr_lane_slot<BN>(wave, lane, I, r, c);
      int col = n0 + c * 8;
      if (col >= a.N) col = 0;
      pb[I] = W + (size_t)r * a.ldw + col;
    }
  }
  const size_t b_step = TRANS_W ? (size_t)BK : (size_t)BK * a.ldw;

  const uint32_t lds0 = __builtin_amdgcn_readfirstlane(lds_address(smem));
  const int uwave = __builtin_amdgcn_readfirstlane(wave);
  auto issue = [&](int stage, int ks) {
    const uint32_t at = lds0 + stage * STAGE, bt = at + A_BYTES;
#pragma unroll
    for (int I = 0; I < BM / 32; ++I) load16_to_lds(pa[I] + (size_t)ks * BK, at + kc_inst_off<BM>(uwave, I));
#pragma unroll
    for (int I = 0; I < BN / 32; ++I)
      load16_to_lds(pb[I] + (size_t)ks * b_step, bt + (TRANS_W ? kc_inst_off<BN>(uwave, I) : tr_inst_off<BN>(uwave, I)));
  };
  auto frags = [&](const char *at, int kk, bf16x8(&fa)[FM], bf16x8(&fb)[FN]) {
    const char *bt = at + A_BYTES;
#pragma unroll
    for (int i = 0; i < FM; ++i) fa[i] = kc_frag(at, wm * (BM / 2) + i * 32, kk, lane);
#pragma unroll
    for (int j = 0; j < FN; ++j)
      fb[j] = TRANS_W ? kc_frag(bt, wn * (BN / 2) + j * 32, kk, lane) : tr_frag<BN>(bt, wn * (BN / 2) + j * 32, kk, lane);
  };

  f32x16 acc[FM][FN];
#pragma unroll
  for (int i = 0; i < FM; ++i)
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int q = 0; q < 16; ++q) acc[i][j][q] = 0.f;

  const int nsteps = a.K / BK;
  issue(0, 0);
  for (int ks = 0; ks < nsteps; ++ks) {
    wait_all_loads();
    __syncthreads();
    const char *at = smem + (ks & 1) * STAGE;
    bf16x8 fa[2][FM], fb[2][FN];
    frags(at, 0, fa[0], fb[0]);
    if (ks + 1 < nsteps) issue((ks + 1) & 1, ks + 1);
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
      if (kk + 1 < BK / 16) frags(at, kk + 1, fa[(kk + 1) & 1], fb[(kk + 1) & 1]);
#pragma unroll
      for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[kk & 1][j], fa[kk & 1][i], acc[i][j], 0, 0, 0);
      if (kk + 1 < BK / 16) interleave_mfma_dsread<FM * FN, FM + (TRANS_W ? FN : 2 * FN)>();
    }
  }
  store_tile_rows<BM, BN, FM, FN>(acc, (bf16_t *)a.C, a.N, a.c_map, row0, row_end, n0, a.N, wm, wn, lane);
}

// ======================================================================================
// groupXTY: dW[e][m0:m0+BM, n0:n0+BN] = sum over the expert's rows i of A[amap(i), m]^T B[bmap(i), n]
// ======================================================================================
template <int BM, int BN>
__global__ void __launch_bounds__(NTHREADS, 1) dw_mfma_kernel(DWArgs a, int tiles_m, int tiles_n) {
  constexpr int FM = BM / 64, FN = BN / 64;
  constexpr int A_BYTES = BM * BK * 2, B_BYTES = BN * BK * 2, STAGE = A_BYTES + B_BYTES;
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  __shared__ int s_expert;
  // Ring of source-row numbers, [slot][operand][row of the step]; -1 marks rows past the segment.
  // The numbers of step s are fetched from the routing arrays two steps early by 128 threads,
  // parked in a register, and published here one step early, so the gathered global->LDS
  // loads never wait on an index lookup.
  __shared__ int s_idx[4][2][BK];

  // Block ids map to tiles directly: consecutive blocks (dealt round-robin to the XCDs) share
  // an expert, so every XCD gets the same mix of long and short contractions.
  const int vid = blockIdx.x;
  const int per_expert = tiles_m * tiles_n;
  const int rank = vid / per_expert;
  if (rank >= a.E) return;
  // experts are visited largest first so that the long contractions start early
  for (int x = threadIdx.x; x < a.E; x += NTHREADS) {
    int nx = a.offsets[x + 1] - a.offsets[x], before = 0;
    for (int y = 0; y < a.E; ++y) {
      int ny = a.offsets[y + 1] - a.offsets[y];
      before += (ny > nx) || (ny == nx && y < x);
    }
    if (before == rank) s_expert = x;
  }
  __syncthreads();
  const int e = s_expert;
  const int t = vid % per_expert;
  const int m0 = (t % tiles_m) * BM, n0 = (t / tiles_m) * BN;
  const int lo = a.offsets[e], hi = a.offsets[e + 1];
  const int nsteps = (hi - lo + BK - 1) / BK;

  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int wm = wave >> 1, wn = wave & 1;
  const bf16_t *A = (const bf16_t *)a.A;
  const bf16_t *B = (const bf16_t *)a.B;

  // per-lane tile slots: contraction row within the step and column offset (elements)
  int ra[BM / 32], ca[BM / 32], rb[BN / 32], cb[BN / 32];
#pragma unroll
  for (int I = 0; I < BM / 32; ++I) {
    int c;
    tr_lane_slot<BM>(wave, lane, I, ra[I], c);
    ca[I] = m0 + c * 8;
    if (ca[I] >= a.M) ca[I] = 0;
  }
#pragma unroll
  for (int I = 0; I < BN / 32; ++I) {
    int c;
    tr_lane_slot<BN>(wave, lane, I, rb[I], c);
    cb[I] = n0 + c * 8;
    if (cb[I] >= a.N) cb[I] = 0;
  }
  const int irow = threadIdx.x & 63, iop = threadIdx.x >> 6;  // waves 0/1 look up rows of A/B
  auto lookup = [&](int ks) -> int {
    int i = lo + ks * BK + irow;
    if (iop >= 2 || i >= hi) return -1;
    return iop == 0 ? map_row(a.a_map, i) : map_row(a.b_map, i);
  };
  // source pointers of one step; rows past the segment read a block of zeros so they add
  // nothing to the sum
  const bf16_t *pa[BM / 32], *pb[BN / 32];
  auto resolve = [&](int ks) {
    const int slot = ks & 3;
#pragma unroll
    for (int I = 0; I < BM / 32; ++I) {
      int row = s_idx[slot][0][ra[I]];
      pa[I] = (row >= 0) ? A + (size_t)row * a.M + ca[I] : (const bf16_t *)g_zero16;
    }
#pragma unroll
    for (int I = 0; I < BN / 32; ++I) {
      int row = s_idx[slot][1][rb[I]];
      pb[I] = (row >= 0) ? B + (size_t)row * a.N + cb[I] : (const bf16_t *)g_zero16;
    }
  };
  const uint32_t lds0 = __builtin_amdgcn_readfirstlane(lds_address(smem));
  const int uwave = __builtin_amdgcn_readfirstlane(wave);
  auto issue = [&](int stage) {
    const uint32_t at = lds0 + stage * STAGE, bt = at + A_BYTES;
#pragma unroll
    for (int I = 0; I < BM / 32; ++I) load16_to_lds(pa[I], at + tr_inst_off<BM>(uwave, I));
#pragma unroll
    for (int I = 0; I < BN / 32; ++I) load16_to_lds(pb[I], bt + tr_inst_off<BN>(uwave, I));
  };
  auto frags = [&](const char *at, int kk, bf16x8(&fa)[FM], bf16x8(&fb)[FN]) {
    const char *bt = at + A_BYTES;
#pragma unroll
    for (int i = 0; i < FM; ++i) fa[i] = tr_frag<BM>(at, wm * (BM / 2) + i * 32, kk, lane);
#pragma unroll
    for (int j = 0; j < FN; ++j) fb[j] = tr_frag<BN>(bt, wn * (BN / 2) + j * 32, kk, lane);
  };

  f32x16 acc[FM][FN];
#pragma unroll
  for (int i = 0; i < FM; ++i)
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int q = 0; q < 16; ++q) acc[i][j][q] = 0.f;

  if (threadIdx.x < 128) {
    s_idx[0][iop][irow] = lookup(0);
    s_idx[1][iop][irow] = lookup(1);
  }
  int parked = lookup(2);
  __syncthreads();
  if (nsteps > 0) {
    resolve(0);
    issue(0);
  }
  for (int ks = 0; ks < nsteps; ++ks) {
    wait_all_loads();
    if (threadIdx.x < 128) s_idx[(ks + 2) & 3][iop][irow] = parked;
    __syncthreads();
    const char *at = smem + (ks & 1) * STAGE;
    bf16x8 fa[2][FM], fb[2][FN];
    frags(at, 0, fa[0], fb[0]);
    if (ks + 1 < nsteps) {
      resolve(ks + 1);
      issue((ks + 1) & 1);
    }
    parked = lookup(ks + 3);
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
      if (kk + 1 < BK / 16) frags(at, kk + 1, fa[(kk + 1) & 1], fb[(kk + 1) & 1]);
#pragma unroll
      for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[kk & 1][j], fa[kk & 1][i], acc[i][j], 0, 0, 0);
      if (kk + 1 < BK / 16) interleave_mfma_dsread<FM * FN, 2 * FM + 2 * FN>();
    }
  }
  bf16_t *dW = (bf16_t *)a.dW + (size_t)e * a.M * a.N;
  RowMap ident{nullptr, 1};
  store_tile_rows<BM, BN, FM, FN>(acc, dW, a.N, ident, m0, a.M, n0, a.N, wm, wn, lane);
}

template <typename K> int set_lds_limit(K kernel, int bytes) {
  return hipFuncSetAttribute((const void *)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes) == hipSuccess
             ? SMOE_OK
             : SMOE_ERR_HIP;
}

template <bool TRANS_W, int BM, int BN>
int launch_s2s_cfg(hipStream_t s, const S2SArgs &a) {
  constexpr int LDS = 2 * (BM + BN) * BK * 2;
  static int attr_rc = set_lds_limit(s2s_mfma_kernel<TRANS_W, BM, BN>, LDS);
  if (attr_rc != SMOE_OK) return attr_rc;
  int tiles_n = ceil_div(a.N, BN);
  int tiles_m = ceil_div(a.Tk, BM) + a.E;     // upper bound on sum_e ceil(n_e / BM)
  int group_m = 4;
  long long total = (long long)ceil_div(tiles_m, group_m) * group_m * tiles_n;
  total = (total + 7) / 8 * 8;
  if (total > 0x7fffffffLL) return SMOE_ERR_UNSUPPORTED;
  hipLaunchKernelGGL((s2s_mfma_kernel<TRANS_W, BM, BN>), dim3((unsigned)total), dim3(NTHREADS), LDS, s, a, tiles_n,
                     group_m);
  SMOE_LAUNCH_CHECK();
  return SMOE_OK;
}

template <int BM, int BN>
int launch_dw_cfg(hipStream_t s, const DWArgs &a) {
  constexpr int LDS = 2 * (BM + BN) * BK * 2;
  static int attr_rc = set_lds_limit(dw_mfma_kernel<BM, BN>, LDS);
  if (attr_rc != SMOE_OK) return attr_rc;
  int tiles_m = ceil_div(a.M, BM), tiles_n = ceil_div(a.N, BN);
  long long total = (long long)a.E * tiles_m * tiles_n;
  total = (total + 7) / 8 * 8;
  if (total > 0x7fffffffLL) return SMOE_ERR_UNSUPPORTED;
  hipLaunchKernelGGL((dw_mfma_kernel<BM, BN>), dim3((unsigned)total), dim3(NTHREADS), LDS, s, a, tiles_m, tiles_n);
  SMOE_LAUNCH_CHECK();
  return SMOE_OK;
}

}  // namespace

// The matrix-core kernels take contraction lengths that are multiples of 64 (no zero fill
// along k) and widths that are multiples of 8 (16-byte chunks never straddle a row end).
bool s2s_mfma_supported(const S2SArgs &a) { return a.K % BK == 0 && a.N % 8 == 0 && a.ldw % 8 == 0 && a.Tk > 0; }
bool dw_mfma_supported(const DWArgs &a) { return a.M % 8 == 0 && a.N % 8 == 0; }

int launch_s2s_mfma(hipStream_t s, const S2SArgs &a, int num_cu) {
  (void)num_cu;
  if (a.trans_w) return launch_s2s_cfg<true, 256, 256>(s, a);
  return launch_s2s_cfg<false, 256, 256>(s, a);
}

int launch_dw_mfma(hipStream_t s, const DWArgs &a, int num_cu) {
  (void)num_cu;
  return launch_dw_cfg<256, 256>(s, a);
}
