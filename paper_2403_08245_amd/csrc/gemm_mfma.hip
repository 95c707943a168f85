// bf16 matrix-core grouped GEMMs for gfx950 (MI355X):
//   * scatter2scatter (Sec. 3.2): rows gathered through the order indices, multiplied by the
//     row's expert matrix W[e] (forward) or W[e]^T (input gradient, Sec. 3.2.1), rows written
//     grouped or scattered.  The grouped copy of the input never exists in HBM: the gather
//     happens in the global->LDS load, the "padded tile" of Sec. 3.1 lives only in LDS.
//   * groupXTY (Sec. 3.2.1): dW[e] = Xbar_e^T dYbar_e over the expert's variable-length row
//     segment of the two grouped operands.
//
// Shape of every kernel: 256 threads = 4 wavefronts in a 2x2 grid over a 256x256 output tile
// (one wavefront per SIMD, 256 fp32 accumulator registers each), v_mfma_f32_32x32x16_bf16.
// The contraction runs in half-steps of 32 elements through a ring of four 32 KB LDS stages
// filled by direct-to-LDS 16-byte global loads (each lane supplies its own gathered address):
// while stage h is multiplied, stage h+1 has landed (its first fragments are prefetched across
// the barrier), stage h+2 is in flight and stage h+3 is being requested, one load instruction
// per four MFMAs so that neither the texture path nor the LDS ever sees a burst.  One barrier
// per half-step; the matrix pipe has its next operands in registers when it is released.
//
// Two LDS tile layouts, both XOR-swizzled at 16-byte granularity so that the fragment reads
// are bank-conflict free:
//   KC tile: rows x 32 contraction elements, contraction contiguous (64 B per row); a lane's
//            8 consecutive-k fragment comes from one ds_read_b128.
//   TR tile: 32 contraction rows x 256 columns, columns contiguous; fragments come from two
//            ds_read_b64_tr_b16 (the transposing LDS read), which hand each lane 4
//            consecutive contraction elements of one column.
// Forward uses KC for X and TR for W; the input gradient uses KC for both (W^T is already
// contraction-contiguous); groupXTY uses TR for both operands.
#include "mfma_common.h"

namespace {

// Epilogue: the accumulators of a wavefront (128 x 128, a lane holds 4 consecutive columns of
// one row per register quad) are rounded to bf16, turned into row-major order through a
// private LDS patch (32 rows x 272 B, the 16 B pad keeps the 8-byte writes conflict free) and
// leave as 16-byte stores that cover 256 contiguous bytes of 4 destination rows each -- whole
// cache lines, also when the rows are scattered.  s_rows[r] is the destination row of tile row
// r, or -1 for rows past the segment / matrix end.
constexpr int EPI_ROW_BYTES = 272;
constexpr int EPI_WAVE_BYTES = 32 * EPI_ROW_BYTES;
__device__ __forceinline__ void store_tile(const f32x16 (&acc)[FR][FR], char *smem, const int *s_rows, bf16_t *C,
                                           int ldc, int col0, int ncols, int wave, int wm, int wn, int lane) {
  __syncthreads();  // every wavefront is done with the stage ring
  char *patch = smem + wave * EPI_WAVE_BYTES;
  const int wcol = col0 + wn * (TB / 2);
#pragma unroll
  for (int fm = 0; fm < FR; ++fm) {
#pragma unroll
    for (int fn = 0; fn < FR; ++fn) {
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        bf16x4 v;
#pragma unroll
        for (int q = 0; q < 4; ++q) v[q] = (bf16_t)acc[fm][fn][g * 4 + q];
        int col = fn * 32 + 8 * g + 4 * (lane >> 5);
        *reinterpret_cast<bf16x4 *>(patch + (lane & 31) * EPI_ROW_BYTES + col * 2) = v;
      }
    }
#pragma unroll
    for (int it = 0; it < 8; ++it) {
      int r = it * 4 + (lane >> 4);
      int chunk = lane & 15;
      bf16x8 v = *reinterpret_cast<const bf16x8 *>(patch + r * EPI_ROW_BYTES + chunk * 16);
      int dst = s_rows[wm * (TB / 2) + fm * 32 + r];
      int col = wcol + chunk * 8;
      if (dst >= 0 && col < ncols) *reinterpret_cast<bf16x8 *>(C + (size_t)dst * ldc + col) = v;
    }
  }
}

// --------------------------------------------------------------------------------------
// The shared contraction loop.  `Ops` supplies the operand-specific parts:
//   ops.begin_group(step)        called once before the 8 loads of a stage are issued
//   ops.load(I, step, lds_addr)  issues load instruction I (0..3 = A tile, 4..7 = B tile)
//   ops.frag_a / frag_b          fragment reads from a landed stage
//   Ops::EXTRA_LOADS             global loads issued by begin_group (counted by the waits)
// Steps past the last one are clamped to it: their loads refill a stage nobody reads again,
// which keeps the loop free of branches and the outstanding-load count constant.
// --------------------------------------------------------------------------------------
template <typename Ops>
__device__ __forceinline__ void contraction_loop(Ops &ops, int nh, char *smem, int wm, int wn, int lane,
                                                 f32x16 (&acc)[FR][FR]) {
  constexpr int PER_GROUP = 2 * NLD + Ops::EXTRA_LOADS;
  const uint32_t lds0 = __builtin_amdgcn_readfirstlane(lds_address(smem));
  const int last = nh - 1;

#pragma unroll
  for (int i = 0; i < FR; ++i)
#pragma unroll
    for (int j = 0; j < FR; ++j)
#pragma unroll
      for (int q = 0; q < 16; ++q) acc[i][j][q] = 0.f;
  if (nh <= 0) return;

  // prologue: stages 0..2 requested at once
#pragma unroll
  for (int st = 0; st < NSTAGE - 1; ++st) {
    int step = min(st, last);
    ops.begin_group(step);
#pragma unroll
    for (int I = 0; I < 2 * NLD; ++I) ops.load(I, step, lds0 + st * STAGE_BYTES + (I / NLD) * TILE_BYTES);
  }
  wait_loads<PER_GROUP>();  // stages 0 and 1 have landed (loads complete in order)
  __syncthreads();
  bf16x8 fa[2][FR], fb[2][FR];
#pragma unroll
  for (int i = 0; i < FR; ++i) fa[0][i] = ops.frag_a(smem, wm * (TB / 2) + i * 32, 0, lane);
#pragma unroll
  for (int j = 0; j < FR; ++j) fb[0][j] = ops.frag_b(smem + TILE_BYTES, wn * (TB / 2) + j * 32, 0, lane);

  for (int h = 0; h < nh; ++h) {
    // stage h+1 has landed for every wavefront and nobody still reads stage h-1
    wait_loads<PER_GROUP>();
    __syncthreads();
    const char *cur = smem + (h & 3) * STAGE_BYTES;
    const char *nxt = smem + ((h + 1) & 3) * STAGE_BYTES;
    const uint32_t fill = lds0 + ((h + 3) & 3) * STAGE_BYTES;
    const int fill_step = min(h + 3, last);
    ops.begin_group(fill_step);
    sched_fence();
#pragma unroll
    for (int kk = 0; kk < 2; ++kk) {
      // fragments read during this sub-step: (stage h, kk = 1) or (stage h+1, kk = 0)
      const char *src = kk == 0 ? cur : nxt;
      const int nkk = 1 - kk;
#pragma unroll
      for (int g = 0; g < FR; ++g) {
#pragma unroll
        for (int j = 0; j < FR; ++j)
          acc[g][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[kk][j], fa[kk][g], acc[g][j], 0, 0, 0);
        // next fragments in the order the next sub-step consumes them: b0 a0 b1 | b2 b3 a1 | a2 a3
        if (g == 0) {
          fb[nkk][0] = ops.frag_b(src + TILE_BYTES, wn * (TB / 2) + 0 * 32, nkk, lane);
          fa[nkk][0] = ops.frag_a(src, wm * (TB / 2) + 0 * 32, nkk, lane);
          fb[nkk][1] = ops.frag_b(src + TILE_BYTES, wn * (TB / 2) + 1 * 32, nkk, lane);
        } else if (g == 1) {
          fb[nkk][2] = ops.frag_b(src + TILE_BYTES, wn * (TB / 2) + 2 * 32, nkk, lane);
          fb[nkk][3] = ops.frag_b(src + TILE_BYTES, wn * (TB / 2) + 3 * 32, nkk, lane);
          fa[nkk][1] = ops.frag_a(src, wm * (TB / 2) + 1 * 32, nkk, lane);
        } else if (g == 2) {
          fa[nkk][2] = ops.frag_a(src, wm * (TB / 2) + 2 * 32, nkk, lane);
          fa[nkk][3] = ops.frag_a(src, wm * (TB / 2) + 3 * 32, nkk, lane);
        }
        // LDS reads ride behind the matrix instructions, then the group's global load
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
        }
        sched_fence();
        const int I = kk * FR + g;
        ops.load(I, fill_step, fill + (I / NLD) * TILE_BYTES);
        sched_fence();
      }
    }
  }
  wait_loads<0>();  // drain the refills of the last three half-steps
}

// ======================================================================================
// scatter2scatter: C[cmap(i), n0:n0+256] = A[amap(i), :] * op(W[e])[:, n0:n0+256]
// ======================================================================================
template <bool TRANS_W> struct S2SOps {
  static constexpr int EXTRA_LOADS = 0;
  const bf16_t *pa[NLD];   // per-lane source of each A load instruction at contraction offset 0
  const bf16_t *pb[NLD];
  size_t b_step;           // elements between consecutive half-steps of the B source
  int uwave;
  __device__ __forceinline__ void begin_group(int) {}
  __device__ __forceinline__ void load(int I, int step, uint32_t tile_lds) {
    if (I < NLD) load16_to_lds(pa[I] + (size_t)step * HK, tile_lds + inst_off(uwave, I));
    else load16_to_lds(pb[I - NLD] + (size_t)step * b_step, tile_lds + inst_off(uwave, I - NLD));
  }
  __device__ __forceinline__ bf16x8 frag_a(const char *tile, int base, int kk, int lane) {
    return kc_frag(tile, base, kk, lane);
  }
  __device__ __forceinline__ bf16x8 frag_b(const char *tile, int base, int kk, int lane) {
    return TRANS_W ? kc_frag(tile, base, kk, lane) : tr_frag(tile, base, kk, lane);
  }
};

template <bool TRANS_W>
__global__ void __launch_bounds__(NTHREADS, 1) s2s_mfma_kernel(S2SArgs a, int tiles_n, int group_m) {
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  __shared__ int s_rows[TB];

  // ---- which tile
  const int vid = xcd_contiguous_id(blockIdx.x, gridDim.x);
  const int tiles_per_group = group_m * tiles_n;
  const int grp = vid / tiles_per_group, in_grp = vid % tiles_per_group;
  const int mt = grp * group_m + in_grp % group_m;
  const int nt = in_grp / group_m;
  int e, row0, row_end;
  if (nt >= tiles_n || !locate_tile(a.offsets, a.E, mt, threadIdx.x & 63, e, row0, row_end)) return;
  const int n0 = nt * TB;

  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int wm = wave >> 1, wn = wave & 1;
  const bf16_t *A = (const bf16_t *)a.A;
  const bf16_t *W = (const bf16_t *)a.W + (size_t)e * a.w_stride;
  {  // destination row of every tile row (read again by the epilogue, after the loop's barriers)
    int i = row0 + (int)threadIdx.x;
    s_rows[threadIdx.x] = (i < row_end) ? map_row(a.c_map, i) : -1;
  }

  // ---- per-lane source pointers; rows past the segment re-read its last row (never stored)
  S2SOps<TRANS_W> ops;
  ops.uwave = __builtin_amdgcn_readfirstlane(wave);
#pragma unroll
  for (int I = 0; I < NLD; ++I) {
    int r, c;
    kc_lane_slot(wave, lane, I, r, c);
    int i = min(row0 + r, row_end - 1);
    ops.pa[I] = A + (size_t)map_row(a.a_map, i) * a.K + c * 8;
  }
#pragma unroll
  for (int I = 0; I < NLD; ++I) {
    int r, c;
    if (TRANS_W) {  // KC tile over rows n of W (row stride ldw), contraction along the row
      kc_lane_slot(wave, lane, I, r, c);
      int n = min(n0 + r, a.N - 1);
      ops.pb[I] = W + (size_t)n * a.ldw + c * 8;
    } else {        // TR tile: contraction rows of W, 256 columns
      tr_lane_slot(wave, lane, I, r, c);
      int col = n0 + c * 8;
      if (col >= a.N) col = 0;
      ops.pb[I] = W + (size_t)r * a.ldw + col;
    }
  }
  ops.b_step = TRANS_W ? (size_t)HK : (size_t)HK * a.ldw;

  f32x16 acc[FR][FR];
  contraction_loop(ops, a.K / HK, smem, wm, wn, lane, acc);
  store_tile(acc, smem, s_rows, (bf16_t *)a.C, a.N, n0, a.N, wave, wm, wn, lane);
}

// ======================================================================================
// groupXTY: dW[e][m0:m0+256, n0:n0+256] = sum over the expert's rows i of A[i, m]^T B[i, n]
// ======================================================================================
// Both operands are in expert-sorted order (Alg. 2 groups them first); rows past the segment
// read a block of zeros so they add nothing to the sum.
struct DWOps {
  static constexpr int EXTRA_LOADS = 0;
  const bf16_t *A, *B;
  int M, N, lo, hi;
  int ra[NLD], ca[NLD], cb[NLD];  // per load instruction: row within the step, column offsets
  int uwave;
  const bf16_t *pa[NLD], *pb[NLD];

  __device__ __forceinline__ void begin_group(int step) {
#pragma unroll
    for (int I = 0; I < NLD; ++I) {
      int i = lo + step * HK + ra[I];
      pa[I] = (i < hi) ? A + (size_t)i * M + ca[I] : (const bf16_t *)g_zero16;
      pb[I] = (i < hi) ? B + (size_t)i * N + cb[I] : (const bf16_t *)g_zero16;
    }
  }
  __device__ __forceinline__ void load(int I, int, uint32_t tile_lds) {
    if (I < NLD) load16_to_lds(pa[I], tile_lds + inst_off(uwave, I));
    else load16_to_lds(pb[I - NLD], tile_lds + inst_off(uwave, I - NLD));
  }
  __device__ __forceinline__ bf16x8 frag_a(const char *tile, int base, int kk, int l) { return tr_frag(tile, base, kk, l); }
  __device__ __forceinline__ bf16x8 frag_b(const char *tile, int base, int kk, int l) { return tr_frag(tile, base, kk, l); }
};

__global__ void __launch_bounds__(NTHREADS, 1) dw_mfma_kernel(DWArgs a, int tiles_m, int tiles_n) {
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  __shared__ int s_expert;
  __shared__ int s_rows[TB];

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
  const int m0 = (t % tiles_m) * TB, n0 = (t / tiles_m) * TB;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int wm = wave >> 1, wn = wave & 1;
  s_rows[threadIdx.x] = (m0 + (int)threadIdx.x < a.M) ? m0 + (int)threadIdx.x : -1;

  DWOps ops;
  ops.A = (const bf16_t *)a.A;
  ops.B = (const bf16_t *)a.B;
  ops.M = a.M;
  ops.N = a.N;
  ops.lo = a.offsets[e];
  ops.hi = a.offsets[e + 1];
  ops.uwave = __builtin_amdgcn_readfirstlane(wave);
#pragma unroll
  for (int I = 0; I < NLD; ++I) {
    int c;
    tr_lane_slot(wave, lane, I, ops.ra[I], c);
    ops.ca[I] = m0 + c * 8;
    if (ops.ca[I] >= a.M) ops.ca[I] = 0;
    ops.cb[I] = n0 + c * 8;
    if (ops.cb[I] >= a.N) ops.cb[I] = 0;
  }
  const int nh = (ops.hi - ops.lo + HK - 1) / HK;

  f32x16 acc[FR][FR];
  contraction_loop(ops, nh, smem, wm, wn, lane, acc);
  bf16_t *dW = (bf16_t *)a.dW + (size_t)e * a.M * a.N;
  store_tile(acc, smem, s_rows, dW, a.N, n0, a.N, wave, wm, wn, lane);
}

constexpr int LDS_BYTES = NSTAGE * STAGE_BYTES;

template <typename K> int set_lds_limit(K kernel, int bytes) {
  return hipFuncSetAttribute((const void *)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes) == hipSuccess
             ? SMOE_OK
             : SMOE_ERR_HIP;
}

template <bool TRANS_W> int launch_s2s_cfg(hipStream_t s, const S2SArgs &a) {
  int tiles_n = ceil_div(a.N, TB);
  int tiles_m = ceil_div(a.Tk, TB) + a.E;     // upper bound on sum_e ceil(n_e / 256)
  int group_m = 4;
  long long total = (long long)ceil_div(tiles_m, group_m) * group_m * tiles_n;
  total = (total + 7) / 8 * 8;
  if (total > 0x7fffffffLL) return SMOE_ERR_UNSUPPORTED;
  hipLaunchKernelGGL((s2s_mfma_kernel<TRANS_W>), dim3((unsigned)total), dim3(NTHREADS), LDS_BYTES, s, a, tiles_n,
                     group_m);
  SMOE_LAUNCH_CHECK();
  return SMOE_OK;
}

int launch_dw_impl(hipStream_t s, const DWArgs &a) {
  int tiles_m = ceil_div(a.M, TB), tiles_n = ceil_div(a.N, TB);
  long long total = (long long)a.E * tiles_m * tiles_n;
  if (total > 0x7fffffffLL) return SMOE_ERR_UNSUPPORTED;
  hipLaunchKernelGGL(dw_mfma_kernel, dim3((unsigned)total), dim3(NTHREADS), LDS_BYTES, s, a, tiles_m, tiles_n);
  SMOE_LAUNCH_CHECK();
  return SMOE_OK;
}

}  // namespace

// The matrix-core kernels take contraction lengths that are multiples of 32 (no zero fill
// along k) and widths that are multiples of 8 (16-byte chunks never straddle a row end).
bool s2s_mfma_supported(const S2SArgs &a) { return a.K % HK == 0 && a.N % 8 == 0 && a.ldw % 8 == 0 && a.Tk > 0; }
bool dw_mfma_supported(const DWArgs &a) { return a.M % 8 == 0 && a.N % 8 == 0 && a.Tk > 0; }

// Raises the dynamic LDS limit of every kernel of this file on the current device (once per context).
int init_mfma_kernels() {
  int rc = set_lds_limit(s2s_mfma_kernel<false>, LDS_BYTES);
  if (rc == SMOE_OK) rc = set_lds_limit(s2s_mfma_kernel<true>, LDS_BYTES);
  if (rc == SMOE_OK) rc = set_lds_limit(dw_mfma_kernel, LDS_BYTES);
  return rc;
}

int launch_s2s_mfma(hipStream_t s, const S2SArgs &a) {
  return a.trans_w ? launch_s2s_cfg<true>(s, a) : launch_s2s_cfg<false>(s, a);
}

int launch_dw_mfma(hipStream_t s, const DWArgs &a) {
  return launch_dw_impl(s, a);
}
