// Persistent ("stream") form of the bf16 matrix-core grouped GEMMs.
//
// One block per compute unit walks a list of 256x256 output tiles.  The four-stage LDS ring of
// the contraction loop never drains between tiles: the loader side runs three half-steps ahead
// of the multiplying side and simply moves on to the next tile's operand rows, so the next
// tile's first stages land while the current tile is being finished and written out.  Per tile
// this removes the block launch, the pipeline fill and the tile search from the critical path;
// what remains is the epilogue (accumulators -> bf16 -> LDS patch -> whole-line stores).
//
// Both sides visit the same sequence of slots (one per half-step, at least one per tile) with a
// fixed lag.  Exactly eight tile loads are issued
// per slot -- slots past the end of the list repeat a valid address -- so one constant
// `s_waitcnt vmcnt` per slot orders everything.  Row indices travel through LDS by
// direct-to-LDS loads as well: no ordinary global load sits in the loop, so the compiler never
// inserts a full wait in front of the loads that are meant to stay in flight.
#include "mfma_common.h"
#include <type_traits>

namespace {

constexpr int RING_BYTES = NSTAGE * STAGE_BYTES;          // 128 KB
constexpr int EPI_ROW_BYTES = 144;                        // 64 bf16 columns + 16 B pad
constexpr int EPI_WAVE_BYTES = 32 * EPI_ROW_BYTES;
constexpr int STREAM_LDS_BYTES = RING_BYTES + 4 * EPI_WAVE_BYTES;
constexpr int MAX_E = 256;                                // expert offsets are cached in LDS
constexpr int MAX_STREAM_GRID = 256;                      // persistent blocks: one per CU; the partial-tile scratch holds this many tiles

// Epilogue of one wavefront: its 128x128 accumulators leave in 8 passes of 32 rows x 64
// columns through a private LDS patch; every store instruction writes full 128-byte lines of
// 8 destination rows.  dst_row(r) gives the destination row of wave-tile row r or -1.
// Moves one accumulator element out of the accumulation register file right where it is
// used.  Left to itself the register allocator copies all 256 accumulators of a lane into
// ordinary registers at the top of the epilogue, which cannot fit beside the operand
// fragments and load addresses that stay live for the next tile.
__device__ __forceinline__ float acc_read(float a) {
  float v;
  __asm__ volatile("v_accvgpr_read_b32 %0, %1" : "=v"(v) : "a"(a));
  return v;
}

// ---- the LDS patch as a pipeline ------------------------------------------------------------------------
// A 32 x 64 block of bf16 results goes accumulator layout -> patch (8-byte writes, a lane's 4 consecutive columns)
// -> whole rows back out (16-byte reads, eight lanes per 128-byte row) -> global memory.  LDS operations of one
// wavefront execute in order, so the block's row reads may be issued right behind its writes and the next block's
// writes right behind those reads, with no wait in between; only the global stores need the read data.  The
// stores of block n are therefore issued after block n+1 has been written and read: the LDS latency of one block
// hides behind the accumulator reads and conversions of the next one instead of being sat out four times per block.
struct PatchRows {
  bf16x8 v[4];
};
__device__ __forceinline__ PatchRows read_patch_rows(const char *patch, int lane) {
  PatchRows r;
#pragma unroll
  for (int it = 0; it < 4; ++it)
    r.v[it] = *reinterpret_cast<const bf16x8 *>(patch + (it * 8 + (lane >> 3)) * EPI_ROW_BYTES + (lane & 7) * 16);
  return r;
}
// The rows read from the patch and where they go: destination rows of the lane's four chunks (-1: none), the
// tensor, its row stride, the lane's column in it, and whether that column exists.
struct RowStore {
  PatchRows rows;
  int drow[4];
  bf16_t *base;
  size_t ld;
  int col;
  bool col_ok, have;
};
__device__ __forceinline__ void issue_row_store(const RowStore &p, int lane) {
#pragma unroll
  for (int it = 0; it < 4; ++it) {
    bf16_t *dst = (p.drow[it] >= 0 && p.col_ok) ? p.base + (size_t)p.drow[it] * p.ld + p.col : (bf16_t *)g_trash + lane * 8;
    // Non-temporal: a launch streams gigabytes of output through each XCD's 4 MB L2, which also holds the operand
    // panels its 32 compute units share; marking the lines for early eviction keeps them from pushing the panels out
    // (3 % on the first product of the Mixtral-shaped layer, neutral on products with narrow outputs).
    __builtin_nontemporal_store(p.rows.v[it], reinterpret_cast<bf16x8 *>(dst));   // masked lanes hit the landing zone
  }
}
// One block through the pipeline: write_block() fills the patch from the accumulators; the previous block's
// stores go out behind this block's LDS traffic.  gcol is the block's first column among the `limit` columns of
// its destination, col0 the offset of those columns inside a row of `base`.
template <typename WriteFn>
__device__ __forceinline__ void pipe_block(RowStore &pend, const char *patch, int lane, WriteFn write_block, const int (&drow)[4],
                                           bf16_t *base, size_t ld, int col0, int gcol, int limit) {
  sched_fence();
  write_block();
  RowStore cur;
  cur.rows = read_patch_rows(patch, lane);
  sched_fence();
  if (pend.have) issue_row_store(pend, lane);
#pragma unroll
  for (int it = 0; it < 4; ++it) cur.drow[it] = drow[it];
  cur.base = base;
  cur.ld = ld;
  cur.col = col0 + gcol + (lane & 7) * 8;
  cur.col_ok = gcol + (lane & 7) * 8 < limit;
  cur.have = true;
  pend = cur;
}
// destination rows of the lane's chunks in every 32-row fragment row of the wave tile
template <typename RowFn> __device__ __forceinline__ void chunk_rows(RowFn dst_row, int lane, int (&drow)[FR][4]) {
#pragma unroll
  for (int fm = 0; fm < FR; ++fm)
#pragma unroll
    for (int it = 0; it < 4; ++it) drow[fm][it] = dst_row(fm * 32 + it * 8 + (lane >> 3));
}
// accumulators of one 32 x 32 fragment pair (64 columns) -> patch, rounded to bf16
__device__ __forceinline__ void acc_block_to_patch(const f32x16 &a0, const f32x16 &a1, char *patch, int lane) {
#pragma unroll
  for (int f2 = 0; f2 < 2; ++f2)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      bf16x4 v;
#pragma unroll
      for (int q = 0; q < 4; ++q) v[q] = (bf16_t)acc_read(f2 == 0 ? a0[g * 4 + q] : a1[g * 4 + q]);
      *reinterpret_cast<bf16x4 *>(patch + (lane & 31) * EPI_ROW_BYTES + (f2 * 32 + 8 * g + 4 * (lane >> 5)) * 2) = v;
    }
}

template <typename RowFn>
__device__ __forceinline__ void store_wave_tile(const f32x16 (&acc)[FR][FR], char *patch, RowFn dst_row, bf16_t *C,
                                                int ldc, int wcol, int ncols, int lane) {
  // the last matrix instructions must have retired before their results are read by hand
  __asm__ volatile("s_nop 15\n\ts_nop 15" ::: "memory");
  int drow[FR][4];
  chunk_rows(dst_row, lane, drow);
  RowStore pend;
  pend.have = false;
#pragma unroll
  for (int fm = 0; fm < FR; ++fm)
#pragma unroll
    for (int half = 0; half < 2; ++half)
      pipe_block(pend, patch, lane, [&] { acc_block_to_patch(acc[fm][half * 2], acc[fm][half * 2 + 1], patch, lane); }, drow[fm], C,
                 (size_t)ldc, 0, wcol + half * 64, ncols);
  sched_fence();
  issue_row_store(pend, lane);
}

// Epilogue of a SwiGLU tile: the wavefront's 128 accumulator columns are 64 gate columns (fragments 0, 1)
// and the 64 up columns that pair with them (fragments 2, 3), so a lane holds both factors of each hidden
// unit in matching registers.  Writes the pre-activation halves (KEEP) and H = silu(gate) * up, each
// through the same pipeline as above.  gcol is the first gate column of this wavefront, half_n the number of
// gate columns of the layer.
template <bool KEEP, typename RowFn>
__device__ __forceinline__ void store_wave_tile_swiglu(const f32x16 (&acc)[FR][FR], char *patch, RowFn dst_row, bf16_t *C,
                                                       bf16_t *H, int half_n, int gcol, int lane) {
  __asm__ volatile("s_nop 15\n\ts_nop 15" ::: "memory");
  int drow[FR][4];
  chunk_rows(dst_row, lane, drow);
  RowStore pend;
  pend.have = false;
#pragma unroll
  for (int fm = 0; fm < FR; ++fm) {
    if (KEEP) {
#pragma unroll
      for (int half = 0; half < 2; ++half)   // gate columns, then up columns of the pre-activation
        pipe_block(pend, patch, lane, [&] { acc_block_to_patch(acc[fm][half * 2], acc[fm][half * 2 + 1], patch, lane); }, drow[fm],
                   C, (size_t)2 * half_n, half * half_n, gcol, half_n);
    }
    pipe_block(pend, patch, lane, [&] {
#pragma unroll
      for (int f2 = 0; f2 < 2; ++f2)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          bf16x4 v;
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            float gate = acc_read(acc[fm][f2][g * 4 + q]), up = acc_read(acc[fm][2 + f2][g * 4 + q]);
            float sig = __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.4426950408889634f * gate));
            v[q] = (bf16_t)(gate * sig * up);
          }
          *reinterpret_cast<bf16x4 *>(patch + (lane & 31) * EPI_ROW_BYTES + (f2 * 32 + 8 * g + 4 * (lane >> 5)) * 2) = v;
        }
    }, drow[fm], H, (size_t)half_n, 0, gcol, half_n);
  }
  sched_fence();
  issue_row_store(pend, lane);
}

// Epilogue of the second ParallelLinear's input-gradient product with the SwiGLU derivative and Alg. 2's dp folded in.
// The accumulators hold dH / p for 128 hidden units of 128 expert-sorted rows (the product ran on the unweighted
// upstream rows).  Per 32-row fragment row the lane fetches the matching gate and up pre-activations (its own row,
// its own 4-column groups: 8-byte loads, the next 64 columns requested before the current ones are used), forms
// h = silu(gate) * up and the partial dot <acc, h> (summed over the wavefront's 128 columns: one slab of dp), scales
// the accumulators by the row's routing weight and writes
//   dgate = dh * up * (sig + silu * (1 - sig)),  dup = dh * silu
// to the two halves of dHpre through the patch pipeline.  Rows past the segment read its last row and columns
// past the width read column 0; neither is stored or added to the dot.
struct GateUp {
  bf16x4 gt[2][4], up[2][4];
};
__device__ __forceinline__ GateUp load_gate_up(const bf16_t *src, int half_n, int col_base, int lane) {
  GateUp r;
#pragma unroll
  for (int f2 = 0; f2 < 2; ++f2)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const int col = col_base + f2 * 32 + 8 * g + 4 * (lane >> 5);
      const int cc = col < half_n ? col : 0;
      r.gt[f2][g] = *reinterpret_cast<const bf16x4 *>(src + cc);
      r.up[f2][g] = *reinterpret_cast<const bf16x4 *>(src + half_n + cc);
    }
  return r;
}
template <typename RowFn>
__device__ __forceinline__ void store_wave_tile_swiglu_bwd(const f32x16 (&acc)[FR][FR], char *patch, RowFn dst_row,
                                                           const bf16_t *Hpre, bf16_t *dHpre, const float *row_scale,
                                                           float *dp_part, int part_ld, int part_col, int half_n, int gcol,
                                                           int row_base, int row_end, int lane) {
  __asm__ volatile("s_nop 15\n\ts_nop 15" ::: "memory");
  const size_t ld = (size_t)2 * half_n;
  // the lane's own row in a fragment row (source of the pre-activations and of the routing weight); rows past the
  // segment read its last row
  auto own_row = [&](int fm) { return min(row_base + fm * 32 + (lane & 31), row_end - 1); };
  RowStore pend;
  pend.have = false;
  GateUp in = load_gate_up(Hpre + (size_t)own_row(0) * ld, half_n, gcol, lane);
  float scale_next = row_scale[own_row(0)];
#pragma unroll
  for (int fm = 0; fm < FR; ++fm) {
    float dp = 0.f;
    const float scale = scale_next;
    int drow[4];      // destination rows of the lane's chunks in this fragment row (the rows are expert-sorted, never scattered)
#pragma unroll
    for (int it = 0; it < 4; ++it) drow[it] = dst_row(fm * 32 + it * 8 + (lane >> 3));
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      const GateUp cur = in;
      if (fm * 2 + half + 1 < 2 * FR) {   // request the next 64 columns (or the next fragment row) now
        const int nfm = half == 0 ? fm : fm + 1;
        in = load_gate_up(Hpre + (size_t)own_row(nfm) * ld, half_n, gcol + (half == 0 ? 64 : 0), lane);
        if (half == 1) scale_next = row_scale[own_row(nfm)];
      }
      bf16x4 du[2][4];
      pipe_block(pend, patch, lane, [&] {
#pragma unroll
        for (int f2 = 0; f2 < 2; ++f2)
#pragma unroll
          for (int g = 0; g < 4; ++g) {
            const int col = gcol + half * 64 + f2 * 32 + 8 * g + 4 * (lane >> 5);
            bf16x4 dg;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
              const float a = acc_read(acc[fm][half * 2 + f2][g * 4 + q]);
              const float gate = (float)cur.gt[f2][g][q], u = (float)cur.up[f2][g][q];
              const float sig = __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.4426950408889634f * gate));
              const float silu = gate * sig;
              if (col < half_n) dp = fmaf(a, silu * u, dp);
              const float dh = scale * a;
              dg[q] = (bf16_t)(dh * u * (sig + silu * (1.0f - sig)));
              du[f2][g][q] = (bf16_t)(dh * silu);
            }
            *reinterpret_cast<bf16x4 *>(patch + (lane & 31) * EPI_ROW_BYTES + (f2 * 32 + 8 * g + 4 * (lane >> 5)) * 2) = dg;
          }
      }, drow, dHpre, ld, 0, gcol + half * 64, half_n);
      pipe_block(pend, patch, lane, [&] {
#pragma unroll
        for (int f2 = 0; f2 < 2; ++f2)
#pragma unroll
          for (int g = 0; g < 4; ++g)
            *reinterpret_cast<bf16x4 *>(patch + (lane & 31) * EPI_ROW_BYTES + (f2 * 32 + 8 * g + 4 * (lane >> 5)) * 2) = du[f2][g];
      }, drow, dHpre, ld, half_n, gcol + half * 64, half_n);
    }
    dp += __shfl_xor(dp, 32, 64);
    if (row_base + fm * 32 + lane < row_end && lane < 32) dp_part[(size_t)(row_base + fm * 32 + lane) * part_ld + part_col] = dp;
  }
  sched_fence();
  issue_row_store(pend, lane);
}

// The activation-agnostic form: the accumulators hold dH / p; the lane fetches the saved hidden activations H of its
// row and column groups, adds <acc, H> to the row's slab of dp, and writes dH = p * acc (and Hw = p * H when asked).
template <typename RowFn>
__device__ __forceinline__ void store_wave_tile_dp(const f32x16 (&acc)[FR][FR], char *patch, RowFn dst_row, const bf16_t *H,
                                                   bf16_t *dH, bf16_t *Hw, const float *row_scale, float *dp_part, int part_ld,
                                                   int part_col, int n, int gcol, int row_base, int row_end, int lane) {
  __asm__ volatile("s_nop 15\n\ts_nop 15" ::: "memory");
  auto own_row = [&](int fm) { return min(row_base + fm * 32 + (lane & 31), row_end - 1); };
  auto load_h = [&](int fm, int half, bf16x4 (&h)[2][4]) {
    const bf16_t *src = H + (size_t)own_row(fm) * n;
#pragma unroll
    for (int f2 = 0; f2 < 2; ++f2)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int col = gcol + half * 64 + f2 * 32 + 8 * g + 4 * (lane >> 5);
        h[f2][g] = *reinterpret_cast<const bf16x4 *>(src + (col < n ? col : 0));
      }
  };
  RowStore pend;
  pend.have = false;
  bf16x4 nxt[2][4];
  load_h(0, 0, nxt);
  float scale_next = row_scale[own_row(0)];
#pragma unroll
  for (int fm = 0; fm < FR; ++fm) {
    float dp = 0.f;
    const float scale = scale_next;
    int drow[4];
#pragma unroll
    for (int it = 0; it < 4; ++it) drow[it] = dst_row(fm * 32 + it * 8 + (lane >> 3));
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      bf16x4 cur[2][4];
#pragma unroll
      for (int f2 = 0; f2 < 2; ++f2)
#pragma unroll
        for (int g = 0; g < 4; ++g) cur[f2][g] = nxt[f2][g];
      if (fm * 2 + half + 1 < 2 * FR) {   // request the next 64 columns (or the next fragment row) now
        load_h(half == 0 ? fm : fm + 1, half == 0 ? 1 : 0, nxt);
        if (half == 1) scale_next = row_scale[own_row(fm + 1)];
      }
      pipe_block(pend, patch, lane, [&] {
#pragma unroll
        for (int f2 = 0; f2 < 2; ++f2)
#pragma unroll
          for (int g = 0; g < 4; ++g) {
            const int col = gcol + half * 64 + f2 * 32 + 8 * g + 4 * (lane >> 5);
            bf16x4 v;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
              const float a = acc_read(acc[fm][half * 2 + f2][g * 4 + q]);
              if (col < n) dp = fmaf(a, (float)cur[f2][g][q], dp);
              v[q] = (bf16_t)(scale * a);
            }
            *reinterpret_cast<bf16x4 *>(patch + (lane & 31) * EPI_ROW_BYTES + (f2 * 32 + 8 * g + 4 * (lane >> 5)) * 2) = v;
          }
      }, drow, dH, (size_t)n, 0, gcol + half * 64, n);
      if (Hw)
        pipe_block(pend, patch, lane, [&] {
#pragma unroll
          for (int f2 = 0; f2 < 2; ++f2)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
              bf16x4 v;
#pragma unroll
              for (int q = 0; q < 4; ++q) v[q] = (bf16_t)(scale * (float)cur[f2][g][q]);
              *reinterpret_cast<bf16x4 *>(patch + (lane & 31) * EPI_ROW_BYTES + (f2 * 32 + 8 * g + 4 * (lane >> 5)) * 2) = v;
            }
        }, drow, Hw, (size_t)n, 0, gcol + half * 64, n);
    }
    dp += __shfl_xor(dp, 32, 64);
    if (row_base + fm * 32 + lane < row_end && lane < 32) dp_part[(size_t)(row_base + fm * 32 + lane) * part_ld + part_col] = dp;
  }
  sched_fence();
  issue_row_store(pend, lane);
}

// A wavefront's 128 x 128 accumulators as fp32 into a 256-wide partial tile (chunks of a split contraction).
__device__ __forceinline__ void store_wave_partial(const f32x16 (&acc)[FR][FR], float *dst, int lane) {
  __asm__ volatile("s_nop 15\n\ts_nop 15" ::: "memory");
#pragma unroll
  for (int fm = 0; fm < FR; ++fm)
#pragma unroll
    for (int fn = 0; fn < FR; ++fn) {
      sched_fence();
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        float4 v = make_float4(acc_read(acc[fm][fn][4 * g]), acc_read(acc[fm][fn][4 * g + 1]), acc_read(acc[fm][fn][4 * g + 2]),
                               acc_read(acc[fm][fn][4 * g + 3]));
        *reinterpret_cast<float4 *>(dst + (size_t)(fm * 32 + (lane & 31)) * TB + fn * 32 + 8 * g + 4 * (lane >> 5)) = v;
      }
    }
}

// One half-step of the contraction: 32 matrix instructions on the landed stage `cur`, the
// fragment reads of its second half and of the next stage's first half riding behind them, and
// the eight loads of the stage being refilled, one per four matrix instructions.  FIRST starts
// a tile: its first sixteen products overwrite the accumulators instead of adding to them.
template <bool FIRST, typename Ops>
__device__ __forceinline__ void half_step(Ops &ops, const char *cur, const char *nxt, uint32_t fill, int wm, int wn,
                                          int lane, bf16x8 (&fa)[2][FR], bf16x8 (&fb)[2][FR], f32x16 (&acc)[FR][FR]) {
  f32x16 zero;
#pragma unroll
  for (int q = 0; q < 16; ++q) zero[q] = 0.f;
  sched_fence();
#pragma unroll
  for (int kk = 0; kk < 2; ++kk) {
    const char *src = kk == 0 ? cur : nxt;
    const int nkk = 1 - kk;
#pragma unroll
    for (int g = 0; g < FR; ++g) {
#pragma unroll
      for (int j = 0; j < FR; ++j)
        acc[g][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[kk][j], fa[kk][g], (FIRST && kk == 0) ? zero : acc[g][j],
                                                            0, 0, 0);
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
      // the source address of this group's load is worked out in the shadow of the matrix instructions
      const int I = kk * FR + g;
      const auto src = ops.prepare(I);
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
      }
      sched_fence();
      ops.issue(I, src, fill + (I / NLD) * TILE_BYTES + inst_off(ops.uwave, I % NLD));
      sched_fence();
    }
  }
}

// ======================================================================================
// scatter2scatter, persistent
// ======================================================================================
struct S2STile {
  int seq;                    // position in this block's tile list (-1 before the first)
  int ord;                    // running number of the tile among the block's valid tiles
  int e, row0, row_end, n0;
  int h0, hn;                 // first half-step and number of half-steps this block contributes
  int part;                   // -1: the whole contraction, result stored directly; else index of the fp32 partial
};

// How the tiles of one launch are dealt to the G persistent blocks.  Tiles are numbered densely
// (groups of group_m M-tiles x all N-tiles); block b takes numbers seq * G + slot(b) for the `rounds`
// full rounds.  The remaining `rest` < G tiles would leave G - rest blocks idle for a whole tile, so
// their contraction is cut into `split` chunks of `chunk` half-steps, one block each; the chunks leave
// fp32 partial tiles that a second kernel adds in chunk order (deterministic) and stores.
struct TilePlan {
  int m_tiles, rounds, rest, split, chunk;
};
// A chunk's fp32 partial tile costs a 256 KB write and a 256 KB read on top of the second kernel's launch,
// about what 48 half-steps of multiplying take: a split must shorten the last round by more than that.
constexpr int SPLIT_MIN_SAVED = 64;
// Largest number of chunks <= max_split (and <= 4) that pays, with the chunk length; 1 = keep whole tiles.
__host__ __device__ inline int choose_split(int nh, int max_split, bool static4, int &chunk) {
  for (int s = max_split < 4 ? max_split : 4; s > 1; --s) {
    int c = (nh + s - 1) / s;
    if (static4) c = (c + 3) & ~3;
    if ((s - 1) * c < nh && nh - c >= SPLIT_MIN_SAVED) {
      chunk = c;
      return s;
    }
  }
  chunk = nh;
  return 1;
}
__device__ __forceinline__ TilePlan plan_tiles(const int32_t *offsets, int E, int tiles_n, int nh, int G, bool static4,
                                               bool may_split, int lane) {
  int sum = 0;
  for (int c0 = 0; c0 < E; c0 += 64) {
    int x = c0 + lane;
    int n = x < E ? (offsets[x + 1] - offsets[x] + TB - 1) / TB : 0;
#pragma unroll
    for (int d = 32; d > 0; d >>= 1) n += __shfl_xor(n, d, 64);
    sum += n;
  }
  TilePlan p;
  p.m_tiles = __builtin_amdgcn_readfirstlane(sum);
  const long long total = (long long)p.m_tiles * tiles_n;
  p.rounds = (int)(total / G);
  p.rest = (int)(total - (long long)p.rounds * G);
  p.split = 1;
  p.chunk = nh;
  if (may_split && p.rest > 0) p.split = choose_split(nh, G / p.rest, static4, p.chunk);
  return p;
}
// dense tile number -> (M-tile, N-tile): groups of group_m M-tiles (the last group may be narrower)
__device__ __forceinline__ void tile_coords(int w, int m_tiles, int tiles_n, int group_m, int &mt, int &nt) {
  const int per_group = group_m * tiles_n, full = m_tiles / group_m;
  int grp = w / per_group;
  if (grp < full) {
    int in_grp = w - grp * per_group;
    mt = grp * group_m + in_grp % group_m;
    nt = in_grp / group_m;
  } else {
    int last = m_tiles - full * group_m, in_grp = w - full * per_group;
    mt = full * group_m + in_grp % last;
    nt = in_grp / last;
  }
}

template <bool TRANS_W> struct S2SStreamOps {
  // Sources of the loader's current tile: wave-uniform bases plus per-lane 32-bit byte offsets at
  // contraction offset 0 (the launcher only takes this kernel when every offset fits 32 bits).
  const char *base_a, *base_b;
  uint32_t oa[NLD], ob[NLD];
  uint32_t b_step;                   // bytes the W source moves per half-step
  int step;                          // half-step the next loads fetch
  int uwave;
  __device__ __forceinline__ uint32_t prepare(int I) const {
    return I < NLD ? oa[I] + (uint32_t)step * (HK * 2) : ob[I - NLD] + (uint32_t)step * b_step;
  }
  __device__ __forceinline__ void issue(int I, uint32_t off, uint32_t lds) const {
    load16_to_lds(I < NLD ? base_a : base_b, off, lds);
  }
  __device__ __forceinline__ void load(int I, uint32_t tile_lds) {
    issue(I, prepare(I), tile_lds + inst_off(uwave, I % NLD));
  }
  __device__ __forceinline__ bf16x8 frag_a(const char *tile, int base, int kk, int lane) {
    return kc_frag(tile, base, kk, lane);
  }
  __device__ __forceinline__ bf16x8 frag_b(const char *tile, int base, int kk, int lane) {
    return TRANS_W ? kc_frag(tile, base, kk, lane) : tr_frag(tile, base, kk, lane);
  }
};

// ACT 1: fused SwiGLU keeping the pre-activation, 2: without, 3: fused SwiGLU derivative and dp (the W2^T input-gradient
// product of Alg. 3's backward, see store_wave_tile_swiglu_bwd), 4: dp from the saved H in that product's epilogue for any
// activation (store_wave_tile_dp).  STATIC4: the contraction is a multiple of four
// half-steps, so every tile starts in LDS stage 0 and the loop is written out four slots at a time with the
// stage as a compile-time constant: all LDS addresses become a loop-invariant register plus an immediate.
template <bool TRANS_W, bool SCATTER_OUT, int ACT = 0, bool STATIC4 = false>
__global__ void __launch_bounds__(NTHREADS, 1) s2s_stream_kernel(S2SArgs a, int tiles_n, int group_m, uint32_t magic_a) {
  constexpr bool SWIGLU = ACT == 1 || ACT == 2;
  constexpr bool SWIGLU_BWD = ACT == 3;
  constexpr bool DP_EPI = ACT == 4;
  static_assert(!SWIGLU || (!TRANS_W && !SCATTER_OUT), "the fused activation belongs to the forward, sorted-output product");
  static_assert(!(SWIGLU_BWD || DP_EPI) || (TRANS_W && !SCATTER_OUT), "the fused derivative belongs to the W^T product with sorted rows in and out");
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  __shared__ int s_off[MAX_E + 1];
  // Order indices of the rows of up to four open tiles.  With the shortest contraction the kernel takes (three
  // half-steps) the loader has opened tile n+2 and requested the rows of tile n+3 while tile n's epilogue still
  // reads its destination rows, so four entries are live at once.
  __shared__ int s_idx[4][TB];

  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int wm = wave >> 1, wn = wave & 1;
  const int uwave = __builtin_amdgcn_readfirstlane(wave);
  const int G = gridDim.x;
  const int slot_in_round = ((int)blockIdx.x & 7) * (G >> 3) + ((int)blockIdx.x >> 3);  // XCD-contiguous tiles
  const int nh = a.K / HK;
  const int32_t *o = a.a_map.o ? a.a_map.o : a.c_map.o;   // both maps use the same order indices
  const bf16_t *A = (const bf16_t *)a.A;

  const unsigned long long probe_c0 = a.clock_probe ? clock64() : 0ull, probe_t0 = a.clock_probe ? wall_clock64() : 0ull;
  for (int i = threadIdx.x; i <= a.E; i += NTHREADS) s_off[i] = a.offsets[i];
  __syncthreads();

  const TilePlan plan = plan_tiles(s_off, a.E, tiles_n, nh, G, STATIC4, ACT == 0 && a.tail_ws != nullptr, lane);
  // next tile (or chunk of a tile of the last round) of this block after t
  auto next_tile = [&](S2STile &t) -> bool {
    const int seq = t.seq + 1;
    int w, chunk = 0;
    bool split = false;
    if (seq < plan.rounds) {
      w = seq * G + slot_in_round;
    } else if (seq == plan.rounds && slot_in_round < plan.rest * plan.split) {
      w = plan.rounds * G + slot_in_round / plan.split;
      chunk = slot_in_round % plan.split;
      split = plan.split > 1;
    } else {
      return false;
    }
    int mt, nt, e, row0, row_end;
    tile_coords(w, plan.m_tiles, tiles_n, group_m, mt, nt);
    locate_tile(s_off, a.E, mt, lane, e, row0, row_end);
    t.seq = seq;
    t.ord += 1;
    t.e = __builtin_amdgcn_readfirstlane(e);
    t.row0 = __builtin_amdgcn_readfirstlane(row0);
    t.row_end = __builtin_amdgcn_readfirstlane(row_end);
    t.n0 = nt * (SWIGLU ? TB / 2 : TB);   // SwiGLU tiles hold 128 gate columns and the 128 up columns pairing with them
    t.h0 = split ? chunk * plan.chunk : 0;
    t.hn = split ? min(nh, t.h0 + plan.chunk) - t.h0 : nh;
    t.part = split ? (w - plan.rounds * G) * plan.split + chunk : -1;
    return true;
  };
  // order indices of a tile's 256 rows -> s_idx[ord & 3] (rows past the segment repeat its last row)
  auto fetch_rows = [&](const S2STile &t) {
    if (!o) return;
    int i = min(t.row0 + wave * 64 + lane, t.row_end - 1);
    load4_to_lds(o + i, __builtin_amdgcn_readfirstlane(lds_address((const char *)&s_idx[t.ord & 3][0])) + uwave * 256);
  };

  S2SStreamOps<TRANS_W> ops;
  ops.uwave = uwave;
  ops.b_step = TRANS_W ? (uint32_t)(HK * 2) : (uint32_t)(HK * 2) * (uint32_t)a.ldw;
  auto setup_pointers = [&](const S2STile &t) {
    // the tile's (chunk of the) contraction starts at half-step h0
    ops.base_b = (const char *)((const bf16_t *)a.W + (size_t)t.e * a.w_stride) + (size_t)t.h0 * ops.b_step;
    // gathered rows are addressed from the start of A, expert-sorted rows from the tile's first row
    ops.base_a = (const char *)(a.a_map.o ? A : A + (size_t)t.row0 * a.K) + (size_t)t.h0 * (HK * 2);
    const int *idx = &s_idx[t.ord & 3][0];
    const uint32_t row_bytes = (uint32_t)a.K * 2u;
#pragma unroll
    for (int I = 0; I < NLD; ++I) {
      int r, c;
      kc_lane_slot(wave, lane, I, r, c);
      uint32_t src;
      if (a.a_map.o) {
        uint32_t slot = (uint32_t)idx[r];
        src = magic_a ? __umulhi(slot, magic_a) : slot;
      } else {
        src = (uint32_t)min(r, t.row_end - 1 - t.row0);
      }
      ops.oa[I] = src * row_bytes + (uint32_t)c * 16u;
    }
#pragma unroll
    for (int I = 0; I < NLD; ++I) {
      int r, c;
      if (TRANS_W) {
        kc_lane_slot(wave, lane, I, r, c);
        int n = min(t.n0 + r, a.N - 1);
        ops.ob[I] = (uint32_t)n * (uint32_t)a.ldw * 2u + (uint32_t)c * 16u;
      } else {
        tr_lane_slot(wave, lane, I, r, c);
        int col = t.n0 + c * 8;
        if (SWIGLU) {
          // tile column v = c * 8: wavefront column half v / 128 takes 64 gate columns then their 64 up columns
          const int v = c * 8, w = v & 127, gate = t.n0 + (v >> 7) * 64 + (w & 63);
          col = (gate < a.N / 2) ? gate + (w >> 6) * (a.N / 2) : a.N;
        }
        if (col >= a.N) col = 0;
        ops.ob[I] = (uint32_t)r * (uint32_t)a.ldw * 2u + (uint32_t)col * 2u;
      }
    }
  };

  // ---- open the first two tiles
  S2STile lt{-1, -1, 0, 0, 0, 0, 0, 0, -1};
  if (!next_tile(lt)) return;
  S2STile ct = lt;             // the multiplying side starts on the same tile
  S2STile upcoming = lt;       // tile the loader will open next
  bool have_upcoming = next_tile(upcoming);
  fetch_rows(lt);
  if (have_upcoming) fetch_rows(upcoming);
  wait_loads<0>();
  __syncthreads();
  setup_pointers(lt);
  ops.step = 0;
  bool loader_live = true;
  // loader moves one slot on; at a tile end it opens the upcoming tile and requests the rows of the one after
  auto advance_loader = [&]() {
    if (!loader_live) return;
    if (++ops.step < lt.hn) return;
    if (!have_upcoming) {
      loader_live = false;
      ops.step = lt.hn - 1;   // slots past the end repeat the last stage's addresses
      return;
    }
    lt = upcoming;
    ops.step = 0;
    have_upcoming = next_tile(upcoming);
    if (have_upcoming) fetch_rows(upcoming);
    setup_pointers(lt);
  };

  const uint32_t lds0 = __builtin_amdgcn_readfirstlane(lds_address(smem));
  char *patch = smem + RING_BYTES + wave * EPI_WAVE_BYTES;
#pragma unroll 1
  for (int st = 0; st < NSTAGE - 1; ++st) {
#pragma unroll
    for (int I = 0; I < 2 * NLD; ++I) ops.load(I, lds0 + st * STAGE_BYTES + (I / NLD) * TILE_BYTES);
    advance_loader();
  }
  wait_loads<2 * NLD>();
  __syncthreads();
  bf16x8 fa[2][FR], fb[2][FR];
  f32x16 acc[FR][FR];
#pragma unroll
  for (int i = 0; i < FR; ++i) fa[0][i] = ops.frag_a(smem, wm * (TB / 2) + i * 32, 0, lane);
#pragma unroll
  for (int j = 0; j < FR; ++j) fb[0][j] = ops.frag_b(smem + TILE_BYTES, wn * (TB / 2) + j * 32, 0, lane);

  int g = 0;   // slot counter: slot g lives in stage g & 3
  auto open_slot = [&]() {
    wait_loads<2 * NLD>();   // stage g+1 has landed for every wavefront, stage g-1 is free
    __syncthreads();
  };
  auto one_slot = [&](auto first) {
    const char *cur = smem + (g & 3) * STAGE_BYTES;
    const char *nxt = smem + ((g + 1) & 3) * STAGE_BYTES;
    const uint32_t fill = lds0 + ((g + 3) & 3) * STAGE_BYTES;
    half_step<decltype(first)::value>(ops, cur, nxt, fill, wm, wn, lane, fa, fb, acc);
    advance_loader();
    ++g;
  };
  auto static_slot = [&](auto first, auto stage) {
    constexpr int S = decltype(stage)::value;
    half_step<decltype(first)::value>(ops, smem + S * STAGE_BYTES, smem + ((S + 1) & 3) * STAGE_BYTES,
                                      lds0 + ((S + 3) & 3) * STAGE_BYTES, wm, wn, lane, fa, fb, acc);
    advance_loader();
  };
  using I0 = std::integral_constant<int, 0>;
  using I1 = std::integral_constant<int, 1>;
  using I2 = std::integral_constant<int, 2>;
  using I3 = std::integral_constant<int, 3>;
  open_slot();
  for (;;) {   // one tile per trip; its first slot has been opened already
    if (STATIC4) {
      static_slot(std::true_type{}, I0{});
      open_slot();
      static_slot(std::false_type{}, I1{});
      open_slot();
      static_slot(std::false_type{}, I2{});
      open_slot();
      static_slot(std::false_type{}, I3{});
      for (int h = 4; h < ct.hn; h += 4) {
        open_slot();
        static_slot(std::false_type{}, I0{});
        open_slot();
        static_slot(std::false_type{}, I1{});
        open_slot();
        static_slot(std::false_type{}, I2{});
        open_slot();
        static_slot(std::false_type{}, I3{});
      }
    } else {
      one_slot(std::true_type{});
      for (int h = 1; h < ct.hn; ++h) {
        open_slot();
        one_slot(std::false_type{});
      }
    }
    // The next tile's first slot is opened before the epilogue: stores share the load counter,
    // so this wait would otherwise also sit out the acknowledgement of every store below.
    open_slot();
    const int *idx = &s_idx[ct.ord & 3][wm * (TB / 2)];
    const int rbase = ct.row0 + wm * (TB / 2);
    auto dst_row = [&](int r) -> int {
      int i = rbase + r;
      int row = SCATTER_OUT ? idx[r] : i;
      return (i < ct.row_end) ? row : -1;
    };
    if (SWIGLU)
      store_wave_tile_swiglu<ACT == 1>(acc, patch, dst_row, (bf16_t *)a.C, (bf16_t *)a.H, a.N / 2, ct.n0 + wn * (TB / 4), lane);
    else if (SWIGLU_BWD)
      store_wave_tile_swiglu_bwd(acc, patch, dst_row, (const bf16_t *)a.Hpre_in, (bf16_t *)a.C, a.row_scale, a.dp_part, 2 * tiles_n,
                                 (ct.n0 / TB) * 2 + wn, a.N, ct.n0 + wn * (TB / 2), rbase, ct.row_end, lane);
    else if (DP_EPI)
      store_wave_tile_dp(acc, patch, dst_row, (const bf16_t *)a.H_in, (bf16_t *)a.C, (bf16_t *)a.Hw_out, a.row_scale, a.dp_part, 2 * tiles_n,
                         (ct.n0 / TB) * 2 + wn, a.N, ct.n0 + wn * (TB / 2), rbase, ct.row_end, lane);
    else if (ct.part >= 0)
      store_wave_partial(acc, a.tail_ws + (size_t)ct.part * TB * TB + (size_t)(wm * (TB / 2)) * TB + wn * (TB / 2), lane);
    else
      store_wave_tile(acc, patch, dst_row, (bf16_t *)a.C, a.N, ct.n0 + wn * (TB / 2), a.N, lane);
    if (!next_tile(ct)) break;
  }
  wait_loads<0>();
  if (a.clock_probe && threadIdx.x == 0) {
    a.clock_probe[2 * blockIdx.x] = clock64() - probe_c0;
    a.clock_probe[2 * blockIdx.x + 1] = wall_clock64() - probe_t0;
  }
}

// Second pass of a split last round: adds the chunks' fp32 partial tiles in chunk order, rounds once and
// stores the rows where the unsplit epilogue would have (expert-sorted or scattered).  TAIL_SLICES blocks
// (32 rows each) per tile of the last round; the plan is recomputed from the same inputs as in the main kernel.
constexpr int TAIL_SLICES = 8;
template <bool SCATTER_OUT>
__global__ void __launch_bounds__(256) s2s_tail_reduce_kernel(S2SArgs a, int tiles_n, int group_m, int G, int static4) {
  __shared__ int s_off[MAX_E + 1];
  const int lane = threadIdx.x & 63;
  for (int i = threadIdx.x; i <= a.E; i += 256) s_off[i] = a.offsets[i];
  __syncthreads();
  const TilePlan plan = plan_tiles(s_off, a.E, tiles_n, a.K / HK, G, static4 != 0, true, lane);
  if (plan.split <= 1 || (int)blockIdx.x >= plan.rest) return;
  int mt, nt, e, row0, row_end;
  tile_coords(plan.rounds * G + (int)blockIdx.x, plan.m_tiles, tiles_n, group_m, mt, nt);
  locate_tile(s_off, a.E, mt, lane, e, row0, row_end);
  const int n0 = nt * TB;
  const float *part = a.tail_ws + (size_t)blockIdx.x * plan.split * TB * TB;
  bf16_t *C = (bf16_t *)a.C;
  constexpr int PER_SLICE = TB * TB / 4 / TAIL_SLICES;
  for (int i = (int)blockIdx.y * PER_SLICE + threadIdx.x; i < ((int)blockIdx.y + 1) * PER_SLICE; i += 256) {
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int c = 0; c < plan.split; ++c) {
      const float4 v = reinterpret_cast<const float4 *>(part + (size_t)c * TB * TB)[i];
      acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
    }
    const int row = row0 + (i * 4) / TB, col = n0 + (i * 4) % TB;
    if (row < row_end && col < a.N) {
      const int dst = SCATTER_OUT ? a.c_map.o[row] : row;
      bf16x4 o;
      o[0] = (bf16_t)acc.x; o[1] = (bf16_t)acc.y; o[2] = (bf16_t)acc.z; o[3] = (bf16_t)acc.w;
      *reinterpret_cast<bf16x4 *>(C + (size_t)dst * a.N + col) = o;
    }
  }
}

// ======================================================================================
// groupXTY, persistent: dW[e] = Xbar_e^T dYbar_e over expert-sorted rows (Alg. 2 groups both
// operands first; gathering the token rows inside this kernel measured a third slower than a
// `group` copy followed by this kernel, the same ranking the paper reports).
// ======================================================================================
// The loader cursor runs three slots ahead of the multiplying cursor over the same slot
// sequence: the half-steps of a tile rounded up to a multiple of four (at least four) slots,
// tiles in largest-expert-first order.  Slots past a segment's end load a block of zeros, so a
// tile of an empty expert multiplies zeros and writes zeros.
struct DWCursor {
  int seq;        // position in this block's tile list
  int step, ns;   // slot within the tile, slots of the tile
  int nh;         // half-steps (0 for an empty expert)
  int e, lo, hi, m0, n0;
  bool live;
};

struct DWStreamOps {
  int ra[NLD], ka[NLD];      // per load instruction: contraction row within a slot, 16-byte column chunk
  int uwave;
  // The loader's current group of four slots: range-checked windows that start at the group's first
  // row and end with the expert's segment (rows past it, padded slots and empty experts read zeros and
  // add nothing to the sum), per-lane byte offsets of the tile's columns inside a slot, and the byte
  // offset of the current slot inside the group.
  int32x4 win_a, win_b;
  uint32_t oa[NLD], ob[NLD];
  uint32_t sub_a, sub_b;
  __device__ __forceinline__ uint32_t prepare(int I) const { return I < NLD ? oa[I] + sub_a : ob[I - NLD] + sub_b; }
  __device__ __forceinline__ void issue(int I, uint32_t off, uint32_t lds) const {
    load16_to_lds_checked(I < NLD ? win_a : win_b, off, lds);
  }
  __device__ __forceinline__ void load(int I, uint32_t tile_lds) { issue(I, prepare(I), tile_lds + inst_off(uwave, I % NLD)); }
  __device__ __forceinline__ bf16x8 frag_a(const char *tile, int base, int kk, int l) { return tr_frag(tile, base, kk, l); }
  __device__ __forceinline__ bf16x8 frag_b(const char *tile, int base, int kk, int l) { return tr_frag(tile, base, kk, l); }
};

// tile number inside an expert -> first row and column of the tile: bands of group_m M-tiles, N-tile by
// N-tile, so that the 32 consecutive tiles an XCD holds at a time form a compact patch sharing few panels
__device__ __forceinline__ void dw_tile_origin(int t, int tiles_m, int tiles_n, int &m0, int &n0) {
  const int group_m = (tiles_m % 8 == 0) ? 8 : ((tiles_m % 4 == 0) ? 4 : ((tiles_m % 2 == 0) ? 2 : 1));
  const int band = t / (group_m * tiles_n), r = t - band * (group_m * tiles_n);
  m0 = (band * group_m + r % group_m) * TB;
  n0 = (r / group_m) * TB;
}
// rows of chunk `chunk` of `split` of the segment [lo, hi): chunks are whole groups of four half-steps
__device__ __forceinline__ void dw_chunk_rows(int lo, int hi, int split, int chunk, int &clo, int &chi) {
  const int nh = (hi - lo + HK - 1) / HK;
  const int len = (((nh + split - 1) / split + 3) & ~3) * HK;
  clo = min(hi, lo + chunk * len);
  chi = min(hi, clo + len);
}

// split > 1 (only when all experts' tiles times split fit one round of the grid): unit T is chunk T % split of
// tile T / split, experts in their own order, and the result is an fp32 partial tile number T in a.split_ws.
__global__ void __launch_bounds__(NTHREADS, 1) dw_stream_kernel(DWArgs a, int tiles_m, int tiles_n, int split) {
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  __shared__ int s_off[MAX_E + 1];
  __shared__ int s_order[MAX_E];      // experts, largest segment first

  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int wm = wave >> 1, wn = wave & 1;
  const int G = gridDim.x;
  const int slot_in_round = ((int)blockIdx.x & 7) * (G >> 3) + ((int)blockIdx.x >> 3);  // XCD-contiguous tiles
  const int per_expert = tiles_m * tiles_n;

  for (int i = threadIdx.x; i <= a.E; i += NTHREADS) s_off[i] = a.offsets[i];
  __syncthreads();
  for (int x = threadIdx.x; x < a.E; x += NTHREADS) {
    int nx = s_off[x + 1] - s_off[x], before = 0;
    for (int y = 0; y < a.E; ++y) {
      int ny = s_off[y + 1] - s_off[y];
      before += (ny > nx) || (ny == nx && y < x);
    }
    s_order[before] = x;
  }
  __syncthreads();

  auto open_tile = [&](DWCursor &c, int seq) {
    c.seq = seq;
    const int U = seq * G + slot_in_round;
    const int T = U / split;
    int rank = T / per_expert;
    c.live = rank < a.E && (split == 1 || seq == 0);
    if (!c.live) return;
    int t = T - rank * per_expert;
    c.e = split > 1 ? rank : __builtin_amdgcn_readfirstlane(s_order[rank]);   // LDS reads land in vector registers: make them scalar again
    c.lo = __builtin_amdgcn_readfirstlane(s_off[c.e]);
    c.hi = __builtin_amdgcn_readfirstlane(s_off[c.e + 1]);
    if (split > 1) dw_chunk_rows(c.lo, c.hi, split, U - T * split, c.lo, c.hi);
    dw_tile_origin(t, tiles_m, tiles_n, c.m0, c.n0);
    c.nh = (c.hi - c.lo + HK - 1) / HK;
    // Slots come in groups of four so that every tile starts in LDS stage 0 and the loop can be written
    // with compile-time stages; the up to three extra slots (four for an empty expert) load the zero
    // block and add nothing.
    c.ns = max((c.nh + 3) & ~3, 4);
    c.step = 0;
  };
  auto advance = [&](DWCursor &c) {
    if (!c.live) return;
    if (++c.step < c.ns) return;
    // keeps the tile lookup behind this (rarely taken) branch: without it the compiler evaluates
    // the lookup's integer divisions in every half-step and selects the results
    __asm__ volatile("" ::: "memory");
    open_tile(c, c.seq + 1);
  };

  DWStreamOps ops;
  ops.uwave = __builtin_amdgcn_readfirstlane(wave);
#pragma unroll
  for (int I = 0; I < NLD; ++I) tr_lane_slot(wave, lane, I, ops.ra[I], ops.ka[I]);
  const bf16_t *A = (const bf16_t *)a.A, *B = (const bf16_t *)a.B;
  const uint32_t row_a = (uint32_t)a.M * 2u, row_b = (uint32_t)a.N * 2u;   // bytes per operand row
  // loader cursor: publish the slot whose eight loads are issued next
  int shown_m0 = -1, shown_n0 = -1;
  auto resolve = [&](const DWCursor &c) {
    const int first = c.lo + (c.step & ~3) * HK;                 // first row of this group of four slots
    const int left = c.live ? max(c.hi - first, 0) : 0;          // rows of the segment from there on
    const int base_row = left > 0 ? first : 0;
    const unsigned long long cap = 0xffffffffull;
    ops.win_a = buffer_window(A + (size_t)base_row * a.M, (uint32_t)min((unsigned long long)left * row_a, cap));
    ops.win_b = buffer_window(B + (size_t)base_row * a.N, (uint32_t)min((unsigned long long)left * row_b, cap));
    ops.sub_a = (uint32_t)(c.step & 3) * HK * row_a;
    ops.sub_b = (uint32_t)(c.step & 3) * HK * row_b;
    if (c.m0 != shown_m0 || c.n0 != shown_n0) {                  // a new tile: its columns' offsets inside a slot
      shown_m0 = c.m0;
      shown_n0 = c.n0;
#pragma unroll
      for (int J = 0; J < NLD; ++J) {
        int ca = c.m0 + ops.ka[J] * 8, cb = c.n0 + ops.ka[J] * 8;
        if (ca >= a.M) ca = 0;
        if (cb >= a.N) cb = 0;
        ops.oa[J] = (uint32_t)ops.ra[J] * row_a + (uint32_t)ca * 2u;
        ops.ob[J] = (uint32_t)ops.ra[J] * row_b + (uint32_t)cb * 2u;
      }
    }
  };

  DWCursor cc, lc;
  open_tile(cc, 0);
  if (!cc.live) return;
  lc = cc;
  const uint32_t lds0 = __builtin_amdgcn_readfirstlane(lds_address(smem));
  char *patch = smem + RING_BYTES + wave * EPI_WAVE_BYTES;
#pragma unroll 1
  for (int st = 0; st < NSTAGE - 1; ++st) {
    resolve(lc);
#pragma unroll
    for (int I = 0; I < 2 * NLD; ++I) ops.load(I, lds0 + st * STAGE_BYTES + (I / NLD) * TILE_BYTES);
    advance(lc);
  }
  wait_loads<2 * NLD>();
  __syncthreads();
  bf16x8 fa[2][FR], fb[2][FR];
  f32x16 acc[FR][FR];
#pragma unroll
  for (int i = 0; i < FR; ++i) fa[0][i] = ops.frag_a(smem, wm * (TB / 2) + i * 32, 0, lane);
#pragma unroll
  for (int j = 0; j < FR; ++j) fb[0][j] = ops.frag_b(smem + TILE_BYTES, wn * (TB / 2) + j * 32, 0, lane);

  auto open_slot = [&]() {
    wait_loads<2 * NLD>();
    __syncthreads();
  };
  auto static_slot = [&](auto first, auto stage) {
    constexpr int S = decltype(stage)::value;
    resolve(lc);
    half_step<decltype(first)::value>(ops, smem + S * STAGE_BYTES, smem + ((S + 1) & 3) * STAGE_BYTES,
                                      lds0 + ((S + 3) & 3) * STAGE_BYTES, wm, wn, lane, fa, fb, acc);
    advance(lc);
  };
  using I0 = std::integral_constant<int, 0>;
  using I1 = std::integral_constant<int, 1>;
  using I2 = std::integral_constant<int, 2>;
  using I3 = std::integral_constant<int, 3>;
  open_slot();
  for (;;) {   // one tile per trip; its first slot has been opened already
    static_slot(std::true_type{}, I0{});
    open_slot();
    static_slot(std::false_type{}, I1{});
    open_slot();
    static_slot(std::false_type{}, I2{});
    open_slot();
    static_slot(std::false_type{}, I3{});
    for (int h = 4; h < cc.ns; h += 4) {
      open_slot();
      static_slot(std::false_type{}, I0{});
      open_slot();
      static_slot(std::false_type{}, I1{});
      open_slot();
      static_slot(std::false_type{}, I2{});
      open_slot();
      static_slot(std::false_type{}, I3{});
    }
    open_slot();   // the next tile's first slot, before the stores below join the load counter
    const int mbase = cc.m0 + wm * (TB / 2);
    auto dst_row = [&](int r) -> int { return (mbase + r < a.M) ? mbase + r : -1; };
    if (split > 1)
      store_wave_partial(acc, a.split_ws + (size_t)(cc.seq * G + slot_in_round) * TB * TB + (size_t)(wm * (TB / 2)) * TB + wn * (TB / 2), lane);
    else
      store_wave_tile(acc, patch, dst_row, (bf16_t *)a.dW + (size_t)cc.e * a.M * a.N, a.N, cc.n0 + wn * (TB / 2), a.N,
                      lane);
    open_tile(cc, cc.seq + 1);
    if (!cc.live) break;
  }
  wait_loads<0>();
}

// Second pass of a row-split groupXTY: adds each tile's partials in chunk order, rounds once, stores dW.
__global__ void __launch_bounds__(256) dw_split_reduce_kernel(DWArgs a, int tiles_m, int tiles_n, int split) {
  const int per_expert = tiles_m * tiles_n;
  const int T = blockIdx.x, e = T / per_expert;
  int m0, n0;
  dw_tile_origin(T - e * per_expert, tiles_m, tiles_n, m0, n0);
  const float *part = a.split_ws + (size_t)T * split * TB * TB;
  bf16_t *dW = (bf16_t *)a.dW + (size_t)e * a.M * a.N;
  constexpr int PER_SLICE = TB * TB / 4 / TAIL_SLICES;
  for (int i = (int)blockIdx.y * PER_SLICE + threadIdx.x; i < ((int)blockIdx.y + 1) * PER_SLICE; i += 256) {
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int c = 0; c < split; ++c) {
      const float4 v = reinterpret_cast<const float4 *>(part + (size_t)c * TB * TB)[i];
      acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
    }
    const int row = m0 + (i * 4) / TB, col = n0 + (i * 4) % TB;
    if (row < a.M && col < a.N) {
      bf16x4 o;
      o[0] = (bf16_t)acc.x; o[1] = (bf16_t)acc.y; o[2] = (bf16_t)acc.z; o[3] = (bf16_t)acc.w;
      *reinterpret_cast<bf16x4 *>(dW + (size_t)row * a.N + col) = o;
    }
  }
}

template <typename K> int set_lds_limit(K kernel, int bytes) {
  return hipFuncSetAttribute((const void *)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes) == hipSuccess
             ? SMOE_OK
             : SMOE_ERR_HIP;
}

uint32_t division_magic(int fan) { return fan > 1 ? (uint32_t)((0x100000000ULL + fan - 1) / fan) : 0u; }

template <bool TRANS_W, bool SCATTER_OUT, int ACT = 0, bool STATIC4 = false> int launch_s2s_stream_one(hipStream_t s, const S2SArgs &a);
template <bool TRANS_W, bool SCATTER_OUT, int ACT = 0> int launch_s2s_stream_cfg(hipStream_t s, const S2SArgs &a) {
  return a.K % (4 * HK) == 0 ? launch_s2s_stream_one<TRANS_W, SCATTER_OUT, ACT, true>(s, a)
                             : launch_s2s_stream_one<TRANS_W, SCATTER_OUT, ACT, false>(s, a);
}
template <bool TRANS_W, bool SCATTER_OUT, int ACT, bool STATIC4> int launch_s2s_stream_one(hipStream_t s, const S2SArgs &a) {
  int tiles_n = (ACT == 1 || ACT == 2) ? ceil_div(a.N / 2, TB / 2) : ceil_div(a.N, TB);
  long long tiles_m = ceil_div(a.Tk, TB) + a.E;     // upper bound on sum_e ceil(n_e / 256)
  const int group_m = a.group_m;
  if (tiles_m * tiles_n > 0x7fffffffLL) return SMOE_ERR_UNSUPPORTED;
  S2SArgs args = a;
  int chunk;
  if (ACT != 0 || choose_split(a.K / HK, 4, STATIC4, chunk) == 1) args.tail_ws = nullptr;   // too short to pay: no second kernel
  hipLaunchKernelGGL((s2s_stream_kernel<TRANS_W, SCATTER_OUT, ACT, STATIC4>), dim3(a.grid), dim3(NTHREADS), STREAM_LDS_BYTES, s, args, tiles_n,
                     group_m, division_magic(a.a_map.o ? a.a_map.fan : 1));
  SMOE_LAUNCH_CHECK();
  if (args.tail_ws) {   // adds and stores the partial tiles of a split last round (no-op when nothing was split)
    hipLaunchKernelGGL(s2s_tail_reduce_kernel<SCATTER_OUT>, dim3(a.grid - 1, TAIL_SLICES), dim3(256), 0, s, a, tiles_n, group_m,
                       a.grid, STATIC4 ? 1 : 0);
    SMOE_LAUNCH_CHECK();
  }
  return SMOE_OK;
}

int launch_dw_stream_impl(hipStream_t s, const DWArgs &a) {
  int tiles_m = ceil_div(a.M, TB), tiles_n = ceil_div(a.N, TB);
  // Row split: only when every tile of every expert, times the split, fits one round of the grid, and only when
  // it shortens the contraction by more than the partial tiles cost (as for the split last round above).
  int split = 1;
  const long long tiles = (long long)a.E * tiles_m * tiles_n;
  if (a.split_ws && tiles * 2 <= a.grid) {
    const long long nh = a.Tk / a.E / HK;            // half-steps of an average segment
    split = (int)(a.grid / tiles < 8 ? a.grid / tiles : 8);
    if (nh - nh / split < SPLIT_MIN_SAVED) split = 1;
  }
  hipLaunchKernelGGL(dw_stream_kernel, dim3(a.grid), dim3(NTHREADS), STREAM_LDS_BYTES, s, a, tiles_m, tiles_n, split);
  SMOE_LAUNCH_CHECK();
  if (split > 1) {
    hipLaunchKernelGGL(dw_split_reduce_kernel, dim3((unsigned)tiles, TAIL_SLICES), dim3(256), 0, s, a, tiles_m, tiles_n, split);
    SMOE_LAUNCH_CHECK();
  }
  return SMOE_OK;
}
}  // namespace

// The persistent kernel keeps three half-steps in flight across tile boundaries, so a tile must
// have at least three; the expert offsets must fit their LDS cache; order indices are divided
// by the fan-out with a multiply-high that is exact while Tk * fan < 2^32.
bool s2s_stream_supported(const S2SArgs &a) {
  long long fan = a.a_map.o ? a.a_map.fan : 1;
  // every per-lane source offset (from the start of a gathered A, from a tile's first row of a
  // sorted A, from the start of an expert's matrix) must fit the 32-bit offset of the loads
  long long a_rows = a.a_map.o ? (long long)a.Tk / fan + 1 : TB;
  long long w_rows = a.trans_w ? a.N : a.K;
  return a.grid >= 8 && a.grid % 8 == 0 && a.grid <= MAX_STREAM_GRID && a.group_m >= 1 && a.K % HK == 0 && a.K >= 3 * HK && a.N % 8 == 0 && a.ldw % 8 == 0 && a.Tk > 0 && a.E <= MAX_E &&
         (long long)a.Tk * fan < 0x100000000LL && a_rows * a.K * 2 < 0x100000000LL &&
         (w_rows + HK) * a.ldw * 2 < 0x100000000LL;
}

bool s2s_stream_swiglu_bwd_supported(const S2SArgs &a) {
  return s2s_stream_supported(a) && a.trans_w && !a.c_map.o && a.Hpre_in && a.row_scale && a.dp_part && a.N % 8 == 0;
}

bool s2s_stream_dp_supported(const S2SArgs &a) {
  return s2s_stream_supported(a) && a.trans_w && !a.c_map.o && a.H_in && !a.Hpre_in && a.row_scale && a.dp_part && a.N % 8 == 0;
}

bool s2s_stream_swiglu_supported(const S2SArgs &a) {
  return s2s_stream_supported(a) && !a.trans_w && !a.c_map.o && a.H && a.N % 16 == 0;
}

int launch_s2s_stream(hipStream_t s, const S2SArgs &a) {
  const bool scatter_out = a.c_map.o != nullptr;
  if (a.dp_part && a.Hpre_in) {
    if (!s2s_stream_swiglu_bwd_supported(a)) return SMOE_ERR_UNSUPPORTED;
    return launch_s2s_stream_cfg<true, false, 3>(s, a);
  }
  if (a.dp_part) {
    if (!s2s_stream_dp_supported(a)) return SMOE_ERR_UNSUPPORTED;
    return launch_s2s_stream_cfg<true, false, 4>(s, a);
  }
  if (a.H) {
    if (!s2s_stream_swiglu_supported(a)) return SMOE_ERR_UNSUPPORTED;
    return a.C ? launch_s2s_stream_cfg<false, false, 1>(s, a) : launch_s2s_stream_cfg<false, false, 2>(s, a);
  }
  if (a.trans_w) return scatter_out ? launch_s2s_stream_cfg<true, true>(s, a) : launch_s2s_stream_cfg<true, false>(s, a);
  return scatter_out ? launch_s2s_stream_cfg<false, true>(s, a) : launch_s2s_stream_cfg<false, false>(s, a);
}

bool dw_stream_supported(const DWArgs &a) {
  long long tiles = (long long)a.E * ceil_div(a.M, TB) * ceil_div(a.N, TB);
  return a.M % 8 == 0 && a.N % 8 == 0 && a.Tk > 0 && a.E <= MAX_E && tiles + MAX_STREAM_GRID < 0x7fffffffLL && a.grid >= 8 && a.grid % 8 == 0 && a.grid <= MAX_STREAM_GRID;
}

int launch_dw_stream(hipStream_t s, const DWArgs &a) { return launch_dw_stream_impl(s, a); }

// Raises the dynamic LDS limit of every persistent kernel on the current device (once per context).
template <bool TRANS_W, bool SCATTER_OUT, int ACT> static int init_s2s_pair() {
  int rc = set_lds_limit(s2s_stream_kernel<TRANS_W, SCATTER_OUT, ACT, false>, STREAM_LDS_BYTES);
  return rc != SMOE_OK ? rc : set_lds_limit(s2s_stream_kernel<TRANS_W, SCATTER_OUT, ACT, true>, STREAM_LDS_BYTES);
}
int init_stream_kernels() {
  int rc = init_s2s_pair<false, false, 0>();
  if (rc == SMOE_OK) rc = init_s2s_pair<false, true, 0>();
  if (rc == SMOE_OK) rc = init_s2s_pair<true, false, 0>();
  if (rc == SMOE_OK) rc = init_s2s_pair<true, true, 0>();
  if (rc == SMOE_OK) rc = init_s2s_pair<false, false, 1>();
  if (rc == SMOE_OK) rc = init_s2s_pair<false, false, 2>();
  if (rc == SMOE_OK) rc = init_s2s_pair<true, false, 3>();
  if (rc == SMOE_OK) rc = init_s2s_pair<true, false, 4>();
  if (rc == SMOE_OK) rc = set_lds_limit(dw_stream_kernel, STREAM_LDS_BYTES);
  return rc;
}
