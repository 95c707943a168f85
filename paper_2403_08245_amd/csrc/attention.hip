// Causal grouped-query attention for the SMoE attention layer (Alg. 4, Sec. 3.3), bf16 in and
// out, fp32 softmax statistics and accumulation on the matrix cores.
//
// Q and O hold one row per routed slot, [B, T, G, h, 128] (G = the k slots of a token, h heads
// per expert); K and V hold one row per token, [B, T, h, 128].  Head hh of every slot attends
// key/value head hh of the positions <= its own inside its sequence.
//
// All three kernels work on transposed score tiles S^T[key][query] = K Q^T so that a lane of
// the 32x32 matrix instruction owns ONE query column: its softmax statistics are per-lane
// scalars, and the probabilities leave the accumulator registers already in the layout the
// next product takes as its B operand (no cross-lane shuffles; the matching operand is read
// from LDS in the same permuted key order).
#include "mfma_common.h"
#include <type_traits>

namespace {

constexpr int AD = 128;             // head width
constexpr int AKT = 32;             // keys (or query rows) per LDS tile
constexpr int AROW = AD * 2;        // bytes per tile row
constexpr int ATILE = AKT * AROW;   // 8 KB
constexpr int AQ = 128;             // rows per block: 32 per wavefront
constexpr int AFS = 3;              // LDS stages of the forward's key walk: tiles j+1 .. j+AFS-2 in flight while j is used; three blocks per CU
constexpr int ADS = 4;              // the same for the dQ pass (two blocks per CU)
constexpr int DKV_WAVES = 4;        // wavefronts (32 keys each) per block of the dK/dV kernel
constexpr int DKV_SORT_MAX = 512;   // key blocks up to which the dK/dV units are dealt in exact longest-first order
constexpr float NEG_BIG = -1.0e30f; // finite stand-in for -inf: exp2 of it is 0 and no inf - inf appears

// 16-byte chunk swizzle of a 256-byte row: conflict free both for the row-per-lane reads
// (16 consecutive rows -> 16 positions) and for the transposing reads (4 consecutive rows ->
// 4 different 64-byte segments).
__device__ __forceinline__ int a_swz(int row) { return ((row & 3) << 2) | ((row >> 2) & 3); }

// One wavefront's share (8 / NW instructions, NW wavefronts per block) of loading a [32 x 128]
// tile whose row r comes from `base + row_index(r) * ld`; rows past `last` repeat row `last`.
template <int NW = 4>
__device__ __forceinline__ void load_tile_rows(const bf16_t *base, size_t ld, int row0, int last, uint32_t lds_tile,
                                               int wave, int uwave, int lane) {
  constexpr int PER = 8 / NW;
#pragma unroll
  for (int u = 0; u < PER; ++u) {
    int i = wave * PER + u;
    int row = 4 * i + (lane >> 4);
    int chunk = (lane & 15) ^ a_swz(row);
    int src = min(row0 + row, last);
    load16_to_lds(base + (size_t)src * ld + chunk * 8, lds_tile + (uwave * PER + u) * 1024);
  }
}

// A operand, tile rows as matrix rows: lane -> row (lane % 32), columns 16*ks + 8*(lane/32) + 0..7
__device__ __forceinline__ bf16x8 a_rows_frag(const char *tile, int ks, int lane) {
  int row = lane & 31;
  int chunk = (2 * ks + (lane >> 5)) ^ a_swz(row);
  return *reinterpret_cast<const bf16x8 *>(tile + row * AROW + (chunk << 4));
}
// A operand, tile columns as matrix rows (the tile transposed): lane -> column c0 + lane % 32 and
// the eight tile rows 16*s + 4*(lane/32) + {0..3, 8..11}: the order in which a lane's accumulator
// registers of a [tile row][x] product enumerate the tile rows, so those registers can be the B
// operand of the next product as they are.
__device__ __forceinline__ bf16x8 a_cols_frag(const char *tile, int c0, int s, int lane) {
  int col = c0 + 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
  int row0 = 16 * s + 4 * (lane >> 5) + ((lane & 15) >> 2);
  union { bf16x8 v; s16x4 h[2]; } u;
#pragma unroll
  for (int t = 0; t < 2; ++t) {
    int row = row0 + 8 * t;
    int off = row * AROW + (((col >> 3) ^ a_swz(row)) << 4) + ((col & 7) << 1);
    u.h[t] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS s16x4 *)(tile + off));
  }
  return u.v;
}
// Per-lane byte offsets of every fragment inside a tile, worked out once: with them (and the LDS stage as a
// compile-time constant in the unrolled loops) a fragment read is one LDS instruction whose address is a
// register plus an immediate, instead of a dozen integer instructions per read.
struct FragOffsets {
  int rows[8];          // a_rows_frag(tile, ks)
  int cols[4][2][2];    // a_cols_frag(tile, 32 * f, s), first and second transposing read
};
__device__ __forceinline__ FragOffsets frag_offsets(int lane) {
  FragOffsets o;
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) {
    int row = lane & 31;
    o.rows[ks] = row * AROW + (((2 * ks + (lane >> 5)) ^ a_swz(row)) << 4);
  }
#pragma unroll
  for (int f = 0; f < 4; ++f)
#pragma unroll
    for (int s = 0; s < 2; ++s)
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        int col = f * 32 + 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
        int row = 16 * s + 4 * (lane >> 5) + ((lane & 15) >> 2) + 8 * t;
        o.cols[f][s][t] = row * AROW + (((col >> 3) ^ a_swz(row)) << 4) + ((col & 7) << 1);
      }
  return o;
}
__device__ __forceinline__ bf16x8 rows_frag(const char *tile, const FragOffsets &o, int ks) {
  return *reinterpret_cast<const bf16x8 *>(tile + o.rows[ks]);
}
__device__ __forceinline__ bf16x8 cols_frag(const char *tile, const FragOffsets &o, int f, int s) {
  union { bf16x8 v; s16x4 h[2]; } u;
#pragma unroll
  for (int t = 0; t < 2; ++t) u.h[t] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS s16x4 *)(tile + o.cols[f][s][t]));
  return u.v;
}

// Makes a value loaded from global memory "arrive" here: the compiler waits for the load at this point and
// not at the value's first use inside a loop, where its counted wait would also sit out the direct-to-LDS
// loads that were just issued for the next tile (the hardware counter does not tell them apart).
template <typename T> __device__ __forceinline__ void settle(T &v) { __asm__ volatile("" : "+v"(v)); }

// tile row that accumulator register q of this lane belongs to (32x32 result layout)
__device__ __forceinline__ int acc_row(int q, int lane) { return 8 * (q >> 2) + 4 * (lane >> 5) + (q & 3); }

__device__ __forceinline__ bf16x8 pack8(const f32x16 &p, int s) {
  bf16x8 v;
#pragma unroll
  for (int c = 0; c < 8; ++c) v[c] = (bf16_t)p[8 * s + c];
  return v;
}

// Split of the dK/dV pass: the slot rows that see key block kb (32 * NW keys) are cut into chunks of
// `ch` 32-row tiles; a (key block, chunk) pair is one work unit.  Key blocks with a single chunk
// store their gradients directly, the others leave fp32 partial sums that a second kernel adds
// in chunk order (deterministic, no atomics).
struct DkvPlan {
  int ch;        // row tiles per chunk
  int units;     // work units per (sequence, head)
  int kblocks;   // key blocks per (sequence, head)
};
__host__ __device__ inline int dkv_first_tile(int kb, int keys_per_block, int G) { return (int)(((long long)kb * keys_per_block * G) / 32); }
__host__ __device__ inline int dkv_chunks(int kb, int keys_per_block, int G, int row_tiles, int ch) {
  return (row_tiles - dkv_first_tile(kb, keys_per_block, G) + ch - 1) / ch;
}

struct AttnDims {
  int B, T, G, h;
  size_t ldq, ldkv;    // row strides in elements: h * 128
  float scale_log2;    // log2(e) / sqrt(128)
};

// ======================================================================================
// forward: block = (query tile of 128 slot rows, head, sequence); keys stream through LDS
// ======================================================================================
__global__ void __launch_bounds__(256, 3) attn_fwd_kernel(const bf16_t *__restrict__ Q, const bf16_t *__restrict__ K,
                                                       const bf16_t *__restrict__ V, bf16_t *__restrict__ O,
                                                       float *__restrict__ LSE, AttnDims d) {
  __shared__ __attribute__((aligned(1024))) char smem[AFS * 2 * ATILE];   // stages of (K tile, V tile)
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int uwave = __builtin_amdgcn_readfirstlane(wave);
  // Blocks are numbered longest key walk first across ALL (sequence, head) pairs: the hardware starts blocks
  // in index order, so the short walks fill in behind the long ones everywhere at once (numbering each pair's
  // tiles separately left the last pairs' long walks to start late: 1.6x the balanced makespan).
  const int nbh = d.h * d.B, rank = (int)blockIdx.x / nbh, bh = (int)blockIdx.x - rank * nbh;
  const int qt = (int)gridDim.x / nbh - 1 - rank;
  const int hh = bh % d.h, b = bh / d.h;
  const int rows = d.T * d.G;                                        // slot rows of one sequence
  const int R0 = qt * AQ;
  const int r_mine = min(R0 + wave * 32 + (lane & 31), rows - 1);
  const int tok = r_mine / d.G;
  const int wave_first = min(R0 + wave * 32, rows - 1) / d.G;
  const int wave_last = min(R0 + wave * 32 + 31, rows - 1) / d.G;
  const int n_tiles = min(R0 + AQ - 1, rows - 1) / d.G / AKT + 1;
  const bool row_valid = R0 + wave * 32 + (lane & 31) < rows;

  const bf16_t *Kb = K + (size_t)b * d.T * d.ldkv + hh * AD;
  const bf16_t *Vb = V + (size_t)b * d.T * d.ldkv + hh * AD;
  const size_t qrow = ((size_t)b * rows + r_mine) * d.ldq + hh * AD;
  bf16x8 qf[8];
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) qf[ks] = *reinterpret_cast<const bf16x8 *>(Q + qrow + 16 * ks + 8 * (lane >> 5));
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) settle(qf[ks]);

  const uint32_t lds0 = __builtin_amdgcn_readfirstlane(lds_address(smem));
  f32x16 acc[4];
#pragma unroll
  for (int f = 0; f < 4; ++f)
#pragma unroll
    for (int q = 0; q < 16; ++q) acc[f][q] = 0.f;
  float m = NEG_BIG, l = 0.f;

  // Every step requests one tile (four loads per wavefront), also past the last one (rows clamp to the
  // sequence's last key and the tile is never read), so that one constant wait count orders the ring.
  auto request = [&](int tile, int stage) {
    const uint32_t dst = lds0 + stage * 2 * ATILE;
    load_tile_rows(Kb, d.ldkv, tile * AKT, d.T - 1, dst, wave, uwave, lane);
    load_tile_rows(Vb, d.ldkv, tile * AKT, d.T - 1, dst + ATILE, wave, uwave, lane);
  };
#pragma unroll
  for (int t = 0; t < AFS - 1; ++t) request(t, t);
  const FragOffsets fo = frag_offsets(lane);
  // the loop is unrolled by the LDS stages so that every tile address below is register + constant
  auto tile_step = [&](auto stage_c, int j) {
    constexpr int STAGE = decltype(stage_c)::value;
    wait_loads<(AFS - 2) * 4>();
    __syncthreads();   // tile j has landed for everyone; everyone is done reading tile j-1, whose stage is refilled
    request(j + AFS - 1, (STAGE + AFS - 1) % AFS);
    const int key0 = j * AKT;
    if (key0 > wave_last) return;   // wave-uniform: every key of the tile is in the future of all 32 rows
    const char *kt = smem + STAGE * 2 * ATILE;
    const char *vt = kt + ATILE;
    f32x16 s;
#pragma unroll
    for (int q = 0; q < 16; ++q) s[q] = 0.f;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(rows_frag(kt, fo, ks), qf[ks], s, 0, 0, 0);
    const bool diag = key0 + AKT - 1 > wave_first;
    // the running maximum m stays in raw score units; the 1/sqrt(d) log2(e) factor enters the exponent's fma
    float mx = NEG_BIG;
    if (diag) {   // wave-uniform: only tiles that straddle the diagonal pay for the mask
#pragma unroll
      for (int q = 0; q < 16; ++q)
        if (key0 + acc_row(q, lane) > tok) s[q] = NEG_BIG;
    }
#pragma unroll
    for (int q = 0; q < 16; ++q) mx = fmaxf(mx, s[q]);
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    const float m_new = fmaxf(m, mx);
    const float alpha = __builtin_amdgcn_exp2f((m - m_new) * d.scale_log2);
    const float shift = -m_new * d.scale_log2;
    float psum = 0.f;
#pragma unroll
    for (int q = 0; q < 16; ++q) {
      float p = __builtin_amdgcn_exp2f(fmaf(s[q], d.scale_log2, shift));
      s[q] = p;
      psum += p;
    }
    l = l * alpha + psum;
    m = m_new;
    if (__any(alpha != 1.0f)) {   // wave-uniform: once the running maxima have settled nothing needs rescaling
#pragma unroll
      for (int f = 0; f < 4; ++f)
#pragma unroll
        for (int q = 0; q < 16; ++q) acc[f][q] *= alpha;
    }
    bf16x8 pb[2] = {pack8(s, 0), pack8(s, 1)};
#pragma unroll
    for (int f = 0; f < 4; ++f)
#pragma unroll
      for (int s2 = 0; s2 < 2; ++s2)
        acc[f] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(cols_frag(vt, fo, f, s2), pb[s2], acc[f], 0, 0, 0);
  };
  static_assert(AFS == 3 || AFS == 4, "the walk below is written out for three or four stages");
  for (int j = 0; j < n_tiles; j += AFS) {
    tile_step(std::integral_constant<int, 0>{}, j);
    if (j + 1 < n_tiles) tile_step(std::integral_constant<int, 1>{}, j + 1);
    if (j + 2 < n_tiles) tile_step(std::integral_constant<int, 2>{}, j + 2);
    if constexpr (AFS > 3)
      if (j + 3 < n_tiles) tile_step(std::integral_constant<int, 3 % AFS>{}, j + 3);
  }
  wait_loads<0>();   // the requests past the last tile

  const float l_tot = l + __shfl_xor(l, 32, 64);
  const float inv = 1.0f / l_tot;
  if (row_valid) {
    bf16_t *orow = O + qrow;
#pragma unroll
    for (int f = 0; f < 4; ++f)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        bf16x4 v;
#pragma unroll
        for (int c = 0; c < 4; ++c) v[c] = (bf16_t)(acc[f][4 * g + c] * inv);
        *reinterpret_cast<bf16x4 *>(orow + f * 32 + 8 * g + 4 * (lane >> 5)) = v;
      }
    if (lane < 32)
      LSE[((size_t)b * rows + r_mine) * d.h + hh] = (m * d.scale_log2 + __builtin_amdgcn_logf(l_tot)) * 0.6931471805599453f;
  }
}


// ======================================================================================
// backward, part 0: delta[row][head] = <dO, O> over the head's 128 columns (sixteen lanes each)
// ======================================================================================
__global__ void __launch_bounds__(256) attn_delta_kernel(const bf16_t *__restrict__ O, const bf16_t *__restrict__ dO,
                                                         float *__restrict__ delta, size_t n) {
  // sixteen lanes per (row, head) pair, 16 bytes each; both tensors are [rows][h][128]
  const size_t i = ((size_t)blockIdx.x * 256 + threadIdx.x) >> 4;
  const int part = threadIdx.x & 15;
  float v = 0.f;
  if (i < n) {
    const bf16x8 a = *reinterpret_cast<const bf16x8 *>(O + i * AD + part * 8);
    const bf16x8 b = *reinterpret_cast<const bf16x8 *>(dO + i * AD + part * 8);
#pragma unroll
    for (int c = 0; c < 8; ++c) v += (float)a[c] * (float)b[c];
  }
#pragma unroll
  for (int d = 8; d > 0; d >>= 1) v += __shfl_xor(v, d, 64);
  if (part == 0 && i < n) delta[i] = v;
}

// ======================================================================================
// backward, part 1: dQ.  Same walk as the forward; a lane owns one query row.
//   S^T = K Q^T, P^T = exp2(S^T * c - lse), dP^T = V dO^T, dS^T = P^T (dP^T - delta) / sqrt(d),
//   dQ^T += K^T dS^T
// ======================================================================================
__global__ void __launch_bounds__(256) attn_bwd_dq_kernel(const bf16_t *__restrict__ Q, const bf16_t *__restrict__ K,
                                                          const bf16_t *__restrict__ V, const bf16_t *__restrict__ dO,
                                                          const float *__restrict__ LSE, const float *__restrict__ delta,
                                                          bf16_t *__restrict__ dQ, AttnDims d) {
  __shared__ __attribute__((aligned(1024))) char smem[ADS * 2 * ATILE];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int uwave = __builtin_amdgcn_readfirstlane(wave);
  const int nbh = d.h * d.B, rank = (int)blockIdx.x / nbh, bh = (int)blockIdx.x - rank * nbh;   // as in the forward
  const int qt = (int)gridDim.x / nbh - 1 - rank;
  const int hh = bh % d.h, b = bh / d.h;
  const int rows = d.T * d.G;
  const int R0 = qt * AQ;
  const int r_mine = min(R0 + wave * 32 + (lane & 31), rows - 1);
  const int tok = r_mine / d.G;
  const int wave_first = min(R0 + wave * 32, rows - 1) / d.G;
  const int wave_last = min(R0 + wave * 32 + 31, rows - 1) / d.G;
  const int n_tiles = min(R0 + AQ - 1, rows - 1) / d.G / AKT + 1;
  const bool row_valid = R0 + wave * 32 + (lane & 31) < rows;

  const bf16_t *Kb = K + (size_t)b * d.T * d.ldkv + hh * AD;
  const bf16_t *Vb = V + (size_t)b * d.T * d.ldkv + hh * AD;
  const size_t qrow = ((size_t)b * rows + r_mine) * d.ldq + hh * AD;
  bf16x8 qf[8], dof[8];
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) {
    qf[ks] = *reinterpret_cast<const bf16x8 *>(Q + qrow + 16 * ks + 8 * (lane >> 5));
    dof[ks] = *reinterpret_cast<const bf16x8 *>(dO + qrow + 16 * ks + 8 * (lane >> 5));
  }
  const size_t stat = ((size_t)b * rows + r_mine) * d.h + hh;
  float lse2 = LSE[stat] * 1.4426950408889634f;
  float dlt = delta[stat];
  const float scale = d.scale_log2 * 0.6931471805599453f;
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) { settle(qf[ks]); settle(dof[ks]); }
  settle(lse2);
  settle(dlt);

  const uint32_t lds0 = __builtin_amdgcn_readfirstlane(lds_address(smem));
  f32x16 acc[4];
#pragma unroll
  for (int f = 0; f < 4; ++f)
#pragma unroll
    for (int q = 0; q < 16; ++q) acc[f][q] = 0.f;

  auto request = [&](int tile, int stage) {   // as in the forward: one tile per step, also past the end
    const uint32_t dst = lds0 + stage * 2 * ATILE;
    load_tile_rows(Kb, d.ldkv, tile * AKT, d.T - 1, dst, wave, uwave, lane);
    load_tile_rows(Vb, d.ldkv, tile * AKT, d.T - 1, dst + ATILE, wave, uwave, lane);
  };
#pragma unroll
  for (int t = 0; t < ADS - 1; ++t) request(t, t);
  const FragOffsets fo = frag_offsets(lane);
  // the loop is unrolled by the LDS stages so that every tile address below is register + constant
  auto tile_step = [&](auto stage_c, int j) {
    constexpr int STAGE = decltype(stage_c)::value;
    wait_loads<(ADS - 2) * 4>();
    __syncthreads();
    request(j + ADS - 1, (STAGE + ADS - 1) % ADS);
    const int key0 = j * AKT;
    if (key0 > wave_last) return;
    const char *kt = smem + STAGE * 2 * ATILE;
    const char *vt = kt + ATILE;
    f32x16 s, dp;
#pragma unroll
    for (int q = 0; q < 16; ++q) { s[q] = 0.f; dp[q] = 0.f; }
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(rows_frag(kt, fo, ks), qf[ks], s, 0, 0, 0);
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(rows_frag(vt, fo, ks), dof[ks], dp, 0, 0, 0);
    const bool diag = key0 + AKT - 1 > wave_first;
    if (diag) {
#pragma unroll
      for (int q = 0; q < 16; ++q)
        if (key0 + acc_row(q, lane) > tok) s[q] = NEG_BIG;   // exp2 of it is 0
    }
#pragma unroll
    for (int q = 0; q < 16; ++q) {
      float p = __builtin_amdgcn_exp2f(fmaf(s[q], d.scale_log2, -lse2));
      s[q] = p * (dp[q] - dlt) * scale;
    }
    bf16x8 db[2] = {pack8(s, 0), pack8(s, 1)};
#pragma unroll
    for (int f = 0; f < 4; ++f)
#pragma unroll
      for (int s2 = 0; s2 < 2; ++s2)
        acc[f] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(cols_frag(kt, fo, f, s2), db[s2], acc[f], 0, 0, 0);
  };
  for (int j = 0; j < n_tiles; j += ADS) {
    tile_step(std::integral_constant<int, 0>{}, j);
    if (j + 1 < n_tiles) tile_step(std::integral_constant<int, 1>{}, j + 1);
    if (j + 2 < n_tiles) tile_step(std::integral_constant<int, 2>{}, j + 2);
    if constexpr (ADS > 3)
      if (j + 3 < n_tiles) tile_step(std::integral_constant<int, 3 % ADS>{}, j + 3);
  }
  wait_loads<0>();   // the requests past the last tile
  if (row_valid) {
    bf16_t *orow = dQ + qrow;
#pragma unroll
    for (int f = 0; f < 4; ++f)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        bf16x4 v;
#pragma unroll
        for (int c = 0; c < 4; ++c) v[c] = (bf16_t)acc[f][4 * g + c];
        *reinterpret_cast<bf16x4 *>(orow + f * 32 + 8 * g + 4 * (lane >> 5)) = v;
      }
  }
}

// ======================================================================================
// backward, part 2: dK and dV.  Block = 32 * NW keys of one (sequence, head), 32 per wavefront, a
// lane owns one key; the slot rows that can see them stream through LDS 32 at a time.
//   S = Q K^T, P = exp2(S c - lse[row]), dV^T += dO^T P, dP = dO V^T,
//   dS = P (dP - delta[row]) / sqrt(d), dK^T += Q^T dS
// ======================================================================================
template <int NW, bool DK, bool DV>
__global__ void __launch_bounds__(64 * NW, 2) attn_bwd_dkv_kernel(const bf16_t *__restrict__ Q, const bf16_t *__restrict__ K,
                                                           const bf16_t *__restrict__ V, const bf16_t *__restrict__ dO,
                                                           const float *__restrict__ LSE, const float *__restrict__ delta,
                                                           bf16_t *__restrict__ dK, bf16_t *__restrict__ dV,
                                                           float *__restrict__ part, DkvPlan plan, AttnDims d) {
  __shared__ __attribute__((aligned(1024))) char smem[4 * ATILE];
  __shared__ __attribute__((aligned(1024))) char s_v[NW * ATILE];   // the block's own V rows, 32 per wavefront
  // log-sum-exp and delta of the 32 rows of a tile; 64 entries per stage because a direct-to-LDS
  // load always lands a whole wavefront's worth (the upper half repeats clamped rows, never read)
  __shared__ __attribute__((aligned(256))) float s_lse[2][64], s_dlt[2][64];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int uwave = __builtin_amdgcn_readfirstlane(wave);
  // units are numbered first key block (longest row list) first, the (sequence, head) pair innermost, so that
  // every pair's long units start together and the short ones fill in behind them
  const int nbh = d.h * d.B, unit = (int)blockIdx.x / nbh, bh = (int)blockIdx.x - unit * nbh;
  const int hh = bh % d.h, b = bh / d.h;
  const int rows = d.T * d.G;
  const int row_tiles = (rows + AKT - 1) / AKT;
  // work unit -> (key block, chunk of its row tiles).  A key block's list is cut into full chunks of plan.ch
  // tiles and one shorter last chunk.  Units in longest-first order: every full chunk (key blocks ascending),
  // then the last chunks by decreasing length (ties: key block ascending) -- with the few units per resident
  // block that a chunked launch has, short units scattered among long ones cost a fifth of the makespan.
  // Beyond DKV_SORT_MAX key blocks the last chunks keep their natural place.
  __shared__ int s_last[DKV_SORT_MAX];   // length of each key block's last chunk
  __shared__ int s_pick;
  const int KB = plan.kblocks;
  auto chunks_of = [&](int i) { return dkv_chunks(i, 32 * NW, d.G, row_tiles, plan.ch); };
  int kb = 0, chunk = 0;
  if (KB > DKV_SORT_MAX || plan.ch >= row_tiles) {
    int before = 0, c = chunks_of(0);
    while (before + c <= unit) {
      before += c;
      ++kb;
      c = chunks_of(kb);
    }
    chunk = unit - before;
  } else if (unit < plan.units - KB) {
    int before = 0, c = chunks_of(0) - 1;
    while (before + c <= unit) {
      before += c;
      ++kb;
      c = chunks_of(kb) - 1;
    }
    chunk = unit - before;
  } else {
    const int want = unit - (plan.units - KB);
    for (int i = threadIdx.x; i < KB; i += 64 * NW)
      s_last[i] = row_tiles - dkv_first_tile(i, 32 * NW, d.G) - (chunks_of(i) - 1) * plan.ch;
    __syncthreads();
    for (int i = threadIdx.x; i < KB; i += 64 * NW) {
      const int mine = s_last[i];
      int ahead = 0;
      for (int o = 0; o < KB; ++o) ahead += (s_last[o] > mine) || (s_last[o] == mine && o < i);
      if (ahead == want) s_pick = i;   // exactly one key block has this position
    }
    __syncthreads();
    kb = __builtin_amdgcn_readfirstlane(s_pick);
    chunk = chunks_of(kb) - 1;
  }
  const int nch = chunks_of(kb);
  int unit0 = 0;                      // units of the earlier key blocks: where this key block's partial sums start
  for (int i = 0; i < kb; ++i) unit0 += chunks_of(i);
  const int k0 = kb * 32 * NW;
  const int key = min(k0 + wave * 32 + (lane & 31), d.T - 1);
  const bool key_valid = k0 + wave * 32 + (lane & 31) < d.T;
  const int wave_key0 = k0 + wave * 32;

  const size_t krow = ((size_t)b * d.T + key) * d.ldkv + hh * AD;
  // K fragments stay in registers; the V fragments are re-read from LDS at every use (keeping both
  // in registers pushes the kernel past 256 registers and down to one wavefront per SIMD)
  bf16x8 kf[8];
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) kf[ks] = *reinterpret_cast<const bf16x8 *>(K + krow + 16 * ks + 8 * (lane >> 5));
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) settle(kf[ks]);
  const char *vmine = s_v + wave * ATILE;
  load_tile_rows<1>(V + (size_t)b * d.T * d.ldkv + hh * AD, d.ldkv, wave_key0, d.T - 1,
                    __builtin_amdgcn_readfirstlane(lds_address(s_v)) + uwave * ATILE, 0, 0, lane);
  const bf16_t *Qb = Q + (size_t)b * rows * d.ldq + hh * AD;
  const bf16_t *dOb = dO + (size_t)b * rows * d.ldq + hh * AD;
  const float *Lb = LSE + (size_t)b * rows * d.h + hh;
  const float *Db = delta + (size_t)b * rows * d.h + hh;
  const float scale = d.scale_log2 * 0.6931471805599453f;

  const uint32_t lds0 = __builtin_amdgcn_readfirstlane(lds_address(smem));
  f32x16 acck[4], accv[4];
#pragma unroll
  for (int f = 0; f < 4; ++f)
#pragma unroll
    for (int q = 0; q < 16; ++q) { acck[f][q] = 0.f; accv[f][q] = 0.f; }

  // first 32-row tile of this unit (the key block's list starts at the tile holding the first row that sees key k0)
  const int t_first = dkv_first_tile(kb, 32 * NW, d.G) + chunk * plan.ch;
  const int n_tiles = min(plan.ch, row_tiles - t_first);
  // the statistics travel like the tiles (direct-to-LDS): an ordinary load here would make the
  // compiler wait for every outstanding load, the next tile's included, before its LDS store
  const uint32_t lds_lse = __builtin_amdgcn_readfirstlane(lds_address((const char *)&s_lse[0][0]));
  const uint32_t lds_dlt = __builtin_amdgcn_readfirstlane(lds_address((const char *)&s_dlt[0][0]));
  auto load_stats = [&](int tile, int stage) {
    if (wave == 0) {
      int r = min(tile * AKT + lane, rows - 1);
      load4_to_lds(Lb + (size_t)r * d.h, lds_lse + stage * 256);
      load4_to_lds(Db + (size_t)r * d.h, lds_dlt + stage * 256);
    }
  };
  load_tile_rows<NW>(Qb, d.ldq, t_first * AKT, rows - 1, lds0, wave, uwave, lane);
  load_tile_rows<NW>(dOb, d.ldq, t_first * AKT, rows - 1, lds0 + ATILE, wave, uwave, lane);
  load_stats(t_first, 0);
  const FragOffsets fo = frag_offsets(lane);
  // the loop is unrolled by the two LDS stages so that every tile address below is register + constant
  auto tile_step = [&](auto stage_c, int j) {
    constexpr int STAGE = decltype(stage_c)::value;
    wait_loads<0>();
    __syncthreads();
    const int tile = t_first + j;
    if (j + 1 < n_tiles) {
      uint32_t nxt = lds0 + (1 - STAGE) * 2 * ATILE;
      load_tile_rows<NW>(Qb, d.ldq, (tile + 1) * AKT, rows - 1, nxt, wave, uwave, lane);
      load_tile_rows<NW>(dOb, d.ldq, (tile + 1) * AKT, rows - 1, nxt + ATILE, wave, uwave, lane);
      load_stats(tile + 1, (j + 1) & 1);
    }
    const int r0 = tile * AKT;
    const int tile_last_tok = min(r0 + AKT - 1, rows - 1) / d.G;
    if (tile_last_tok < wave_key0) return;                    // none of these rows sees any key of this wavefront
    const char *qt = smem + STAGE * 2 * ATILE;
    const char *dot = qt + ATILE;
    f32x16 s, dp;
#pragma unroll
    for (int q = 0; q < 16; ++q) { s[q] = 0.f; dp[q] = 0.f; }
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(rows_frag(qt, fo, ks), kf[ks], s, 0, 0, 0);
    if (DK) {
#pragma unroll
      for (int ks = 0; ks < 8; ++ks)
        dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(rows_frag(dot, fo, ks), rows_frag(vmine, fo, ks), dp, 0, 0, 0);
    }
    // rows of this tile that are earlier than the wavefront's last key, or past the end, need the mask
    const bool edge = (r0 / d.G < wave_key0 + 31) || (r0 + AKT > rows);
    f32x16 p;
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const int rr = 8 * g + 4 * (lane >> 5);
      const float4 l4 = *reinterpret_cast<const float4 *>(&s_lse[j & 1][rr]);
      const float4 d4 = *reinterpret_cast<const float4 *>(&s_dlt[j & 1][rr]);
      const float lv[4] = {l4.x, l4.y, l4.z, l4.w}, dv[4] = {d4.x, d4.y, d4.z, d4.w};
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const int q = 4 * g + c;
        float pv = __builtin_amdgcn_exp2f(s[q] * d.scale_log2 - lv[c] * 1.4426950408889634f);
        if (edge) {
          int r = r0 + rr + c;
          if (r >= rows || r / d.G < key) pv = 0.f;
        }
        p[q] = pv;
        s[q] = pv * (dp[q] - dv[c]) * scale;
      }
    }
    bf16x8 pb[2] = {pack8(p, 0), pack8(p, 1)};
    bf16x8 db[2] = {pack8(s, 0), pack8(s, 1)};
#pragma unroll
    for (int f = 0; f < 4; ++f)
#pragma unroll
      for (int s2 = 0; s2 < 2; ++s2) {
        if (DV) accv[f] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(cols_frag(dot, fo, f, s2), pb[s2], accv[f], 0, 0, 0);
        if (DK) acck[f] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(cols_frag(qt, fo, f, s2), db[s2], acck[f], 0, 0, 0);
      }
  };
  for (int j = 0; j < n_tiles; j += 2) {
    tile_step(std::integral_constant<int, 0>{}, j);
    if (j + 1 < n_tiles) tile_step(std::integral_constant<int, 1>{}, j + 1);
  }
  if (nch > 1) {   // partial sums of this chunk: [unit][dK | dV][key][128] fp32
    float *pk = part + ((((size_t)b * d.h + hh) * plan.units + unit0 + chunk) * 2) * (32 * NW) * AD +
                (size_t)(wave * 32 + (lane & 31)) * AD;
    float *pv = pk + (size_t)(32 * NW) * AD;
#pragma unroll
    for (int f = 0; f < 4; ++f)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int col = f * 32 + 8 * g + 4 * (lane >> 5);
        if (DK) *reinterpret_cast<float4 *>(pk + col) = make_float4(acck[f][4 * g], acck[f][4 * g + 1], acck[f][4 * g + 2], acck[f][4 * g + 3]);
        if (DV) *reinterpret_cast<float4 *>(pv + col) = make_float4(accv[f][4 * g], accv[f][4 * g + 1], accv[f][4 * g + 2], accv[f][4 * g + 3]);
      }
  } else if (key_valid) {
#pragma unroll
    for (int f = 0; f < 4; ++f)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        bf16x4 vk, vv;
#pragma unroll
        for (int c = 0; c < 4; ++c) { vk[c] = (bf16_t)acck[f][4 * g + c]; vv[c] = (bf16_t)accv[f][4 * g + c]; }
        if (DK) *reinterpret_cast<bf16x4 *>(dK + krow + f * 32 + 8 * g + 4 * (lane >> 5)) = vk;
        if (DV) *reinterpret_cast<bf16x4 *>(dV + krow + f * 32 + 8 * g + 4 * (lane >> 5)) = vv;
      }
  }
}

// adds the chunk partials of one key block in chunk order and rounds once
template <int NW>
__global__ void __launch_bounds__(256) attn_bwd_dkv_reduce_kernel(const float *__restrict__ part, bf16_t *__restrict__ dK,
                                                                  bf16_t *__restrict__ dV, DkvPlan plan, AttnDims d) {
  constexpr int SPLIT = 8;   // blocks per key block
  const int kb = blockIdx.x / SPLIT, part_id = blockIdx.x % SPLIT, hh = blockIdx.y, b = blockIdx.z;
  const int row_tiles = (d.T * d.G + AKT - 1) / AKT;
  int unit0 = 0;
  for (int i = 0; i < kb; ++i) unit0 += dkv_chunks(i, 32 * NW, d.G, row_tiles, plan.ch);
  const int nch = dkv_chunks(kb, 32 * NW, d.G, row_tiles, plan.ch);
  if (nch <= 1) return;
  constexpr int KEYS = 32 * NW;
  const float *base = part + (((size_t)b * d.h + hh) * plan.units + unit0) * 2 * KEYS * AD;
  constexpr int PER = 2 * KEYS * AD / 4 / SPLIT;
  for (int i = part_id * PER + threadIdx.x; i < (part_id + 1) * PER; i += 256) {
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int c = 0; c < nch; ++c) {
      const float4 v = reinterpret_cast<const float4 *>(base + (size_t)c * 2 * KEYS * AD)[i];
      acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
    }
    const int which = i / (KEYS * AD / 4), rem = i % (KEYS * AD / 4);
    const int key = kb * KEYS + rem / (AD / 4), col = (rem % (AD / 4)) * 4;
    if (key < d.T) {
      bf16x4 o;
      o[0] = (bf16_t)acc.x; o[1] = (bf16_t)acc.y; o[2] = (bf16_t)acc.z; o[3] = (bf16_t)acc.w;
      bf16_t *dst = (which ? dV : dK) + ((size_t)b * d.T + key) * d.ldkv + hh * AD + col;
      *reinterpret_cast<bf16x4 *>(dst) = o;
    }
  }
}

}  // namespace

int launch_attn_fwd(hipStream_t s, const void *Q, const void *K, const void *V, void *O, float *LSE, int B, int T, int G,
                    int h) {
  AttnDims d{B, T, G, h, (size_t)h * AD, (size_t)h * AD, 1.4426950408889634f / sqrtf((float)AD)};
  int q_tiles = ceil_div(T * G, AQ);
  hipLaunchKernelGGL(attn_fwd_kernel, dim3(q_tiles * h * B), dim3(256), 0, s, (const bf16_t *)Q, (const bf16_t *)K,
                     (const bf16_t *)V, (bf16_t *)O, LSE, d);
  SMOE_LAUNCH_CHECK();
  return SMOE_OK;
}

// The row list of a key block is cut into chunks only when that is needed to fill the chip: with enough
// (sequence, head) pairs the whole lists, longest first, already pack to within a few percent of the balanced
// makespan, and whole lists leave no partial sums behind.
static DkvPlan dkv_plan(int T, int G, int nbh) {
  const int row_tiles = ceil_div(T * G, AKT), keys = 32 * DKV_WAVES;
  DkvPlan p;
  p.kblocks = ceil_div(T, keys);
  long long tiles = 0;                       // row tiles over all key blocks of one pair
  for (int kb = 0; kb < p.kblocks; ++kb) tiles += row_tiles - dkv_first_tile(kb, keys, G);
  const long long balanced = tiles * nbh / 512;   // per resident block: two per compute unit
  if ((long long)row_tiles * 20 <= balanced * 21)
    p.ch = row_tiles;
  else
    p.ch = row_tiles / 8 > 16 ? ceil_div(row_tiles, 8) : 16;   // the longest row list splits into about eight units
  p.units = 0;
  for (int kb = 0; kb < p.kblocks; ++kb) p.units += dkv_chunks(kb, keys, G, row_tiles, p.ch);
  return p;
}

size_t attn_bwd_workspace_bytes(int B, int T, int G, int h) {
  DkvPlan p = dkv_plan(T, G, B * h);
  size_t delta = ((size_t)B * T * G * h * sizeof(float) + 255) & ~(size_t)255;
  if (p.ch >= ceil_div(T * G, AKT)) return delta;   // whole row lists: no partial sums
  return delta + (size_t)B * h * p.units * 2 * (32 * DKV_WAVES) * AD * sizeof(float);
}

int launch_attn_bwd(hipStream_t s, const void *Q, const void *K, const void *V, const void *O, const void *dO,
                    const float *LSE, void *ws, void *dQ, void *dK, void *dV, int B, int T, int G, int h) {
  AttnDims d{B, T, G, h, (size_t)h * AD, (size_t)h * AD, 1.4426950408889634f / sqrtf((float)AD)};
  size_t n = (size_t)B * T * G * h;
  float *delta = (float *)ws;
  float *part = (float *)((char *)ws + ((n * sizeof(float) + 255) & ~(size_t)255));
  constexpr int NW = DKV_WAVES;
  const DkvPlan plan = dkv_plan(T, G, B * h);
  if ((long long)plan.units * h * B > 0x7fffffffLL) return SMOE_ERR_UNSUPPORTED;
  hipLaunchKernelGGL(attn_delta_kernel, dim3((unsigned)((n + 15) / 16)), dim3(256), 0, s, (const bf16_t *)O, (const bf16_t *)dO,
                     delta, n);
  SMOE_LAUNCH_CHECK();
  hipLaunchKernelGGL(attn_bwd_dq_kernel, dim3(ceil_div(T * G, AQ) * h * B), dim3(256), 0, s, (const bf16_t *)Q,
                     (const bf16_t *)K, (const bf16_t *)V, (const bf16_t *)dO, LSE, (const float *)delta, (bf16_t *)dQ, d);
  SMOE_LAUNCH_CHECK();
  hipLaunchKernelGGL((attn_bwd_dkv_kernel<NW, true, true>), dim3(plan.units * h * B), dim3(64 * NW), 0, s, (const bf16_t *)Q,
                     (const bf16_t *)K, (const bf16_t *)V, (const bf16_t *)dO, LSE, (const float *)delta, (bf16_t *)dK,
                     (bf16_t *)dV, part, plan, d);
  SMOE_LAUNCH_CHECK();
  if (plan.ch < ceil_div(T * G, AKT)) {   // some key block was cut into chunks
    hipLaunchKernelGGL(attn_bwd_dkv_reduce_kernel<NW>, dim3(plan.kblocks * 8, h, B), dim3(256), 0, s, (const float *)part,
                       (bf16_t *)dK, (bf16_t *)dV, plan, d);
    SMOE_LAUNCH_CHECK();
  }
  return SMOE_OK;
}
