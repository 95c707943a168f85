// Plain LDS-tiled grouped GEMMs (scalar FMA, fp32 accumulation) for the fp32 validation
// path and for shapes the matrix-core kernels do not take.  Same operations as the MFMA
// kernels: scatter2scatter (Sec. 3.2) with W or W^T, and groupXTY (Sec. 3.2.1).
#include "common.h"

namespace {
constexpr int PT = 64;   // tile edge (rows and columns)
constexpr int PK = 16;   // contraction step

// Finds the expert segment and first row of M-tile `tile` when every expert's rows are cut
// into tiles of `bm` rows.  Returns false when `tile` is past the last tile.
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

template <typename T>
__global__ void __launch_bounds__(256) s2s_plain_kernel(S2SArgs a) {
  __shared__ float As[PK][PT + 1];
  __shared__ float Bs[PK][PT + 1];
  int e, row0, row_end;
  if (!locate_tile(a.offsets, a.E, PT, blockIdx.x, e, row0, row_end)) return;
  const T *A = (const T *)a.A;
  const T *W = (const T *)a.W + (size_t)e * a.w_stride;
  T *C = (T *)a.C;
  const int n0 = blockIdx.y * PT;
  const int tx = threadIdx.x % 16, ty = threadIdx.x / 16;  // thread -> 4x4 outputs
  float acc[4][4] = {};
  for (int k0 = 0; k0 < a.K; k0 += PK) {
    for (int idx = threadIdx.x; idx < PT * PK; idx += 256) {
      int r = idx / PK, kk = idx % PK;   // A tile: row r, column k0+kk
      int i = row0 + r;
      float v = 0.f;
      if (i < row_end && k0 + kk < a.K) v = to_f32<T>(A[(size_t)map_row(a.a_map, i) * a.K + k0 + kk]);
      As[kk][r] = v;
    }
    for (int idx = threadIdx.x; idx < PT * PK; idx += 256) {
      int kk, c;
      if (a.trans_w) { c = idx / PK; kk = idx % PK; } else { kk = idx / PT; c = idx % PT; }
      float v = 0.f;
      if (k0 + kk < a.K && n0 + c < a.N)
        v = to_f32<T>(a.trans_w ? W[(size_t)(n0 + c) * a.ldw + k0 + kk] : W[(size_t)(k0 + kk) * a.ldw + n0 + c]);
      Bs[kk][c] = v;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < PK; ++kk) {
      float av[4], bv[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) { av[q] = As[kk][ty * 4 + q]; bv[q] = Bs[kk][tx * 4 + q]; }
#pragma unroll
      for (int p = 0; p < 4; ++p)
#pragma unroll
        for (int q = 0; q < 4; ++q) acc[p][q] = fmaf(av[p], bv[q], acc[p][q]);
    }
    __syncthreads();
  }
  for (int p = 0; p < 4; ++p) {
    int i = row0 + ty * 4 + p;
    if (i >= row_end) continue;
    size_t orow = (size_t)map_row(a.c_map, i) * a.N;
    for (int q = 0; q < 4; ++q) {
      int n = n0 + tx * 4 + q;
      if (n < a.N) C[orow + n] = from_f32<T>(acc[p][q]);
    }
  }
}

template <typename T>
__global__ void __launch_bounds__(256) dw_plain_kernel(DWArgs a) {
  __shared__ float As[PK][PT + 1];
  __shared__ float Bs[PK][PT + 1];
  const int e = blockIdx.z;
  const int lo = a.offsets[e], hi = a.offsets[e + 1];
  const T *A = (const T *)a.A;
  const T *B = (const T *)a.B;
  T *dW = (T *)a.dW + (size_t)e * a.M * a.N;
  const int m0 = blockIdx.y * PT, n0 = blockIdx.x * PT;
  const int tx = threadIdx.x % 16, ty = threadIdx.x / 16;
  float acc[4][4] = {};
  for (int i0 = lo; i0 < hi; i0 += PK) {
    for (int idx = threadIdx.x; idx < PT * PK; idx += 256) {
      int kk = idx / PT, c = idx % PT;
      int i = i0 + kk;
      float va = 0.f, vb = 0.f;
      if (i < hi) {
        if (m0 + c < a.M) va = to_f32<T>(A[(size_t)i * a.M + m0 + c]);
        if (n0 + c < a.N) vb = to_f32<T>(B[(size_t)i * a.N + n0 + c]);
      }
      As[kk][c] = va;
      Bs[kk][c] = vb;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < PK; ++kk) {
      float av[4], bv[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) { av[q] = As[kk][ty * 4 + q]; bv[q] = Bs[kk][tx * 4 + q]; }
#pragma unroll
      for (int p = 0; p < 4; ++p)
#pragma unroll
        for (int q = 0; q < 4; ++q) acc[p][q] = fmaf(av[p], bv[q], acc[p][q]);
    }
    __syncthreads();
  }
  for (int p = 0; p < 4; ++p) {
    int m = m0 + ty * 4 + p;
    if (m >= a.M) continue;
    for (int q = 0; q < 4; ++q) {
      int n = n0 + tx * 4 + q;
      if (n < a.N) dW[(size_t)m * a.N + n] = from_f32<T>(acc[p][q]);
    }
  }
}
}  // namespace

int launch_s2s_plain(hipStream_t s, smoe_dtype dt, const S2SArgs &a) {
  if (a.Tk == 0) return SMOE_OK;
  dim3 grid(ceil_div(a.Tk, PT) + a.E, ceil_div(a.N, PT)), block(256);
  if (dt == SMOE_BF16) hipLaunchKernelGGL((s2s_plain_kernel<bf16_t>), grid, block, 0, s, a);
  else hipLaunchKernelGGL((s2s_plain_kernel<float>), grid, block, 0, s, a);
  SMOE_LAUNCH_CHECK();
  return SMOE_OK;
}

int launch_dw_plain(hipStream_t s, smoe_dtype dt, const DWArgs &a) {
  dim3 grid(ceil_div(a.N, PT), ceil_div(a.M, PT), a.E), block(256);
  if (dt == SMOE_BF16) hipLaunchKernelGGL((dw_plain_kernel<bf16_t>), grid, block, 0, s, a);
  else hipLaunchKernelGGL((dw_plain_kernel<float>), grid, block, 0, s, a);
  SMOE_LAUNCH_CHECK();
  return SMOE_OK;
}
