// Shared declarations of the libsmoe kernels (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include "smoe.h"

typedef __bf16 bf16_t;

struct smoe_ctx {
  int device;
  int num_cu;
  int stream_grid;  // blocks of the persistent kernels: one per compute unit, a multiple of 8 (one share per XCD), at most 256
  unsigned long long *clock_probe;  // device array the persistent s2s kernels report their clocks to, or NULL (smoe_set_clock_probe)
  int group_m;      // M-tiles per group of the persistent scatter2scatter kernels' tile order (4; smoe_set_tile_group)
  int kernel_mode;  // 0 auto, 1 plain tiled kernels only, 2 one block per tile (testing aid, see smoe_set_kernel_mode)
  int32_t *route_scratch;  // this device's copy of the routing kernels' static scratch array (smoe_route_noalloc)
};

#define SMOE_LAUNCH_CHECK()                                   \
  do {                                                        \
    if (hipGetLastError() != hipSuccess) return SMOE_ERR_HIP; \
  } while (0)

static inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }
static inline size_t dtype_size(smoe_dtype d) { return d == SMOE_BF16 ? 2 : 4; }
static inline int ceil_div(int a, int b) { return (a + b - 1) / b; }

template <typename T> __device__ __forceinline__ float to_f32(T v);
template <> __device__ __forceinline__ float to_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ float to_f32<bf16_t>(bf16_t v) { return (float)v; }
template <typename T> __device__ __forceinline__ T from_f32(float v);
template <> __device__ __forceinline__ float from_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16_t from_f32<bf16_t>(float v) { return (bf16_t)v; }  // RNE

// How a GEMM operand's rows are addressed through the routing arrays.
//   sorted position i -> row i (grouped) or o[i] / fan (scattered source with fan-out)
//   or o[i] (scattered destination).
struct RowMap {
  const int32_t *o;  // sorted_scattered_idxs, or nullptr when rows are already grouped
  int fan;           // divisor applied to o[i]; 1 for slot-indexed tensors
};
__device__ __forceinline__ int map_row(const RowMap &m, int i) {
  return m.o ? (m.fan > 1 ? m.o[i] / m.fan : m.o[i]) : i;
}

// ---- routing.hip
int launch_topk_gate(hipStream_t s, const float *logits, int T, int E, int k, int32_t *idx, float *gates);
int launch_attn_fwd(hipStream_t s, const void *Q, const void *K, const void *V, void *O, float *LSE, int B, int T, int G,
                    int h);
size_t attn_bwd_workspace_bytes(int B, int T, int G, int h);
int launch_attn_bwd(hipStream_t s, const void *Q, const void *K, const void *V, const void *O, const void *dO,
                    const float *LSE, void *ws, void *dQ, void *dK, void *dV, int B, int T, int G, int h);
int launch_dense_offsets(hipStream_t s, int32_t *off, int n);
int launch_add3(hipStream_t s, const void *a, const void *b, const void *c, void *out, size_t n);
int launch_topk_gate_bwd(hipStream_t s, const int32_t *idx, const float *gates, const float *dgates, int T, int E, int k,
                         float *dlogits);
constexpr int ROUTE_MAX_E = 16384;   // the routing kernels keep one 4-byte counter per expert in LDS (64 KB without raising the limit)
size_t route_workspace_bytes(int Tk, int E);
// Static device scratch of smoe_route_noalloc: its size, and the address of the current device's copy.
constexpr size_t ROUTE_SCRATCH_BYTES = (size_t)1 << 20;
int route_scratch_address(int32_t **ptr);
int launch_route(hipStream_t s, const int32_t *expert_idxs, int Tk, int E, int32_t *sorted_e,
                 int32_t *sorted_s, int32_t *offsets, void *ws);

// ---- elementwise.hip
int launch_act_fwd(hipStream_t s, smoe_dtype dt, smoe_act act, const void *Hpre, void *H, int rows, int d_expert);
int launch_act_bwd(hipStream_t s, smoe_dtype dt, smoe_act act, const void *Hpre, const void *dH, void *dHpre,
                   int rows, int d_expert);
// Y[t] = sum_j g[t*k+j] * Yhat[t*k+j]; g == nullptr means all ones.
int launch_combine(hipStream_t s, smoe_dtype dt, const void *Yhat, const float *g, void *Y, int T, int k, int d);
int launch_group(hipStream_t s, smoe_dtype dt, const void *in, const int32_t *o, int fan, const float *g,
                 void *out, int Tk, int d);
// dg[o[i]] = sum_c part[i, c] (c ascending): finishes the routing-weight gradient left in slabs by the fused
// SwiGLU backward epilogue.
int launch_dp_reduce(hipStream_t s, const float *part, int ld, const int32_t *o, float *dg, int Tk);
// g_sorted[i] = g[o[i]]: the routing weight of every expert-sorted row
int launch_sorted_weights(hipStream_t s, const int32_t *o, const float *g, float *g_sorted, int Tk);
// dg[s] = <dY[s / kp], Yhat[s]>
int launch_rowdot(hipStream_t s, smoe_dtype dt, const void *dY, const void *Yhat, float *dg, int Tk, int kp, int d);

// ---- GEMM launchers (gemm_plain.hip, gemm_mfma.hip)
struct S2SArgs {      // C[out(i), :] = A[in(i), :] * op(W[e(i)])   for sorted rows i
  const void *A;      // [*, K] rows addressed through a_map
  const void *W;      // [E, d_in, d_out]
  void *C;            // [*, N] rows addressed through c_map
  RowMap a_map, c_map;
  const int32_t *offsets;  // [E+1]
  int E, Tk;
  int K, N;           // contraction length and output width
  int ldw;            // row stride of W[e] (= d_out)
  size_t w_stride;    // elements between experts (= d_in * d_out)
  int trans_w;        // 0: op(W) = W (K = d_in, N = d_out); 1: op(W) = W^T (K = d_out, N = d_in)
  // Optional scratch for splitting the contraction of the last, partly filled round of tiles over the
  // compute units that would otherwise idle (S2S_TAIL_WS_BYTES of device memory, or NULL: no split).
  float *tail_ws;
  int grid = 256;     // blocks of the persistent kernel (smoe_ctx::stream_grid)
  int group_m = 4;    // tiles are numbered in groups of this many M-tiles x all N-tiles (smoe_ctx::group_m)
  // Optional fused SwiGLU of Alg. 3 (forward, expert-sorted output only): W's columns are
  // [gate | up] halves of width N / 2 and H [*, N / 2] receives silu(gate) * up; C may then be
  // NULL when the pre-activation is not kept.
  void *H;
  // Optional fused SwiGLU backward of Alg. 3 (input-gradient product of the second ParallelLinear, expert-sorted
  // out, op(W) = W^T, N = d_expert): A holds the UNWEIGHTED upstream rows (gathered through a_map or already
  // expert-sorted), so the fp32 accumulators are dH / p.  With Hpre_in [Tk, 2N] (the saved pre-activation), row_scale [Tk] (the routing
  // weight of every sorted row) and dp_part [Tk, 2 * ceil(N / 256)] fp32 set, the epilogue writes
  // C = dHpre [Tk, 2N] = sigma'(Hpre) * row_scale * acc instead of dH, and per row and 128-column slab the
  // partial dot <acc, silu(gate) * up> whose sum over the slabs is Alg. 2's dp for that row.
  // Optional [2 * grid] device array: block b leaves the shader-clock cycles and the 100 MHz real-time ticks between its
  // first and last instruction in entries 2b and 2b+1 (measurement aid: the ratio is the clock the block ran at).
  unsigned long long *clock_probe = nullptr;
  const void *Hpre_in = nullptr;
  const float *row_scale = nullptr;
  float *dp_part = nullptr;
  // The same idea for any activation (still the W2^T product on unweighted rows): with H_in [Tk, N] (the saved
  // hidden activations), row_scale and dp_part set and Hpre_in NULL, the epilogue writes C = dH = row_scale * acc, the
  // slabs of dp = <acc, H>, and, when Hw_out [Tk, N] is given, Hw = row_scale * H (the routing-weighted hidden rows
  // that let groupXTY take the unweighted sorted dY for dW2 as well).  The activation's derivative stays a row kernel.
  const void *H_in = nullptr;
  void *Hw_out = nullptr;
};
struct DWArgs {       // dW[e] = sum_{i in segment e} A[i, :]^T B[i, :]   (both operands expert-sorted)
  const void *A;      // [Tk, M]
  const void *B;      // [Tk, N]
  void *dW;           // [E, M, N]
  const int32_t *offsets;
  int E, Tk, M, N;
  // Optional scratch (S2S_TAIL_WS_BYTES of device memory, or NULL): when the output tiles of all experts fill
  // only a fraction of the chip (a dense projection run as one expert), each segment's rows are cut into chunks
  // that leave fp32 partial tiles here, added in chunk order by a second kernel.
  float *split_ws = nullptr;
  int grid = 256;     // blocks of the persistent kernel (smoe_ctx::stream_grid)
};
int launch_s2s_plain(hipStream_t s, smoe_dtype dt, const S2SArgs &a);
int launch_dw_plain(hipStream_t s, smoe_dtype dt, const DWArgs &a);
bool s2s_mfma_supported(const S2SArgs &a);
bool dw_mfma_supported(const DWArgs &a);
int launch_s2s_mfma(hipStream_t s, const S2SArgs &a);
int launch_dw_mfma(hipStream_t s, const DWArgs &a);
// Per-device set-up of the kernels that need more dynamic LDS than the default limit (called by
// smoe_create with the context's device current).
int init_mfma_kernels();
int init_stream_kernels();
// persistent tile-stream kernels (gemm_stream.hip)
constexpr size_t S2S_TAIL_WS_BYTES = (size_t)256 * 256 * 256 * sizeof(float);   // 256 partial tiles of 256 x 256 fp32
bool s2s_stream_supported(const S2SArgs &a);
bool s2s_stream_swiglu_supported(const S2SArgs &a);
bool s2s_stream_swiglu_bwd_supported(const S2SArgs &a);
bool s2s_stream_dp_supported(const S2SArgs &a);
int launch_s2s_stream(hipStream_t s, const S2SArgs &a);
// Small-batch (decoding) forward products: 32-row tiles, one wavefront each, bound by the weight stream.
// Takes a.H like the persistent kernel (fused SwiGLU).
bool s2s_decode_supported(const S2SArgs &a);
int launch_s2s_decode(hipStream_t s, const S2SArgs &a);
bool dw_stream_supported(const DWArgs &a);
int launch_dw_stream(hipStream_t s, const DWArgs &a);
