// Routing kernels: top-k gate (Sec. 3.1 step 1) and the stable bucket sort of the routed
// slots by expert (Sec. 3.1 step 2), integer-exact.
#include "common.h"

// ---------------------------------------------------------------------------------------
// top-k gate: one thread per token.  Slot j takes the largest logit that comes after slot
// j-1's pick in the order (value descending, expert id ascending), so ties go to the lower
// id and no per-thread array is needed.  Gates are the softmax over the k picks.  A NaN logit
// counts as -inf (it can only be kept after every number), and picks that are all -inf share
// the weight equally, so every token writes all k slots whatever its logits hold.
// ---------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256) topk_gate_kernel(const float *__restrict__ logits, int T, int E, int k,
                                                        int32_t *__restrict__ idx, float *__restrict__ gates) {
  int t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= T) return;
  const float *row = logits + (size_t)t * E;
  float prev_v = 0.f, first_v = 0.f, sum = 0.f;
  int prev_i = -1;
  for (int j = 0; j < k; ++j) {
    float best_v = 0.f;
    int best_i = -1;
    for (int e = 0; e < E; ++e) {
      float v = row[e];
      if (v != v) v = -INFINITY;
      bool after_prev = (prev_i < 0) || (v < prev_v) || (v == prev_v && e > prev_i);
      bool better = (best_i < 0) || (v > best_v);  // first hit wins ties -> lower id
      if (after_prev && better) { best_v = v; best_i = e; }
    }
    if (j == 0) first_v = best_v;
    float w = first_v == -INFINITY ? 1.0f : expf(best_v - first_v);
    idx[(size_t)t * k + j] = best_i;
    gates[(size_t)t * k + j] = w;
    sum += w;
    prev_v = best_v;
    prev_i = best_i;
  }
  float inv = 1.0f / sum;
  for (int j = 0; j < k; ++j) gates[(size_t)t * k + j] *= inv;
}

// Same selection with one wavefront per token for E <= 64 * VPL, by ranking: lane x holds logits x,
// x + 64, ...; the token's row sits in LDS and every lane counts, for each of its logits, how many
// come before it in the order (value descending, expert id ascending).  A logit of rank r < k is slot r.
template <int VPL>
__global__ void __launch_bounds__(256) topk_gate_wave_kernel(const float *__restrict__ logits, int T, int E, int k,
                                                             int32_t *__restrict__ idx, float *__restrict__ gates) {
  __shared__ __attribute__((aligned(16))) float rows[4][64 * VPL];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int t = blockIdx.x * 4 + wave;
  if (t >= T) return;
  float *row = rows[wave];
  float v[VPL];
  int rank[VPL];
#pragma unroll
  for (int i = 0; i < VPL; ++i) {
    int e = lane + 64 * i;
    // padding ranks after every real logit and never before one (-inf loses ties to the lower real ids)
    v[i] = e < E ? logits[(size_t)t * E + e] : -INFINITY;
    if (v[i] != v[i]) v[i] = -INFINITY;   // NaN counts as -inf
    row[e] = v[i];
    rank[i] = 0;
  }
  const int E4 = (E + 3) & ~3;   // the row is read four logits at a time; entries up to 64 * VPL are initialised
  for (int e0 = 0; e0 < E4; e0 += 4) {
    const float4 o4 = *reinterpret_cast<const float4 *>(row + e0);   // same address in every lane: a broadcast read
    const float o[4] = {o4.x, o4.y, o4.z, o4.w};
#pragma unroll
    for (int c = 0; c < 4; ++c)
#pragma unroll
      for (int i = 0; i < VPL; ++i) rank[i] += (o[c] > v[i]) || (o[c] == v[i] && e0 + c < lane + 64 * i);
  }
  // the rank-0 logit is the maximum; the gates are the softmax over the k kept logits
  float top = v[0];
#pragma unroll
  for (int i = 1; i < VPL; ++i) top = fmaxf(top, v[i]);
#pragma unroll
  for (int d = 32; d > 0; d >>= 1) top = fmaxf(top, __shfl_xor(top, d, 64));
  float w[VPL], sum = 0.f;
#pragma unroll
  for (int i = 0; i < VPL; ++i) {
    w[i] = (rank[i] < k && lane + 64 * i < E) ? (top == -INFINITY ? 1.0f : expf(v[i] - top)) : 0.f;
    sum += w[i];
  }
#pragma unroll
  for (int d = 32; d > 0; d >>= 1) sum += __shfl_xor(sum, d, 64);
  const float inv = 1.0f / sum;
#pragma unroll
  for (int i = 0; i < VPL; ++i)
    if (rank[i] < k && lane + 64 * i < E) {
      idx[(size_t)t * k + rank[i]] = lane + 64 * i;
      gates[(size_t)t * k + rank[i]] = w[i] * inv;
    }
}

int launch_topk_gate(hipStream_t s, const float *logits, int T, int E, int k, int32_t *idx, float *gates) {
  if (T == 0) return SMOE_OK;
  dim3 grid(ceil_div(T, 4)), block(256);
  if (E <= 64)
    hipLaunchKernelGGL(topk_gate_wave_kernel<1>, grid, block, 0, s, logits, T, E, k, idx, gates);
  else if (E <= 128)
    hipLaunchKernelGGL(topk_gate_wave_kernel<2>, grid, block, 0, s, logits, T, E, k, idx, gates);
  else if (E <= 256)
    hipLaunchKernelGGL(topk_gate_wave_kernel<4>, grid, block, 0, s, logits, T, E, k, idx, gates);
  else
    hipLaunchKernelGGL(topk_gate_kernel, dim3(ceil_div(T, 256)), dim3(256), 0, s, logits, T, E, k, idx, gates);
  SMOE_LAUNCH_CHECK();
  return SMOE_OK;
}

// Gradient of the gate with respect to the router logits: softmax Jacobian on the k kept
// experts (g_j (dp_j - sum_i g_i dp_i)), zero elsewhere.  One thread per (token, expert)
// element so the [T,E] row is written whole and coalesced.
__global__ void __launch_bounds__(256) topk_gate_bwd_kernel(const int32_t *__restrict__ idx,
                                                            const float *__restrict__ gates,
                                                            const float *__restrict__ dgates, size_t total, int E, int k,
                                                            float *__restrict__ dlogits) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= total) return;
  size_t t = i / E;
  int e = (int)(i - t * E);
  const size_t base = t * k;
  float dot = 0.f, g_mine = 0.f, dp_mine = 0.f;
  for (int j = 0; j < k; ++j) {
    float g = gates[base + j], dp = dgates[base + j];
    dot += g * dp;
    if (idx[base + j] == e) { g_mine = g; dp_mine = dp; }
  }
  dlogits[i] = g_mine * (dp_mine - dot);
}

int launch_topk_gate_bwd(hipStream_t s, const int32_t *idx, const float *gates, const float *dgates, int T, int E, int k,
                         float *dlogits) {
  size_t total = (size_t)T * E;
  if (total == 0) return SMOE_OK;
  hipLaunchKernelGGL(topk_gate_bwd_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, idx, gates, dgates, total,
                     E, k, dlogits);
  SMOE_LAUNCH_CHECK();
  return SMOE_OK;
}

// ---------------------------------------------------------------------------------------
// Stable bucket sort by expert in three launches:
//   1. each 64-lane block counts the experts of its contiguous chunk of slots,
//   2. one block turns the [chunk][expert] counts into start positions (expert-major
//      exclusive scan) and writes expert_offsets,
//   3. each block walks its chunk again 64 slots at a time; a lane's rank among the lanes
//      of the same expert comes from wavefront ballots over the bits of the expert id.
// Slots keep their order inside an expert because chunks, steps and lanes are all visited
// in ascending slot order.
// ---------------------------------------------------------------------------------------
static constexpr int ROUTE_CHUNK = 1024;  // slots per block

__device__ __forceinline__ int clamp_expert(int e, int E) { return e < 0 ? 0 : (e >= E ? E - 1 : e); }

__global__ void __launch_bounds__(64) route_count_kernel(const int32_t *__restrict__ expert_idxs, int Tk, int E,
                                                         int32_t *__restrict__ counts /*[E][nchunk]*/) {
  extern __shared__ int32_t hist[];
  for (int e = threadIdx.x; e < E; e += 64) hist[e] = 0;
  __syncthreads();
  int base = blockIdx.x * ROUTE_CHUNK;
  int end = min(base + ROUTE_CHUNK, Tk);
  for (int s = base + threadIdx.x; s < end; s += 64) atomicAdd(&hist[clamp_expert(expert_idxs[s], E)], 1);
  __syncthreads();
  // expert-major so that the scan below reads each expert's chunk counts contiguously
  for (int e = threadIdx.x; e < E; e += 64) counts[(size_t)e * gridDim.x + blockIdx.x] = hist[e];
}

// counts[e][c] -> start position of (chunk c, expert e); offsets[e] = rows before expert e.  One wavefront
// per expert at a time: lanes take chunks, a wave prefix sum orders them.
__global__ void __launch_bounds__(1024) route_scan_kernel(int32_t *__restrict__ counts, int nchunk, int E,
                                                          int32_t *__restrict__ offsets, int Tk) {
  extern __shared__ int32_t totals[];  // [E] rows per expert, then exclusive prefix
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nwave = blockDim.x >> 6;
  for (int e = wave; e < E; e += nwave) {
    int sum = 0;
    for (int c = lane; c < nchunk; c += 64) sum += counts[(size_t)e * nchunk + c];
#pragma unroll
    for (int d = 32; d > 0; d >>= 1) sum += __shfl_xor(sum, d, 64);
    if (lane == 0) totals[e] = sum;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    int run = 0;
    for (int e = 0; e < E; ++e) {
      int n = totals[e];
      totals[e] = run;
      offsets[e] = run;
      run += n;
    }
    offsets[E] = run;
  }
  __syncthreads();
  for (int e = wave; e < E; e += nwave) {
    int run = totals[e];
    for (int c0 = 0; c0 < nchunk; c0 += 64) {
      int c = c0 + lane;
      int n = (c < nchunk) ? counts[(size_t)e * nchunk + c] : 0;
      int incl = n;
#pragma unroll
      for (int d = 1; d < 64; d <<= 1) {
        int up = __shfl_up(incl, d, 64);
        if (lane >= d) incl += up;
      }
      if (c < nchunk) counts[(size_t)e * nchunk + c] = run + incl - n;
      run += __shfl(incl, 63, 64);
    }
  }
}

__global__ void __launch_bounds__(64) route_place_kernel(const int32_t *__restrict__ expert_idxs, int Tk, int E,
                                                         const int32_t *__restrict__ starts /*[E][nchunk]*/,
                                                         int32_t *__restrict__ sorted_e,
                                                         int32_t *__restrict__ sorted_s) {
  extern __shared__ int32_t next[];  // next free position per expert for this chunk
  for (int e = threadIdx.x; e < E; e += 64) next[e] = starts[(size_t)e * gridDim.x + blockIdx.x];
  __syncthreads();
  int nbits = 32 - __clz(max(E - 1, 1));
  int base = blockIdx.x * ROUTE_CHUNK;
  int end = min(base + ROUTE_CHUNK, Tk);
  int lane = threadIdx.x;
  unsigned long long lt_mask = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
  for (int s0 = base; s0 < end; s0 += 64) {
    int s = s0 + lane;
    bool live = s < end;
    int e = live ? clamp_expert(expert_idxs[s], E) : 0;
    unsigned long long peers = __ballot(live);
    for (int b = 0; b < nbits; ++b) {
      unsigned long long set = __ballot(live && ((e >> b) & 1));
      peers &= ((e >> b) & 1) ? set : ~set;
    }
    int rank = __popcll(peers & lt_mask);
    int pos = 0;
    if (live) pos = next[e] + rank;
    __syncthreads();
    if (live && rank == 0) next[e] += __popcll(peers);  // lowest lane of each expert updates
    __syncthreads();
    if (live) {
      sorted_e[pos] = e;
      sorted_s[pos] = s;
    }
  }
}

// All three steps in one wavefront when the slots fit one chunk (decoding batches): histogram, exclusive
// scan over the experts, stable placement.  Nothing passes through global memory in between.
__global__ void __launch_bounds__(64) route_single_chunk_kernel(const int32_t *__restrict__ expert_idxs, int Tk, int E,
                                                                int32_t *__restrict__ offsets,
                                                                int32_t *__restrict__ sorted_e,
                                                                int32_t *__restrict__ sorted_s) {
  extern __shared__ int32_t next[];  // rows per expert, then next free position per expert
  const int lane = threadIdx.x;
  for (int e = lane; e < E; e += 64) next[e] = 0;
  __syncthreads();
  for (int s = lane; s < Tk; s += 64) atomicAdd(&next[clamp_expert(expert_idxs[s], E)], 1);
  __syncthreads();
  int run = 0;
  for (int c0 = 0; c0 < E; c0 += 64) {
    const int e = c0 + lane;
    const int n = e < E ? next[e] : 0;
    int incl = n;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
      int up = __shfl_up(incl, d, 64);
      if (lane >= d) incl += up;
    }
    if (e < E) {
      next[e] = run + incl - n;
      offsets[e] = run + incl - n;
    }
    run += __shfl(incl, 63, 64);
  }
  if (lane == 0) offsets[E] = run;
  __syncthreads();
  const int nbits = 32 - __clz(max(E - 1, 1));
  const unsigned long long lt_mask = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
  for (int s0 = 0; s0 < Tk; s0 += 64) {
    const int s = s0 + lane;
    const bool live = s < Tk;
    const int e = live ? clamp_expert(expert_idxs[s], E) : 0;
    unsigned long long peers = __ballot(live);
    for (int b = 0; b < nbits; ++b) {
      unsigned long long set = __ballot(live && ((e >> b) & 1));
      peers &= ((e >> b) & 1) ? set : ~set;
    }
    const int rank = __popcll(peers & lt_mask);
    int pos = 0;
    if (live) pos = next[e] + rank;
    __syncthreads();
    if (live && rank == 0) next[e] += __popcll(peers);  // lowest lane of each expert updates
    __syncthreads();
    if (live) {
      sorted_e[pos] = e;
      sorted_s[pos] = s;
    }
  }
}

// Scratch of the no-allocation routing entry point: the per-chunk expert counts that smoe_route keeps in
// caller workspace live here instead.  One copy per device, held until the process ends.  In host code the
// array's name is only a handle for hipGetSymbolAddress: kernels get the address looked up below.
static __device__ __align__(256) int32_t scratch[ROUTE_SCRATCH_BYTES / sizeof(int32_t)];

// Address of the current device's copy of the scratch array (called once per context, with the context's
// device current).
int route_scratch_address(int32_t **ptr) {
  void *p = nullptr;
  if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) return SMOE_ERR_HIP;
  *ptr = (int32_t *)p;
  return SMOE_OK;
}

size_t route_workspace_bytes(int Tk, int E) {
  size_t nchunk = (size_t)ceil_div(Tk > 0 ? Tk : 1, ROUTE_CHUNK);
  return align256(nchunk * (size_t)E * sizeof(int32_t));
}

int launch_route(hipStream_t s, const int32_t *expert_idxs, int Tk, int E, int32_t *sorted_e, int32_t *sorted_s,
                 int32_t *offsets, void *ws) {
  int nchunk = ceil_div(Tk > 0 ? Tk : 1, ROUTE_CHUNK);
  int32_t *counts = (int32_t *)ws;
  size_t shm = (size_t)E * sizeof(int32_t);
  if (nchunk == 1) {
    hipLaunchKernelGGL(route_single_chunk_kernel, dim3(1), dim3(64), shm, s, expert_idxs, Tk, E, offsets, sorted_e, sorted_s);
    SMOE_LAUNCH_CHECK();
    return SMOE_OK;
  }
  hipLaunchKernelGGL(route_count_kernel, dim3(nchunk), dim3(64), shm, s, expert_idxs, Tk, E, counts);
  SMOE_LAUNCH_CHECK();
  hipLaunchKernelGGL(route_scan_kernel, dim3(1), dim3(1024), shm, s, counts, nchunk, E, offsets, Tk);
  SMOE_LAUNCH_CHECK();
  if (Tk > 0) {
    hipLaunchKernelGGL(route_place_kernel, dim3(nchunk), dim3(64), shm, s, expert_idxs, Tk, E, counts, sorted_e,
                       sorted_s);
    SMOE_LAUNCH_CHECK();
  }
  return SMOE_OK;
}
