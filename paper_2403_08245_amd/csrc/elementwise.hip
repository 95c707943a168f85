// Memory-bound row kernels around the grouped GEMMs: the activation of Alg. 3, the weighted
// sum over a token's k slots (Alg. 1), the `group` copy and the routing-weight gradient of
// Alg. 2.  All read/write 16 bytes per lane when the row width allows it.
#include "common.h"

template <typename T> struct Vec16 { static constexpr int N = 16 / sizeof(T); T v[N]; } __attribute__((aligned(16)));

template <typename T> __device__ __forceinline__ void load_vec(const T *p, float (&f)[16 / sizeof(T)]) {
  Vec16<T> r = *reinterpret_cast<const Vec16<T> *>(p);
#pragma unroll
  for (int i = 0; i < Vec16<T>::N; ++i) f[i] = to_f32<T>(r.v[i]);
}
template <typename T> __device__ __forceinline__ void store_vec(T *p, const float (&f)[16 / sizeof(T)]) {
  Vec16<T> r;
#pragma unroll
  for (int i = 0; i < Vec16<T>::N; ++i) r.v[i] = from_f32<T>(f[i]);
  *reinterpret_cast<Vec16<T> *>(p) = r;
}

__device__ __forceinline__ float gelu_f(float x) { return 0.5f * x * (1.0f + erff(x * 0.70710678118654752440f)); }
__device__ __forceinline__ float gelu_grad_f(float x) {
  float cdf = 0.5f * (1.0f + erff(x * 0.70710678118654752440f));
  float pdf = expf(-0.5f * x * x) * 0.39894228040143267794f;
  return cdf + x * pdf;
}
__device__ __forceinline__ float sigmoid_f(float x) { return 1.0f / (1.0f + expf(-x)); }

// ---- activation forward: H = act(Hpre).  Work item = VEC consecutive hidden units of a row.
template <typename T, int ACT>
__global__ void __launch_bounds__(256) act_fwd_kernel(const T *__restrict__ Hpre, T *__restrict__ H, size_t rows,
                                                      int d_expert) {
  constexpr int V = 16 / sizeof(T);
  const int d_h = (ACT == SMOE_ACT_SWIGLU) ? 2 * d_expert : d_expert;
  const size_t per_row = d_expert / V;
  const size_t total = rows * per_row;
  for (size_t w = blockIdx.x * (size_t)blockDim.x + threadIdx.x; w < total; w += (size_t)gridDim.x * blockDim.x) {
    size_t r = w / per_row;
    int c = (int)(w % per_row) * V;
    float a[V], out[V];
    load_vec<T>(Hpre + r * d_h + c, a);
    if (ACT == SMOE_ACT_SWIGLU) {
      float u[V];
      load_vec<T>(Hpre + r * d_h + d_expert + c, u);
#pragma unroll
      for (int i = 0; i < V; ++i) out[i] = a[i] * sigmoid_f(a[i]) * u[i];
    } else if (ACT == SMOE_ACT_GELU) {
#pragma unroll
      for (int i = 0; i < V; ++i) out[i] = gelu_f(a[i]);
    } else {
#pragma unroll
      for (int i = 0; i < V; ++i) out[i] = a[i];
    }
    store_vec<T>(H + r * d_expert + c, out);
  }
}

// ---- activation backward: dHpre = act'(Hpre) * dH.
template <typename T, int ACT>
__global__ void __launch_bounds__(256) act_bwd_kernel(const T *__restrict__ Hpre, const T *__restrict__ dH,
                                                      T *__restrict__ dHpre, size_t rows, int d_expert) {
  constexpr int V = 16 / sizeof(T);
  const int d_h = (ACT == SMOE_ACT_SWIGLU) ? 2 * d_expert : d_expert;
  const size_t per_row = d_expert / V;
  const size_t total = rows * per_row;
  for (size_t w = blockIdx.x * (size_t)blockDim.x + threadIdx.x; w < total; w += (size_t)gridDim.x * blockDim.x) {
    size_t r = w / per_row;
    int c = (int)(w % per_row) * V;
    float a[V], g[V], o1[V];
    load_vec<T>(Hpre + r * d_h + c, a);
    load_vec<T>(dH + r * d_expert + c, g);
    if (ACT == SMOE_ACT_SWIGLU) {
      float u[V], o2[V];
      load_vec<T>(Hpre + r * d_h + d_expert + c, u);
#pragma unroll
      for (int i = 0; i < V; ++i) {
        float sg = sigmoid_f(a[i]);
        float silu = a[i] * sg;
        o1[i] = g[i] * u[i] * (sg + silu * (1.0f - sg));
        o2[i] = g[i] * silu;
      }
      store_vec<T>(dHpre + r * d_h + c, o1);
      store_vec<T>(dHpre + r * d_h + d_expert + c, o2);
    } else {
#pragma unroll
      for (int i = 0; i < V; ++i) o1[i] = (ACT == SMOE_ACT_GELU) ? g[i] * gelu_grad_f(a[i]) : g[i];
      store_vec<T>(dHpre + r * d_h + c, o1);
    }
  }
}

// ---- weighted sum over a token's k slots: Y[t] = sum_j g[t*k+j] * Yhat[t*k+j]  (g may be null = 1)
template <typename T>
__global__ void __launch_bounds__(256) combine_kernel(const T *__restrict__ Yhat, const float *__restrict__ g,
                                                      T *__restrict__ Y, size_t T_rows, int k, int d) {
  constexpr int V = 16 / sizeof(T);
  const size_t per_row = d / V;
  const size_t total = T_rows * per_row;
  for (size_t w = blockIdx.x * (size_t)blockDim.x + threadIdx.x; w < total; w += (size_t)gridDim.x * blockDim.x) {
    size_t t = w / per_row;
    int c = (int)(w % per_row) * V;
    float acc[V];
#pragma unroll
    for (int i = 0; i < V; ++i) acc[i] = 0.f;
    for (int j = 0; j < k; ++j) {
      float a[V];
      load_vec<T>(Yhat + (t * k + j) * d + c, a);
      float gj = g ? g[t * k + j] : 1.0f;
#pragma unroll
      for (int i = 0; i < V; ++i) acc[i] = fmaf(gj, a[i], acc[i]);
    }
    store_vec<T>(Y + t * d + c, acc);
  }
}

// ---- group: out[i] = scale * in[o[i] / fan]
template <typename T>
__global__ void __launch_bounds__(256) group_kernel(const T *__restrict__ in, const int32_t *__restrict__ o, int fan,
                                                    const float *__restrict__ g, T *__restrict__ out, size_t Tk,
                                                    int d) {
  constexpr int V = 16 / sizeof(T);
  const size_t per_row = d / V;
  const size_t total = Tk * per_row;
  for (size_t w = blockIdx.x * (size_t)blockDim.x + threadIdx.x; w < total; w += (size_t)gridDim.x * blockDim.x) {
    size_t i = w / per_row;
    int c = (int)(w % per_row) * V;
    int s = o[i];
    float a[V];
    load_vec<T>(in + (size_t)(s / fan) * d + c, a);
    if (g) {
      float gs = g[s];
#pragma unroll
      for (int q = 0; q < V; ++q) a[q] *= gs;
    }
    store_vec<T>(out + i * d + c, a);
  }
}

// ---- dg[o[i]] = sum_c part[i, c], c ascending (fixed order): one thread per sorted row
__global__ void __launch_bounds__(256) dp_reduce_kernel(const float *__restrict__ part, int ld, const int32_t *__restrict__ o,
                                                        float *__restrict__ dg, int Tk) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= Tk) return;
  const float *p = part + (size_t)i * ld;
  float acc = 0.f;
  for (int c = 0; c < ld; ++c) acc += p[c];
  dg[o[i]] = acc;
}

// ---- dg[s] = <dY[s / kp], Yhat[s]> : one wavefront per slot, lanes stride the row.
template <typename T>
__global__ void __launch_bounds__(256) rowdot_kernel(const T *__restrict__ dY, const T *__restrict__ Yhat,
                                                     float *__restrict__ dg, int Tk, int kp, int d) {
  constexpr int V = 16 / sizeof(T);
  int lane = threadIdx.x & 63;
  int s = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (s >= Tk) return;
  const T *a = dY + (size_t)(s / kp) * d;
  const T *b = Yhat + (size_t)s * d;
  float acc = 0.f;
  for (int c = lane * V; c < d; c += 64 * V) {
    float x[V], y[V];
    load_vec<T>(a + c, x);
    load_vec<T>(b + c, y);
#pragma unroll
    for (int i = 0; i < V; ++i) acc = fmaf(x[i], y[i], acc);
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) acc += __shfl_xor(acc, off, 64);
  if (lane == 0) dg[s] = acc;
}

// -----------------------------------------------------------------------------------------
static inline int grid_for(size_t work_items) {
  size_t b = (work_items + 255) / 256;
  if (b > 256 * 64) b = 256 * 64;
  return (int)(b ? b : 1);
}
template <typename T> static bool vec_ok(int d) { return d % (16 / (int)sizeof(T)) == 0; }

template <typename T>
static int act_fwd_t(hipStream_t s, smoe_act act, const void *Hpre, void *H, int rows, int d_expert) {
  if (!vec_ok<T>(d_expert)) return SMOE_ERR_UNSUPPORTED;
  size_t items = (size_t)rows * (d_expert / (16 / sizeof(T)));
  if (!items) return SMOE_OK;
  dim3 g(grid_for(items)), b(256);
  const T *in = (const T *)Hpre;
  T *out = (T *)H;
  if (act == SMOE_ACT_SWIGLU) hipLaunchKernelGGL((act_fwd_kernel<T, SMOE_ACT_SWIGLU>), g, b, 0, s, in, out, (size_t)rows, d_expert);
  else if (act == SMOE_ACT_GELU) hipLaunchKernelGGL((act_fwd_kernel<T, SMOE_ACT_GELU>), g, b, 0, s, in, out, (size_t)rows, d_expert);
  else hipLaunchKernelGGL((act_fwd_kernel<T, SMOE_ACT_NONE>), g, b, 0, s, in, out, (size_t)rows, d_expert);
  SMOE_LAUNCH_CHECK();
  return SMOE_OK;
}
int launch_act_fwd(hipStream_t s, smoe_dtype dt, smoe_act act, const void *Hpre, void *H, int rows, int d_expert) {
  return dt == SMOE_BF16 ? act_fwd_t<bf16_t>(s, act, Hpre, H, rows, d_expert) : act_fwd_t<float>(s, act, Hpre, H, rows, d_expert);
}

template <typename T>
static int act_bwd_t(hipStream_t s, smoe_act act, const void *Hpre, const void *dH, void *dHpre, int rows, int d_expert) {
  if (!vec_ok<T>(d_expert)) return SMOE_ERR_UNSUPPORTED;
  size_t items = (size_t)rows * (d_expert / (16 / sizeof(T)));
  if (!items) return SMOE_OK;
  dim3 g(grid_for(items)), b(256);
  const T *a = (const T *)Hpre; const T *gr = (const T *)dH; T *out = (T *)dHpre;
  if (act == SMOE_ACT_SWIGLU) hipLaunchKernelGGL((act_bwd_kernel<T, SMOE_ACT_SWIGLU>), g, b, 0, s, a, gr, out, (size_t)rows, d_expert);
  else if (act == SMOE_ACT_GELU) hipLaunchKernelGGL((act_bwd_kernel<T, SMOE_ACT_GELU>), g, b, 0, s, a, gr, out, (size_t)rows, d_expert);
  else hipLaunchKernelGGL((act_bwd_kernel<T, SMOE_ACT_NONE>), g, b, 0, s, a, gr, out, (size_t)rows, d_expert);
  SMOE_LAUNCH_CHECK();
  return SMOE_OK;
}
int launch_act_bwd(hipStream_t s, smoe_dtype dt, smoe_act act, const void *Hpre, const void *dH, void *dHpre, int rows, int d_expert) {
  return dt == SMOE_BF16 ? act_bwd_t<bf16_t>(s, act, Hpre, dH, dHpre, rows, d_expert)
                         : act_bwd_t<float>(s, act, Hpre, dH, dHpre, rows, d_expert);
}

template <typename T>
static int combine_t(hipStream_t s, const void *Yhat, const float *g, void *Y, int T_rows, int k, int d) {
  if (!vec_ok<T>(d)) return SMOE_ERR_UNSUPPORTED;
  size_t items = (size_t)T_rows * (d / (16 / sizeof(T)));
  if (!items) return SMOE_OK;
  hipLaunchKernelGGL((combine_kernel<T>), dim3(grid_for(items)), dim3(256), 0, s, (const T *)Yhat, g, (T *)Y, (size_t)T_rows, k, d);
  SMOE_LAUNCH_CHECK();
  return SMOE_OK;
}
int launch_combine(hipStream_t s, smoe_dtype dt, const void *Yhat, const float *g, void *Y, int T, int k, int d) {
  return dt == SMOE_BF16 ? combine_t<bf16_t>(s, Yhat, g, Y, T, k, d) : combine_t<float>(s, Yhat, g, Y, T, k, d);
}

template <typename T>
static int group_t(hipStream_t s, const void *in, const int32_t *o, int fan, const float *g, void *out, int Tk, int d) {
  if (!vec_ok<T>(d)) return SMOE_ERR_UNSUPPORTED;
  size_t items = (size_t)Tk * (d / (16 / sizeof(T)));
  if (!items) return SMOE_OK;
  hipLaunchKernelGGL((group_kernel<T>), dim3(grid_for(items)), dim3(256), 0, s, (const T *)in, o, fan, g, (T *)out, (size_t)Tk, d);
  SMOE_LAUNCH_CHECK();
  return SMOE_OK;
}
int launch_group(hipStream_t s, smoe_dtype dt, const void *in, const int32_t *o, int fan, const float *g, void *out, int Tk, int d) {
  return dt == SMOE_BF16 ? group_t<bf16_t>(s, in, o, fan, g, out, Tk, d) : group_t<float>(s, in, o, fan, g, out, Tk, d);
}

__global__ void __launch_bounds__(256) sorted_weights_kernel(const int32_t *__restrict__ o, const float *__restrict__ g,
                                                             float *__restrict__ g_sorted, int Tk) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < Tk) g_sorted[i] = g[o[i]];
}
int launch_sorted_weights(hipStream_t s, const int32_t *o, const float *g, float *g_sorted, int Tk) {
  if (!Tk) return SMOE_OK;
  hipLaunchKernelGGL(sorted_weights_kernel, dim3(ceil_div(Tk, 256)), dim3(256), 0, s, o, g, g_sorted, Tk);
  SMOE_LAUNCH_CHECK();
  return SMOE_OK;
}

int launch_dp_reduce(hipStream_t s, const float *part, int ld, const int32_t *o, float *dg, int Tk) {
  if (!Tk) return SMOE_OK;
  hipLaunchKernelGGL(dp_reduce_kernel, dim3(ceil_div(Tk, 256)), dim3(256), 0, s, part, ld, o, dg, Tk);
  SMOE_LAUNCH_CHECK();
  return SMOE_OK;
}

template <typename T>
static int rowdot_t(hipStream_t s, const void *dY, const void *Yhat, float *dg, int Tk, int kp, int d) {
  if (!vec_ok<T>(d)) return SMOE_ERR_UNSUPPORTED;
  if (!Tk) return SMOE_OK;
  hipLaunchKernelGGL((rowdot_kernel<T>), dim3(ceil_div(Tk, 4)), dim3(256), 0, s, (const T *)dY, (const T *)Yhat, dg, Tk, kp, d);
  SMOE_LAUNCH_CHECK();
  return SMOE_OK;
}
int launch_rowdot(hipStream_t s, smoe_dtype dt, const void *dY, const void *Yhat, float *dg, int Tk, int kp, int d) {
  return dt == SMOE_BF16 ? rowdot_t<bf16_t>(s, dY, Yhat, dg, Tk, kp, d) : rowdot_t<float>(s, dY, Yhat, dg, Tk, kp, d);
}

// ------------------------------------------------------------------------------------------
// helpers of the attention layer: offsets of a single all-rows segment (a dense product run
// through the grouped kernels as one expert), and the sum of three bf16 arrays
// ------------------------------------------------------------------------------------------
__global__ void dense_offsets_kernel(int32_t *off, int n) {
  if (threadIdx.x == 0) { off[0] = 0; off[1] = n; }
}
int launch_dense_offsets(hipStream_t s, int32_t *off, int n) {
  hipLaunchKernelGGL(dense_offsets_kernel, dim3(1), dim3(64), 0, s, off, n);
  SMOE_LAUNCH_CHECK();
  return SMOE_OK;
}

__global__ void __launch_bounds__(256) add3_kernel(const bf16_t *__restrict__ a, const bf16_t *__restrict__ b,
                                                   const bf16_t *__restrict__ c, bf16_t *__restrict__ out, size_t n8) {
  typedef bf16_t v8 __attribute__((ext_vector_type(8)));
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n8; i += (size_t)gridDim.x * blockDim.x) {
    v8 x = reinterpret_cast<const v8 *>(a)[i], y = reinterpret_cast<const v8 *>(b)[i], z = reinterpret_cast<const v8 *>(c)[i], r;
#pragma unroll
    for (int q = 0; q < 8; ++q) r[q] = (bf16_t)((float)x[q] + (float)y[q] + (float)z[q]);
    reinterpret_cast<v8 *>(out)[i] = r;
  }
}
int launch_add3(hipStream_t s, const void *a, const void *b, const void *c, void *out, size_t n) {
  if (n % 8) return SMOE_ERR_UNSUPPORTED;
  if (!n) return SMOE_OK;
  hipLaunchKernelGGL(add3_kernel, dim3(grid_for(n / 8)), dim3(256), 0, s, (const bf16_t *)a, (const bf16_t *)b,
                     (const bf16_t *)c, (bf16_t *)out, n / 8);
  SMOE_LAUNCH_CHECK();
  return SMOE_OK;
}
