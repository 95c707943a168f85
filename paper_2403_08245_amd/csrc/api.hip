// C ABI of libsmoe: argument checks, workspace layout and the order of kernel launches for
// ParallelLinear (Alg. 1, Alg. 2) and the SMoE MLP (Alg. 3).  No entry point allocates,
// synchronises or touches the host copy of any tensor.
#include "common.h"
#include <new>

namespace {
inline bool aligned16(const void *p) { return ((uintptr_t)p & 15) == 0; }

bool routing_ok(const smoe_routing *r) {
  if (!r || r->Tk < 0 || r->E < 1 || !r->expert_offsets) return false;
  return r->Tk == 0 || (r->sorted_expert_idxs && r->sorted_scattered_idxs);  // empty index arrays may be null
}
// Row widths must allow 16-byte accesses in the row kernels.
bool width_ok(smoe_dtype dt, int d) { return d > 0 && d % (int)(16 / dtype_size(dt)) == 0; }
bool dtype_ok(int dt) { return dt == SMOE_F32 || dt == SMOE_BF16; }

int run_s2s(smoe_ctx *ctx, hipStream_t s, smoe_dtype dt, S2SArgs a) {
  a.grid = ctx->stream_grid;
  a.group_m = ctx->group_m;
  a.clock_probe = ctx->clock_probe;
  if (dt == SMOE_BF16 && ctx->kernel_mode == 0 && s2s_decode_supported(a)) return launch_s2s_decode(s, a);
  if (dt == SMOE_BF16 && ctx->kernel_mode == 0 && s2s_stream_supported(a)) return launch_s2s_stream(s, a);
  if (dt == SMOE_BF16 && ctx->kernel_mode != 1 && s2s_mfma_supported(a)) return launch_s2s_mfma(s, a);
  return launch_s2s_plain(s, dt, a);
}
int run_dw(smoe_ctx *ctx, hipStream_t s, smoe_dtype dt, DWArgs a) {
  a.grid = ctx->stream_grid;
  if (dt == SMOE_BF16 && ctx->kernel_mode == 0 && dw_stream_supported(a)) return launch_dw_stream(s, a);
  if (dt == SMOE_BF16 && ctx->kernel_mode != 1 && dw_mfma_supported(a)) return launch_dw_mfma(s, a);
  return launch_dw_plain(s, dt, a);
}

S2SArgs make_s2s(const void *A, const void *W, void *C, const smoe_routing *r, int d_in, int d_out, bool trans_w,
                 bool a_grouped, int a_fan, bool c_grouped) {
  S2SArgs a;
  a.A = A; a.W = W; a.C = C;
  a.a_map = RowMap{a_grouped ? nullptr : r->sorted_scattered_idxs, a_fan};
  a.c_map = RowMap{c_grouped ? nullptr : r->sorted_scattered_idxs, 1};
  a.offsets = r->expert_offsets;
  a.E = r->E; a.Tk = r->Tk;
  a.K = trans_w ? d_out : d_in;
  a.N = trans_w ? d_in : d_out;
  a.ldw = d_out;
  a.w_stride = (size_t)d_in * d_out;
  a.trans_w = trans_w ? 1 : 0;
  a.H = nullptr;
  a.tail_ws = nullptr;
  return a;
}
}  // namespace

extern "C" {

int smoe_abi_version(void) { return 1; }

const char *smoe_strerror(int status) {
  switch (status) {
    case SMOE_OK: return "ok";
    case SMOE_ERR_INVALID_ARG: return "invalid argument";
    case SMOE_ERR_UNSUPPORTED: return "unsupported shape or option (row widths must be multiples of 16 bytes)";
    case SMOE_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case SMOE_ERR_HIP: return "HIP runtime error";
    case SMOE_ERR_TOO_LARGE: return "problem exceeds the fixed scratch capacity of a no-allocation entry point";
    default: return "unknown status";
  }
}

int smoe_create(smoe_ctx **out, int device) {
  if (!out) return SMOE_ERR_INVALID_ARG;
  *out = nullptr;
  int count = 0;
  if (hipGetDeviceCount(&count) != hipSuccess) return SMOE_ERR_HIP;
  if (device < 0 || device >= count) return SMOE_ERR_INVALID_ARG;
  hipDeviceProp_t prop;
  if (hipGetDeviceProperties(&prop, device) != hipSuccess) return SMOE_ERR_HIP;
  smoe_ctx *c = new (std::nothrow) smoe_ctx;
  if (!c) return SMOE_ERR_HIP;
  c->device = device;
  c->num_cu = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
  // persistent kernels: one block per compute unit, dealt to the XCDs in eight equal shares
  c->stream_grid = c->num_cu >= 256 ? 256 : (c->num_cu & ~7);
  c->kernel_mode = 0;
  c->group_m = 4;
  c->clock_probe = nullptr;
  c->route_scratch = nullptr;
  // kernel attributes and the address of a __device__ array are per device: set them with this context's device current, then restore the caller's
  int prev = -1;
  int rc = SMOE_ERR_HIP;
  if (hipGetDevice(&prev) == hipSuccess && hipSetDevice(device) == hipSuccess) {
    rc = init_stream_kernels();
    if (rc == SMOE_OK) rc = init_mfma_kernels();
    if (rc == SMOE_OK) rc = route_scratch_address(&c->route_scratch);
    if (hipSetDevice(prev) != hipSuccess && rc == SMOE_OK) rc = SMOE_ERR_HIP;
  }
  if (rc != SMOE_OK) {
    delete c;
    return rc;
  }
  *out = c;
  return SMOE_OK;
}

void smoe_destroy(smoe_ctx *ctx) { delete ctx; }

int smoe_set_kernel_mode(smoe_ctx *ctx, int mode) {
  if (!ctx || mode < 0 || mode > 2) return SMOE_ERR_INVALID_ARG;
  ctx->kernel_mode = mode;
  return SMOE_OK;
}

int smoe_set_tile_group(smoe_ctx *ctx, int group_m) {
  if (!ctx || group_m < 1 || group_m > 64) return SMOE_ERR_INVALID_ARG;
  ctx->group_m = group_m;
  return SMOE_OK;
}

int smoe_set_clock_probe(smoe_ctx *ctx, uint64_t *device_array) {
  if (!ctx) return SMOE_ERR_INVALID_ARG;
  ctx->clock_probe = (unsigned long long *)device_array;
  return SMOE_OK;
}

int smoe_topk_gate(smoe_ctx *ctx, void *stream, const float *logits, int T, int E, int k, int32_t *expert_idxs,
                   float *gates) {
  if (!ctx || T < 0 || E < 1 || k < 1 || k > E) return SMOE_ERR_INVALID_ARG;
  if (T == 0) return SMOE_OK;
  if (!logits || !expert_idxs || !gates) return SMOE_ERR_INVALID_ARG;
  if ((long long)T * k > 0x7fffffffLL) return SMOE_ERR_UNSUPPORTED;
  return launch_topk_gate((hipStream_t)stream, logits, T, E, k, expert_idxs, gates);
}

int smoe_topk_gate_bwd(smoe_ctx *ctx, void *stream, const int32_t *expert_idxs, const float *gates, const float *dgates,
                       int T, int E, int k, float *dlogits) {
  if (!ctx || T < 0 || E < 1 || k < 1 || k > E) return SMOE_ERR_INVALID_ARG;
  if (T == 0) return SMOE_OK;
  if (!expert_idxs || !gates || !dgates || !dlogits) return SMOE_ERR_INVALID_ARG;
  if ((long long)T * k > 0x7fffffffLL) return SMOE_ERR_UNSUPPORTED;
  return launch_topk_gate_bwd((hipStream_t)stream, expert_idxs, gates, dgates, T, E, k, dlogits);
}

static int attention_args_ok(smoe_dtype dtype, int B, int T, int G, int h, int d_head) {
  if (B < 1 || T < 1 || G < 1 || h < 1 || d_head < 1) return SMOE_ERR_INVALID_ARG;
  if (dtype != SMOE_BF16 || d_head != 128) return SMOE_ERR_UNSUPPORTED;
  if ((long long)T * G > 0x3fffffffLL || (long long)B * T * G > 0x7fffffffLL || h > 65535 || B > 65535)
    return SMOE_ERR_UNSUPPORTED;
  if ((((long long)T * G + 127) / 128) * h * B > 0x7fffffffLL) return SMOE_ERR_UNSUPPORTED;   // one-dimensional grids
  return SMOE_OK;
}

int smoe_attention_fwd(smoe_ctx *ctx, void *stream, smoe_dtype dtype, const void *Q, const void *K, const void *V, int B,
                       int T, int G, int h, int d_head, void *O, float *LSE) {
  if (!ctx || !Q || !K || !V || !O || !LSE) return SMOE_ERR_INVALID_ARG;
  int rc = attention_args_ok(dtype, B, T, G, h, d_head);
  if (rc != SMOE_OK) return rc;
  return launch_attn_fwd((hipStream_t)stream, Q, K, V, O, LSE, B, T, G, h);
}

size_t smoe_attention_bwd_workspace_bytes(int B, int T, int G, int h) {
  if (B < 1 || T < 1 || G < 1 || h < 1) return 0;
  return align256(attn_bwd_workspace_bytes(B, T, G, h));
}

int smoe_attention_bwd(smoe_ctx *ctx, void *stream, smoe_dtype dtype, const void *dO, const void *Q, const void *K,
                       const void *V, const void *O, const float *LSE, int B, int T, int G, int h, int d_head, void *dQ,
                       void *dK, void *dV, void *ws, size_t ws_bytes) {
  if (!ctx || !dO || !Q || !K || !V || !O || !LSE || !dQ || !dK || !dV) return SMOE_ERR_INVALID_ARG;
  int rc = attention_args_ok(dtype, B, T, G, h, d_head);
  if (rc != SMOE_OK) return rc;
  if (!ws || ((uintptr_t)ws & 255) || ws_bytes < smoe_attention_bwd_workspace_bytes(B, T, G, h)) return SMOE_ERR_WORKSPACE;
  return launch_attn_bwd((hipStream_t)stream, Q, K, V, O, dO, LSE, ws, dQ, dK, dV, B, T, G, h);
}

size_t smoe_route_workspace_bytes(int T, int k, int E) {
  if (T < 0 || k < 1 || E < 1) return 0;
  return route_workspace_bytes(T * k, E);
}

int smoe_route(smoe_ctx *ctx, void *stream, const int32_t *expert_idxs, int T, int k, int E,
               int32_t *sorted_expert_idxs, int32_t *sorted_scattered_idxs, int32_t *expert_offsets, void *ws,
               size_t ws_bytes) {
  if (!ctx || T < 0 || k < 1 || E < 1 || !expert_offsets) return SMOE_ERR_INVALID_ARG;
  if ((long long)T * k > 0x7fffffffLL || E > ROUTE_MAX_E) return SMOE_ERR_UNSUPPORTED;
  if (T > 0 && (!expert_idxs || !sorted_expert_idxs || !sorted_scattered_idxs)) return SMOE_ERR_INVALID_ARG;
  if (!ws || ((uintptr_t)ws & 255) || ws_bytes < route_workspace_bytes(T * k, E)) return SMOE_ERR_WORKSPACE;
  return launch_route((hipStream_t)stream, expert_idxs, T * k, E, sorted_expert_idxs, sorted_scattered_idxs,
                      expert_offsets, ws);
}

int smoe_route_noalloc(smoe_ctx *ctx, void *stream, const int32_t *expert_idxs, int T, int k, int E,
                       int32_t *sorted_expert_idxs, int32_t *sorted_scattered_idxs, int32_t *expert_offsets) {
  if (!ctx || T < 0 || k < 1 || E < 1 || !expert_offsets) return SMOE_ERR_INVALID_ARG;
  if ((long long)T * k > 0x7fffffffLL || E > ROUTE_MAX_E) return SMOE_ERR_UNSUPPORTED;
  if (T > 0 && (!expert_idxs || !sorted_expert_idxs || !sorted_scattered_idxs)) return SMOE_ERR_INVALID_ARG;
  if (route_workspace_bytes(T * k, E) > ROUTE_SCRATCH_BYTES) return SMOE_ERR_TOO_LARGE;
  if (!ctx->route_scratch) return SMOE_ERR_HIP;
  // Nothing in the scratch has to start at zero: the counting kernel writes every (expert, chunk) counter
  // before the scan reads it, and a one-chunk problem does not touch the scratch at all.
  return launch_route((hipStream_t)stream, expert_idxs, T * k, E, sorted_expert_idxs, sorted_scattered_idxs,
                      expert_offsets, ctx->route_scratch);
}

int smoe_group(smoe_ctx *ctx, void *stream, smoe_dtype dtype, const void *in, int d, const smoe_routing *r, int fan,
               const float *gates, void *out) {
  if (!ctx || !dtype_ok(dtype) || !routing_ok(r) || fan < 1 || d < 1) return SMOE_ERR_INVALID_ARG;
  if (r->Tk == 0) return SMOE_OK;
  if (!in || !out || r->Tk % fan) return SMOE_ERR_INVALID_ARG;
  if (!width_ok(dtype, d) || !aligned16(in) || !aligned16(out)) return SMOE_ERR_UNSUPPORTED;
  return launch_group((hipStream_t)stream, dtype, in, r->sorted_scattered_idxs, fan, gates, out, r->Tk, d);
}

// ------------------------------------------------------------------------------ Alg. 1
int smoe_plinear_fwd(smoe_ctx *ctx, void *stream, smoe_dtype dtype, const void *X, int x_rows, int d_in,
                     const void *W, int d_out, const smoe_routing *r, int k, const float *gates, int gates_k,
                     int grouped_in, int grouped_out, void *Yhat, void *Y) {
  if (!ctx || !dtype_ok(dtype) || !routing_ok(r) || d_in < 1 || d_out < 1 || k < 1 || x_rows < 0)
    return SMOE_ERR_INVALID_ARG;
  const int Tk = r->Tk;
  if (grouped_in ? (k != 1 || x_rows != Tk) : ((long long)x_rows * k != Tk)) return SMOE_ERR_INVALID_ARG;
  if (gates) {
    if (grouped_out || gates_k < 1 || Tk % gates_k || !Y) return SMOE_ERR_INVALID_ARG;
  } else if (Y) {
    return SMOE_ERR_INVALID_ARG;
  }
  if (Tk == 0) return SMOE_OK;
  if (!X || !W || !Yhat) return SMOE_ERR_INVALID_ARG;
  if (!width_ok(dtype, d_in) || !width_ok(dtype, d_out) || !aligned16(X) || !aligned16(W) || !aligned16(Yhat) ||
      (Y && !aligned16(Y)))
    return SMOE_ERR_UNSUPPORTED;
  hipStream_t s = (hipStream_t)stream;
  S2SArgs a = make_s2s(X, W, Yhat, r, d_in, d_out, false, grouped_in != 0, k, grouped_out != 0);
  int rc = run_s2s(ctx, s, dtype, a);
  if (rc != SMOE_OK) return rc;
  if (gates) rc = launch_combine(s, dtype, Yhat, gates, Y, Tk / gates_k, gates_k, d_out);
  return rc;
}

// ------------------------------------------------------------------------------ Alg. 2
// Workspace: [dYbar: Tk x d_out, when dY arrives scattered (weighted or not) -- Alg. 2's group(dY, o, p)]
//            [Xbar:  Tk x d_in, when X was scattered -- Alg. 2's group(X, o); the same array then
//                    receives dXbar, the reuse Sec. 3.2.1 points out]
static void plinear_bwd_layout(smoe_dtype dt, int d_in, int d_out, int Tk, int grouped_in, int grouped_out,
                               size_t &off_dybar, size_t &off_xbar, size_t &total) {
  size_t es = dtype_size(dt), off = 0;
  off_dybar = off_xbar = (size_t)-1;
  if (!grouped_out) { off_dybar = off; off += align256((size_t)Tk * d_out * es); }
  if (!grouped_in) { off_xbar = off; off += align256((size_t)Tk * d_in * es); }
  total = off + S2S_TAIL_WS_BYTES;   // fp32 partial tiles of the input-gradient product's split last round
}

size_t smoe_plinear_bwd_workspace_bytes(smoe_dtype dtype, int x_rows, int d_in, int d_out, int Tk, int k,
                                        int has_gates, int grouped_in, int grouped_out) {
  (void)x_rows; (void)k; (void)has_gates;
  if (!dtype_ok(dtype) || d_in < 1 || d_out < 1 || Tk < 0) return 0;
  size_t a, b, total;
  plinear_bwd_layout(dtype, d_in, d_out, Tk, grouped_in, grouped_out, a, b, total);
  return total;
}

int smoe_plinear_bwd(smoe_ctx *ctx, void *stream, smoe_dtype dtype, const void *dY, const void *X, int x_rows,
                     int d_in, const void *W, int d_out, const void *Yhat, const smoe_routing *r, int k,
                     const float *gates, int gates_k, int grouped_in, int grouped_out, void *dX, void *dW,
                     float *dgates, void *ws, size_t ws_bytes) {
  if (!ctx || !dtype_ok(dtype) || !routing_ok(r) || d_in < 1 || d_out < 1 || k < 1 || x_rows < 0)
    return SMOE_ERR_INVALID_ARG;
  const int Tk = r->Tk;
  if (grouped_in ? (k != 1 || x_rows != Tk) : ((long long)x_rows * k != Tk)) return SMOE_ERR_INVALID_ARG;
  if (gates && (grouped_out || gates_k < 1 || Tk % gates_k)) return SMOE_ERR_INVALID_ARG;
  if (!gates && dgates) return SMOE_ERR_INVALID_ARG;
  if (dgates && !Yhat) return SMOE_ERR_INVALID_ARG;
  if (!width_ok(dtype, d_in) || !width_ok(dtype, d_out)) return SMOE_ERR_UNSUPPORTED;
  if (!W && dX) return SMOE_ERR_INVALID_ARG;
  size_t off_dybar, off_xbar, need;
  plinear_bwd_layout(dtype, d_in, d_out, Tk, grouped_in, grouped_out, off_dybar, off_xbar, need);
  if (need && (!ws || ((uintptr_t)ws & 255) || ws_bytes < need)) return SMOE_ERR_WORKSPACE;
  hipStream_t s = (hipStream_t)stream;
  int rc = SMOE_OK;
  if (Tk == 0) {  // no routed rows: dW is all zeros, nothing else to write
    if (dW) {
      DWArgs z{nullptr, nullptr, dW, r->expert_offsets, r->E, 0, d_in, d_out};
      rc = launch_dw_plain(s, dtype, z);
    }
    return rc;
  }
  if (!dY || !X) return SMOE_ERR_INVALID_ARG;
  if (!aligned16(dY) || !aligned16(X) || (W && !aligned16(W)) || (dX && !aligned16(dX)) || (dW && !aligned16(dW)))
    return SMOE_ERR_UNSUPPORTED;

  // dp = bmm(dY, Yhat); dYbar = group(dY, o, p)  (Alg. 2: "weight and group")
  const void *dYbar = dY;
  if (!grouped_out) {
    if (gates && dgates) {
      rc = launch_rowdot(s, dtype, dY, Yhat, dgates, Tk, gates_k, d_out);
      if (rc != SMOE_OK) return rc;
    }
    void *buf = (char *)ws + off_dybar;
    rc = launch_group(s, dtype, dY, r->sorted_scattered_idxs, gates ? gates_k : 1, gates, buf, Tk, d_out);
    if (rc != SMOE_OK) return rc;
    dYbar = buf;
  }
  // Xbar = group(X, o);  dW = groupXTY(Xbar, dYbar)
  void *xbar = grouped_in ? nullptr : (void *)((char *)ws + off_xbar);
  if (dW) {
    const void *Xg = X;
    if (!grouped_in) {
      rc = launch_group(s, dtype, X, r->sorted_scattered_idxs, k, nullptr, xbar, Tk, d_in);
      if (rc != SMOE_OK) return rc;
      Xg = xbar;
    }
    DWArgs a{Xg, dYbar, dW, r->expert_offsets, r->E, Tk, d_in, d_out};
    a.split_ws = (float *)((char *)ws + need - S2S_TAIL_WS_BYTES);   // the input-gradient product below uses it afterwards
    rc = run_dw(ctx, s, dtype, a);
    if (rc != SMOE_OK) return rc;
  }
  // dXbar = scatter2scatter(dYbar, W^T, o, 1): grouped or scattered like the forward input;
  // with fan-out k the k slot gradients of a row are then summed.
  if (dX) {
    bool need_sum = !grouped_in && k > 1;
    void *dst = need_sum ? xbar : dX;   // Xbar is dead once dW is done
    S2SArgs a = make_s2s(dYbar, W, dst, r, d_in, d_out, true, true, 1, grouped_in != 0);
    a.tail_ws = (float *)((char *)ws + need - S2S_TAIL_WS_BYTES);
    rc = run_s2s(ctx, s, dtype, a);
    if (rc != SMOE_OK) return rc;
    if (need_sum) rc = launch_combine(s, dtype, dst, nullptr, dX, x_rows, k, d_in);
  }
  return rc;
}

// ------------------------------------------------------------------------------ Alg. 3
static inline int hidden_width(smoe_act act, int d_expert) { return act == SMOE_ACT_SWIGLU ? 2 * d_expert : d_expert; }

// Hpre = ParallelLinear(X, W1, scattered -> grouped);  H = sigma(Hpre)   (first two lines of Alg. 3).
// Hpre always points at room for the pre-activation; keep_hpre says whether the caller wants it written
// (when the activation is applied in the product's epilogue it is otherwise never stored).
static int hidden_forward(smoe_ctx *ctx, hipStream_t s, smoe_dtype dtype, smoe_act act, const void *X, int d_model,
                          int d_expert, const void *W1, const smoe_routing *r, int k, void *Hpre, bool keep_hpre, void *H,
                          float *tail_ws) {
  const int d_h = hidden_width(act, d_expert);
  S2SArgs a1 = make_s2s(X, W1, Hpre, r, d_model, d_h, false, false, k, true);
  a1.tail_ws = tail_ws;
  S2SArgs fused = a1;
  fused.H = H;
  fused.grid = ctx->stream_grid;
  fused.group_m = ctx->group_m;
  fused.clock_probe = ctx->clock_probe;
  if (act == SMOE_ACT_SWIGLU && dtype == SMOE_BF16 && ctx->kernel_mode == 0 &&
      (s2s_decode_supported(fused) || s2s_stream_swiglu_supported(fused))) {
    // SwiGLU in the product's epilogue: H comes straight from the fp32 accumulators, and the
    // pre-activation is written only when the caller keeps it for the backward pass
    if (!keep_hpre) fused.C = nullptr;
    return s2s_decode_supported(fused) ? launch_s2s_decode(s, fused) : launch_s2s_stream(s, fused);
  }
  int rc = run_s2s(ctx, s, dtype, a1);
  if (rc != SMOE_OK) return rc;
  return launch_act_fwd(s, dtype, act, Hpre, H, r->Tk, d_expert);
}

size_t smoe_plinear_act_fwd_workspace_bytes(smoe_dtype dtype, smoe_act act, int T, int k, int d_model, int d_expert,
                                            int keep_hpre) {
  if (!dtype_ok(dtype) || T < 0 || k < 1 || d_model < 1 || d_expert < 1) return 0;
  size_t hpre = keep_hpre ? 0 : align256((size_t)T * k * hidden_width(act, d_expert) * dtype_size(dtype));
  return hpre + S2S_TAIL_WS_BYTES;
}

int smoe_plinear_act_fwd(smoe_ctx *ctx, void *stream, smoe_dtype dtype, smoe_act act, const void *X, int T, int d_model,
                         int d_expert, const void *W1, const smoe_routing *r, int k, void *Hpre, void *H, void *ws,
                         size_t ws_bytes) {
  if (!ctx || !dtype_ok(dtype) || !routing_ok(r) || T < 0 || k < 1 || d_model < 1 || d_expert < 1)
    return SMOE_ERR_INVALID_ARG;
  if (act != SMOE_ACT_NONE && act != SMOE_ACT_GELU && act != SMOE_ACT_SWIGLU) return SMOE_ERR_INVALID_ARG;
  if ((long long)T * k != r->Tk) return SMOE_ERR_INVALID_ARG;
  if (T == 0) return SMOE_OK;
  if (!X || !W1 || !H) return SMOE_ERR_INVALID_ARG;
  if (!width_ok(dtype, d_model) || !width_ok(dtype, d_expert)) return SMOE_ERR_UNSUPPORTED;
  size_t need = smoe_plinear_act_fwd_workspace_bytes(dtype, act, T, k, d_model, d_expert, Hpre != nullptr);
  if (!ws || ((uintptr_t)ws & 255) || ws_bytes < need) return SMOE_ERR_WORKSPACE;
  float *tail_ws = (float *)((char *)ws + need - S2S_TAIL_WS_BYTES);
  void *pre = Hpre ? Hpre : ws;
  if (!aligned16(X) || !aligned16(W1) || !aligned16(H) || !aligned16(pre)) return SMOE_ERR_UNSUPPORTED;
  return hidden_forward(ctx, (hipStream_t)stream, dtype, act, X, d_model, d_expert, W1, r, k, pre, Hpre != nullptr, H, tail_ws);
}

size_t smoe_mlp_fwd_workspace_bytes(smoe_dtype dtype, smoe_act act, int T, int k, int d_model, int d_expert,
                                    int training) {
  if (!dtype_ok(dtype) || T < 0 || k < 1 || d_model < 1 || d_expert < 1) return 0;
  size_t es = dtype_size(dtype), Tk = (size_t)T * k;
  if (training == 1) return S2S_TAIL_WS_BYTES;
  if (training == 2) return align256(Tk * d_model * es) + S2S_TAIL_WS_BYTES;      // Hpre and H kept, Yhat lives here
  return align256(Tk * hidden_width(act, d_expert) * es) + align256(Tk * d_expert * es) +
         align256(Tk * d_model * es) + S2S_TAIL_WS_BYTES;
}

int smoe_mlp_fwd(smoe_ctx *ctx, void *stream, smoe_dtype dtype, smoe_act act, const void *X, int T, int d_model,
                 int d_expert, const void *W1, const void *W2, const smoe_routing *r, int k, const float *gates,
                 void *Y, void *saved_Hpre, void *saved_H, void *saved_Yhat, void *ws, size_t ws_bytes) {
  if (!ctx || !dtype_ok(dtype) || !routing_ok(r) || T < 0 || k < 1 || d_model < 1 || d_expert < 1)
    return SMOE_ERR_INVALID_ARG;
  if (act != SMOE_ACT_NONE && act != SMOE_ACT_GELU && act != SMOE_ACT_SWIGLU) return SMOE_ERR_INVALID_ARG;
  if ((long long)T * k != r->Tk) return SMOE_ERR_INVALID_ARG;
  const int nhid = (saved_Hpre != nullptr) + (saved_H != nullptr);
  if (nhid == 1 || (nhid == 0 && saved_Yhat)) return SMOE_ERR_INVALID_ARG;
  const int nsaved = nhid ? 3 : 0;                      // 3: training (Yhat may still live in the workspace)
  const int mode = nhid == 0 ? 0 : (saved_Yhat ? 1 : 2);
  if (T == 0) return SMOE_OK;
  if (!X || !W1 || !W2 || !gates || !Y) return SMOE_ERR_INVALID_ARG;
  const int d_h = hidden_width(act, d_expert), Tk = r->Tk;
  if (!width_ok(dtype, d_model) || !width_ok(dtype, d_expert)) return SMOE_ERR_UNSUPPORTED;
  size_t es = dtype_size(dtype);
  size_t need = smoe_mlp_fwd_workspace_bytes(dtype, act, T, k, d_model, d_expert, mode);
  if (!ws || ((uintptr_t)ws & 255) || ws_bytes < need) return SMOE_ERR_WORKSPACE;
  float *tail_ws = (float *)((char *)ws + need - S2S_TAIL_WS_BYTES);   // partial tiles of a split last round
  if (mode == 2) saved_Yhat = ws;
  if (nsaved == 0) {
    saved_Hpre = ws;
    saved_H = (char *)saved_Hpre + align256((size_t)Tk * d_h * es);
    saved_Yhat = (char *)saved_H + align256((size_t)Tk * d_expert * es);
  }
  if (!aligned16(X) || !aligned16(W1) || !aligned16(W2) || !aligned16(Y) || !aligned16(saved_Hpre) ||
      !aligned16(saved_H) || !aligned16(saved_Yhat))
    return SMOE_ERR_UNSUPPORTED;
  hipStream_t s = (hipStream_t)stream;
  int rc = hidden_forward(ctx, s, dtype, act, X, d_model, d_expert, W1, r, k, saved_Hpre, nsaved != 0, saved_H, tail_ws);
  if (rc != SMOE_OK) return rc;
  // Y = ParallelLinear(H, W2, p, grouped -> scattered)
  S2SArgs a2 = make_s2s(saved_H, W2, saved_Yhat, r, d_expert, d_model, false, true, 1, false);
  a2.tail_ws = tail_ws;
  rc = run_s2s(ctx, s, dtype, a2);
  if (rc != SMOE_OK) return rc;
  return launch_combine(s, dtype, saved_Yhat, gates, Y, T, k, d_model);
}

// Workspace of the backward pass: dYbar [Tk,d_model] (later reused for dXbar), dH [Tk,d_expert],
// dHpre [Tk,d_h].
// Backward passes that form dp in the epilogue of the W2^T product (bf16 through the persistent kernels).
// That product gathers the rows of dY itself; the one expert-sorted copy of dY [Tk,d_model] is for groupXTY (its array later
// holds Xbar, then dXbar).
//   mode 1 (SwiGLU): the activation's derivative is applied there too; scratch = the routing-weighted sorted copy of dY,
//     dHpre [Tk,d_h].
//   mode 2 (other activations): dp from the saved H; scratch = the weighted sorted copy of dY or, when d_expert < d_model
//     makes them the smaller tensor, the plain sorted copy plus the routing-weighted hidden rows Hw [Tk,d_expert] that let
//     groupXTY form dW2 from the plain copy; dH [Tk,d_expert]; dHpre [Tk,d_h].
//   both: the sorted routing weights [Tk] and the slabs of dp [Tk, 2 * ceil(d_expert / 256)] fp32.
struct MlpBwdEpiLayout {
  size_t dybar_u, second, dh, dhpre, gsorted, dp_part, total;
  int part_ld;
  bool use_hw;
};
static MlpBwdEpiLayout mlp_bwd_epi_layout(int mode, size_t es, size_t Tk, int d_model, int d_expert, int d_h) {
  MlpBwdEpiLayout L;
  size_t off = 0;
  L.part_ld = 2 * ceil_div(d_expert, 256);
  L.use_hw = mode == 2 && d_expert < d_model;
  L.dybar_u = off;  off += L.use_hw ? align256(Tk * d_model * es) : 0;
  L.second = off;   off += align256(Tk * (size_t)(L.use_hw ? d_expert : d_model) * es);
  L.dh = off;       off += mode == 2 ? align256(Tk * (size_t)d_expert * es) : 0;
  L.dhpre = off;    off += align256(Tk * (size_t)d_h * es);
  L.gsorted = off;  off += align256(Tk * sizeof(float));
  L.dp_part = off;  off += align256(Tk * (size_t)L.part_ld * sizeof(float));
  L.total = off + S2S_TAIL_WS_BYTES;
  return L;
}

size_t smoe_mlp_bwd_workspace_bytes(smoe_dtype dtype, smoe_act act, int T, int k, int d_model, int d_expert) {
  if (!dtype_ok(dtype) || T < 0 || k < 1 || d_model < 1 || d_expert < 1) return 0;
  size_t es = dtype_size(dtype), Tk = (size_t)T * k;
  const int d_h = hidden_width(act, d_expert);
  size_t plain = align256(Tk * d_model * es) + align256(Tk * d_expert * es) + align256(Tk * d_h * es) + S2S_TAIL_WS_BYTES;
  if (dtype != SMOE_BF16) return plain;
  size_t epi = mlp_bwd_epi_layout(act == SMOE_ACT_SWIGLU ? 1 : 2, es, Tk, d_model, d_expert, d_h).total;
  return epi > plain ? epi : plain;   // whichever path the shape takes fits
}

// How the backward pass of this shape runs: 0 = Alg. 2 step by step (dp from the forward's saved Yhat), 1 / 2 = dp in the
// epilogue of the W2^T product as described above (the forward's unweighted Yhat is then not needed).
static int mlp_bwd_mode(const smoe_ctx *ctx, smoe_dtype dtype, smoe_act act, int Tk, int k, int E, int d_model, int d_expert) {
  if (dtype != SMOE_BF16 || ctx->kernel_mode != 0 || Tk < 1) return 0;
  S2SArgs x;
  x.A = x.W = nullptr;  x.C = nullptr;
  x.a_map = RowMap{(const int32_t *)1, k};  x.c_map = RowMap{nullptr, 1};   // the product gathers the rows of dY [T, d_model]
  x.offsets = nullptr;  x.E = E;  x.Tk = Tk;
  x.K = d_model;  x.N = d_expert;  x.ldw = d_model;  x.w_stride = (size_t)d_expert * d_model;  x.trans_w = 1;
  x.tail_ws = nullptr;  x.H = nullptr;
  x.grid = ctx->stream_grid;
  x.row_scale = (const float *)1;  x.dp_part = (float *)1;   // only tested for presence
  if (act == SMOE_ACT_SWIGLU) {
    x.Hpre_in = (const void *)1;
    return s2s_stream_swiglu_bwd_supported(x) ? 1 : 0;
  }
  x.H_in = (const void *)1;
  return s2s_stream_dp_supported(x) ? 2 : 0;
}

int smoe_mlp_saves_yhat(smoe_ctx *ctx, smoe_dtype dtype, smoe_act act, int T, int k, int E, int d_model, int d_expert) {
  if (!ctx || !dtype_ok(dtype) || T < 0 || k < 1 || E < 1 || d_model < 1 || d_expert < 1) return SMOE_ERR_INVALID_ARG;
  return mlp_bwd_mode(ctx, dtype, act, T * k, k, E, d_model, d_expert) ? 0 : 1;
}

int smoe_mlp_bwd(smoe_ctx *ctx, void *stream, smoe_dtype dtype, smoe_act act, const void *dY, const void *X, int T,
                 int d_model, int d_expert, const void *W1, const void *W2, const smoe_routing *r, int k,
                 const float *gates, const void *saved_Hpre, const void *saved_H, const void *saved_Yhat, void *dX,
                 void *dW1, void *dW2, float *dgates, void *ws, size_t ws_bytes) {
  if (!ctx || !dtype_ok(dtype) || !routing_ok(r) || T < 0 || k < 1 || d_model < 1 || d_expert < 1)
    return SMOE_ERR_INVALID_ARG;
  if (act != SMOE_ACT_NONE && act != SMOE_ACT_GELU && act != SMOE_ACT_SWIGLU) return SMOE_ERR_INVALID_ARG;
  if ((long long)T * k != r->Tk) return SMOE_ERR_INVALID_ARG;
  if (!dW1 || !dW2) return SMOE_ERR_INVALID_ARG;
  if (!width_ok(dtype, d_model) || !width_ok(dtype, d_expert)) return SMOE_ERR_UNSUPPORTED;
  const int d_h = hidden_width(act, d_expert), Tk = r->Tk;
  size_t es = dtype_size(dtype);
  size_t need = smoe_mlp_bwd_workspace_bytes(dtype, act, T, k, d_model, d_expert);
  if (need && (!ws || ((uintptr_t)ws & 255) || ws_bytes < need)) return SMOE_ERR_WORKSPACE;
  hipStream_t s = (hipStream_t)stream;
  int rc;
  if (T == 0) {
    DWArgs z1{nullptr, nullptr, dW1, r->expert_offsets, r->E, 0, d_model, d_h};
    rc = launch_dw_plain(s, dtype, z1);
    if (rc != SMOE_OK) return rc;
    DWArgs z2{nullptr, nullptr, dW2, r->expert_offsets, r->E, 0, d_expert, d_model};
    return launch_dw_plain(s, dtype, z2);
  }
  const int mode = mlp_bwd_mode(ctx, dtype, act, Tk, k, r->E, d_model, d_expert);
  if (!dY || !X || !W1 || !W2 || !gates || !saved_Hpre || !saved_H || (!saved_Yhat && !mode) || !dX || !dgates)
    return SMOE_ERR_INVALID_ARG;
  if (!aligned16(dY) || !aligned16(X) || !aligned16(W1) || !aligned16(W2) || !aligned16(saved_Hpre) ||
      !aligned16(saved_H) || (saved_Yhat && !aligned16(saved_Yhat)) || !aligned16(dX) || !aligned16(dW1) || !aligned16(dW2))
    return SMOE_ERR_UNSUPPORTED;
  if (mode) {
    // Alg. 2 for both ParallelLinears with dp taken in the epilogue of the W2^T product: that product runs on the
    // UNWEIGHTED sorted copy of dY, so its fp32 accumulators are dH / p and dp[row] = <acc, H[row]> needs neither the
    // forward's Yhat nor a division by a routing weight.
    const MlpBwdEpiLayout L = mlp_bwd_epi_layout(mode, es, (size_t)Tk, d_model, d_expert, d_h);
    char *base = (char *)ws;
    void *dYu = base + L.dybar_u, *second = base + L.second, *dH = base + L.dh, *dHpre = base + L.dhpre;
    float *gsorted = (float *)(base + L.gsorted), *dp_part = (float *)(base + L.dp_part);
    float *tail_ws = (float *)(base + L.total - S2S_TAIL_WS_BYTES);
    // The W2^T product gathers the rows of dY itself (Alg. 1's scattered input, fan-out k); groupXTY needs sorted rows, so
    // one sorted copy is made for it: the routing-weighted one, or the plain one when the weights go into Hw instead.
    rc = launch_group(s, dtype, dY, r->sorted_scattered_idxs, k, L.use_hw ? nullptr : gates, L.use_hw ? dYu : second, Tk, d_model);
    if (rc != SMOE_OK) return rc;
    rc = launch_sorted_weights(s, r->sorted_scattered_idxs, gates, gsorted, Tk);
    if (rc != SMOE_OK) return rc;
    S2SArgs x2 = make_s2s(dY, W2, mode == 1 ? dHpre : dH, r, d_expert, d_model, true, false, k, true);
    if (mode == 1) {
      x2.Hpre_in = saved_Hpre;           // dHpre = sigma'(Hpre) p (dYu W2^T) straight from the accumulators
    } else {
      x2.H_in = saved_H;                 // dH = p (dYu W2^T), Hw = p H
      x2.Hw_out = L.use_hw ? second : nullptr;
    }
    x2.row_scale = gsorted;
    x2.dp_part = dp_part;
    x2.grid = ctx->stream_grid;
    x2.group_m = ctx->group_m;
    x2.clock_probe = ctx->clock_probe;
    rc = launch_s2s_stream(s, x2);
    if (rc != SMOE_OK) return rc;
    rc = launch_dp_reduce(s, dp_part, L.part_ld, r->sorted_scattered_idxs, dgates, Tk);
    if (rc != SMOE_OK) return rc;
    if (mode == 2) {
      rc = launch_act_bwd(s, dtype, act, saved_Hpre, dH, dHpre, Tk, d_expert);
      if (rc != SMOE_OK) return rc;
    }
    DWArgs w2{L.use_hw ? (const void *)second : saved_H, L.use_hw ? (const void *)dYu : (const void *)second, dW2,
              r->expert_offsets, r->E, Tk, d_expert, d_model};
    w2.split_ws = tail_ws;
    rc = run_dw(ctx, s, dtype, w2);
    if (rc != SMOE_OK) return rc;
    void *Xbar = L.use_hw ? dYu : second;                // the sorted copy of dY is dead: its array holds Xbar, then dXbar
    rc = launch_group(s, dtype, X, r->sorted_scattered_idxs, k, nullptr, Xbar, Tk, d_model);
    if (rc != SMOE_OK) return rc;
    DWArgs w1{Xbar, dHpre, dW1, r->expert_offsets, r->E, Tk, d_model, d_h};
    w1.split_ws = tail_ws;
    rc = run_dw(ctx, s, dtype, w1);
    if (rc != SMOE_OK) return rc;
    S2SArgs x1 = make_s2s(dHpre, W1, k == 1 ? dX : Xbar, r, d_model, d_h, true, true, 1, false);
    x1.tail_ws = tail_ws;
    rc = run_s2s(ctx, s, dtype, x1);
    if (rc != SMOE_OK || k == 1) return rc;
    return launch_combine(s, dtype, Xbar, nullptr, dX, T, k, d_model);
  }
  char *p = (char *)ws;
  void *dYbar = p;                 p += align256((size_t)Tk * d_model * es);
  void *dH = p;                    p += align256((size_t)Tk * d_expert * es);
  void *dHpre = p;
  float *tail_ws = (float *)((char *)ws + need - S2S_TAIL_WS_BYTES);   // partial tiles of a split last round
  void *Xbar = dYbar;  // dYbar is dead once dH and dW2 are done; its array then holds Xbar, then dXbar

  // ---- second ParallelLinear (grouped in, scattered weighted out)
  rc = launch_rowdot(s, dtype, dY, saved_Yhat, dgates, Tk, k, d_model);                 // dp = bmm(dY, Yhat)
  if (rc != SMOE_OK) return rc;
  rc = launch_group(s, dtype, dY, r->sorted_scattered_idxs, k, gates, dYbar, Tk, d_model);  // weight and group
  if (rc != SMOE_OK) return rc;
  DWArgs w2{saved_H, dYbar, dW2, r->expert_offsets, r->E, Tk, d_expert, d_model};
  w2.split_ws = tail_ws;
  rc = run_dw(ctx, s, dtype, w2);                                                      // groupXTY
  if (rc != SMOE_OK) return rc;
  S2SArgs x2 = make_s2s(dYbar, W2, dH, r, d_expert, d_model, true, true, 1, true);      // dH = dYbar W2^T
  x2.tail_ws = tail_ws;
  rc = run_s2s(ctx, s, dtype, x2);
  if (rc != SMOE_OK) return rc;
  // ---- activation
  rc = launch_act_bwd(s, dtype, act, saved_Hpre, dH, dHpre, Tk, d_expert);
  if (rc != SMOE_OK) return rc;
  // ---- first ParallelLinear (scattered in with fan-out k, grouped out): its one `group`
  rc = launch_group(s, dtype, X, r->sorted_scattered_idxs, k, nullptr, Xbar, Tk, d_model);
  if (rc != SMOE_OK) return rc;
  DWArgs w1{Xbar, dHpre, dW1, r->expert_offsets, r->E, Tk, d_model, d_h};
  w1.split_ws = tail_ws;
  rc = run_dw(ctx, s, dtype, w1);
  if (rc != SMOE_OK) return rc;
  if (k == 1) {  // slot id == token id: scatter straight into dX
    S2SArgs x1 = make_s2s(dHpre, W1, dX, r, d_model, d_h, true, true, 1, false);
    x1.tail_ws = tail_ws;
    return run_s2s(ctx, s, dtype, x1);
  }
  S2SArgs x1 = make_s2s(dHpre, W1, Xbar, r, d_model, d_h, true, true, 1, false);        // grouped -> scattered dXbar
  x1.tail_ws = tail_ws;
  rc = run_s2s(ctx, s, dtype, x1);
  if (rc != SMOE_OK) return rc;
  return launch_combine(s, dtype, Xbar, nullptr, dX, T, k, d_model);                    // sum the k slots
}

// ------------------------------------------------------------------------------ Alg. 4
namespace {
struct MomhaSizes {
  size_t kv, q, lse, yhat, x;   // bytes, each rounded up to 256
};
MomhaSizes momha_sizes(int B, int T, int k, int d_model, int h_expert, int d_head) {
  size_t N = (size_t)B * T, Tk = N * k, d_out = (size_t)h_expert * d_head;
  return MomhaSizes{align256(N * d_out * 2), align256(Tk * d_out * 2), align256(Tk * h_expert * sizeof(float)),
                    align256(Tk * d_model * 2), align256(N * d_model * 2)};
}
int momha_args_ok(smoe_ctx *ctx, smoe_dtype dtype, int B, int T, int d_model, int h_expert, int d_head,
                  const smoe_routing *r, int k) {
  if (!ctx || !routing_ok(r) || d_model < 1 || k < 1) return SMOE_ERR_INVALID_ARG;
  int rc = attention_args_ok(dtype, B, T, k, h_expert, d_head);
  if (rc != SMOE_OK) return rc;
  if ((long long)B * T * k != r->Tk) return SMOE_ERR_INVALID_ARG;
  if (!width_ok(dtype, d_model)) return SMOE_ERR_UNSUPPORTED;
  return SMOE_OK;
}
// a dense product A [n, d_in] x W (or W^T) run through the grouped kernels as one expert
S2SArgs dense_s2s(const void *A, const void *W, void *C, const int32_t *offsets, int n, int d_in, int d_out, bool trans_w) {
  smoe_routing r{nullptr, nullptr, offsets, n, 1};
  return make_s2s(A, W, C, &r, d_in, d_out, trans_w, true, 1, true);
}
}  // namespace

size_t smoe_momha_fwd_workspace_bytes(int B, int T, int k, int d_model, int h_expert, int d_head, int training) {
  if (B < 1 || T < 1 || k < 1 || d_model < 1 || h_expert < 1 || d_head < 1) return 0;
  MomhaSizes z = momha_sizes(B, T, k, d_model, h_expert, d_head);
  return 256 + S2S_TAIL_WS_BYTES + (training ? 0 : 2 * z.kv + 2 * z.q + z.lse + z.yhat);
}

int smoe_momha_fwd(smoe_ctx *ctx, void *stream, smoe_dtype dtype, const void *X, int B, int T, int d_model,
                   int h_expert, int d_head, const void *W_K, const void *W_V, const void *W_Q, const void *W_O,
                   const smoe_routing *r, int k, const float *gates, void *O, void *saved_K, void *saved_V,
                   void *saved_Q, void *saved_Ohat, float *saved_LSE, void *saved_Yhat, void *ws, size_t ws_bytes) {
  int rc = momha_args_ok(ctx, dtype, B, T, d_model, h_expert, d_head, r, k);
  if (rc != SMOE_OK) return rc;
  if (!X || !W_K || !W_V || !W_Q || !W_O || !gates || !O) return SMOE_ERR_INVALID_ARG;
  const int n_saved = !!saved_K + !!saved_V + !!saved_Q + !!saved_Ohat + !!saved_LSE + !!saved_Yhat;
  if (n_saved != 0 && n_saved != 6) return SMOE_ERR_INVALID_ARG;
  size_t need = smoe_momha_fwd_workspace_bytes(B, T, k, d_model, h_expert, d_head, n_saved == 6);
  if (!ws || ((uintptr_t)ws & 255) || ws_bytes < need) return SMOE_ERR_WORKSPACE;
  const int N = B * T, Tk = r->Tk, d_out = h_expert * d_head;
  MomhaSizes z = momha_sizes(B, T, k, d_model, h_expert, d_head);
  char *p = (char *)ws;
  int32_t *dense_off = (int32_t *)p;  p += 256;
  float *tail_ws = (float *)p;  p += S2S_TAIL_WS_BYTES;
  if (n_saved == 0) {
    saved_K = p;  p += z.kv;
    saved_V = p;  p += z.kv;
    saved_Q = p;  p += z.q;
    saved_Ohat = p;  p += z.q;
    saved_LSE = (float *)p;  p += z.lse;
    saved_Yhat = p;
  }
  hipStream_t s = (hipStream_t)stream;
  rc = launch_dense_offsets(s, dense_off, N);
  if (rc != SMOE_OK) return rc;
  // V = X W_V, K = X W_K
  auto product = [&](S2SArgs a) { a.tail_ws = tail_ws; return run_s2s(ctx, s, dtype, a); };
  rc = product(dense_s2s(X, W_V, saved_V, dense_off, N, d_model, d_out, false));
  if (rc != SMOE_OK) return rc;
  rc = product(dense_s2s(X, W_K, saved_K, dense_off, N, d_model, d_out, false));
  if (rc != SMOE_OK) return rc;
  // Q = ParallelLinear(X, W_Q, o, no p, scattered -> scattered)
  rc = product(make_s2s(X, W_Q, saved_Q, r, d_model, d_out, false, false, k, false));
  if (rc != SMOE_OK) return rc;
  // Ohat = Attention(Q, K, V)
  rc = launch_attn_fwd(s, saved_Q, saved_K, saved_V, saved_Ohat, saved_LSE, B, T, k, h_expert);
  if (rc != SMOE_OK) return rc;
  // O = ParallelLinear(Ohat, W_O, o, p, scattered -> scattered)
  rc = product(make_s2s(saved_Ohat, W_O, saved_Yhat, r, d_out, d_model, false, false, 1, false));
  if (rc != SMOE_OK) return rc;
  return launch_combine(s, dtype, saved_Yhat, gates, O, N, k, d_model);
}

size_t smoe_momha_bwd_workspace_bytes(int B, int T, int k, int d_model, int h_expert, int d_head) {
  if (B < 1 || T < 1 || k < 1 || d_model < 1 || h_expert < 1 || d_head < 1) return 0;
  MomhaSizes z = momha_sizes(B, T, k, d_model, h_expert, d_head);
  // dense offsets, dOhat, dQ, dK, dV, three partial dX, delta, and the ParallelLinear backward scratch
  // (a grouped [Tk, d_model] and a grouped [Tk, d_out] array, used by both projections in turn)
  return 256 + 2 * z.q + 2 * z.kv + 3 * z.x + smoe_attention_bwd_workspace_bytes(B, T, k, h_expert) + z.yhat + z.q +
         S2S_TAIL_WS_BYTES;
}

int smoe_momha_bwd(smoe_ctx *ctx, void *stream, smoe_dtype dtype, const void *dO, const void *X, int B, int T,
                   int d_model, int h_expert, int d_head, const void *W_K, const void *W_V, const void *W_Q,
                   const void *W_O, const smoe_routing *r, int k, const float *gates, const void *saved_K,
                   const void *saved_V, const void *saved_Q, const void *saved_Ohat, const float *saved_LSE,
                   const void *saved_Yhat, void *dX, void *dW_K, void *dW_V, void *dW_Q, void *dW_O, float *dgates,
                   void *ws, size_t ws_bytes) {
  int rc = momha_args_ok(ctx, dtype, B, T, d_model, h_expert, d_head, r, k);
  if (rc != SMOE_OK) return rc;
  if (!dO || !X || !W_K || !W_V || !W_Q || !W_O || !gates || !saved_K || !saved_V || !saved_Q || !saved_Ohat ||
      !saved_LSE || !saved_Yhat || !dX || !dW_K || !dW_V || !dW_Q || !dW_O || !dgates)
    return SMOE_ERR_INVALID_ARG;
  size_t need = smoe_momha_bwd_workspace_bytes(B, T, k, d_model, h_expert, d_head);
  if (!ws || ((uintptr_t)ws & 255) || ws_bytes < need) return SMOE_ERR_WORKSPACE;
  const int N = B * T, Tk = r->Tk, d_out = h_expert * d_head;
  MomhaSizes z = momha_sizes(B, T, k, d_model, h_expert, d_head);
  char *p = (char *)ws;
  int32_t *dense_off = (int32_t *)p;  p += 256;
  void *dOhat = p;  p += z.q;
  void *dQ = p;     p += z.q;
  void *dK = p;     p += z.kv;
  void *dV = p;     p += z.kv;
  void *dXq = p;    p += z.x;
  void *dXk = p;    p += z.x;
  void *dXv = p;    p += z.x;
  void *attn_ws = p;  p += smoe_attention_bwd_workspace_bytes(B, T, k, h_expert);
  void *sub = p;
  const size_t sub_bytes = z.yhat + z.q + S2S_TAIL_WS_BYTES;
  float *tail_ws = (float *)((char *)sub + z.yhat + z.q);   // where the ParallelLinear backward puts its own, too
  hipStream_t s = (hipStream_t)stream;
  rc = launch_dense_offsets(s, dense_off, N);
  if (rc != SMOE_OK) return rc;
  // output projection (Alg. 2 with p, scattered in with fan-out 1, scattered out): dOhat, dW_O, dp
  rc = smoe_plinear_bwd(ctx, stream, dtype, dO, saved_Ohat, Tk, d_out, W_O, d_model, saved_Yhat, r, 1, gates, k, 0, 0,
                        dOhat, dW_O, dgates, sub, sub_bytes);
  if (rc != SMOE_OK) return rc;
  rc = launch_attn_bwd(s, saved_Q, saved_K, saved_V, saved_Ohat, dOhat, saved_LSE, attn_ws, dQ, dK, dV, B, T, k, h_expert);
  if (rc != SMOE_OK) return rc;
  // query projection (Alg. 2 without p, scattered in with fan-out k, scattered out): dX part, dW_Q
  rc = smoe_plinear_bwd(ctx, stream, dtype, dQ, X, N, d_model, W_Q, d_out, nullptr, r, k, nullptr, 0, 0, 0, dXq, dW_Q,
                        nullptr, sub, sub_bytes);
  if (rc != SMOE_OK) return rc;
  // dense key / value projections
  DWArgs wk{X, dK, dW_K, dense_off, 1, N, d_model, d_out}, wv{X, dV, dW_V, dense_off, 1, N, d_model, d_out};
  wk.split_ws = wv.split_ws = (float *)((char *)sub + z.yhat + z.q);
  rc = run_dw(ctx, s, dtype, wk);
  if (rc != SMOE_OK) return rc;
  rc = run_dw(ctx, s, dtype, wv);
  if (rc != SMOE_OK) return rc;
  S2SArgs xk = dense_s2s(dK, W_K, dXk, dense_off, N, d_model, d_out, true);
  S2SArgs xv = dense_s2s(dV, W_V, dXv, dense_off, N, d_model, d_out, true);
  xk.tail_ws = xv.tail_ws = tail_ws;
  rc = run_s2s(ctx, s, dtype, xk);
  if (rc != SMOE_OK) return rc;
  rc = run_s2s(ctx, s, dtype, xv);
  if (rc != SMOE_OK) return rc;
  return launch_add3(s, dXq, dXk, dXv, dX, (size_t)N * d_model);
}

}  // extern "C"
