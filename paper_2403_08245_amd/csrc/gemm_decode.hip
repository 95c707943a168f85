// scatter2scatter for the decoding regime (Sec. 5 names it as the open case): a few rows per
// expert, so the product is a stream of every used expert's weights past a handful of rows and
// the only thing that matters is keeping HBM busy.
//
// One wavefront per block owns a 32-row x 128-column output tile of one expert and walks the whole
// contraction by itself: no barrier anywhere, a private four-stage LDS ring filled by
// direct-to-LDS loads (three stages = 30 KB in flight per wavefront, four wavefronts per compute
// unit), and two matrix instructions per fragment per stage on whatever rows the tile has.  The
// matrix cores idle most of the time by design; a 256-row tile would spend eight times the matrix
// and LDS work per weight byte on padding rows, which is what bounds the large-tile kernels here.
// Forward products only (W as stored); the gradients of such small batches use the large-tile kernels.
#include "mfma_common.h"

namespace {

constexpr int DM = 32;                        // rows of a tile
constexpr int DN = 128;                       // columns of a tile
constexpr int DST = 4;                        // LDS stages of a wavefront
constexpr int DW_BYTES = HK * DN * 2;         // W part of a stage: 32 contraction rows x 256 B
constexpr int DA_BYTES = DM * HK * 2;         // A part of a stage: 32 rows x 64 B
constexpr int DSTAGE_BYTES = DW_BYTES + DA_BYTES;
constexpr int NLW = DW_BYTES / 1024;          // load instructions per stage (1 KB per instruction)
constexpr int NLA = DA_BYTES / 1024;
constexpr int NLOADS = NLW + NLA;
constexpr int DECODE_LDS_BYTES = DST * DSTAGE_BYTES;
static_assert((DST - 1) * NLOADS < 64, "the load counter has six bits");

__device__ __forceinline__ int dw_swz(int krow) { return (krow & 3) << 2; }
// fragment of the W part (32 x 128, columns contiguous): lane holds column cbase + lane%32 and the
// contraction rows kk*16 + 8*(lane/32) + 0..7, gathered by two transposing reads
__device__ __forceinline__ bf16x8 dw_frag(const char *tile, int cbase, int kk, int lane) {
  int col = cbase + 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
  int row0 = kk * 16 + 8 * (lane >> 5) + ((lane & 15) >> 2);
  union { bf16x8 v; s16x4 h[2]; } u;
#pragma unroll
  for (int t = 0; t < 2; ++t) {
    int row = row0 + 4 * t;
    int off = row * (DN * 2) + (((col >> 3) ^ dw_swz(row)) << 4) + ((col & 7) << 1);
    u.h[t] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS s16x4 *)(tile + off));
  }
  return u.v;
}

// ACT 0: C = A W.  ACT 1 / 2: fused SwiGLU (a tile is 64 gate columns and the 64 up columns pairing with
// them), keeping / not keeping the pre-activation.
template <int ACT, bool SCATTER_OUT>
__global__ void __launch_bounds__(64) s2s_decode_kernel(S2SArgs a, int n_chunks) {
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  const int lane = threadIdx.x;
  const int mt = (int)blockIdx.x / n_chunks, nc = (int)blockIdx.x - mt * n_chunks;
  int e, row0, row_end;
  if (!locate_rows<DM>(a.offsets, a.E, mt, lane, e, row0, row_end)) return;   // grid is an upper bound
  e = __builtin_amdgcn_readfirstlane(e);
  const int half_n = a.N / 2;
  const int n0 = nc * (ACT ? DN / 2 : DN);           // first (gate) column of the tile
  const int nh = a.K / HK;
  const bf16_t *A = (const bf16_t *)a.A;
  const bf16_t *W = (const bf16_t *)a.W + (size_t)e * a.w_stride;

  // per-lane sources at contraction offset 0
  const bf16_t *pw[NLW], *pa[NLA];
#pragma unroll
  for (int I = 0; I < NLW; ++I) {
    const int krow = I * 4 + (lane >> 4);
    const int c = (lane & 15) ^ dw_swz(krow);         // source chunk (8 columns) landing at LDS position lane%16
    int col;
    if (ACT) {
      const int gate = n0 + (c & 7) * 8;
      col = gate < half_n ? gate + (c >> 3) * half_n : 0;
    } else {
      col = n0 + c * 8;
      if (col >= a.N) col = 0;
    }
    pw[I] = W + (size_t)krow * a.ldw + col;
  }
#pragma unroll
  for (int I = 0; I < NLA; ++I) {
    const int r = I * 16 + (lane >> 2);
    const int i = min(row0 + r, row_end - 1);         // rows past the segment repeat its last row
    const int src = a.a_map.o ? a.a_map.o[i] / a.a_map.fan : i;
    pa[I] = A + (size_t)src * a.K + (((lane & 3) ^ kc_swz(r)) << 3);
  }
  const size_t w_step = (size_t)HK * a.ldw;

  const uint32_t lds0 = __builtin_amdgcn_readfirstlane(lds_address(smem));
  auto issue = [&](int step, int slot) {
    const int st = min(step, nh - 1);                 // steps past the end repeat the last one (never read)
    const uint32_t lds = lds0 + (uint32_t)slot * DSTAGE_BYTES;
#pragma unroll
    for (int I = 0; I < NLW; ++I) load16_to_lds(pw[I] + (size_t)st * w_step, lds + I * 1024);
#pragma unroll
    for (int I = 0; I < NLA; ++I) load16_to_lds(pa[I] + (size_t)st * HK, lds + DW_BYTES + I * 1024);
  };

  f32x16 acc[4];
#pragma unroll
  for (int f = 0; f < 4; ++f)
#pragma unroll
    for (int q = 0; q < 16; ++q) acc[f][q] = 0.f;

#pragma unroll 1
  for (int s = 0; s < DST - 1; ++s) issue(s, s);
#pragma unroll 1
  for (int s = 0; s < nh; ++s) {
    // refills the stage read one step ago (its fragments went into matrix instructions already issued)
    issue(s + DST - 1, (s + DST - 1) % DST);
    wait_loads<(DST - 1) * NLOADS>();                 // stage s has landed
    const char *tile = smem + (s % DST) * DSTAGE_BYTES;
#pragma unroll
    for (int kk = 0; kk < 2; ++kk) {
      const bf16x8 fa = kc_frag(tile + DW_BYTES, 0, kk, lane);
#pragma unroll
      for (int f = 0; f < 4; ++f)
        acc[f] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(dw_frag(tile, f * 32, kk, lane), fa, acc[f], 0, 0, 0);
    }
  }
  wait_loads<0>();

  // a lane holds row lane%32 and, per fragment f and group g, the four columns f*32 + 8g + 4*(lane/32) + 0..3
  const int i = row0 + (lane & 31);
  if (i >= row_end) return;
  const size_t dst = SCATTER_OUT ? (size_t)a.c_map.o[i] : (size_t)i;
  if (ACT == 0) {
    bf16_t *C = (bf16_t *)a.C + dst * a.N;
#pragma unroll
    for (int f = 0; f < 4; ++f)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int col = n0 + f * 32 + 8 * g + 4 * (lane >> 5);
        if (col < a.N) {
          bf16x4 v;
#pragma unroll
          for (int q = 0; q < 4; ++q) v[q] = (bf16_t)acc[f][4 * g + q];
          *reinterpret_cast<bf16x4 *>(C + col) = v;
        }
      }
  } else {
    bf16_t *Hpre = ACT == 1 ? (bf16_t *)a.C + dst * a.N : nullptr;
    bf16_t *H = (bf16_t *)a.H + dst * half_n;
#pragma unroll
    for (int f = 0; f < 2; ++f)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int col = n0 + f * 32 + 8 * g + 4 * (lane >> 5);   // hidden unit = gate column
        if (col < half_n) {
          bf16x4 vg, vu, vh;
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const float gate = acc[f][4 * g + q], up = acc[2 + f][4 * g + q];
            const float sig = __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.4426950408889634f * gate));
            vg[q] = (bf16_t)gate;
            vu[q] = (bf16_t)up;
            vh[q] = (bf16_t)(gate * sig * up);
          }
          if (ACT == 1) {
            *reinterpret_cast<bf16x4 *>(Hpre + col) = vg;
            *reinterpret_cast<bf16x4 *>(Hpre + half_n + col) = vu;
          }
          *reinterpret_cast<bf16x4 *>(H + col) = vh;
        }
      }
  }
}

template <int ACT, bool SCATTER_OUT> int launch_decode(hipStream_t s, const S2SArgs &a) {
  const int n_chunks = ACT ? ceil_div(a.N / 2, DN / 2) : ceil_div(a.N, DN);
  const long long m_bound = a.Tk / DM + a.E;           // >= sum_e ceil(n_e / 32)
  hipLaunchKernelGGL((s2s_decode_kernel<ACT, SCATTER_OUT>), dim3((unsigned)(m_bound * n_chunks)), dim3(64), DECODE_LDS_BYTES, s, a,
                     n_chunks);
  SMOE_LAUNCH_CHECK();
  return SMOE_OK;
}

}  // namespace

// The decoding regime: on average at most one 32-row tile per expert.  Gathered or expert-sorted input,
// W as stored, any output order; widths as the 16-byte loads and 8-byte stores need them.
bool s2s_decode_supported(const S2SArgs &a) {
  if (a.trans_w || a.Tk <= 0 || a.E < 1 || (long long)a.Tk > (long long)DM * a.E) return false;
  if (a.K < HK || a.K % HK || a.N % 8) return false;
  if (a.H && (a.N % 16 || a.c_map.o)) return false;
  const long long blocks = ((long long)a.Tk / DM + a.E) * ceil_div(a.N, DN / 2);
  return blocks < 0x7fffffffLL;
}

int launch_s2s_decode(hipStream_t s, const S2SArgs &a) {
  if (!s2s_decode_supported(a)) return SMOE_ERR_UNSUPPORTED;
  if (a.H) return a.C ? launch_decode<1, false>(s, a) : launch_decode<2, false>(s, a);
  return a.c_map.o ? launch_decode<0, true>(s, a) : launch_decode<0, false>(s, a);
}
