// Dense projections for 17..96 activation rows on the matrix cores, bf16 weights:
//     Y[m][n] (op)= sum_k X'[m][k] * W[n][k],   X' = X (+ X2) or rmsnorm(X (+ X2)) * norm_w.
// (batched draft steps and verification passes of a few dozen sequences).  As in the kernel for
// up to 16 rows the weights are the A operand of v_mfma_f32_16x16x32_bf16 exactly as the packed
// tiles store them and the activations, split exactly into three bf16 terms, are the B operand;
// here every weight fragment meets all MT row tiles of the activations, so the weights stream
// from HBM once whatever the row count.
//
// A workgroup owns one K window (KSW steps of 32 columns) of the activations: it stages the three
// terms of all rows of that window in LDS once (a wavefront stages whole rows, so the sums of
// squares for the RMSNorm are plain wavefront sums), and each of its wavefronts then takes units
// of two weight tiles (or one gate/up tile pair) of that window: KSW fragments per tile in
// registers, every B fragment read from LDS feeds two MFMAs.  No sums across wavefronts; the
// window's partial product goes to scratch and the reduction kernel adds the windows in order,
// applies the norm scale and the epilogue.
#include <stdlib.h>

#include "hh_internal.h"
#include "bf16_split.h"
#include "trace.h"

namespace hh {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// bf16 terms an activation is split into: three (exact); with two (16 mantissa bits) the test
// with order-one activations loses a token to a near tie
static constexpr int kMidTerms = 3;

union MFrag {
  uint4 u;
  bf16x8 v;
};

struct MidArgs {
  const float* X; int ldx, M, K;
  const float* X2;                         // optional second addend of the input
  const float* norm_w;
  const uint16_t* W; const uint16_t* W2;   // packed tiles (W2: the "up" matrix for SwiGLU)
  int N, kst_row;                          // weight rows; steps of 32 columns a packed row holds
  float* partial;                          // [windows][NF][M][N]
  float* ssq;                              // [windows][ssq_ld] sums of squares per row, or nullptr
  int ssq_ld;
  int units;                               // wavefront units: pairs of tiles (NF = 1) or gate/up tile pairs (NF = 2)
};

template <int CTRL>
__device__ __forceinline__ float mid_dpp(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, false));
}
// sum over the 64 lanes (all lanes active)
__device__ __forceinline__ float mid_wave_sum(float v) {
  v += mid_dpp<0xB1>(v); v += mid_dpp<0x4E>(v); v += mid_dpp<0x141>(v); v += mid_dpp<0x140>(v);
  const int iv = __float_as_int(v);
  return (__int_as_float(__builtin_amdgcn_readlane(iv, 0)) + __int_as_float(__builtin_amdgcn_readlane(iv, 16))) +
         (__int_as_float(__builtin_amdgcn_readlane(iv, 32)) + __int_as_float(__builtin_amdgcn_readlane(iv, 48)));
}

// grid: x = groups of NW units (strided), y = K windows.  NF = 2: SwiGLU pair.  MT row tiles of 16.
// KSW steps of 32 columns per window (4 or 8).  NW wavefronts per workgroup: 4 (one per SIMD, so
// that the MFMA work of a small product spreads over all compute units) or 8.
template <int NF, int MT, int KSW, int NW>
__global__ __launch_bounds__(64 * NW) void mid_mfma_kernel(const MidArgs a) {
  constexpr int KW = KSW * 32, SL = KW + 8;      // window columns; staged row stride (bf16, padded)
  constexpr int ROWS = MT * 16;
  constexpr int CG = KW / 4;                     // float4 column groups per row
  constexpr int RPW = 64 / CG;                   // rows a wavefront stages per pass (1 or 2)
  extern __shared__ __align__(16) unsigned char smem_raw[];
  uint16_t* xs = reinterpret_cast<uint16_t*>(smem_raw);     // [kMidTerms][ROWS][SL]
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int g = lane >> 4, n = lane & 15;
  const int M = a.M, K = a.K, N = a.N;
  const int win = blockIdx.y, k0 = win * KW;

  // the weight fragments of a unit
  const int n_tiles = (N + 15) >> 4;
  const int KST = (K + 31) >> 5, step0 = win * KSW;
  MFrag wf[2][KSW];
  int tile[2] = {0, 0};
  auto load_unit = [&](int unit) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      tile[i] = NF == 2 ? unit : unit * 2 + i;
      const uint16_t* Wp = (NF == 2 && i == 1) ? a.W2 : a.W;
      const size_t row = (size_t)min(tile[i], n_tiles - 1) * a.kst_row;
#pragma unroll
      for (int s = 0; s < KSW; ++s)   // steps past the end of the row re-read the last one and meet zero activations
        wf[i][s].u = *reinterpret_cast<const uint4*>(Wp + (row + min(step0 + s, KST - 1)) * 512 + lane * 8);
    }
  };
  int unit = blockIdx.x * NW + wave;
  TR(0);

  // ---- stage the window: rows wave*RPW + NW*RPW*i, lane = (row in pass, column group).  The
  // loads of the first NB passes are requested before the weights (they would wait behind them).
  {
    const int cgi = lane % CG, rsub = lane / CG;
    const int col = k0 + 4 * cgi;
    const bool okc = col < K;                    // K % 4 == 0: a group is inside or outside
    const int colc = okc ? col : 0;
    float4 nw = make_float4(1.f, 1.f, 1.f, 1.f);
    if (a.norm_w != nullptr) nw = *reinterpret_cast<const float4*>(a.norm_w + colc);
    constexpr int PASS = NW * RPW;               // rows per pass of the workgroup
    constexpr int NP = (ROWS + PASS - 1) / PASS;
    constexpr int NB = NP < 12 ? NP : 12;        // passes whose loads are in flight together
    float4 v[NB];
    auto issue = [&](int p0) {
#pragma unroll
      for (int u = 0; u < NB; ++u) {
        const int r = (p0 + u) * PASS + wave * RPW + rsub;
        v[u] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (p0 + u < NP && r < M && okc) {
          v[u] = *reinterpret_cast<const float4*>(a.X + (size_t)r * a.ldx + col);
          if (a.X2 != nullptr) {
            const float4 w2 = *reinterpret_cast<const float4*>(a.X2 + (size_t)r * a.ldx + col);
            v[u].x += w2.x; v[u].y += w2.y; v[u].z += w2.z; v[u].w += w2.w;
          }
        }
      }
    };
    auto process = [&](int p0) {
#pragma unroll
      for (int u = 0; u < NB; ++u) {
        if (p0 + u >= NP) break;                 // wavefront-uniform
        const int r = (p0 + u) * PASS + wave * RPW + rsub;
        if (a.ssq != nullptr) {
          float sq = v[u].x * v[u].x + v[u].y * v[u].y + v[u].z * v[u].z + v[u].w * v[u].w;
          float tot;
          if (RPW == 1) {
            tot = mid_wave_sum(sq);
          } else {                               // two rows per wavefront: halves of 32 lanes
            sq += mid_dpp<0xB1>(sq); sq += mid_dpp<0x4E>(sq); sq += mid_dpp<0x141>(sq); sq += mid_dpp<0x140>(sq);
            const int iv = __float_as_int(sq);
            const float lo = __int_as_float(__builtin_amdgcn_readlane(iv, 0)) + __int_as_float(__builtin_amdgcn_readlane(iv, 16));
            const float hi = __int_as_float(__builtin_amdgcn_readlane(iv, 32)) + __int_as_float(__builtin_amdgcn_readlane(iv, 48));
            tot = rsub == 0 ? lo : hi;
          }
          if (blockIdx.x == 0 && cgi == 0 && r < M) a.ssq[(size_t)win * a.ssq_ld + r] = tot;
        }
        if (r < ROWS) {
          uint32_t a0, a1, a2, b0, b1, b2;
          split3_bf16_pair(v[u].x * nw.x, v[u].y * nw.y, a0, a1, a2);
          split3_bf16_pair(v[u].z * nw.z, v[u].w * nw.w, b0, b1, b2);
          uint16_t* dst = xs + (size_t)r * SL + 4 * cgi;
          *reinterpret_cast<uint2*>(dst) = make_uint2(a0, b0);
          *reinterpret_cast<uint2*>(dst + (size_t)ROWS * SL) = make_uint2(a1, b1);
          if (kMidTerms == 3) *reinterpret_cast<uint2*>(dst + (size_t)(kMidTerms - 1) * ROWS * SL) = make_uint2(a2, b2);
        }
      }
    };
    issue(0);
    if (unit < a.units) load_unit(unit);         // the first unit's weights stream in meanwhile
    TR(1);
    process(0);
    for (int p0 = NB; p0 < NP; p0 += NB) { issue(p0); process(p0); }
  }
  TR(2);
  __syncthreads();
  TR(3);

  // ---- the units of this wavefront
  while (unit < a.units) {
    f32x4 acc[2][MT];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) acc[i][mt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      const uint16_t* xrow = xs + (size_t)(mt * 16 + n) * SL + 8 * g;
#pragma unroll
      for (int s = 0; s < KSW; ++s) {
        // keeps the scheduler from hoisting the LDS reads of the whole unit (registers)
        if ((s & 1) == 0) asm volatile("" ::: "memory");
#pragma unroll
        for (int t = 0; t < kMidTerms; ++t) {
          MFrag xb;
          xb.u = *reinterpret_cast<const uint4*>(xrow + (size_t)t * ROWS * SL + s * 32);
          acc[0][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[0][s].v, xb.v, acc[0][mt], 0, 0, 0);
          acc[1][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[1][s].v, xb.v, acc[1][mt], 0, 0, 0);
        }
      }
    }
    TR(4);
    // the next unit's weights are requested before this unit's results are stored
    const int tl[2] = {tile[0], tile[1]};
    unit += (int)gridDim.x * NW;
    if (unit < a.units) load_unit(unit);
    // lane (g, n) holds Y[activation row mt*16 + n][weight rows tile*16 + 4g .. + 3]
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      if (tl[i] >= n_tiles) continue;
      const int f = NF == 2 ? i : 0;
      float* pb = a.partial + ((size_t)(win * NF + f) * M) * N;
      const int c0 = tl[i] * 16 + 4 * g;
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        const int m = mt * 16 + n;
        if (m >= M) continue;
        float* y = pb + (size_t)m * N + c0;
        if (c0 + 3 < N && (N & 3) == 0) {
          *reinterpret_cast<float4*>(y) = make_float4(acc[i][mt][0], acc[i][mt][1], acc[i][mt][2], acc[i][mt][3]);
        } else {
#pragma unroll
          for (int r = 0; r < 4; ++r)
            if (c0 + r < N) y[r] = acc[i][mt][r];
        }
      }
    }
  }
  TR(5);
}

struct MidPlan { int mt, ksw, nw, windows, units, blocks; size_t lds, partial_elems; };

static bool mid_plan(const GemvArgs& g, MidPlan& p) {
  if (!g.bf16 || g.n_seg != 1 || g.seg[0].P == nullptr || g.best != nullptr) return false;
  if (g.M <= 16 || g.M > 96 || g.K % 8 != 0 || g.K < 32 || g.ldx % 4 != 0) return false;
  if (g.epi == EPI_SWIGLU && g.seg[0].P2 == nullptr) return false;
  const int nf = g.epi == EPI_SWIGLU ? 2 : 1, N = g.seg[0].n_rows, tiles = (N + 15) / 16;
  p.mt = (g.M + 15) / 16;
  p.units = nf == 2 ? tiles : (tiles + 1) / 2;
  // Windows of 256 columns, of 128 when that leaves too few wavefront units for the chip's 1024
  // SIMDs (the MFMA work of a unit is what bounds a small product); 4 wavefronts per workgroup
  // (one per SIMD) unless there are units for 8.
  static const int min_units = getenv("HH_MID_MINUNITS") ? atoi(getenv("HH_MID_MINUNITS")) : 1024;
  p.ksw = 8;
  if ((long)p.units * ((g.K + 255) / 256) < min_units) p.ksw = 4;
  const int kw = p.ksw * 32;
  p.windows = (g.K + kw - 1) / kw;
  p.nw = (long)p.units * p.windows >= 4096 ? 8 : 4;
  p.blocks = (p.units + p.nw - 1) / p.nw;
  // more than ~4 workgroups per compute unit: several units per wavefront instead
  while ((long)p.blocks * p.windows > 1024 && p.blocks > 1) p.blocks = (p.blocks + 1) / 2;
  p.lds = (size_t)kMidTerms * p.mt * 16 * (kw + 8) * 2;
  p.partial_elems = (size_t)p.windows * nf * g.M * N + (size_t)p.windows * 96;
  return p.lds <= 160 * 1024 && p.partial_elems <= gemm_partial_elems() && p.windows <= 65535;
}

bool mid_mfma_fits(const GemvArgs& g) {
  static const bool off = getenv("HH_MID_OFF") != nullptr && atoi(getenv("HH_MID_OFF")) != 0;
  MidPlan p;
  return !off && mid_plan(g, p);
}

template <int NF, int MT, int KSW, int NW>
static hipError_t mid_launch(const MidArgs& a, const MidPlan& p, hipStream_t s) {
  auto kern = mid_mfma_kernel<NF, MT, KSW, NW>;
  static size_t lds_enabled = 48 * 1024;
  if (p.lds > lds_enabled) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)p.lds);
    if (e != hipSuccess) return e;
    lds_enabled = p.lds;
  }
  hipLaunchKernelGGL(kern, dim3(p.blocks, p.windows), dim3(64 * NW), p.lds, s, a);
  return hipGetLastError();
}
template <int NF, int MT>
static hipError_t mid_dispatch_k(const MidArgs& a, const MidPlan& p, hipStream_t s) {
  if (p.nw == 8) return p.ksw == 8 ? mid_launch<NF, MT, 8, 8>(a, p, s) : mid_launch<NF, MT, 4, 8>(a, p, s);
  return p.ksw == 8 ? mid_launch<NF, MT, 8, 4>(a, p, s) : mid_launch<NF, MT, 4, 4>(a, p, s);
}
template <int NF>
static hipError_t mid_dispatch(const MidArgs& a, const MidPlan& p, hipStream_t s) {
  switch (p.mt) {
    case 2: return mid_dispatch_k<NF, 2>(a, p, s);
    case 3: return mid_dispatch_k<NF, 3>(a, p, s);
    case 4: return mid_dispatch_k<NF, 4>(a, p, s);
    case 5: return mid_dispatch_k<NF, 5>(a, p, s);
    case 6: return mid_dispatch_k<NF, 6>(a, p, s);
  }
  return hipErrorInvalidValue;
}

// `partial`: scratch of gemm_partial_elems() floats
hipError_t launch_mid_mfma(const GemvArgs& g, float* partial, hipStream_t s) {
  MidPlan p;
  if (!mid_plan(g, p) || partial == nullptr) return hipErrorInvalidValue;
  const int N = g.seg[0].n_rows;
  if (N <= 0) return hipSuccess;
  const int nf = g.epi == EPI_SWIGLU ? 2 : 1;
  MidArgs a{};
  a.X = g.X; a.ldx = g.ldx; a.M = g.M; a.K = g.K; a.X2 = g.X2; a.norm_w = g.norm_w;
  a.W = static_cast<const uint16_t*>(g.seg[0].P); a.W2 = static_cast<const uint16_t*>(g.seg[0].P2);
  a.N = N; a.kst_row = (g.K + 31) / 32; a.partial = partial; a.units = p.units;
  a.ssq_ld = 96;
  a.ssq = g.norm_w != nullptr ? partial + (size_t)p.windows * nf * g.M * N : nullptr;
  hipError_t e = nf == 2 ? mid_dispatch<2>(a, p, s) : mid_dispatch<1>(a, p, s);
  if (e != hipSuccess) return e;
  return launch_gemm_reduce(g.epi, partial, p.windows, g.M, N, g.seg[0].Y, g.seg[0].ldy, g.R2, a.ssq, a.ssq_ld,
                            1.0f / (float)g.K, g.eps, s);
}

}  // namespace hh
