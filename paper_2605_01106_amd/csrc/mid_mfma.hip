// Dense projections for 17..96 activation rows on the matrix cores, bf16 weights:
//     Y[m][n] (op)= sum_k X'[m][k] * W[n][k],   X' = X (+ X2) or rmsnorm(X (+ X2)) * norm_w.
// (batched draft steps and verification passes of a few dozen sequences).  As in the kernel for
// up to 16 rows the weights are the A operand of v_mfma_f32_16x16x32_bf16 exactly as the packed
// tiles store them and the activations, split exactly into three bf16 terms, are the B operand;
// here every weight fragment meets all MT row tiles of the activations, so the weights stream
// from HBM once whatever the row count.
//
// A workgroup owns 8 units - a unit is two weight tiles, or one gate/up tile pair, one per
// wavefront - and a range of K windows of 128 columns.  Per window it stages the three terms of
// all activation rows in LDS (a wavefront stages whole rows; the sums of squares for the RMSNorm
// accumulate per lane) and every wavefront multiplies its unit's fragments of that window with
// every row tile: each B fragment read from LDS feeds two MFMAs, no sums across wavefronts, the
// accumulators stay in registers over the K range.  The K chunks of a product (gridDim.y) write
// partial products to scratch; the reduction kernel adds them in order and applies the norm
// scale and the epilogue.
#include <stdlib.h>

#include "hh_internal.h"
#include "wave_ops.h"
#include "bf16_split.h"
#include "trace.h"

namespace hh {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// bf16 terms an activation is split into: three (exact); with two (16 mantissa bits) the test
// with order-one activations loses a token to a near tie
static constexpr int kMidTerms = 3;
// padding of a staged activation row in LDS (bf16 elements): with 16 the row stride is 288 or 160 bytes and the
// 16-byte operand reads of a wavefront (row = lane % 16, 16-byte group = lane / 16) are free of bank conflicts
// (measured 156 bytes per cycle against 116 with a padding of 8)
// (8 where 16 would not fit the LDS: 96 rows with 128-column windows)
static constexpr int mid_pad(int mt, int kw) { return (size_t)2 * kMidTerms * mt * 16 * (kw + 16) * 2 <= 160 * 1024 ? 16 : 8; }

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
  int wpb;                                 // K-loop kernel: windows per workgroup (K chunk)
};

// The K loop: the staged activations are double-buffered in LDS and the weight fragments
// triple-buffered in registers: while window i is multiplied, the activations of window i+1 are
// loaded, split and written to the other buffer and the weights of window i+2 are requested;
// one workgroup barrier per window.  The
// grid: x = groups of 8 units, y = K chunks of a.wpb windows.
// NW wavefronts per workgroup (one unit each), KSW steps of 32 columns per window: 8 x 4 (one
// workgroup per compute unit: 104 KB of LDS at 64 rows) or 4 x 2 (half the columns and half the window:
// 55 KB of LDS and half the registers, so that two workgroups share a compute unit and one's loads,
// staging and barriers hide behind the other's MFMAs).
template <int NF, int MT, int NW, int KSW>
__global__ __launch_bounds__(64 * NW) void mid_loop_kernel(const MidArgs a) {
  constexpr int KW = KSW * 32, SL = KW + mid_pad(MT, KW);
  constexpr int ROWS = MT * 16;
  constexpr int GPR = KW / 4;                    // float4 column groups per staged row: 32 or 16 lanes
  constexpr int RPW = 64 / GPR;                  // rows a wavefront stages per pass: 2 or 4
  constexpr int PASS = NW * RPW;                 // rows staged per pass (16 in both shapes)
  constexpr int NP = ROWS / PASS;
  static_assert(PASS == 16 && (KSW == 4 || KSW == 2), "a staging pass is one row tile");
  constexpr size_t BUF = (size_t)kMidTerms * ROWS * SL;   // bf16 elements per LDS buffer
  extern __shared__ __align__(16) unsigned char smem_raw[];
  uint16_t* xs = reinterpret_cast<uint16_t*>(smem_raw);     // [2][kMidTerms][ROWS][SL]
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int g = lane >> 4, n = lane & 15;
  const int M = a.M, K = a.K, N = a.N;
  const int n_tiles = (N + 15) >> 4, KST = (K + 31) >> 5;
  const int n_win = (K + KW - 1) / KW;
  const int win0 = blockIdx.y * a.wpb, win1 = min(n_win, win0 + a.wpb);   // win0 < n_win by construction
  const int unit = blockIdx.x * NW + wave;
  int tile[2];
  const uint16_t* wrow[2];
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    tile[i] = NF == 2 ? unit : unit * 2 + i;
    wrow[i] = ((NF == 2 && i == 1) ? a.W2 : a.W) + (size_t)min(tile[i], n_tiles - 1) * a.kst_row * 512 + lane * 8;
  }
  // staging: lane = (row in pass, float4 column group)
  const int cgi = lane & (GPR - 1), rsub = lane / GPR;
  float4 v[NP], nw;
  float sq[NP];
#pragma unroll
  for (int u = 0; u < NP; ++u) sq[u] = 0.f;
  // unconditional loads from clamped addresses (a branch around them would make the waits for
  // the current window's operands wait for these too); what lies outside is zeroed when staged
  bool okc = false;
  auto issue_x = [&](int win) {
    const int col = win * KW + 4 * cgi;
    okc = col < K;                               // K % 4 == 0: a group is inside or outside
    const int colc = okc ? col : 0;
    nw = make_float4(1.f, 1.f, 1.f, 1.f);
    if (a.norm_w != nullptr) nw = *reinterpret_cast<const float4*>(a.norm_w + colc);
#pragma unroll
    for (int u = 0; u < NP; ++u) {
      const int r = min(u * PASS + wave * RPW + rsub, M - 1);
      v[u] = *reinterpret_cast<const float4*>(a.X + (size_t)r * a.ldx + colc);
    }
    if (a.X2 != nullptr) {
#pragma unroll
      for (int u = 0; u < NP; ++u) {
        const int r = min(u * PASS + wave * RPW + rsub, M - 1);
        const float4 w2 = *reinterpret_cast<const float4*>(a.X2 + (size_t)r * a.ldx + colc);
        v[u].x += w2.x; v[u].y += w2.y; v[u].z += w2.z; v[u].w += w2.w;
      }
    }
  };
  auto issue_w = [&](int win, MFrag(&w)[2][KSW]) {
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int s = 0; s < KSW; ++s)   // steps past the end of the row re-read the last one and meet zero activations
        w[i][s].u = *reinterpret_cast<const uint4*>(wrow[i] + (size_t)min(win * KSW + s, KST - 1) * 512);
  };
  auto stage = [&](uint16_t* buf) {
#pragma unroll
    for (int u = 0; u < NP; ++u) {
      const int r = u * PASS + wave * RPW + rsub;
      if (!(okc && r < M)) v[u] = make_float4(0.f, 0.f, 0.f, 0.f);
      sq[u] += v[u].x * v[u].x + v[u].y * v[u].y + v[u].z * v[u].z + v[u].w * v[u].w;
      uint32_t a0, a1, a2, b0, b1, b2;
      split3_bf16_pair(v[u].x * nw.x, v[u].y * nw.y, a0, a1, a2);
      split3_bf16_pair(v[u].z * nw.z, v[u].w * nw.w, b0, b1, b2);
      uint16_t* dst = buf + (size_t)r * SL + 4 * cgi;
      *reinterpret_cast<uint2*>(dst) = make_uint2(a0, b0);
      *reinterpret_cast<uint2*>(dst + (size_t)ROWS * SL) = make_uint2(a1, b1);
      if (kMidTerms == 3) *reinterpret_cast<uint2*>(dst + (size_t)(kMidTerms - 1) * ROWS * SL) = make_uint2(a2, b2);
    }
  };
  f32x4 acc[2][MT];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) acc[i][mt] = f32x4{0.f, 0.f, 0.f, 0.f};
  // B fragments in batches of two steps (6 fragments), the next batch read from LDS while the
  // current one is multiplied; the fences keep the scheduler from hoisting more reads than that
  // (registers).
  auto multiply = [&](const uint16_t* buf, const MFrag(&w)[2][KSW]) {
    constexpr int NBATCH = MT * KSW / 2;
    const uint16_t* xbase = buf + (size_t)n * SL + 8 * g;
    MFrag xb[2][2 * kMidTerms];
    auto read_batch = [&](int b, MFrag(&x)[2 * kMidTerms]) {
      const int mt = b / (KSW / 2), s0 = (b % (KSW / 2)) * 2;
      const uint16_t* xrow = xbase + (size_t)mt * 16 * SL;
#pragma unroll
      for (int ds = 0; ds < 2; ++ds)
#pragma unroll
        for (int t = 0; t < kMidTerms; ++t)
          x[ds * kMidTerms + t].u = *reinterpret_cast<const uint4*>(xrow + (size_t)t * ROWS * SL + (s0 + ds) * 32);
    };
    read_batch(0, xb[0]);
#pragma unroll
    for (int b = 0; b < NBATCH; ++b) {
      asm volatile("" ::: "memory");
      if (b + 1 < NBATCH) read_batch(b + 1, xb[(b + 1) & 1]);
      const int mt = b / (KSW / 2), s0 = (b % (KSW / 2)) * 2;
#pragma unroll
      for (int ds = 0; ds < 2; ++ds)
#pragma unroll
        for (int t = 0; t < kMidTerms; ++t) {
          acc[0][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w[0][s0 + ds].v, xb[b & 1][ds * kMidTerms + t].v, acc[0][mt], 0, 0, 0);
          acc[1][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w[1][s0 + ds].v, xb[b & 1][ds * kMidTerms + t].v, acc[1][mt], 0, 0, 0);
        }
    }
  };
  // One window: request the activations of the next one and the weights of the one after it
  // (HBM latency exceeds one window's multiplication; past the end the last window is requested
  // again and not used), multiply this one, stage the next one in the other LDS buffer.  Three
  // weight buffers in rotation: the loop body is three windows, straight-line.
  MFrag w0[2][KSW], w1[2][KSW], w2[2][KSW];
  auto window = [&](int win, const MFrag(&wc)[2][KSW], MFrag(&wn2)[2][KSW]) {
    uint16_t* cur = xs + (size_t)((win - win0) & 1) * BUF;
    uint16_t* nxt = xs + (size_t)((win - win0 + 1) & 1) * BUF;
    issue_x(min(win + 1, win1 - 1));
    issue_w(min(win + 2, win1 - 1), wn2);
    multiply(cur, wc);
    if (win + 1 < win1) stage(nxt);
    __syncthreads();
  };
  TR(0);
  issue_x(win0);
  issue_w(win0, w0);
  issue_w(min(win0 + 1, win1 - 1), w1);
  TR(1);
  stage(xs);
  __syncthreads();
  TR(2);
  int win = win0;
  for (; win + 2 < win1; win += 3) {
    window(win, w0, w2);
    window(win + 1, w1, w0);
    window(win + 2, w2, w1);
  }
  if (win < win1) window(win, w0, w2);
  if (win + 1 < win1) window(win + 1, w1, w0);
  TR(3);
  // sums of squares of the rows this wavefront staged (GPR lanes per row), for the norm scale
  if (a.ssq != nullptr && blockIdx.x == 0) {
#pragma unroll
    for (int u = 0; u < NP; ++u) {
      float t = row16_sum(sq[u]);                                   // every row of 16 lanes holds its total
      if (GPR == 32) t += __shfl_xor(t, 16, 64);                    // a staged row spans two rows of lanes
      const int r = u * PASS + wave * RPW + rsub;
      if (cgi == 0 && r < M) a.ssq[(size_t)blockIdx.y * a.ssq_ld + r] = t;
    }
  }
  // lane (g, n) holds Y[activation row mt*16 + n][weight rows tile*16 + 4g .. + 3]
  TR(4);
  if (unit >= a.units) return;
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    if (tile[i] >= n_tiles) continue;
    const int f = NF == 2 ? i : 0;
    float* pb = a.partial + ((size_t)(blockIdx.y * NF + f) * M) * N;
    const int c0 = tile[i] * 16 + 4 * g;
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
  TR(5);
}


struct MidPlan { int mt, windows, units, blocks, wpb, small; size_t lds, partial_elems; };   // windows: K chunks = partial products

static bool mid_plan(const GemvArgs& g, MidPlan& p) {
  if (!g.bf16 || g.n_seg != 1 || g.seg[0].P == nullptr || g.best != nullptr) return false;   // (argmax: through g.row_best)
  if (g.M <= 16 || g.M > 96 || g.K % 8 != 0 || g.K < 32 || g.ldx % 4 != 0) return false;
  if (g.epi == EPI_SWIGLU && g.seg[0].P2 == nullptr) return false;
  const int nf = g.epi == EPI_SWIGLU ? 2 : 1, N = g.seg[0].n_rows, tiles = (N + 15) / 16;
  p.mt = (g.M + 15) / 16;
  p.units = nf == 2 ? tiles : (tiles + 1) / 2;
  // the small shape (4 wavefronts, windows of 64 columns, two workgroups per compute unit) for up to 80 rows
  // (96 rows: two workgroups' staging buffers no longer fit the LDS)
  p.small = p.mt <= 5 && !(g.flags & HH_KF_MID_WIDE) ? 1 : 0;
  const int upb = p.small ? 4 : 8, kw = p.small ? 64 : 128;
  // K chunks so that the launch has at most one (two) workgroup(s) per compute unit
  const int target = p.small ? 512 : 256;
  const int n_win = (g.K + kw - 1) / kw;
  p.blocks = (p.units + upb - 1) / upb;
  int ks = target / p.blocks;
  if (ks > n_win) ks = n_win;
  if (ks < 1) ks = 1;
  p.wpb = (n_win + ks - 1) / ks;
  if (p.small) {
    // The small shape picks its windows per workgroup from a cost model fitted to the 3B shape at 64 rows (us):
    // a window costs a workgroup 0.305 us per row tile, 1.4 times that when the launch has more than one workgroup
    // per compute unit; a K chunk costs 0.49 us per 64 x 2560 partial sums (written, then read by the reduction).
    // Few long workgroups beat many short ones for the narrow products: out_proj 18.2 -> 14.5 us with 8 chunks of
    // 5 windows instead of 20 of 2, in_proj 19.0 -> 17.4 us with 5 chunks of 8 instead of 10 of 4.  The longest
    // workgroups within 3 % of the cheapest plan win (fewer partial sums).
    const double tw = 0.305 * p.mt, cc = 0.49 * (g.M / 64.0) * nf * (N / 2560.0);
    double t_min = 1e30;
    for (int pass = 0; pass < 2; ++pass) {
      for (int w = 1; w <= n_win; ++w) {
        const int ch = (n_win + w - 1) / w;
        const long wgs = (long)p.blocks * ch;
        if (wgs > 512 && w < n_win) continue;            // at most two workgroups per compute unit
        const double t = tw * w * (wgs > 256 ? 1.4 : 1.0) + cc * ch;
        if (pass == 0) { if (t < t_min) t_min = t; }
        else if (t <= 1.03 * t_min) p.wpb = w;
      }
    }
  }
  p.windows = (n_win + p.wpb - 1) / p.wpb;          // K chunks = partial products
  p.lds = (size_t)2 * kMidTerms * p.mt * 16 * (kw + mid_pad(p.mt, kw)) * 2;
  p.partial_elems = (size_t)p.windows * nf * g.M * N + (size_t)p.windows * 96;
  return p.lds <= 160 * 1024 && p.partial_elems <= gemm_partial_elems() && p.windows <= 65535;
}

bool mid_mfma_fits(const GemvArgs& g) {
  MidPlan p;
  return !(g.flags & HH_KF_MID_OFF) && mid_plan(g, p);
}

template <int NF, int MT, int NW, int KSW>
static hipError_t mid_launch_loop(const MidArgs& a, const MidPlan& p, hipStream_t s) {
  auto kern = mid_loop_kernel<NF, MT, NW, KSW>;
  static size_t lds_enabled = 48 * 1024;
  if (p.lds > lds_enabled) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)p.lds);
    if (e != hipSuccess) return e;
    lds_enabled = p.lds;
  }
  hipLaunchKernelGGL(kern, dim3(p.blocks, p.windows), dim3(64 * NW), p.lds, s, a);
  return hipGetLastError();
}
template <int NF>
static hipError_t mid_dispatch(const MidArgs& a, const MidPlan& p, hipStream_t s) {
  if (p.small) {
    switch (p.mt) {
      case 2: return mid_launch_loop<NF, 2, 4, 2>(a, p, s);
      case 3: return mid_launch_loop<NF, 3, 4, 2>(a, p, s);
      case 4: return mid_launch_loop<NF, 4, 4, 2>(a, p, s);
      case 5: return mid_launch_loop<NF, 5, 4, 2>(a, p, s);
    }
    return hipErrorInvalidValue;
  }
  switch (p.mt) {
    case 2: return mid_launch_loop<NF, 2, 8, 4>(a, p, s);
    case 3: return mid_launch_loop<NF, 3, 8, 4>(a, p, s);
    case 4: return mid_launch_loop<NF, 4, 8, 4>(a, p, s);
    case 5: return mid_launch_loop<NF, 5, 8, 4>(a, p, s);
    case 6: return mid_launch_loop<NF, 6, 8, 4>(a, p, s);
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
  a.N = N; a.kst_row = (g.K + 31) / 32; a.partial = partial; a.units = p.units; a.wpb = p.wpb;
  a.ssq_ld = 96;
  a.ssq = g.norm_w != nullptr ? partial + (size_t)p.windows * nf * g.M * N : nullptr;
  hipError_t e = nf == 2 ? mid_dispatch<2>(a, p, s) : mid_dispatch<1>(a, p, s);
  if (e != hipSuccess) return e;
  return launch_gemm_reduce(g.epi, partial, p.windows, g.M, N, g.seg[0].Y, g.seg[0].ldy, g.R2, a.ssq, a.ssq_ld,
                            1.0f / (float)g.K, g.eps, g.row_best, g.no_store ? 0 : 1, s);
}

}  // namespace hh
