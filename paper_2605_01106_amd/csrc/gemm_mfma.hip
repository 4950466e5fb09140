// Dense projections on the matrix cores for passes with many activation rows (more than 96:
// verification of large batches, prefill): Y[M x N] (op)= X'[M x K] * W[N x K]^T, bf16 weights in
// the packed operand tiles.
//
// A first kernel applies the fused RMSNorm and splits every activation into bf16 terms stored
// as planes: x = t0 + t1 + t2 exactly (two terms, 16 mantissa bits, as an option); the product
// is the sum of the per-term bf16 MFMA products accumulated in float32.
//
// GEMM kernel: a wavefront is an independent unit of work - NT strips of 16 weight rows x
// MTW tiles of 16 activation rows x a range of K steps - with all accumulators in registers
// and no LDS.  Per step of 32 columns it loads NT weight tiles (A operand, 1 KB contiguous each,
// from HBM) and terms x MTW activation fragments (B operand, from the planes, which stay in L2)
// and issues terms x NT x MTW MFMAs; the next step is requested before the current one is
// multiplied.  The activation fragments are shared by the NT strips, so L2 traffic is
// terms MTW / NT times the weight traffic.  When N is small the K range is split over units to
// cover the chip; the partial products go to a scratch buffer and a second kernel adds them
// in split order (deterministic) and applies the epilogue.  With one split the epilogue runs
// in the GEMM kernel.  Accumulator layout: lane l holds D[weight row 4(l/16)+r][activation row l%16].
#include <stdlib.h>

#include "hh_internal.h"
#include "bf16_split.h"
#include "wave_ops.h"
#include "gemm_lds.h"

namespace hh {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// bf16 terms an activation is split into for this kernel (planes per row tile and step): three
// (exact).  Two terms (16 mantissa bits) would be about twice as fast, and the benign
// random-weight workloads would still match the float64 reference, but models with order-one
// activations and recurrences amplify the 2^-17 relative error beyond the logit tolerance (seen
// on the test initialisation with 160 prefill rows).
static int gemm_terms(int) { return 3; }

// split activations in MFMA operand order (see below); rows >= M and columns >= K are zero.
// One workgroup per row; a thread handles groups of 8 consecutive columns (two float4 loads,
// one 16-byte store per term): K % 8 == 0 and 16-byte aligned rows (VEC), else element by element.
template <bool VEC>
__global__ __launch_bounds__(256) void split_rows_kernel(const float* __restrict__ X, const float* __restrict__ X2, int ldx, int M, int K, int Mp, int Kp,
                                                         const float* __restrict__ norm_w, float eps,
                                                         uint16_t* __restrict__ planes, const int kTerms) {
  const int m = blockIdx.x;
  __shared__ float red[4];
  const float* xr = X + (size_t)m * ldx;
  const float* xr2 = X2 != nullptr ? X2 + (size_t)m * ldx : nullptr;
  float rstd = 1.f;
  if (m < M && norm_w != nullptr) {
    float ss = 0.f;
    if (VEC) {
      for (int k = threadIdx.x * 4; k < K; k += 1024) {
        float4 v = *reinterpret_cast<const float4*>(xr + k);
        if (xr2 != nullptr) { const float4 w = *reinterpret_cast<const float4*>(xr2 + k); v.x += w.x; v.y += w.y; v.z += w.z; v.w += w.w; }
        ss = fmaf(v.x, v.x, ss); ss = fmaf(v.y, v.y, ss); ss = fmaf(v.z, v.z, ss); ss = fmaf(v.w, v.w, ss);
      }
    } else {
      for (int k = threadIdx.x; k < K; k += 256) {
        const float v = xr[k] + (xr2 != nullptr ? xr2[k] : 0.f);
        ss = fmaf(v, v, ss);
      }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) ss += __shfl_xor(ss, o, 64);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
    __syncthreads();
    rstd = 1.0f / sqrtf((red[0] + red[1] + red[2] + red[3]) / (float)K + eps);
  }
  // operand order: block (row tile, step of 32 columns, term) of 512 elements, lane 16 g + n at
  // element 8 (16 g + n), n = row % 16, g = (column % 32) / 8: a wavefront load is 1 KB contiguous
  const int KST = Kp >> 5;
  if (VEC) {
    for (int k = threadIdx.x * 8; k < Kp; k += 2048) {
      float v[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) v[i] = 0.f;
      if (m < M && k < K) {                       // K % 8 == 0: a group is inside or outside
        const float4 a0 = *reinterpret_cast<const float4*>(xr + k), a1 = *reinterpret_cast<const float4*>(xr + k + 4);
        v[0] = a0.x; v[1] = a0.y; v[2] = a0.z; v[3] = a0.w; v[4] = a1.x; v[5] = a1.y; v[6] = a1.z; v[7] = a1.w;
        if (xr2 != nullptr) {
          const float4 b0 = *reinterpret_cast<const float4*>(xr2 + k), b1 = *reinterpret_cast<const float4*>(xr2 + k + 4);
          v[0] += b0.x; v[1] += b0.y; v[2] += b0.z; v[3] += b0.w; v[4] += b1.x; v[5] += b1.y; v[6] += b1.z; v[7] += b1.w;
        }
        if (norm_w != nullptr) {
          const float4 n0 = *reinterpret_cast<const float4*>(norm_w + k), n1 = *reinterpret_cast<const float4*>(norm_w + k + 4);
          const float nw[8] = {n0.x, n0.y, n0.z, n0.w, n1.x, n1.y, n1.z, n1.w};
#pragma unroll
          for (int i = 0; i < 8; ++i) v[i] = v[i] * nw[i] * rstd;   // same order as the element-wise path
        }
      }
      uint32_t w0[4], w1[4], w2[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) split3_bf16_pair(v[2 * i], v[2 * i + 1], w0[i], w1[i], w2[i]);
      uint16_t* dst = planes + (((size_t)(m >> 4) * KST + (k >> 5)) * kTerms) * 512 + (size_t)((((k & 31) >> 3) * 16 + (m & 15)) * 8);
      *reinterpret_cast<uint4*>(dst) = make_uint4(w0[0], w0[1], w0[2], w0[3]);
      *reinterpret_cast<uint4*>(dst + 512) = make_uint4(w1[0], w1[1], w1[2], w1[3]);
      if (kTerms == 3) *reinterpret_cast<uint4*>(dst + 1024) = make_uint4(w2[0], w2[1], w2[2], w2[3]);
    }
    return;
  }
  for (int k = threadIdx.x; k < Kp; k += 256) {
    uint16_t t0 = 0, t1 = 0, t2 = 0;
    if (m < M && k < K) {
      float v = xr[k] + (xr2 != nullptr ? xr2[k] : 0.f);
      if (norm_w != nullptr) v = v * norm_w[k] * rstd;
      uint32_t b0, b1, b2;
      split3_bf16(v, b0, b1, b2);
      t0 = (uint16_t)b0; t1 = (uint16_t)b1; t2 = (uint16_t)b2;
    }
    const size_t at = (((size_t)(m >> 4) * KST + (k >> 5)) * kTerms) * 512 + (size_t)((((k & 31) >> 3) * 16 + (m & 15)) * 8 + (k & 7));
    planes[at] = t0; planes[at + 512] = t1;
    if (kTerms == 3) planes[at + 1024] = t2;
  }
}

// The same planes for passes of many rows (three terms, K % 8 == 0, 16-byte aligned rows): one workgroup of 16
// wavefronts per tile of 16 rows.  Thread = (row r = tid % 16, column group tid / 16 of 8 columns), so that a
// wavefront holds the 16 rows x 32 columns of one step and each of its three stores is one whole fragment:
// 1 KB contiguous (the row-wise kernel above writes a fragment as 64 separate 16-byte pieces from 16
// workgroups).  Rows with a norm are read twice, as there: sums of squares first (the four lanes of a row
// within the wavefront, then the 16 wavefronts through LDS in a fixed order), then the split.
// grid: x = row tiles, y = column slices of `slice` columns (a multiple of 512) for passes with few row tiles:
// every workgroup of a tile then sums the squares of the whole rows (from L2) and splits its slice.
__global__ __launch_bounds__(1024) void split_tiles_kernel(const float* __restrict__ X, const float* __restrict__ X2, int ldx, int M, int K, int Kp,
                                                           const float* __restrict__ norm_w, float eps, uint16_t* __restrict__ planes, int slice) {
  __shared__ float red[16][16];
  const int tid = threadIdx.x, r = tid & 15, kg = tid >> 4, wave = tid >> 6;
  const int m = blockIdx.x * 16 + r;
  const bool row_ok = m < M;
  const float* xr = X + (size_t)min(m, M - 1) * ldx;
  const float* xr2 = X2 != nullptr ? X2 + (size_t)min(m, M - 1) * ldx : nullptr;
  float rstd = 1.f;
  if (norm_w != nullptr) {
    float ss = 0.f;
    for (int k = kg * 8; k < K; k += 512) {
      float4 a0 = *reinterpret_cast<const float4*>(xr + k), a1 = *reinterpret_cast<const float4*>(xr + k + 4);
      if (xr2 != nullptr) {
        const float4 b0 = *reinterpret_cast<const float4*>(xr2 + k), b1 = *reinterpret_cast<const float4*>(xr2 + k + 4);
        a0.x += b0.x; a0.y += b0.y; a0.z += b0.z; a0.w += b0.w; a1.x += b1.x; a1.y += b1.y; a1.z += b1.z; a1.w += b1.w;
      }
      ss = fmaf(a0.x, a0.x, ss); ss = fmaf(a0.y, a0.y, ss); ss = fmaf(a0.z, a0.z, ss); ss = fmaf(a0.w, a0.w, ss);
      ss = fmaf(a1.x, a1.x, ss); ss = fmaf(a1.y, a1.y, ss); ss = fmaf(a1.z, a1.z, ss); ss = fmaf(a1.w, a1.w, ss);
    }
    ss += __shfl_xor(ss, 16, 64);
    ss += __shfl_xor(ss, 32, 64);
    if ((tid & 63) < 16) red[wave][r] = ss;
    __syncthreads();
    float tot = 0.f;
#pragma unroll
    for (int w = 0; w < 16; ++w) tot += red[w][r];
    rstd = 1.0f / sqrtf(tot / (float)K + eps);
  }
  const int KST = Kp >> 5;
  const int k_end = min(Kp, ((int)blockIdx.y + 1) * slice);
  for (int k = (int)blockIdx.y * slice + kg * 8; k < k_end; k += 512) {
    float v[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = 0.f;
    if (row_ok && k < K) {                        // K % 8 == 0: a group is inside or outside
      const float4 a0 = *reinterpret_cast<const float4*>(xr + k), a1 = *reinterpret_cast<const float4*>(xr + k + 4);
      v[0] = a0.x; v[1] = a0.y; v[2] = a0.z; v[3] = a0.w; v[4] = a1.x; v[5] = a1.y; v[6] = a1.z; v[7] = a1.w;
      if (xr2 != nullptr) {
        const float4 b0 = *reinterpret_cast<const float4*>(xr2 + k), b1 = *reinterpret_cast<const float4*>(xr2 + k + 4);
        v[0] += b0.x; v[1] += b0.y; v[2] += b0.z; v[3] += b0.w; v[4] += b1.x; v[5] += b1.y; v[6] += b1.z; v[7] += b1.w;
      }
      if (norm_w != nullptr) {
        const float4 n0 = *reinterpret_cast<const float4*>(norm_w + k), n1 = *reinterpret_cast<const float4*>(norm_w + k + 4);
        const float nw[8] = {n0.x, n0.y, n0.z, n0.w, n1.x, n1.y, n1.z, n1.w};
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] = v[i] * nw[i] * rstd;
      }
    }
    uint32_t w0[4], w1[4], w2[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) split3_bf16_pair(v[2 * i], v[2 * i + 1], w0[i], w1[i], w2[i]);
    // fragment (row tile, step k / 32): element 8 * (16 * ((k % 32) / 8) + r) = 8 * (tid % 64)
    uint16_t* dst = planes + (((size_t)blockIdx.x * KST + (k >> 5)) * 3) * 512 + (size_t)(tid & 63) * 8;
    *reinterpret_cast<uint4*>(dst) = make_uint4(w0[0], w0[1], w0[2], w0[3]);
    *reinterpret_cast<uint4*>(dst + 512) = make_uint4(w1[0], w1[1], w1[2], w1[3]);
    *reinterpret_cast<uint4*>(dst + 1024) = make_uint4(w2[0], w2[1], w2[2], w2[3]);
  }
}

struct GemmArgs {
  const uint16_t* planes; int Mp, Kp;     // split activations [3][Mp][Kp]
  const uint16_t* W; const uint16_t* W2;  // packed tiles (W2: the "up" matrix for SwiGLU)
  float* Y; int ldy;
  const float* R2;                        // optional second residual (EPI_ADD)
  float* partial;                         // [ksplit][NF][M][N] when ksplit > 1
  int M, N, K;
  int strip_groups, m_groups, ksplit;     // units = strip_groups * m_groups * ksplit
  int ksteps;                             // steps of 32 columns per unit
  // reduction only: per-split sums of squares of the activation rows [ksplit][ssq_ld] (or
  // nullptr); the row sum is then scaled by 1 / sqrt(sum * rnorm_k + eps)
  const float* ssq; int ssq_ld; float rnorm_k, eps;
  int terms;                              // bf16 terms per activation in the planes (2 or 3)
  // EPI_STORE: per-row argmax keys [M], zeroed by the caller and raised with atomic maxima (the
  // maximum of the keys is the same in any order), or nullptr; store = 0: Y itself is not written
  unsigned long long* row_best; int store;
};

union GFrag {
  uint4 u;
  bf16x8 v;
};

template <int EPI, int NT, int MTW, int kTerms>
__global__ __launch_bounds__(256, 2) void gemm_tiled_kernel(const GemmArgs a) {
  constexpr int NF = EPI == EPI_SWIGLU ? 2 : 1;
  const int lane = threadIdx.x & 63;
  const int unit = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int n_units = a.strip_groups * a.m_groups * a.ksplit;
  if (unit >= n_units) return;
  const int g = lane >> 4, n = lane & 15;
  // unit -> (strip group, m group, k split); consecutive units share the K range and the m group
  const int sg = unit % a.strip_groups, mg = (unit / a.strip_groups) % a.m_groups, kp = unit / (a.strip_groups * a.m_groups);
  const int KST = (a.K + 31) >> 5, n_tiles = (a.N + 15) >> 4, m_tiles = a.Mp >> 4;
  const int k_begin = kp * a.ksteps, k_end = min(KST, k_begin + a.ksteps);
  const int t0 = sg * NT, mt0 = mg * MTW;

  f32x4 acc[NF][NT][MTW];
#pragma unroll
  for (int f = 0; f < NF; ++f)
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
      for (int m = 0; m < MTW; ++m) acc[f][t][m] = f32x4{0.f, 0.f, 0.f, 0.f};

  GFrag wf[2][NF][NT], xf[2][kTerms][MTW];
  auto load_step = [&](int ks, GFrag(&w)[NF][NT], GFrag(&x)[kTerms][MTW]) {
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      const size_t at = ((size_t)min(t0 + t, n_tiles - 1) * KST + ks) * 512 + lane * 8;
      w[0][t].u = *reinterpret_cast<const uint4*>(a.W + at);
      if (NF == 2) w[NF - 1][t].u = *reinterpret_cast<const uint4*>(a.W2 + at);
    }
#pragma unroll
    for (int m = 0; m < MTW; ++m) {
      const uint16_t* src = a.planes + (((size_t)min(mt0 + m, m_tiles - 1) * KST + ks) * kTerms) * 512 + lane * 8;
#pragma unroll
      for (int term = 0; term < kTerms; ++term) x[term][m].u = *reinterpret_cast<const uint4*>(src + term * 512);
    }
  };
  auto mul_step = [&](const GFrag(&w)[NF][NT], const GFrag(&x)[kTerms][MTW]) {
#pragma unroll
    for (int term = 0; term < kTerms; ++term)
#pragma unroll
      for (int m = 0; m < MTW; ++m)
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
          for (int f = 0; f < NF; ++f)
            acc[f][t][m] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w[f][t].v, x[term][m].v, acc[f][t][m], 0, 0, 0);
  };
  if (k_begin < k_end) load_step(k_begin, wf[0], xf[0]);
  for (int ks = k_begin; ks < k_end; ks += 2) {
    if (ks + 1 < k_end) load_step(ks + 1, wf[1], xf[1]);
    mul_step(wf[0], xf[0]);
    if (ks + 1 < k_end) {
      if (ks + 2 < k_end) load_step(ks + 2, wf[0], xf[0]);
      mul_step(wf[1], xf[1]);
    }
  }

  // ---- results: D[weight row 4g+r][activation row n] of every (strip, m tile)
  unsigned long long best[MTW];
#pragma unroll
  for (int m = 0; m < MTW; ++m) best[m] = 0ull;
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    const int row0 = (t0 + t) * 16 + 4 * g;
    if (t0 + t >= n_tiles) continue;
#pragma unroll
    for (int m = 0; m < MTW; ++m) {
      const int am = (mt0 + m) * 16 + n;
      if (mt0 + m >= m_tiles || am >= a.M) continue;
      if (a.ksplit > 1) {
#pragma unroll
        for (int f = 0; f < NF; ++f) {
          float* p = a.partial + (((size_t)kp * NF + f) * a.M + am) * a.N + row0;
          if (row0 + 3 < a.N && (a.N & 3) == 0) *reinterpret_cast<float4*>(p) = make_float4(acc[f][t][m][0], acc[f][t][m][1], acc[f][t][m][2], acc[f][t][m][3]);
          else
#pragma unroll
            for (int r = 0; r < 4; ++r) if (row0 + r < a.N) p[r] = acc[f][t][m][r];
        }
      } else {
        float* y = a.Y + (size_t)am * a.ldy + row0;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          if (row0 + r < a.N) {
            float v = acc[0][t][m][r];
            if (EPI == EPI_SWIGLU) v = v / (1.0f + expf(-v)) * acc[NF - 1][t][m][r];
            if (EPI == EPI_ADD) v += y[r] + (a.R2 != nullptr ? a.R2[(size_t)am * a.ldy + row0 + r] : 0.f);
            if (EPI != EPI_STORE || a.store) y[r] = v;
            if (EPI == EPI_STORE) { const unsigned long long key = argmax_key(v, row0 + r); if (key > best[m]) best[m] = key; }
          }
        }
      }
    }
  }
  if (EPI == EPI_STORE && a.row_best != nullptr && a.ksplit == 1) {
    // largest key of this lane's activation row over the unit's weight rows: across the four lane
    // groups, then one atomic maximum per row and wavefront
#pragma unroll
    for (int m = 0; m < MTW; ++m) {
      unsigned long long b = best[m];
      unsigned long long o = __shfl_xor(b, 16, 64); if (o > b) b = o;
      o = __shfl_xor(b, 32, 64); if (o > b) b = o;
      const int am = (mt0 + m) * 16 + n;
      if (g == 0 && mt0 + m < m_tiles && am < a.M && b != 0ull) atomicMax(a.row_best + am, b);
    }
  }
}

// second pass when K is split: sum of the partial products in split order + epilogue
// (4 consecutive columns per thread when the shapes allow vector accesses: VEC)
// ARGMAX (EPI_STORE): the grid is (column blocks, rows) so that a workgroup stays inside one row;
// it raises the row's argmax key by one atomic maximum.
template <int EPI, bool VEC, bool ARGMAX = false>
__global__ __launch_bounds__(256) void gemm_reduce_kernel(const GemmArgs a) {
  constexpr int NF = EPI == EPI_SWIGLU ? 2 : 1;
  constexpr int W = VEC ? 4 : 1;
  const size_t total = (size_t)a.M * a.N;
  unsigned long long best = 0ull;
  const size_t it_first = ARGMAX ? (size_t)blockIdx.y * a.N + (blockIdx.x * (size_t)256 + threadIdx.x) * W
                                 : (blockIdx.x * (size_t)256 + threadIdx.x) * W;
  const size_t it_stride = ARGMAX ? total : (size_t)gridDim.x * 256 * W;
  const size_t it_end = ARGMAX ? ((blockIdx.x * (size_t)256 + threadIdx.x) * W < (size_t)a.N ? total : 0) : total;
  for (size_t it = it_first; it < it_end; it += it_stride) {
    const size_t m = it / a.N, nn = it - m * a.N;
    // the sums of squares are requested first, so that they arrive with the partial products
    // (in batches of 8 independent loads: one load per loop pass would cost a cache round trip per split)
    float tot = 0.f;
    if (a.ssq != nullptr) {
      for (int s0 = 0; s0 < a.ksplit; s0 += 8) {
        float q[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) q[u] = a.ssq[(size_t)min(s0 + u, a.ksplit - 1) * a.ssq_ld + m];
#pragma unroll
        for (int u = 0; u < 8; ++u)
          if (s0 + u < a.ksplit) tot += q[u];
      }
    }
    float* y = a.Y + m * a.ldy + nn;
    float4 old = make_float4(0.f, 0.f, 0.f, 0.f);          // residual(s), requested with them
    if (EPI == EPI_ADD && VEC) {
      old = *reinterpret_cast<const float4*>(y);
      if (a.R2 != nullptr) {
        const float4 r2 = *reinterpret_cast<const float4*>(a.R2 + m * a.ldy + nn);
        old.x += r2.x; old.y += r2.y; old.z += r2.z; old.w += r2.w;
      }
    }
    float v[NF][W];
#pragma unroll
    for (int f = 0; f < NF; ++f) {
#pragma unroll
      for (int w = 0; w < W; ++w) v[f][w] = 0.f;
      // 8 splits per pass, their loads issued together; added in split order
      for (int s0 = 0; s0 < a.ksplit; s0 += 8) {
        float4 q[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          const float* src = a.partial + ((size_t)min(s0 + u, a.ksplit - 1) * NF + f) * total + it;
          if (VEC) q[u] = *reinterpret_cast<const float4*>(src);
          else q[u].x = *src;
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          if (s0 + u < a.ksplit) {
            v[f][0] += q[u].x;
            if (VEC) { v[f][1 % W] += q[u].y; v[f][2 % W] += q[u].z; v[f][3 % W] += q[u].w; }
          }
        }
      }
    }
    const float scale = a.ssq != nullptr ? 1.0f / sqrtf(tot * a.rnorm_k + a.eps) : 1.f;
    float o[W];
#pragma unroll
    for (int w = 0; w < W; ++w) {
      o[w] = v[0][w] * scale;
      if (EPI == EPI_SWIGLU) o[w] = o[w] / (1.0f + expf(-o[w])) * (v[NF - 1][w] * scale);
    }
    if (ARGMAX) {
#pragma unroll
      for (int w = 0; w < W; ++w) { const unsigned long long key = argmax_key(o[w], (int)nn + w); if (key > best) best = key; }
    }
    if (VEC) {
      float4 r = make_float4(o[0], o[1 % W], o[2 % W], o[3 % W]);
      if (EPI == EPI_ADD) { r.x += old.x; r.y += old.y; r.z += old.z; r.w += old.w; }
      if (!ARGMAX || a.store) *reinterpret_cast<float4*>(y) = r;
    } else {
      if (EPI == EPI_ADD) o[0] += *y + (a.R2 != nullptr ? a.R2[m * a.ldy + nn] : 0.f);
      if (!ARGMAX || a.store) *y = o[0];
    }
  }
  if (ARGMAX) {
    __shared__ unsigned long long wb[4];
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) { const unsigned long long v = __shfl_xor(best, o, 64); if (v > best) best = v; }
    if ((threadIdx.x & 63) == 0) wb[threadIdx.x >> 6] = best;
    __syncthreads();
    if (threadIdx.x == 0) {
      for (int i = 1; i < 4; ++i) if (wb[i] > best) best = wb[i];
      if (best != 0ull) atomicMax(a.row_best + blockIdx.y, best);
    }
  }
}

template <int EPI>
static hipError_t reduce_launch(const GemmArgs& a, hipStream_t s) {
  const size_t total = (size_t)a.M * a.N;
  const bool vec = a.N % 4 == 0 && a.ldy % 4 == 0;
  if (EPI == EPI_STORE && a.row_best != nullptr) {
    if (a.M > 65535) return hipErrorInvalidValue;
    const int per = vec ? 1024 : 256;
    const dim3 grid((a.N + per - 1) / per, a.M);
    if (vec) hipLaunchKernelGGL((gemm_reduce_kernel<EPI_STORE, true, true>), grid, dim3(256), 0, s, a);
    else hipLaunchKernelGGL((gemm_reduce_kernel<EPI_STORE, false, true>), grid, dim3(256), 0, s, a);
    return hipGetLastError();
  }
  const size_t items = vec ? total / 4 : total;
  const int rb = (int)((items + 255) / 256 < 2048 ? (items + 255) / 256 : 2048);
  if (vec) hipLaunchKernelGGL((gemm_reduce_kernel<EPI, true>), dim3(rb), dim3(256), 0, s, a);
  else hipLaunchKernelGGL((gemm_reduce_kernel<EPI, false>), dim3(rb), dim3(256), 0, s, a);
  return hipGetLastError();
}

size_t gemm_planes_elems(int M, int K) {
  const size_t Mp = ((size_t)M + 15) / 16 * 16, Kp = ((size_t)K + 31) / 32 * 32;
  return 3 * Mp * Kp;
}
// float elements of scratch for the partial products of split-K launches
size_t gemm_partial_elems() { return (size_t)24 << 20; }

// The LDS-staged kernel with MTW row tiles per wavefront (2 MTW per workgroup)
template <int EPI, int MTW>
static hipError_t lds_launch_m(const LdsGemmArgs& a, hipStream_t s) {
  auto kern = gemm_lds_kernel<EPI, MTW>;
  static bool enabled = false;
  if (!enabled) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, lds_stages(MTW) * lds_stage_bytes(MTW));
    if (e != hipSuccess) return e;
    enabled = true;
  }
  hipLaunchKernelGGL(kern, dim3(a.n_blocks * a.m_blocks * a.ksplit), dim3(64 * kLdsWaves), lds_stages(MTW) * lds_stage_bytes(MTW), s, a);
  return hipGetLastError();
}
template <int EPI>
static hipError_t lds_launch(const LdsGemmArgs& a, int mtw, hipStream_t s) {
  switch (mtw) {
    case 1: return lds_launch_m<EPI, 1>(a, s);
    case 2: return lds_launch_m<EPI, 2>(a, s);
    case 3: return lds_launch_m<EPI, 3>(a, s);
    case 6: return lds_launch_m<EPI, 6>(a, s);
  }
  return hipErrorInvalidValue;
}

template <int EPI, int NT, int MTW>
static hipError_t gemm_launch(const GemmArgs& a, int units, hipStream_t s) {
  if (a.terms == 3) hipLaunchKernelGGL((gemm_tiled_kernel<EPI, NT, MTW, 3>), dim3((units + 3) / 4), dim3(256), 0, s, a);
  else hipLaunchKernelGGL((gemm_tiled_kernel<EPI, NT, MTW, 2>), dim3((units + 3) / 4), dim3(256), 0, s, a);
  return hipGetLastError();
}
template <int EPI, int NT>
static hipError_t gemm_dispatch_m(const GemmArgs& a, int mtw, int units, hipStream_t s) {
  switch (mtw) {
    case 1: return gemm_launch<EPI, NT, 1>(a, units, s);
    case 2: return gemm_launch<EPI, NT, 2>(a, units, s);
    case 3: return gemm_launch<EPI, NT, 3>(a, units, s);
    case 4: return gemm_launch<EPI, NT, 4>(a, units, s);
    case 5: return gemm_launch<EPI, NT, 5>(a, units, s);
  }
  return hipErrorInvalidValue;
}

// Row tiles per wavefront (workgroup = 256 weight rows x 32 MTW activation rows) and K split of the
// LDS-staged kernel, by a cost model in microseconds: a workgroup step takes the longer of its MFMAs
// (384 MTW cycles per SIMD) and its copies ((16 + 6 MTW) KB at 28 bytes per cycle and compute unit);
// the workgroups run in rounds of one per compute unit; a K split adds the reduction kernel and
// ks * M * N floats of partial products written and read again (about 4 TB/s).  Up to 96 rows one
// workgroup holds all rows; many rows choose between 192-row and 96-row workgroups.
static void lds_plan(int m_tiles, int steps, int n_blocks, int nf, int M, int N, int& mtw, int& ks) {
  mtw = 0; ks = 1;
  double best = 1e30;
  const int mtw_lo = m_tiles > 6 ? 3 : (m_tiles + 1) / 2, mtw_hi = m_tiles > 6 ? 6 : (m_tiles + 1) / 2;
  for (int cand = mtw_lo; cand <= mtw_hi; cand += 3) {
    const int m_blocks = (m_tiles + lds_row_tiles(cand) - 1) / lds_row_tiles(cand);
    const double mfma = 384.0 * cand, copy = (16.0 + 6.0 * cand) * 1024.0 / 28.0;
    const double step_us = (mfma > copy ? mfma : copy) / 2400.0;
    const int min_steps = m_tiles > 6 ? 8 : 3;
    for (int k = 1; k <= 32; ++k) {
      if (k > 1 && (steps / k < min_steps || (size_t)k * nf * M * N > gemm_partial_elems())) break;
      const int ksteps = (steps + k - 1) / k, kk = (steps + ksteps - 1) / ksteps;
      const long wgs = (long)n_blocks * m_blocks * kk;
      const double rounds = (double)((wgs + 255) / 256);
      double t = rounds * (ksteps + 3) * step_us;
      if (kk > 1) t += 3.0 + (double)kk * nf * M * N * 8.0 / 4e6;
      if (t < best) { best = t; mtw = cand; ks = kk; }
    }
  }
}

static bool lds_path(const GemvArgs& g, int m_tiles) { return (m_tiles > 6 || (g.flags & HH_KF_ROWS_LDS)) && gemm_terms(g.M) == 3; }

bool gemm_hands_over_planes(const GemvArgs& g) {
  if (!g.bf16 || g.n_seg != 1 || g.epi != EPI_SWIGLU || g.seg[0].P == nullptr || g.seg[0].P2 == nullptr || g.K % 8 != 0 || g.K < 8) return false;
  const int M = g.M, N = g.seg[0].n_rows, m_tiles = (M + 15) / 16, steps = (g.K + 31) / 32, tiles = (N + 15) / 16;
  if (M <= 0 || N <= 0 || N % 32 != 0 || !lds_path(g, m_tiles)) return false;
  int mtw = 0, ks = 1;
  lds_plan(m_tiles, steps, (tiles + kLdsA / 2 - 1) / (kLdsA / 2), 2, M, N, mtw, ks);
  return ks == 1;
}

// Y (op)= norm(X) * W^T on the matrix cores.  `planes` is scratch of gemm_planes_elems(M, K) bf16,
// `partial` of gemm_partial_elems() floats; the weights are the packed tiles (seg[0].P / P2).
hipError_t launch_gemm_mfma(const GemvArgs& g, uint16_t* planes, float* partial, hipStream_t s) {
  if (!g.bf16 || g.n_seg != 1 || g.K % 8 != 0 || g.K < 8 || g.seg[0].P == nullptr) return hipErrorInvalidValue;
  const int M = g.M, K = g.K, N = g.seg[0].n_rows;
  if (M <= 0 || N <= 0) return hipSuccess;
  const int Mp = (M + 15) / 16 * 16, Kp = (K + 31) / 32 * 32;
  const bool vec = K % 8 == 0 && g.ldx % 4 == 0 && (reinterpret_cast<uintptr_t>(g.X) & 15) == 0 &&
                   (g.X2 == nullptr || (reinterpret_cast<uintptr_t>(g.X2) & 15) == 0) &&
                   (g.norm_w == nullptr || (reinterpret_cast<uintptr_t>(g.norm_w) & 15) == 0);
  hipError_t e = hipSuccess;
  if (g.planes_in != nullptr) {
    if (g.norm_w != nullptr || g.X2 != nullptr) return hipErrorInvalidValue;   // the producer wrote the operand as it is multiplied
    planes = const_cast<uint16_t*>(g.planes_in);
  } else {
    if (vec && M >= 256 && gemm_terms(M) == 3) {
      // tile-wise; column slices so that about 256 workgroups run where the row tiles alone are fewer
      const int tiles = Mp / 16, iters = (Kp + 511) / 512;
      int slices = (256 + tiles - 1) / tiles;
      if (slices > iters) slices = iters;
      const int per = (iters + slices - 1) / slices;
      slices = (iters + per - 1) / per;
      hipLaunchKernelGGL(split_tiles_kernel, dim3(tiles, slices), dim3(1024), 0, s, g.X, g.X2, g.ldx, M, K, Kp, g.norm_w, g.eps, planes, per * 512);
    } else if (vec) hipLaunchKernelGGL(split_rows_kernel<true>, dim3(Mp), dim3(256), 0, s, g.X, g.X2, g.ldx, M, K, Mp, Kp, g.norm_w, g.eps, planes, gemm_terms(M));
    else hipLaunchKernelGGL(split_rows_kernel<false>, dim3(Mp), dim3(256), 0, s, g.X, g.X2, g.ldx, M, K, Mp, Kp, g.norm_w, g.eps, planes, gemm_terms(M));
    e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  const int nf = g.epi == EPI_SWIGLU ? 2 : 1, nt = nf == 2 ? 2 : 4;
  GemmArgs a{};
  a.planes = planes; a.Mp = Mp; a.Kp = Kp; a.terms = gemm_terms(M);
  a.W = static_cast<const uint16_t*>(g.seg[0].P); a.W2 = static_cast<const uint16_t*>(g.seg[0].P2);
  a.Y = g.seg[0].Y; a.ldy = g.seg[0].ldy; a.R2 = g.R2; a.partial = partial; a.M = M; a.N = N; a.K = K;
  a.row_best = g.epi == EPI_STORE ? g.row_best : nullptr; a.store = g.no_store && a.row_best != nullptr ? 0 : 1;
  const int steps = Kp / 32, tiles = (N + 15) / 16, m_tiles = Mp / 16;
  if (lds_path(g, m_tiles)) {
    LdsGemmArgs l{};
    l.planes = planes; l.m_tiles = m_tiles; l.KST = steps;
    l.W = a.W; l.W2 = a.W2; l.Y = a.Y; l.ldy = a.ldy; l.R2 = a.R2; l.partial = partial;
    l.M = M; l.N = N; l.n_tiles = tiles; l.row_best = a.row_best; l.store = a.store;
    l.n_blocks = (tiles + kLdsA / nf - 1) / (kLdsA / nf);

    int mtw = 0, ks = 1;
    lds_plan(m_tiles, steps, l.n_blocks, nf, M, N, mtw, ks);
    l.m_blocks = (m_tiles + lds_row_tiles(mtw) - 1) / lds_row_tiles(mtw);
    // per-XCD tile ranges where few workgroups share a block of weights (verification: 3 row blocks; measured
    // 63 against 67 us for the down projection of the 3B shape); with the 22 row blocks of a prefill pass the
    // plain numbering is 2.5 % faster (there every XCD reads every weight block either way)
    l.xcd_ranges = l.m_blocks <= 4;
    l.ksteps = (steps + ks - 1) / ks;
    l.ksplit = (steps + l.ksteps - 1) / l.ksteps;
    if (g.planes_out != nullptr) {
      if (!gemm_hands_over_planes(g) || l.ksplit != 1) return hipErrorInvalidValue;
      l.planes_out = g.planes_out; l.out_KST = N / 32;
    }
    switch (g.epi) {
      case EPI_STORE: e = lds_launch<EPI_STORE>(l, mtw, s); break;
      case EPI_ADD: e = lds_launch<EPI_ADD>(l, mtw, s); break;
      case EPI_SWIGLU: e = lds_launch<EPI_SWIGLU>(l, mtw, s); break;
      default: return hipErrorInvalidValue;
    }
    if (e != hipSuccess || l.ksplit == 1) return e;
    a.ksplit = l.ksplit;
    switch (g.epi) {
      case EPI_STORE: return reduce_launch<EPI_STORE>(a, s);
      case EPI_ADD: return reduce_launch<EPI_ADD>(a, s);
      case EPI_SWIGLU: return reduce_launch<EPI_SWIGLU>(a, s);
    }
    return hipErrorInvalidValue;
  }
  a.strip_groups = (tiles + nt - 1) / nt;
  // row tiles per unit: 5 with two terms; 4 with three (5 would spill under the two-workgroups-per-CU register cap)
  const int mtw_cap = a.terms == 3 ? 4 : 5;
  a.m_groups = (m_tiles + mtw_cap - 1) / mtw_cap;
  const int mtw = (m_tiles + a.m_groups - 1) / a.m_groups;
  // K split: enough units (wavefronts) to cover the chip, at least 4 steps each, partial buffer permitting
  constexpr int unit_target = 2048;
  int ksplit = 1;
  while (a.strip_groups * a.m_groups * ksplit * 2 <= unit_target && steps / (ksplit * 2) >= 4 &&
         (size_t)(ksplit * 2) * nf * M * N <= gemm_partial_elems())
    ksplit *= 2;
  a.ksplit = ksplit;
  a.ksteps = (steps + ksplit - 1) / ksplit;
  const int units = a.strip_groups * a.m_groups * ksplit;
  switch (g.epi) {
    case EPI_STORE: e = gemm_dispatch_m<EPI_STORE, 4>(a, mtw, units, s); break;
    case EPI_ADD: e = gemm_dispatch_m<EPI_ADD, 4>(a, mtw, units, s); break;
    case EPI_SWIGLU: e = gemm_dispatch_m<EPI_SWIGLU, 2>(a, mtw, units, s); break;
    default: return hipErrorInvalidValue;
  }
  if (e != hipSuccess || ksplit == 1) return e;
  switch (g.epi) {
    case EPI_STORE: return reduce_launch<EPI_STORE>(a, s);
    case EPI_ADD: return reduce_launch<EPI_ADD>(a, s);
    case EPI_SWIGLU: return reduce_launch<EPI_SWIGLU>(a, s);
  }
  return hipErrorInvalidValue;
}

// Sum of `ksplit` partial products [ksplit][NF][M][N] in order + norm scale + epilogue, for the K
// windows of the in-kernel-split products.  ssq: per-window sums of squares [ksplit][ssq_ld] of the
// activation rows, or nullptr (no norm).
hipError_t launch_gemm_reduce(int epi, float* partial, int ksplit, int M, int N, float* Y, int ldy, const float* R2,
                              const float* ssq, int ssq_ld, float rnorm_k, float eps, unsigned long long* row_best, int store,
                              hipStream_t s) {
  if (ssq != nullptr && M > ssq_ld) return hipErrorInvalidValue;
  GemmArgs a{};
  a.partial = partial; a.ksplit = ksplit; a.M = M; a.N = N; a.Y = Y; a.ldy = ldy; a.R2 = R2;
  a.ssq = ssq; a.ssq_ld = ssq_ld; a.rnorm_k = rnorm_k; a.eps = eps;
  a.row_best = epi == EPI_STORE ? row_best : nullptr; a.store = a.row_best != nullptr ? store : 1;
  switch (epi) {
    case EPI_STORE: return reduce_launch<EPI_STORE>(a, s);
    case EPI_ADD: return reduce_launch<EPI_ADD>(a, s);
    case EPI_SWIGLU: return reduce_launch<EPI_SWIGLU>(a, s);
  }
  return hipErrorInvalidValue;
}

}  // namespace hh
