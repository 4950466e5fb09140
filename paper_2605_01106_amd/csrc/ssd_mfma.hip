// SSM branch of a pass with many positions per sequence (prefill chunks) in the matmul
// ("state-space dual") form, on the matrix cores in float32.
//
// The scalar-decay recurrence  S_t = a_t S_{t-1} + dt_t x_t (outer) B_t,  y_t = S_t C_t + D x_t
// over a chunk of L positions with the state S entering it is, with cum_t = sum_{i<=t} log a_i,
//     y_t = exp(cum_t) * (S C_t)  +  sum_{i<=t} [ (C_t . B_i) * exp(cum_t - cum_i) * dt_i ] x_i  +  D x_t
//     S'  = exp(cum_L) * S        +  sum_i  exp(cum_L - cum_i) * dt_i * x_i (outer) B_i
// - four small matrix products per chunk instead of L dependent state updates.  All exponents are
// <= 0, so nothing overflows whatever the decay.  Products are v_mfma_f32_16x16x4_f32 (exact
// float32 products, float32 accumulation): the rounding differs from the sequential kernels only
// in the order of the sums.
//
// One workgroup of four wavefronts per (sequence, head), head dimension P = 64; wavefront w owns
// the 16 rows p = 16 w .. 16 w + 15 of the head for everything - its slice of the state, transposed
// (n down, p across), lives in MFMA accumulator registers for the whole pass and is fed back as
// the A operand of the read-out product as it is: lane (g, j) holds S[p = 16 w + j][n = 16 tile +
// 4 g + r], which the instruction takes as A[row j][k = g] when the B operand is read with the same
// n for k = g.  Per chunk of 32 positions: the convolution + SiLU of x, B, C (a thread walks 4
// channels through the positions with a sliding window of raw rows), the step sizes and their
// running sum, then  G = C B^T  (three 16 x 16 tiles at or below the diagonal), the masked and
// scaled M to LDS, the read-out of the old state, the intra-chunk product M x, the outputs
// y * silu(z), and the state update.  B is kept row-major and C transposed in LDS, padded so
// that the operand reads of the two large products are free of bank conflicts.
#include <stdlib.h>

#include "hh_internal.h"
#include "wave_ops.h"
#include "trace.h"

namespace hh {

typedef float ssd_f32x4 __attribute__((ext_vector_type(4)));

static constexpr int kSsdL = 32;    // positions per chunk
static constexpr int kSsdP = 64;    // head dimension

__device__ __forceinline__ float ssd_silu(float v) { return v * __frcp_rn(1.0f + __expf(-v)); }
__device__ __forceinline__ float ssd_softplus(float v) { return v > 20.0f ? v : log1pf(expf(v)); }

template <int N>
struct SsdLds {
  static constexpr int LDB = N + 16, LDT = kSsdL + 4, LDX = kSsdP + 16, LDM = kSsdL + 4;
  static constexpr int kB = 0;                         // B  [L][LDB]   (position, n)
  static constexpr int kCt = kB + kSsdL * LDB;         // C^T [N][LDT]  (n, position)
  static constexpr int kX = kCt + N * LDT;             // x  [L][LDX]   (position, p)
  static constexpr int kM = kX + kSsdL * LDX;          // M  [L][LDM]   (t, i)
  static constexpr int kDt = kM + kSsdL * LDM;         // dt_i
  static constexpr int kCum = kDt + kSsdL;             // cum_i
  static constexpr int kFloats = kCum + kSsdL;
};

template <int N>
__global__ __launch_bounds__(256) void ssd_mfma_kernel(const Dims d, const SsmArgs a) {
  typedef SsdLds<N> Lds;
  constexpr int L = kSsdL, P = kSsdP, NT = N / 16;
  constexpr int LDB = Lds::LDB, LDT = Lds::LDT, LDX = Lds::LDX, LDM = Lds::LDM;
  constexpr int NG = (P + 2 * N) / 4;                  // conv channel groups of 4: x | B | C
  static_assert(NG <= 192, "the staging threads are the first three wavefronts");
  extern __shared__ __align__(16) float ssd_smem[];
  float* Bs = ssd_smem + Lds::kB;
  float* Ct = ssd_smem + Lds::kCt;
  float* Xs = ssd_smem + Lds::kX;
  float* Ms = ssd_smem + Lds::kM;
  float* dts = ssd_smem + Lds::kDt;
  float* cums = ssd_smem + Lds::kCum;

  const int tid = threadIdx.x, lane = tid & 63, w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int g = lane >> 4, j = lane & 15;
  const int h = blockIdx.x, b = blockIdx.y;
  const LayerDev& ly = a.one;
  int nt = a.T;
  if (a.n_tok != nullptr) nt = a.n_tok[b];
  if (nt <= 0) return;
  const int pos0 = a.pos0[b];
  const int rmask = d.ring_slots - 1;
  float* ring = ly.ring + (size_t)b * d.ring_slots * d.ring_w;
  const float* zx = a.zx + (size_t)b * a.T * d.ldzx;

  // ---- state slice of this wavefront, transposed: acc[tile][r] = S[16 w + j][16 tile + 4 g + r]
  ssd_f32x4 S[NT];
  {
    const float* src = a.state_in == 0 ? ly.S : (a.state_in == 1 ? ly.S_draft : nullptr);
    if (src != nullptr) {
      const float* sp = src + (((size_t)b * d.Hm + h) * P + 16 * w + j) * N + 4 * g;
#pragma unroll
      for (int t = 0; t < NT; ++t) {
        const float4 v = *reinterpret_cast<const float4*>(sp + 16 * t);
        S[t] = ssd_f32x4{v.x, v.y, v.z, v.w};
      }
    } else {
#pragma unroll
      for (int t = 0; t < NT; ++t) S[t] = ssd_f32x4{0.f, 0.f, 0.f, 0.f};
    }
  }
  const float dskip = ly.d_skip[h], dtb = ly.dt_bias[h], negA = -expf(ly.a_log[h]);

  // ---- staging role: thread q < NG owns 4 conv channels
  const bool stager = tid < NG;
  int ch = 0;                                          // first of the 4 channels (index into xBC)
  if (stager) ch = tid < P / 4 ? h * P + 4 * tid : d.d_inner + 4 * (tid - P / 4);
  float4 tw[4], bias = make_float4(0.f, 0.f, 0.f, 0.f), r0, r1, r2;
  // raw xBC row of a position: this pass's projections, or the ring for the three positions before it
  auto raw_row = [&](int pos) -> float4 {
    if (pos < 0) return make_float4(0.f, 0.f, 0.f, 0.f);
    const float* p = pos >= pos0 ? zx + (size_t)(pos - pos0) * d.ldzx + d.d_inner + ch : ring + (size_t)(pos & rmask) * d.ring_w + ch;
    return *reinterpret_cast<const float4*>(p);
  };
  if (stager) {
#pragma unroll
    for (int q = 0; q < 4; ++q) tw[q] = *reinterpret_cast<const float4*>(ly.conv_w + (size_t)(ch + q) * 4);
    bias = *reinterpret_cast<const float4*>(ly.conv_b + ch);
    r0 = raw_row(pos0 - 3); r1 = raw_row(pos0 - 2); r2 = raw_row(pos0 - 1);
  }

  TR(0);
  for (int j0 = 0; j0 < nt; j0 += L) {
    const int tc = min(L, nt - j0);
    if (j0 == 0) TR(1);
    // ================= staging: conv + SiLU of x, B, C; dt and its running log-decay sum
    if (stager) {
#pragma unroll 1
      for (int jb = 0; jb < L; jb += 8) {
        float4 cur[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) cur[u] = raw_row(pos0 + j0 + min(jb + u, tc - 1));   // (clamped: loads stay inside this pass)
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          const int jj = jb + u;
          const bool on = jj < tc;
          const float4 c4 = cur[u];
          float o[4];
          const float x0[4] = {r0.x, r0.y, r0.z, r0.w}, x1[4] = {r1.x, r1.y, r1.z, r1.w}, x2[4] = {r2.x, r2.y, r2.z, r2.w},
                      x3[4] = {c4.x, c4.y, c4.z, c4.w}, bq[4] = {bias.x, bias.y, bias.z, bias.w};
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            float acc = tw[q].x * x0[q];
            acc = fmaf(tw[q].y, x1[q], acc); acc = fmaf(tw[q].z, x2[q], acc); acc = fmaf(tw[q].w, x3[q], acc);
            o[q] = on ? ssd_silu(acc + bq[q]) : 0.f;
          }
          if (tid < P / 4) {
            *reinterpret_cast<float4*>(Xs + jj * LDX + 4 * tid) = make_float4(o[0], o[1], o[2], o[3]);
          } else if (tid < P / 4 + N / 4) {
            *reinterpret_cast<float4*>(Bs + jj * LDB + 4 * (tid - P / 4)) = make_float4(o[0], o[1], o[2], o[3]);
          } else {
            const int n0 = 4 * (tid - P / 4 - N / 4);
#pragma unroll
            for (int q = 0; q < 4; ++q) Ct[(n0 + q) * LDT + jj] = o[q];
          }
          if (on) {
            // the raw inputs stay in the ring for the next pass's window and for rollbacks (x of this
            // head by every workgroup, B and C by the workgroup of head 0)
            if (a.write_ring && (tid < P / 4 || h == 0))
              *reinterpret_cast<float4*>(ring + (size_t)((pos0 + j0 + jj) & rmask) * d.ring_w + ch) = c4;
            r0 = r1; r1 = r2; r2 = c4;
          }
        }
      }
    } else if (w == 3 && lane < L) {
      const bool on = lane < tc;
      const float rawdt = zx[(size_t)(j0 + min(lane, tc - 1)) * d.ldzx + d.d_inner + d.conv_dim + h];
      const float dt = on ? ssd_softplus(rawdt + dtb) : 0.f;
      if (on && a.write_ring) ring[(size_t)((pos0 + j0 + lane) & rmask) * d.ring_w + d.conv_dim + h] = rawdt;
      float c = negA * dt;                             // log a_t, summed over the positions up to t
#pragma unroll
      for (int o = 1; o < L; o <<= 1) {
        const float up = __shfl_up(c, o, 64);
        if (lane >= o) c += up;
      }
      dts[lane] = dt;
      cums[lane] = c;
    }
    __syncthreads();
    if (j0 == 0) TR(2);

    // ================= G = C B^T on the tiles at or below the diagonal, M = G * decay * dt to LDS
    {
      const int tt = w == 0 ? 0 : 1, it = w == 2 ? 1 : 0;          // wavefront 3: the tile above the diagonal is zero
      ssd_f32x4 G = {0.f, 0.f, 0.f, 0.f};
      if (w < 3) {
#pragma unroll 4
        for (int kk = 0; kk < N / 4; ++kk) {
          const float av = Ct[(4 * kk + g) * LDT + 16 * tt + j];   // A[row t = j][k = g] = C[t][n = 4 kk + g]
          const float bv = Bs[(16 * it + j) * LDB + 4 * kk + g];   // B[k = g][col i = j] = B[i][n = 4 kk + g]
          G = __builtin_amdgcn_mfma_f32_16x16x4f32(av, bv, G, 0, 0, 0);
        }
      }
      // lane (g, j) holds G[t = 16 tt' + 4 g + r][i = 16 it' + j]
      const int tt_w = w == 3 ? 0 : tt, it_w = w == 3 ? 1 : it;
      const int i = 16 * it_w + j;
      const float ci = cums[i], di = dts[i];
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int t = 16 * tt_w + 4 * g + r;
        const float m = (w < 3 && i <= t) ? G[r] * di * expf(cums[t] - ci) : 0.f;
        Ms[t * LDM + i] = m;
      }
    }
    __syncthreads();
    if (j0 == 0) TR(3);

    // ================= read-out of the entering state, intra-chunk product, outputs
    ssd_f32x4 Y[2] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};   // Y[tt][r] = y[p = 16 w + 4 g + r][t = 16 tt + j]
#pragma unroll
    for (int t = 0; t < NT; ++t) {
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const float* crow = Ct + (16 * t + 4 * g + r) * LDT + j;   // B[k = g][col j] = C[position][n = 16 t + 4 g + r]
        Y[0] = __builtin_amdgcn_mfma_f32_16x16x4f32(S[t][r], crow[0], Y[0], 0, 0, 0);
        Y[1] = __builtin_amdgcn_mfma_f32_16x16x4f32(S[t][r], crow[16], Y[1], 0, 0, 0);
      }
    }
    {
      const float e0 = expf(cums[j]), e1 = expf(cums[16 + j]);
#pragma unroll
      for (int r = 0; r < 4; ++r) { Y[0][r] *= e0; Y[1][r] *= e1; }
    }
#pragma unroll
    for (int kk = 0; kk < L / 4; ++kk) {
      const float xv = Xs[(4 * kk + g) * LDX + 16 * w + j];        // A[row p = j][k = g] = x[i = 4 kk + g][p]
      if (kk < 4) Y[0] = __builtin_amdgcn_mfma_f32_16x16x4f32(xv, Ms[j * LDM + 4 * kk + g], Y[0], 0, 0, 0);
      Y[1] = __builtin_amdgcn_mfma_f32_16x16x4f32(xv, Ms[(16 + j) * LDM + 4 * kk + g], Y[1], 0, 0, 0);
    }
#pragma unroll
    for (int tt = 0; tt < 2; ++tt) {
      const int t = 16 * tt + j;
      if (t < tc) {
        const size_t m = (size_t)b * a.T + j0 + t;
        const int p = 16 * w + 4 * g;
        const float4 xv = *reinterpret_cast<const float4*>(Xs + t * LDX + p);
        const float4 z = *reinterpret_cast<const float4*>(a.zx + m * d.ldzx + h * P + p);
        float4 o;
        o.x = (Y[tt][0] + dskip * xv.x) * ssd_silu(z.x);
        o.y = (Y[tt][1] + dskip * xv.y) * ssd_silu(z.y);
        o.z = (Y[tt][2] + dskip * xv.z) * ssd_silu(z.z);
        o.w = (Y[tt][3] + dskip * xv.w) * ssd_silu(z.w);
        *reinterpret_cast<float4*>(a.g + m * d.d_inner + h * P + p) = o;
      }
    }

    if (j0 == 0) TR(4);
    // ================= state update: S' = exp(cum_L) S + sum_i w_i x_i (outer) B_i
    {
      const float cl = cums[L - 1], el = expf(cl);
#pragma unroll
      for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int r = 0; r < 4; ++r) S[t][r] *= el;
#pragma unroll
      for (int kk = 0; kk < L / 4; ++kk) {
        const int i = 4 * kk + g;
        const float xw = Xs[i * LDX + 16 * w + j] * (dts[i] * expf(cl - cums[i]));   // B[k = g][col p = j]
        const float* brow = Bs + i * LDB + j;                                        // A[row n = j][k = g] = B[i][n]
#pragma unroll
        for (int t = 0; t < NT; ++t) S[t] = __builtin_amdgcn_mfma_f32_16x16x4f32(brow[16 * t], xw, S[t], 0, 0, 0);
      }
    }
    __syncthreads();
    if (j0 == 0) TR(5);
  }
  TR(6);

  if (a.state_out != 0) {
    float* dp = (a.state_out == 1 ? ly.S : ly.S_draft) + (((size_t)b * d.Hm + h) * P + 16 * w + j) * N + 4 * g;
#pragma unroll
    for (int t = 0; t < NT; ++t) *reinterpret_cast<float4*>(dp + 16 * t) = make_float4(S[t][0], S[t][1], S[t][2], S[t][3]);
  }
  TR(7);
}

template <int N>
static hipError_t ssd_launch(const Dims& d, const SsmArgs& a, hipStream_t s) {
  auto kern = ssd_mfma_kernel<N>;
  constexpr int lds = SsdLds<N>::kFloats * (int)sizeof(float);
  static bool enabled = false;
  if (!enabled && lds > 48 * 1024) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (e != hipSuccess) return e;
    enabled = true;
  }
  hipLaunchKernelGGL(kern, dim3(d.Hm, a.B), dim3(256), lds, s, d, a);
  return hipGetLastError();
}

// true if the pass was taken by the matmul-form kernel: a single layer's pass over this call's
// projections with outputs, at least 16 positions, head dimension 64, state size 64, 128 or 256,
// 16-byte aligned rows
bool launch_ssd_mfma(const Dims& d, const SsmArgs& a, hipStream_t s, hipError_t* err) {
  if ((d.flags & HH_KF_SSM_SEQUENTIAL) || a.layers != nullptr || a.zx == nullptr || a.g == nullptr || a.n_acc != nullptr ||
      a.skip != nullptr || a.T < 16 || d.P != kSsdP || d.d_inner % 4 != 0 || d.ldzx % 4 != 0 || d.ring_w % 4 != 0 ||
      d.conv_dim % 4 != 0 || (reinterpret_cast<uintptr_t>(a.zx) & 15) != 0 || (reinterpret_cast<uintptr_t>(a.g) & 15) != 0)
    return false;
  switch (d.N) {
    case 64: *err = ssd_launch<64>(d, a, s); return true;
    case 128: *err = ssd_launch<128>(d, a, s); return true;
    case 256: *err = ssd_launch<256>(d, a, s); return true;
  }
  return false;
}

}  // namespace hh
