// Dense projections on the matrix cores, for passes with more than a handful of activation
// rows (batched drafting, batched verification, prefill): Y[M x N] = X'[M x K] * W[N x K]^T with
// bf16 weights.
//
// Activations stay float32-accurate: a first kernel applies the fused RMSNorm and splits every
// value into three bf16 terms, x = t0 + t1 + t2 exactly (8 + 8 + 8 mantissa bits); the product
// is the sum of three bf16 MFMA products accumulated in float32.  While the pass is bound by
// streaming the weights the two extra MFMAs per weight fragment are free.
//
// GEMM kernel: a workgroup owns a strip of 16 output columns (16 gate + 16 up columns for
// SwiGLU) and up to 128 activation rows; its wavefronts split K.  Per step of 32 columns of K a
// wavefront loads its weight fragment straight from global memory into registers (v_mfma_f32_16x16x32_bf16 B operand:
// lane l holds W[n0 + l%16][k0 + 8*(l/16) .. +7], one 16-byte load) and reuses them for every
// 16-row tile and every split term of the activations (A operand: lane l holds
// A[m0 + l%16][k0 + 8*(l/16) .. +7], read from the split planes through L1/L2).  No LDS.
// Accumulator layout: lane l holds C[4*(l/16) + r][l%16], r = 0..3.
#include "hh_internal.h"

namespace hh {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

static constexpr int kTiles = 8;   // 16-row tiles per launch (128 activation rows)

__device__ __forceinline__ uint16_t bf16_rne(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}
__device__ __forceinline__ float bf16_f32(uint16_t h) { return __uint_as_float((uint32_t)h << 16); }

// planes [3][Mp][Kp] bf16; rows >= M and columns >= K are zero
__global__ __launch_bounds__(256) void split_rows_kernel(const float* __restrict__ X, int ldx, int M, int K, int Mp, int Kp,
                                                         const float* __restrict__ norm_w, float eps,
                                                         uint16_t* __restrict__ planes) {
  const int m = blockIdx.x;
  __shared__ float red[4];
  float rstd = 1.f;
  if (m < M && norm_w != nullptr) {
    float ss = 0.f;
    for (int k = threadIdx.x; k < K; k += 256) { const float v = X[(size_t)m * ldx + k]; ss = fmaf(v, v, ss); }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) ss += __shfl_xor(ss, o, 64);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
    __syncthreads();
    rstd = 1.0f / sqrtf((red[0] + red[1] + red[2] + red[3]) / (float)K + eps);
  }
  const size_t plane = (size_t)Mp * Kp;
  for (int k = threadIdx.x; k < Kp; k += 256) {
    uint16_t t0 = 0, t1 = 0, t2 = 0;
    if (m < M && k < K) {
      float v = X[(size_t)m * ldx + k];
      if (norm_w != nullptr) v = v * norm_w[k] * rstd;
      t0 = bf16_rne(v);
      const float r1 = v - bf16_f32(t0);
      t1 = bf16_rne(r1);
      const float r2 = r1 - bf16_f32(t1);
      t2 = bf16_rne(r2);
    }
    const size_t at = (size_t)m * Kp + k;
    planes[at] = t0; planes[plane + at] = t1; planes[2 * plane + at] = t2;
  }
}

struct GemmArgs {
  const uint16_t* planes; int Mp, Kp;     // split activations
  const uint16_t* W; const uint16_t* W2;  // [N][K] bf16 (W2: the "up" matrix for SwiGLU)
  float* Y; int ldy;
  int M, N, K, m0, mt;                    // rows m0 .. m0 + 16*mt of the planes in this launch
  int ksteps;                             // steps of 32 columns per wavefront (K split over the workgroup)
};

static constexpr int kGroupK = 2;   // weight fragments loaded ahead, in steps of 32 columns

// One workgroup per strip of 16 output columns; its KS wavefronts split K between them and add
// their partial tiles through LDS.  Small per-wavefront work, many wavefronts: the weights of a
// wavefront's K slice are requested up to 8 steps ahead.
template <int EPI>
__global__ __launch_bounds__(512) void gemm_mfma_kernel(const GemmArgs a) {
  constexpr int NF = EPI == EPI_SWIGLU ? 2 : 1;
  extern __shared__ __align__(16) float red[];   // [KS][mt][NF][64][4]
  const int lane = threadIdx.x & 63;
  const int ks = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int KS = blockDim.x >> 6;
  const int i = lane & 15, g = lane >> 4;
  const int n0 = blockIdx.x * 16;
  const size_t wr = (size_t)min(n0 + i, a.N - 1) * a.K;
  const uint16_t* wrow[2] = {a.W + wr, EPI == EPI_SWIGLU ? a.W2 + wr : a.W + wr};
  const size_t plane = (size_t)a.Mp * a.Kp;
  const uint16_t* arow = a.planes + (size_t)(a.m0 + i) * a.Kp + g * 8;
  const int kbeg = ks * a.ksteps * 32, kend = min(a.Kp, kbeg + a.ksteps * 32);

  f32x4 acc[kTiles][NF];
#pragma unroll
  for (int t = 0; t < kTiles; ++t)
#pragma unroll
    for (int f = 0; f < NF; ++f) acc[t][f] = f32x4{0.f, 0.f, 0.f, 0.f};

  for (int kg = kbeg; kg < kend; kg += 32 * kGroupK) {
    bf16x8 bw[kGroupK][NF];
#pragma unroll
    for (int u = 0; u < kGroupK; ++u) {
      const int kb = min(kg + u * 32 + g * 8, a.K - 8);   // past K: clamped, meets zero activations
#pragma unroll
      for (int f = 0; f < NF; ++f) bw[u][f] = *reinterpret_cast<const bf16x8*>(wrow[f] + kb);
    }
#pragma unroll
    for (int u = 0; u < kGroupK; ++u) {
      const int k0 = kg + u * 32;
      if (k0 < kend) {
#pragma unroll
        for (int t = 0; t < kTiles; ++t) {
          if (t < a.mt) {
            const uint16_t* ap = arow + (size_t)t * 16 * a.Kp + k0;
#pragma unroll
            for (int term = 0; term < 3; ++term) {
              const bf16x8 av = *reinterpret_cast<const bf16x8*>(ap + term * plane);
#pragma unroll
              for (int f = 0; f < NF; ++f)
                acc[t][f] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, bw[u][f], acc[t][f], 0, 0, 0);
            }
          }
        }
      }
      // keep the activation loads of later steps from being hoisted above this step's MFMAs
      // (hoisting all of them exhausts the register file)
      __builtin_amdgcn_sched_barrier(0);
    }
  }

  // ---- add the partial tiles of the KS wavefronts; wavefront ks finishes tiles ks, ks+KS, ...
  if (KS > 1) {
#pragma unroll
    for (int t = 0; t < kTiles; ++t)
      if (t < a.mt)
#pragma unroll
        for (int f = 0; f < NF; ++f)
          *reinterpret_cast<f32x4*>(&red[((((size_t)ks * a.mt + t) * NF + f) * 64 + lane) * 4]) = acc[t][f];
    __syncthreads();
  }
#pragma unroll
  for (int t = 0; t < kTiles; ++t) {
    if (t < a.mt && (KS == 1 || t % KS == ks)) {
      f32x4 sum[NF];
#pragma unroll
      for (int f = 0; f < NF; ++f) {
        if (KS == 1) sum[f] = acc[t][f];
        else {
          sum[f] = f32x4{0.f, 0.f, 0.f, 0.f};
          for (int j = 0; j < KS; ++j)
            sum[f] += *reinterpret_cast<const f32x4*>(&red[((((size_t)j * a.mt + t) * NF + f) * 64 + lane) * 4]);
        }
      }
      const int n = n0 + i;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int m = a.m0 + t * 16 + g * 4 + r;
        if (m < a.M && n < a.N) {
          float* y = a.Y + (size_t)m * a.ldy + n;
          if (EPI == EPI_SWIGLU) {
            const float gt = sum[0][r], up = sum[NF - 1][r];
            *y = gt / (1.0f + expf(-gt)) * up;
          } else {
            *y = EPI == EPI_ADD ? *y + sum[0][r] : sum[0][r];
          }
        }
      }
    }
  }
}

size_t gemm_planes_elems(int M, int K) {
  const size_t Mp = ((size_t)M + 15) / 16 * 16, Kp = ((size_t)K + 31) / 32 * 32;
  return 3 * Mp * Kp;
}

// Y (op)= norm(X) * W^T on the matrix cores.  `planes` is scratch of gemm_planes_elems(M, K) bf16.
hipError_t launch_gemm_mfma(const GemvArgs& g, uint16_t* planes, hipStream_t s) {
  if (!g.bf16 || g.n_seg != 1 || g.K % 8 != 0 || g.K < 8) return hipErrorInvalidValue;
  const int M = g.M, K = g.K, N = g.seg[0].n_rows;
  if (M <= 0 || N <= 0) return hipSuccess;
  const int Mp = (M + 15) / 16 * 16, Kp = (K + 31) / 32 * 32;
  hipLaunchKernelGGL(split_rows_kernel, dim3(Mp), dim3(256), 0, s, g.X, g.ldx, M, K, Mp, Kp, g.norm_w, g.eps, planes);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  GemmArgs a{};
  a.planes = planes; a.Mp = Mp; a.Kp = Kp;
  a.W = static_cast<const uint16_t*>(g.seg[0].W); a.W2 = static_cast<const uint16_t*>(g.seg[0].W2);
  a.Y = g.seg[0].Y; a.ldy = g.seg[0].ldy; a.M = M; a.N = N; a.K = K;
  const int strips = (N + 15) / 16, nf = g.epi == EPI_SWIGLU ? 2 : 1, steps = Kp / 32;
  for (int m0 = 0; m0 < Mp; m0 += 16 * kTiles) {
    a.m0 = m0;
    a.mt = (Mp - m0) / 16 < kTiles ? (Mp - m0) / 16 : kTiles;
    // K split: enough wavefronts to cover the chip, bounded by the steps available and by the
    // LDS the partial tiles need (1 KB per wavefront, tile and fragment)
    int KS = 1;
    while (KS < 8 && strips * KS < 1024 && steps / (KS * 2) >= 2 && (size_t)KS * 2 * a.mt * nf * 1024 <= 96 * 1024) KS *= 2;
    a.ksteps = (steps + KS - 1) / KS;
    const size_t lds = KS > 1 ? (size_t)KS * a.mt * nf * 1024 : 0;
#define HH_GEMM_LAUNCH(E)                                                                              \
    {                                                                                                  \
      auto kern = gemm_mfma_kernel<E>;                                                                 \
      static size_t lds_enabled = 48 * 1024;                                                           \
      if (lds > lds_enabled) {                                                                         \
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),                                   \
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);                 \
        if (e != hipSuccess) return e;                                                                 \
        lds_enabled = lds;                                                                             \
      }                                                                                                \
      hipLaunchKernelGGL(kern, dim3(strips), dim3(64 * KS), lds, s, a);                                \
    }
    switch (g.epi) {
      case EPI_STORE: HH_GEMM_LAUNCH(EPI_STORE) break;
      case EPI_ADD: HH_GEMM_LAUNCH(EPI_ADD) break;
      case EPI_SWIGLU: HH_GEMM_LAUNCH(EPI_SWIGLU) break;
      default: return hipErrorInvalidValue;
    }
#undef HH_GEMM_LAUNCH
    e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

// argmax of each row of logits [M][ld] (largest value, lowest index on ties):
// row m = b*T + j -> out[b*out_stride + out_off + j]
__global__ __launch_bounds__(256) void argmax_rows_kernel(const float* __restrict__ logits, int ld, int V, int* out,
                                                          int out_stride, int out_off, int T) {
  const int m = blockIdx.x;
  const float* row = logits + (size_t)m * ld;
  float bv = -INFINITY;
  int bi = 0x7fffffff;
  for (int n = threadIdx.x; n < V; n += 256) {
    const float v = row[n];
    if (v > bv) { bv = v; bi = n; }   // strided ascending n per thread: first maximum kept
  }
  __shared__ float sv[256];
  __shared__ int si[256];
  sv[threadIdx.x] = bv; si[threadIdx.x] = bi;
  __syncthreads();
  for (int o = 128; o > 0; o >>= 1) {
    if ((int)threadIdx.x < o) {
      const float v2 = sv[threadIdx.x + o];
      const int i2 = si[threadIdx.x + o];
      if (v2 > sv[threadIdx.x] || (v2 == sv[threadIdx.x] && i2 < si[threadIdx.x])) { sv[threadIdx.x] = v2; si[threadIdx.x] = i2; }
    }
    __syncthreads();
  }
  if (threadIdx.x == 0) out[(size_t)(m / T) * out_stride + out_off + m % T] = si[0];
}

hipError_t launch_argmax_rows(const float* logits, int ld, int V, int M, int* out, int out_stride, int out_off, int T,
                              hipStream_t s) {
  hipLaunchKernelGGL(argmax_rows_kernel, dim3(M), dim3(256), 0, s, logits, ld, V, out, out_stride, out_off, T);
  return hipGetLastError();
}

}  // namespace hh
