// Skinny GEMM for the dense projections (in/out/QKV/MLP/LM head) when only a few
// rows of activations meet each weight: Y[m][n] = sum_k X'[m][k] * W[n][k].
//
// The weights are streamed from HBM exactly once per launch (16-byte loads, one
// output row per wavefront pass), so the kernel is bound by HBM bandwidth.  The
// activation rows live in LDS in float32 and are never rounded: products of a
// bf16 weight and a float32 activation are accumulated in float32.
//
// Fused around the product:
//   prologue  RMSNorm of the activation row (x / sqrt(mean(x^2)+eps) * w);
//   epilogue  plain store, in-place residual add, SwiGLU (silu(gate) * up with
//             the two matrices paired row by row), and per-block argmax
//             partials for the LM head (largest value, lowest index on ties).
#include "hh_internal.h"

namespace hh {

static constexpr int kThreads = 256;
static constexpr int kWaves = 4;
static constexpr int kMaxBlocks = 2048;

int gemv_max_blocks() { return kMaxBlocks; }

__device__ __forceinline__ float bf16lo(uint32_t v) { return __uint_as_float(v << 16); }
__device__ __forceinline__ float bf16hi(uint32_t v) { return __uint_as_float(v & 0xffff0000u); }

template <int BF16>
__device__ __forceinline__ void load_w8(const void* base, size_t elem, float (&w)[8]) {
  if (BF16) {
    const uint4 v = *reinterpret_cast<const uint4*>(static_cast<const uint16_t*>(base) + elem);
    w[0] = bf16lo(v.x); w[1] = bf16hi(v.x); w[2] = bf16lo(v.y); w[3] = bf16hi(v.y);
    w[4] = bf16lo(v.z); w[5] = bf16hi(v.z); w[6] = bf16lo(v.w); w[7] = bf16hi(v.w);
  } else {
    const float4* p = reinterpret_cast<const float4*>(static_cast<const float*>(base) + elem);
    const float4 a = p[0], b = p[1];
    w[0] = a.x; w[1] = a.y; w[2] = a.z; w[3] = a.w; w[4] = b.x; w[5] = b.y; w[6] = b.z; w[7] = b.w;
  }
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

__device__ __forceinline__ unsigned long long argmax_key(float v, int n) {
  uint32_t u = __float_as_uint(v);
  u = (u & 0x80000000u) ? ~u : (u | 0x80000000u);
  return (static_cast<unsigned long long>(u) << 32) | static_cast<unsigned long long>(0xFFFFFFFFu - (uint32_t)n);
}

// LDS layout of one activation row: the 8 floats a lane multiplies in chunk c
// (k = c*512 + lane*8 + i) are stored as two float4 at [(2c + i/4)*64 + lane],
// so both 16-byte LDS reads of a wavefront are unit-stride across lanes.
__device__ __forceinline__ int xs_index(int k) {
  const int c = k >> 9, r = k & 511, lane = r >> 3, i = r & 7;
  return (((c * 2 + (i >> 2)) * 64 + lane) << 2) + (i & 3);
}

template <int BF16, int MT, int R, int EPI>
__global__ __launch_bounds__(kThreads) void gemv_kernel(const GemvArgs a, const int m0, const int n_total) {
  extern __shared__ __align__(16) float smem[];
  const int K = a.K;
  const int Kpad = (K + 511) & ~511;
  float* xs = smem;                       // [MT][Kpad]
  float* red = smem + (size_t)MT * Kpad;  // [kWaves][MT] + argmax scratch
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int mt = min(MT, a.M - m0);

  // ---- prologue: stage (and normalise) the activation rows
  for (int m = 0; m < MT; ++m) {
    float ss = 0.f;
    if (m < mt) {
      const float* x = a.X + (size_t)(m0 + m) * a.ldx;
      for (int k = tid; k < Kpad; k += kThreads) {
        const float v = k < K ? x[k] : 0.f;
        xs[(size_t)m * Kpad + xs_index(k)] = v;
        ss += v * v;
      }
    } else {
      for (int k = tid; k < Kpad; k += kThreads) xs[(size_t)m * Kpad + xs_index(k)] = 0.f;
    }
    if (a.norm_w != nullptr) {
      ss = wave_sum(ss);
      if (lane == 0) red[wave * MT + m] = ss;
    }
  }
  __syncthreads();
  if (a.norm_w != nullptr) {
    for (int m = 0; m < mt; ++m) {
      float tot = 0.f;
      for (int w = 0; w < kWaves; ++w) tot += red[w * MT + m];
      const float rstd = 1.0f / sqrtf(tot / (float)K + a.eps);
      for (int k = tid; k < K; k += kThreads) {
        float* p = &xs[(size_t)m * Kpad + xs_index(k)];
        *p = *p * rstd * a.norm_w[k];
      }
    }
    __syncthreads();
  }

  unsigned long long best[MT];
#pragma unroll
  for (int m = 0; m < MT; ++m) best[m] = 0ull;

  // ---- main loop: each wavefront owns R output rows per pass
  for (int base = blockIdx.x * (kWaves * R); base < n_total; base += gridDim.x * (kWaves * R)) {
    const void* wp[R];
    const void* wp2[R];
    float* yp[R];
    int ncol[R], ldy[R];
    bool live[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
      int n = base + wave * R + r;
      live[r] = n < n_total;
      if (!live[r]) n = n_total - 1;
      int s = 0;
      while (s + 1 < a.n_seg && n >= a.seg[s].n_rows) { n -= a.seg[s].n_rows; ++s; }
      const size_t esz = BF16 ? 2 : 4;
      wp[r] = static_cast<const char*>(a.seg[s].W) + (size_t)n * K * esz;
      wp2[r] = EPI == EPI_SWIGLU ? static_cast<const char*>(a.seg[s].W2) + (size_t)n * K * esz : nullptr;
      yp[r] = a.seg[s].Y; ncol[r] = n; ldy[r] = a.seg[s].ldy;
    }
    float acc[R][MT], acc2[EPI == EPI_SWIGLU ? R : 1][MT];
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
      for (int m = 0; m < MT; ++m) { acc[r][m] = 0.f; if (EPI == EPI_SWIGLU) acc2[r][m] = 0.f; }

    for (int c = 0; c * 512 + lane * 8 < K; ++c) {
      const size_t k0 = (size_t)c * 512 + lane * 8;
      float w[R][8], w2[EPI == EPI_SWIGLU ? R : 1][8];
#pragma unroll
      for (int r = 0; r < R; ++r) {
        load_w8<BF16>(wp[r], k0, w[r]);
        if (EPI == EPI_SWIGLU) load_w8<BF16>(wp2[r], k0, w2[r]);
      }
#pragma unroll
      for (int m = 0; m < MT; ++m) {
        const float4 xa = *reinterpret_cast<const float4*>(&xs[(size_t)m * Kpad + (((c * 2) * 64 + lane) << 2)]);
        const float4 xb = *reinterpret_cast<const float4*>(&xs[(size_t)m * Kpad + (((c * 2 + 1) * 64 + lane) << 2)]);
        const float x[8] = {xa.x, xa.y, xa.z, xa.w, xb.x, xb.y, xb.z, xb.w};
#pragma unroll
        for (int r = 0; r < R; ++r) {
#pragma unroll
          for (int i = 0; i < 8; ++i) acc[r][m] = fmaf(w[r][i], x[i], acc[r][m]);
          if (EPI == EPI_SWIGLU) {
#pragma unroll
            for (int i = 0; i < 8; ++i) acc2[r][m] = fmaf(w2[r][i], x[i], acc2[r][m]);
          }
        }
      }
    }
#pragma unroll
    for (int r = 0; r < R; ++r) {
#pragma unroll
      for (int m = 0; m < MT; ++m) {
        float v = wave_sum(acc[r][m]);
        if (EPI == EPI_SWIGLU) {
          const float u = wave_sum(acc2[r][m]);
          v = v / (1.0f + expf(-v)) * u;
        }
        if (lane == 0 && live[r] && m < mt) {
          float* y = yp[r] + (size_t)(m0 + m) * ldy[r] + ncol[r];
          if (EPI == EPI_ADD) v += *y;
          *y = v;
          if (a.best != nullptr) {
            const unsigned long long key = argmax_key(v, ncol[r]);
            if (key > best[m]) best[m] = key;
          }
        }
      }
    }
  }

  if (a.best != nullptr) {
    unsigned long long* bw = reinterpret_cast<unsigned long long*>(red + kWaves * MT + (kWaves * MT & 1));
    __syncthreads();
    if (lane == 0)
      for (int m = 0; m < MT; ++m) bw[wave * MT + m] = best[m];
    __syncthreads();
    if (tid < mt) {
      unsigned long long b = 0ull;
      for (int w = 0; w < kWaves; ++w) b = max(b, bw[w * MT + tid]);
      a.best[(size_t)(m0 + tid) * gridDim.x + blockIdx.x] = b;
    }
  }
}

template <int BF16, int MT, int R, int EPI>
static hipError_t launch_one(const GemvArgs& a, int m0, int n_total, int blocks, size_t lds, hipStream_t s) {
  auto kern = gemv_kernel<BF16, MT, R, EPI>;
  static bool big_lds_enabled = false;  // per instantiation; set once, outside any stream capture
  if (lds > 48 * 1024 && !big_lds_enabled) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (e != hipSuccess) return e;
    big_lds_enabled = true;
  }
  hipLaunchKernelGGL(kern, dim3(blocks), dim3(kThreads), lds, s, a, m0, n_total);
  return hipGetLastError();
}

template <int BF16, int MT, int R>
static hipError_t launch_epi(const GemvArgs& a, int m0, int n_total, int blocks, size_t lds, hipStream_t s) {
  switch (a.epi) {
    case EPI_STORE: return launch_one<BF16, MT, R, EPI_STORE>(a, m0, n_total, blocks, lds, s);
    case EPI_ADD: return launch_one<BF16, MT, R, EPI_ADD>(a, m0, n_total, blocks, lds, s);
    case EPI_SWIGLU: return launch_one<BF16, MT, (R > 2 ? 2 : R), EPI_SWIGLU>(a, m0, n_total, blocks, lds, s);
  }
  return hipErrorInvalidValue;
}

static int rows_per_pass(const GemvArgs& a, int n_total) {
  // rows per wavefront pass: enough blocks to cover the chip first, then fatter passes
  int R = 1;
  if (n_total >= 256 * kWaves * 2 * 2) R = 2;
  if (n_total >= 256 * kWaves * 4 * 2) R = 4;
  if (a.epi == EPI_SWIGLU && R == 4) R = 2;
  return R;
}

template <int BF16, int MT>
static hipError_t launch_r(const GemvArgs& a, int m0, int n_total, int* nblk, hipStream_t s) {
  const int Kpad = (a.K + 511) & ~511;
  const size_t lds = ((size_t)MT * Kpad + kWaves * MT + 2) * sizeof(float) + (size_t)kWaves * MT * 8 + 16;
  const int R = rows_per_pass(a, n_total);
  int blocks = (n_total + kWaves * R - 1) / (kWaves * R);
  if (blocks > kMaxBlocks) blocks = kMaxBlocks;
  if (nblk) *nblk = blocks;
  switch (R) {
    case 1: return launch_epi<BF16, MT, 1>(a, m0, n_total, blocks, lds, s);
    case 2: return launch_epi<BF16, MT, 2>(a, m0, n_total, blocks, lds, s);
    default: return launch_epi<BF16, MT, 4>(a, m0, n_total, blocks, lds, s);
  }
}

static constexpr size_t kLdsBudget = 150 * 1024;

template <int BF16>
static hipError_t launch_m(const GemvArgs& a, int* nblk, hipStream_t s) {
  int n_total = 0;
  for (int i = 0; i < a.n_seg; ++i) n_total += a.seg[i].n_rows;
  if (n_total <= 0 || a.M <= 0) return hipSuccess;
  const int Kpad = (a.K + 511) & ~511;
  // largest row tile whose activations fit in LDS
  int mt_cap = 8;
  while (mt_cap > 1 && (size_t)mt_cap * Kpad * 4 + 1024 > kLdsBudget) --mt_cap;
  if (mt_cap == 7 || mt_cap == 6) mt_cap = 5;
  for (int m0 = 0; m0 < a.M;) {
    const int left = a.M - m0;
    int mt = left >= 8 ? 8 : (left > 5 ? 8 : left);
    if (mt > mt_cap) mt = mt_cap;
    hipError_t e;
    switch (mt) {
      case 1: e = launch_r<BF16, 1>(a, m0, n_total, nblk, s); break;
      case 2: e = launch_r<BF16, 2>(a, m0, n_total, nblk, s); break;
      case 3: e = launch_r<BF16, 3>(a, m0, n_total, nblk, s); break;
      case 4: e = launch_r<BF16, 4>(a, m0, n_total, nblk, s); break;
      case 5: e = launch_r<BF16, 5>(a, m0, n_total, nblk, s); break;
      default: e = launch_r<BF16, 8>(a, m0, n_total, nblk, s); break;
    }
    if (e != hipSuccess) return e;
    m0 += mt;
  }
  return hipSuccess;
}

hipError_t launch_gemv(const GemvArgs& a, int* n_blocks_out, hipStream_t s) {
  if (a.K % 8 != 0) return hipErrorInvalidValue;
  return a.bf16 ? launch_m<1>(a, n_blocks_out, s) : launch_m<0>(a, n_blocks_out, s);
}

}  // namespace hh
