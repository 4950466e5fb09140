// Skinny-GEMM kernel template (see gemv.hip for the description).  Included by one translation
// unit per epilogue so that the instantiations compile in parallel.
#pragma once
#include "hh_internal.h"
#include "wave_ops.h"

namespace hh {

static constexpr int kGemvThreads = 256;
static constexpr int kGemvWaves = 4;

__device__ __forceinline__ float bf16lo(uint32_t v) { return __uint_as_float(v << 16); }
__device__ __forceinline__ float bf16hi(uint32_t v) { return __uint_as_float(v & 0xffff0000u); }

// 8 consecutive weights held as loaded (converted only when used)
template <int BF16> struct W8;
template <> struct W8<1> {
  uint4 v;
  __device__ __forceinline__ void load(const void* row, int k) {
    v = *reinterpret_cast<const uint4*>(static_cast<const uint16_t*>(row) + k);
  }
  __device__ __forceinline__ float dot(const float4& a, const float4& b, float s) const {
    s = fmaf(bf16lo(v.x), a.x, s); s = fmaf(bf16hi(v.x), a.y, s);
    s = fmaf(bf16lo(v.y), a.z, s); s = fmaf(bf16hi(v.y), a.w, s);
    s = fmaf(bf16lo(v.z), b.x, s); s = fmaf(bf16hi(v.z), b.y, s);
    s = fmaf(bf16lo(v.w), b.z, s); s = fmaf(bf16hi(v.w), b.w, s);
    return s;
  }
};
template <> struct W8<0> {
  uint4 p, q;   // raw bits of 8 floats
  __device__ __forceinline__ void load(const void* row, int k) {
    const uint4* s = reinterpret_cast<const uint4*>(static_cast<const float*>(row) + k);
    p = s[0]; q = s[1];
  }
  __device__ __forceinline__ float dot(const float4& a, const float4& b, float s) const {
    s = fmaf(__uint_as_float(p.x), a.x, s); s = fmaf(__uint_as_float(p.y), a.y, s);
    s = fmaf(__uint_as_float(p.z), a.z, s); s = fmaf(__uint_as_float(p.w), a.w, s);
    s = fmaf(__uint_as_float(q.x), b.x, s); s = fmaf(__uint_as_float(q.y), b.y, s);
    s = fmaf(__uint_as_float(q.z), b.z, s); s = fmaf(__uint_as_float(q.w), b.w, s);
    return s;
  }
};

// Sum over the 64 lanes of a wavefront without LDS traffic: butterfly inside each row of 16
// lanes with DPP lane permutations, then the four row totals are read out and added.
// Every lane returns the total.  Must be called with all 64 lanes active.
__device__ __forceinline__ float wave_sum(float v) {
  v += dpp_move<0xB1>(v);    // quad_perm [1,0,3,2]: lane ^ 1
  v += dpp_move<0x4E>(v);    // quad_perm [2,3,0,1]: lane ^ 2
  v += dpp_move<0x141>(v);   // row_half_mirror: lane i <-> 7 - i inside each 8
  v += dpp_move<0x140>(v);   // row_mirror: lane i <-> 15 - i inside each 16
  const int iv = __float_as_int(v);
  const float r0 = __int_as_float(__builtin_amdgcn_readlane(iv, 0));
  const float r1 = __int_as_float(__builtin_amdgcn_readlane(iv, 16));
  const float r2 = __int_as_float(__builtin_amdgcn_readlane(iv, 32));
  const float r3 = __int_as_float(__builtin_amdgcn_readlane(iv, 48));
  return (r0 + r1) + (r2 + r3);
}

// LDS layout of one activation row: the 8 floats a lane multiplies in chunk c
// (k = c*512 + lane*8 + i) are stored as two float4 at slots (2c)*64 + lane and (2c+1)*64 + lane,
// so both 16-byte LDS reads of a wavefront are unit-stride across lanes.
__device__ __forceinline__ int xs_slot4(int k4) {       // k4 = k / 4 -> float4 slot
  const int c = k4 >> 7, r = k4 & 127;
  return (c * 2 + (r & 1)) * 64 + (r >> 1);
}

// A workgroup of 4 wavefronts.  A wavefront owns R consecutive output rows and a slice of
// NCW chunks of 512 columns (lane l owns columns 8l .. 8l+7 of each chunk); KS wavefronts
// share the rows of one row group and split its columns between them, so a workgroup covers
// 4/KS row groups per iteration.  All weight loads of a unit are issued together and
// unconditionally (columns past K read a clamped, valid address and meet zero activations);
// the first unit is issued before the activations are staged.  Latency is hidden by the other
// resident wavefronts (up to 8 per SIMD), not by software pipelining.
template <int BF16, int MT, int R, int NCW, int KS, int EPI>
__global__ __launch_bounds__(kGemvThreads) void gemv_kernel(const GemvArgs a, const int m0, const int iters) {
  constexpr int NW = EPI == EPI_SWIGLU ? 2 * R : R;   // weight rows held per wavefront
  constexpr int RGB = kGemvWaves / KS;                // row groups per workgroup per iteration
  constexpr int NOUT = R * MT;                        // outputs per row group
  constexpr int PN = EPI == EPI_SWIGLU ? 2 * NOUT : NOUT;
  extern __shared__ __align__(16) float smem[];
  const int K = a.K;
  const int Kpad = (K + 511) & ~511;
  const int nch = Kpad >> 9;
  const int N = a.seg[0].n_rows;
  const int nrg = N / R;
  float4* xs4 = reinterpret_cast<float4*>(smem);          // [MT][Kpad/4]
  float* red = smem + (size_t)MT * Kpad;                  // [4][MT] sums of squares
  float* part = red + kGemvWaves * MT;                    // [2][4][PN] split-K partial sums
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int ks = wave % KS, slot = wave / KS;
  const int mt = min(MT, a.M - m0);
  const size_t row_bytes = (size_t)K * (BF16 ? 2 : 4);
  const char* const Wb = static_cast<const char*>(a.seg[0].W);
  const char* const W2b = static_cast<const char*>(a.seg[0].W2);
  const int ldy = a.seg[0].ldy;
  float* const Yb = a.seg[0].Y + (size_t)m0 * ldy;
  const int out_r = lane / MT, out_m = lane - out_r * MT;   // output owned by this lane (lane < NOUT)
  const bool owner = ks == 0 && lane < NOUT && out_m < mt;

  W8<BF16> w[NW][NCW];
  float resid = 0.f;
  auto row_group = [&](int it) { return (blockIdx.x * iters + it) * RGB + slot; };
  auto load_unit = [&](int rg) {
    const int n = min(rg, nrg - 1) * R;
#pragma unroll
    for (int c = 0; c < NCW; ++c) {
      const int k0 = min((ks * NCW + c) * 512 + lane * 8, K - 8);
#pragma unroll
      for (int r = 0; r < R; ++r) {
        w[r][c].load(Wb + (size_t)(n + r) * row_bytes, k0);
        if (EPI == EPI_SWIGLU) w[R + r][c].load(W2b + (size_t)(n + r) * row_bytes, k0);
      }
    }
    if (EPI == EPI_ADD) {
      if (owner && rg < nrg) {
        resid = Yb[(size_t)out_m * ldy + n + out_r];
        if (a.R2 != nullptr) resid += a.R2[(size_t)(m0 + out_m) * ldy + n + out_r];
      }
    }
  };
  load_unit(row_group(0));   // in flight while the activations are staged

  // ---- prologue: stage x[k] * norm_w[k] (float4 at a time) and the sums of squares.  The
  // loads of all MT rows of a column group are issued together (one memory round trip, not MT).
  const bool normed = a.norm_w != nullptr;
  {
    float ss[MT];
#pragma unroll
    for (int m = 0; m < MT; ++m) ss[m] = 0.f;
    const float4* n4 = reinterpret_cast<const float4*>(a.norm_w);
    for (int k4 = tid; k4 < (Kpad >> 2); k4 += kGemvThreads) {
      const bool in_k = k4 < (K >> 2);
      const int k4c = min(k4, (K >> 2) - 1);
      float4 v[MT];
      float4 nw = make_float4(1.f, 1.f, 1.f, 1.f);
      if (normed) nw = n4[k4c];
#pragma unroll
      for (int m = 0; m < MT; ++m) {
        const size_t ro = (size_t)(m0 + min(m, mt - 1)) * a.ldx;
        v[m] = reinterpret_cast<const float4*>(a.X + ro)[k4c];
        if (a.X2 != nullptr) {
          const float4 w2 = reinterpret_cast<const float4*>(a.X2 + ro)[k4c];
          v[m].x += w2.x; v[m].y += w2.y; v[m].z += w2.z; v[m].w += w2.w;
        }
      }
#pragma unroll
      for (int m = 0; m < MT; ++m) {
        float4 o = make_float4(0.f, 0.f, 0.f, 0.f);
        if (in_k && m < mt) {
          o = v[m];
          ss[m] += o.x * o.x + o.y * o.y + o.z * o.z + o.w * o.w;
          o.x *= nw.x; o.y *= nw.y; o.z *= nw.z; o.w *= nw.w;
        }
        xs4[(size_t)m * (Kpad >> 2) + xs_slot4(k4)] = o;
      }
    }
    if (normed) {
#pragma unroll
      for (int m = 0; m < MT; ++m) {
        const float t = wave_sum(ss[m]);
        if (lane == 0) red[wave * MT + m] = t;
      }
    }
  }
  __syncthreads();
  float rstd = 1.f;   // of the activation row this lane stores
  if (normed && lane < NOUT) {
    float tot = 0.f;
#pragma unroll
    for (int i = 0; i < kGemvWaves; ++i) tot += red[i * MT + out_m];
    rstd = 1.0f / sqrtf(tot / (float)K + a.eps);
  }

  unsigned long long best = 0ull;
  for (int it = 0; it < iters; ++it) {
    const int rg = row_group(it);
    if (it > 0) load_unit(rg);
    float acc[NW][MT];
#pragma unroll
    for (int r = 0; r < NW; ++r)
#pragma unroll
      for (int m = 0; m < MT; ++m) acc[r][m] = 0.f;
#pragma unroll
    for (int c = 0; c < NCW; ++c) {
      const int ch = ks * NCW + c;
      if (ch < nch) {
#pragma unroll
        for (int m = 0; m < MT; ++m) {
          const float4* xr = &xs4[(size_t)m * (Kpad >> 2) + (ch * 2) * 64 + lane];
          const float4 xa = xr[0], xb = xr[64];
#pragma unroll
          for (int r = 0; r < NW; ++r) acc[r][m] = w[r][c].dot(xa, xb, acc[r][m]);
        }
      }
    }
    // lane r*MT + m collects the wavefront's sum for output (r, m)
    float mine = 0.f, mine2 = 0.f;
#pragma unroll
    for (int r = 0; r < R; ++r) {
#pragma unroll
      for (int m = 0; m < MT; ++m) {
        const float v = wave_sum(acc[r][m]);
        if (lane == r * MT + m) mine = v;
        if (EPI == EPI_SWIGLU) {
          const float u = wave_sum(acc[R + r][m]);
          if (lane == r * MT + m) mine2 = u;
        }
      }
    }
    if (KS > 1) {   // add the partial sums of the wavefronts that share these rows
      float* pb = part + (size_t)(it & 1) * kGemvWaves * PN;
      if (lane < NOUT) {
        pb[wave * PN + lane] = mine;
        if (EPI == EPI_SWIGLU) pb[wave * PN + NOUT + lane] = mine2;
      }
      __syncthreads();
      if (ks == 0 && lane < NOUT) {
#pragma unroll
        for (int j = 1; j < KS; ++j) {
          mine += pb[(wave + j) * PN + lane];
          if (EPI == EPI_SWIGLU) mine2 += pb[(wave + j) * PN + NOUT + lane];
        }
      }
    }
    if (owner && rg < nrg) {
      float v = mine * rstd;
      if (EPI == EPI_SWIGLU) v = v / (1.0f + expf(-v)) * (mine2 * rstd);
      if (EPI == EPI_ADD) v += resid;
      const int n = rg * R + out_r;
      Yb[(size_t)out_m * ldy + n] = v;
      if (a.best != nullptr) {
        const unsigned long long key = argmax_key(v, n);
        if (key > best) best = key;
      }
    }
  }

  if (a.best != nullptr) {
    // per activation row m: max over every output this workgroup produced
    __shared__ unsigned long long bw[kGemvWaves * NOUT];
    if (lane < NOUT) bw[wave * NOUT + lane] = best;   // zero for wavefronts that do not store
    __syncthreads();
    if (tid < mt) {
      unsigned long long b = 0ull;
      for (int i = 0; i < kGemvWaves; ++i)
        for (int r = 0; r < R; ++r) b = max(b, bw[i * NOUT + r * MT + tid]);
      a.best[(size_t)(m0 + tid) * gridDim.x + blockIdx.x] = b;
    }
  }
}

// shape of one launch, chosen on the host
struct GemvPlan { int MT, R, NCW, KS, iters, blocks; size_t lds; };

template <int BF16, int MT, int R, int NCW, int KS, int EPI>
hipError_t gemv_launch_one(const GemvArgs& a, int m0, const GemvPlan& p, hipStream_t s) {
  auto kern = gemv_kernel<BF16, MT, R, NCW, KS, EPI>;
  static size_t lds_enabled = 48 * 1024;  // per instantiation: dynamic LDS the kernel may use so far
  if (p.lds > lds_enabled) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)p.lds);
    if (e != hipSuccess) return e;
    lds_enabled = p.lds;
  }
  hipLaunchKernelGGL(kern, dim3(p.blocks), dim3(kGemvThreads), p.lds, s, a, m0, p.iters);
  return hipGetLastError();
}

// Dispatch over (MT, R, NCW, KS) for one epilogue and storage type.
template <int BF16, int EPI, int MT, int R>
hipError_t gemv_dispatch_ks(const GemvArgs& a, int m0, const GemvPlan& p, hipStream_t s) {
  if (p.NCW == 2 && p.KS == 1) return gemv_launch_one<BF16, MT, R, 2, 1, EPI>(a, m0, p, s);
  if (p.NCW == 2 && p.KS == 2) return gemv_launch_one<BF16, MT, R, 2, 2, EPI>(a, m0, p, s);
  if (p.NCW == 2 && p.KS == 4) return gemv_launch_one<BF16, MT, R, 2, 4, EPI>(a, m0, p, s);
  if (p.NCW == 4 && p.KS == 4) return gemv_launch_one<BF16, MT, R, 4, 4, EPI>(a, m0, p, s);
  return hipErrorInvalidValue;
}
template <int BF16, int EPI, int MT>
hipError_t gemv_dispatch_r(const GemvArgs& a, int m0, const GemvPlan& p, hipStream_t s) {
  if (p.R == 1) return gemv_dispatch_ks<BF16, EPI, MT, 1>(a, m0, p, s);
  if (BF16) {
    if (p.R == 2) return gemv_dispatch_ks<BF16, EPI, MT, 2>(a, m0, p, s);
    if (EPI != EPI_SWIGLU && MT <= 5 && p.R == 4) return gemv_dispatch_ks<BF16, EPI, MT, 4>(a, m0, p, s);
  }
  return hipErrorInvalidValue;
}
template <int BF16, int EPI>
hipError_t gemv_dispatch(const GemvArgs& a, int m0, const GemvPlan& p, hipStream_t s) {
  switch (p.MT) {
    case 1: return gemv_dispatch_r<BF16, EPI, 1>(a, m0, p, s);
    case 3: return gemv_dispatch_r<BF16, EPI, 3>(a, m0, p, s);
    case 5: return gemv_dispatch_r<BF16, EPI, 5>(a, m0, p, s);
    case 8: return gemv_dispatch_r<BF16, EPI, 8>(a, m0, p, s);
  }
  return hipErrorInvalidValue;
}

hipError_t gemv_dispatch_store(const GemvArgs& a, int m0, const GemvPlan& p, hipStream_t s);
hipError_t gemv_dispatch_add(const GemvArgs& a, int m0, const GemvPlan& p, hipStream_t s);
hipError_t gemv_dispatch_swiglu(const GemvArgs& a, int m0, const GemvPlan& p, hipStream_t s);

}  // namespace hh
