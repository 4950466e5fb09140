// Skinny-GEMM kernel template (see gemv.hip for the description).  Included by one translation
// unit per epilogue so that the instantiations compile in parallel.
#pragma once
#include "hh_internal.h"

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
  __device__ __forceinline__ void zero() { v = make_uint4(0, 0, 0, 0); }
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
  __device__ __forceinline__ void zero() { p = make_uint4(0, 0, 0, 0); q = make_uint4(0, 0, 0, 0); }
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
// Every lane returns the total.
template <int CTRL>
__device__ __forceinline__ float dpp_perm(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, false));
}
__device__ __forceinline__ float wave_sum(float v) {
  v += dpp_perm<0xB1>(v);    // quad_perm [1,0,3,2]: lane ^ 1
  v += dpp_perm<0x4E>(v);    // quad_perm [2,3,0,1]: lane ^ 2
  v += dpp_perm<0x141>(v);   // row_half_mirror: lane i <-> 7 - i inside each 8
  v += dpp_perm<0x140>(v);   // row_mirror: lane i <-> 15 - i inside each 16
  const int iv = __float_as_int(v);
  const float r0 = __int_as_float(__builtin_amdgcn_readlane(iv, 0));
  const float r1 = __int_as_float(__builtin_amdgcn_readlane(iv, 16));
  const float r2 = __int_as_float(__builtin_amdgcn_readlane(iv, 32));
  const float r3 = __int_as_float(__builtin_amdgcn_readlane(iv, 48));
  return (r0 + r1) + (r2 + r3);
}

__device__ __forceinline__ unsigned long long argmax_key(float v, int n) {
  uint32_t u = __float_as_uint(v);
  u = (u & 0x80000000u) ? ~u : (u | 0x80000000u);
  return (static_cast<unsigned long long>(u) << 32) | static_cast<unsigned long long>(0xFFFFFFFFu - (uint32_t)n);
}

// One unit of work of a wavefront: R output rows x G chunks of 512 columns (lane l owns columns
// c*512 + 8l .. 8l+7 of chunk c).  Units are walked row group by row group (stride = number of
// wavefronts in the grid), chunk group by chunk group inside a row group; the loads of unit u+1
// (weights AND the lane's own activation columns) are issued before the arithmetic of unit u.
// Wavefronts never synchronise with each other: no LDS, no barrier.
template <int BF16, int MT, int R, int G, int EPI>
__global__ __launch_bounds__(kGemvThreads) void gemv_kernel(const GemvArgs a, const int m0, const int n_total) {
  constexpr int NW = EPI == EPI_SWIGLU ? 2 * R : R;   // weight rows held per wavefront
  const int K = a.K;
  const int nch = (K + 511) >> 9;
  const int ncg = (nch + G - 1) / G;
  const int nrg = (n_total + R - 1) / R;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int mt = min(MT, a.M - m0);
  const int wave_g = blockIdx.x * kGemvWaves + wave, n_waves = gridDim.x * kGemvWaves;
  const size_t esz = BF16 ? 2 : 4;
  const bool normed = a.norm_w != nullptr;

  struct Rows { const char* w[NW]; float* y[R]; int col[R], ldy[R]; bool live[R]; };
  auto resolve = [&](int rg, Rows& q) {
#pragma unroll
    for (int r = 0; r < R; ++r) {
      int n = rg * R + r;
      q.live[r] = n < n_total;
      if (!q.live[r]) n = n_total - 1;
      // segment of row n, without a data-dependent loop (at most 4 segments)
      int s = 0, first = 0;
#pragma unroll
      for (int i = 0; i < 3; ++i) {
        const bool next = i + 1 < a.n_seg && n >= first + a.seg[i].n_rows;
        if (next && s == i) { first += a.seg[i].n_rows; s = i + 1; }
      }
      n -= first;
      const void* W = s == 0 ? a.seg[0].W : s == 1 ? a.seg[1].W : s == 2 ? a.seg[2].W : a.seg[3].W;
      const void* W2 = s == 0 ? a.seg[0].W2 : s == 1 ? a.seg[1].W2 : s == 2 ? a.seg[2].W2 : a.seg[3].W2;
      float* Y = s == 0 ? a.seg[0].Y : s == 1 ? a.seg[1].Y : s == 2 ? a.seg[2].Y : a.seg[3].Y;
      const int ld = s == 0 ? a.seg[0].ldy : s == 1 ? a.seg[1].ldy : s == 2 ? a.seg[2].ldy : a.seg[3].ldy;
      q.w[r] = static_cast<const char*>(W) + (size_t)n * K * esz;
      if (EPI == EPI_SWIGLU) q.w[R + r] = static_cast<const char*>(W2) + (size_t)n * K * esz;
      q.y[r] = Y + (size_t)m0 * ld + n;
      q.col[r] = n;
      q.ldy[r] = ld;
    }
  };

  struct XBuf { float4 lo[MT][G], hi[MT][G]; };
  W8<BF16> wbuf0[NW][G], wbuf1[NW][G];
  XBuf xbuf0, xbuf1;
  float resid_e = 0.f, resid_o = 0.f;   // old outputs of the row groups in flight, by row-group parity
  const float4 zero4 = make_float4(0.f, 0.f, 0.f, 0.f);

  auto issue = [&](W8<BF16> (&wb)[NW][G], XBuf& xb, int par, int rg, int cg) {
    Rows q;
    resolve(rg, q);
#pragma unroll
    for (int c = 0; c < G; ++c) {
      const int k0 = (cg * G + c) * 512 + lane * 8;
      const bool in = k0 < K;
#pragma unroll
      for (int r = 0; r < NW; ++r) {
        if (in) wb[r][c].load(q.w[r], k0);
        else wb[r][c].zero();
      }
#pragma unroll
      for (int m = 0; m < MT; ++m) {
        if (in && m < mt) {
          const float4* xp = reinterpret_cast<const float4*>(a.X + (size_t)(m0 + m) * a.ldx + k0);
          xb.lo[m][c] = xp[0]; xb.hi[m][c] = xp[1];
        } else {
          xb.lo[m][c] = zero4; xb.hi[m][c] = zero4;
        }
      }
    }
    if (EPI == EPI_ADD && cg == 0 && lane < R * MT) {   // old value of the output this lane will store
      const int r = lane / MT, m = lane % MT;
#pragma unroll
      for (int rr = 0; rr < R; ++rr)
        if (rr == r && q.live[rr] && m < mt) {
          if (par) resid_o = q.y[rr][(size_t)m * q.ldy[rr]];
          else resid_e = q.y[rr][(size_t)m * q.ldy[rr]];
        }
    }
  };

  // first unit in flight before anything else
  int rg = wave_g, cg = 0, par = 0;
  const bool any = rg < nrg;
  if (any) issue(wbuf0, xbuf0, par, rg, cg);

  // ---- RMSNorm scale of every activation row: each wavefront sums the squares itself
  float rstd[MT];
#pragma unroll
  for (int m = 0; m < MT; ++m) rstd[m] = 1.f;
  if (normed && any) {
    float ss[MT];
#pragma unroll
    for (int m = 0; m < MT; ++m) ss[m] = 0.f;
    for (int c = 0; c < nch; ++c) {
      const int k0 = c * 512 + lane * 8;
      if (k0 < K) {
#pragma unroll
        for (int m = 0; m < MT; ++m) {
          if (m < mt) {
            const float4* xp = reinterpret_cast<const float4*>(a.X + (size_t)(m0 + m) * a.ldx + k0);
            const float4 u = xp[0], v = xp[1];
            ss[m] += u.x * u.x + u.y * u.y + u.z * u.z + u.w * u.w + v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
          }
        }
      }
    }
#pragma unroll
    for (int m = 0; m < MT; ++m) rstd[m] = 1.0f / sqrtf(wave_sum(ss[m]) / (float)K + a.eps);
  }

  float acc[NW][MT];
#pragma unroll
  for (int r = 0; r < NW; ++r)
#pragma unroll
    for (int m = 0; m < MT; ++m) acc[r][m] = 0.f;
  unsigned long long best = 0ull;

  auto compute = [&](const W8<BF16> (&wb)[NW][G], const XBuf& xb, int cgi) {
#pragma unroll
    for (int c = 0; c < G; ++c) {
      const int k0 = (cgi * G + c) * 512 + lane * 8;
      float4 nlo = make_float4(1.f, 1.f, 1.f, 1.f), nhi = nlo;
      if (normed && k0 < K) {
        const float4* np = reinterpret_cast<const float4*>(a.norm_w + k0);
        nlo = np[0]; nhi = np[1];
      }
#pragma unroll
      for (int m = 0; m < MT; ++m) {
        float4 xa = xb.lo[m][c], xc = xb.hi[m][c];
        xa.x *= nlo.x; xa.y *= nlo.y; xa.z *= nlo.z; xa.w *= nlo.w;
        xc.x *= nhi.x; xc.y *= nhi.y; xc.z *= nhi.z; xc.w *= nhi.w;
#pragma unroll
        for (int r = 0; r < NW; ++r) acc[r][m] = wb[r][c].dot(xa, xc, acc[r][m]);
      }
    }
  };
  // reduce across lanes, apply the epilogue, store; lane r*MT + m owns output (r, m)
  auto finish = [&](int rgi, int pari) {
    const float resid = pari ? resid_o : resid_e;
    Rows q;
    resolve(rgi, q);
    float mine = 0.f;
#pragma unroll
    for (int r = 0; r < R; ++r) {
#pragma unroll
      for (int m = 0; m < MT; ++m) {
        float v = wave_sum(acc[r][m]) * rstd[m];
        acc[r][m] = 0.f;
        if (EPI == EPI_SWIGLU) {
          const float u = wave_sum(acc[R + r][m]) * rstd[m];
          acc[R + r][m] = 0.f;
          v = v / (1.0f + expf(-v)) * u;
        }
        if (lane == r * MT + m) mine = v;
      }
    }
    if (lane < R * MT) {
      const int r = lane / MT, m = lane % MT;
#pragma unroll
      for (int rr = 0; rr < R; ++rr) {
        if (rr == r && q.live[rr] && m < mt) {
          const float v = EPI == EPI_ADD ? mine + resid : mine;
          q.y[rr][(size_t)m * q.ldy[rr]] = v;
          if (a.best != nullptr) {
            const unsigned long long key = argmax_key(v, q.col[rr]);
            if (key > best) best = key;
          }
        }
      }
    }
  };
  auto advance = [&](int& rgi, int& cgi, int& pari) {
    if (++cgi == ncg) { cgi = 0; rgi += n_waves; pari ^= 1; }
  };

  // ---- software pipeline over units, two per trip so that both buffers are named statically
  if (any) {
    while (true) {
      int rg1 = rg, cg1 = cg, par1 = par;
      advance(rg1, cg1, par1);
      const bool has1 = rg1 < nrg;
      if (has1) issue(wbuf1, xbuf1, par1, rg1, cg1);
      compute(wbuf0, xbuf0, cg);
      if (cg == ncg - 1) finish(rg, par);
      if (!has1) break;
      int rg2 = rg1, cg2 = cg1, par2 = par1;
      advance(rg2, cg2, par2);
      const bool has2 = rg2 < nrg;
      if (has2) issue(wbuf0, xbuf0, par2, rg2, cg2);
      compute(wbuf1, xbuf1, cg1);
      if (cg1 == ncg - 1) finish(rg1, par1);
      if (!has2) break;
      rg = rg2; cg = cg2; par = par2;
    }
  }

  if (a.best != nullptr) {
    // per activation row m: max over every output this workgroup produced
    __shared__ unsigned long long bw[kGemvWaves * R * MT];
    if (lane < R * MT) bw[(wave * R + lane / MT) * MT + lane % MT] = best;
    __syncthreads();
    if ((int)threadIdx.x < mt) {
      unsigned long long b = 0ull;
      for (int w = 0; w < kGemvWaves * R; ++w) b = max(b, bw[w * MT + threadIdx.x]);
      a.best[(size_t)(m0 + threadIdx.x) * gridDim.x + blockIdx.x] = b;
    }
  }
}

template <int BF16, int MT, int R, int G, int EPI>
hipError_t gemv_launch_one(const GemvArgs& a, int m0, int n_total, int blocks, hipStream_t s) {
  hipLaunchKernelGGL((gemv_kernel<BF16, MT, R, G, EPI>), dim3(blocks), dim3(kGemvThreads), 0, s, a, m0, n_total);
  return hipGetLastError();
}

// shape of one launch, chosen on the host
struct GemvPlan { int MT, R, G, blocks; };

// Dispatch over (MT, R, G) for one epilogue and storage type; defined once per epilogue TU.
template <int BF16, int EPI>
hipError_t gemv_dispatch(const GemvArgs& a, int m0, int n_total, const GemvPlan& p, hipStream_t s) {
#define HH_RG(MTV)                                                                                          \
  if (p.R == 1 && p.G == 2) return gemv_launch_one<BF16, MTV, 1, 2, EPI>(a, m0, n_total, p.blocks, s); \
  if (p.R == 1 && p.G == 4) return gemv_launch_one<BF16, MTV, 1, 4, EPI>(a, m0, n_total, p.blocks, s); \
  if (p.R == 2 && p.G == 2) return gemv_launch_one<BF16, MTV, 2, 2, EPI>(a, m0, n_total, p.blocks, s); \
  if (BF16 && EPI != EPI_SWIGLU) {                                                                          \
    if (p.R == 2 && p.G == 4) return gemv_launch_one<BF16, MTV, 2, 4, EPI>(a, m0, n_total, p.blocks, s); \
    if (p.R == 4 && p.G == 2) return gemv_launch_one<BF16, MTV, 4, 2, EPI>(a, m0, n_total, p.blocks, s); \
  }                                                                                                         \
  return hipErrorInvalidValue;
  switch (p.MT) {
    case 1: HH_RG(1)
    case 2: HH_RG(2)
    case 3: HH_RG(3)
    case 4: HH_RG(4)
    case 5: HH_RG(5)
  }
#undef HH_RG
  return hipErrorInvalidValue;
}

hipError_t gemv_dispatch_store(const GemvArgs& a, int m0, int n_total, const GemvPlan& p, hipStream_t s);
hipError_t gemv_dispatch_add(const GemvArgs& a, int m0, int n_total, const GemvPlan& p, hipStream_t s);
hipError_t gemv_dispatch_swiglu(const GemvArgs& a, int m0, int n_total, const GemvPlan& p, hipStream_t s);

}  // namespace hh
