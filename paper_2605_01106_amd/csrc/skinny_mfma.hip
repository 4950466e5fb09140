// Dense projections for 1..16 activation rows on the matrix cores, bf16 weights:
//     Y[m][n] (op)= sum_k X'[m][k] * W[n][k],   X' = X or rmsnorm(X) * norm_w.
// The pass is bound by streaming W once, so the kernel is built to do nothing else per weight
// byte: with v_mfma_f32_16x16x32_bf16 a wavefront loads 16 weight rows x 32 columns as the A
// operand exactly as they lie in memory (lane l: row l%16, 16 bytes at column 8(l/16)) - no
// conversion, no FMA per weight, no cross-lane sum.  The activations are the B operand
// (lane l: activation row l%16, the same 8 columns; rows >= M are zero).
//
// Activations stay float32-accurate: each value is split exactly into three bf16 terms
// (x = t0 + t1 + t2), one MFMA per term accumulating in float32.  The split, with the fused
// RMSNorm, happens once per workgroup: every wavefront owns a slice of K, stages the three
// terms of its slice in LDS, and multiplies it with the same slice of every weight tile the
// workgroup visits.  The partial tiles of the wavefronts are added through LDS in wavefront
// order (deterministic); the wavefront that finishes a tile holds D[4(l/16)+r][l%16] =
// Y[activation row l%16][weight row 4(l/16)+r] and applies the epilogue (store, residual add,
// SwiGLU, argmax partials for the LM head: largest value, lowest index on ties).
#include <stdlib.h>

#include "hh_internal.h"
#include "wave_ops.h"
#include "trace.h"
#include "bf16_split.h"

namespace hh {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

union SFrag {
  uint4 u;
  bf16x8 v;
};

__device__ __forceinline__ void sk_split3(float x, uint32_t& t0, uint32_t& t1, uint32_t& t2) { split3_bf16(x, t0, t1, t2); }

// sum over the 64 lanes: DPP butterflies inside each row of 16 lanes, then the four row totals
__device__ __forceinline__ float sk_wave_sum(float v) {
  v += dpp_move<0xB1>(v); v += dpp_move<0x4E>(v); v += dpp_move<0x141>(v); v += dpp_move<0x140>(v);
  const int iv = __float_as_int(v);
  return (__int_as_float(__builtin_amdgcn_readlane(iv, 0)) + __int_as_float(__builtin_amdgcn_readlane(iv, 16))) +
         (__int_as_float(__builtin_amdgcn_readlane(iv, 32)) + __int_as_float(__builtin_amdgcn_readlane(iv, 48)));
}

struct SkinnyArgs {
  const float* X; int ldx, M, K;
  const float* X2;                         // optional second addend of the input
  const float* R2;                         // optional second residual (EPI_ADD)
  const float* norm_w; float eps;
  const uint16_t* W; const uint16_t* W2;   // packed tiles (W2: the "up" matrix for SwiGLU)
  float* Y; int ldy, N;
  unsigned long long* best;                // [M][gridDim.x] argmax partials, or nullptr
  int rounds;                              // weight tiles per workgroup (tile = blockIdx.x + round * gridDim.x)
  int k0, kst_row;                         // workgroup (x, y) covers columns k0 + y K .. + K of rows that hold kst_row steps
  float rnorm_k;                           // 1 / (columns the RMSNorm averages over)
  // K windows side by side (gridDim.y > 1): window y stores its raw partial product at
  // Y + y * ywin (EPI_STORE) and, with a norm, its sums of squares at ssq[y * 16 + row]; a
  // reduction kernel adds the windows in order and applies norm scale and epilogue.
  size_t ywin;
  float* ssq;
};

// NWAVES wavefronts split K, each taking KSTEPS steps of 32 columns; a round is one tile of 16
// weight rows.  The weights of round r+1 are requested before round r is multiplied; the
// partial tiles are double-buffered in LDS so that a round costs one workgroup barrier, and
// the wavefront that finishes a tile (round mod NWAVES) does so while the others go on.
template <int EPI, int NWAVES, int KSTEPS>
__global__ __launch_bounds__(64 * NWAVES) void skinny_mfma_kernel(const SkinnyArgs a) {
  constexpr int NF = EPI == EPI_SWIGLU ? 2 : 1;
  // two weight matrices and long slices: one set of fragments, the next round is requested
  // after the multiplication instead of before it
  constexpr bool DB = !(NF == 2 && KSTEPS > 5);
  constexpr int SL = KSTEPS * 32 + 8;                       // staged columns per wavefront (+ pad)
  constexpr int SL4 = KSTEPS * 8;                           // float4 groups per row of a slice
  extern __shared__ __align__(16) unsigned char smem_raw[];
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int g = lane >> 4, n = lane & 15;
  const int K = a.K, M = a.M, N = a.N;
  const int k0 = a.k0 + (int)blockIdx.y * K;                // first column of this workgroup's window
  float* const Yw = a.Y + (size_t)blockIdx.y * a.ywin;
  const int kb = wave * KSTEPS * 32;                        // first column of this wavefront's slice
  uint16_t* xs = reinterpret_cast<uint16_t*>(smem_raw) + (size_t)wave * 3 * M * SL;          // [3][M][SL]
  float* red = reinterpret_cast<float*>(smem_raw + (size_t)NWAVES * 3 * M * SL * 2);         // [NWAVES][16]
  f32x4* part = reinterpret_cast<f32x4*>(red + NWAVES * 16);                                 // [2][NF][NWAVES][64]
  unsigned long long* bestb = reinterpret_cast<unsigned long long*>(part + 2 * NF * NWAVES * 64);   // [NWAVES][16]
  float* ssb = reinterpret_cast<float*>(part) + (size_t)wave * M * SL4;   // [M][SL4] per wavefront; shares the partial-tile buffer (used before it)

  const int n_tiles = (N + 15) >> 4;
  const int KST = (K + 31) >> 5;                            // steps of 32 columns covered by this launch
  const int ks0 = wave * KSTEPS;                            // first step of this wavefront's slice
  TR(0);
  SFrag wf[DB ? 2 : 1][NF][KSTEPS];
  auto load_round = [&](int rd, SFrag(&w)[NF][KSTEPS]) {
    const int tile = min(blockIdx.x + rd * (int)gridDim.x, n_tiles - 1);
#pragma unroll
    for (int s = 0; s < KSTEPS; ++s) {
      // steps past the end of the row (last wavefronts only) re-read the last step and meet zero activations
      const size_t at = ((size_t)tile * a.kst_row + (k0 >> 5) + min(ks0 + s, KST - 1)) * 512 + lane * 8;
      w[0][s].u = *reinterpret_cast<const uint4*>(a.W + at);
      if (NF == 2) w[NF - 1][s].u = *reinterpret_cast<const uint4*>(a.W2 + at);
    }
  };
  // ---- stage this wavefront's slice of the activations: norm weight, 3-term split, squares.
  // Items (row, group of 4 columns) are spread over the lanes, 4 loads in flight per lane; the
  // first batch is requested before the weights so that it does not wait behind them.
  {
    const bool normed = a.norm_w != nullptr;
    const int items = M * SL4;
    float4 v[4], nw[4];
    int mi[4], ci[4];
    bool ok[4];
    auto issue = [&](int it0) {
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int it = it0 + u * 64 + lane;
        mi[u] = min(it / SL4, M - 1); ci[u] = it % SL4;
        const int col = kb + 4 * ci[u];
        ok[u] = it < items && col < K;
        const int colc = min(col, K - 4);
        v[u] = *reinterpret_cast<const float4*>(a.X + (size_t)mi[u] * a.ldx + k0 + colc);
        if (a.X2 != nullptr) {
          const float4 w2 = *reinterpret_cast<const float4*>(a.X2 + (size_t)mi[u] * a.ldx + k0 + colc);
          v[u].x += w2.x; v[u].y += w2.y; v[u].z += w2.z; v[u].w += w2.w;
        }
        nw[u] = normed ? *reinterpret_cast<const float4*>(a.norm_w + k0 + colc) : make_float4(1.f, 1.f, 1.f, 1.f);
      }
    };
    auto process = [&](int it0) {
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        if (it0 + u * 64 + lane < items) {
          if (!ok[u]) v[u] = make_float4(0.f, 0.f, 0.f, 0.f);
          ssb[mi[u] * SL4 + ci[u]] = v[u].x * v[u].x + v[u].y * v[u].y + v[u].z * v[u].z + v[u].w * v[u].w;
          uint32_t t0[4], t1[4], t2[4];
          sk_split3(v[u].x * nw[u].x, t0[0], t1[0], t2[0]); sk_split3(v[u].y * nw[u].y, t0[1], t1[1], t2[1]);
          sk_split3(v[u].z * nw[u].z, t0[2], t1[2], t2[2]); sk_split3(v[u].w * nw[u].w, t0[3], t1[3], t2[3]);
          uint16_t* dst = xs + (size_t)mi[u] * SL + 4 * ci[u];
          *reinterpret_cast<uint2*>(dst) = make_uint2(t0[0] | (t0[1] << 16), t0[2] | (t0[3] << 16));
          *reinterpret_cast<uint2*>(dst + (size_t)M * SL) = make_uint2(t1[0] | (t1[1] << 16), t1[2] | (t1[3] << 16));
          *reinterpret_cast<uint2*>(dst + (size_t)2 * M * SL) = make_uint2(t2[0] | (t2[1] << 16), t2[2] | (t2[3] << 16));
        }
      }
    };
    issue(0);
    load_round(0, wf[0]);   // the weights of the first tile stream in while the activations are staged
    TR(1);
    process(0);
    for (int it0 = 256; it0 < items; it0 += 256) { issue(it0); process(it0); }
    if (normed) {
      // lane (g, n) adds the squares of row n over the groups c = g, g+4, ...; then across g
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
      float ss = 0.f;
      if (n < M)
        for (int c = g; c < SL4; c += 4) ss += ssb[n * SL4 + c];
      ss += __shfl_xor(ss, 16, 64);
      ss += __shfl_xor(ss, 32, 64);
      if (g == 0) red[wave * 16 + n] = ss;
    }
  }
  TR(2);
  __syncthreads();
  TR(3);
  float rstd = 1.f;   // of activation row n (this lane's column of every tile)
  if (a.norm_w != nullptr && n < M) {
    float tot = 0.f;
#pragma unroll
    for (int w = 0; w < NWAVES; ++w) tot += red[w * 16 + n];
    if (a.ssq == nullptr) rstd = 1.0f / sqrtf(tot * a.rnorm_k + a.eps);
    else if (blockIdx.x == 0 && wave == 0 && g == 0) a.ssq[blockIdx.y * 16 + n] = tot;   // the reduction kernel scales
  }
  // this lane's activation fragments; lanes n >= M hold copies of a valid row (their columns of
  // the product are never stored)
  const uint16_t* xrow = xs + (size_t)min(n, M - 1) * SL + 8 * g;

  unsigned long long best = 0ull;
  auto round = [&](int rd, SFrag(&w)[NF][KSTEPS], SFrag(&wnext)[NF][KSTEPS]) {
    if (DB && rd + 1 < a.rounds) load_round(rd + 1, wnext);
    const int tile = blockIdx.x + rd * (int)gridDim.x;
    const int fin = rd % NWAVES;                 // the wavefront that finishes this tile
    // residual of the tile: requested now, needed after the reduction
    float4 old = make_float4(0.f, 0.f, 0.f, 0.f);
    const int row0 = tile * 16 + 4 * g;
    const bool vec = n < M && row0 + 3 < N && (a.ldy & 3) == 0;
    if (EPI == EPI_ADD && wave == fin && vec) {
      old = *reinterpret_cast<const float4*>(Yw + (size_t)n * a.ldy + row0);
      if (a.R2 != nullptr) {
        const float4 o2 = *reinterpret_cast<const float4*>(a.R2 + (size_t)n * a.ldy + row0);
        old.x += o2.x; old.y += o2.y; old.z += o2.z; old.w += o2.w;
      }
    }
    if (KSTEPS > 5 || !DB) asm volatile("" ::: "memory");   // long slices: re-read the activation fragments every round
    f32x4 acc[NF][3];
#pragma unroll
    for (int f = 0; f < NF; ++f)
#pragma unroll
      for (int t = 0; t < 3; ++t) acc[f][t] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int s = 0; s < KSTEPS; ++s) {
#pragma unroll
      for (int t = 0; t < 3; ++t) {
        SFrag xb;
        xb.u = *reinterpret_cast<const uint4*>(xrow + (size_t)t * M * SL + s * 32);
#pragma unroll
        for (int f = 0; f < NF; ++f) acc[f][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w[f][s].v, xb.v, acc[f][t], 0, 0, 0);
      }
    }
    if (!DB && rd + 1 < a.rounds) load_round(rd + 1, wnext);
    f32x4* pb = part + (size_t)(rd & 1) * NF * NWAVES * 64;
#pragma unroll
    for (int f = 0; f < NF; ++f) pb[(f * NWAVES + wave) * 64 + lane] = (acc[f][0] + acc[f][1]) + acc[f][2];
    __syncthreads();
    if (wave == fin) {
      f32x4 sum[NF];
#pragma unroll
      for (int f = 0; f < NF; ++f) {
        sum[f] = pb[(f * NWAVES) * 64 + lane];
#pragma unroll
        for (int w2 = 1; w2 < NWAVES; ++w2) sum[f] += pb[(f * NWAVES + w2) * 64 + lane];
      }
      if (tile < n_tiles && n < M) {
        float* y = Yw + (size_t)n * a.ldy + row0;
        float v[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          v[r] = sum[0][r] * rstd;
          if (EPI == EPI_SWIGLU) v[r] = v[r] / (1.0f + expf(-v[r])) * (sum[NF - 1][r] * rstd);
        }
        if (vec) {
          float4 o = make_float4(v[0], v[1], v[2], v[3]);
          if (EPI == EPI_ADD) { o.x += old.x; o.y += old.y; o.z += old.z; o.w += old.w; }
          *reinterpret_cast<float4*>(y) = o;
          v[0] = o.x; v[1] = o.y; v[2] = o.z; v[3] = o.w;
        } else {
#pragma unroll
          for (int r = 0; r < 4; ++r)
            if (row0 + r < N) {
              if (EPI == EPI_ADD) v[r] += y[r] + (a.R2 != nullptr ? a.R2[(size_t)n * a.ldy + row0 + r] : 0.f);
              y[r] = v[r];
            }
        }
        if (a.best != nullptr) {
#pragma unroll
          for (int r = 0; r < 4; ++r)
            if (row0 + r < N) { const unsigned long long key = argmax_key(v[r], row0 + r); if (key > best) best = key; }
        }
      }
    }
  };
  for (int rd = 0; rd < a.rounds; rd += 2) {
    round(rd, wf[0], wf[DB ? 1 : 0]);
    if (rd + 1 < a.rounds) round(rd + 1, wf[DB ? 1 : 0], wf[0]);
  }
  TR(4);

  if (a.best != nullptr) {
    // per activation row: maximum over the 4 lane groups, then over the wavefronts
    unsigned long long o = __shfl_xor(best, 16, 64); if (o > best) best = o;
    o = __shfl_xor(best, 32, 64); if (o > best) best = o;
    if (g == 0) bestb[wave * 16 + n] = best;
    __syncthreads();
    if (tid < M) {
      unsigned long long b = 0ull;
#pragma unroll
      for (int w = 0; w < NWAVES; ++w) b = max(b, bestb[w * 16 + tid]);
      a.best[(size_t)tid * gridDim.x + blockIdx.x] = b;
    }
  }
  TR(5);
}

// Weight layout of the matrix-core kernels: tiles of 16 rows x 32 columns stored in operand
// order, tile (t, s) at element ((t * ceil(K/32) + s) * 512, lane l = 16 g + n of the tile
// holding W[16 t + n][32 s + 8 g .. + 7] at element 8 l; rows >= N and columns >= K are zero.
// A wavefront load of one tile is 1 KB contiguous, a K slice of one row tile is contiguous.
__host__ __device__ size_t packed_weight_elems(int N, int K) { return (size_t)((N + 15) / 16) * ((K + 31) / 32) * 512; }

__global__ __launch_bounds__(256) void pack_weights_kernel(const uint16_t* __restrict__ W, int N, int K, size_t ldw,
                                                           uint16_t* __restrict__ P) {
  const int KST = (K + 31) >> 5;
  const size_t total = packed_weight_elems(N, K) / 8;     // 16-byte groups
  for (size_t it = blockIdx.x * (size_t)256 + threadIdx.x; it < total; it += (size_t)gridDim.x * 256) {
    const int l = (int)(it & 63);
    const size_t ts = it >> 6;
    const int s = (int)(ts % KST);
    const size_t t = ts / KST;
    const size_t row = t * 16 + (l & 15);
    const int col = s * 32 + 8 * (l >> 4);
    uint4 v = make_uint4(0, 0, 0, 0);
    if (row < (size_t)N && col < K) v = *reinterpret_cast<const uint4*>(W + row * ldw + col);   // K % 8 == 0
    *reinterpret_cast<uint4*>(P + it * 8) = v;
  }
}

hipError_t launch_pack_weights(const void* W, int N, int K, size_t ldw, void* P, hipStream_t s) {
  if (K % 8 != 0 || ldw % 8 != 0) return hipErrorInvalidValue;
  const size_t groups = packed_weight_elems(N, K) / 8;
  const int blocks = (int)((groups + 255) / 256 < 4096 ? (groups + 255) / 256 : 4096);
  hipLaunchKernelGGL(pack_weights_kernel, dim3(blocks), dim3(256), 0, s, static_cast<const uint16_t*>(W), N, K, ldw,
                     static_cast<uint16_t*>(P));
  return hipGetLastError();
}

struct SkinnyPlan { int nwaves, ksteps, rounds, blocks, windows; size_t lds; };

// plan for a window of K columns of the product (the whole row, or a part when the staged
// activations of the whole row would not fit in LDS)
static bool skinny_plan_k(const GemvArgs& g, int K, SkinnyPlan& p) {
  constexpr int blk_target = 768;
  const int M = g.M, N = g.seg[0].n_rows, nf = g.epi == EPI_SWIGLU ? 2 : 1;
  const int steps = (K + 31) / 32, tiles = (N + 15) / 16;
  // K split: 8 wavefronts, 16 for long rows; a slice is at most 8 steps (the fragments of two
  // rounds live in registers)
  p.nwaves = steps > 64 && nf == 1 ? 16 : 8;
  p.ksteps = (steps + p.nwaves - 1) / p.nwaves;
  if (p.ksteps > 8 && p.nwaves == 8 && nf == 1) { p.nwaves = 16; p.ksteps = (steps + 15) / 16; }
  static const int allowed8[] = {1, 2, 3, 4, 5, 6, 8, 10}, allowed16[] = {4, 5, 6, 8, 10, 14};
  int ks = 0;
  if (p.nwaves == 8) { for (int v : allowed8) if (v >= p.ksteps) { ks = v; break; } }
  else { for (int v : allowed16) if (v >= p.ksteps) { ks = v; break; } }
  if (ks == 0 || (ks == 10 && p.nwaves == 8 && nf == 1)) return false;
  p.ksteps = ks;
  p.blocks = tiles < blk_target ? tiles : blk_target;
  p.rounds = (tiles + p.blocks - 1) / p.blocks;
  p.blocks = (tiles + p.rounds - 1) / p.rounds;
  const size_t part = (size_t)2 * nf * p.nwaves * 64 * 16, ssb = (size_t)p.nwaves * M * ks * 8 * 4;
  p.lds = (size_t)p.nwaves * 3 * M * (ks * 32 + 8) * 2 + (size_t)p.nwaves * 16 * 4 + (part > ssb ? part : ssb) +
          (size_t)p.nwaves * 16 * 8;
  return p.lds <= 160 * 1024 && p.blocks <= gemv_max_blocks();
}

// Number of K windows (1, 2, 4 or 8) the product is computed in, 0 if it does not fit this kernel.
// Windows are used when the staged activations of a whole row do not fit in LDS, and when the
// product has too few weight tiles to occupy the chip (N small, K long): the windows run side
// by side as gridDim.y and a reduction kernel adds them.
static int skinny_windows(const GemvArgs& g, SkinnyPlan& p) {
  constexpr int min_blocks = 192;
  const int tiles = (g.seg[0].n_rows + 15) / 16;
  // the reduction handles store / residual add and the norm scale; not SwiGLU or argmax partials
  const bool can_split = g.epi != EPI_SWIGLU && g.best == nullptr &&
                         (size_t)8 * g.M * g.seg[0].n_rows + 256 <= gemm_partial_elems();
  int best = 0;
  SkinnyPlan q;
  for (int w = 1; w <= 8; w *= 2) {
    if (w > 1 && (!can_split || g.K % (32 * w) != 0 || g.K / w < 256)) break;
    if (!skinny_plan_k(g, g.K / w, q)) continue;
    q.windows = w;
    p = q; best = w;
    if (tiles >= 128 || tiles * w >= min_blocks) break;   // half the chip by tiles alone: no split
  }
  return best;
}

template <int EPI, int NWAVES, int KSTEPS>
static hipError_t skinny_launch_one(const SkinnyArgs& a, const SkinnyPlan& p, hipStream_t s) {
  auto kern = skinny_mfma_kernel<EPI, NWAVES, KSTEPS>;
  static size_t lds_enabled = 48 * 1024;
  if (p.lds > lds_enabled) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)p.lds);
    if (e != hipSuccess) return e;
    lds_enabled = p.lds;
  }
  hipLaunchKernelGGL(kern, dim3(p.blocks, p.windows), dim3(64 * NWAVES), p.lds, s, a);
  return hipGetLastError();
}

template <int EPI>
static hipError_t skinny_dispatch(const SkinnyArgs& a, const SkinnyPlan& p, hipStream_t s) {
  constexpr bool sw = EPI == EPI_SWIGLU;
  if (p.nwaves == 8) {
    switch (p.ksteps) {
      case 1: return skinny_launch_one<EPI, 8, 1>(a, p, s);
      case 2: return skinny_launch_one<EPI, 8, 2>(a, p, s);
      case 3: return skinny_launch_one<EPI, 8, 3>(a, p, s);
      case 4: return skinny_launch_one<EPI, 8, 4>(a, p, s);
      case 5: return skinny_launch_one<EPI, 8, 5>(a, p, s);
      case 6: return skinny_launch_one<EPI, 8, 6>(a, p, s);
      case 8: return skinny_launch_one<EPI, 8, 8>(a, p, s);
      case 10: if (sw) return skinny_launch_one<EPI, 8, (sw ? 10 : 1)>(a, p, s); break;
    }
  } else if (!sw) {
    constexpr int E2 = sw ? EPI_STORE : EPI;
    switch (p.ksteps) {
      case 4: return skinny_launch_one<E2, 16, 4>(a, p, s);
      case 5: return skinny_launch_one<E2, 16, 5>(a, p, s);
      case 6: return skinny_launch_one<E2, 16, 6>(a, p, s);
      case 8: return skinny_launch_one<E2, 16, 8>(a, p, s);
      case 10: return skinny_launch_one<E2, 16, 10>(a, p, s);
      case 14: return skinny_launch_one<E2, 16, 14>(a, p, s);
    }
  }
  return hipErrorInvalidValue;
}

// true if the product fits this kernel (bf16 weights, 1..16 rows, K slices that fit registers and LDS)
bool skinny_mfma_fits(const GemvArgs& g) {
  SkinnyPlan p;
  return g.bf16 && g.n_seg == 1 && g.M >= 1 && g.M <= 16 && g.K % 8 == 0 && g.K >= 32 && g.ldx % 4 == 0 &&
         skinny_windows(g, p) > 0;
}

// `partial`: scratch of gemm_partial_elems() floats, used when the product is computed in K windows
hipError_t launch_skinny_mfma(const GemvArgs& g, float* partial, int* n_blocks_out, hipStream_t s) {
  SkinnyPlan p;
  if (!skinny_mfma_fits(g)) return hipErrorInvalidValue;
  const int windows = skinny_windows(g, p);
  if (g.seg[0].n_rows <= 0) return hipSuccess;
  if (windows > 1 && partial == nullptr) return hipErrorInvalidValue;
  SkinnyArgs a{};
  a.X = g.X; a.X2 = g.X2; a.R2 = g.R2; a.ldx = g.ldx; a.M = g.M; a.norm_w = g.norm_w; a.eps = g.eps;
  a.W = static_cast<const uint16_t*>(g.seg[0].W); a.W2 = static_cast<const uint16_t*>(g.seg[0].W2);
  a.Y = g.seg[0].Y; a.ldy = g.seg[0].ldy; a.N = g.seg[0].n_rows; a.best = g.best;
  a.rounds = p.rounds; a.kst_row = (g.K + 31) / 32; a.rnorm_k = 1.0f / (float)g.K;
  a.K = g.K / windows; a.k0 = 0;
  if (n_blocks_out) *n_blocks_out = p.blocks;
  int epi = g.epi;
  const size_t total = (size_t)g.M * a.N;
  // Windows that are only there because a whole row does not fit LDS, on a product that fills the
  // chip by itself: one launch per window, each accumulating on the output (side by side they
  // would need a second round of workgroups and the reduction pass).
  const int tiles = (a.N + 15) / 16;
  if (windows > 1 && tiles * windows > 256 && g.norm_w == nullptr && g.epi != EPI_SWIGLU && g.best == nullptr) {
    p.windows = 1;
    for (int w = 0; w < windows; ++w) {
      a.k0 = w * a.K;
      if (w > 0) a.R2 = nullptr;                   // the second residual goes in with the first window
      const int e1 = w == 0 ? g.epi : EPI_ADD;     // later windows accumulate
      hipError_t e = e1 == EPI_STORE ? skinny_dispatch<EPI_STORE>(a, p, s) : skinny_dispatch<EPI_ADD>(a, p, s);
      if (e != hipSuccess) return e;
    }
    return hipSuccess;
  }
  if (windows > 1) {
    a.Y = partial; a.ldy = a.N; a.ywin = total; a.R2 = nullptr; epi = EPI_STORE;
    a.ssq = g.norm_w != nullptr ? partial + (size_t)windows * total : nullptr;
  }
  hipError_t e = hipErrorInvalidValue;
  switch (epi) {
    case EPI_STORE: e = skinny_dispatch<EPI_STORE>(a, p, s); break;
    case EPI_ADD: e = skinny_dispatch<EPI_ADD>(a, p, s); break;
    case EPI_SWIGLU: e = skinny_dispatch<EPI_SWIGLU>(a, p, s); break;
  }
  if (e != hipSuccess || windows == 1) return e;
  return launch_gemm_reduce(g.epi, partial, windows, g.M, a.N, g.seg[0].Y, g.seg[0].ldy, g.R2, a.ssq, 16, a.rnorm_k, g.eps, nullptr, 1, s);
}

}  // namespace hh
