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
// One workgroup of eight wavefronts per (sequence, pair of heads), head dimension P = 64: B, C
// and G = C B^T do not depend on the head, so their convolution is shared by the pair, and two
// wavefronts per SIMD hide each other's LDS latency.  Wavefront 4 hh + wq owns the 16 rows
// p = 16 wq .. 16 wq + 15 of head hh of the pair for everything - its slice of the state,
// transposed (n down, p across), lives in MFMA accumulator registers for the whole pass and is
// fed back as the A operand of the read-out product as it is: lane (g, j) holds S[p = 16 wq + j]
// [n = 16 tile + 4 g + r], which the instruction takes as A[row j][k = g] when the B operand is
// read with the same n for k = g.  Per chunk of 32 positions: the convolution + SiLU of x, B, C (a
// thread takes 4 channels through 16 positions; the raw rows of the next chunk are requested
// before the products of this one, so their latency hides behind the MFMAs), the step sizes and
// their running sum, then  G = C B^T  (three 16 x 16 tiles at or below the diagonal), the masked
// and scaled M of each head to LDS, the read-out of the old state, the intra-chunk product M x,
// the outputs y * silu(z), and the state update.  B is kept row-major and C transposed in LDS,
// padded so that the operand reads of the two large products are free of bank conflicts.
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
  static constexpr int kB = 0;                         // B  [L][LDB]      (position, n)
  static constexpr int kCt = kB + kSsdL * LDB;         // C^T [N][LDT]     (n, position)
  static constexpr int kX = kCt + N * LDT;             // x  [2][L][LDX]   (head of the pair, position, p)
  static constexpr int kM = kX + 2 * kSsdL * LDX;      // M  [2][L][LDM]   (head of the pair, t, i)
  static constexpr int kDt = kM + 2 * kSsdL * LDM;     // dt [2][L]
  static constexpr int kCum = kDt + 2 * kSsdL;         // cum [2][L]
  static constexpr int kFloats = kCum + 2 * kSsdL;
};

template <int N>
__global__ __launch_bounds__(512) void ssd_mfma_kernel(const Dims d, const SsmArgs a) {
  typedef SsdLds<N> Lds;
  constexpr int L = kSsdL, P = kSsdP, NT = N / 16, HALF = L / 2;
  constexpr int LDB = Lds::LDB, LDT = Lds::LDT, LDX = Lds::LDX, LDM = Lds::LDM;
  constexpr int NG = (2 * P + 2 * N) / 4;              // conv channel groups of 4: x of head 0 | x of head 1 | B | C
  static_assert(2 * ((NG + 63) / 64) <= 6, "the staging tasks (a channel group x half a chunk) fit the first six wavefronts");
  extern __shared__ __align__(16) float ssd_smem[];
  float* Bs = ssd_smem + Lds::kB;
  float* Ct = ssd_smem + Lds::kCt;

  const int tid = threadIdx.x, lane = tid & 63, w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int hh = w >> 2, wq = w & 3;                   // head of the pair, 16-row slice of the head
  const int g = lane >> 4, j = lane & 15;
  const int h = 2 * blockIdx.x + hh, b = blockIdx.y;
  float* Xs = ssd_smem + Lds::kX + hh * L * LDX;
  float* Ms = ssd_smem + Lds::kM + hh * L * LDM;
  float* dts = ssd_smem + Lds::kDt + hh * L;
  float* cums = ssd_smem + Lds::kCum + hh * L;
  const LayerDev& ly = a.one;
  int nt = a.T;
  if (a.n_tok != nullptr) nt = a.n_tok[b];
  if (nt <= 0) return;
  const int pos0 = a.pos0[b];
  const int rmask = d.ring_slots - 1;
  float* ring = ly.ring + (size_t)b * d.ring_slots * d.ring_w;
  const float* zx = a.zx + (size_t)b * a.T * d.ldzx;

  // ---- state slice of this wavefront, transposed: acc[tile][r] = S[16 wq + j][16 tile + 4 g + r]
  ssd_f32x4 S[NT];
  {
    const float* src = a.state_in == 0 ? ly.S : (a.state_in == 1 ? ly.S_draft : nullptr);
    if (src != nullptr) {
      const float* sp = src + (((size_t)b * d.Hm + h) * P + 16 * wq + j) * N + 4 * g;
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

  // ---- staging role: a task is (channel group sg < NG, half sh of the chunk); the tasks of a half fill whole
  // wavefronts (WPH of them), so that the row a wavefront loads is uniform and its address scalar
  constexpr int WPH = (NG + 63) / 64;
  const int sh = w / WPH < 2 ? w / WPH : 0, sg_raw = tid - 64 * WPH * sh;
  const bool stager = w < 2 * WPH && sg_raw < NG;
  const int sg = stager ? sg_raw : 0;
  // first of the 4 channels (index into xBC) and where its outputs go
  const int ch = sg < P / 4 ? (2 * blockIdx.x) * P + 4 * sg : sg < 2 * (P / 4) ? (2 * blockIdx.x + 1) * P + 4 * (sg - P / 4) : d.d_inner + 4 * (sg - 2 * (P / 4));
  float4 tw[4], bias = make_float4(0.f, 0.f, 0.f, 0.f);
  // raw xBC row of a position: this pass's projections, or the ring for the three positions before it
  // (rows[0..2]: the window before the task's first position; rows[3 + u]: its positions, clamped to
  // the pass; a macro, not a lambda: an array captured by reference may end up in scratch memory)
  const unsigned choff = (unsigned)(d.d_inner + ch), rchoff = (unsigned)ch;
  float4 rows[3 + HALF / 2];
  // rows[LO_ .. 3 + HALF / 2) <- raw rows of the positions first_ - 3 + LO_ ... (first_: chunk-local index of the
  // batch's first position, uniform over the wavefront: scalar row address + the lane's channel offset)
#define HH_SSD_REQUEST(first_, LO_)                                                                      \
  do {                                                                                                   \
    _Pragma("unroll") for (int u = (LO_); u < 3 + HALF / 2; ++u) {                                       \
      const int pos_ = pos0 + min((first_) - 3 + u, nt - 1);                                             \
      const bool here_ = pos_ >= pos0;                                                                   \
      const float* rb_ = here_ ? zx + (size_t)(pos_ - pos0) * d.ldzx : ring + (size_t)(max(pos_, 0) & rmask) * d.ring_w; \
      const float4 v_ = *reinterpret_cast<const float4*>(rb_ + (here_ ? choff : rchoff));                \
      rows[u] = pos_ < 0 ? make_float4(0.f, 0.f, 0.f, 0.f) : v_;                                         \
    }                                                                                                    \
  } while (0)
  if (stager) HH_SSD_REQUEST(HALF * sh, 0);

  TR(0);
  for (int j0 = 0; j0 < nt; j0 += L) {
    const int tc = min(L, nt - j0);
    if (j0 == 0) TR(1);
    // ================= staging: conv + SiLU of x, B, C; dt and its running log-decay sum
    if (stager) {
      // (taps and biases are re-read per chunk from the cache rather than held in 20 registers across the products)
#pragma unroll
      for (int q = 0; q < 4; ++q) tw[q] = *reinterpret_cast<const float4*>(ly.conv_w + (size_t)(ch + q) * 4);
      bias = *reinterpret_cast<const float4*>(ly.conv_b + ch);
      const float bq[4] = {bias.x, bias.y, bias.z, bias.w};
      // two batches of 8 positions: the first one's rows were requested a chunk ago, the second one's are
      // requested when the first is done (registers: 11 rows at a time)
#pragma unroll
      for (int half2 = 0; half2 < 2; ++half2) {
        if (half2 == 1) {
          asm volatile("" ::: "memory");
          rows[0] = rows[HALF / 2]; rows[1] = rows[HALF / 2 + 1]; rows[2] = rows[HALF / 2 + 2];
          HH_SSD_REQUEST(j0 + HALF * sh + HALF / 2, 3);
        }
#pragma unroll
        for (int u = 0; u < HALF / 2; ++u) {
          const int jj = HALF * sh + (HALF / 2) * half2 + u;
          const bool on = jj < tc;
          const float4 q0 = rows[u], q1 = rows[u + 1], q2 = rows[u + 2], q3 = rows[u + 3];
          const float x0[4] = {q0.x, q0.y, q0.z, q0.w}, x1[4] = {q1.x, q1.y, q1.z, q1.w}, x2[4] = {q2.x, q2.y, q2.z, q2.w},
                      x3[4] = {q3.x, q3.y, q3.z, q3.w};
          float o[4];
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            float acc = tw[q].x * x0[q];
            acc = fmaf(tw[q].y, x1[q], acc); acc = fmaf(tw[q].z, x2[q], acc); acc = fmaf(tw[q].w, x3[q], acc);
            o[q] = on ? ssd_silu(acc + bq[q]) : 0.f;
          }
          if (sg < 2 * (P / 4)) {
            *reinterpret_cast<float4*>(ssd_smem + Lds::kX + (sg / (P / 4)) * L * LDX + jj * LDX + 4 * (sg % (P / 4))) = make_float4(o[0], o[1], o[2], o[3]);
          } else if (sg < 2 * (P / 4) + N / 4) {
            *reinterpret_cast<float4*>(Bs + jj * LDB + 4 * (sg - 2 * (P / 4))) = make_float4(o[0], o[1], o[2], o[3]);
          } else {
            const int n0 = 4 * (sg - 2 * (P / 4) - N / 4);
#pragma unroll
            for (int q = 0; q < 4; ++q) Ct[(n0 + q) * LDT + jj] = o[q];
          }
          // the raw inputs stay in the ring for the next pass's window and for rollbacks (x of this pair
          // of heads by every workgroup, B and C by the workgroup of the first pair)
          if (on && a.write_ring && (sg < 2 * (P / 4) || blockIdx.x == 0))
            *reinterpret_cast<float4*>(ring + (size_t)((pos0 + j0 + jj) & rmask) * d.ring_w + ch) = q3;
        }
      }
      asm volatile("" ::: "memory");                   // (not before this chunk's rows are dead: registers)
      if (j0 + L < nt) HH_SSD_REQUEST(j0 + L + HALF * sh, 0);   // the next chunk's first rows travel while this one is multiplied
    } else if (w >= 6 && lane < L) {
      // wavefront 6 + hh': step sizes and log-decay sums of head hh' (= this wavefront's own head: 6 >> 2 = 7 >> 2 = 1
      // does not hold, so index explicitly)
      const int hp = w - 6, hd = 2 * blockIdx.x + hp;
      const bool on = lane < tc;
      const float rawdt = zx[(size_t)(j0 + min(lane, tc - 1)) * d.ldzx + d.d_inner + d.conv_dim + hd];
      const float dt = on ? ssd_softplus(rawdt + ly.dt_bias[hd]) : 0.f;
      if (on && a.write_ring) ring[(size_t)((pos0 + j0 + lane) & rmask) * d.ring_w + d.conv_dim + hd] = rawdt;
      float c = -expf(ly.a_log[hd]) * dt;              // log a_t, summed over the positions up to t
#pragma unroll
      for (int o = 1; o < L; o <<= 1) {
        const float up = __shfl_up(c, o, 64);
        if (lane >= o) c += up;
      }
      ssd_smem[Lds::kDt + hp * L + lane] = dt;
      ssd_smem[Lds::kCum + hp * L + lane] = c;
    }
    __syncthreads();
    if (j0 == 0) TR(2);

    // ================= G = C B^T on the tiles at or below the diagonal, M = G * decay * dt to LDS
    {
      const int tt = wq == 0 ? 0 : 1, it = wq == 2 ? 1 : 0;        // slice 3: the tile above the diagonal is zero
      ssd_f32x4 G = {0.f, 0.f, 0.f, 0.f};
      if (wq < 3) {
#pragma unroll 4
        for (int kk = 0; kk < N / 4; ++kk) {
          const float av = Ct[(4 * kk + g) * LDT + 16 * tt + j];   // A[row t = j][k = g] = C[t][n = 4 kk + g]
          const float bv = Bs[(16 * it + j) * LDB + 4 * kk + g];   // B[k = g][col i = j] = B[i][n = 4 kk + g]
          G = __builtin_amdgcn_mfma_f32_16x16x4f32(av, bv, G, 0, 0, 0);
        }
      }
      // lane (g, j) holds G[t = 16 tt' + 4 g + r][i = 16 it' + j]
      const int tt_w = wq == 3 ? 0 : tt, it_w = wq == 3 ? 1 : it;
      const int i = 16 * it_w + j;
      const float ci = cums[i], di = dts[i];
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int t = 16 * tt_w + 4 * g + r;
        const float m = (wq < 3 && i <= t) ? G[r] * di * expf(cums[t] - ci) : 0.f;
        Ms[t * LDM + i] = m;
      }
    }
    __syncthreads();
    if (j0 == 0) TR(3);

    // ================= read-out of the entering state, intra-chunk product, outputs
    ssd_f32x4 Y[2] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};   // Y[tt][r] = y[p = 16 wq + 4 g + r][t = 16 tt + j]
#pragma unroll
    for (int t = 0; t < NT; ++t) {
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const float* crow = Ct + (16 * t + 4 * g + r) * LDT + j;   // B[k = g][col j] = C[position][n = 16 t + 4 g + r]
        Y[0] = __builtin_amdgcn_mfma_f32_16x16x4f32(S[t][r], crow[0], Y[0], 0, 0, 0);
        Y[1] = __builtin_amdgcn_mfma_f32_16x16x4f32(S[t][r], crow[16], Y[1], 0, 0, 0);
      }
      if ((t & 1) == 1) asm volatile("" ::: "memory");   // operand reads at most two state tiles ahead (registers)
    }
    {
      const float e0 = expf(cums[j]), e1 = expf(cums[16 + j]);
#pragma unroll
      for (int r = 0; r < 4; ++r) { Y[0][r] *= e0; Y[1][r] *= e1; }
    }
#pragma unroll
    for (int kk = 0; kk < L / 4; ++kk) {
      const float xv = Xs[(4 * kk + g) * LDX + 16 * wq + j];       // A[row p = j][k = g] = x[i = 4 kk + g][p]
      if (kk < 4) Y[0] = __builtin_amdgcn_mfma_f32_16x16x4f32(xv, Ms[j * LDM + 4 * kk + g], Y[0], 0, 0, 0);
      Y[1] = __builtin_amdgcn_mfma_f32_16x16x4f32(xv, Ms[(16 + j) * LDM + 4 * kk + g], Y[1], 0, 0, 0);
    }
#pragma unroll
    for (int tt = 0; tt < 2; ++tt) {
      const int t = 16 * tt + j;
      if (t < tc) {
        const size_t m = (size_t)b * a.T + j0 + t;
        const int p = 16 * wq + 4 * g;
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
        const float xw = Xs[i * LDX + 16 * wq + j] * (dts[i] * expf(cl - cums[i]));  // B[k = g][col p = j]
        const float* brow = Bs + i * LDB + j;                                        // A[row n = j][k = g] = B[i][n]
#pragma unroll
        for (int t = 0; t < NT; ++t) S[t] = __builtin_amdgcn_mfma_f32_16x16x4f32(brow[16 * t], xw, S[t], 0, 0, 0);
        asm volatile("" ::: "memory");
      }
    }
    __syncthreads();
    if (j0 == 0) TR(5);
  }
  TR(6);

  if (a.state_out != 0) {
    float* dp = (a.state_out == 1 ? ly.S : ly.S_draft) + (((size_t)b * d.Hm + h) * P + 16 * wq + j) * N + 4 * g;
#pragma unroll
    for (int t = 0; t < NT; ++t) *reinterpret_cast<float4*>(dp + 16 * t) = make_float4(S[t][0], S[t][1], S[t][2], S[t][3]);
  }
  TR(7);
  (void)dtb; (void)negA;
#undef HH_SSD_REQUEST
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
  hipLaunchKernelGGL(kern, dim3(d.Hm / 2, a.B), dim3(512), lds, s, d, a);
  return hipGetLastError();
}

// true if the pass was taken by the matmul-form kernel: a single layer's pass over this call's
// projections with outputs, at least 16 positions, an even number of heads of dimension 64, state size 64, 128 or 256,
// 16-byte aligned rows
bool launch_ssd_mfma(const Dims& d, const SsmArgs& a, hipStream_t s, hipError_t* err) {
  if ((d.flags & HH_KF_SSM_SEQUENTIAL) || a.layers != nullptr || a.zx == nullptr || a.g == nullptr || a.n_acc != nullptr ||
      a.skip != nullptr || a.T < 16 || d.P != kSsdP || d.Hm % 2 != 0 || d.d_inner % 4 != 0 || d.ldzx % 4 != 0 || d.ring_w % 4 != 0 ||
      d.conv_dim % 4 != 0 || (reinterpret_cast<uintptr_t>(a.zx) & 15) != 0 || (reinterpret_cast<uintptr_t>(a.g) & 15) != 0)
    return false;
  // one workgroup per (sequence, pair of heads) walks the whole pass chunk by chunk: with few of them
  // (one sequence in prefill: 12 at the 0.5B shape, 20 at the 3B shape) the position-by-position kernel,
  // which splits every head over several workgroups and stages on wavefronts of its own, is faster
  // (measured: 12.1 against 15.2 ms, 164 against 184 ms; 16 sequences: 277 against 220 ms)
  if ((d.Hm / 2) * a.B < 128 && !(d.flags & HH_KF_SSM_MATMUL)) return false;
  switch (d.N) {
    case 64: *err = ssd_launch<64>(d, a, s); return true;
    case 128: *err = ssd_launch<128>(d, a, s); return true;
    case 256: *err = ssd_launch<256>(d, a, s); return true;
  }
  return false;
}

}  // namespace hh
