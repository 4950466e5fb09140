// SSM branch of the hybrid block: causal depthwise conv over a ring of raw inputs,
// then the scalar-decay selective state update
//     S <- a * S + (dt * x) (outer) B,   y = S C + D x,   out = y * silu(z)
// for up to T consecutive positions per sequence, with the state held in registers.
//
// One kernel serves the three uses of the recurrence on the hot path:
//   draft step   T = 1, reads the committed state (first step) or the draft scratch, writes the scratch;
//   verification T = k+1, reads the committed state and writes nothing back: the raw inputs of the
//                T positions go to the ring, which is all a later rollback needs;
//   commit       re-runs the first n+1 of those positions from the ring and writes the committed
//                state: the state after position n, bit-identical to what verification held.
// Prefill uses the verification form with a state write-back per chunk.
//
// Layout: S[b][h][p][n] float32, n fastest.  A workgroup owns kRows (8 or 32) rows p of one head; 8 lanes
// share a row, each holding N/8 consecutive n in registers; the read-out over n is reduced
// across those 8 lanes.  Ring row for position q: slot q mod ring_slots, [conv_dim raw xBC | Hm raw dt].
#include "hh_internal.h"

namespace hh {

static constexpr int kSub = 8;     // lanes per row
static constexpr int kTS = 16;     // positions staged per pass through LDS

__device__ __forceinline__ float silu_f(float v) { return v / (1.0f + expf(-v)); }
__device__ __forceinline__ float softplus_f(float v) { return v > 20.0f ? v : log1pf(expf(v)); }

template <int CTRL>
__device__ __forceinline__ float dpp_perm_f(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, false));
}

// kRows = 8: one wavefront per workgroup, many small workgroups (latency-bound small batches);
// kRows = 32: four wavefronts, the conv of B and C is shared by four times as many state rows.
template <int NV, int kRows>
__global__ __launch_bounds__(kRows * kSub) void ssm_kernel(const Dims d, const SsmArgs a) {
  constexpr int N = NV * kSub;
  __shared__ float xs[kTS][kRows];
  __shared__ float Bs[kTS][N];
  __shared__ float Cs[kTS][N];
  __shared__ float dts[kTS], as[kTS];

  const int tid = threadIdx.x, row = tid >> 3, sub = tid & 7;
  const int p0 = blockIdx.x * kRows, h = blockIdx.y;
  const int lz = blockIdx.z / a.B, b = blockIdx.z % a.B;
  // one layer: its pointers arrive by value in the kernel arguments; several: from the table
  const LayerDev& ly = a.layers != nullptr ? a.layers[a.layer0 + lz] : a.one;
  if (a.skip != nullptr && a.skip[b]) return;
  int nt = a.T;
  if (a.n_acc != nullptr) nt = a.n_acc[b] + 1;
  else if (a.n_tok != nullptr) nt = a.n_tok[b];
  if (nt <= 0) return;
  const int pos0 = a.pos0[b];
  const int p = p0 + row;
  const bool prow = p < d.P;
  const int rmask = d.ring_slots - 1;
  const float* ring = ly.ring + (size_t)b * d.ring_slots * d.ring_w;
  const float* zx = a.zx != nullptr ? a.zx + (size_t)b * a.T * d.ldzx : nullptr;

  // raw (pre-conv) input of channel c (c < conv_dim: xBC, else dt of head c - conv_dim) at position pos
  // (one unconditional load from a selected address, so that independent loads overlap)
  auto raw = [&](int pos, int c) -> float {
    const float* p = (zx != nullptr && pos >= pos0) ? zx + (size_t)(pos - pos0) * d.ldzx + d.d_inner + c
                                                    : ring + (size_t)(max(pos, 0) & rmask) * d.ring_w + c;
    const float v = *p;
    return pos < 0 ? 0.f : v;
  };

  float S[NV];
  {
    const float* src = a.state_in == 0 ? ly.S : (a.state_in == 1 ? ly.S_draft : nullptr);
    if (src != nullptr && prow) {
      const float* sp = src + (((size_t)b * d.Hm + h) * d.P + p) * N + sub * NV;
      if (NV % 4 == 0) {
#pragma unroll
        for (int i = 0; i < NV; i += 4) {
          const float4 v = *reinterpret_cast<const float4*>(sp + i);
          S[i] = v.x; S[i + 1] = v.y; S[i + 2] = v.z; S[i + 3] = v.w;
        }
      } else {
#pragma unroll
        for (int i = 0; i < NV; ++i) S[i] = sp[i];
      }
    } else {
#pragma unroll
      for (int i = 0; i < NV; ++i) S[i] = 0.f;
    }
  }
  const float dskip = ly.d_skip[h];
  const float dtb = ly.dt_bias[h];
  const float negA = -expf(ly.a_log[h]);

  for (int j0 = 0; j0 < nt; j0 += kTS) {
    const int tc = min(kTS, nt - j0);
    // ---- conv + SiLU for this workgroup's x rows and for B, C
    const int nch = kRows + 2 * N;
    for (int it = tid; it < tc * nch; it += kRows * kSub) {
      const int jj = it / nch, ci = it % nch;
      int c;
      bool ok = true;
      if (ci < kRows) { c = h * d.P + p0 + ci; ok = p0 + ci < d.P; }
      else c = d.d_inner + (ci - kRows);
      float out = 0.f;
      if (ok) {
        const int pos = pos0 + j0 + jj;
        const float4 taps = *reinterpret_cast<const float4*>(ly.conv_w + (size_t)c * 4);
        const float bias = ly.conv_b[c];
        const float r0 = raw(pos - 3, c), r1 = raw(pos - 2, c), r2 = raw(pos - 1, c), r3 = raw(pos, c);
        float acc = taps.x * r0;
        acc = fmaf(taps.y, r1, acc); acc = fmaf(taps.z, r2, acc); acc = fmaf(taps.w, r3, acc);
        out = silu_f(acc + bias);
      }
      if (ci < kRows) xs[jj][ci] = out;
      else if (ci < kRows + N) Bs[jj][ci - kRows] = out;
      else Cs[jj][ci - kRows - N] = out;
    }
    if (tid < tc) {
      const float dt = softplus_f(raw(pos0 + j0 + tid, d.conv_dim + h) + dtb);
      dts[tid] = dt;
      as[tid] = expf(negA * dt);
    }
    // ---- keep the raw inputs of these positions for later windows and for rollback
    if (a.write_ring && zx != nullptr) {
      float* wr = ly.ring + (size_t)b * d.ring_slots * d.ring_w;
      for (int it = tid; it < tc * kRows; it += kRows * kSub) {
        const int jj = it / kRows, ci = it % kRows;
        if (p0 + ci < d.P) {
          const int c = h * d.P + p0 + ci, pos = pos0 + j0 + jj;
          wr[(size_t)(pos & rmask) * d.ring_w + c] = raw(pos, c);
        }
      }
      if (h == 0 && blockIdx.x == 0) {
        const int extra = 2 * N + d.Hm;
        for (int it = tid; it < tc * extra; it += kRows * kSub) {
          const int jj = it / extra, c = d.d_inner + it % extra, pos = pos0 + j0 + jj;
          wr[(size_t)(pos & rmask) * d.ring_w + c] = raw(pos, c);
        }
      }
    }
    __syncthreads();
    // ---- recurrence over the staged positions
    for (int jj = 0; jj < tc; ++jj) {
      const float xv = xs[jj][row];
      const float coef = dts[jj] * xv, aj = as[jj];
      float part = 0.f;
#pragma unroll
      for (int i = 0; i < NV; ++i) {
        S[i] = fmaf(aj, S[i], coef * Bs[jj][sub * NV + i]);
        part = fmaf(S[i], Cs[jj][sub * NV + i], part);
      }
      part += dpp_perm_f<0xB1>(part);    // lane ^ 1
      part += dpp_perm_f<0x4E>(part);    // lane ^ 2
      part += dpp_perm_f<0x141>(part);   // the other quad of the 8 lanes that share a row
      if (a.g != nullptr && sub == 0 && prow) {
        const size_t m = (size_t)b * a.T + j0 + jj;
        const float z = a.zx[m * d.ldzx + h * d.P + p];
        a.g[m * d.d_inner + h * d.P + p] = (part + dskip * xv) * silu_f(z);
      }
    }
    __syncthreads();
  }

  if (a.state_out != 0 && prow) {
    float* dst = (a.state_out == 1 ? ly.S : ly.S_draft) + (((size_t)b * d.Hm + h) * d.P + p) * N + sub * NV;
    if (NV % 4 == 0) {
#pragma unroll
      for (int i = 0; i < NV; i += 4) *reinterpret_cast<float4*>(dst + i) = make_float4(S[i], S[i + 1], S[i + 2], S[i + 3]);
    } else {
#pragma unroll
      for (int i = 0; i < NV; ++i) dst[i] = S[i];
    }
  }
}

template <int kRows>
static hipError_t launch_ssm_rows(const Dims& d, const SsmArgs& a, hipStream_t s) {
  const dim3 grid((d.P + kRows - 1) / kRows, d.Hm, a.n_layers_z * a.B);
  const dim3 block(kRows * kSub);
  switch (d.N / kSub) {
    case 1: hipLaunchKernelGGL((ssm_kernel<1, kRows>), grid, block, 0, s, d, a); break;
    case 2: hipLaunchKernelGGL((ssm_kernel<2, kRows>), grid, block, 0, s, d, a); break;
    case 4: hipLaunchKernelGGL((ssm_kernel<4, kRows>), grid, block, 0, s, d, a); break;
    case 8: hipLaunchKernelGGL((ssm_kernel<8, kRows>), grid, block, 0, s, d, a); break;
    case 16: hipLaunchKernelGGL((ssm_kernel<16, kRows>), grid, block, 0, s, d, a); break;
    case 32: hipLaunchKernelGGL((ssm_kernel<32, kRows>), grid, block, 0, s, d, a); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

hipError_t launch_ssm(const Dims& d, const SsmArgs& a, hipStream_t s) {
  if (d.N % kSub != 0) return hipErrorInvalidValue;
  // enough 32-row workgroups to cover the chip twice: take them, else 8-row ones
  const long big = (long)((d.P + 31) / 32) * d.Hm * a.n_layers_z * a.B;
  (void)big;
  return launch_ssm_rows<32>(d, a, s);
}

// Committed conv window (the d_conv-1 raw inputs before position kv_len, oldest first) of one layer,
// exported as [B][conv_dim][3] for read-back.
__global__ void export_conv_kernel(const Dims d, const LayerDev* layer, const int* kv_len, float* out) {
  const int b = blockIdx.x;
  const int len = kv_len[b];
  const float* ring = layer->ring + (size_t)b * d.ring_slots * d.ring_w;
  for (int it = threadIdx.x; it < d.conv_dim * 3; it += blockDim.x) {
    const int c = it / 3, t = it % 3, pos = len - 3 + t;
    out[((size_t)b * d.conv_dim + c) * 3 + t] =
        pos < 0 ? 0.f : ring[(size_t)(pos & (d.ring_slots - 1)) * d.ring_w + c];
  }
}

hipError_t launch_export_state(const Dims& d, const LayerDev* layer, const int* kv_len, int B, float* conv_out,
                               hipStream_t s) {
  hipLaunchKernelGGL(export_conv_kernel, dim3(B), dim3(256), 0, s, d, layer, kv_len, conv_out);
  return hipGetLastError();
}

}  // namespace hh
