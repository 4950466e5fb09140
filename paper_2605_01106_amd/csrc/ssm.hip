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
#include <stdlib.h>

#include "hh_internal.h"
#include "wave_ops.h"
#include "trace.h"

namespace hh {

static constexpr int kSub = 8;     // lanes per row
static constexpr int kTS = 16;     // positions staged per pass through LDS

// v * sigmoid(v) with the hardware exponential and reciprocal (each within 1 ulp; the argument
// scaling of the exponential adds |v| * 2^-24 relative): the kernels below evaluate it for
// every conv channel of every position, with one wavefront per SIMD
__device__ __forceinline__ float silu_f(float v) { return v * __frcp_rn(1.0f + __expf(-v)); }
__device__ __forceinline__ float softplus_f(float v) { return v > 20.0f ? v : log1pf(expf(v)); }


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
      part += dpp_move<0xB1>(part);    // lane ^ 1
      part += dpp_move<0x4E>(part);    // lane ^ 2
      part += dpp_move<0x141>(part);   // the other quad of the 8 lanes that share a row
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

// ---- few positions per pass (draft steps, verification, rollback), 16-byte aligned rows.
// One wavefront per workgroup owns 64/SUBS rows p of one head, SUBS lanes share a row.  Every
// global load of the workgroup (state, conv taps and biases, the raw inputs of the T positions
// and of the 3 before them, dt, z) is issued before the first result is used, so the kernel
// costs about one memory round trip plus the recurrence.  The conv of B and C is computed
// once per workgroup, 4 channels per lane, and handed to the lanes through LDS.
// The same for aligned shapes (rows, channels and row strides multiples of 4): the convolution of a
// chunk of positions is done by one thread per group of 4 channels (B, C and this workgroup's x
// rows) walking the positions with a sliding window of float4 rows - all loads of a half chunk in
// flight together, taps and bias loaded once - instead of one scalar item per channel and position,
// and the gate inputs z are staged with x, so the recurrence loop touches no global memory but
// its output.  (Prefill chunks: the scalar staging made the pass latency-bound.)
// Threads of the staging role of ssm_chunk_kernel when it has wavefronts of its own: kPipeSets sets
// (one per part of a chunk, so that the loads of all parts are in flight together) of one thread
// per group of 4 conv channels (B | C | the workgroup's x rows), plus one per staged position (step
// and decay), rounded up to whole wavefronts.
static constexpr int kPipeSets = 4;
template <int NV, int kRows>
constexpr int chunk_stage_threads() { return ((kPipeSets * (2 * NV * kSub / 4 + kRows / 4) + kTS + 63) / 64) * 64; }

// PIPE: the staging role gets wavefronts of its own (behind the kRows * kSub recurrence threads) and
// stages chunk c+1 into the other LDS buffer while the recurrence runs over chunk c, so the global
// loads and the convolution of a chunk are off the recurrence's path: for small launches (one
// sequence in prefill), where no other workgroup on the compute unit hides them.
template <int NV, int kRows, bool PIPE>
__global__ __launch_bounds__(kRows * kSub + (PIPE ? chunk_stage_threads<NV, kRows>() : 0)) void ssm_chunk_kernel(const Dims d, const SsmArgs a) {
  constexpr int N = NV * kSub;
  constexpr int NSETS = PIPE ? kPipeSets : 1;                      // conv thread sets (one part of a chunk each)
  constexpr int NPARTS = PIPE ? kPipeSets : 2;                     // parts a chunk is staged in
  constexpr int NGBC = 2 * N / 4, NGX = kRows / 4, HP = kTS / NPARTS;
  constexpr int NREC = kRows * kSub;                               // recurrence threads
  constexpr int NSTG = PIPE ? chunk_stage_threads<NV, kRows>() : NREC;   // threads that can take the staging role
  constexpr int NBUF = PIPE ? 2 : 1;
  static_assert(NSETS * (NGBC + NGX) + kTS <= NSTG, "one thread per channel group and per staged position");
  __shared__ __align__(16) float xs[NBUF][kTS][kRows];
  __shared__ __align__(16) float zs[NBUF][kTS][kRows];
  __shared__ __align__(16) float Bs[NBUF][kTS][N];
  __shared__ __align__(16) float Cs[NBUF][kTS][N];
  __shared__ float dts[NBUF][kTS], as[NBUF][kTS];

  const int tid = threadIdx.x, row = (tid >> 3) % kRows, sub = tid & 7;
  const bool stager = !PIPE || tid >= NREC;
  const bool worker = !PIPE || tid < NREC;
  const int stid = PIPE ? tid - NREC : tid;                        // index within the staging role
  const int p0 = blockIdx.x * kRows, h = blockIdx.y;
  const int lz = blockIdx.z / a.B, b = blockIdx.z % a.B;
  const LayerDev& ly = a.layers != nullptr ? a.layers[a.layer0 + lz] : a.one;
  if (a.skip != nullptr && a.skip[b]) return;
  int nt = a.T;
  if (a.n_acc != nullptr) nt = a.n_acc[b] + 1;
  else if (a.n_tok != nullptr) nt = a.n_tok[b];
  if (nt <= 0) return;
  const int pos0 = a.pos0[b];
  const int p = p0 + row;
  const bool prow = worker && p < d.P;
  const int rmask = d.ring_slots - 1;
  float* ring = ly.ring + (size_t)b * d.ring_slots * d.ring_w;
  const float* zx = a.zx != nullptr ? a.zx + (size_t)b * a.T * d.ldzx : nullptr;
  // row of raw inputs (xBC | dt) of position pos (positions < 0 read slot 0 and count as 0)
  auto raw_row = [&](int pos) -> const float* {
    return (zx != nullptr && pos >= pos0) ? zx + (size_t)(pos - pos0) * d.ldzx + d.d_inner
                                          : ring + (size_t)(max(pos, 0) & rmask) * d.ring_w;
  };

  float S[NV];
  {
    const float* src = a.state_in == 0 ? ly.S : (a.state_in == 1 ? ly.S_draft : nullptr);
    if (src != nullptr && prow) {
      const float* sp = src + (((size_t)b * d.Hm + h) * d.P + p) * N + sub * 4;   // float4 i of a lane is elements (i/4)*4*kSub + 4*sub ..: a row group reads 16*kSub contiguous bytes
#pragma unroll
      for (int i = 0; i < NV; i += 4) {
        const float4 v = *reinterpret_cast<const float4*>(sp + i * kSub);
        S[i] = v.x; S[i + 1] = v.y; S[i + 2] = v.z; S[i + 3] = v.w;
      }
    } else {
#pragma unroll
      for (int i = 0; i < NV; ++i) S[i] = 0.f;
    }
  }
  const float dskip = ly.d_skip[h];
  const float dtb = ly.dt_bias[h];
  const float negA = -expf(ly.a_log[h]);
  // this thread's channel group: B|C groups first, then the x rows of the workgroup
  const bool conv_thread = stager && stid >= 0 && stid < NSETS * (NGBC + NGX);
  const int cset = max(stid, 0) / (NGBC + NGX);              // which part of a chunk this thread stages (several sets)
  const int cid = max(stid, 0) % (NGBC + NGX);               // channel group
  const bool is_x = cid >= NGBC;
  const int xg = cid - NGBC;                                 // x group (is_x)
  const bool active = conv_thread && (!is_x || p0 + 4 * xg < d.P);
  const int c4 = is_x ? h * d.P + min(p0 + 4 * xg, d.P - 4) : d.d_inner + 4 * cid;
  // the step-and-decay threads: the last kTS of the staging role
  const int dt_jj = stid - (NSTG - kTS);
  float4 taps[4], bias;
#pragma unroll
  for (int t = 0; t < 4; ++t) taps[t] = *reinterpret_cast<const float4*>(ly.conv_w + (size_t)(c4 + t) * 4);
  bias = *reinterpret_cast<const float4*>(ly.conv_b + c4);

  // conv inputs, gate inputs, step and decay of positions j0 .. j0 + kTS - 1 into LDS buffer `buf`
  auto stage = [&](int j0, int buf) {
    const int tc = min(kTS, nt - j0);
    if (conv_thread) {
      for (int hp = (NSETS > 1 ? cset : 0); hp < (NSETS > 1 ? cset + 1 : NPARTS); ++hp) {
        const int jb = j0 + hp * HP;                           // first position of the part (relative)
        if (jb >= j0 + tc) break;
        // raw rows of positions jb-3 .. jb+HP-1 (clamped to the last valid one), z of jb .. jb+HP-1
        float4 r[HP + 3], z[HP];
#pragma unroll
        for (int u = 0; u < HP + 3; ++u) {
          const int pos = pos0 + min(jb + u - 3, nt - 1);
          r[u] = *reinterpret_cast<const float4*>(raw_row(pos) + c4);
          if (pos < 0) r[u] = make_float4(0.f, 0.f, 0.f, 0.f);
        }
        if (is_x && a.g != nullptr) {
#pragma unroll
          for (int u = 0; u < HP; ++u)
            z[u] = *reinterpret_cast<const float4*>(zx + (size_t)min(jb + u, nt - 1) * d.ldzx + (c4 - 0));
        }
#pragma unroll
        for (int u = 0; u < HP; ++u) {
          const int jj = hp * HP + u;
          if (jb + u >= j0 + tc) break;
          float o[4];
#pragma unroll
          for (int ch = 0; ch < 4; ++ch) {
            const float* r0 = reinterpret_cast<const float*>(&r[u]);
            const float* r1 = reinterpret_cast<const float*>(&r[u + 1]);
            const float* r2 = reinterpret_cast<const float*>(&r[u + 2]);
            const float* r3 = reinterpret_cast<const float*>(&r[u + 3]);
            const float* tp = reinterpret_cast<const float*>(&taps[ch]);
            float acc = tp[0] * r0[ch];
            acc = fmaf(tp[1], r1[ch], acc); acc = fmaf(tp[2], r2[ch], acc); acc = fmaf(tp[3], r3[ch], acc);
            o[ch] = silu_f(acc + reinterpret_cast<const float*>(&bias)[ch]);
          }
          const float4 ov = make_float4(o[0], o[1], o[2], o[3]);
          if (!is_x) {
            if (cid < NGBC / 2) *reinterpret_cast<float4*>(&Bs[buf][jj][4 * cid]) = ov;
            else *reinterpret_cast<float4*>(&Cs[buf][jj][4 * cid - N]) = ov;
          } else if (active) {
            *reinterpret_cast<float4*>(&xs[buf][jj][4 * xg]) = ov;
            if (a.g != nullptr) *reinterpret_cast<float4*>(&zs[buf][jj][4 * xg]) = z[u];
          }
          // keep the raw inputs of these positions for later windows and for rollback
          if (a.write_ring && zx != nullptr && active && (is_x || (h == 0 && blockIdx.x == 0)))
            *reinterpret_cast<float4*>(ring + (size_t)((pos0 + jb + u) & rmask) * d.ring_w + c4) = r[u + 3];
        }
      }
    }
    if (stager && dt_jj >= 0 && dt_jj < tc) {   // step and decay of the head
      const float dt = softplus_f(raw_row(pos0 + j0 + dt_jj)[d.conv_dim + h] + dtb);
      dts[buf][dt_jj] = dt;
      as[buf][dt_jj] = expf(negA * dt);
    }
    if (stager && a.write_ring && zx != nullptr && h == 0 && blockIdx.x == 0) {
      for (int it = stid; it < tc * d.Hm; it += NSTG) {
        const int jj = it / d.Hm, hh = it - jj * d.Hm, pos = pos0 + j0 + jj;
        ring[(size_t)(pos & rmask) * d.ring_w + d.conv_dim + hh] = raw_row(pos)[d.conv_dim + hh];
      }
    }
  };

  // recurrence over the staged positions of buffer `buf`
  auto recur = [&](int j0, int buf) {
    const int tc = min(kTS, nt - j0);
    for (int jj = 0; jj < tc; ++jj) {
      const float xv = xs[buf][jj][row];
      const float coef = dts[buf][jj] * xv, aj = as[buf][jj];
      float part = 0.f;
#pragma unroll
      for (int i = 0; i < NV; i += 4) {
        const float4 Bv = *reinterpret_cast<const float4*>(&Bs[buf][jj][i * kSub + sub * 4]);
        const float4 Cv = *reinterpret_cast<const float4*>(&Cs[buf][jj][i * kSub + sub * 4]);
        S[i] = fmaf(aj, S[i], coef * Bv.x); part = fmaf(S[i], Cv.x, part);
        S[i + 1] = fmaf(aj, S[i + 1], coef * Bv.y); part = fmaf(S[i + 1], Cv.y, part);
        S[i + 2] = fmaf(aj, S[i + 2], coef * Bv.z); part = fmaf(S[i + 2], Cv.z, part);
        S[i + 3] = fmaf(aj, S[i + 3], coef * Bv.w); part = fmaf(S[i + 3], Cv.w, part);
      }
      part += dpp_move<0xB1>(part);    // lane ^ 1
      part += dpp_move<0x4E>(part);    // lane ^ 2
      part += dpp_move<0x141>(part);   // the other quad of the 8 lanes that share a row
      if (a.g != nullptr && sub == 0 && prow)
        a.g[((size_t)b * a.T + j0 + jj) * d.d_inner + h * d.P + p] = (part + dskip * xv) * silu_f(zs[buf][jj][row]);
    }
  };

  if (!PIPE) {
    for (int j0 = 0; j0 < nt; j0 += kTS) {
      stage(j0, 0);
      __syncthreads();
      recur(j0, 0);
      __syncthreads();
    }
  } else {
    if (stager) stage(0, 0);
    __syncthreads();
    int buf = 0;
    for (int j0 = 0; j0 < nt; j0 += kTS, buf ^= 1) {
      // the other buffer was last read by the recurrence of the chunk before this one, which
      // ended before the barrier that closed the previous iteration
      if (stager) {
        if (j0 + kTS < nt) stage(j0 + kTS, buf ^ 1);
      } else {
        recur(j0, buf);
      }
      __syncthreads();
    }
  }

  if (a.state_out != 0 && prow) {
    float* dst = (a.state_out == 1 ? ly.S : ly.S_draft) + (((size_t)b * d.Hm + h) * d.P + p) * N + sub * 4;
#pragma unroll
    for (int i = 0; i < NV; i += 4) *reinterpret_cast<float4*>(dst + i * kSub) = make_float4(S[i], S[i + 1], S[i + 2], S[i + 3]);
  }
}

// RG row groups of 64 / SUBS rows per workgroup, one after the other: the B/C convolution and the
// per-head scalars are shared by all of them, which is what a large batch needs (there a
// workgroup's fixed loads would otherwise exceed its share of the state).
// NWV wavefronts per workgroup (1 or 4), each with its own rows: with tens of thousands of
// one-wavefront workgroups the launch is bound by the workgroup dispatch rate (measured: 3
// resident wavefronts per compute unit), and four wavefronts share one B/C convolution.
// OUT = false (no outputs wanted: the commit's rebuild of the state from the ring): the read-out S C and
// the gate are not computed and positions behind the sequence's count are skipped (the count is
// uniform over the workgroup), which halves the arithmetic per position and leaves n + 1 instead of
// TMAX positions of it.
// CW (4 or 2) consecutive channels as one load or store; with 2 the upper half of the float4 is never used
template <int CW>
__device__ __forceinline__ float4 load_channels(const float* p) {
  if (CW == 4) return *reinterpret_cast<const float4*>(p);
  const float2 v = *reinterpret_cast<const float2*>(p);
  return make_float4(v.x, v.y, 0.f, 0.f);
}
template <int CW>
__device__ __forceinline__ void store_channels(float* p, const float4& v) {
  if (CW == 4) *reinterpret_cast<float4*>(p) = v;
  else *reinterpret_cast<float2*>(p) = make_float2(v.x, v.y);
}

template <int NV, int SUBS, int TMAX, int RG, int NWV, bool OUT = true>
__global__ __launch_bounds__(64 * NWV) void ssm_small_kernel(const Dims d, const SsmArgs a) {
  constexpr int NTHR = 64 * NWV;
  constexpr int ROWS = 64 / SUBS, N = NV * SUBS;
  // B|C channels per thread and group: 4, or 2 where groups of 4 would leave threads of the workgroup idle (half
  // the registers for the taps and the raw rows of the convolution: one more resident wavefront per SIMD)
  constexpr int CW = 2 * N / 4 >= NTHR ? 4 : 2;
  constexpr int NGR = 2 * N / CW;                      // groups in all
  constexpr int NG = (NGR + NTHR - 1) / NTHR;          // groups per thread
  __shared__ __align__(16) float BCs[TMAX][2 * N];

  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int row = lane / SUBS, sub = lane % SUBS;
  const int p0 = (blockIdx.x * NWV + wave) * ROWS * RG, h = blockIdx.y;
  const int lz = blockIdx.z / a.B, b = blockIdx.z % a.B;
  const LayerDev& ly = a.layers != nullptr ? a.layers[a.layer0 + lz] : a.one;
  TR(0);
  // Loads in the order of what they wait for.  Nothing here depends on the per-sequence
  // scalars except the ring rows (slot = position mod ring size), which come last.
  int pr[RG], cx[RG];
  bool prow[RG];
#pragma unroll
  for (int rg = 0; rg < RG; ++rg) {
    pr[rg] = min(p0 + rg * ROWS + row, d.P - 1);
    prow[rg] = p0 + rg * ROWS + row < d.P;
    cx[rg] = h * d.P + pr[rg];
  }
  const int rmask = d.ring_slots - 1;
  float* ring = ly.ring + (size_t)b * d.ring_slots * d.ring_w;
  const float* zx = a.zx != nullptr ? a.zx + (size_t)b * a.T * d.ldzx : nullptr;
  const int skip_v = (a.skip != nullptr ? a.skip : a.pos0)[b];   // absent arrays read pos0 instead and are ignored
  const int nacc_v = (a.n_acc != nullptr ? a.n_acc : a.pos0)[b];
  const int ntok_v = (a.n_tok != nullptr ? a.n_tok : a.pos0)[b];
  const int pos0 = a.pos0[b];
  float S[RG][NV];
  // (a macro, not a lambda: the state must stay in registers)
#define HH_LOAD_STATE()                                                                                                   \
  {                                                                                                                       \
    const float* src = a.state_in == 0 ? ly.S : (a.state_in == 1 ? ly.S_draft : nullptr);                                 \
    _Pragma("unroll") for (int rg = 0; rg < RG; ++rg) {                                                                   \
      if (src != nullptr) {                                                                                               \
        /* float4 i of a lane: elements (i/4)*4*SUBS + 4*sub .. */                                                        \
        const float* sp = src + (((size_t)b * d.Hm + h) * d.P + pr[rg]) * N + sub * 4;                                    \
        _Pragma("unroll") for (int i = 0; i < NV; i += 4) {                                                               \
          const float4 v = *reinterpret_cast<const float4*>(sp + i * SUBS);                                               \
          S[rg][i] = v.x; S[rg][i + 1] = v.y; S[rg][i + 2] = v.z; S[rg][i + 3] = v.w;                                     \
        }                                                                                                                 \
      } else {                                                                                                            \
        _Pragma("unroll") for (int i = 0; i < NV; ++i) S[rg][i] = 0.f;                                                    \
      }                                                                                                                   \
    }                                                                                                                     \
  }
  // With outputs the state is requested first (the longest wait).  The rebuild holds up to TMAX + 3 ring rows of
  // B | C per thread until the convolution is done; it requests the state behind that, which keeps it at the
  // register count of the one-position kernel (more resident wavefronts cover the wait instead).
  if (OUT) HH_LOAD_STATE();
  float4 bw[NG][CW], bb[NG], braw[NG][TMAX + 3];
  float xraw[RG][TMAX + 3], zg[RG][TMAX];
  float dtraw_l = 0.f;   // raw dt of position `lane` (lanes < T): softplus and decay are evaluated once, lane-parallel
#pragma unroll
  for (int u = 0; u < NG; ++u) {
    const int c = d.d_inner + CW * min(tid + NTHR * u, NGR - 1);
#pragma unroll
    for (int t = 0; t < CW; ++t) bw[u][t] = *reinterpret_cast<const float4*>(ly.conv_w + (size_t)(c + t) * 4);
    bb[u] = load_channels<CW>(ly.conv_b + c);
  }
  float4 xw[RG];
  float xb[RG];
#pragma unroll
  for (int rg = 0; rg < RG; ++rg) {
    xw[rg] = *reinterpret_cast<const float4*>(ly.conv_w + (size_t)cx[rg] * 4);
    xb[rg] = ly.conv_b[cx[rg]];
  }
  const float dskip = ly.d_skip[h];
  const float dtb = ly.dt_bias[h];
  const float alog = ly.a_log[h];
  if (zx != nullptr) {   // inputs of this pass: rows 0 .. T-1 of the projection buffer (rows >= nt are read but not used)
#pragma unroll
    for (int j = 0; j < TMAX; ++j) {
      const float* r = zx + (size_t)min(j, a.T - 1) * d.ldzx + d.d_inner;
#pragma unroll
      for (int u = 0; u < NG; ++u) braw[u][j + 3] = load_channels<CW>(r + d.d_inner + CW * min(tid + NTHR * u, NGR - 1));
#pragma unroll
      for (int rg = 0; rg < RG; ++rg) {
        xraw[rg][j + 3] = r[cx[rg]];
        zg[rg][j] = a.g != nullptr ? r[cx[rg] - d.d_inner] : 0.f;   // z precedes xBC in the row
      }
    }
    dtraw_l = zx[(size_t)min(lane, a.T - 1) * d.ldzx + d.d_inner + d.conv_dim + h];
  }
  if (a.skip != nullptr && skip_v) return;
  int nt = a.T;
  if (a.n_acc != nullptr) nt = nacc_v + 1;
  else if (a.n_tok != nullptr) nt = ntok_v;
  if (nt <= 0) return;
  nt = min(nt, TMAX);
  // row of raw inputs (xBC | dt) of position pos0 + j in the ring (positions before 0 read slot 0 and count as 0)
  auto ring_row = [&](int j) -> const float* { return ring + (size_t)(max(pos0 + j, 0) & rmask) * d.ring_w; };
#pragma unroll
  for (int j = -3; j < (int)TMAX; ++j) {
    if (j >= 0 && zx != nullptr) continue;
    if (!OUT && j >= nt) continue;               // the rebuild never uses positions behind the count: no loads for them
    const float* r = ring_row(min(j, nt - 1));
#pragma unroll
    for (int u = 0; u < NG; ++u) braw[u][j + 3] = load_channels<CW>(r + d.d_inner + CW * min(tid + NTHR * u, NGR - 1));
#pragma unroll
    for (int rg = 0; rg < RG; ++rg) {
      xraw[rg][j + 3] = r[cx[rg]];
      if (j >= 0) zg[rg][j] = 0.f;
    }
  }
  if (zx == nullptr) dtraw_l = ring_row(min(lane, nt - 1))[d.conv_dim + h];
  const float negA = -expf(alog);
  TR(1);

  // ---- conv + SiLU: B and C for the whole workgroup (branch-free: clamped inputs, every
  // position computed; positions >= nt are never used)
#pragma unroll
  for (int u = 0; u < NG; ++u) {
    const int gi = tid + NTHR * u;
#pragma unroll
    for (int j = 0; j < TMAX; ++j) {
      if (!OUT && j >= nt) continue;             // (a guard per position, not a loop exit: the unrolled arrays stay in registers)
      float4 o = make_float4(0.f, 0.f, 0.f, 0.f);
      float* op = reinterpret_cast<float*>(&o);
#pragma unroll
      for (int ch = 0; ch < CW; ++ch) {
        const float r0 = pos0 + j - 3 < 0 ? 0.f : reinterpret_cast<const float*>(&braw[u][j])[ch];
        const float r1 = pos0 + j - 2 < 0 ? 0.f : reinterpret_cast<const float*>(&braw[u][j + 1])[ch];
        const float r2 = pos0 + j - 1 < 0 ? 0.f : reinterpret_cast<const float*>(&braw[u][j + 2])[ch];
        const float r3 = reinterpret_cast<const float*>(&braw[u][j + 3])[ch];
        float acc = bw[u][ch].x * r0;
        acc = fmaf(bw[u][ch].y, r1, acc); acc = fmaf(bw[u][ch].z, r2, acc); acc = fmaf(bw[u][ch].w, r3, acc);
        op[ch] = silu_f(acc + reinterpret_cast<const float*>(&bb[u])[ch]);
      }
      if (gi < NGR) store_channels<CW>(&BCs[j][CW * gi], o);
    }
  }
  // ---- per-position scalars of the head (step and decay), all positions at once
  float dtj[TMAX], aj[TMAX];
  const float dt_l = softplus_f(dtraw_l + dtb);
  const float a_l = expf(negA * dt_l);
#pragma unroll
  for (int j = 0; j < TMAX; ++j) {
    const bool on = j < nt;
    dtj[j] = on ? __int_as_float(__builtin_amdgcn_readlane(__float_as_int(dt_l), j)) : 0.f;
    aj[j] = on ? __int_as_float(__builtin_amdgcn_readlane(__float_as_int(a_l), j)) : 1.f;   // positions >= nt leave the state as it is
  }
  // ---- keep the raw inputs of these positions for later windows and for rollback
  if (a.write_ring && zx != nullptr) {
#pragma unroll
    for (int rg = 0; rg < RG; ++rg) {
      if (sub == 0 && prow[rg]) {
#pragma unroll
        for (int j = 0; j < TMAX; ++j)
          if (j < nt) ring[(size_t)((pos0 + j) & rmask) * d.ring_w + cx[rg]] = xraw[rg][j + 3];
      }
    }
    if (h == 0 && blockIdx.x == 0) {
#pragma unroll
      for (int u = 0; u < NG; ++u) {
        const int gi = tid + NTHR * u;
        if (gi < NGR) {
#pragma unroll
          for (int j = 0; j < TMAX; ++j)
            if (j < nt) store_channels<CW>(ring + (size_t)((pos0 + j) & rmask) * d.ring_w + d.d_inner + CW * gi, braw[u][j + 3]);
        }
      }
      for (int it = tid; it < nt * d.Hm; it += NTHR) {
        const int j = it / d.Hm, hh = it - j * d.Hm;
        ring[(size_t)((pos0 + j) & rmask) * d.ring_w + d.conv_dim + hh] = zx[(size_t)j * d.ldzx + d.d_inner + d.conv_dim + hh];
      }
    }
  }
  TR(2);
  __syncthreads();
  TR(3);
  if (!OUT) HH_LOAD_STATE();
#undef HH_LOAD_STATE

  // ---- per row group: conv + SiLU of x, recurrence, outputs
#pragma unroll
  for (int rg = 0; rg < RG; ++rg) {
    float y[TMAX];
#pragma unroll
    for (int j = 0; j < TMAX; ++j) {
      if (!OUT && j >= nt) continue;
      const float r0 = pos0 + j - 3 < 0 ? 0.f : xraw[rg][j];
      const float r1 = pos0 + j - 2 < 0 ? 0.f : xraw[rg][j + 1];
      const float r2 = pos0 + j - 1 < 0 ? 0.f : xraw[rg][j + 2];
      float acc = xw[rg].x * r0;
      acc = fmaf(xw[rg].y, r1, acc); acc = fmaf(xw[rg].z, r2, acc); acc = fmaf(xw[rg].w, xraw[rg][j + 3], acc);
      const float xv = silu_f(acc + xb[rg]);
      const float coef = dtj[j] * xv;
      if (!OUT) {
#pragma unroll
        for (int i = 0; i < NV; i += 4) {
          const float4 Bv = *reinterpret_cast<const float4*>(&BCs[j][i * SUBS + sub * 4]);
          S[rg][i] = fmaf(aj[j], S[rg][i], coef * Bv.x);
          S[rg][i + 1] = fmaf(aj[j], S[rg][i + 1], coef * Bv.y);
          S[rg][i + 2] = fmaf(aj[j], S[rg][i + 2], coef * Bv.z);
          S[rg][i + 3] = fmaf(aj[j], S[rg][i + 3], coef * Bv.w);
        }
        continue;
      }
      const float gate = silu_f(zg[rg][j]);
      float part = 0.f;
#pragma unroll
      for (int i = 0; i < NV; i += 4) {
        const float4 Bv = *reinterpret_cast<const float4*>(&BCs[j][i * SUBS + sub * 4]);
        const float4 Cv = *reinterpret_cast<const float4*>(&BCs[j][N + i * SUBS + sub * 4]);
        S[rg][i] = fmaf(aj[j], S[rg][i], coef * Bv.x); part = fmaf(S[rg][i], Cv.x, part);
        S[rg][i + 1] = fmaf(aj[j], S[rg][i + 1], coef * Bv.y); part = fmaf(S[rg][i + 1], Cv.y, part);
        S[rg][i + 2] = fmaf(aj[j], S[rg][i + 2], coef * Bv.z); part = fmaf(S[rg][i + 2], Cv.z, part);
        S[rg][i + 3] = fmaf(aj[j], S[rg][i + 3], coef * Bv.w); part = fmaf(S[rg][i + 3], Cv.w, part);
      }
      part += dpp_move<0xB1>(part);    // lane ^ 1
      part += dpp_move<0x4E>(part);    // lane ^ 2
      part += dpp_move<0x141>(part);   // the other quad of 8 lanes
      if (SUBS == 16) part += dpp_move<0x140>(part);   // the other half of 16 lanes
      y[j] = (part + dskip * xv) * gate;
    }
    if (a.g != nullptr && sub == 0 && prow[rg]) {
#pragma unroll
      for (int j = 0; j < TMAX; ++j)
        if (j < nt) a.g[((size_t)b * a.T + j) * d.d_inner + cx[rg]] = y[j];
    }
    if (a.state_out != 0 && prow[rg]) {
      float* dst = (a.state_out == 1 ? ly.S : ly.S_draft) + (((size_t)b * d.Hm + h) * d.P + pr[rg]) * N + sub * 4;
#pragma unroll
      for (int i = 0; i < NV; i += 4)
        *reinterpret_cast<float4*>(dst + i * SUBS) = make_float4(S[rg][i], S[rg][i + 1], S[rg][i + 2], S[rg][i + 3]);
    }
  }
  TR(5);
}

template <int NV, int SUBS, int RG, int NWV>
static hipError_t launch_ssm_small_r(const Dims& d, const SsmArgs& a, int tmax, hipStream_t s) {
  constexpr int rows = 64 / SUBS * RG * NWV;
  const dim3 grid((d.P + rows - 1) / rows, d.Hm, a.n_layers_z * a.B);
  if (a.g == nullptr && a.zx == nullptr) {   // the rebuild from the ring: no outputs
    switch (tmax) {
      case 1: hipLaunchKernelGGL((ssm_small_kernel<NV, SUBS, 1, RG, NWV, false>), grid, dim3(64 * NWV), 0, s, d, a); break;
      case 3: hipLaunchKernelGGL((ssm_small_kernel<NV, SUBS, 3, RG, NWV, false>), grid, dim3(64 * NWV), 0, s, d, a); break;
      case 5: hipLaunchKernelGGL((ssm_small_kernel<NV, SUBS, 5, RG, NWV, false>), grid, dim3(64 * NWV), 0, s, d, a); break;
      case 9: hipLaunchKernelGGL((ssm_small_kernel<NV, SUBS, 9, RG, NWV, false>), grid, dim3(64 * NWV), 0, s, d, a); break;
      default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
  }
  switch (tmax) {
    case 1: hipLaunchKernelGGL((ssm_small_kernel<NV, SUBS, 1, RG, NWV>), grid, dim3(64 * NWV), 0, s, d, a); break;
    case 3: hipLaunchKernelGGL((ssm_small_kernel<NV, SUBS, 3, RG, NWV>), grid, dim3(64 * NWV), 0, s, d, a); break;
    case 5: hipLaunchKernelGGL((ssm_small_kernel<NV, SUBS, 5, RG, NWV>), grid, dim3(64 * NWV), 0, s, d, a); break;
    case 9: hipLaunchKernelGGL((ssm_small_kernel<NV, SUBS, 9, RG, NWV>), grid, dim3(64 * NWV), 0, s, d, a); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}
template <int NV, int SUBS>
static hipError_t launch_ssm_small_t(const Dims& d, const SsmArgs& a, int tmax, hipStream_t s) {
  // Several row groups per workgroup pay off only in the rebuild from the ring (commit: all layers
  // in one launch, every load of a workgroup besides the state is fixed cost); measured, the
  // draft step and the verification pass are no faster with them.
  constexpr int min_wg = 1024;
  const int groups = (d.P + 64 / SUBS - 1) / (64 / SUBS);
  const long wgs = (long)groups * d.Hm * a.n_layers_z * a.B;
  if (a.zx == nullptr && NV <= 16) {            // (32 values per lane and row group: registers; four wavefronts instead)
    if (groups % 4 == 0 && wgs / 4 >= min_wg) return launch_ssm_small_r<NV, SUBS, 4, 1>(d, a, tmax, s);
    if (groups % 2 == 0 && wgs / 2 >= min_wg) return launch_ssm_small_r<NV, SUBS, 2, 1>(d, a, tmax, s);
  }
  // large launches: four wavefronts per workgroup (workgroup dispatch rate, shared B/C convolution)
  constexpr int wide_wg = 2048;
  if (groups % 4 == 0 && wgs >= wide_wg) return launch_ssm_small_r<NV, SUBS, 1, 4>(d, a, tmax, s);
  return launch_ssm_small_r<NV, SUBS, 1, 1>(d, a, tmax, s);
}

// true if the pass was taken by the few-positions kernel
static bool launch_ssm_small(const Dims& d, const SsmArgs& a, hipStream_t s, hipError_t* err) {
  if ((d.flags & HH_KF_SSM_GENERAL) || a.T > 9 || d.Hm % 4 != 0 || d.P % 4 != 0 || d.N % 32 != 0 || d.ldzx % 4 != 0 || d.d_inner % 4 != 0) return false;
  const int tmax = a.T <= 1 ? 1 : a.T <= 3 ? 3 : a.T <= 5 ? 5 : 9;
  const long waves8 = (long)((d.P + 7) / 8) * d.Hm * a.n_layers_z * a.B;
  const bool wide = d.N % 64 == 0 && waves8 < 1024;     // 16 lanes per row: twice the wavefronts
  switch (wide ? d.N / 16 : d.N / 8) {
    case 4: *err = wide ? launch_ssm_small_t<4, 16>(d, a, tmax, s) : launch_ssm_small_t<4, 8>(d, a, tmax, s); return true;
    case 8: *err = wide ? launch_ssm_small_t<8, 16>(d, a, tmax, s) : launch_ssm_small_t<8, 8>(d, a, tmax, s); return true;
    case 16: *err = wide ? launch_ssm_small_t<16, 16>(d, a, tmax, s) : launch_ssm_small_t<16, 8>(d, a, tmax, s); return true;
    case 32: if (!wide) { *err = launch_ssm_small_t<32, 8>(d, a, tmax, s); return true; } break;
  }
  return false;
}

template <int kRows>
static hipError_t launch_ssm_rows(const Dims& d, const SsmArgs& a, hipStream_t s) {
  const dim3 grid((d.P + kRows - 1) / kRows, d.Hm, a.n_layers_z * a.B);
  const dim3 block(kRows * kSub);
  // aligned shapes: the kernel with the vectorised chunk convolution
  const bool scalar = (d.flags & HH_KF_SSM_SCALAR_CONV) != 0;
  const int nv = d.N / kSub;
  const bool vec = !scalar && d.P % 4 == 0 && d.d_inner % 4 == 0 && d.ldzx % 4 == 0 && d.ring_w % 4 == 0 &&
                   d.conv_dim % 4 == 0 && nv % 4 == 0 && 2 * d.N / 4 + kRows / 4 <= kRows * kSub - kTS &&
                   (a.zx == nullptr || (reinterpret_cast<uintptr_t>(a.zx) & 15) == 0);
  if (vec) {
    // few workgroups per compute unit and several chunks: staging on wavefronts of its own
    constexpr int pipe_wg = 512;
    const bool pipe = (long long)grid.x * grid.y * grid.z <= pipe_wg && a.T > kTS;
#define HH_CHUNK(NV_)                                                                                          \
  case NV_:                                                                                                    \
    if (pipe)                                                                                                  \
      hipLaunchKernelGGL((ssm_chunk_kernel<NV_, kRows, true>), grid,                                           \
                         dim3(kRows * kSub + chunk_stage_threads<NV_, kRows>()), 0, s, d, a);                  \
    else                                                                                                       \
      hipLaunchKernelGGL((ssm_chunk_kernel<NV_, kRows, false>), grid, block, 0, s, d, a);                      \
    return hipGetLastError();
    switch (nv) {
      HH_CHUNK(4)
      HH_CHUNK(8)
      HH_CHUNK(16)
      HH_CHUNK(32)
    }
#undef HH_CHUNK
  }
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
  hipError_t e = hipSuccess;
  if (launch_ssm_small(d, a, s, &e)) return e;
  if (launch_ssd_mfma(d, a, s, &e)) return e;
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
