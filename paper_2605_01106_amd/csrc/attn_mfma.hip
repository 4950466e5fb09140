// Attention branch on the matrix cores (bf16 KV cache): causal grouped-query attention of the
// T new positions of every sequence over all keys up to each position, rotary embedding of q
// fused, keys split over the wavefronts of a workgroup and over workgroups, log-sum-exp merge
// in slice order.  The keys and values of the new positions are already in the cache.
//
// Everything is computed transposed so that no operand ever has to be transposed in LDS.
// With v_mfma_f32_16x16x32_bf16 (D[m][n] += sum_k A[m][k] B[k][n]; lane l holds A[l%16][8(l/16)..+7],
// B[8(l/16)..+7][l%16] and D[4(l/16)+r][l%16]):
//   scores   S^T[key][row] = sum_dim K[key][dim] Q[row][dim]      A = 16 keys of the cache (one
//            16-byte load per lane: a key row is contiguous), B = query rows from LDS;
//   softmax  a lane then holds 8 keys of one query row: running maximum and sum per lane,
//            combined across the 4 lane groups with two lane exchanges;
//   output   O^T[dim][row] = sum_key V^T[dim][key] P^T[key][row]   A = V pages, stored
//            transposed (16 bytes = 8 consecutive tokens of one dimension), B = the lane's own
//            8 probabilities; the accumulator of a lane belongs to one query row, so the
//            rescaling of the online softmax is a per-lane scalar.
// The A rows of the two key blocks of a step are assigned so that a lane's 8 scores are the
// 8 consecutive keys its V load covers (block 0 row m <-> key 8(m/4) + m%4, block 1: + 4).
// Queries and probabilities are float32 values split exactly into three bf16 terms, so the
// products carry float32 accuracy (with two-term probabilities, 16 mantissa bits, models with
// order-one activations lost tokens to near ties that the float32 reference path keeps); K and V
// are used as stored.  The scores
// are kept in base-2 units (log2(e) folded into the query scale) so that the exponentials are
// single v_exp_f32 instructions.
#include <stdlib.h>

#include "attn_common.h"
#include "bf16_split.h"

namespace hh {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

int attention_mfma_row_chunks(const Dims& d, int T);

static constexpr int kStepKeys = 32;   // keys per wavefront step
static constexpr int kMergeLd = 20;    // row stride (floats) of the in-workgroup merge buffer

union Frag {
  uint4 u;
  bf16x8 v;
};

__device__ __forceinline__ void split3(float x, uint32_t& t0, uint32_t& t1, uint32_t& t2) { split3_bf16(x, t0, t1, t2); }

// maximum over the lanes l, l^16, l^32, l^48 (the four lanes that hold one query row), through
// the row swaps of the vector unit instead of LDS permutes: v_permlane16_swap exchanges the odd
// 16-lane rows of its first operand with the even rows of its second, v_permlane32_swap the upper
// half of the first with the lower half of the second.
__device__ __forceinline__ float xor_max(float v) {
  const uint32_t x = __float_as_uint(v);
  const auto s16 = __builtin_amdgcn_permlane16_swap(x, x, false, false);
  v = fmaxf(__uint_as_float(s16[0]), __uint_as_float(s16[1]));
  const uint32_t y = __float_as_uint(v);
  const auto s32 = __builtin_amdgcn_permlane32_swap(y, y, false, false);
  return fmaxf(__uint_as_float(s32[0]), __uint_as_float(s32[1]));
}
// 2^x through the hardware instruction (scores are kept in base-2 units)
__device__ __forceinline__ float ex2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float xor_add(float v) {
  v += __shfl_xor(v, 16, 64);
  return v + __shfl_xor(v, 32, 64);
}

// grid: x = row_chunks * n_splits, y = Hkv, z = B.  RT = 16-row tiles per workgroup,
// KS = ceil(Dh / 32).
//
// FUSE (verification: at most 16 new positions, one row chunk): the keys and values of the new
// positions are not in the cache yet.  The cached keys (positions < pos0) are visible to every
// row; one wavefront of the launch builds the operands of the new positions from the projection
// buffer (rotating and rounding k, rounding v), appends them to the cache and scores them as
// one more step with the causal mask.  Otherwise the cache already holds them (prefill).
//
// NW wavefronts per workgroup split the keys of its slice and meet in LDS.
template <int RT, int KS, bool FUSE, int NW>
__global__ __launch_bounds__(64 * NW) void attn_mfma_kernel(const Dims d, const AttnArgs a, const int row_chunks) {
  constexpr int NT = 64 * NW;            // threads
  constexpr int NDB = 2 * KS;            // blocks of 16 output dimensions
  constexpr int Dhp = 32 * KS;           // head dimension padded to the MFMA depth
  constexpr int QS = 3 * Dhp + 8;        // bf16 elements per staged query row (3 split terms + pad)
  constexpr int R = RT * 16;
  extern __shared__ __align__(16) unsigned char smem_raw[];
  __shared__ int s_last;
  int* pg = reinterpret_cast<int*>(smem_raw);                                  // [NW][64] page numbers of a wavefront's steps
  uint16_t* qT = reinterpret_cast<uint16_t*>(smem_raw + NT * 4);               // [R][QS]
  float* mrg = reinterpret_cast<float*>(smem_raw + NT * 4 + (size_t)R * QS * 2);   // merge scratch
  float* mrg_o = mrg;                                                          // [NW-1][Dhp][kMergeLd]
  float* mrg_ml = mrg + (NW - 1) * Dhp * kMergeLd;                             // [NW-1][16][2]

  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int g = lane >> 4, n = lane & 15;
  const int chunk = blockIdx.x % row_chunks, sp = blockIdx.x / row_chunks;
  const int kvh = blockIdx.y, b = blockIdx.z;
  TR(0);
  const int nt = a.n_tok != nullptr ? a.n_tok[b] : a.T;
  const int pos0 = a.pos0[b];
  const int Dh = d.Dh, G = d.Hq / d.Hkv, half = Dh >> 1, S = a.n_splits;
  const int n_rows = a.T * G;
  const int row_lim = min(n_rows, nt * G);     // row = position j * G + query head of the group; valid while j < nt
  const int row0 = chunk * R;
  const int jmax = row0 < row_lim ? (min(row_lim, row0 + R) - 1) / G : -1;
  const int nk_all = jmax < 0 ? 0 : pos0 + jmax + 1;      // keys 0 .. nk_all-1 are visible to some row of this chunk
  const int nk = FUSE ? min(nk_all, pos0) : nk_all;       // ... of which the cache holds 0 .. nk-1
  const int* pt_row = a.page_table + (size_t)b * d.pages_per_seq;
  const int pshift = 31 - __clz(d.page_tokens), pmask = d.page_tokens - 1;
  const uint16_t* kp = static_cast<const uint16_t*>(a.kpool);
  const uint16_t* vp = static_cast<const uint16_t*>(a.vpool);
  const float* xrow = a.qkv + (size_t)b * a.T * d.ldzx;

  // key steps of this workgroup and of this wavefront
  const int steps = (nk + kStepKeys - 1) / kStepKeys;
  const int sps = (steps + S - 1) / S;
  const int sb = sp * sps, se = min(steps, sb + sps);
  const int per = (max(se - sb, 0) + NW - 1) / NW;
  const int ws = sb + wave * per, we = min(se, ws + per);

  // Operand loads of one step.  A step's 32 keys lie in one page (the page size is a multiple of
  // 32 on this path), so the page number is a scalar load and the lane offsets within the page
  // are computed once.
  Frag kA[KS], kB[KS], vT[NDB];
  const size_t head_elems = (size_t)d.page_tokens * Dh;              // elements per (page, head)
  const int kofsA = 8 * (n >> 2) + (n & 3);                          // key of block A row n within the step
  int voff[NDB];                                                     // dimension (clamped) * page_tokens
#pragma unroll
  for (int db = 0; db < NDB; ++db) voff[db] = min(db * 16 + n, Dh - 1) * d.page_tokens;
  const bool dh32 = (Dh & 31) == 0;
  // The page numbers of 64 steps at a time go through LDS (one per lane, read back by the whole
  // wavefront): a page-table load in the step loop would expose its memory latency every step.
  int* pgw = pg + wave * 64;
  auto stage_pages = [&](int step0) { pgw[lane] = pt_row[(max(min(step0 + lane, steps - 1), 0) * kStepKeys) >> pshift]; };
  stage_pages(ws);
  auto load_step = [&](int step, Frag(&ka)[KS], Frag(&kb)[KS], Frag(&vt)[NDB]) {
    const int key0 = step * kStepKeys;
    if (step != ws && ((step - ws) & 63) == 0) stage_pages(step);
    const int page = __builtin_amdgcn_readfirstlane(pgw[(step - ws) & 63]);
    const size_t base = ((size_t)page * d.Hkv + kvh) * head_elems;
    const int in0 = key0 & pmask, last = nk - 1 - (key0 - in0);      // in-page index of the step's first key / of the last cached key
    // past the end: a valid key, masked later
    const uint16_t* pa = kp + base + (size_t)(min(in0 + kofsA, last) * Dh + 8 * g);
    const uint16_t* pb = kp + base + (size_t)(min(in0 + kofsA + 4, last) * Dh + 8 * g);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      // unconditional loads (a branch around them would make the wait for the previous step's
      // operands wait for these as well); lanes past the head dimension re-read dimension 0
      const int off = (dh32 || ks * 32 + 8 * g < Dh) ? ks * 32 : -8 * g;
      ka[ks].u = *reinterpret_cast<const uint4*>(pa + off);
      kb[ks].u = *reinterpret_cast<const uint4*>(pb + off);
    }
    if (!dh32) {
#pragma unroll
      for (int ks = 0; ks < KS; ++ks)
        if (ks * 32 + 8 * g >= Dh) { ka[ks].u = make_uint4(0, 0, 0, 0); kb[ks].u = make_uint4(0, 0, 0, 0); }
    }
    // 8 consecutive tokens of one dimension (tokens >= nk are zeroed when the step is scored)
    const int tok = in0 + 8 * g;
    const int cnt = min(max(last + 1 - tok, 0), 8);
    const uint16_t* pv = vp + base + (cnt > 0 ? tok : (last & ~7));
#pragma unroll
    for (int db = 0; db < NDB; ++db) vt[db].u = *reinterpret_cast<const uint4*>(pv + voff[db]);
  };
  if (ws < we) load_step(ws, kA, kB, vT);
  TR(1);

  // ---- the new positions (FUSE): one wavefront of the launch builds their operands from the
  // projection buffer and appends them to the cache, before the queries are staged (it only
  // needs the queries to score them)
  const bool new_wave = FUSE && sp == S - 1 && wave == NW - 1 && nk_all > pos0;
  Frag nA[KS], nB[KS], nV[NDB];
  if (new_wave) {
    const float2* rope = reinterpret_cast<const float2*>(a.rope);
    const bool al4 = (d.ldzx & 3) == 0 && (reinterpret_cast<uintptr_t>(xrow) & 15) == 0;   // 16-byte aligned rows (dq, Dh are multiples of 8)
    uint16_t* kpw = static_cast<uint16_t*>(a.kpool);
    uint16_t* vpw = static_cast<uint16_t*>(a.vpool);
    auto load8 = [&](const float* src, float(&o)[8]) {
      if (al4) {
        const float4 x = *reinterpret_cast<const float4*>(src), y = *reinterpret_cast<const float4*>(src + 4);
        o[0] = x.x; o[1] = x.y; o[2] = x.z; o[3] = x.w; o[4] = y.x; o[5] = y.y; o[6] = y.z; o[7] = y.w;
      } else {
#pragma unroll
        for (int i = 0; i < 8; ++i) o[i] = src[i];
      }
    };
    // values of the new positions first (their loads overlap the rotation of the keys below)
    float vraw[NDB][8];
    size_t vat[8];
    {
      const float* vbase = xrow + d.dq + d.dkv + (size_t)kvh * Dh;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int jc = min(8 * g + i, nt - 1), pos = pos0 + jc;
        vat[i] = ((size_t)pt_row[pos >> pshift] * d.Hkv + kvh) * Dh * d.page_tokens + (pos & pmask);
#pragma unroll
        for (int db = 0; db < NDB; ++db) vraw[db][i] = vbase[(size_t)jc * d.ldzx + min(db * 16 + n, Dh - 1)];
      }
    }
#pragma unroll
    for (int blk = 0; blk < 2; ++blk) {
      const int j = 8 * (n >> 2) + (n & 3) + 4 * blk;            // new position of this lane's key row
      const bool live = j < nt;
      const int jc = min(j, nt - 1);
      const float* kr = xrow + (size_t)jc * d.ldzx + d.dq + (size_t)kvh * Dh;
      const size_t kat = (((size_t)pt_row[(pos0 + jc) >> pshift] * d.Hkv + kvh) * d.page_tokens + ((pos0 + jc) & pmask)) * Dh;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        const int d0 = ks * 32 + 8 * g;
        Frag f;
        f.u = make_uint4(0, 0, 0, 0);
        if (d0 < Dh && (blk == 0 || nt > 4)) {                   // the second block only holds positions 4..7, 12..15
          const bool low = d0 < half;                            // an 8-dim group lies in one half (Dh % 16 == 0 here)
          float x[8], xp[8];
          load8(kr + d0, x);
          load8(kr + (low ? d0 + half : d0 - half), xp);
          const float2* cs = rope + (size_t)(pos0 + jc) * half + (low ? d0 : d0 - half);
          uint32_t h[8];
#pragma unroll
          for (int i = 0; i < 8; ++i) {
            const float2 c = cs[i];
            const float r = low ? x[i] * c.x - xp[i] * c.y : x[i] * c.x + xp[i] * c.y;
            h[i] = live ? f32_to_bf16_rne(r) : 0u;
          }
          f.u = make_uint4(h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16));
          if (live) *reinterpret_cast<uint4*>(kpw + kat + d0) = f.u;
        }
        if (blk == 0) nA[ks] = f; else nB[ks] = f;
      }
    }
#pragma unroll
    for (int db = 0; db < NDB; ++db) {
      const int dim = db * 16 + n;
      uint32_t h[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        h[i] = 0u;
        if (8 * g + i < nt && dim < Dh) {
          h[i] = f32_to_bf16_rne(vraw[db][i]);
          vpw[vat[i] + (size_t)dim * d.page_tokens] = (uint16_t)h[i];
        }
      }
      nV[db].u = make_uint4(h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16));
    }
  }

  // ---- query rows: rotate to their positions, scale, split into 3 bf16 terms, stage in LDS
  {
    const float scale = 1.4426950408889634f / sqrtf((float)Dh);   // scores in base-2 units: softmax through 2^x
    const float2* rope = reinterpret_cast<const float2*>(a.rope);
    // (the wavefront that builds the new positions' operands takes no part in the staging)
    const int stagers = FUSE && sp == S - 1 && nk_all > pos0 ? NT - 64 : NT;
    // four items per thread and pass, their loads issued together
    for (int it0 = tid; it0 < R * half && tid < stagers; it0 += 4 * stagers) {
      float x0[4], x1[4];
      float2 c[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int it = it0 + u * stagers, r = it / half, i = it - r * half, rr = row0 + r;
        x0[u] = 0.f; x1[u] = 0.f; c[u] = make_float2(0.f, 0.f);
        if (it < R * half && rr < row_lim) {
          const int j = rr / G;
          const float* q = xrow + (size_t)j * d.ldzx + (size_t)(kvh * G + rr % G) * Dh;
          c[u] = rope[(size_t)(pos0 + j) * half + i];
          x0[u] = q[i]; x1[u] = q[i + half];
        }
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int it = it0 + u * stagers, r = it / half, i = it - r * half;
        if (it >= R * half) break;
        const float lo = (x0[u] * c[u].x - x1[u] * c[u].y) * scale, hi = (x1[u] * c[u].x + x0[u] * c[u].y) * scale;
        uint32_t l0, l1, l2, h0, h1, h2;
        split3(lo, l0, l1, l2);
        split3(hi, h0, h1, h2);
        uint16_t* row = qT + (size_t)r * QS;
        row[i] = (uint16_t)l0; row[Dhp + i] = (uint16_t)l1; row[2 * Dhp + i] = (uint16_t)l2;
        row[i + half] = (uint16_t)h0; row[Dhp + i + half] = (uint16_t)h1; row[2 * Dhp + i + half] = (uint16_t)h2;
      }
    }
    if (Dh < Dhp) {
      const int padw = Dhp - Dh;
      for (int it = tid; it < R * padw * 3 && tid < stagers; it += stagers) {
        const int r = it / (padw * 3), rem = it - r * padw * 3, term = rem / padw, i = rem - term * padw;
        qT[(size_t)r * QS + term * Dhp + Dh + i] = 0;
      }
    }
  }
  __syncthreads();
  TR(2);

  // the key limit of this lane's query row in each tile (row n of tile rt)
  int lim[RT];
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) {
    const int rr = row0 + rt * 16 + n;
    lim[rt] = rr < row_lim ? (FUSE ? pos0 - 1 : pos0 + rr / G) : 0x7fffffff;   // rows past the end: never stored
  }
  const int lim_min = FUSE ? pos0 - 1 : pos0 + row0 / G;     // the smallest limit of the chunk's rows
  float mrun[RT], lrun[RT];
  f32x4 acc[RT][NDB];
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) {
    mrun[rt] = -INFINITY; lrun[rt] = 0.f;
#pragma unroll
    for (int db = 0; db < NDB; ++db) acc[rt][db] = f32x4{0.f, 0.f, 0.f, 0.f};
  }

  // one step of 32 keys: scores, online softmax, output.  The lane's 8 keys are kbase .. kbase+7,
  // visible to the lane's row of tile rt while <= limit[rt].
  // `masked` (wavefront-uniform): some key of the step may be invisible to some row; otherwise
  // all 32 keys are visible to every row and the comparisons are skipped.
  // `nvalid`: keys >= nvalid of a cached step are not in the cache: their value operands are
  // zeroed here (0 * stale bits must not be a NaN).
  auto score_step = [&](const Frag(&ka)[KS], const Frag(&kb)[KS], Frag(&vt)[NDB], const int kbase, const int(&limit)[RT],
                        const bool masked, const int nvalid) {
    if (kbase - 8 * g + kStepKeys > nvalid) {             // wavefront-uniform: the last step of the sequence
      const int cnt = min(max(nvalid - kbase, 0), 8);
      uint32_t mw[4];
#pragma unroll
      for (int w = 0; w < 4; ++w) mw[w] = (2 * w < cnt ? 0x0000FFFFu : 0u) | (2 * w + 1 < cnt ? 0xFFFF0000u : 0u);
#pragma unroll
      for (int db = 0; db < NDB; ++db) { vt[db].u.x &= mw[0]; vt[db].u.y &= mw[1]; vt[db].u.z &= mw[2]; vt[db].u.w &= mw[3]; }
    }
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
      // large tiles: re-read the query fragments from LDS every step instead of keeping all
      // of them in registers across the loop
      if (RT * KS > 4) asm volatile("" ::: "memory");
      f32x4 sA = f32x4{0.f, 0.f, 0.f, 0.f}, sB = f32x4{0.f, 0.f, 0.f, 0.f};
      const uint16_t* qrow = qT + (size_t)(rt * 16 + n) * QS + 8 * g;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
#pragma unroll
        for (int term = 0; term < 3; ++term) {
          Frag q;
          q.u = *reinterpret_cast<const uint4*>(qrow + term * Dhp + ks * 32);
          sA = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka[ks].v, q.v, sA, 0, 0, 0);
          sB = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kb[ks].v, q.v, sB, 0, 0, 0);
        }
      }
      float sc[8] = {sA[0], sA[1], sA[2], sA[3], sB[0], sB[1], sB[2], sB[3]};
      if (masked) {
#pragma unroll
        for (int i = 0; i < 8; ++i) sc[i] = kbase + i <= limit[rt] ? sc[i] : -INFINITY;
      }
      const float mx = fmaxf(fmaxf(fmaxf(sc[0], sc[1]), fmaxf(sc[2], sc[3])), fmaxf(fmaxf(sc[4], sc[5]), fmaxf(sc[6], sc[7])));
      const float mold = mrun[rt];
      const float mnew = fmaxf(mold, xor_max(mx));
      // every key masked so far: keep the state (2^(-inf - -inf) is not a number)
      const float msub = masked && mnew == -INFINITY ? 0.f : mnew;
      float pr[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) pr[i] = ex2(sc[i] - msub);       // 2^-inf = 0 for masked keys
      const float psum = ((pr[0] + pr[1]) + (pr[2] + pr[3])) + ((pr[4] + pr[5]) + (pr[6] + pr[7]));
      const float corr = ex2(mold - msub);                         // 0 while nothing was accumulated
      lrun[rt] = lrun[rt] * corr + psum;
      mrun[rt] = mnew;
      // the probabilities go into the value product split exactly into three bf16 terms
      Frag p0, p1, p2;
      split3_bf16_pair(pr[0], pr[1], p0.u.x, p1.u.x, p2.u.x);
      split3_bf16_pair(pr[2], pr[3], p0.u.y, p1.u.y, p2.u.y);
      split3_bf16_pair(pr[4], pr[5], p0.u.z, p1.u.z, p2.u.z);
      split3_bf16_pair(pr[6], pr[7], p0.u.w, p1.u.w, p2.u.w);
      // the accumulators are rescaled only when some row's maximum rose (and it holds something)
      if (__builtin_amdgcn_ballot_w64(corr != 1.f && mold != -INFINITY) != 0) {
#pragma unroll
        for (int db = 0; db < NDB; ++db) {
          acc[rt][db][0] *= corr; acc[rt][db][1] *= corr; acc[rt][db][2] *= corr; acc[rt][db][3] *= corr;
        }
      }
#pragma unroll
      for (int db = 0; db < NDB; ++db) {
        f32x4 c = acc[rt][db];
        c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vt[db].v, p0.v, c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vt[db].v, p1.v, c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vt[db].v, p2.v, c, 0, 0, 0);
        acc[rt][db] = c;
      }
    }
  };

  // ---- the new positions (FUSE): scored as one more step by the wavefront that built their operands
  if (new_wave) {
    int limn[RT];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
      const int rr = row0 + rt * 16 + n;
      limn[rt] = rr < row_lim ? rr / G : -1;                     // new position j is visible to position rr / G >= j
    }
    score_step(nA, nB, nV, 8 * g, limn, true, 0x7fffffff);
  }

  // Two operand sets in turn: the loads of a step are issued before the previous step is scored.
  // The loop body is branch-free (two steps, loads unconditional: past the last step they repeat
  // it) so that each wait counts exactly the loads issued after the operands it needs; an odd
  // last step follows the loop.
  {
    Frag kA2[KS], kB2[KS], vT2[NDB];
    const int n_steps = max(we - ws, 0);
    for (int step = ws; step + 1 < we; step += 2) {
      load_step(step + 1, kA2, kB2, vT2);
      score_step(kA, kB, vT, step * kStepKeys + 8 * g, lim, (step + 1) * kStepKeys - 1 > lim_min, nk);
      load_step(min(step + 2, we - 1), kA, kB, vT);
      score_step(kA2, kB2, vT2, (step + 1) * kStepKeys + 8 * g, lim, (step + 2) * kStepKeys - 1 > lim_min, nk);
    }
    if (n_steps & 1) score_step(kA, kB, vT, (we - 1) * kStepKeys + 8 * g, lim, we * kStepKeys - 1 > lim_min, nk);
  }
  TR(3);
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) lrun[rt] = xor_add(lrun[rt]);

  // ---- merge the wavefronts (key slices in order) into wavefront 0, one row tile at a time
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) {
    if (wave > 0) {
      if (g == 0) { mrg_ml[((wave - 1) * 16 + n) * 2] = mrun[rt]; mrg_ml[((wave - 1) * 16 + n) * 2 + 1] = lrun[rt]; }
#pragma unroll
      for (int db = 0; db < NDB; ++db)
#pragma unroll
        for (int r = 0; r < 4; ++r) mrg_o[((wave - 1) * Dhp + db * 16 + 4 * g + r) * kMergeLd + n] = acc[rt][db][r];
    }
    __syncthreads();
    if (wave == 0) {
      float mw[NW - 1], lw[NW - 1], M = mrun[rt];
#pragma unroll
      for (int w = 0; w < NW - 1; ++w) { mw[w] = mrg_ml[(w * 16 + n) * 2]; lw[w] = mrg_ml[(w * 16 + n) * 2 + 1]; M = fmaxf(M, mw[w]); }
      const float f0 = mrun[rt] == -INFINITY ? 0.f : ex2(mrun[rt] - M);
      float fw[NW - 1];
      float lsum = f0 * lrun[rt];
#pragma unroll
      for (int w = 0; w < NW - 1; ++w) { fw[w] = mw[w] == -INFINITY ? 0.f : ex2(mw[w] - M); lsum = fmaf(fw[w], lw[w], lsum); }
      lrun[rt] = lsum;
      mrun[rt] = M;
#pragma unroll
      for (int db = 0; db < NDB; ++db)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          float v = f0 * acc[rt][db][r];
#pragma unroll
          for (int w = 0; w < NW - 1; ++w) v = fmaf(fw[w], mrg_o[(w * Dhp + db * 16 + 4 * g + r) * kMergeLd + n], v);
          acc[rt][db][r] = v;
        }
    }
    __syncthreads();
  }
  TR(4);

  // ---- results of the workgroup (held by wavefront 0): final, or the partial of its key slice
  if (wave == 0) {
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
      const int rr = row0 + rt * 16 + n;
      if (rr >= n_rows) continue;
      const int j = rr / G, hq = kvh * G + rr % G;
      if (S == 1) {
        const float inv = (rr < row_lim && lrun[rt] > 0.f) ? 1.0f / lrun[rt] : 0.f;
        float* orow = a.o + ((size_t)b * a.T + j) * d.dq + (size_t)hq * Dh;
#pragma unroll
        for (int db = 0; db < NDB; ++db) {
          const int dim = db * 16 + 4 * g;
          if (dim < Dh)
            *reinterpret_cast<float4*>(orow + dim) =
                make_float4(acc[rt][db][0] * inv, acc[rt][db][1] * inv, acc[rt][db][2] * inv, acc[rt][db][3] * inv);
        }
      } else {
        const size_t rid = (((size_t)b * a.T + j) * d.Hq + hq) * S + sp;
#pragma unroll
        for (int db = 0; db < NDB; ++db) {
          const int dim = db * 16 + 4 * g;
          if (dim < Dh)
            *reinterpret_cast<float4*>(a.part_o + rid * Dh + dim) =
                make_float4(acc[rt][db][0], acc[rt][db][1], acc[rt][db][2], acc[rt][db][3]);
        }
        if (g == 0) { a.part_ml[rid * 2] = mrun[rt]; a.part_ml[rid * 2 + 1] = lrun[rt]; }
      }
    }
  }
  if (S == 1 || a.counters == nullptr) return;   // no counters: a merge kernel follows

  // Make the partials visible device-wide (release), then take a ticket; the workgroup that
  // draws the last ticket sees all of them after its acquire fence and merges the slices.
  TR(5);
  __threadfence();
  __syncthreads();
  int* counter = a.counters + ((size_t)b * d.Hkv + kvh) * row_chunks + chunk;
  if (tid == 0) {
    const int ticket = atomicAdd(counter, 1);
    s_last = ticket == S - 1;
    if (s_last) *counter = 0;   // ready for the next launch (launches on a context are ordered)
  }
  __syncthreads();
  TR(6);
  if (!s_last) return;
  __threadfence();
  float2* gm = reinterpret_cast<float2*>(mrg);   // [R][S] (maximum, sum) of every slice
  const int d4n = Dh >> 2;
  // the first 8 slices of this thread's first output item are requested together with the
  // slice statistics (they do not depend on them)
  float4 pv0[8];
  {
    const int it = min(tid, R * d4n - 1), r = it / d4n, c4 = it - r * d4n, rr = min(row0 + r, n_rows - 1);
    const size_t rid = ((size_t)b * a.T + rr / G) * d.Hq + kvh * G + rr % G;
#pragma unroll
    for (int u = 0; u < 8; ++u) pv0[u] = *reinterpret_cast<const float4*>(a.part_o + (rid * S + min(u, S - 1)) * Dh + 4 * c4);
  }
  for (int it = tid; it < R * S; it += NT) {
    const int r = it / S, s = it - r * S, rr = row0 + r;
    float2 v = make_float2(-INFINITY, 0.f);
    if (rr < n_rows) {
      const size_t rid = ((size_t)b * a.T + rr / G) * d.Hq + kvh * G + rr % G;
      v = reinterpret_cast<const float2*>(a.part_ml)[rid * S + s];
    }
    gm[it] = v;
  }
  __syncthreads();
  TR(7);
  for (int it = tid; it < R * d4n; it += NT) {
    const int r = it / d4n, c4 = it - r * d4n, rr = row0 + r;
    if (rr >= n_rows) continue;
    const int j = rr / G, hq = kvh * G + rr % G;
    const size_t rid = ((size_t)b * a.T + j) * d.Hq + hq;
    float M = -INFINITY;
    for (int s = 0; s < S; ++s) M = fmaxf(M, gm[r * S + s].x);
    float4 out = make_float4(0.f, 0.f, 0.f, 0.f);
    float L = 0.f;
    for (int s0 = 0; s0 < S; s0 += 16) {                // slice order: deterministic; 16 loads in flight
      float4 pv[16];
#pragma unroll
      for (int u = 0; u < 16; ++u)
        if (u < 8 || s0 + 8 < S)
          pv[u] = (it == tid && s0 == 0 && u < 8)
                      ? pv0[u & 7]
                      : *reinterpret_cast<const float4*>(a.part_o + (rid * S + min(s0 + u, S - 1)) * Dh + 4 * c4);
#pragma unroll
      for (int u = 0; u < 16; ++u) {
        if (s0 + u < S) {
          const float2 ml = gm[r * S + s0 + u];
          const float w = ml.x == -INFINITY ? 0.f : ex2(ml.x - M);
          L = fmaf(w, ml.y, L);
          out.x = fmaf(w, pv[u].x, out.x); out.y = fmaf(w, pv[u].y, out.y);
          out.z = fmaf(w, pv[u].z, out.z); out.w = fmaf(w, pv[u].w, out.w);
        }
      }
    }
    const float inv = (rr < row_lim && L > 0.f) ? 1.0f / L : 0.f;
    *reinterpret_cast<float4*>(a.o + ((size_t)b * a.T + j) * d.dq + (size_t)hq * Dh + 4 * c4) =
        make_float4(out.x * inv, out.y * inv, out.z * inv, out.w * inv);
  }
  TR(8);
}

// Merge of the key slices as a kernel of its own, for launches with many workgroups (there the
// device-wide fence of the ticket scheme costs more than a kernel boundary) or with much partial
// data per row chunk (one workgroup would pull all of it through one compute unit).
// grid: x = T * G rows, y = Hkv, z = B; one workgroup per output row.  Thread = (slice group sg,
// float4 column c4): it sums the slices sg, sg + SG, ... of its column; the groups meet in LDS.
__global__ __launch_bounds__(256) void attn_merge_kernel(const Dims d, const AttnArgs a) {
  __shared__ float2 gm[64];        // (maximum, sum) of every slice
  __shared__ float4 red[256];
  const int tid = threadIdx.x;
  const int rr = blockIdx.x, kvh = blockIdx.y, b = blockIdx.z;
  const int Dh = d.Dh, G = d.Hq / d.Hkv, S = a.n_splits, d4n = Dh >> 2;
  const int SG = min(256 / d4n, S), sg = tid / d4n, c4 = tid - sg * d4n;
  const bool active = sg < SG;
  const int j = rr / G, hq = kvh * G + rr % G;
  const size_t rid = ((size_t)b * a.T + j) * d.Hq + hq;
  const float* prow = a.part_o + rid * S * Dh + 4 * c4;
  float4 pv[4];                    // the first pass of loads does not wait for the statistics
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int sl = sg + u * SG;
    pv[u] = active && sl < S ? *reinterpret_cast<const float4*>(prow + (size_t)sl * Dh) : make_float4(0.f, 0.f, 0.f, 0.f);
  }
  if (tid < S) gm[tid] = reinterpret_cast<const float2*>(a.part_ml)[rid * S + tid];
  __syncthreads();
  float M = -INFINITY;
  for (int sl = 0; sl < S; ++sl) M = fmaxf(M, gm[sl].x);
  float4 out = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int s0 = 0; s0 < S; s0 += 4 * SG) {
    if (s0 > 0) {
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int sl = s0 + sg + u * SG;
        pv[u] = active && sl < S ? *reinterpret_cast<const float4*>(prow + (size_t)sl * Dh) : make_float4(0.f, 0.f, 0.f, 0.f);
      }
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int sl = s0 + sg + u * SG;
      if (active && sl < S) {
        const float mx = gm[sl].x;
        const float w = mx == -INFINITY ? 0.f : ex2(mx - M);
        out.x = fmaf(w, pv[u].x, out.x); out.y = fmaf(w, pv[u].y, out.y);
        out.z = fmaf(w, pv[u].z, out.z); out.w = fmaf(w, pv[u].w, out.w);
      }
    }
  }
  red[tid] = out;
  __syncthreads();
  if (sg != 0) return;
  for (int q = 1; q < SG; ++q) {                           // fixed order: deterministic
    const float4 v = red[q * d4n + c4];
    out.x += v.x; out.y += v.y; out.z += v.z; out.w += v.w;
  }
  float L = 0.f;
  for (int sl = 0; sl < S; ++sl) {
    const float2 ml = gm[sl];
    L = fmaf(ml.x == -INFINITY ? 0.f : ex2(ml.x - M), ml.y, L);
  }
  const int nt = a.n_tok != nullptr ? a.n_tok[b] : a.T;
  const float inv = j < nt && L > 0.f ? 1.0f / L : 0.f;    // positions past the valid ones give zeros
  *reinterpret_cast<float4*>(a.o + ((size_t)b * a.T + j) * d.dq + (size_t)hq * Dh + 4 * c4) =
      make_float4(out.x * inv, out.y * inv, out.z * inv, out.w * inv);
}

template <int RT, int KS, bool FUSE, int NW>
static hipError_t launch_w(const Dims& d, const AttnArgs& a, int row_chunks, hipStream_t s) {
  constexpr int Dhp = 32 * KS, QS = 3 * Dhp + 8;
  size_t scratch = (size_t)((NW - 1) * Dhp * kMergeLd + (NW - 1) * 16 * 2) * sizeof(float);
  const size_t gm = (size_t)RT * 16 * a.n_splits * sizeof(float2);
  if (gm > scratch) scratch = gm;
  const size_t lds = (size_t)NW * 64 * 4 + (size_t)RT * 16 * QS * 2 + scratch;
  static size_t lds_enabled = 48 * 1024;
  if (lds > lds_enabled) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(attn_mfma_kernel<RT, KS, FUSE, NW>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    lds_enabled = lds;
  }
  hipLaunchKernelGGL((attn_mfma_kernel<RT, KS, FUSE, NW>), dim3(row_chunks * a.n_splits, d.Hkv, a.B), dim3(64 * NW), lds, s, d, a,
                     row_chunks);
  return hipGetLastError();
}
template <int RT, int KS, bool FUSE>
static hipError_t launch_t(const Dims& d, const AttnArgs& a, int row_chunks, hipStream_t s) {
  // 4 wavefronts: with 8 a wavefront is left with 256 registers and the step loop spills
  return launch_w<RT, KS, FUSE, 4>(d, a, row_chunks, s);
}

template <int KS, bool FUSE>
static hipError_t launch_ks(const Dims& d, const AttnArgs& a, int rt, int row_chunks, hipStream_t s) {
  switch (rt) {
    case 1: return launch_t<1, KS, FUSE>(d, a, row_chunks, s);
    case 2: return launch_t<2, KS, FUSE>(d, a, row_chunks, s);
    case 3: if (KS < 8) return launch_t<(KS < 8 ? 3 : 1), KS, FUSE>(d, a, row_chunks, s); break;
    case 4: if (KS < 8) return launch_t<(KS < 8 ? 4 : 1), KS, FUSE>(d, a, row_chunks, s); break;
  }
  return hipErrorInvalidValue;
}

// the kernel appends the new keys itself: few new positions, one row chunk, 8-dim groups that do not straddle the rotation halves
bool attention_mfma_fuses_append(const Dims& d, int T) {
  return T <= 16 && attention_mfma_row_chunks(d, T) == 1 && d.Dh % 16 == 0;
}

// rows (position x query head of a KV group) per workgroup, in tiles of 16
static int mfma_row_tiles(const Dims& d, int T) {
  const int rows = T * (d.Hq / d.Hkv);
  const int rt_max = d.Dh > 128 ? 2 : 4;
  const int tiles = (rows + 15) / 16;
  return tiles < rt_max ? tiles : rt_max;
}
int attention_mfma_row_chunks(const Dims& d, int T) {
  const int rows = T * (d.Hq / d.Hkv);
  const int per = 16 * mfma_row_tiles(d, T);
  return (rows + per - 1) / per;
}

static constexpr int kTicketMaxBlocks = 64;          // larger launches merge in a second kernel,
static constexpr size_t kTicketMaxBytes = 64 << 10;  // and so do those with more partial data per row chunk

hipError_t launch_attention_mfma(const Dims& d, const AttnArgs& a_in, hipStream_t s) {
  AttnArgs a = a_in;
  if (!d.bf16 || d.page_tokens % 32 != 0 || d.Dh > 256 || d.Dh % 8 != 0 || d.Dh < 8 || a.n_splits > 64 || a.n_splits < 1 || a.T < 1 || a.B < 1 ||
      d.page_tokens % 8 != 0 || (d.page_tokens & (d.page_tokens - 1)) != 0)
    return hipErrorInvalidValue;
  const int rt = mfma_row_tiles(d, a.T), row_chunks = attention_mfma_row_chunks(d, a.T);
  const int ks = (d.Dh + 31) / 32;
  const bool two_kernels = a.n_splits > 1 && ((long)row_chunks * a.n_splits * d.Hkv * a.B > kTicketMaxBlocks ||
                                              (size_t)a.n_splits * rt * 16 * d.Dh * sizeof(float) > kTicketMaxBytes);
  if (two_kernels) a.counters = nullptr;
  hipError_t e;
  if (attention_mfma_fuses_append(d, a.T)) {
    if (ks == 1) e = launch_ks<1, true>(d, a, rt, row_chunks, s);
    else if (ks == 2) e = launch_ks<2, true>(d, a, rt, row_chunks, s);
    else if (ks <= 4) e = launch_ks<4, true>(d, a, rt, row_chunks, s);
    else e = launch_ks<8, true>(d, a, rt, row_chunks, s);
  } else {
    if (ks == 1) e = launch_ks<1, false>(d, a, rt, row_chunks, s);
    else if (ks == 2) e = launch_ks<2, false>(d, a, rt, row_chunks, s);
    else if (ks <= 4) e = launch_ks<4, false>(d, a, rt, row_chunks, s);
    else e = launch_ks<8, false>(d, a, rt, row_chunks, s);
  }
  if (e != hipSuccess || !two_kernels) return e;
  const int rows = a.T * (d.Hq / d.Hkv);
  hipLaunchKernelGGL(attn_merge_kernel, dim3(rows, d.Hkv, a.B), dim3(256), 0, s, d, a);
  return hipGetLastError();
}

}  // namespace hh
