// Attention branch of the hybrid block for multi-position passes (verification, prefill):
// the float32-FMA kernel (float32 KV cache; any head dimension that is a multiple of 8), the
// append of new keys and values to the paged cache, and the dispatch between this kernel and
// the matrix-core kernel used for a bf16 cache.
//
// One kernel per layer: rotary embedding of q and k, append of k and v to the paged KV cache
// (rounded to the storage type), causal grouped-query attention of the T new positions over
// all keys up to each position, split along the keys, and the log-sum-exp merge of the key
// slices in slice order.
//
// A workgroup owns 16 query rows (row = position j x query head of one KV group) and one
// slice of the keys.  K and V tiles of 64 keys are staged through LDS in float32: cached keys
// come from the pages; the keys of the new positions are rotated from the projection buffer,
// rounded, written to the cache by the one workgroup that owns them, and used as rounded.
// Lane t scores key t for the wavefront's 4 rows, the softmax is kept online per row, lane d
// accumulates output dimension d.  With several key slices every workgroup stores its partial
// result; the last one to finish (a counter per row chunk) merges them, so no second launch.
#include <stdlib.h>
#include "wave_ops.h"

#include "attn_common.h"

namespace hh {

static constexpr int kKeys = 64;      // keys per LDS tile
static constexpr int kRowsPerWave = 4;
static constexpr int kRowsPerBlock = 16;
static constexpr int kMaxDh = 256;

// Reductions over the 64 lanes without LDS traffic: DPP butterflies inside each row of 16
// lanes, then the four row results are read out and combined.  All lanes must be active.
__device__ __forceinline__ float wave_max(float v) {
  v = fmaxf(v, dpp_move<0xB1>(v));
  v = fmaxf(v, dpp_move<0x4E>(v));
  v = fmaxf(v, dpp_move<0x141>(v));
  v = fmaxf(v, dpp_move<0x140>(v));
  const int iv = __float_as_int(v);
  return fmaxf(fmaxf(__int_as_float(__builtin_amdgcn_readlane(iv, 0)), __int_as_float(__builtin_amdgcn_readlane(iv, 16))),
               fmaxf(__int_as_float(__builtin_amdgcn_readlane(iv, 32)), __int_as_float(__builtin_amdgcn_readlane(iv, 48))));
}
__device__ __forceinline__ float wave_add(float v) {
  v += dpp_move<0xB1>(v);
  v += dpp_move<0x4E>(v);
  v += dpp_move<0x141>(v);
  v += dpp_move<0x140>(v);
  const int iv = __float_as_int(v);
  return (__int_as_float(__builtin_amdgcn_readlane(iv, 0)) + __int_as_float(__builtin_amdgcn_readlane(iv, 16))) +
         (__int_as_float(__builtin_amdgcn_readlane(iv, 32)) + __int_as_float(__builtin_amdgcn_readlane(iv, 48)));
}


__device__ __forceinline__ float round_store(float v, int bf16) {
  return bf16 ? __uint_as_float((uint32_t)f32_to_bf16_rne(v) << 16) : v;
}

// grid: x = row_chunks * n_splits, y = Hkv, z = B.  E = ceil(Dh / 64).
//
// Order of the global loads of a workgroup (each later group needs the one before): position
// of the sequence -> page numbers, query rows, rotation table, new keys -> cached keys of the
// first tile.  The cached keys of tile t + 1 are requested before tile t is scored.
template <int BF16, int E>
__global__ __launch_bounds__(256) void attention_kernel(const Dims d, const AttnArgs a, const int row_chunks) {
  constexpr int EPI = BF16 ? 8 : 4;          // elements per 16-byte item
  constexpr int NI = BF16 ? 2 * E : 4 * E;   // items of a K (or V) tile per thread
  constexpr int NQ = 2 * E;                  // rotation pairs of the query rows per thread
  extern __shared__ __align__(16) float smem[];
  __shared__ int s_last;
  const int Dh = d.Dh, G = d.Hq / d.Hkv, half = Dh >> 1;
  const int ldk = Dh + 1;
  float* Ks = smem;                         // [kKeys][Dh+1]
  float* Vs = Ks + kKeys * ldk;             // [kKeys][Dh]
  float* qs = Vs + kKeys * Dh;              // [kRowsPerBlock][Dh]
  float* ps = qs + kRowsPerBlock * Dh;      // [4 waves][kRowsPerWave][kKeys]

  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int chunk = blockIdx.x % row_chunks, sp = blockIdx.x / row_chunks;
  const int kvh = blockIdx.y, b = blockIdx.z;
  TR(0);
  const int nt = a.n_tok != nullptr ? a.n_tok[b] : a.T;
  const int pos0 = a.pos0[b];
  const int n_rows = a.T * G;
  const int* pt_row = a.page_table + (size_t)b * d.pages_per_seq;
  const float scale = 1.0f / sqrtf((float)Dh);
  const float2* rope = reinterpret_cast<const float2*>(a.rope);
  const float* xrow = a.qkv + (size_t)b * a.T * d.ldzx;   // q | k | v of this sequence's positions
  const size_t esz = BF16 ? 2 : 4;
  const char* kbytes = static_cast<const char*>(a.kpool);
  const char* vbytes = static_cast<const char*>(a.vpool);

  // rows of this workgroup: row = position j * G + query head of the group; valid while j < nt
  const int row_lim = min(n_rows, nt * G);
  const int row0 = chunk * kRowsPerBlock;
  const int jmax = row0 < row_lim ? (min(row_lim, row0 + kRowsPerBlock) - 1) / G : -1;
  int rj[kRowsPerWave], rq[kRowsPerWave];
  bool rok[kRowsPerWave];
#pragma unroll
  for (int r = 0; r < kRowsPerWave; ++r) {
    const int rg = row0 + wave * kRowsPerWave + r;
    rj[r] = rg / G; rq[r] = kvh * G + rg % G;
    rok[r] = rg < row_lim;
  }

  // key slice of this workgroup (whole tiles)
  const int nk = jmax < 0 ? 0 : pos0 + jmax + 1;
  const int tiles = (nk + kKeys - 1) / kKeys;
  const int tps = (tiles + a.n_splits - 1) / a.n_splits;
  const int t_begin = sp * tps, t_end = min(tiles, (sp + 1) * tps);
  const int cpk = Dh / EPI;                 // items per key
  const int n_items = kKeys * cpk;

  // ---- cached keys of a tile: pages -> registers -> LDS as float32.  A K item is 16 bytes of
  // one key row; a V item is 16 bytes of one dimension (consecutive tokens of a page).
  uint4 kreg[NI], vreg[NI];
  constexpr int TPI = EPI;                   // tokens per V item
  auto load_tile = [&](int t) {
    const int key0 = t * kKeys;
    const int n_old = min(max(pos0 - key0, 0), kKeys);          // keys of this tile already in the cache
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      const int it = tid + 256 * i;
      const int kk = it / cpk, c = (it - kk * cpk) * EPI;
      if (kk < n_old) kreg[i] = *reinterpret_cast<const uint4*>(kbytes + (k_index(d, pt_row, kvh, key0 + kk) + c) * esz);
      const int grp = it / Dh, dd = it - grp * Dh;
      if (grp * TPI < n_old) vreg[i] = *reinterpret_cast<const uint4*>(vbytes + v_index(d, pt_row, kvh, key0 + grp * TPI, dd) * esz);
    }
  };
  auto store_tile = [&](int t) {
    const int key0 = t * kKeys;
    const int n_old = min(max(pos0 - key0, 0), kKeys);
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      const int it = tid + 256 * i;
      if (it >= n_items) continue;
      const int kk = it / cpk, c = (it - kk * cpk) * EPI;
      float* kd = Ks + kk * ldk + c;
      if (kk < n_old) {
        const uint32_t kw[4] = {kreg[i].x, kreg[i].y, kreg[i].z, kreg[i].w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          if (BF16) { kd[2 * e] = __uint_as_float(kw[e] << 16); kd[2 * e + 1] = __uint_as_float(kw[e] & 0xffff0000u); }
          else kd[e] = __uint_as_float(kw[e]);
        }
      } else if (key0 + kk >= nk) {           // past the last key: zeros (the new keys are staged separately)
#pragma unroll
        for (int e = 0; e < EPI; ++e) kd[e] = 0.f;
      }
      const int grp = it / Dh, dd = it - grp * Dh;
      const uint32_t vw[4] = {vreg[i].x, vreg[i].y, vreg[i].z, vreg[i].w};
#pragma unroll
      for (int e = 0; e < TPI; ++e) {
        const int vk = grp * TPI + e;
        float val = 0.f;
        if (vk < n_old) val = BF16 ? ((e & 1) ? __uint_as_float(vw[e >> 1] & 0xffff0000u) : __uint_as_float(vw[e >> 1] << 16))
                                   : __uint_as_float(vw[e & 3]);
        if (vk < n_old || key0 + vk >= nk) Vs[vk * Dh + dd] = val;
      }
    }
  };
  // ---- keys of the new positions in a tile: rotate, round, append to the cache, use as rounded
  struct NewKey { float k0, k1, v0, v1; float2 c; };
  auto new_count = [&](int t) {
    const int key0 = t * kKeys;
    return min(nk - key0, kKeys) - min(max(pos0 - key0, 0), kKeys);
  };
  auto load_new = [&](int t, int it, NewKey& nw) {
    const int key0 = t * kKeys;
    const int n_old = min(max(pos0 - key0, 0), kKeys);
    const int kk = n_old + it / half, i = it % half;
    const int j = key0 + kk - pos0;
    const float* kr = xrow + (size_t)j * d.ldzx + d.dq + (size_t)kvh * Dh;
    const float* vr = kr + d.dkv;
    nw.c = rope[(size_t)(pos0 + j) * half + i];
    nw.k0 = kr[i]; nw.k1 = kr[i + half]; nw.v0 = vr[i]; nw.v1 = vr[i + half];
  };
  auto store_new = [&](int t, int it, const NewKey& nw) {
    const int key0 = t * kKeys;
    const int n_old = min(max(pos0 - key0, 0), kKeys);
    const int kk = n_old + it / half, i = it % half;
    const int j = key0 + kk - pos0;
    const float klo = round_store(nw.k0 * nw.c.x - nw.k1 * nw.c.y, BF16), khi = round_store(nw.k1 * nw.c.x + nw.k0 * nw.c.y, BF16);
    const float vlo = round_store(nw.v0, BF16), vhi = round_store(nw.v1, BF16);
    Ks[kk * ldk + i] = klo; Ks[kk * ldk + i + half] = khi;
    Vs[kk * Dh + i] = vlo; Vs[kk * Dh + i + half] = vhi;
    if (chunk == (j * G) / kRowsPerBlock) {   // the one row chunk that owns position j writes it
      const size_t at = k_index(d, pt_row, kvh, pos0 + j);
      const size_t v0 = v_index(d, pt_row, kvh, pos0 + j, i), v1 = v_index(d, pt_row, kvh, pos0 + j, i + half);
      if (BF16) {
        uint16_t* kp = static_cast<uint16_t*>(a.kpool) + at;
        uint16_t* vp = static_cast<uint16_t*>(a.vpool);
        kp[i] = (uint16_t)(__float_as_uint(klo) >> 16); kp[i + half] = (uint16_t)(__float_as_uint(khi) >> 16);
        vp[v0] = (uint16_t)(__float_as_uint(vlo) >> 16); vp[v1] = (uint16_t)(__float_as_uint(vhi) >> 16);
      } else {
        float* kp = static_cast<float*>(a.kpool) + at;
        float* vp = static_cast<float*>(a.vpool);
        kp[i] = klo; kp[i + half] = khi; vp[v0] = vlo; vp[v1] = vhi;
      }
    }
  };

  // ---- loads of the prologue, all in flight together
  float qx0[NQ], qx1[NQ];
  float2 qc[NQ];
#pragma unroll
  for (int i = 0; i < NQ; ++i) {
    const int it = tid + 256 * i;
    const int r = it / half, ii = it - r * half, rg = row0 + r;
    qx0[i] = 0.f; qx1[i] = 0.f; qc[i] = make_float2(0.f, 0.f);
    if (r < kRowsPerBlock && rg < row_lim) {
      const int j = rg / G;
      const float* q = xrow + (size_t)j * d.ldzx + (size_t)(kvh * G + rg % G) * Dh;
      qc[i] = rope[(size_t)(pos0 + j) * half + ii];
      qx0[i] = q[ii]; qx1[i] = q[ii + half];
    }
  }
  NewKey nw0;
  const int n_new0 = t_begin < t_end ? new_count(t_begin) * half : 0;   // rotation pairs of new keys in the first tile
  if (tid < n_new0) load_new(t_begin, tid, nw0);
  if (t_begin < t_end) load_tile(t_begin);
  TR(1);
  // query rows, rotated to their positions and scaled
#pragma unroll
  for (int i = 0; i < NQ; ++i) {
    const int it = tid + 256 * i;
    const int r = it / half, ii = it - r * half;
    if (r < kRowsPerBlock) {
      qs[r * Dh + ii] = (qx0[i] * qc[i].x - qx1[i] * qc[i].y) * scale;
      qs[r * Dh + ii + half] = (qx1[i] * qc[i].x + qx0[i] * qc[i].y) * scale;
    }
  }

  float mrun[kRowsPerWave], lrun[kRowsPerWave], acc[kRowsPerWave][E];
#pragma unroll
  for (int r = 0; r < kRowsPerWave; ++r) {
    mrun[r] = -INFINITY; lrun[r] = 0.f;
#pragma unroll
    for (int e = 0; e < E; ++e) acc[r][e] = 0.f;
  }

  for (int t = t_begin; t < t_end; ++t) {
    const int key0 = t * kKeys;
    if (t != t_begin) __syncthreads();      // the previous tile has been consumed
    const int n_new = new_count(t) * half;
    if (t == t_begin) {
      if (tid < n_new) store_new(t, tid, nw0);
      for (int it = tid + 256; it < n_new; it += 256) { NewKey nw; load_new(t, it, nw); store_new(t, it, nw); }
    } else {
      for (int it = tid; it < n_new; it += 256) { NewKey nw; load_new(t, it, nw); store_new(t, it, nw); }
    }
    TR(2);
    store_tile(t);
    __syncthreads();
    TR(3);
    if (t + 1 < t_end) load_tile(t + 1);
    // scores: lane = key
    float sc[kRowsPerWave];
#pragma unroll
    for (int r = 0; r < kRowsPerWave; ++r) sc[r] = 0.f;
#pragma unroll 8
    for (int dd = 0; dd < Dh; ++dd) {
      const float kvv = Ks[lane * ldk + dd];
#pragma unroll
      for (int r = 0; r < kRowsPerWave; ++r) sc[r] = fmaf(qs[(wave * kRowsPerWave + r) * Dh + dd], kvv, sc[r]);
    }
    TR(4);
    const int key = key0 + lane;
#pragma unroll
    for (int r = 0; r < kRowsPerWave; ++r) {
      const bool vis = rok[r] && key <= pos0 + rj[r];
      const float sv = vis ? sc[r] : -INFINITY;
      const float mnew = fmaxf(mrun[r], wave_max(sv));
      float pr = 0.f, corr = 1.f;
      if (mnew != -INFINITY) {
        pr = vis ? expf(sv - mnew) : 0.f;
        corr = mrun[r] == -INFINITY ? 0.f : expf(mrun[r] - mnew);
      }
      lrun[r] = lrun[r] * corr + wave_add(pr);
      mrun[r] = mnew;
#pragma unroll
      for (int e = 0; e < E; ++e) acc[r][e] *= corr;
      ps[(wave * kRowsPerWave + r) * kKeys + lane] = pr;
    }
    // (ps is written and read by the same wavefront only)
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    TR(5);
    // output: lane = dimension
#pragma unroll 4
    for (int kk = 0; kk < kKeys; ++kk) {
#pragma unroll
      for (int e = 0; e < E; ++e) {
        const int dd = lane + 64 * e;
        if (dd < Dh) {
          const float vv = Vs[kk * Dh + dd];
#pragma unroll
          for (int r = 0; r < kRowsPerWave; ++r) acc[r][e] = fmaf(ps[(wave * kRowsPerWave + r) * kKeys + kk], vv, acc[r][e]);
        }
      }
    }
  }

  TR(6);
  // ---- results: final when there is one key slice, else partial + merge by the last workgroup
  if (a.n_splits == 1) {
#pragma unroll
    for (int r = 0; r < kRowsPerWave; ++r) {
      const int rg = row0 + wave * kRowsPerWave + r;
      if (rg >= n_rows) continue;
      const size_t mrow = (size_t)b * a.T + rj[r];
      const float inv = (rok[r] && lrun[r] > 0.f) ? 1.0f / lrun[r] : 0.f;
#pragma unroll
      for (int e = 0; e < E; ++e) {
        const int dd = lane + 64 * e;
        if (dd < Dh) a.o[mrow * d.dq + (size_t)rq[r] * Dh + dd] = acc[r][e] * inv;
      }
    }
    return;
  }
  const int S = a.n_splits;
#pragma unroll
  for (int r = 0; r < kRowsPerWave; ++r) {
    const int rg = row0 + wave * kRowsPerWave + r;
    if (rg >= n_rows) continue;
    const size_t rid = (((size_t)b * a.T + rj[r]) * d.Hq + rq[r]) * S + sp;
#pragma unroll
    for (int e = 0; e < E; ++e) {
      const int dd = lane + 64 * e;
      if (dd < Dh) a.part_o[rid * Dh + dd] = acc[r][e];
    }
    if (lane == 0) { a.part_ml[rid * 2] = mrun[r]; a.part_ml[rid * 2 + 1] = lrun[r]; }
  }
  // Make the partials visible device-wide (release), then take a ticket; the workgroup that
  // draws the last ticket sees all of them after its acquire fence and merges.
  TR(7);
  __threadfence();
  __syncthreads();
  TR(8);
  int* counter = a.counters + ((size_t)b * d.Hkv + kvh) * row_chunks + chunk;
  if (tid == 0) {
    const int ticket = atomicAdd(counter, 1);
    s_last = ticket == S - 1;
    if (s_last) *counter = 0;   // ready for the next launch (launches on a context are ordered)
  }
  __syncthreads();
  TR(9);
  if (!s_last) return;
  __threadfence();
  TR(10);
  // lane s holds slice s of each of the wavefront's rows (S <= 64); all loads are issued
  // before the first of them is used
  constexpr int kAhead = 4;
  float ms[kRowsPerWave], ls[kRowsPerWave], po[kRowsPerWave][E][kAhead];
  size_t rid0[kRowsPerWave];
#pragma unroll
  for (int r = 0; r < kRowsPerWave; ++r) {
    const int rg = min(row0 + wave * kRowsPerWave + r, n_rows - 1);
    rid0[r] = (((size_t)b * a.T + rg / G) * d.Hq + kvh * G + rg % G) * S;
    const float2 ml = reinterpret_cast<const float2*>(a.part_ml)[rid0[r] + min(lane, S - 1)];
    ms[r] = lane < S ? ml.x : -INFINITY; ls[r] = lane < S ? ml.y : 0.f;
  }
#pragma unroll
  for (int r = 0; r < kRowsPerWave; ++r)
#pragma unroll
    for (int e = 0; e < E; ++e)
#pragma unroll
      for (int u = 0; u < kAhead; ++u)
        po[r][e][u] = a.part_o[(rid0[r] + min(u, S - 1)) * Dh + min(lane + 64 * e, Dh - 1)];
  TR(11);
#pragma unroll
  for (int r = 0; r < kRowsPerWave; ++r) {
    const int rg = row0 + wave * kRowsPerWave + r;
    if (rg >= n_rows) continue;                     // uniform per wavefront
    const float M = wave_max(ms[r]);
    const float ws = ms[r] != -INFINITY ? expf(ms[r] - M) : 0.f;
    const float L = wave_add(ws * ls[r]);
    const int wbits = __float_as_int(ws);
    float out[E];
#pragma unroll
    for (int e = 0; e < E; ++e) out[e] = 0.f;
#pragma unroll
    for (int u = 0; u < kAhead; ++u) {              // slice order: deterministic
      if (u < S) {
        const float w = __int_as_float(__builtin_amdgcn_readlane(wbits, u));
#pragma unroll
        for (int e = 0; e < E; ++e) out[e] = fmaf(w, po[r][e][u], out[e]);
      }
    }
    for (int s0 = kAhead; s0 < S; s0 += kAhead) {
      float pn[E][kAhead];
#pragma unroll
      for (int e = 0; e < E; ++e)
#pragma unroll
        for (int u = 0; u < kAhead; ++u)
          pn[e][u] = a.part_o[(rid0[r] + min(s0 + u, S - 1)) * Dh + min(lane + 64 * e, Dh - 1)];
#pragma unroll
      for (int u = 0; u < kAhead; ++u) {
        if (s0 + u < S) {
          const float w = __int_as_float(__builtin_amdgcn_readlane(wbits, s0 + u));
#pragma unroll
          for (int e = 0; e < E; ++e) out[e] = fmaf(w, pn[e][u], out[e]);
        }
      }
    }
    const size_t mrow = (size_t)b * a.T + rj[r];
    const float inv = (rok[r] && L > 0.f) ? 1.0f / L : 0.f;
#pragma unroll
    for (int e = 0; e < E; ++e) {
      const int dd = lane + 64 * e;
      if (dd < Dh) a.o[mrow * d.dq + (size_t)rq[r] * Dh + dd] = out[e] * inv;
    }
  }
  TR(12);
}

template <int BF16, int E>
static hipError_t launch_attention_t(const Dims& d, const AttnArgs& a, int row_chunks, size_t lds, hipStream_t s) {
  static size_t lds_enabled = 48 * 1024;
  if (lds > lds_enabled) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(attention_kernel<BF16, E>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    lds_enabled = lds;
  }
  hipLaunchKernelGGL((attention_kernel<BF16, E>), dim3(row_chunks * a.n_splits, d.Hkv, a.B), dim3(256), lds, s, d, a,
                     row_chunks);
  return hipGetLastError();
}

// Keys and values of the new positions: rotate k, round to the storage type, write to the pages.
// grid: one workgroup per (sequence, new position).
__global__ __launch_bounds__(256) void kv_append_kernel(const Dims d, const AttnArgs a) {
  const int m = blockIdx.x, b = m / a.T, j = m - b * a.T;
  const int nt = a.n_tok != nullptr ? a.n_tok[b] : a.T;
  if (j >= nt) return;
  const int pos = a.pos0[b] + j;
  const int Dh = d.Dh, half = Dh >> 1;
  const float* krow = a.qkv + (size_t)m * d.ldzx + d.dq;
  const float* vrow = krow + d.dkv;
  const int* pt_row = a.page_table + (size_t)b * d.pages_per_seq;
  const float2* cs = reinterpret_cast<const float2*>(a.rope) + (size_t)pos * half;
  for (int it = threadIdx.x; it < d.Hkv * half; it += 256) {
    const int kvh = it / half, i = it - kvh * half;
    const float2 c = cs[i];
    const float x0 = krow[kvh * Dh + i], x1 = krow[kvh * Dh + i + half];
    const float lo = x0 * c.x - x1 * c.y, hi = x1 * c.x + x0 * c.y;
    const size_t at = k_index(d, pt_row, kvh, pos);
    if (d.bf16) {
      uint16_t* kp = static_cast<uint16_t*>(a.kpool) + at;
      kp[i] = f32_to_bf16_rne(lo); kp[i + half] = f32_to_bf16_rne(hi);
    } else {
      float* kp = static_cast<float*>(a.kpool) + at;
      kp[i] = lo; kp[i + half] = hi;
    }
  }
  for (int it = threadIdx.x; it < d.Hkv * Dh; it += 256) {
    const int kvh = it / Dh, dd = it - kvh * Dh;
    const size_t at = v_index(d, pt_row, kvh, pos, dd);
    if (d.bf16) static_cast<uint16_t*>(a.vpool)[at] = f32_to_bf16_rne(vrow[it]);
    else static_cast<float*>(a.vpool)[at] = vrow[it];
  }
}

// The same for a bf16 cache whose pages hold a multiple of 8 tokens, in groups of 8 consecutive positions
// (aligned to 8, so a group lies in one page): the values of one dimension for the 8 tokens are 16 contiguous
// bytes of the transposed V page and are written as one store (the kernel above writes them as 8 separate
// 2-byte stores from 8 workgroups).  Same arithmetic and rounding.  grid: sequence x groups_per_seq.
__global__ __launch_bounds__(256) void kv_append8_kernel(const Dims d, const AttnArgs a, int groups_per_seq) {
  const int b = blockIdx.x / groups_per_seq, gl = blockIdx.x - b * groups_per_seq;
  const int nt = min(a.n_tok != nullptr ? a.n_tok[b] : a.T, a.T);
  const int pos0 = a.pos0[b];
  const int p_first = ((pos0 >> 3) + gl) << 3;               // first position of this group
  if (nt <= 0 || p_first >= pos0 + nt) return;
  const int Dh = d.Dh, half = Dh >> 1;
  const int* pt_row = a.page_table + (size_t)b * d.pages_per_seq;
  const float* rows = a.qkv + (size_t)b * a.T * d.ldzx + d.dq;   // row j: k | v of position pos0 + j
  const bool whole = p_first >= pos0 && p_first + 8 <= pos0 + nt;
  uint16_t* vpool = static_cast<uint16_t*>(a.vpool);
  for (int it = threadIdx.x; it < d.Hkv * Dh; it += 256) {
    const int kvh = it / Dh, dd = it - kvh * Dh;
    const size_t at = v_index(d, pt_row, kvh, p_first, dd);
    if (whole) {
      uint32_t h[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) h[u] = f32_to_bf16_rne(rows[(size_t)(p_first - pos0 + u) * d.ldzx + d.dkv + it]);
      *reinterpret_cast<uint4*>(vpool + at) = make_uint4(h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16));
    } else {
      for (int u = 0; u < 8; ++u) {
        const int j = p_first + u - pos0;
        if (j >= 0 && j < nt) vpool[at + u] = f32_to_bf16_rne(rows[(size_t)j * d.ldzx + d.dkv + it]);
      }
    }
  }
  uint16_t* kpool = static_cast<uint16_t*>(a.kpool);
  const int per = d.Hkv * half;
  for (int it = threadIdx.x; it < 8 * per; it += 256) {
    const int u = it / per, rem = it - u * per, kvh = rem / half, i = rem - kvh * half;
    const int pos = p_first + u, j = pos - pos0;
    if (j < 0 || j >= nt) continue;
    const float2 c = reinterpret_cast<const float2*>(a.rope)[(size_t)pos * half + i];
    const float* krow = rows + (size_t)j * d.ldzx;
    const float x0 = krow[kvh * Dh + i], x1 = krow[kvh * Dh + i + half];
    const float lo = x0 * c.x - x1 * c.y, hi = x1 * c.x + x0 * c.y;
    uint16_t* kp = kpool + k_index(d, pt_row, kvh, pos);
    kp[i] = f32_to_bf16_rne(lo); kp[i + half] = f32_to_bf16_rne(hi);
  }
}

// bf16 cache: matrix-core kernel (HH_KF_ATTN_SCALAR selects the float32-FMA kernel instead, for cross-checks)
bool attention_uses_mfma(const Dims& d) {
  return d.bf16 && !(d.flags & HH_KF_ATTN_SCALAR) && d.page_tokens % 32 == 0;   // a 32-key step of that kernel lies in one page
}

hipError_t launch_attention(const Dims& d, const AttnArgs& a, hipStream_t s) {
  if (d.Dh > kMaxDh || d.Dh % 8 != 0 || a.n_splits > 64 || a.n_splits < 1 || a.T < 1 || a.B < 1) return hipErrorInvalidValue;
  if (attention_uses_mfma(d)) {
    if (!attention_mfma_fuses_append(d, a.T)) {
      if (a.T >= 16 && d.page_tokens % 8 == 0) {
        const int groups = (a.T + 7) / 8 + 1;      // 8-aligned groups that T consecutive positions can touch
        hipLaunchKernelGGL(kv_append8_kernel, dim3(a.B * groups), dim3(256), 0, s, d, a, groups);
      } else {
        hipLaunchKernelGGL(kv_append_kernel, dim3(a.B * a.T), dim3(256), 0, s, d, a);
      }
      hipError_t e = hipGetLastError();
      if (e != hipSuccess) return e;
    }
    return launch_attention_mfma(d, a, s);
  }
  const int G = d.Hq / d.Hkv;
  const int row_chunks = (a.T * G + kRowsPerBlock - 1) / kRowsPerBlock;
  const size_t lds = ((size_t)kKeys * (d.Dh + 1) + (size_t)kKeys * d.Dh + (size_t)kRowsPerBlock * d.Dh +
                      4 * kRowsPerWave * kKeys) * sizeof(float);
  const int E = (d.Dh + 63) / 64;
  if (d.bf16) {
    if (E == 1) return launch_attention_t<1, 1>(d, a, row_chunks, lds, s);
    if (E == 2) return launch_attention_t<1, 2>(d, a, row_chunks, lds, s);
    return launch_attention_t<1, 4>(d, a, row_chunks, lds, s);
  }
  if (E == 1) return launch_attention_t<0, 1>(d, a, row_chunks, lds, s);
  if (E == 2) return launch_attention_t<0, 2>(d, a, row_chunks, lds, s);
  return launch_attention_t<0, 4>(d, a, row_chunks, lds, s);
}

// upper bound on the row chunks of either kernel (sizes the ticket counters)
int attention_row_chunks(const Dims& d, int T) { return (T * (d.Hq / d.Hkv) + kRowsPerBlock - 1) / kRowsPerBlock; }

__global__ void export_kv_kernel(const Dims d, const LayerDev* layer, const int* page_table, int seq, int tok0,
                                 int n_tokens, float* k, float* v) {
  const int* pt_row = page_table + (size_t)seq * d.pages_per_seq;
  const size_t total = (size_t)n_tokens * d.Hkv * d.Dh;
  for (size_t it = blockIdx.x * (size_t)blockDim.x + threadIdx.x; it < total; it += (size_t)gridDim.x * blockDim.x) {
    const int dd = it % d.Dh, kvh = (it / d.Dh) % d.Hkv, pos = tok0 + (int)(it / ((size_t)d.Dh * d.Hkv));
    const size_t at = k_index(d, pt_row, kvh, pos) + dd, vat = v_index(d, pt_row, kvh, pos, dd);
    if (d.bf16) {
      k[it] = __uint_as_float((uint32_t) static_cast<const uint16_t*>(layer->kpool)[at] << 16);
      v[it] = __uint_as_float((uint32_t) static_cast<const uint16_t*>(layer->vpool)[vat] << 16);
    } else {
      k[it] = static_cast<const float*>(layer->kpool)[at];
      v[it] = static_cast<const float*>(layer->vpool)[vat];
    }
  }
}

hipError_t launch_export_kv(const Dims& d, const LayerDev* layer, const int* page_table, int seq, int tok0,
                            int n_tokens, float* k, float* v, hipStream_t s) {
  if (n_tokens <= 0) return hipSuccess;
  hipLaunchKernelGGL(export_kv_kernel, dim3(64), dim3(256), 0, s, d, layer, page_table, seq, tok0, n_tokens, k, v);
  return hipGetLastError();
}

}  // namespace hh
