// Attention branch of the hybrid block for multi-position passes (verification, prefill):
// rotary embedding of q and k, append of k and v to the paged KV cache (rounded to the
// storage type), and causal grouped-query attention of the T new positions over all keys
// up to each position, split along the keys with a deterministic log-sum-exp merge.
//
// Cache layout per layer: pages [page][kv_head][token_in_page][Dh]; page_table[b][i] is the
// page holding tokens i*page_tokens .. of sequence b.
//
// Attention kernel: a workgroup owns 16 query rows (row = position j x query head of one
// KV group) and one slice of the keys.  K and V tiles of 64 keys are staged through LDS in
// float32; lane t scores key t for the wavefront's 4 rows, the softmax is kept online per
// row, and lane d accumulates output dimension d.
#include "hh_internal.h"

namespace hh {

static constexpr int kKeys = 64;      // keys per LDS tile
static constexpr int kRowsPerWave = 4;
static constexpr int kRowsPerBlock = 16;
static constexpr int kMaxDh = 256;

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

__device__ __forceinline__ size_t kv_index(const Dims& d, const int* pt_row, int kvh, int pos) {
  const int page = pt_row[pos / d.page_tokens], off = pos % d.page_tokens;
  return (((size_t)page * d.Hkv + kvh) * d.page_tokens + off) * d.Dh;
}

__global__ __launch_bounds__(256) void rope_append_kernel(const Dims d, const AttnArgs a) {
  const int m = blockIdx.x, b = m / a.T, j = m % a.T;
  const int nt = a.n_tok != nullptr ? a.n_tok[b] : a.T;
  if (j >= nt) return;
  const int pos = a.pos0[b] + j;
  const int half = d.Dh / 2;
  float* row = a.qkv + (size_t)m * d.ldzx;
  const int* pt_row = a.page_table + (size_t)b * d.pages_per_seq;
  const float2* cs = reinterpret_cast<const float2*>(a.rope) + (size_t)pos * half;
  const int n_rot = (d.Hq + d.Hkv) * half;
  for (int it = threadIdx.x; it < n_rot + d.Hkv * half; it += blockDim.x) {
    const int hd = it / half, i = it % half;
    if (hd < d.Hq + d.Hkv) {
      float* v = row + (size_t)hd * d.Dh;
      const float2 c = cs[i];
      const float lo = v[i], hi = v[i + half];
      const float rlo = lo * c.x - hi * c.y, rhi = hi * c.x + lo * c.y;
      if (hd < d.Hq) {
        v[i] = rlo; v[i + half] = rhi;
      } else {
        const size_t at = kv_index(d, pt_row, hd - d.Hq, pos);
        if (d.bf16) {
          uint16_t* kp = static_cast<uint16_t*>(a.kpool) + at;
          kp[i] = f32_to_bf16_rne(rlo); kp[i + half] = f32_to_bf16_rne(rhi);
        } else {
          float* kp = static_cast<float*>(a.kpool) + at;
          kp[i] = rlo; kp[i + half] = rhi;
        }
      }
    } else {
      const int kvh = hd - d.Hq - d.Hkv;
      const float* v = row + (size_t)(d.Hq + d.Hkv + kvh) * d.Dh;
      const size_t at = kv_index(d, pt_row, kvh, pos);
      if (d.bf16) {
        uint16_t* vp = static_cast<uint16_t*>(a.vpool) + at;
        vp[i] = f32_to_bf16_rne(v[i]); vp[i + half] = f32_to_bf16_rne(v[i + half]);
      } else {
        float* vp = static_cast<float*>(a.vpool) + at;
        vp[i] = v[i]; vp[i + half] = v[i + half];
      }
    }
  }
}

hipError_t launch_rope_append(const Dims& d, const AttnArgs& a, hipStream_t s) {
  hipLaunchKernelGGL(rope_append_kernel, dim3(a.B * a.T), dim3(256), 0, s, d, a);
  return hipGetLastError();
}

// Reductions over the 64 lanes without LDS traffic: DPP butterflies inside each row of 16
// lanes, then the four row results are read out and combined.  All lanes must be active.
template <int CTRL>
__device__ __forceinline__ float dpp_perm_a(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, false));
}
__device__ __forceinline__ float wave_max(float v) {
  v = fmaxf(v, dpp_perm_a<0xB1>(v));
  v = fmaxf(v, dpp_perm_a<0x4E>(v));
  v = fmaxf(v, dpp_perm_a<0x141>(v));
  v = fmaxf(v, dpp_perm_a<0x140>(v));
  const int iv = __float_as_int(v);
  return fmaxf(fmaxf(__int_as_float(__builtin_amdgcn_readlane(iv, 0)), __int_as_float(__builtin_amdgcn_readlane(iv, 16))),
               fmaxf(__int_as_float(__builtin_amdgcn_readlane(iv, 32)), __int_as_float(__builtin_amdgcn_readlane(iv, 48))));
}
__device__ __forceinline__ float wave_add(float v) {
  v += dpp_perm_a<0xB1>(v);
  v += dpp_perm_a<0x4E>(v);
  v += dpp_perm_a<0x141>(v);
  v += dpp_perm_a<0x140>(v);
  const int iv = __float_as_int(v);
  return (__int_as_float(__builtin_amdgcn_readlane(iv, 0)) + __int_as_float(__builtin_amdgcn_readlane(iv, 16))) +
         (__int_as_float(__builtin_amdgcn_readlane(iv, 32)) + __int_as_float(__builtin_amdgcn_readlane(iv, 48)));
}

// grid: x = row_chunks * n_splits, y = Hkv, z = B
__global__ __launch_bounds__(256) void attention_kernel(const Dims d, const AttnArgs a, const int row_chunks) {
  extern __shared__ __align__(16) float smem[];
  const int Dh = d.Dh, G = d.Hq / d.Hkv;
  const int ldk = Dh + 1;
  float* Ks = smem;                         // [kKeys][Dh+1]
  float* Vs = Ks + kKeys * ldk;             // [kKeys][Dh]
  float* qs = Vs + kKeys * Dh;              // [kRowsPerBlock][Dh]
  float* ps = qs + kRowsPerBlock * Dh;      // [4 waves][kRowsPerWave][kKeys]

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int chunk = blockIdx.x % row_chunks, sp = blockIdx.x / row_chunks;
  const int kvh = blockIdx.y, b = blockIdx.z;
  const int nt = a.n_tok != nullptr ? a.n_tok[b] : a.T;
  const int pos0 = a.pos0[b];
  const int n_rows = a.T * G;
  const int* pt_row = a.page_table + (size_t)b * d.pages_per_seq;
  const float scale = 1.0f / sqrtf((float)Dh);

  // rows of this wavefront
  int rj[kRowsPerWave], rq[kRowsPerWave];
  bool rok[kRowsPerWave];
  int jmax = -1;
  for (int r = 0; r < kRowsPerBlock; ++r) {
    const int rg = chunk * kRowsPerBlock + r;
    if (rg < n_rows && rg / G < nt) jmax = max(jmax, rg / G);
  }
#pragma unroll
  for (int r = 0; r < kRowsPerWave; ++r) {
    const int rg = chunk * kRowsPerBlock + wave * kRowsPerWave + r;
    rj[r] = rg / G; rq[r] = kvh * G + rg % G;
    rok[r] = rg < n_rows && rj[r] < nt;
  }
  // stage the query rows
  for (int it = tid; it < kRowsPerBlock * Dh; it += 256) {
    const int r = it / Dh, dd = it % Dh, rg = chunk * kRowsPerBlock + r;
    float v = 0.f;
    if (rg < n_rows && rg / G < nt)
      v = a.qkv[((size_t)b * a.T + rg / G) * d.ldzx + (size_t)(kvh * G + rg % G) * Dh + dd];
    qs[it] = v;
  }

  // key slice of this workgroup (whole tiles)
  const int nk = jmax < 0 ? 0 : pos0 + jmax + 1;
  const int tiles = (nk + kKeys - 1) / kKeys;
  const int tps = (tiles + a.n_splits - 1) / a.n_splits;
  const int t_begin = sp * tps, t_end = min(tiles, (sp + 1) * tps);

  float mrun[kRowsPerWave], lrun[kRowsPerWave], acc[kRowsPerWave][kMaxDh / 64];
#pragma unroll
  for (int r = 0; r < kRowsPerWave; ++r) {
    mrun[r] = -INFINITY; lrun[r] = 0.f;
#pragma unroll
    for (int e = 0; e < kMaxDh / 64; ++e) acc[r][e] = 0.f;
  }

  for (int t = t_begin; t < t_end; ++t) {
    const int key0 = t * kKeys;
    __syncthreads();
    // stage K and V tiles as float32
    for (int it = tid; it < kKeys * (Dh / 8); it += 256) {
      const int kk = it / (Dh / 8), c8 = (it % (Dh / 8)) * 8;
      const int key = key0 + kk;
      float kv8[8], vv8[8];
      if (key < nk) {
        const size_t at = kv_index(d, pt_row, kvh, key) + c8;
        if (d.bf16) {
          const uint4 ku = *reinterpret_cast<const uint4*>(static_cast<const uint16_t*>(a.kpool) + at);
          const uint4 vu = *reinterpret_cast<const uint4*>(static_cast<const uint16_t*>(a.vpool) + at);
          const uint32_t kw[4] = {ku.x, ku.y, ku.z, ku.w}, vw[4] = {vu.x, vu.y, vu.z, vu.w};
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            kv8[2 * i] = __uint_as_float(kw[i] << 16); kv8[2 * i + 1] = __uint_as_float(kw[i] & 0xffff0000u);
            vv8[2 * i] = __uint_as_float(vw[i] << 16); vv8[2 * i + 1] = __uint_as_float(vw[i] & 0xffff0000u);
          }
        } else {
          const float* kp = static_cast<const float*>(a.kpool) + at;
          const float* vp = static_cast<const float*>(a.vpool) + at;
#pragma unroll
          for (int i = 0; i < 8; ++i) { kv8[i] = kp[i]; vv8[i] = vp[i]; }
        }
      } else {
#pragma unroll
        for (int i = 0; i < 8; ++i) { kv8[i] = 0.f; vv8[i] = 0.f; }
      }
#pragma unroll
      for (int i = 0; i < 8; ++i) { Ks[kk * ldk + c8 + i] = kv8[i]; Vs[kk * Dh + c8 + i] = vv8[i]; }
    }
    __syncthreads();
    // scores: lane = key
    float sc[kRowsPerWave];
#pragma unroll
    for (int r = 0; r < kRowsPerWave; ++r) sc[r] = 0.f;
    for (int dd = 0; dd < Dh; ++dd) {
      const float kvv = Ks[lane * ldk + dd];
#pragma unroll
      for (int r = 0; r < kRowsPerWave; ++r) sc[r] = fmaf(qs[(wave * kRowsPerWave + r) * Dh + dd], kvv, sc[r]);
    }
    const int key = key0 + lane;
#pragma unroll
    for (int r = 0; r < kRowsPerWave; ++r) {
      const bool vis = rok[r] && key <= pos0 + rj[r];
      const float sv = vis ? sc[r] * scale : -INFINITY;
      const float mnew = fmaxf(mrun[r], wave_max(sv));
      float pr = 0.f, corr = 1.f;
      if (mnew != -INFINITY) {
        pr = vis ? expf(sv - mnew) : 0.f;
        corr = mrun[r] == -INFINITY ? 0.f : expf(mrun[r] - mnew);
      }
      lrun[r] = lrun[r] * corr + wave_add(pr);
      mrun[r] = mnew;
#pragma unroll
      for (int e = 0; e < kMaxDh / 64; ++e) acc[r][e] *= corr;
      ps[(wave * kRowsPerWave + r) * kKeys + lane] = pr;
    }
    __syncthreads();
    // output: lane = dimension
    for (int kk = 0; kk < kKeys; ++kk) {
#pragma unroll
      for (int e = 0; e < kMaxDh / 64; ++e) {
        const int dd = lane + 64 * e;
        if (dd < Dh) {
          const float vv = Vs[kk * Dh + dd];
#pragma unroll
          for (int r = 0; r < kRowsPerWave; ++r) acc[r][e] = fmaf(ps[(wave * kRowsPerWave + r) * kKeys + kk], vv, acc[r][e]);
        }
      }
    }
  }

  // ---- write results
#pragma unroll
  for (int r = 0; r < kRowsPerWave; ++r) {
    const int rg = chunk * kRowsPerBlock + wave * kRowsPerWave + r;
    if (rg >= n_rows) continue;
    const size_t mrow = (size_t)b * a.T + rj[r];
    if (a.n_splits == 1) {
      const float inv = (rok[r] && lrun[r] > 0.f) ? 1.0f / lrun[r] : 0.f;
#pragma unroll
      for (int e = 0; e < kMaxDh / 64; ++e) {
        const int dd = lane + 64 * e;
        if (dd < Dh) a.o[mrow * d.dq + (size_t)rq[r] * Dh + dd] = acc[r][e] * inv;
      }
    } else {
      const size_t rid = (mrow * d.Hq + rq[r]) * a.n_splits + sp;
#pragma unroll
      for (int e = 0; e < kMaxDh / 64; ++e) {
        const int dd = lane + 64 * e;
        if (dd < Dh) a.part_o[rid * Dh + dd] = acc[r][e];
      }
      if (lane == 0) { a.part_ml[rid * 2] = mrun[r]; a.part_ml[rid * 2 + 1] = lrun[r]; }
    }
  }
}

// grid: B*T*Hq rows; merges the key slices in slice order
__global__ void attention_merge_kernel(const Dims d, const AttnArgs a) {
  const size_t row = blockIdx.x;
  const int hq = row % d.Hq;
  const size_t m = row / d.Hq;
  const int S = a.n_splits;
  float M = -INFINITY;
  for (int s = 0; s < S; ++s) M = fmaxf(M, a.part_ml[(row * S + s) * 2]);
  float L = 0.f;
  for (int s = 0; s < S; ++s) {
    const float ms = a.part_ml[(row * S + s) * 2];
    if (ms != -INFINITY) L += expf(ms - M) * a.part_ml[(row * S + s) * 2 + 1];
  }
  for (int dd = threadIdx.x; dd < d.Dh; dd += blockDim.x) {
    float v = 0.f;
    if (L > 0.f) {
      for (int s = 0; s < S; ++s) {
        const float ms = a.part_ml[(row * S + s) * 2];
        if (ms != -INFINITY) v += expf(ms - M) * a.part_o[(row * S + s) * d.Dh + dd];
      }
      v /= L;
    }
    a.o[m * d.dq + (size_t)hq * d.Dh + dd] = v;
  }
}

hipError_t launch_attention(const Dims& d, const AttnArgs& a, hipStream_t s) {
  if (d.Dh > kMaxDh || d.Dh % 8 != 0) return hipErrorInvalidValue;
  const int G = d.Hq / d.Hkv;
  const int row_chunks = (a.T * G + kRowsPerBlock - 1) / kRowsPerBlock;
  const size_t lds = ((size_t)kKeys * (d.Dh + 1) + (size_t)kKeys * d.Dh + (size_t)kRowsPerBlock * d.Dh +
                      4 * kRowsPerWave * kKeys) * sizeof(float);
  static bool big = false;
  if (lds > 48 * 1024 && !big) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(attention_kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (e != hipSuccess) return e;
    big = true;
  }
  hipLaunchKernelGGL(attention_kernel, dim3(row_chunks * a.n_splits, d.Hkv, a.B), dim3(256), lds, s, d, a, row_chunks);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (a.n_splits > 1) {
    hipLaunchKernelGGL(attention_merge_kernel, dim3(a.B * a.T * d.Hq), dim3(64), 0, s, d, a);
    e = hipGetLastError();
  }
  return e;
}

__global__ void export_kv_kernel(const Dims d, const LayerDev* layer, const int* page_table, int seq, int tok0,
                                 int n_tokens, float* k, float* v) {
  const int* pt_row = page_table + (size_t)seq * d.pages_per_seq;
  const size_t total = (size_t)n_tokens * d.Hkv * d.Dh;
  for (size_t it = blockIdx.x * (size_t)blockDim.x + threadIdx.x; it < total; it += (size_t)gridDim.x * blockDim.x) {
    const int dd = it % d.Dh, kvh = (it / d.Dh) % d.Hkv, pos = tok0 + (int)(it / ((size_t)d.Dh * d.Hkv));
    const size_t at = kv_index(d, pt_row, kvh, pos) + dd;
    if (d.bf16) {
      k[it] = __uint_as_float((uint32_t) static_cast<const uint16_t*>(layer->kpool)[at] << 16);
      v[it] = __uint_as_float((uint32_t) static_cast<const uint16_t*>(layer->vpool)[at] << 16);
    } else {
      k[it] = static_cast<const float*>(layer->kpool)[at];
      v[it] = static_cast<const float*>(layer->vpool)[at];
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
