// Token choice at temperature T > 0 (Section 3.3, Eq. 6 of the paper): draws from
// softmax(logits / T) for the draft steps and for the first token, and the rejection test of
// the round with its correction token drawn from norm(max(0, P_H - P_S)).
//
// A draw from unnormalised masses p_0 .. p_{V-1} with a uniform u is the inverse CDF in index
// order: the smallest i with p_0 + .. + p_i > u * sum(p).  The uniforms are 24-bit values of a
// counter-based generator: output number c of SplitMix64 (Steele, Lea, Flood 2014) started at
// the caller's seed, c = sequence * 2^34 + stream position * 4 + purpose (0 draft draw,
// 1 acceptance test, 2 correction / bonus / first token), so any decision can be recomputed alone.
//
// The outcome of a round is written in the form the commit step already consumes: targets[i] =
// drafts[i] for the kept positions, targets[n] = the emitted token, later entries -1; the
// longest-matching-prefix rule then returns n, because the residual has no mass at a rejected draft.
#include <mutex>

#include "hh_internal.h"

namespace hh {
namespace {

constexpr int kDrawThreads = 1024;
constexpr int kDrawWaves = kDrawThreads / 64;

__device__ __forceinline__ uint64_t splitmix64_at(uint64_t seed, uint64_t counter) {
  uint64_t z = seed + (counter + 1) * 0x9E3779B97F4A7C15ull;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

__device__ __forceinline__ float uniform24(uint64_t seed, int b, int idx, int purpose) {
  const uint64_t c = (static_cast<uint64_t>(b) << 34) + (static_cast<uint64_t>(idx) << 2) + static_cast<uint64_t>(purpose);
  return static_cast<float>(splitmix64_at(seed, c) >> 40) * 0x1p-24f;
}

__device__ __forceinline__ float wave_max(float v) {
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}

// softmax(l / T) entry from the row's maximum m and 1 / sum: the one expression every kernel here uses,
// so that a probability computed in two places has the same bits.  The product is rounded on its own
// (never contracted into a following subtraction: fma(a, b, -round(a * b)) is the rounding error of
// the product, which would give the residual of two identical distributions a noise mass).
__device__ __forceinline__ float prob(float l, float m, float inv_t, float rsum) {
#pragma clang fp contract(off)
  return expf((l - m) * inv_t) * rsum;
}
// max(0, P_H - P_S) of one entry, the subtraction kept apart from the two products
__device__ __forceinline__ float residual_mass(float ph, float ps) {
#pragma clang fp contract(off)
  const float d = ph - ps;
  return fmaxf(0.f, d);
}

constexpr float kNoLogit = -3.0e38f;   // stands for an entry past the end of the row: exp((kNoLogit - m) / T) = 0

// entries jj .. jj+3 of a row (jj a multiple of 4); past `end` they read as kNoLogit.  vec: the row
// starts on a 16-byte boundary
__device__ __forceinline__ void load_group(const float* __restrict__ row, int jj, int end, bool vec, float (&l)[4]) {
  if (vec && jj + 3 < end) {
    const float4 t = *reinterpret_cast<const float4*>(row + jj);
    l[0] = t.x; l[1] = t.y; l[2] = t.z; l[3] = t.w;
  } else {
    for (int e = 0; e < 4; ++e) l[e] = jj + e < end ? row[jj + e] : kNoLogit;
  }
}
__device__ __forceinline__ bool row_is_vec(const float* row) { return (reinterpret_cast<uintptr_t>(row) & 15) == 0; }

// max over the row, by a whole workgroup; `red` holds blockDim.x / 64 floats
__device__ float row_max(const float* __restrict__ row, int V, float* red) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, nw = blockDim.x >> 6;
  const bool vec = row_is_vec(row);
  float m = kNoLogit;
#pragma unroll 4
  for (int j = threadIdx.x * 4; j < V; j += blockDim.x * 4) {
    float l[4];
    load_group(row, j, V, vec, l);
    m = fmaxf(fmaxf(m, fmaxf(l[0], l[1])), fmaxf(l[2], l[3]));
  }
  m = wave_max(m);
  if (lane == 0) red[w] = m;
  __syncthreads();
  m = red[0];
  for (int i = 1; i < nw; ++i) m = fmaxf(m, red[i]);
  __syncthreads();
  return m;
}

// max over the row and sum of exp((l - max) / T), by a whole workgroup; `red` holds blockDim.x / 64 floats
__device__ void row_stats(const float* __restrict__ row, int V, float inv_t, float* red, float& m_out, float& s_out) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, nw = blockDim.x >> 6;
  const bool vec = row_is_vec(row);
  const float m = row_max(row, V, red);
  float s = 0.f;
#pragma unroll 4
  for (int j = threadIdx.x * 4; j < V; j += blockDim.x * 4) {
    float l[4];
    load_group(row, j, V, vec, l);
    s += (expf((l[0] - m) * inv_t) + expf((l[1] - m) * inv_t)) + (expf((l[2] - m) * inv_t) + expf((l[3] - m) * inv_t));
  }
  s = wave_sum(s);
  if (lane == 0) red[w] = s;
  __syncthreads();
  s = 0.f;
  for (int i = 0; i < nw; ++i) s += red[i];
  __syncthreads();
  m_out = m; s_out = s;
}

// Inverse-CDF draw by a workgroup of kDrawThreads threads.  val(jj, end, v) fills v[0..3] with the
// masses (>= 0) of indices jj .. jj+3, zero past `end`.
// Wavefront w owns the contiguous segment [w * seg, (w + 1) * seg); the segment sums give the
// segment that holds u * total, and that wavefront alone scans its segment in index order.
// red: kDrawWaves floats, res: one int (both in LDS).  Every thread returns the drawn index, or -1
// when no entry has mass.
template <typename F>
__device__ int block_draw(F val, int V, float u, float* red, int* res) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int seg = ((V + kDrawWaves * 256 - 1) / (kDrawWaves * 256)) * 256;
  const int j0 = min(V, w * seg), j1 = min(V, j0 + seg);
  float acc = 0.f;
#pragma unroll 4
  for (int j = j0 + lane * 4; j < j1; j += 256) {
    float v[4];
    val(j, j1, v);
    acc += (v[0] + v[1]) + (v[2] + v[3]);
  }
  acc = wave_sum(acc);
  if (lane == 0) red[w] = acc;
  __syncthreads();
  float total = 0.f;
  for (int i = 0; i < kDrawWaves; ++i) total += red[i];
  if (!(total > 0.f)) {          // uniform over the workgroup: every thread summed the same values
    __syncthreads();
    return -1;
  }
  const float target = u * total;
  int ws = -1;
  float carry = 0.f, c = 0.f;
  for (int i = 0; i < kDrawWaves; ++i) {
    const float nx = c + red[i];
    if (ws < 0 && nx > target) { ws = i; carry = c; }
    c = nx;
  }
  if (ws < 0) {   // u * total rounded up to the total: the last segment that has mass
    ws = 0;
    c = 0.f;
    for (int i = 0; i < kDrawWaves; ++i) {
      if (red[i] > 0.f) { ws = i; carry = c; }
      c += red[i];
    }
  }
  if (w == ws) {
    int result = -1;
    int last_mass = -1;        // last index with mass seen so far (the answer if rounding hides the crossing)
    float cw = carry;
    for (int j = j0; j < j1 && result < 0; j += 256) {
      const int jj = j + lane * 4;
      float v[4];
      val(jj, j1, v);
      float t = 0.f;
      int lm = -1;
      for (int e = 0; e < 4; ++e) {
        t += v[e];
        if (v[e] > 0.f) lm = jj + e;
      }
      float incl = t;
      for (int o = 1; o < 64; o <<= 1) {
        const float up = __shfl_up(incl, o);
        if (lane >= o) incl += up;
      }
      float excl = __shfl_up(incl, 1);
      if (lane == 0) excl = 0.f;
      const unsigned long long hit = __ballot(cw + incl > target);
      if (hit != 0ull) {
        const int fl = __ffsll(hit) - 1;
        int r = -1;
        if (lane == fl) {
          float c2 = cw + excl;
          for (int e = 0; e < 4; ++e) {
            c2 += v[e];
            if (r < 0 && v[e] > 0.f && c2 > target) r = jj + e;
          }
          if (r < 0) r = lm;
        }
        r = __shfl(r, fl);
        if (r < 0) {   // the lane's own walk fell short by rounding and it holds no mass: nearest mass before it
          int prev = lane < fl ? lm : -1;
          for (int o = 32; o > 0; o >>= 1) prev = max(prev, __shfl_xor(prev, o));
          r = prev >= 0 ? prev : last_mass;
          if (r < 0) r = min(jj, j1 - 1);
          r = __shfl(r, fl);
        }
        result = r;
      } else {
        cw += __shfl(incl, 63);
        int blk = lm;
        for (int o = 32; o > 0; o >>= 1) blk = max(blk, __shfl_xor(blk, o));
        if (blk >= 0) last_mass = blk;
      }
    }
    if (result < 0) result = last_mass >= 0 ? last_mass : max(j1 - 1, 0);
    if (lane == 0) *res = result;
  }
  __syncthreads();
  const int out = *res;
  __syncthreads();
  return out;
}

// One row per workgroup: token drawn from softmax(row / T).
__global__ __launch_bounds__(kDrawThreads) void sample_rows_kernel(const float* __restrict__ logits, size_t row_stride, int V,
                                                                    const SamplingParams* __restrict__ prm_dev,
                                                                    const SamplingParams prm_val,
                                                                    const int* __restrict__ idx_base, int idx_off,
                                                                    int purpose, int* __restrict__ out, int out_stride,
                                                                    int out_off) {
  __shared__ float red[kDrawWaves];
  __shared__ int res;
  const int b = blockIdx.x;
  const float* row = logits + static_cast<size_t>(b) * row_stride;
  const SamplingParams prm = prm_dev ? *prm_dev : prm_val;
  const float inv_t = prm.inv_t;
  const bool vec = row_is_vec(row);
  const float m = row_max(row, V, red);
  const int idx = (idx_base ? idx_base[b] : 0) + idx_off;
  const float u = uniform24(prm.seed, b, idx, purpose);
  const int tok = block_draw(
      [&](int jj, int end, float (&v)[4]) {
        float l[4];
        load_group(row, jj, end, vec, l);
        for (int e = 0; e < 4; ++e) v[e] = expf((l[e] - m) * inv_t);
      },
      V, u, red, &res);
  if (threadIdx.x == 0) out[static_cast<size_t>(b) * out_stride + out_off] = tok;
}

// (max, sum) of the k draft rows and the k + 1 verification rows of every sequence:
// stats[b][r][2], r < kmax: draft row r; r >= kmax: verification row r - kmax.
__global__ __launch_bounds__(kDrawThreads) void softmax_stats_kernel(const float* __restrict__ logits_d,
                                                            const float* __restrict__ logits_v, int V, int k, int kmax,
                                                            const SamplingParams* __restrict__ prm_dev,
                                                            const SamplingParams prm_val, float* __restrict__ stats) {
  __shared__ float red[kDrawWaves];
  const int r = blockIdx.x, b = blockIdx.y;
  const float* row;
  int slot;
  if (r < k) { row = logits_d + (static_cast<size_t>(b) * kmax + r) * V; slot = r; }
  else { row = logits_v + (static_cast<size_t>(b) * (k + 1) + (r - k)) * V; slot = kmax + (r - k); }
  float m, s;
  row_stats(row, V, prm_dev ? prm_dev->inv_t : prm_val.inv_t, red, m, s);
  if (threadIdx.x == 0) {
    float* st = stats + (static_cast<size_t>(b) * (2 * kmax + 1) + slot) * 2;
    st[0] = m; st[1] = s;
  }
}

// The round's acceptance for one sequence per workgroup (Eq. 6) and its targets row.
__global__ __launch_bounds__(kDrawThreads) void spec_targets_kernel(const float* __restrict__ logits_d,
                                                                     const float* __restrict__ logits_v, int V, int k,
                                                                     int kmax, const SamplingParams* __restrict__ prm_dev,
                                                                     const SamplingParams prm_val,
                                                                     const float* __restrict__ stats,
                                                                     const int* __restrict__ drafts,
                                                                     const int* __restrict__ committed,
                                                                     int* __restrict__ targets) {
  __shared__ float red[kDrawWaves];
  __shared__ int res;
  __shared__ int n_sh;
  const int b = blockIdx.x;
  const SamplingParams prm = prm_dev ? *prm_dev : prm_val;
  const float inv_t = prm.inv_t;
  const uint64_t seed = prm.seed;
  const int base = committed[b];
  const int* d = drafts + static_cast<size_t>(b) * kmax;
  const float* st = stats + static_cast<size_t>(b) * (2 * kmax + 1) * 2;
  const float* rows_d = logits_d + static_cast<size_t>(b) * kmax * V;
  const float* rows_v = logits_v + static_cast<size_t>(b) * (k + 1) * V;
  if (threadIdx.x == 0) {
    int n = k;
    for (int i = 0; i < k; ++i) {
      const int di = d[i];
      if (di < 0 || di >= V) { n = i; break; }   // not a token: rejected, never used as an index
      const float ps = prob(rows_d[static_cast<size_t>(i) * V + di], st[2 * i], inv_t, 1.0f / st[2 * i + 1]);
      const float ph = prob(rows_v[static_cast<size_t>(i) * V + di], st[2 * (kmax + i)], inv_t, 1.0f / st[2 * (kmax + i) + 1]);
      const float u = uniform24(seed, b, base + i, 1);
      if (!(u < ph / ps)) { n = i; break; }      // kept with probability min(1, P_H / P_S)
    }
    n_sh = n;
  }
  __syncthreads();
  const int n = n_sh;
  const float u = uniform24(seed, b, base + n, 2);
  const float* lh = rows_v + static_cast<size_t>(n) * V;
  const float mh = st[2 * (kmax + n)], rsh = 1.0f / st[2 * (kmax + n) + 1];
  int tok;
  if (n < k) {
    const float* ls = rows_d + static_cast<size_t>(n) * V;
    const float ms = st[2 * n], rss = 1.0f / st[2 * n + 1];
    const bool vec = row_is_vec(lh) && row_is_vec(ls);
    tok = block_draw(
        [&](int jj, int end, float (&v)[4]) {
          float a[4], c[4];
          load_group(lh, jj, end, vec, a);
          load_group(ls, jj, end, vec, c);
          for (int e = 0; e < 4; ++e) v[e] = residual_mass(prob(a[e], mh, inv_t, rsh), prob(c[e], ms, inv_t, rss));
        },
        V, u, red, &res);
    if (tok < 0) {
      // The residual has no mass (the two distributions agree to rounding; in exact arithmetic a
      // rejection implies mass elsewhere): the token is drawn from P_H with the same uniform, and
      // should that be the rejected draft itself, its successor in index order is taken, so that
      // the targets row still encodes n.
      tok = block_draw(
          [&](int jj, int end, float (&v)[4]) {
            float l[4];
            load_group(lh, jj, end, row_is_vec(lh), l);
            for (int e = 0; e < 4; ++e) v[e] = expf((l[e] - mh) * inv_t);
          },
          V, u, red, &res);
      if (tok == d[n]) tok = tok + 1 < V ? tok + 1 : 0;
    }
  } else {
    const bool vec = row_is_vec(lh);
    tok = block_draw(
        [&](int jj, int end, float (&v)[4]) {
          float l[4];
          load_group(lh, jj, end, vec, l);
          for (int e = 0; e < 4; ++e) v[e] = expf((l[e] - mh) * inv_t);
        },
        V, u, red, &res);
  }
  int* g = targets + static_cast<size_t>(b) * (kmax + 1);
  for (int i = threadIdx.x; i <= k; i += blockDim.x) g[i] = i < n ? d[i] : (i == n ? tok : -1);
}

}  // namespace

hipError_t launch_sample_rows(const float* logits, size_t row_stride, int V, int B, const SamplingParams* prm,
                              SamplingParams prm_val, const int* idx_base, int idx_off, int purpose, int* out,
                              int out_stride, int out_off, hipStream_t s) {
  hipLaunchKernelGGL(sample_rows_kernel, dim3(B), dim3(kDrawThreads), 0, s, logits, row_stride, V, prm, prm_val, idx_base,
                     idx_off, purpose, out, out_stride, out_off);
  return hipGetLastError();
}

// ---- statistics buffer of the entry point that allocates nothing (hh_accept_tokens_static):
// one array per GPU, held until the process ends.  In host code the array's name is only a
// stand-in for the symbol; the device address comes from hipGetSymbolAddress, once per device.
constexpr size_t kStaticScratchFloats = 1 << 16;
static __device__ __align__(256) float scratch[kStaticScratchFloats];

hipError_t static_accept_scratch(float** ptr, size_t* n_floats) {
  constexpr int kMaxDevices = 64;
  static std::mutex mu;
  static float* per_device[kMaxDevices] = {};
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(mu);
  if (per_device[dev] == nullptr) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));   // the current device's copy of the array
    if (e != hipSuccess) return e;
    if (p == nullptr) return hipErrorInvalidSymbol;
    per_device[dev] = static_cast<float*>(p);
  }
  *ptr = per_device[dev];
  *n_floats = kStaticScratchFloats;
  return hipSuccess;
}

hipError_t launch_spec_targets(const float* logits_d, const float* logits_v, int V, int B, int k, int kmax,
                               const SamplingParams* prm, SamplingParams prm_val, float* stats, const int* drafts,
                               const int* committed, int* targets, hipStream_t s) {
  hipLaunchKernelGGL(softmax_stats_kernel, dim3(2 * k + 1, B), dim3(kDrawThreads), 0, s, logits_d, logits_v, V, k, kmax, prm,
                     prm_val, stats);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(spec_targets_kernel, dim3(B), dim3(kDrawThreads), 0, s, logits_d, logits_v, V, k, kmax, prm, prm_val,
                     stats, drafts, committed, targets);
  return hipGetLastError();
}

}  // namespace hh
