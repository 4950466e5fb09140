// Small kernels of the round protocol: token gathering and embedding lookup, the final
// step of the LM-head argmax, greedy acceptance with its bookkeeping, and helpers for
// prefill.  All token ids, lengths and counts stay on the device between the calls of a
// round; nothing here is read back by the host.
#include "hh_internal.h"

namespace hh {

// h[m][:] = E[tok[m]][:]
__global__ void embed_kernel(const void* embed, int bf16, const int* tok, int D, int V, float* h) {
  const int m = blockIdx.x;
  const size_t src = (size_t)min(max(tok[m], 0), V - 1) * D;   // an id that is no token reads a valid row, never out of bounds
  for (int k = threadIdx.x; k < D; k += blockDim.x) {
    float v;
    if (bf16) v = __uint_as_float((uint32_t) static_cast<const uint16_t*>(embed)[src + k] << 16);
    else v = static_cast<const float*>(embed)[src + k];
    h[(size_t)m * D + k] = v;
  }
}

hipError_t launch_embed(const Dims& d, const void* embed, const int* tok, int M, float* h, hipStream_t s) {
  hipLaunchKernelGGL(embed_kernel, dim3(M), dim3(256), 0, s, embed, d.bf16, tok, d.D, d.V, h);
  return hipGetLastError();
}

// mode 0: draft step `step`: tok[b] = step == 0 ? pending[b] : drafts[b][step-1]; pos0[b] = kv_len[b] + step
// mode 1: verification:      tok[b*T + 0] = pending[b], tok[b*T + j] = drafts[b][j-1]; pos0[b] = kv_len[b]
__global__ void gather_tokens_kernel(const int* pending, const int* drafts, int kmax, int B, int T, int mode, int step,
                                     int* tok, const int* kv_len, int* pos0) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (mode == 0) {
    if (i < B) {
      tok[i] = step == 0 ? pending[i] : drafts[i * kmax + step - 1];
      pos0[i] = kv_len[i] + step;
    }
  } else if (i < B * T) {
    const int b = i / T, j = i % T;
    tok[i] = j == 0 ? pending[b] : drafts[b * kmax + j - 1];
    if (j == 0) pos0[b] = kv_len[b];
  }
}

hipError_t launch_gather_tokens(const int* pending, const int* drafts, int kmax, int B, int T, int mode, int step,
                                int* tok, const int* kv_len, int* pos0, hipStream_t s) {
  const int n = mode == 0 ? B : B * T;
  hipLaunchKernelGGL(gather_tokens_kernel, dim3((n + 255) / 256), dim3(256), 0, s, pending, drafts, kmax, B, T, mode,
                     step, tok, kv_len, pos0);
  return hipGetLastError();
}

// Prefill pass: tok[b*T + j] = prompt[b][off + j] for j < n_tok[b] (0 beyond); pos0[b] = kv_len[b]
__global__ void gather_prompt_kernel(const int* prompt, int row_stride, int off, const int* n_tok, int B, int T,
                                     int* tok, const int* kv_len, int* pos0) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= B * T) return;
  const int b = i / T, j = i % T;
  tok[i] = j < n_tok[b] ? prompt[(size_t)b * row_stride + off + j] : 0;
  if (j == 0) pos0[b] = kv_len[b];
}

hipError_t launch_gather_prompt(const int* prompt, int row_stride, int off, const int* n_tok, int B, int T, int* tok,
                                const int* kv_len, int* pos0, hipStream_t s) {
  hipLaunchKernelGGL(gather_prompt_kernel, dim3((B * T + 255) / 256), dim3(256), 0, s, prompt, row_stride, off, n_tok,
                     B, T, tok, kv_len, pos0);
  return hipGetLastError();
}

// Reduce the per-workgroup argmax partials of the LM head: row m = b*T + j -> out[b*out_stride + out_off + j]
__global__ void argmax_finish_kernel(const unsigned long long* best, int n_part, int M, int* out, int out_stride,
                                     int out_off, int T) {
  const int m = blockIdx.x;
  unsigned long long v = 0ull;
  for (int i = threadIdx.x; i < n_part; i += blockDim.x) v = max(v, best[(size_t)m * n_part + i]);
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = max(v, (unsigned long long)__shfl_xor((long long)v, o, 64));
  __shared__ unsigned long long w[4];
  if ((threadIdx.x & 63) == 0) w[threadIdx.x >> 6] = v;
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int i = 1; i < (int)(blockDim.x >> 6); ++i) v = max(v, w[i]);
    const int b = m / T, j = m % T;
    out[(size_t)b * out_stride + out_off + j] = (int)(0xFFFFFFFFu - (uint32_t)(v & 0xFFFFFFFFull));
  }
}

hipError_t launch_argmax_finish(const unsigned long long* best, int n_part, int M, int* out, int out_stride,
                                int out_off, int T, hipStream_t s) {
  hipLaunchKernelGGL(argmax_finish_kernel, dim3(M), dim3(256), 0, s, best, n_part, M, out, out_stride, out_off, T);
  return hipGetLastError();
}

// Greedy acceptance (longest prefix with drafts[i] == targets[i]) or a forced count, then the
// bookkeeping of the commit: emitted tokens, pending token, committed count.  The cache length
// is advanced later (after the state rebuild has used it) by adding adv[b].
__global__ void accept_kernel(const CommitArgs a) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= a.B) return;
  const int done = a.committed[b] >= a.G;
  a.skip[b] = done;
  if (done) { a.n_acc[b] = 0; a.adv[b] = 0; return; }
  const int* d = a.drafts + (size_t)b * a.kmax;
  const int* g = a.targets + (size_t)b * (a.kmax + 1);
  int n = 0;
  if (a.forced != nullptr) {
    n = min(max(a.forced[b], 0), a.k);
  } else {
    while (n < a.k && d[n] == g[n]) ++n;
  }
  int c = a.committed[b];
  int* out = a.out_tok + (size_t)b * a.out_stride;
  for (int i = 0; i < n && c < a.G; ++i) out[c++] = d[i];
  if (c < a.G) out[c++] = g[n];
  a.committed[b] = c;
  a.pending[b] = g[n];
  a.last_n[b] = n;
  a.n_acc[b] = n;
  a.adv[b] = n + 1;
  // acceptance statistics: drafts 1..n passed their test, draft n+1 (if there is one) failed it
  if (a.acc_stats != nullptr && a.k > 0) {
    atomicAdd(a.acc_stats, (unsigned long long)n);
    atomicAdd(a.acc_stats + 1, (unsigned long long)min(n + 1, a.k));
  }
}

hipError_t launch_accept(const CommitArgs& a, hipStream_t s) {
  hipLaunchKernelGGL(accept_kernel, dim3((a.B + 63) / 64), dim3(64), 0, s, a);
  return hipGetLastError();
}

__global__ void advance_kernel(int* kv_len, const int* n, int B) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b < B) kv_len[b] += n[b];
}

hipError_t launch_advance(int* kv_len, const int* n, int B, hipStream_t s) {
  hipLaunchKernelGGL(advance_kernel, dim3((B + 63) / 64), dim3(64), 0, s, kv_len, n, B);
  return hipGetLastError();
}

// After a prefill pass: keep the stream of each sequence's last prompt position (input of the
// LM head) and advance the cache length by the positions consumed.
__global__ void prefill_tail_kernel(const float* h, int T, int D, const int* n_tok, const int* is_last, float* lasth,
                                    int* kv_len) {
  const int b = blockIdx.x;
  const int nt = n_tok[b];
  if (nt > 0 && is_last[b]) {
    const float* src = h + ((size_t)b * T + nt - 1) * D;
    for (int k = threadIdx.x; k < D; k += blockDim.x) lasth[(size_t)b * D + k] = src[k];
  }
  if (threadIdx.x == 0) kv_len[b] += nt;
}

hipError_t launch_prefill_tail(const float* h, int T, int D, const int* n_tok, const int* is_last, float* lasth,
                               int* kv_len, int B, hipStream_t s) {
  hipLaunchKernelGGL(prefill_tail_kernel, dim3(B), dim3(256), 0, s, h, T, D, n_tok, is_last, lasth, kv_len);
  return hipGetLastError();
}

// First generated token: pending, first entry of the output, committed = 1
__global__ void prefill_finish_kernel(const int* first_tok, int* pending, int* out_tok, int out_stride, int* committed,
                                      int* last_n, int B) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= B) return;
  pending[b] = first_tok[b];
  out_tok[(size_t)b * out_stride] = first_tok[b];
  committed[b] = 1;
  last_n[b] = 0;
}

hipError_t launch_prefill_finish(const int* first_tok, int* pending, int* out_tok, int out_stride, int* committed,
                                 int* last_n, int B, hipStream_t s) {
  hipLaunchKernelGGL(prefill_finish_kernel, dim3((B + 63) / 64), dim3(64), 0, s, first_tok, pending, out_tok, out_stride,
                     committed, last_n, B);
  return hipGetLastError();
}

__global__ void fill_i32_kernel(int* p, int v, size_t n) {
  for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = v;
}
__global__ void fill_f32_kernel(float* p, float v, size_t n) {
  for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = v;
}

hipError_t launch_fill_i32(int* p, int v, size_t n, hipStream_t s) {
  if (n == 0) return hipSuccess;
  const int blocks = (int)((n + 255) / 256 < 4096 ? (n + 255) / 256 : 4096);
  hipLaunchKernelGGL(fill_i32_kernel, dim3(blocks), dim3(256), 0, s, p, v, n);
  return hipGetLastError();
}
hipError_t launch_fill_f32(float* p, float v, size_t n, hipStream_t s) {
  if (n == 0) return hipSuccess;
  const int blocks = (int)((n + 255) / 256 < 4096 ? (n + 255) / 256 : 4096);
  hipLaunchKernelGGL(fill_f32_kernel, dim3(blocks), dim3(256), 0, s, p, v, n);
  return hipGetLastError();
}

}  // namespace hh
