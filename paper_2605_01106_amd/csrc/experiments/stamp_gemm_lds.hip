// Development aid: timing and in-kernel phase stamps (csrc/trace.h) of the many-row LDS-staged GEMM at the 3B shape
// (576 verification rows, 4096 prefill rows).  Stamps: 0 start, 1 first copies issued, 2 end of the K loop, 3 end.
// Build: hipcc --offload-arch=gfx950 -O3 -std=c++17 -Xclang -target-feature -Xclang -packed-fp32-ops -I../../../include -o stamp_gemm_lds stamp_gemm_lds.hip
#define HH_KERNEL_TRACE 1
#include <stdio.h>
#include <stdlib.h>
#include <vector>
#include <algorithm>
#include "../trace.h"
#include "../skinny_mfma.hip"
#include "../gemm_mfma.hip"
namespace hh { int gemv_max_blocks() { return 1 << 15; } }
using namespace hh;
#define CK(x) do { hipError_t e=(x); if(e!=hipSuccess){printf("ERR %s line %d: %s\n",#x,__LINE__,hipGetErrorString(e)); exit(1);} } while(0)
int main() {
  CK(hipSetDevice(0));
  hipStream_t s; CK(hipStreamCreate(&s));
  hipEvent_t e0, e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
  struct Case { const char* name; int M, K, N, epi, norm; };
  std::vector<Case> cases = {{"c4v in_proj", 576, 2560, 8232, EPI_STORE, 1}, {"c4v out_proj", 576, 2560, 2560, EPI_ADD, 1},
                             {"c4v gate_up", 576, 2560, 6912, EPI_SWIGLU, 1}, {"c4v down", 576, 6912, 2560, EPI_ADD, 0},
                             {"c4p in_proj", 4096, 2560, 8232, EPI_STORE, 1}, {"c4p gate_up", 4096, 2560, 6912, EPI_SWIGLU, 1}, {"c4p down", 4096, 6912, 2560, EPI_ADD, 0}};
  const int L = 6;
  for (auto& c : cases) {
    const size_t pe = packed_weight_elems(c.N, c.K);
    std::vector<uint16_t*> P(L), P2(L);
    for (int l = 0; l < L; ++l) { CK(hipMalloc(&P[l], pe * 2)); CK(hipMalloc(&P2[l], pe * 2)); CK(hipMemset(P[l], 0x3c, pe * 2)); CK(hipMemset(P2[l], 0x3c, pe * 2)); }
    float *X, *Y, *nw, *partial; uint16_t* planes;
    CK(hipMalloc(&X, (size_t)c.M * c.K * 4)); CK(hipMemset(X, 0, (size_t)c.M * c.K * 4));
    CK(hipMalloc(&Y, (size_t)c.M * c.N * 4)); CK(hipMemset(Y, 0, (size_t)c.M * c.N * 4));
    CK(hipMalloc(&nw, c.K * 4)); CK(hipMemset(nw, 0, c.K * 4));
    CK(hipMalloc(&partial, gemm_partial_elems() * 4));
    CK(hipMalloc(&planes, gemm_planes_elems(c.M, c.K) * 2));
    auto run = [&](int it) {
      GemvArgs g{};
      g.X = X; g.ldx = c.K; g.M = c.M; g.K = c.K; g.norm_w = c.norm ? nw : nullptr; g.eps = 1e-5f; g.epi = c.epi; g.bf16 = 1; g.n_seg = 1;
      g.seg[0] = {nullptr, nullptr, P[it % L], P2[it % L], Y, c.N, c.N};
      CK(launch_gemm_mfma(g, planes, partial, s));
    };
    const int iters = 20;
    for (int it = 0; it < 3; ++it) run(it);
    CK(hipEventRecord(e0, s));
    for (int it = 0; it < iters; ++it) run(it);
    CK(hipEventRecord(e1, s)); CK(hipStreamSynchronize(s));
    float ms; CK(hipEventElapsedTime(&ms, e0, e1));
    const double flop = 2.0 * c.M * c.N * c.K * 3 * (c.epi == EPI_SWIGLU ? 2 : 1);
    printf("%-12s M=%d K=%d N=%d : %8.2f us per product (split + GEMM + reduction), %.0f TFLOP/s on the three terms\n", c.name, c.M, c.K, c.N, ms * 1e3 / iters, flop / (ms * 1e-3 / iters) / 1e12);
    std::vector<long long> tr(4096 * 16);
    CK(hipMemcpyFromSymbol(tr.data(), HIP_SYMBOL(g_kernel_trace), tr.size() * 8));
    int nb = 0; long long t0 = 0;
    for (int i = 0; i < 4096; ++i) if (tr[i * 16]) { if (!nb || tr[i * 16] < t0) t0 = tr[i * 16]; nb = i + 1; }
    printf("  %d workgroups stamped\n", nb);
    for (int k = 0; k < 4; ++k) {
      std::vector<double> v;
      for (int i = 0; i < nb; ++i) if (tr[i * 16]) v.push_back((tr[i * 16 + k] - t0) * 0.01);
      std::sort(v.begin(), v.end());
      if (!v.empty()) printf("  stamp %d: min %7.2f median %7.2f max %7.2f us\n", k, v.front(), v[v.size() / 2], v.back());
    }
    { std::vector<long long> z(4096 * 16, 0); CK(hipMemcpyToSymbol(HIP_SYMBOL(g_kernel_trace), z.data(), z.size() * 8)); }
    fflush(stdout);
    for (int l = 0; l < L; ++l) { CK(hipFree(P[l])); CK(hipFree(P2[l])); }
    CK(hipFree(X)); CK(hipFree(Y)); CK(hipFree(nw)); CK(hipFree(partial)); CK(hipFree(planes));
  }
  return 0;
}
