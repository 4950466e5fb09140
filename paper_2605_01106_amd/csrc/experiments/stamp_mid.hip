// Development aid: timing and in-kernel phase stamps (csrc/trace.h) of the 17..96-row matrix-core product at the
// 3B shape with 64 rows (the batched draft step).  Stamps: 0 start, 1 first loads issued, 2 first window staged,
// 3 end of the K loop, 4 sums of squares written, 5 partial products written.
// Build: hipcc --offload-arch=gfx950 -O3 -std=c++17 -Xclang -target-feature -Xclang -packed-fp32-ops -I../../../include -o stamp_mid stamp_mid.hip
#define HH_KERNEL_TRACE 1
#include <stdio.h>
#include <stdlib.h>
#include <vector>
#include "../trace.h"
#include "../skinny_mfma.hip"
#include "../gemm_mfma.hip"
#include "../mid_mfma.hip"
#include <algorithm>
namespace hh { int gemv_max_blocks() { return 1 << 15; } }
using namespace hh;
#define CK(x) do { hipError_t e=(x); if(e!=hipSuccess){printf("ERR %s line %d: %s\n",#x,__LINE__,hipGetErrorString(e)); exit(1);} } while(0)
int main() {
  CK(hipSetDevice(0));
  hipStream_t s; CK(hipStreamCreate(&s));
  hipEvent_t e0, e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
  struct Case { const char* name; int M, K, N, epi, norm; };
  std::vector<Case> cases = {{"c4 in_proj", 64, 2560, 5672, EPI_STORE, 1}, {"c4 out_proj", 64, 2560, 2560, EPI_ADD, 1},
                             {"c4 gate_up", 64, 2560, 6912, EPI_SWIGLU, 1}, {"c4 down", 64, 6912, 2560, EPI_ADD, 0}};
  const int L = 8;
  for (auto& c : cases) {
    const size_t pe = packed_weight_elems(c.N, c.K);
    std::vector<uint16_t*> P(L), P2(L);
    for (int l = 0; l < L; ++l) { CK(hipMalloc(&P[l], pe * 2)); CK(hipMalloc(&P2[l], pe * 2)); CK(hipMemset(P[l], 0x3c, pe * 2)); CK(hipMemset(P2[l], 0x3c, pe * 2)); }
    float *X, *Y, *nw, *partial;
    CK(hipMalloc(&X, (size_t)c.M * c.K * 4)); CK(hipMemset(X, 0, (size_t)c.M * c.K * 4));
    CK(hipMalloc(&Y, (size_t)c.M * c.N * 4)); CK(hipMemset(Y, 0, (size_t)c.M * c.N * 4));
    CK(hipMalloc(&nw, c.K * 4)); CK(hipMemset(nw, 0, c.K * 4));
    CK(hipMalloc(&partial, gemm_partial_elems() * 4));
    auto run = [&](int it) {
      GemvArgs g{};
      g.X = X; g.ldx = c.K; g.M = c.M; g.K = c.K; g.norm_w = c.norm ? nw : nullptr; g.eps = 1e-5f; g.epi = c.epi; g.bf16 = 1; g.n_seg = 1;
      g.seg[0] = {nullptr, nullptr, P[it % L], P2[it % L], Y, c.N, c.N};
      CK(launch_mid_mfma(g, partial, s));
    };
    const int iters = 40;
    for (int it = 0; it < 5; ++it) run(it);
    CK(hipEventRecord(e0, s));
    for (int it = 0; it < iters; ++it) run(it);
    CK(hipEventRecord(e1, s)); CK(hipStreamSynchronize(s));
    float ms; CK(hipEventElapsedTime(&ms, e0, e1));
    printf("%-12s M=%d K=%d N=%d : %7.2f us per product (kernel + reduction)\n", c.name, c.M, c.K, c.N, ms * 1e3 / iters);
    std::vector<long long> tr(4096 * 16);
    CK(hipMemcpyFromSymbol(tr.data(), HIP_SYMBOL(g_kernel_trace), tr.size() * 8));
    MidPlan pl; GemvArgs gg{}; gg.M = c.M; gg.K = c.K; gg.bf16 = 1; gg.n_seg = 1; gg.epi = c.epi; gg.ldx = c.K; gg.seg[0].P = P[0]; gg.seg[0].P2 = P2[0]; gg.seg[0].n_rows = c.N;
    mid_plan(gg, pl);
    const int nb = pl.blocks * pl.windows;
    long long t0 = tr[0];
    for (int i = 0; i < nb; ++i) if (tr[i * 16] && tr[i * 16] < t0) t0 = tr[i * 16];
    printf("  plan: blocks %d x windows %d (wpb %d) = %d workgroups\n", pl.blocks, pl.windows, pl.wpb, nb);
    for (int k = 0; k < 6; ++k) {
      std::vector<double> v;
      for (int i = 0; i < nb && i < 4096; ++i) v.push_back((tr[i * 16 + k] - t0) * 0.01);
      std::sort(v.begin(), v.end());
      printf("  stamp %d: min %6.2f median %6.2f max %6.2f us\n", k, v.front(), v[v.size() / 2], v.back());
    }
    fflush(stdout);
    for (int l = 0; l < L; ++l) { CK(hipFree(P[l])); CK(hipFree(P2[l])); }
    CK(hipFree(X)); CK(hipFree(Y)); CK(hipFree(nw)); CK(hipFree(partial));
  }
  return 0;
}
