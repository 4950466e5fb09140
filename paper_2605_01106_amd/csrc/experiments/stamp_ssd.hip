// Development aid: timing and in-kernel phase stamps (csrc/trace.h) of the matmul-form scan for one prefill pass
// at the 3B shape (64 sequences x 64 positions, 40 heads, N = 256).
// Build: hipcc --offload-arch=gfx950 -O3 -std=c++17 -Xclang -target-feature -Xclang -packed-fp32-ops -I../../../include -o stamp_ssd stamp_ssd.hip
#define HH_KERNEL_TRACE 1
#include <stdio.h>
#include <stdlib.h>
#include <vector>
#include <algorithm>
#include "../trace.h"
#include "../ssd_mfma.hip"
using namespace hh;
#define CK(x) do { hipError_t e=(x); if(e!=hipSuccess){printf("ERR %s line %d: %s\n",#x,__LINE__,hipGetErrorString(e)); exit(1);} } while(0)
int main() {
  CK(hipSetDevice(0));
  hipStream_t s; CK(hipStreamCreate(&s));
  hipEvent_t e0, e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
  Dims d{};
  d.L = 1; d.D = 2560; d.Hm = 40; d.P = 64; d.N = 256; d.d_inner = 2560; d.conv_dim = 2560 + 512; d.d_in_proj = 2 * 2560 + 512 + 40;
  d.ring_w = d.conv_dim + d.Hm; d.ldzx = d.d_in_proj + 1792; d.ring_slots = 128; d.flags = 0;
  const int B = 64, T = 64;
  LayerDev ly{};
  auto dev = [&](size_t n, float fill) { float* p; CK(hipMalloc(&p, n * 4)); std::vector<float> h(n); for (size_t i = 0; i < n; ++i) h[i] = fill * (float)((i * 2654435761u >> 8) & 1023) / 1024.f - fill * 0.5f; CK(hipMemcpy(p, h.data(), n * 4, hipMemcpyHostToDevice)); return p; };
  ly.conv_w = dev((size_t)d.conv_dim * 4, 0.5f); ly.conv_b = dev(d.conv_dim, 0.1f); ly.a_log = dev(d.Hm, 0.5f); ly.d_skip = dev(d.Hm, 1.f); ly.dt_bias = dev(d.Hm, 0.5f);
  ly.S = dev((size_t)B * d.Hm * d.P * d.N, 0.1f); ly.S_draft = nullptr; ly.ring = dev((size_t)B * d.ring_slots * d.ring_w, 0.5f);
  SsmArgs a{};
  a.layers = nullptr; a.one = ly; a.layer0 = 0; a.n_layers_z = 1;
  float* zx = dev((size_t)B * T * d.ldzx, 1.f); float* g = dev((size_t)B * T * d.d_inner, 0.f);
  int* pos0; CK(hipMalloc(&pos0, B * 4)); CK(hipMemset(pos0, 0, B * 4));
  a.zx = zx; a.g = g; a.pos0 = pos0; a.n_tok = nullptr; a.T = T; a.B = B; a.state_in = 0; a.state_out = 1; a.write_ring = 1;
  hipError_t err = hipSuccess;
  for (int it = 0; it < 3; ++it) { if (!launch_ssd_mfma(d, a, s, &err)) { printf("not taken\n"); return 1; } CK(err); }
  CK(hipEventRecord(e0, s));
  const int iters = 10;
  for (int it = 0; it < iters; ++it) { launch_ssd_mfma(d, a, s, &err); CK(err); }
  CK(hipEventRecord(e1, s)); CK(hipStreamSynchronize(s));
  float ms; CK(hipEventElapsedTime(&ms, e0, e1));
  printf("ssd_mfma B=%d T=%d Hm=%d N=%d: %.1f us per launch\n", B, T, d.Hm, d.N, ms * 1e3 / iters);
  std::vector<long long> tr(4096 * 16);
  CK(hipMemcpyFromSymbol(tr.data(), HIP_SYMBOL(g_kernel_trace), tr.size() * 8));
  const int nb = d.Hm / 2 * B;
  // per-workgroup phase durations (stamps are per workgroup; slot 0 = start)
  const char* names[] = {"start->loop", "stage(chunk0)", "G+M", "readout+intra+out", "state update", "rest of chunks", "state store"};
  for (int k = 0; k < 7; ++k) {
    std::vector<double> v;
    for (int i = 0; i < nb && i < 4096; ++i) v.push_back((tr[i * 16 + k + 1] - tr[i * 16 + k]) * 0.01);
    std::sort(v.begin(), v.end());
    printf("  %-20s median %7.2f  p90 %7.2f us\n", names[k], v[v.size() / 2], v[v.size() * 9 / 10]);
  }
  { std::vector<double> v; for (int i = 0; i < nb && i < 4096; ++i) v.push_back((tr[i * 16 + 7] - tr[i * 16]) * 0.01); std::sort(v.begin(), v.end()); printf("  workgroup total      median %7.2f  p90 %7.2f us\n", v[v.size() / 2], v[v.size() * 9 / 10]); }
  return 0;
}
