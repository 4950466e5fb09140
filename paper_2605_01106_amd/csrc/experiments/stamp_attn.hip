// Development aid: timing of the matrix-core attention kernel for one verification pass at the 3B shape
// (64 sequences x 9 positions, 10 query / 2 KV heads of dimension 128, bf16 cache in 64-token pages), with the
// cache of every sequence in pages of its own ("streamed": every key comes from HBM) and with every page-table
// entry pointing at the same few pages ("cached": every key comes from the caches) - the difference tells how
// much of the kernel's time is memory and how much is arithmetic.
// Build: hipcc --offload-arch=gfx950 -O3 -std=c++17 -Xclang -target-feature -Xclang -packed-fp32-ops -I../../../include -o stamp_attn stamp_attn.hip
#include <stdio.h>
#include <stdlib.h>
#include <vector>
#include "../trace.h"
#include "../attn.hip"
#include "../attn_mfma.hip"
using namespace hh;
#define CK(x) do { hipError_t e=(x); if(e!=hipSuccess){printf("ERR %s line %d: %s\n",#x,__LINE__,hipGetErrorString(e)); exit(1);} } while(0)
int main(int argc, char** argv) {
  const int len = argc > 1 ? atoi(argv[1]) : 8192;
  CK(hipSetDevice(0));
  hipStream_t s; CK(hipStreamCreate(&s));
  hipEvent_t e0, e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
  Dims d{};
  d.Hq = 10; d.Hkv = 2; d.Dh = 128; d.dq = 1280; d.dkv = 256; d.dqkv = 1792; d.d_in_proj = 5672; d.ldzx = 5672 + 1792;
  d.page_tokens = 64; d.bf16 = 1; d.flags = 0; d.max_seq = len + 64;
  const int B = 64, T = 9;
  d.pages_per_seq = (d.max_seq + 63) / 64; d.n_pages = d.pages_per_seq * B; d.Bmax = B; d.Tmax = 64;
  const size_t pool = (size_t)d.n_pages * d.Hkv * 64 * d.Dh;   // bf16 elements
  uint16_t *kp, *vp; CK(hipMalloc(&kp, pool * 2)); CK(hipMalloc(&vp, pool * 2));
  CK(hipMemset(kp, 0x3c, pool * 2)); CK(hipMemset(vp, 0x3c, pool * 2));      // finite bf16 values
  std::vector<float> hq((size_t)B * T * d.ldzx);
  for (size_t i = 0; i < hq.size(); ++i) hq[i] = (float)((i * 2654435761u >> 8) & 255) / 256.f - 0.5f;
  float *qkv, *o, *rope, *part_o, *part_ml; int *pos0, *pt, *counters;
  CK(hipMalloc(&qkv, hq.size() * 4)); CK(hipMemcpy(qkv, hq.data(), hq.size() * 4, hipMemcpyHostToDevice));
  CK(hipMalloc(&o, (size_t)B * T * d.dq * 4));
  std::vector<float> hr((size_t)d.max_seq * d.Dh);
  for (int p = 0; p < d.max_seq; ++p) for (int i = 0; i < d.Dh / 2; ++i) { hr[((size_t)p * 64 + i) * 2] = 1.f; hr[((size_t)p * 64 + i) * 2 + 1] = 0.f; }
  CK(hipMalloc(&rope, hr.size() * 4)); CK(hipMemcpy(rope, hr.data(), hr.size() * 4, hipMemcpyHostToDevice));
  CK(hipMalloc(&part_o, (size_t)B * T * d.Hq * 32 * d.Dh * 4)); CK(hipMalloc(&part_ml, (size_t)B * T * d.Hq * 32 * 2 * 4));
  std::vector<int> hp(B, len); CK(hipMalloc(&pos0, B * 4)); CK(hipMemcpy(pos0, hp.data(), B * 4, hipMemcpyHostToDevice));
  CK(hipMalloc(&counters, (size_t)B * d.Hkv * 64 * 4)); CK(hipMemset(counters, 0, (size_t)B * d.Hkv * 64 * 4));
  CK(hipMalloc(&pt, (size_t)B * d.pages_per_seq * 4));
  for (int mode = 0; mode < 2; ++mode) {
    std::vector<int> hpt((size_t)B * d.pages_per_seq);
    for (int b = 0; b < B; ++b) for (int i = 0; i < d.pages_per_seq; ++i) hpt[(size_t)b * d.pages_per_seq + i] = mode == 0 ? b * d.pages_per_seq + i : (b % 4) * 2 + (i & 1);
    CK(hipMemcpy(pt, hpt.data(), hpt.size() * 4, hipMemcpyHostToDevice));
    for (int splits : {1, 2, 4}) {
      AttnArgs a{};
      a.kpool = kp; a.vpool = vp; a.qkv = qkv + d.d_in_proj; a.o = o; a.pos0 = pos0; a.n_tok = nullptr; a.page_table = pt; a.rope = rope;
      a.part_o = part_o; a.part_ml = part_ml; a.counters = counters; a.T = T; a.B = B; a.n_splits = splits;
      for (int it = 0; it < 3; ++it) CK(launch_attention(d, a, s));
      CK(hipEventRecord(e0, s));
      const int iters = 10;
      for (int it = 0; it < iters; ++it) CK(launch_attention(d, a, s));
      CK(hipEventRecord(e1, s)); CK(hipStreamSynchronize(s));
      float ms; CK(hipEventElapsedTime(&ms, e0, e1));
      const double kv = (double)B * len * 2 * d.Hkv * d.Dh * 2;
      printf("%s cache, %5d keys, %d key slices: %8.1f us per launch (%.2f TB/s of KV)\n", mode == 0 ? "streamed" : "cached  ", len, splits, ms * 1e3 / iters, kv / (ms * 1e-3 / iters) / 1e12);
      fflush(stdout);
    }
  }
  return 0;
}
