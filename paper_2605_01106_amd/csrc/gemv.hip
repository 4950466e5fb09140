// Skinny GEMM for the dense projections (in/out/QKV/MLP/LM head) when only a few
// rows of activations meet each weight: Y[m][n] = sum_k X'[m][k] * W[n][k].
//
// The weights are streamed from HBM exactly once per launch, so the kernel is bound by HBM
// bandwidth and, for the small matrices of a batch-1 decode step, by latency.  Hence:
//   * a wavefront owns R output rows and up to 2048 of their columns and issues all of its
//     16-byte weight loads at once, BEFORE it touches the activations; rows longer than
//     that are split between the wavefronts of a workgroup and added through LDS;
//   * many small workgroups (up to 8 wavefronts resident per SIMD) rather than deep software
//     pipelines: measured on MI355X this streams at 5.4-5.8 TB/s;
//   * the activation rows are staged once per workgroup in LDS in float32 and never rounded:
//     a bf16 weight times a float32 activation, accumulated in float32;
//   * RMSNorm is fused as a prologue in one pass: LDS holds x[k] * w[k], and the scalar
//     1 / sqrt(mean(x^2) + eps) multiplies the finished dot product;
//   * epilogues: plain store, in-place residual add (the old value is fetched with the first
//     loads), SwiGLU (gate and up matrices paired row by row: silu(gate) * up), and
//     per-workgroup argmax partials for the LM head (largest value, lowest index on ties).
#include <stdlib.h>

#include "gemv_kernel.h"

namespace hh {

static constexpr int kMaxBlocks = 1 << 15;
static constexpr size_t kLdsBudget = 150 * 1024;

int gemv_max_blocks() { return kMaxBlocks; }

static bool make_plan(const GemvArgs& a, int MT, GemvPlan& p) {
  const int N = a.seg[0].n_rows;
  const int Kpad = (a.K + 511) & ~511;
  const int nch = Kpad >> 9;
  p.MT = MT;
  // column split: each wavefront takes NCW chunks, KS wavefronts per row group
  if (nch <= 2) { p.NCW = 2; p.KS = 1; }
  else if (nch <= 4) { p.NCW = 2; p.KS = 2; }
  else if (nch <= 8) { p.NCW = 2; p.KS = 4; }
  else if (nch <= 16) { p.NCW = 4; p.KS = 4; }
  else return false;
  // rows per wavefront: R * NCW (* 2 for SwiGLU) loads of 16 bytes in flight per lane
  int rmax = 4;
  if (a.epi == EPI_SWIGLU || MT > 5) rmax = 2;
  if (!a.bf16) rmax = 1;
  p.R = rmax;
  const int rgb = kGemvWaves / p.KS;
  // R must divide N; use fewer rows per wavefront while that is needed to cover the CUs
  constexpr int min_blocks = 256;
  while (p.R > 1 && (N % p.R || N / p.R / rgb < min_blocks)) p.R >>= 1;
  const int nrg = N / p.R;
  // several row groups per workgroup, so that staging the activations (MT * K floats per
  // workgroup, from L2) stays small next to the weights it meets
  constexpr int tb1 = 1024, tbm = 1024;
  const int per = (nrg + rgb - 1) / rgb;
  const int target = MT == 1 ? tb1 : tbm;
  p.iters = (per + target - 1) / target;
  if (p.iters < 1) p.iters = 1;
  if (p.iters > 64) p.iters = 64;
  p.blocks = (nrg + rgb * p.iters - 1) / (rgb * p.iters);
  if (p.blocks > kMaxBlocks) return false;
  const int pn = (a.epi == EPI_SWIGLU ? 2 : 1) * p.R * MT;
  p.lds = ((size_t)MT * Kpad + kGemvWaves * MT + 2 * kGemvWaves * pn + 4) * sizeof(float);
  return true;
}

hipError_t launch_gemv(const GemvArgs& a, int* n_blocks_out, hipStream_t s) {
  if (a.K % 8 != 0 || a.K < 8 || a.ldx % 4 != 0 || a.n_seg != 1) return hipErrorInvalidValue;
  if (a.seg[0].n_rows <= 0 || a.M <= 0) return hipSuccess;
  const int Kpad = (a.K + 511) & ~511;
  // largest row tile whose activations fit in LDS
  int mt_cap = 8;
  while (mt_cap > 1 && (size_t)mt_cap * Kpad * 4 + 4096 > kLdsBudget) --mt_cap;
  mt_cap = mt_cap >= 8 ? 8 : mt_cap >= 5 ? 5 : mt_cap >= 3 ? 3 : 1;
  int mt_first = 0;
  for (int m0 = 0; m0 < a.M;) {
    const int left = a.M - m0;
    int mt = left > 5 ? 8 : left > 3 ? 5 : left > 1 ? 3 : 1;
    if (mt > mt_cap) mt = mt_cap;
    // the argmax partials of all row tiles share one layout: keep one launch shape
    if (a.best != nullptr) { if (mt_first == 0) mt_first = mt; mt = mt_first; }
    GemvPlan p;
    if (!make_plan(a, mt, p)) return hipErrorInvalidValue;
    if (n_blocks_out) *n_blocks_out = p.blocks;
    hipError_t e;
    switch (a.epi) {
      case EPI_STORE: e = gemv_dispatch_store(a, m0, p, s); break;
      case EPI_ADD: e = gemv_dispatch_add(a, m0, p, s); break;
      case EPI_SWIGLU: e = gemv_dispatch_swiglu(a, m0, p, s); break;
      default: e = hipErrorInvalidValue;
    }
    if (e != hipSuccess) return e;
    m0 += mt;
  }
  return hipSuccess;
}

}  // namespace hh
