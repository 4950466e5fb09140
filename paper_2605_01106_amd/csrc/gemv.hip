// Skinny GEMM for the dense projections (in/out/QKV/MLP/LM head) when only a few
// rows of activations meet each weight: Y[m][n] = sum_k X'[m][k] * W[n][k].
//
// The weights are streamed from HBM exactly once per launch, so the kernel is bound by HBM
// bandwidth and, for the small matrices of a batch-1 decode step, by latency.  Hence:
//   * a wavefront walks "units" of R output rows x G chunks of 512 columns and issues the
//     16-byte loads of unit u+1 before the arithmetic of unit u; the first unit is issued
//     BEFORE the activations are touched, so the HBM round trip overlaps the prologue;
//   * the grid is at most two workgroups per CU; a wavefront loops over its row groups, so
//     big matrices (LM head) pay the prologue once and keep the load pipeline full;
//   * wavefronts are independent: each lane loads its own eight activation columns per chunk
//     from global memory (L1/L2 hits) together with the weights, in float32, never rounded:
//     a bf16 weight times a float32 activation, accumulated in float32.  No LDS, no barrier;
//   * RMSNorm is fused: every wavefront sums the squares of the activation row itself, the
//     norm weight multiplies the activations as they are used, and the scalar
//     1 / sqrt(mean(x^2) + eps) multiplies the finished dot product;
//   * epilogues: plain store, in-place residual add (the old value is fetched with the first
//     loads), SwiGLU (gate and up matrices paired row by row: silu(gate) * up), and
//     per-workgroup argmax partials for the LM head (largest value, lowest index on ties).
#include "gemv_kernel.h"

namespace hh {

static constexpr int kMaxBlocks = 512;   // two workgroups per CU

int gemv_max_blocks() { return kMaxBlocks; }

static GemvPlan make_plan(const GemvArgs& a, int n_total, int MT) {
  GemvPlan p;
  const int nch = (a.K + 511) >> 9;
  p.MT = MT;
  p.G = nch <= 2 ? 2 : 4;
  // registers per lane: weights 2 buffers * R * G * 4 (bf16; 8 for float32), activations
  // 2 buffers * MT * G * 8.  Keep the sum near 200.
  if (MT >= 3) p.G = 2;
  int rmax = 8 / p.G;
  if (a.epi == EPI_SWIGLU) rmax /= 2;
  if (!a.bf16) rmax = a.epi == EPI_SWIGLU ? 1 : (rmax > 2 ? 2 : rmax);
  if (!a.bf16 && p.G == 4) rmax = 1;
  if (MT >= 3 && rmax > 2) rmax = 2;
  if (rmax < 1) rmax = 1;
  // fewer rows per wavefront while that is needed to give every CU a workgroup
  p.R = rmax;
  while (p.R > 1 && (n_total + p.R - 1) / p.R < 256 * kGemvWaves) p.R >>= 1;
  const int nrg = (n_total + p.R - 1) / p.R;
  p.blocks = (nrg + kGemvWaves - 1) / kGemvWaves;
  if (p.blocks > kMaxBlocks) p.blocks = kMaxBlocks;
  return p;
}

hipError_t launch_gemv(const GemvArgs& a, int* n_blocks_out, hipStream_t s) {
  if (a.K % 8 != 0 || a.ldx % 4 != 0) return hipErrorInvalidValue;
  int n_total = 0;
  for (int i = 0; i < a.n_seg; ++i) n_total += a.seg[i].n_rows;
  if (n_total <= 0 || a.M <= 0) return hipSuccess;
  for (int m0 = 0; m0 < a.M;) {
    const int left = a.M - m0;
    const int mt = left > 5 ? 4 : left;
    const GemvPlan p = make_plan(a, n_total, mt);
    if (n_blocks_out) *n_blocks_out = p.blocks;
    hipError_t e;
    switch (a.epi) {
      case EPI_STORE: e = gemv_dispatch_store(a, m0, n_total, p, s); break;
      case EPI_ADD: e = gemv_dispatch_add(a, m0, n_total, p, s); break;
      case EPI_SWIGLU: e = gemv_dispatch_swiglu(a, m0, n_total, p, s); break;
      default: e = hipErrorInvalidValue;
    }
    if (e != hipSuccess) return e;
    m0 += mt;
  }
  return hipSuccess;
}

}  // namespace hh
