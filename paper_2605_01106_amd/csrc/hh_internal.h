// Internal declarations shared by the translation units of libhh (not installed).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/hh.h"

namespace hh {

// ---- model dimensions derived from hh_cfg
struct Dims {
  int L, D, V;
  int Hm, P, N, d_inner, conv_dim, d_in_proj, ring_w;  // ring_w = conv_dim + Hm (raw xBC inputs | raw dt)
  int Hq, Hkv, Dh, dq, dkv, dqkv;
  int ldzx;         // row stride of the projection buffer: d_in_proj + dqkv (z | xBC | dt | q | k | v)
  int F;
  int ring_slots;   // power of two >= d_conv-1 + max_draft+1 and >= d_conv-1 + prefill chunk
  int page_tokens, pages_per_seq, n_pages;
  int Bmax, Tmax, Gmax, Kmax, max_seq;
  int bf16;         // storage type of matrices and KV
  float eps, rope_base;
  int flags;        // hh_cfg.kernel_flags (HH_KF_* bits)
};

// ---- per-layer device pointers (an array of these lives in the workspace)
struct LayerDev {
  const float *norm1, *conv_w, *conv_b, *a_log, *d_skip, *dt_bias, *gnorm, *norm2;
  const void *w_in, *w_out, *w_q, *w_k, *w_v, *w_o, *w_gate, *w_up, *w_down;
  void* w_inqkv;   // library-owned copy [d_in_proj + dqkv][D]: rows of w_in, w_q, w_k, w_v stacked
  // library-owned copies in the tile layout of the matrix-core kernels (bf16 weights only, else nullptr)
  void *p_inqkv, *p_out, *p_o, *p_gate, *p_up, *p_down;
  float* S;        // committed SSM state of this layer   [B][Hm][P][N]
  float* S_draft;  // draft scratch state                 [B][Hm][P][N]
  float* ring;     // raw conv inputs, ring over positions [B][ring_slots][ring_w]
  void* kpool;     // K pages [n_pages][Hkv][page_tokens][Dh]
  void* vpool;     // V pages
};

// ---- skinny GEMM: Y[m][n] (op)= sum_k norm(X)[m][k] * W[n][k]
enum { EPI_STORE = 0, EPI_ADD = 1, EPI_SWIGLU = 2 };
struct GemvSeg {
  const void* W;    // [n_rows][K]
  const void* W2;   // EPI_SWIGLU: the "up" matrix paired row by row with W (gate)
  const void* P;    // the same matrices in the packed tile layout (nullptr: not available)
  const void* P2;
  float* Y;         // [M][ldy], row n of this segment lands in column n
  int n_rows, ldy;
};
struct GemvArgs {
  const float* X; int ldx; int M; int K;
  const float* X2;                         // optional second addend of the input, same shape as X: X' = X + X2
  const float* R2;                         // EPI_ADD: optional second residual [M][ldy] added with the old Y
  const float* norm_w; float eps;          // rmsnorm prologue when norm_w != nullptr
  GemvSeg seg[4]; int n_seg;
  int epi;
  unsigned long long* best;                // optional per-block argmax partials [M][gridDim.x]
  int bf16;
  int flags;                               // hh_cfg.kernel_flags (HH_KF_* bits)
  int no_store;                            // EPI_STORE with an argmax output: only the argmax is wanted, Y need not be written
  unsigned long long* row_best;            // EPI_STORE, many-row kernels: per-row argmax keys [M] (zeroed by the caller), or nullptr
  // hand-over between two many-row products without a float32 round trip (see gemm_hands_over_planes):
  const uint16_t* planes_in;               // X already split into bf16 planes (X itself is not read)
  uint16_t* planes_out;                    // EPI_SWIGLU: the result goes out as split planes [gemm_planes_elems(M, N)] instead of Y
};
hipError_t launch_gemv(const GemvArgs& a, int* n_blocks_out, hipStream_t s);
int gemv_max_blocks();   // upper bound on gridDim.x of launch_gemv (size of the argmax partial rows)

// ---- the same product for 1..16 activation rows on the matrix cores (bf16 weights; activations split in-kernel)
// (weights in the packed tile layout written by launch_pack_weights; seg[0].W / W2 point to packed copies)
__host__ __device__ size_t packed_weight_elems(int N, int K);
hipError_t launch_pack_weights(const void* W, int N, int K, size_t ldw, void* P, hipStream_t s);
bool skinny_mfma_fits(const GemvArgs& a);
hipError_t launch_skinny_mfma(const GemvArgs& a, float* partial, int* n_blocks_out, hipStream_t s);
// row_best (EPI_STORE only): per-row argmax keys [M], zeroed by the caller, raised with atomic maxima; store = 0: Y is not written
hipError_t launch_gemm_reduce(int epi, float* partial, int ksplit, int M, int N, float* Y, int ldy, const float* R2,
                              const float* ssq, int ssq_ld, float rnorm_k, float eps, unsigned long long* row_best, int store,
                              hipStream_t s);

// ---- the same product for 17..96 activation rows on the matrix cores (bf16 weights from seg[0].P / P2,
// activations split in-kernel per K window; partial: scratch of gemm_partial_elems() floats)
bool mid_mfma_fits(const GemvArgs& a);
hipError_t launch_mid_mfma(const GemvArgs& a, float* partial, hipStream_t s);

// ---- the same product on the matrix cores (bf16 weights, more than a few activation rows)
size_t gemm_planes_elems(int M, int K);   // bf16 elements of scratch for the split activations
size_t gemm_partial_elems();              // float elements of scratch for split-K partial products
hipError_t launch_gemm_mfma(const GemvArgs& a, uint16_t* planes, float* partial, hipStream_t s);
// whether launch_gemm_mfma honours a.planes_out for these arguments (SwiGLU product through the LDS-staged
// kernel without a K split, result columns a multiple of 32): the caller then passes the same buffer as
// planes_in of the product that consumes the result
bool gemm_hands_over_planes(const GemvArgs& a);

// ---- SSM branch: causal conv + selective scan over up to T positions per sequence
struct SsmArgs {
  const LayerDev* layers; int layer0; int n_layers_z;  // blockIdx.z = (layer - layer0) * B + b
  LayerDev one;        // used instead of the table when layers == nullptr (single-layer launch)
  const float* zx;     // [B*T][ldzx] projections of this pass (nullptr: inputs come from the ring only)
  float* g;            // [B*T][d_inner]  y * silu(z)  (nullptr: no output)
  const int* pos0;     // [B] position of the first token of this pass
  const int* n_tok;    // [B] valid positions (<= T); nullptr: T for all
  const int* n_acc;    // [B] rebuild mode: positions = n_acc[b] + 1
  const int* skip;     // [B] nonzero: leave this sequence untouched (may be nullptr)
  int T, B;
  int state_in, state_out;   // in: 0 committed S, 1 S_draft, 2 zeros.  out: 0 none, 1 S, 2 S_draft
  int write_ring;
};
hipError_t launch_ssm(const Dims& d, const SsmArgs& a, hipStream_t s);
// matmul-form kernel for passes with many positions (ssd_mfma.hip); true if it took the pass
bool launch_ssd_mfma(const Dims& d, const SsmArgs& a, hipStream_t s, hipError_t* err);

// ---- attention branch
struct AttnArgs {
  void* kpool; void* vpool;  // this layer's K and V pages
  const float* qkv;       // [B*T][ldzx] (offset to the q column): raw q | k | v of this pass
  float* o;               // [B*T][dq]
  const int* pos0; const int* n_tok; const int* page_table;  // [B], [B], [B][pages_per_seq]
  const float* rope;      // [max_seq][Dh/2][2] (cos, sin)
  float* part_o; float* part_ml;  // split scratch: [B*T*Hq][S][Dh], [B*T*Hq][S][2]
  int* counters;          // [B][Hkv][row chunks], zero between launches: tickets of the key slices
  int T, B, n_splits;
};
int attention_row_chunks(const Dims& d, int T);
hipError_t launch_attention(const Dims& d, const AttnArgs& a, hipStream_t s);
bool attention_uses_mfma(const Dims& d);
int attention_mfma_row_chunks(const Dims& d, int T);
bool attention_mfma_fuses_append(const Dims& d, int T);
// bf16 cache, new keys already appended: the matrix-core kernel alone
hipError_t launch_attention_mfma(const Dims& d, const AttnArgs& a, hipStream_t s);

// ---- small kernels
hipError_t launch_embed(const Dims& d, const void* embed, const int* tok, int M, float* h, hipStream_t s);
// tokens of one draft step: step 0 reads pending[b], step i reads drafts[b][i-1]
hipError_t launch_gather_tokens(const int* pending, const int* drafts, int kmax, int B, int T, int mode,
                                int step, int* tok, const int* kv_len, int* pos0, hipStream_t s);
hipError_t launch_argmax_finish(const unsigned long long* best, int n_part, int M, int* out, int out_stride,
                                int out_off, int T, hipStream_t s);
struct CommitArgs {
  const int* drafts; const int* targets; const int* forced;  // [B][kmax], [B][kmax+1], [B] or nullptr
  int *committed, *last_n, *pending, *out_tok, *n_acc, *skip, *adv;
  unsigned long long* acc_stats;   // [2] running sums over rounds and active sequences: accepted drafts, tested drafts
  int B, k, kmax, G, out_stride;
};
hipError_t launch_accept(const CommitArgs& a, hipStream_t s);
hipError_t launch_advance(int* kv_len, const int* n, int B, hipStream_t s);
hipError_t launch_gather_prompt(const int* prompt, int row_stride, int off, const int* n_tok, int B, int T, int* tok,
                                const int* kv_len, int* pos0, hipStream_t s);
hipError_t launch_prefill_tail(const float* h, int T, int D, const int* n_tok, const int* is_last, float* lasth,
                               int* kv_len, int B, hipStream_t s);
hipError_t launch_prefill_finish(const int* first_tok, int* pending, int* out_tok, int out_stride, int* committed,
                                 int* last_n, int B, hipStream_t s);
// ---- token choice at temperature > 0 (rejection test of the round and its draws)
struct SamplingParams { float inv_t; uint32_t pad; uint64_t seed; };   // lives in device memory
// one row per sequence b at logits + b * row_stride -> out[b * out_stride + out_off];
// stream position of the drawn token: (idx_base ? idx_base[b] : 0) + idx_off.
// Parameters: *prm (device memory) when prm != nullptr, else prm_val.
hipError_t launch_sample_rows(const float* logits, size_t row_stride, int V, int B, const SamplingParams* prm,
                              SamplingParams prm_val, const int* idx_base, int idx_off, int purpose, int* out,
                              int out_stride, int out_off, hipStream_t s);
// logits_d [B][kmax][V], logits_v [B][k+1][V], stats: scratch of B * (2 * kmax + 1) * 2 floats
hipError_t launch_spec_targets(const float* logits_d, const float* logits_v, int V, int B, int k, int kmax,
                               const SamplingParams* prm, SamplingParams prm_val, float* stats, const int* drafts,
                               const int* committed, int* targets, hipStream_t s);
// device address and size of the current GPU's file-scope statistics array (no allocation)
hipError_t static_accept_scratch(float** ptr, size_t* n_floats);
hipError_t launch_fill_i32(int* p, int v, size_t n, hipStream_t s);
hipError_t launch_fill_f32(float* p, float v, size_t n, hipStream_t s);
hipError_t launch_export_state(const Dims& d, const LayerDev* layer, const int* kv_len, int B, float* conv_out,
                               hipStream_t s);
hipError_t launch_export_kv(const Dims& d, const LayerDev* layer, const int* page_table, int seq, int tok0,
                            int n_tokens, float* k, float* v, hipStream_t s);

}  // namespace hh
