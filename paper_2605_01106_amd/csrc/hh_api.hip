// C ABI of libhh: context, workspace carving, the round state machine and the per-layer
// kernel schedules of the two forward modes -- the full hybrid M_H (Eq. 2 of the paper: SSM
// branch + attention branch summed) and the SSM-only draft M_S (Eq. 4: the attention branch
// is simply not launched).  Host code only enqueues; every value a round depends on (tokens,
// lengths, accepted counts) stays in device memory.
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <algorithm>
#include <map>
#include <string>
#include <vector>

#include "hh_internal.h"

using namespace hh;

namespace {

enum Phase { PH_CREATED = 0, PH_READY = 1, PH_DRAFTED = 2, PH_VERIFIED = 3 };

constexpr int kMaxSplits = 32;
constexpr size_t kProfCap = 1 << 15;   // timed launches kept per profiling session
constexpr size_t kAlign = 256;

std::string g_create_error;

constexpr size_t kCanaryBytes = 256;
constexpr int kCanaryByte = 0xA5;

struct Carver {
  char* base;
  size_t off = 0;
  bool canaries = false;               // HH_KF_CANARIES: every region is followed by kCanaryBytes of guard bytes
  std::vector<size_t>* marks = nullptr;   // their offsets (recorded when carving for real)
  template <typename T>
  T* take(size_t n) {
    off = (off + kAlign - 1) / kAlign * kAlign;
    T* p = base ? reinterpret_cast<T*>(base + off) : nullptr;
    off += n * sizeof(T);
    if (canaries) {
      off = (off + kAlign - 1) / kAlign * kAlign;
      if (base && marks) marks->push_back(off);
      off += kCanaryBytes;
    }
    return p;
  }
};

}  // namespace

struct hh_ctx {
  hh_cfg cfg;
  Dims d;
  const void *embed, *final_norm, *lm_head;
  std::vector<LayerDev> layers_host;
  LayerDev* layers_dev;
  // strict draft state (cfg.draft_state_mode = 1): the same layers with M_S's own committed
  // recurrent state and ring of raw convolution inputs in place of the full model's
  std::vector<LayerDev> layers_ms_host;
  LayerDev* layers_ms_dev = nullptr;
  bool strict = false;
  std::vector<int> draft_modes;   // per layer HH_DRAFT_*; empty: every layer SSM-only (Eq. 4)
  std::vector<size_t> canaries;   // offsets of the guard bytes behind every workspace region (HH_KF_CANARIES)
  bool draft_has_full = false;
  // device int state
  int *kv_len, *committed, *last_n, *pending, *n_acc, *skip, *adv, *drafts, *targets, *tok, *pos0, *out_tok,
      *page_table, *plan_ntok, *plan_last, *first_tok;
  unsigned long long* best;
  unsigned long long* acc_stats;   // accepted / tested drafts since the last prefill
  SamplingParams* sampling;   // temperature and seed read by the drawing kernels
  float* softmax_stats;       // (max, sum) of the round's logit rows
  float temperature = 0.f;    // 0: greedy
  int* attn_counters;   // tickets of the attention key slices (zero between launches)
  uint16_t* planes;   // split activations of the matrix-core products
  float* gemm_partial;   // partial products of split-K launches
  uint16_t* planes_side; // the same two scratch areas for products enqueued on the side stream
  uint16_t* planes_act;  // SwiGLU result of a many-row pass, handed to the down projection as split planes
  float* gemm_partial_side;
  float* ho;             // [Mmax][D] attention branch after its output projection (full mode)
  float *rope, *h, *zx, *qkv, *g, *o, *act, *logits_d, *logits_v, *logits_p, *lasth, *part_o, *part_ml, *export_buf;
  int max_passes;
  // host state
  int phase = PH_CREATED;
  int B = 0, G = 0, k = 0;
  int len_upper = 0;
  std::vector<int> h_page_table, h_plan;
  std::string err;
  // optional per-launch timing (hh_profile): event pairs tagged phase*16 + kind
  bool prof_on = false;
  void* p_lm_head = nullptr;   // LM head in the packed tile layout (bf16 weights)
  int only_kind = -1;   // hh_time_kind: launch only this kind of kernel
  int prof_phase = 0;
  std::vector<hipEvent_t> prof_ev;
  std::vector<int> prof_tag;
  // captured launch sequences of draft and verify, by (kind, batch, k, key splits); a key is run
  // eagerly on its first use (which also sets kernel attributes), captured on its second
  // side stream on which the attention branch of a block runs beside its SSM branch
  hipStream_t side = nullptr;
  std::vector<hipEvent_t> fork_ev, join_ev;   // one pair per layer
  struct GraphSlot { hipGraphExec_t exec = nullptr; int uses = 0; };
  std::map<long long, GraphSlot> graphs;
  ~hh_ctx() {
    for (hipEvent_t e : prof_ev) (void)hipEventDestroy(e);
    for (auto& kv : graphs)
      if (kv.second.exec) (void)hipGraphExecDestroy(kv.second.exec);
    for (hipEvent_t e : fork_ev) (void)hipEventDestroy(e);
    for (hipEvent_t e : join_ev) (void)hipEventDestroy(e);
    if (side) (void)hipStreamDestroy(side);
  }
};

namespace {

// Prompt positions per sequence per prefill pass.  Default: about 4096 activation rows per pass
// over the whole batch (enough rows for the tiled matrix-core GEMM and few passes over the
// weights), in multiples of 64, between 64 and 512.
int prefill_chunk_of(const hh_cfg& c) {
  if (c.prefill_chunk != 0) return c.prefill_chunk;
  const int rows = 4096 / (c.max_batch > 0 ? c.max_batch : 1);
  const int chunk = rows / 64 * 64;
  return chunk < 64 ? 64 : (chunk > 512 ? 512 : chunk);
}

bool derive_dims(const hh_cfg& c, Dims& d, std::string& why) {
  auto bad = [&](const char* m) { why = m; return false; };
  if (c.struct_size != sizeof(hh_cfg)) return bad("struct_size does not match this library's hh_cfg");
  if (c.n_layers < 1 || c.d_model < 8 || c.vocab < 2) return bad("n_layers/d_model/vocab out of range");
  if (c.m_heads < 1 || c.m_head_dim < 1 || c.d_state < 8) return bad("m_heads/m_head_dim/d_state out of range");
  if (c.n_groups != 1) return bad("n_groups must be 1");
  if (c.d_conv != 4) return bad("d_conv must be 4");
  if (c.n_q_heads < 1 || c.n_kv_heads < 1 || c.n_q_heads % c.n_kv_heads != 0) return bad("n_q_heads must be a multiple of n_kv_heads");
  if (c.head_dim < 8 || c.head_dim % 8 != 0 || c.head_dim > 256) return bad("head_dim must be a multiple of 8 in 8..256");
  if (c.w_dtype != HH_F32 && c.w_dtype != HH_BF16) return bad("unknown w_dtype");
  const int ns = c.d_state / 8;
  if (c.d_state % 8 != 0 || (ns & (ns - 1)) != 0 || ns > 32) return bad("d_state must be 8, 16, 32, 64, 128 or 256");
  if (c.max_batch < 1 || c.max_draft < 0 || c.max_new_tokens < 1 || c.max_seq_len < 2) return bad("capacities out of range");
  if (!(c.rms_eps > 0.f) || !(c.rope_base > 1.f)) return bad("rms_eps / rope_base out of range");
  d.L = c.n_layers; d.D = c.d_model; d.V = c.vocab;
  d.Hm = c.m_heads; d.P = c.m_head_dim; d.N = c.d_state;
  d.d_inner = d.Hm * d.P; d.conv_dim = d.d_inner + 2 * d.N; d.d_in_proj = 2 * d.d_inner + 2 * d.N + d.Hm;
  d.ring_w = d.conv_dim + d.Hm;
  d.Hq = c.n_q_heads; d.Hkv = c.n_kv_heads; d.Dh = c.head_dim;
  d.dq = d.Hq * d.Dh; d.dkv = d.Hkv * d.Dh; d.dqkv = d.dq + 2 * d.dkv;
  d.ldzx = d.d_in_proj + d.dqkv;
  d.F = c.d_ff;
  if (d.D % 8 || d.d_inner % 8 || d.dq % 8 || d.F % 8 || d.F < 8) return bad("d_model, d_inner, n_q_heads*head_dim and d_ff must be multiples of 8");
  if (d.D > 8192 || d.d_inner > 8192 || d.dq > 8192 || d.F > 8192) return bad("d_model, d_inner, n_q_heads*head_dim and d_ff must not exceed 8192");
  d.page_tokens = c.kv_page_tokens == 0 ? 64 : c.kv_page_tokens;
  if (d.page_tokens != 16 && d.page_tokens != 32 && d.page_tokens != 64 && d.page_tokens != 128 && d.page_tokens != 256)
    return bad("kv_page_tokens must be 16, 32, 64, 128 or 256");
  const int chunk = prefill_chunk_of(c);
  if (chunk < 1 || chunk > 1024) return bad("prefill_chunk must be in 1..1024");
  d.Kmax = c.max_draft; d.Bmax = c.max_batch; d.Gmax = c.max_new_tokens; d.max_seq = c.max_seq_len;
  d.Tmax = d.Kmax + 1 > chunk ? d.Kmax + 1 : chunk;
  d.ring_slots = 4;
  while (d.ring_slots < d.Tmax + 3) d.ring_slots <<= 1;
  d.pages_per_seq = (d.max_seq + d.page_tokens - 1) / d.page_tokens;
  d.n_pages = d.pages_per_seq * d.Bmax;
  d.bf16 = c.w_dtype == HH_BF16;
  d.eps = c.rms_eps; d.rope_base = c.rope_base;
  if (c.overlap_mode < 0 || c.overlap_mode > 3) return bad("overlap_mode must be in 0..3");
  if (c.attn_max_splits < 0 || c.attn_max_splits > kMaxSplits) return bad("attn_max_splits must be in 0..32");
  if (c.attn_target_blocks != 0 && (c.attn_target_blocks < 64 || c.attn_target_blocks > 8192)) return bad("attn_target_blocks must be 0 or in 64..8192");
  if (c.attn_single_slice_steps < -1) return bad("attn_single_slice_steps must be -1, 0 or a step count");
  if (c.kernel_flags & ~(HH_KF_ATTN_SCALAR | HH_KF_SSM_GENERAL | HH_KF_MID_OFF | HH_KF_SKINNY_OFF | HH_KF_SSM_SCALAR_CONV | HH_KF_ROWS_LDS | HH_KF_SSM_SEQUENTIAL | HH_KF_NO_HANDOVER | HH_KF_CANARIES | HH_KF_SSM_MATMUL | HH_KF_MID_WIDE))
    return bad("unknown bit in kernel_flags");
  if (c.prefill_progress < 0) return bad("prefill_progress must not be negative");
  if (c.draft_state_mode != 0 && c.draft_state_mode != 1) return bad("draft_state_mode must be 0 (shared) or 1 (strict)");
  if (c.keep_logits != 0 && c.keep_logits != 1) return bad("keep_logits must be 0 or 1");
  if (c.use_graphs != 0 && c.use_graphs != 1) return bad("use_graphs must be 0 or 1");
  d.flags = c.kernel_flags;
  return true;
}

// Assigns (or, with base == nullptr, only sizes) every region of the workspace.
size_t carve(hh_ctx* x, char* base) {
  const Dims& d = x->d;
  Carver c{base};
  c.canaries = (x->cfg.kernel_flags & HH_KF_CANARIES) != 0;
  if (base) { x->canaries.clear(); c.marks = &x->canaries; }
  const size_t B = d.Bmax, Mmax = B * d.Tmax, Mv = B * (d.Kmax + 1);
  const size_t esz = d.bf16 ? 2 : 4;
  x->layers_dev = c.take<LayerDev>(d.L);
  const bool strict = x->cfg.draft_state_mode == 1;
  x->layers_ms_dev = strict ? c.take<LayerDev>(d.L) : nullptr;
  x->kv_len = c.take<int>(B); x->committed = c.take<int>(B); x->last_n = c.take<int>(B);
  x->pending = c.take<int>(B); x->n_acc = c.take<int>(B); x->skip = c.take<int>(B); x->adv = c.take<int>(B);
  x->first_tok = c.take<int>(B);
  x->drafts = c.take<int>(B * (d.Kmax > 0 ? d.Kmax : 1));
  x->targets = c.take<int>(B * (d.Kmax + 1));
  x->tok = c.take<int>(Mmax); x->pos0 = c.take<int>(B);
  x->out_tok = c.take<int>(B * d.Gmax);
  x->page_table = c.take<int>(B * d.pages_per_seq);
  const int chunk = prefill_chunk_of(x->cfg);
  x->max_passes = (d.max_seq + chunk - 1) / chunk;
  x->plan_ntok = c.take<int>((size_t)x->max_passes * B);
  x->plan_last = c.take<int>((size_t)x->max_passes * B);
  x->best = c.take<unsigned long long>(Mv * gemv_max_blocks());
  x->acc_stats = c.take<unsigned long long>(2);
  x->sampling = c.take<SamplingParams>(1);
  x->softmax_stats = c.take<float>(B * (2 * d.Kmax + 1) * 2);
  x->attn_counters = c.take<int>(B * d.Hkv * attention_row_chunks(d, d.Tmax));
  {
    int kmax = d.D > d.d_inner ? d.D : d.d_inner;
    if (d.dq > kmax) kmax = d.dq;
    if (d.F > kmax) kmax = d.F;
    x->planes = c.take<uint16_t>(gemm_planes_elems((int)Mmax, kmax));
    x->gemm_partial = d.bf16 ? c.take<float>(gemm_partial_elems()) : nullptr;
    x->planes_side = c.take<uint16_t>(gemm_planes_elems((int)Mmax, kmax));
    x->planes_act = d.bf16 && Mmax > 16 ? c.take<uint16_t>(gemm_planes_elems((int)Mmax, d.F)) : nullptr;
    x->gemm_partial_side = d.bf16 ? c.take<float>(gemm_partial_elems()) : nullptr;
  }
  x->rope = c.take<float>((size_t)d.max_seq * d.Dh);
  x->h = c.take<float>(Mmax * d.D);
  x->zx = c.take<float>(Mmax * d.ldzx);
  x->qkv = x->zx ? x->zx + d.d_in_proj : nullptr;
  x->g = c.take<float>(Mmax * d.d_inner);
  x->o = c.take<float>(Mmax * d.dq);
  x->ho = c.take<float>(Mmax * d.D);
  x->act = c.take<float>(Mmax * d.F);
  x->logits_d = c.take<float>(B * (d.Kmax > 0 ? d.Kmax : 1) * d.V);
  x->logits_v = c.take<float>(Mv * d.V);
  x->logits_p = c.take<float>(B * d.V);
  x->lasth = c.take<float>(B * d.D);
  x->part_o = c.take<float>(Mv * d.Hq * kMaxSplits * d.Dh);
  x->part_ml = c.take<float>(Mv * d.Hq * kMaxSplits * 2);
  x->export_buf = c.take<float>(B * d.conv_dim * 3);
  const size_t state = B * d.Hm * d.P * d.N;
  const size_t ring = B * d.ring_slots * d.ring_w;
  const size_t pool = (size_t)d.n_pages * d.Hkv * d.page_tokens * d.Dh * esz;
  if (base) x->layers_host.resize(d.L);
  if (base && strict) x->layers_ms_host.resize(d.L);
  for (int l = 0; l < d.L; ++l) {
    float* S = c.take<float>(state);
    float* Sd = c.take<float>(state);
    float* rg = c.take<float>(ring);
    float* S_ms = strict ? c.take<float>(state) : nullptr;
    float* rg_ms = strict ? c.take<float>(ring) : nullptr;
    char* kp = c.take<char>(pool);
    char* vp = c.take<char>(pool);
    char* wf = c.take<char>((size_t)d.ldzx * d.D * esz);
    uint16_t *pi = nullptr, *po = nullptr, *poo = nullptr, *pg = nullptr, *pu = nullptr, *pd = nullptr;
    if (d.bf16) {
      pi = c.take<uint16_t>(packed_weight_elems(d.ldzx, d.D));
      po = c.take<uint16_t>(packed_weight_elems(d.D, d.d_inner));
      poo = c.take<uint16_t>(packed_weight_elems(d.D, d.dq));
      pg = c.take<uint16_t>(packed_weight_elems(d.F, d.D));
      pu = c.take<uint16_t>(packed_weight_elems(d.F, d.D));
      pd = c.take<uint16_t>(packed_weight_elems(d.D, d.F));
    }
    if (base) {
      LayerDev& ld = x->layers_host[l];
      ld.S = S; ld.S_draft = Sd; ld.ring = rg; ld.kpool = kp; ld.vpool = vp; ld.w_inqkv = wf;
      ld.p_inqkv = pi; ld.p_out = po; ld.p_o = poo; ld.p_gate = pg; ld.p_up = pu; ld.p_down = pd;
      if (strict) {   // completed in hh_create, once the weight pointers are in place
        x->layers_ms_host[l].S = S_ms;
        x->layers_ms_host[l].ring = rg_ms;
      }
    }
  }
  x->p_lm_head = d.bf16 ? c.take<uint16_t>(packed_weight_elems(d.V, d.D)) : nullptr;
  return (c.off + kAlign - 1) / kAlign * kAlign;
}

hh_status fail(hh_ctx* x, hh_status st, const std::string& msg) {
  if (x) x->err = msg; else g_create_error = msg;
  return st;
}

#define HH_HIP(call)                                                                           \
  do {                                                                                         \
    hipError_t e_ = (call);                                                                    \
    if (e_ != hipSuccess)                                                                      \
      return fail(x, HH_EDEVICE, std::string(#call) + ": " + hipGetErrorString(e_));           \
  } while (0)

// Launch `call`, bracketed by an event pair when profiling is on.
#define HH_LAUNCH(kind, call)                                                                  \
  do {                                                                                         \
    if (x->only_kind >= 0 && x->only_kind != (kind)) break;                                    \
    const bool p_ = x->prof_on && x->prof_ev.size() < kProfCap * 2;                            \
    if (p_) {                                                                                  \
      hipEvent_t a_, b_;                                                                       \
      HH_HIP(hipEventCreate(&a_)); x->prof_ev.push_back(a_);                                   \
      HH_HIP(hipEventCreate(&b_)); x->prof_ev.push_back(b_);                                   \
      x->prof_tag.push_back(x->prof_phase * 16 + (kind));                                      \
      HH_HIP(hipEventRecord(a_, s));                                                           \
    }                                                                                          \
    HH_HIP(call);                                                                              \
    if (p_) HH_HIP(hipEventRecord(x->prof_ev.back(), s));                                      \
  } while (0)

// One dense projection with bf16 weights: the weight-streaming FMA kernel for up to 3 activation
// rows, the matrix-core kernel with in-kernel activation split for 4..16 rows where it fits, the
// matrix-core GEMM over pre-split activations for 9 rows and more otherwise.  float32 weights:
// the FMA kernel.
constexpr int kMfmaMinRows = 9;
constexpr int kSkinnyMinRows = 4;
// the arguments with the packed weights in place of the row-major ones, if this product can take the skinny kernel
bool skinny_args(const GemvArgs& a, GemvArgs& b) {
  if (!a.bf16 || (a.flags & HH_KF_SKINNY_OFF) || a.M < kSkinnyMinRows || a.M > 16 || a.seg[0].P == nullptr) return false;
  b = a;
  b.seg[0].W = a.seg[0].P; b.seg[0].W2 = a.seg[0].P2;
  return skinny_mfma_fits(b);
}
// side: the product is enqueued on the side stream (its own scratch, so that it may overlap a product on the main stream)
hipError_t product(hh_ctx* x, const GemvArgs& a, hipStream_t s, bool side = false) {
  GemvArgs b;
  if (a.planes_in != nullptr || a.planes_out != nullptr)   // hand-over between two many-row products
    return launch_gemm_mfma(a, side ? x->planes_side : x->planes, side ? x->gemm_partial_side : x->gemm_partial, s);
  if (skinny_args(a, b)) return launch_skinny_mfma(b, side ? x->gemm_partial_side : x->gemm_partial, nullptr, s);
  if (mid_mfma_fits(a)) return launch_mid_mfma(a, side ? x->gemm_partial_side : x->gemm_partial, s);
  if (a.bf16 && a.M >= kMfmaMinRows && a.seg[0].P != nullptr)
    return launch_gemm_mfma(a, side ? x->planes_side : x->planes, side ? x->gemm_partial_side : x->gemm_partial, s);
  return launch_gemv(a, nullptr, s);
}

// Whether a full pass runs its attention branch on the side stream beside the SSM branch.
// Prefill passes do (both branches are long there).  A verification pass does not unless asked:
// what can overlap is the shorter branch (scan + out projection: 130 us of 900 us per layer at the 3B
// shape with 32k-token caches), both branches are bound by the same HBM bandwidth, and a forked
// graph makes every launch of the following single-stream draft graphs about 0.9 us longer;
// measured at that workload the pass takes 30.1 ms without the fork and 30.4 ms with it.
// cfg.overlap_mode: 0 automatic (= 2), 1 never, 2 prefill passes only, 3 always.
bool branch_overlap(const hh_ctx* x, int B, int T, bool prefill) {
  (void)B; (void)T;
  const int mode = x->cfg.overlap_mode;
  if (mode == 1) return false;
  if (mode == 3) return true;
  return prefill;
}

// ---- one pass of the block stack over M = B*T rows.  all_full: M_H (both branches of every
// block, Eq. 2); otherwise M_S (Eq. 4), or, with `modes` (one HH_DRAFT_* per layer), the draft
// model in which a layer keeps both branches, only its SSM branch, or is passed over whole
// (identity on the residual stream, Eq. 5 applied to the block).  table: the layers with the
// recurrent state and ring this pass works on.
hh_status run_layers(hh_ctx* x, const std::vector<LayerDev>& table, bool all_full, const int* modes, int B, int T,
                     const int* n_tok, int state_in, int state_out, int n_splits, bool prefill, hipStream_t s) {
  const Dims& d = x->d;
  const int M = B * T;
  for (int l = 0; l < d.L; ++l) {
    const int mode = all_full ? HH_DRAFT_FULL : (modes ? modes[l] : HH_DRAFT_SSM);
    if (mode == HH_DRAFT_SKIP) continue;
    const bool full = mode == HH_DRAFT_FULL;
    const LayerDev& w = table[l];
    {  // shared input norm, Mamba-2 input projection (+ q, k, v of the attention branch)
      GemvArgs a{};
      a.X = x->h; a.ldx = d.D; a.M = M; a.K = d.D; a.norm_w = w.norm1; a.eps = d.eps; a.epi = EPI_STORE; a.bf16 = d.bf16; a.flags = d.flags;
      a.seg[0] = {w.w_inqkv, nullptr, w.p_inqkv, nullptr, x->zx, full ? d.ldzx : d.d_in_proj, d.ldzx};
      a.n_seg = 1;
      HH_LAUNCH(HH_K_IN_PROJ, product(x, a, s));
    }
    // The two branches of the block (Eq. 2) only share their input.  The attention branch
    // (attention, then its output projection into a buffer of its own) is enqueued on a side
    // stream beside the SSM branch (scan, then out projection into the residual stream); the
    // branches meet at the MLP, whose input is h + ho and whose down projection adds both.
    const bool overlap = full && !x->prof_on && x->side != nullptr && branch_overlap(x, B, T, prefill);
    hipStream_t sa = s;
    if (overlap) {
      sa = x->side;
      HH_HIP(hipEventRecord(x->fork_ev[l], s));
      HH_HIP(hipStreamWaitEvent(sa, x->fork_ev[l], 0));
    }
    if (full) {
      AttnArgs a{};
      a.kpool = w.kpool; a.vpool = w.vpool; a.qkv = x->qkv; a.o = x->o; a.pos0 = x->pos0; a.n_tok = n_tok;
      a.page_table = x->page_table; a.rope = x->rope; a.part_o = x->part_o; a.part_ml = x->part_ml;
      a.counters = x->attn_counters;
      a.T = T; a.B = B; a.n_splits = n_splits;
      GemvArgs b{};
      b.X = x->o; b.ldx = d.dq; b.M = M; b.K = d.dq; b.norm_w = nullptr; b.epi = EPI_STORE; b.bf16 = d.bf16; b.flags = d.flags;
      b.seg[0] = {w.w_o, nullptr, w.p_o, nullptr, x->ho, d.D, d.D}; b.n_seg = 1;
      if (overlap) {
        HH_HIP(launch_attention(d, a, sa));
        HH_HIP(product(x, b, sa, true));
        HH_HIP(hipEventRecord(x->join_ev[l], sa));
      } else {
        HH_LAUNCH(HH_K_ATTN, launch_attention(d, a, s));
        HH_LAUNCH(HH_K_O_PROJ, product(x, b, s));
      }
    }
    {  // conv + selective scan -> y * silu(z)
      SsmArgs a{};
      a.layers = nullptr; a.one = w; a.layer0 = 0; a.n_layers_z = 1;
      a.zx = x->zx; a.g = x->g; a.pos0 = x->pos0; a.n_tok = n_tok; a.T = T; a.B = B;
      a.state_in = state_in; a.state_out = state_out; a.write_ring = 1;
      HH_LAUNCH(HH_K_SSM, launch_ssm(d, a, s));
    }
    {  // h += W_out * gated_norm(g)
      GemvArgs a{};
      a.X = x->g; a.ldx = d.d_inner; a.M = M; a.K = d.d_inner; a.norm_w = w.gnorm; a.eps = d.eps; a.epi = EPI_ADD; a.bf16 = d.bf16; a.flags = d.flags;
      a.seg[0] = {w.w_out, nullptr, w.p_out, nullptr, x->h, d.D, d.D}; a.n_seg = 1;
      HH_LAUNCH(HH_K_OUT_PROJ, product(x, a, s));
    }
    if (overlap) HH_HIP(hipStreamWaitEvent(s, x->join_ev[l], 0));
    {  // SwiGLU MLP on r = rmsnorm(h + ho); h += ho + W_d(...)   (ho: full mode only)
      const float* ho = full ? x->ho : nullptr;
      GemvArgs a{};
      a.X = x->h; a.X2 = ho; a.ldx = d.D; a.M = M; a.K = d.D; a.norm_w = w.norm2; a.eps = d.eps; a.epi = EPI_SWIGLU; a.bf16 = d.bf16; a.flags = d.flags;
      a.seg[0] = {w.w_gate, w.w_up, w.p_gate, w.p_up, x->act, d.F, d.F}; a.n_seg = 1;
      GemvArgs b{};
      b.X = x->act; b.ldx = d.F; b.M = M; b.K = d.F; b.norm_w = nullptr; b.epi = EPI_ADD; b.bf16 = d.bf16; b.flags = d.flags; b.R2 = ho;
      b.seg[0] = {w.w_down, nullptr, w.p_down, nullptr, x->h, d.D, d.D}; b.n_seg = 1;
      // many rows: the SwiGLU result goes to the down projection as split bf16 planes, without the float32
      // round trip through `act` and without a split kernel of its own
      if (x->planes_act != nullptr && !(d.flags & HH_KF_NO_HANDOVER) && !mid_mfma_fits(a)) {
        GemvArgs sk;
        if (!skinny_args(a, sk) && gemm_hands_over_planes(a)) {
          a.planes_out = x->planes_act;
          b.planes_in = x->planes_act;
        }
      }
      HH_LAUNCH(HH_K_MLP_UP, product(x, a, s));
      HH_LAUNCH(HH_K_MLP_DOWN, product(x, b, s));
    }
  }
  return HH_OK;
}

// final norm + LM head + argmax of M rows of X; row m = b*T + j -> out[b*out_stride + out_off + j]
hh_status run_head(hh_ctx* x, const float* X, int M, int T, float* logits, int ld_logits, int* out, int out_stride,
                   int out_off, hipStream_t s) {
  const Dims& d = x->d;
  GemvArgs a{};
  a.X = X; a.ldx = d.D; a.M = M; a.K = d.D; a.norm_w = static_cast<const float*>(x->final_norm); a.eps = d.eps;
  a.epi = EPI_STORE; a.bf16 = d.bf16; a.flags = d.flags; a.best = x->best;
  // greedy rounds of a context created with keep_logits = 0 only need the argmax of every row
  a.no_store = !x->cfg.keep_logits && !(x->temperature > 0.f);
  a.seg[0] = {x->lm_head, nullptr, x->p_lm_head, nullptr, logits, d.V, ld_logits}; a.n_seg = 1;
  GemvArgs sk;
  if (skinny_args(a, sk)) {
    int nb = 0;
    HH_LAUNCH(HH_K_LM_HEAD, launch_skinny_mfma(sk, x->gemm_partial, &nb, s));
    HH_HIP(launch_argmax_finish(x->best, nb, M, out, out_stride, out_off, T, s));
    return HH_OK;
  }
  if (a.bf16 && M >= kMfmaMinRows) {
    // many-row kernels: every row's argmax key is raised with atomic maxima in the epilogue (the first
    // M entries of the partials buffer, cleared here), so the logits need not be written or re-read
    a.best = nullptr; a.row_best = x->best;
    HH_HIP(launch_fill_i32(reinterpret_cast<int*>(x->best), 0, (size_t)2 * M, s));
    if (mid_mfma_fits(a)) HH_LAUNCH(HH_K_LM_HEAD, launch_mid_mfma(a, x->gemm_partial, s));
    else HH_LAUNCH(HH_K_LM_HEAD, launch_gemm_mfma(a, x->planes, x->gemm_partial, s));
    HH_HIP(launch_argmax_finish(x->best, 1, M, out, out_stride, out_off, T, s));
    return HH_OK;
  }
  int nblk = 0;
  HH_LAUNCH(HH_K_LM_HEAD, launch_gemv(a, &nblk, s));
  HH_HIP(launch_argmax_finish(x->best, nblk, M, out, out_stride, out_off, T, s));
  return HH_OK;
}

// Replays `enqueue` (a fixed sequence of kernel launches whose arguments never change for this
// key) as a HIP graph.  Not used on the NULL stream (it cannot be captured) or while profiling.
template <typename F>
hh_status run_graphed(hh_ctx* x, long long key, hipStream_t s, F enqueue) {
  if (!x->cfg.use_graphs || x->prof_on || s == nullptr) return enqueue();
  hh_ctx::GraphSlot& g = x->graphs[key];
  if (g.exec != nullptr) {
    HH_HIP(hipGraphLaunch(g.exec, s));
    return HH_OK;
  }
  if (g.uses++ == 0) return enqueue();
  HH_HIP(hipStreamBeginCapture(s, hipStreamCaptureModeThreadLocal));
  const hh_status st = enqueue();
  hipGraph_t graph = nullptr;
  const hipError_t e = hipStreamEndCapture(s, &graph);
  if (st != HH_OK || e != hipSuccess || graph == nullptr) {
    if (graph) (void)hipGraphDestroy(graph);
    if (st != HH_OK) return st;
    return fail(x, HH_EDEVICE, std::string("hipStreamEndCapture: ") + hipGetErrorString(e));
  }
  const hipError_t ei = hipGraphInstantiate(&g.exec, graph, nullptr, nullptr, 0);
  (void)hipGraphDestroy(graph);
  if (ei != hipSuccess) {
    g.exec = nullptr;
    return fail(x, HH_EDEVICE, std::string("hipGraphInstantiate: ") + hipGetErrorString(ei));
  }
  HH_HIP(hipGraphLaunch(g.exec, s));
  return HH_OK;
}

// Key slices per (sequence, KV head, row chunk) of a verification pass: enough workgroups to
// cover the chip once (more slices cost more in partial results and their merge than they gain:
// at 64 sequences x 2 KV heads over 8192-token caches 2 slices take 133 us per layer, 4 slices 151,
// 8 slices 188), but no slice smaller than the unit of work of the kernel.
int pick_splits(const hh_cfg& c, const Dims& d, int B, int T, int len_upper) {
  const int cap = c.attn_max_splits > 0 ? c.attn_max_splits : 16;
  const int target = c.attn_target_blocks > 0 ? c.attn_target_blocks : 256;   // one workgroup per compute unit: measured best at every workload
  const int single = c.attn_single_slice_steps == 0 ? 28 : c.attn_single_slice_steps;   // -1: never a single slice by this rule
  int s;
  if (attention_uses_mfma(d)) {
    const int blocks = attention_mfma_row_chunks(d, T) * d.Hkv * B;
    const int steps = (len_upper + T + 31) / 32;      // 32 keys per wavefront step, 4 wavefronts per workgroup
    s = (target + blocks - 1) / blocks;
    if (s > (steps + 3) / 4) s = (steps + 3) / 4;
    // short caches: the ticket and the merge across workgroups (about 4 us) cost more than the
    // few extra steps per wavefront of a single slice
    if (steps <= single) s = 1;
  } else {
    const int G = d.Hq / d.Hkv;
    const int row_chunks = (T * G + 15) / 16;
    const int blocks = row_chunks * d.Hkv * B;
    const int tiles = (len_upper + T + 63) / 64;
    s = (target + blocks - 1) / blocks;
    if (s > tiles) s = tiles;
  }
  if (s > kMaxSplits) s = kMaxSplits;
  if (s > cap) s = cap;
  return s < 1 ? 1 : s;
}

// Strict draft state: M_S (no head) over positions first..last of the round (position 0 consumes
// the pending token, position i draft i), continuing from the draft scratch state (from M_S's
// committed state at position 0); leaves the raw inputs of those positions in M_S's ring (the
// scratch state after the last of them is not needed and not written).
hh_status ms_consume(hh_ctx* x, int B, int first, int last, hipStream_t s) {
  const Dims& d = x->d;
  for (int i = first; i <= last; ++i) {
    HH_HIP(launch_gather_tokens(x->pending, x->drafts, d.Kmax, B, 1, 0, i, x->tok, x->kv_len, x->pos0, s));
    HH_HIP(launch_embed(d, x->embed, x->tok, B, x->h, s));
    const hh_status st = run_layers(x, x->layers_ms_host, false, nullptr, B, 1, nullptr, i == 0 ? 0 : 1, i == last ? 0 : 2, 1, false, s);
    if (st != HH_OK) return st;
  }
  return HH_OK;
}

}  // namespace

extern "C" {

size_t hh_workspace_bytes(const hh_cfg* cfg) {
  if (!cfg) return 0;
  hh_ctx tmp;
  std::string why;
  tmp.cfg = *cfg;
  if (!derive_dims(*cfg, tmp.d, why)) { g_create_error = why; return 0; }
  return carve(&tmp, nullptr);
}

hh_status hh_create(const hh_weights* weights, const hh_cfg* cfg, hh_ctx** out) {
  hh_ctx* x = nullptr;
  if (out) *out = nullptr;
  if (!weights || !cfg || !out) return fail(nullptr, HH_EINVAL, "hh_create: NULL argument");
  Dims d;
  std::string why;
  if (!derive_dims(*cfg, d, why)) return fail(nullptr, HH_EINVAL, "hh_create: " + why);
  if (!weights->embed || !weights->final_norm || !weights->lm_head || !weights->layers)
    return fail(nullptr, HH_EINVAL, "hh_create: NULL weight pointer");
  for (int l = 0; l < d.L; ++l) {
    const void* const* p = reinterpret_cast<const void* const*>(&weights->layers[l]);
    for (size_t i = 0; i < sizeof(hh_layer_weights) / sizeof(void*); ++i)
      if (!p[i]) return fail(nullptr, HH_EINVAL, "hh_create: NULL layer weight pointer");
  }
  hh_ctx* ctx = new hh_ctx();
  ctx->cfg = *cfg; ctx->d = d;
  const size_t need = carve(ctx, nullptr);
  if (!cfg->workspace || (reinterpret_cast<uintptr_t>(cfg->workspace) % kAlign) != 0 || cfg->workspace_bytes < need) {
    char msg[160];
    snprintf(msg, sizeof msg, "hh_create: workspace missing, misaligned or too small (need %zu bytes, 256-byte aligned)", need);
    delete ctx;
    return fail(nullptr, HH_EWORKSPACE, msg);
  }
  carve(ctx, static_cast<char*>(cfg->workspace));
  for (size_t off : ctx->canaries) {
    const hipError_t ce = hipMemset(static_cast<char*>(cfg->workspace) + off, kCanaryByte, kCanaryBytes);
    if (ce != hipSuccess) {
      delete ctx;
      return fail(nullptr, HH_EDEVICE, std::string("hh_create: writing the region guards: ") + hipGetErrorString(ce));
    }
  }
  ctx->embed = weights->embed; ctx->final_norm = weights->final_norm; ctx->lm_head = weights->lm_head;
  for (int l = 0; l < d.L; ++l) {
    const hh_layer_weights& w = weights->layers[l];
    LayerDev& ld = ctx->layers_host[l];
    ld.norm1 = (const float*)w.norm1; ld.conv_w = (const float*)w.conv_w; ld.conv_b = (const float*)w.conv_b;
    ld.a_log = (const float*)w.a_log; ld.d_skip = (const float*)w.d_skip; ld.dt_bias = (const float*)w.dt_bias;
    ld.gnorm = (const float*)w.gnorm; ld.norm2 = (const float*)w.norm2;
    ld.w_in = w.w_in; ld.w_out = w.w_out; ld.w_q = w.w_q; ld.w_k = w.w_k; ld.w_v = w.w_v; ld.w_o = w.w_o;
    ld.w_gate = w.w_gate; ld.w_up = w.w_up; ld.w_down = w.w_down;
  }
  x = nullptr;  // errors below are reported through g_create_error
  // stacked copy of the four input-side projections, so that one product yields z|xBC|dt|q|k|v
  {
    const size_t esz = d.bf16 ? 2 : 4, rowb = (size_t)d.D * esz;
    for (int l = 0; l < d.L; ++l) {
      LayerDev& ld = ctx->layers_host[l];
      char* dst = static_cast<char*>(ld.w_inqkv);
      const void* src[4] = {ld.w_in, ld.w_q, ld.w_k, ld.w_v};
      const size_t rows[4] = {(size_t)d.d_in_proj, (size_t)d.dq, (size_t)d.dkv, (size_t)d.dkv};
      for (int i = 0; i < 4; ++i) {
        hipError_t ce = hipMemcpy(dst, src[i], rows[i] * rowb, hipMemcpyDeviceToDevice);
        if (ce != hipSuccess) {
          delete ctx;
          return fail(nullptr, HH_EDEVICE, std::string("hh_create: stacking projections: ") + hipGetErrorString(ce));
        }
        dst += rows[i] * rowb;
      }
    }
  }
  auto bail = [&](hipError_t e, const char* what) {
    delete ctx;
    return fail(nullptr, HH_EDEVICE, std::string(what) + ": " + hipGetErrorString(e));
  };
  if (d.bf16) {   // copies of every matrix in the tile layout of the matrix-core kernels
    hipError_t pe = hipSuccess;
    auto pack = [&](const void* W, int N, int K, void* P) { if (pe == hipSuccess) pe = launch_pack_weights(W, N, K, (size_t)K, P, nullptr); };
    for (int l = 0; l < d.L; ++l) {
      const LayerDev& ld = ctx->layers_host[l];
      pack(ld.w_inqkv, d.ldzx, d.D, ld.p_inqkv);
      pack(ld.w_out, d.D, d.d_inner, ld.p_out);
      pack(ld.w_o, d.D, d.dq, ld.p_o);
      pack(ld.w_gate, d.F, d.D, ld.p_gate);
      pack(ld.w_up, d.F, d.D, ld.p_up);
      pack(ld.w_down, d.D, d.F, ld.p_down);
    }
    pack(ctx->lm_head, d.V, d.D, ctx->p_lm_head);
    if (pe == hipSuccess) pe = hipDeviceSynchronize();
    if (pe != hipSuccess) return bail(pe, "hh_create: packing the weights");
  }
  hipError_t e = hipMemcpy(ctx->layers_dev, ctx->layers_host.data(), sizeof(LayerDev) * d.L, hipMemcpyHostToDevice);
  if (e != hipSuccess) return bail(e, "hh_create: upload of layer table");
  ctx->strict = cfg->draft_state_mode == 1;
  if (ctx->strict) {
    for (int l = 0; l < d.L; ++l) {
      LayerDev ms = ctx->layers_host[l];
      ms.S = ctx->layers_ms_host[l].S;
      ms.ring = ctx->layers_ms_host[l].ring;
      ctx->layers_ms_host[l] = ms;
    }
    e = hipMemcpy(ctx->layers_ms_dev, ctx->layers_ms_host.data(), sizeof(LayerDev) * d.L, hipMemcpyHostToDevice);
    if (e != hipSuccess) return bail(e, "hh_create: upload of the draft model's layer table");
  }
  e = hipMemset(ctx->attn_counters, 0, sizeof(int) * (size_t)d.Bmax * d.Hkv * attention_row_chunks(d, d.Tmax));
  if (e != hipSuccess) return bail(e, "hh_create: clearing the attention tickets");
  // rotary table: angle pos * base^(-2i/Dh) evaluated in double, stored as float (cos, sin)
  {
    const int half = d.Dh / 2;
    std::vector<float> tab((size_t)d.max_seq * d.Dh);
    for (int i = 0; i < half; ++i) {
      const double inv = pow((double)d.rope_base, -2.0 * i / d.Dh);
      for (int pos = 0; pos < d.max_seq; ++pos) {
        const double ang = (double)pos * inv;
        tab[((size_t)pos * half + i) * 2] = (float)cos(ang);
        tab[((size_t)pos * half + i) * 2 + 1] = (float)sin(ang);
      }
    }
    e = hipMemcpy(ctx->rope, tab.data(), tab.size() * sizeof(float), hipMemcpyHostToDevice);
    if (e != hipSuccess) return bail(e, "hh_create: upload of rotary table");
  }
  // side stream (default priority) and per-layer fork/join events for the branch overlap
  e = hipStreamCreateWithFlags(&ctx->side, hipStreamNonBlocking);
  if (e != hipSuccess) return bail(e, "hh_create: side stream");
  ctx->fork_ev.resize(d.L); ctx->join_ev.resize(d.L);
  for (int l = 0; l < d.L; ++l) {
    ctx->fork_ev[l] = nullptr; ctx->join_ev[l] = nullptr;
  }
  for (int l = 0; l < d.L; ++l) {
    e = hipEventCreateWithFlags(&ctx->fork_ev[l], hipEventDisableTiming);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&ctx->join_ev[l], hipEventDisableTiming);
    if (e != hipSuccess) return bail(e, "hh_create: events");
  }
  *out = ctx;
  return HH_OK;
}

hh_status hh_destroy(hh_ctx* ctx) {
  if (!ctx) return HH_EINVAL;
  delete ctx;
  return HH_OK;
}

hh_status hh_prefill(hh_ctx* x, const int32_t* tokens, int32_t row_stride, const int32_t* lens, int32_t batch,
                     int32_t max_new, void* stream) {
  if (!x) return HH_EINVAL;
  if (!tokens || !lens) return fail(x, HH_EINVAL, "hh_prefill: NULL argument");
  const Dims& d = x->d;
  if (batch < 1 || batch > d.Bmax) return fail(x, HH_ECAPACITY, "hh_prefill: batch exceeds max_batch");
  if (max_new < 1 || max_new > d.Gmax) return fail(x, HH_ECAPACITY, "hh_prefill: max_new exceeds max_new_tokens");
  int maxlen = 0;
  for (int b = 0; b < batch; ++b) {
    if (lens[b] < 1 || lens[b] > row_stride) return fail(x, HH_EINVAL, "hh_prefill: lens[b] must be in 1..row_stride");
    if ((long long)lens[b] + max_new + 2LL * d.Kmax + 2 > d.max_seq)
      return fail(x, HH_ECAPACITY, "hh_prefill: lens[b] + max_new + 2*max_draft + 2 exceeds max_seq_len");
    if (lens[b] > maxlen) maxlen = lens[b];
  }
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int B = batch;
  const int chunk = prefill_chunk_of(x->cfg);
  const int n_pass = (maxlen + chunk - 1) / chunk;
  x->prof_phase = HH_PHASE_PREFILL;

  // pages: each sequence gets what its final length can need, handed out round-robin so that
  // the pages of one sequence are not contiguous in the pool
  x->h_page_table.assign((size_t)B * d.pages_per_seq, 0);
  {
    std::vector<int> need(B), got(B, 0);
    int most = 0;
    for (int b = 0; b < B; ++b) {
      need[b] = (lens[b] + max_new + 2 * d.Kmax + 2 + d.page_tokens - 1) / d.page_tokens;
      if (need[b] > d.pages_per_seq) need[b] = d.pages_per_seq;
      if (need[b] > most) most = need[b];
    }
    int next = 0;
    for (int i = 0; i < most; ++i)
      for (int b = 0; b < B; ++b)
        if (got[b] < need[b]) x->h_page_table[(size_t)b * d.pages_per_seq + got[b]++] = next++;
    if (next > d.n_pages) return fail(x, HH_ECAPACITY, "hh_prefill: KV page pool exhausted");
  }
  x->h_plan.assign((size_t)2 * n_pass * B, 0);
  for (int p = 0; p < n_pass; ++p)
    for (int b = 0; b < B; ++b) {
      int nt = lens[b] - p * chunk;
      nt = nt < 0 ? 0 : (nt > chunk ? chunk : nt);
      x->h_plan[(size_t)p * B + b] = nt;
      x->h_plan[(size_t)(n_pass + p) * B + b] = (nt > 0 && lens[b] <= (p + 1) * chunk) ? 1 : 0;
    }
  HH_HIP(hipMemcpyAsync(x->page_table, x->h_page_table.data(), x->h_page_table.size() * sizeof(int), hipMemcpyHostToDevice, s));
  HH_HIP(hipMemcpyAsync(x->plan_ntok, x->h_plan.data(), (size_t)n_pass * B * sizeof(int), hipMemcpyHostToDevice, s));
  HH_HIP(hipMemcpyAsync(x->plan_last, x->h_plan.data() + (size_t)n_pass * B, (size_t)n_pass * B * sizeof(int), hipMemcpyHostToDevice, s));
  HH_HIP(launch_fill_i32(x->kv_len, 0, B, s));
  HH_HIP(launch_fill_i32(x->committed, 0, B, s));
  HH_HIP(launch_fill_i32(reinterpret_cast<int*>(x->acc_stats), 0, 4, s));

  for (int p = 0; p < n_pass; ++p) {
    const int T = maxlen - p * chunk < chunk ? maxlen - p * chunk : chunk;
    const int* nt = x->plan_ntok + (size_t)p * B;
    HH_HIP(launch_gather_prompt(tokens, row_stride, p * chunk, nt, B, T, x->tok, x->kv_len, x->pos0, s));
    HH_HIP(launch_embed(d, x->embed, x->tok, B * T, x->h, s));
    hh_status st = HH_OK;
    if (x->strict) {   // M_S over the same positions first, into its own state and ring (Eq. 4 at every prefix position)
      st = run_layers(x, x->layers_ms_host, false, nullptr, B, T, nt, p == 0 ? 2 : 0, 1, 1, true, s);
      if (st != HH_OK) return st;
      HH_HIP(launch_embed(d, x->embed, x->tok, B * T, x->h, s));
    }
    st = run_layers(x, x->layers_host, true, nullptr, B, T, nt, p == 0 ? 2 : 0, 1, 1, true, s);
    if (st != HH_OK) return st;
    HH_HIP(launch_prefill_tail(x->h, T, d.D, nt, x->plan_last + (size_t)p * B, x->lasth, x->kv_len, B, s));
    // cfg.prefill_progress = n: wait for every n-th pass and report it (long prompts; otherwise the call only enqueues)
    const int progress = x->cfg.prefill_progress;
    if (progress > 0 && (p + 1) % progress == 0) {
      HH_HIP(hipStreamSynchronize(s));
      fprintf(stderr, "[hh] prefill pass %d of %d done\n", p + 1, n_pass);
      fflush(stderr);
    }
  }
  hh_status st = run_head(x, x->lasth, B, 1, x->logits_p, d.V, x->first_tok, 1, 0, s);
  if (st != HH_OK) return st;
  if (x->temperature > 0.f)
    HH_HIP(launch_sample_rows(x->logits_p, d.V, d.V, B, x->sampling, SamplingParams{}, nullptr, 0, 2, x->first_tok, 1, 0, s));
  HH_HIP(launch_prefill_finish(x->first_tok, x->pending, x->out_tok, d.Gmax, x->committed, x->last_n, B, s));
  x->B = B; x->G = max_new; x->k = 0; x->len_upper = maxlen;
  x->phase = PH_READY;
  return HH_OK;
}

hh_status hh_set_sampling(hh_ctx* x, float temperature, uint64_t seed, void* stream) {
  if (!x) return HH_EINVAL;
  if (x->phase != PH_CREATED && x->phase != PH_READY)
    return fail(x, HH_ESTATE, "hh_set_sampling: not while a round is in flight");
  if (!(temperature >= 0.f) || !(temperature < 1e30f)) return fail(x, HH_EINVAL, "hh_set_sampling: temperature must be finite and >= 0");
  hipStream_t s = static_cast<hipStream_t>(stream);
  SamplingParams p{};
  p.inv_t = temperature > 0.f ? 1.0f / temperature : 0.f;
  p.seed = seed;
  // ordered after the rounds already enqueued on the stream; the source is copied before the call returns
  HH_HIP(hipMemcpyAsync(x->sampling, &p, sizeof(p), hipMemcpyHostToDevice, s));
  HH_HIP(hipStreamSynchronize(s));
  x->temperature = temperature;
  return HH_OK;
}

static bool sampling_value(float temperature, uint64_t seed, SamplingParams& p) {
  if (!(temperature > 0.f) || !(temperature < 1e30f)) return false;
  p.inv_t = 1.0f / temperature; p.pad = 0; p.seed = seed;
  return true;
}

hh_status hh_draw_tokens(const float* logits, int64_t row_stride, int32_t vocab, int32_t rows, float temperature,
                         uint64_t seed, const int32_t* positions, int32_t position_offset, int32_t purpose, int32_t* out,
                         void* stream) {
  SamplingParams p{};
  if (!logits || !out || vocab < 1 || rows < 0 || row_stride < vocab || purpose < 0 || purpose > 3 || position_offset < 0 ||
      !sampling_value(temperature, seed, p))
    return HH_EINVAL;
  if (rows == 0) return HH_OK;
  if (launch_sample_rows(logits, (size_t)row_stride, vocab, rows, nullptr, p, positions, position_offset, purpose, out, 1, 0,
                         static_cast<hipStream_t>(stream)) != hipSuccess)
    return HH_EDEVICE;
  return HH_OK;
}

hh_status hh_accept_tokens(const float* draft_logits, const float* verify_logits, int32_t vocab, int32_t batch, int32_t k,
                           const int32_t* drafts, const int32_t* positions, float temperature, uint64_t seed,
                           float* scratch, int32_t* targets, void* stream) {
  SamplingParams p{};
  if (!verify_logits || !positions || !scratch || !targets || vocab < 1 || batch < 0 || k < 0 ||
      (k > 0 && (!draft_logits || !drafts)) || !sampling_value(temperature, seed, p))
    return HH_EINVAL;
  if (batch == 0) return HH_OK;
  if (launch_spec_targets(draft_logits, verify_logits, vocab, batch, k, k, nullptr, p, scratch, drafts, positions, targets,
                          static_cast<hipStream_t>(stream)) != hipSuccess)
    return HH_EDEVICE;
  return HH_OK;
}

hh_status hh_accept_tokens_static(const float* draft_logits, const float* verify_logits, int32_t vocab, int32_t batch,
                                  int32_t k, const int32_t* drafts, const int32_t* positions, float temperature,
                                  uint64_t seed, int32_t* targets, void* stream) {
  SamplingParams p{};
  if (!verify_logits || !positions || !targets || vocab < 1 || batch < 0 || k < 0 || (k > 0 && (!draft_logits || !drafts)) ||
      !sampling_value(temperature, seed, p))
    return fail(nullptr, HH_EINVAL, "hh_accept_tokens_static: bad argument");
  if (batch == 0) return HH_OK;
  float* stats = nullptr;
  size_t cap = 0;
  const hipError_t e = static_accept_scratch(&stats, &cap);
  if (e != hipSuccess) return fail(nullptr, HH_EDEVICE, std::string("hh_accept_tokens_static: ") + hipGetErrorString(e));
  const unsigned long long need = (unsigned long long)batch * (2ull * (unsigned long long)k + 1ull) * 2ull;
  if (need > cap) {
    char msg[200];
    snprintf(msg, sizeof msg, "hh_accept_tokens_static: batch * (2k + 1) * 2 = %llu floats of statistics exceed the built-in %zu",
             need, cap);
    return fail(nullptr, HH_ECAPACITY, msg);
  }
  if (launch_spec_targets(draft_logits, verify_logits, vocab, batch, k, k, nullptr, p, stats, drafts, positions, targets,
                          static_cast<hipStream_t>(stream)) != hipSuccess)
    return fail(nullptr, HH_EDEVICE, "hh_accept_tokens_static: launch failed");
  return HH_OK;
}

hh_status hh_draft(hh_ctx* x, int32_t k, void* stream) {
  if (!x) return HH_EINVAL;
  if (x->phase != PH_READY) return fail(x, HH_ESTATE, "hh_draft: needs a prefilled context with no round in flight");
  const Dims& d = x->d;
  if (k < 0 || k > d.Kmax) return fail(x, HH_ECAPACITY, "hh_draft: k outside 0..max_draft");
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int B = x->B;
  const bool stochastic = x->temperature > 0.f;
  x->prof_phase = HH_PHASE_DRAFT;
  const std::vector<LayerDev>& table = x->strict ? x->layers_ms_host : x->layers_host;
  const int* modes = x->draft_modes.empty() ? nullptr : x->draft_modes.data();
  const int splits = x->draft_has_full ? pick_splits(x->cfg, d, B, 1, x->len_upper) : 1;
  auto enqueue = [&]() -> hh_status {
    for (int i = 0; i < k; ++i) {
      HH_HIP(launch_gather_tokens(x->pending, x->drafts, d.Kmax, B, 1, 0, i, x->tok, x->kv_len, x->pos0, s));
      HH_HIP(launch_embed(d, x->embed, x->tok, B, x->h, s));
      // the scratch state after the last step is never read (unless M_S goes on to consume d_k): not written
      const int state_out = (i == k - 1 && !x->strict) ? 0 : 2;
      hh_status st = run_layers(x, table, false, modes, B, 1, nullptr, i == 0 ? 0 : 1, state_out, splits, false, s);
      if (st != HH_OK) return st;
      st = run_head(x, x->h, B, 1, x->logits_d + (size_t)i * d.V, d.Kmax * d.V, x->drafts, d.Kmax, i, s);
      if (st != HH_OK) return st;
      if (stochastic)
        HH_HIP(launch_sample_rows(x->logits_d + (size_t)i * d.V, (size_t)d.Kmax * d.V, d.V, B, x->sampling, SamplingParams{},
                                  x->committed, i, 0, x->drafts, d.Kmax, i, s));
    }
    // strict state: M_S also consumes d_k (no head), so that its ring holds the raw inputs of all
    // k+1 positions a commit may keep
    if (x->strict) return ms_consume(x, B, k, k, s);
    return HH_OK;
  };
  if (k > 0 || x->strict) {
    const hh_status st = run_graphed(x, (1LL << 40) | ((long long)stochastic << 38) | ((long long)B << 20) | ((long long)splits << 8) | k, s, enqueue);
    if (st != HH_OK) return st;
  }
  x->k = k;
  x->phase = PH_DRAFTED;
  return HH_OK;
}

hh_status hh_set_drafts(hh_ctx* x, const int32_t* drafts, void* stream) {
  if (!x) return HH_EINVAL;
  if (x->phase != PH_DRAFTED) return fail(x, HH_ESTATE, "hh_set_drafts: only between hh_draft and hh_verify");
  if (x->temperature > 0.f)
    return fail(x, HH_ESTATE, "hh_set_drafts: replaced drafts have no draft distribution to test against at temperature > 0");
  if (!drafts) return fail(x, HH_EINVAL, "hh_set_drafts: NULL argument");
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (x->k > 0)
    HH_HIP(hipMemcpy2DAsync(x->drafts, (size_t)x->d.Kmax * sizeof(int), drafts, (size_t)x->k * sizeof(int),
                            (size_t)x->k * sizeof(int), x->B, hipMemcpyDeviceToDevice, s));
  // strict state: M_S's ring must hold the raw inputs of the tokens that may be committed
  if (x->strict) return ms_consume(x, x->B, 0, x->k, s);
  return HH_OK;
}

hh_status hh_set_draft_mask(hh_ctx* x, const int32_t* modes) {
  if (!x) return HH_EINVAL;
  if (x->phase != PH_CREATED && x->phase != PH_READY)
    return fail(x, HH_ESTATE, "hh_set_draft_mask: not while a round is in flight");
  const Dims& d = x->d;
  std::vector<int> m;
  bool any = false, has_full = false;
  if (modes) {
    m.assign(modes, modes + d.L);
    for (int v : m) {
      if (v != HH_DRAFT_SSM && v != HH_DRAFT_FULL && v != HH_DRAFT_SKIP)
        return fail(x, HH_EINVAL, "hh_set_draft_mask: modes must be HH_DRAFT_SSM, HH_DRAFT_FULL or HH_DRAFT_SKIP");
      any |= v != HH_DRAFT_SSM;
      has_full |= v == HH_DRAFT_FULL;
    }
  }
  if (any && x->strict)
    return fail(x, HH_ESTATE, "hh_set_draft_mask: the strict draft state is defined for the SSM-only draft (all HH_DRAFT_SSM)");
  if (!any) m.clear();
  if (m != x->draft_modes) {
    // captured draft sequences belong to the old mask
    for (auto it = x->graphs.begin(); it != x->graphs.end();) {
      if ((it->first >> 40) == 1) {
        if (it->second.exec) (void)hipGraphExecDestroy(it->second.exec);
        it = x->graphs.erase(it);
      } else {
        ++it;
      }
    }
  }
  x->draft_modes = m;
  x->draft_has_full = has_full;
  return HH_OK;
}

int32_t hh_optimal_draft_length(double alpha, double cost_ratio, const int32_t* candidates, int32_t n_candidates) {
  if (!candidates || n_candidates < 1 || !(alpha >= 0.0) || !(alpha <= 1.0) || !(cost_ratio >= 0.0) || !(cost_ratio < 1e30))
    return -1;
  std::vector<int32_t> ks(candidates, candidates + n_candidates);
  std::sort(ks.begin(), ks.end());
  if (ks.front() < 0) return -1;
  int32_t best = -1;
  double best_s = -1.0;
  for (int32_t k : ks) {   // ascending, so that the shortest of equally good lengths wins
    // Eq. 1: expected tokens per round 1 + alpha + .. + alpha^k over the round's cost 1 + k * c
    double tokens = 0.0, pw = 1.0;
    for (int32_t j = 0; j <= k; ++j) { tokens += pw; pw *= alpha; }
    const double sp = tokens / (1.0 + (double)k * cost_ratio);
    if (sp > best_s + 1e-15) { best = k; best_s = sp; }
  }
  return best;
}

hh_status hh_verify(hh_ctx* x, void* stream) {
  if (!x) return HH_EINVAL;
  if (x->phase != PH_DRAFTED) return fail(x, HH_ESTATE, "hh_verify: needs hh_draft first");
  const Dims& d = x->d;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int B = x->B, T = x->k + 1;
  const bool stochastic = x->temperature > 0.f;
  x->prof_phase = HH_PHASE_VERIFY;
  const int splits = pick_splits(x->cfg, d, B, T, x->len_upper);
  auto enqueue = [&]() -> hh_status {
    HH_HIP(launch_gather_tokens(x->pending, x->drafts, d.Kmax, B, T, 1, 0, x->tok, x->kv_len, x->pos0, s));
    HH_HIP(launch_embed(d, x->embed, x->tok, B * T, x->h, s));
    hh_status st = run_layers(x, x->layers_host, true, nullptr, B, T, nullptr, 0, 0, splits, false, s);
    if (st != HH_OK) return st;
    st = run_head(x, x->h, B * T, T, x->logits_v, d.V, x->targets, d.Kmax + 1, 0, s);
    if (st != HH_OK) return st;
    if (stochastic)
      HH_HIP(launch_spec_targets(x->logits_d, x->logits_v, d.V, B, x->k, d.Kmax, x->sampling, SamplingParams{}, x->softmax_stats, x->drafts,
                                 x->committed, x->targets, s));
    return HH_OK;
  };
  const hh_status st = run_graphed(x, (2LL << 40) | ((long long)branch_overlap(x, B, T, false) << 39) | ((long long)stochastic << 38) | ((long long)B << 20) | ((long long)splits << 8) | T, s, enqueue);
  if (st != HH_OK) return st;
  x->phase = PH_VERIFIED;
  return HH_OK;
}

hh_status hh_commit(hh_ctx* x, const int32_t* n_accepted, void* stream) {
  if (!x) return HH_EINVAL;
  if (x->phase != PH_VERIFIED) return fail(x, HH_ESTATE, "hh_commit: needs hh_verify first");
  if (n_accepted && x->temperature > 0.f)
    return fail(x, HH_ESTATE, "hh_commit: a forced count has no correction token at temperature > 0");
  const Dims& d = x->d;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int B = x->B;
  x->prof_phase = HH_PHASE_COMMIT;
  CommitArgs c{};
  c.drafts = x->drafts; c.targets = x->targets; c.forced = n_accepted;
  c.committed = x->committed; c.last_n = x->last_n; c.pending = x->pending; c.out_tok = x->out_tok;
  c.n_acc = x->n_acc; c.skip = x->skip; c.adv = x->adv; c.acc_stats = x->acc_stats;
  c.B = B; c.k = x->k; c.kmax = d.Kmax; c.G = x->G; c.out_stride = d.Gmax;
  HH_HIP(launch_accept(c, s));
  // rollback: rebuild the state after position n from the committed state and the ring
  SsmArgs a{};
  a.layers = x->layers_dev; a.layer0 = 0; a.n_layers_z = d.L;
  a.zx = nullptr; a.g = nullptr; a.pos0 = x->kv_len; a.n_tok = nullptr; a.n_acc = x->n_acc; a.skip = x->skip;
  a.T = x->k + 1; a.B = B; a.state_in = 0; a.state_out = 1; a.write_ring = 0;
  HH_LAUNCH(HH_K_SSM, launch_ssm(d, a, s));
  if (x->strict) {   // M_S has consumed the same n+1 tokens: its state after position n, from its own ring
    a.layers = x->layers_ms_dev;
    HH_LAUNCH(HH_K_SSM, launch_ssm(d, a, s));
  }
  HH_HIP(launch_advance(x->kv_len, x->adv, B, s));
  x->len_upper += x->k + 1;
  if (x->len_upper > d.max_seq) x->len_upper = d.max_seq;
  x->phase = PH_READY;
  return HH_OK;
}

// ------------------------------------------------------------------ read-back

static hh_status sync_stream(hh_ctx* x, void* stream) {
  HH_HIP(hipStreamSynchronize(static_cast<hipStream_t>(stream)));
  return HH_OK;
}

hh_status hh_get_tokens(hh_ctx* x, int32_t seq, int32_t* out, int32_t cap, int32_t* n_out, void* stream) {
  if (!x) return HH_EINVAL;
  if (x->phase == PH_CREATED) return fail(x, HH_ESTATE, "hh_get_tokens: nothing prefilled");
  if (seq < 0 || seq >= x->B || !out || !n_out || cap < 0) return fail(x, HH_EINVAL, "hh_get_tokens: bad argument");
  hh_status st = sync_stream(x, stream);
  if (st != HH_OK) return st;
  int c = 0;
  HH_HIP(hipMemcpy(&c, x->committed + seq, sizeof(int), hipMemcpyDeviceToHost));
  if (c > cap) c = cap;
  if (c > 0) HH_HIP(hipMemcpy(out, x->out_tok + (size_t)seq * x->d.Gmax, (size_t)c * sizeof(int), hipMemcpyDeviceToHost));
  *n_out = c;
  return HH_OK;
}

hh_status hh_get_lengths(hh_ctx* x, int32_t* kv_len, int32_t* committed, int32_t* last_n, void* stream) {
  if (!x) return HH_EINVAL;
  if (x->phase == PH_CREATED) return fail(x, HH_ESTATE, "hh_get_lengths: nothing prefilled");
  hh_status st = sync_stream(x, stream);
  if (st != HH_OK) return st;
  const size_t n = (size_t)x->B * sizeof(int);
  if (kv_len) HH_HIP(hipMemcpy(kv_len, x->kv_len, n, hipMemcpyDeviceToHost));
  if (committed) HH_HIP(hipMemcpy(committed, x->committed, n, hipMemcpyDeviceToHost));
  if (last_n) HH_HIP(hipMemcpy(last_n, x->last_n, n, hipMemcpyDeviceToHost));
  return HH_OK;
}

hh_status hh_check_canaries(hh_ctx* x, int32_t* n_damaged, void* stream) {
  if (!x) return HH_EINVAL;
  if (!n_damaged) return fail(x, HH_EINVAL, "hh_check_canaries: NULL argument");
  if (!(x->cfg.kernel_flags & HH_KF_CANARIES)) return fail(x, HH_ESTATE, "hh_check_canaries: the context was created without HH_KF_CANARIES");
  hh_status st = sync_stream(x, stream);
  if (st != HH_OK) return st;
  int bad = 0;
  unsigned char buf[kCanaryBytes];
  for (size_t i = 0; i < x->canaries.size(); ++i) {
    HH_HIP(hipMemcpy(buf, static_cast<char*>(x->cfg.workspace) + x->canaries[i], kCanaryBytes, hipMemcpyDeviceToHost));
    for (size_t k = 0; k < kCanaryBytes; ++k)
      if (buf[k] != kCanaryByte) {
        if (bad++ == 0) {
          char msg[160];
          snprintf(msg, sizeof msg, "hh_check_canaries: guard %zu of %zu (workspace offset %zu) overwritten at byte %zu", i,
                   x->canaries.size(), x->canaries[i], k);
          x->err = msg;
        }
        break;
      }
  }
  *n_damaged = bad;
  return HH_OK;
}

hh_status hh_get_acceptance(hh_ctx* x, uint64_t* accepted, uint64_t* tested, void* stream) {
  if (!x) return HH_EINVAL;
  if (x->phase == PH_CREATED) return fail(x, HH_ESTATE, "hh_get_acceptance: nothing prefilled");
  if (!accepted || !tested) return fail(x, HH_EINVAL, "hh_get_acceptance: NULL argument");
  hh_status st = sync_stream(x, stream);
  if (st != HH_OK) return st;
  unsigned long long v[2] = {0, 0};
  HH_HIP(hipMemcpy(v, x->acc_stats, sizeof v, hipMemcpyDeviceToHost));
  *accepted = v[0]; *tested = v[1];
  return HH_OK;
}

hh_status hh_get_round(hh_ctx* x, int32_t* drafts, int32_t* targets, void* stream) {
  if (!x) return HH_EINVAL;
  if (x->phase == PH_CREATED) return fail(x, HH_ESTATE, "hh_get_round: nothing prefilled");
  hh_status st = sync_stream(x, stream);
  if (st != HH_OK) return st;
  const Dims& d = x->d;
  if (drafts && x->k > 0)
    HH_HIP(hipMemcpy2D(drafts, (size_t)x->k * sizeof(int), x->drafts, (size_t)d.Kmax * sizeof(int),
                       (size_t)x->k * sizeof(int), x->B, hipMemcpyDeviceToHost));
  if (targets)
    HH_HIP(hipMemcpy2D(targets, (size_t)(x->k + 1) * sizeof(int), x->targets, (size_t)(d.Kmax + 1) * sizeof(int),
                       (size_t)(x->k + 1) * sizeof(int), x->B, hipMemcpyDeviceToHost));
  return HH_OK;
}

hh_status hh_get_logits(hh_ctx* x, int32_t which, float* out, void* stream) {
  if (!x) return HH_EINVAL;
  if (x->phase == PH_CREATED) return fail(x, HH_ESTATE, "hh_get_logits: nothing prefilled");
  if (!out || which < 0 || which > 2) return fail(x, HH_EINVAL, "hh_get_logits: bad argument");
  if (!x->cfg.keep_logits) return fail(x, HH_ESTATE, "hh_get_logits: the context was created with keep_logits = 0");
  hh_status st = sync_stream(x, stream);
  if (st != HH_OK) return st;
  const Dims& d = x->d;
  const size_t V = d.V;
  if (which == 0) {
    if (x->k > 0)
      HH_HIP(hipMemcpy2D(out, (size_t)x->k * V * 4, x->logits_d, (size_t)d.Kmax * V * 4, (size_t)x->k * V * 4, x->B,
                         hipMemcpyDeviceToHost));
  } else if (which == 1) {
    HH_HIP(hipMemcpy(out, x->logits_v, (size_t)x->B * (x->k + 1) * V * 4, hipMemcpyDeviceToHost));
  } else {
    HH_HIP(hipMemcpy(out, x->logits_p, (size_t)x->B * V * 4, hipMemcpyDeviceToHost));
  }
  return HH_OK;
}

hh_status hh_get_state(hh_ctx* x, int32_t layer, float* ssm, float* conv, void* stream) {
  if (!x) return HH_EINVAL;
  if (x->phase == PH_CREATED) return fail(x, HH_ESTATE, "hh_get_state: nothing prefilled");
  const Dims& d = x->d;
  if (layer < 0 || layer >= d.L) return fail(x, HH_EINVAL, "hh_get_state: layer out of range");
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (conv) HH_HIP(launch_export_state(d, x->layers_dev + layer, x->kv_len, x->B, x->export_buf, s));
  hh_status st = sync_stream(x, stream);
  if (st != HH_OK) return st;
  if (ssm)
    HH_HIP(hipMemcpy(ssm, x->layers_host[layer].S, (size_t)x->B * d.Hm * d.P * d.N * 4, hipMemcpyDeviceToHost));
  if (conv) HH_HIP(hipMemcpy(conv, x->export_buf, (size_t)x->B * d.conv_dim * 3 * 4, hipMemcpyDeviceToHost));
  return HH_OK;
}

hh_status hh_get_draft_state(hh_ctx* x, int32_t layer, float* ssm, float* conv, void* stream) {
  if (!x) return HH_EINVAL;
  if (x->phase == PH_CREATED) return fail(x, HH_ESTATE, "hh_get_draft_state: nothing prefilled");
  if (!x->strict) return fail(x, HH_ESTATE, "hh_get_draft_state: needs cfg.draft_state_mode = 1");
  const Dims& d = x->d;
  if (layer < 0 || layer >= d.L) return fail(x, HH_EINVAL, "hh_get_draft_state: layer out of range");
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (conv) HH_HIP(launch_export_state(d, x->layers_ms_dev + layer, x->kv_len, x->B, x->export_buf, s));
  hh_status st = sync_stream(x, stream);
  if (st != HH_OK) return st;
  if (ssm)
    HH_HIP(hipMemcpy(ssm, x->layers_ms_host[layer].S, (size_t)x->B * d.Hm * d.P * d.N * 4, hipMemcpyDeviceToHost));
  if (conv) HH_HIP(hipMemcpy(conv, x->export_buf, (size_t)x->B * d.conv_dim * 3 * 4, hipMemcpyDeviceToHost));
  return HH_OK;
}

hh_status hh_get_kv(hh_ctx* x, int32_t layer, int32_t seq, int32_t n_tokens, float* k, float* v, void* stream) {
  if (!x) return HH_EINVAL;
  if (x->phase == PH_CREATED) return fail(x, HH_ESTATE, "hh_get_kv: nothing prefilled");
  const Dims& d = x->d;
  if (layer < 0 || layer >= d.L || seq < 0 || seq >= x->B || n_tokens < 0 || n_tokens > d.max_seq || !k || !v)
    return fail(x, HH_EINVAL, "hh_get_kv: bad argument");
  // staged through the (idle between calls) projection buffer, a slab of tokens at a time
  const size_t per_tok = (size_t)d.Hkv * d.Dh;
  const size_t cap = (size_t)d.Bmax * d.Tmax * d.ldzx / 2;
  const int slab = (int)(cap / per_tok);
  if (slab < 1) return fail(x, HH_ECAPACITY, "hh_get_kv: staging buffer too small");
  hipStream_t s = static_cast<hipStream_t>(stream);
  float* kb = x->zx;
  float* vb = x->zx + cap;
  for (int t0 = 0; t0 < n_tokens; t0 += slab) {
    const int nt = n_tokens - t0 < slab ? n_tokens - t0 : slab;
    HH_HIP(launch_export_kv(d, x->layers_dev + layer, x->page_table, seq, t0, nt, kb, vb, s));
    hh_status st = sync_stream(x, stream);
    if (st != HH_OK) return st;
    HH_HIP(hipMemcpy(k + (size_t)t0 * per_tok, kb, (size_t)nt * per_tok * 4, hipMemcpyDeviceToHost));
    HH_HIP(hipMemcpy(v + (size_t)t0 * per_tok, vb, (size_t)nt * per_tok * 4, hipMemcpyDeviceToHost));
  }
  return HH_OK;
}

hh_status hh_time_kind(hh_ctx* x, int32_t phase, int32_t kind, int32_t k, int32_t reps, float* total_ms,
                       int32_t* launches, void* stream) {
  if (!x) return HH_EINVAL;
  if (x->phase != PH_READY) return fail(x, HH_ESTATE, "hh_time_kind: needs a prefilled context with no round in flight");
  const Dims& d = x->d;
  if ((phase != HH_PHASE_DRAFT && phase != HH_PHASE_VERIFY) || kind < 0 || kind > HH_K_LM_HEAD || reps < 1 ||
      k < 0 || k > d.Kmax || !total_ms || !launches)
    return fail(x, HH_EINVAL, "hh_time_kind: bad argument");
  hipStream_t s = static_cast<hipStream_t>(stream);
  const bool full = phase == HH_PHASE_VERIFY;
  const int B = x->B, T = full ? k + 1 : 1;
  hipEvent_t e0, e1;
  HH_HIP(hipEventCreate(&e0));
  HH_HIP(hipEventCreate(&e1));
  // positions and tokens of an ordinary pass, so that every kernel sees valid inputs
  HH_HIP(launch_gather_tokens(x->pending, x->drafts, d.Kmax, B, T, full ? 1 : 0, 0, x->tok, x->kv_len, x->pos0, s));
  HH_HIP(launch_embed(d, x->embed, x->tok, B * T, x->h, s));
  const bool prof = x->prof_on;
  x->prof_on = true;            // serial launches on one stream (no side stream), but no event pairs:
  const size_t cap = x->prof_ev.size();
  x->only_kind = kind;
  hh_status st = HH_OK;
  int n = 0;
  {
    // suppress the per-launch events by pretending the record is full
    std::vector<hipEvent_t> saved;
    saved.swap(x->prof_ev);
    x->prof_ev.resize(kProfCap * 2, nullptr);
    HH_HIP(hipEventRecord(e0, s));
    for (int r = 0; r < reps && st == HH_OK; ++r) {
      if (kind == HH_K_LM_HEAD) {
        st = run_head(x, x->h, B * T, T, full ? x->logits_v : x->logits_d, full ? d.V : d.Kmax * d.V,
                      full ? x->targets : x->drafts, full ? d.Kmax + 1 : d.Kmax, 0, s);
        n += 1;
      } else {
        st = run_layers(x, x->layers_host, full, nullptr, B, T, nullptr, 0, full ? 0 : 2, pick_splits(x->cfg, d, B, T, x->len_upper), false, s);
        n += d.L;
      }
    }
    hipError_t er = hipEventRecord(e1, s);
    x->prof_ev.swap(saved);
    (void)cap;
    x->only_kind = -1;
    x->prof_on = prof;
    if (st != HH_OK) return st;
    HH_HIP(er);
  }
  HH_HIP(hipEventSynchronize(e1));
  HH_HIP(hipEventElapsedTime(total_ms, e0, e1));
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  *launches = n;
  return HH_OK;
}

hh_status hh_profile(hh_ctx* x, int32_t enable) {
  if (!x) return HH_EINVAL;
  if (enable) {
    for (hipEvent_t e : x->prof_ev) (void)hipEventDestroy(e);
    x->prof_ev.clear();
    x->prof_tag.clear();
  }
  x->prof_on = enable != 0;
  return HH_OK;
}

hh_status hh_profile_read(hh_ctx* x, int32_t n_tags, int32_t* launches, float* total_ms, void* stream) {
  if (!x) return HH_EINVAL;
  if (!launches || !total_ms || n_tags < 1) return fail(x, HH_EINVAL, "hh_profile_read: bad argument");
  hh_status st = sync_stream(x, stream);
  if (st != HH_OK) return st;
  for (int i = 0; i < n_tags; ++i) { launches[i] = 0; total_ms[i] = 0.f; }
  for (size_t i = 0; i < x->prof_tag.size(); ++i) {
    const int tag = x->prof_tag[i];
    if (tag < 0 || tag >= n_tags) continue;
    float ms = 0.f;
    HH_HIP(hipEventElapsedTime(&ms, x->prof_ev[2 * i], x->prof_ev[2 * i + 1]));
    launches[tag] += 1;
    total_ms[tag] += ms;
  }
  return HH_OK;
}

const char* hh_last_error(const hh_ctx* ctx) { return ctx ? ctx->err.c_str() : g_create_error.c_str(); }

}  // extern "C"
