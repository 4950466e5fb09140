// Many-row dense projections (more than 96 activation rows: verification of large batches,
// prefill passes) on the matrix cores with both operands staged through LDS.
//
// Operands are the same as in the register-tiled kernel: the weights in packed tiles (a 16 x 32
// tile is 1 KB in MFMA operand order) and the activations as three bf16 planes in the same order
// (x = t0 + t1 + t2 exactly, written by split_rows_kernel).  A fragment therefore is 1 KB
// contiguous in global memory and in LDS alike: it is copied with one 16-byte load per lane and
// read back with one 16-byte LDS read per lane, without bank conflicts and without any transpose.
//
// A workgroup of eight wavefronts owns 16 weight fragments (16 strips of 16 weight rows, or 8
// gate/up strip pairs) x 12 row tiles (256 x 192 outputs) and a range of K.  Per step of 32
// columns it brings 16 + 36 fragments (52 KB) into LDS once; wavefront (wn, wm) multiplies its
// 4 weight fragments with its 6 row tiles (72 MFMAs per step, 96 accumulator registers).  A
// compute unit takes in well under 30 bytes per cycle this way (the register-tiled kernel, where
// every wavefront loads its own operands, asks for 85 and is bound by exactly that).  The copies
// are LDS-direct loads (global_load_lds_dwordx4: lane l's 16 bytes land at the wavefront's LDS
// base + 16 l, no registers in between) into three to six stages of LDS (what fits 160 KB): the
// copies of step s + stages - 1 are issued before step s is multiplied, so that many steps of
// copies are in flight behind the MFMAs; one workgroup barrier per step.
#pragma once
#include "hh_internal.h"
#include "wave_ops.h"
#include "trace.h"

namespace hh {

typedef __bf16 lds_bf16x8 __attribute__((ext_vector_type(8)));
typedef float lds_f32x4 __attribute__((ext_vector_type(4)));
union LFrag {
  uint4 u;
  lds_bf16x8 v;
};

constexpr int kLdsWaves = 8;                  // 4 along the weight rows x 2 along the activation rows
constexpr int kLdsA = 16;                     // weight fragments per workgroup and step
// MTW = activation row tiles per wavefront (6, or 1..3 for passes of at most 96 rows): the
// workgroup covers 2 MTW row tiles, 6 MTW plane fragments per step
constexpr int lds_row_tiles(int mtw) { return 2 * mtw; }
constexpr int lds_frags(int mtw) { return kLdsA + 6 * mtw; }
constexpr int lds_stage_bytes(int mtw) { return lds_frags(mtw) * 1024; }
constexpr int lds_items(int mtw) { return (lds_frags(mtw) + kLdsWaves - 1) / kLdsWaves; }   // 16-byte copies per thread and step

struct LdsGemmArgs {
  const uint16_t* planes; int m_tiles, KST;    // split activations: block (row tile, step, term) of 512 elements
  const uint16_t* W; const uint16_t* W2;       // packed tiles (W2: the "up" matrix for SwiGLU)
  float* Y; int ldy; const float* R2;
  float* partial;                              // [ksplit][NF][M][N] when ksplit > 1
  int M, N, n_tiles;
  int n_blocks, m_blocks, ksplit, ksteps;      // grid = n_blocks * m_blocks * ksplit
  unsigned long long* row_best; int store;     // EPI_STORE: per-row argmax keys (atomic maxima); store = 0: Y not written
  int xcd_ranges;                              // 1: tiles numbered in per-XCD ranges (see the kernel)
  uint16_t* planes_out; int out_KST;           // EPI_SWIGLU, ksplit == 1: result as split planes (out_KST = N / 32 steps per row tile) instead of Y
};

// LDS stages of the copy pipeline: as many as fit 160 KB, at most 6 (three for 192-row workgroups)
constexpr int lds_stages(int mtw) { return 160 * 1024 / lds_stage_bytes(mtw) > 6 ? 6 : 160 * 1024 / lds_stage_bytes(mtw); }

template <int EPI, int MTW>
__global__ __launch_bounds__(64 * kLdsWaves) void gemm_lds_kernel(const LdsGemmArgs a) {
  constexpr int NSTAGE = lds_stages(MTW);
  constexpr int NF = EPI == EPI_SWIGLU ? 2 : 1;
  constexpr int NS = 4 / NF;                   // strips (strip pairs) per wavefront
  constexpr int SPB = kLdsA / NF;              // strips (pairs) per workgroup
  constexpr int ROW_TILES = lds_row_tiles(MTW), FRAGS = lds_frags(MTW), STAGE = lds_stage_bytes(MTW), ITEMS = lds_items(MTW);
  static_assert(ITEMS >= 3 && ITEMS <= 7 && kLdsA == 2 * kLdsWaves, "two weight fragments and one to five plane fragments per wavefront and step");
  extern __shared__ __align__(16) unsigned char smem_raw[];
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wn = wave & 3, wm = wave >> 2;
  const int g = lane >> 4, n = lane & 15;
  // Workgroups are handed to the 8 XCDs (each with an L2 of its own) in turn: workgroup i runs on XCD i % 8.
  // The tiles are numbered so that each XCD works on one contiguous range of them: XCD x takes the tiles
  // x * q + min(x, r) ... (q, r = quotient and remainder of the grid size by 8) in the order it receives its
  // workgroups.  Consecutive tiles share the K range and the weights (m block fastest), so the workgroups that
  // read the same weights meet in one L2 instead of fetching them into all eight.
  int lid = blockIdx.x;
  if (a.xcd_ranges) {
    const int q = gridDim.x >> 3, r = gridDim.x & 7, x = blockIdx.x & 7;
    lid = x * q + min(x, r) + (blockIdx.x >> 3);
  }
  const int mb = lid % a.m_blocks, nb = (lid / a.m_blocks) % a.n_blocks, kp = lid / (a.m_blocks * a.n_blocks);
  const int k_begin = kp * a.ksteps, k_end = min(a.KST, k_begin + a.ksteps);
  const int n_steps = k_end - k_begin;

  // ---- the copies of this thread: wavefront w copies the fragments w, w + 8, ... (a fragment is
  // 1 KB: one 16-byte copy per lane); the first two are weight fragments, the rest plane
  // fragments.  Every wavefront issues exactly ITEMS copies per step (a wavefront without a
  // fragment of its own in the last round repeats its previous one), so that "at most ITEMS
  // copies outstanding" means for each of them: the copies of the step before the newest one
  // have landed.
  const uint16_t* src[ITEMS];
  unsigned dst[ITEMS];      // byte offset of the fragment within a stage
  int stride[ITEMS];        // elements from one step's fragment to the next step's
#pragma unroll
  for (int j = 0; j < ITEMS; ++j) {
    const int frag = wave + kLdsWaves * j < FRAGS ? wave + kLdsWaves * j : wave + kLdsWaves * (j - 1);
    dst[j] = (unsigned)frag * 1024;
    if (frag < kLdsA) {
      // fragment wn' * 4 + i of the workgroup: NF == 1: strip wn' * 4 + i; NF == 2: pair wn' * 2 + i % 2 of matrix i / 2
      const int w4 = frag >> 2, i = frag & 3;
      const int strip = nb * SPB + (NF == 2 ? w4 * 2 + (i & 1) : frag);
      const uint16_t* base = (NF == 2 && i >= 2) ? a.W2 : a.W;
      src[j] = base + ((size_t)min(strip, a.n_tiles - 1) * a.KST + k_begin) * 512 + lane * 8;
      stride[j] = 512;
    } else {
      const int pf = frag - kLdsA, rt = pf / 3, term = pf - rt * 3;
      const int mt = min(mb * ROW_TILES + rt, a.m_tiles - 1);
      src[j] = a.planes + (((size_t)mt * a.KST + k_begin) * 3 + term) * 512 + lane * 8;
      stride[j] = 1536;
    }
  }
  // The copies are issued through inline assembly (M0 = LDS byte address of the wavefront's 1 KB
  // slot): issued through the compiler's builtin, every LDS read after them is made to wait for
  // ALL outstanding copies, which would serialise the pipeline.  The waits are explicit below.
  typedef __attribute__((address_space(3))) void* lptr_t;
  const unsigned lds0 = (unsigned)(size_t)(lptr_t)smem_raw;
  auto copy16 = [](const void* gsrc, unsigned lds_byte_address) {
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(gsrc), "s"(lds_byte_address) : "memory", "m0");
  };
#define HH_LDS_COPY1(j, s_, b_) \
  if (ITEMS > (j)) copy16(src[(j) < ITEMS ? (j) : 0] + s_ * (size_t)stride[(j) < ITEMS ? (j) : 0], b_ + dst[(j) < ITEMS ? (j) : 0])
#define HH_LDS_COPY(step, stage)                                                                       \
  do {                                                                                                 \
    const size_t s_ = (size_t)min((step), n_steps - 1);   /* past the end: the last step again */      \
    const unsigned b_ = lds0 + (unsigned)(stage) * STAGE;                                              \
    HH_LDS_COPY1(0, s_, b_); HH_LDS_COPY1(1, s_, b_); HH_LDS_COPY1(2, s_, b_); HH_LDS_COPY1(3, s_, b_); \
    HH_LDS_COPY1(4, s_, b_); HH_LDS_COPY1(5, s_, b_); HH_LDS_COPY1(6, s_, b_);                         \
  } while (0)
  // the copies of the NSTAGE - 2 newest steps may still be in flight; everything older has landed
#define HH_LDS_WAIT_PREVIOUS() asm volatile("s_waitcnt vmcnt(%0)" ::"n"((NSTAGE - 2) * ITEMS) : "memory")
  static_assert((NSTAGE - 2) * ITEMS <= 63, "vmcnt is a 6-bit counter");

  lds_f32x4 acc[NF][NS][MTW];
#pragma unroll
  for (int f = 0; f < NF; ++f)
#pragma unroll
    for (int t = 0; t < NS; ++t)
#pragma unroll
      for (int m = 0; m < MTW; ++m) acc[f][t][m] = lds_f32x4{0.f, 0.f, 0.f, 0.f};

#define HH_LDS_FENCE() asm volatile("" ::: "memory")
  // one step: this wavefront's 4 weight fragments, then row tile by row tile three plane fragments
  // (the next row tile's are read while this one is multiplied)
  auto compute = [&](int stage) {
    const unsigned char* base = smem_raw + (size_t)stage * STAGE + lane * 16;
    LFrag wf[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) wf[i].u = *reinterpret_cast<const uint4*>(base + (wn * 4 + i) * 1024);
    const unsigned char* pb = base + kLdsA * 1024 + (size_t)(wm * MTW) * 3 * 1024;
    LFrag pn[3];
#pragma unroll
    for (int t = 0; t < 3; ++t) pn[t].u = *reinterpret_cast<const uint4*>(pb + t * 1024);
#pragma unroll
    for (int m = 0; m < MTW; ++m) {
      LFrag pc[3] = {pn[0], pn[1], pn[2]};
      if (m + 1 < MTW) {
#pragma unroll
        for (int t = 0; t < 3; ++t) pn[t].u = *reinterpret_cast<const uint4*>(pb + ((m + 1) * 3 + t) * 1024);
      }
      HH_LDS_FENCE();
#pragma unroll
      for (int t = 0; t < 3; ++t)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          // NF == 1: fragment i is strip i; NF == 2: fragment i is strip i % 2 of matrix i / 2
          lds_f32x4& c = acc[NF == 2 ? (i >> 1) : 0][NF == 2 ? (i & 1) : (i % NS)][m];
          c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[i].v, pc[t].v, c, 0, 0, 0);
        }
    }
  };

  // ---- pipeline: LDS stage s % NSTAGE holds step s.  Before step s is multiplied its copies
  // are waited for, a barrier makes them (and the end of step s-1 everywhere) known to all
  // wavefronts, and the copies of step s + NSTAGE - 1 are issued into the stage step s-1 has just
  // left: NSTAGE - 1 steps of copies are in flight behind the MFMAs.
  TR(0);
#pragma unroll
  for (int p = 0; p < NSTAGE - 1; ++p) HH_LDS_COPY(p, p);
  TR(1);
  int st = 0;                                    // stage of step s
#pragma unroll 1
  for (int s = 0; s < n_steps; ++s) {
    HH_LDS_WAIT_PREVIOUS();
    __syncthreads();
    const int st2 = st == 0 ? NSTAGE - 1 : st - 1;   // (s + NSTAGE - 1) % NSTAGE: the stage step s-1 has just left
    HH_LDS_COPY(s + NSTAGE - 1, st2);
    compute(st);
    HH_LDS_FENCE();
    st = st == NSTAGE - 1 ? 0 : st + 1;
  }
  TR(2);
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");     // the copies issued past the end land before the workgroup leaves
#undef HH_LDS_FENCE
#undef HH_LDS_COPY
#undef HH_LDS_COPY1
#undef HH_LDS_WAIT_PREVIOUS

  // ---- results: lane (g, n) holds D[weight row 4g+r][activation row n] of every (strip, row tile).
  // The block and lane coordinates pass through an empty asm statement first: otherwise the
  // compiler computes the addresses of all 24 tiles before the loop and keeps them in registers
  // across it (the loop then spills).
  int nb_e = nb, mb_e = mb, g_e = g, n_e = n;
  asm volatile("" : "+s"(nb_e), "+s"(mb_e), "+v"(g_e), "+v"(n_e));
  unsigned long long best[MTW];
#pragma unroll
  for (int m = 0; m < MTW; ++m) best[m] = 0ull;
  const int mt0 = mb_e * ROW_TILES + wm * MTW;
#pragma unroll
  for (int t = 0; t < NS; ++t) {
    const int strip = nb_e * SPB + wn * NS + t;
    const int row0 = strip * 16 + 4 * g_e;
    if (strip >= a.n_tiles) continue;
#pragma unroll
    for (int m = 0; m < MTW; ++m) {
      asm volatile("" ::: "memory");          // one tile after the other (interleaved, the 24 tiles' temporaries overflow the registers)
      const int am = (mt0 + m) * 16 + n_e;
      if (mt0 + m >= a.m_tiles || am >= a.M) continue;
      if (a.ksplit > 1) {
#pragma unroll
        for (int f = 0; f < NF; ++f) {
          float* p = a.partial + (((size_t)kp * NF + f) * a.M + am) * a.N + row0;
          if (row0 + 3 < a.N && (a.N & 3) == 0) *reinterpret_cast<float4*>(p) = make_float4(acc[f][t][m][0], acc[f][t][m][1], acc[f][t][m][2], acc[f][t][m][3]);
          else
#pragma unroll
            for (int r = 0; r < 4; ++r) if (row0 + r < a.N) p[r] = acc[f][t][m][r];
        }
      } else {
        float* y = a.Y + (size_t)am * a.ldy + row0;
        float v[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          v[r] = acc[0][t][m][r];
          if (EPI == EPI_SWIGLU) v[r] = v[r] / (1.0f + expf(-v[r])) * acc[NF - 1][t][m][r];
        }
        if (EPI == EPI_SWIGLU && a.planes_out != nullptr) {
          // the consumer's operand layout: block (row tile, step of 32 columns, term) of 512 elements, element
          // ((column % 32) / 8 * 16 + row % 16) * 8 + column % 8; this lane's 4 columns are half a group of 8
          uint32_t a0, a1, a2, b0, b1, b2;
          split3_bf16_pair(v[0], v[1], a0, a1, a2);
          split3_bf16_pair(v[2], v[3], b0, b1, b2);
          uint16_t* dst = a.planes_out + (((size_t)(am >> 4) * a.out_KST + (row0 >> 5)) * 3) * 512 +
                          ((((row0 & 31) >> 3) * 16 + (am & 15)) * 8 + (row0 & 7));
          *reinterpret_cast<uint2*>(dst) = make_uint2(a0, b0);
          *reinterpret_cast<uint2*>(dst + 512) = make_uint2(a1, b1);
          *reinterpret_cast<uint2*>(dst + 1024) = make_uint2(a2, b2);
          continue;
        }
        const bool vec = row0 + 3 < a.N && (a.ldy & 3) == 0;
        if (EPI == EPI_ADD) {
          if (vec) {
            const float4 o = *reinterpret_cast<const float4*>(y);
            v[0] += o.x; v[1] += o.y; v[2] += o.z; v[3] += o.w;
            if (a.R2 != nullptr) {
              const float4 o2 = *reinterpret_cast<const float4*>(a.R2 + (size_t)am * a.ldy + row0);
              v[0] += o2.x; v[1] += o2.y; v[2] += o2.z; v[3] += o2.w;
            }
          } else {
#pragma unroll
            for (int r = 0; r < 4; ++r)
              if (row0 + r < a.N) v[r] += y[r] + (a.R2 != nullptr ? a.R2[(size_t)am * a.ldy + row0 + r] : 0.f);
          }
        }
        if (EPI != EPI_STORE || a.store) {
          if (vec) *reinterpret_cast<float4*>(y) = make_float4(v[0], v[1], v[2], v[3]);
          else
#pragma unroll
            for (int r = 0; r < 4; ++r) if (row0 + r < a.N) y[r] = v[r];
        }
        if (EPI == EPI_STORE) {
#pragma unroll
          for (int r = 0; r < 4; ++r)
            if (row0 + r < a.N) { const unsigned long long key = argmax_key(v[r], row0 + r); if (key > best[m]) best[m] = key; }
        }
      }
    }
  }
  if (EPI == EPI_STORE && a.row_best != nullptr && a.ksplit == 1) {
#pragma unroll
    for (int m = 0; m < MTW; ++m) {
      unsigned long long b = best[m];
      unsigned long long o = __shfl_xor(b, 16, 64); if (o > b) b = o;
      o = __shfl_xor(b, 32, 64); if (o > b) b = o;
      const int am = (mt0 + m) * 16 + n_e;
      if (g_e == 0 && mt0 + m < a.m_tiles && am < a.M && b != 0ull) atomicMax(a.row_best + am, b);
    }
  }
  TR(3);
}

}  // namespace hh
