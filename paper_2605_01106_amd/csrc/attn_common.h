// Paged KV cache addressing and small helpers shared by the attention kernels.
//
// Cache layout per layer: K pages [page][kv_head][token_in_page][Dh] (a key is one contiguous
// row) and V pages [page][kv_head][Dh][token_in_page] (transposed: the values of one
// dimension for consecutive tokens are contiguous, which is the operand layout of the matrix
// cores for P x V).  page_table[b][i] is the page holding tokens i*page_tokens .. of
// sequence b.
#pragma once
#include "hh_internal.h"
#include "trace.h"
#include "wave_ops.h"

namespace hh {

// element index of K[pos][0] of one KV head
__device__ __forceinline__ size_t k_index(const Dims& d, const int* pt_row, int kvh, int pos) {
  const int page = pt_row[pos / d.page_tokens], off = pos % d.page_tokens;
  return (((size_t)page * d.Hkv + kvh) * d.page_tokens + off) * d.Dh;
}
// element index of V[pos][dim] of one KV head (consecutive pos of a page are adjacent)
__device__ __forceinline__ size_t v_index(const Dims& d, const int* pt_row, int kvh, int pos, int dim) {
  const int page = pt_row[pos / d.page_tokens], off = pos % d.page_tokens;
  return (((size_t)page * d.Hkv + kvh) * d.Dh + dim) * d.page_tokens + off;
}

}  // namespace hh
