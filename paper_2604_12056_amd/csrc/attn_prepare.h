// Device routine that builds the prepared inputs of the matrix-core attention kernel.
#pragma once
#include "losa_device.h"
#include "losa_internal.h"

namespace losa {

// Builds the prepared inputs of attn_mfma_kernel for one (sequence, KV head): resolves the
// page list (logical ids, or every page when `list` is NULL) to entries and gathers the
// query rows of the active tokens (every token when active_idx is NULL).  One workgroup.
__device__ inline void prepare_head(const KvView& kv, const Shape& sh, int b, int j, const int32_t* list, int U,
                             const int32_t* active_idx, int n_act, const bf16_t* q, const AttnPrepared& prep) {
  const int tid = threadIdx.x, nthr = blockDim.x;
  const int head = b * sh.Hkv + j;
  const int base = kv.page_indptr[b];
  const int P = min(kv.page_indptr[b + 1] - base, sh.max_pages);
  const int L = kv.seq_lens[b];
  U = max(0, min(U, sh.max_pages));
  int32_t* ent = prep.entries + (size_t)head * sh.max_pages;
  for (int i = tid; i < U; i += nthr) {
    const int logical = list ? list[i] : i;
    int e = 0;
    if ((unsigned)logical < (unsigned)P) {
      const int ph = kv.page_indices[base + logical];
      const int nv = max(0, min(sh.g, L - logical * sh.g));
      if ((unsigned)ph < (unsigned)kv.num_pages && ph < (1 << kEntryShift)) e = ph | (nv << kEntryShift);
    }
    ent[i] = e;
  }
  const int M = max(0, min(n_act, sh.B)) * sh.G;
  const int vpr = sh.d / 8;   // 16-byte vectors per query row
  uint4* dst = reinterpret_cast<uint4*>(prep.q_act + (size_t)head * sh.rows_max * sh.d);
  for (int v = tid; v < M * vpr; v += nthr) {
    const int r = v / vpr, cv = v % vpr;
    const int a = r / sh.G, hg = r % sh.G;
    const int tok = active_idx ? active_idx[(size_t)b * sh.B + a] : a;
    uint4 val = make_uint4(0u, 0u, 0u, 0u);
    if ((unsigned)tok < (unsigned)sh.B)
      val = reinterpret_cast<const uint4*>(q + (((size_t)b * sh.B + tok) * sh.Hq + j * sh.G + hg) * sh.d)[cv];
    dst[v] = val;
  }
  if (tid == 0) {
    prep.ucount[head] = U;
    prep.mrows[head] = M;
  }
}


}  // namespace losa
