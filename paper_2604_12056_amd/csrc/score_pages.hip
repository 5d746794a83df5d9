// QUEST page scoring, per-query top pages and their union per KV head
// (paper: Preliminaries, Sparse Attention Algorithms for LLMs; Methodology, eq. quest_union).
//
//   page_scores   s[b,j,r,p] = sum_c max(q_c*min_c, q_c*max_c)   r = a*G + hg over the active slots a
//   select_pages  per row r: exact top-K by radix select on order-preserving keys (ties:
//                 smaller page); the last row of a KV head to finish ORs the row bitmaps,
//                 compacts the union into an ascending page list and, inside losa_step,
//                 also builds the attention kernel's inputs
//
// Everything that decides a set is integer work on float bit patterns: no float atomics,
// so the outcome does not depend on scheduling.
#include "losa_device.h"
#include "losa_internal.h"

namespace losa {

// What the scoring kernel leaves ready for the selection kernel that follows it: the ticket
// counter of every (sequence, KV head) at zero, and - when no token is active, so that no
// selection workgroup will run - empty results.
struct ScoreAux {
  int32_t* tickets;
  int32_t* sel_count;
  int32_t* ucount;   // nullable
  int32_t* mrows;    // nullable
  __device__ void reset(int head, int M) const {
    tickets[head] = 0;
    if (M <= 0) {
      sel_count[head] = 0;
      if (ucount) {
        ucount[head] = 0;
        mrows[head] = 0;
      }
    }
  }
};

// In-kernel locality pruning (paper: Methodology, Locality Pruning): when `delta` is given,
// every scoring workgroup ranks the block's locality scores itself (B <= kRankTokens, one
// thread per token, ranking by counting as in the stand-alone kernel) instead of reading an
// active list some earlier launch produced, and the first workgroup of each sequence writes
// mask / list / count out for the kernels that follow.  This replaces the hand-over at the end
// of the locality kernel (store, wait, ticket, reload, rank) by B compares per thread here.
constexpr int kRankTokens = 256;
constexpr int kMaxTilesPerWg = 4;   // 64-page tiles one scoring workgroup may take
struct RankArgs {
  const float* delta;     // [batch*B] locality scores; NULL: use the active list passed to the kernel
  int mode, n;            // LOSA_SEL_TOPK / FRACTION (n = count), LOSA_SEL_THRESHOLD or LOSA_SEL_MASS (tau)
  float tau;
  uint8_t* mask;          // outputs, written by workgroup (0, 0, b)
  int32_t* active_idx;
  int32_t* active_count;
};

constexpr int kScorePages = 32;  // pages per workgroup in page_scores
constexpr int kScoreRows = 32;   // query rows staged at a time

template <typename T, int D>
__global__ __launch_bounds__(256) void page_scores_kernel(KvView kv, Shape sh, const T* __restrict__ q,
                                                          const int32_t* __restrict__ active_idx,
                                                          const int32_t* __restrict__ active_count,
                                                          float* __restrict__ scores, ScoreAux aux) {
  constexpr int V = Vec16<T>::n;
  constexpr int PT = kScorePages, RC = kScoreRows;
  __shared__ float mn[PT][D + 1];
  __shared__ float mx[PT][D + 1];
  __shared__ float qs[RC][D];
  const int b = blockIdx.z, j = blockIdx.y, p0 = blockIdx.x * PT, tid = threadIdx.x;
  const int base = kv.page_indptr[b];
  const int P = seq_pages(kv, sh, b);
  const int n = min(active_count[b], sh.B);
  const int M = n * sh.G;
  if (blockIdx.x == 0 && tid == 0) aux.reset(b * sh.Hkv + j, M);
  if (p0 >= P) return;
  if (M <= 0) return;

  constexpr int VPR = D / V;  // vectors per metadata row
  for (int v = tid; v < PT * 2 * VPR; v += 256) {
    const int pg = v / (2 * VPR), rem = v % (2 * VPR), which = rem / VPR, cv = rem % VPR;
    float f[V];
#pragma unroll
    for (int e = 0; e < V; ++e) f[e] = 0.f;
    if (p0 + pg < P) {
      const int phys = kv.page_indices[base + p0 + pg];
      if ((unsigned)phys < (unsigned)kv.num_pages) {
        const uint4 raw = reinterpret_cast<const uint4*>((const T*)kv.meta + (((size_t)phys * sh.Hkv + j) * 2 + which) * D)[cv];
        widen16(raw, f, T());
      }
    }
    float* dst = which ? &mx[pg][cv * V] : &mn[pg][cv * V];
#pragma unroll
    for (int e = 0; e < V; ++e) dst[e] = f[e];
  }

  const int pg = tid % PT, rs = tid / PT;  // 8 row lanes
  for (int r0 = 0; r0 < M; r0 += RC) {
    __syncthreads();
    for (int v = tid; v < RC * VPR; v += 256) {
      const int rr = v / VPR, cv = v % VPR, r = r0 + rr;
      float f[V];
#pragma unroll
      for (int e = 0; e < V; ++e) f[e] = 0.f;
      if (r < M) {
        const int a = r / sh.G, hg = r % sh.G;
        const int tok = active_idx[(size_t)b * sh.B + a];
        if ((unsigned)tok < (unsigned)sh.B) {
          const uint4 raw = reinterpret_cast<const uint4*>(q + (((size_t)b * sh.B + tok) * sh.Hq + j * sh.G + hg) * D)[cv];
          widen16(raw, f, T());
        }
      }
#pragma unroll
      for (int e = 0; e < V; ++e) qs[rr][cv * V + e] = f[e];
    }
    __syncthreads();
    for (int rr = rs; rr < RC && r0 + rr < M; rr += 256 / PT) {
      float s = 0.f;
#pragma unroll 8
      for (int c = 0; c < D; ++c) {
        const float qv = qs[rr][c];
        s += fmaxf(qv * mn[pg][c], qv * mx[pg][c]);
      }
      if (p0 + pg < P)
        scores[(((size_t)b * sh.Hkv + j) * sh.rows_max + r0 + rr) * sh.max_pages + p0 + pg] = s;
    }
  }
}

// Matrix-core page scoring for bfloat16.  Since max >= min per channel,
//   max(q*min, q*max) = q+ * max + q- * min      with q+ = max(q,0), q- = min(q,0),
// and one of the two terms is exactly zero, so each channel contributes the same exact
// product either way: the score matrix of a KV head is the dense contraction
//   S^T [pages x rows] = [max | min] (pages x 2d) . [Q+ | Q-]^T (2d x rows).
// A wavefront takes 16 pages: its A operands are the 16 metadata rows read straight from
// memory (one 16-byte load per lane and k-step, 8 KiB per wavefront all in flight at once);
// the B operands are the sign-split query fragments.  Output leaves the matrix core as 4
// consecutive pages per lane and query row: one 16-byte store.
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;

template <int D, int MAXT>
__global__ __launch_bounds__(256) void page_scores_mfma_kernel(KvView kv, Shape sh, const bf16_t* __restrict__ q,
                                                               const int32_t* __restrict__ active_idx,
                                                               const int32_t* __restrict__ active_count,
                                                               float* __restrict__ scores, ScoreAux aux, RankArgs ra,
                                                               int tpw) {
  // A workgroup scores tpw (<= MAXT, a template argument so that the one-tile form carries no
  // code for more) consecutive 64-page tiles: what it does before
  // the first product (ranking, query staging) is then paid once for all of them, and a
  // batch of many sequences still fits the machine in one round of workgroups.
  const int bx = blockIdx.x * tpw, j = blockIdx.y, b = blockIdx.z;
  constexpr int KS = D / 32;
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6, l16 = lane & 15, qd = lane >> 4;
  const int base = kv.page_indptr[b];
  const int P = seq_pages(kv, sh, b);
  const int p0 = bx * 64 + wave * 16;
  __shared__ __attribute__((aligned(16))) float sdelta[kRankTokens];
  __shared__ int act_list[kRankTokens];
  __shared__ int rscan[17];
  const bool ranked = ra.delta != nullptr;   // uniform over the launch
  const bool writes_active = ranked && bx == 0 && j == 0;   // this workgroup publishes the active set
  auto tile_phys = [&](int t) {   // page whose metadata rows lane l16 feeds for tile t of this workgroup (clamped: always valid)
    const int pg = max(0, min((bx + t) * 64 + wave * 16 + l16, P - 1));
    int ph = P > 0 ? kv.page_indices[base + pg] : 0;
    return (unsigned)ph < (unsigned)kv.num_pages ? ph : 0;
  };
  if (bx * 64 >= P && !writes_active) {                      // no pages here and nothing to publish
    if (bx == 0 && tid == 0) aux.reset(b * sh.Hkv + j, 0);   // (P == 0: nothing will be selected either)
    return;
  }

  // Everything that can be fetched before the active set is known is requested first: the
  // locality scores, then the metadata rows of this wavefront's pages (two dependent round
  // trips: page table, then the rows), which then travel while the ranking runs.
  float my_delta = 0.f;
  if (ranked && tid < sh.B) my_delta = ra.delta[(size_t)b * sh.B + tid];
  // A operands: metadata rows of page p0 + l16 (a valid page is read for lanes past P, never stored).
  // The page ids of all of this workgroup's tiles are fetched at once.
  int physv[MAXT];
#pragma unroll
  for (int t = 0; t < MAXT; ++t) physv[t] = t < tpw ? tile_phys(t) : 0;
  bf16x8_t amin[KS], amax[KS];
  auto load_meta = [&](int phys, bf16x8_t (&mn)[KS], bf16x8_t (&mx)[KS]) {
    const bf16_t* mrow = (const bf16_t*)kv.meta + ((size_t)phys * sh.Hkv + j) * 2 * D;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      mn[ks] = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const uint4*>(mrow + ks * 32 + qd * 8));
      mx[ks] = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const uint4*>(mrow + D + ks * 32 + qd * 8));
    }
  };
  load_meta(physv[0], amin, amax);

  int M;
  if (ranked) {
    const int B = sh.B;   // <= kRankTokens (checked by the launcher)
    sdelta[tid] = tid < B ? my_delta : -INFINITY;   // 256 threads, kRankTokens entries: the padding never outranks a token
    __syncthreads();
    int act = 0, rank = 0;
    if (tid < B && ra.mode != LOSA_SEL_THRESHOLD) {
      // four scores per LDS read, reads independent of one another (a scalar loop pays one LDS
      // latency per token)
#pragma unroll 4
      for (int k = 0; k < B; k += 4) {
        const f32x4_t dk = *reinterpret_cast<const f32x4_t*>(&sdelta[k]);
#pragma unroll
        for (int e = 0; e < 4; ++e)   // bitwise on purpose: the short-circuit forms compile to a branch per element
          rank += (int)(dk[e] > my_delta) | ((int)(dk[e] == my_delta) & (int)(k + e < tid));
      }
    }
    int n_take = ra.n;
    if (ra.mode == LOSA_SEL_MASS) {
      // Cumulative-mass rule, as in the stand-alone kernel: scores in descending order, summed
      // in that order in float by one thread; A is the shortest prefix reaching tau * total.
      __shared__ float sorted[kRankTokens];
      __shared__ int s_take;
      if (tid < B) sorted[rank] = my_delta;
      __syncthreads();
      if (tid == 0) {
        float total = 0.f;
        for (int k = 0; k < B; ++k) total += sorted[k];
        const float target = ra.tau * total;
        int cnt = 0;
        if (total > 0.f) {
          float run = 0.f;
          cnt = B;
          for (int k = 0; k < B; ++k) {
            run += sorted[k];
            if (run >= target) {
              cnt = k + 1;
              break;
            }
          }
          if (!(ra.tau > 0.f)) cnt = 0;
        }
        s_take = cnt;
      }
      __syncthreads();
      n_take = s_take;
    }
    if (tid < B) act = ra.mode == LOSA_SEL_THRESHOLD ? my_delta > ra.tau : rank < n_take;
    int n_act;
    const int pos = block_exclusive_scan(act, rscan, &n_act);
    if (act) act_list[pos] = tid;
    if (writes_active) {
      if (tid < B) ra.mask[(size_t)b * B + tid] = (uint8_t)act;
      if (act) ra.active_idx[(size_t)b * B + pos] = tid;
      for (int i = n_act + tid; i < B; i += 256) ra.active_idx[(size_t)b * B + i] = -1;
      if (tid == 0) ra.active_count[b] = n_act;
    }
    __syncthreads();   // act_list is read below
    M = n_act * sh.G;
  } else {
    M = min(active_count[b], sh.B) * sh.G;
  }
  if (bx == 0 && tid == 0) aux.reset(b * sh.Hkv + j, M);
  if (bx * 64 >= P) return;   // whole workgroup (only the publishing one gets here without pages)
  if (M <= 0) return;

  float* out_base = scores + ((size_t)b * sh.Hkv + j) * sh.rows_max * sh.max_pages;

  // Query rows go through LDS, kRows at a time, so that the four wavefronts (64 pages) fetch
  // each row once instead of once per wavefront.  A row is D bfloat16 plus 16 bytes of padding:
  // the 16 lanes that read the same 16-byte column of 16 consecutive rows then fall on
  // different banks.
  constexpr int kRows = 64, VPR = D / 8, STRIDE = D * 2 + 16;   // bytes; 64 rows cover the usual active sets in one go and keep LDS small enough for 8 workgroups per CU
  // Staged already split by sign (score = q+ . max + q- . min): the split is done once per
  // workgroup by the staging threads, not once per wavefront, tile and row tile.
  __shared__ __attribute__((aligned(16))) unsigned char qs[2][kRows * STRIDE];   // [0]: q+, [1]: q-
  bool staged = false;   // LDS holds rows [0, kRows) of this head's active queries
#pragma unroll
  for (int t = 0; t < MAXT; ++t) {
    if (t >= tpw || (bx + t) * 64 >= P) break;   // uniform over the workgroup
    const int p0t = p0 + t * 64;
    const bool live = p0t < P;   // a wavefront without pages still helps staging and keeps the barriers
    const bool vec_ok = (sh.max_pages & 3) == 0 && p0t + 16 <= P;
    // the next tile's metadata rows travel while this tile is scored
    bf16x8_t nmin[KS], nmax[KS];
    if (t + 1 < MAXT && t + 1 < tpw) load_meta(physv[t + 1 < MAXT ? t + 1 : t], nmin, nmax);
    for (int r0 = 0; r0 < M; r0 += kRows) {
      const int nrows = min(kRows, M - r0);
      if (!(staged && M <= kRows)) {   // with a single chunk of rows the first tile's staging serves all tiles
        if (staged) __syncthreads();   // everyone is done reading the previous chunk
        // staging: thread -> (row, 16-byte vector); token ids first, then all the row loads
        constexpr int PER = kRows * VPR / 256;
        int tok[PER];
#pragma unroll
        for (int k = 0; k < PER; ++k) {
          const int rr = min((tid + 256 * k) / VPR, nrows - 1);
          tok[k] = ranked ? act_list[(r0 + rr) / sh.G] : active_idx[(size_t)b * sh.B + (r0 + rr) / sh.G];
        }
        uint4 v[PER];
#pragma unroll
        for (int k = 0; k < PER; ++k) {
          const int rr = min((tid + 256 * k) / VPR, nrows - 1), cv = (tid + 256 * k) % VPR;
          const int tc = (unsigned)tok[k] < (unsigned)sh.B ? tok[k] : 0;
          v[k] = reinterpret_cast<const uint4*>(q + (((size_t)b * sh.B + tc) * sh.Hq + j * sh.G + (r0 + rr) % sh.G) * D)[cv];
        }
#pragma unroll
        for (int k = 0; k < PER; ++k) {
          const int rr = (tid + 256 * k) / VPR, cv = (tid + 256 * k) % VPR;
          if (rr < nrows) {
            // per 16-bit half: all-ones where the sign bit is set
            typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
            const uint32_t keep = (unsigned)tok[k] < (unsigned)sh.B ? 0xFFFFFFFFu : 0u;
            const u32x4_t x = u32x4_t{v[k].x, v[k].y, v[k].z, v[k].w} & keep;
            const u32x4_t mk = ((x >> 15) & 0x00010001u) * 0xFFFFu;
            *reinterpret_cast<u32x4_t*>(qs[0] + rr * STRIDE + cv * 16) = x & ~mk;
            *reinterpret_cast<u32x4_t*>(qs[1] + rr * STRIDE + cv * 16) = x & mk;
          }
        }
        __syncthreads();
        staged = true;
      }
      if (!live) continue;
      for (int t0 = 0; t0 < nrows; t0 += 16) {
        const int rr = t0 + l16;           // row of this lane inside the chunk (may be past nrows: masked below)
        uint4 qpos[KS], qneg[KS];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
          qpos[ks] = *reinterpret_cast<const uint4*>(qs[0] + min(rr, nrows - 1) * STRIDE + ks * 64 + qd * 16);
          qneg[ks] = *reinterpret_cast<const uint4*>(qs[1] + min(rr, nrows - 1) * STRIDE + ks * 64 + qd * 16);
        }
        f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
          acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(amax[ks], __builtin_bit_cast(bf16x8_t, qpos[ks]), acc, 0, 0, 0);
          acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(amin[ks], __builtin_bit_cast(bf16x8_t, qneg[ks]), acc, 0, 0, 0);
        }
        // acc[e] = score of page p0t + 4*qd + e for query row r0 + t0 + l16
        if (rr < nrows) {
          float* dst = out_base + (size_t)(r0 + rr) * sh.max_pages + p0t + 4 * qd;
          if (vec_ok) {
            __builtin_nontemporal_store(acc, reinterpret_cast<f32x4_t*>(dst));
          } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
              if (p0t + 4 * qd + e < P) dst[e] = acc[e];
          }
        }
      }
    }
    if (t + 1 < MAXT && t + 1 < tpw) {
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        amin[ks] = nmin[ks];
        amax[ks] = nmax[ks];
      }
    }
  }
}

// float -> uint32 whose unsigned order is the float order (-0 and +0 made equal first).
__device__ __forceinline__ uint32_t order_key(float f) {
  f += 0.0f;
  const uint32_t u = __float_as_uint(f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// Device-wide hand-over used by the selection kernel: every row's workgroup stores its pick
// bitmap, then takes a ticket; the workgroup that draws the last ticket of a (sequence, KV
// head) ORs the rows, compacts the union and builds what the attention kernel consumes.
// (How the stores are made visible to that workgroup is described at the hand-over.)
struct SelectOut {
  int32_t* topk_out;    // nullable [batch, B, Hq, topk]
  int32_t* sel_pages;   // [batch, Hkv, cap] logical pages of the union, ascending
  int32_t* sel_count;   // [batch, Hkv]
  int cap;
  uint32_t* rowmaps;    // workspace [heads, rows_max, words]: pick bitmap of every query row
  int32_t* tickets;     // workspace [heads], zero on entry (zeroed by the scoring kernel), zero on exit
  AttnPrepared prep;    // entries == NULL: do not build the attention inputs
  const void* q;        // query tensor (for the gather into prep.q_act)
  const int32_t* active_idx;
  bool rows_known;      // the grid has exactly one workgroup per existing row (+ the gather workgroup)
  bool bitmaps_only;    // heads with at most kUnionRows rows: leave the row bitmaps to the attention kernel (no hand-over, no union, no list)
};

// Inclusive suffix scan over 256 histogram buckets by one wavefront: lane l owns buckets
// 255-4l .. 252-4l (descending).  Returns through LDS the bucket where the running count from
// the top first reaches `need`, how many are still needed inside that bucket, and how many
// keys the bucket holds.
__device__ __forceinline__ void find_bucket_wave0(const uint32_t* hist, int need, uint32_t* s_bucket, int* s_need,
                                                  int* s_count) {
  const int lane = threadIdx.x;   // caller guarantees threadIdx.x < 64
  int c[4], tot = 0;
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    c[k] = (int)hist[255 - 4 * lane - k];
    tot += c[k];
  }
  const int incl = wave_inclusive_scan(tot);
  int above = incl - tot;   // keys in buckets owned by lower lanes (= higher buckets)
  if (above < need && incl >= need) {
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      if (above < need && above + c[k] >= need) {
        *s_bucket = (uint32_t)(255 - 4 * lane - k);
        *s_need = need - above;
        *s_count = c[k];
      }
      above += c[k];
    }
  }
}

// A bucket of at most this many keys is ranked directly instead of by further histogram passes.
template <int E> struct RankMax { static constexpr int value = E >= 32 ? 256 : 64; };

// LDS state of radix_kth.  hist must be all zero when radix_kth is entered (the caller clears it
// early; the first barrier inside radix_kth orders that clear before its first use).
template <int E, int NT>
struct RadixLds {
  uint32_t hist[256];
  __attribute__((aligned(16))) uint32_t cand[RankMax<E>::value];
  uint32_t bucket, lo[NT / 64], hi[NT / 64], kth;
  int need, count, ncand;
};

// Radix select.  It runs on keys relative to the row's smallest key and starts at the highest
// bit of the row's largest one (a block min/max finds both), so the first histogram is already
// spread over many buckets instead of piling every key onto the few exponent patterns the
// scores share.  As soon as the bucket that holds the K-th key has at most RankMax<E> keys,
// those are copied to LDS and ranked against each other directly (one thread per candidate),
// which replaces the remaining histogram passes.
//
// The K-th largest of the workgroup's keys (thread t holds key[0..nmine)), Kp < number of keys:
// on return every key > prefix is among the Kp largest, and of the keys == prefix the first
// `need` in page order are (all of them when ties_cut is false).  On return the keys have been
// rebased (the row minimum subtracted); prefix is in the same units.  all: Kp covers every key,
// nothing to find.  Every thread of the workgroup must call it.
template <int E, int NT>
__device__ __forceinline__ void radix_kth(uint32_t (&key)[E], int nmine, int Kp, bool all, RadixLds<E, NT>& L,
                                          uint32_t& prefix, int& need, bool& ties_cut) {
  const int tid = threadIdx.x;
  constexpr int NW = NT / 64;
  uint32_t pmask = 0u;
  prefix = 0u;
  need = Kp;
  ties_cut = true;   // false once it is known that every key equal to the K-th is picked
  if (!all) {
    // highest differing bit of the row's keys
    uint32_t lo = 0xFFFFFFFFu, hi = 0u;
#pragma unroll
    for (int i = 0; i < E; ++i)
      if (i < nmine) {
        lo = min(lo, key[i]);
        hi = max(hi, key[i]);
      }
    lo = wave_min_u32(lo);
    hi = wave_max_u32(hi);
    if ((tid & 63) == 0) {
      L.lo[tid >> 6] = lo;
      L.hi[tid >> 6] = hi;
    }
    if (tid == 0) L.ncand = 0;
    __syncthreads();
    lo = L.lo[0];
    hi = L.hi[0];
#pragma unroll
    for (int w = 1; w < NW; ++w) {
      lo = min(lo, L.lo[w]);
      hi = max(hi, L.hi[w]);
    }
    // Keys are taken relative to the row minimum from here on (order is unchanged): the
    // first digit then resolves the row's actual range into 128..256 buckets wherever that
    // range lies, instead of splitting at whatever power of two happens to fall inside it.
#pragma unroll
    for (int i = 0; i < E; ++i) key[i] -= lo;   // entries past the row's pages are never looked at
    hi -= lo;
    const uint32_t diff = hi;
    if (diff != 0u) {
      const int hb = 31 - __clz((int)diff);          // no key has a bit above hb
      pmask = hb >= 31 ? 0u : ~((2u << hb) - 1u);
      prefix = 0u;
      bool first_pass = true;   // the histogram was cleared at the top (a barrier has passed since)
      for (int shift = max(hb - 7, 0);; shift = max(shift - 8, 0)) {
        if (!first_pass) {
          if (tid < 256) L.hist[tid] = 0u;
          __syncthreads();
        }
        first_pass = false;
#pragma unroll
        for (int i = 0; i < E; ++i)
          if (i < nmine && (key[i] & pmask) == prefix) atomicAdd(&L.hist[(key[i] >> shift) & 255u], 1u);
        __syncthreads();
        if (tid < 64) find_bucket_wave0(L.hist, need, &L.bucket, &L.need, &L.count);
        __syncthreads();
        // bits of the digit that lie above bit hb (only when hb < 7) are common to all keys
        const uint32_t dmask = 0xFFu << shift;
        prefix = (prefix & ~dmask) | (L.bucket << shift);
        pmask |= dmask;
        need = L.need;
        const int count = L.count;
        if (shift == 0) {
          ties_cut = count != need;
          break;
        }
        if (count <= RankMax<E>::value) {
          // the K-th key is the need-th largest of `count` candidates: rank them directly.
          // Candidates are packed wavefront by wavefront (one LDS atomic each); their order
          // in the array does not matter to the ranks.
          int mine_n = 0;
#pragma unroll
          for (int i = 0; i < E; ++i) mine_n += (int)(i < nmine) & (int)((key[i] & pmask) == prefix);
          const int incl = wave_inclusive_scan(mine_n);
          int wbase = 0;
          if ((tid & 63) == 63) wbase = atomicAdd(&L.ncand, incl);
          wbase = __builtin_amdgcn_readlane(wbase, 63);
          int at = wbase + incl - mine_n;
#pragma unroll
          for (int i = 0; i < E; ++i)
            if (i < nmine && (key[i] & pmask) == prefix) L.cand[at++] = key[i];
          // pad to a whole number of 16-candidate steps with keys that rank below everything
          if (tid < 16 && count + tid < RankMax<E>::value) L.cand[count + tid] = 0u;
          __syncthreads();
          if (tid < count) {
            const uint32_t mine = L.cand[tid];
            int gt = 0, ge = 0;
            for (int u = 0; u < count; u += 16) {
              uint4 c4[4];
#pragma unroll
              for (int k = 0; k < 4; ++k) c4[k] = *reinterpret_cast<const uint4*>(&L.cand[u + 4 * k]);
#pragma unroll
              for (int k = 0; k < 4; ++k) {
                gt += (c4[k].x > mine) + (c4[k].y > mine) + (c4[k].z > mine) + (c4[k].w > mine);
                ge += (c4[k].x >= mine) + (c4[k].y >= mine) + (c4[k].z >= mine) + (c4[k].w >= mine);
              }
            }
            // the padding keys (0) count as ">= mine" only for a key that is 0 itself
            if (mine == 0u) ge -= ((count + 15) & ~15) - count;
            if (gt < need && need <= ge) {   // every thread that holds the K-th value writes the same
              L.kth = mine;
              L.need = need - gt;
              L.count = ge - gt;
            }
          }
          __syncthreads();
          prefix = L.kth;
          pmask = 0xFFFFFFFFu;
          need = L.need;
          ties_cut = L.count != need;
          break;
        }
      }
    } else {
      prefix = 0u;          // every key is the same: ties by page order
      pmask = 0xFFFFFFFFu;
    }
  } else {
    __syncthreads();
  }
}

// Per-query top pages, register resident (thread t of NT owns the E consecutive pages
// [t*E, t*E+E); P <= NT*E: 256 threads x 8 up to 2048 pages, 1024 threads x 8 or 16 beyond),
// fused with the union and the hand-over described above.
template <int E, int NT, bool MULTI>
__global__ __launch_bounds__(NT) void select_pages_kernel(KvView kv, Shape sh, const int32_t* __restrict__ active_count,
                                                           const float* __restrict__ scores, int topk, SelectOut out,
                                                           int rpw) {
  // A workgroup selects for up to rpw query rows, one after the other (the next row's
  // scores travel while the current row is selected).  rpw is 1 unless the grid would not fit
  // the machine in one round: a second round of workgroups costs more than a second row.
  // MULTI = false is the one-row form (rpw == 1) without the loop's register cost.
  constexpr int WORDS = NT * E / 32;
  __shared__ RadixLds<E, NT> rl;
  __shared__ uint32_t rowbits[WORDS];   // this row's picks
  __shared__ uint32_t ubits[WORDS];     // union of the head's rows (used by the workgroup that builds it)
  __shared__ int s_last;
  __shared__ int scan[17];
  // A workgroup's rows are r_first, r_first + r_step, ...: dealt round-robin over the row workgroups, so
  // that when the grid was sized for more rows than exist (a count only the device knows) the rows
  // that do exist still spread over as many workgroups as possible.
  const int r_step = MULTI ? (int)gridDim.x - 1 : 1;
  const int r_first = blockIdx.x, j = blockIdx.y, b = blockIdx.z, tid = threadIdx.x;
  const int head = b * sh.Hkv + j;
  const int p_first_all = tid * E;
  const int p_first = p_first_all;
  // When the host knows the row count (every workgroup of the grid has a row), the row's
  // scores are fetched before anything else: the address depends on kernel arguments only,
  // so these loads travel together with the loads of the counts below (entries past the
  // sequence's pages are masked later).  Otherwise they wait until the row is known to exist.
  float raw[E];
  auto load_row = [&](float (&dst)[E], int r) {   // thread t: pages [t*E, t*E+E), 32 or 64 contiguous bytes
    const float* row = scores + ((size_t)head * sh.rows_max + min(r, sh.rows_max - 1)) * sh.max_pages;
    if (p_first + E <= sh.max_pages && (sh.max_pages & 3) == 0) {
#pragma unroll
      for (int i = 0; i < E; i += 4) {
        const f32x4_t v = *reinterpret_cast<const f32x4_t*>(row + p_first + i);
        dst[i] = v[0];
        dst[i + 1] = v[1];
        dst[i + 2] = v[2];
        dst[i + 3] = v[3];
      }
    } else {
#pragma unroll
      for (int i = 0; i < E; ++i) dst[i] = row[min(p_first + i, sh.max_pages - 1)];
    }
  };
  if (out.rows_known) load_row(raw, r_first);
  const int n_act = min(active_count[b], sh.B);
  const int M = n_act * sh.G;
  const int base = kv.page_indptr[b];
  const int P = min(seq_pages(kv, sh, b), NT * E);   // (the launcher picks NT * E >= the page limit)
  const int L = kv.seq_lens[b];

  if (blockIdx.x == gridDim.x - 1) {
    // The extra workgroup of every (sequence, head) gathers the head's active query rows into
    // the dense buffer the attention kernel reads, off the path of the selection.  Indices are
    // clamped so that every load can be issued before the one it depends on has been checked.
    if (out.prep.entries == nullptr || M <= 0) return;
    if (out.bitmaps_only && M <= kUnionRows) {
      // nobody builds the union here, who would otherwise publish the row count; and the row slots
      // past it are cleared, so that the attention kernel can OR all slots without looking at the count
      if (tid == 0) out.prep.mrows[head] = M;
      const int wds = (sh.max_pages + 31) / 32, spare = kUnionRows - min(M, kUnionRows);
      uint32_t* slots = out.rowmaps + (size_t)head * union_region_words(sh.rows_max, wds);
      for (int i = tid; i < wds * spare; i += NT) slots[(size_t)(i / spare) * kUnionRows + (kUnionRows - spare) + i % spare] = 0u;
      // ... and the head gets its page table in the form the attention kernel consumes (physical id
      // and valid-token count of every logical page), at an address that kernel knows when it starts
      int32_t* tab = out.prep.entries + (size_t)head * sh.max_pages;
      for (int p0 = tid; p0 < P; p0 += NT * 4) {
        int ph[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) ph[k] = kv.page_indices[base + min(p0 + NT * k, P - 1)];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          const int pg = p0 + NT * k;
          if (pg < P) {
            const int nv = max(0, min(sh.g, L - pg * sh.g));
            tab[pg] = ((unsigned)ph[k] < (unsigned)kv.num_pages && ph[k] < (1 << kEntryShift)) ? (ph[k] | (nv << kEntryShift)) : 0;
          }
        }
      }
    }
    constexpr int QV = 4;   // 16-byte vectors per thread per sweep
    const int vpr = sh.d / 8;
    const bf16_t* q = (const bf16_t*)out.q;
    uint4* dst = reinterpret_cast<uint4*>(out.prep.q_act + (size_t)head * sh.rows_max * sh.d);
    for (int v0 = tid; v0 < M * vpr; v0 += NT * QV) {
      int tok[QV];
#pragma unroll
      for (int k = 0; k < QV; ++k) tok[k] = out.active_idx[(size_t)b * sh.B + min((v0 + NT * k) / vpr, M - 1) / sh.G];
      uint4 qv[QV];
#pragma unroll
      for (int k = 0; k < QV; ++k) {
        const int rr = min((v0 + NT * k) / vpr, M - 1), cv = (v0 + NT * k) % vpr;
        const int tc = (unsigned)tok[k] < (unsigned)sh.B ? tok[k] : 0;
        qv[k] = reinterpret_cast<const uint4*>(q + (((size_t)b * sh.B + tc) * sh.Hq + j * sh.G + rr % sh.G) * sh.d)[cv];
      }
#pragma unroll
      for (int k = 0; k < QV; ++k)
        if (v0 + NT * k < M * vpr)
          dst[v0 + NT * k] = (unsigned)tok[k] < (unsigned)sh.B ? qv[k] : make_uint4(0u, 0u, 0u, 0u);
    }
    return;
  }
  if (r_first >= M) return;
  if (!out.rows_known) load_row(raw, r_first);
  const int words = (sh.max_pages + 31) / 32;
  const int Kp = min(topk, P);
  const int nmine_all = max(0, min(E, P - p_first));   // pages of this thread that exist
  // LDS that must start at zero is cleared now, while the scores are still on their way
  for (int w = tid; w < WORDS; w += NT) {
    rowbits[w] = 0u;
    ubits[w] = 0u;
  }
  if (tid < 256) rl.hist[tid] = 0u;
  const int r_end = MULTI ? M : r_first + 1;
#pragma unroll 1
  for (int r = r_first; r < r_end; r += r_step) {
    // Per-thread constants are made opaque once per row: otherwise everything derived from them
    // (bit masks, predicates, addresses) is computed once ahead of the loop and kept in registers
    // across it, which costs half the kernel's occupancy.
    int p_first_r = p_first_all, nmine_r = nmine_all;
    if constexpr (MULTI) asm volatile("" : "+v"(p_first_r), "+v"(nmine_r));
    const int p_first = p_first_r, nmine = nmine_r;
    const int a = r / sh.G, h = j * sh.G + r % sh.G;
    int32_t* tk = out.topk_out ? out.topk_out + (((size_t)b * sh.B + a) * sh.Hq + h) * topk : nullptr;
    uint32_t key[E];
#pragma unroll
    for (int i = 0; i < E; ++i) key[i] = i < nmine ? order_key(raw[i]) : 0u;
    if (r + r_step < r_end) load_row(raw, r + r_step);   // the next row's scores, on their way during this row's selection

    const bool all = Kp >= P;
    uint32_t prefix;
    int need;
    bool ties_cut;
    radix_kth<E, NT>(key, nmine, Kp, all, rl, prefix, need, ties_cut);
    // picks: keys above the K-th, plus the first `need` keys equal to it in page order.
    // (Bitwise logic on purpose: the short-circuit forms compile to a branch per key.)
    int my_eq = 0, my_gt = 0;
    if (ties_cut || tk) {   // the counts feed the scans below and nothing else
  #pragma unroll
      for (int i = 0; i < E; ++i) {
        const int in = i < nmine;
        my_gt += in & ((int)all | (int)(key[i] > prefix));
        my_eq += in & (int)!all & (int)(key[i] == prefix);
      }
    }
    int tot_eq;
    int eq_rank = 0;   // block-uniform branch: ties_cut derives from LDS values every thread read
    if (ties_cut) eq_rank = block_exclusive_scan(my_eq, scan, &tot_eq);
    int pos = 0, tot_sel = 0;
    if (tk) pos = block_exclusive_scan(my_gt + (ties_cut ? max(0, min(my_eq, need - eq_rank)) : my_eq), scan, &tot_sel);
    uint32_t bits[(E + 31) / 32];
  #pragma unroll
    for (int w = 0; w < (E + 31) / 32; ++w) bits[w] = 0u;
  #pragma unroll
    for (int i = 0; i < E; ++i) {
      const int in = i < nmine;
      const int eq = in & (int)!all & (int)(key[i] == prefix);
      const int sel = (in & ((int)all | (int)(key[i] > prefix))) | (eq & ((int)!ties_cut | (int)(eq_rank < need)));
      eq_rank += eq;
      bits[i / 32] |= (uint32_t)sel << ((p_first + i) & 31);
      if (tk && sel) tk[pos++] = p_first + i;
    }
    if (E >= 32) {
  #pragma unroll
      for (int w = 0; w < (E + 31) / 32; ++w) rowbits[p_first / 32 + w] = bits[w];   // this thread owns whole words
    } else {
      if (bits[0]) atomicOr(&rowbits[p_first / 32], bits[0]);
    }
    if (tk)
      for (int k = tot_sel + tid; k < topk; k += NT) tk[k] = -1;
    __syncthreads();
    // ---- hand-over: the last row of this (sequence, head) builds the union.
    // The row bitmap travels in agent-scope atomic stores (written through to memory, past the
    // per-die L2 slices); ordering is "my stores have completed (wait count zero), then my
    // ticket".  A full agent-scope fence would also work but writes back and invalidates whole
    // L2 slices, once per workgroup.
    uint32_t* myrow = out.rowmaps + (size_t)head * union_region_words(sh.rows_max, words) + (size_t)r * words;
    if (out.bitmaps_only && M <= kUnionRows) {   // read by the next launch: ordinary stores, into the word-major layout
      uint32_t* slots = out.rowmaps + (size_t)head * union_region_words(sh.rows_max, words);
      if (r < kUnionRows)
        for (int w = tid; w < words; w += NT) slots[(size_t)w * kUnionRows + r] = w < WORDS ? rowbits[w] : 0u;
    } else {
      for (int w = tid; w < words; w += NT)
        __hip_atomic_store(&myrow[w], w < WORDS ? rowbits[w] : 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    if (r + r_step < r_end) {
      // the row bitmap has been read out (the stores above take their data at issue): clear the
      // LDS state of the next row; its first barrier (inside radix_kth) orders these writes
      __syncthreads();
      for (int w = tid; w < WORDS; w += NT) rowbits[w] = 0u;
      if (tid < 256) rl.hist[tid] = 0u;
    }
  }
  if (out.bitmaps_only && M <= kUnionRows) return;
  const int rows_done = (r_end - 1 - r_first) / r_step + 1;
  __builtin_amdgcn_s_waitcnt(0);
  __atomic_signal_fence(__ATOMIC_SEQ_CST);
  __syncthreads();
  // the ticket counts rows: the workgroup whose rows complete the head's M builds the union
  if (tid == 0)
    s_last = __hip_atomic_fetch_add(&out.tickets[head], rows_done, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + rows_done == M;
  __syncthreads();
  if (!s_last) return;
  if (tid == 0) out.tickets[head] = 0;
  // Union of the M row bitmaps -> ascending page list (+ page entries for the attention kernel).
  // Pages are handled a thread each, kTailPages per thread: their physical ids are fetched
  // before the bits are known, together with the row bitmaps, so the tail is one memory
  // round trip.  A page's slot in the list is the popcount prefix of its bitmap word plus
  // the set bits below it in the word: no serial walk, stores ascend with the thread id.
  const int wordsP = (P + 31) / 32;
  int32_t* sel = out.sel_pages + (size_t)head * out.cap;
  int32_t* ent = out.prep.entries ? out.prep.entries + (size_t)head * sh.max_pages : nullptr;
  __shared__ int wordbase[WORDS];
  int phys[E];
  if (ent) {
#pragma unroll
    for (int i = 0; i < E; ++i)   // (an empty sequence has no entry of its own in the page table)
      phys[i] = P > 0 ? kv.page_indices[base + min(tid + NT * i, P - 1)] : 0;
  }
  const uint32_t* maps = out.rowmaps + (size_t)head * union_region_words(sh.rows_max, words);
  {
    // Thread t ORs bitmap word (t mod nw) of every `groups`-th row in registers, 16 independent
    // loads at a time (a loop of load-then-use would pay one memory latency per iteration),
    // and only the per-thread results meet in LDS.  Agent-scope atomic loads: they are served
    // from the coherence point, not from a line this compute unit or its die's L2 holds.  The
    // writers' stores went through to memory (agent scope) and had completed before their
    // tickets were drawn, but the bitmap regions of two (sequence, head) pairs can share a
    // cache line (rows * words * 4 need not be a multiple of the line), and the union
    // workgroup of the other pair may have fetched that line while this pair's rows were
    // still being written.
    for (int w0 = 0; w0 < wordsP; w0 += NT) {
      const int nw = min(NT, wordsP - w0);
      const int groups = NT / nw;
      const int ww = w0 + tid % nw, rg = tid / nw;
      if (rg < groups) {
        uint32_t acc = 0u;
        for (int r0 = rg; r0 < M; r0 += groups * 16) {
          uint32_t v[16];
#pragma unroll
          for (int k = 0; k < 16; ++k) {
            const int rr = r0 + groups * k;
            v[k] = __hip_atomic_load(&maps[(size_t)min(rr, M - 1) * words + ww], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          }
#pragma unroll
          for (int k = 0; k < 16; ++k) acc |= (r0 + groups * k < M) ? v[k] : 0u;
        }
        if (acc) atomicOr(&ubits[ww], acc);
      }
    }
  }
  __syncthreads();
  int base_out = 0;
  for (int w0 = 0; w0 < WORDS; w0 += NT) {   // exclusive popcount prefix per word
    const int w = w0 + tid;
    const int c = w < wordsP ? __popc(ubits[w]) : 0;
    int total;
    const int ex = block_exclusive_scan(c, scan, &total);
    if (w < WORDS) wordbase[w] = base_out + ex;
    base_out += total;
  }
  __syncthreads();
  // Every load of this thread has landed by now; saying so keeps the stores below from each
  // waiting for the one before it (loads and stores share one in-order counter).
  __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0) only
  uint32_t wd[E];
  int wb[E];
#pragma unroll
  for (int i = 0; i < E; ++i) {   // all LDS reads first: one latency, not one per page
    wd[i] = ubits[(tid + NT * i) >> 5];
    wb[i] = wordbase[(tid + NT * i) >> 5];
  }
#pragma unroll
  for (int i = 0; i < E; ++i) {
    const int page = tid + NT * i;
    if (page < P && ((wd[i] >> (page & 31)) & 1u)) {
      const int at = wb[i] + __popc(wd[i] & ((1u << (page & 31)) - 1u));
      if (at < out.cap) {
        sel[at] = page;
        if (ent) {
          const int nv = max(0, min(sh.g, L - page * sh.g));
          const int ph = phys[i];
          ent[at] = ((unsigned)ph < (unsigned)kv.num_pages && ph < (1 << kEntryShift)) ? (ph | (nv << kEntryShift)) : 0;
        }
      }
    }
  }
  const int U = min(base_out, out.cap);
  if (tid == 0) {
    out.sel_count[head] = U;
    if (ent) {
      out.prep.ucount[head] = U;
      out.prep.mrows[head] = M;
    }
  }
}

// One page set per (sequence, KV head) shared by all of its active queries (not in the paper:
// the other reading of a per-KV-head budget): every page takes the largest bound any active
// query of the head gives it, and the K best pages are kept, so exactly min(K, P) pages are
// read.  One workgroup per (sequence, head): the row maxima are taken in registers on the
// order-preserving keys (the same pages-per-thread layout as select_pages_kernel), the K-th
// is found by the same radix select, and the list is emitted in ascending page order by a
// prefix sum over the threads' pick counts - no hand-over between workgroups is needed.
template <int E, int NT>
__global__ __launch_bounds__(NT) void shared_select_kernel(KvView kv, Shape sh, const int32_t* __restrict__ active_count,
                                                            const float* __restrict__ scores, int topk,
                                                            int32_t* __restrict__ sel_pages,
                                                            int32_t* __restrict__ sel_count, int cap) {
  __shared__ RadixLds<E, NT> rl;
  __shared__ int scan[17];
  const int j = blockIdx.x, b = blockIdx.y, tid = threadIdx.x;
  const int head = b * sh.Hkv + j;
  const int p_first = tid * E;
  if (tid < 256) rl.hist[tid] = 0u;
  const int M = min(active_count[b], sh.B) * sh.G;
  const int P = min(seq_pages(kv, sh, b), NT * E);
  if (M <= 0 || P <= 0) {
    if (tid == 0) sel_count[head] = 0;
    return;
  }
  const int nmine = max(0, min(E, P - p_first));
  const bool vec = p_first + E <= sh.max_pages && (sh.max_pages & 3) == 0;
  const float* rows = scores + (size_t)head * sh.rows_max * sh.max_pages;
  uint32_t key[E];
#pragma unroll
  for (int i = 0; i < E; ++i) key[i] = 0u;
  constexpr int RB = E >= 16 ? 2 : 4;   // rows in flight (fewer with more keys per thread: 128 registers at 1024 threads)
  for (int r0 = 0; r0 < M; r0 += RB) {
    float v[RB][E];
#pragma unroll
    for (int rr = 0; rr < RB; ++rr) {
      const float* row = rows + (size_t)min(r0 + rr, M - 1) * sh.max_pages;   // clamped: the repeat changes no maximum
      if (vec) {
#pragma unroll
        for (int i = 0; i < E; i += 4) {
          const float4 x = *reinterpret_cast<const float4*>(row + p_first + i);
          v[rr][i] = x.x;
          v[rr][i + 1] = x.y;
          v[rr][i + 2] = x.z;
          v[rr][i + 3] = x.w;
        }
      } else {
#pragma unroll
        for (int i = 0; i < E; ++i) v[rr][i] = row[min(p_first + i, sh.max_pages - 1)];
      }
    }
#pragma unroll
    for (int rr = 0; rr < RB; ++rr)
#pragma unroll
      for (int i = 0; i < E; ++i) key[i] = max(key[i], order_key(v[rr][i]));
  }
#pragma unroll
  for (int i = 0; i < E; ++i)
    if (i >= nmine) key[i] = 0u;

  const int Kp = min(topk, P);
  const bool all = Kp >= P;
  uint32_t prefix;
  int need;
  bool ties_cut;
  radix_kth<E, NT>(key, nmine, Kp, all, rl, prefix, need, ties_cut);

  int my_eq = 0, my_gt = 0;
#pragma unroll
  for (int i = 0; i < E; ++i) {
    const bool in = i < nmine;
    my_gt += in && (all || key[i] > prefix);
    my_eq += in && !all && key[i] == prefix;
  }
  int tot_eq, eq_rank = 0;
  if (ties_cut) eq_rank = block_exclusive_scan(my_eq, scan, &tot_eq);
  const int mine = my_gt + (ties_cut ? max(0, min(my_eq, need - eq_rank)) : my_eq);
  int total;
  int pos = block_exclusive_scan(mine, scan, &total);
  int32_t* sel = sel_pages + (size_t)head * cap;
#pragma unroll
  for (int i = 0; i < E; ++i) {
    const bool in = i < nmine;
    bool take = in && (all || key[i] > prefix);
    if (in && !all && key[i] == prefix) {
      take = !ties_cut || eq_rank < need;
      ++eq_rank;
    }
    if (take) {
      if (pos < cap) sel[pos] = p_first + i;
      ++pos;
    }
  }
  if (tid == 0) sel_count[head] = min(total, cap);
}

hipError_t launch_page_scores(hipStream_t st, int dtype, const KvView& kv, const Shape& sh, int batch,
                              int max_seq_pages, const void* q, const int32_t* active_idx,
                              const int32_t* active_count, float* scores, int32_t* tickets, int32_t* sel_count,
                              const AttnPrepared* prep, const InKernelRanking* ranking, long workgroups_per_round) {
  if (batch <= 0) return hipSuccess;
  ScoreAux aux{tickets, sel_count, prep ? prep->ucount : nullptr, prep ? prep->mrows : nullptr};
  RankArgs ra{nullptr, 0, 0, 0.f, nullptr, nullptr, nullptr};
  if (ranking) {
    if (dtype != LOSA_BF16 || sh.B > kRankTokens) return hipErrorInvalidValue;
    ra = RankArgs{ranking->delta, ranking->mode, ranking->n, ranking->tau, ranking->mask, ranking->active_idx,
                  ranking->active_count};
  }
  dim3 grid((max_seq_pages + kScorePages - 1) / kScorePages, sh.Hkv, batch);
  if (grid.x == 0) grid.x = 1;
  if (dtype == LOSA_BF16) {
    // One 64-page tile per workgroup while the grid fits the machine in one round; beyond
    // that, more tiles per workgroup rather than a second round.
    const long tiles = max((max_seq_pages + 63) / 64, 1);
    const long round = max(workgroups_per_round, 1L);
    int tpw = (int)((tiles * sh.Hkv * batch + round - 1) / round);
    tpw = max(1, min(tpw, kMaxTilesPerWg));
    dim3 mgrid((unsigned)((tiles + tpw - 1) / tpw), sh.Hkv, batch);
    if (sh.d == 128) {
      if (tpw == 1)
        page_scores_mfma_kernel<128, 1><<<mgrid, 256, 0, st>>>(kv, sh, (const bf16_t*)q, active_idx, active_count, scores, aux, ra, 1);
      else
        page_scores_mfma_kernel<128, kMaxTilesPerWg><<<mgrid, 256, 0, st>>>(kv, sh, (const bf16_t*)q, active_idx, active_count, scores, aux, ra, tpw);
    } else {
      if (tpw == 1)
        page_scores_mfma_kernel<64, 1><<<mgrid, 256, 0, st>>>(kv, sh, (const bf16_t*)q, active_idx, active_count, scores, aux, ra, 1);
      else
        page_scores_mfma_kernel<64, kMaxTilesPerWg><<<mgrid, 256, 0, st>>>(kv, sh, (const bf16_t*)q, active_idx, active_count, scores, aux, ra, tpw);
    }
  } else {
    if (sh.d == 128)
      page_scores_kernel<float, 128><<<grid, 256, 0, st>>>(kv, sh, (const float*)q, active_idx, active_count, scores, aux);
    else
      page_scores_kernel<float, 64><<<grid, 256, 0, st>>>(kv, sh, (const float*)q, active_idx, active_count, scores, aux);
  }
  return hipGetLastError();
}

hipError_t launch_select_pages(hipStream_t st, const KvView& kv, const Shape& sh, int batch, int max_seq_pages,
                               const void* q, const int32_t* active_idx, const int32_t* active_count,
                               const float* scores, int topk, int32_t* topk_out, int32_t* sel_pages,
                               int32_t* sel_count, int cap, uint32_t* rowmaps, int32_t* tickets,
                               const AttnPrepared* prep, int rows_hint, long workgroups_per_round, bool bitmaps_only) {
  if (batch <= 0) return hipSuccess;
  if (bitmaps_only && (!prep || topk_out)) return hipErrorInvalidValue;
  SelectOut out;
  out.bitmaps_only = bitmaps_only;
  out.topk_out = topk_out;
  out.sel_pages = sel_pages;
  out.sel_count = sel_count;
  out.cap = cap;
  out.rowmaps = rowmaps;
  out.tickets = tickets;
  out.prep = prep ? *prep : AttnPrepared{nullptr, nullptr, nullptr, nullptr};
  out.q = q;
  out.active_idx = active_idx;
  out.rows_known = rows_hint >= 1;
  // rows_hint: an upper bound on |A| * G the host happens to know (0: none); rows past it get no workgroup
  const int rows = rows_hint >= 1 && rows_hint < sh.rows_max ? rows_hint : sh.rows_max;
  const int pages = max_seq_pages < sh.max_pages ? max_seq_pages : sh.max_pages;
  // One row per workgroup while the grid fits the machine in one round (seven 256-thread
  // workgroups per CU for the one-row form, five for the several-row form, by their register
  // counts; one 1024-thread workgroup); beyond that, up to four rows per workgroup.
  const bool small = pages <= 256 * 8;
  // (without the union hand-over at its end a workgroup is short enough that a grid somewhat past
  // one round still beats two rows per workgroup: measured on 16 sequences of 36 rows x 4 heads)
  const long fit_one = workgroups_per_round > 0 ? workgroups_per_round : (small ? (bitmaps_only ? 10L : 7L) * 256 : 256L);
  const long fit_many = workgroups_per_round > 0 ? workgroups_per_round : (small ? 5L * 256 : 256L);
  // (a count the host does not know: the grid has a workgroup for every possible row, and those past
  // the count leave at once; sized as if a quarter of the rows existed, so that a typical active set
  // is not made to share workgroups for the sake of rows that are not there)
  const long wgs = (long)(rows + 1) * sh.Hkv * batch / (out.rows_known ? 1 : 4);
  int rpw = wgs <= fit_one ? 1 : (int)((wgs + fit_many - 1) / fit_many);
  rpw = rpw < 1 ? 1 : (rpw > 4 ? 4 : rpw);
  dim3 grid((rows + rpw - 1) / rpw + 1, sh.Hkv, batch);   // + the query-gather workgroup
  // Few keys per thread keep the unrolled code small (it has to come through the instruction
  // cache on every launch) and the loads contiguous: longer sequences get more threads, not
  // more keys per thread.
  if (pages <= 256 * 8)
    if (rpw == 1)
      select_pages_kernel<8, 256, false><<<grid, 256, 0, st>>>(kv, sh, active_count, scores, topk, out, 1);
    else
      select_pages_kernel<8, 256, true><<<grid, 256, 0, st>>>(kv, sh, active_count, scores, topk, out, rpw);
  else if (pages <= 1024 * 8)
    if (rpw == 1)
      select_pages_kernel<8, 1024, false><<<grid, 1024, 0, st>>>(kv, sh, active_count, scores, topk, out, 1);
    else
      select_pages_kernel<8, 1024, true><<<grid, 1024, 0, st>>>(kv, sh, active_count, scores, topk, out, rpw);
  else if (pages <= kMaxSelectPages)
    if (rpw == 1)
      select_pages_kernel<16, 1024, false><<<grid, 1024, 0, st>>>(kv, sh, active_count, scores, topk, out, 1);
    else
      select_pages_kernel<16, 1024, true><<<grid, 1024, 0, st>>>(kv, sh, active_count, scores, topk, out, rpw);
  else
    return hipErrorInvalidValue;
  return hipGetLastError();
}

hipError_t launch_shared_select(hipStream_t st, const KvView& kv, const Shape& sh, int batch, int max_seq_pages,
                                const int32_t* active_count, const float* scores, int topk, int32_t* sel_pages,
                                int32_t* sel_count, int cap) {
  if (batch <= 0) return hipSuccess;
  dim3 grid(sh.Hkv, batch);
  const int pages = max_seq_pages < sh.max_pages ? max_seq_pages : sh.max_pages;
  if (pages <= 256 * 8)
    shared_select_kernel<8, 256><<<grid, 256, 0, st>>>(kv, sh, active_count, scores, topk, sel_pages, sel_count, cap);
  else if (pages <= 1024 * 8)
    shared_select_kernel<8, 1024><<<grid, 1024, 0, st>>>(kv, sh, active_count, scores, topk, sel_pages, sel_count, cap);
  else if (pages <= kMaxSelectPages)
    shared_select_kernel<16, 1024><<<grid, 1024, 0, st>>>(kv, sh, active_count, scores, topk, sel_pages, sel_count, cap);
  else
    return hipErrorInvalidValue;
  return hipGetLastError();
}

}  // namespace losa
