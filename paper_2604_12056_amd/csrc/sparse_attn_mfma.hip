// Split-K paged sparse prefix attention on the gfx950 matrix cores, bfloat16 inputs
// (paper: Preliminaries, Attention Decomposition With Online Softmax; Methodology, eq. update_rule).
//
// One wavefront owns up to R*16 query rows of one KV head and walks 32-token tiles of that
// head's page list with v_mfma_f32_16x16x32_bf16:
//
//   S^T = K_tile . Q^T      A operand = 16 keys x 32 channels, read straight from the
//                           token-major key page (each lane one 16-byte load);
//                           B operand = the query fragment, resident in registers.
//   O^T += V_tile^T . P^T   A operand = 16 channels x 32 tokens, read straight from the
//                           channel-major value page (one 16-byte load per lane);
//                           B operand = P^T, which is exactly how S^T leaves the matrix core
//                           (lane = query column, 4+4 tokens), so probabilities never cross
//                           lanes and the per-row rescale factor is lane-local as well.
//
// The 16 rows of a score-product half are a chosen subset of the tile's 32 tokens such that
// each lane ends up with 8 consecutive tokens; both operands of the second product use that
// same token order, which is all a contraction needs.
//
// Two work shapes:
//   split-pages (rows <= 64, the sparse steps): the four wavefronts of a workgroup take
//       interleaved tiles, K/V go global -> registers in operand layout one tile ahead (no LDS
//       and no barrier in the main loop), and the four combine their (reference, sum, O)
//       through LDS at the end, so one partial leaves the workgroup;
//   many rows (rows > 64, e.g. the dense initialisation): eight wavefronts of 32 rows walk the
//       same tiles; a tile is fetched from memory once per workgroup, its values converted to
//       half precision, and shared through LDS (one barrier per tile).  Four independent
//       wavefronts of 64 rows, each loading every tile itself, remain as a switchable fallback.
// Tiles of a (sequence, head) list are dealt round-robin to its workgroups, so every
// workgroup gets the same number of tiles (within one) whatever the union size turns out to be.
#include <hip/hip_ext.h>
#include <math.h>

#include <type_traits>

#include "losa_device.h"
#include "losa_internal.h"

namespace losa {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;
typedef __attribute__((ext_vector_type(8))) float f32x8_t;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8_t;
typedef uint32_t u32x4v_t __attribute__((ext_vector_type(4)));   // a plain vector value (stays in registers)

constexpr float kNegBig = -1.0e30f;   // finite stand-in for "no token seen yet"

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// max over the 4 lanes {l, l^16, l^32, l^48} with the gfx950 lane-swap instructions (vector ALU,
// no LDS round trip): after a swap of a register with itself the pair holds both halves.
__device__ __forceinline__ float max_over_lane_groups(float v) {
  const unsigned u = __float_as_uint(v);
  const auto a = __builtin_amdgcn_permlane16_swap(u, u, false, false);
  const float m16 = fmaxf(__uint_as_float(a[0]), __uint_as_float(a[1]));
  const unsigned w = __float_as_uint(m16);
  const auto c = __builtin_amdgcn_permlane32_swap(w, w, false, false);
  return fmaxf(__uint_as_float(c[0]), __uint_as_float(c[1]));
}
__device__ __forceinline__ float sum_over_lane_groups(float v) {
  const unsigned u = __float_as_uint(v);
  const auto a = __builtin_amdgcn_permlane16_swap(u, u, false, false);
  const float s16 = __uint_as_float(a[0]) + __uint_as_float(a[1]);
  const unsigned w = __float_as_uint(s16);
  const auto c = __builtin_amdgcn_permlane32_swap(w, w, false, false);
  return __uint_as_float(c[0]) + __uint_as_float(c[1]);
}

template <int D, int R>
struct MergeSlot {   // LDS image of one wavefront's state: O as [row tile][channel tile][lane] 16-byte
                     // vectors (every access is lane-linear, so bank-conflict free), then ref[], sum[]
  static constexpr int kOFloats = R * (D / 16) * 64 * 4;
  static constexpr int kFloats = kOFloats + 2 * R * 16;
};

// Inputs of the matrix-core kernel are *prepared* per (sequence, KV head) by whoever decided
// the selection (the union kernel inside losa_step, or attn_prepare_kernel for the
// stand-alone entry point and the dense initialisation):
//   entries[i] = physical page id | (valid tokens << kEntryShift)   for the i-th page of the list
//   q_act      = the query rows of the active tokens, gathered densely, [rows_max, d] bfloat16
//   ucount     = number of list entries,  mrows = number of query rows (|A| * G)
// so that a wavefront can issue its page-entry loads, its query loads and the two counts all
// at once when it starts: the only dependent memory round trip left before key/value data
// flows is entries -> pages.
// F16V (shared-tile shape only): the value product runs in half precision.  The value tile is
// converted bfloat16 -> half once per workgroup while it is staged into LDS (exact for
// 2^-14 <= |v| <= 65504, truncated towards zero below that range, i.e. off by less than 2^-24,
// and held at +-65504 above it), and the numerators go to the matrix core as ONE half-precision
// operand (11 significant bits, round to nearest) instead of a bfloat16 hi + lo pair: a third
// fewer matrix products per tile and no hi/lo split on the vector ALUs.  The reference point of
// the exponentials sits 7 (log2 units) above where it would otherwise be, so that numerators use
// the upper end of the half-precision range (they stay <= 2^15) and only values below 2^-31 of
// a row's largest fall into its subnormals.
//
// UNION (split-pages shape only): there is no prepared page list.  The selection kernel left the
// pick bitmap of every query row (word-major) and a copy of the head's page table; the four
// wavefronts of a workgroup fetch a quarter of each, meet in LDS (one barrier), and then every
// wavefront ORs the quarters (lane = bitmap word), ranks the union with a popcount prefix sum,
// keeps words and ranks in LDS (in its own merge slot, which is idle until the combine), and finds
// the pages of its own tiles by rank: a binary search over the word ranks, a 5-step search inside
// the word, then the page's entry from the table in LDS (from memory for pages beyond the first
// 2048).  That is more start-up work than with a prepared list (about 2 us at 2048 pages), in
// exchange for the selection kernel's whole hand-over tail (about 4 us).
constexpr int kMaxUnionWords = kMaxSelectPages / 32;
constexpr int kTablePagesInLds = 2048;   // the first so many entries of a head's page table are kept in LDS
// LDS of the split-pages shape, in floats: the four wavefronts' merge slots, then (UNION) an area the
// workgroup fills together at start-up: each wavefront's share of the bitmap OR, and the page table.
constexpr int kUnionShared = 4 * kMaxUnionWords + kTablePagesInLds;
template <int D, int GP, int R, bool SPLIT_PAGES, int NBUF, int NWAVE = 4, bool LDS_TILES = false, bool F16V = false,
          bool UNION = false>
__device__ __forceinline__ void attn_mfma_body(AttnPrepared prep, int nchunk, int nrbg, Shape sh, KvView kv, Partials part,
                                               float scale_log2e, int m_lo, int m_hi, UnionInKernel uni, float* lds) {
  static_assert(!UNION || SPLIT_PAGES, "the union is built in the kernel only in the split-pages shape");
  static_assert(!UNION || MergeSlot<D, R>::kFloats >= 2 * kMaxUnionWords, "the union's words and ranks do not fit a merge slot");
  constexpr int kSlotStride = MergeSlot<D, R>::kFloats;
  constexpr int KS = D / 32;    // k-steps of the score product
  constexpr int NT = D / 16;    // channel tiles of the output
  constexpr int PPT = 32 / GP;  // pages per 32-token tile
  constexpr int TPR = 64 / PPT; // tiles covered by one page-entry fetch (one entry per lane)

  // the wavefront number is the same for all lanes; saying so keeps what derives from it (tile
  // numbers, loop bounds, page ids, base addresses) in scalar registers and scalar arithmetic
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int l16 = lane & 15, qd = lane >> 4;
  const int chunk = blockIdx.x, b = blockIdx.z;
  const int j = SPLIT_PAGES ? blockIdx.y : blockIdx.y / nrbg;
  const int rb = SPLIT_PAGES ? 0 : (blockIdx.y % nrbg) * NWAVE + wave;
  const int head = b * sh.Hkv + j;

  // Tiles are dealt round-robin: workgroup `chunk` owns tiles chunk, chunk+nchunk, ... of the
  // list, and in the split-pages shape its four wavefronts deal those out again.  Which tiles
  // a wavefront owns therefore does not depend on the list length, only whether they exist.
  const int wstart = SPLIT_PAGES ? wave : 0, wstride = SPLIT_PAGES ? 4 : 1;
  const int tfirst = chunk + nchunk * wstart;   // first tile of this wavefront
  const int tstep = nchunk * wstride;           // distance between its tiles
  const int32_t* ent = prep.entries + (size_t)head * sh.max_pages;

  // ---- start-up.  What gates the kernel is when the first key/value load leaves, and that
  // needs only the counts and the page entries: they are fetched first, the exit tests follow,
  // and the query fragments are requested next but not waited for until after the first tiles
  // have been requested (they arrive long before the first tile does).
  const int M_raw = prep.mrows[head];
  int U_raw;
  int pg_entry = 0;
  auto fetch_entries = [&](int first_local_tile) {
    if constexpr (!UNION) {
      const long lp = ((long)tfirst + (long)(first_local_tile + lane / PPT) * tstep) * PPT + lane % PPT;
      pg_entry = lp < sh.max_pages ? ent[lp] : 0;   // inside the array whatever U is; checked against U at use
    }
  };
  // UNION: words and ranks of the head's union, in this wavefront's own merge slot; the page table and
  // the staging of the OR in the area behind the slots
  [[maybe_unused]] uint32_t* u_bits = reinterpret_cast<uint32_t*>(lds + (SPLIT_PAGES ? wave : 0) * kSlotStride);
  [[maybe_unused]] int* u_base = reinterpret_cast<int*>(u_bits) + kMaxUnionWords;
  [[maybe_unused]] uint32_t* u_stage = reinterpret_cast<uint32_t*>(lds + 4 * kSlotStride);   // [4][kMaxUnionWords]
  [[maybe_unused]] int* u_tab = reinterpret_cast<int*>(u_stage) + 4 * kMaxUnionWords;     // entries by logical page
  [[maybe_unused]] int u_words = 0;
  // pages whose entries the LDS copy holds: whole 16-byte pieces of the table, up to what fits
  [[maybe_unused]] const int tab_lds_pages = min(sh.max_pages & ~3, kTablePagesInLds);
  if constexpr (UNION) {
    // The four wavefronts share the start-up fetches (every workgroup of a head needs the same
    // 16 KiB of bitmaps and 8 KiB of page table; fetched once per wavefront they cost the compute
    // unit four times the traffic): each takes a quarter of the row slots and of the table, the
    // pieces meet in LDS, one barrier.
    const int words = (sh.max_pages + 31) >> 5;
    // the head's page table, written by the selection kernel at an address known here: its first
    // kTablePagesInLds entries go to LDS, so that resolving a page needs no dependent load
    // (pages beyond them are looked up in memory)
    constexpr int TPW = kTablePagesInLds / 4 / 256;   // 16-byte pieces per lane per wavefront
    u32x4v_t tabv[TPW];
#pragma unroll
    for (int k = 0; k < TPW; ++k) {
      const int i4 = min(wave * (64 * TPW) + lane + 64 * k, max(sh.max_pages / 4 - 1, 0));   // clamped inside the head's table
      tabv[k] = reinterpret_cast<const u32x4v_t*>(ent)[i4];
    }
    // word-major bitmaps: the kUnionRows row slots of one bitmap word are contiguous (slots past the
    // head's row count were cleared by the selection kernel), so a lane ORs its word over rows with
    // 16-byte loads at constant offsets: one memory latency, no per-row addressing
    const uint32_t* maps = uni.rowmaps + (size_t)head * union_region_words(sh.rows_max, words);
    // (the loads of up to four groups of 64 words are issued before the first is used: taken one
    // group at a time, each group costs a memory round trip of its own - 8192 pages are four groups)
    constexpr int kGroupsInFlight = 4;
    for (int g0 = 0; g0 < words; g0 += 64 * kGroupsInFlight) {
      u32x4v_t v[kGroupsInFlight][R];
#pragma unroll
      for (int u = 0; u < kGroupsInFlight; ++u) {
        if (g0 + 64 * u < words) {   // uniform over the workgroup
          const int w = g0 + 64 * u + lane;
          const u32x4v_t* col = reinterpret_cast<const u32x4v_t*>(maps + (size_t)min(w, words - 1) * kUnionRows) + wave * R;
#pragma unroll
          for (int k = 0; k < R; ++k) v[u][k] = col[k];   // this wavefront's quarter of the R * 16 row slots
        }
      }
#pragma unroll
      for (int u = 0; u < kGroupsInFlight; ++u) {
        if (g0 + 64 * u < words) {
          const int w = g0 + 64 * u + lane;
          uint32_t acc = 0u;
#pragma unroll
          for (int k = 0; k < R; ++k) acc |= (v[u][k][0] | v[u][k][1]) | (v[u][k][2] | v[u][k][3]);
          if (w < words) u_stage[wave * kMaxUnionWords + w] = acc;   // words <= kMaxUnionWords: max_pages <= 32 * kMaxUnionWords
        }
      }
    }
#pragma unroll
    for (int k = 0; k < TPW; ++k) reinterpret_cast<u32x4v_t*>(u_tab)[wave * (64 * TPW) + lane + 64 * k] = tabv[k];
    const int P = seq_pages(kv, sh, b);
    u_words = (P + 31) >> 5;
    __syncthreads();
    int total = 0;
    for (int g0 = 0; g0 < words; g0 += 64) {
      const int w = g0 + lane;
      uint32_t acc = (u_stage[w] | u_stage[kMaxUnionWords + w]) | (u_stage[2 * kMaxUnionWords + w] | u_stage[3 * kMaxUnionWords + w]);
      // pages past the sequence's last one are never picked; the masks only keep a stale bitmap harmless
      if (w >= u_words) acc = 0u;
      if (w == u_words - 1 && (P & 31)) acc &= (1u << (P & 31)) - 1u;
      const int c = __popc(acc);
      const int incl = wave_inclusive_scan(c);
      u_bits[w] = acc;
      u_base[w] = total + incl - c;
      total += __builtin_amdgcn_readlane(incl, 63);
    }
    U_raw = total;
    if (chunk == 0 && threadIdx.x == 0 && M_raw > 0) {   // for the merge kernel and the caller's diagnostics
      prep.ucount[head] = total;
      if (uni.sel_count) uni.sel_count[head] = total;
    }
  } else {
    U_raw = prep.ucount[head];
    fetch_entries(0);
  }
  const int U = min(U_raw, sh.max_pages);
  const int M = min(M_raw, min(sh.rows_max, part.rows));   // (rows past the partial stride have nowhere to go: the host sizes it from an upper bound)
  const int ntiles = (U + PPT - 1) / PPT;
  // M <= 0: nothing active; chunk >= ntiles: this workgroup owns no tile; third: no rows for this
  // wavefront in the split-rows shape (which uses no barrier)
  // fourth: this launch only serves row counts in (m_lo, m_hi] (the host may not know the count
  // and then launches both work shapes, each taking its own range)
  const bool has_rows = SPLIT_PAGES || rb * (R * 16) < M;
  // shared-tile shape: a workgroup none of whose wavefronts has rows leaves; one with some rows
  // keeps its row-less wavefronts (they help with staging and keep the barriers)
  const bool group_has_rows = !LDS_TILES || (int)(blockIdx.y % nrbg) * (NWAVE * R * 16) < M;
  if ((M <= 0) | (chunk >= ntiles) | (!LDS_TILES && !has_rows) | !group_has_rows | (M <= m_lo) | (M > m_hi)) return;
  const int ntw = tfirst < ntiles ? (ntiles - 1 - tfirst) / tstep + 1 : 0;   // this wavefront's tiles

  bf16x8_t qf[R][KS];
  {
    const bf16_t* qa = prep.q_act + (size_t)head * sh.rows_max * D;
#pragma unroll
    for (int mt = 0; mt < R; ++mt) {
      const int rg = min(rb * (R * 16) + mt * 16 + l16, sh.rows_max - 1);
#pragma unroll
      for (int ks = 0; ks < KS; ++ks)
        qf[mt][ks] = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const uint4*>(qa + (size_t)rg * D + ks * 32 + qd * 8));
    }
  }
  __builtin_amdgcn_sched_barrier(0);   // the query loads stay ahead of the tile loads below

  float m_run[R], l_run[R], up_thr[R];   // up_thr: the raw score above which a row's reference has to move
  const float inv_scale_log2e = 1.0f / scale_log2e;
  [[maybe_unused]] const f16x8_t ones_h = {1, 1, 1, 1, 1, 1, 1, 1};
  f32x4_t o[R][NT];
#pragma unroll
  for (int mt = 0; mt < R; ++mt) {
    m_run[mt] = kNegBig;
    up_thr[mt] = -INFINITY;
    l_run[mt] = 0.f;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) o[mt][nt] = (f32x4_t){0.f, 0.f, 0.f, 0.f};
  }

  // ---- decoded page entries of this wavefront's next 64 pages, one per lane
  int pg_phys = 0, pg_valid = 0;
  auto decode_entries = [&](int first_local_tile) {
    const long lp = ((long)tfirst + (long)(first_local_tile + lane / PPT) * tstep) * PPT + lane % PPT;
    if constexpr (UNION) {
      // the page of rank lp in the union: the last bitmap word whose rank is <= lp, then the
      // (lp - rank)-th set bit of that word; its physical id comes from the page table
      int page = 0;
      const bool want = lp < U;
      if (want) {
        int lo = 0, hi = u_words, k = (int)lp;
        while (hi - lo > 1) {   // (the trip count depends on u_words only: uniform over the wavefront)
          const int mid = (lo + hi) >> 1;
          if (u_base[mid] <= k) lo = mid; else hi = mid;
        }
        const uint32_t word = u_bits[lo];
        k -= u_base[lo];
        int pos = 0;
#pragma unroll
        for (int sft = 16; sft >= 1; sft >>= 1) {
          const int c = __popc((word >> pos) & ((1u << sft) - 1u));
          if (k >= c) {
            k -= c;
            pos += sft;
          }
        }
        page = lo * 32 + pos;
      }
      // (page < P <= max_pages: inside the table either way)
      const bool from_lds = page < tab_lds_pages;
      pg_entry = !want ? 0 : (from_lds ? u_tab[page] : ent[page]);
    }
    const int e = lp < U ? pg_entry : 0;   // UNION: the entry of the page just found
    const int ph = e & ((1 << kEntryShift) - 1);
    const bool ok = (unsigned)ph < (unsigned)kv.num_pages;
    pg_phys = ok ? ph : 0;
    pg_valid = ok ? min(GP, (int)((unsigned)e >> kEntryShift)) : 0;
  };

  // A 32-token tile is fed to the matrix core as two 16-row halves.  Row i of half h is token
  //   tt(h, i) = 8*(i/4) + 4*h + (i%4)
  // of the tile, so that after the score product lane group qd holds tokens 8*qd .. 8*qd+7
  // (half 0 gives +0..3, half 1 gives +4..7): the 8 k-slots of the second product are 8
  // CONSECUTIVE tokens and its value operand is one 16-byte load from the channel-major page.
  struct Tile {
    bf16x8_t k[2][KS];
    uint4 v[NT];
    int nv[2];   // GP == 16: valid tokens of the tile's two pages; GP == 32: {min(nv,16), max(nv-16,0)}
  };

  // n >= ne asks for a tile that does not exist: the same number of loads is issued (so the
  // count of loads in flight stays a compile-time constant), but all lanes read the first few
  // lines of the pool, which costs a handful of cache hits instead of a tile of traffic.
  auto load_tile = [&](Tile& t, int n, int ne) {
    const bool real = n < ne;
    const int slot = (n * PPT) & 63;
    const bf16_t *k0, *k1, *vp;
    if (GP == 16) {
      const int pa = real ? __builtin_amdgcn_readlane(pg_phys, slot) : 0;
      const int pb = real ? __builtin_amdgcn_readlane(pg_phys, slot + 1) : 0;
      t.nv[0] = real ? __builtin_amdgcn_readlane(pg_valid, slot) : 0;
      t.nv[1] = real ? __builtin_amdgcn_readlane(pg_valid, slot + 1) : 0;
      // lanes l16 < 8 read rows of the first page, the others of the second; row within the page:
      // half 0 -> {0..3, 8..11}, half 1 -> {4..7, 12..15}
      const size_t tk = (size_t)(l16 < 8 ? pa : pb) * sh.Hkv + j;
      const int row0 = real ? 8 * ((l16 >> 2) & 1) + (l16 & 3) : 0;
      k0 = (const bf16_t*)kv.k_pages + tk * (GP * D) + row0 * D;
      k1 = k0 + (real ? 4 * D : 0);
      const size_t tv = (size_t)(qd < 2 ? pa : pb) * sh.Hkv + j;
      vp = (const bf16_t*)kv.v_pages + tv * (GP * D) + (real ? l16 * GP : 0) + 8 * (qd & 1);
    } else {
      const int pa = real ? __builtin_amdgcn_readlane(pg_phys, slot) : 0;
      const int nv = real ? __builtin_amdgcn_readlane(pg_valid, slot) : 0;
      t.nv[0] = nv;
      t.nv[1] = nv;
      const size_t ta = (size_t)pa * sh.Hkv + j;
      const int row0 = real ? 8 * (l16 >> 2) + (l16 & 3) : 0;
      k0 = (const bf16_t*)kv.k_pages + ta * (GP * D) + row0 * D;
      k1 = k0 + (real ? 4 * D : 0);
      vp = (const bf16_t*)kv.v_pages + ta * (GP * D) + (real ? l16 * GP : 0) + 8 * qd;
    }
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      // (streaming loads: a key / value tile is read once per step, and keeping it out of the caches'
      // allocation measured 1 us at C1 and 10 us at C4 per step)
      t.k[0][ks] = __builtin_bit_cast(bf16x8_t, __builtin_nontemporal_load(reinterpret_cast<const u32x4v_t*>(k0 + ks * 32 + qd * 8)));
      t.k[1][ks] = __builtin_bit_cast(bf16x8_t, __builtin_nontemporal_load(reinterpret_cast<const u32x4v_t*>(k1 + ks * 32 + qd * 8)));
    }
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) t.v[nt] = __builtin_bit_cast(uint4, __builtin_nontemporal_load(reinterpret_cast<const u32x4v_t*>(vp + nt * 16 * GP)));
  };

  // Exponentials are taken against a reference point m_run that is allowed to lag the true
  // row maximum by up to kLag (log2 units): the accumulators are rescaled only when a row's
  // maximum overtakes its reference by more than that, which after the first tile is rare.
  // exp2(kLag) = 256 is far inside float / bfloat16 range, and (m_run, l, O) stay consistent.
  constexpr float kLag = 8.0f;
  constexpr float kRefBias = F16V ? 7.0f : 0.0f;   // numerators are exp2(s - m_run) with m_run = reference - kRefBias

  // all score products of a tile, back to back: S^T = K_tile . Q^T for both 16-row halves
  auto score_products = [&](const bf16x8_t (&k)[2][KS], f32x4_t (&sc)[R][2]) {
#pragma unroll
    for (int mt = 0; mt < R; ++mt) {
      sc[mt][0] = (f32x4_t){0.f, 0.f, 0.f, 0.f};
      sc[mt][1] = (f32x4_t){0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        sc[mt][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(k[0][ks], qf[mt][ks], sc[mt][0], 0, 0, 0);
        sc[mt][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(k[1][ks], qf[mt][ks], sc[mt][1], 0, 0, 0);
      }
    }
  };

  // Softmax update and value products of a tile whose scores `sc` are given.  `between` is code
  // the caller wants issued after the rescale decision, in the same straight-line region as the
  // numerators (the shared-tile loop puts the NEXT tile's score products there, so that the matrix
  // core works on them while the vector ALU takes this tile's exponentials).
  auto softmax_values = [&](Tile& t, f32x4_t (&sc)[R][2], auto&& between, auto mfma_between_c) {
    constexpr int MB = decltype(mfma_between_c)::value;   // matrix instructions `between` issues
    // valid tokens among this lane's 8 (tile tokens 8*qd .. 8*qd+7)
    int lane_valid;
    bool full;
    if (GP == 16) {
      full = (t.nv[0] == 16) && (t.nv[1] == 16);
      lane_valid = (qd < 2 ? t.nv[0] : t.nv[1]) - 8 * (qd & 1);
    } else {
      full = t.nv[0] == 32;
      lane_valid = t.nv[0] - 8 * qd;
    }
    if (!LDS_TILES && !full) {   // (the shared-tile shape clears them once per workgroup, while staging the tile)
      // slots past the end of the sequence may hold anything: clear them in V (0 * NaN = NaN)
      const int cnt = max(0, min(8, lane_valid));
      const uint32_t m0 = cnt >= 2 ? ~0u : (cnt == 1 ? 0xFFFFu : 0u);
      const uint32_t m1 = cnt >= 4 ? ~0u : (cnt == 3 ? 0xFFFFu : 0u);
      const uint32_t m2 = cnt >= 6 ? ~0u : (cnt == 5 ? 0xFFFFu : 0u);
      const uint32_t m3 = cnt >= 8 ? ~0u : (cnt == 7 ? 0xFFFFu : 0u);
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
        t.v[nt].x &= m0;
        t.v[nt].y &= m1;
        t.v[nt].z &= m2;
        t.v[nt].w &= m3;
      }
    }
    // ---- phase 2: one lazy-rescale decision for the wavefront.  Whether some row's maximum
    // has overtaken its reference by more than kLag is decided from each lane's own maximum
    // (a row's lanes share m_run, and scaling by a positive factor keeps the order, so "some
    // lane exceeds" and "the row maximum exceeds" are the same event); the cross-lane maximum
    // itself is only taken when that happens, which after the first tile is rare.
    // (Every instruction that reads a matrix-core result here is an ordinary compiler-visible
    // one: the wait states such a read needs are inserted by the compiler, which it cannot do
    // for inline assembly.)
    // The scores are used where the matrix core left them (element e of the lane's 8 tokens is
    // sc[mt][e / 4][e % 4]); the test against the reference is one compare per row tile against a
    // threshold in score units, kept up to date with the reference.
    float tm[R];
    bool any_up = false;
#pragma unroll
    for (int mt = 0; mt < R; ++mt) {
      if (!full) {
#pragma unroll
        for (int e = 0; e < 8; ++e)
          if (e >= lane_valid) sc[mt][e >> 2][e & 3] = -INFINITY;
      }
      const f32x4_t a = sc[mt][0], b = sc[mt][1];
      tm[mt] = fmaxf(fmaxf(fmaxf(fmaxf(a[0], a[1]), a[2]), fmaxf(fmaxf(a[3], b[0]), b[1])), fmaxf(b[2], b[3]));
      any_up |= tm[mt] > up_thr[mt];
    }
    if (__any(any_up)) {
#pragma unroll
      for (int mt = 0; mt < R; ++mt) {
        const float m_cand = max_over_lane_groups(tm[mt]) * scale_log2e - kRefBias;
        const bool up = m_cand > m_run[mt] + kLag;
        const float alpha = up ? fast_exp2(m_run[mt] - m_cand) : 1.0f;
        m_run[mt] = up ? m_cand : m_run[mt];
        up_thr[mt] = (m_run[mt] + (kLag + kRefBias)) * inv_scale_log2e;
        l_run[mt] *= alpha;
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) o[mt][nt] *= alpha;
      }
    }
    // ---- phase 3: numerators as a bfloat16 pair, value products.
    // P = hi + lo with hi = p truncated to its top 16 bits (exact, no conversion) and
    // lo = p - hi rounded: 16 mantissa bits in all.  A single bfloat16 would cost 2^-9 of the
    // spread of V per row, which outlier value channels push past the 2e-2 bound.
    // The hi products of a row tile are issued right after its numerators, so the matrix core
    // works while the vector ALU does the next row tile; all lo products come last, far from
    // the hi product that feeds the same accumulator.
    between();
    if constexpr (F16V) {
      // half-precision form: one operand per row tile (the value tile in t.v is already half precision)
#pragma unroll
      for (int mt = 0; mt < R; ++mt) {
        const float neg_m = -m_run[mt];
        f32x8_t p;
#pragma unroll
        for (int e = 0; e < 8; ++e) p[e] = fast_exp2(fmaf(sc[mt][e >> 2][e & 3], scale_log2e, neg_m));
        const f16x8_t ph = __builtin_convertvector(p, f16x8_t);
        // The row sum comes from the matrix core as well: a product with an all-ones operand sums the
        // (rounded) numerators of the tile's 32 tokens into every element of the result, so the
        // normaliser is exactly the sum of the weights the value product uses, and the vector ALU
        // adds one number per row tile instead of eight.
        const f32x4_t rs = __builtin_amdgcn_mfma_f32_16x16x32_f16(ones_h, ph, (f32x4_t){0.f, 0.f, 0.f, 0.f}, 0, 0, 0);
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
          o[mt][nt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8_t, t.v[nt]), ph, o[mt][nt], 0, 0, 0);
        l_run[mt] += rs[0];
      }
      // scheduling hint for this region: one matrix instruction, then a few vector instructions
#pragma unroll
      for (int i = 0; i < R * NT + R + MB; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // 1 MFMA
        __builtin_amdgcn_sched_group_barrier(0x002, 3, 0);   // 3 VALU
      }
    } else {
    bf16x8_t p_lo[R];
#pragma unroll
    for (int mt = 0; mt < R; ++mt) {
      const float neg_m = -m_run[mt];
      float p[8], psum = 0.f;
      f32x8_t lo;
      uint32_t pb[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        p[e] = fast_exp2(fmaf(sc[mt][e >> 2][e & 3], scale_log2e, neg_m));
        psum += p[e];
        pb[e] = __float_as_uint(p[e]);
        lo[e] = p[e] - __uint_as_float(pb[e] & 0xFFFF0000u);
      }
      l_run[mt] += psum;
      uint4 hi_bits;
      hi_bits.x = __builtin_amdgcn_perm(pb[1], pb[0], 0x07060302u);
      hi_bits.y = __builtin_amdgcn_perm(pb[3], pb[2], 0x07060302u);
      hi_bits.z = __builtin_amdgcn_perm(pb[5], pb[4], 0x07060302u);
      hi_bits.w = __builtin_amdgcn_perm(pb[7], pb[6], 0x07060302u);
      const bf16x8_t p_hi = __builtin_bit_cast(bf16x8_t, hi_bits);
      p_lo[mt] = __builtin_convertvector(lo, bf16x8_t);
#pragma unroll
      for (int nt = 0; nt < NT; ++nt)
        o[mt][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, t.v[nt]), p_hi, o[mt][nt], 0, 0, 0);
    }
#pragma unroll
    for (int mt = 0; mt < R; ++mt)
#pragma unroll
      for (int nt = 0; nt < NT; ++nt)
        o[mt][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, t.v[nt]), p_lo[mt], o[mt][nt], 0, 0, 0);
    // Scheduling hint for this region: alternate one matrix instruction with a few vector
    // instructions, so the numerators of the next row tile are computed while the matrix core
    // works on the products of the previous one (one wavefront per SIMD: nobody else would).
#pragma unroll
    for (int i = 0; i < 2 * R * NT; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // 1 MFMA
      __builtin_amdgcn_sched_group_barrier(0x002, 3, 0);   // 3 VALU
    }
    }
  };
  auto compute_tile = [&](Tile& t) {
    f32x4_t sc[R][2];
    score_products(t.k, sc);
    softmax_values(t, sc, [] {}, std::integral_constant<int, 0>{});
  };

  // ---- main loop: NBUF tile buffers in registers, NBUF-1 tiles of lookahead (how many: see
  // the launcher).  A wavefront has a SIMD to itself, so memory latency is hidden by its own
  // lookahead, not by occupancy.  Every load is issued unconditionally (see load_tile) so that
  // the number of loads in flight at each use is a compile-time constant: a load behind a
  // branch would force a full drain at the join.
  if constexpr (LDS_TILES) {
    // ---- shared-tile variant (many rows, 8 wavefronts of R*16 rows, 2 per SIMD): every
    // wavefront of the workgroup walks the same tiles, so a tile is fetched from memory once per
    // workgroup (not once per wavefront), put into LDS and read from there by all.  Measured on
    // the dense initialisation this is 9-14% faster than 4 independent wavefronts of 64 rows.
    // What it does not buy is overlap of matrix and vector work: counters show matrix-core busy
    // plus vector-ALU busy adding up to the run time with one or two wavefronts per SIMD, also
    // when the two of a SIMD are made to alternate their matrix and vector pieces with barriers
    // (tried: same time), so the many-row shape is bound by the sum of the two, not by memory.
    //
    // LDS image of a tile: the matrix-core operands themselves, one 1 KiB block per operand
    // (2*KS key blocks: half h, k-step ks; then NT value blocks), lane L's 16 bytes at L*16.
    // Writes and reads are then both lane-linear, hence free of bank conflicts whichever way
    // the hardware groups lanes; the permutation lives in the global addresses, where it only
    // costs some coalescing.  Each wavefront fetches BPW of the blocks.  Two LDS buffers: tile
    // n+1 is written while tile n is computed on; one barrier per tile.
    constexpr int NBLK = 2 * KS + NT;          // operand blocks per tile
    constexpr int BPW = NBLK / NWAVE;          // blocks fetched by each wavefront
    constexpr int BUF = NBLK * 1024;           // bytes of one tile image
    static_assert(NBLK % NWAVE == 0 && (BPW == 1 || BPW == 2), "operand blocks do not split evenly over the wavefronts");
    unsigned char* lbase = reinterpret_cast<unsigned char*>(lds);
    // PD tiles are in flight per workgroup: one register set each (this lane's 16-byte pieces
    // of its blocks and, in scalar registers, the tile's valid-token counts).  Tile n sits in set
    // n % PD; all indices below are compile-time constants once the loops are unrolled.
    constexpr int PD = 2;
    static_assert(PD <= TPR, "the first PD tiles come from the first batch of page entries");
    typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));   // a plain vector value: stays in registers
    struct Stage {
      u32x4_t v[BPW];
      int nv[2];
    };
    Stage g[PD];
    // Byte offset of this lane's piece of block i (of this wavefront) inside its page, and which
    // of the tile's pages it is in (0 or 1): fixed for the whole kernel.
    int piece_off[BPW];
    bool piece_second[BPW], piece_is_k[BPW];
#pragma unroll
    for (int i = 0; i < BPW; ++i) {
      const int blk = wave + NWAVE * i;
      piece_is_k[i] = blk < 2 * KS;
      if (piece_is_k[i]) {
        const int h = blk / KS, ks = blk % KS;
        const int r = 8 * (l16 >> 2) + 4 * h + (l16 & 3);   // token row tt(h, l16) of the tile
        piece_second[i] = GP == 16 && r >= 16;
        piece_off[i] = (r % GP) * (D * 2) + ks * 64 + qd * 16;
      } else {
        const int ch = (blk - 2 * KS) * 16 + l16;           // value channel
        piece_second[i] = GP == 16 && qd >= 2;
        piece_off[i] = ch * (GP * 2) + (GP == 16 ? (qd & 1) : qd) * 16;
      }
    }
    // tile n of this workgroup -> registers.  n >= ntw asks for a tile that does not exist: the
    // loads are issued all the same (no load behind a branch, so the number in flight at every
    // wait is a compile-time constant) but read the first page of the pool.
    auto gload = [&](Stage& st, int n) {
      const bool real = n < ntw;
      const int slot = (n * PPT) & 63;
      const int pa = real ? __builtin_amdgcn_readlane(pg_phys, slot) : 0;
      const int pb = real ? __builtin_amdgcn_readlane(pg_phys, slot + PPT - 1) : 0;
      st.nv[0] = real ? __builtin_amdgcn_readlane(pg_valid, slot) : 0;
      st.nv[1] = real ? __builtin_amdgcn_readlane(pg_valid, slot + PPT - 1) : 0;
#pragma unroll
      for (int i = 0; i < BPW; ++i) {
        const size_t tile = (size_t)(piece_second[i] ? pb : pa) * sh.Hkv + j;
        const unsigned char* src = reinterpret_cast<const unsigned char*>(piece_is_k[i] ? kv.k_pages : kv.v_pages) +
                                   tile * (size_t)(GP * D * 2) + piece_off[i];
        st.v[i] = *reinterpret_cast<const u32x4_t*>(src);
      }
    };
    // bfloat16 pair -> half pair, towards zero: exact inside the half range, never infinite
    auto to_half2 = [](uint32_t two_bf16) -> uint32_t {
      const auto h = __builtin_amdgcn_cvt_pkrtz(__uint_as_float(two_bf16 << 16), __uint_as_float(two_bf16 & 0xFFFF0000u));
      return __builtin_bit_cast(uint32_t, h);
    };
    auto lstore = [&](const Stage& st, int buf) {
      // a tile that ends inside its page(s): the value slots past the end may hold anything and are
      // cleared here, once per workgroup, so that the consumers need not look at them (0 * NaN = NaN)
      const bool full = GP == 16 ? (st.nv[0] == 16) && (st.nv[1] == 16) : st.nv[0] == 32;
#pragma unroll
      for (int i = 0; i < BPW; ++i) {
        u32x4_t x = st.v[i];
        if (!full && !piece_is_k[i]) {
          // this lane's piece of a value block: 8 consecutive tokens of one channel
          const int first = GP == 16 ? 8 * (qd & 1) : 8 * qd;
          const int cnt = max(0, min(8, (GP == 16 && qd >= 2 ? st.nv[1] : st.nv[0]) - first));
          x[0] &= cnt >= 2 ? ~0u : (cnt == 1 ? 0xFFFFu : 0u);
          x[1] &= cnt >= 4 ? ~0u : (cnt == 3 ? 0xFFFFu : 0u);
          x[2] &= cnt >= 6 ? ~0u : (cnt == 5 ? 0xFFFFu : 0u);
          x[3] &= cnt >= 8 ? ~0u : (cnt == 7 ? 0xFFFFu : 0u);
        }
        if (F16V && !piece_is_k[i]) {   // (uniform over the wavefront: a block is all keys or all values)
          x[0] = to_half2(x[0]);
          x[1] = to_half2(x[1]);
          x[2] = to_half2(x[2]);
          x[3] = to_half2(x[3]);
        }
        *reinterpret_cast<u32x4_t*>(lbase + buf * BUF + (wave + NWAVE * i) * 1024 + lane * 16) = x;
      }
    };
    auto lread = [&](Tile& t, int buf) {
      const unsigned char* tb_ = lbase + buf * BUF + lane * 16;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        t.k[0][ks] = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const uint4*>(tb_ + ks * 1024));
        t.k[1][ks] = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const uint4*>(tb_ + (KS + ks) * 1024));
      }
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) t.v[nt] = *reinterpret_cast<const uint4*>(tb_ + (2 * KS + nt) * 1024);
    };
    // rows past M hold whatever the workspace held: make them zero queries
#pragma unroll
    for (int mt = 0; mt < R; ++mt) {
      const uint32_t keep = rb * (R * 16) + mt * 16 + l16 < M ? 0xFFFFFFFFu : 0u;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        uint4 x = __builtin_bit_cast(uint4, qf[mt][ks]);
        x.x &= keep;
        x.y &= keep;
        x.z &= keep;
        x.w &= keep;
        qf[mt][ks] = __builtin_bit_cast(bf16x8_t, x);
      }
    }
    decode_entries(0);
#pragma unroll
    for (int k = 0; k < PD; ++k) gload(g[k], k);
    lstore(g[0], 0);   // waits for tile 0 only
    __syncthreads();
    Tile t;
    // Iteration n: request tile n + PD into the set tile n has just left, compute on tile n from
    // LDS buffer n & 1, move tile n + 1 (requested PD - 1 iterations ago) from its registers into
    // the other buffer, barrier.  The loop runs in groups of PD iterations so that set indices
    // are constants; iterations past the last tile of a group only keep the barriers in step.
    for (int n0 = 0; n0 < ntw; n0 += PD) {
#pragma unroll
      for (int k = 0; k < PD; ++k) {
        const int n = n0 + k;
        t.nv[0] = g[k].nv[0];
        t.nv[1] = g[k].nv[1];
        // page entries come in batches of TPR tiles, requested one iteration before they are decoded
        if ((n + PD) % TPR == 0 && n + PD < ntw) decode_entries(n + PD);
        if ((n + PD + 1) % TPR == 0) fetch_entries(n + PD + 1);
        gload(g[k], n + PD);
        if (has_rows && n < ntw) {
          lread(t, n & 1);
          compute_tile(t);
        }
        lstore(g[(k + 1) % PD], (n + 1) & 1);
        __syncthreads();
      }
    }
    if (!has_rows) return;
  }
  Tile tb[NBUF];
  if constexpr (!LDS_TILES) {
  decode_entries(0);
#pragma unroll
  for (int k = 0; k < NBUF - 1; ++k) load_tile(tb[k], k, min(ntw, TPR));
  __builtin_amdgcn_sched_barrier(0);
  // rows past M hold whatever the workspace held: make them zero queries (first wait for them)
#pragma unroll
  for (int mt = 0; mt < R; ++mt) {
    const uint32_t keep = rb * (R * 16) + mt * 16 + l16 < M ? 0xFFFFFFFFu : 0u;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      uint4 x = __builtin_bit_cast(uint4, qf[mt][ks]);
      x.x &= keep;
      x.y &= keep;
      x.z &= keep;
      x.w &= keep;
      qf[mt][ks] = __builtin_bit_cast(bf16x8_t, x);
    }
  }
  for (int nb = 0; nb < ntw; nb += TPR) {
    const int ne = min(ntw, nb + TPR);
    if (nb > 0) {
      fetch_entries(nb);
      decode_entries(nb);
#pragma unroll
      for (int k = 0; k < NBUF - 1; ++k) load_tile(tb[k], nb + k, ne);
    }
    for (int n = nb; n < ne; n += NBUF) {
#pragma unroll
      for (int k = 0; k < NBUF; ++k) {
        load_tile(tb[(k + NBUF - 1) % NBUF], n + k + NBUF - 1, ne);
        if (n + k < ne) compute_tile(tb[k]);
      }
    }
  }
  }   // !LDS_TILES

  // each lane summed its own tokens; rows are spread over the 4 lane groups (the half-precision
  // form took whole-row sums from the matrix core: nothing to add up)
  if constexpr (!F16V) {
#pragma unroll
    for (int mt = 0; mt < R; ++mt) l_run[mt] = sum_over_lane_groups(l_run[mt]);
  }

  const size_t item = ((size_t)head * nchunk + chunk);
  if (SPLIT_PAGES) {
    // ---- one-round combine of the 4 wavefronts: wavefront w owns channel tiles {w*NTW ..} of
    // the partial.  Everyone publishes (ref, sum) and the O tiles it does NOT own in LDS (its
    // own stay in registers), then reads the three other wavefronts' versions of its tiles,
    // combines the four in wavefront order and stores its slice.  One barrier; the order is
    // fixed, so is the result.  The register file is indexed by the wavefront number, hence
    // one specialisation per wavefront behind a uniform branch.
    typedef MergeSlot<D, R> Slot;
    constexpr int NTW = NT / 4;   // channel tiles per wavefront
    auto publish = [&](auto wv) {
      constexpr int W = decltype(wv)::value;
      {
        float* so = lds + W * kSlotStride;
        float* sm = so + Slot::kOFloats;
        float* sl = sm + R * 16;
#pragma unroll
        for (int mt = 0; mt < R; ++mt) {
          const int r = mt * 16 + l16;
          if (qd == 0) {
            sm[r] = m_run[mt];
            sl[r] = l_run[mt];
          }
#pragma unroll
          for (int nt = 0; nt < NT; ++nt)
            if (nt / NTW != W) *reinterpret_cast<f32x4_t*>(so + ((mt * NT + nt) * 64 + lane) * 4) = o[mt][nt];
        }
      }
    };
    auto combine = [&](auto wv) {
      constexpr int W = decltype(wv)::value;
      // all LDS reads of the combine are issued before the first is used
      float mw[R][4], lw[R][4];
      f32x4_t ov[R][NTW][4];
#pragma unroll
      for (int mt = 0; mt < R; ++mt) {
        const int r = mt * 16 + l16;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          const float* sm = lds + w * kSlotStride + Slot::kOFloats;
          mw[mt][w] = sm[r];
          lw[mt][w] = sm[R * 16 + r];
#pragma unroll
          for (int k = 0; k < NTW; ++k)
            ov[mt][k][w] = w == W ? o[mt][W * NTW + k]
                                  : *reinterpret_cast<const f32x4_t*>(lds + w * kSlotStride +
                                                                      ((mt * NT + W * NTW + k) * 64 + lane) * 4);
        }
      }
#pragma unroll
      for (int mt = 0; mt < R; ++mt) {
        const float m_all = fmaxf(fmaxf(mw[mt][0], mw[mt][1]), fmaxf(mw[mt][2], mw[mt][3]));
        float wgt[4], l_all = 0.f;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          wgt[w] = fast_exp2(mw[mt][w] - m_all);
          l_all = fmaf(lw[mt][w], wgt[w], l_all);
        }
        const int rg = mt * 16 + l16;
        if (rg < M) {
          const size_t prow = item * part.rows + rg;
          if (W == 0 && qd == 0) {
            // (streaming stores: the partials are read once, by the next launch; leaving them out of the
            // caches' write-back at the kernel's end measured 0.3 us per step at 48 MB launches)
            __builtin_nontemporal_store(m_all, &part.m[prow]);
            __builtin_nontemporal_store(l_all, &part.l[prow]);
          }
#pragma unroll
          for (int k = 0; k < NTW; ++k) {
            f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int w = 0; w < 4; ++w) acc += ov[mt][k][w] * wgt[w];
            __builtin_nontemporal_store(acc, reinterpret_cast<f32x4_t*>(part.o + prow * D + (W * NTW + k) * 16 + qd * 4));
          }
        }
      }
    };
    switch (wave) {
      case 0: publish(std::integral_constant<int, 0>{}); break;
      case 1: publish(std::integral_constant<int, 1>{}); break;
      case 2: publish(std::integral_constant<int, 2>{}); break;
      default: publish(std::integral_constant<int, 3>{}); break;
    }
    __syncthreads();
    switch (wave) {
      case 0: combine(std::integral_constant<int, 0>{}); break;
      case 1: combine(std::integral_constant<int, 1>{}); break;
      case 2: combine(std::integral_constant<int, 2>{}); break;
      default: combine(std::integral_constant<int, 3>{}); break;
    }
    return;
  }

  // ---- partial of this (sequence, head, chunk): un-normalised O, running max (log2 units), sum
#pragma unroll
  for (int mt = 0; mt < R; ++mt) {
    const int rg = rb * (R * 16) + mt * 16 + l16;
    if (rg < M) {
      const size_t prow = item * part.rows + rg;
      if (qd == 0) {
        part.m[prow] = m_run[mt];
        part.l[prow] = l_run[mt];
      }
#pragma unroll
      for (int nt = 0; nt < NT; ++nt)
        *reinterpret_cast<f32x4_t*>(part.o + prow * D + nt * 16 + qd * 4) = o[mt][nt];
    }
  }
}

template <int D, int GP, int R, bool SPLIT_PAGES, int NBUF, int NWAVE = 4, bool LDS_TILES = false, bool F16V = false,
          bool UNION = false>
__global__ __launch_bounds__(64 * NWAVE) void attn_mfma_kernel(AttnPrepared prep, int nchunk, int nrbg, Shape sh, KvView kv,
                                                        Partials part, float scale_log2e, int m_lo, int m_hi,
                                                        UnionInKernel uni) {
  extern __shared__ __attribute__((aligned(16))) float lds[];
  attn_mfma_body<D, GP, R, SPLIT_PAGES, NBUF, NWAVE, LDS_TILES, F16V, UNION>(prep, nchunk, nrbg, sh, kv, part, scale_log2e,
                                                                            m_lo, m_hi, uni, lds);
}

// The split-pages shape with the union built in the kernel, for launches whose row counts only the
// device knows (threshold / cumulative-mass selection): every (sequence, KV head) runs the body
// compiled for its own number of 16-row tiles, read from the count the selection kernel left, so a
// head with a few active rows does not pay for the 64 the launch has to allow.  Heads with more than
// 64 rows are not served here (m_hi).
template <int D, int GP>
__global__ __launch_bounds__(256) void attn_mfma_rows_kernel(AttnPrepared prep, int nchunk, Shape sh, KvView kv, Partials part,
                                                             float scale_log2e, int m_lo, int m_hi, UnionInKernel uni) {
  extern __shared__ __attribute__((aligned(16))) float lds[];
  const int M = __builtin_amdgcn_readfirstlane(prep.mrows[blockIdx.z * sh.Hkv + blockIdx.y]);
  if (M <= 0 || M > kUnionRows) return;
  if (M <= 16)
    attn_mfma_body<D, GP, 1, true, 2, 4, false, false, true>(prep, nchunk, 1, sh, kv, part, scale_log2e, m_lo, m_hi, uni, lds);
  else if (M <= 32)
    attn_mfma_body<D, GP, 2, true, 2, 4, false, false, true>(prep, nchunk, 1, sh, kv, part, scale_log2e, m_lo, m_hi, uni, lds);
  else if (M <= 48)
    attn_mfma_body<D, GP, 3, true, 2, 4, false, false, true>(prep, nchunk, 1, sh, kv, part, scale_log2e, m_lo, m_hi, uni, lds);
  else
    attn_mfma_body<D, GP, 4, true, 2, 4, false, false, true>(prep, nchunk, 1, sh, kv, part, scale_log2e, m_lo, m_hi, uni, lds);
}

// Builds the prepared inputs of attn_mfma_kernel when the selection kernel has not done so
// (stand-alone losa_sparse_attn, and the dense initialisation): resolves the page list
// (logical ids, or every page when sel_pages is NULL) to entries and gathers the query rows
// of the active tokens (every token when active_idx is NULL).  kPrepSlices workgroups per
// (sequence, KV head) share the work, so no thread walks a long chain of dependent loads.
constexpr int kPrepSlices = 16;

__global__ __launch_bounds__(256) void attn_prepare_kernel(KvView kv, Shape sh, const bf16_t* __restrict__ q,
                                                           const int32_t* __restrict__ active_idx,
                                                           const int32_t* __restrict__ active_count,
                                                           const int32_t* __restrict__ sel_pages,
                                                           const int32_t* __restrict__ sel_count, int cap,
                                                           AttnPrepared prep) {
  const int j = blockIdx.x, b = blockIdx.y;
  const int gtid = blockIdx.z * 256 + threadIdx.x, gthreads = kPrepSlices * 256;
  const int head = b * sh.Hkv + j;
  const int base = kv.page_indptr[b];
  const int P = seq_pages(kv, sh, b);
  const int L = kv.seq_lens[b];
  const int32_t* list = sel_pages ? sel_pages + (size_t)head * cap : nullptr;
  const int U = max(0, min(list ? min(sel_count[head], cap) : P, sh.max_pages));
  const int n_act = active_idx ? active_count[b] : sh.B;
  int32_t* ent = prep.entries + (size_t)head * sh.max_pages;
  for (int i = gtid; i < U; i += gthreads) {
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
  for (int v = gtid; v < M * vpr; v += gthreads) {
    const int r = v / vpr, cv = v % vpr;
    const int a = r / sh.G, hg = r % sh.G;
    const int tok = active_idx ? active_idx[(size_t)b * sh.B + a] : a;
    uint4 val = make_uint4(0u, 0u, 0u, 0u);
    if ((unsigned)tok < (unsigned)sh.B)
      val = reinterpret_cast<const uint4*>(q + (((size_t)b * sh.B + tok) * sh.Hq + j * sh.G + hg) * sh.d)[cv];
    dst[v] = val;
  }
  if (gtid == 0) {
    prep.ucount[head] = U;
    prep.mrows[head] = M;
  }
}

hipError_t launch_attn_prepare(hipStream_t st, const KvView& kv, const Shape& sh, int batch, const void* q,
                               const int32_t* active_idx, const int32_t* active_count, const int32_t* sel_pages,
                               const int32_t* sel_count, int cap, const AttnPrepared& prep) {
  if (batch <= 0) return hipSuccess;
  dim3 grid(sh.Hkv, batch, kPrepSlices);
  attn_prepare_kernel<<<grid, 256, 0, st>>>(kv, sh, (const bf16_t*)q, active_idx, active_count, sel_pages, sel_count,
                                            cap, prep);
  return hipGetLastError();
}

// Bytes of LDS the shared-tile variant needs: two images of a 32-token tile (keys and values).
template <int D, int GP>
constexpr size_t shared_tile_lds_bytes() {
  return 2 * (2 * 32 * D * 2);
}

template <int D, int GP, int R, bool SPLIT, int NWAVE = 4, bool LDS_TILES = false, bool F16V = false, bool UNION = false>
static hipError_t launch_one(hipStream_t st, const KvView& kv, const Shape& sh, int batch, const AttnPrepared& prep,
                             int nchunk, const Partials& part, hipEvent_t ev_start, hipEvent_t ev_stop, int m_lo,
                             int m_hi, const UnionInKernel& uni = UnionInKernel{nullptr, nullptr}) {
  static_assert(!(SPLIT && LDS_TILES) && (SPLIT ? NWAVE == 4 : true), "the split-pages combine is written for 4 wavefronts");
  const int nrbg = SPLIT ? 1 : (sh.rows_max + R * 16 * NWAVE - 1) / (R * 16 * NWAVE);
  const size_t lds_bytes = SPLIT ? (4 * MergeSlot<D, R>::kFloats + (UNION ? kUnionShared : 0)) * sizeof(float)
                                 : (LDS_TILES ? shared_tile_lds_bytes<D, GP>() : 0);
  // Tile buffers per wavefront (one is being computed on, the others are in flight).  The sparse
  // shape wants exactly one tile of lookahead: with more, every wavefront has its whole share
  // of the list requested at once, the memory system completes those requests in no useful
  // order, and the first tile of every wavefront lands only near the end of the stream, so
  // nothing is left to overlap the arithmetic with (C1: 17.9 us with 3 tiles of lookahead,
  // 15.2 us with 1).  The dense shape has arithmetic to hide behind and keeps a deeper queue.
  constexpr int NBUF = (SPLIT || LDS_TILES) ? 2 : ((D == 128 && R == 4) ? 3 : 4);
  static_assert(!F16V || LDS_TILES, "the half-precision value product converts the tile while staging it");
  auto kern = attn_mfma_kernel<D, GP, R, SPLIT, NBUF, NWAVE, LDS_TILES, F16V, UNION>;
  static bool attr_set = false;   // per instantiation
  if (lds_bytes > 48 * 1024 && !attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)lds_bytes);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  const float scale_log2e = sh.sm_scale * 1.4426950408889634f;
  dim3 grid(nchunk, sh.Hkv * nrbg, batch);
  if (ev_start && ev_stop)   // events bound to this dispatch: they read the kernel's own begin and end
    hipExtLaunchKernelGGL(kern, grid, dim3(64 * NWAVE), (uint32_t)lds_bytes, st, ev_start, ev_stop, 0, prep, nchunk,
                          nrbg, sh, kv, part, scale_log2e, m_lo, m_hi, uni);
  else
    kern<<<grid, 64 * NWAVE, lds_bytes, st>>>(prep, nchunk, nrbg, sh, kv, part, scale_log2e, m_lo, m_hi, uni);
  return hipGetLastError();
}

// Many rows (many_rows: ManyRowForm): 8 wavefronts of 32 rows sharing tiles through LDS, with the value
// product in half precision or as a bfloat16 pair, or 4 independent wavefronts of 64 rows.
template <int D, int GP>
static hipError_t launch_dg(hipStream_t st, const KvView& kv, const Shape& sh, int batch, const AttnPrepared& prep,
                            int nchunk, int rows_upper, const Partials& part, hipEvent_t e0, hipEvent_t e1, int m_lo,
                            int m_hi, const UnionInKernel* uni, int many_rows) {
  if (uni && uni->rowmaps && uni->rows_on_device) {   // ... and takes every head's row-tile count from the device
    const size_t lds_bytes = (4 * MergeSlot<D, 4>::kFloats + kUnionShared) * sizeof(float);
    auto kern = attn_mfma_rows_kernel<D, GP>;
    static bool attr_set = false;   // per instantiation
    if (lds_bytes > 48 * 1024 && !attr_set) {
      hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                         (int)lds_bytes);
      if (e != hipSuccess) return e;
      attr_set = true;
    }
    kern<<<dim3(nchunk, sh.Hkv, batch), 256, lds_bytes, st>>>(prep, nchunk, sh, kv, part, sh.sm_scale * 1.4426950408889634f,
                                                              m_lo, m_hi, *uni);
    return hipGetLastError();
  }
  if (uni && uni->rowmaps) {   // the kernel builds the union from the row bitmaps itself
    if (rows_upper <= 16) return launch_one<D, GP, 1, true, 4, false, false, true>(st, kv, sh, batch, prep, nchunk, part, e0, e1, m_lo, m_hi, *uni);
    if (rows_upper <= 32) return launch_one<D, GP, 2, true, 4, false, false, true>(st, kv, sh, batch, prep, nchunk, part, e0, e1, m_lo, m_hi, *uni);
    if (rows_upper <= 48) return launch_one<D, GP, 3, true, 4, false, false, true>(st, kv, sh, batch, prep, nchunk, part, e0, e1, m_lo, m_hi, *uni);
    if (rows_upper <= 64) return launch_one<D, GP, 4, true, 4, false, false, true>(st, kv, sh, batch, prep, nchunk, part, e0, e1, m_lo, m_hi, *uni);
    return hipErrorInvalidValue;
  }
  if (rows_upper <= 16) return launch_one<D, GP, 1, true>(st, kv, sh, batch, prep, nchunk, part, e0, e1, m_lo, m_hi);
  if (rows_upper <= 32) return launch_one<D, GP, 2, true>(st, kv, sh, batch, prep, nchunk, part, e0, e1, m_lo, m_hi);
  if (rows_upper <= 48) return launch_one<D, GP, 3, true>(st, kv, sh, batch, prep, nchunk, part, e0, e1, m_lo, m_hi);
  if (rows_upper <= 64) return launch_one<D, GP, 4, true>(st, kv, sh, batch, prep, nchunk, part, e0, e1, m_lo, m_hi);
  // (16 rows per wavefront for up to 128 rows, so that all 8 wavefronts have work, was measured
  // and is slower than 4 busy wavefronts of 32 rows: every wavefront reads the whole tile from
  // LDS whatever its row count, so halving the rows halves the reuse of each operand read.)
  if (many_rows == kManyRowsSharedHalf)
    return launch_one<D, GP, 2, false, 8, true, true>(st, kv, sh, batch, prep, nchunk, part, e0, e1, m_lo, m_hi);
  if (many_rows == kManyRowsSharedPair)
    return launch_one<D, GP, 2, false, 8, true, false>(st, kv, sh, batch, prep, nchunk, part, e0, e1, m_lo, m_hi);
  return launch_one<D, GP, 4, false>(st, kv, sh, batch, prep, nchunk, part, e0, e1, m_lo, m_hi);
}

hipError_t launch_attn_mfma(hipStream_t st, const KvView& kv, const Shape& sh, int batch, const AttnPrepared& prep,
                            int nchunk, int rows_upper, const Partials& part, hipEvent_t e0, hipEvent_t e1, int m_lo,
                            int m_hi, const UnionInKernel* uni, int many_rows) {
  if (batch <= 0 || nchunk <= 0) return hipSuccess;
  if (sh.d == 128) {
    if (sh.g == 16) return launch_dg<128, 16>(st, kv, sh, batch, prep, nchunk, rows_upper, part, e0, e1, m_lo, m_hi, uni, many_rows);
    return launch_dg<128, 32>(st, kv, sh, batch, prep, nchunk, rows_upper, part, e0, e1, m_lo, m_hi, uni, many_rows);
  }
  if (sh.g == 16) return launch_dg<64, 16>(st, kv, sh, batch, prep, nchunk, rows_upper, part, e0, e1, m_lo, m_hi, uni, many_rows);
  return launch_dg<64, 32>(st, kv, sh, batch, prep, nchunk, rows_upper, part, e0, e1, m_lo, m_hi, uni, many_rows);
}

}  // namespace losa
