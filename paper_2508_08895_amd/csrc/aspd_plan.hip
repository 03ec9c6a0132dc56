// The plan of a step's attention launches (see aspd_plan.h): which workgroup takes which run of KV
// pages of which (sequence, row group, KV head) item.  One small kernel per step; integer work.
//
// Work decomposition of the attention kernels (ASPD Sec. 3.2 Eq. 1-3 evaluate, per query row, a softmax
// over the KV slots the row may see; rows that share a sequence and a KV head share the pages they
// read): the (sequence, row group, KV head, page) space is flattened and every workgroup takes a
// contiguous share of it.  A share may cut an item: the workgroups that hold parts of one item combine
// their partial results inside the attention launch.
#include <algorithm>
#include <atomic>

#include "aspd_plan.h"

namespace {

constexpr int PLAN_THREADS = 1024;  // one workgroup; a thread per workgroup of the largest attention grid

struct PlanArgs {
  const int32_t* stage_base;
  const int32_t* seq_len;
  const int32_t* cu_seq_new;
  const int32_t* block_tables;
  int32_t*       plan;
  int            B, nwg, qpg, pad, num_kv_heads, max_blocks_per_seq, num_blocks;
  int            has_owner;
};

struct Item {
  int s, rg, h;     // sequence, row group, KV head
  int np;           // pages of the item
  int lp;           // pages of it that lie wholly before stage_base (no owner tags, no masking)
  int q0, nq;       // first packed query row and number of queries of the row group
  int first_unit;   // flattened index of the item's page 0
};

// Per-sequence scalars in LDS and the table of share boundaries.
struct Sched {
  int* cu_units;  // [B+1] exclusive scan of (pages + pad) * row groups * KV heads
  int* T;         // [B]   seq_len
  int* L;         // [B]   stage_base
  int* q0;        // [B+1] cu_seq_new
  int* wgb;       // [MAX_WG+1] first unit of every workgroup's share (ragged regime only)
};
__device__ __forceinline__ Sched sched_at(int* base, int B) {
  Sched sc;
  sc.cu_units = base;
  sc.T = base + (B + 1);
  sc.L = sc.T + B;
  sc.q0 = sc.L + B;
  sc.wgb = sc.q0 + (B + 1);
  return sc;
}
constexpr int sched_ints(int B) { return (4 * B + 2 + MAX_WG + 1 + 3) & ~3; }  // (what follows stays 16-byte aligned)

__device__ __forceinline__ int pages_of(const PlanArgs& a, const Sched& sc, int s) {
  return min((sc.T[s] + ASPD_BLOCK - 1) / ASPD_BLOCK, a.max_blocks_per_seq);
}
__device__ __forceinline__ int groups_of(const PlanArgs& a, const Sched& sc, int s) {
  return (sc.q0[s + 1] - sc.q0[s] + a.qpg - 1) / a.qpg;
}

// Shares of the unit space, one per workgroup used.  A unit is a page of an item or, in the ragged
// regime, one of `pad` virtual units in front of every item: they price the fixed cost a workgroup
// pays for starting a segment (start-up, reduction, a partial to be merged), so that equal shares of
// units are about equal shares of time.  Two regimes, chosen per step:
//
// EVEN (no more items than workgroups, and pieces that come out about as long as the shares of the
// ragged regime would).  Every workgroup has exactly one segment: item i is cut evenly among
// k_i = ceil(np_i / p) workgroups of its own, with p the smallest piece length for which the pieces of
// all items fit the grid.  A workgroup pays a segment's fixed cost once, and an item that fits one piece
// needs no merge.
//
// RAGGED.  Workgroup w nominally takes [w * total / n, (w + 1) * total / n); a boundary inside an
// item's padding, or within `tol` units after it or before the item's end, is moved onto the item
// boundary: a sliver of a neighbouring item would cost a whole extra segment for a few pages.  The
// boundaries are tabulated in LDS (wgb), which also gives the owner of a unit by binary search.
struct Shares {
  int total, n, tol, pad;
  bool even;
  int piece;        // EVEN: p, the length no piece exceeds
  double share;     // RAGGED: total / n, units per workgroup
  __device__ __forceinline__ int nominal_begin(int w) const { return min(total, (int)((double)w * share)); }
};

// The item that holds unit `u`, and the unit's index within it (padding first, then the pages).
// `hint`: a sequence at or before the one that holds u, or -1 (a walk moves forward: the item it was at).
__device__ Item locate(const PlanArgs& a, const Sched& sc, int pad, int u, int* vpage, int hint = -1) {
  int lo = 0, hi = a.B - 1;  // the last sequence that starts at or before u
  if (hint >= 0) {
    // the same sequence or one of the next two, else search from there on
    lo = hint;
#pragma unroll
    for (int d = 0; d < 3; ++d) {
      if (lo < hi && sc.cu_units[lo + 1] <= u) ++lo; else hi = lo;
    }
    if (lo < a.B - 1 && sc.cu_units[lo + 1] <= u) hi = a.B - 1;  // further on: bisect the rest
  }
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (sc.cu_units[mid] <= u) lo = mid; else hi = mid - 1;
  }
  Item it;
  it.s = lo;
  it.np = pages_of(a, sc, lo);
  const int vl = it.np + pad;
  const int rel = u - sc.cu_units[lo];
  const int idx = rel / vl;
  *vpage = rel - idx * vl;
  const int ngroups = groups_of(a, sc, lo);
  it.h = idx / ngroups;       // row groups of one KV head are neighbours: they read the same pages
  it.rg = idx - it.h * ngroups;
  it.first_unit = sc.cu_units[lo] + idx * vl;
  it.lp = a.has_owner ? min(it.np, sc.L[lo] / ASPD_BLOCK) : it.np;
  const int qs = sc.q0[lo];
  const int nq = sc.q0[lo + 1] - qs;
  it.q0 = qs + it.rg * a.qpg;
  it.nq = min(a.qpg, nq - it.rg * a.qpg);
  return it;
}

// Cutting one item among its k workgroups (even regime).  A page of the branch region costs a wave
// more than a page before it (owner tags, masking, scores that are thrown away): measured between 1.1
// and 1.5 times, taken as 1.25.  The cut is therefore even in cost(p) = 4p + max(0, p - lp) rather than
// in pages: piece j starts at the first page p with cost(p) * k >= j * cost(np), and page p belongs to
// piece cost(p) * k / cost(np).
__device__ __forceinline__ int item_cut(const Item& it, int j, int k) {
  const int total = 4 * it.np + (it.np - it.lp);
  const int t = (int)(((unsigned)j * (unsigned)total + (unsigned)k - 1u) / (unsigned)k);
  return t <= 4 * it.lp ? (t + 3) >> 2 : it.lp + (t - 4 * it.lp + 4) / 5;
}
__device__ __forceinline__ int item_piece(const Item& it, int page, int k) {
  const int total = 4 * it.np + (it.np - it.lp);
  const int cost = 4 * page + max(0, page - it.lp);
  return min(k - 1, (int)((unsigned)cost * (unsigned)k / (unsigned)total));
}

__device__ int share_begin(const PlanArgs& a, const Sched& sc, const Shares& sh, int w) {
  if (w <= 0) return 0;
  if (w >= sh.n) return sh.total;
  const int nominal = sh.nominal_begin(w);
  int vpage;
  const Item it = locate(a, sc, sh.pad, nominal, &vpage);
  const int vl = it.np + sh.pad;
  if (vpage <= sh.pad + sh.tol) return it.first_unit;
  if (vl - vpage <= sh.tol) return it.first_unit + vl;
  return nominal;
}

// Fills the LDS tables and returns the shares.  All threads of the workgroup call it.
__device__ Shares build_schedule(const PlanArgs& a, const Sched& sc, int* scratch /* 3 * PLAN_THREADS / 64 + 2 ints */) {
  constexpr int PER = (ASPD_MAX_BATCH + PLAN_THREADS - 1) / PLAN_THREADS;  // sequences per thread
  constexpr int NWV = PLAN_THREADS / 64;
  const int tid = threadIdx.x;
  int mine_p[PER], mine_i[PER];
  int sum_p = 0, sum_i = 0;
  int longest = 0;
#pragma unroll
  for (int j = 0; j < PER; ++j) {
    const int s = tid * PER + j;
    mine_p[j] = 0;
    mine_i[j] = 0;
    if (s < a.B) {
      const int T = a.seq_len[s];
      const int q0 = a.cu_seq_new[s];
      const int q1 = a.cu_seq_new[s + 1];
      sc.T[s] = T;
      sc.L[s] = a.stage_base[s];
      sc.q0[s] = q0;
      if (s == a.B - 1) sc.q0[a.B] = q1;
      const int np = min((T + ASPD_BLOCK - 1) / ASPD_BLOCK, a.max_blocks_per_seq);
      const int ng = (q1 - q0 + a.qpg - 1) / a.qpg;
      if (np > 0 && ng > 0) {
        mine_i[j] = ng * a.num_kv_heads;
        mine_p[j] = np * mine_i[j];
        longest = max(longest, np);
      }
      // (for the search below; both tables are filled in for good later)
      sc.cu_units[s] = mine_i[j];
      sc.wgb[s] = mine_i[j] > 0 ? np : 0;
    }
    sum_p += mine_p[j];
    sum_i += mine_i[j];
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) longest = max(longest, __shfl_xor(longest, off));
  // scans: inside the wave by shuffles, across the waves through LDS (one barrier)
  int incl_p = sum_p, incl_i = sum_i;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const int vp = __shfl_up(incl_p, off);
    const int vi = __shfl_up(incl_i, off);
    if ((tid & 63) >= off) {
      incl_p += vp;
      incl_i += vi;
    }
  }
  if ((tid & 63) == 63) {
    scratch[tid >> 6] = incl_p;
    scratch[NWV + (tid >> 6)] = incl_i;
    scratch[2 * NWV + (tid >> 6)] = longest;
  }
  __syncthreads();
  int run_p = incl_p - sum_p, run_i = incl_i - sum_i;  // exclusive within the wave
  int pages = 0, items = 0;
  longest = 0;
#pragma unroll
  for (int w = 0; w < NWV; ++w) {
    const int tp = scratch[w], ti = scratch[NWV + w];
    if (w < (tid >> 6)) {
      run_p += tp;
      run_i += ti;
    }
    pages += tp;
    items += ti;
    longest = max(longest, scratch[2 * NWV + w]);
  }
  Shares sh;
  sh.pad = a.pad;
  sh.piece = 0;
  sh.even = false;
  // ---- EVEN regime?  Thread t tries piece length p_t; the smallest that fits the grid wins.
  int* best = scratch + 3 * NWV;  // [2]: smallest piece length that fits; workgroups it takes
  if (tid == 0) best[0] = 0x7fffffff;
  __syncthreads();
  if (items > 0 && items <= a.nwg) {
    const int span = max(longest - MIN_PAGES_PER_WG, 0);
    const int step = span / PLAN_THREADS + 1;
    const int p = min(max(longest, 1), MIN_PAGES_PER_WG + tid * step);
    // pieces of all items at this length: ceil(np / p) by a float reciprocal, made exact by one correction
    // (np + p < 2^24, the estimate is off by one at most)
    const float rp = __builtin_amdgcn_rcpf((float)p);
    long need = 0;
    for (int s = 0; s < a.B; ++s) {
      const int x = sc.wgb[s] + p - 1;
      int q = (int)((float)x * rp);
      if ((q + 1) * p <= x) ++q;
      else if (q * p > x) --q;
      need += (long)sc.cu_units[s] * q;
    }
    int mine = need <= a.nwg ? p : 0x7fffffff;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) mine = min(mine, __shfl_xor(mine, off));
    if ((tid & 63) == 0 && mine != 0x7fffffff) atomicMin(best, mine);
  }
  __syncthreads();
  if (best[0] != 0x7fffffff) {
    // pieces of this length against what the ragged regime's longest workgroups would carry (a share and two
    // segment starts)
    sh.piece = best[0];
    sh.even = (long)sh.piece + a.pad <= (long)pages / a.nwg + 2L * a.pad;
  }
  __syncthreads();  // (best is read by all before anyone reuses scratch)
  if (sh.even) {
    // cu_units[s]: first workgroup of sequence s' items (the unit of this regime is the workgroup)
    sh.pad = 0;
    int mine_w[PER], sum_w = 0;
#pragma unroll
    for (int j = 0; j < PER; ++j) {
      const int s = tid * PER + j;
      mine_w[j] = 0;
      if (s < a.B && mine_i[j] > 0) mine_w[j] = mine_i[j] * ((mine_p[j] / mine_i[j] + sh.piece - 1) / sh.piece);
      sum_w += mine_w[j];
    }
    int incl_w = sum_w;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const int v = __shfl_up(incl_w, off);
      if ((tid & 63) >= off) incl_w += v;
    }
    if ((tid & 63) == 63) scratch[tid >> 6] = incl_w;
    __syncthreads();
    int run_w = incl_w - sum_w, total_w = 0;
#pragma unroll
    for (int w = 0; w < NWV; ++w) {
      if (w < (tid >> 6)) run_w += scratch[w];
      total_w += scratch[w];
    }
#pragma unroll
    for (int j = 0; j < PER; ++j) {
      const int s = tid * PER + j;
      if (s < a.B) sc.cu_units[s] = run_w;
      run_w += mine_w[j];
    }
    if (tid == 0) sc.cu_units[a.B] = total_w;
    sh.total = total_w;
    sh.n = total_w;
    sh.tol = 0;
    sh.share = 1.0;
    __syncthreads();
    return sh;
  }
  sh.total = pages + sh.pad * items;
  sh.n = pages > 0 ? max(1, min(a.nwg, sh.total / MIN_PAGES_PER_WG)) : 0;
  sh.tol = min((sh.total / max(sh.n, 1)) >> 3, a.pad);
  sh.share = (double)sh.total / (double)max(sh.n, 1);
#pragma unroll
  for (int j = 0; j < PER; ++j) {
    const int s = tid * PER + j;
    if (s < a.B) sc.cu_units[s] = run_p + sh.pad * run_i;
    run_p += mine_p[j];
    run_i += mine_i[j];
  }
  if (tid == 0) sc.cu_units[a.B] = sh.total;
  __syncthreads();
  for (int w = tid; w <= sh.n; w += PLAN_THREADS) sc.wgb[w] = share_begin(a, sc, sh, w);
  __syncthreads();
  return sh;
}

// RAGGED: the workgroup whose share holds unit u.
__device__ int share_owner(const Sched& sc, const Shares& sh, int u) {
  // boundaries sit within a padding's length of w * share: try the nominal owner and its neighbours first
  {
    const int g = min(sh.n - 1, max(0, (int)((float)u / (float)sh.share)));
#pragma unroll
    for (int d = -1; d <= 1; ++d) {
      const int w = g + d;
      if (w >= 0 && w < sh.n && sc.wgb[w] <= u && (w == sh.n - 1 || sc.wgb[w + 1] > u)) return w;
    }
  }
  int lo = 0, hi = sh.n - 1;  // last w with wgb[w] <= u
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (sc.wgb[mid] <= u) lo = mid; else hi = mid - 1;
  }
  return lo;
}

// EVEN: the one segment of workgroup w, and the first and last workgroup of its item.
__device__ bool even_share(const PlanArgs& a, const Sched& sc, const Shares& sh, int w, Item* out, int* page0,
                           int* page1, int* owner, int* w_last) {
  int lo = 0, hi = a.B - 1;  // the last sequence whose first workgroup is at or before w
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (sc.cu_units[mid] <= w) lo = mid; else hi = mid - 1;
  }
  Item it;
  it.s = lo;
  it.np = pages_of(a, sc, lo);
  const int k = (it.np + sh.piece - 1) / sh.piece;  // workgroups per item of this sequence
  const int local = w - sc.cu_units[lo];
  const int idx = local / k, j = local - idx * k;
  const int ngroups = groups_of(a, sc, lo);
  it.h = idx / ngroups;       // row groups of one KV head are neighbours: they read the same pages
  it.rg = idx - it.h * ngroups;
  it.first_unit = 0;
  it.lp = a.has_owner ? min(it.np, sc.L[lo] / ASPD_BLOCK) : it.np;
  const int qs = sc.q0[lo];
  it.q0 = qs + it.rg * a.qpg;
  it.nq = min(a.qpg, sc.q0[lo + 1] - qs - it.rg * a.qpg);
  *out = it;
  *page0 = item_cut(it, j, k);
  *page1 = item_cut(it, j + 1, k);
  *owner = w - j;
  *w_last = w - j + k - 1;
  return *page1 > *page0;
}

// Ragged regime: the next run of real pages in [*u, end), or false at the end.
__device__ bool next_segment(const PlanArgs& a, const Sched& sc, const Shares& sh, int* u, int end, int* s_hint,
                             Item* it, int* page0, int* page1) {
  while (*u < end) {
    int v0;
    *it = locate(a, sc, sh.pad, *u, &v0, *s_hint);
    *s_hint = it->s;
    const int v1 = min(it->np + sh.pad, v0 + (end - *u));
    *u += v1 - v0;
    *page0 = max(0, v0 - sh.pad);
    *page1 = max(0, v1 - sh.pad);
    if (*page1 > *page0) return true;
  }
  return false;
}

// A workgroup's walk over its share, as an iterator: each step gives a segment and the first and last
// workgroup that hold a part of its item.
struct Walk {
  int u, end;
  int s_hint;  // sequence of the item the walk was at last (-1: none yet)
  bool even_pending;
};
__device__ __forceinline__ Walk walk_begin(const Sched& sc, const Shares& sh, int w) {
  Walk wk;
  wk.u = wk.end = 0;
  wk.s_hint = -1;
  wk.even_pending = sh.even && w < sh.n;
  if (!sh.even && w < sh.n) {
    wk.u = sc.wgb[w];
    wk.end = sc.wgb[w + 1];
  }
  return wk;
}
__device__ __forceinline__ bool walk_next(const PlanArgs& a, const Sched& sc, const Shares& sh, int w, Walk* wk,
                                          Item* it, int* page0, int* page1, int* owner, int* w_last) {
  if (sh.even) {
    if (!wk->even_pending) return false;
    wk->even_pending = false;
    return even_share(a, sc, sh, w, it, page0, page1, owner, w_last);
  }
  if (!next_segment(a, sc, sh, &wk->u, wk->end, &wk->s_hint, it, page0, page1)) return false;
  *owner = *page0 == 0 ? w : share_owner(sc, sh, it->first_unit + sh.pad);
  *w_last = *page1 == it->np ? w : share_owner(sc, sh, it->first_unit + sh.pad + it->np - 1);
  return true;
}

// Segments of a workgroup that pass 1 keeps in LDS for pass 2 (8 words each); a workgroup with more is walked
// on from where pass 1 stood when the room ran out.
__host__ __device__ constexpr int plan_cached_segments(int nwg) { return nwg <= 256 ? 4 : (nwg <= 512 ? 2 : 1); }

__global__ __launch_bounds__(PLAN_THREADS) void plan_kernel(PlanArgs a) {
  extern __shared__ int lds[];
  __shared__ int scratch[3 * PLAN_THREADS / 64 + 2];
  __shared__ int wave_tot[PLAN_THREADS / 64];
  const Sched sc = sched_at(lds, a.B);
  int* seg_cache = lds + sched_ints(a.B);
  const int CS = plan_cached_segments(a.nwg);
  const int tid = threadIdx.x;
  const Shares sh = build_schedule(a, sc, scratch);

  // ---- pass 1: the segments of each workgroup (thread w: workgroup w); the first few are kept in LDS
  static_assert(PLAN_THREADS >= MAX_WG, "a thread per workgroup");
  typedef int i32x4 __attribute__((ext_vector_type(4)));
  const int w = tid;
  int cnt = 0;
  Walk resume;  // where the walk stood after the cached segments
  if (w < a.nwg) {
    Walk wk = walk_begin(sc, sh, w);
    resume = wk;
    Item it;
    int p0, p1, owner, w_last;
    while (cnt < CS && walk_next(a, sc, sh, w, &wk, &it, &p0, &p1, &owner, &w_last)) {
      int* c = seg_cache + (w * CS + cnt) * PLAN_SEG;
      *(i32x4*)c = i32x4{it.s | (it.h << 16), it.q0, it.nq, p0};
      *(i32x4*)(c + 4) = i32x4{p1, it.np, owner | (w_last << 16), sc.L[it.s]};
      ++cnt;
    }
    resume = wk;
    // the rest is only counted here (most of a step of the walk is then dead code)
    if (cnt == CS)
      while (walk_next(a, sc, sh, w, &wk, &it, &p0, &p1, &owner, &w_last)) ++cnt;
  }
  // exclusive scan, over the workgroups, of the segments beyond the first
  const int extra = max(cnt - 1, 0);
  int incl = extra;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const int v = __shfl_up(incl, off);
    if ((tid & 63) >= off) incl += v;
  }
  if ((tid & 63) == 63) wave_tot[tid >> 6] = incl;
  __syncthreads();
  int run = incl - extra;
  for (int wv = 0; wv < (tid >> 6); ++wv) run += wave_tot[wv];

  // ---- pass 2: headers and segments
  if (w >= a.nwg) return;
  int32_t* seg_list = a.plan + PLAN_HDR * a.nwg;
  int32_t* hdr = a.plan + PLAN_HDR * w;
  hdr[PLAN_HDR_NSEG] = cnt;
  hdr[PLAN_HDR_NEXT] = run;
  const int cached = min(cnt, CS);
  for (int i = 0; i < cached; ++i) {
    const int* c = seg_cache + (w * CS + i) * PLAN_SEG;
    const i32x4 lo = *(const i32x4*)c, hi = *(const i32x4*)(c + 4);
    int32_t* d = i == 0 ? hdr : seg_list + PLAN_SEG * (run + i - 1);
    *(i32x4*)d = lo;
    *(i32x4*)(d + 4) = hi;
    if (i == 0) {
      const int p0 = lo[3], p1 = hi[0];
      const int32_t* bt = a.block_tables + (long)(lo[0] & 0xffff) * a.max_blocks_per_seq;
      int ids[PLAN_IDS];
#pragma unroll
      for (int k = 0; k < PLAN_IDS; ++k) ids[k] = bt[min(p0 + k, p1 - 1)];  // all on their way at once
#pragma unroll
      for (int k = 0; k < PLAN_IDS; k += 4)
        *(i32x4*)(hdr + PLAN_HDR_IDS + k) =
            i32x4{min(max(ids[k], 0), a.num_blocks - 1), min(max(ids[k + 1], 0), a.num_blocks - 1),
                  min(max(ids[k + 2], 0), a.num_blocks - 1), min(max(ids[k + 3], 0), a.num_blocks - 1)};
    }
  }
  if (cnt > CS) {
    Walk wk = resume;
    Item it;
    int p0, p1, owner, w_last;
    int i = CS;
    while (walk_next(a, sc, sh, w, &wk, &it, &p0, &p1, &owner, &w_last)) {
      int32_t* d = seg_list + PLAN_SEG * (run + i - 1);
      *(i32x4*)d = i32x4{it.s | (it.h << 16), it.q0, it.nq, p0};
      *(i32x4*)(d + 4) = i32x4{p1, it.np, owner | (w_last << 16), sc.L[it.s]};
      ++i;
    }
  }
}

std::atomic<int> g_cu_count[64];

}  // namespace

int aspd_device_cu_count() {
  int dev = 0, n = 0;
  if (hipGetDevice(&dev) != hipSuccess) return 256;
  const bool slot = dev >= 0 && dev < 64;
  if (slot && (n = g_cu_count[dev].load(std::memory_order_relaxed)) > 0) return n;
  if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) return 256;
  if (slot) g_cu_count[dev].store(n, std::memory_order_relaxed);
  return n;
}

int aspd_choose_variant(const aspd_kv* kv, int32_t B, int32_t NQ, int32_t max_new_per_seq, int32_t max_workgroups,
                        bool chunk_call, bool has_owner, AttnVariant* v) {
  const int G = kv->num_q_heads / kv->num_kv_heads;
  v->has_owner = has_owner;
  v->nt = 0;
  if (kv->dtype == ASPD_BF16) {
    // Row group of the streaming kernel: `nt` MFMA tiles of 16 rows, as few as the caller's bound on new
    // tokens per sequence allows (fewer tiles leave more registers for loads in flight), three when there
    // is no bound.  A sequence with more rows than one group holds is processed in several groups.
    int tiles = NT_MAX;
    if (max_new_per_seq > 0) tiles = std::min(NT_MAX, (max_new_per_seq * G + 15) / 16);
    while (tiles < NT_MAX && 16 * tiles < G) ++tiles;
    if (G > 16 * tiles) return 0;
    // Many rows per KV head (branch chunks, prefills): the waves split the rows instead of the keys.
    const bool many_rows = (long)max_new_per_seq * G > 16 * NT_MAX;
    const bool by_rows = (long)NQ * G > 16 * NT_MAX && (many_rows || (chunk_call && max_new_per_seq == 0));
    v->kernel = by_rows ? KERNEL_BF16_ROWS : KERNEL_BF16_STREAM;
    v->nt = by_rows ? ROWS_NT : tiles;
    v->rows_cap = by_rows ? ROWS_NW * 16 * ROWS_NT : 16 * tiles;
  } else {
    if (G > F32_ROWS) return 0;
    v->kernel = KERNEL_F32;
    v->rows_cap = F32_ROWS;
  }
  v->qpg = v->rows_cap / G;
  // A segment's fixed cost (start-up, reduction across waves, partial, merge) in units of the time one
  // more page takes its workgroup.
  v->pad = v->kernel == KERNEL_BF16_STREAM ? PAD_STREAM * 128 / kv->head_dim
           : (v->kernel == KERNEL_BF16_ROWS ? PAD_ROWS : PAD_COMPUTE);
  // Grid: as many workgroups as stay resident at once (one per compute unit: every kernel here needs more
  // than half of a compute unit's LDS or registers), never more than the pages can feed, never more than
  // the caller allows.
  long nwg = aspd_device_cu_count();
  if (v->kernel == KERNEL_BF16_ROWS) nwg = std::min(nwg, (long)MAX_WG_ROWS);
  const long groups_max = (long)B + NQ / v->qpg;
  const long units_max = groups_max * kv->num_kv_heads * kv->max_blocks_per_seq;
  // (... but a workgroup per item when the items are few: four items of six pages each are done sooner by
  // four workgroups than by two that take them in turn)
  nwg = std::min(nwg, std::max((units_max + MIN_PAGES_PER_WG - 1) / MIN_PAGES_PER_WG, groups_max * kv->num_kv_heads));
  if (max_workgroups > 0) nwg = std::min(nwg, (long)max_workgroups);
  v->nwg = (int)std::max(1L, std::min(nwg, (long)MAX_WG));
  v->stream_once = max_new_per_seq > 0 && max_new_per_seq <= v->qpg;
  return 1;
}

uint64_t aspd_plan_key(const AttnVariant& v, int32_t B) {
  // every field the plan kernel's result depends on besides the device arrays
  uint64_t k = 1;
  k = k * 4 + (uint64_t)v.kernel;
  k = k * 2 + (v.has_owner ? 1 : 0);
  k = k * 2048 + (uint64_t)v.nwg;
  k = k * 512 + (uint64_t)v.qpg;
  k = k * 256 + (uint64_t)v.pad;
  k = k * 1024 + (uint64_t)B;
  return k;  // 42 bits
}

size_t aspd_plan_words(const aspd_kv* kv, const AttnVariant& v, int32_t B, int32_t NQ) {
  const size_t items = ((size_t)B + (size_t)NQ / v.qpg) * kv->num_kv_heads;
  return (size_t)PLAN_HDR * v.nwg + (size_t)PLAN_SEG * (items + v.nwg);
}

int aspd_plan_launch(const aspd_kv* kv, const AttnVariant& v, int32_t B, const int32_t* stage_base_d,
                     const int32_t* seq_len_d, const int32_t* cu_seq_new_d, int32_t* plan_d, hipStream_t stream) {
  PlanArgs a;
  a.stage_base = stage_base_d;
  a.seq_len = seq_len_d;
  a.cu_seq_new = cu_seq_new_d;
  a.block_tables = kv->block_tables_d;
  a.plan = plan_d;
  a.B = B;
  a.nwg = v.nwg;
  a.qpg = v.qpg;
  a.pad = v.pad;
  a.num_kv_heads = kv->num_kv_heads;
  a.max_blocks_per_seq = kv->max_blocks_per_seq;
  a.num_blocks = kv->num_blocks;
  a.has_owner = v.has_owner ? 1 : 0;
  const size_t lds = (size_t)(sched_ints(B) + v.nwg * plan_cached_segments(v.nwg) * PLAN_SEG) * sizeof(int);
  hipLaunchKernelGGL(plan_kernel, dim3(1), dim3(PLAN_THREADS), lds, stream, a);
  ASPD_HIP_CHECK(hipGetLastError());
  return ASPD_OK;
}
