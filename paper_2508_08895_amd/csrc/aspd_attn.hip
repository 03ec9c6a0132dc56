// Branch-isolated attention over a paged KV cache for gfx950 (ASPD Sec. 3.2 Eq. 1-3, Sec. 3.3).
//
// The three attention entry points share one rule, one plan and one way of combining partial
// results; two bf16 kernels (one that streams keys past few rows, one that splits many rows among its
// waves) and an fp32 kernel apply it.  A query row q of sequence s sees key slot j iff
//     j <= slot(q)  and  ( j < stage_base[s]  or  tag(q) == 0  or  slot_owner[s][j] == tag(q) )
// with tag(q) = 0 for a main-branch token and the 1-based branch number otherwise.  This is Eq. 2-3
// in cache terms: slots below stage_base belong to earlier stages (visible to all), slots above it to
// the running parallel stage (visible to their own branch), and a token's own slot bounds what has
// been decoded before it.  Parallel decode, branch chunk and serial decode differ only in which rows
// they bring.
//
// Work decomposition: the (sequence, row group, KV head, page) space is flattened; every workgroup
// takes a contiguous share of pages and walks the segments in it.  Which workgroup takes what is the
// step's plan (aspd_plan.h): a kernel only loads its workgroup's header and starts.  All rows of a row
// group (the active branches of the sequence times the query heads of the KV-head's group) are
// processed against a KV page while it is in the workgroup's LDS, so the shared prefix is fetched once
// for all branches.  A segment that covers its item completely writes the output; otherwise it writes
// an unnormalised partial (running max, sum, accumulator); the workgroup that delivers the last partial
// of an item combines them, in the same launch.
#include <algorithm>
#include <cmath>
#include <mutex>
#include <set>
#include <utility>

#include "aspd_plan.h"

namespace {

constexpr int NW = 4;                 // waves per workgroup, fp32 kernel
constexpr int THREADS = NW * 64;
// bf16 streaming kernel: one workgroup of 4 waves per compute unit (one wave per SIMD, so up to 512
// registers each) and one pair of pages in flight per wave, 64 KB per compute unit.  Measured: deeper
// prefetch (rings of 2 or 3 pairs per wave) and 8 waves both lower the read rate of the whole device
// and make it uneven between the XCDs; the ring depth stays a template parameter.
constexpr int STREAM_NW = 4;
constexpr int STREAM_PF = 1;
constexpr int BF16_ROWS = 16 * NT_MAX;
constexpr int ROWS_PREFETCH = 1;      // groups of pages the row-splitting kernel keeps on their way per workgroup
constexpr int ROWS_PPS = 2;           // pairs of pages it stages (and computes) between two barriers
constexpr int COUNTER_BYTES = 4096;   // MAX_WG arrival counters at the head of the workspace
static_assert(COUNTER_BYTES == MAX_WG * 4, "workspace head");
constexpr float LOG2E = 1.4426950408889634f;
constexpr float LN2 = 0.6931471805599453f;
constexpr float LAZY = 6.f;           // log2 slack of the running softmax reference (bf16 path)

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;  // 16 bytes in registers (a native
                                                                  // vector, so arrays of it stay in VGPRs)

struct AttnArgs {
  // (what a workgroup needs before its first page loads leave comes first: one line of the argument block)
  const int32_t* plan;          // the step's plan for this launch shape (aspd_plan.h)
  KvView         kv;
  int            NQ;            // rows of q / out
  int            B;
  int            nwg;
  int            qpg;           // queries per row group
  const int32_t* cu_branches;   // null when no row carries a branch tag
  const uint8_t* slot_owner;
  int            owner_stride;
  const int32_t* q_branch;
  const int32_t* logical_slot;
  const void*    q;
  void*          out;
  float*         lse;
  float*         partial;       // [2 * nwg] slots of {[rows_cap][D] accumulators, [rows_cap][4]: reference, sum, pad}
  int*           counters;      // [nwg] arrivals per split item, zero between calls
  float          scale_log2;    // sm_scale * log2(e)
  int            G;             // query heads per KV head
  int            rows_cap;      // rows per row group the partial slots are sized for
  const int32_t* row_base;      // whole-sequence launches: per packed row, the first slot of the row's stage
};

// ---------------------------------------------------------------------------------------------
// The plan, as the kernels read it.
// ---------------------------------------------------------------------------------------------
struct Seg {
  int s, h;           // sequence, KV head
  int q0, nq;         // first packed query row and number of queries of the row group
  int page0, page1;   // the segment's pages
  int np;             // pages of the whole item
  int owner, w_last;  // first and last workgroup that hold a part of the item
  int L;              // stage_base of the sequence
};

// Plan words through the scalar (constant) path: the address is the same in every lane, the words were
// written by an earlier kernel, and scalar loads neither take vector registers nor queue up with the
// page loads.
typedef int i32x16 __attribute__((ext_vector_type(16)));
typedef int i32x8 __attribute__((ext_vector_type(8)));
typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef int i32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ i32x16 load_words16(const int32_t* p /* 64-byte aligned, uniform */) {
  return *(const __attribute__((address_space(4))) i32x16*)(uintptr_t)p;
}
__device__ __forceinline__ i32x8 load_words8(const int32_t* p /* 32-byte aligned, uniform */) {
  return *(const __attribute__((address_space(4))) i32x8*)(uintptr_t)p;
}
__device__ __forceinline__ i32x2 load_words2(const int32_t* p /* 8-byte aligned, uniform */) {
  return *(const __attribute__((address_space(4))) i32x2*)(uintptr_t)p;
}
template <typename V>
__device__ __forceinline__ Seg seg_of(const V& w) {
  Seg g;
  g.s = w[0] & 0xffff;
  g.h = (int)((unsigned)w[0] >> 16);
  g.q0 = w[1];
  g.nq = w[2];
  g.page0 = w[3];
  g.page1 = w[4];
  g.np = w[5];
  g.owner = w[6] & 0xffff;
  g.w_last = (int)((unsigned)w[6] >> 16);
  g.L = w[7];
  return g;
}
__device__ __forceinline__ Seg load_seg(const int32_t* p) { return seg_of(load_words8(p)); }
// Everything a kernel derives an address from.  A plan is written by the library's own kernel; the
// check keeps a workgroup that is handed anything else (a buffer of the wrong step, say) from reading
// or writing outside the call's arrays: it then does nothing.
__device__ __forceinline__ bool seg_ok(const AttnArgs& a, const Seg& g) {
  // (no short-circuit: one straight run of scalar compares instead of a chain of branches)
  return (int)(g.s < a.B) & (int)(g.h < a.kv.num_kv_heads) & (int)(g.q0 >= 0) & (int)(g.nq >= 1) & (int)(g.nq <= a.qpg) &
         (int)(g.q0 <= a.NQ - g.nq) & (int)(g.page0 >= 0) & (int)(g.page0 < g.page1) & (int)(g.page1 <= g.np) &
         (int)(g.np <= a.kv.max_blocks_per_seq) & (int)(g.L >= 0) & (int)(g.owner <= (int)blockIdx.x) &
         (int)((int)blockIdx.x <= g.w_last) & (int)(g.w_last < a.nwg);
}
__device__ __forceinline__ bool seg_complete(const Seg& g) { return g.page0 == 0 && g.page1 == g.np; }

// Called by every thread of a workgroup that has written a partial of the item of `g` (defined after
// the kernels: it needs the merge).
template <int D, bool BF16, int THREADS, int ELEMS>
__device__ void announce_partial(const AttnArgs& a, const Seg& g, int* flag /* LDS */);

__device__ __forceinline__ float* partial_slot(const AttnArgs& a, int wg, int starts_item, int D) {
  return a.partial + ((long)(2 * wg + starts_item)) * a.rows_cap * (D + 4);
}
// Inside a slot the accumulator rows come first, D floats each and nothing between them, so that rows
// start on 64-byte lines and the lanes of one store fill whole lines (a partly written line costs a
// full line of write traffic); the softmax statistics of all rows follow, 16 bytes per row.
__device__ __forceinline__ float* partial_acc(float* slot, int r, int D) { return slot + (long)r * D; }
__device__ __forceinline__ float* partial_stat(const AttnArgs& a, float* slot, int r, int D) {
  return slot + (long)a.rows_cap * D + 4 * r;
}

__device__ __forceinline__ float exp2_safe_ref(float m) { return (m == -INFINITY) ? 0.f : m; }

// Partials travel between workgroups that may sit on different XCDs, whose L2 caches are not kept
// coherent for ordinary accesses.  Device-scope relaxed atomic stores write through and device-scope
// atomic loads read past the local L2, so no cache write-back or invalidate is needed on this path.
__device__ __forceinline__ void store_device_scope(float* p, float v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float load_device_scope(const float* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// The same write-through store, 16 bytes wide (narrow write-through stores cost a partial-line
// write each).  Callers order it like the 4-byte form: a later s_waitcnt vmcnt(0) covers it.
// A store of more than 8 bytes reads its data registers a little after it issues, and the compiler, which
// does not look inside inline assembly, may let the very next instruction overwrite them: the s_nop keeps
// the wait states the compiler would have inserted for a store of its own.
__device__ __forceinline__ void store_device_scope_x4(float* p, f32x4 v) {
  asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1\n\ts_nop 1" ::"v"(p), "v"(v) : "memory");
}

// ---------------------------------------------------------------------------------------------
// bf16 path: MFMA 16x16x32, transposed scores.
//
// Per wave and per pair of pages (32 keys): S^T[key][row] = K * Q^T  (A = K page, B = Q^T), so a lane
// holds four keys of one row per page; the accumulator layout of S^T is exactly the B-operand layout
// of the second product O^T[d][row] = V^T * P^T, whose A operand (V^T) comes from the LDS
// transpose read.  Softmax statistics of a row live in the 4 lanes {c, c+16, c+32, c+48}.
// ---------------------------------------------------------------------------------------------
template <int D>
struct Bf16Cfg {
  static constexpr int CH = D / 8;              // 16-byte chunks per row
  static constexpr int PAGE_U4 = 16 * CH;       // uint4 per page
  static constexpr int LPP = PAGE_U4 / 64;      // loads per page per lane
  static constexpr int RPL = 64 / CH;           // rows of a page one load covers
  static constexpr int KSTEPS = D / 32;
  static constexpr int MT = D / 16;
  // In LDS a row (one key, or one query row) is followed by 32 bytes of padding.  Measured with all
  // waves of a compute unit reading: the K / Q operand reads (16 rows x one 16-byte chunk per quarter
  // wave) and the transposing V reads then run at the rate of linear reads, where the XOR swizzles
  // tried before them (chunk ^ row) cost 1.6 times that; writes are not affected.
  static constexpr int LROW = CH + 2;            // uint4 per row in LDS
  static constexpr int LPAGE_U4 = 16 * LROW;     // uint4 per page in LDS
  static constexpr int STAGE_BYTES = 4 * LPAGE_U4 * 16;  // K0 K1 V0 V1
};

// Position (in 16-byte units) of 16-byte chunk `chunk` of row `row` inside a page or Q tile in LDS.
template <int D>
__device__ __forceinline__ int lds_pos(int row, int chunk) { return row * Bf16Cfg<D>::LROW + chunk; }

// One pair of pages in flight: K page 0, K page 1, V page 0, V page 1.
template <int D>
struct PairRegs {
  u32x4 r[4][Bf16Cfg<D>::LPP];
  uint32_t own[2];  // owner tags of this lane's four keys in either page (pairs that need masking only)
};

// Owner tags through the scalar (constant) path, for the kernel whose waves fetch pages cooperatively:
// the address is the same for the whole wave, and scalar loads are counted apart from the vector
// loads, so waiting for the tags of a pair never means waiting for the pages of the next pair.
typedef u32x4 __attribute__((aligned(4))) u32x4_a4;
__device__ __forceinline__ u32x4 load_tags_uniform(const uint8_t* p /* same in all lanes, 4-byte aligned */) {
  return *(const __attribute__((address_space(4))) u32x4_a4*)(uintptr_t)p;
}
// The lane's four keys (4g .. 4g + 3) out of a page's sixteen tags.
__device__ __forceinline__ uint32_t lane_tags(const u32x4& t, int g) {
  uint32_t r = t[0];
  r = (g == 1) ? t[1] : r;
  r = (g == 2) ? t[2] : r;
  r = (g == 3) ? t[3] : r;
  return r;
}
// A pointer every lane holds, as a value the compiler knows to be the same in all of them.
__device__ __forceinline__ const uint8_t* uniform_ptr(const uint8_t* p) {
  const uint64_t v = (uint64_t)p;
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
  const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
  return (const uint8_t*)(((uint64_t)hi << 32) | lo);
}

// STREAM: the pages are read once by this launch, so they are fetched with non-temporal loads, which
// on this device sustain a visibly higher read rate than ordinary loads; launches that revisit pages
// (several row groups per KV head) use ordinary loads and find them in the L2 / memory-side cache.
template <int D, bool STREAM>
__device__ __forceinline__ void issue_pair(PairRegs<D>& pr, const AttnArgs& a, int h, int b0, int b1, int lane,
                                           const uint8_t* own_p0 /* tags of the lane's keys in page 0, or null */,
                                           int own_step /* bytes from there to the same keys in page 1 */) {
  using C = Bf16Cfg<D>;
  const long o0 = ((long)b0 * a.kv.num_kv_heads + h) * C::PAGE_U4 + lane;
  const long o1 = ((long)b1 * a.kv.num_kv_heads + h) * C::PAGE_U4 + lane;
  const u32x4* k0 = (const u32x4*)a.kv.k + o0;
  const u32x4* k1 = (const u32x4*)a.kv.k + o1;
  const u32x4* v0 = (const u32x4*)a.kv.v + o0;
  const u32x4* v1 = (const u32x4*)a.kv.v + o1;
#pragma unroll
  for (int i = 0; i < C::LPP; ++i) {
    if (STREAM) {
      pr.r[0][i] = __builtin_nontemporal_load(k0 + i * 64);
      pr.r[1][i] = __builtin_nontemporal_load(k1 + i * 64);
      pr.r[2][i] = __builtin_nontemporal_load(v0 + i * 64);
      pr.r[3][i] = __builtin_nontemporal_load(v1 + i * 64);
    } else {
      pr.r[0][i] = k0[i * 64];
      pr.r[1][i] = k1[i * 64];
      pr.r[2][i] = v0[i * 64];
      pr.r[3][i] = v1[i * 64];
    }
  }
  // Fetched with the pages, so that waiting for the tags never means waiting for younger pairs.
  if (own_p0) {
    pr.own[0] = *(const uint32_t*)own_p0;
    pr.own[1] = *(const uint32_t*)(own_p0 + own_step);
  }
}

// Running state of the rows one wave owns: output accumulators (transposed: [d][row]), softmax
// reference and sum per row, and what each row may see.
template <int D, int NT>
struct RowState {
  f32x4 acc[NT][D / 16];
  float m_run[NT], l_run[NT];
  int slot[NT], tag[NT];
  int base[NT];  // first slot of the row's own stage (kernels whose rows may belong to different stages)
};

// Largest of eight scores in four instructions.  Written as assembly because fmaxf() makes the compiler
// quiet a possible signalling NaN in every operand first (one more instruction each: 11 instead of 4
// per tile of every pair); scores are MFMA results or -inf and never NaN here, and the three-operand
// maximum returns a number whenever one operand is a number.
__device__ __forceinline__ float max8(const float (&x)[8]) {
  float r1, r2, r3, m;
  asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r1) : "v"(x[0]), "v"(x[1]), "v"(x[2]));
  asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r2) : "v"(x[3]), "v"(x[4]), "v"(x[5]));
  asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r3) : "v"(x[6]), "v"(x[7]), "v"(r1));
  asm("v_max_f32 %0, %1, %2" : "=v"(m) : "v"(r2), "v"(r3));
  return m;
}

// One pair of pages (32 keys) against NT 16-row tiles: scores, mask, running softmax, accumulation.
// `stage` holds K page 0, K page 1, V page 0, V page 1 (padded rows), `qtile` the rows' Q (padded rows).
// kr_even / kr_odd / vu are the lane's LDS bases (see the caller).  KB k-steps of K and VB d-tiles of
// V are fetched from LDS at a time: large batches hide the LDS latency, small ones save registers.
// QREG: the rows' Q operands come from registers (qr[n * KSTEPS + t]) instead of `qtile`.
// ROWBASE: every row brings the first slot of its own stage (ts.base) instead of the common `L`.
template <int D, int NT, int KB, int VB, bool QREG = false, bool ROWBASE = false>
__device__ __forceinline__ void pair_compute(const u32x4* stage, const u32x4* qtile, RowState<D, NT>& ts,
                                             int kr_even, int kr_odd, const int (&vu)[4], int g, int L,
                                             int mask_from, int P0, bool second_valid, uint32_t own0,
                                             uint32_t own1, float scale_log2, const bf16x8* qr = nullptr) {
  using C = Bf16Cfg<D>;
    // ---- S^T = K Q^T for both pages.  LDS operands are fetched KB k-steps (VB d-tiles below) at a
    // time: large batches hide the LDS latency, small ones leave registers to wide row groups.
    f32x4 st[2][NT];
#pragma unroll
    for (int n = 0; n < NT; ++n) {
      st[0][n] = f32x4{0.f, 0.f, 0.f, 0.f};
      st[1][n] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
#pragma unroll
    for (int t0 = 0; t0 < C::KSTEPS; t0 += KB) {
      bf16x8 ka[KB], kb[KB];
#pragma unroll
      for (int tt = 0; tt < KB; ++tt) {
        const int kr = (((t0 + tt) & 1) ? kr_odd : kr_even) + 8 * ((t0 + tt) >> 1);
        ka[tt] = *(const bf16x8*)&stage[0 * C::LPAGE_U4 + kr];
        kb[tt] = *(const bf16x8*)&stage[1 * C::LPAGE_U4 + kr];
      }
#pragma unroll
      for (int n = 0; n < NT; ++n) {
#pragma unroll
        for (int tt = 0; tt < KB; ++tt) {
          const int kr = (((t0 + tt) & 1) ? kr_odd : kr_even) + 8 * ((t0 + tt) >> 1);
          const bf16x8 qb = QREG ? qr[n * C::KSTEPS + t0 + tt] : *(const bf16x8*)&qtile[16 * n * C::LROW + kr];
          st[0][n] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka[tt], qb, st[0][n], 0, 0, 0);
          st[1][n] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kb[tt], qb, st[1][n], 0, 0, 0);
        }
      }
    }

    // ---- V^T operands through the LDS transpose read; the first batch is issued ahead of the
    // softmax so that its latency is hidden
    const s16x4* vs0 = (const s16x4*)(stage + 2 * C::LPAGE_U4);
    const s16x4* vs1 = (const s16x4*)(stage + 3 * C::LPAGE_U4);
#define ASPD_V_UNIT(mt) (vu[(mt) & 3] + 16 * ((mt) >> 2))
    s16x4 va[VB], vb[VB];
#pragma unroll
    for (int mm = 0; mm < VB; ++mm) {
      va[mm] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(vs0 + ASPD_V_UNIT(mm)));
      vb[mm] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(vs1 + ASPD_V_UNIT(mm)));
    }

    // ---- mask (only pages that reach into the branch region or the tail need it)
    const int slot0 = P0 * ASPD_BLOCK + 4 * g;  // first of this lane's four keys in page 0
    const bool need_mask = (P0 + 2) * ASPD_BLOCK > mask_from || !second_valid;

    // Running softmax with a lazily updated reference: ts.m_run[n] is a per-row reference exponent
    // (log2 domain, scaled scores), not necessarily the row maximum.  It is raised, and the
    // accumulators rescaled, only when a score exceeds it by more than LAZY (weights then stay
    // below 2^LAZY, harmless in fp32 and in the bf16 P operand, whose precision is relative).
    // The four lanes of a row always hold the same reference.
    s16x8 pb[NT];
#pragma unroll
    for (int n = 0; n < NT; ++n) {
      float sc[8];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        sc[e] = st[0][n][e];
        sc[4 + e] = st[1][n][e];
      }
      if (need_mask) {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const int jk = slot0 + (e & 3) + (e >> 2) * ASPD_BLOCK;
          const int own = (int)(((e < 4 ? own0 : own1) >> (8 * (e & 3))) & 0xff);
          const int stage_first = ROWBASE ? ts.base[n] : L;
          bool vis = (jk <= ts.slot[n]) && (jk < stage_first || ts.tag[n] == 0 || own == ts.tag[n]);
          if (e >= 4 && !second_valid) vis = false;
          sc[e] = vis ? sc[e] : -INFINITY;
        }
      }
      float mx = max8(sc);
      mx *= scale_log2;  // scale > 0: the maximum commutes with it
      if (__any(mx > ts.m_run[n] + LAZY)) {
        mx = fmaxf(mx, __shfl_xor(mx, 16));
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        const float m_new = fmaxf(ts.m_run[n], mx);
        const float alpha = __builtin_amdgcn_exp2f(ts.m_run[n] - exp2_safe_ref(m_new));
        ts.m_run[n] = m_new;
        ts.l_run[n] *= alpha;
#pragma unroll
        for (int mt = 0; mt < C::MT; ++mt) ts.acc[n][mt] *= alpha;
      }
      const float neg_ref = -exp2_safe_ref(ts.m_run[n]);
      float psum = 0.f;
      bf16x8 pv;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float w = __builtin_amdgcn_exp2f(fmaf(sc[e], scale_log2, neg_ref));
        psum += w;
        pv[e] = (__bf16)w;
      }
      ts.l_run[n] += psum;
      pb[n] = __builtin_bit_cast(s16x8, pv);
    }

    // ---- O^T += V^T P^T
#pragma unroll
    for (int m0 = 0; m0 < C::MT; m0 += VB) {
      if (m0 > 0) {
#pragma unroll
        for (int mm = 0; mm < VB; ++mm) {
          va[mm] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
              (__attribute__((address_space(3))) s16x4*)(vs0 + ASPD_V_UNIT(m0 + mm)));
          vb[mm] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
              (__attribute__((address_space(3))) s16x4*)(vs1 + ASPD_V_UNIT(m0 + mm)));
        }
      }
#pragma unroll
      for (int mm = 0; mm < VB; ++mm) {
        s16x8 v8;
        v8[0] = va[mm][0]; v8[1] = va[mm][1]; v8[2] = va[mm][2]; v8[3] = va[mm][3];
        v8[4] = vb[mm][0]; v8[5] = vb[mm][1]; v8[6] = vb[mm][2]; v8[7] = vb[mm][3];
        const bf16x8 vop = __builtin_bit_cast(bf16x8, v8);
#pragma unroll
        for (int n = 0; n < NT; ++n)
          ts.acc[n][m0 + mm] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vop, __builtin_bit_cast(bf16x8, pb[n]),
                                                                    ts.acc[n][m0 + mm], 0, 0, 0);
      }
    }
#undef ASPD_V_UNIT
}

constexpr int BLK_WIN = 512;   // pages of a segment whose block ids are staged in LDS at once

// The start-up loads of a segment, in registers: block ids of the first window, the Q rows, the row
// descriptors, and the first pair of pages of every wave (pair `wave` of the segment).
template <int D, int NT, int NW>
struct SegLoads {
  static constexpr int THREADS = NW * 64;
  static constexpr int BPT = BLK_WIN / THREADS;  // block ids per thread and window
  static constexpr int QL = (16 * NT * Bf16Cfg<D>::CH + THREADS - 1) / THREADS;  // Q chunks per thread
  int blkreg[BPT];
  u32x4 qreg[QL];
  int d_slot, d_branch, first_branch;  // of the thread's row: logical slot, global branch; the sequence's first branch
  int b0, b1;                          // block ids of the wave's first pair, as loaded from the block table
  int used0, used1;                    // the block ids `first` was fetched with
  PairRegs<D> first;
};

// Segment start-up, part one: the loads that depend on nothing but the segment.  The Q rows and row
// descriptors are fetched alongside the block ids, and each wave fetches the two block ids of its
// first pair itself.  Touches no LDS; every address stays in bounds for any `d` that passed seg_ok.
template <int D, int NT, int NW>
__device__ __forceinline__ void segment_issue_ids(const AttnArgs& a, const Seg& d, SegLoads<D, NT, NW>& ld) {
  using C = Bf16Cfg<D>;
  using LD = SegLoads<D, NT, NW>;
  constexpr int ROWS = 16 * NT;
  constexpr int THREADS = NW * 64;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int g = lane >> 4;
  const int R = d.nq * a.G;
  const int* bt = a.kv.block_tables + (long)d.s * a.kv.max_blocks_per_seq;
  const uint8_t* owner_row = a.slot_owner ? a.slot_owner + (long)d.s * a.owner_stride : nullptr;
  // The wave's own first pair: the same two addresses in every lane.  A wave past the end of a short
  // segment fetches the last page again (and never uses it) rather than branch: with the same loads in
  // flight on every path, the compiler's wait counts stay exact.
  const int P0 = min(d.page0 + 2 * wave, d.page1 - 1);
  ld.b0 = bt[P0];
  ld.b1 = bt[min(P0 + 1, d.page1 - 1)];
  // no load below depends on another, so that all of them are one round trip
  ld.first_branch = a.cu_branches ? a.cu_branches[d.s] : 0;
#pragma unroll
  for (int k = 0; k < LD::BPT; ++k) {
    const int P = min(d.page0 + tid + k * THREADS, d.page1 - 1);
    ld.blkreg[k] = bt[P];
  }
#pragma unroll
  for (int k = 0; k < LD::QL; ++k) {
    const int i = tid + k * THREADS;
    if (i < ROWS * C::CH) {
      const int r = i / C::CH, ch = i - r * C::CH;
      const int rr = min(r, R - 1);
      const int q = d.q0 + rr / a.G;
      const int head = d.h * a.G + rr % a.G;
      ld.qreg[k] = *((const u32x4*)a.q + ((long)q * a.kv.num_q_heads + head) * C::CH + ch);
    }
  }
  ld.d_slot = 0;
  ld.d_branch = -1;
  if (tid < ROWS) {
    const int rr = min(tid, R - 1);
    const int q = d.q0 + rr / a.G;
    ld.d_slot = a.logical_slot[q];
    ld.d_branch = a.q_branch[q];
  }
  // Owner tags travel with the pair whenever the call has any (the rows that need them are not known yet).
  // A call without tags loads two words it never looks at instead of branching: with the same loads in
  // flight on every path the compiler's wait counts stay exact (a branch here made the page loads below
  // wait for every load above).
  const uint8_t* own_p0 = owner_row ? owner_row + P0 * ASPD_BLOCK + 4 * g : (const uint8_t*)a.logical_slot;
  const int own_step = owner_row ? min(ASPD_BLOCK, a.owner_stride - 4 - (P0 * ASPD_BLOCK + 4 * g)) : 0;  // stays inside the owner row
  ld.first.own[0] = *(const uint32_t*)own_p0;
  ld.first.own[1] = *(const uint32_t*)(own_p0 + own_step);
}
// ... and the pages of the wave's first pair, from two block ids: those the plan carries for a
// workgroup's first segment (one round trip after the kernel starts), or those just loaded from the
// block table.  Any two blocks of the pool are safe to read; the segment compares them with the block
// table before it uses the pages.
template <int D, int NT, int NW, bool STREAM>
__device__ __forceinline__ void segment_issue_pair(const AttnArgs& a, const Seg& d, SegLoads<D, NT, NW>& ld, int b0,
                                                   int b1) {
  ld.used0 = min(max(__builtin_amdgcn_readfirstlane(b0), 0), a.kv.num_blocks - 1);
  ld.used1 = min(max(__builtin_amdgcn_readfirstlane(b1), 0), a.kv.num_blocks - 1);
  issue_pair<D, STREAM>(ld.first, a, d.h, ld.used0, ld.used1, threadIdx.x & 63, nullptr, 0);
}

// Segment start-up, part two, the stream and the epilogue.  `ld` holds the loads made for this very
// segment.
template <int D, int NT, int NW, int PF, bool STREAM>
__device__ void segment_bf16(const AttnArgs& a, char* smem, const Seg& it, bool complete, float* pslot,
                             const SegLoads<D, NT, NW>& ld) {
  using C = Bf16Cfg<D>;
  using LD = SegLoads<D, NT, NW>;
  constexpr int ROWS = 16 * NT;
  constexpr int THREADS = NW * 64;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int c = lane & 15;
  const int g = lane >> 4;
  const int R = it.nq * a.G;
  const int page0 = it.page0, page1 = it.page1, L = it.L;

  u32x4* stage = (u32x4*)(smem + wave * C::STAGE_BYTES);                // this wave's K0 K1 V0 V1
  u32x4* qtile = (u32x4*)(smem + NW * C::STAGE_BYTES);                  // [ROWS][LROW]
  int* rowslot = (int*)(smem + NW * C::STAGE_BYTES + ROWS * C::LROW * 16);
  int* rowtag = rowslot + ROWS;
  float* wm = (float*)(rowtag + ROWS);                                  // [NW][ROWS]
  float* wl = wm + NW * ROWS;
  int* blk_lds = (int*)(wl + NW * ROWS);                                // [BLK_WIN] block ids of the window
  int* pair_counter = blk_lds + BLK_WIN;                                // next pair nobody has taken yet

  const int* bt = a.kv.block_tables + (long)it.s * a.kv.max_blocks_per_seq;
  const uint8_t* owner_row = a.slot_owner ? a.slot_owner + (long)it.s * a.owner_stride : nullptr;

  __syncthreads();  // LDS of the previous segment is free
#pragma unroll
  for (int k = 0; k < LD::BPT; ++k) blk_lds[tid + k * THREADS] = min(max(ld.blkreg[k], 0), a.kv.num_blocks - 1);
  if (tid == 0) *pair_counter = NW;  // pairs 0 .. NW - 1 of the first window are on their way already
#pragma unroll
  for (int k = 0; k < LD::QL; ++k) {
    const int i = tid + k * THREADS;
    if (i < ROWS * C::CH) {
      const int r = i / C::CH, ch = i - r * C::CH;
      qtile[lds_pos<D>(r, ch)] = ld.qreg[k];
    }
  }
  if (tid < ROWS) {
    rowslot[tid] = ld.d_slot;
    rowtag[tid] = (ld.d_branch < 0 || !a.cu_branches) ? 0 : ld.d_branch - ld.first_branch + 1;
  }
  __syncthreads();

  RowState<D, NT> ts;
  int mask_from = L;  // keys below this slot are visible to every row of the group
  int last_slot = 0;  // keys above this slot are visible to none
#pragma unroll
  for (int n = 0; n < NT; ++n) {
    ts.slot[n] = rowslot[16 * n + c];
    ts.tag[n] = rowtag[16 * n + c];
    mask_from = min(mask_from, ts.slot[n]);
    last_slot = max(last_slot, ts.slot[n]);
  }
#pragma unroll
  for (int off = 1; off < 16; off <<= 1) {
    mask_from = min(mask_from, __shfl_xor(mask_from, off));
    last_slot = max(last_slot, __shfl_xor(last_slot, off));
  }
  mask_from = __builtin_amdgcn_readfirstlane(mask_from);
  last_slot = __builtin_amdgcn_readfirstlane(last_slot);

  // LDS addressing: every position used in the loop is one of a few lane-dependent bases
  // plus a compile-time offset (which the LDS instructions carry as an immediate).
  //   stage writes: lane owns 16-byte chunk (lane % CH) of row (lane / CH) + i * RPL
  const int wrow = lane / C::CH, wch = lane % C::CH;
  const int kw = lds_pos<D>(wrow, wch);
  //   K / Q operand reads: row c, chunk 4t + g; t even and t odd differ in bit 2 of the chunk
  const int kr_even = lds_pos<D>(c, g);
  const int kr_odd = lds_pos<D>(c, 4 + g);
  //   V transpose reads in 8-byte units: key 4g + c/4, d-tile mt at units 4 mt .. 4 mt + 3 of the row
  const int vkey = 4 * g + (c >> 2);
  int vu[4];
#pragma unroll
  for (int b = 0; b < 4; ++b) vu[b] = vkey * (2 * C::LROW) + 4 * b + (c & 3);

#pragma unroll
  for (int n = 0; n < NT; ++n) {
    ts.m_run[n] = -INFINITY;
    ts.l_run[n] = 0.f;
#pragma unroll
    for (int mt = 0; mt < C::MT; ++mt) ts.acc[n][mt] = f32x4{0.f, 0.f, 0.f, 0.f};
  }

  // ---- the stream.  Pairs of pages are handed out dynamically: a wave that gets its data sooner
  // takes the next pair sooner, so the waves of the workgroup finish together whatever the memory
  // system does to each of them.  A wave keeps PF pairs in flight in a ring of register sets (the
  // ring is unrolled so that every set has fixed registers); the set it has just emptied into its
  // LDS stage is refilled at once, before the pair is computed.
  PairRegs<D> pr[PF];
  int idx[PF];
  // owner tags are needed (and fetched) only for pairs that reach past mask_from
  auto own_ptr = [&](int P0) -> const uint8_t* {
    return (owner_row && (P0 + 2) * ASPD_BLOCK > mask_from) ? owner_row + P0 * ASPD_BLOCK + 4 * g : nullptr;
  };
  auto own_step = [&](int P0) -> int {
    return min(ASPD_BLOCK, a.owner_stride - 4 - (P0 * ASPD_BLOCK + 4 * g));  // stays inside the owner row
  };
  for (int wbase = page0; wbase < page1; wbase += BLK_WIN) {  // windows of block ids; normally one
    const int wend = min(page1, wbase + BLK_WIN);
    const int wpages = wend - wbase;
    const int npairs = (wpages + 1) >> 1;
    if (wbase != page0) {
      __syncthreads();  // every wave is done with the previous window's ids and counter
#pragma unroll
      for (int k = 0; k < LD::BPT; ++k) {
        const int P = min(wbase + tid + k * THREADS, page1 - 1);
        blk_lds[tid + k * THREADS] = min(max(bt[P], 0), a.kv.num_blocks - 1);
      }
      if (tid == 0) *pair_counter = 0;
      __syncthreads();
    }
    auto take = [&]() -> int {  // next pair nobody has taken (may be past the end)
      int v = 0;
      if (lane == 0) v = atomicAdd(pair_counter, 1);
      return __builtin_amdgcn_readfirstlane(v);
    };
#pragma unroll
    for (int sl = 0; sl < PF; ++sl) {
      if (sl == 0 && wbase == page0) {  // fetched at start-up
        idx[0] = wave;
        pr[0] = ld.first;
        // ... with block ids that may have come from the plan: fetched again if the block table the
        // call was given says otherwise
        const int a0 = __builtin_amdgcn_readfirstlane(blk_lds[min(2 * wave, wpages - 1)]);
        const int a1 = __builtin_amdgcn_readfirstlane(blk_lds[min(2 * wave + 1, wpages - 1)]);
        if (a0 != ld.used0 || a1 != ld.used1) issue_pair<D, STREAM>(pr[0], a, it.h, a0, a1, lane, nullptr, 0);
        continue;
      }
      idx[sl] = take();
      if (idx[sl] < npairs) {
        const int b0 = __builtin_amdgcn_readfirstlane(blk_lds[2 * idx[sl]]);
        const int b1 = __builtin_amdgcn_readfirstlane(blk_lds[min(2 * idx[sl] + 1, wpages - 1)]);
        issue_pair<D, STREAM>(pr[sl], a, it.h, b0, b1, lane, own_ptr(wbase + 2 * idx[sl]), own_step(wbase + 2 * idx[sl]));
      }
    }
    int ahead = take();  // always one hand-out ahead, so that a refill never waits for the counter
    bool more = true;
    while (more) {
#pragma unroll
      for (int sl = 0; sl < PF; ++sl) {
        // pairs are handed out in increasing order: once the oldest outstanding one is past the end,
        // all are
        if (idx[sl] >= npairs) {
          more = false;
          break;
        }
        const int pair = idx[sl];
        const int P0 = wbase + 2 * pair;
        // Slots past the last row's own slot have never been written (the tail of the last page) and may
        // hold anything: their V rows enter the second product with weight zero, and zero times a NaN
        // is a NaN, so they are cleared on the way into LDS.  (Their K rows only reach scores that the
        // mask replaces.)
        if ((P0 + 2) * ASPD_BLOCK > last_slot + 1) {
#pragma unroll
          for (int i = 0; i < C::LPP; ++i) {
            const int key = P0 * ASPD_BLOCK + wrow + i * C::RPL;
            if (key > last_slot) pr[sl].r[2][i] = u32x4{0u, 0u, 0u, 0u};
            if (key + ASPD_BLOCK > last_slot) pr[sl].r[3][i] = u32x4{0u, 0u, 0u, 0u};
          }
        }
        // ---- registers -> this wave's LDS stage
#pragma unroll
        for (int i = 0; i < C::LPP; ++i) {
          // the position is a lane-dependent base plus a compile-time offset
          constexpr int STEP = C::RPL * C::LROW;  // load i of a page is rows i * RPL .. of it
          stage[0 * C::LPAGE_U4 + i * STEP + kw] = pr[sl].r[0][i];
          stage[1 * C::LPAGE_U4 + i * STEP + kw] = pr[sl].r[1][i];
          stage[2 * C::LPAGE_U4 + i * STEP + kw] = pr[sl].r[2][i];
          stage[3 * C::LPAGE_U4 + i * STEP + kw] = pr[sl].r[3][i];
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        // ---- refill the set: the next pair streams in while this one is computed
        idx[sl] = ahead;
        const uint32_t own0 = pr[sl].own[0], own1 = pr[sl].own[1];  // of the pair about to be computed
        if (ahead < npairs) {
          const int b0 = __builtin_amdgcn_readfirstlane(blk_lds[2 * ahead]);
          const int b1 = __builtin_amdgcn_readfirstlane(blk_lds[min(2 * ahead + 1, wpages - 1)]);
          issue_pair<D, STREAM>(pr[sl], a, it.h, b0, b1, lane, own_ptr(wbase + 2 * ahead), own_step(wbase + 2 * ahead));
        }
        ahead = take();

        const bool second_valid = (P0 + 1) < wend;

        constexpr bool ROOMY = (NW <= 4);  // one wave per SIMD: 512 registers
        constexpr int KB = (NT == 1 || ROOMY) ? C::KSTEPS : (NT == 2 ? 2 : 1);
        constexpr int VB = (NT == 1 || ROOMY) ? C::MT : (NT == 2 ? 4 : 2);
        pair_compute<D, NT, KB, VB>(stage, qtile, ts, kr_even, kr_odd, vu, g, L, mask_from, P0, second_valid, own0,
                                    own1, a.scale_log2);
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
      }
    }
  }

  // ---- combine the waves of the workgroup
#pragma unroll
  for (int n = 0; n < NT; ++n) {
    ts.l_run[n] += __shfl_xor(ts.l_run[n], 16);
    ts.l_run[n] += __shfl_xor(ts.l_run[n], 32);
    if (g == 0) {
      wm[wave * ROWS + 16 * n + c] = ts.m_run[n];
      wl[wave * ROWS + 16 * n + c] = ts.l_run[n];
    }
  }
  __syncthreads();  // also: every wave is done with its stage, which `red` aliases from here on
  float* red = (float*)smem;  // [NW][16][D + 4]: rows padded by four banks so that the 16 rows a wave
                              // writes at once fall on different banks
  constexpr int RS = D + 4;
#pragma unroll
  for (int n = 0; n < NT; ++n) {
    {
      float mg = -INFINITY;
#pragma unroll
      for (int w = 0; w < NW; ++w) mg = fmaxf(mg, wm[w * ROWS + 16 * n + c]);
      const float f = __builtin_amdgcn_exp2f(ts.m_run[n] - exp2_safe_ref(mg));
#pragma unroll
      for (int mt = 0; mt < C::MT; ++mt) {
        f32x4 v = ts.acc[n][mt] * f;
        *(f32x4*)&red[(wave * 16 + c) * RS + 16 * mt + 4 * g] = v;
      }
    }
    __syncthreads();
    {
      // Consecutive lanes take consecutive 16-byte chunks of the tile: every store fills whole lines.
      constexpr int CPR = D / 4;  // chunks per row
      constexpr int PASSES = (16 * CPR + THREADS - 1) / THREADS;
      auto row_stats = [&](int r, float* mg_out, float* lg_out) {
        float mg = -INFINITY;
#pragma unroll
        for (int w = 0; w < NW; ++w) mg = fmaxf(mg, wm[w * ROWS + r]);
        const float mref = exp2_safe_ref(mg);
        float lg = 0.f;
#pragma unroll
        for (int w = 0; w < NW; ++w) lg += wl[w * ROWS + r] * __builtin_amdgcn_exp2f(wm[w * ROWS + r] - mref);
        *mg_out = mg;
        *lg_out = lg;
      };
      // The index arithmetic below (divisions by G among it) depends on nothing the main loop produces;
      // tying it to a value defined here keeps it, and the registers it needs, out of that loop.
      int tid_here = tid;
      asm volatile("" : "+v"(tid_here)::"memory");
#pragma unroll
      for (int k = 0; k < PASSES; ++k) {
        const int ci = tid_here + k * THREADS;
        if ((16 * CPR) % THREADS != 0 && ci >= 16 * CPR) break;
        const int row = ci / CPR;
        const int d0 = 4 * (ci % CPR);
        const int r = 16 * n + row;
        f32x4 o = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int w = 0; w < NW; ++w) o += *(const f32x4*)&red[(w * 16 + row) * RS + d0];
        if (r >= R) continue;
        if (complete) {
          float mg, lg;
          row_stats(r, &mg, &lg);
          const int q = it.q0 + r / a.G;
          const int head = it.h * a.G + r % a.G;
          const float inv = 1.f / lg;
          __bf16* dst = (__bf16*)a.out + ((long)q * a.kv.num_q_heads + head) * D + d0;
          typedef __attribute__((ext_vector_type(4))) __bf16 out_vec;
          out_vec ov;
#pragma unroll
          for (int e = 0; e < 4; ++e) ov[e] = (__bf16)(o[e] * inv);
          *(out_vec*)dst = ov;
          if (a.lse && d0 == 0) a.lse[(long)q * a.kv.num_q_heads + head] = (mg + log2f(lg)) * LN2;
        } else {
          store_device_scope_x4(partial_acc(pslot, r, D) + d0, o);
        }
      }
      if (!complete && tid_here < 16 && 16 * n + tid_here < R) {
        float mg, lg;
        row_stats(16 * n + tid_here, &mg, &lg);
        store_device_scope_x4(partial_stat(a, pslot, 16 * n + tid_here, D), f32x4{mg, lg, 0.f, 0.f});
      }
    }
    __syncthreads();
  }
}


template <int D, int NT, int NW>
size_t bf16_smem_bytes() {
  return NW * Bf16Cfg<D>::STAGE_BYTES + 16 * NT * Bf16Cfg<D>::LROW * 16 + 2 * 16 * NT * 4 + 2 * NW * 16 * NT * 4 +
         (BLK_WIN + 4) * 4;
}

// What every kernel does first: its workgroup's header of the plan.  Returns the number of segments
// (0: nothing to do, also for a header that fails seg_ok).  `ids`: the block ids of the pages
// first_id, first_id + 1 of the first segment (first_id even, below PLAN_IDS).  Two loads, no branch
// between them and their uses: scalar loads return in any order, so a wait between them would make each
// a memory round trip of its own.
__device__ __forceinline__ int plan_begin(const AttnArgs& a, Seg* first, int* next, int first_id = 0,
                                          i32x2* ids = nullptr) {
  static_assert(PLAN_HDR_NSEG == 8 && PLAN_HDR_NEXT == 9, "segment and counts in one 64-byte load");
  const int32_t* hdr = a.plan + (long)PLAN_HDR * blockIdx.x;
  const i32x16 w = load_words16(hdr);
  const i32x2 b = load_words2(hdr + PLAN_HDR_IDS + first_id);
  // (both are needed here, so neither load is moved further down, behind other waits)
  asm volatile("" ::"s"(w[0]), "s"(b[0]), "s"(b[1]));
  if (ids) *ids = b;
  *first = seg_of(w);
  *next = w[PLAN_HDR_NEXT];
  return ((int)(w[PLAN_HDR_NSEG] > 0) & (int)seg_ok(a, *first)) ? w[PLAN_HDR_NSEG] : 0;
}
__device__ __forceinline__ Seg plan_segment(const AttnArgs& a, int index) {
  return load_seg(a.plan + (long)PLAN_HDR * a.nwg + (long)PLAN_SEG * index);
}

template <int D, int NT, int NW, int PF, bool STREAM>
__global__ __launch_bounds__(NW * 64) __attribute__((amdgpu_waves_per_eu(NW / 4, NW / 4))) void attn_bf16_kernel(
    AttnArgs a) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  __shared__ int merge_flag;
  constexpr int THREADS = NW * 64;
  static_assert(2 * NW <= PLAN_IDS, "the plan carries two block ids per wave");
  // One memory round trip after the kernel starts the workgroup knows its first segment and the blocks
  // of each wave's first pair of pages (scalar loads of the plan header), and the pages, the block ids of
  // the whole segment, the Q rows and the row descriptors all leave together.
  Seg seg;
  int next;
  i32x2 ids;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int nseg = plan_begin(a, &seg, &next, 2 * wave, &ids);
  if (nseg == 0) return;
  SegLoads<D, NT, NW> ld;
  // (loads return in order: the small ones first, the LDS set-up waits for them and not for the pages)
  segment_issue_ids<D, NT, NW>(a, seg, ld);
  segment_issue_pair<D, NT, NW, STREAM>(a, seg, ld, ids[0], ids[1]);
  asm volatile("" ::: "memory");  // the loads leave here, not where their results are first used
  for (int i = 0;;) {
    // the next segment's words are on their way while this one streams
    Seg after = seg;
    if (i + 1 < nseg) after = plan_segment(a, next + i);
    const bool complete = seg_complete(seg);
    float* pslot = partial_slot(a, blockIdx.x, seg.page0 == 0 ? 1 : 0, D);
    segment_bf16<D, NT, NW, PF, STREAM>(a, smem, seg, complete, pslot, ld);
    // the merging workgroup has 16 * NT rows of D / 4 chunks to combine: one pass of its 64 * NW threads
    if (!complete) announce_partial<D, true, THREADS, (NT == 1 ? 2 : 3)>(a, seg, &merge_flag);
    if (++i >= nseg) break;
    seg = after;
    if (!seg_ok(a, seg)) break;
    segment_issue_ids<D, NT, NW>(a, seg, ld);
    segment_issue_pair<D, NT, NW, STREAM>(a, seg, ld, ld.b0, ld.b1);
  }
}

// ---------------------------------------------------------------------------------------------
// bf16, many rows per KV head (branch chunks): the waves of a workgroup split the ROWS instead of
// the keys.  Every group of ROWS_PPS pairs of pages is loaded once per workgroup, cooperatively, into a
// double-buffered LDS stage that all waves read; each wave keeps its own 16*NT rows (Q operands,
// accumulators, softmax state, all in registers) for the whole segment, so there is no reduction
// across waves.  One barrier per group.  With NW waves a row group holds NW * 16 * NT rows, and the pages of a KV head
// are fetched once per that many rows.  The product per pair is compute-bound here (rows x 32 keys x
// D on the MFMA units, the softmax on the vector ALU, the operands out of LDS), which is why the
// waves share the loads rather than the keys.  Measured: 8 waves of 32 rows beat 8 of 48 (whose Q
// operands no longer fit in registers) and 4 of 64 (one wave per SIMD overlaps nothing).
// A wave skips the arithmetic for pairs that none of its rows can see (the chunks and earlier
// tokens of other branches).
// ---------------------------------------------------------------------------------------------
template <int D, int NT, int NW>
size_t rows_smem_bytes() {
  return 2 * ROWS_PPS * Bf16Cfg<D>::STAGE_BYTES + (BLK_WIN + 4) * 4;
}

// SEQ: the rows are tokens of a whole multi-stage sequence (aspd_attn_full_sequence): each brings the first
// slot of its own stage (a.row_base) and its branch number within that stage; otherwise all rows belong to
// the sequence's running stage, which starts at it.L.
template <int D, int NT, int NW, bool SEQ = false>
__device__ void segment_rows(const AttnArgs& a, char* smem, const Seg& it, bool complete, float* pslot) {
  using C = Bf16Cfg<D>;
  constexpr int ROWS = 16 * NT;        // rows per wave
  constexpr int THREADS = NW * 64;
  constexpr int PPS = ROWS_PPS;          // pairs per stage: all of them are staged, then computed, between two barriers
  constexpr int ARR = 4 * PPS;           // page arrays of a stage: K0 K1 V0 V1 of every pair
  constexpr int PER_PAGE = THREADS / ARR;  // threads that share the load of one page
  static_assert(THREADS % ARR == 0 && C::PAGE_U4 % PER_PAGE == 0, "page not divisible among its loaders");
  constexpr int LPT = C::PAGE_U4 / PER_PAGE;  // 16-byte loads per thread and page
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int c = lane & 15;
  const int g = lane >> 4;
  const int R = it.nq * a.G;                       // rows of the whole row group
  const int page0 = it.page0, page1 = it.page1;
  const int Rw = min(ROWS, R - wave * ROWS);       // rows this wave owns (<= 0: none)
  const bool wave_active = Rw > 0;

  u32x4* stage0 = (u32x4*)smem;                 // [2][PPS][K0 K1 V0 V1]
  int* blk_lds = (int*)(smem + 2 * PPS * C::STAGE_BYTES);

  const int* bt = a.kv.block_tables + (long)it.s * a.kv.max_blocks_per_seq;
  const uint8_t* owner_row = a.slot_owner ? uniform_ptr(a.slot_owner + (long)it.s * a.owner_stride) : nullptr;
  // The rows of a group are packed in the order of their slots: the last row's slot bounds what any row
  // of the group may see.  Slots past it have never been written (the tail of the last page) and may hold
  // anything; their V rows are cleared on the way into LDS (zero weight times a NaN would be a NaN).
  const int last_slot = __builtin_amdgcn_readfirstlane(a.logical_slot[it.q0 + it.nq - 1]);

  // ---- start-up: block ids of the first window; this wave's Q operands and row descriptors go
  // straight to registers (lane (c, g) holds, of row c of every tile, the 16-byte pieces 4t + g)
  constexpr int BPT = BLK_WIN / THREADS;
  int blkreg[BPT];
#pragma unroll
  for (int k = 0; k < BPT; ++k) blkreg[k] = bt[min(page0 + tid + k * THREADS, page1 - 1)];
  RowState<D, NT> ts;
  bf16x8 qr[NT * C::KSTEPS];
  // What the wave's rows have in common decides which pairs need a mask and which can be left out:
  //   mask_from  every key below this slot is visible to every row (below every row's stage and slot);
  //   slot_hi    no key above this slot is visible to any row;
  //   base_hi    the latest stage start among the rows.  A row of an earlier stage lies below it, so keys
  //              from base_hi on are visible, if at all, only to the rows of that latest stage, and only
  //              where their branch tags match: [tag_lo, tag_hi] is the range of those rows' tags.
  int mask_from = 0x7fffffff, slot_hi = 0, base_hi = 0;
#pragma unroll
  for (int n = 0; n < NT; ++n) {
    const int rr = min(wave * ROWS + 16 * n + c, R - 1);  // padding rows (and idle waves) repeat the last row
    const int q = it.q0 + rr / a.G;
    const int head = it.h * a.G + rr % a.G;
    const u32x4* qsrc = (const u32x4*)a.q + ((long)q * a.kv.num_q_heads + head) * C::CH + g;
#pragma unroll
    for (int t = 0; t < C::KSTEPS; ++t) qr[n * C::KSTEPS + t] = __builtin_bit_cast(bf16x8, qsrc[4 * t]);
    ts.slot[n] = a.logical_slot[q];
    const int qb = a.q_branch[q];
    if (SEQ) {
      // (no owner tags: the shared mask, every row is treated like a main-branch row)
      ts.tag[n] = a.slot_owner ? max(qb, -1) + 1 : 0;
      ts.base[n] = a.slot_owner ? a.row_base[q] : ts.slot[n];
    } else {
      ts.tag[n] = (qb < 0 || !a.cu_branches) ? 0 : qb - a.cu_branches[it.s] + 1;
      ts.base[n] = it.L;
    }
    mask_from = min(mask_from, min(ts.slot[n], ts.base[n]));
    slot_hi = max(slot_hi, ts.slot[n]);
    base_hi = max(base_hi, ts.base[n]);
    ts.m_run[n] = -INFINITY;
    ts.l_run[n] = 0.f;
#pragma unroll
    for (int mt = 0; mt < C::MT; ++mt) ts.acc[n][mt] = f32x4{0.f, 0.f, 0.f, 0.f};
  }
  __syncthreads();  // LDS of the previous segment is free
#pragma unroll
  for (int k = 0; k < BPT; ++k) blk_lds[tid + k * THREADS] = min(max(blkreg[k], 0), a.kv.num_blocks - 1);
  __syncthreads();
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    mask_from = min(mask_from, __shfl_xor(mask_from, off));
    slot_hi = max(slot_hi, __shfl_xor(slot_hi, off));
    base_hi = max(base_hi, __shfl_xor(base_hi, off));
  }
  mask_from = __builtin_amdgcn_readfirstlane(mask_from);
  slot_hi = __builtin_amdgcn_readfirstlane(slot_hi);
  base_hi = __builtin_amdgcn_readfirstlane(base_hi);
  int tag_lo = 0x7fffffff, tag_hi = 0;
#pragma unroll
  for (int n = 0; n < NT; ++n) {
    if (ts.base[n] == base_hi) {
      tag_lo = min(tag_lo, ts.tag[n]);
      tag_hi = max(tag_hi, ts.tag[n]);
    }
  }
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    tag_lo = min(tag_lo, __shfl_xor(tag_lo, off));
    tag_hi = max(tag_hi, __shfl_xor(tag_hi, off));
  }
  tag_lo = __builtin_amdgcn_readfirstlane(tag_lo);
  tag_hi = __builtin_amdgcn_readfirstlane(tag_hi);

  // LDS bases of this lane (same layout as the streaming kernel)
  const int kr_even = lds_pos<D>(c, g);
  const int kr_odd = lds_pos<D>(c, 4 + g);
  const int vkey = 4 * g + (c >> 2);
  int vu[4];
#pragma unroll
  for (int b = 0; b < 4; ++b) vu[b] = vkey * (2 * C::LROW) + 4 * b + (c & 3);
  // cooperative load: PER_PAGE threads share one page array, consecutive threads consecutive 16 bytes
  const int lpage = tid / PER_PAGE;          // pair lpage / 4 of the group, array lpage % 4: K0, K1, V0, V1
  const int lt = tid - lpage * PER_PAGE;
  const bool l_is_k = (lpage & 3) < 2;
  int lpos[LPT];                             // positions inside the page in LDS
#pragma unroll
  for (int k = 0; k < LPT; ++k) {
    const int i = lt + k * PER_PAGE;         // chunk index inside the page
    const int row = i / C::CH, ch = i - row * C::CH;
    lpos[k] = lds_pos<D>(row, ch);
  }

  constexpr int RD = ROWS_PREFETCH;  // groups on their way per workgroup (a ring of register sets)
  u32x4 nxt[RD][LPT];
  for (int wbase = page0; wbase < page1; wbase += BLK_WIN) {  // windows of block ids; normally one
    const int wend = min(page1, wbase + BLK_WIN);
    const int wpages = wend - wbase;
    const int npairs = (wpages + 1) >> 1;
    const int ngroups = (npairs + PPS - 1) / PPS;
    if (wbase != page0) {
      __syncthreads();
#pragma unroll
      for (int k = 0; k < BPT; ++k)
        blk_lds[tid + k * THREADS] = min(max(bt[min(wbase + tid + k * THREADS, page1 - 1)], 0), a.kv.num_blocks - 1);
      __syncthreads();
    }
    // This thread's slice of group gi.  Issued for every ring slot, also past the end of the window (the
    // last pages again, which the caches hold): the number of loads younger than a slot is then fixed,
    // so waiting for the oldest slot leaves the younger ones in flight.
    // the page (of the window) this thread loads for group gi
    auto page_of = [&](int gi) -> int {
      const int p = min(gi * PPS + (lpage >> 2), npairs - 1);
      return min(2 * p + (lpage & 1), wpages - 1);
    };
    auto issue = [&](u32x4 (&dst)[LPT], int gi) {
      const int pg = page_of(gi);
      const int b = blk_lds[pg];
      const u32x4* src = (const u32x4*)(l_is_k ? a.kv.k : a.kv.v) + ((long)b * a.kv.num_kv_heads + it.h) * C::PAGE_U4;
#pragma unroll
      for (int k = 0; k < LPT; ++k) dst[k] = src[lt + k * PER_PAGE];
    };
    // owner tags of the pairs that reach into the branch region, fetched one group ahead like the pages
    auto tags_of = [&](int gi, u32x4 (&t)[PPS][2]) {
#pragma unroll
      for (int h = 0; h < PPS; ++h) {
        const int P = wbase + 2 * (gi * PPS + h);
        if (owner_row && P < wend && (P + 2) * ASPD_BLOCK > mask_from) {
          t[h][0] = load_tags_uniform(owner_row + P * ASPD_BLOCK);
          t[h][1] = load_tags_uniform(owner_row + min(P + 1, page1 - 1) * ASPD_BLOCK);  // stays inside the owner row
        }
      }
    };
    u32x4 tn[PPS][2];
#pragma unroll
    for (int h = 0; h < PPS; ++h) tn[h][0] = tn[h][1] = u32x4{0, 0, 0, 0};
#pragma unroll
    for (int d = 0; d < RD; ++d) issue(nxt[d], d);
    tags_of(0, tn);
    for (int gbase = 0; gbase < ngroups; gbase += RD) {
#pragma unroll
    for (int d = 0; d < RD; ++d) {  // the ring is unrolled so that every slot has fixed registers
      const int gi = gbase + d;
      if (gi >= ngroups) break;
      u32x4* stage = stage0 + (gi & 1) * (PPS * C::STAGE_BYTES / 16);
      const int key0 = (wbase + page_of(gi)) * ASPD_BLOCK;  // first slot of the page this thread staged
      if (!l_is_k && key0 + ASPD_BLOCK > last_slot + 1) {
#pragma unroll
        for (int k = 0; k < LPT; ++k)
          if (key0 + (lt + k * PER_PAGE) / C::CH > last_slot) nxt[d][k] = u32x4{0u, 0u, 0u, 0u};
      }
#pragma unroll
      for (int k = 0; k < LPT; ++k) stage[lpage * C::LPAGE_U4 + lpos[k]] = nxt[d][k];
      u32x4 tc[PPS][2];
#pragma unroll
      for (int h = 0; h < PPS; ++h) {
        tc[h][0] = tn[h][0];
        tc[h][1] = tn[h][1];
      }
      issue(nxt[d], gi + RD);
      if (gi + 1 < ngroups) tags_of(gi + 1, tn);
      __syncthreads();  // the group is staged; everyone is done with the other buffer's previous group

      if (!wave_active) continue;
#pragma unroll
      for (int h = 0; h < PPS; ++h) {
        const int P0 = wbase + 2 * (gi * PPS + h);
        if (P0 >= wend) break;
        // keys past the last of this wave's rows (whole sequences only: the rows of a decode or chunk step
        // sit at the tail of their sequence, and the test costs the chunk launch 3 %)
        if (SEQ && P0 * ASPD_BLOCK > slot_hi) continue;
        const bool second_valid = (P0 + 1) < wend;
        uint32_t own0 = 0, own1 = 0;
        if (owner_row && (P0 + 2) * ASPD_BLOCK > mask_from) {
          own0 = lane_tags(tc[h][0], g);
          own1 = lane_tags(tc[h][1], g);
          // pairs wholly inside the latest stage: skip if no key belongs to a branch of this wave's rows there
          if (P0 * ASPD_BLOCK >= base_hi && tag_lo > 0) {
            bool mine = false;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
              const int own = (int)(((e < 4 ? own0 : own1) >> (8 * (e & 3))) & 0xff);
              mine |= (own >= tag_lo && own <= tag_hi);
            }
            if (!__any(mine)) continue;
          }
        }
        constexpr int KB = 2;
        constexpr int VB = 4;
        pair_compute<D, NT, KB, VB, true, true>(stage + h * 4 * C::LPAGE_U4, nullptr, ts, kr_even, kr_odd, vu, g, 0,
                                                mask_from, P0, second_valid, own0, own1, a.scale_log2, qr);
      }
    }
    }
  }

  // ---- every wave writes its own rows
  if (!wave_active) return;
#pragma unroll
  for (int n = 0; n < NT; ++n) {
    ts.l_run[n] += __shfl_xor(ts.l_run[n], 16);
    ts.l_run[n] += __shfl_xor(ts.l_run[n], 32);
    const int r = wave * ROWS + 16 * n + c;  // row inside the row group
    if (16 * n + c >= Rw) continue;
    if (complete) {
      const int q = it.q0 + r / a.G;
      const int head = it.h * a.G + r % a.G;
      const float inv = 1.f / ts.l_run[n];
      __bf16* dst = (__bf16*)a.out + ((long)q * a.kv.num_q_heads + head) * D;
      typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
#pragma unroll
      for (int mt = 0; mt < C::MT; ++mt) {
        bf16x4 ov;
#pragma unroll
        for (int e = 0; e < 4; ++e) ov[e] = (__bf16)(ts.acc[n][mt][e] * inv);
        *(bf16x4*)(dst + 16 * mt + 4 * g) = ov;
      }
      if (a.lse && g == 0) a.lse[(long)q * a.kv.num_q_heads + head] = (ts.m_run[n] + log2f(ts.l_run[n])) * LN2;
    } else {
      float* dst = partial_acc(pslot, r, D);
#pragma unroll
      for (int mt = 0; mt < C::MT; ++mt) store_device_scope_x4(dst + 16 * mt + 4 * g, ts.acc[n][mt]);
      if (g == 0) store_device_scope_x4(partial_stat(a, pslot, r, D), f32x4{ts.m_run[n], ts.l_run[n], 0.f, 0.f});
    }
  }
}

template <int D, int NT, int NW>
__global__ __launch_bounds__(NW * 64) __attribute__((amdgpu_waves_per_eu(NW / 4, NW / 4))) void attn_bf16_rows_kernel(
    AttnArgs a) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  __shared__ int merge_flag;
  constexpr int THREADS = NW * 64;
  Seg seg;
  int next;
  const int nseg = plan_begin(a, &seg, &next);
  for (int i = 0; i < nseg; ++i) {
    if (i > 0) {
      seg = plan_segment(a, next + i - 1);
      if (!seg_ok(a, seg)) break;
    }
    const bool complete = seg_complete(seg);
    float* pslot = partial_slot(a, blockIdx.x, seg.page0 == 0 ? 1 : 0, D);
    segment_rows<D, NT, NW>(a, smem, seg, complete, pslot);
    if (!complete) announce_partial<D, true, THREADS, 2>(a, seg, &merge_flag);
  }
}

// ---------------------------------------------------------------------------------------------
// Whole sequences (teacher forcing, re-prefill): every token of the batch is a query row.  The row
// groups (qpg consecutive tokens of a sequence, one KV head) are listed in the step's plan, longest key
// range first; workgroups take them from the list as they become free (the ranges differ by two orders
// of magnitude, so no static split would balance), through one counter in the workspace that the last
// workgroup to finish puts back to zero.  Every group is computed whole by one workgroup with the
// row-splitting arithmetic above: nothing is split, nothing merged.
// ---------------------------------------------------------------------------------------------
template <int D, int NT, int NW>
__global__ __launch_bounds__(NW * 64) __attribute__((amdgpu_waves_per_eu(NW / 4, NW / 4))) void attn_bf16_seq_kernel(
    AttnArgs a) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  __shared__ int next_item;
  const int n_groups = a.plan[0];
  const int32_t* items = a.plan + SEQ_PLAN_HDR + ((a.NQ + 3) & ~3);
  const int Hkv = a.kv.num_kv_heads;
  const long total = (long)n_groups * Hkv;
  for (;;) {
    if (threadIdx.x == 0) next_item = atomicAdd(a.counters, 1);
    __syncthreads();
    const int e = next_item;
    __syncthreads();  // everyone has read it before the next round overwrites it
    if (e >= total) break;
    const i32x4 w = *(const i32x4*)(items + 4 * (e / Hkv));
    Seg seg;
    seg.s = w[0];
    seg.h = e % Hkv;
    seg.q0 = w[1];
    seg.nq = w[2];
    seg.page0 = 0;
    seg.page1 = seg.np = w[3];
    seg.owner = seg.w_last = 0;
    seg.L = 0;
    // the list is the library's own; the check keeps a workgroup that is handed anything else inside the
    // call's arrays
    const bool ok = (int)(seg.s >= 0) & (int)(seg.s < a.B) & (int)(seg.q0 >= 0) & (int)(seg.nq >= 1) &
                    (int)(seg.nq <= a.qpg) & (int)(seg.q0 <= a.NQ - seg.nq) & (int)(seg.np >= 1) &
                    (int)(seg.np <= a.kv.max_blocks_per_seq);
    if (!ok) continue;
    segment_rows<D, NT, NW, true>(a, smem, seg, true, nullptr);
  }
  // the last workgroup to leave puts the two counters back to zero for the next launch
  if (threadIdx.x == 0) {
    const int gone = atomicAdd(a.counters + 1, 1);
    if (gone == (int)gridDim.x - 1) {
      atomicExch(a.counters, 0);
      atomicExch(a.counters + 1, 0);
    }
  }
}

// ---------------------------------------------------------------------------------------------
// fp32 path: vector ALU, fp32 throughout.  Lane (k = lane % 16, g = lane / 16) owns key k of each
// page and the g-th quarter of head_dim; a row's score is completed across the four quarters with
// two butterfly adds.  Every lane keeps a private running softmax over the keys it has seen
// (one per page) and they are combined once at the end of the segment.
// ---------------------------------------------------------------------------------------------
template <int D>
__device__ void segment_f32(const AttnArgs& a, char* smem, const Seg& it, bool complete, float* pslot) {
  constexpr int QD = D / 4;  // floats per lane per key
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int k = lane & 15;
  const int g = lane >> 4;
  const int R = it.nq * a.G;
  const int page0 = it.page0, page1 = it.page1, L = it.L;

  float* qtile = (float*)smem;                           // [F32_ROWS][D]
  int* rowslot = (int*)(qtile + F32_ROWS * D);
  int* rowtag = rowslot + F32_ROWS;
  float* red = (float*)(rowtag + F32_ROWS);              // [THREADS][F32_ROWS][QD + 2]

  __syncthreads();
  for (int i = tid; i < F32_ROWS * D; i += THREADS) {
    const int r = i / D, d = i - r * D;
    const int rr = min(r, R - 1);
    const int q = it.q0 + rr / a.G;
    const int head = it.h * a.G + rr % a.G;
    qtile[i] = ((const float*)a.q)[((long)q * a.kv.num_q_heads + head) * D + d];
  }
  if (tid < F32_ROWS) {
    const int rr = min(tid, R - 1);
    const int q = it.q0 + rr / a.G;
    rowslot[tid] = a.logical_slot[q];
    const int qb = a.q_branch[q];
    rowtag[tid] = (qb < 0 || !a.cu_branches) ? 0 : qb - a.cu_branches[it.s] + 1;
  }
  __syncthreads();

  float acc[F32_ROWS][QD];
  float m_run[F32_ROWS], l_run[F32_ROWS];
#pragma unroll
  for (int r = 0; r < F32_ROWS; ++r) {
    m_run[r] = -INFINITY;
    l_run[r] = 0.f;
#pragma unroll
    for (int e = 0; e < QD; ++e) acc[r][e] = 0.f;
  }
  // slots past the last row's own slot have never been written and may hold anything: see below
  int last_slot = 0;
#pragma unroll
  for (int r = 0; r < F32_ROWS; ++r) last_slot = max(last_slot, rowslot[r]);
  const long bt_base = (long)it.s * a.kv.max_blocks_per_seq;
  const uint8_t* owner_row = a.slot_owner ? a.slot_owner + (long)it.s * a.owner_stride : nullptr;

  for (int P = page0 + wave; P < page1; P += NW) {
    // The query rows are re-read from LDS for every page: kept in registers across the loop (4 rows x
    // D / 4 values per lane) they would not fit beside the accumulators.
    asm volatile("" ::: "memory");
    int blk = __builtin_amdgcn_readfirstlane(a.kv.block_tables[bt_base + P]);
    blk = min(max(blk, 0), a.kv.num_blocks - 1);
    const long off = (((long)blk * a.kv.num_kv_heads + it.h) * ASPD_BLOCK + k) * D + g * QD;
    float kv_k[QD], kv_v[QD];
#pragma unroll
    for (int e = 0; e < QD; e += 4) {
      const float4 x = *(const float4*)((const float*)a.kv.k + off + e);
      const float4 y = *(const float4*)((const float*)a.kv.v + off + e);
      kv_k[e] = x.x; kv_k[e + 1] = x.y; kv_k[e + 2] = x.z; kv_k[e + 3] = x.w;
      kv_v[e] = y.x; kv_v[e + 1] = y.y; kv_v[e + 2] = y.z; kv_v[e + 3] = y.w;
    }
    const int j = P * ASPD_BLOCK + k;
    if (j > last_slot) {  // zero weight times a NaN would be a NaN
#pragma unroll
      for (int e = 0; e < QD; ++e) kv_v[e] = 0.f;
    }
    const int own = (owner_row && j >= L && j < a.owner_stride) ? owner_row[j] : 0;
#pragma unroll
    for (int r = 0; r < F32_ROWS; ++r) {
      float s = 0.f;
#pragma unroll
      for (int e = 0; e < QD; ++e) s = fmaf(qtile[r * D + g * QD + e], kv_k[e], s);
      s += __shfl_xor(s, 16);
      s += __shfl_xor(s, 32);
      s *= a.scale_log2;
      const bool vis = (j <= rowslot[r]) && (j < L || rowtag[r] == 0 || own == rowtag[r]);
      // No branch on vis (an invisible key enters with weight zero): the lanes of one key agree on vis
      // and on s, so their statistics stay identical, and the whole update runs with all lanes active.
      const float sv = vis ? s : -INFINITY;
      const float m_new = fmaxf(m_run[r], sv);
      const float mref = exp2_safe_ref(m_new);
      const float alpha = exp2f(m_run[r] - mref);
      const float p = exp2f(sv - mref);
      m_run[r] = m_new;
      l_run[r] = l_run[r] * alpha + p;
#pragma unroll
      for (int e = 0; e < QD; ++e) acc[r][e] = fmaf(p, kv_v[e], acc[r][e] * alpha);
    }
  }

  // ---- combine all lanes that hold the same quarter g: 16 key classes x NW waves
  float* mine = red + (long)tid * F32_ROWS * (QD + 2);
#pragma unroll
  for (int r = 0; r < F32_ROWS; ++r) {
#pragma unroll
    for (int e = 0; e < QD; ++e) mine[r * (QD + 2) + e] = acc[r][e];
    mine[r * (QD + 2) + QD] = m_run[r];
    mine[r * (QD + 2) + QD + 1] = l_run[r];
  }
  __syncthreads();
  // one thread per (row, d)
  for (int i = tid; i < F32_ROWS * D; i += THREADS) {
    const int r = i / D, d = i - r * D;
    const int gq = d / QD, e = d - gq * QD;
    float mg = -INFINITY;
    for (int w = 0; w < NW; ++w)
      for (int kk = 0; kk < 16; ++kk)
        mg = fmaxf(mg, red[((long)(w * 64 + gq * 16 + kk) * F32_ROWS + r) * (QD + 2) + QD]);
    const float mref = exp2_safe_ref(mg);
    float lg = 0.f, o = 0.f;
    for (int w = 0; w < NW; ++w)
      for (int kk = 0; kk < 16; ++kk) {
        const float* src = red + ((long)(w * 64 + gq * 16 + kk) * F32_ROWS + r) * (QD + 2);
        const float f = exp2f(src[QD] - mref);
        lg += src[QD + 1] * f;
        o += src[e] * f;
      }
    if (r < R) {
      if (complete) {
        const int q = it.q0 + r / a.G;
        const int head = it.h * a.G + r % a.G;
        ((float*)a.out)[((long)q * a.kv.num_q_heads + head) * D + d] = o / lg;
        if (a.lse && d == 0) a.lse[(long)q * a.kv.num_q_heads + head] = (mg + log2f(lg)) * LN2;
      } else {
        store_device_scope(partial_acc(pslot, r, D) + d, o);
        if (d == 0) {
          float* stat = partial_stat(a, pslot, r, D);
          store_device_scope(stat, mg);
          store_device_scope(stat + 1, lg);
        }
      }
    }
  }
}

template <int D>
size_t f32_smem_bytes() {
  return F32_ROWS * D * 4 + 2 * F32_ROWS * 4 + (size_t)THREADS * F32_ROWS * (D / 4 + 2) * 4;
}

// One workgroup per compute unit (255 vector registers per lane and 138 KB of LDS at head_dim 128), one wave
// per SIMD; the grid is sized for that.
static_assert(F32_ROWS * 128 * 4 + 2 * F32_ROWS * 4 + THREADS * F32_ROWS * (128 / 4 + 2) * 4 <= 160 * 1024 - 256,
              "fp32 kernel: query tile, row descriptors and one reduction slot per thread fit the LDS of a compute unit");
template <int D>
__global__ __launch_bounds__(THREADS) __attribute__((amdgpu_waves_per_eu(1, 1))) void attn_f32_kernel(AttnArgs a) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  __shared__ int merge_flag;
  Seg seg;
  int next;
  const int nseg = plan_begin(a, &seg, &next);
  for (int i = 0; i < nseg; ++i) {
    if (i > 0) {
      seg = plan_segment(a, next + i - 1);
      if (!seg_ok(a, seg)) break;
    }
    const bool complete = seg_complete(seg);
    float* pslot = partial_slot(a, blockIdx.x, seg.page0 == 0 ? 1 : 0, D);
    segment_f32<D>(a, smem, seg, complete, pslot);
    // F32_ROWS rows of D / 4 chunks never exceed the workgroup's threads: one element per thread
    if (!complete) announce_partial<D, false, THREADS, 1>(a, seg, &merge_flag);
  }
}

// ---------------------------------------------------------------------------------------------
// Items split over several workgroups: every workgroup that has written a partial for the item
// announces it on the item's counter (indexed by the workgroup in whose share the item starts);
// the one that arrives last combines all partials and writes the output.  No workgroup waits for
// another.  The partials are the "starts item" slot of the first workgroup and the "continues
// item" slots of the following ones.
// ---------------------------------------------------------------------------------------------
template <int D, bool BF16, int THREADS, int ELEMS, int BATCH>
__device__ void merge_parts(const AttnArgs& a, const Seg& it, int owner, int w_last) {
  constexpr int CPR = D / 4;  // float4 chunks per row
  // ELEMS: (row, chunk) elements a thread combines concurrently; BATCH: partials fetched at once, per
  // element.
  const int R = it.nq * a.G;
  const long stride = (long)a.rows_cap * (D + 4);
  const int nparts = w_last - owner + 1;
  const int total = R * CPR;
  // The loads miss the caches and are latency-bound: a thread keeps the loads of up to ELEMS
  // elements x BATCH partials in flight at once.
  for (int i0 = threadIdx.x; i0 < total; i0 += ELEMS * THREADS) {
    int r[ELEMS], cc[ELEMS];
    float m[ELEMS], l[ELEMS];
    f32x4 o[ELEMS];
#pragma unroll
    for (int x = 0; x < ELEMS; ++x) {
      const int i = min(i0 + x * THREADS, total - 1);  // a clamped duplicate is computed and not stored
      r[x] = i / CPR;
      cc[x] = i - r[x] * CPR;
      m[x] = -INFINITY;
      l[x] = 0.f;
      o[x] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    for (int p0 = 0; p0 < nparts; p0 += BATCH) {
      float pm[ELEMS][BATCH], pl[ELEMS][BATCH];
      f32x4 po[ELEMS][BATCH];
#pragma unroll
      for (int x = 0; x < ELEMS; ++x) {
#pragma unroll
        for (int k = 0; k < BATCH; ++k) {
          const int ww = owner + min(p0 + k, nparts - 1);
          const float* slot = a.partial + (long)(2 * ww + (ww == owner ? 1 : 0)) * stride;
          const f32x4 ml = *(const f32x4*)(slot + (long)a.rows_cap * D + 4 * r[x]);  // reference, sum, padding
          pm[x][k] = ml[0];
          pl[x][k] = ml[1];
          po[x][k] = *(const f32x4*)(slot + (long)r[x] * D + 4 * cc[x]);
        }
      }
#pragma unroll
      for (int x = 0; x < ELEMS; ++x) {
        float mb = m[x];
#pragma unroll
        for (int k = 0; k < BATCH; ++k)
          if (p0 + k < nparts) mb = fmaxf(mb, pm[x][k]);
        const float mref = exp2_safe_ref(mb);
        const float f0 = __builtin_amdgcn_exp2f(m[x] - mref);
        l[x] *= f0;
        o[x] *= f0;
#pragma unroll
        for (int k = 0; k < BATCH; ++k) {
          if (p0 + k < nparts) {
            const float f = __builtin_amdgcn_exp2f(pm[x][k] - mref);
            l[x] += pl[x][k] * f;
            o[x] += po[x][k] * f;
          }
        }
        m[x] = mb;
      }
    }
#pragma unroll
    for (int x = 0; x < ELEMS; ++x) {
      if (i0 + x * THREADS >= total) continue;
      const int q = it.q0 + r[x] / a.G;
      const int head = it.h * a.G + r[x] % a.G;
      const long oi = ((long)q * a.kv.num_q_heads + head) * D + 4 * cc[x];
      const float inv = 1.f / l[x];
      if (BF16) {
        typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
        bf16x4 ov;
#pragma unroll
        for (int e = 0; e < 4; ++e) ov[e] = (__bf16)(o[x][e] * inv);
        *(bf16x4*)((__bf16*)a.out + oi) = ov;
      } else {
        *(f32x4*)((float*)a.out + oi) = o[x] * inv;
      }
      if (a.lse && cc[x] == 0) a.lse[(long)q * a.kv.num_q_heads + head] = (m[x] + log2f(l[x])) * LN2;
    }
  }
}

// A second batch costs a second round trip to memory, so the batch is as large as the registers allow
// (sixteen in the one-tile streaming kernel, one wave per SIMD) - but no larger than the parts there are:
// with one wave per SIMD the merge is bound by the instructions it issues, and every slot of a batch costs
// its loads and its arithmetic whether a part stands behind it or not.
template <int D, bool BF16, int THREADS, int ELEMS>
__device__ void merge_item(const AttnArgs& a, const Seg& it, int owner, int w_last) {
  constexpr bool WIDE = BF16 && ELEMS == 2 && THREADS == 256;
  const int nparts = w_last - owner + 1;
  if (nparts <= 4) merge_parts<D, BF16, THREADS, ELEMS, 4>(a, it, owner, w_last);
  else if (!WIDE || nparts <= 8) merge_parts<D, BF16, THREADS, ELEMS, 8>(a, it, owner, w_last);
  else merge_parts<D, BF16, THREADS, ELEMS, WIDE ? 16 : 8>(a, it, owner, w_last);
}

// Called by every thread of the workgroup after it has written a partial of the item of `it`.
template <int D, bool BF16, int THREADS, int ELEMS>
__device__ void announce_partial(const AttnArgs& a, const Seg& it, int* flag /* LDS */) {
  const int owner = it.owner, w_last = it.w_last;
  // the write-through stores of the partial have completed before the arrival is counted
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  if (threadIdx.x == 0) {
    const int old = atomicAdd(a.counters + owner, 1);
    const int last = (old == w_last - owner) ? 1 : 0;
    if (last) atomicExch(a.counters + owner, 0);  // every part has arrived: leave it clean for the next call
    *flag = last;
  }
  __syncthreads();
  if (*flag == 0) return;
  // Only the merging workgroup pays for an acquire at device scope (it drops whatever stale copies of
  // the partial slots its caches may hold from earlier launches); the partials themselves were
  // written through by their producers, so ordinary wide loads now fetch them.
  // One wave issues it for the workgroup: the invalidate acts on the compute unit's L1 and the XCD's L2,
  // which all waves of the workgroup share.
  if (threadIdx.x < 64) __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
  __syncthreads();
  merge_item<D, BF16, THREADS, ELEMS>(a, it, owner, w_last);
}

// ---------------------------------------------------------------------------------------------
// Host side
// ---------------------------------------------------------------------------------------------
constexpr int LDS_BYTES = 160 * 1024;  // per compute unit on gfx950
constexpr int STATIC_LDS_RESERVE = 256;  // room for the kernels' few static LDS variables

// Dynamic LDS above 64 KB has to be allowed once per kernel and device.
int allow_big_lds(const void* kernel) {
  static std::mutex mu;
  static std::set<std::pair<int, const void*>> done;
  int dev = 0;
  ASPD_HIP_CHECK(hipGetDevice(&dev));
  std::lock_guard<std::mutex> lock(mu);
  if (done.count({dev, kernel})) return ASPD_OK;
  ASPD_HIP_CHECK(hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES - STATIC_LDS_RESERVE));
  done.insert({dev, kernel});
  return ASPD_OK;
}

// Workspace: arrival counters, room for a plan (used when the step brings none that fits the launch),
// two partial slots per workgroup.
size_t plan_area_bytes(size_t plan_words) { return (plan_words * sizeof(int32_t) + 255) & ~(size_t)255; }
size_t scratch_need(int head_dim, size_t plan_words, long nwg, int rows_cap) {
  return COUNTER_BYTES + plan_area_bytes(plan_words) + (size_t)2 * nwg * rows_cap * (head_dim + 4) * sizeof(float);
}

enum Mode { MODE_PARALLEL, MODE_CHUNK, MODE_SERIAL };

int attn_launch(Mode mode, const aspd_kv* kv, const aspd_state* state, const aspd_step* step, const void* q_d,
                void* out_d, float* lse_d, float sm_scale, void* workspace_d, size_t workspace_bytes,
                void* stream) {
  int rc = aspd_check_kv(kv);
  if (rc != ASPD_OK) return rc;
  if (!state || !step || state->B <= 0 || !state->stage_base_d || !state->seq_len_d) return ASPD_ERR_INVALID_ARG;
  if (state->B > ASPD_MAX_BATCH) return ASPD_ERR_UNSUPPORTED;
  if (step->NQ < 0 || step->max_new_per_seq < 0 || step->max_workgroups < 0 || !step->cu_seq_new_d)
    return ASPD_ERR_INVALID_ARG;
  if (step->NQ == 0) return ASPD_OK;
  if (!step->q_branch_d || !step->logical_slot_d || !q_d || !out_d) return ASPD_ERR_INVALID_ARG;
  if (((uintptr_t)q_d & 15) || ((uintptr_t)out_d & 15)) return ASPD_ERR_INVALID_ARG;
  if (!(sm_scale >= 0.f)) return ASPD_ERR_INVALID_ARG;
  const bool branches = (mode != MODE_SERIAL) && step->shared_mask == 0;  // rows that may carry branch tags
  if (branches) {
    if (!state->cu_branches_d || !state->slot_owner_d) return ASPD_ERR_INVALID_ARG;
    if (state->owner_stride < kv->max_blocks_per_seq * ASPD_BLOCK || (state->owner_stride & 3) ||
        ((uintptr_t)state->slot_owner_d & 3))
      return ASPD_ERR_INVALID_ARG;
  }
  AttnVariant v;
  if (!aspd_choose_variant(kv, state->B, step->NQ, step->max_new_per_seq, step->max_workgroups, mode == MODE_CHUNK,
                           branches, &v))
    return ASPD_ERR_UNSUPPORTED;
  if (!workspace_d || ((uintptr_t)workspace_d & 255)) return ASPD_ERR_INVALID_ARG;
  const size_t plan_words = aspd_plan_words(kv, v, state->B, step->NQ);
  if (workspace_bytes < scratch_need(kv->head_dim, plan_words, v.nwg, v.rows_cap)) return ASPD_ERR_WORKSPACE;
  hipStream_t hs = (hipStream_t)stream;

  // The step's own plan when it was built for this launch shape; otherwise (no plan buffer, a hint that
  // changed since, the other entry point) one is built now, into the workspace, by the same kernel.
  const int32_t* plan = step->plan_d;
  if (!plan || step->plan_key != aspd_plan_key(v, state->B) || step->plan_bytes < plan_words * sizeof(int32_t)) {
    int32_t* own = (int32_t*)((char*)workspace_d + COUNTER_BYTES);
    rc = aspd_plan_launch(kv, v, state->B, state->stage_base_d, state->seq_len_d, step->cu_seq_new_d, own, hs);
    if (rc != ASPD_OK) return rc;
    plan = own;
  }

  AttnArgs a;
  a.kv = make_view(kv);
  a.cu_branches = branches ? state->cu_branches_d : nullptr;
  a.slot_owner = branches ? state->slot_owner_d : nullptr;
  a.owner_stride = branches ? state->owner_stride : 0;
  a.q_branch = step->q_branch_d;
  a.logical_slot = step->logical_slot_d;
  a.q = q_d;
  a.out = out_d;
  a.lse = lse_d;
  a.counters = (int*)workspace_d;
  a.partial = (float*)((char*)workspace_d + COUNTER_BYTES + plan_area_bytes(plan_words));
  a.plan = plan;
  a.row_base = nullptr;
  a.NQ = step->NQ;
  a.scale_log2 = (sm_scale == 0.f ? 1.0f / sqrtf((float)kv->head_dim) : sm_scale) * LOG2E;
  a.B = state->B;
  a.nwg = v.nwg;
  a.G = kv->num_q_heads / kv->num_kv_heads;
  a.qpg = v.qpg;
  a.rows_cap = v.rows_cap;

  const int D = kv->head_dim;
#define ASPD_LAUNCH(KERNEL, NTHREADS, SMEM)                                          \
  do {                                                                               \
    rc = allow_big_lds((const void*)KERNEL);                                         \
    if (rc != ASPD_OK) return rc;                                                    \
    if ((SMEM) > (size_t)(LDS_BYTES - STATIC_LDS_RESERVE)) return ASPD_ERR_UNSUPPORTED;                     \
    hipLaunchKernelGGL(KERNEL, dim3(a.nwg), dim3(NTHREADS), SMEM, hs, a);            \
    ASPD_HIP_CHECK(hipGetLastError());                                               \
  } while (0)
  if (v.kernel == KERNEL_BF16_ROWS) {
    if (D == 128)
      ASPD_LAUNCH((attn_bf16_rows_kernel<128, ROWS_NT, ROWS_NW>), ROWS_NW * 64,
                  (rows_smem_bytes<128, ROWS_NT, ROWS_NW>()));
    else
      ASPD_LAUNCH((attn_bf16_rows_kernel<64, ROWS_NT, ROWS_NW>), ROWS_NW * 64,
                  (rows_smem_bytes<64, ROWS_NT, ROWS_NW>()));
  } else if (v.kernel == KERNEL_BF16_STREAM) {
    // pages that no second row group reads are fetched with non-temporal loads
#define ASPD_BF16_CASE(DD, NN)                                                                            \
  do {                                                                                                    \
    if (v.stream_once)                                                                                    \
      ASPD_LAUNCH((attn_bf16_kernel<DD, NN, STREAM_NW, STREAM_PF, true>), STREAM_NW * 64,                 \
                  (bf16_smem_bytes<DD, NN, STREAM_NW>()));                                                \
    else                                                                                                  \
      ASPD_LAUNCH((attn_bf16_kernel<DD, NN, STREAM_NW, STREAM_PF, false>), STREAM_NW * 64,                \
                  (bf16_smem_bytes<DD, NN, STREAM_NW>()));                                                \
  } while (0)
    if (D == 128) {
      if (v.nt == 1) ASPD_BF16_CASE(128, 1);
      else if (v.nt == 2) ASPD_BF16_CASE(128, 2);
      else ASPD_BF16_CASE(128, 3);
    } else {
      if (v.nt == 1) ASPD_BF16_CASE(64, 1);
      else if (v.nt == 2) ASPD_BF16_CASE(64, 2);
      else ASPD_BF16_CASE(64, 3);
    }
#undef ASPD_BF16_CASE
  } else {
    if (D == 128) ASPD_LAUNCH(attn_f32_kernel<128>, THREADS, f32_smem_bytes<128>());
    else ASPD_LAUNCH(attn_f32_kernel<64>, THREADS, f32_smem_bytes<64>());
  }
#undef ASPD_LAUNCH
  return ASPD_OK;
}

}  // namespace

extern "C" size_t aspd_workspace_bytes(const aspd_kv* kv, int32_t B, int32_t NQ) {
  if (!kv || B <= 0 || NQ < 0 || kv->num_kv_heads <= 0 || kv->num_q_heads <= 0) return 0;
  if (kv->head_dim != 64 && kv->head_dim != 128) return 0;
  if (kv->dtype != ASPD_F32 && kv->dtype != ASPD_BF16) return 0;
  if (kv->num_q_heads % kv->num_kv_heads != 0 || kv->max_blocks_per_seq <= 0) return 0;
  // the largest need over the launch shapes the NQ rows may take (hints 0 .. 3 tiles' worth, either call)
  const int G = kv->num_q_heads / kv->num_kv_heads;
  size_t need = 0;
  for (int tiles = 0; tiles <= NT_MAX + 1; ++tiles) {
    for (int chunk = 0; chunk < 2; ++chunk) {
      AttnVariant v;
      const int hint = tiles == 0 ? 0 : std::max(1, 16 * tiles / G);
      if (!aspd_choose_variant(kv, B, NQ, hint, 0, chunk != 0, true, &v)) continue;
      need = std::max(need, scratch_need(kv->head_dim, aspd_plan_words(kv, v, B, NQ), v.nwg, v.rows_cap));
    }
  }
  return need;
}

extern "C" size_t aspd_plan_bytes(const aspd_kv* kv, int32_t B, int32_t NQ) {
  if (!kv || B <= 0 || NQ < 0 || kv->num_kv_heads <= 0 || kv->num_q_heads <= 0) return 0;
  if (kv->num_q_heads % kv->num_kv_heads != 0) return 0;
  // a row group holds at least one query; a grid at most MAX_WG workgroups
  const size_t items = ((size_t)B + (size_t)NQ) * kv->num_kv_heads;
  return ((size_t)PLAN_HDR * MAX_WG + (size_t)PLAN_SEG * (items + MAX_WG)) * sizeof(int32_t);
}

namespace {
__global__ void zero_counters_kernel(int* head) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < COUNTER_BYTES / 4) head[i] = 0;
}
}  // namespace

namespace {
// Plain streaming read (non-temporal loads, the fastest plain read on this device): every lane loads 16 bytes per step, consecutive lanes consecutive addresses,
// each workgroup a contiguous share.  The XOR of everything read goes to one word per workgroup so
// that the loads cannot be dropped.
__global__ __launch_bounds__(256) void probe_read_kernel(const u32x4* __restrict__ src, size_t n16,
                                                         unsigned* __restrict__ sink) {
  const size_t per = (n16 + gridDim.x - 1) / gridDim.x;
  const size_t lo = per * blockIdx.x;
  const size_t hi = lo + per < n16 ? lo + per : n16;
  u32x4 acc = {0u, 0u, 0u, 0u};
  size_t i = lo + threadIdx.x;
  for (; i + 3 * 256 < hi; i += 4 * 256) {
    const u32x4 a0 = __builtin_nontemporal_load(src + i), a1 = __builtin_nontemporal_load(src + i + 256),
                a2 = __builtin_nontemporal_load(src + i + 512), a3 = __builtin_nontemporal_load(src + i + 768);
    acc ^= a0 ^ a1 ^ a2 ^ a3;
  }
  for (; i < hi; i += 256) acc ^= src[i];
  unsigned x = acc[0] ^ acc[1] ^ acc[2] ^ acc[3];
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) x ^= __shfl_xor(x, off);
  __shared__ unsigned part[4];
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = x;
  __syncthreads();
  if (threadIdx.x == 0) sink[blockIdx.x] = part[0] ^ part[1] ^ part[2] ^ part[3];
}
}  // namespace

extern "C" int aspd_probe_read_bandwidth(const void* src_d, size_t bytes, void* sink_d, void* stream) {
  if (!src_d || !sink_d || ((uintptr_t)src_d & 15) || bytes < 16) return ASPD_ERR_INVALID_ARG;
  const int grid = 8 * aspd_device_cu_count();
  hipLaunchKernelGGL(probe_read_kernel, dim3(grid), dim3(256), 0, (hipStream_t)stream, (const u32x4*)src_d,
                     bytes / 16, (unsigned*)sink_d);
  ASPD_HIP_CHECK(hipGetLastError());
  return ASPD_OK;
}

extern "C" int aspd_workspace_init(void* workspace_d, size_t workspace_bytes, void* stream) {
  if (!workspace_d || ((uintptr_t)workspace_d & 255)) return ASPD_ERR_INVALID_ARG;
  if (workspace_bytes < (size_t)COUNTER_BYTES) return ASPD_ERR_WORKSPACE;
  hipLaunchKernelGGL(zero_counters_kernel, dim3(COUNTER_BYTES / 4 / 256), dim3(256), 0, (hipStream_t)stream,
                     (int*)workspace_d);
  ASPD_HIP_CHECK(hipGetLastError());
  return ASPD_OK;
}

extern "C" int aspd_attn_parallel_decode(const aspd_kv* kv, const aspd_state* state, const aspd_step* step,
                                         const void* q_d, void* out_d, float* lse_d, float sm_scale,
                                         void* workspace_d, size_t workspace_bytes, void* stream) {
  return attn_launch(MODE_PARALLEL, kv, state, step, q_d, out_d, lse_d, sm_scale, workspace_d, workspace_bytes,
                     stream);
}

extern "C" int aspd_attn_branch_chunk(const aspd_kv* kv, const aspd_state* state, const aspd_step* step,
                                      const void* q_d, void* out_d, float* lse_d, float sm_scale,
                                      void* workspace_d, size_t workspace_bytes, void* stream) {
  return attn_launch(MODE_CHUNK, kv, state, step, q_d, out_d, lse_d, sm_scale, workspace_d, workspace_bytes,
                     stream);
}

extern "C" int aspd_attn_serial_decode(const aspd_kv* kv, const aspd_state* state, const aspd_step* step,
                                       const void* q_d, void* out_d, float* lse_d, float sm_scale,
                                       void* workspace_d, size_t workspace_bytes, void* stream) {
  return attn_launch(MODE_SERIAL, kv, state, step, q_d, out_d, lse_d, sm_scale, workspace_d, workspace_bytes,
                     stream);
}

extern "C" int aspd_attn_full_sequence(const aspd_kv* kv, const aspd_state* state, const aspd_step* step,
                                       const void* q_d, void* out_d, float* lse_d, float sm_scale,
                                       void* workspace_d, size_t workspace_bytes, void* stream) {
  int rc = aspd_check_kv(kv);
  if (rc != ASPD_OK) return rc;
  if (!state || !step || state->B <= 0) return ASPD_ERR_INVALID_ARG;
  if (state->B > ASPD_MAX_BATCH) return ASPD_ERR_UNSUPPORTED;
  const int G = kv->num_q_heads / kv->num_kv_heads;
  const int qpg = aspd_sequence_qpg(G);
  if (kv->dtype != ASPD_BF16 || qpg < 1) return ASPD_ERR_UNSUPPORTED;
  if (step->NQ < 0) return ASPD_ERR_INVALID_ARG;
  if (step->NQ == 0) return ASPD_OK;
  if (!step->plan_d || step->plan_key != aspd_sequence_plan_key(qpg, state->B) ||
      step->plan_bytes < aspd_sequence_plan_words(kv, state->B, step->NQ) * sizeof(int32_t))
    return ASPD_ERR_INVALID_ARG;  // not a step of aspd_build_sequence_meta
  if (!step->q_branch_d || !step->logical_slot_d || !q_d || !out_d) return ASPD_ERR_INVALID_ARG;
  if (((uintptr_t)q_d & 15) || ((uintptr_t)out_d & 15)) return ASPD_ERR_INVALID_ARG;
  if (!(sm_scale >= 0.f)) return ASPD_ERR_INVALID_ARG;
  const bool branches = step->shared_mask == 0;
  if (branches && (!state->slot_owner_d || state->owner_stride < kv->max_blocks_per_seq * ASPD_BLOCK ||
                   (state->owner_stride & 3) || ((uintptr_t)state->slot_owner_d & 3)))
    return ASPD_ERR_INVALID_ARG;
  if (!workspace_d || ((uintptr_t)workspace_d & 255)) return ASPD_ERR_INVALID_ARG;
  if (workspace_bytes < (size_t)COUNTER_BYTES) return ASPD_ERR_WORKSPACE;
  if (step->max_workgroups < 0) return ASPD_ERR_INVALID_ARG;

  AttnArgs a;
  a.kv = make_view(kv);
  a.cu_branches = nullptr;
  a.slot_owner = branches ? state->slot_owner_d : nullptr;
  a.owner_stride = branches ? state->owner_stride : 0;
  a.q_branch = step->q_branch_d;
  a.logical_slot = step->logical_slot_d;
  a.q = q_d;
  a.out = out_d;
  a.lse = lse_d;
  a.counters = (int*)workspace_d;
  a.partial = nullptr;
  a.plan = step->plan_d;
  a.row_base = step->plan_d + SEQ_PLAN_HDR;
  a.NQ = step->NQ;
  a.scale_log2 = (sm_scale == 0.f ? 1.0f / sqrtf((float)kv->head_dim) : sm_scale) * LOG2E;
  a.B = state->B;
  a.G = G;
  a.qpg = qpg;
  a.rows_cap = ROWS_NW * 16 * ROWS_NT;
  // one workgroup per compute unit, never more than there are row groups to take
  long nwg = aspd_device_cu_count();
  nwg = std::min(nwg, ((long)state->B + step->NQ / qpg) * kv->num_kv_heads);
  if (step->max_workgroups > 0) nwg = std::min(nwg, (long)step->max_workgroups);
  a.nwg = (int)std::max(1L, nwg);
  hipStream_t hs = (hipStream_t)stream;
  if (kv->head_dim == 128) {
    rc = allow_big_lds((const void*)attn_bf16_seq_kernel<128, ROWS_NT, ROWS_NW>);
    if (rc != ASPD_OK) return rc;
    hipLaunchKernelGGL((attn_bf16_seq_kernel<128, ROWS_NT, ROWS_NW>), dim3(a.nwg), dim3(ROWS_NW * 64),
                       (rows_smem_bytes<128, ROWS_NT, ROWS_NW>()), hs, a);
  } else {
    rc = allow_big_lds((const void*)attn_bf16_seq_kernel<64, ROWS_NT, ROWS_NW>);
    if (rc != ASPD_OK) return rc;
    hipLaunchKernelGGL((attn_bf16_seq_kernel<64, ROWS_NT, ROWS_NW>), dim3(a.nwg), dim3(ROWS_NW * 64),
                       (rows_smem_bytes<64, ROWS_NT, ROWS_NW>()), hs, a);
  }
  ASPD_HIP_CHECK(hipGetLastError());
  return ASPD_OK;
}

// ---------------------------------------------------------------------------------------------
// Parallel decode for callers that cannot allocate: the scratch is an array of the code object itself,
// one copy per device, alive until the process ends.  It starts zeroed (which is what a prepared
// workspace looks like) and every attention launch leaves its counters at zero again.
// ---------------------------------------------------------------------------------------------
static __device__ __align__(256) unsigned char scratch[ASPD_STATIC_SCRATCH_BYTES];

namespace {
// Device address of `scratch` on the current device (the array's name is only a host-side handle).
int static_scratch(void** out) {
  static std::mutex mu;
  constexpr int MAX_DEVICES = 64;
  static void* ptrs[MAX_DEVICES];
  int dev = 0;
  ASPD_HIP_CHECK(hipGetDevice(&dev));
  if (dev < 0 || dev >= MAX_DEVICES) return ASPD_ERR_UNSUPPORTED;
  std::lock_guard<std::mutex> lock(mu);
  if (!ptrs[dev]) {
    void* p = nullptr;
    ASPD_HIP_CHECK(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p || ((uintptr_t)p & 255)) return ASPD_ERR_HIP;
    ptrs[dev] = p;
  }
  *out = ptrs[dev];
  return ASPD_OK;
}
}  // namespace

extern "C" int aspd_attn_parallel_decode_static(const aspd_kv* kv, const aspd_state* state, const aspd_step* step,
                                                const void* q_d, void* out_d, float* lse_d, float sm_scale,
                                                void* stream) {
  void* ws = nullptr;
  int rc = static_scratch(&ws);
  if (rc != ASPD_OK) return rc;
  rc = attn_launch(MODE_PARALLEL, kv, state, step, q_d, out_d, lse_d, sm_scale, ws, ASPD_STATIC_SCRATCH_BYTES, stream);
  return rc == ASPD_ERR_WORKSPACE ? ASPD_ERR_SCRATCH_LIMIT : rc;
}
