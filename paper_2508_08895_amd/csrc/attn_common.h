// Shared by the attention kernels (internal to libaspd): launch arguments, the plan as the kernels read it,
// partial-result slots and the device-scope stores they are written with.
#pragma once

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
// the wait states the compiler would have inserted for a store of its own.  The data are usually MFMA
// results, which a memory instruction must not read too soon after the MFMA was issued either (no hardware
// interlock, and again the compiler's padding does not cover assembly): hence the wait states in front.
__device__ __forceinline__ void store_device_scope_x4(float* p, f32x4 v) {
  asm volatile("s_nop 15\n\tglobal_store_dwordx4 %0, %1, off sc0 sc1\n\ts_nop 1" ::"v"(p), "v"(v) : "memory");
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

}  // namespace
