// Combining the partial results of an item that several workgroups share (internal to libaspd).
#pragma once

#include "attn_common.h"

namespace {

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

}  // namespace
