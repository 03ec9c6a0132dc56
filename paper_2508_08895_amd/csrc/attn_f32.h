// The fp32 kernel (internal to libaspd).
#pragma once

#include "attn_common.h"

namespace {

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

}  // namespace
