// The row-splitting bf16 kernels (internal to libaspd): many rows per KV head (branch chunks, whole sequences).
#pragma once

#include "attn_bf16_math.h"

namespace {

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
// tokens of other branches).  The groups of a window that lie wholly below everything a wave's rows must
// mask (the prefix, earlier stages) are taken first, in a loop of their own without tags, masks or
// per-pair tests: the kernel's time follows the number of instructions a wave issues per pair.
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

  u32x4 nxt[LPT];  // this thread's slice of the group on its way
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
    // the page (of the window) this thread loads for group gi; past the end of the window the last pages
    // again, which the caches hold
    auto page_of = [&](int gi) -> int {
      const int p = min(gi * PPS + (lpage >> 2), npairs - 1);
      return min(2 * p + (lpage & 1), wpages - 1);
    };
    auto issue = [&](int gi) {
      const int pg = page_of(gi);
      const int b = blk_lds[pg];
      const u32x4* src = (const u32x4*)(l_is_k ? a.kv.k : a.kv.v) + ((long)b * a.kv.num_kv_heads + it.h) * C::PAGE_U4;
#pragma unroll
      for (int k = 0; k < LPT; ++k) nxt[k] = src[lt + k * PER_PAGE];
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
    issue(0);

    // ---- the leading groups of the window that every row of this wave sees in full (whole pairs below
    // mask_from): nothing to mask, no tags, nothing to clear (they end below the last row's slot).  The
    // count differs between the waves of a workgroup; every group costs one barrier in either loop, and
    // what a wave stages for a group does not depend on the loop it is in.
    const int g_open = max(0, min(ngroups, (min(wend, mask_from / ASPD_BLOCK) - wbase) / (2 * PPS)));
    for (int gi = 0; gi < g_open; ++gi) {
      u32x4* stage = stage0 + (gi & 1) * (PPS * C::STAGE_BYTES / 16);
#pragma unroll
      for (int k = 0; k < LPT; ++k) stage[lpage * C::LPAGE_U4 + lpos[k]] = nxt[k];
      issue(gi + 1);
      __syncthreads();  // the group is staged; everyone is done with the other buffer's previous group
      if (wave_active) group_compute_open<D, NT, PPS>(stage, ts, kr_even, kr_odd, vu, a.scale_log2, qr);
    }

    // ---- the rest of the window: pairs that may need the mask, the tags, the tail
    u32x4 tn[PPS][2];
#pragma unroll
    for (int h = 0; h < PPS; ++h) tn[h][0] = tn[h][1] = u32x4{0, 0, 0, 0};
    if (g_open < ngroups) tags_of(g_open, tn);
    for (int gi = g_open; gi < ngroups; ++gi) {
      u32x4* stage = stage0 + (gi & 1) * (PPS * C::STAGE_BYTES / 16);
      const int key0 = (wbase + page_of(gi)) * ASPD_BLOCK;  // first slot of the page this thread staged
      if (!l_is_k && key0 + ASPD_BLOCK > last_slot + 1) {
#pragma unroll
        for (int k = 0; k < LPT; ++k)
          if (key0 + (lt + k * PER_PAGE) / C::CH > last_slot) nxt[k] = u32x4{0u, 0u, 0u, 0u};
      }
#pragma unroll
      for (int k = 0; k < LPT; ++k) stage[lpage * C::LPAGE_U4 + lpos[k]] = nxt[k];
      u32x4 tc[PPS][2];
#pragma unroll
      for (int h = 0; h < PPS; ++h) {
        tc[h][0] = tn[h][0];
        tc[h][1] = tn[h][1];
      }
      issue(gi + 1);
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

}  // namespace
