// The streaming bf16 kernel (internal to libaspd): few rows per KV head, the waves of a workgroup split the keys
// (parallel decode, serial decode, narrow chunks).
#pragma once

#include "attn_bf16_math.h"

namespace {

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

}  // namespace
