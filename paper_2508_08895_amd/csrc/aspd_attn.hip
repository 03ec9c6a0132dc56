// Branch-isolated attention over a paged KV cache for gfx950 (ASPD Sec. 3.2 Eq. 1-3, Sec. 3.3).
//
// One streaming kernel serves the three attention entry points.  A query row q of sequence s sees
// key slot j iff
//     j <= slot(q)  and  ( j < stage_base[s]  or  tag(q) == 0  or  slot_owner[s][j] == tag(q) )
// with tag(q) = 0 for a main-branch token and the 1-based branch number otherwise.  This is Eq. 2-3
// in cache terms: slots below stage_base belong to earlier stages (visible to all), slots above it to
// the running parallel stage (visible to their own branch), and a token's own slot bounds what has
// been decoded before it.  Parallel decode, branch chunk and serial decode differ only in which rows
// they bring.
//
// Work decomposition: the (sequence, row group, KV head, page) space is flattened; every workgroup
// takes an equal contiguous share of pages and walks the segments in it.  All rows of a row group
// (the active branches of the sequence times the query heads of the KV-head's group) are processed
// against a KV page while it is in the workgroup's LDS, so the shared prefix is fetched once for all
// branches.  A segment that covers its item completely writes the output; otherwise it writes an
// unnormalised partial (running max, sum, accumulator) and a second kernel combines the partials.
#include <algorithm>
#include <cmath>
#include <mutex>
#include <set>
#include <utility>

#include "aspd_common.h"

namespace {

constexpr int NW = 4;                 // waves per workgroup
constexpr int THREADS = NW * 64;
constexpr int NT_MAX = 3;             // 16-row MFMA tiles per row group (bf16 path)
constexpr int BF16_ROWS = 16 * NT_MAX;
constexpr int F32_ROWS = 4;           // rows per row group (fp32 vector path)
constexpr int MIN_PAGES_PER_WG = 16;  // do not split finer than this
constexpr int MAX_WG = 1024;          // upper bound of the grid (workspace is sized for it)
constexpr float LOG2E = 1.4426950408889634f;
constexpr float LN2 = 0.6931471805599453f;

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;

struct AttnArgs {
  KvView         kv;
  const int32_t* stage_base;
  const int32_t* seq_len;
  const int32_t* cu_branches;   // null when no row carries a branch tag
  const uint8_t* slot_owner;
  int            owner_stride;
  const int32_t* cu_seq_new;
  const int32_t* q_branch;
  const int32_t* logical_slot;
  const void*    q;
  void*          out;
  float*         lse;
  float*         partial;       // [2 * nwg][rows_per_group][D + 2]
  float          scale_log2;    // sm_scale * log2(e)
  int            B;
  int            nwg;
  int            G;             // query heads per KV head
  int            qpg;           // queries per row group
  int            rows_cap;      // rows per row group the partial slots are sized for
};

// ---------------------------------------------------------------------------------------------
// Scheduling: identical in the attention kernels and in the merge kernel.
// ---------------------------------------------------------------------------------------------
struct Item {
  int s, rg, h;     // sequence, row group, KV head
  int np;           // pages of the item
  int q0, nq;       // first packed query row and number of queries of the row group
  int first_unit;   // flattened index of the item's page 0
};

__device__ __forceinline__ int pages_of(const AttnArgs& a, int s) {
  int np = (a.seq_len[s] + ASPD_BLOCK - 1) / ASPD_BLOCK;
  return min(np, a.kv.max_blocks_per_seq);
}
__device__ __forceinline__ int groups_of(const AttnArgs& a, int s) {
  int nq = a.cu_seq_new[s + 1] - a.cu_seq_new[s];
  return (nq + a.qpg - 1) / a.qpg;
}

// cu_units[0..B] = exclusive scan of pages * KV heads * row groups per sequence.  Returns the total.
__device__ int build_units(const AttnArgs& a, int* cu_units, int* scratch /*THREADS ints*/) {
  constexpr int PER = ASPD_MAX_BATCH / THREADS;  // sequences per thread
  const int tid = threadIdx.x;
  int mine[PER];
  int sum = 0;
#pragma unroll
  for (int j = 0; j < PER; ++j) {
    int s = tid * PER + j;
    mine[j] = (s < a.B) ? pages_of(a, s) * groups_of(a, s) * a.kv.num_kv_heads : 0;
    sum += mine[j];
  }
  scratch[tid] = sum;
  __syncthreads();
  for (int d = 1; d < THREADS; d <<= 1) {
    int v = (tid >= d) ? scratch[tid - d] : 0;
    __syncthreads();
    scratch[tid] += v;
    __syncthreads();
  }
  int run = scratch[tid] - sum;  // exclusive
#pragma unroll
  for (int j = 0; j < PER; ++j) {
    int s = tid * PER + j;
    if (s < a.B) cu_units[s] = run;
    run += mine[j];
  }
  const int total = scratch[THREADS - 1];
  if (tid == 0) cu_units[a.B] = total;
  __syncthreads();
  return total;
}

__device__ __forceinline__ int chunk_of(int total, int nwg) {
  int c = (total + nwg - 1) / nwg;
  return max(c, MIN_PAGES_PER_WG);
}

// The item that holds flattened page `u`, and the page's index within it.
__device__ Item locate(const AttnArgs& a, const int* cu_units, int u, int* page) {
  int lo = 0, hi = a.B - 1;
  while (lo < hi) {
    int mid = (lo + hi + 1) >> 1;
    if (cu_units[mid] <= u) lo = mid; else hi = mid - 1;
  }
  Item it;
  it.s = lo;
  it.np = pages_of(a, lo);
  const int rel = u - cu_units[lo];
  const int idx = rel / it.np;
  *page = rel - idx * it.np;
  const int ngroups = groups_of(a, lo);
  it.h = idx / ngroups;       // row groups of one KV head are neighbours: they read the same pages
  it.rg = idx - it.h * ngroups;
  it.first_unit = cu_units[lo] + idx * it.np;
  const int qs = a.cu_seq_new[lo];
  const int nq = a.cu_seq_new[lo + 1] - qs;
  it.q0 = qs + it.rg * a.qpg;
  it.nq = min(a.qpg, nq - it.rg * a.qpg);
  return it;
}

__device__ __forceinline__ float* partial_slot(const AttnArgs& a, int wg, int starts_item, int D) {
  return a.partial + ((long)(2 * wg + starts_item)) * a.rows_cap * (D + 2);
}

__device__ __forceinline__ float exp2_safe_ref(float m) { return (m == -INFINITY) ? 0.f : m; }

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
  static constexpr int KSTEPS = D / 32;
  static constexpr int MT = D / 16;
  static constexpr int STAGE_BYTES = 4 * PAGE_U4 * 16;  // K0 K1 V0 V1
};

template <int D>
__device__ __forceinline__ int k_swz(int row, int chunk) { return row * Bf16Cfg<D>::CH + (chunk ^ (row & 7)); }
template <int D>
__device__ __forceinline__ int v_swz(int row, int chunk) {
  return row * Bf16Cfg<D>::CH + ((((chunk >> 1) ^ (row & 3)) << 1) | (chunk & 1));
}

template <int D, int NT>
__device__ void segment_bf16(const AttnArgs& a, char* smem, const Item& it, int page0, int page1, int L,
                             bool complete, float* pslot) {
  using C = Bf16Cfg<D>;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int c = lane & 15;
  const int g = lane >> 4;
  const int R = it.nq * a.G;

  uint4* stage = (uint4*)(smem + wave * C::STAGE_BYTES);                // this wave's K0 K1 V0 V1
  uint4* qtile = (uint4*)(smem + NW * C::STAGE_BYTES);                  // [BF16_ROWS][CH] swizzled
  int* rowslot = (int*)(smem + NW * C::STAGE_BYTES + BF16_ROWS * D * 2);
  int* rowtag = rowslot + BF16_ROWS;
  float* wm = (float*)(rowtag + BF16_ROWS);                             // [NW][BF16_ROWS]
  float* wl = wm + NW * BF16_ROWS;

  __syncthreads();  // LDS of the previous segment is free
  // ---- Q tile and row descriptors into LDS (padding rows repeat the last row)
  for (int i = tid; i < 16 * NT * C::CH; i += THREADS) {
    const int r = i / C::CH, ch = i - r * C::CH;
    const int rr = min(r, R - 1);
    const int q = it.q0 + rr / a.G;
    const int head = it.h * a.G + rr % a.G;
    const uint4* src = (const uint4*)a.q + ((long)q * a.kv.num_q_heads + head) * C::CH + ch;
    qtile[k_swz<D>(r, ch)] = *src;
  }
  if (tid < 16 * NT) {
    const int rr = min(tid, R - 1);
    const int q = it.q0 + rr / a.G;
    rowslot[tid] = a.logical_slot[q];
    const int qb = a.q_branch[q];
    rowtag[tid] = (qb < 0 || !a.cu_branches) ? 0 : qb - a.cu_branches[it.s] + 1;
  }
  __syncthreads();

  int my_slot[NT], my_tag[NT];
  int mask_from = L;  // keys below this slot are visible to every row of the group
#pragma unroll
  for (int n = 0; n < NT; ++n) {
    my_slot[n] = rowslot[16 * n + c];
    my_tag[n] = rowtag[16 * n + c];
    mask_from = min(mask_from, my_slot[n]);
  }
#pragma unroll
  for (int off = 1; off < 16; off <<= 1) mask_from = min(mask_from, __shfl_xor(mask_from, off));

  f32x4 acc[NT][C::MT];
  float m_run[NT], l_run[NT];
#pragma unroll
  for (int n = 0; n < NT; ++n) {
    m_run[n] = -INFINITY;
    l_run[n] = 0.f;
#pragma unroll
    for (int mt = 0; mt < C::MT; ++mt) acc[n][mt] = f32x4{0.f, 0.f, 0.f, 0.f};
  }

  const int npairs = (page1 - page0 + 1) >> 1;
  const long bt_base = (long)it.s * a.kv.max_blocks_per_seq;
  const uint8_t* owner_row = a.slot_owner ? a.slot_owner + (long)it.s * a.owner_stride : nullptr;

  auto page_ptrs = [&](int pair, const uint4*& k0, const uint4*& k1, const uint4*& v0, const uint4*& v1) {
    const int P0 = page0 + 2 * pair;
    const int P1 = min(P0 + 1, page1 - 1);
    int b0 = __builtin_amdgcn_readfirstlane(a.kv.block_tables[bt_base + P0]);
    int b1 = __builtin_amdgcn_readfirstlane(a.kv.block_tables[bt_base + P1]);
    b0 = min(max(b0, 0), a.kv.num_blocks - 1);
    b1 = min(max(b1, 0), a.kv.num_blocks - 1);
    const long o0 = ((long)b0 * a.kv.num_kv_heads + it.h) * C::PAGE_U4;
    const long o1 = ((long)b1 * a.kv.num_kv_heads + it.h) * C::PAGE_U4;
    k0 = (const uint4*)a.kv.k + o0; v0 = (const uint4*)a.kv.v + o0;
    k1 = (const uint4*)a.kv.k + o1; v1 = (const uint4*)a.kv.v + o1;
  };

  uint4 ld[4][C::LPP];  // in-flight page pair: K0 K1 V0 V1
  auto issue = [&](int pair) {
    const uint4 *k0, *k1, *v0, *v1;
    page_ptrs(pair, k0, k1, v0, v1);
#pragma unroll
    for (int i = 0; i < C::LPP; ++i) {
      ld[0][i] = k0[i * 64 + lane];
      ld[1][i] = k1[i * 64 + lane];
      ld[2][i] = v0[i * 64 + lane];
      ld[3][i] = v1[i * 64 + lane];
    }
  };

  if (wave < npairs) issue(wave);
  for (int pair = wave; pair < npairs; pair += NW) {
    // ---- registers -> this wave's LDS stage (swizzled)
#pragma unroll
    for (int i = 0; i < C::LPP; ++i) {
      const int idx = i * 64 + lane;
      const int row = idx / C::CH, ch = idx % C::CH;
      stage[0 * C::PAGE_U4 + k_swz<D>(row, ch)] = ld[0][i];
      stage[1 * C::PAGE_U4 + k_swz<D>(row, ch)] = ld[1][i];
      stage[2 * C::PAGE_U4 + v_swz<D>(row, ch)] = ld[2][i];
      stage[3 * C::PAGE_U4 + v_swz<D>(row, ch)] = ld[3][i];
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    if (pair + NW < npairs) issue(pair + NW);  // next pair streams in while this one is computed

    const int P0 = page0 + 2 * pair;
    const bool second_valid = (P0 + 1) < page1;

    // ---- S^T = K Q^T for both pages
    f32x4 st[2][NT];
#pragma unroll
    for (int p = 0; p < 2; ++p)
#pragma unroll
      for (int n = 0; n < NT; ++n) st[p][n] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int t = 0; t < C::KSTEPS; ++t) {
      const bf16x8 ka = *(const bf16x8*)&stage[0 * C::PAGE_U4 + k_swz<D>(c, 4 * t + g)];
      const bf16x8 kb = *(const bf16x8*)&stage[1 * C::PAGE_U4 + k_swz<D>(c, 4 * t + g)];
#pragma unroll
      for (int n = 0; n < NT; ++n) {
        const bf16x8 qb = *(const bf16x8*)&qtile[k_swz<D>(16 * n + c, 4 * t + g)];
        st[0][n] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka, qb, st[0][n], 0, 0, 0);
        st[1][n] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kb, qb, st[1][n], 0, 0, 0);
      }
    }

    // ---- mask (only pages that reach into the branch region or the tail need it)
    const int slot0 = P0 * ASPD_BLOCK + 4 * g;  // first of this lane's four keys in page 0
    const bool need_mask = (P0 + 2) * ASPD_BLOCK > mask_from || !second_valid;
    uint32_t own0 = 0, own1 = 0;
    if (need_mask && owner_row) {
      own0 = *(const uint32_t*)(owner_row + slot0);
      own1 = *(const uint32_t*)(owner_row + min(slot0 + ASPD_BLOCK, a.owner_stride - 4));
    }

    s16x8 pb[NT];
#pragma unroll
    for (int n = 0; n < NT; ++n) {
      float sc[8];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        sc[e] = st[0][n][e] * a.scale_log2;
        sc[4 + e] = st[1][n][e] * a.scale_log2;
      }
      if (need_mask) {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const int j = slot0 + (e & 3) + (e >> 2) * ASPD_BLOCK;
          const int own = (int)(((e < 4 ? own0 : own1) >> (8 * (e & 3))) & 0xff);
          bool vis = (j <= my_slot[n]) && (j < L || my_tag[n] == 0 || own == my_tag[n]);
          if (e >= 4 && !second_valid) vis = false;
          sc[e] = vis ? sc[e] : -INFINITY;
        }
      }
      float mx = sc[0];
#pragma unroll
      for (int e = 1; e < 8; ++e) mx = fmaxf(mx, sc[e]);
      mx = fmaxf(mx, __shfl_xor(mx, 16));
      mx = fmaxf(mx, __shfl_xor(mx, 32));
      const float m_new = fmaxf(m_run[n], mx);
      const float m_ref = exp2_safe_ref(m_new);
      const float alpha = exp2f(m_run[n] - m_ref);
      m_run[n] = m_new;
      float psum = 0.f;
      float pr[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        pr[e] = exp2f(sc[e] - m_ref);
        psum += pr[e];
      }
      l_run[n] = l_run[n] * alpha + psum;
      if (__any(alpha != 1.f)) {
#pragma unroll
        for (int mt = 0; mt < C::MT; ++mt) acc[n][mt] *= alpha;
      }
      bf16x8 pv;
#pragma unroll
      for (int e = 0; e < 8; ++e) pv[e] = (__bf16)pr[e];
      pb[n] = __builtin_bit_cast(s16x8, pv);
    }

    // ---- O^T += V^T P^T
    const s16x4* vs0 = (const s16x4*)(stage + 2 * C::PAGE_U4);
    const s16x4* vs1 = (const s16x4*)(stage + 3 * C::PAGE_U4);
    const int vkey = 4 * g + (c >> 2);
#pragma unroll
    for (int mt = 0; mt < C::MT; ++mt) {
      // 8-byte units: a row has D/4 of them; 32-byte chunk mt is swizzled by the key
      const int unit = vkey * (D / 4) + (((mt ^ (vkey & 3)) << 2) | (c & 3));
      const s16x4 va = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
          (__attribute__((address_space(3))) s16x4*)(vs0 + unit));
      const s16x4 vb = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
          (__attribute__((address_space(3))) s16x4*)(vs1 + unit));
      s16x8 v8;
      v8[0] = va[0]; v8[1] = va[1]; v8[2] = va[2]; v8[3] = va[3];
      v8[4] = vb[0]; v8[5] = vb[1]; v8[6] = vb[2]; v8[7] = vb[3];
      const bf16x8 vop = __builtin_bit_cast(bf16x8, v8);
#pragma unroll
      for (int n = 0; n < NT; ++n)
        acc[n][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vop, __builtin_bit_cast(bf16x8, pb[n]),
                                                             acc[n][mt], 0, 0, 0);
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
  }

  // ---- combine the waves of the workgroup
#pragma unroll
  for (int n = 0; n < NT; ++n) {
    l_run[n] += __shfl_xor(l_run[n], 16);
    l_run[n] += __shfl_xor(l_run[n], 32);
    if (g == 0) {
      wm[wave * BF16_ROWS + 16 * n + c] = m_run[n];
      wl[wave * BF16_ROWS + 16 * n + c] = l_run[n];
    }
  }
  __syncthreads();  // also: every wave is done with its stage, which `red` aliases from here on
  float* red = (float*)smem;  // [NW][16][D]
#pragma unroll
  for (int n = 0; n < NT; ++n) {
    {
      float mg = -INFINITY;
#pragma unroll
      for (int w = 0; w < NW; ++w) mg = fmaxf(mg, wm[w * BF16_ROWS + 16 * n + c]);
      const float f = exp2f(m_run[n] - exp2_safe_ref(mg));
#pragma unroll
      for (int mt = 0; mt < C::MT; ++mt) {
        f32x4 v = acc[n][mt] * f;
        *(f32x4*)&red[(wave * 16 + c) * D + 16 * mt + 4 * g] = v;
      }
    }
    __syncthreads();
    {
      constexpr int PER = 16 * D / THREADS;  // consecutive floats per thread
      const int row = tid / (D / PER);
      const int d0 = (tid % (D / PER)) * PER;
      const int r = 16 * n + row;
      float mg = -INFINITY;
#pragma unroll
      for (int w = 0; w < NW; ++w) mg = fmaxf(mg, wm[w * BF16_ROWS + r]);
      const float mref = exp2_safe_ref(mg);
      float lg = 0.f;
#pragma unroll
      for (int w = 0; w < NW; ++w) lg += wl[w * BF16_ROWS + r] * exp2f(wm[w * BF16_ROWS + r] - mref);
      float o[PER];
#pragma unroll
      for (int e = 0; e < PER; ++e) {
        o[e] = 0.f;
#pragma unroll
        for (int w = 0; w < NW; ++w) o[e] += red[(w * 16 + row) * D + d0 + e];
      }
      if (r < R) {
        if (complete) {
          const int q = it.q0 + r / a.G;
          const int head = it.h * a.G + r % a.G;
          const float inv = 1.f / lg;
          __bf16* dst = (__bf16*)a.out + ((long)q * a.kv.num_q_heads + head) * D + d0;
#pragma unroll
          for (int e = 0; e < PER; ++e) dst[e] = (__bf16)(o[e] * inv);
          if (a.lse && d0 == 0) a.lse[(long)q * a.kv.num_q_heads + head] = (mg + log2f(lg)) * LN2;
        } else {
          float* dst = pslot + (long)r * (D + 2);
#pragma unroll
          for (int e = 0; e < PER; ++e) dst[d0 + e] = o[e];
          if (d0 == 0) {
            dst[D] = mg;
            dst[D + 1] = lg;
          }
        }
      }
    }
    __syncthreads();
  }
}

template <int D>
__global__ __launch_bounds__(THREADS) __attribute__((amdgpu_waves_per_eu(2, 2))) void attn_bf16_kernel(AttnArgs a) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  using C = Bf16Cfg<D>;
  // after the stages, the Q tile, row descriptors and wave statistics: the unit scan
  int* cu_units = (int*)(smem + NW * C::STAGE_BYTES + BF16_ROWS * D * 2 + 2 * BF16_ROWS * 4 +
                         2 * NW * BF16_ROWS * 4);
  int* scratch = (int*)smem;  // the stage area is idle until the first segment
  const int total = build_units(a, cu_units, scratch);
  const int chunk = chunk_of(total, a.nwg);
  const int begin = blockIdx.x * chunk;
  const int end = min(total, begin + chunk);
  int u = begin;
  while (u < end) {
    int page0;
    const Item it = locate(a, cu_units, u, &page0);
    const int page1 = min(it.np, page0 + (end - u));
    const bool complete = (page0 == 0) && (page1 == it.np);
    float* pslot = partial_slot(a, blockIdx.x, page0 == 0 ? 1 : 0, D);
    const int L = a.stage_base[it.s];
    const int nt = (it.nq * a.G + 15) >> 4;
    if (nt <= 1) segment_bf16<D, 1>(a, smem, it, page0, page1, L, complete, pslot);
    else if (nt == 2) segment_bf16<D, 2>(a, smem, it, page0, page1, L, complete, pslot);
    else segment_bf16<D, 3>(a, smem, it, page0, page1, L, complete, pslot);
    u += page1 - page0;
  }
}

template <int D>
size_t bf16_smem_bytes(int B) {
  return NW * Bf16Cfg<D>::STAGE_BYTES + BF16_ROWS * D * 2 + 2 * BF16_ROWS * 4 + 2 * NW * BF16_ROWS * 4 +
         (size_t)(B + 1) * 4;
}

// ---------------------------------------------------------------------------------------------
// fp32 path: vector ALU, fp32 throughout.  Lane (k = lane % 16, g = lane / 16) owns key k of each
// page and the g-th quarter of head_dim; a row's score is completed across the four quarters with
// two butterfly adds.  Every lane keeps a private running softmax over the keys it has seen
// (one per page) and they are combined once at the end of the segment.
// ---------------------------------------------------------------------------------------------
template <int D>
__device__ void segment_f32(const AttnArgs& a, char* smem, const Item& it, int page0, int page1, int L,
                            bool complete, float* pslot) {
  constexpr int QD = D / 4;  // floats per lane per key
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int k = lane & 15;
  const int g = lane >> 4;
  const int R = it.nq * a.G;

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
  const long bt_base = (long)it.s * a.kv.max_blocks_per_seq;
  const uint8_t* owner_row = a.slot_owner ? a.slot_owner + (long)it.s * a.owner_stride : nullptr;

  for (int P = page0 + wave; P < page1; P += NW) {
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
      if (vis) {  // lanes of one key agree on vis and on s, so their statistics stay identical
        const float m_new = fmaxf(m_run[r], s);
        const float alpha = exp2f(m_run[r] - m_new);
        const float p = exp2f(s - m_new);
        m_run[r] = m_new;
        l_run[r] = l_run[r] * alpha + p;
#pragma unroll
        for (int e = 0; e < QD; ++e) acc[r][e] = fmaf(p, kv_v[e], acc[r][e] * alpha);
      }
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
        float* dst = pslot + (long)r * (D + 2);
        dst[d] = o;
        if (d == 0) {
          dst[D] = mg;
          dst[D + 1] = lg;
        }
      }
    }
  }
}

template <int D>
size_t f32_smem_bytes(int B) {
  return F32_ROWS * D * 4 + 2 * F32_ROWS * 4 + (size_t)THREADS * F32_ROWS * (D / 4 + 2) * 4 + (size_t)(B + 1) * 4;
}

template <int D>
__global__ __launch_bounds__(THREADS) void attn_f32_kernel(AttnArgs a) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  int* cu_units = (int*)(smem + F32_ROWS * D * 4 + 2 * F32_ROWS * 4 +
                         (size_t)THREADS * F32_ROWS * (D / 4 + 2) * 4);
  int* scratch = (int*)(smem + F32_ROWS * D * 4 + 2 * F32_ROWS * 4);  // idle until the first segment ends
  const int total = build_units(a, cu_units, scratch);
  const int chunk = chunk_of(total, a.nwg);
  const int begin = blockIdx.x * chunk;
  const int end = min(total, begin + chunk);
  int u = begin;
  while (u < end) {
    int page0;
    const Item it = locate(a, cu_units, u, &page0);
    const int page1 = min(it.np, page0 + (end - u));
    const bool complete = (page0 == 0) && (page1 == it.np);
    float* pslot = partial_slot(a, blockIdx.x, page0 == 0 ? 1 : 0, D);
    segment_f32<D>(a, smem, it, page0, page1, a.stage_base[it.s], complete, pslot);
    u += page1 - page0;
  }
}

// ---------------------------------------------------------------------------------------------
// Merge of the partials of items that were split over several workgroups.  Workgroup w owns the
// item that starts inside w's share and runs past its end; the item's partials are w's
// "starts item" slot and the "continues item" slots of the following workgroups.
// ---------------------------------------------------------------------------------------------
template <int D, bool BF16>
__global__ __launch_bounds__(THREADS) void merge_kernel(AttnArgs a) {
  __shared__ int cu_units[ASPD_MAX_BATCH + 1];
  __shared__ int scratch[THREADS];
  const int total = build_units(a, cu_units, scratch);
  const int chunk = chunk_of(total, a.nwg);
  const int w = blockIdx.x;
  const long begin = (long)w * chunk;
  if (begin >= total) return;
  const int end = min((long)total, begin + chunk);
  int page;
  const Item it = locate(a, cu_units, end - 1, &page);
  const int item_end = it.first_unit + it.np;
  if (item_end <= end) return;               // the item finishes here: complete, or merged by its owner
  if (it.first_unit < begin) return;         // started in an earlier workgroup: that one owns it
  const int w_last = (item_end - 1) / chunk;
  const int R = it.nq * a.G;
  const int stride = a.rows_cap * (D + 2);
  for (int i = threadIdx.x; i < R * D; i += THREADS) {
    const int r = i / D, d = i - r * D;
    float mg = -INFINITY;
    for (int ww = w; ww <= w_last; ++ww) {
      const float* p = a.partial + (long)(2 * ww + (ww == w ? 1 : 0)) * stride + (long)r * (D + 2);
      mg = fmaxf(mg, p[D]);
    }
    const float mref = exp2_safe_ref(mg);
    float lg = 0.f, o = 0.f;
    for (int ww = w; ww <= w_last; ++ww) {
      const float* p = a.partial + (long)(2 * ww + (ww == w ? 1 : 0)) * stride + (long)r * (D + 2);
      const float f = exp2f(p[D] - mref);
      lg += p[D + 1] * f;
      o += p[d] * f;
    }
    const int q = it.q0 + r / a.G;
    const int head = it.h * a.G + r % a.G;
    const long oi = ((long)q * a.kv.num_q_heads + head) * D + d;
    if (BF16) ((__bf16*)a.out)[oi] = (__bf16)(o / lg);
    else ((float*)a.out)[oi] = o / lg;
    if (a.lse && d == 0) a.lse[(long)q * a.kv.num_q_heads + head] = (mg + log2f(lg)) * LN2;
  }
}

// ---------------------------------------------------------------------------------------------
// Host side
// ---------------------------------------------------------------------------------------------
int rows_per_group(const aspd_kv* kv, int* qpg) {
  const int G = kv->num_q_heads / kv->num_kv_heads;
  const int cap = (kv->dtype == ASPD_BF16) ? BF16_ROWS : F32_ROWS;
  if (G > cap) return 0;
  *qpg = cap / G;
  return cap;
}

int device_cu_count() {
  static int cached = 0;
  if (cached > 0) return cached;
  int dev = 0, n = 0;
  if (hipGetDevice(&dev) != hipSuccess) return 256;
  if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) return 256;
  cached = n;
  return n;
}

constexpr int LDS_BYTES = 160 * 1024;  // per compute unit on gfx950

// Dynamic LDS above 64 KB has to be allowed once per kernel and device.
int allow_big_lds(const void* kernel) {
  static std::mutex mu;
  static std::set<std::pair<int, const void*>> done;
  int dev = 0;
  ASPD_HIP_CHECK(hipGetDevice(&dev));
  std::lock_guard<std::mutex> lock(mu);
  if (done.count({dev, kernel})) return ASPD_OK;
  ASPD_HIP_CHECK(hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES));
  done.insert({dev, kernel});
  return ASPD_OK;
}

enum Mode { MODE_PARALLEL, MODE_CHUNK, MODE_SERIAL };

int attn_launch(Mode mode, const aspd_kv* kv, const aspd_state* state, const aspd_step* step, const void* q_d,
                void* out_d, float* lse_d, float sm_scale, void* workspace_d, size_t workspace_bytes,
                void* stream) {
  int rc = aspd_check_kv(kv);
  if (rc != ASPD_OK) return rc;
  if (!state || !step || state->B <= 0 || !state->stage_base_d || !state->seq_len_d) return ASPD_ERR_INVALID_ARG;
  if (state->B > ASPD_MAX_BATCH) return ASPD_ERR_UNSUPPORTED;
  if (step->NQ < 0 || !step->cu_seq_new_d) return ASPD_ERR_INVALID_ARG;
  if (step->NQ == 0) return ASPD_OK;
  if (!step->q_branch_d || !step->logical_slot_d || !q_d || !out_d) return ASPD_ERR_INVALID_ARG;
  if (((uintptr_t)q_d & 15) || ((uintptr_t)out_d & 15)) return ASPD_ERR_INVALID_ARG;
  if (!(sm_scale >= 0.f)) return ASPD_ERR_INVALID_ARG;
  const bool branches = (mode != MODE_SERIAL);
  if (branches) {
    if (!state->cu_branches_d || !state->slot_owner_d) return ASPD_ERR_INVALID_ARG;
    if (state->owner_stride < kv->max_blocks_per_seq * ASPD_BLOCK || (state->owner_stride & 3) ||
        ((uintptr_t)state->slot_owner_d & 3))
      return ASPD_ERR_INVALID_ARG;
  }
  int qpg = 0;
  const int rows_cap = rows_per_group(kv, &qpg);
  if (rows_cap == 0) return ASPD_ERR_UNSUPPORTED;
  const size_t need = aspd_workspace_bytes(kv, state->B, step->NQ);
  if (need == 0) return ASPD_ERR_INVALID_ARG;
  if (!workspace_d || ((uintptr_t)workspace_d & 255)) return ASPD_ERR_INVALID_ARG;
  if (workspace_bytes < need) return ASPD_ERR_WORKSPACE;

  AttnArgs a;
  a.kv = make_view(kv);
  a.stage_base = state->stage_base_d;
  a.seq_len = state->seq_len_d;
  a.cu_branches = branches ? state->cu_branches_d : nullptr;
  a.slot_owner = branches ? state->slot_owner_d : nullptr;
  a.owner_stride = branches ? state->owner_stride : 0;
  a.cu_seq_new = step->cu_seq_new_d;
  a.q_branch = step->q_branch_d;
  a.logical_slot = step->logical_slot_d;
  a.q = q_d;
  a.out = out_d;
  a.lse = lse_d;
  a.partial = (float*)workspace_d;
  a.scale_log2 = (sm_scale == 0.f ? 1.0f / sqrtf((float)kv->head_dim) : sm_scale) * LOG2E;
  a.B = state->B;
  a.G = kv->num_q_heads / kv->num_kv_heads;
  a.qpg = qpg;
  a.rows_cap = rows_cap;

  // Grid: two workgroups per compute unit, never more than the pages can feed.
  const long groups_max = (long)state->B + step->NQ / qpg;
  const long units_max = groups_max * kv->num_kv_heads * kv->max_blocks_per_seq;
  long nwg = 2L * device_cu_count();
  nwg = std::min(nwg, (units_max + MIN_PAGES_PER_WG - 1) / MIN_PAGES_PER_WG);
  nwg = std::max(1L, std::min(nwg, (long)MAX_WG));
  a.nwg = (int)nwg;

  hipStream_t hs = (hipStream_t)stream;
  const int D = kv->head_dim;
#define ASPD_LAUNCH(KERNEL, MERGE, SMEM)                                             \
  do {                                                                               \
    rc = allow_big_lds((const void*)KERNEL);                                         \
    if (rc != ASPD_OK) return rc;                                                    \
    if ((SMEM) > (size_t)LDS_BYTES) return ASPD_ERR_UNSUPPORTED;                     \
    hipLaunchKernelGGL(KERNEL, dim3(a.nwg), dim3(THREADS), SMEM, hs, a);             \
    ASPD_HIP_CHECK(hipGetLastError());                                               \
    hipLaunchKernelGGL(MERGE, dim3(a.nwg), dim3(THREADS), 0, hs, a);                 \
    ASPD_HIP_CHECK(hipGetLastError());                                               \
  } while (0)
  if (kv->dtype == ASPD_BF16) {
    if (D == 128) ASPD_LAUNCH(attn_bf16_kernel<128>, (merge_kernel<128, true>), bf16_smem_bytes<128>(state->B));
    else ASPD_LAUNCH(attn_bf16_kernel<64>, (merge_kernel<64, true>), bf16_smem_bytes<64>(state->B));
  } else {
    if (D == 128) ASPD_LAUNCH(attn_f32_kernel<128>, (merge_kernel<128, false>), f32_smem_bytes<128>(state->B));
    else ASPD_LAUNCH(attn_f32_kernel<64>, (merge_kernel<64, false>), f32_smem_bytes<64>(state->B));
  }
#undef ASPD_LAUNCH
  return ASPD_OK;
}

}  // namespace

extern "C" size_t aspd_workspace_bytes(const aspd_kv* kv, int32_t B, int32_t NQ) {
  if (!kv || B <= 0 || NQ < 0 || kv->num_kv_heads <= 0 || kv->num_q_heads <= 0) return 0;
  if (kv->head_dim != 64 && kv->head_dim != 128) return 0;
  if (kv->dtype != ASPD_F32 && kv->dtype != ASPD_BF16) return 0;
  int qpg = 0;
  const int rows_cap = rows_per_group(kv, &qpg);
  if (rows_cap == 0) return 0;
  // two partial slots per workgroup of the largest grid any device would get
  return (size_t)2 * MAX_WG * rows_cap * (kv->head_dim + 2) * sizeof(float);
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
