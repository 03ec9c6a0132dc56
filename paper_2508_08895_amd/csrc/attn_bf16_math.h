// bf16 arithmetic of the attention kernels (internal to libaspd): LDS layout of a pair of pages, the MFMA
// products and the running softmax of one pair against a wave's row tiles.
#pragma once

#include "attn_common.h"

namespace {

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
// The operands are usually MFMA results, and a vector instruction that reads one too soon after the MFMA
// was issued gets the old register contents: the hardware does not interlock, the compiler pads with
// wait states for the instructions it emits itself, and it does not look into assembly.  So the block
// brings its own wait states (16: more than the 8-pass MFMA used here needs) and is ONE statement, so
// that no MFMA can be scheduled between them and the reads.
__device__ __forceinline__ float max8(const float (&x)[8]) {
  float r1, r2, m;
  asm("s_nop 15\n\t"
      "v_max3_f32 %0, %3, %4, %5\n\t"
      "v_max3_f32 %1, %6, %7, %8\n\t"
      "v_max3_f32 %2, %9, %10, %0\n\t"
      "v_max_f32 %2, %1, %2"
      : "=&v"(r1), "=&v"(r2), "=&v"(m)
      : "v"(x[0]), "v"(x[1]), "v"(x[2]), "v"(x[3]), "v"(x[4]), "v"(x[5]), "v"(x[6]), "v"(x[7]));
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

// ---------------------------------------------------------------------------------------------
// A staged group of PPS pairs of pages that every row of the wave sees in full (keys of the prefix and of
// earlier stages: most of a long context).  No mask, no owner tags, and straight-line code but for one rarely
// taken branch per group: all score products first, then one test whether any row's softmax reference must
// be raised (the lazy reference of pair_compute, against the largest score of the whole group), then the
// weights and second products of all pairs.  Counters on the general path show the row-splitting kernel
// bound by the number of instructions a wave issues per pair (about 240, of which 32 MFMA), not by a
// pipeline: this form issues about a third fewer.
// ---------------------------------------------------------------------------------------------
template <int D, int NT, int PPS>
__device__ __forceinline__ void group_compute_open(const u32x4* stage, RowState<D, NT>& ts, int kr_even, int kr_odd,
                                                   const int (&vu)[4], float scale_log2, const bf16x8* qr) {
  using C = Bf16Cfg<D>;
  // LDS operands are fetched a whole pair at a time and one step ahead of their use (the K pages of the next
  // pair before the score products of this one, the V pages of a pair before its weights are computed), so
  // that a wave waits for LDS once per phase and not once per MFMA.
  auto fetch_k = [&](const u32x4* sp, bf16x8 (&k)[2][C::KSTEPS]) {
#pragma unroll
    for (int t = 0; t < C::KSTEPS; ++t) {
      const int kr = ((t & 1) ? kr_odd : kr_even) + 8 * (t >> 1);
      k[0][t] = *(const bf16x8*)&sp[0 * C::LPAGE_U4 + kr];
      k[1][t] = *(const bf16x8*)&sp[1 * C::LPAGE_U4 + kr];
    }
  };
  auto fetch_v = [&](const u32x4* sp, bf16x8 (&v)[C::MT]) {
    const s16x4* vs0 = (const s16x4*)(sp + 2 * C::LPAGE_U4);
    const s16x4* vs1 = (const s16x4*)(sp + 3 * C::LPAGE_U4);
#pragma unroll
    for (int mt = 0; mt < C::MT; ++mt) {
      const int unit = vu[mt & 3] + 16 * (mt >> 2);
      const s16x4 va = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(vs0 + unit));
      const s16x4 vb = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(vs1 + unit));
      s16x8 v8;
      v8[0] = va[0]; v8[1] = va[1]; v8[2] = va[2]; v8[3] = va[3];
      v8[4] = vb[0]; v8[5] = vb[1]; v8[6] = vb[2]; v8[7] = vb[3];
      v[mt] = __builtin_bit_cast(bf16x8, v8);
    }
  };
  f32x4 st[PPS][2][NT];
  {
    bf16x8 kop[2][2][C::KSTEPS];
    fetch_k(stage, kop[0]);
#pragma unroll
    for (int h = 0; h < PPS; ++h) {
      if (h + 1 < PPS) fetch_k(stage + (h + 1) * 4 * C::LPAGE_U4, kop[(h + 1) & 1]);
#pragma unroll
      for (int n = 0; n < NT; ++n) st[h][0][n] = st[h][1][n] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int t = 0; t < C::KSTEPS; ++t) {
#pragma unroll
        for (int n = 0; n < NT; ++n) {
          st[h][0][n] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kop[h & 1][0][t], qr[n * C::KSTEPS + t], st[h][0][n], 0, 0, 0);
          st[h][1][n] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kop[h & 1][1][t], qr[n * C::KSTEPS + t], st[h][1][n], 0, 0, 0);
        }
      }
    }
  }
  bf16x8 vop[C::MT];
  fetch_v(stage, vop);
  // ---- the rows' references against the largest score of the group
  float mx[NT];
  bool up = false;
#pragma unroll
  for (int n = 0; n < NT; ++n) {
#pragma unroll
    for (int h = 0; h < PPS; ++h) {
      float sc[8];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        sc[e] = st[h][0][n][e];
        sc[4 + e] = st[h][1][n][e];
      }
      const float m8 = max8(sc);
      mx[n] = (h == 0) ? m8 : fmaxf(mx[n], m8);
    }
    mx[n] *= scale_log2;  // scale > 0: the maximum commutes with it
    up |= mx[n] > ts.m_run[n] + LAZY;
  }
  if (__any(up)) {
#pragma unroll
    for (int n = 0; n < NT; ++n) {
      float m = mx[n];
      m = fmaxf(m, __shfl_xor(m, 16));
      m = fmaxf(m, __shfl_xor(m, 32));
      const float m_new = fmaxf(ts.m_run[n], m);
      const float alpha = __builtin_amdgcn_exp2f(ts.m_run[n] - exp2_safe_ref(m_new));
      ts.m_run[n] = m_new;
      ts.l_run[n] *= alpha;
#pragma unroll
      for (int mt = 0; mt < C::MT; ++mt) ts.acc[n][mt] *= alpha;
    }
  }
  // ---- weights and second products
#pragma unroll
  for (int h = 0; h < PPS; ++h) {
    bf16x8 p[NT];
#pragma unroll
    for (int n = 0; n < NT; ++n) {
      const float neg_ref = -exp2_safe_ref(ts.m_run[n]);
      float psum = 0.f;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float w = __builtin_amdgcn_exp2f(fmaf(st[h][e >> 2][n][e & 3], scale_log2, neg_ref));
        psum += w;
        p[n][e] = (__bf16)w;
      }
      ts.l_run[n] += psum;
    }
#pragma unroll
    for (int mt = 0; mt < C::MT; ++mt) {
#pragma unroll
      for (int n = 0; n < NT; ++n) ts.acc[n][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vop[mt], p[n], ts.acc[n][mt], 0, 0, 0);
    }
    if (h + 1 < PPS) fetch_v(stage + (h + 1) * 4 * C::LPAGE_U4, vop);
  }
}

}  // namespace
