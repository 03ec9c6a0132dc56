// aspd_rope_append: the step between the metadata and the attention call.  The position ids of
// ASPD Sec. 3.2, Eq. 4 act on the attention scores through the rotary encoding of the queries and
// keys; this kernel rotates the new tokens' Q rows in place, rotates their K rows into the paged
// cache at slot_mapping and copies their V rows there.
//
// Rotary encoding as defined by RoFormer, in the rotate-half layout: head_dim D is split into the
// pairs (i, i + D/2); pair i of a vector at position p turns by the angle p * theta^(-2i/D).
//
// Memory-trivial (a few hundred bytes per token and head), so the launch is shaped for latency: one
// workgroup per new token, a thread owns pair i of every HL-th head, the angle is formed in double
// (a float product would lose 1e-3 rad at positions of a few ten thousand) and its sine and cosine
// are computed once per thread.
#include "aspd_common.h"

namespace {

constexpr int ROPE_THREADS = 256;

template <typename T>
__device__ __forceinline__ float to_f32(T x) { return (float)x; }

template <typename T, int D>
__global__ __launch_bounds__(ROPE_THREADS) void rope_append_kernel(KvView kv, const int32_t* __restrict__ position_ids,
                                                                   const int64_t* __restrict__ slot_mapping, T* q,
                                                                   const T* __restrict__ k_new,
                                                                   const T* __restrict__ v_new, double log2_theta) {
  constexpr int HALF = D / 2;
  constexpr int HL = ROPE_THREADS / HALF;  // heads handled at once
  const int row = blockIdx.x;
  const int i = threadIdx.x % HALF;
  const int hsub = threadIdx.x / HALF;
  const int pos = position_ids[row];
  const long slot = slot_mapping[row];

  const double freq = exp2(-(2.0 * i / D) * log2_theta);
  double sn, cs;
  sincos((double)pos * freq, &sn, &cs);
  const float c = (float)cs, s = (float)sn;

  T* qrow = q + (long)row * kv.num_q_heads * D;
  for (int h = hsub; h < kv.num_q_heads; h += HL) {
    const float a = to_f32(qrow[h * D + i]);
    const float b = to_f32(qrow[h * D + i + HALF]);
    qrow[h * D + i] = (T)(a * c - b * s);
    qrow[h * D + i + HALF] = (T)(b * c + a * s);
  }
  if (slot < 0 || slot >= (long)kv.num_blocks * ASPD_BLOCK) return;  // never write outside the pools
  const long blk = slot / ASPD_BLOCK, off = slot % ASPD_BLOCK;
  const T* krow = k_new + (long)row * kv.num_kv_heads * D;
  const T* vrow = v_new + (long)row * kv.num_kv_heads * D;
  for (int h = hsub; h < kv.num_kv_heads; h += HL) {
    const long dst = ((blk * kv.num_kv_heads + h) * ASPD_BLOCK + off) * D;
    const float a = to_f32(krow[h * D + i]);
    const float b = to_f32(krow[h * D + i + HALF]);
    T* kc = (T*)kv.k + dst;
    T* vc = (T*)kv.v + dst;
    kc[i] = (T)(a * c - b * s);
    kc[i + HALF] = (T)(b * c + a * s);
    vc[i] = vrow[h * D + i];
    vc[i + HALF] = vrow[h * D + i + HALF];
  }
}

}  // namespace

extern "C" int aspd_rope_append(const aspd_kv* kv, const aspd_step* step, void* q_d, const void* k_new_d,
                                const void* v_new_d, float rope_theta, void* stream) {
  int rc = aspd_check_kv(kv);
  if (rc != ASPD_OK) return rc;
  if (!step || step->NQ < 0) return ASPD_ERR_INVALID_ARG;
  if (step->NQ == 0) return ASPD_OK;
  if (!step->position_ids_d || !step->slot_mapping_d || !q_d || !k_new_d || !v_new_d) return ASPD_ERR_INVALID_ARG;
  if (!(rope_theta > 1.f)) return ASPD_ERR_INVALID_ARG;
  const KvView kvv = make_view(kv);
  const double l2 = log2((double)rope_theta);
  hipStream_t hs = (hipStream_t)stream;
  const dim3 grid(step->NQ), block(ROPE_THREADS);
#define ASPD_ROPE(TYPE, DD)                                                                                   \
  hipLaunchKernelGGL((rope_append_kernel<TYPE, DD>), grid, block, 0, hs, kvv, step->position_ids_d,            \
                     step->slot_mapping_d, (TYPE*)q_d, (const TYPE*)k_new_d, (const TYPE*)v_new_d, l2)
  if (kv->dtype == ASPD_BF16) {
    if (kv->head_dim == 128) ASPD_ROPE(__bf16, 128); else ASPD_ROPE(__bf16, 64);
  } else {
    if (kv->head_dim == 128) ASPD_ROPE(float, 128); else ASPD_ROPE(float, 64);
  }
#undef ASPD_ROPE
  ASPD_HIP_CHECK(hipGetLastError());
  return ASPD_OK;
}
