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
//
// One translation unit: attn_common.h (arguments, plan readers, partial slots), attn_bf16_math.h (one pair
// of pages against a wave's rows), attn_bf16_stream.h (the streaming kernel), attn_bf16_rows.h (the
// row-splitting kernels for chunks and whole sequences), attn_f32.h, attn_merge.h, and the host side below.
#include <algorithm>
#include <cmath>
#include <mutex>
#include <set>
#include <utility>

#include "aspd_plan.h"

#include "attn_common.h"
#include "attn_bf16_math.h"
#include "attn_bf16_stream.h"
#include "attn_bf16_rows.h"
#include "attn_f32.h"
#include "attn_merge.h"

namespace {

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
