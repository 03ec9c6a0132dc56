// The per-step plan of the attention launches (internal to libaspd, not part of the public ABI).
//
// The three attention calls of a step (ASPD Sec. 3.2-3.3: parallel decode, branch chunk, serial
// decode) split the key ranges of their (sequence, row group, KV head) items among the workgroups of
// one launch.  How they are split depends on nothing but the lengths of the batch and a few launch
// constants, so it is worked out once per step, by a small kernel that runs right after the metadata
// kernel of aspd_build_branch_meta, and every attention launch of the step (one per layer) starts from
// the result: a workgroup loads its 128-byte header and has its first pages on their way after one
// memory round trip.
//
// Layout of a plan (32-bit words), for a grid of `nwg` workgroups:
//   [0, 32 nwg)                    one header per workgroup
//   [32 nwg, 32 nwg + 8 nsegs)     the segments that are not the first of their workgroup, in the
//                                  order the workgroups walk them
// Header: words 0-7 the workgroup's first segment, 8 the number of its segments (0: nothing to do),
//   9 the index of its second segment in the list above, 16-31 the block ids of the first sixteen
//   pages of its first segment (read again from the block table before they count, see the kernels).
// Segment: a run of pages [page0, page1) of one item, for all rows of the item's row group:
//   0  sequence | KV head << 16        1  first packed query row of the row group
//   2  queries of the row group        3  page0        4  page1
//   5  pages of the whole item (the segment is the whole item iff page0 = 0 and page1 = this)
//   6  first | last << 16 workgroup that holds a part of the item (they combine their partial results)
//   7  stage_base of the sequence
#pragma once

#include "aspd_common.h"

constexpr int PLAN_HDR = 32;         // words per workgroup header
constexpr int PLAN_SEG = 8;          // words per segment
constexpr int PLAN_HDR_NSEG = 8;
constexpr int PLAN_HDR_NEXT = 9;
constexpr int PLAN_HDR_IDS = 16;
constexpr int PLAN_IDS = 16;

constexpr int MAX_WG = 1024;         // upper bound of any attention grid
constexpr int NT_MAX = 3;            // 16-row MFMA tiles per row group of the streaming bf16 kernel
constexpr int F32_ROWS = 4;          // rows per row group of the fp32 kernel
constexpr int ROWS_NW = 8;           // waves per workgroup of the row-splitting (chunk) kernel
constexpr int ROWS_NT = 2;           // 16-row tiles per wave there
constexpr int MAX_WG_ROWS = 256;     // its largest grid
constexpr int MIN_PAGES_PER_WG = 16; // key ranges are not split finer than this
constexpr int PAD_STREAM = 32;       // fixed cost of a segment in pages, bandwidth-bound kernel at head_dim 128
constexpr int PAD_COMPUTE = 8;       // the same for the fp32 kernel
constexpr int PAD_ROWS = 32;         // and for the row-splitting kernel: a segment there costs about 17 us (Q operands
                                     // of 256 rows into registers, 64-128 KB of output or partial, its share of a
                                     // merge), 25-40 pages' worth; measured on a 64-sequence chunk step: 8 -> 828 us,
                                     // 16 -> 818, 24 -> 809, 32 -> 804, 48 -> 822, 64 -> 827

enum AttnKernel { KERNEL_F32 = 0, KERNEL_BF16_STREAM = 1, KERNEL_BF16_ROWS = 2 };

// Which kernel an attention call takes and how its launch is shaped: decided on the host from the
// cache's shape and the step's host fields, by the metadata call (which builds the plan for it) and by
// the attention call (which checks that the plan it is given was built for the same launch).
struct AttnVariant {
  int  kernel;       // AttnKernel
  int  nt;           // 16-row tiles per row group (streaming bf16 kernel)
  int  qpg;          // queries per row group
  int  rows_cap;     // rows per row group the partial slots are sized for
  int  nwg;          // workgroups of the launch
  int  pad;          // virtual pages in front of every item (ragged batches)
  bool stream_once;  // no page is read by more than one row group
  bool has_owner;    // rows may carry branch tags (all calls but serial decode)
};

// 0 when the shape is not supported.  `chunk_call`: the call is aspd_attn_branch_chunk (matters only
// when the step gives no bound on the new tokens per sequence).
int aspd_choose_variant(const aspd_kv* kv, int32_t B, int32_t NQ, int32_t max_new_per_seq, int32_t max_workgroups,
                        bool chunk_call, bool has_owner, AttnVariant* out);

// Identifies the launch a plan was built for; never 0.
uint64_t aspd_plan_key(const AttnVariant& v, int32_t B);

// Words a plan for `v` may take.
size_t aspd_plan_words(const aspd_kv* kv, const AttnVariant& v, int32_t B, int32_t NQ);

// Enqueues the kernel that writes the plan of the step for launch shape `v` to plan_d.
int aspd_plan_launch(const aspd_kv* kv, const AttnVariant& v, int32_t B, const int32_t* stage_base_d,
                     const int32_t* seq_len_d, const int32_t* cu_seq_new_d, int32_t* plan_d, hipStream_t stream);

// ---- The plan of a whole-sequence step (aspd_build_sequence_meta / aspd_attn_full_sequence) -------
// Layout (32-bit words):
//   [0, 16)                 header: 0 row groups in the list, 1 tokens per row group, 2 NQ, 3 B
//   [16, 16 + NQ4)          per packed row, the first slot of the row's own stage (its own slot for a
//                           main-branch row); NQ4 = NQ rounded up to a multiple of 4
//   then 4 words per row group, in the order workgroups take them: sequence, first packed row,
//                           tokens, pages of its key range
constexpr int SEQ_PLAN_HDR = 16;
// Tokens per row group: what the row-splitting kernel holds per workgroup.
static inline int aspd_sequence_qpg(int G) { return ROWS_NW * 16 * ROWS_NT / G; }
// Identifies such a plan; no value aspd_plan_key returns has bit 62 set.
static inline uint64_t aspd_sequence_plan_key(int qpg, int32_t B) {
  return ((uint64_t)1 << 62) | ((uint64_t)qpg << 16) | (uint64_t)B;
}
size_t aspd_sequence_plan_words(const aspd_kv* kv, int32_t B, int32_t NQ);

// Compute units of the current device (256 when there is none to ask, as on a build host).
int aspd_device_cu_count();
