/* aspd.h - branch-isolated attention over one reusable paged KV cache, for AMD MI355X (gfx950).
 *
 * The operations are those of the Hybrid Decoding Engine of "ASPD: Adaptive Serial-Parallel
 * Decoding" (arXiv 2508.08895), Sec. 3.2-3.3.  A sequence is decoded in stages.  In a serial stage
 * one main branch grows token by token.  In a parallel stage K branches grow at once; a branch token
 * attends the tokens of all earlier stages plus the earlier tokens of its own branch, never a sibling
 * branch (Eq. 2-3), and branches share position ids at equal depth (Eq. 4).  After the stage the
 * main branch attends everything; the KV cache is reused as it is, nothing is recomputed or moved.
 *
 * Conventions fixed here where the paper leaves them open:
 *   - Position ids are 0-based (Eq. 4 minus one; rotary encodings see differences only).
 *   - A token sees itself (Eq. 2 read as pos(i) > pos(j) or i = j).
 *   - One cache per sequence, addressed by LOGICAL SLOT = index of the token in append order.
 *     One append call lays its new tokens at the tail ordered by (branch ascending, token
 *     ascending).  Physical slot = block_tables[s][slot / block_size] * block_size + slot % block_size.
 *   - Query head h reads KV head h / (num_q_heads / num_kv_heads).  Scores are scaled by
 *     sm_scale (0 selects 1/sqrt(head_dim), Eq. 1); natural exponent.
 *   - The K/V rows of the tokens of an append call must already be in the cache (at
 *     slot_mapping) when the attention call for them runs.
 *
 * Memory: every pointer named *_d is DEVICE memory owned by the caller.  Structs themselves are
 * host memory, read during the call only.  The library allocates nothing, frees nothing, never
 * synchronises: each call enqueues kernels on `stream` (a hipStream_t passed as void*; NULL = the
 * default stream) and returns.  Calls read no device data on the host, so they may be captured
 * into a HIP graph.
 *
 * Errors: every entry point returns ASPD_OK (0) or a negative code.  Host-checkable arguments are
 * validated before anything is launched; contents of device arrays are trusted, except that
 * aspd_build_branch_meta never writes outside the arrays described to it (see aspd_state.fault_d).
 */
#ifndef ASPD_H
#define ASPD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#if defined(__GNUC__)
#define ASPD_API __attribute__((visibility("default")))
#else
#define ASPD_API
#endif

#define ASPD_OK               0
#define ASPD_ERR_INVALID_ARG (-1) /* null pointer, negative size, misaligned buffer            */
#define ASPD_ERR_UNSUPPORTED (-2) /* dtype / head_dim / block_size / head ratio / batch limits */
#define ASPD_ERR_WORKSPACE   (-3) /* workspace_bytes below aspd_workspace_bytes(...)           */
#define ASPD_ERR_HIP         (-4) /* a HIP call or launch failed                               */
#define ASPD_ERR_SCRATCH_LIMIT (-5) /* aspd_attn_parallel_decode_static: the call needs more scratch
                                       than ASPD_STATIC_SCRATCH_BYTES                             */

#define ASPD_F32  0 /* fp32 in, fp32 accumulate, fp32 out                                 */
#define ASPD_BF16 1 /* bf16 in, fp32 accumulate, bf16 out (round to nearest even)         */

#define ASPD_STAGE_PARALLEL 0 /* append new_len[b] tokens to branch b of the running parallel stage */
#define ASPD_STAGE_SERIAL   1 /* append new_len[s] main-branch tokens to sequence s                 */
#define ASPD_STAGE_MERGE    2 /* the parallel stage ends; no token is appended, no KV is touched     */
#define ASPD_STAGE_MIXED    3 /* PARALLEL for the sequences with open branches, SERIAL for the others */

/* Position-id paradigms (Sec. 4.5.3).  What a token may attend to is the same under all of them. */
#define ASPD_POS_SAME_SEQ 0 /* Eq. 4 as adopted by the paper ("Same-Sequential"): after a parallel stage
                               the main branch continues at the number of tokens decoded so far         */
#define ASPD_POS_SAME_MAX 1 /* branches share positions as in Eq. 4; after the stage the main branch
                               continues right after the largest position any branch reached           */
#define ASPD_POS_FIX_N(n) (2 | ((n) << 8)) /* branch k of a stage owns the pre-allocated interval
                               [stage_start + k n, stage_start + (k+1) n), 1 <= n < 2^22; the main branch
                               continues after the last interval                                        */

#define ASPD_MAX_BATCH             512  /* sequences per call                                      */
#define ASPD_MAX_BRANCHES_PER_SEQ  255  /* owner tags are one byte                                 */

/* bits of *aspd_state.fault_d */
#define ASPD_FAULT_BLOCK_TABLE 1 /* a sequence outgrew max_blocks_per_seq or hit a negative block id */
#define ASPD_FAULT_OWNER_ROW   2 /* a sequence outgrew owner_stride                                   */
#define ASPD_FAULT_ROW_COUNT   4 /* the sum of new_len exceeded aspd_step.NQ                          */
#define ASPD_FAULT_BRANCHES    8 /* a sequence has more than ASPD_MAX_BRANCHES_PER_SEQ branches        */
#define ASPD_FAULT_STAGE      16 /* main-branch tokens for a sequence whose parallel stage has not been
                                    merged, or a running stage whose branch count changes             */
#define ASPD_FAULT_INTERVAL   32 /* ASPD_POS_FIX_N: a branch would outgrow its interval of n positions  */

/* The one reusable KV cache (paper: abstract, Sec. 2.3).  K and V each are
 * [num_blocks][num_kv_heads][block_size][head_dim] elements of `dtype`, so the rows one KV head
 * keeps for one block are one contiguous page.  block_size must be 16; head_dim 64 or 128;
 * num_q_heads a multiple of num_kv_heads.  "Contiguous KV" is the identity block table. */
typedef struct aspd_kv {
  void*          k_cache_d;
  void*          v_cache_d;
  const int32_t* block_tables_d; /* [B][max_blocks_per_seq], physical block of logical block i */
  int32_t        num_blocks;
  int32_t        block_size;
  int32_t        num_q_heads;
  int32_t        num_kv_heads;
  int32_t        head_dim;
  int32_t        max_blocks_per_seq;
  int32_t        dtype;          /* ASPD_F32 | ASPD_BF16 */
} aspd_kv;

/* Decode state of a batch.  Caller-owned; only aspd_build_branch_meta writes it.
 * Sequence s: slots [0, stage_base[s]) are visible to every current query (everything before the
 * running parallel stage: Eq. 3, "different stage"); slots [stage_base[s], seq_len[s]) belong to the
 * branches of the running parallel stage, slot j to branch slot_owner[s][j] in 1..K_s.  Branches are
 * numbered globally over the batch: sequence s owns branches [cu_branches[s], cu_branches[s+1]).
 * To open a parallel stage the caller provides cu_branches and zeroes branch_len (stage_base equals
 * seq_len after any serial append or merge). */
typedef struct aspd_state {
  int32_t        B;              /* sequences                                                      */
  int32_t        NB;             /* branches over the whole batch (0 when every sequence is serial) */
  int32_t*       stage_base_d;   /* [B]                                                            */
  int32_t*       seq_len_d;      /* [B]  logical slots in use                                      */
  const int32_t* cu_branches_d;  /* [B+1] exclusive scan of branches per sequence                  */
  int32_t*       branch_len_d;   /* [NB] tokens held by each branch                                */
  uint8_t*       slot_owner_d;   /* [B][owner_stride], indexed by logical slot                     */
  int32_t        owner_stride;
  int32_t*       fault_d;        /* nullable; ASPD_FAULT_* bits are OR-ed in, tokens that would not
                                    fit are dropped instead of written out of bounds               */
  int32_t*       main_pos_d;     /* [B] position id the next main-branch token of each sequence takes.
                                    Required (and kept up to date by aspd_build_branch_meta, from 0 for
                                    an empty sequence) for ASPD_POS_SAME_MAX and ASPD_POS_FIX_N, where it
                                    differs from seq_len; may be NULL for ASPD_POS_SAME_SEQ              */
  int32_t*       stage_open_d;   /* [B] 1 while the sequence is in a parallel stage, tokens or not; 0 otherwise.
                                    Set by aspd_renumber_branches (sequences that are given branches) and by
                                    PARALLEL / MIXED appends, cleared by MERGE; a caller that opens a stage by
                                    writing cu_branches itself sets it too.  Required for ASPD_POS_FIX_N, whose
                                    intervals are spent when the stage opens (a stage that ends without a
                                    token cannot be told from no stage by stage_base and seq_len); may be
                                    NULL otherwise                                                        */
} aspd_state;

/* What one aspd_build_branch_meta call produces for the NQ tokens it appends (caller-allocated).
 * Packed row order: sequence-major, then branch, then token: the order of the query rows in
 * q_d / out_d of the attention call that follows. */
typedef struct aspd_step {
  int32_t  NQ;              /* host: total tokens appended (sum of new_len)                        */
  int32_t  max_new_per_seq; /* host: upper bound of the tokens this step appends to any ONE sequence,
                               0 = unknown.  A tuning hint for the attention calls only (it sizes the
                               row tile); results do not depend on it, even when it is wrong.        */
  int32_t  max_workgroups;  /* host: most workgroups an attention launch of this step may use, for callers
                               that run other kernels next to attention and want compute units left for
                               them; 0 = one per compute unit.  Results do not depend on it.            */
  int32_t  shared_mask;     /* host: 0 = the branch-independent mask of Eq. 2-3 (the paper's choice); 1 = the
                               "Shared" mask of the ablation (Sec. 4.5.2, Table "PosId x mask"): branch tokens are
                               treated like main-branch tokens, every row attends every slot of its sequence up
                               to and including its own, sibling branches included.  Read by the metadata call
                               (for the plan) and by aspd_attn_parallel_decode / aspd_attn_branch_chunk        */
  int32_t* cu_new_d;        /* [NB+1] (PARALLEL) or [B+1] (SERIAL): first row of each branch / sequence */
  int32_t* cu_seq_new_d;    /* [B+1] first row of each sequence                                    */
  int32_t* q_seq_d;         /* [NQ] sequence of the token                                          */
  int32_t* q_branch_d;      /* [NQ] global branch index, -1 for main-branch tokens                 */
  int32_t* position_ids_d;  /* [NQ] Eq. 4, 0-based                                                 */
  int32_t* logical_slot_d;  /* [NQ]                                                                */
  int64_t* slot_mapping_d;  /* [NQ] physical slot: where the caller writes the token's K and V      */
  int32_t* kv_len_d;        /* [NQ] number of keys the token attends to, itself included           */
  int32_t* plan_d;          /* nullable, 256-byte aligned, plan_bytes >= aspd_plan_bytes(kv, B, NQ): the plan of
                               the step's attention launches (which workgroup reads which pages for which
                               rows), written by aspd_build_branch_meta and read by every attention call of
                               the step, i.e. by all layers.  Without it each attention call works the plan
                               out itself (one more small kernel per call)                              */
  size_t   plan_bytes;
  uint64_t plan_key;        /* host, written by aspd_build_branch_meta: the launch shape the plan in plan_d
                               was built for (0: none).  An attention call whose shape differs (the two
                               hints above were changed, or aspd_attn_branch_chunk is called on a step that
                               gives no max_new_per_seq) ignores the plan and builds its own           */
} aspd_step;

/* Sec. 3.2 Eq. 4 and the bookkeeping behind Eq. 2-3; Sec. 3.3 for the stage switches.
 * PARALLEL: new_len_d[NB]; token t (0-based, counting tokens already held) of a branch of sequence s
 *   gets position stage_base[s] + t; branch_len and seq_len grow; slot_owner is tagged.  Entries may
 *   be 0 (finished branch: its KV stays, it gets no query) or > 1 (chunk append).
 * SERIAL:   new_len_d[B]; main-branch token gets position = number of tokens already in the sequence
 *   (its flattened index); seq_len grows and stage_base follows it.  state->NB / branch arrays unused.
 *   A sequence whose parallel stage has not been merged (stage_base < seq_len, or stage_open set) takes
 *   no main-branch token: it is left as it is and ASPD_FAULT_STAGE is raised.
 * MERGE:    out may be NULL; stage_base[s] <- seq_len[s] for every sequence, or, when new_len_d is
 *   given, for the sequences with new_len_d[s] != 0 ([B]; Sec. 3.3: every response switches modes on
 *   its own).  No KV is read or written.
 * MIXED:    new_len_d[NB + B]: first the tokens per open branch as in PARALLEL, then the main-branch
 *   tokens per sequence as in SERIAL.  A sequence that owns branches (cu_branches) takes its branch
 *   entries and must have main entry 0; a sequence that owns none takes its main entry.  Rows stay
 *   sequence-major; out->cu_new_d [NB+1] holds the first row of every branch, then NQ.  The attention
 *   call for such a step is aspd_attn_parallel_decode or aspd_attn_branch_chunk.
 * pos_mode: one of ASPD_POS_*, the same in every call on a state.  out->NQ must equal the sum of new_len (known to the caller;
 * rows beyond it are dropped and ASPD_FAULT_ROW_COUNT is raised).
 * When out->plan_d is given, a second small kernel writes the step's attention plan there, for the launch
 * shape that out->max_new_per_seq and out->max_workgroups select, and out->plan_key (a HOST field of the
 * caller's struct, the only one the library writes) names that shape.  The plan holds copies of block-table
 * entries; the attention kernels check them against the block table they are given. */
ASPD_API int aspd_build_branch_meta(const aspd_kv* kv, aspd_state* state, int32_t stage, int32_t pos_mode,
                           const int32_t* new_len_d, aspd_step* out, void* stream);

/* Sequences open and end their parallel stages at different times (Sec. 3.3), which renumbers the
 * batch's branches.  Given the new exclusive scan of branches per sequence, writes the new branch_len
 * array [new NB]: the branches of a stage still running (stage_base < seq_len; their count must not
 * change, else ASPD_FAULT_STAGE) keep the tokens they hold, every other entry starts at 0.  The new
 * arrays must not be the ones in `state`; afterwards the caller points state->cu_branches_d,
 * branch_len_d and NB at them.  Reads no KV. */
ASPD_API int aspd_renumber_branches(const aspd_state* state, const int32_t* new_cu_branches_d,
                                    int32_t* new_branch_len_d, void* stream);

/* The step between aspd_build_branch_meta and the attention call: Eq. 4's position ids act on the
 * scores through the rotary encoding of queries and keys (RoFormer's definition, rotate-half layout:
 * pairs (i, i + head_dim/2), pair i turns by position * rope_theta^(-2i/head_dim); the layout of the
 * base models of Sec. 4).  For every new token r of `step`:
 *   q_d[r]      [num_q_heads][head_dim]  rotated in place by position_ids[r];
 *   k_new_d[r]  [num_kv_heads][head_dim] rotated and written to the cache at slot_mapping[r];
 *   v_new_d[r]  [num_kv_heads][head_dim] written to the cache at slot_mapping[r] as it is.
 * All three are device arrays of kv->dtype, rows in the packed order of the step.  Arithmetic in
 * fp32 with the angle formed in fp64; bf16 results are rounded to nearest even.  rope_theta > 1. */
ASPD_API int aspd_rope_append(const aspd_kv* kv, const aspd_step* step, void* q_d, const void* k_new_d,
                              const void* v_new_d, float rope_theta, void* stream);

/* Bytes of device scratch the attention calls of a step with NQ rows need at most: arrival counters, room
 * for a plan, and the partial softmax results of split key ranges (host-only computation; sized for the
 * current device's compute units, for 256 of them when there is no device).  Returns 0 on invalid arguments. */
ASPD_API size_t aspd_workspace_bytes(const aspd_kv* kv, int32_t B, int32_t NQ);

/* Bytes a step's plan buffer (aspd_step.plan_d) needs at most for B sequences and NQ rows (host-only). */
ASPD_API size_t aspd_plan_bytes(const aspd_kv* kv, int32_t B, int32_t NQ);

/* Prepares a freshly allocated workspace (256-byte aligned, at least aspd_workspace_bytes): enqueues
 * a small kernel that clears the arrival counters at its head.  Call once after allocation, on the stream
 * (or ordered before the stream) of the first attention call.  Attention calls leave the counters
 * cleared, so one workspace serves any number of calls, one at a time: two attention calls that run
 * concurrently must not share a workspace.  Nothing else in the workspace outlives a call. */
ASPD_API int aspd_workspace_init(void* workspace_d, size_t workspace_bytes, void* stream);

/* Sec. 3.2 Eq. 1-3, "The Parallel Branch's Perspective"; Sec. 3.3.  One new token per active branch
 * (the step built with ASPD_STAGE_PARALLEL and new_len in {0,1}): row r attends slots
 * [0, stage_base) plus the slots of its own branch up to and including its own.
 * q_d, out_d: [NQ][num_q_heads][head_dim] in kv->dtype, 16-byte aligned.  lse_d: nullable
 * [NQ][num_q_heads] float, natural-log sum of exp of the scaled scores.  workspace_d: 256-byte
 * aligned.  The KV pages shared by the branches of a sequence are read once for all of them. */
ASPD_API int aspd_attn_parallel_decode(const aspd_kv* kv, const aspd_state* state, const aspd_step* step,
                              const void* q_d, void* out_d, float* lse_d, float sm_scale,
                              void* workspace_d, size_t workspace_bytes, void* stream);

/* Sec. 3.3 (the per-branch prefix the engine forces at the start of each branch) under the mask
 * of Eq. 2-3: a step built with ASPD_STAGE_PARALLEL and any new_len >= 0.  Chunk token j of branch b
 * attends [0, stage_base), b's earlier tokens, and b's chunk tokens up to and including j.
 * Arguments as aspd_attn_parallel_decode. */
ASPD_API int aspd_attn_branch_chunk(const aspd_kv* kv, const aspd_state* state, const aspd_step* step,
                           const void* q_d, void* out_d, float* lse_d, float sm_scale,
                           void* workspace_d, size_t workspace_bytes, void* stream);

/* Sec. 3.2 "The Main Branch's Perspective"; Eq. 3 case 1.  Rows of a step built with
 * ASPD_STAGE_SERIAL: each attends every slot of its sequence up to and including its own -
 * serial prefix, all branches of all finished parallel stages, earlier main tokens.
 * Arguments as aspd_attn_parallel_decode (state->NB and branch arrays unused). */
ASPD_API int aspd_attn_serial_decode(const aspd_kv* kv, const aspd_state* state, const aspd_step* step,
                            const void* q_d, void* out_d, float* lse_d, float sm_scale,
                            void* workspace_d, size_t workspace_bytes, void* stream);

/* ---- A whole sequence in one call (teacher forcing, re-prefill) -----------------------------------
 * Fig. 5 (training arrangement: the branches of a stage laid one after the other), Eq. 2-4 over all
 * tokens of a multi-stage sequence at once, and the re-prefill that the "Same-Re" paradigm of Sec. 4.5.3
 * performs after every stage.  The cache of every sequence is (re)built from slot 0.
 *
 * The layout of sequence s is the list of its runs cu_runs[s] .. cu_runs[s+1]-1 in cache order.  Run r holds
 * run_len[r] >= 0 consecutive tokens of one branch: run_branch[r] = 0 for main-branch tokens, k >= 1 for the
 * k-th branch of a parallel stage.  A parallel stage is a succession of runs numbered 1, 2, .., K (K <=
 * ASPD_MAX_BRANCHES_PER_SEQ), each branch exactly one run; a run numbered 1 always opens a new stage.  Any
 * other numbering raises ASPD_FAULT_LAYOUT and leaves the sequence without tokens.
 * At most ASPD_MAX_RUNS_PER_SEQ runs per sequence. */
#define ASPD_MAX_RUNS_PER_SEQ 2048
#define ASPD_FAULT_LAYOUT     64 /* aspd_build_sequence_meta: branch runs of a stage not numbered 1..K in order,
                                    or too many runs                                                      */
typedef struct aspd_layout {
  int32_t        num_runs;      /* host: R, runs over the whole batch                                  */
  const int32_t* cu_runs_d;     /* [B+1] exclusive scan of runs per sequence                            */
  const int32_t* run_branch_d;  /* [R]                                                                  */
  const int32_t* run_len_d;     /* [R]                                                                  */
} aspd_layout;

/* Bytes of aspd_step.plan_d that aspd_build_sequence_meta needs for a batch of B sequences and NQ tokens
 * (0 for arguments the library does not support). */
ASPD_API size_t aspd_sequence_plan_bytes(const aspd_kv* kv, int32_t B, int32_t NQ);

/* Metadata of all tokens of the batch, row r of sequence s being the token at logical slot r - cu_seq_new[s]:
 * position ids by Eq. 4 under pos_mode (main-branch tokens as in ASPD_STAGE_SERIAL appends, tokens of a stage
 * as in one ASPD_STAGE_PARALLEL append of whole branches, every stage followed by a merge), logical and
 * physical slots, kv_len (the keys Eq. 2-3 let the token see, itself included), q_seq, and in q_branch the
 * token's branch number within its own stage minus one (-1 for main-branch tokens).  cu_new_d is not
 * written.  out->NQ must equal the sum of run_len (else ASPD_FAULT_ROW_COUNT); out->plan_d is required
 * (aspd_sequence_plan_bytes): it receives, per row, the first slot of the row's own stage, and the list of
 * row groups the attention call works through.  The state is left as after a merge of the last stage:
 * seq_len = stage_base = tokens of the sequence, stage_open = 0, main_pos = the next main-branch position,
 * branch_len of the sequence's entries untouched; slot_owner[s][j] = branch number of slot j within its
 * stage (0 for main-branch slots).  Decoding continues from there with aspd_build_branch_meta.
 * Faults as in aspd_build_branch_meta (a sequence that does not fit its block table or owner row, or breaks
 * the layout rules, gets no tokens: seq_len = 0, the packed rows its layout gave it stay unwritten and the
 * attention call skips them; ASPD_FAULT_ROW_COUNT accompanies the cause). */
ASPD_API int aspd_build_sequence_meta(const aspd_kv* kv, aspd_state* state, const aspd_layout* layout,
                                      int32_t pos_mode, aspd_step* out, void* stream);

/* Eq. 1-3 for every token of every sequence in one launch: row r attends the slots up to and including its
 * own that are main-branch slots, slots of other stages, or slots of its own branch.  `step` is one built by
 * aspd_build_sequence_meta (anything else: ASPD_ERR_INVALID_ARG); the K and V rows of all its tokens are in
 * the cache (aspd_rope_append with the same step writes them).  bf16 only (ASPD_ERR_UNSUPPORTED for fp32).
 * Key pages beyond a row group's last slot are never read, and a wave skips the pages of a stage that hold
 * only sibling branches of its rows.  With step->shared_mask = 1 every row attends every slot up to and including its
 * own (plain causal attention over the sequence: the "Shared" mask of Sec. 4.5.2, and what a re-prefill of a
 * sequence without parallel stages computes).  Other arguments as aspd_attn_parallel_decode; the workspace needs
 * aspd_workspace_bytes(kv, B, NQ) like any other call (only its counters are used). */
ASPD_API int aspd_attn_full_sequence(const aspd_kv* kv, const aspd_state* state, const aspd_step* step,
                                     const void* q_d, void* out_d, float* lse_d, float sm_scale,
                                     void* workspace_d, size_t workspace_bytes, void* stream);

/* aspd_attn_parallel_decode for callers that cannot allocate device memory (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): same arguments without the workspace,
 * same results.  The scratch is an array inside the library's code object, ASPD_STATIC_SCRATCH_BYTES per
 * device, held from the first use on that device until the process ends; the call allocates and frees
 * nothing.  A call whose grid and row groups need more (ASPD_ERR_SCRATCH_LIMIT; on a device of 256 compute
 * units every step with up to 48 query rows per sequence and KV head fits, as does any fp32 step) has to
 * go through aspd_attn_parallel_decode with a workspace.  All calls on one device share the one array:
 * two of them must not run concurrently (they would mix their partial results), and the first call on a
 * device looks the array's address up, so make it outside graph capture. */
#define ASPD_STATIC_SCRATCH_BYTES ((size_t)16 << 20)
ASPD_API int aspd_attn_parallel_decode_static(const aspd_kv* kv, const aspd_state* state, const aspd_step* step,
                                              const void* q_d, void* out_d, float* lse_d, float sm_scale,
                                              void* stream);

/* Measurement aid, not part of the method: enqueues one plain, fully coalesced read of
 * bytes / 16 * 16 bytes from src_d (16-byte aligned) and writes one 32-bit word per workgroup to
 * sink_d (room for 64 KiB is enough on any device).  Benchmarks time it to report what a read-only
 * stream reaches on the device at hand, next to the 8 TB/s datasheet figure, and profilers use its
 * known size to calibrate HBM byte counters. */
ASPD_API int aspd_probe_read_bandwidth(const void* src_d, size_t bytes, void* sink_d, void* stream);

/* Static string for a return code. */
ASPD_API const char* aspd_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* ASPD_H */
