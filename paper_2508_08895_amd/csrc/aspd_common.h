// Internal helpers shared by the gfx950 kernels of libaspd (not part of the public ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "aspd.h"

#define ASPD_BLOCK 16  // tokens per KV block (the only block size the kernels are written for)

#define ASPD_HIP_CHECK(expr)                       \
  do {                                             \
    hipError_t _e = (expr);                        \
    if (_e != hipSuccess) return ASPD_ERR_HIP;     \
  } while (0)

// Flat-argument views of the public structs: kernels take these by value.
struct KvView {
  const void*    k;
  const void*    v;
  const int32_t* block_tables;
  int32_t        num_blocks, num_q_heads, num_kv_heads, head_dim, max_blocks_per_seq;
};

struct StateView {
  int32_t        B, NB;
  int32_t*       stage_base;
  int32_t*       seq_len;
  const int32_t* cu_branches;
  int32_t*       branch_len;
  uint8_t*       slot_owner;
  int32_t        owner_stride;
  int32_t*       fault;
  int32_t*       main_pos;
  int32_t*       stage_open;
};

struct StepView {
  int32_t  NQ;
  int32_t  max_new_per_seq;
  int32_t* cu_new;
  int32_t* cu_seq_new;
  int32_t* q_seq;
  int32_t* q_branch;
  int32_t* position_ids;
  int32_t* logical_slot;
  int64_t* slot_mapping;
  int32_t* kv_len;
};

static inline KvView make_view(const aspd_kv* kv) {
  return KvView{kv->k_cache_d, kv->v_cache_d, kv->block_tables_d, kv->num_blocks, kv->num_q_heads,
                kv->num_kv_heads, kv->head_dim, kv->max_blocks_per_seq};
}
static inline StateView make_view(const aspd_state* st) {
  return StateView{st->B, st->NB, st->stage_base_d, st->seq_len_d, st->cu_branches_d, st->branch_len_d,
                   st->slot_owner_d, st->owner_stride, st->fault_d, st->main_pos_d, st->stage_open_d};
}
static inline StepView make_view(const aspd_step* sp) {
  return StepView{sp->NQ, sp->max_new_per_seq, sp->cu_new_d, sp->cu_seq_new_d, sp->q_seq_d, sp->q_branch_d, sp->position_ids_d,
                  sp->logical_slot_d, sp->slot_mapping_d, sp->kv_len_d};
}

// Host-side validation of the cache descriptor; returns an ASPD_* code.
int aspd_check_kv(const aspd_kv* kv);
