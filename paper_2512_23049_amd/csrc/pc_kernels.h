// Launch wrappers of the kernels (internal to the library).
#ifndef PC_KERNELS_H_
#define PC_KERNELS_H_

#include "pc_internal.h"

void pc_launch_append(int dtype, const void *k, const void *v, int len, int n_kv_heads, int D,
                      int64_t slot_start, int64_t slots, const double *inv_freq, void *k_store,
                      void *v_store, PcMsgEntry *table, int msg_id, hipStream_t st);

// several whole messages in one launch
void pc_launch_append_batch(int dtype, const PcAppendItem *items, int n_items, int max_len, int n_kv_heads, int D,
                            int64_t slots, const double *inv_freq, void *k_store, void *v_store, PcMsgEntry *table,
                            hipStream_t st);

// n tokens (rows of k, v: [n, H_kv, D]) into the slots the items name
void pc_launch_append_tokens(int dtype, const PcTokenItem *items, int n, const void *k, const void *v, int n_kv_heads,
                             int D, int64_t slots, const double *inv_freq, void *k_store, void *v_store,
                             PcMsgEntry *table, hipStream_t st);

// the same for at most PC_TOKEN_PACK items, passed in the kernel's arguments (no staging copy)
void pc_launch_append_tokens_packed(int dtype, const PcTokenPack &pack, int n, const void *k, const void *v, int n_kv_heads,
                                    int D, int64_t slots, const double *inv_freq, void *k_store, void *v_store,
                                    PcMsgEntry *table, hipStream_t st);

// zero the rows of n_slots slots from slot_start on (both multiples of the tile) of the K or the V store, every KV head
void pc_launch_zero_span(int dtype, void *store, int64_t slots, int n_kv_heads, int D, int64_t slot_start, int64_t n_slots,
                           hipStream_t st);

// turn the stored keys of one message by delta positions, in place
void pc_launch_reposition(int dtype, int len, int n_kv_heads, int D, int64_t slot_start, int64_t slots, int delta,
                          int new_base, const double *inv_freq, void *k_store, PcMsgEntry *table, int msg_id,
                          hipStream_t st);

// the same for a staged list of messages, one launch (blockIdx.y = message)
void pc_launch_reposition_batch(int dtype, const PcMoveItem *items, int n_items, int n_kv_heads, int D, int64_t slots,
                                const double *inv_freq, void *k_store, PcMsgEntry *table, hipStream_t st);

// tok (may be empty): tokens the same launch appends to existing messages (a decode step: one launch for both)
struct PcTokenWork {
    const PcTokenItem *items = nullptr; int n = 0;
    const void *k = nullptr, *v = nullptr;        // [n, H_kv, D] rows in item order
    void *k_store = nullptr, *v_store = nullptr;
    int64_t slots = 0; int n_kv_heads = 0, D = 0, dtype = 0;
};
void pc_launch_build_plan(const PcCallDesc *calls, int n_calls, const int2 *sel, const int32_t *q_pos,
                          PcMsgEntry *table, const double *inv_freq, int half, int total_seg,
                          int total_q, PcSegment *segs, int32_t *seg_kvoff, float2 *rot_seg,
                          float2 *rot_q, float2 *rot_qw, PcTile *tiles, const PcTokenWork &tok, hipStream_t st);

void pc_launch_expand_tables(const PcSegment *segs, const int32_t *seg_kvoff, int n_seg, int64_t n_kv,
                             int32_t *kv_slot, int32_t *kv_pos, hipStream_t st);

// split_lanes: 1, or 4 for rows with many splits (their splits are shared out over four lanes)
void pc_launch_merge(int dtype, const PcMergeRow *merge_rows, int n_merge_rows, int split_lanes, const uint16_t *part_o,
                     const float *part_ml, void *out, float *lse, int n_q_heads, int D, hipStream_t st);

void pc_launch_attend_f32(const PcLaunch &L, const int32_t *row_call, int total_q, int D, hipStream_t st);

// gradient of the attention (dtype of q, d_out and the cache: 0 fp32, 1 bf16; gradients fp32); d_k collects the
// gradient w.r.t. the stored keys until the finalize pass
void pc_launch_attend_bwd(int dtype, const PcLaunch &L, const int32_t *row_call, int n_calls, int total_q, int total_seg,
                          int max_seg_len, int D, const float *lse, const void *d_out, float scale, float *delta,
                          float *d_q, float *d_k, float *d_v, hipStream_t st);
void pc_launch_grad_keys_finalize(const PcMsgEntry *msgs, int n_msgs, int n_kv_heads, int D, const double *inv_freq,
                                  float *d_k, hipStream_t st);

// keys (turned to the positions their call gives them) and values of the listed calls, token after token, into
// L.k_gather / L.v_gather
void pc_launch_gather(const PcLaunch &L, const PcGatherItem *items, int n_items, int64_t n_tiles, const int32_t *seg_kvoff,
                      hipStream_t st);

// bf16 MFMA kernels (D = 128)
void pc_launch_decode_bf16(const PcLaunch &L, int n_items, hipStream_t st);
void pc_launch_prefill_bf16(const PcLaunch &L, int n_items, bool packed, hipStream_t st);   // packed: the items of calls that gathered

// shared decode: rotation table of the listed (message, row) pairs, then the attention kernel
void pc_launch_shared_rot(const int32_t *pos, int64_t n_ent, const double *inv_freq, int half, float2 *rot, hipStream_t st);
void pc_launch_decode_shared_bf16(const PcLaunch &L, const PcShLaunch &S, int n_items, hipStream_t st);

#endif
