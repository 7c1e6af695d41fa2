/*
 * pc.h - C ABI of the choreographed-attention library for AMD MI355X (gfx950).
 *
 * The library implements the attention step of Prompt Choreography
 * (arXiv 2512.23049): a dynamic, global, append-only KV cache of messages, and
 * attention calls whose query tokens attend over an arbitrary, reordered subset
 * of cached messages, each placed at a caller-chosen start position (gaps and
 * overlaps allowed), with many parallel calls batched (Sec. 2.1 "Core Idea",
 * Sec. 2.3 "A Prompt Choreography API", Sec. 2.4 "Managing the KV Cache").
 *
 * The unit of this interface is tensors, not text: the caller (an LLM layer)
 * supplies K/V of a new message and the query rows; tokenisation, sampling and
 * the rest of the model are outside.
 *
 * Conventions
 *  - Every function returns an int32 status: PC_OK (0) or a negative PC_ERR_*.
 *    pc_last_error() returns a NUL-terminated description owned by the cache
 *    (valid until the next failing call on that cache).  Nothing throws.
 *  - Pointers named k, v, q, out, lse, kv_slot, kv_pos are DEVICE pointers owned
 *    by the caller.  All other pointers are HOST pointers; list arguments are
 *    copied before the function returns, so the caller may free them at once.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).  All
 *    device work is enqueued on it and is stream-ordered; no function waits for
 *    the device, except that a workspace may be (re)allocated on first use of a
 *    larger batch shape.  Calls on one cache must come from one thread at a time
 *    and on one stream (or on streams the caller orders with events).
 *  - Errors that the host can detect (unknown id, capacity, bad shapes, positions
 *    out of range) are returned BEFORE anything is enqueued.
 *  - Message ids are 0, 1, 2, ... in append order (Sec. 2.4: ids map to
 *    contiguous physical spans of the cache).
 */
#ifndef PC_H_
#define PC_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define PC_OK               0
#define PC_ERR_INVALID_ARG (-1)
#define PC_ERR_BAD_MSG_ID  (-2)
#define PC_ERR_NO_SPACE    (-3)
#define PC_ERR_SHAPE       (-4)
#define PC_ERR_HIP         (-5)

#define PC_F32  0
#define PC_BF16 1

/* An omitted offset (Sec. 2.3, the rule for offsets that are left out): the position
 * right after the end of the preceding list entry.  For the first entry it means 0; for
 * the new message it means right after the last list entry (0 if the list is empty). */
#define PC_POS_AUTO INT32_MIN

/* Every message starts at a slot that is a multiple of this (cache layout rule:
 * message i starts at the first such slot at or after the end of message i-1's
 * reserved span; message 0 starts at slot 0). */
#define PC_SLOT_ALIGN 32

/* pc_config.flags */
#define PC_FLAG_HOST_ONLY 1u  /* no device memory, no launches: validation, allocation
                                 and position resolution only (k/v/q/out are ignored) */
#define PC_FLAG_GROW_EXTENTS 2u /* a message whose reserve is used up grows into a further extent
                                 (Sec. 2.4: the message table maps an id to where its tokens
                                 live; here to one or more spans) instead of PC_ERR_NO_SPACE:
                                 pc_append_tokens* then takes slots for it by the allocation
                                 rule, room for the tokens the call still brings and at least
                                 the message's first reserve and PC_SLOT_ALIGN tokens.  Every
                                 extent uses one row of the
                                 message table (max_messages bounds messages plus further
                                 extents), so message ids stay ascending but need not be
                                 consecutive.  To every call the message is one sequence of
                                 tokens; the query rows of a call must lie in the last extent
                                 of its new message (PC_ERR_SHAPE otherwise). */

typedef struct pc_cache pc_cache;

typedef struct {
    int32_t  n_q_heads;        /* H_q  (multiple of n_kv_heads; PC_BF16: at most 16 per KV head) */
    int32_t  n_kv_heads;       /* H_kv                                                  */
    int32_t  head_dim;         /* D: 64 or 128 (PC_BF16: 128); other shapes: PC_ERR_SHAPE */
    int32_t  dtype;            /* PC_F32 | PC_BF16: type of k, v, q, out and of storage */
    float    rope_theta;       /* RoPE base, e.g. 1e4 or 5e5                            */
    float    softmax_scale;    /* 0 -> 1/sqrt(D)                                        */
    int64_t  capacity_tokens;  /* slots in the cache (rounded up to PC_SLOT_ALIGN)      */
    int32_t  max_messages;
    int32_t  max_position;     /* every token / query position p obeys |p| <= this      */
    uint32_t flags;
    void    *arena;            /* optional caller-owned DEVICE memory for K/V storage,  */
    size_t   arena_bytes;      /*   >= pc_cache_storage_bytes(cfg); NULL -> hipMalloc   */
} pc_config;

/* Bytes of device memory the K/V storage needs for this configuration. */
size_t  pc_cache_storage_bytes(const pc_config *cfg);

/* Create / destroy the global cache (Sec. 2.4: pre-allocated, append-only store of
 * K and V for every cached token plus the message -> span map).  One attention
 * layer per cache object. */
int32_t pc_cache_create(const pc_config *cfg, pc_cache **out);
int32_t pc_cache_destroy(pc_cache *c);
const char *pc_last_error(const pc_cache *c);

/* Append one message (Sec. 2.3: prefill/decode "append a newly encoded message to
 * the global KV cache and return a unique new identifier"; Sec. 2.4: new messages go
 * at the end of the occupied part of the cache).
 *   k, v     device, [len, n_kv_heads, head_dim] contiguous, cache dtype, 16-byte aligned
 *            (PC_ERR_INVALID_ARG otherwise); k is the UNROTATED key (no positional rotation
 *            applied by the caller).
 *   reserve  slots to reserve for the message (0 or < len means len).
 *   msg_id   receives the new id.
 * The fused append kernel stores K turned to its in-message index (delta-rotated
 * form) and V in the tile layout the attention kernels read. */
int32_t pc_append_message(pc_cache *c, const void *k, const void *v, int32_t len,
                          int32_t reserve, int32_t *msg_id, void *stream);

/* The same for n messages in one launch (Sec. 2.4 "Parallel API Calls": the new messages
 * of parallel calls).  k, v: host arrays of n device pointers; lens, reserves (may be NULL:
 * no extra room), msg_ids: host arrays of n entries; all copied / filled before return.
 * Ids are consecutive in list order.  All or nothing: on any error (a length < 1, a null
 * pointer, no room for one of them) nothing is appended. */
int32_t pc_append_messages(pc_cache *c, int32_t n, const void *const *k, const void *const *v,
                           const int32_t *lens, const int32_t *reserves, int32_t *msg_ids,
                           void *stream);

/* Growth of existing messages within the room reserved at pc_append_message
 * (Sec. 2.4: decode tails grow token by token; parallel calls grow theirs in step).
 * pc_append_tokens: n more tokens for one message, k, v device [n, n_kv_heads, head_dim].
 * pc_append_tokens_batch: one more token for each of n_msgs distinct messages in one
 * launch; msg_ids host (copied before return), row j of k, v ([n_msgs, n_kv_heads,
 * head_dim]) goes to message msg_ids[j].
 * Keys are turned to base + in-message index like those of pc_append_message.  Stream
 * ordered: a later pc_attend on the same stream sees the longer messages.
 * Errors (nothing enqueued): unknown id, an id listed twice in a batch, n < 1, more
 * tokens than the reserve has room for (PC_ERR_NO_SPACE; with PC_FLAG_GROW_EXTENTS the
 * message takes a further extent instead, and PC_ERR_NO_SPACE means the cache or the
 * message table has no room for it). */
int32_t pc_append_tokens(pc_cache *c, int32_t msg_id, const void *k, const void *v, int32_t n,
                         void *stream);
int32_t pc_append_tokens_batch(pc_cache *c, const int32_t *msg_ids, int32_t n_msgs, const void *k,
                               const void *v, void *stream);

/* One parent of a call: message id and the position of its first token
 * (Sec. 2.3 `parents` and `offsets`). */
typedef struct { int32_t msg_id; int32_t start_pos; } pc_sel;

/* One attention call (Sec. 2.3 prefill/decode; Sec. 2.4 "Dynamic Masking": the new
 * message's tokens see all tokens of `sel` and the earlier tokens of their own
 * message; nothing else).
 *   sel/n_sel   parents in list order; repeats allowed; any order of positions.
 *   self_msg    id of the (already appended) new message, or -1 for none.
 *   self_start  position of its first token (Sec. 2.3 `new_offset`) or PC_POS_AUTO.
 *   n_q         number of query rows, >= 1; row r is the (len(self) - n_q + r)-th
 *               token of the new message and sees own tokens up to and including
 *               itself (prefill: n_q = len; decode: n_q = 1).  With self_msg = -1
 *               the rows see the parents only.
 *   q_pos       host, n_q positions of the query rows, or NULL for
 *               self_start + token index. */
typedef struct {
    const pc_sel  *sel;
    int32_t        n_sel;
    int32_t        self_msg;
    int32_t        self_start;
    int32_t        n_q;
    const int32_t *q_pos;
} pc_call;

/* Batched choreographed attention (Sec. 2.4 "Parallel API Calls": a list of calls
 * that each see exactly what they list).
 *   q    device, [sum n_q, n_q_heads, head_dim], rows packed in call order, unrotated.
 *   out  device, same shape and dtype as q.
 *   lse  device, optional fp32 [sum n_q, n_q_heads]: natural-log sum of exp(scores).
 * A row with nothing visible yields zeros and -inf. */
int32_t pc_attend(pc_cache *c, const pc_call *calls, int32_t n_calls,
                  const void *q, void *out, float *lse, void *stream);

/* One decode step of parallel calls in one call (Sec. 2.4 "Parallel API Calls" and the interleaved decoding of
 * parallel calls): pc_append_tokens_batch(msg_ids, n_msgs, k, v) followed by pc_attend(calls, ...), with the same
 * arguments, results and errors as the two.  What the fused form saves: the tokens are written by the plan builder's
 * own launch and their item list rides in the same staging copy as the call list (one launch and one copy fewer per
 * step).  The append keeps a launch of its own when a grown message is listed as a PARENT by one of the calls or
 * needs a further extent.  If the append is refused nothing is enqueued; if the call list is refused the tokens
 * stay appended, as with the two separate calls. */
int32_t pc_decode_step(pc_cache *c, const int32_t *msg_ids, int32_t n_msgs, const void *k, const void *v,
                       const pc_call *calls, int32_t n_calls, const void *q, void *out, float *lse, void *stream);

/* pc_attend for callers that cannot allocate device memory: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments, same kernels, same results (bit for bit) as pc_attend; the
 * per-call workspace (staged descriptors, the device-built plan, split partials) lives in a fixed array of
 * PC_STATIC_WS_BYTES (32 MiB) that the library holds on every GPU it runs on until the process ends, and the
 * function calls no hipMalloc, hipFree or other allocating routine.  A batch whose workspace exceeds that size, or
 * whose staged descriptors exceed one slot of the cache's pinned staging ring (1 MiB), is rejected with
 * PC_ERR_NO_SPACE before anything is enqueued (pc_last_error names both sizes).  Kernel timing (pc_profile_enable)
 * does not cover it.  Every cache on a GPU shares that GPU's array, which keeps the last call's contents (nothing
 * in it has to start at zero: every call writes what it reads): calls on one GPU that overlap in time - two
 * streams, or two caches - race; order them on one stream or with events. */
#define PC_STATIC_WS_BYTES ((size_t)32 << 20)
int32_t pc_attend_static(pc_cache *c, const pc_call *calls, int32_t n_calls,
                         const void *q, void *out, float *lse, void *stream);

/* In-place position update of a cached message (Sec. 2.4 "Position Updates": the
 * paper's mechanism, a rotation of the cached keys through a table of the D/2
 * rotations for the move).  The stored key of token t, so far turned to position
 * base + t (base = 0 after pc_append_message), is turned to new_base + t; one read
 * and one write of the message's K, V untouched, stream-ordered.
 * What pc_attend computes does not change (a call may still place the message
 * anywhere: the difference start_pos - base is applied to the queries), except for
 * one more rounding of the keys to the cache dtype per move.  What changes is the
 * cost: consecutive parents of a call whose start_pos - base agree (all zero when
 * every parent sits where it was last repositioned to) share one turn of the queries.
 * Errors: unknown id, |new_base| > max_position.  new_base equal to the current base
 * launches nothing. */
int32_t pc_reposition(pc_cache *c, int32_t msg_id, int32_t new_base, void *stream);
/* The same for n_msgs distinct messages in one launch (msg_ids, new_bases: host lists,
 * copied before return).  Nothing is enqueued if any entry is in error (also: an id
 * listed twice). */
int32_t pc_reposition_batch(pc_cache *c, const int32_t *msg_ids, const int32_t *new_bases,
                            int32_t n_msgs, void *stream);

/* Parity/debug: the expanded gather table and position map of one call, in list
 * order then the new message: kv_slot[i] = physical slot, kv_pos[i] = logical
 * position (the (m, j) metadata of Sec. 2.4 in gathered form).  kv_slot and kv_pos
 * are device int32 arrays of `cap` entries each.  The function writes the number of
 * gathered tokens to *n_kv and fills the arrays only if cap >= that number (pass
 * cap = 0 and NULL arrays to query the count). */
int32_t pc_build_tables(pc_cache *c, const pc_call *call, int32_t *kv_slot, int32_t *kv_pos,
                        int64_t cap, int64_t *n_kv, void *stream);

/* Host-side resolution of a call: starts_out[n_sel] receives each parent's resolved
 * start position, *self_start_out the new message's, *n_kv the gathered token count.
 * Any output pointer may be NULL. */
int32_t pc_resolve_call(pc_cache *c, const pc_call *call, int32_t *starts_out,
                        int32_t *self_start_out, int64_t *n_kv);

/* Gives a message's reserved slots back (Sec. 2.4: the cache is a map from message id to
 * physical span; a message no call will select again can make room).  Host bookkeeping
 * only, nothing is enqueued: work already enqueued that reads the message is not
 * disturbed by a later pc_append_message on the same stream that reuses the slots, but the
 * caller must not reuse them from another stream before that work has finished.
 * The id becomes unknown to every function (PC_ERR_BAD_MSG_ID) and is never given out
 * again: ids keep counting up, and max_messages bounds the appends of a cache's lifetime.
 * Allocation rule after frees: pc_append_message takes the first freed span (lowest slot)
 * that holds the reserve rounded up to PC_SLOT_ALIGN, else the end of the used region;
 * adjacent freed spans merge; a span freed at the end shrinks the used region. */
int32_t pc_message_free(pc_cache *c, int32_t msg_id);

/* Swap (Sec. 2.2 "Simplifying Assumptions", the note on caches that do not fit GPU memory, and
 * the note to Sec. 2.4's append-only cache: messages may be moved out to CPU memory for a while).
 * pc_message_swap_out copies the stored K and V of a live message (its whole reserved span, as
 * stored: keys turned to their stored base) into `blob`, then gives the slots back exactly as
 * pc_message_free does.  `blob`: caller-owned, pc_message_swap_bytes(msg) bytes, pinned host or
 * device memory (any memory hipMemcpyDefault can write); the copy is enqueued on `stream`, so
 * appends that reuse the slots must go to the same stream or wait for it, and the blob is complete
 * once the stream has passed this point.  Until it is swapped in again the id is unknown to every
 * other function (PC_ERR_BAD_MSG_ID), but it is kept: pc_message_swap_in(msg, blob) takes slots by
 * the allocation rule above (PC_ERR_NO_SPACE if there is no room; nothing changed then), copies the
 * blob back on `stream` and the message is what it was: same id, length, reserve and stored base,
 * bit-identical K and V, possibly at other slots.  The blob's layout is private to the library
 * and tied to the cache's configuration.  pc_message_swap_bytes returns the blob size for a live
 * or swapped-out message, or a negative error code. */
int64_t pc_message_swap_bytes(pc_cache *c, int32_t msg_id);
int32_t pc_message_swap_out(pc_cache *c, int32_t msg_id, void *blob, void *stream);
int32_t pc_message_swap_in(pc_cache *c, int32_t msg_id, const void *blob, void *stream);

/* Message and cache bookkeeping (Sec. 2.4: count of cached tokens, id -> span). */
int32_t pc_message_info(pc_cache *c, int32_t msg_id, int32_t *len, int64_t *slot_start,
                        int32_t *reserved);
/* The extents of a message in token order: *n_extents (always written), and for the first
 * min(cap, *n_extents) of them the first slot and the tokens held.  pc_message_info reports
 * the first extent's slot_start and the totals over all extents. */
int32_t pc_message_extents(pc_cache *c, int32_t msg_id, int32_t *n_extents, int64_t *slot_starts,
                           int32_t *lens, int32_t cap);
/* *base_pos: the position the message's stored keys are currently turned to (see
 * pc_reposition). */
int32_t pc_message_base(pc_cache *c, int32_t msg_id, int32_t *base_pos);
int32_t pc_cache_info(pc_cache *c, int32_t *n_messages, int64_t *slots_used,
                      int64_t *capacity_slots);

/* Kernel timing for benchmarks.  When enabled, every kernel the library launches is
 * bracketed by events on the caller's stream.  pc_profile_read waits for the stream
 * work recorded so far, then returns per-kernel-class totals since the last reset.
 * Classes: 0 append, 1 plan builder, 2 prefill attention, 3 decode attention,
 * 4 split merge, 5 fp32 attention, 6 table expansion, 7 reposition, 8 key gather. */
#define PC_N_KERNEL_CLASSES 9
int32_t pc_profile_enable(pc_cache *c, int32_t on);
int32_t pc_profile_read(pc_cache *c, double ms_total[PC_N_KERNEL_CLASSES],
                        int64_t launches[PC_N_KERNEL_CLASSES], int32_t reset);

/* Tuning knobs (0 keeps the default): KV tiles (of 32 keys) per split for decode
 * and for prefill work items. */
int32_t pc_set_tuning(pc_cache *c, int32_t decode_tiles_per_split, int32_t prefill_tiles_per_split);

/* Gather pass (Sec. 2.4 "Position Updates", applied to a copy).  A prefill call with many query rows can have the
 * keys and values it lists copied once into the call's workspace: tokens in list order without gaps between
 * messages, every key turned to the position the call gives it.  The attention kernel then reads plain tiles of the
 * copy and turns the queries by their own position only, instead of once more per listed message.  The cache itself
 * is not changed; results are the same up to one more rounding of the copied keys to bf16.  mode 0 (default): calls
 * with rows x query heads >= 32768 (below that the copy costs more than it saves); 1: never; 2: every prefill call.
 * PC_BF16 caches only; pc_attend_static never gathers (the copy may not fit its fixed workspace). */
int32_t pc_set_key_gather(pc_cache *c, int32_t mode);

/* Gradient of pc_attend for fine-tuning (Sec. 2.4: while fine-tuning, a position update is
 * applied to the keys without destroying them, so that gradients flow back through it to the
 * cached keys).  For the scalar sum(out * d_out) of a pc_attend with the same cache state,
 * calls and q (q and d_out in the cache dtype, like out; gradients are fp32 for both dtypes):
 *   d_q   [sum n_q][n_q_heads][head_dim] fp32, device: written, the gradient w.r.t. q;
 *   d_k, d_v [capacity slots][n_kv_heads][head_dim] fp32, device, indexed by physical slot
 *         (a message's rows start at its slot_start, see pc_message_info / pc_message_extents):
 *         ADDED to, so that the gradients of several calls and batches collect in one buffer
 *         the caller zeroed.
 * lse: the [sum n_q][n_q_heads] fp32 log-sum-exp pc_attend wrote for these calls.
 * d_v is the gradient w.r.t. the appended V.  d_k collects the gradient w.r.t. the keys AS
 * STORED (turned to their stored base; in a PC_BF16 cache also rounded once more); once every
 * backward call has been enqueued, pc_grad_keys_finalize(d_k) turns the rows of every live
 * message into the gradient w.r.t. the K that was appended.  No message may be repositioned,
 * freed or swapped between the first backward call into a buffer and its finalize.  A
 * functional path (plain fp32 vector kernels, no matrix cores): not tuned. */
int32_t pc_attend_backward(pc_cache *c, const pc_call *calls, int32_t n_calls, const void *q, const float *lse,
                           const void *d_out, float *d_q, float *d_k, float *d_v, void *stream);
int32_t pc_grad_keys_finalize(pc_cache *c, float *d_k, void *stream);

/* Shared decode (Sec. 2.4 "Parallel decoding": parallel calls read the same cached
 * messages).  Consecutive one-row calls of a pc_attend batch (up to 32 * 8 / g of them, g =
 * query heads per KV head, for g in {1, 2, 4, 8}) can be served as a group that reads the
 * union of their messages once per KV head instead of once per call; results are the same
 * up to rounding.  mode 0 (default): a group takes the shared walk when its calls together
 * list at least six times the tokens of the union; 1: never; 2: always when the shape
 * allows it.  Applies to PC_BF16 caches; other calls are unaffected. */
int32_t pc_set_decode_sharing(pc_cache *c, int32_t mode);

#ifdef __cplusplus
}
#endif
#endif /* PC_H_ */
