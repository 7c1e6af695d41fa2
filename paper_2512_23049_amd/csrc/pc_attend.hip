// Host side of the library: the attention entry points (forward, gradient, expanded tables).
#include "pc_host.h"

// ---------------------------------------------------------------------------------------------------------
// The library's fixed scratch memory: the per-call workspace (staged descriptors, the device-built plan, split
// partials) of pc_attend_static, for callers that must not allocate.  Every device the library runs on holds its
// own copy of the array, at its own address, until the process ends.  In host code the array's NAME is only a
// handle: the address kernels and copies can use comes from hipGetSymbolAddress, looked up once per device with
// that device current, and only that pointer is ever passed on.
// ---------------------------------------------------------------------------------------------------------
static __device__ __align__(256) unsigned char scratch[PC_STATIC_WS_BYTES];

int32_t pc_static_scratch(void **ptr, size_t *bytes)
{
    constexpr int MAX_DEV = 64;
    static void *per_device[MAX_DEV] = {nullptr};
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEV) return PC_ERR_HIP;
    if (!per_device[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return PC_ERR_HIP;
        per_device[dev] = p;
    }
    *ptr = per_device[dev];
    *bytes = PC_STATIC_WS_BYTES;
    return PC_OK;
}

// fixed_ws: nullptr = the cache's own workspace (grows on demand), else a buffer of fixed_cap bytes the call must fit into
static int32_t attend_impl(pc_cache *c, const pc_call *calls, int32_t n_calls, const void *q, void *out, float *lse,
                           hipStream_t st, void *fixed_ws, size_t fixed_cap, Planned *with_tokens = nullptr)
{
    Planned own;
    Planned &P = with_tokens ? *with_tokens : own;       // (a decode step hands in the tokens the plan builder's launch appends)
    P.fixed_ws = fixed_ws; P.fixed_cap = fixed_cap;
    const int32_t rc = pc_plan_and_stage(c, calls, n_calls, true, st, P);
    if (rc != PC_OK || c->host_only) return rc;

    char *w = (char *)P.ws;
    PcLaunch L{};
    L.calls = (const PcCallDesc *)(w + P.lay.calls);
    L.segs = (const PcSegment *)(w + P.lay.segs);
    L.rot_seg = (const float2 *)(w + P.lay.rot_seg);
    L.rot_q = (const float2 *)(w + P.lay.rot_q);
    L.rot_qw = (const float2 *)(w + P.lay.rot_qw);
    L.tiles = (const PcTile *)(w + P.lay.tiles);
    L.k_store = c->k_store; L.v_store = c->v_store; L.q = q; L.out = out; L.lse = lse;
    L.part_o = (uint16_t *)(w + P.lay.part_o); L.part_ml = (float *)(w + P.lay.part_ml);
    L.slots = c->slots; L.n_q_heads = c->cfg.n_q_heads; L.n_kv_heads = c->cfg.n_kv_heads;
    L.scale_log2 = c->scale * 1.4426950408889634f;
    L.k_gather = w + P.lay.k_gather; L.v_gather = w + P.lay.v_gather; L.kg_slots = P.kg_tiles * PC_TILE;
    L.kg_norm = (float *)(w + P.lay.kg_norm);
    const int32_t *row_call = (const int32_t *)(w + P.lay.row_call);
    if (c->cfg.dtype == PC_F32) {
        ProfScope ps(c, 5, st);
        pc_launch_attend_f32(L, row_call, P.total_q, c->D, st);
        PC_HIP(c, hipGetLastError());
        return PC_OK;
    }
    // A mixed batch (Sec. 2.4 "Parallel API Calls": prefill and decode calls in one batch): the one-row calls run on a
    // second stream beside the prefill calls' kernels, forked behind the plan builder and joined in front of the split
    // merge.  They start together with the gather pass (both stream from HBM) and end under the first prefill
    // workgroups; a prefill workgroup fills a compute unit, so the two kinds do not share units and the prefill takes
    // a unit over when its decode workgroup ends.  With kernel timing on, everything stays on the caller's stream: the
    // events around a kernel would otherwise time its neighbours as well.
    const bool has_pre = P.n_pre > 0 || P.n_pre_pk > 0, has_dec = P.n_dec > 0 || P.n_sh_items > 0;
    const bool fork = has_pre && has_dec && !c->prof && c->side;
    hipStream_t st_dec = st;
    if (fork) {
        PC_HIP(c, hipEventRecord(c->ev_fork, st));
        PC_HIP(c, hipStreamWaitEvent(c->side, c->ev_fork, 0));
        st_dec = c->side;
    }
    if (P.n_dec > 0) {
        ProfScope ps(c, 3, st_dec);
        L.items = (const PcItem *)(w + P.lay.items_dec);
        pc_launch_decode_bf16(L, P.n_dec, st_dec);
        PC_HIP(c, hipGetLastError());
    }
    if (P.n_sh_items > 0) {
        ProfScope ps(c, 3, st_dec);
        PcShLaunch S{};
        S.groups = (const PcShGroup *)(w + P.lay.sh_groups);
        S.segs = (const PcShSeg *)(w + P.lay.sh_segs);
        S.items = (const PcShItem *)(w + P.lay.sh_items);
        S.rot = (const float2 *)(w + P.lay.sh_rot);
        pc_launch_decode_shared_bf16(L, S, P.n_sh_items, st_dec);
        PC_HIP(c, hipGetLastError());
    }
    if (fork) PC_HIP(c, hipEventRecord(c->ev_join, c->side));
    if (P.n_kg_items > 0) {
        ProfScope ps(c, 8, st);
        pc_launch_gather(L, (const PcGatherItem *)(w + P.lay.kg_items), P.n_kg_items, P.kg_tiles, (const int32_t *)(w + P.lay.seg_kvoff), st);
        PC_HIP(c, hipGetLastError());
    }
    if (P.n_pre_pk > 0) {
        ProfScope ps(c, 2, st);
        L.items = (const PcItem *)(w + P.lay.items_pk);
        pc_launch_prefill_bf16(L, P.n_pre_pk, true, st);
        PC_HIP(c, hipGetLastError());
    }
    if (P.n_pre > 0) {
        ProfScope ps(c, 2, st);
        L.items = (const PcItem *)(w + P.lay.items_pre);
        pc_launch_prefill_bf16(L, P.n_pre, false, st);
        PC_HIP(c, hipGetLastError());
    }
    if (fork) PC_HIP(c, hipStreamWaitEvent(st, c->ev_join, 0));
    if (P.n_merge_rows > 0) {
        ProfScope ps(c, 4, st);
        const PcMergeRow *rows = (const PcMergeRow *)(w + P.lay.merge_rows);
        pc_launch_merge(c->cfg.dtype, rows, P.n_merge_few, 1, L.part_o, L.part_ml, out, lse, c->cfg.n_q_heads, c->D, st);
        pc_launch_merge(c->cfg.dtype, rows + P.n_merge_few, P.n_merge_rows - P.n_merge_few, 4, L.part_o, L.part_ml, out, lse,
                        c->cfg.n_q_heads, c->D, st);
        PC_HIP(c, hipGetLastError());
    }
    return PC_OK;
}

extern "C" {

int32_t pc_attend(pc_cache *c, const pc_call *calls, int32_t n_calls, const void *q, void *out, float *lse, void *stream)
{
    if (!c) return PC_ERR_INVALID_ARG;
    if (n_calls < 0 || (n_calls > 0 && !calls)) return pc_fail(c, PC_ERR_INVALID_ARG, "attend: bad call list");
    if (n_calls == 0) return PC_OK;
    if (!c->host_only && (!q || !out)) return pc_fail(c, PC_ERR_INVALID_ARG, "attend: null q or out");
    return attend_impl(c, calls, n_calls, q, out, lse, (hipStream_t)stream, nullptr, 0);
}

int32_t pc_decode_step(pc_cache *c, const int32_t *msg_ids, int32_t n_msgs, const void *k, const void *v,
                       const pc_call *calls, int32_t n_calls, const void *q, void *out, float *lse, void *stream)
{
    if (!c) return PC_ERR_INVALID_ARG;
    if (n_calls < 0 || (n_calls > 0 && !calls)) return pc_fail(c, PC_ERR_INVALID_ARG, "decode_step: bad call list");
    if (!c->host_only && n_calls > 0 && (!q || !out)) return pc_fail(c, PC_ERR_INVALID_ARG, "decode_step: null q or out");
    int32_t rc = pc_check_token_batch(c, msg_ids, n_msgs, k, v);
    if (rc != PC_OK) return rc;
    hipStream_t st = (hipStream_t)stream;
    const std::vector<int32_t> ids(msg_ids, msg_ids + std::max(n_msgs, 0));
    // The tokens can be written by the plan builder's own launch (one launch and one staging copy for the whole step) when
    // nothing the plan builder reads from the device table changes under it: the new message's length travels with the
    // call (host side), so what remains is a grown message that some call lists as a PARENT (its length is read from the
    // table) and a message that needs a further extent (a new table row).  Then the append gets a launch of its own.
    bool fuse = !c->host_only && n_msgs > 0 && n_calls > 0;
    if (fuse) {
        std::vector<char> grows(c->msgs.size(), 0);
        for (int32_t m : ids) grows[(size_t)m] = 1;
        for (int i = 0; i < n_calls && fuse; ++i)
            for (int e = 0; e < calls[i].n_sel && calls[i].sel && fuse; ++e) {
                const int32_t m = calls[i].sel[e].msg_id;
                if (m >= 0 && m < (int32_t)grows.size() && grows[(size_t)m]) fuse = false;
            }
    }
    Planned P;
    if (n_msgs > 0) {
        rc = pc_append_token_items(c, ids, k, v, st, fuse ? &P.tok_items : nullptr);
        if (rc != PC_OK) return rc;
        P.tok_k = k; P.tok_v = v;
    }
    auto append_alone = [&]() -> int32_t {               // the tokens are in the host's books: they must reach the cache
        if (P.tok_items.empty() || P.tok_done) return PC_OK;
        const int32_t r2 = pc_stage_items(c, P.tok_items.data(), sizeof(PcTokenItem) * P.tok_items.size(), st);
        if (r2 != PC_OK) return r2;
        pc_launch_append_tokens(c->cfg.dtype, (const PcTokenItem *)c->tok_dev, (int)P.tok_items.size(), k, v, c->cfg.n_kv_heads, c->D,
                                c->slots, c->inv_freq_dev, c->k_store, c->v_store, c->table_dev, st);
        PC_HIP(c, hipGetLastError());
        P.tok_done = true;
        return PC_OK;
    };
    if (n_calls == 0) return append_alone();
    rc = attend_impl(c, calls, n_calls, q, out, lse, st, nullptr, 0, &P);
    if (rc != PC_OK) {                                   // a refused call list: the tokens stay appended, as with the two separate calls
        const std::string why = c->err;
        const int32_t r2 = append_alone();
        c->err = why;
        return r2 != PC_OK && rc == PC_OK ? r2 : rc;
    }
    return PC_OK;
}

int32_t pc_attend_static(pc_cache *c, const pc_call *calls, int32_t n_calls, const void *q, void *out, float *lse, void *stream)
{
    if (!c) return PC_ERR_INVALID_ARG;
    if (n_calls < 0 || (n_calls > 0 && !calls)) return pc_fail(c, PC_ERR_INVALID_ARG, "attend_static: bad call list");
    if (n_calls == 0) return PC_OK;
    if (c->host_only) return attend_impl(c, calls, n_calls, q, out, lse, nullptr, nullptr, 0);
    if (!q || !out) return pc_fail(c, PC_ERR_INVALID_ARG, "attend_static: null q or out");
    if (!c->static_ws) return pc_fail(c, PC_ERR_HIP, "attend_static: the fixed scratch array was not found on this device");
    const bool prof = c->prof;                           // kernel timing takes events from a pool that may have to grow
    c->prof = false;
    const int32_t rc = attend_impl(c, calls, n_calls, q, out, lse, (hipStream_t)stream, c->static_ws, PC_STATIC_WS_BYTES);
    c->prof = prof;
    return rc;
}

int32_t pc_attend_backward(pc_cache *c, const pc_call *calls, int32_t n_calls, const void *q, const float *lse,
                           const void *d_out, float *d_q, float *d_k, float *d_v, void *stream)
{
    if (!c) return PC_ERR_INVALID_ARG;
    if (n_calls < 0 || (n_calls > 0 && !calls)) return pc_fail(c, PC_ERR_INVALID_ARG, "attend_backward: bad call list");
    if (n_calls == 0) return PC_OK;
    if (!c->host_only && (!q || !lse || !d_out || !d_q || !d_k || !d_v))
        return pc_fail(c, PC_ERR_INVALID_ARG, "attend_backward: null argument");
    hipStream_t st = (hipStream_t)stream;
    Planned P;
    const int32_t rc = pc_plan_and_stage(c, calls, n_calls, false, st, P);
    if (rc != PC_OK || c->host_only) return rc;
    char *w = (char *)P.ws;
    PcLaunch L{};
    L.calls = (const PcCallDesc *)(w + P.lay.calls);
    L.segs = (const PcSegment *)(w + P.lay.segs);
    L.rot_seg = (const float2 *)(w + P.lay.rot_seg);
    L.rot_q = (const float2 *)(w + P.lay.rot_q);
    L.rot_qw = (const float2 *)(w + P.lay.rot_qw);
    L.k_store = c->k_store; L.v_store = c->v_store; L.q = q;
    L.slots = c->slots; L.n_q_heads = c->cfg.n_q_heads; L.n_kv_heads = c->cfg.n_kv_heads;
    L.scale_log2 = c->scale * 1.4426950408889634f;
    ProfScope ps(c, 5, st);
    int max_seg_len = 0;
    for (const Resolved &r : P.res) {
        for (const int2 &e : r.sel) max_seg_len = std::max(max_seg_len, c->msgs[(size_t)e.x].len);
        max_seg_len = std::max(max_seg_len, r.self_len);
    }
    if ((max_seg_len + 15) / 16 > 65535) return pc_fail(c, PC_ERR_SHAPE, "attend_backward: a message of %d tokens is too long", max_seg_len);
    L.calls = (const PcCallDesc *)(w + P.lay.calls);
    pc_launch_attend_bwd(c->cfg.dtype, L, (const int32_t *)(w + P.lay.row_call), n_calls, P.total_q, P.total_seg, max_seg_len, c->D,
                         lse, d_out, c->scale, (float *)(w + P.lay.row_scalar), d_q, d_k, d_v, st);
    PC_HIP(c, hipGetLastError());
    return PC_OK;
}

int32_t pc_grad_keys_finalize(pc_cache *c, float *d_k, void *stream)
{
    if (!c) return PC_ERR_INVALID_ARG;
    if (c->host_only) return PC_OK;
    if (!d_k) return pc_fail(c, PC_ERR_INVALID_ARG, "grad_keys_finalize: null d_k");
    std::vector<PcMsgEntry> live;
    for (const HostMsg &m : c->msgs)
        if (m.live && m.len > 0) live.push_back(PcMsgEntry{(int32_t)m.slot_start, m.len, m.base_pos, 0});
    if (live.empty()) return PC_OK;
    hipStream_t st = (hipStream_t)stream;
    const int32_t rc = pc_stage_items(c, live.data(), sizeof(PcMsgEntry) * live.size(), st);
    if (rc != PC_OK) return rc;
    ProfScope ps(c, 5, st);
    pc_launch_grad_keys_finalize((const PcMsgEntry *)c->tok_dev, (int)live.size(), c->cfg.n_kv_heads, c->D, c->inv_freq_dev, d_k, st);
    PC_HIP(c, hipGetLastError());
    return PC_OK;
}

int32_t pc_build_tables(pc_cache *c, const pc_call *call, int32_t *kv_slot, int32_t *kv_pos, int64_t cap,
                        int64_t *n_kv, void *stream)
{
    if (!c) return PC_ERR_INVALID_ARG;
    hipStream_t st = (hipStream_t)stream;
    Planned P;
    const int32_t rc = pc_plan_and_stage(c, call, 1, false, st, P);
    if (rc != PC_OK) return rc;
    const int64_t n = P.res[0].n_kv;
    if (n_kv) *n_kv = n;
    if (c->host_only || cap < n || n == 0) return PC_OK;
    if (!kv_slot || !kv_pos) return pc_fail(c, PC_ERR_INVALID_ARG, "build_tables: null output with cap > 0");
    ProfScope ps(c, 6, st);
    char *w = (char *)P.ws;
    pc_launch_expand_tables((const PcSegment *)(w + P.lay.segs), (const int32_t *)(w + P.lay.seg_kvoff), P.total_seg, n,
                            kv_slot, kv_pos, st);
    PC_HIP(c, hipGetLastError());
    return PC_OK;
}

}  // extern "C"
