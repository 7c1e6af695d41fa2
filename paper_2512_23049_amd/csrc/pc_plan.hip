// Host side of the library: a call's validation and position resolution, the split of a batch into
// work items (prefill, per-call decode, shared decode), staging, and the launch of the plan builder.
#include "pc_host.h"

int32_t pc_resolve(pc_cache *c, const pc_call *call, int idx, Resolved &out)
{
    if (!call) return pc_fail(c, PC_ERR_INVALID_ARG, "call %d: null", idx);
    if (call->n_sel < 0 || (call->n_sel > 0 && !call->sel))
        return pc_fail(c, PC_ERR_INVALID_ARG, "call %d: bad parent list", idx);
    if (call->n_q < 1) return pc_fail(c, PC_ERR_INVALID_ARG, "call %d: n_q = %d must be >= 1", idx, call->n_q);
    const int64_t maxp = c->cfg.max_position;
    // a listed message becomes one (extent record, start) pair per extent that holds tokens
    out.sel.clear();
    out.sel.reserve((size_t)call->n_sel);
    out.entry_start.resize((size_t)call->n_sel);
    int64_t nxt = 0, n_kv = 0, tiles = 0;
    for (int e = 0; e < call->n_sel; ++e) {
        const int32_t m = call->sel[e].msg_id;
        if (!known(c, m)) return pc_fail(c, PC_ERR_BAD_MSG_ID, "call %d: parent %d names unknown message %d", idx, e, m);
        const int64_t len = chain_len(c, m);
        const int64_t s = call->sel[e].start_pos == PC_POS_AUTO ? nxt : (int64_t)call->sel[e].start_pos;
        if (s < -maxp || s + len - 1 > maxp)
            return pc_fail(c, PC_ERR_INVALID_ARG, "call %d: parent %d spans positions [%lld, %lld], limit is +-%lld", idx, e,
                        (long long)s, (long long)(s + len - 1), (long long)maxp);
        out.entry_start[(size_t)e] = (int32_t)s;
        int64_t at = s;
        for (int32_t r = m; r >= 0; r = c->msgs[(size_t)r].next) {
            const int32_t rl = c->msgs[(size_t)r].len;
            if (rl > 0 || r == m) out.sel.push_back(make_int2(r, (int)at));
            at += rl; tiles += (rl + PC_TILE - 1) / PC_TILE;
        }
        nxt = s + len; n_kv += len;
    }
    out.self_msg = -1; out.self_len = 0;
    int64_t s_self = call->self_start == PC_POS_AUTO ? nxt : (int64_t)call->self_start;
    int64_t self_total = 0;
    if (call->self_msg >= 0) {
        if (!known(c, call->self_msg)) return pc_fail(c, PC_ERR_BAD_MSG_ID, "call %d: new message id %d unknown", idx, call->self_msg);
        self_total = chain_len(c, call->self_msg);
        if (call->n_q > self_total)
            return pc_fail(c, PC_ERR_SHAPE, "call %d: n_q = %d exceeds the new message's %lld tokens", idx, call->n_q, (long long)self_total);
        if (s_self < -maxp || s_self + self_total - 1 > maxp)
            return pc_fail(c, PC_ERR_INVALID_ARG, "call %d: new message spans positions beyond +-%lld", idx, (long long)maxp);
        // The causal part lives in the message's last extent; the extents before it are seen whole by
        // every query row, like parents.
        const int32_t last = chain_last(c, call->self_msg);
        if (call->n_q > c->msgs[(size_t)last].len)
            return pc_fail(c, PC_ERR_SHAPE, "call %d: the %d query rows must lie in the new message's last extent (%d tokens)", idx,
                        call->n_q, c->msgs[(size_t)last].len);
        int64_t at = s_self;
        for (int32_t r = call->self_msg; r != last; r = c->msgs[(size_t)r].next) {
            const int32_t rl = c->msgs[(size_t)r].len;
            if (rl > 0) out.sel.push_back(make_int2(r, (int)at));
            at += rl; tiles += (rl + PC_TILE - 1) / PC_TILE;
        }
        out.self_msg = last;
        out.self_len = c->msgs[(size_t)last].len;
        out.self_start = (int32_t)at;
        n_kv += self_total; tiles += (out.self_len + PC_TILE - 1) / PC_TILE;
    } else if (call->self_msg != -1) {
        return pc_fail(c, PC_ERR_BAD_MSG_ID, "call %d: self_msg must be -1 or a message id", idx);
    } else if (s_self < -maxp || s_self + call->n_q - 1 > maxp) {
        return pc_fail(c, PC_ERR_INVALID_ARG, "call %d: query positions beyond +-%lld", idx, (long long)maxp);
    }
    out.msg_start = (int32_t)s_self;
    if (out.self_msg < 0) out.self_start = (int32_t)s_self;
    out.n_q = call->n_q;
    out.q_pos.resize(call->n_q);
    const int64_t tok0 = out.self_msg >= 0 ? self_total - call->n_q : 0;
    for (int r = 0; r < call->n_q; ++r) {
        const int64_t p = call->q_pos ? (int64_t)call->q_pos[r] : s_self + tok0 + r;
        if (p < -maxp || p > maxp) return pc_fail(c, PC_ERR_INVALID_ARG, "call %d: query position %lld beyond +-%lld", idx, (long long)p, (long long)maxp);
        out.q_pos[r] = (int32_t)p;
    }
    if (n_kv > INT32_MAX / 2) return pc_fail(c, PC_ERR_SHAPE, "call %d: gathers %lld tokens, too many", idx, (long long)n_kv);
    out.n_kv = n_kv; out.tiles = (int32_t)tiles;
    return PC_OK;
}

PlanLayout make_layout(int n_calls, int total_sel, int total_q, int total_seg, int n_dec, int n_pre, int n_pre_pk,
                       int64_t part_rows, int64_t total_tiles, int H_q, int D,
                       size_t n_sh_groups = 0, size_t n_sh_segs = 0, size_t n_sh_items = 0, size_t n_sh_pos = 0,
                       size_t n_kg_items = 0, int64_t kg_tiles = 0, int H_kv = 1, size_t n_tok = 0)
{
    PlanLayout L{};
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o = align_up(o + bytes, 256); return at; };
    L.calls = take(sizeof(PcCallDesc) * (size_t)std::max(n_calls, 1));
    L.sel = take(sizeof(int2) * (size_t)std::max(total_sel, 1));
    L.q_pos = take(sizeof(int32_t) * (size_t)std::max(total_q, 1));
    L.row_call = take(sizeof(int32_t) * (size_t)std::max(total_q, 1));
    L.merge_rows = take(sizeof(PcMergeRow) * (size_t)std::max(total_q, 1));
    L.items_dec = take(sizeof(PcItem) * (size_t)std::max(n_dec, 1));
    L.items_pre = take(sizeof(PcItem) * (size_t)std::max(n_pre, 1));
    L.items_pk = take(sizeof(PcItem) * (size_t)std::max(n_pre_pk, 1));
    L.sh_groups = take(sizeof(PcShGroup) * std::max<size_t>(n_sh_groups, 1));
    L.sh_segs = take(sizeof(PcShSeg) * std::max<size_t>(n_sh_segs, 1));
    L.sh_items = take(sizeof(PcShItem) * std::max<size_t>(n_sh_items, 1));
    L.sh_pos = take(sizeof(int32_t) * std::max<size_t>(n_sh_pos, 1));
    L.kg_items = take(sizeof(PcGatherItem) * std::max<size_t>(n_kg_items, 1));
    L.tok_items = take(sizeof(PcTokenItem) * std::max<size_t>(n_tok, 1));
    L.h2d_bytes = o;
    L.segs = take(sizeof(PcSegment) * (size_t)std::max(total_seg, 1));
    L.seg_kvoff = take(sizeof(int32_t) * (size_t)std::max(total_seg, 1));
    L.rot_seg = take(sizeof(float2) * (size_t)std::max(total_seg, 1) * (D / 2));
    L.rot_q = take(sizeof(float2) * (size_t)std::max(total_q, 1) * (D / 2));
    L.rot_qw = take(D == 128 ? sizeof(float2) * (size_t)((std::max(total_q, 1) + 31) / 32) * 32 * (D / 2) : 0);   // whole blocks of 32 rows
    L.tiles = take(sizeof(PcTile) * (size_t)std::max<int64_t>(total_tiles, 1));
    L.sh_rot = take(sizeof(float2) * std::max<size_t>(n_sh_pos, 1) * (D / 2));
    L.part_o = take(sizeof(uint16_t) * (size_t)std::max<int64_t>(part_rows, 1) * H_q * D);
    L.part_ml = take(sizeof(float) * (size_t)std::max<int64_t>(part_rows, 1) * H_q * 2);
    L.row_scalar = take(sizeof(float) * (size_t)std::max(total_q, 1) * H_q);      // one float per (row, head): the gradient path's Delta
    L.k_gather = take((size_t)std::max<int64_t>(kg_tiles, 0) * PC_TILE * (size_t)H_kv * (size_t)D * 2);   // bf16 keys ...
    L.v_gather = take((size_t)std::max<int64_t>(kg_tiles, 0) * PC_TILE * (size_t)H_kv * (size_t)D * 2);   // ... and values of the calls that gather
    L.kg_norm = take(sizeof(float) * (size_t)std::max<int64_t>(kg_tiles, 0) * (size_t)H_kv);             // ... and the largest key norm of each of their tiles
    L.total = o;
    return L;
}

// a decode call's parents in ascending cache-slot order; ties (a message listed twice) go by start
static void sort_by_slot(const pc_cache *c, Resolved &r)
{
    if (r.sel.size() < 2) return;
    // While ids ascend with slots (no freed span was ever refilled) and the list is long, one pass over
    // a table indexed by message id does it; a message listed twice sends the call to the general sort.
    if (c->slots_in_id_order && r.sel.size() * 8 > c->msgs.size()) {
        static thread_local std::vector<int32_t> where;
        static thread_local std::vector<int2> sorted;
        where.assign(c->msgs.size(), -1);
        bool twice = false;
        for (size_t e = 0; e < r.sel.size() && !twice; ++e) {
            int32_t &w = where[(size_t)r.sel[e].x];
            twice = w >= 0;
            w = (int32_t)e;
        }
        if (!twice) {
            sorted.clear();
            for (size_t m = 0; m < where.size(); ++m)
                if (where[m] >= 0) sorted.push_back(r.sel[(size_t)where[m]]);
            r.sel.assign(sorted.begin(), sorted.end());
            return;
        }
    }
    struct SortKey { uint64_t key; int2 v; };
    static thread_local std::vector<SortKey> keys;
    keys.resize(r.sel.size());
    for (size_t e = 0; e < r.sel.size(); ++e)
        keys[e] = {((uint64_t)(uint32_t)c->msgs[(size_t)r.sel[e].x].slot_start << 32) | ((uint32_t)r.sel[e].y ^ 0x80000000u), r.sel[e]};
    std::sort(keys.begin(), keys.end(), [](const SortKey &a, const SortKey &b) { return a.key < b.key; });
    for (size_t e = 0; e < r.sel.size(); ++e) r.sel[e] = keys[e].v;
}

// Shared decode (message-major): runs of consecutive one-row calls are cut into groups of up to
// 32 * 8 / g rows; a group whose calls overlap enough walks the union of their messages once.
struct SharedPlan {
    std::vector<char> in_shared;                 // per call
    std::vector<PcShGroup> groups;
    std::vector<PcShSeg> segs;
    std::vector<PcShItem> items;
    std::vector<int32_t> pos;                    // rotation positions, PC_SH_ABSENT where a row does not list the message
};

// Calls that together list n times the tokens of the union gain from the shared walk once n
// exceeds what a union tile costs there (a workgroup's pass over it for all rows: 8.7 ns per tile
// and KV head with the chip full) relative to a tile streamed by one call (1.5 to 1.7 ns).
constexpr double SHARE_MIN = 6.0;
// rows with more splits than this are merged by four lanes per 8 dimensions
constexpr int MERGE_MANY_SPLITS = 8;

static void plan_shared(const pc_cache *c, std::vector<Resolved> &res, const std::vector<int> &q_off, int g, SharedPlan &sp)
{
    const int n_calls = (int)res.size();
    sp.in_shared.assign((size_t)n_calls, 0);
    if (c->decode_sharing == 1 || !(g == 1 || g == 2 || g == 4 || g == 8)) return;
    const int rows_max = 32 * (8 / g);
    std::vector<int32_t> useg_of_msg(c->msgs.size(), -1);
    struct USeg { int32_t msg, occ; int64_t slot; int32_t len; };
    struct Entry { int32_t useg, row, pos; };
    std::vector<USeg> usegs;
    std::vector<Entry> entries;
    std::vector<std::pair<int64_t, int32_t>> extra;       // (msg << 20 | occurrence) -> useg, for repeats within a call
    std::vector<int32_t> order, new_index;
    for (int i = 0; i < n_calls;) {
        if (res[i].n_q != 1) { ++i; continue; }
        int j = i;
        while (j < n_calls && res[j].n_q == 1 && j - i < rows_max) ++j;
        usegs.clear(); entries.clear(); extra.clear();
        int64_t call_tiles = 0;
        auto lookup = [&](int32_t m, int32_t occ) -> int32_t {
            if (occ == 0) {
                if (useg_of_msg[(size_t)m] < 0) {
                    useg_of_msg[(size_t)m] = (int32_t)usegs.size();
                    usegs.push_back({m, 0, c->msgs[(size_t)m].slot_start, c->msgs[(size_t)m].len});
                }
                return useg_of_msg[(size_t)m];
            }
            const int64_t key = ((int64_t)m << 20) | occ;
            for (auto &kv : extra) if (kv.first == key) return kv.second;
            extra.push_back({key, (int32_t)usegs.size()});
            usegs.push_back({m, occ, c->msgs[(size_t)m].slot_start, c->msgs[(size_t)m].len});
            return extra.back().second;
        };
        for (int r = 0; r < j - i; ++r) {
            Resolved &rc = res[(size_t)(i + r)];
            sort_by_slot(c, rc);
            call_tiles += rc.tiles;
            int32_t prev = -1, occ = 0, self_occ = 0;
            for (const int2 &e : rc.sel) {
                occ = (e.x == prev) ? occ + 1 : 0;
                prev = e.x;
                if (e.x == rc.self_msg) ++self_occ;
                if (c->msgs[(size_t)e.x].len > 0)
                    entries.push_back({lookup(e.x, occ), r, e.y - c->msgs[(size_t)e.x].base_pos});
            }
            if (rc.self_msg >= 0 && rc.self_len > 0)      // the call's own tail: one row, one token from the end -> all of it visible
                entries.push_back({lookup(rc.self_msg, self_occ), r, rc.self_start - c->msgs[(size_t)rc.self_msg].base_pos});
        }
        int64_t union_tiles = 0;
        for (const USeg &u : usegs) union_tiles += (u.len + PC_TILE - 1) / PC_TILE;
        // (the rotation table has one 512-byte row per (message, row) pair: keep it under 256 MB)
        const bool take = union_tiles > 0 && union_tiles < INT32_MAX / 2 &&
                          (int64_t)usegs.size() * (j - i) <= ((int64_t)1 << 19) &&
                          (c->decode_sharing == 2 || (j - i >= 2 && (double)call_tiles >= SHARE_MIN * (double)union_tiles));
        if (take) {
            // union in cache-slot order
            order.resize(usegs.size()); new_index.resize(usegs.size());
            for (size_t u = 0; u < usegs.size(); ++u) order[u] = (int32_t)u;
            std::sort(order.begin(), order.end(), [&](int32_t a, int32_t b) {
                return usegs[(size_t)a].slot != usegs[(size_t)b].slot ? usegs[(size_t)a].slot < usegs[(size_t)b].slot
                                                                      : usegs[(size_t)a].occ < usegs[(size_t)b].occ; });
            PcShGroup gr{};
            gr.seg_off = (int32_t)sp.segs.size(); gr.n_seg = (int32_t)usegs.size();
            gr.row0 = q_off[(size_t)i]; gr.n_rows = j - i; gr.rot_off = (int32_t)sp.pos.size();
            gr.n_splits = 1; gr.part_off = 0;
            int32_t tile_off = 0;
            for (size_t k = 0; k < order.size(); ++k) {
                const USeg &u = usegs[(size_t)order[k]];
                new_index[(size_t)order[k]] = (int32_t)k;
                PcShSeg sg{};
                sg.slot_start = (int32_t)u.slot; sg.len = u.len; sg.tile_off = tile_off;
                tile_off += (u.len + PC_TILE - 1) / PC_TILE;
                sp.segs.push_back(sg);
            }
            gr.n_tiles = tile_off;
            sp.pos.resize(sp.pos.size() + usegs.size() * (size_t)gr.n_rows, PC_SH_ABSENT);
            for (const Entry &en : entries) {
                const int32_t k = new_index[(size_t)en.useg];
                sp.segs[(size_t)gr.seg_off + (size_t)k].vis[en.row >> 5] |= 1u << (en.row & 31);
                sp.pos[(size_t)gr.rot_off + (size_t)k * (size_t)gr.n_rows + (size_t)en.row] = en.pos;
            }
            sp.groups.push_back(gr);
            for (int k = i; k < j; ++k) sp.in_shared[(size_t)k] = 1;
        }
        for (const USeg &u : usegs) if (u.occ == 0) useg_of_msg[(size_t)u.msg] = -1;
        i = j;
    }
}

int32_t pc_plan_and_stage(pc_cache *c, const pc_call *calls, int32_t n_calls, bool want_items,
                              hipStream_t st, Planned &P)
{
    P.n_calls = n_calls;
    P.res.resize((size_t)n_calls);
    for (int i = 0; i < n_calls; ++i) {
        const int32_t rc = pc_resolve(c, &calls[i], i, P.res[i]);
        if (rc != PC_OK) return rc;
        P.total_q += P.res[i].n_q;
    }
    const int g = c->g, H_kv = c->cfg.n_kv_heads;
    const bool bf16 = c->cfg.dtype == PC_BF16;
    // work-group shape of the prefill kernel: 8 row units (32 rows x 1 q head each) per group
    P.pre_waves = 8;
    std::vector<PcCallDesc> cds((size_t)n_calls);
    std::vector<PcItem> dec, pre, pre_pk;
    std::vector<PcGatherItem> kg;
    int64_t kg_tiles = 0;
    int64_t part_rows = 0, total_tiles = 0;
    int sel_off = 0, q_off = 0, seg_off = 0;
    // groups of one-row calls that share enough of their messages take the shared walk
    SharedPlan sp;
    sp.in_shared.assign((size_t)n_calls, 0);
    if (want_items && bf16) {
        std::vector<int> q_offs((size_t)n_calls);
        for (int i = 0, o = 0; i < n_calls; ++i) { q_offs[(size_t)i] = o; o += P.res[(size_t)i].n_q; }
        plan_shared(c, P.res, q_offs, g, sp);
    }
    // first pass: how many prefill groups without splitting (to decide on KV splits)
    int64_t pre_groups = 0, dec_groups = 0;
    if (want_items && bf16)
        for (int i = 0; i < n_calls; ++i) {
            const Resolved &r = P.res[(size_t)i];
            if (sp.in_shared[(size_t)i]) continue;
            if (r.n_q * g > 16) pre_groups += (int64_t)(((r.n_q + 31) / 32) * g + P.pre_waves - 1) / P.pre_waves * H_kv;
            else dec_groups += H_kv;
        }
    for (int i = 0; i < n_calls; ++i) {
        Resolved &r = P.res[i];
        PcCallDesc &cd = cds[i];
        // a call served by the shared walk needs no segments, tiles or rotation rows of its own: the plan
        // builder sees it as a call that lists nothing
        const bool own_plan = !sp.in_shared[(size_t)i];
        cd.sel_off = sel_off; cd.n_sel = own_plan ? (int)r.sel.size() : 0;
        cd.self_msg = own_plan ? r.self_msg : -1; cd.self_start = r.self_start;
        cd.n_q = r.n_q; cd.q_off = q_off; cd.seg_off = seg_off; cd.n_seg = cd.n_sel + (cd.self_msg >= 0 ? 1 : 0);
        cd.self_len = own_plan ? r.self_len : 0; cd.n_splits = 1; cd.part_off = 0; cd.tile_off = (int32_t)total_tiles;
        cd.kg_tile0 = -1; cd.n_par = 0; cd.pad[0] = cd.pad[1] = 0;
        if (own_plan) total_tiles += r.tiles;
        sel_off += cd.n_sel; q_off += cd.n_q; seg_off += cd.n_seg;
        if (!want_items || !bf16 || !own_plan) continue;
        const int T = r.tiles;
        if (r.n_q * g <= 16) {                       // decode-shaped: all rows x heads of a KV head in one wave
            // Attention does not depend on the order the keys are visited in (each keeps its own
            // position), so a decode call walks its parents in ascending cache-slot order: calls that
            // share messages then touch them at about the same time and the later ones hit in L2.
            sort_by_slot(c, r);
            // as few splits as fill the chip (256 workgroups): the kernel is bound by memory, and every
            // split beyond that only adds partial results to write and merge
            int ns = c->decode_tiles_per_split > 0 ? (T + c->decode_tiles_per_split - 1) / c->decode_tiles_per_split
                                                   : (int)std::min<int64_t>((256 + dec_groups - 1) / dec_groups, std::max(1, T / 16));
            ns = std::max(1, std::min(MAX_SPLITS, ns));
            const int chunk = std::max(1, (T + ns - 1) / ns);
            ns = std::max(1, (T + chunk - 1) / chunk);
            cd.n_splits = ns;
            for (int s = 0; s < ns; ++s) {
                PcItem it{}; it.call = i; it.unit0 = 0; it.tile_begin = s * chunk; it.tile_end = std::min(T, (s + 1) * chunk); it.split = s;
                it.tile_tab0 = cd.tile_off;
                dec.push_back(it);
            }
        } else {
            // Gather: a call with many query rows reads its keys and values from a packed copy (the gather pass: keys
            // turned to the call's positions, no padding between messages), which moves 8192 bytes per listed token once
            // (about 1.8 ns) and saves the turns of the queries at every message, the ragged tile at every message's end
            // and the per-tile lookups: 15 to 25 % of the attention's own time, which is rows x heads x 0.47 ps per token.
            // The copy pays from rows x query heads of about 20 thousand on; taken from 32768 on.  (Not with a fixed
            // workspace, which the copy may not fit into.)
            const int self_tiles = r.self_msg >= 0 ? (r.self_len + PC_TILE - 1) / PC_TILE : 0;
            int64_t n_par = 0;
            for (const int2 &e : r.sel) n_par += c->msgs[(size_t)e.x].len;
            const int p_tiles = (int)((n_par + PC_TILE - 1) / PC_TILE);
            const bool packed = T > 0 && !P.fixed_ws && kg_tiles + p_tiles + self_tiles < ((int64_t)1 << 24) &&
                                (c->key_gather == 2 || (c->key_gather == 0 && (int64_t)r.n_q * c->cfg.n_q_heads >= 32768));
            if (packed) {
                cd.kg_tile0 = (int32_t)kg_tiles; cd.n_par = (int32_t)n_par;
                kg.push_back(PcGatherItem{i, (int32_t)kg_tiles, p_tiles + self_tiles, (int32_t)n_par});
                kg_tiles += p_tiles + self_tiles;
            }
            const int Tc = packed ? p_tiles + self_tiles : T;        // tiles the attention kernel walks for this call
            const int units = ((r.n_q + 31) / 32) * g;
            const int groups = (units + P.pre_waves - 1) / P.pre_waves;
            int ns = 1;
            if (c->prefill_tiles_per_split > 0) ns = (Tc + c->prefill_tiles_per_split - 1) / c->prefill_tiles_per_split;
            else if (pre_groups < 256) ns = (int)std::min<int64_t>((256 + pre_groups - 1) / pre_groups, std::max(1, Tc / 16));
            ns = std::max(1, std::min(MAX_SPLITS, ns));
            const int chunk = std::max(1, (Tc + ns - 1) / ns);
            ns = std::max(1, (Tc + chunk - 1) / chunk);
            cd.n_splits = ns;
            // A group of row units walks the parents' tiles and the tiles of the new message up to the
            // causal limit of its last row (the kernel relies on tile_end being cut there); its splits
            // divide THAT count evenly, so the groups with early rows do not end up with a nearly empty
            // last split.
            const int parent_tiles = Tc - self_tiles;
            for (int gidx = 0; gidx < groups; ++gidx) {
                int Tg = Tc;
                if (r.self_msg >= 0) {
                    const int last_unit = std::min(gidx * P.pre_waves + P.pre_waves - 1, units - 1);
                    const int lim = (r.self_len - r.n_q) + std::min(32 * (last_unit / g) + 31, r.n_q - 1);   // last own token seen
                    Tg = parent_tiles + std::min(self_tiles, lim / PC_TILE + 1);
                }
                const int chunk_g = std::max(1, (Tg + ns - 1) / ns);
                for (int s = 0; s < ns; ++s) {
                    PcItem it{}; it.call = i; it.unit0 = gidx * P.pre_waves; it.split = s; it.tile_tab0 = cd.tile_off;
                    it.tile_begin = std::min(Tg, s * chunk_g);
                    it.tile_end = s == ns - 1 ? Tg : std::min(Tg, (s + 1) * chunk_g);
                    (packed ? pre_pk : pre).push_back(it);
                }
            }
        }
        if (cd.n_splits > 1) { cd.part_off = (int32_t)part_rows; part_rows += (int64_t)cd.n_splits * cd.n_q; }
    }
    // shared groups: as many splits of the union as fill the chip together
    for (size_t gi = 0; gi < sp.groups.size(); ++gi) {
        PcShGroup &gr = sp.groups[gi];
        const int T = gr.n_tiles;
        int ns = c->decode_tiles_per_split > 0 ? (T + c->decode_tiles_per_split - 1) / c->decode_tiles_per_split
                                               : (int)std::min<int64_t>((256 + (int64_t)sp.groups.size() * H_kv - 1) / ((int64_t)sp.groups.size() * H_kv),
                                                                        std::max(1, T / 8));
        ns = std::max(1, std::min(MAX_SPLITS, ns));
        const int chunk = std::max(1, (T + ns - 1) / ns);
        ns = std::max(1, (T + chunk - 1) / chunk);
        gr.n_splits = ns;
        if (ns > 1) { gr.part_off = (int32_t)part_rows; part_rows += (int64_t)ns * gr.n_rows; }
        int seg = 0;                                     // the message that owns a split's first tile (splits ascend)
        for (int sidx = 0; sidx < ns; ++sidx) {
            const int t0 = sidx * chunk;
            while (seg + 1 < gr.n_seg && sp.segs[(size_t)gr.seg_off + (size_t)seg + 1].tile_off <= t0) ++seg;
            sp.items.push_back(PcShItem{(int32_t)gi, t0, std::min(T, (sidx + 1) * chunk), sidx, seg, {0, 0, 0}});
        }
    }
    if (part_rows > INT32_MAX) return pc_fail(c, PC_ERR_SHAPE, "attend: partial buffer too large");
    P.total_sel = sel_off; P.total_seg = seg_off;
    P.n_dec = (int)dec.size(); P.n_pre = (int)pre.size(); P.n_pre_pk = (int)pre_pk.size();
    P.n_sh_items = (int)sp.items.size(); P.n_sh_pos = sp.pos.size();
    P.n_kg_items = (int)kg.size(); P.kg_tiles = kg_tiles;
    if (total_tiles > INT32_MAX / 2) return pc_fail(c, PC_ERR_SHAPE, "attend: too many KV tiles");
    if (sp.pos.size() > (size_t)INT32_MAX / 2) return pc_fail(c, PC_ERR_SHAPE, "attend: shared decode table too large");
    P.lay = make_layout(n_calls, P.total_sel, P.total_q, P.total_seg, P.n_dec, P.n_pre, P.n_pre_pk, part_rows, total_tiles, c->cfg.n_q_heads, c->D,
                        sp.groups.size(), sp.segs.size(), sp.items.size(), sp.pos.size(), kg.size(), kg_tiles, H_kv, P.tok_items.size());
    if (c->host_only) return PC_OK;

    int32_t rc = PC_OK;
    if (P.fixed_ws) {                                    // nothing may be allocated: the plan fits or the call fails
        if (P.lay.total > P.fixed_cap)
            return pc_fail(c, PC_ERR_NO_SPACE, "attend: this batch needs %zu bytes of workspace, the fixed one holds %zu",
                           P.lay.total, P.fixed_cap);
        if (P.lay.h2d_bytes > c->stage[c->stage_next].cap)
            return pc_fail(c, PC_ERR_NO_SPACE, "attend: this batch stages %zu bytes of descriptors, the pinned ring slot holds %zu",
                           P.lay.h2d_bytes, c->stage[c->stage_next].cap);
        P.ws = P.fixed_ws;
    } else {
        rc = pc_ensure_ws(c, P.lay.total, st);
        if (rc != PC_OK) return rc;
        P.ws = c->ws;
    }
    StageSlot *slot = nullptr;
    rc = pc_stage_acquire(c, P.lay.h2d_bytes, &slot);
    if (rc != PC_OK) return rc;
    char *h = (char *)slot->host;
    std::memcpy(h + P.lay.calls, cds.data(), sizeof(PcCallDesc) * cds.size());
    int2 *hs = (int2 *)(h + P.lay.sel);
    int32_t *hq = (int32_t *)(h + P.lay.q_pos), *hr = (int32_t *)(h + P.lay.row_call);
    PcMergeRow *hm = (PcMergeRow *)(h + P.lay.merge_rows);
    for (int i = 0; i < n_calls; ++i) {
        const Resolved &r = P.res[i];
        if (cds[i].n_sel > 0) std::memcpy(hs + cds[i].sel_off, r.sel.data(), sizeof(int2) * (size_t)cds[i].n_sel);
        std::memcpy(hq + cds[i].q_off, r.q_pos.data(), sizeof(int32_t) * r.q_pos.size());
        for (int q = 0; q < r.n_q; ++q) hr[cds[i].q_off + q] = i;
    }
    // rows to merge: those with few splits first, then those with many (they get four lanes per 8 dimensions)
    for (int pass = 0; pass < 2; ++pass) {
        auto wanted = [&](int n_splits) { return n_splits > 1 && (n_splits > MERGE_MANY_SPLITS) == (pass == 1); };
        for (int i = 0; i < n_calls; ++i)
            if (wanted(cds[i].n_splits))
                for (int q = 0; q < P.res[i].n_q; ++q)
                    hm[P.n_merge_rows++] = PcMergeRow{cds[i].q_off + q, cds[i].part_off + q, cds[i].n_splits, P.res[i].n_q};
        for (const PcShGroup &gr : sp.groups)
            if (wanted(gr.n_splits))
                for (int q = 0; q < gr.n_rows; ++q) hm[P.n_merge_rows++] = PcMergeRow{gr.row0 + q, gr.part_off + q, gr.n_splits, gr.n_rows};
        if (pass == 0) P.n_merge_few = P.n_merge_rows;
    }
    if (!dec.empty()) std::memcpy(h + P.lay.items_dec, dec.data(), sizeof(PcItem) * dec.size());
    if (!pre.empty()) std::memcpy(h + P.lay.items_pre, pre.data(), sizeof(PcItem) * pre.size());
    if (!pre_pk.empty()) std::memcpy(h + P.lay.items_pk, pre_pk.data(), sizeof(PcItem) * pre_pk.size());
    if (!kg.empty()) std::memcpy(h + P.lay.kg_items, kg.data(), sizeof(PcGatherItem) * kg.size());
    if (!P.tok_items.empty()) std::memcpy(h + P.lay.tok_items, P.tok_items.data(), sizeof(PcTokenItem) * P.tok_items.size());
    if (!sp.items.empty()) {
        std::memcpy(h + P.lay.sh_groups, sp.groups.data(), sizeof(PcShGroup) * sp.groups.size());
        std::memcpy(h + P.lay.sh_segs, sp.segs.data(), sizeof(PcShSeg) * sp.segs.size());
        std::memcpy(h + P.lay.sh_items, sp.items.data(), sizeof(PcShItem) * sp.items.size());
        std::memcpy(h + P.lay.sh_pos, sp.pos.data(), sizeof(int32_t) * sp.pos.size());
    }
    PC_HIP(c, hipMemcpyAsync(P.ws, h, P.lay.h2d_bytes, hipMemcpyHostToDevice, st));
    PC_HIP(c, hipEventRecord(slot->ev, st));
    slot->used = true;
    {
        ProfScope ps(c, 1, st);
        char *w = (char *)P.ws;
        PcTokenWork tok;
        if (!P.tok_items.empty()) {
            tok.items = (const PcTokenItem *)(w + P.lay.tok_items); tok.n = (int)P.tok_items.size();
            tok.k = P.tok_k; tok.v = P.tok_v; tok.k_store = c->k_store; tok.v_store = c->v_store;
            tok.slots = c->slots; tok.n_kv_heads = c->cfg.n_kv_heads; tok.D = c->D; tok.dtype = c->cfg.dtype;
        }
        pc_launch_build_plan((const PcCallDesc *)(w + P.lay.calls), n_calls, (const int2 *)(w + P.lay.sel),
                             (const int32_t *)(w + P.lay.q_pos), c->table_dev, c->inv_freq_dev, c->half, P.total_seg,
                             P.total_q, (PcSegment *)(w + P.lay.segs), (int32_t *)(w + P.lay.seg_kvoff),
                             (float2 *)(w + P.lay.rot_seg), (float2 *)(w + P.lay.rot_q),
                             c->cfg.head_dim == 128 ? (float2 *)(w + P.lay.rot_qw) : nullptr, (PcTile *)(w + P.lay.tiles), tok, st);
        PC_HIP(c, hipGetLastError());
        P.tok_done = !P.tok_items.empty();
        if (P.n_sh_items > 0) {
            pc_launch_shared_rot((const int32_t *)(w + P.lay.sh_pos), (int64_t)P.n_sh_pos, c->inv_freq_dev, c->half,
                                 (float2 *)(w + P.lay.sh_rot), st);
            PC_HIP(c, hipGetLastError());
        }
    }
    return PC_OK;
}

extern "C" {

int32_t pc_resolve_call(pc_cache *c, const pc_call *call, int32_t *starts_out, int32_t *self_start_out, int64_t *n_kv)
{
    if (!c) return PC_ERR_INVALID_ARG;
    Resolved r;
    const int32_t rc = pc_resolve(c, call, 0, r);
    if (rc != PC_OK) return rc;
    if (starts_out) for (size_t e = 0; e < r.entry_start.size(); ++e) starts_out[e] = r.entry_start[e];
    if (self_start_out) *self_start_out = r.msg_start;
    if (n_kv) *n_kv = r.n_kv;
    return PC_OK;
}

}  // extern "C"
