// Host side of the library: the cache object, message table, slot allocator, appends, position
// updates, free / swap, bookkeeping and profiling.
#include "pc_host.h"

int32_t pc_fail(pc_cache *c, int32_t code, const char *fmt, ...)
{
    if (c) {
        char buf[512];
        va_list ap; va_start(ap, fmt); vsnprintf(buf, sizeof buf, fmt, ap); va_end(ap);
        c->err = buf;
    }
    return code;
}

size_t pc_storage_bytes(const pc_config *cfg)
{
    const int64_t slots = (int64_t)align_up((size_t)std::max<int64_t>(cfg->capacity_tokens, 1), PC_SLOT_ALIGN);
    const size_t es = cfg->dtype == PC_BF16 ? 2 : 4;
    return 2 * (size_t)slots * cfg->n_kv_heads * cfg->head_dim * es;
}

void pc_prof_collect(pc_cache *c)
{
    for (auto &r : c->prof_recs) {
        (void)hipEventSynchronize(r.b);
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, r.a, r.b) == hipSuccess) { c->prof_ms[r.cls] += ms; c->prof_n[r.cls] += 1; }
        c->ev_pool.push_back(r.a); c->ev_pool.push_back(r.b);
    }
    c->prof_recs.clear();
}

int32_t pc_ensure_ws(pc_cache *c, size_t bytes, hipStream_t st)
{
    if (bytes <= c->ws_cap) return PC_OK;
    if (c->ws) {                                         // work in flight may still use the old one
        PC_HIP(c, hipStreamSynchronize(st));
        PC_HIP(c, hipDeviceSynchronize());
        PC_HIP(c, hipFree(c->ws));
    }
    c->ws = nullptr; c->ws_cap = 0;
    const size_t cap = align_up(bytes + bytes / 4, 1 << 20);
    PC_HIP(c, hipMalloc(&c->ws, cap));
    c->ws_cap = cap;
    return PC_OK;
}

int32_t pc_stage_acquire(pc_cache *c, size_t bytes, StageSlot **out)
{
    StageSlot &s = c->stage[c->stage_next];
    c->stage_next = (c->stage_next + 1) % N_STAGE;
    if (s.used) PC_HIP(c, hipEventSynchronize(s.ev));
    if (!s.ev) PC_HIP(c, hipEventCreateWithFlags(&s.ev, hipEventDisableTiming));
    if (bytes > s.cap) {
        if (s.host) PC_HIP(c, hipHostFree(s.host));
        s.host = nullptr; s.cap = 0;
        const size_t cap = align_up(bytes * 2, 4096);
        PC_HIP(c, hipHostMalloc(&s.host, cap, hipHostMallocDefault));
        s.cap = cap;
    }
    *out = &s;
    return PC_OK;
}

// =====================================================================================
extern "C" {

size_t pc_cache_storage_bytes(const pc_config *cfg)
{
    if (!cfg || cfg->n_kv_heads <= 0 || cfg->head_dim <= 0) return 0;
    return pc_storage_bytes(cfg);
}

int32_t pc_cache_create(const pc_config *cfg, pc_cache **out)
{
    if (!cfg || !out) return PC_ERR_INVALID_ARG;
    *out = nullptr;
    if (cfg->n_q_heads <= 0 || cfg->n_kv_heads <= 0 || cfg->n_q_heads % cfg->n_kv_heads) return PC_ERR_SHAPE;
    if (cfg->head_dim != 64 && cfg->head_dim != 128) return PC_ERR_SHAPE;
    if (cfg->dtype != PC_F32 && cfg->dtype != PC_BF16) return PC_ERR_INVALID_ARG;
    if (cfg->dtype == PC_BF16 && cfg->head_dim != 128) return PC_ERR_SHAPE;
    if (cfg->dtype == PC_BF16 && cfg->n_q_heads / cfg->n_kv_heads > 16) return PC_ERR_SHAPE;
    if (cfg->capacity_tokens <= 0 || cfg->max_messages <= 0 || !(cfg->rope_theta > 0.f)) return PC_ERR_INVALID_ARG;
    pc_cache *c = new pc_cache();
    c->cfg = *cfg;
    if (c->cfg.max_position <= 0) c->cfg.max_position = 1 << 24;
    c->host_only = (cfg->flags & PC_FLAG_HOST_ONLY) != 0;
    c->grow_extents = (cfg->flags & PC_FLAG_GROW_EXTENTS) != 0;
    c->D = cfg->head_dim; c->half = c->D / 2; c->g = cfg->n_q_heads / cfg->n_kv_heads;
    c->slots = (int64_t)align_up((size_t)cfg->capacity_tokens, PC_SLOT_ALIGN);
    if (c->slots > INT32_MAX) { delete c; return PC_ERR_SHAPE; }
    c->esize = cfg->dtype == PC_BF16 ? 2 : 4;
    c->scale = cfg->softmax_scale > 0.f ? cfg->softmax_scale : 1.0f / std::sqrt((float)c->D);
    c->msgs.reserve((size_t)cfg->max_messages);
    *out = c;
    if (c->host_only) return PC_OK;

    const size_t bytes = pc_storage_bytes(cfg);
    auto bail = [&](int32_t code) { pc_cache_destroy(c); *out = nullptr; return code; };
    if (cfg->arena) {
        if (cfg->arena_bytes < bytes || ((uintptr_t)cfg->arena & 255)) return bail(PC_ERR_NO_SPACE);
        c->storage = cfg->arena;
    } else {
        if (hipMalloc(&c->storage, bytes) != hipSuccess) return bail(PC_ERR_HIP);
        c->owns_storage = true;
    }
    // zero once: slots past a message's end inside its last tile are read (and masked)
    if (hipMemset(c->storage, 0, bytes) != hipSuccess) return bail(PC_ERR_HIP);
    c->k_store = c->storage;
    c->v_store = (char *)c->storage + bytes / 2;
    if (hipMalloc((void **)&c->table_dev, sizeof(PcMsgEntry) * (size_t)cfg->max_messages) != hipSuccess) return bail(PC_ERR_HIP);
    if (hipMemset(c->table_dev, 0, sizeof(PcMsgEntry) * (size_t)cfg->max_messages) != hipSuccess) return bail(PC_ERR_HIP);
    std::vector<double> f((size_t)c->half);
    for (int i = 0; i < c->half; ++i) f[i] = std::pow((double)cfg->rope_theta, -2.0 * i / c->D);
    if (hipMalloc((void **)&c->inv_freq_dev, sizeof(double) * f.size()) != hipSuccess) return bail(PC_ERR_HIP);
    if (hipMemcpy(c->inv_freq_dev, f.data(), sizeof(double) * f.size(), hipMemcpyHostToDevice) != hipSuccess) return bail(PC_ERR_HIP);
    // first buffers of a modest size, so that ordinary calls do not allocate on their way (they grow on demand)
    if (hipMalloc(&c->ws, (size_t)32 << 20) != hipSuccess) return bail(PC_ERR_HIP);
    c->ws_cap = (size_t)32 << 20;
    if (hipMalloc(&c->tok_dev, (size_t)1 << 16) != hipSuccess) return bail(PC_ERR_HIP);
    c->tok_cap = (size_t)1 << 16;
    for (int i = 0; i < N_STAGE; ++i) {
        if (hipHostMalloc(&c->stage[i].host, (size_t)1 << 20, hipHostMallocDefault) != hipSuccess) return bail(PC_ERR_HIP);
        c->stage[i].cap = (size_t)1 << 20;
        if (hipEventCreateWithFlags(&c->stage[i].ev, hipEventDisableTiming) != hipSuccess) return bail(PC_ERR_HIP);
    }
    if (hipStreamCreateWithFlags(&c->side, hipStreamNonBlocking) != hipSuccess) return bail(PC_ERR_HIP);
    if (hipEventCreateWithFlags(&c->ev_fork, hipEventDisableTiming) != hipSuccess) return bail(PC_ERR_HIP);
    if (hipEventCreateWithFlags(&c->ev_join, hipEventDisableTiming) != hipSuccess) return bail(PC_ERR_HIP);
    {   // this device's address of the library's fixed scratch array (pc_attend_static works in it)
        size_t n = 0;
        if (pc_static_scratch(&c->static_ws, &n) != PC_OK) return bail(PC_ERR_HIP);
    }
    if (hipDeviceSynchronize() != hipSuccess) return bail(PC_ERR_HIP);
    return PC_OK;
}

int32_t pc_cache_destroy(pc_cache *c)
{
    if (!c) return PC_ERR_INVALID_ARG;
    if (!c->host_only) {
        (void)hipDeviceSynchronize();
        pc_prof_collect(c);
        for (auto e : c->ev_pool) (void)hipEventDestroy(e);
        for (auto &s : c->stage) { if (s.host) (void)hipHostFree(s.host); if (s.ev) (void)hipEventDestroy(s.ev); }
        if (c->ev_fork) (void)hipEventDestroy(c->ev_fork);
        if (c->ev_join) (void)hipEventDestroy(c->ev_join);
        if (c->side) (void)hipStreamDestroy(c->side);
        if (c->ws) (void)hipFree(c->ws);
        if (c->tok_dev) (void)hipFree(c->tok_dev);
        if (c->inv_freq_dev) (void)hipFree(c->inv_freq_dev);
        if (c->table_dev) (void)hipFree(c->table_dev);
        if (c->owns_storage && c->storage) (void)hipFree(c->storage);
    }
    delete c;
    return PC_OK;
}

const char *pc_last_error(const pc_cache *c) { return c ? c->err.c_str() : "null cache"; }

// Takes the slots of one message out of (spans, next): the first freed span that holds the reserve
// rounded up to the slot alignment, else the end of the used region.  False (nothing changed) if neither has room.
static bool take_slots(std::vector<FreeSpan> &spans, int64_t &next, int64_t capacity, int32_t res, int64_t &start)
{
    const int64_t need = (int64_t)align_up((size_t)res, PC_SLOT_ALIGN);
    for (size_t i = 0; i < spans.size(); ++i)
        if (spans[i].size >= need) {
            start = spans[i].start;
            spans[i].start += need; spans[i].size -= need;
            if (spans[i].size == 0) spans.erase(spans.begin() + (long)i);
            return true;
        }
    if (next + res > capacity) return false;
    start = next;
    next += need;
    return true;
}

// A span taken where a freed or swapped-out message may have lived: its K and V rows are cleared before the new
// owner's append kernel runs (the attention kernels mask what lies behind a message's last token, inside its last
// tile, by adding -inf to its scores and multiply its V rows by exact zeros, both of which need finite values there).
static void clear_if_reused(pc_cache *c, int64_t start, int32_t res, hipStream_t st)
{
    if (c->host_only || start >= c->dirty_end) return;
    const int64_t need = (int64_t)align_up((size_t)res, PC_SLOT_ALIGN);
    const int64_t n = std::min(need, c->dirty_end - start);
    pc_launch_zero_span(c->cfg.dtype, c->k_store, c->slots, c->cfg.n_kv_heads, c->D, start, n, st);
    pc_launch_zero_span(c->cfg.dtype, c->v_store, c->slots, c->cfg.n_kv_heads, c->D, start, n, st);
}

int32_t pc_append_message(pc_cache *c, const void *k, const void *v, int32_t len, int32_t reserve,
                          int32_t *msg_id, void *stream)
{
    if (!c) return PC_ERR_INVALID_ARG;
    if (len < 1) return pc_fail(c, PC_ERR_INVALID_ARG, "append: len = %d must be >= 1", len);
    if (!c->host_only && (!k || !v)) return pc_fail(c, PC_ERR_INVALID_ARG, "append: null k or v");
    if (!c->host_only && (((uintptr_t)k | (uintptr_t)v) & 15)) return pc_fail(c, PC_ERR_INVALID_ARG, "append: k and v must be 16-byte aligned");
    if (!msg_id) return pc_fail(c, PC_ERR_INVALID_ARG, "append: null msg_id");
    if ((int64_t)c->msgs.size() >= c->cfg.max_messages)
        return pc_fail(c, PC_ERR_NO_SPACE, "append: message table full (%d)", c->cfg.max_messages);
    const int32_t res = std::max(reserve, len);
    // the bookkeeping changes only once the launch has been accepted
    std::vector<FreeSpan> spans = c->free_spans;
    int64_t next = c->next_slot, start = 0;
    if (!take_slots(spans, next, c->slots, res, start))
        return pc_fail(c, PC_ERR_NO_SPACE, "append: needs slots [%lld, %lld), capacity %lld", (long long)c->next_slot,
                    (long long)(c->next_slot + res), (long long)c->slots);
    const int id = (int)c->msgs.size();
    if (!c->host_only) {
        hipStream_t st = (hipStream_t)stream;
        clear_if_reused(c, start, res, st);
        ProfScope ps(c, 0, st);
        pc_launch_append(c->cfg.dtype, k, v, len, c->cfg.n_kv_heads, c->D, start, c->slots, c->inv_freq_dev,
                         c->k_store, c->v_store, c->table_dev, id, st);
        PC_HIP(c, hipGetLastError());
    }
    if (!c->msgs.empty() && start < c->msgs.back().slot_start) c->slots_in_id_order = false;
    c->msgs.push_back({start, len, res, 0, true});
    c->free_spans.swap(spans);
    c->next_slot = next;
    *msg_id = id;
    return PC_OK;
}

// small host-built item lists go through the pinned ring into one device buffer that grows on demand
int32_t pc_stage_items(pc_cache *c, const void *items, size_t bytes, hipStream_t st)
{
    if (bytes > c->tok_cap) {
        if (c->tok_dev) {                                // work in flight may still use the old one
            PC_HIP(c, hipStreamSynchronize(st));
            PC_HIP(c, hipDeviceSynchronize());
            PC_HIP(c, hipFree(c->tok_dev));
        }
        c->tok_dev = nullptr; c->tok_cap = 0;
        const size_t cap = std::max<size_t>(1 << 16, bytes * 2);
        PC_HIP(c, hipMalloc(&c->tok_dev, cap));
        c->tok_cap = cap;
    }
    StageSlot *slot = nullptr;
    const int32_t rc = pc_stage_acquire(c, bytes, &slot);
    if (rc != PC_OK) return rc;
    std::memcpy(slot->host, items, bytes);
    PC_HIP(c, hipMemcpyAsync(c->tok_dev, slot->host, bytes, hipMemcpyHostToDevice, st));
    PC_HIP(c, hipEventRecord(slot->ev, st));
    slot->used = true;
    return PC_OK;
}

int32_t pc_append_messages(pc_cache *c, int32_t n, const void *const *k, const void *const *v, const int32_t *lens,
                           const int32_t *reserves, int32_t *msg_ids, void *stream)
{
    if (!c) return PC_ERR_INVALID_ARG;
    if (n < 0 || (n > 0 && (!lens || !msg_ids))) return pc_fail(c, PC_ERR_INVALID_ARG, "append_messages: bad lists");
    if (n == 0) return PC_OK;
    if (!c->host_only && (!k || !v)) return pc_fail(c, PC_ERR_INVALID_ARG, "append_messages: null k or v list");
    if ((int64_t)c->msgs.size() + n > c->cfg.max_messages)
        return pc_fail(c, PC_ERR_NO_SPACE, "append_messages: message table full (%d)", c->cfg.max_messages);
    // all or nothing: allocate on copies first
    std::vector<FreeSpan> spans = c->free_spans;
    int64_t next = c->next_slot;
    std::vector<PcAppendItem> items((size_t)n);
    std::vector<HostMsg> fresh((size_t)n);
    int max_len = 0;
    for (int j = 0; j < n; ++j) {
        if (lens[j] < 1) return pc_fail(c, PC_ERR_INVALID_ARG, "append_messages: message %d has len = %d", j, lens[j]);
        if (!c->host_only && (!k[j] || !v[j])) return pc_fail(c, PC_ERR_INVALID_ARG, "append_messages: message %d has null k or v", j);
        if (!c->host_only && (((uintptr_t)k[j] | (uintptr_t)v[j]) & 15))
            return pc_fail(c, PC_ERR_INVALID_ARG, "append_messages: k and v of message %d must be 16-byte aligned", j);
        const int32_t res = std::max(reserves ? reserves[j] : 0, lens[j]);
        int64_t start = 0;
        if (!take_slots(spans, next, c->slots, res, start))
            return pc_fail(c, PC_ERR_NO_SPACE, "append_messages: message %d (%d slots) does not fit, capacity %lld", j, res,
                        (long long)c->slots);
        fresh[(size_t)j] = HostMsg{start, lens[j], res, 0, true};
        items[(size_t)j] = PcAppendItem{c->host_only ? nullptr : k[j], c->host_only ? nullptr : v[j],
                                        (int32_t)c->msgs.size() + j, (int32_t)start, lens[j], 0};
        max_len = std::max(max_len, lens[j]);
    }
    if (!c->host_only) {
        hipStream_t st = (hipStream_t)stream;
        const int32_t rc = pc_stage_items(c, items.data(), sizeof(PcAppendItem) * (size_t)n, st);
        if (rc != PC_OK) return rc;
        for (int j = 0; j < n; ++j) clear_if_reused(c, fresh[(size_t)j].slot_start, fresh[(size_t)j].reserve, st);
        ProfScope ps(c, 0, st);
        pc_launch_append_batch(c->cfg.dtype, (const PcAppendItem *)c->tok_dev, n, max_len, c->cfg.n_kv_heads, c->D, c->slots,
                               c->inv_freq_dev, c->k_store, c->v_store, c->table_dev, st);
        PC_HIP(c, hipGetLastError());
    }
    for (int j = 0; j < n; ++j) {
        msg_ids[j] = (int32_t)c->msgs.size();
        if (!c->msgs.empty() && fresh[(size_t)j].slot_start < c->msgs.back().slot_start) c->slots_in_id_order = false;
        c->msgs.push_back(fresh[(size_t)j]);
    }
    c->free_spans.swap(spans);
    c->next_slot = next;
    return PC_OK;
}

// shared by pc_append_tokens and pc_append_tokens_batch: token j of k, v goes to message ids[j]
// (the tokens of one message are consecutive and in order, no message has two runs; validated by
// the callers).  Host work is proportional to the tokens, not to the messages the cache holds.
// defer: if given and the tokens need no new table row (no further extent), nothing is launched: the items are handed
// back for the caller to write them with a kernel of its own (the decode step's plan builder); the host bookkeeping is
// done either way.  An empty *defer on return means the append was enqueued here.
int32_t pc_append_token_items(pc_cache *c, const std::vector<int32_t> &ids, const void *k, const void *v, hipStream_t st,
                              std::vector<PcTokenItem> *defer)
{
    if (defer) defer->clear();
    const int n = (int)ids.size();
    std::vector<PcTokenItem> items((size_t)n);
    std::vector<HostMsg> fresh;                              // new extent records: ids msgs.size(), msgs.size() + 1, ...
    std::vector<std::pair<int32_t, int32_t>> links;          // (record, its new next)
    std::vector<std::pair<int32_t, int32_t>> grown;          // (record, its length after this call)
    std::vector<FreeSpan> spans = c->free_spans;             // nothing is committed before the launch is accepted
    int64_t next = c->next_slot;
    const int32_t first_new = (int32_t)c->msgs.size();
    for (int j = 0; j < n;) {
        const int32_t m = ids[(size_t)j];
        int run_end = j;
        while (run_end < n && ids[(size_t)run_end] == m) ++run_end;
        // the extent the message is writing into, as it will be
        const int32_t last = chain_last(c, m);
        const HostMsg &hm = c->msgs[(size_t)last];
        int32_t rec = last, len = hm.len, reserve = hm.reserve, base = hm.base_pos;
        int64_t slot = hm.slot_start;
        int first_item = j;                                  // first token of this call in the current extent
        // every item carries the final length of the extent it goes to
        auto close_extent = [&](int upto) {
            if (upto == first_item) return;
            for (int t = first_item; t < upto; ++t) items[(size_t)t].new_len = len;
            grown.push_back({rec, len});
        };
        for (; j < run_end; ++j) {
            if (len == reserve) {
                if (!c->grow_extents)
                    return pc_fail(c, PC_ERR_NO_SPACE, "append_tokens: message %d holds %d of %d reserved tokens, %d more do not fit",
                                (int)m, chain_len(c, m), chain_len(c, m), run_end - j);
                // a further extent: room for what this call still brings, at least the message's first reserve
                if ((int64_t)c->msgs.size() + (int64_t)fresh.size() >= c->cfg.max_messages)
                    return pc_fail(c, PC_ERR_NO_SPACE, "append_tokens: message table full (%d)", c->cfg.max_messages);
                const int32_t res = std::max(run_end - j, std::max<int32_t>(PC_SLOT_ALIGN, c->msgs[(size_t)m].reserve));
                int64_t start = 0;
                if (!take_slots(spans, next, c->slots, res, start))
                    return pc_fail(c, PC_ERR_NO_SPACE, "append_tokens: no room for a further extent of %d slots for message %d", res, (int)m);
                close_extent(j);
                const int32_t id = first_new + (int32_t)fresh.size();
                HostMsg ext{start, 0, res, base + len, true};
                ext.is_ext = true;
                fresh.push_back(ext);
                links.push_back({rec, id});
                rec = id; len = 0; reserve = res; base = ext.base_pos; slot = start;
                first_item = j;
            }
            items[(size_t)j] = PcTokenItem{rec, (int32_t)(slot + len), base + len, 0};
            len += 1;
        }
        close_extent(run_end);
    }
    if (!c->host_only && defer && fresh.empty()) {
        defer->swap(items);
    } else if (!c->host_only) {
        for (const HostMsg &rec : fresh) clear_if_reused(c, rec.slot_start, rec.reserve, st);
        if (!fresh.empty()) {                                // the device table learns the new extents (length 0 until the kernel sets it)
            StageSlot *slot = nullptr;
            const int32_t rc = pc_stage_acquire(c, sizeof(PcMsgEntry) * fresh.size(), &slot);
            if (rc != PC_OK) return rc;
            PcMsgEntry *en = (PcMsgEntry *)slot->host;
            for (size_t r = 0; r < fresh.size(); ++r) en[r] = PcMsgEntry{(int32_t)fresh[r].slot_start, 0, fresh[r].base_pos, 0};
            PC_HIP(c, hipMemcpyAsync(c->table_dev + first_new, slot->host, sizeof(PcMsgEntry) * fresh.size(), hipMemcpyHostToDevice, st));
            PC_HIP(c, hipEventRecord(slot->ev, st));
            slot->used = true;
        }
        if (n <= PC_TOKEN_PACK) {                            // a decode step's handful of tokens rides in the kernel arguments
            PcTokenPack pack;
            std::memcpy(pack.it, items.data(), sizeof(PcTokenItem) * (size_t)n);
            ProfScope ps(c, 0, st);
            pc_launch_append_tokens_packed(c->cfg.dtype, pack, n, k, v, c->cfg.n_kv_heads, c->D, c->slots, c->inv_freq_dev,
                                           c->k_store, c->v_store, c->table_dev, st);
            PC_HIP(c, hipGetLastError());
        } else {
            const int32_t rc = pc_stage_items(c, items.data(), sizeof(PcTokenItem) * (size_t)n, st);
            if (rc != PC_OK) return rc;
            ProfScope ps(c, 0, st);
            pc_launch_append_tokens(c->cfg.dtype, (const PcTokenItem *)c->tok_dev, n, k, v, c->cfg.n_kv_heads, c->D, c->slots, c->inv_freq_dev,
                                    c->k_store, c->v_store, c->table_dev, st);
            PC_HIP(c, hipGetLastError());
        }
    }
    for (const HostMsg &rec : fresh) {
        if (!c->msgs.empty() && rec.slot_start < c->msgs.back().slot_start) c->slots_in_id_order = false;
        c->msgs.push_back(rec);
    }
    for (const auto &lk : links) c->msgs[(size_t)lk.first].next = lk.second;
    for (const auto &g : grown) c->msgs[(size_t)g.first].len = g.second;
    c->free_spans.swap(spans);
    c->next_slot = next;
    return PC_OK;
}

int32_t pc_append_tokens(pc_cache *c, int32_t msg_id, const void *k, const void *v, int32_t n, void *stream)
{
    if (!c) return PC_ERR_INVALID_ARG;
    if (!known(c, msg_id)) return pc_fail(c, PC_ERR_BAD_MSG_ID, "append_tokens: unknown message %d", msg_id);
    if (n < 1) return pc_fail(c, PC_ERR_INVALID_ARG, "append_tokens: n = %d must be >= 1", n);
    if (!c->host_only && (!k || !v)) return pc_fail(c, PC_ERR_INVALID_ARG, "append_tokens: null k or v");
    return pc_append_token_items(c, std::vector<int32_t>((size_t)n, msg_id), k, v, (hipStream_t)stream, nullptr);
}

int32_t pc_check_token_batch(pc_cache *c, const int32_t *msg_ids, int32_t n_msgs, const void *k, const void *v)
{
    if (n_msgs < 0 || (n_msgs > 0 && !msg_ids)) return pc_fail(c, PC_ERR_INVALID_ARG, "append_tokens_batch: bad id list");
    if (n_msgs == 0) return PC_OK;
    if (!c->host_only && (!k || !v)) return pc_fail(c, PC_ERR_INVALID_ARG, "append_tokens_batch: null k or v");
    for (int j = 0; j < n_msgs; ++j)
        if (!known(c, msg_ids[j])) return pc_fail(c, PC_ERR_BAD_MSG_ID, "append_tokens_batch: unknown message %d", msg_ids[j]);
    std::vector<int32_t> sorted(msg_ids, msg_ids + n_msgs);
    std::sort(sorted.begin(), sorted.end());
    const auto twice = std::adjacent_find(sorted.begin(), sorted.end());
    if (twice != sorted.end()) return pc_fail(c, PC_ERR_INVALID_ARG, "append_tokens_batch: message %d listed twice", *twice);
    return PC_OK;
}

int32_t pc_append_tokens_batch(pc_cache *c, const int32_t *msg_ids, int32_t n_msgs, const void *k, const void *v, void *stream)
{
    if (!c) return PC_ERR_INVALID_ARG;
    const int32_t rc = pc_check_token_batch(c, msg_ids, n_msgs, k, v);
    if (rc != PC_OK || n_msgs == 0) return rc;
    return pc_append_token_items(c, std::vector<int32_t>(msg_ids, msg_ids + n_msgs), k, v, (hipStream_t)stream, nullptr);
}

int32_t pc_message_info(pc_cache *c, int32_t msg_id, int32_t *len, int64_t *slot_start, int32_t *reserved)
{
    if (!c) return PC_ERR_INVALID_ARG;
    if (!known(c, msg_id)) return pc_fail(c, PC_ERR_BAD_MSG_ID, "unknown message %d", msg_id);
    if (len) *len = chain_len(c, msg_id);
    if (slot_start) *slot_start = c->msgs[msg_id].slot_start;
    if (reserved) {
        int32_t r = 0;
        for (int32_t e = msg_id; e >= 0; e = c->msgs[(size_t)e].next) r += c->msgs[(size_t)e].reserve;
        *reserved = r;
    }
    return PC_OK;
}

int32_t pc_message_extents(pc_cache *c, int32_t msg_id, int32_t *n_extents, int64_t *slot_starts, int32_t *lens, int32_t cap)
{
    if (!c) return PC_ERR_INVALID_ARG;
    if (!known(c, msg_id)) return pc_fail(c, PC_ERR_BAD_MSG_ID, "unknown message %d", msg_id);
    int32_t n = 0;
    for (int32_t e = msg_id; e >= 0; e = c->msgs[(size_t)e].next, ++n)
        if (n < cap) {
            if (slot_starts) slot_starts[n] = c->msgs[(size_t)e].slot_start;
            if (lens) lens[n] = c->msgs[(size_t)e].len;
        }
    if (n_extents) *n_extents = n;
    return PC_OK;
}

int32_t pc_message_base(pc_cache *c, int32_t msg_id, int32_t *base_pos)
{
    if (!c) return PC_ERR_INVALID_ARG;
    if (!known(c, msg_id)) return pc_fail(c, PC_ERR_BAD_MSG_ID, "unknown message %d", msg_id);
    if (base_pos) *base_pos = c->msgs[msg_id].base_pos;
    return PC_OK;
}

int32_t pc_reposition_batch(pc_cache *c, const int32_t *msg_ids, const int32_t *new_bases, int32_t n_msgs, void *stream);

int32_t pc_reposition(pc_cache *c, int32_t msg_id, int32_t new_base, void *stream)
{
    if (!c) return PC_ERR_INVALID_ARG;
    if (!known(c, msg_id)) return pc_fail(c, PC_ERR_BAD_MSG_ID, "reposition: unknown message %d", msg_id);
    if (new_base > c->cfg.max_position || new_base < -c->cfg.max_position)
        return pc_fail(c, PC_ERR_INVALID_ARG, "reposition: position %d outside [-%d, %d]", new_base, c->cfg.max_position,
                    c->cfg.max_position);
    if (c->msgs[(size_t)msg_id].next >= 0) return pc_reposition_batch(c, &msg_id, &new_base, 1, stream);   // every extent moves
    HostMsg &m = c->msgs[(size_t)msg_id];
    const int64_t delta = (int64_t)new_base - m.base_pos;
    if (delta == 0) return PC_OK;
    if (!c->host_only) {
        hipStream_t st = (hipStream_t)stream;
        ProfScope ps(c, 7, st);
        pc_launch_reposition(c->cfg.dtype, m.len, c->cfg.n_kv_heads, c->D, m.slot_start, c->slots, (int)delta, new_base,
                             c->inv_freq_dev, c->k_store, c->table_dev, msg_id, st);
        PC_HIP(c, hipGetLastError());
    }
    m.base_pos = new_base;
    return PC_OK;
}

int32_t pc_reposition_batch(pc_cache *c, const int32_t *msg_ids, const int32_t *new_bases, int32_t n_msgs, void *stream)
{
    if (!c) return PC_ERR_INVALID_ARG;
    if (n_msgs < 0 || (n_msgs > 0 && (!msg_ids || !new_bases))) return pc_fail(c, PC_ERR_INVALID_ARG, "reposition_batch: bad lists");
    std::vector<PcMoveItem> items;
    std::vector<char> listed(c->msgs.size(), 0);
    for (int j = 0; j < n_msgs; ++j) {
        const int32_t m = msg_ids[j];
        if (!known(c, m)) return pc_fail(c, PC_ERR_BAD_MSG_ID, "reposition_batch: unknown message %d", m);
        if (listed[(size_t)m]) return pc_fail(c, PC_ERR_INVALID_ARG, "reposition_batch: message %d listed twice", m);
        listed[(size_t)m] = 1;
        if (new_bases[j] > c->cfg.max_position || new_bases[j] < -c->cfg.max_position)
            return pc_fail(c, PC_ERR_INVALID_ARG, "reposition_batch: position %d outside [-%d, %d]", new_bases[j],
                        c->cfg.max_position, c->cfg.max_position);
        const int64_t delta = (int64_t)new_bases[j] - c->msgs[(size_t)m].base_pos;
        if (delta != 0)
            for (int32_t r = m; r >= 0; r = c->msgs[(size_t)r].next) {          // every extent turns by the same angle
                const HostMsg &hm = c->msgs[(size_t)r];
                items.push_back(PcMoveItem{r, (int32_t)hm.slot_start, hm.len, (int32_t)delta, (int32_t)(hm.base_pos + delta), {0, 0, 0}});
            }
    }
    if (!items.empty() && !c->host_only) {
        hipStream_t st = (hipStream_t)stream;
        const int32_t rc = pc_stage_items(c, items.data(), sizeof(PcMoveItem) * items.size(), st);
        if (rc != PC_OK) return rc;
        ProfScope ps(c, 7, st);
        pc_launch_reposition_batch(c->cfg.dtype, (const PcMoveItem *)c->tok_dev, (int)items.size(), c->cfg.n_kv_heads, c->D,
                                   c->slots, c->inv_freq_dev, c->k_store, c->table_dev, st);
        PC_HIP(c, hipGetLastError());
    }
    for (const PcMoveItem &it : items) c->msgs[(size_t)it.msg].base_pos = it.new_base;
    return PC_OK;
}

// gives a span of slots back: sorted insert, merge with its neighbours, shrink the used region
static void release_span(pc_cache *c, FreeSpan f)
{
    c->dirty_end = std::max(c->dirty_end, f.start + f.size);
    auto &fs = c->free_spans;
    size_t i = 0;
    while (i < fs.size() && fs[i].start < f.start) ++i;
    fs.insert(fs.begin() + (long)i, f);
    if (i + 1 < fs.size() && fs[i].start + fs[i].size == fs[i + 1].start) {           // merge with the span behind
        fs[i].size += fs[i + 1].size;
        fs.erase(fs.begin() + (long)i + 1);
    }
    if (i > 0 && fs[i - 1].start + fs[i - 1].size == fs[i].start) {                   // ... and the one in front
        fs[i - 1].size += fs[i].size;
        fs.erase(fs.begin() + (long)i);
    }
    if (!fs.empty() && fs.back().start + fs.back().size == c->next_slot) {            // freed at the end: the used region shrinks
        c->next_slot = fs.back().start;
        fs.pop_back();
    }
}

int32_t pc_message_free(pc_cache *c, int32_t msg_id)
{
    if (!c) return PC_ERR_INVALID_ARG;
    if (!known(c, msg_id)) return pc_fail(c, PC_ERR_BAD_MSG_ID, "free: unknown message %d", msg_id);
    for (int32_t r = msg_id; r >= 0; r = c->msgs[(size_t)r].next) {
        HostMsg &m = c->msgs[(size_t)r];
        m.live = false;
        release_span(c, FreeSpan{m.slot_start, (int64_t)align_up((size_t)m.reserve, PC_SLOT_ALIGN)});
    }
    return PC_OK;
}

// ---- swap: a message's stored K and V leave the cache as one blob and come back later -----------
static inline bool swapped_out(const pc_cache *c, int32_t m) { return m >= 0 && m < (int32_t)c->msgs.size() && c->msgs[(size_t)m].swapped; }

int64_t pc_message_swap_bytes(pc_cache *c, int32_t msg_id)
{
    if (!c) return PC_ERR_INVALID_ARG;
    if ((!known(c, msg_id) && !swapped_out(c, msg_id)) || c->msgs[(size_t)msg_id].is_ext)
        return pc_fail(c, PC_ERR_BAD_MSG_ID, "swap_bytes: unknown message %d", msg_id);
    int64_t span = 0;                                    // every extent's reserved span, one after the other
    for (int32_t r = msg_id; r >= 0; r = c->msgs[(size_t)r].next) span += (int64_t)align_up((size_t)c->msgs[(size_t)r].reserve, PC_SLOT_ALIGN);
    return 2 * span * c->cfg.n_kv_heads * c->D * (int64_t)c->esize;
}

// the span [slot_start, slot_start + span) of every KV head, K heads first then V heads; both stores keep a
// head's slots contiguous (V in groups of 8 slots, and spans are multiples of 32), so each is one strided copy
static int32_t copy_span(pc_cache *c, int64_t slot_start, int64_t span, void *blob, bool out, hipStream_t st)
{
    const size_t row = (size_t)span * (size_t)c->D * c->esize;                 // one head's share of the span
    const size_t pitch = (size_t)c->slots * (size_t)c->D * c->esize;           // one head's share of the store
    const size_t at = (size_t)slot_start * (size_t)c->D * c->esize;
    char *bk = (char *)blob, *bv = bk + row * (size_t)c->cfg.n_kv_heads;
    char *sk = (char *)c->k_store + at, *sv = (char *)c->v_store + at;
    if (out) {
        PC_HIP(c, hipMemcpy2DAsync(bk, row, sk, pitch, row, (size_t)c->cfg.n_kv_heads, hipMemcpyDefault, st));
        PC_HIP(c, hipMemcpy2DAsync(bv, row, sv, pitch, row, (size_t)c->cfg.n_kv_heads, hipMemcpyDefault, st));
    } else {
        PC_HIP(c, hipMemcpy2DAsync(sk, pitch, bk, row, row, (size_t)c->cfg.n_kv_heads, hipMemcpyDefault, st));
        PC_HIP(c, hipMemcpy2DAsync(sv, pitch, bv, row, row, (size_t)c->cfg.n_kv_heads, hipMemcpyDefault, st));
    }
    return PC_OK;
}

int32_t pc_message_swap_out(pc_cache *c, int32_t msg_id, void *blob, void *stream)
{
    if (!c) return PC_ERR_INVALID_ARG;
    if (!known(c, msg_id)) return pc_fail(c, PC_ERR_BAD_MSG_ID, "swap_out: unknown message %d", msg_id);
    if (!c->host_only && !blob) return pc_fail(c, PC_ERR_INVALID_ARG, "swap_out: null blob");
    const size_t per_slot = 2 * (size_t)c->cfg.n_kv_heads * (size_t)c->D * c->esize;
    if (!c->host_only) {
        char *at = (char *)blob;
        for (int32_t r = msg_id; r >= 0; r = c->msgs[(size_t)r].next) {
            const HostMsg &m = c->msgs[(size_t)r];
            const int64_t span = (int64_t)align_up((size_t)m.reserve, PC_SLOT_ALIGN);
            const int32_t rc = copy_span(c, m.slot_start, span, at, true, (hipStream_t)stream);
            if (rc != PC_OK) return rc;
            at += (size_t)span * per_slot;
        }
    }
    for (int32_t r = msg_id; r >= 0; r = c->msgs[(size_t)r].next) {
        HostMsg &m = c->msgs[(size_t)r];
        m.live = false; m.swapped = true;
        release_span(c, FreeSpan{m.slot_start, (int64_t)align_up((size_t)m.reserve, PC_SLOT_ALIGN)});
    }
    return PC_OK;
}

int32_t pc_message_swap_in(pc_cache *c, int32_t msg_id, const void *blob, void *stream)
{
    if (!c) return PC_ERR_INVALID_ARG;
    if (!swapped_out(c, msg_id) || c->msgs[(size_t)msg_id].is_ext)
        return pc_fail(c, PC_ERR_BAD_MSG_ID, "swap_in: message %d is not swapped out", msg_id);
    if (!c->host_only && !blob) return pc_fail(c, PC_ERR_INVALID_ARG, "swap_in: null blob");
    // slots for every extent first: all or nothing
    std::vector<FreeSpan> spans = c->free_spans;
    int64_t next = c->next_slot;
    std::vector<std::pair<int32_t, int64_t>> placed;      // (record, new slot_start)
    for (int32_t r = msg_id; r >= 0; r = c->msgs[(size_t)r].next) {
        int64_t start = 0;
        if (!take_slots(spans, next, c->slots, c->msgs[(size_t)r].reserve, start))
            return pc_fail(c, PC_ERR_NO_SPACE, "swap_in: message %d does not fit (an extent of %d slots), capacity %lld", msg_id,
                        c->msgs[(size_t)r].reserve, (long long)c->slots);
        placed.push_back({r, start});
    }
    if (!c->host_only) {
        hipStream_t st = (hipStream_t)stream;
        const size_t per_slot = 2 * (size_t)c->cfg.n_kv_heads * (size_t)c->D * c->esize;
        const char *at = (const char *)blob;
        for (const auto &pl : placed) {
            const HostMsg &m = c->msgs[(size_t)pl.first];
            const int64_t span = (int64_t)align_up((size_t)m.reserve, PC_SLOT_ALIGN);
            int32_t rc = copy_span(c, pl.second, span, const_cast<char *>(at), false, st);
            if (rc != PC_OK) return rc;
            at += (size_t)span * per_slot;
            // the device table learns where the extent lives now
            StageSlot *slot = nullptr;
            rc = pc_stage_acquire(c, sizeof(PcMsgEntry), &slot);
            if (rc != PC_OK) return rc;
            const PcMsgEntry en{(int32_t)pl.second, m.len, m.base_pos, 0};
            std::memcpy(slot->host, &en, sizeof en);
            PC_HIP(c, hipMemcpyAsync(c->table_dev + pl.first, slot->host, sizeof en, hipMemcpyHostToDevice, st));
            PC_HIP(c, hipEventRecord(slot->ev, st));
            slot->used = true;
        }
    }
    for (const auto &pl : placed) {
        HostMsg &m = c->msgs[(size_t)pl.first];
        m.slot_start = pl.second; m.live = true; m.swapped = false;
    }
    c->slots_in_id_order = false;                       // an old id may now sit behind newer ones
    c->free_spans.swap(spans);
    c->next_slot = next;
    return PC_OK;
}

int32_t pc_cache_info(pc_cache *c, int32_t *n_messages, int64_t *slots_used, int64_t *capacity_slots)
{
    if (!c) return PC_ERR_INVALID_ARG;
    if (n_messages) *n_messages = (int32_t)c->msgs.size();
    if (slots_used) *slots_used = c->next_slot;
    if (capacity_slots) *capacity_slots = c->slots;
    return PC_OK;
}

int32_t pc_profile_enable(pc_cache *c, int32_t on)
{
    if (!c) return PC_ERR_INVALID_ARG;
    if (c->host_only) return pc_fail(c, PC_ERR_INVALID_ARG, "profiling needs a device cache");
    c->prof = on != 0;
    return PC_OK;
}

int32_t pc_profile_read(pc_cache *c, double ms_total[PC_N_KERNEL_CLASSES], int64_t launches[PC_N_KERNEL_CLASSES], int32_t reset)
{
    if (!c) return PC_ERR_INVALID_ARG;
    if (c->host_only) return pc_fail(c, PC_ERR_INVALID_ARG, "profiling needs a device cache");
    pc_prof_collect(c);
    for (int i = 0; i < PC_N_KERNEL_CLASSES; ++i) {
        if (ms_total) ms_total[i] = c->prof_ms[i];
        if (launches) launches[i] = c->prof_n[i];
        if (reset) { c->prof_ms[i] = 0; c->prof_n[i] = 0; }
    }
    return PC_OK;
}

int32_t pc_set_decode_sharing(pc_cache *c, int32_t mode)
{
    if (!c || mode < 0 || mode > 2) return PC_ERR_INVALID_ARG;
    c->decode_sharing = mode;
    return PC_OK;
}

int32_t pc_set_key_gather(pc_cache *c, int32_t mode)
{
    if (!c || mode < 0 || mode > 2) return PC_ERR_INVALID_ARG;
    c->key_gather = mode;
    return PC_OK;
}

int32_t pc_set_tuning(pc_cache *c, int32_t decode_tiles_per_split, int32_t prefill_tiles_per_split)
{
    if (!c || decode_tiles_per_split < 0 || prefill_tiles_per_split < 0) return PC_ERR_INVALID_ARG;
    c->decode_tiles_per_split = decode_tiles_per_split;
    c->prefill_tiles_per_split = prefill_tiles_per_split;
    return PC_OK;
}

}  // extern "C"
