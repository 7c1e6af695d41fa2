// Host side of the library: message table, slot allocator, validation, position
// resolution, work-item planning, staging and kernel launches.
#include "../../include/pc.h"
#include "pc_kernels.h"

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <string>
#include <vector>

namespace {

// One extent of a message.  A message is a chain of extents: the record under the message's id, then the
// records it grew into once its reserve was used up (PC_FLAG_GROW_EXTENTS); those sit in the same table under
// ids no caller is given.  base_pos of an extent = base of the message + tokens in the extents before it.
struct HostMsg { int64_t slot_start; int32_t len; int32_t reserve; int32_t base_pos; bool live; bool swapped = false;
                 int32_t next = -1; bool is_ext = false; };
struct FreeSpan { int64_t start, size; };            // freed slots, multiples of PC_SLOT_ALIGN

struct StageSlot { void *host = nullptr; size_t cap = 0; hipEvent_t ev = nullptr; bool used = false; };

struct ProfRec { int cls; hipEvent_t a, b; };

constexpr int N_STAGE = 4;
constexpr int MAX_SPLITS = 128;

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

}  // namespace

struct pc_cache {
    pc_config cfg;
    bool host_only = false;
    bool grow_extents = false;
    int D = 0, half = 0, g = 0;
    int64_t slots = 0;
    size_t esize = 0;
    float scale = 0.f;
    std::vector<HostMsg> msgs;
    std::vector<FreeSpan> free_spans;                // sorted by start, neighbours merged, none touches next_slot
    int64_t next_slot = 0;
    bool slots_in_id_order = true;                   // no message was ever placed in a freed span: ids ascend with slots
    // device
    void *storage = nullptr; bool owns_storage = false;
    void *k_store = nullptr, *v_store = nullptr;
    PcMsgEntry *table_dev = nullptr;
    double *inv_freq_dev = nullptr;
    void *ws = nullptr; size_t ws_cap = 0;
    void *tok_dev = nullptr; size_t tok_cap = 0;          // staged items of pc_append_tokens* / pc_reposition_batch (bytes)
    StageSlot stage[N_STAGE]; int stage_next = 0;
    // profiling
    bool prof = false;
    std::vector<ProfRec> prof_recs;
    std::vector<hipEvent_t> ev_pool;
    double prof_ms[PC_N_KERNEL_CLASSES] = {0};
    int64_t prof_n[PC_N_KERNEL_CLASSES] = {0};
    // tuning
    int decode_tiles_per_split = 0, prefill_tiles_per_split = 0;
    int decode_sharing = 0;                            // 0 auto, 1 never, 2 whenever possible
    std::string err;
};

namespace {

int32_t fail(pc_cache *c, int32_t code, const char *fmt, ...)
{
    if (c) {
        char buf[512];
        va_list ap; va_start(ap, fmt); vsnprintf(buf, sizeof buf, fmt, ap); va_end(ap);
        c->err = buf;
    }
    return code;
}

#define PC_HIP(c, expr)                                                                        \
    do { hipError_t e_ = (expr);                                                               \
         if (e_ != hipSuccess) return fail((c), PC_ERR_HIP, "%s: %s", #expr, hipGetErrorString(e_)); } while (0)

size_t storage_bytes(const pc_config *cfg)
{
    const int64_t slots = (int64_t)align_up((size_t)std::max<int64_t>(cfg->capacity_tokens, 1), PC_SLOT_ALIGN);
    const size_t es = cfg->dtype == PC_BF16 ? 2 : 4;
    return 2 * (size_t)slots * cfg->n_kv_heads * cfg->head_dim * es;
}

struct ProfScope {
    pc_cache *c; int cls; hipStream_t st; hipEvent_t a = nullptr, b = nullptr;
    ProfScope(pc_cache *c_, int cls_, hipStream_t st_) : c(c_), cls(cls_), st(st_) {
        if (!c->prof) return;
        auto get = [&]() { hipEvent_t e = nullptr;
            if (!c->ev_pool.empty()) { e = c->ev_pool.back(); c->ev_pool.pop_back(); }
            else if (hipEventCreate(&e) != hipSuccess) e = nullptr;
            return e; };
        a = get(); b = get();
        if (a) (void)hipEventRecord(a, st);
    }
    ~ProfScope() {
        if (!c->prof || !a || !b) return;
        (void)hipEventRecord(b, st);
        c->prof_recs.push_back({cls, a, b});
    }
};

void prof_collect(pc_cache *c)
{
    for (auto &r : c->prof_recs) {
        (void)hipEventSynchronize(r.b);
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, r.a, r.b) == hipSuccess) { c->prof_ms[r.cls] += ms; c->prof_n[r.cls] += 1; }
        c->ev_pool.push_back(r.a); c->ev_pool.push_back(r.b);
    }
    c->prof_recs.clear();
}

// ---- validated, resolved form of one call -------------------------------------------
struct Resolved {
    std::vector<int2> sel;        // (extent record, resolved start), the caller's entries expanded
    std::vector<int32_t> entry_start;   // resolved start of each entry of the caller's list
    int32_t self_msg = -1, self_start = 0, self_len = 0, n_q = 0;   // the new message's LAST extent
    int32_t msg_start = 0;        // resolved start of the new message's first token
    std::vector<int32_t> q_pos;
    int64_t n_kv = 0;
    int32_t tiles = 0;            // KV tiles incl. the new message
};

inline bool known(const pc_cache *c, int32_t m)
{
    return m >= 0 && m < (int32_t)c->msgs.size() && c->msgs[(size_t)m].live && !c->msgs[(size_t)m].is_ext;
}
inline int32_t chain_len(const pc_cache *c, int32_t m)
{
    int32_t n = 0;
    for (int32_t r = m; r >= 0; r = c->msgs[(size_t)r].next) n += c->msgs[(size_t)r].len;
    return n;
}
inline int32_t chain_last(const pc_cache *c, int32_t m)
{
    while (c->msgs[(size_t)m].next >= 0) m = c->msgs[(size_t)m].next;
    return m;
}

int32_t resolve_call(pc_cache *c, const pc_call *call, int idx, Resolved &out)
{
    if (!call) return fail(c, PC_ERR_INVALID_ARG, "call %d: null", idx);
    if (call->n_sel < 0 || (call->n_sel > 0 && !call->sel))
        return fail(c, PC_ERR_INVALID_ARG, "call %d: bad parent list", idx);
    if (call->n_q < 1) return fail(c, PC_ERR_INVALID_ARG, "call %d: n_q = %d must be >= 1", idx, call->n_q);
    const int64_t maxp = c->cfg.max_position;
    // a listed message becomes one (extent record, start) pair per extent that holds tokens
    out.sel.clear();
    out.sel.reserve((size_t)call->n_sel);
    out.entry_start.resize((size_t)call->n_sel);
    int64_t nxt = 0, n_kv = 0, tiles = 0;
    for (int e = 0; e < call->n_sel; ++e) {
        const int32_t m = call->sel[e].msg_id;
        if (!known(c, m)) return fail(c, PC_ERR_BAD_MSG_ID, "call %d: parent %d names unknown message %d", idx, e, m);
        const int64_t len = chain_len(c, m);
        const int64_t s = call->sel[e].start_pos == PC_POS_AUTO ? nxt : (int64_t)call->sel[e].start_pos;
        if (s < -maxp || s + len - 1 > maxp)
            return fail(c, PC_ERR_INVALID_ARG, "call %d: parent %d spans positions [%lld, %lld], limit is +-%lld", idx, e,
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
        if (!known(c, call->self_msg)) return fail(c, PC_ERR_BAD_MSG_ID, "call %d: new message id %d unknown", idx, call->self_msg);
        self_total = chain_len(c, call->self_msg);
        if (call->n_q > self_total)
            return fail(c, PC_ERR_SHAPE, "call %d: n_q = %d exceeds the new message's %lld tokens", idx, call->n_q, (long long)self_total);
        if (s_self < -maxp || s_self + self_total - 1 > maxp)
            return fail(c, PC_ERR_INVALID_ARG, "call %d: new message spans positions beyond +-%lld", idx, (long long)maxp);
        // The causal part lives in the message's last extent; the extents before it are seen whole by
        // every query row, like parents.
        const int32_t last = chain_last(c, call->self_msg);
        if (call->n_q > c->msgs[(size_t)last].len)
            return fail(c, PC_ERR_SHAPE, "call %d: the %d query rows must lie in the new message's last extent (%d tokens)", idx,
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
        return fail(c, PC_ERR_BAD_MSG_ID, "call %d: self_msg must be -1 or a message id", idx);
    } else if (s_self < -maxp || s_self + call->n_q - 1 > maxp) {
        return fail(c, PC_ERR_INVALID_ARG, "call %d: query positions beyond +-%lld", idx, (long long)maxp);
    }
    out.msg_start = (int32_t)s_self;
    if (out.self_msg < 0) out.self_start = (int32_t)s_self;
    out.n_q = call->n_q;
    out.q_pos.resize(call->n_q);
    const int64_t tok0 = out.self_msg >= 0 ? self_total - call->n_q : 0;
    for (int r = 0; r < call->n_q; ++r) {
        const int64_t p = call->q_pos ? (int64_t)call->q_pos[r] : s_self + tok0 + r;
        if (p < -maxp || p > maxp) return fail(c, PC_ERR_INVALID_ARG, "call %d: query position %lld beyond +-%lld", idx, (long long)p, (long long)maxp);
        out.q_pos[r] = (int32_t)p;
    }
    if (n_kv > INT32_MAX / 2) return fail(c, PC_ERR_SHAPE, "call %d: gathers %lld tokens, too many", idx, (long long)n_kv);
    out.n_kv = n_kv; out.tiles = (int32_t)tiles;
    return PC_OK;
}

int32_t ensure_ws(pc_cache *c, size_t bytes, hipStream_t st)
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

int32_t stage_acquire(pc_cache *c, size_t bytes, StageSlot **out)
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

// layout of the staged (host -> device) block and of the device-built block
struct PlanLayout {
    size_t calls, sel, q_pos, row_call, merge_rows, items_dec, items_pre, sh_groups, sh_segs, sh_items, sh_pos, h2d_bytes;
    size_t segs, seg_kvoff, rot_seg, rot_q, tiles, sh_rot, part_o, part_ml, row_scalar, total;
};

PlanLayout make_layout(int n_calls, int total_sel, int total_q, int total_seg, int n_dec, int n_pre,
                       int64_t part_rows, int64_t total_tiles, int H_q, int D,
                       size_t n_sh_groups = 0, size_t n_sh_segs = 0, size_t n_sh_items = 0, size_t n_sh_pos = 0)
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
    L.sh_groups = take(sizeof(PcShGroup) * std::max<size_t>(n_sh_groups, 1));
    L.sh_segs = take(sizeof(PcShSeg) * std::max<size_t>(n_sh_segs, 1));
    L.sh_items = take(sizeof(PcShItem) * std::max<size_t>(n_sh_items, 1));
    L.sh_pos = take(sizeof(int32_t) * std::max<size_t>(n_sh_pos, 1));
    L.h2d_bytes = o;
    L.segs = take(sizeof(PcSegment) * (size_t)std::max(total_seg, 1));
    L.seg_kvoff = take(sizeof(int32_t) * (size_t)std::max(total_seg, 1));
    L.rot_seg = take(sizeof(float2) * (size_t)std::max(total_seg, 1) * (D / 2));
    L.rot_q = take(sizeof(float2) * (size_t)std::max(total_q, 1) * (D / 2));
    L.tiles = take(sizeof(PcTile) * (size_t)std::max<int64_t>(total_tiles, 1));
    L.sh_rot = take(sizeof(float2) * std::max<size_t>(n_sh_pos, 1) * (D / 2));
    L.part_o = take(sizeof(uint16_t) * (size_t)std::max<int64_t>(part_rows, 1) * H_q * D);
    L.part_ml = take(sizeof(float) * (size_t)std::max<int64_t>(part_rows, 1) * H_q * 2);
    L.row_scalar = take(sizeof(float) * (size_t)std::max(total_q, 1) * H_q);      // one float per (row, head): the gradient path's Delta
    L.total = o;
    return L;
}

}  // namespace

// =====================================================================================
extern "C" {

size_t pc_cache_storage_bytes(const pc_config *cfg)
{
    if (!cfg || cfg->n_kv_heads <= 0 || cfg->head_dim <= 0) return 0;
    return storage_bytes(cfg);
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

    const size_t bytes = storage_bytes(cfg);
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
    if (hipDeviceSynchronize() != hipSuccess) return bail(PC_ERR_HIP);
    return PC_OK;
}

int32_t pc_cache_destroy(pc_cache *c)
{
    if (!c) return PC_ERR_INVALID_ARG;
    if (!c->host_only) {
        (void)hipDeviceSynchronize();
        prof_collect(c);
        for (auto e : c->ev_pool) (void)hipEventDestroy(e);
        for (auto &s : c->stage) { if (s.host) (void)hipHostFree(s.host); if (s.ev) (void)hipEventDestroy(s.ev); }
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

int32_t pc_append_message(pc_cache *c, const void *k, const void *v, int32_t len, int32_t reserve,
                          int32_t *msg_id, void *stream)
{
    if (!c) return PC_ERR_INVALID_ARG;
    if (len < 1) return fail(c, PC_ERR_INVALID_ARG, "append: len = %d must be >= 1", len);
    if (!c->host_only && (!k || !v)) return fail(c, PC_ERR_INVALID_ARG, "append: null k or v");
    if (!msg_id) return fail(c, PC_ERR_INVALID_ARG, "append: null msg_id");
    if ((int64_t)c->msgs.size() >= c->cfg.max_messages)
        return fail(c, PC_ERR_NO_SPACE, "append: message table full (%d)", c->cfg.max_messages);
    const int32_t res = std::max(reserve, len);
    // the bookkeeping changes only once the launch has been accepted
    std::vector<FreeSpan> spans = c->free_spans;
    int64_t next = c->next_slot, start = 0;
    if (!take_slots(spans, next, c->slots, res, start))
        return fail(c, PC_ERR_NO_SPACE, "append: needs slots [%lld, %lld), capacity %lld", (long long)c->next_slot,
                    (long long)(c->next_slot + res), (long long)c->slots);
    const int id = (int)c->msgs.size();
    if (!c->host_only) {
        hipStream_t st = (hipStream_t)stream;
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
static int32_t stage_items(pc_cache *c, const void *items, size_t bytes, hipStream_t st)
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
    const int32_t rc = stage_acquire(c, bytes, &slot);
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
    if (n < 0 || (n > 0 && (!lens || !msg_ids))) return fail(c, PC_ERR_INVALID_ARG, "append_messages: bad lists");
    if (n == 0) return PC_OK;
    if (!c->host_only && (!k || !v)) return fail(c, PC_ERR_INVALID_ARG, "append_messages: null k or v list");
    if ((int64_t)c->msgs.size() + n > c->cfg.max_messages)
        return fail(c, PC_ERR_NO_SPACE, "append_messages: message table full (%d)", c->cfg.max_messages);
    // all or nothing: allocate on copies first
    std::vector<FreeSpan> spans = c->free_spans;
    int64_t next = c->next_slot;
    std::vector<PcAppendItem> items((size_t)n);
    std::vector<HostMsg> fresh((size_t)n);
    int max_len = 0;
    for (int j = 0; j < n; ++j) {
        if (lens[j] < 1) return fail(c, PC_ERR_INVALID_ARG, "append_messages: message %d has len = %d", j, lens[j]);
        if (!c->host_only && (!k[j] || !v[j])) return fail(c, PC_ERR_INVALID_ARG, "append_messages: message %d has null k or v", j);
        const int32_t res = std::max(reserves ? reserves[j] : 0, lens[j]);
        int64_t start = 0;
        if (!take_slots(spans, next, c->slots, res, start))
            return fail(c, PC_ERR_NO_SPACE, "append_messages: message %d (%d slots) does not fit, capacity %lld", j, res,
                        (long long)c->slots);
        fresh[(size_t)j] = HostMsg{start, lens[j], res, 0, true};
        items[(size_t)j] = PcAppendItem{c->host_only ? nullptr : k[j], c->host_only ? nullptr : v[j],
                                        (int32_t)c->msgs.size() + j, (int32_t)start, lens[j], 0};
        max_len = std::max(max_len, lens[j]);
    }
    if (!c->host_only) {
        hipStream_t st = (hipStream_t)stream;
        const int32_t rc = stage_items(c, items.data(), sizeof(PcAppendItem) * (size_t)n, st);
        if (rc != PC_OK) return rc;
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
// (ids sorted by message with a message's tokens in order; validated by the callers)
static int32_t append_token_items(pc_cache *c, const std::vector<int32_t> &ids, const void *k, const void *v, hipStream_t st)
{
    const int n = (int)ids.size();
    std::vector<PcTokenItem> items((size_t)n);
    std::vector<int32_t> left(c->msgs.size(), 0);            // tokens of this call still to place, per message
    for (int j = 0; j < n; ++j) left[(size_t)ids[j]] += 1;
    // the extent each message is writing into, as it will be (nothing is committed before the launch is accepted)
    struct Cur { int32_t rec, len, reserve, base; int64_t slot; };
    std::vector<int32_t> cur_of(c->msgs.size(), -1);
    std::vector<Cur> cur;
    std::vector<HostMsg> fresh;                              // new extent records: ids msgs.size(), msgs.size() + 1, ...
    std::vector<std::pair<int32_t, int32_t>> links;          // (record, its new next)
    std::vector<FreeSpan> spans = c->free_spans;
    int64_t next = c->next_slot;
    const int32_t first_new = (int32_t)c->msgs.size();
    for (int j = 0; j < n; ++j) {
        const int32_t m = ids[j];
        if (cur_of[(size_t)m] < 0) {
            const int32_t last = chain_last(c, m);
            const HostMsg &hm = c->msgs[(size_t)last];
            cur_of[(size_t)m] = (int32_t)cur.size();
            cur.push_back(Cur{last, hm.len, hm.reserve, hm.base_pos, hm.slot_start});
        }
        Cur &cu = cur[(size_t)cur_of[(size_t)m]];
        if (cu.len == cu.reserve) {
            if (!c->grow_extents)
                return fail(c, PC_ERR_NO_SPACE, "append_tokens: message %d holds %d of %d reserved tokens, %d more do not fit",
                            (int)m, chain_len(c, m), chain_len(c, m), left[(size_t)m]);
            // a further extent: room for what this call still brings, at least the message's first reserve
            if ((int64_t)c->msgs.size() + (int64_t)fresh.size() >= c->cfg.max_messages)
                return fail(c, PC_ERR_NO_SPACE, "append_tokens: message table full (%d)", c->cfg.max_messages);
            const int32_t res = std::max(left[(size_t)m], std::max<int32_t>(PC_SLOT_ALIGN, c->msgs[(size_t)m].reserve));
            int64_t start = 0;
            if (!take_slots(spans, next, c->slots, res, start))
                return fail(c, PC_ERR_NO_SPACE, "append_tokens: no room for a further extent of %d slots for message %d", res, (int)m);
            const int32_t id = first_new + (int32_t)fresh.size();
            HostMsg rec{start, 0, res, cu.base + cu.len, true};
            rec.is_ext = true;
            fresh.push_back(rec);
            links.push_back({cu.rec, id});
            cu = Cur{id, 0, res, rec.base_pos, start};
        }
        items[(size_t)j] = PcTokenItem{cu.rec, (int32_t)(cu.slot + cu.len), cu.base + cu.len, 0};
        cu.len += 1;
        left[(size_t)m] -= 1;
    }
    // every item carries the final length of the extent it goes to
    std::vector<int32_t> final_len(c->msgs.size() + fresh.size(), 0);
    for (size_t r = 0; r < c->msgs.size(); ++r) final_len[r] = c->msgs[r].len;
    for (int j = 0; j < n; ++j) final_len[(size_t)items[(size_t)j].msg] += 1;
    for (int j = 0; j < n; ++j) items[(size_t)j].new_len = final_len[(size_t)items[(size_t)j].msg];
    if (!c->host_only) {
        if (!fresh.empty()) {                                // the device table learns the new extents (length 0 until the kernel sets it)
            StageSlot *slot = nullptr;
            const int32_t rc = stage_acquire(c, sizeof(PcMsgEntry) * fresh.size(), &slot);
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
            const int32_t rc = stage_items(c, items.data(), sizeof(PcTokenItem) * (size_t)n, st);
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
    for (size_t r = 0; r < c->msgs.size(); ++r) c->msgs[r].len = final_len[r];
    c->free_spans.swap(spans);
    c->next_slot = next;
    return PC_OK;
}

int32_t pc_append_tokens(pc_cache *c, int32_t msg_id, const void *k, const void *v, int32_t n, void *stream)
{
    if (!c) return PC_ERR_INVALID_ARG;
    if (!known(c, msg_id)) return fail(c, PC_ERR_BAD_MSG_ID, "append_tokens: unknown message %d", msg_id);
    if (n < 1) return fail(c, PC_ERR_INVALID_ARG, "append_tokens: n = %d must be >= 1", n);
    if (!c->host_only && (!k || !v)) return fail(c, PC_ERR_INVALID_ARG, "append_tokens: null k or v");
    return append_token_items(c, std::vector<int32_t>((size_t)n, msg_id), k, v, (hipStream_t)stream);
}

int32_t pc_append_tokens_batch(pc_cache *c, const int32_t *msg_ids, int32_t n_msgs, const void *k, const void *v, void *stream)
{
    if (!c) return PC_ERR_INVALID_ARG;
    if (n_msgs < 0 || (n_msgs > 0 && !msg_ids)) return fail(c, PC_ERR_INVALID_ARG, "append_tokens_batch: bad id list");
    if (n_msgs == 0) return PC_OK;
    if (!c->host_only && (!k || !v)) return fail(c, PC_ERR_INVALID_ARG, "append_tokens_batch: null k or v");
    std::vector<char> listed(c->msgs.size(), 0);
    for (int j = 0; j < n_msgs; ++j) {
        const int32_t m = msg_ids[j];
        if (!known(c, m)) return fail(c, PC_ERR_BAD_MSG_ID, "append_tokens_batch: unknown message %d", m);
        if (listed[(size_t)m]) return fail(c, PC_ERR_INVALID_ARG, "append_tokens_batch: message %d listed twice", m);
        listed[(size_t)m] = 1;
    }
    return append_token_items(c, std::vector<int32_t>(msg_ids, msg_ids + n_msgs), k, v, (hipStream_t)stream);
}

int32_t pc_resolve_call(pc_cache *c, const pc_call *call, int32_t *starts_out, int32_t *self_start_out, int64_t *n_kv)
{
    if (!c) return PC_ERR_INVALID_ARG;
    Resolved r;
    const int32_t rc = resolve_call(c, call, 0, r);
    if (rc != PC_OK) return rc;
    if (starts_out) for (size_t e = 0; e < r.entry_start.size(); ++e) starts_out[e] = r.entry_start[e];
    if (self_start_out) *self_start_out = r.msg_start;
    if (n_kv) *n_kv = r.n_kv;
    return PC_OK;
}

int32_t pc_message_info(pc_cache *c, int32_t msg_id, int32_t *len, int64_t *slot_start, int32_t *reserved)
{
    if (!c) return PC_ERR_INVALID_ARG;
    if (!known(c, msg_id)) return fail(c, PC_ERR_BAD_MSG_ID, "unknown message %d", msg_id);
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
    if (!known(c, msg_id)) return fail(c, PC_ERR_BAD_MSG_ID, "unknown message %d", msg_id);
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
    if (!known(c, msg_id)) return fail(c, PC_ERR_BAD_MSG_ID, "unknown message %d", msg_id);
    if (base_pos) *base_pos = c->msgs[msg_id].base_pos;
    return PC_OK;
}

int32_t pc_reposition_batch(pc_cache *c, const int32_t *msg_ids, const int32_t *new_bases, int32_t n_msgs, void *stream);

int32_t pc_reposition(pc_cache *c, int32_t msg_id, int32_t new_base, void *stream)
{
    if (!c) return PC_ERR_INVALID_ARG;
    if (!known(c, msg_id)) return fail(c, PC_ERR_BAD_MSG_ID, "reposition: unknown message %d", msg_id);
    if (new_base > c->cfg.max_position || new_base < -c->cfg.max_position)
        return fail(c, PC_ERR_INVALID_ARG, "reposition: position %d outside [-%d, %d]", new_base, c->cfg.max_position,
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
    if (n_msgs < 0 || (n_msgs > 0 && (!msg_ids || !new_bases))) return fail(c, PC_ERR_INVALID_ARG, "reposition_batch: bad lists");
    std::vector<PcMoveItem> items;
    std::vector<char> listed(c->msgs.size(), 0);
    for (int j = 0; j < n_msgs; ++j) {
        const int32_t m = msg_ids[j];
        if (!known(c, m)) return fail(c, PC_ERR_BAD_MSG_ID, "reposition_batch: unknown message %d", m);
        if (listed[(size_t)m]) return fail(c, PC_ERR_INVALID_ARG, "reposition_batch: message %d listed twice", m);
        listed[(size_t)m] = 1;
        if (new_bases[j] > c->cfg.max_position || new_bases[j] < -c->cfg.max_position)
            return fail(c, PC_ERR_INVALID_ARG, "reposition_batch: position %d outside [-%d, %d]", new_bases[j],
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
        const int32_t rc = stage_items(c, items.data(), sizeof(PcMoveItem) * items.size(), st);
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
    if (!known(c, msg_id)) return fail(c, PC_ERR_BAD_MSG_ID, "free: unknown message %d", msg_id);
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
        return fail(c, PC_ERR_BAD_MSG_ID, "swap_bytes: unknown message %d", msg_id);
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
    if (!known(c, msg_id)) return fail(c, PC_ERR_BAD_MSG_ID, "swap_out: unknown message %d", msg_id);
    if (!c->host_only && !blob) return fail(c, PC_ERR_INVALID_ARG, "swap_out: null blob");
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
        return fail(c, PC_ERR_BAD_MSG_ID, "swap_in: message %d is not swapped out", msg_id);
    if (!c->host_only && !blob) return fail(c, PC_ERR_INVALID_ARG, "swap_in: null blob");
    // slots for every extent first: all or nothing
    std::vector<FreeSpan> spans = c->free_spans;
    int64_t next = c->next_slot;
    std::vector<std::pair<int32_t, int64_t>> placed;      // (record, new slot_start)
    for (int32_t r = msg_id; r >= 0; r = c->msgs[(size_t)r].next) {
        int64_t start = 0;
        if (!take_slots(spans, next, c->slots, c->msgs[(size_t)r].reserve, start))
            return fail(c, PC_ERR_NO_SPACE, "swap_in: message %d does not fit (an extent of %d slots), capacity %lld", msg_id,
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
            rc = stage_acquire(c, sizeof(PcMsgEntry), &slot);
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
    if (c->host_only) return fail(c, PC_ERR_INVALID_ARG, "profiling needs a device cache");
    c->prof = on != 0;
    return PC_OK;
}

int32_t pc_profile_read(pc_cache *c, double ms_total[PC_N_KERNEL_CLASSES], int64_t launches[PC_N_KERNEL_CLASSES], int32_t reset)
{
    if (!c) return PC_ERR_INVALID_ARG;
    if (c->host_only) return fail(c, PC_ERR_INVALID_ARG, "profiling needs a device cache");
    prof_collect(c);
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

int32_t pc_set_tuning(pc_cache *c, int32_t decode_tiles_per_split, int32_t prefill_tiles_per_split)
{
    if (!c || decode_tiles_per_split < 0 || prefill_tiles_per_split < 0) return PC_ERR_INVALID_ARG;
    c->decode_tiles_per_split = decode_tiles_per_split;
    c->prefill_tiles_per_split = prefill_tiles_per_split;
    return PC_OK;
}

// -------------------------------------------------------------------------------------
// shared by pc_attend and pc_build_tables: validate, plan, stage, run the plan builder
// -------------------------------------------------------------------------------------
struct Planned {
    PlanLayout lay;
    int n_calls = 0, total_sel = 0, total_q = 0, total_seg = 0, n_dec = 0, n_pre = 0, pre_waves = 4;
    int n_merge_rows = 0;
    int n_sh_items = 0;
    size_t n_sh_pos = 0;
    std::vector<Resolved> res;
};

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

static int32_t plan_and_stage(pc_cache *c, const pc_call *calls, int32_t n_calls, bool want_items,
                              hipStream_t st, Planned &P)
{
    P.n_calls = n_calls;
    P.res.resize((size_t)n_calls);
    for (int i = 0; i < n_calls; ++i) {
        const int32_t rc = resolve_call(c, &calls[i], i, P.res[i]);
        if (rc != PC_OK) return rc;
        P.total_q += P.res[i].n_q;
    }
    const int g = c->g, H_kv = c->cfg.n_kv_heads;
    const bool bf16 = c->cfg.dtype == PC_BF16;
    // work-group shape of the prefill kernel: 8 row units (32 rows x 1 q head each) per group
    P.pre_waves = 8;
    std::vector<PcCallDesc> cds((size_t)n_calls);
    std::vector<PcItem> dec, pre;
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
                dec.push_back(it);
            }
        } else {
            const int units = ((r.n_q + 31) / 32) * g;
            const int groups = (units + P.pre_waves - 1) / P.pre_waves;
            int ns = 1;
            if (c->prefill_tiles_per_split > 0) ns = (T + c->prefill_tiles_per_split - 1) / c->prefill_tiles_per_split;
            else if (pre_groups < 256) ns = (int)std::min<int64_t>((256 + pre_groups - 1) / pre_groups, std::max(1, T / 16));
            ns = std::max(1, std::min(MAX_SPLITS, ns));
            const int chunk = std::max(1, (T + ns - 1) / ns);
            ns = std::max(1, (T + chunk - 1) / chunk);
            cd.n_splits = ns;
            // A group of row units walks the parents' tiles and the tiles of the new message up to the
            // causal limit of its last row; its splits divide THAT count evenly, so the groups with
            // early rows do not end up with a nearly empty last split.
            const int self_tiles = r.self_msg >= 0 ? (r.self_len + PC_TILE - 1) / PC_TILE : 0;
            const int parent_tiles = T - self_tiles;
            for (int gidx = 0; gidx < groups; ++gidx) {
                int Tg = T;
                if (r.self_msg >= 0) {
                    const int last_unit = std::min(gidx * P.pre_waves + P.pre_waves - 1, units - 1);
                    const int lim = (r.self_len - r.n_q) + std::min(32 * (last_unit / g) + 31, r.n_q - 1);   // last own token seen
                    Tg = parent_tiles + std::min(self_tiles, lim / PC_TILE + 1);
                }
                const int chunk_g = std::max(1, (Tg + ns - 1) / ns);
                for (int s = 0; s < ns; ++s) {
                    PcItem it{}; it.call = i; it.unit0 = gidx * P.pre_waves; it.split = s;
                    it.tile_begin = std::min(Tg, s * chunk_g);
                    it.tile_end = s == ns - 1 ? T : std::min(Tg, (s + 1) * chunk_g);
                    pre.push_back(it);
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
    if (part_rows > INT32_MAX) return fail(c, PC_ERR_SHAPE, "attend: partial buffer too large");
    P.total_sel = sel_off; P.total_seg = seg_off;
    P.n_dec = (int)dec.size(); P.n_pre = (int)pre.size();
    P.n_sh_items = (int)sp.items.size(); P.n_sh_pos = sp.pos.size();
    if (total_tiles > INT32_MAX / 2) return fail(c, PC_ERR_SHAPE, "attend: too many KV tiles");
    if (sp.pos.size() > (size_t)INT32_MAX / 2) return fail(c, PC_ERR_SHAPE, "attend: shared decode table too large");
    P.lay = make_layout(n_calls, P.total_sel, P.total_q, P.total_seg, P.n_dec, P.n_pre, part_rows, total_tiles, c->cfg.n_q_heads, c->D,
                        sp.groups.size(), sp.segs.size(), sp.items.size(), sp.pos.size());
    if (c->host_only) return PC_OK;

    int32_t rc = ensure_ws(c, P.lay.total, st);
    if (rc != PC_OK) return rc;
    StageSlot *slot = nullptr;
    rc = stage_acquire(c, P.lay.h2d_bytes, &slot);
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
        if (cds[i].n_splits > 1)
            for (int q = 0; q < r.n_q; ++q) hm[P.n_merge_rows++] = PcMergeRow{cds[i].q_off + q, cds[i].part_off + q, cds[i].n_splits, r.n_q};
    }
    for (const PcShGroup &gr : sp.groups)
        if (gr.n_splits > 1)
            for (int q = 0; q < gr.n_rows; ++q) hm[P.n_merge_rows++] = PcMergeRow{gr.row0 + q, gr.part_off + q, gr.n_splits, gr.n_rows};
    if (!dec.empty()) std::memcpy(h + P.lay.items_dec, dec.data(), sizeof(PcItem) * dec.size());
    if (!pre.empty()) std::memcpy(h + P.lay.items_pre, pre.data(), sizeof(PcItem) * pre.size());
    if (!sp.items.empty()) {
        std::memcpy(h + P.lay.sh_groups, sp.groups.data(), sizeof(PcShGroup) * sp.groups.size());
        std::memcpy(h + P.lay.sh_segs, sp.segs.data(), sizeof(PcShSeg) * sp.segs.size());
        std::memcpy(h + P.lay.sh_items, sp.items.data(), sizeof(PcShItem) * sp.items.size());
        std::memcpy(h + P.lay.sh_pos, sp.pos.data(), sizeof(int32_t) * sp.pos.size());
    }
    PC_HIP(c, hipMemcpyAsync(c->ws, h, P.lay.h2d_bytes, hipMemcpyHostToDevice, st));
    PC_HIP(c, hipEventRecord(slot->ev, st));
    slot->used = true;
    {
        ProfScope ps(c, 1, st);
        char *w = (char *)c->ws;
        pc_launch_build_plan((const PcCallDesc *)(w + P.lay.calls), n_calls, (const int2 *)(w + P.lay.sel),
                             (const int32_t *)(w + P.lay.q_pos), c->table_dev, c->inv_freq_dev, c->half, P.total_seg,
                             P.total_q, (PcSegment *)(w + P.lay.segs), (int32_t *)(w + P.lay.seg_kvoff),
                             (float2 *)(w + P.lay.rot_seg), (float2 *)(w + P.lay.rot_q), (PcTile *)(w + P.lay.tiles), st);
        PC_HIP(c, hipGetLastError());
        if (P.n_sh_items > 0) {
            pc_launch_shared_rot((const int32_t *)(w + P.lay.sh_pos), (int64_t)P.n_sh_pos, c->inv_freq_dev, c->half,
                                 (float2 *)(w + P.lay.sh_rot), st);
            PC_HIP(c, hipGetLastError());
        }
    }
    return PC_OK;
}

int32_t pc_attend(pc_cache *c, const pc_call *calls, int32_t n_calls, const void *q, void *out, float *lse, void *stream)
{
    if (!c) return PC_ERR_INVALID_ARG;
    if (n_calls < 0 || (n_calls > 0 && !calls)) return fail(c, PC_ERR_INVALID_ARG, "attend: bad call list");
    if (n_calls == 0) return PC_OK;
    if (!c->host_only && (!q || !out)) return fail(c, PC_ERR_INVALID_ARG, "attend: null q or out");
    hipStream_t st = (hipStream_t)stream;
    Planned P;
    const int32_t rc = plan_and_stage(c, calls, n_calls, true, st, P);
    if (rc != PC_OK || c->host_only) return rc;

    char *w = (char *)c->ws;
    PcLaunch L{};
    L.calls = (const PcCallDesc *)(w + P.lay.calls);
    L.segs = (const PcSegment *)(w + P.lay.segs);
    L.rot_seg = (const float2 *)(w + P.lay.rot_seg);
    L.rot_q = (const float2 *)(w + P.lay.rot_q);
    L.tiles = (const PcTile *)(w + P.lay.tiles);
    L.k_store = c->k_store; L.v_store = c->v_store; L.q = q; L.out = out; L.lse = lse;
    L.part_o = (uint16_t *)(w + P.lay.part_o); L.part_ml = (float *)(w + P.lay.part_ml);
    L.slots = c->slots; L.n_q_heads = c->cfg.n_q_heads; L.n_kv_heads = c->cfg.n_kv_heads;
    L.scale_log2 = c->scale * 1.4426950408889634f;
    const int32_t *row_call = (const int32_t *)(w + P.lay.row_call);
    if (c->cfg.dtype == PC_F32) {
        ProfScope ps(c, 5, st);
        pc_launch_attend_f32(L, row_call, P.total_q, c->D, st);
        PC_HIP(c, hipGetLastError());
        return PC_OK;
    }
    if (P.n_pre > 0) {
        ProfScope ps(c, 2, st);
        L.items = (const PcItem *)(w + P.lay.items_pre);
        pc_launch_prefill_bf16(L, P.n_pre, st);
        PC_HIP(c, hipGetLastError());
    }
    if (P.n_dec > 0) {
        ProfScope ps(c, 3, st);
        L.items = (const PcItem *)(w + P.lay.items_dec);
        pc_launch_decode_bf16(L, P.n_dec, st);
        PC_HIP(c, hipGetLastError());
    }
    if (P.n_sh_items > 0) {
        ProfScope ps(c, 3, st);
        PcShLaunch S{};
        S.groups = (const PcShGroup *)(w + P.lay.sh_groups);
        S.segs = (const PcShSeg *)(w + P.lay.sh_segs);
        S.items = (const PcShItem *)(w + P.lay.sh_items);
        S.rot = (const float2 *)(w + P.lay.sh_rot);
        pc_launch_decode_shared_bf16(L, S, P.n_sh_items, st);
        PC_HIP(c, hipGetLastError());
    }
    if (P.n_merge_rows > 0) {
        ProfScope ps(c, 4, st);
        pc_launch_merge(c->cfg.dtype, (const PcMergeRow *)(w + P.lay.merge_rows), P.n_merge_rows, L.part_o, L.part_ml, out, lse,
                        c->cfg.n_q_heads, c->D, st);
        PC_HIP(c, hipGetLastError());
    }
    return PC_OK;
}

int32_t pc_attend_backward(pc_cache *c, const pc_call *calls, int32_t n_calls, const void *q, const float *lse,
                           const void *d_out, float *d_q, float *d_k, float *d_v, void *stream)
{
    if (!c) return PC_ERR_INVALID_ARG;
    if (n_calls < 0 || (n_calls > 0 && !calls)) return fail(c, PC_ERR_INVALID_ARG, "attend_backward: bad call list");
    if (n_calls == 0) return PC_OK;
    if (!c->host_only && (!q || !lse || !d_out || !d_q || !d_k || !d_v))
        return fail(c, PC_ERR_INVALID_ARG, "attend_backward: null argument");
    hipStream_t st = (hipStream_t)stream;
    Planned P;
    const int32_t rc = plan_and_stage(c, calls, n_calls, false, st, P);
    if (rc != PC_OK || c->host_only) return rc;
    char *w = (char *)c->ws;
    PcLaunch L{};
    L.calls = (const PcCallDesc *)(w + P.lay.calls);
    L.segs = (const PcSegment *)(w + P.lay.segs);
    L.rot_seg = (const float2 *)(w + P.lay.rot_seg);
    L.rot_q = (const float2 *)(w + P.lay.rot_q);
    L.k_store = c->k_store; L.v_store = c->v_store; L.q = q;
    L.slots = c->slots; L.n_q_heads = c->cfg.n_q_heads; L.n_kv_heads = c->cfg.n_kv_heads;
    L.scale_log2 = c->scale * 1.4426950408889634f;
    ProfScope ps(c, 5, st);
    int max_seg_len = 0;
    for (const Resolved &r : P.res) {
        for (const int2 &e : r.sel) max_seg_len = std::max(max_seg_len, c->msgs[(size_t)e.x].len);
        max_seg_len = std::max(max_seg_len, r.self_len);
    }
    if ((max_seg_len + 15) / 16 > 65535) return fail(c, PC_ERR_SHAPE, "attend_backward: a message of %d tokens is too long", max_seg_len);
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
    if (!d_k) return fail(c, PC_ERR_INVALID_ARG, "grad_keys_finalize: null d_k");
    std::vector<PcMsgEntry> live;
    for (const HostMsg &m : c->msgs)
        if (m.live && m.len > 0) live.push_back(PcMsgEntry{(int32_t)m.slot_start, m.len, m.base_pos, 0});
    if (live.empty()) return PC_OK;
    hipStream_t st = (hipStream_t)stream;
    const int32_t rc = stage_items(c, live.data(), sizeof(PcMsgEntry) * live.size(), st);
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
    const int32_t rc = plan_and_stage(c, call, 1, false, st, P);
    if (rc != PC_OK) return rc;
    const int64_t n = P.res[0].n_kv;
    if (n_kv) *n_kv = n;
    if (c->host_only || cap < n || n == 0) return PC_OK;
    if (!kv_slot || !kv_pos) return fail(c, PC_ERR_INVALID_ARG, "build_tables: null output with cap > 0");
    ProfScope ps(c, 6, st);
    char *w = (char *)c->ws;
    pc_launch_expand_tables((const PcSegment *)(w + P.lay.segs), (const int32_t *)(w + P.lay.seg_kvoff), P.total_seg, n,
                            kv_slot, kv_pos, st);
    PC_HIP(c, hipGetLastError());
    return PC_OK;
}

}  // extern "C"
