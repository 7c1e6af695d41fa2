// Host side of the library, shared by its source files: the cache object, the message table and slot
// allocator records, the resolved form of a call, the plan layout, and the helpers they all use.
#ifndef PC_HOST_H_
#define PC_HOST_H_

#include "../../include/pc.h"
#include "pc_kernels.h"

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <string>
#include <vector>


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
    int64_t dirty_end = 0;                           // slots below this may hold what a freed or swapped-out message left
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
    int key_gather = 0;                                // gather pass for prefill calls: 0 by size, 1 never, 2 always
    void *static_ws = nullptr;                         // this device's copy of the library's fixed scratch array
    // a mixed batch runs its one-row calls beside its prefill calls: a second stream (default priority) forked from
    // and joined to the caller's with these two events
    hipStream_t side = nullptr; hipEvent_t ev_fork = nullptr, ev_join = nullptr;
    std::string err;
};

#define PC_HIP(c, expr)                                                                        \
    do { hipError_t e_ = (expr);                                                               \
         if (e_ != hipSuccess) return pc_fail((c), PC_ERR_HIP, "%s: %s", #expr, hipGetErrorString(e_)); } while (0)

int32_t pc_fail(pc_cache *c, int32_t code, const char *fmt, ...);
size_t pc_storage_bytes(const pc_config *cfg);
void pc_prof_collect(pc_cache *c);

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

// layout of the staged (host -> device) block and of the device-built block
struct PlanLayout {
    size_t calls, sel, q_pos, row_call, merge_rows, items_dec, items_pre, items_pk, sh_groups, sh_segs, sh_items, sh_pos, kg_items, tok_items, h2d_bytes;
    size_t segs, seg_kvoff, rot_seg, rot_q, rot_qw, tiles, sh_rot, part_o, part_ml, row_scalar, k_gather, v_gather, kg_norm, total;
};

// -------------------------------------------------------------------------------------
// shared by pc_attend and pc_build_tables: validate, plan, stage, run the plan builder
// -------------------------------------------------------------------------------------
struct Planned {
    PlanLayout lay;
    int n_calls = 0, total_sel = 0, total_q = 0, total_seg = 0, n_dec = 0, n_pre = 0, n_pre_pk = 0, pre_waves = 4;
    int n_merge_rows = 0, n_merge_few = 0;               // rows to merge; the first n_merge_few have few splits
    int n_sh_items = 0;
    size_t n_sh_pos = 0;
    int n_kg_items = 0; int64_t kg_tiles = 0;            // calls whose keys are gathered, and their tiles in all
    std::vector<Resolved> res;
    // Where the call's workspace lives.  On entry: fixed_ws != nullptr names a buffer of fixed_cap bytes the plan
    // must fit into (nothing is allocated then: a plan or staging block that does not fit is an error); nullptr
    // means the cache's own workspace, which grows on demand.  On return ws is the buffer the plan was staged to.
    void *fixed_ws = nullptr; size_t fixed_cap = 0;
    void *ws = nullptr;
    // pc_decode_step: tokens the plan builder's launch writes into the cache beside its own work (device k, v rows in
    // item order); tok_done: that launch was enqueued
    std::vector<PcTokenItem> tok_items; const void *tok_k = nullptr, *tok_v = nullptr; bool tok_done = false;
};

// pc_lib.hip
extern "C" int32_t pc_check_token_batch(pc_cache *c, const int32_t *msg_ids, int32_t n_msgs, const void *k, const void *v);
extern "C" int32_t pc_append_token_items(pc_cache *c, const std::vector<int32_t> &ids, const void *k, const void *v, hipStream_t st,
                                         std::vector<PcTokenItem> *defer);
int32_t pc_ensure_ws(pc_cache *c, size_t bytes, hipStream_t st);
int32_t pc_stage_acquire(pc_cache *c, size_t bytes, StageSlot **out);
extern "C" int32_t pc_stage_items(pc_cache *c, const void *items, size_t bytes, hipStream_t st);
// pc_attend.hip: the address, on the current device, of the library's fixed scratch array (looked up once per device)
int32_t pc_static_scratch(void **ptr, size_t *bytes);
// pc_plan.hip
int32_t pc_resolve(pc_cache *c, const pc_call *call, int idx, Resolved &out);
int32_t pc_plan_and_stage(pc_cache *c, const pc_call *calls, int32_t n_calls, bool want_items, hipStream_t st, Planned &P);

#endif
