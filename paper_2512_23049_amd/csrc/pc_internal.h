// Structures shared by the host side of the library and its kernels.
#ifndef PC_INTERNAL_H_
#define PC_INTERNAL_H_

#include <hip/hip_runtime.h>
#include <stdint.h>

#define PC_TILE 32            // keys per KV tile; equals the slot alignment, so a
                              // tile never straddles two messages
#define PC_VGROUP 8           // V is stored key-transposed in groups of 8 slots

// Device copy of one message-table entry (Sec. 2.4: message id -> physical span).
struct PcMsgEntry {
    int32_t slot_start;       // first slot (multiple of PC_TILE)
    int32_t len;              // tokens stored
    int32_t base_pos;         // the stored key of token t is turned to position base_pos + t
                              // (0 after an append; moved by pc_reposition)
    int32_t pad;
};

// One message of a batched append (staged by the host).
struct PcAppendItem {
    const void *k, *v;        // device, [len, H_kv, D] each
    int32_t msg;
    int32_t slot_start;
    int32_t len;
    int32_t pad;
};

// One token appended to an existing message (staged by the host).
struct PcTokenItem {
    int32_t msg;              // message that grows
    int32_t slot;             // physical slot the token goes to
    int32_t pos;              // base_pos + in-message index: what its key is turned to
    int32_t new_len;          // the message's length once this token is in
};

#define PC_TOKEN_PACK 128     // token items that travel in a kernel's arguments (2 KB)
struct PcTokenPack { PcTokenItem it[PC_TOKEN_PACK]; };

// One message of a batched position update (staged by the host).
struct PcMoveItem {
    int32_t msg;
    int32_t slot_start;
    int32_t len;
    int32_t delta;            // positions the stored keys are turned by
    int32_t new_base;
    int32_t pad[3];
};

// One call of a batch as staged by the host.
struct PcCallDesc {
    int32_t sel_off;          // first entry in the packed (msg, start) list
    int32_t n_sel;
    int32_t self_msg;         // -1: none
    int32_t self_start;       // resolved
    int32_t n_q;
    int32_t q_off;            // first packed query row
    int32_t seg_off;          // first segment of this call in the segment arrays
    int32_t n_seg;            // n_sel + (self_msg >= 0)
    int32_t self_len;         // tokens in the new message (0 if none)
    int32_t n_splits;         // KV splits of this call's work items
    int32_t part_off;         // first partial row (units of rows) when n_splits > 1
    int32_t tile_off;         // first entry of this call in the tile table
    int32_t kg_tile0;         // -1, or the call's first tile in the gather buffers: its keys (turned to the positions
                              // the call gives them) and values were copied there token after token, the parents'
                              // part padded to whole tiles, then the new message
    int32_t n_par;            // tokens of the parents' part (all segments but the new message)
    int32_t pad[2];
};

// One call whose keys the gather pass copies (staged by the host).
struct PcGatherItem {
    int32_t call;
    int32_t kg_tile0;         // its first tile in the gathered-keys buffer
    int32_t n_tiles;          // tiles of its copy: ceil(n_par / 32) + ceil(self_len / 32)
    int32_t n_par;            // tokens of the parents' part
};

// A gathered segment = one whole message placed at pos_start (built on device).
struct PcSegment {
    int32_t slot_start;
    int32_t len;
    int32_t pos_start;        // position the call assigns to the message's first token
    int32_t tile_off;         // KV tiles of this call before this segment
    int32_t rot_pos;          // pos_start - the message's stored base: what the queries are turned back by
    int32_t same_rot;         // 1: rot_pos equals that of the segment before (no new turn of the queries)
    int32_t pad[2];
};

// One 32-key KV tile of a call's gathered sequence (built on device from the segments).
#define PC_TILE_FRESH 0x100   // first tile of a segment whose query rotation differs from the one before
#define PC_TILE_SELF  0x200   // tile of the new message (causal limit applies)
struct PcTile {
    int32_t slot0;            // first physical slot of the tile (multiple of PC_TILE)
    int32_t key0;             // in-message index of its first token
    int32_t seg;              // segment index within the call
    int32_t valid_flags;      // low byte: tokens that exist (1..32); PC_TILE_* flags above
};

// One workgroup's share of an attention launch.
struct PcItem {
    int32_t call;
    int32_t unit0;            // prefill: first row unit of the workgroup; decode: 0
    int32_t tile_begin;       // KV tile range [begin, end) within the call
    int32_t tile_end;
    int32_t split;            // split index within the call
    int32_t tile_tab0;        // the call's first entry in the tile table (a copy of its PcCallDesc::tile_off, so that
                              // the first tile descriptors can be requested without waiting for the call descriptor)
    int32_t pad[2];
};

// One output row whose KV splits the merge kernel combines (staged by the host).
struct PcMergeRow {
    int32_t row;              // packed query row
    int32_t part_row0;        // partial row of split 0 (split s is n_q rows further)
    int32_t n_splits;
    int32_t n_q;
};

// ---- shared decode: a group of one-row calls walks the union of its calls' messages once ----
#define PC_SH_ABSENT INT32_MIN    // rotation-table entry of a (message, row) pair the row's call does not list

// One message of a group's union list, in cache-slot order (staged by the host).
struct PcShSeg {
    int32_t slot_start;
    int32_t len;
    int32_t tile_off;         // KV tiles of the union before this message
    int32_t pad;
    uint32_t vis[8];          // bit n of word b: row 32*b + n of the group lists this message
};

// One group: consecutive one-row calls (staged by the host).
struct PcShGroup {
    int32_t seg_off, n_seg;   // its messages in the PcShSeg array
    int32_t n_tiles;          // KV tiles of the union
    int32_t row0;             // packed query row of the group's first call
    int32_t n_rows;           // calls in the group (<= 32 * 8 / g)
    int32_t rot_off;          // entry (message s, row r) of the rotation table is rot_off + s * n_rows + r
    int32_t part_off;         // first partial row when n_splits > 1 (split s is n_rows rows further)
    int32_t n_splits;
};

struct PcShItem {
    int32_t group;
    int32_t tile_begin, tile_end;     // range of the union's tiles
    int32_t split;
    int32_t seg_begin;                // message of the union that owns tile_begin
    int32_t pad[3];
};

struct PcShLaunch {
    const PcShGroup *groups;
    const PcShSeg   *segs;
    const PcShItem  *items;
    const float2    *rot;     // [entries][D/2] (cos, sin)((start - stored base) * theta_i)
};

// Everything an attention kernel needs, passed by value.
struct PcLaunch {
    const PcCallDesc *calls;
    const PcSegment  *segs;
    const float2     *rot_seg;    // [total_seg][D/2] (cos, sin)((pos_start - stored base) * theta_i)
    const float2     *rot_q;      // [total_q][D/2]   (cos, sin)(q_pos * theta_i)
    const float2     *rot_qw;     // the same values laid out for the bf16 prefill kernel's lanes (D = 128 only, else null):
                                  // pair 16 ks + 8 hh + 2 jq + e of row R at float2 index
                                  // ((R / 32 * 1024 + ks * 256 + jq * 64 + hh * 32 + R % 32) * 2 + e
    const PcItem     *items;
    const PcTile     *tiles;      // [total tiles] per-call tile tables
    const void       *k_store;    // [H_kv][slots][D]            K turned to its in-message index
    const void       *v_store;    // bf16: [H_kv][slots/8][D][8] ; f32: [H_kv][slots][D]
    const void       *q;          // [total_q][H_q][D]
    void             *out;        // [total_q][H_q][D]
    float            *lse;        // [total_q][H_q] or null
    uint16_t         *part_o;     // [part rows][H_q][D]   partial outputs, each normalised by its own sum, fp16
    float            *part_ml;    // [part rows][H_q][2]   running max (scaled log2 domain), sum
    void             *k_gather;   // [H_kv][kg_slots][D]       keys of the calls that gather, turned to their positions
    void             *v_gather;   // [H_kv][kg_slots/8][D][8]  their values, in the cache's group-of-8 layout
    int64_t           kg_slots;   // slots of that buffer per KV head (32 per gathered tile)
    float            *kg_norm;    // [H_kv][kg_slots/32]       per tile of that buffer: the largest squared norm of its keys (as stored, bf16)
    int64_t           slots;      // capacity in slots (stride between KV heads)
    int32_t           n_q_heads, n_kv_heads;
    float             scale_log2; // softmax scale * log2(e)
};

#endif
