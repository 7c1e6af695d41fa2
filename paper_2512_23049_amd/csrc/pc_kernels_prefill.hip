// K3: bf16 MFMA prefill attention for gfx950.
//
// Work decomposition.  A row unit is 32 query rows of one query head; units of a (call, KV
// head) are numbered head-fastest.  A workgroup is 8 waves = 8 consecutive units (two waves
// per SIMD), so the heads that share a KV head sit in one workgroup and share every staged
// K/V tile.
//
// Formulation (shared with the decode kernel): S^T = K~ . Q^T and O^T = V^T . P^T, so a query
// row's softmax statistics live in one lane column and P goes from the first MFMA's
// accumulators to the second MFMA's B operand without leaving registers.
//
// Vector-ALU diet.  On this chip the softmax costs about as many cycles as the MFMAs, so the
// loop keeps it to the essentials: the softmax scale (times log2 e) is folded into the turned
// queries; probabilities are 2^(score - m_ref) with a reference m_ref that starts at 0 and only
// moves (and the accumulators are only rescaled) when a tile's maximum exceeds it by more than
// 64 (a probability above 2^64: fp32 sums over 2^17 keys and bf16 probabilities hold that with room
// to spare) or the first scores of a row lie more than 64 below it.  While no lane of a wave has
// moved its reference the scores are not shifted at all, so a score costs one v_exp, one add
// and half a convert.  The packed walk goes one step further: the gather pass leaves the largest
// key norm of every tile, and when |q| |k| cannot reach 64 for any row of the wave and any key of
// the call, its loop does not look for the maximum at all (a quarter of its vector instructions).
//
// Overlap.  Every wave runs a software pipeline over the tiles in which the vector ALU work of
// the softmax sits a few instructions behind each MFMA: iteration i issues the eight score
// MFMAs of tile i+1 beside 12 of tile i's 16 exponentials, then the eight P.V MFMAs of tile i
// beside the last four exponentials, the column maximum of tile i+1 and the test whether the
// reference has to move.  A wave that issues about four vector instructions behind each MFMA
// runs close to the MFMA-only rate; separate MFMA and vector phases, even on the two waves
// of a SIMD in opposite order, overlap far less.  Rare work (a segment change, a ragged or
// causal tile, a moving reference) is laid out off the hot path.
//
// Staging.  K and V tiles go global -> LDS directly (global_load_lds, 16 bytes per lane, no
// staging registers) into rings of 5 slots; K(i+5) and V(i+4) are requested inside iteration
// i's two MFMA runs (not all at one point: the requests of eight waves would queue up) and
// K(i+3), V(i+1) must have landed at its closing barrier, so a request has two to three
// iterations to complete.  A direct load writes 1 KB of consecutive LDS per wave, so K rows
// cannot be padded; instead the 16-byte chunks of row r are stored at chunk position
// (c ^ (r & 15)), which keeps the fragment reads (16 rows x one logical chunk) free of bank
// conflicts.  Which tile comes next (physical slot, in-message index, segment, ragged length)
// is read from the per-call tile table the plan builder wrote, with a scalar load requested
// at the top of an iteration and awaited between its two MFMA runs.
//
// Position: keys are stored turned to base + in-message index (base 0 unless the message was
// repositioned); whenever start - base changes from one segment to the next the queries are
// turned by (q_pos - start + base) from an fp32 master copy, half in registers and half in
// LDS (Sec. 2.4 "Position Updates", applied to the query side).  The kernel uses no
// accumulation registers on purpose: with all 256 registers of a wave in one file the MFMA
// results are read by the vector ALU without copies.
//
// Two walks, one template.  In place (the text above): tiles wherever the messages lie in the cache.  Packed: calls
// with many rows read a copy of their keys and values that the gather pass wrote token after token, keys already
// turned to the call's positions; then nothing is looked up per tile, and the loop splits into a plain pipelined loop
// for the tiles every row of the wave sees whole and a simple loop for the few on the causal diagonal.
//
// Queries and results move as whole cache lines: the 32 query rows of a wave come in by direct loads into LDS (16
// lanes per 256-byte row), the results leave through LDS the same way.  A lane that fetches or stores its own row's
// pieces touches 32 lines per instruction with 16 or 32 bytes used of each, which cost a launch several microseconds.
#include "pc_mfma_common.h"

#include <type_traits>

#define TILE_BYTES 8192
#define RING 5
#define LAZY_LOG2 64.0f
#define MFMA32(a, b, c) __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0)

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

__device__ __forceinline__ float max3(float a, float b, float c) { return __builtin_fmaxf(__builtin_fmaxf(a, b), c); }
// The same on the bit patterns, as signed integers: equal to the float maximum whenever some input is positive (among
// positive floats the patterns order like the values, and any positive pattern beats any negative one), which is all
// a test against a positive threshold needs; integer maxima are not preceded by the quieting v_max(x, x) that the
// compiler puts in front of a float maximum of MFMA results.
__device__ __forceinline__ int imax3(int a, int b, int c) { return max(max(a, b), c); }
__device__ __forceinline__ int imax_across_halves(int x)
{
    auto r = __builtin_amdgcn_permlane32_swap((unsigned)x, (unsigned)x, false, false);
    return max((int)r[0], (int)r[1]);
}
__device__ __forceinline__ float max_across_halves(float x)
{
    // lanes l and l^32 hold the two halves of one column
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float sum_across_halves(float x)
{
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// One 16-byte-per-lane direct load: lane l's 16 bytes land at lds_wave_base + 16*l.  Written
// as assembly on purpose: the compiler then keeps no record of the LDS write, so it neither
// drains every outstanding request (vmcnt(0)) in front of later LDS reads of the same array nor
// at barriers; completion is awaited explicitly with s_waitcnt vmcnt(n) where the ring needs it.
__device__ __forceinline__ void dma16(const void *gbase_uniform, unsigned lane_off, unsigned lds_wave_base)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 ::"s"(lds_wave_base), "v"(lane_off), "s"(gbase_uniform) : "memory", "m0");
}
// workgroup barrier without the fence __syncthreads() implies (which would wait for every
// outstanding direct load); LDS accesses are not moved across it
__device__ __forceinline__ void ring_barrier() { asm volatile("s_barrier" ::: "memory"); }

template <int I> using IC = std::integral_constant<int, I>;

// PACKED: the call's keys and values were copied by the gather pass into a buffer of their own, token after token in
// the order the call lists them (keys already turned to the positions the call gives them), the parents' part padded
// to whole tiles, then the new message.  Tile t of the call then sits at slot 32 t of that copy, only the last tile
// of each part can be ragged, the queries are turned once by their own position, and nothing has to be looked up per
// tile: no tile table, no rotation tables, no fp32 copy of the queries.
template <bool PACKED>
__global__ __launch_bounds__(512, 1) void pc_prefill_bf16_kernel(PcLaunch L)
{
    __shared__ __attribute__((aligned(1024))) unsigned char s_k[RING][TILE_BYTES];
    __shared__ __attribute__((aligned(1024))) unsigned char s_v[RING][TILE_BYTES];
    __shared__ __attribute__((aligned(1024))) float2 s_rot[RING][PC_D / 2];
    __shared__ __attribute__((aligned(16))) float4 s_qm[8][8][64];    // upper half (dims 64..127) of the fp32 query master
    // what a lane adds to its 16 scores of a tile of which it may see the first `lim` keys only (0 <= lim <= 32):
    // 0 for a visible key, -inf for the others; row [lim][lane >> 5], register r = key 16 (r / 8) + 8 (lane >> 5) + r % 8
    __shared__ __attribute__((aligned(16))) float s_bias[PC_TILE + 1][2][16];
    __shared__ float s_red[8];

    for (int idx = threadIdx.x; idx < (PC_TILE + 1) * 32; idx += 512) {           // (visible after the barrier in front of the first tile)
        const int lim = idx >> 5, half = (idx >> 4) & 1, r = idx & 15;
        s_bias[lim][half][r] = (16 * (r >> 3) + 8 * half + (r & 7) < lim) ? 0.f : -INFINITY;
    }
    const int kh = blockIdx.x % L.n_kv_heads;          // consecutive workgroups (one per XCD) take different KV heads
    const PcItem item = L.items[blockIdx.x / L.n_kv_heads];
    const PcCallDesc cd = L.calls[item.call];
    const int g = L.n_q_heads / L.n_kv_heads;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wave_s = __builtin_amdgcn_readfirstlane(wave);       // (in a scalar register)
    const int n = lane & 31, hh = lane >> 5;
    const int n_units = ((cd.n_q + 31) >> 5) * g;
    const int unit = item.unit0 + wave;
    const bool unit_ok = unit < n_units;
    const int ub = unit_ok ? unit / g : 0;               // 32-row block
    const int uj = unit_ok ? unit - ub * g : 0;          // head within the group
    const int h = kh * g + uj;
    const int tok0 = cd.self_len - cd.n_q;               // own token index of query row 0
    const int row = 32 * ub + n;
    const bool row_ok = unit_ok && row < cd.n_q;
    const int Rg = cd.q_off + (row_ok ? row : 0);
    const int self_lim = tok0 + row;                     // last own token this row sees
    const int blk_lim_lo = __builtin_amdgcn_readfirstlane(tok0 + 32 * ub);   // ... the wave's first row sees (wave uniform)

    // query turned by its own position and scaled by softmax_scale * log2(e), fp32; element
    // (ks, j) is dim 16*ks + 8*hh + j.  Lower half in registers, upper half in LDS (read back
    // once per segment).  Filled while the first tiles are on their way.
    float qm[4][8];
    bf16x8 qop[8];
    // PACKED: the same values go straight into the bf16 MFMA operands (qop[ks]: dims 16 ks + 8 hh + j, qop[ks + 4]: 64 up)
    float qn2 = 0.f;                                     // PACKED: the largest squared norm of the wave's query rows (scaled, turned)
    auto load_query_direct = [&]() __attribute__((always_inline)) {
        float ss = 0.f;
        const uint16_t *qp = (const uint16_t *)L.q + ((int64_t)Rg * L.n_q_heads + h) * PC_D + 8 * hh;
        const float2 *rq = L.rot_q + (int64_t)Rg * (PC_D / 2) + 8 * hh;
        const float sc = row_ok ? L.scale_log2 : 0.f;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            uint4 lo = ldg16(qp + 16 * ks), hi = ldg16(qp + 16 * ks + 64);
            const uint32_t lw[4] = {lo.x, lo.y, lo.z, lo.w}, hw[4] = {hi.x, hi.y, hi.z, hi.w};
            float xx[8], yy[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const float x = ((j & 1) ? bf_hi(lw[j >> 1]) : bf_lo(lw[j >> 1])) * sc;
                const float y = ((j & 1) ? bf_hi(hw[j >> 1]) : bf_lo(hw[j >> 1])) * sc;
                const float2 cs = rq[16 * ks + j];
                xx[j] = x * cs.x - y * cs.y;
                yy[j] = x * cs.y + y * cs.x;
                ss += xx[j] * xx[j] + yy[j] * yy[j];
            }
            qop[ks] = __builtin_bit_cast(bf16x8, make_uint4(pack_bf16(xx[0], xx[1]), pack_bf16(xx[2], xx[3]), pack_bf16(xx[4], xx[5]), pack_bf16(xx[6], xx[7])));
            qop[ks + 4] = __builtin_bit_cast(bf16x8, make_uint4(pack_bf16(yy[0], yy[1]), pack_bf16(yy[2], yy[3]), pack_bf16(yy[4], yy[5]), pack_bf16(yy[6], yy[7])));
        }
        ss = sum_across_halves(ss);                      // the row's squared norm, then the largest of the wave's 32 rows
#pragma unroll
        for (int o = 1; o < 32; o <<= 1) ss = __builtin_fmaxf(ss, __shfl_xor(ss, o));
        qn2 = __uint_as_float(__builtin_amdgcn_readfirstlane(__float_as_uint(ss)));
    };
    // In-place walk: the wave's 32 query rows of its head (256 bytes each) arrive by direct loads in the wave's part of
    // s_qm, which is free until the master copy is written: instruction i brings rows 4 i .. 4 i + 3, sixteen lanes to a
    // row, whole cache lines (a lane fetching its own row's pieces touches 32 lines per instruction instead of 8).
    // Chunk c of row r lands at position c ^ (r & 15) of the row, so that the 16 lanes that later read one chunk
    // index of 16 different rows hit different banks.  The rotation rows come from the copy of the table that is laid
    // out for this access (rot_qw: 16 bytes per lane, lanes of consecutive rows side by side).
    float4 rqw[4][4];
    const unsigned lds_q = (unsigned)(size_t)&s_qm[0][0][0] + __builtin_amdgcn_readfirstlane(wave) * 8192u;
    auto request_query = [&]() __attribute__((always_inline)) {
        const int ub_u = __builtin_amdgcn_readfirstlane(ub), h_u = __builtin_amdgcn_readfirstlane(h);
        const unsigned char *qb = (const unsigned char *)L.q + ((int64_t)(cd.q_off + 32 * ub_u) * L.n_q_heads + h_u) * (PC_D * 2);
        const int r4 = lane >> 4, c = lane & 15;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int r = 4 * i + r4;
            const int src = (unit_ok && 32 * ub_u + r < cd.n_q) ? r : 0;          // rows past the call's end: any valid row
            dma16(qb, (unsigned)(src * L.n_q_heads * (PC_D * 2) + ((c ^ (r & 15)) << 4)), lds_q + i * 1024);
        }
        const float4 *rw = reinterpret_cast<const float4 *>(L.rot_qw) + ((int64_t)(Rg >> 5) * 32 + hh) * 32 + (Rg & 31);
#pragma unroll
        for (int ks = 0; ks < 4; ++ks)
#pragma unroll
            for (int jq = 0; jq < 4; ++jq) rqw[ks][jq] = rw[(ks * 4 + jq) * 64];
    };
    // ... once they have landed (the caller has waited): into the fp32 master, turned by the row's own position and scaled
    auto finish_query = [&]() __attribute__((always_inline)) {
        const float sc = row_ok ? L.scale_log2 : 0.f;
        const unsigned char *ql = reinterpret_cast<const unsigned char *>(&s_qm[wave][0][0]) + n * 256;
        uint4 lo[4], hi[4];
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            lo[ks] = *reinterpret_cast<const uint4 *>(ql + (((2 * ks + hh) ^ (n & 15)) << 4));
            hi[ks] = *reinterpret_cast<const uint4 *>(ql + (((2 * ks + hh + 8) ^ (n & 15)) << 4));
        }
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            const uint32_t lw[4] = {lo[ks].x, lo[ks].y, lo[ks].z, lo[ks].w}, hw[4] = {hi[ks].x, hi[ks].y, hi[ks].z, hi[ks].w};
            float yy[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const float x = ((j & 1) ? bf_hi(lw[j >> 1]) : bf_lo(lw[j >> 1])) * sc;
                const float y = ((j & 1) ? bf_hi(hw[j >> 1]) : bf_lo(hw[j >> 1])) * sc;
                const float4 t = rqw[ks][j >> 1];
                const float cs_x = (j & 1) ? t.z : t.x, cs_y = (j & 1) ? t.w : t.y;
                qm[ks][j] = x * cs_x - y * cs_y;
                yy[j] = x * cs_y + y * cs_x;
            }
            s_qm[wave][2 * ks][lane] = make_float4(yy[0], yy[1], yy[2], yy[3]);
            s_qm[wave][2 * ks + 1][lane] = make_float4(yy[4], yy[5], yy[6], yy[7]);
        }
    };

    const unsigned char *kb, *vb;
    if constexpr (PACKED) {
        const int64_t at = ((int64_t)kh * L.kg_slots + (int64_t)cd.kg_tile0 * PC_TILE) * PC_D * 2;
        kb = (const unsigned char *)L.k_gather + at;
        vb = (const unsigned char *)L.v_gather + at;
    } else {
        kb = (const unsigned char *)L.k_store + (int64_t)kh * L.slots * PC_D * 2;
        vb = (const unsigned char *)L.v_store + (int64_t)kh * L.slots * PC_D * 2;
    }

    // tiles this workgroup walks: its split's range (the host has cut it at the causal limit of the
    // workgroup's last row, so nothing has to be looked up for it)
    const int tile_end = item.tile_end;
    const int tile0 = item.tile_begin;
    const int T = tile_end - tile0;

    // softmax state of this lane's column.  Probabilities are 2^(score - m_ref) with scores in
    // the log2 domain.  m_ref starts at 0 and moves only when it has to: when a tile's maximum
    // exceeds it by more than LAZY_LOG2, or when the first scores seen lie more than that below it.  For
    // ordinary attention logits it never moves, and then no lane of the wave needs to shift its
    // scores at all (`shifted` is false) and a score costs one v_exp, one add and half a convert.
    float m_ref = 0.f, thr_lo = -LAZY_LOG2, l_run = 0.f;
    bool shifted = false;                                // some lane of this wave has m_ref != 0
    bool all_seen = false;                               // every lane of this wave has met a visible key (thr_lo is -inf everywhere)
    f32x16 acc[4];
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[db][r] = 0.f;

    // tile descriptors come from the per-call tile table the plan builder wrote; they are
    // fetched with scalar loads a few tiles ahead (uniform over the workgroup)
    struct Desc {                                        // as in the table: 4 scalar registers per tile
        int slot0, key0, seg, flags;
        // (read through readfirstlane: the values are wave uniform, which the compiler cannot
        // see for the ones that arrive through request_desc)
        __device__ int valid() const { return __builtin_amdgcn_readfirstlane(flags) & 0xFF; }
        __device__ bool fresh() const { return (__builtin_amdgcn_readfirstlane(flags) & PC_TILE_FRESH) != 0; }
        __device__ bool is_self() const { return (__builtin_amdgcn_readfirstlane(flags) & PC_TILE_SELF) != 0; }
        __device__ int key() const { return __builtin_amdgcn_readfirstlane(key0); }
    };
    const PcTile *tile_tab = L.tiles + item.tile_tab0;   // (from the work item: no need to wait for the call descriptor)
    typedef int i32x4 __attribute__((ext_vector_type(4)));
    auto decode = [&](const i32x4 &v) {
        Desc d;
        d.slot0 = v.x; d.key0 = v.y; d.seg = v.z; d.flags = v.w;
        return d;
    };
    // PACKED: what the table would say follows from the tile's number
    // (the parents' part is padded IN FRONT to whole tiles: only the call's very first tile has keys that do not
    // exist, its first `front_pad` ones, and that tile is always met outside the pipelined loop)
    const int p_tiles = (cd.n_par + PC_TILE - 1) / PC_TILE;          // tiles of the parents' part
    const int front_pad = p_tiles * PC_TILE - cd.n_par;
    auto packed_desc = [&](int t) {
        const bool own = t >= p_tiles;
        const int key0 = own ? (t - p_tiles) * PC_TILE : 0;
        const int valid = own ? min(cd.self_len - key0, PC_TILE) : PC_TILE;
        return (i32x4){t * PC_TILE, key0, 0, valid | (own ? PC_TILE_SELF : 0)};
    };
    auto describe = [&](int t) {
        if constexpr (PACKED) return decode(packed_desc(t));
        const i32x4 v = *reinterpret_cast<const __attribute__((address_space(4))) i32x4 *>(reinterpret_cast<uintptr_t>(tile_tab + t));
        return decode(v);
    };
    // The same load in two halves, so that a whole iteration lies between request and use: the
    // compiler would wait for the data right behind the load.  The request is invisible to the
    // compiler's wait counting, which stays correct for its own LDS reads (an extra outstanding
    // scalar load only makes those waits stricter); await_desc waits for everything.
    auto request_desc = [&](int t) {
        if constexpr (PACKED) return packed_desc(t);
        i32x4 v;
        asm volatile("s_load_dwordx4 %0, %1, 0x0" : "=&s"(v) : "s"(tile_tab + t));
        return v;
    };
    auto await_desc = [&](i32x4 &v) { if constexpr (!PACKED) asm volatile("s_waitcnt lgkmcnt(0)" : "+s"(v)); };

    // direct global -> LDS requests.  A tile is 512 16-byte chunks, one per thread.  Chunk
    // position p of a K tile holds logical chunk (p & 15) ^ ((p >> 4) & 15) of row p >> 4.
    const unsigned k_src_off = (threadIdx.x >> 4) * 256 + (((threadIdx.x & 15) ^ ((threadIdx.x >> 4) & 15)) << 4);
    const unsigned v_src_off = threadIdx.x * 16;
    const unsigned wave_lds = __builtin_amdgcn_readfirstlane(wave) * 1024;
    const unsigned lds_k = (unsigned)(size_t)&s_k[0][0] + wave_lds, lds_v = (unsigned)(size_t)&s_v[0][0] + wave_lds;
    const unsigned lds_rot = (unsigned)(size_t)&s_rot[0][0];
    const unsigned char *rot_base = (const unsigned char *)(L.rot_seg + (int64_t)cd.seg_off * (PC_D / 2));
    auto dma_k = [&](const Desc &d, int slot) {         // the rotation table first: it must be the oldest request
        if constexpr (!PACKED) {
            if (d.fresh() && threadIdx.x < 32)
                dma16(rot_base + (int64_t)__builtin_amdgcn_readfirstlane(d.seg) * (PC_D / 2) * sizeof(float2), threadIdx.x * 16, lds_rot + slot * (unsigned)sizeof(s_rot[0]));
        }
        dma16(kb + (int64_t)__builtin_amdgcn_readfirstlane(d.slot0) * 256, k_src_off, lds_k + slot * TILE_BYTES);
    };
    auto dma_v = [&](const Desc &d, int slot) {
        dma16(vb + (int64_t)__builtin_amdgcn_readfirstlane(d.slot0) * 256, v_src_off, lds_v + slot * TILE_BYTES);
    };

    // K row read by this lane for MFMA row (lane & 31): rows are permuted so that the score
    // registers 0..7 / 8..15 of a lane are keys 8*hh + 0..7 / 16 + 8*hh + 0..7
    const int krow = 16 * (n >> 4) + 8 * ((n >> 2) & 1) + 4 * ((n >> 3) & 1) + (n & 3);
    // LDS addresses of fragment ks in ring slot 0, kept as eight ready-made registers (the empty
    // asm stops the compiler from re-deriving them with an add in front of every read)
    unsigned k_rd[8];
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
        k_rd[ks] = (unsigned)(size_t)&s_k[0][krow * 256 + (((2 * ks + hh) ^ (krow & 15)) << 4)];
        asm volatile("" : "+v"(k_rd[ks]));
    }
    const unsigned char *v_rd = &s_v[0][(hh * PC_D + n) * 16];

    // turn the queries by -segment start (table in s_rot[slot]) into bf16 MFMA operands
    auto turn_query = [&](int slot) __attribute__((always_inline)) {
        const float4 *rs = reinterpret_cast<const float4 *>(&s_rot[slot][8 * hh]);
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            uint32_t lo[4], hi[4];
#pragma unroll
            for (int j4 = 0; j4 < 2; ++j4) {
                const float4 c0 = rs[(16 * ks + 4 * j4) >> 1];          // (cos, sin) of pairs 4*j4, 4*j4+1
                const float4 c1 = rs[((16 * ks + 4 * j4) >> 1) + 1];    // ... 4*j4+2, 4*j4+3
                const float x0 = qm[ks][4 * j4], x1 = qm[ks][4 * j4 + 1], x2 = qm[ks][4 * j4 + 2], x3 = qm[ks][4 * j4 + 3];
                const float4 yv = s_qm[wave][2 * ks + j4][lane];
                const float y0 = yv.x, y1 = yv.y, y2 = yv.z, y3 = yv.w;
                lo[2 * j4] = pack_bf16(x0 * c0.x + y0 * c0.y, x1 * c0.z + y1 * c0.w);
                hi[2 * j4] = pack_bf16(y0 * c0.x - x0 * c0.y, y1 * c0.z - x1 * c0.w);
                lo[2 * j4 + 1] = pack_bf16(x2 * c1.x + y2 * c1.y, x3 * c1.z + y3 * c1.w);
                hi[2 * j4 + 1] = pack_bf16(y2 * c1.x - x2 * c1.y, y3 * c1.z - x3 * c1.w);
            }
            qop[ks] = __builtin_bit_cast(bf16x8, make_uint4(lo[0], lo[1], lo[2], lo[3]));
            qop[ks + 4] = __builtin_bit_cast(bf16x8, make_uint4(hi[0], hi[1], hi[2], hi[3]));
        }
    };

    // K / V fragments of ring slot `slot` as MFMA A operands.  One register set `fr` of 8
    // fragments is recycled: as soon as an MFMA has consumed fr[j], the fragment the NEXT MFMA
    // phase needs is requested into it, so LDS latency hides behind the current phase.
    typedef const __attribute__((address_space(3))) bf16x8 *lds_frag_ptr;
    auto kfrag = [&](int slot, int ks) { return *(lds_frag_ptr)(k_rd[ks] + slot * TILE_BYTES); };
    // V fragment f: d block f & 3, key step f >> 2
    auto vfrag = [&](int slot, int f) { return *reinterpret_cast<const bf16x8 *>(v_rd + slot * TILE_BYTES + (((f >> 2) * 2) * PC_D + 32 * (f & 3)) * 16); };
    bf16x8 fr[8];

    // ---- the softmax in two parts, each written to run in the shadow of eight MFMAs ----
    // Part 1 of a tile: mask what a row may not see (ragged tile end, causal limit in the new
    // message) and shift by the reference if some lane has moved it; both are rare and wave
    // uniform.  Register r of the scores is key 16*(r/8) + 8*hh + (r%8).
    auto mask_and_shift = [&](f32x16 &s, const Desc &d) __attribute__((always_inline)) {
        const bool is_self = d.is_self();
        if (__builtin_expect(d.valid() < PC_TILE || (is_self && d.key() + PC_TILE - 1 > blk_lim_lo), 0)) {
            // (added, not selected: sixteen additions and four LDS reads instead of sixteen compares and selects;
            // the scores of keys that do not exist are finite, because the slots behind a message's end hold zeros
            // or what an earlier, finite message left there)
            const int lim = is_self ? max(0, min(d.valid(), self_lim - d.key() + 1)) : d.valid();
            const float4 *b = reinterpret_cast<const float4 *>(&s_bias[lim][hh][0]);
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                const float4 bv = b[q4];
                s[4 * q4] += bv.x; s[4 * q4 + 1] += bv.y; s[4 * q4 + 2] += bv.z; s[4 * q4 + 3] += bv.w;
            }
        }
        if (__builtin_expect(shifted, 0)) {
#pragma unroll
            for (int r = 0; r < 16; ++r) s[r] -= m_ref;
        }
    };
    // ... then, given the column maximum mx (relative to m_ref), move the reference if needed.
    // The test is three compares whose lane masks are combined on the scalar side.
    auto rebase = [&](f32x16 &s, float mx) __attribute__((always_inline)) {
        const uint64_t above = __builtin_amdgcn_ballot_w64(mx > LAZY_LOG2);
        uint64_t need_mask = above;
        if (__builtin_expect(!all_seen, 0)) {            // until every row of the wave has met a visible key
            const uint64_t below = __builtin_amdgcn_ballot_w64(mx < thr_lo);
            const bool seen = mx > -INFINITY;
            need_mask |= below & __builtin_amdgcn_ballot_w64(seen);
            thr_lo = seen ? -INFINITY : thr_lo;
            all_seen = __builtin_amdgcn_ballot_w64(thr_lo == -INFINITY) == ~0ull;
        }
        if (__builtin_expect(need_mask != 0, 0)) {
            const bool need = (need_mask >> lane) & 1;
            const float shift = need ? mx : 0.f;
            // The reference moves down only at a row's first scores, when nothing has been accumulated yet:
            // the factor is then irrelevant, and 2^-shift could overflow (0 * inf); it is taken as 1.
            const float alpha = fast_exp2(-__builtin_fmaxf(shift, 0.f));
            l_run *= alpha;
#pragma unroll
            for (int db = 0; db < 4; ++db) acc[db] *= alpha;
            m_ref += shift;
#pragma unroll
            for (int r = 0; r < 16; ++r) s[r] -= shift;
            shifted = __builtin_amdgcn_ballot_w64(m_ref != 0.f) != 0;
        }
    };
    auto col_max = [&](const f32x16 &s) {
        float mx = __builtin_fmaxf(s[0], s[1]);
#pragma unroll
        for (int r = 2; r < 16; r += 2) mx = __builtin_fmaxf(mx, __builtin_fmaxf(s[r], s[r + 1]));
        return max_across_halves(mx);
    };

    // An iteration is two runs of eight MFMAs with the vector ALU work of the softmax placed in
    // their shadow, a few instructions behind each MFMA (the sched_group_barrier calls pin that
    // order).  e^x of score register r, added to the row sum; odd r completes a bf16 pair.
    float ps;
    uint32_t pk[8];
    float ev[16];
    auto expo = [&](const f32x16 &s, int r) __attribute__((always_inline)) {
        ev[r] = fast_exp2(s[r]);
        ps = r == 0 ? ev[0] : ps + ev[r];                // (r == 0 opens a tile's sum)
        if (r & 1) {
            pk[r >> 1] = pack_bf16(ev[r - 1], ev[r]);
            asm volatile("" : "+v"(pk[r >> 1]), "+v"(ps));    // keeps the vector work from sinking below its MFMA
        }
    };
    // Phase A: the scores of the NEXT tile (K fragments in fr, one MFMA chain into a fresh
    // accumulator) beside the first 12 exponentials of THIS tile's finished scores `s`.  Each
    // consumed K fragment register is refilled with a V fragment of this tile (ring slot
    // v_slot).  `between` runs after the second MFMA: the direct loads of a later tile are
    // requested there, not all at one point of the iteration.
    auto phase_a = [&](int v_slot, const f32x16 &s, auto between) __attribute__((always_inline)) {
        f32x16 sn;
#pragma unroll
        for (int r = 0; r < 16; ++r) sn[r] = 0.f;
        ps = 0.f;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            sn = MFMA32(fr[ks], qop[ks], sn);
            fr[ks] = vfrag(v_slot, ks);
            if (ks == 1) between();
#pragma unroll
            for (int r = (3 * ks) / 2; r < (3 * ks + 3) / 2; ++r) expo(s, r);
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            if (ks & 1) {
                __builtin_amdgcn_sched_group_barrier(0x400, 2, 0);
                __builtin_amdgcn_sched_group_barrier(0x002, 3, 0);
            } else {
                __builtin_amdgcn_sched_group_barrier(0x400, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x002, 2, 0);
            }
        }
        return sn;
    };
    // Phase B: O^T += V^T . P^T of this tile (V fragments in fr, refilled with the K fragments
    // of ring slot k_slot).  Its first two MFMAs cover the last 4 exponentials (the second key
    // step's probabilities are first needed by the fifth MFMA), the others the column maximum of
    // the next tile's scores sn and the test whether the reference has to move.  It moves after
    // the MFMAs: the accumulators they update are relative to the old reference.
    auto phase_b = [&](auto plain_c, int k_slot, const f32x16 &s, f32x16 &sn, const Desc &dn, auto between) __attribute__((always_inline)) {
        // plain_c: 0 the general form; 1 nothing to mask (PACKED, plain loop); 2 nor can a score exceed the reference by
        // more than 2^LAZY_LOG2, by the norms of the wave's queries and the call's keys, and no reference has moved
        constexpr int FORM = decltype(plain_c)::value;
        constexpr bool PLAIN = FORM != 0, BOUNDED = FORM == 2;
        if constexpr (BOUNDED) {
        } else if constexpr (PLAIN) {                    // nothing to mask; a moved reference still has to be subtracted
            if (__builtin_expect(shifted, 0)) {
#pragma unroll
                for (int r = 0; r < 16; ++r) sn[r] -= m_ref;
            }
        } else {
            mask_and_shift(sn, dn);
        }
        const bf16x8 p0 = __builtin_bit_cast(bf16x8, make_uint4(pk[0], pk[1], pk[2], pk[3]));
        int mxi = 0;
        auto fi = [](float x) { return __float_as_int(x); };
#pragma unroll
        for (int f = 0; f < 4; ++f) {
            acc[f] = MFMA32(fr[f], p0, acc[f]);
            fr[f] = kfrag(k_slot, f);
            if (f == 1) between();
            if (f < 2) { expo(s, 12 + 2 * f); expo(s, 13 + 2 * f); }
            else if constexpr (BOUNDED) {}
            else if (f == 2) mxi = imax3(imax3(fi(sn[0]), fi(sn[1]), fi(sn[2])), fi(sn[3]), fi(sn[4]));     // three-input maxima: 8 for 16 scores
            else mxi = imax3(imax3(mxi, fi(sn[5]), fi(sn[6])), fi(sn[7]), fi(sn[8]));
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            if (f < 2) __builtin_amdgcn_sched_group_barrier(0x400, 2, 0);
            __builtin_amdgcn_sched_group_barrier(0x002, 3, 0);
        }
        l_run += ps;
        const bf16x8 p1 = __builtin_bit_cast(bf16x8, make_uint4(pk[4], pk[5], pk[6], pk[7]));
#pragma unroll
        for (int f = 4; f < 8; ++f) {
            acc[f & 3] = MFMA32(fr[f], p1, acc[f & 3]);
            fr[f] = kfrag(k_slot, f);
            if constexpr (!BOUNDED) {
                if (f == 4) mxi = imax3(imax3(mxi, fi(sn[9]), fi(sn[10])), fi(sn[11]), fi(sn[12]));
                if (f == 5) mxi = imax3(imax3(mxi, fi(sn[13]), fi(sn[14])), fi(sn[15]), fi(sn[15]));
            }
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x002, 4, 0);
        }
        // The column maximum is taken on the bit patterns (see imax3): once every row of the wave has met a key, all that
        // is asked of it is whether it exceeds the threshold, and in the lanes where it does the pattern's maximum is
        // the float maximum (the other lanes' references stay where they are).  Until then the rare path takes the float
        // maximum again, for the test against the lower threshold.
        if constexpr (!BOUNDED) {
            mxi = imax_across_halves(mxi);
            const bool above = __builtin_amdgcn_ballot_w64(mxi > fi(LAZY_LOG2)) != 0;
            bool early = false;
            if constexpr (!PLAIN) early = !all_seen;
            if (__builtin_expect(above || early, 0)) rebase(sn, early ? col_max(sn) : __int_as_float(mxi));
        }
    };

    if (T > 0) {
        const int last = tile_end - 1;
        Desc d0 = describe(tile0);
        if constexpr (!PACKED) d0.flags |= PC_TILE_FRESH;          // a split may start in the middle of a segment
        Desc d1 = describe(min(tile0 + 1, last));
        Desc d2 = describe(min(tile0 + 2, last));
        Desc d3 = describe(min(tile0 + 3, last));
        Desc d4 = describe(min(tile0 + 4, last));
        Desc d5 = describe(min(tile0 + 5, last));
        // PACKED: the largest squared key norm of the call (the gather pass left one per tile)
        float kn2 = 0.f;
        if constexpr (PACKED) {
            const float *kn = L.kg_norm + (int64_t)kh * (L.kg_slots / PC_TILE) + cd.kg_tile0;
            const int n_all = p_tiles + (cd.self_len + PC_TILE - 1) / PC_TILE;
            for (int t = threadIdx.x; t < n_all; t += 512) kn2 = __builtin_fmaxf(kn2, kn[t]);
        }
        dma_k(d0, 0); dma_v(d0, 0);
        if constexpr (!PACKED) request_query();          // right behind the first tile: requests come back in order
        dma_k(d1, 1); dma_v(d1, 1);
        dma_k(d2, 2); dma_v(d2, 2);
        dma_k(d3, 3); dma_v(d3, 3);
        dma_k(d4, 4);
        if constexpr (PACKED) load_query_direct();
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        if constexpr (!PACKED) finish_query();
        if constexpr (PACKED) {
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) kn2 = __builtin_fmaxf(kn2, __shfl_xor(kn2, o));
            if (lane == 0) s_red[wave] = kn2;
        }
        __syncthreads();
        // |q.k| <= |q| |k|: when that bound (with room for the operands' rounding) stays below the threshold at which the
        // softmax reference would move, no score of the plain loop can cross it and the loop need not look
        bool bounded = false;
        if constexpr (PACKED) {
            kn2 = s_red[0];
#pragma unroll
            for (int w8 = 1; w8 < 8; ++w8) kn2 = __builtin_fmaxf(kn2, s_red[w8]);
            bounded = qn2 * kn2 * 1.05f <= LAZY_LOG2 * LAZY_LOG2;
        }

        // tile 0: scores and softmax part 1, nothing to overlap with yet; leaves the K fragments
        // of tile 1 in fr
#pragma unroll
        for (int f = 0; f < 8; ++f) fr[f] = kfrag(0, f);
        if constexpr (!PACKED) turn_query(0);
        f32x16 sc;                                       // scores of the current tile, part 1 done
#pragma unroll
        for (int r = 0; r < 16; ++r) sc[r] = 0.f;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            sc = MFMA32(fr[ks], qop[ks], sc);
            fr[ks] = kfrag(1, ks);
        }
        if constexpr (!PACKED) { if (d1.fresh()) turn_query(1); }   // (from tile 2 on the queries are turned at the end of an iteration)
        if constexpr (PACKED) {
            if (tile0 == 0 && front_pad > 0) {           // the padding in front of the parents' part
#pragma unroll
                for (int r = 0; r < 16; ++r) sc[r] = (16 * (r >> 3) + 8 * hh + (r & 7) >= front_pad) ? sc[r] : -INFINITY;
            }
        }
        mask_and_shift(sc, d0);
        rebase(sc, col_max(sc));
        // every wave has read tile 0's K before any wave overwrites its slot with tile 5's
        __builtin_amdgcn_s_waitcnt(0xC07F);              // lgkmcnt(0)
        ring_barrier();

        // Iteration i (tiles i and i+1); u = i mod RING is a compile-time constant so that ring
        // slots are immediates.  On entry: sc = scores of tile i (part 1 done), fr = K fragments
        // of tile i+1, d1..d5 = descriptors of tiles i+1..i+5.  K(i+2) and V(i) are in LDS.
        // PLAIN (PACKED calls only): the form of the iteration for the tiles nothing special happens around: tile i+1 is
        // a whole tile every row of the wave sees all of (nothing to mask) and every row of the wave has met a key; it
        // tests one thing, whether some score exceeds the reference by more than LAZY_LOG2 (form 1), or, when the norms
        // of the wave's queries and the call's keys rule that out, nothing at all (form 2).
        auto iteration = [&](auto uc, auto plain_c, int i) {
            constexpr int u = decltype(uc)::value;
            constexpr int s0 = u, s1 = (u + 1) % RING, s2 = (u + 2) % RING, s4 = (u + 4) % RING;
            i32x4 raw6 = request_desc(min(tile0 + i + 6, last));     // first used in the next iteration's requests
            f32x16 sn = phase_a(s0, sc, [&] { dma_k(d5, s0); });             // K(i+5) takes the slot of K(i)
            // the descriptor is awaited here, where the wait costs nothing: it waits for every LDS
            // read too, and the V fragments requested during phase A arrived while its vector work
            // finished
            await_desc(raw6);
            const Desc d6 = decode(raw6);
            phase_b(plain_c, s2, sc, sn, d1, [&] { dma_v(d4, s4); });        // V(i+4) takes the slot of V(i-1)
            // the score MFMAs of this iteration have been issued, so the query operands are free:
            // turn them now if the tile after next starts a new rotation (its table came with K(i+2));
            // the P.V MFMAs just issued keep the matrix pipe busy meanwhile
            if constexpr (!PACKED) { if (__builtin_expect(d2.fresh(), 0)) turn_query(s2); }
            sc = sn;
            // K(i+3), V(i+1) (requested two and three iterations ago) must have landed; the requests
            // of this and the previous iteration (a K and a V each, rotation tables in front of
            // their K) may stay in flight.  The K fragment reads of phase B may still be in flight
            // too: their slot is not written again before the barrier after next.
            __builtin_amdgcn_s_waitcnt(0x0F74);          // vmcnt(4)
            ring_barrier();
            d1 = d2; d2 = d3; d3 = d4; d4 = d5; d5 = d6;
        };
        const int n_it = T - 1;
        if constexpr (PACKED) {
            auto dsc = [&](int t) { return decode(packed_desc(min(t, last))); };
            // The plain form of the iteration, software-pipelined, ring slots as immediates: for tiles of which every
            // row of the wave sees every key (the parents' part; the tiles of the new message below the wave's first
            // row), once every row has met a key.
            auto plain_iteration = [&](auto uc, auto form, int i) {
                constexpr int u = decltype(uc)::value;
                constexpr int s0 = u, s2 = (u + 2) % RING, s4 = (u + 4) % RING;
                f32x16 sn = phase_a(s0, sc, [&] { dma_k(dsc(tile0 + i + 5), s0); });
                phase_b(form, s2, sc, sn, d1, [&] { dma_v(dsc(tile0 + i + 4), s4); });
                sc = sn;
                __builtin_amdgcn_s_waitcnt(0x0F74);      // vmcnt(4), as in the general form below
                ring_barrier();
            };
            // the first tile not of that kind for this wave: behind the parents' part and the tiles of the new message
            // that lie wholly below the wave's first row
            const int whole_own = cd.self_len > 0 ? max(0, (blk_lim_lo + 1) / PC_TILE) : 0;
            const int n_plain = max(0, min(n_it, p_tiles + whole_own - tile0 - 1));
            auto ok = [&](int i) { return i < n_plain && all_seen; };
            int i = 0;
            auto plain_loop = [&](auto form) __attribute__((always_inline)) {
                for (;; i += RING) {
                    if (!ok(i)) break;
                    plain_iteration(IC<0>{}, form, i);
                    if (!ok(i + 1)) { i += 1; break; }
                    plain_iteration(IC<1>{}, form, i + 1);
                    if (!ok(i + 2)) { i += 2; break; }
                    plain_iteration(IC<2>{}, form, i + 2);
                    if (!ok(i + 3)) { i += 3; break; }
                    plain_iteration(IC<3>{}, form, i + 3);
                    if (!ok(i + 4)) { i += 4; break; }
                    plain_iteration(IC<4>{}, form, i + 4);
                }
            };
            if (bounded && !shifted) plain_loop(IC<2>{});            // (no reference moves in that loop, so none has moved at its end)
            else plain_loop(IC<1>{});
            // The general form for what is left (the tiles on and beyond the causal diagonal, or everything once a
            // reference has moved): the same steps one after the other, ring slots computed, nothing overlapped.  It
            // serves a few tiles per workgroup.
            int u = i % RING;
            for (; i < n_it; ++i) {
                const int s0 = u, s2 = u + 2 >= RING ? u + 2 - RING : u + 2, s4 = u + 4 >= RING ? u + 4 - RING : u + 4;
                dma_k(dsc(tile0 + i + 5), s0);           // K(i+5) takes the slot of K(i)
                f32x16 sn;
#pragma unroll
                for (int r = 0; r < 16; ++r) sn[r] = 0.f;
#pragma unroll
                for (int ks = 0; ks < 8; ++ks) sn = MFMA32(fr[ks], qop[ks], sn);       // scores of tile i+1
#pragma unroll
                for (int f = 0; f < 8; ++f) fr[f] = vfrag(s0, f);
                dma_v(dsc(tile0 + i + 4), s4);           // V(i+4) takes the slot of V(i-1)
                ps = 0.f;
#pragma unroll
                for (int r = 0; r < 16; ++r) expo(sc, r);
                l_run += ps;
                const bf16x8 p0 = __builtin_bit_cast(bf16x8, make_uint4(pk[0], pk[1], pk[2], pk[3]));
                const bf16x8 p1 = __builtin_bit_cast(bf16x8, make_uint4(pk[4], pk[5], pk[6], pk[7]));
#pragma unroll
                for (int f = 0; f < 8; ++f) acc[f & 3] = MFMA32(fr[f], (f >> 2) ? p1 : p0, acc[f & 3]);
#pragma unroll
                for (int ks = 0; ks < 8; ++ks) fr[ks] = kfrag(s2, ks);
                mask_and_shift(sn, dsc(tile0 + i + 1));
                rebase(sn, col_max(sn));
                sc = sn;
                __builtin_amdgcn_s_waitcnt(0x0F74);      // vmcnt(4)
                ring_barrier();
                u = u + 1 == RING ? 0 : u + 1;
            }
        } else {
            for (int i = 0; i < n_it; i += RING) {
                iteration(IC<0>{}, IC<0>{}, i);
                if (i + 1 >= n_it) break;
                iteration(IC<1>{}, IC<0>{}, i + 1);
                if (i + 2 >= n_it) break;
                iteration(IC<2>{}, IC<0>{}, i + 2);
                if (i + 3 >= n_it) break;
                iteration(IC<3>{}, IC<0>{}, i + 3);
                if (i + 4 >= n_it) break;
                iteration(IC<4>{}, IC<0>{}, i + 4);
            }
        }
        __builtin_amdgcn_s_waitcnt(0x0F70);              // drain outstanding direct loads
        // the last tile: softmax part 2 and P.V with nothing to overlap with
        {
            const unsigned char *vl = v_rd + ((T - 1) % RING) * TILE_BYTES;
#pragma unroll
            for (int f = 0; f < 8; ++f) fr[f] = *reinterpret_cast<const bf16x8 *>(vl + (((f >> 2) * 2) * PC_D + 32 * (f & 3)) * 16);
            // outside the pipelined loop the row sum can afford to take the probabilities as the MFMA sees them
            // (rounded to bf16): for calls of a single tile the rounding then cancels between numerator and
            // denominator (a row with one visible key returns its V exactly)
            uint32_t pl[8];
            float ps = 0.f;
#pragma unroll
            for (int r = 0; r < 8; ++r) {
                pl[r] = pack_bf16(fast_exp2(sc[2 * r]), fast_exp2(sc[2 * r + 1]));
                ps += bf_lo(pl[r]) + bf_hi(pl[r]);
            }
            l_run += ps;
            const bf16x8 p0 = __builtin_bit_cast(bf16x8, make_uint4(pl[0], pl[1], pl[2], pl[3]));
            const bf16x8 p1 = __builtin_bit_cast(bf16x8, make_uint4(pl[4], pl[5], pl[6], pl[7]));
#pragma unroll
            for (int f = 0; f < 8; ++f) acc[f & 3] = MFMA32(fr[f], (f >> 2) ? p1 : p0, acc[f & 3]);
        }
    }

    // epilogue: a lane holds, for its row, dims 32*db + 8*(r/4) + 4*hh + (r%4).  The 2-byte results (bf16 outputs, or
    // fp16 partials of a split) are turned round in the wave's part of s_qm so that a row's 256 bytes leave as whole cache
    // lines: 16 lanes per row, 4 rows per store (written straight from the accumulators a store would touch 32 lines
    // with 16 bytes each).  Chunk c (16 bytes) of row r sits at position c ^ (r & 15).
    // (Which lane this is, and everything that follows from it, is derived again here from the hardware's lane count and
    // the wave's number in a scalar register: held in vector registers across the loops they would cost a spill.)
    const float l = sum_across_halves(l_run);
    const float inv = l > 0.f ? 1.f / l : 0.f;
    const bool whole = cd.n_splits == 1;
    const int lane_e = (int)__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
    const int n_e = lane_e & 31, hh_e = lane_e >> 5;
    const int unit_e = item.unit0 + wave_s;
    const bool unit_ok_e = unit_e < n_units;
    const int ub_e = unit_ok_e ? unit_e / g : 0;
    const int h_e = kh * g + (unit_ok_e ? unit_e - ub_e * g : 0);
    const int row_e = 32 * ub_e + n_e;
    {
        unsigned char *stg = reinterpret_cast<unsigned char *>(&s_qm[0][0][0]) + wave_s * 8192;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                const float a0 = acc[db][4 * q4] * inv, a1 = acc[db][4 * q4 + 1] * inv, a2 = acc[db][4 * q4 + 2] * inv, a3 = acc[db][4 * q4 + 3] * inv;
                uint2 w;
                w.x = whole ? pack_bf16(a0, a1) : pack_f16(a0, a1);
                w.y = whole ? pack_bf16(a2, a3) : pack_f16(a2, a3);
                *reinterpret_cast<uint2 *>(stg + n_e * 256 + (((4 * db + q4) ^ (n_e & 15)) << 4) + 8 * hh_e) = w;
            }
        const int64_t row0 = whole ? (int64_t)cd.q_off : (int64_t)cd.part_off + (int64_t)item.split * cd.n_q;
        unsigned char *dst = reinterpret_cast<unsigned char *>(whole ? (uint16_t *)L.out : L.part_o) + ((row0 * L.n_q_heads + h_e) * PC_D) * 2;
        const int r4 = lane_e >> 4, c = lane_e & 15;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int r = 4 * i + r4, rw = 32 * ub_e + r;
            const uint4 v = *reinterpret_cast<const uint4 *>(stg + r * 256 + ((c ^ (r & 15)) << 4));
            if (unit_ok_e && rw < cd.n_q) *reinterpret_cast<uint4 *>(dst + (int64_t)rw * L.n_q_heads * (PC_D * 2) + 16 * c) = v;
        }
    }
    if (!unit_ok_e || row_e >= cd.n_q || hh_e != 0) return;
    if (whole) {
        if (L.lse) L.lse[((int64_t)cd.q_off + row_e) * L.n_q_heads + h_e] = (l > 0.f) ? (m_ref + log2f(l)) * 0.6931471805599453f : -INFINITY;
    } else {
        const int64_t pr = (int64_t)cd.part_off + (int64_t)item.split * cd.n_q + row_e;
        L.part_ml[(pr * L.n_q_heads + h_e) * 2] = (l > 0.f) ? m_ref : -INFINITY;
        L.part_ml[(pr * L.n_q_heads + h_e) * 2 + 1] = l;
    }
}

void pc_launch_prefill_bf16(const PcLaunch &L, int n_items, bool packed, hipStream_t st)
{
    if (n_items <= 0) return;
    dim3 grid((unsigned)n_items * L.n_kv_heads);
    if (packed) pc_prefill_bf16_kernel<true><<<grid, 512, 0, st>>>(L);
    else pc_prefill_bf16_kernel<false><<<grid, 512, 0, st>>>(L);
}
