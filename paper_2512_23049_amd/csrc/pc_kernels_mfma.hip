// bf16 MFMA attention kernels for gfx950: split-K decode and flash-style prefill.
//
// Both work on the transposed problem: scores S^T = K~ . Q^T (rows = keys, columns =
// query rows), so that the softmax statistics of a query row live in one lane column and
// the probabilities come out of the first MFMA already in the register layout the second
// MFMA (O^T = V^T . P^T) wants for its B operand.  V is stored key-transposed in groups of
// 8 slots, so the A operand of the second MFMA is one 16-byte load per lane.
//
// Keys are stored turned to their in-message index t; a message placed at start s then
// needs the query turned by (q_pos - s): <R(p)q, R(s+t)k> = <R(p-s)q, R(t)k>.  The query is
// turned once by p (table rot_q) and once more per segment by -s (table rot_seg).
#include "pc_kernels.h"

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

#define PC_D 128

__device__ __forceinline__ float bf_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float bf_hi(uint32_t u) { return __uint_as_float(u & 0xFFFF0000u); }
__device__ __forceinline__ uint32_t pack_bf16(float a, float b)
{
    bf16x2 r = {(__bf16)a, (__bf16)b};
    return __builtin_bit_cast(uint32_t, r);
}
__device__ __forceinline__ uint16_t to_bf16(float a)
{
    __bf16 r = (__bf16)a;
    return __builtin_bit_cast(uint16_t, r);
}
__device__ __forceinline__ uint4 ldg16(const void *p) { return *reinterpret_cast<const uint4 *>(p); }

// ----------------------------------------------------------------------------------------
// K4: split-K decode.  One workgroup of 4 waves per (work item, KV head); the g query heads
// of the KV head times the call's (few) query rows are the <= 16 columns of 16x16x32 MFMAs.
// Each wave streams a contiguous run of 32-key tiles straight from HBM into registers
// (K rows as MFMA A operands, V groups as A operands of the second MFMA), double buffered.
// ----------------------------------------------------------------------------------------
struct DecTile {
    uint4 k[2][4];      // [16-key half][d step of 32]
    uint4 v[8];         // [16-d block]
    int seg;            // segment index within the call
    int key0;           // first in-message token of the tile
    int valid;          // tokens of the tile that exist (1..32)
};

__device__ __forceinline__ void dec_load(DecTile &T, const uint16_t *__restrict__ kb, const uint16_t *__restrict__ vb,
                                         int slot0, int valid, int lane)
{
    const int m = lane & 15, a = lane >> 4;
    const uint4 z = make_uint4(0, 0, 0, 0);
#pragma unroll
    for (int tau = 0; tau < 2; ++tau) {
        const int key = 8 * (m >> 2) + 4 * tau + (m & 3);
        const uint16_t *row = kb + (int64_t)(slot0 + key) * PC_D + 8 * a;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) T.k[tau][ks] = (key < valid) ? ldg16(row + 32 * ks) : z;
    }
    const uint16_t *vg = vb + ((int64_t)(slot0 / PC_VGROUP + a) * PC_D + m) * PC_VGROUP;
#pragma unroll
    for (int db = 0; db < 8; ++db) T.v[db] = (8 * a < valid) ? ldg16(vg + 16 * db * PC_VGROUP) : z;
}

__global__ __launch_bounds__(256) void pc_decode_bf16_kernel(PcLaunch L)
{
    __shared__ float s_acc[4][PC_D][17];
    __shared__ float s_m[4][16], s_l[4][16];

    const int kh = blockIdx.x % L.n_kv_heads;          // consecutive workgroups (one per XCD) take different KV heads
    const PcItem item = L.items[blockIdx.x / L.n_kv_heads];
    const PcCallDesc cd = L.calls[item.call];
    const int g = L.n_q_heads / L.n_kv_heads;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n = lane & 15, a = lane >> 4;
    const int n_cols = cd.n_q * g;
    const int qr = n / g, qj = n - qr * g;               // column -> (query row, head in group)
    const bool col_ok = n < n_cols;
    const int R = cd.q_off + (col_ok ? qr : 0);
    const int h = kh * g + (col_ok ? qj : 0);
    const int self_seg = cd.self_msg >= 0 ? cd.n_seg - 1 : -1;
    const int self_lim = cd.self_len - cd.n_q + qr;      // last own token this column sees

    // query turned by its own position, kept in fp32: element (ks, j) is dim 32*ks + 8*a + j
    float qh[4][8];
    {
        const uint16_t *qp = (const uint16_t *)L.q + ((int64_t)R * L.n_q_heads + h) * PC_D + 8 * a;
        const float2 *rq = L.rot_q + (int64_t)R * (PC_D / 2) + 8 * a;
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            uint4 lo = ldg16(qp + 32 * ks), hi = ldg16(qp + 32 * ks + 64);
            const uint32_t lw[4] = {lo.x, lo.y, lo.z, lo.w}, hw[4] = {hi.x, hi.y, hi.z, hi.w};
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const float x = (j & 1) ? bf_hi(lw[j >> 1]) : bf_lo(lw[j >> 1]);
                const float y = (j & 1) ? bf_hi(hw[j >> 1]) : bf_lo(hw[j >> 1]);
                const float2 cs = rq[32 * ks + j];
                qh[ks][j] = col_ok ? x * cs.x - y * cs.y : 0.f;
                qh[ks + 2][j] = col_ok ? x * cs.y + y * cs.x : 0.f;
            }
        }
    }

    const uint16_t *kb = (const uint16_t *)L.k_store + (int64_t)kh * L.slots * PC_D;
    const uint16_t *vb = (const uint16_t *)L.v_store + (int64_t)kh * L.slots * PC_D;

    // this wave's contiguous run of tiles
    const int n_tiles = item.tile_end - item.tile_begin;
    const int per_wave = (n_tiles + 3) >> 2;
    int tile = item.tile_begin + wave * per_wave;
    const int tile_stop = min(item.tile_end, tile + per_wave);

    float m_run = -INFINITY, l_run = 0.f;
    f32x4 acc[8];
#pragma unroll
    for (int db = 0; db < 8; ++db) acc[db] = (f32x4){0.f, 0.f, 0.f, 0.f};

    // segment cursor
    int e = 0;
    PcSegment sg = {0, 0, 0, 0};
    int seg_tiles_end = 0;
    auto seek = [&](int t) {           // make (e, sg) the segment that owns tile t
        while (t >= seg_tiles_end) {
            // binary search on first use, then linear steps
            if (seg_tiles_end == 0) {
                int lo = 0, hi = cd.n_seg - 1;
                while (lo < hi) {
                    const int mid = (lo + hi + 1) >> 1;
                    if (L.segs[cd.seg_off + mid].tile_off <= t) lo = mid; else hi = mid - 1;
                }
                e = lo;
            } else {
                ++e;
            }
            sg = L.segs[cd.seg_off + e];
            seg_tiles_end = sg.tile_off + (sg.len + PC_TILE - 1) / PC_TILE;
        }
    };
    auto fetch = [&](DecTile &T, int t) {
        seek(t);
        const int key0 = (t - sg.tile_off) * PC_TILE;
        T.seg = e; T.key0 = key0; T.valid = min(PC_TILE, sg.len - key0);
        dec_load(T, kb, vb, sg.slot_start + key0, T.valid, lane);
    };

    int cur_seg = -1;
    bf16x8 qop[4];
    auto compute = [&](const DecTile &T) {
        if (T.seg != cur_seg) {                          // turn the query by -segment start
            cur_seg = T.seg;
            const float2 *rs = L.rot_seg + (int64_t)(cd.seg_off + cur_seg) * (PC_D / 2) + 8 * a;
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) {
                uint32_t lo[4], hi[4];
#pragma unroll
                for (int j = 0; j < 8; j += 2) {
                    const float2 c0 = rs[32 * ks + j], c1 = rs[32 * ks + j + 1];
                    const float x0 = qh[ks][j], y0 = qh[ks + 2][j], x1 = qh[ks][j + 1], y1 = qh[ks + 2][j + 1];
                    lo[j >> 1] = pack_bf16(x0 * c0.x + y0 * c0.y, x1 * c1.x + y1 * c1.y);
                    hi[j >> 1] = pack_bf16(y0 * c0.x - x0 * c0.y, y1 * c1.x - x1 * c1.y);
                }
                qop[ks] = __builtin_bit_cast(bf16x8, make_uint4(lo[0], lo[1], lo[2], lo[3]));
                qop[ks + 2] = __builtin_bit_cast(bf16x8, make_uint4(hi[0], hi[1], hi[2], hi[3]));
            }
        }
        f32x4 s[2];
#pragma unroll
        for (int tau = 0; tau < 2; ++tau) {
            s[tau] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < 4; ++ks)
                s[tau] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, T.k[tau][ks]), qop[ks], s[tau], 0, 0, 0);
        }
        // lane holds keys 8a + 0..7 of column n
        const int lim = (T.seg == self_seg) ? min(T.valid, self_lim - T.key0 + 1) : T.valid;
        float sc[8];
        float mx = -INFINITY;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const float v = s[j >> 2][j & 3] * L.scale_log2;
            sc[j] = (8 * a + j < lim) ? v : -INFINITY;
            mx = fmaxf(mx, sc[j]);
        }
        mx = fmaxf(mx, __shfl_xor(mx, 16));
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        const float m_new = fmaxf(m_run, mx);
        const float m_safe = (m_new == -INFINITY) ? 0.f : m_new;
        const float alpha = exp2f(m_run - m_safe);
        float p[8], ps = 0.f;
#pragma unroll
        for (int j = 0; j < 8; ++j) { p[j] = exp2f(sc[j] - m_safe); ps += p[j]; }
        l_run = l_run * alpha + ps;
        m_run = m_new;
        const bf16x8 pop = __builtin_bit_cast(bf16x8, make_uint4(pack_bf16(p[0], p[1]), pack_bf16(p[2], p[3]),
                                                                 pack_bf16(p[4], p[5]), pack_bf16(p[6], p[7])));
#pragma unroll
        for (int db = 0; db < 8; ++db) {
            acc[db] *= alpha;
            acc[db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, T.v[db]), pop, acc[db], 0, 0, 0);
        }
    };

    DecTile A, B;
    if (tile < tile_stop) fetch(A, tile);
    while (tile < tile_stop) {
        if (tile + 1 < tile_stop) fetch(B, tile + 1);
        compute(A);
        ++tile;
        if (tile >= tile_stop) break;
        if (tile + 1 < tile_stop) fetch(A, tile + 1);
        compute(B);
        ++tile;
    }

    // combine lane groups, then the 4 waves
    l_run += __shfl_xor(l_run, 16);
    l_run += __shfl_xor(l_run, 32);
    if (a == 0) { s_m[wave][n] = m_run; s_l[wave][n] = l_run; }
#pragma unroll
    for (int db = 0; db < 8; ++db)
#pragma unroll
        for (int r = 0; r < 4; ++r) s_acc[wave][16 * db + 4 * a + r][n] = acc[db][r];
    __syncthreads();
    for (int idx = threadIdx.x; idx < n_cols * PC_D; idx += 256) {
        const int col = idx / PC_D, d = idx - col * PC_D;
        float mm = fmaxf(fmaxf(s_m[0][col], s_m[1][col]), fmaxf(s_m[2][col], s_m[3][col]));
        float o = 0.f, l = 0.f;
        if (mm > -INFINITY) {
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                const float sc = (s_m[w][col] > -INFINITY) ? exp2f(s_m[w][col] - mm) : 0.f;
                o += s_acc[w][d][col] * sc;
                l += s_l[w][col] * sc;
            }
        }
        const int r = col / g, hq = kh * g + (col - r * g);
        const int64_t Rr = cd.q_off + r;
        if (cd.n_splits == 1) {
            ((uint16_t *)L.out)[(Rr * L.n_q_heads + hq) * PC_D + d] = to_bf16(l > 0.f ? o / l : 0.f);
            if (L.lse && d == 0) L.lse[Rr * L.n_q_heads + hq] = (l > 0.f) ? (mm + log2f(l)) * 0.6931471805599453f : -INFINITY;
        } else {
            const int64_t pr = (int64_t)cd.part_off + (int64_t)item.split * cd.n_q + r;
            L.part_o[(pr * L.n_q_heads + hq) * PC_D + d] = o;
            if (d == 0) { L.part_ml[(pr * L.n_q_heads + hq) * 2] = mm; L.part_ml[(pr * L.n_q_heads + hq) * 2 + 1] = l; }
        }
    }
}

void pc_launch_decode_bf16(const PcLaunch &L, int n_items, hipStream_t st)
{
    if (n_items <= 0) return;
    dim3 grid((unsigned)n_items * L.n_kv_heads);
    pc_decode_bf16_kernel<<<grid, 256, 0, st>>>(L);
}

// ----------------------------------------------------------------------------------------
// K3: prefill.  A workgroup of NW waves handles NW row units of one KV head; a row unit is
// 32 query rows of one query head (units are numbered head-fastest, so the g heads that
// share the KV head sit in one workgroup and share every staged K/V tile).  32-key tiles
// are staged through LDS, double buffered; each wave runs 32x32x16 MFMAs against them.
// Softmax runs in the log2 domain with a lazily updated reference maximum: the running
// reference only moves (and the accumulators are only rescaled) when a tile's maximum
// exceeds it by more than 2^8, so the common tile costs one fma + one exp per score.
// ----------------------------------------------------------------------------------------
#define KROW 272        // bytes per K row in LDS (256 + 16 padding: conflict-free 16 B reads)
#define KTILE_BYTES (32 * KROW)
#define VTILE_BYTES (4 * PC_D * 16)
#define LAZY_LOG2 8.0f

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

__device__ __forceinline__ float max_across_halves(float x)
{
    // lanes l and l^32 hold the two halves of one column
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

#define SGB(mask, n) __builtin_amdgcn_sched_group_barrier(mask, n, 0)

template <int NW>
__global__ __launch_bounds__(NW * 64) void pc_prefill_bf16_kernel(PcLaunch L)
{
    __shared__ __attribute__((aligned(16))) unsigned char s_k[2][KTILE_BYTES];
    __shared__ __attribute__((aligned(16))) unsigned char s_v[2][VTILE_BYTES];
    __shared__ __attribute__((aligned(16))) float2 s_rot[2][PC_D / 2];

    const int kh = blockIdx.x % L.n_kv_heads;
    const PcItem item = L.items[blockIdx.x / L.n_kv_heads];
    const PcCallDesc cd = L.calls[item.call];
    const int g = L.n_q_heads / L.n_kv_heads;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n = lane & 31, hh = lane >> 5;
    const int n_units = ((cd.n_q + 31) >> 5) * g;
    const int unit = item.unit0 + wave;
    const bool unit_ok = unit < n_units;
    const int ub = unit_ok ? unit / g : 0;               // 32-row block
    const int uj = unit_ok ? unit - ub * g : 0;          // head within the group
    const int row = 32 * ub + n;
    const bool row_ok = unit_ok && row < cd.n_q;
    const int R = cd.q_off + (row_ok ? row : 0);
    const int h = kh * g + uj;
    const int self_seg = cd.self_msg >= 0 ? cd.n_seg - 1 : -1;
    const int self_lim = cd.self_len - cd.n_q + row;     // last own token this row sees
    const int wave_lim_lo = cd.self_len - cd.n_q + 32 * ub;       // ... the wave's first row sees
    const int last_unit = min(item.unit0 + NW - 1, n_units - 1);
    const int wg_lim = cd.self_len - cd.n_q + min(32 * (last_unit / g) + 31, cd.n_q - 1);
    const float c_log2 = L.scale_log2;

    // query turned by its own position, fp32: element (ks, j) is dim 16*ks + 8*hh + j
    float qh[8][8];
    {
        const uint16_t *qp = (const uint16_t *)L.q + ((int64_t)R * L.n_q_heads + h) * PC_D + 8 * hh;
        const float2 *rq = L.rot_q + (int64_t)R * (PC_D / 2) + 8 * hh;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            uint4 lo = ldg16(qp + 16 * ks), hi = ldg16(qp + 16 * ks + 64);
            const uint32_t lw[4] = {lo.x, lo.y, lo.z, lo.w}, hw[4] = {hi.x, hi.y, hi.z, hi.w};
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const float x = (j & 1) ? bf_hi(lw[j >> 1]) : bf_lo(lw[j >> 1]);
                const float y = (j & 1) ? bf_hi(hw[j >> 1]) : bf_lo(hw[j >> 1]);
                const float2 cs = rq[16 * ks + j];
                qh[ks][j] = row_ok ? x * cs.x - y * cs.y : 0.f;
                qh[ks + 4][j] = row_ok ? x * cs.y + y * cs.x : 0.f;
            }
        }
    }

    const unsigned char *kb = (const unsigned char *)L.k_store + (int64_t)kh * L.slots * PC_D * 2;
    const unsigned char *vb = (const unsigned char *)L.v_store + (int64_t)kh * L.slots * PC_D * 2;

    // tiles this workgroup walks: its split's range, cut at the causal limit of its last row
    int tile_end = item.tile_end;
    if (self_seg >= 0) {
        const int self_tile_off = L.segs[cd.seg_off + self_seg].tile_off;
        tile_end = min(tile_end, self_tile_off + (wg_lim + PC_TILE) / PC_TILE);
    }
    const int tile0 = item.tile_begin;
    const int T = tile_end - tile0;

    float m_ref = -INFINITY, neg_m = 0.f, l_run = 0.f;
    f32x16 acc[4];
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[db][r] = 0.f;

    // segment cursor (uniform over the workgroup); tiles are described in non-decreasing order
    int e = 0, seg_tiles_end = 0;
    PcSegment sg = {0, 0, 0, 0};
    struct Desc { int seg, key0, valid, slot0; bool fresh; };
    auto describe = [&](int t, int prev_seg) {
        while (t >= seg_tiles_end) {
            if (seg_tiles_end == 0) {
                int lo = 0, hi = cd.n_seg - 1;
                while (lo < hi) {
                    const int mid = (lo + hi + 1) >> 1;
                    if (L.segs[cd.seg_off + mid].tile_off <= t) lo = mid; else hi = mid - 1;
                }
                e = lo;
            } else {
                ++e;
            }
            sg = L.segs[cd.seg_off + e];
            seg_tiles_end = sg.tile_off + (sg.len + PC_TILE - 1) / PC_TILE;
        }
        Desc d;
        d.seg = e; d.key0 = (t - sg.tile_off) * PC_TILE; d.valid = min(PC_TILE, sg.len - d.key0);
        d.slot0 = sg.slot_start + d.key0; d.fresh = e != prev_seg;
        return d;
    };

    // global -> register -> LDS staging: 512 16-byte chunks per K tile and per V tile, plus the
    // 512-byte rotation table of a segment when a K tile opens it
    constexpr int CH = 512 / (NW * 64);
    uint4 stg_k[CH], stg_v[CH], stg_r;
    auto g_load_k = [&](const Desc &d) {
#pragma unroll
        for (int i = 0; i < CH; ++i) stg_k[i] = ldg16(kb + (int64_t)d.slot0 * 256 + (threadIdx.x + i * NW * 64) * 16);
        if (d.fresh && threadIdx.x < 32)
            stg_r = ldg16((const unsigned char *)(L.rot_seg + (int64_t)(cd.seg_off + d.seg) * (PC_D / 2)) + threadIdx.x * 16);
    };
    auto g_load_v = [&](const Desc &d) {
#pragma unroll
        for (int i = 0; i < CH; ++i) stg_v[i] = ldg16(vb + (int64_t)d.slot0 * 256 + (threadIdx.x + i * NW * 64) * 16);
    };
    auto s_store_k = [&](int buf, bool fresh) {
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            const int c = threadIdx.x + i * NW * 64;
            *reinterpret_cast<uint4 *>(&s_k[buf][(c >> 4) * KROW + (c & 15) * 16]) = stg_k[i];
        }
        if (fresh && threadIdx.x < 32)
            *reinterpret_cast<uint4 *>((unsigned char *)&s_rot[buf][0] + threadIdx.x * 16) = stg_r;
    };
    auto s_store_v = [&](int buf) {
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            const int c = threadIdx.x + i * NW * 64;
            *reinterpret_cast<uint4 *>(&s_v[buf][c * 16]) = stg_v[i];
        }
    };

    bf16x8 qop[8];
    // K row read by this lane for MFMA row (lane & 31): rows are permuted so that the score
    // registers 0..7 / 8..15 of a lane are keys 8*hh + 0..7 / 16 + 8*hh + 0..7
    const int krow = 16 * (n >> 4) + 8 * ((n >> 2) & 1) + 4 * ((n >> 3) & 1) + (n & 3);
    const int k_lane_off = krow * KROW + hh * 16;
    const int v_lane_off = (hh * PC_D + n) * 16;

    auto turn_query = [&](int buf) {           // query turned by -segment start, as bf16 MFMA operands
        const float4 *rs = reinterpret_cast<const float4 *>(&s_rot[buf][8 * hh]);
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            uint32_t lo[4], hi[4];
#pragma unroll
            for (int j = 0; j < 8; j += 2) {
                const float4 cc = rs[(16 * ks + j) >> 1];      // (cos, sin) of pairs j and j+1
                const float x0 = qh[ks][j], y0 = qh[ks + 4][j], x1 = qh[ks][j + 1], y1 = qh[ks + 4][j + 1];
                lo[j >> 1] = pack_bf16(x0 * cc.x + y0 * cc.y, x1 * cc.z + y1 * cc.w);
                hi[j >> 1] = pack_bf16(y0 * cc.x - x0 * cc.y, y1 * cc.z - x1 * cc.w);
            }
            qop[ks] = __builtin_bit_cast(bf16x8, make_uint4(lo[0], lo[1], lo[2], lo[3]));
            qop[ks + 4] = __builtin_bit_cast(bf16x8, make_uint4(hi[0], hi[1], hi[2], hi[3]));
        }
    };

    // after the scores of a tile are complete: mask what this row may not see, take the column
    // maximum, and move the reference maximum (rescaling the accumulators) only when needed.
    // Register r of this lane is key 16*(r/8) + 8*hh + (r%8) of column n.
    auto prep = [&](f32x16 &s, const Desc &d) {
        const bool is_self = d.seg == self_seg;
        if (d.valid < PC_TILE || (is_self && d.key0 + PC_TILE - 1 > wave_lim_lo)) {
            const int lim = is_self ? min(d.valid, self_lim - d.key0 + 1) : d.valid;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int key = 16 * (r >> 3) + 8 * hh + (r & 7);
                s[r] = (key < lim) ? s[r] : -INFINITY;
            }
        }
        float mx = fmaxf(s[0], s[1]);
#pragma unroll
        for (int r = 2; r < 16; r += 2) mx = fmaxf(mx, fmaxf(s[r], s[r + 1]));
        mx = max_across_halves(mx) * c_log2;
        const bool need = mx > m_ref + LAZY_LOG2;
        if (__builtin_amdgcn_ballot_w64(need) != 0) {
            const float m_new = need ? mx : m_ref;
            const float alpha = need ? fast_exp2(m_ref - m_new) : 1.f;
            l_run *= alpha;
#pragma unroll
            for (int db = 0; db < 4; ++db) acc[db] *= alpha;
            m_ref = m_new;
            neg_m = (m_ref == -INFINITY) ? 0.f : -m_ref;
        }
    };

    if (T > 0) {
        const int last = tile_end - 1;
        Desc d0 = describe(tile0, -1);
        Desc d1 = describe(min(tile0 + 1, last), d0.seg);
        g_load_k(d0); g_load_v(d0);
        s_store_k(0, true); s_store_v(0);
        g_load_k(d1);
        s_store_k(1, d1.fresh);
        __syncthreads();
        turn_query(0);
        f32x16 sc;
#pragma unroll
        for (int r = 0; r < 16; ++r) sc[r] = 0.f;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks)
            sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<const bf16x8 *>(&s_k[0][k_lane_off + ks * 32]), qop[ks], sc, 0, 0, 0);
        prep(sc, d0);

        for (int i = 0; i < T; ++i) {
            const Desc d2 = describe(min(tile0 + i + 2, last), d1.seg);
            g_load_k(d2);
            g_load_v(d1);
            const int kbuf = (i + 1) & 1, vbuf = i & 1;
            if (d1.fresh) turn_query(kbuf);

            // ---- scores of tile i+1 (MFMA) overlapped with the exponentials of tile i (VALU)
            const unsigned char *kr = &s_k[kbuf][k_lane_off];
            const unsigned char *vr = &s_v[vbuf][v_lane_off];
            f32x16 sn;
#pragma unroll
            for (int r = 0; r < 16; ++r) sn[r] = 0.f;
            float p[16];
            float ps = 0.f;
            uint32_t pw[8];
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) {
                const bf16x8 ka = *reinterpret_cast<const bf16x8 *>(kr + ks * 32);
                sn = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, qop[ks], sn, 0, 0, 0);
                p[ks] = fast_exp2(fmaf(sc[ks], c_log2, neg_m));
                ps += p[ks];
                if (ks & 1) pw[ks >> 1] = pack_bf16(p[ks - 1], p[ks]);
            }
            const bf16x8 pop0 = __builtin_bit_cast(bf16x8, make_uint4(pw[0], pw[1], pw[2], pw[3]));
            // ---- first half of P.V overlapped with the second half of the exponentials
#pragma unroll
            for (int db = 0; db < 4; ++db) {
                const bf16x8 va = *reinterpret_cast<const bf16x8 *>(vr + (32 * db) * 16);
                acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, pop0, acc[db], 0, 0, 0);
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    const int r = 8 + 2 * db + j;
                    p[r] = fast_exp2(fmaf(sc[r], c_log2, neg_m));
                    ps += p[r];
                }
                pw[4 + db] = pack_bf16(p[8 + 2 * db], p[9 + 2 * db]);
            }
            const bf16x8 pop1 = __builtin_bit_cast(bf16x8, make_uint4(pw[4], pw[5], pw[6], pw[7]));
#pragma unroll
            for (int db = 0; db < 4; ++db) {
                const bf16x8 va = *reinterpret_cast<const bf16x8 *>(vr + (2 * PC_D + 32 * db) * 16);
                acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, pop1, acc[db], 0, 0, 0);
            }
            l_run += ps;

            s_store_k(i & 1, d2.fresh);
            s_store_v((i + 1) & 1);
            __syncthreads();
            if (i + 1 < T) prep(sn, d1);
            sc = sn;
            d0 = d1; d1 = d2;
        }
    }

    // epilogue: this lane holds, for row n, dims 32*db + 8*(r/4) + 4*hh + (r%4)
    {
        auto r2 = __builtin_amdgcn_permlane32_swap(__float_as_uint(l_run), __float_as_uint(l_run), false, false);
        l_run = __uint_as_float(r2[0]) + __uint_as_float(r2[1]);
    }
    if (!row_ok) return;
    if (cd.n_splits == 1) {
        const float inv = l_run > 0.f ? 1.f / l_run : 0.f;
        uint16_t *o = (uint16_t *)L.out + ((int64_t)R * L.n_q_heads + h) * PC_D;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                const int d = 32 * db + 8 * q4 + 4 * hh;
                uint2 w;
                w.x = pack_bf16(acc[db][4 * q4] * inv, acc[db][4 * q4 + 1] * inv);
                w.y = pack_bf16(acc[db][4 * q4 + 2] * inv, acc[db][4 * q4 + 3] * inv);
                *reinterpret_cast<uint2 *>(o + d) = w;
            }
        if (L.lse && hh == 0)
            L.lse[(int64_t)R * L.n_q_heads + h] = (l_run > 0.f) ? (m_ref + log2f(l_run)) * 0.6931471805599453f : -INFINITY;
    } else {
        const int64_t pr = (int64_t)cd.part_off + (int64_t)item.split * cd.n_q + row;
        float *o = L.part_o + (pr * L.n_q_heads + h) * PC_D;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                const int d = 32 * db + 8 * q4 + 4 * hh;
                *reinterpret_cast<float4 *>(o + d) = make_float4(acc[db][4 * q4], acc[db][4 * q4 + 1], acc[db][4 * q4 + 2], acc[db][4 * q4 + 3]);
            }
        if (hh == 0) { L.part_ml[(pr * L.n_q_heads + h) * 2] = m_ref; L.part_ml[(pr * L.n_q_heads + h) * 2 + 1] = l_run; }
    }
}

void pc_launch_prefill_bf16(const PcLaunch &L, int n_items, int waves, hipStream_t st)
{
    if (n_items <= 0) return;
    dim3 grid((unsigned)n_items * L.n_kv_heads);
    if (waves == 8) pc_prefill_bf16_kernel<8><<<grid, 512, 0, st>>>(L);
    else pc_prefill_bf16_kernel<4><<<grid, 256, 0, st>>>(L);
}
