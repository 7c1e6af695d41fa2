// bf16 MFMA attention kernels for gfx950: split-K decode (the prefill kernel is in
// pc_kernels_prefill.hip and shares the formulation described here).
//
// Both work on the transposed problem: scores S^T = K~ . Q^T (rows = keys, columns =
// query rows), so that the softmax statistics of a query row live in one lane column and
// the probabilities come out of the first MFMA already in the register layout the second
// MFMA (O^T = V^T . P^T) wants for its B operand.  V is stored key-transposed in groups of
// 8 slots, so the A operand of the second MFMA is one 16-byte load per lane.
//
// Keys are stored turned to b + t (in-message index t, base b = 0 unless the message was
// repositioned); a message placed at start s then needs the query turned by (q_pos - s + b):
// <R(p)q, R(s+t)k> = <R(p-s+b)q, R(b+t)k>.  The query is turned once by p (table rot_q) and
// once more per segment by -(s - b) (table rot_seg).
#include "pc_mfma_common.h"

// ----------------------------------------------------------------------------------------
// K4: split-K decode.  One workgroup of 4 waves per (work item, KV head); the g query heads
// of the KV head times the call's (few) query rows are the <= 16 columns of 16x16x32 MFMAs.
// Each wave streams a contiguous run of 32-key tiles straight from HBM into registers
// (K rows as MFMA A operands, V groups as A operands of the second MFMA), double buffered.
// Two workgroups per CU (256 registers per wave): the kernel lives on bytes in flight, and
// with one workgroup per CU (what an unconstrained register allocation gives) it reached
// only four fifths of the bandwidth it reaches with two.
// ----------------------------------------------------------------------------------------
// maximum over the lane pairs (l, l ^ 16) and (l, l ^ 32) without a trip through LDS: the swap
// instructions exchange 16- resp. 32-lane rows between their two operands
__device__ __forceinline__ float max_lanes_xor16(float x)
{
    auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float max_lanes_xor32(float x)
{
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

struct DecTile {
    uint4 k[2][4];      // [16-key half][d step of 32]
    uint4 v[8];         // [16-d block]
    int seg;            // segment index within the call
    int key0;           // first in-message token of the tile
    int valid;          // tokens of the tile that exist (1..32)
    bool fresh;         // first tile of a segment whose query rotation differs from the one before
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

__global__ __launch_bounds__(256, 2) void pc_decode_bf16_kernel(PcLaunch L)
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

    // this wave's contiguous run of tiles
    const int n_tiles = item.tile_end - item.tile_begin;
    const int per_wave = (n_tiles + 3) >> 2;
    int tile = item.tile_begin + wave * per_wave;
    const int tile_stop = min(item.tile_end, tile + per_wave);
    // Where a tile lives comes from the call's tile table (written by the plan builder), read with a
    // scalar load one tile ahead of the loads it steers; the first one is requested here, in front of
    // the query, so that the wave's first K/V loads do not wait behind a search through the segments.
    typedef int i32x4 __attribute__((ext_vector_type(4)));
    const PcTile *tile_tab = L.tiles + item.tile_tab0;   // (from the work item: requested beside the call descriptor, not behind it)
    auto describe = [&](int t) {
        const int tc = __builtin_amdgcn_readfirstlane(max(0, min(t, item.tile_end - 1)));
        if (item.tile_end <= 0) return (i32x4){0, 0, 0, 0};                   // a call that sees nothing has no table
        return *reinterpret_cast<const __attribute__((address_space(4))) i32x4 *>(reinterpret_cast<uintptr_t>(tile_tab + tc));
    };
    i32x4 next_desc = describe(tile);                    // {slot0, key0, seg, valid | flags}

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
                // (the softmax scale, times log2 e, rides on the query: scores come out of the MFMA ready for exp2)
                qh[ks][j] = col_ok ? (x * cs.x - y * cs.y) * L.scale_log2 : 0.f;
                qh[ks + 2][j] = col_ok ? (x * cs.y + y * cs.x) * L.scale_log2 : 0.f;
            }
        }
    }

    const uint16_t *kb = (const uint16_t *)L.k_store + (int64_t)kh * L.slots * PC_D;
    const uint16_t *vb = (const uint16_t *)L.v_store + (int64_t)kh * L.slots * PC_D;

    float m_run = -INFINITY, l_run = 0.f;
    f32x4 acc[8];
#pragma unroll
    for (int db = 0; db < 8; ++db) acc[db] = (f32x4){0.f, 0.f, 0.f, 0.f};

    auto fetch = [&](DecTile &T, int t) {                // t is the tile next_desc describes
        const i32x4 d = next_desc;
        next_desc = describe(t + 1);
        T.seg = d.z; T.key0 = d.y; T.valid = d.w & 0xFF; T.fresh = (d.w & PC_TILE_FRESH) != 0;
        dec_load(T, kb, vb, d.x, T.valid, lane);
    };

    int cur_seg = -1;
    bf16x8 qop[4];
    auto compute = [&](const DecTile &T) {
        if (T.fresh || cur_seg < 0) {                    // turn the query by -(segment start - stored base): a new
            cur_seg = T.seg;                             // rotation starts here, or the wave starts inside a segment
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
#pragma unroll
        for (int j = 0; j < 8; ++j) sc[j] = s[j >> 2][j & 3];
        if (T.valid < PC_TILE || T.seg == self_seg) {      // ragged or causal tile (uniform over the wave): mask
#pragma unroll
            for (int j = 0; j < 8; ++j) sc[j] = (8 * a + j < lim) ? sc[j] : -INFINITY;
        }
        float mx = fmaxf(fmaxf(fmaxf(sc[0], sc[1]), fmaxf(sc[2], sc[3])), fmaxf(fmaxf(sc[4], sc[5]), fmaxf(sc[6], sc[7])));
        mx = max_lanes_xor16(mx);
        mx = max_lanes_xor32(mx);
        const float m_new = fmaxf(m_run, mx);
        const float m_safe = (m_new == -INFINITY) ? 0.f : m_new;
        const float alpha = __builtin_amdgcn_exp2f(m_run - m_safe);
        // the row sum is taken over the probabilities as the second MFMA sees them (rounded to bf16): the
        // rounding then cancels between numerator and denominator (a row with a single key returns its V exactly)
        uint32_t pk[4];
        float ps = 0.f;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            pk[j] = pack_bf16(__builtin_amdgcn_exp2f(sc[2 * j] - m_safe), __builtin_amdgcn_exp2f(sc[2 * j + 1] - m_safe));
            ps += bf_lo(pk[j]) + bf_hi(pk[j]);
        }
        l_run = l_run * alpha + ps;
        m_run = m_new;
        const bool rescale = __builtin_amdgcn_ballot_w64(alpha != 1.f) != 0;   // rare once the running maxima have settled
        const bf16x8 pop = __builtin_bit_cast(bf16x8, make_uint4(pk[0], pk[1], pk[2], pk[3]));
#pragma unroll
        for (int db = 0; db < 8; ++db) {
            if (rescale) acc[db] *= alpha;
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
            L.part_o[(pr * L.n_q_heads + hq) * PC_D + d] = to_f16(l > 0.f ? o / l : 0.f);
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

