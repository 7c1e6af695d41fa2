// Shared decode for gfx950: a group of one-row calls that select largely the same messages
// walks the UNION of their messages once, instead of every call streaming its own copy
// (Sec. 2.4 "Parallel decoding": many calls read the same cached messages; here a K/V tile
// is loaded once per KV head for all of them).
//
// The query rows of the group (one per call) times the g query heads of a KV head are the
// columns of 32x32x16 MFMAs, as in the prefill kernel: a workgroup is 8 waves, a wave owns 32
// rows of one head.  What differs from prefill:
//   * a row sees a message only if its call lists it: one bit per (message, row);
//   * each call places a message at its own start, so the queries are turned per (message, row)
//     from a table of (cos, sin)((start - stored base) theta_i) the host lists and a small
//     kernel fills;
//   * the rows are independent calls, so there is no causal structure: a call's own growing
//     tail is just one more message that only its row sees.
// The loop is the plain one (stage a tile through registers into one of two LDS buffers, one
// barrier per tile, ordinary online softmax): the path is bound by the one pass over the
// union's bytes, not by the MFMA rate.
//
// Register/LDS layouts (fragment addressing, key permutation of the score rows, accumulator
// layout) are those of the prefill kernel, so that split partials and the merge are shared.
#include "pc_mfma_common.h"

#define MFMA32(a, b, c) __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0)

namespace {

__device__ __forceinline__ float sh_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float sh_max_halves(float x)
{
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float sh_sum_halves(float x)
{
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

}  // namespace

// (cos, sin)(pos * theta_i) for every listed (message, row) pair; PC_SH_ABSENT entries are skipped
__global__ __launch_bounds__(256) void pc_shared_rot_kernel(const int32_t *__restrict__ pos, int64_t n_ent,
                                                            const double *__restrict__ inv_freq, int half,
                                                            float2 *__restrict__ rot)
{
    const int64_t tid = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (tid >= n_ent * half) return;
    const int64_t ent = tid / half;
    const int i = (int)(tid - ent * half);
    const int p = pos[ent];
    if (p == PC_SH_ABSENT) return;
    double s, c;
    sincos((double)p * inv_freq[i], &s, &c);
    rot[tid] = make_float2((float)c, (float)s);
}

__global__ __launch_bounds__(512, 1) void pc_decode_shared_bf16_kernel(PcLaunch L, PcShLaunch S)
{
    __shared__ __attribute__((aligned(1024))) unsigned char s_k[2][8192];
    __shared__ __attribute__((aligned(1024))) unsigned char s_v[2][8192];

    const int kh = blockIdx.x % L.n_kv_heads;          // consecutive workgroups (one per XCD) take different KV heads
    const PcShItem item = S.items[blockIdx.x / L.n_kv_heads];
    const PcShGroup gr = S.groups[item.group];
    const int g = L.n_q_heads / L.n_kv_heads;            // 1, 2, 4 or 8: a workgroup covers 8 / g blocks of 32 rows
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n = lane & 31, hh = lane >> 5;
    const int ub = wave / g, uj = wave - ub * g;
    const int h = kh * g + uj;
    const int row = 32 * ub + n;
    const bool row_ok = row < gr.n_rows;
    const int Rg = gr.row0 + (row_ok ? row : 0);         // the group's calls are consecutive one-row calls

    // query turned by its own position, scaled by softmax_scale * log2(e), fp32:
    // x[ks][j] is dim 16*ks + 8*hh + j, y[ks][j] is dim 64 + 16*ks + 8*hh + j
    float x[4][8], y[4][8];
    {
        const uint16_t *qp = (const uint16_t *)L.q + ((int64_t)Rg * L.n_q_heads + h) * PC_D + 8 * hh;
        const float2 *rq = L.rot_q + (int64_t)Rg * (PC_D / 2) + 8 * hh;
        const float sc = row_ok ? L.scale_log2 : 0.f;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            const uint4 lo = ldg16(qp + 16 * ks), hi = ldg16(qp + 16 * ks + 64);
            const uint32_t lw[4] = {lo.x, lo.y, lo.z, lo.w}, hw[4] = {hi.x, hi.y, hi.z, hi.w};
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const float a = ((j & 1) ? bf_hi(lw[j >> 1]) : bf_lo(lw[j >> 1])) * sc;
                const float b = ((j & 1) ? bf_hi(hw[j >> 1]) : bf_lo(hw[j >> 1])) * sc;
                const float2 cs = rq[16 * ks + j];
                x[ks][j] = a * cs.x - b * cs.y;
                y[ks][j] = a * cs.y + b * cs.x;
            }
        }
    }

    const unsigned char *kb = (const unsigned char *)L.k_store + (int64_t)kh * L.slots * PC_D * 2;
    const unsigned char *vb = (const unsigned char *)L.v_store + (int64_t)kh * L.slots * PC_D * 2;
    // staging: a tile is 512 16-byte chunks, one per thread; LDS chunk position p of a K tile
    // holds logical chunk (p & 15) ^ ((p >> 4) & 15) of key row p >> 4 (bank-conflict-free fragment reads)
    const unsigned k_src_off = (threadIdx.x >> 4) * 256 + (((threadIdx.x & 15) ^ ((threadIdx.x >> 4) & 15)) << 4);
    const unsigned v_src_off = threadIdx.x * 16;
    // K row read by this lane for MFMA row n: rows are permuted so that score registers 0..7 / 8..15
    // of a lane are keys 8*hh + 0..7 / 16 + 8*hh + 0..7 (the layout the second MFMA's B operand wants)
    const int krow = 16 * (n >> 4) + 8 * ((n >> 2) & 1) + 4 * ((n >> 3) & 1) + (n & 3);

    float m_run = -INFINITY, l_run = 0.f;
    f32x16 acc[4];
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[db][r] = 0.f;

    // segment cursor over the group's union list (uniform over the workgroup)
    const PcShSeg *segs = S.segs + gr.seg_off;
    int e = 0, seg_slot = 0, seg_len = 0, seg_tile0 = 0, seg_tiles_end = 0;
    bool vis = false;
    auto seek = [&](int t) {
        if (seg_tiles_end == 0) {                        // first use: binary search
            int lo = 0, hi = gr.n_seg - 1;
            while (lo < hi) {
                const int mid = (lo + hi + 1) >> 1;
                if (segs[mid].tile_off <= t) lo = mid; else hi = mid - 1;
            }
            e = lo - 1;
        }
        while (t >= seg_tiles_end) {
            ++e;
            seg_slot = segs[e].slot_start; seg_len = segs[e].len; seg_tile0 = segs[e].tile_off;
            seg_tiles_end = seg_tile0 + (seg_len + PC_TILE - 1) / PC_TILE;
        }
    };

    bf16x8 qop[8];
    int cur_seg = -1;
    // turn this lane's row by -(start - base) of the message for its call; rows that do not list the
    // message keep whatever operands they have (their scores are masked)
    auto turn = [&](int seg) {
        cur_seg = seg;
        vis = row_ok && ((segs[seg].vis[ub] >> n) & 1u);
        if (vis) {
            const float4 *rs = reinterpret_cast<const float4 *>(S.rot + ((int64_t)gr.rot_off + (int64_t)seg * gr.n_rows + row) * (PC_D / 2) + 8 * hh);
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                uint32_t lo[4], hi[4];
#pragma unroll
                for (int j2 = 0; j2 < 4; ++j2) {
                    const float4 c = rs[(16 * ks + 2 * j2) >> 1];       // (cos, sin) of pairs 2*j2, 2*j2 + 1
                    const float x0 = x[ks][2 * j2], y0 = y[ks][2 * j2], x1 = x[ks][2 * j2 + 1], y1 = y[ks][2 * j2 + 1];
                    lo[j2] = pack_bf16(x0 * c.x + y0 * c.y, x1 * c.z + y1 * c.w);
                    hi[j2] = pack_bf16(y0 * c.x - x0 * c.y, y1 * c.z - x1 * c.w);
                }
                qop[ks] = __builtin_bit_cast(bf16x8, make_uint4(lo[0], lo[1], lo[2], lo[3]));
                qop[ks + 4] = __builtin_bit_cast(bf16x8, make_uint4(hi[0], hi[1], hi[2], hi[3]));
            }
        }
    };
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) qop[ks] = __builtin_bit_cast(bf16x8, make_uint4(0, 0, 0, 0));

    auto compute = [&](int buf, int valid) {
        const unsigned char *kt = &s_k[buf][0], *vt = &s_v[buf][0];
        f32x16 s;
#pragma unroll
        for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            const bf16x8 kf = *reinterpret_cast<const bf16x8 *>(kt + krow * 256 + (((2 * ks + hh) ^ (krow & 15)) << 4));
            s = MFMA32(kf, qop[ks], s);
        }
        const int lim = vis ? valid : 0;
        float mx = -INFINITY;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int key = 16 * (r >> 3) + 8 * hh + (r & 7);
            s[r] = (key < lim) ? s[r] : -INFINITY;
            mx = fmaxf(mx, s[r]);
        }
        mx = sh_max_halves(mx);
        const float m_new = fmaxf(m_run, mx);
        const float m_safe = (m_new == -INFINITY) ? 0.f : m_new;
        const float alpha = sh_exp2(m_run - m_safe);     // 0 while nothing has been seen
        float ps = 0.f;
        uint32_t pk[8];
#pragma unroll
        for (int r = 0; r < 16; r += 2) {
            const float p0 = sh_exp2(s[r] - m_safe), p1 = sh_exp2(s[r + 1] - m_safe);
            ps += p0 + p1;
            pk[r >> 1] = pack_bf16(p0, p1);
        }
        l_run = l_run * alpha + ps;
        m_run = m_new;
        if (__builtin_amdgcn_ballot_w64(alpha != 1.f) != 0) {
#pragma unroll
            for (int db = 0; db < 4; ++db) acc[db] *= alpha;
        }
        const bf16x8 p0 = __builtin_bit_cast(bf16x8, make_uint4(pk[0], pk[1], pk[2], pk[3]));
        const bf16x8 p1 = __builtin_bit_cast(bf16x8, make_uint4(pk[4], pk[5], pk[6], pk[7]));
#pragma unroll
        for (int f = 0; f < 8; ++f) {
            // V fragment f: d block f & 3, key step f >> 2; group 2*(f >> 2) + hh, dim 32*(f & 3) + n
            const bf16x8 vf = *reinterpret_cast<const bf16x8 *>(vt + ((2 * (f >> 2) + hh) * PC_D + 32 * (f & 3) + n) * 16);
            acc[f & 3] = MFMA32(vf, (f >> 2) ? p1 : p0, acc[f & 3]);
        }
    };

    // the walk: tile t is computed from LDS buffer (t - tile_begin) & 1 while tile t + 1 is on its way
    // from global memory in two registers per thread
    const int t0 = item.tile_begin, t1 = item.tile_end;
    if (t0 < t1) {
        seek(t0);
        int c_seg = e, c_valid = min(PC_TILE, seg_len - (t0 - seg_tile0) * PC_TILE);
        {
            const int64_t slot0 = (int64_t)seg_slot + (int64_t)(t0 - seg_tile0) * PC_TILE;
            const uint4 a = ldg16(kb + slot0 * 256 + k_src_off), b = ldg16(vb + slot0 * 256 + v_src_off);
            *reinterpret_cast<uint4 *>(&s_k[0][threadIdx.x * 16]) = a;
            *reinterpret_cast<uint4 *>(&s_v[0][threadIdx.x * 16]) = b;
        }
        __syncthreads();
        for (int t = t0; t < t1; ++t) {
            const int buf = (t - t0) & 1;
            const bool more = t + 1 < t1;
            uint4 nk = make_uint4(0, 0, 0, 0), nv = nk;
            int n_seg_i = c_seg, n_valid = 0;
            if (more) {
                seek(t + 1);
                n_seg_i = e; n_valid = min(PC_TILE, seg_len - (t + 1 - seg_tile0) * PC_TILE);
                const int64_t slot0 = (int64_t)seg_slot + (int64_t)(t + 1 - seg_tile0) * PC_TILE;
                nk = ldg16(kb + slot0 * 256 + k_src_off);
                nv = ldg16(vb + slot0 * 256 + v_src_off);
            }
            if (c_seg != cur_seg) turn(c_seg);
            compute(buf, c_valid);
            if (more) {
                *reinterpret_cast<uint4 *>(&s_k[buf ^ 1][threadIdx.x * 16]) = nk;
                *reinterpret_cast<uint4 *>(&s_v[buf ^ 1][threadIdx.x * 16]) = nv;
            }
            __syncthreads();
            c_seg = n_seg_i; c_valid = n_valid;
        }
    }

    // epilogue: a lane holds, for its row, dims 32*db + 8*(r/4) + 4*hh + (r%4)
    const float l = sh_sum_halves(l_run);
    if (!row_ok) return;
    const float inv = l > 0.f ? 1.f / l : 0.f;
    if (gr.n_splits == 1) {
        uint16_t *o = (uint16_t *)L.out + ((int64_t)Rg * L.n_q_heads + h) * PC_D;
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
            L.lse[(int64_t)Rg * L.n_q_heads + h] = (l > 0.f) ? (m_run + log2f(l)) * 0.6931471805599453f : -INFINITY;
    } else {
        const int64_t pr = (int64_t)gr.part_off + (int64_t)item.split * gr.n_rows + row;
        uint16_t *o = L.part_o + (pr * L.n_q_heads + h) * PC_D;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                const int d = 32 * db + 8 * q4 + 4 * hh;
                uint2 w;
                w.x = pack_f16(acc[db][4 * q4] * inv, acc[db][4 * q4 + 1] * inv);
                w.y = pack_f16(acc[db][4 * q4 + 2] * inv, acc[db][4 * q4 + 3] * inv);
                *reinterpret_cast<uint2 *>(o + d) = w;
            }
        if (hh == 0) {
            L.part_ml[(pr * L.n_q_heads + h) * 2] = (l > 0.f) ? m_run : -INFINITY;
            L.part_ml[(pr * L.n_q_heads + h) * 2 + 1] = l;
        }
    }
}

void pc_launch_shared_rot(const int32_t *pos, int64_t n_ent, const double *inv_freq, int half, float2 *rot, hipStream_t st)
{
    if (n_ent <= 0) return;
    const int64_t n = n_ent * half;
    pc_shared_rot_kernel<<<(unsigned)((n + 255) / 256), 256, 0, st>>>(pos, n_ent, inv_freq, half, rot);
}

void pc_launch_decode_shared_bf16(const PcLaunch &L, const PcShLaunch &S, int n_items, hipStream_t st)
{
    if (n_items <= 0) return;
    dim3 grid((unsigned)n_items * L.n_kv_heads);
    pc_decode_shared_bf16_kernel<<<grid, 512, 0, st>>>(L, S);
}
