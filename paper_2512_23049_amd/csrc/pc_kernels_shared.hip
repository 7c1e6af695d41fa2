// Shared decode for gfx950: a group of one-row calls that select largely the same messages
// walks the UNION of their messages once, instead of every call streaming its own copy
// (Sec. 2.4 "Parallel decoding": many calls read the same cached messages; here a K/V tile
// is loaded once per KV head for all of them).
//
// The query rows of the group (one per call) times the g query heads of a KV head are the
// columns of 32x32x16 MFMAs, as in the prefill kernel: a workgroup is 8 waves, a wave owns 32 / g
// rows times the g heads.  What differs from prefill:
//   * a row sees a message only if its call lists it: one bit per (message, row);
//   * each call places a message at its own start, so the queries are turned per (message, row)
//     from a table of (cos, sin)((start - stored base) theta_i) the host lists and a small
//     kernel fills;
//   * the rows are independent calls, so there is no causal structure: a call's own growing
//     tail is just one more message that only its row sees.
// K and V tiles go global -> LDS directly (16 bytes per lane, no staging registers) into a
// ring of four slots, requested three tiles ahead (the two requests of a tile are issued between the
// score MFMAs, where they queue behind nothing); one barrier per tile; the softmax keeps the prefill
// kernel's lazily moved reference, and a row that does not list the message subtracts +inf instead of
// its reference, which takes its probabilities to zero without a select per score.  The tile step is
// not software-pipelined: score MFMAs, softmax and P.V MFMAs of a wave follow each other.
//
// Register/LDS layouts (fragment addressing, key permutation of the score rows, accumulator
// layout) are those of the prefill kernel, so that split partials and the merge are shared.
#include "pc_mfma_common.h"

#define MFMA32(a, b, c) __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0)

namespace {

__device__ __forceinline__ float sh_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float sh_max3(float a, float b, float c) { return __builtin_fmaxf(__builtin_fmaxf(a, b), c); }
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

// One 16-byte-per-lane direct load: lane l's 16 bytes land at lds_wave_base + 16*l.  Assembly, so
// that the compiler keeps no record of the LDS write and does not drain every outstanding request
// in front of later LDS reads or at barriers; completion is awaited with s_waitcnt vmcnt(n).
__device__ __forceinline__ void sh_dma16(const void *gbase_uniform, unsigned lane_off, unsigned lds_wave_base)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 ::"s"(lds_wave_base), "v"(lane_off), "s"(gbase_uniform) : "memory", "m0");
}
// workgroup barrier without the fence of __syncthreads() (which would wait for every direct load)
__device__ __forceinline__ void sh_barrier() { asm volatile("s_barrier" ::: "memory"); }

#define SH_RING 4                 // ring slots of 16 KB (K and V tile)
#define SH_AHEAD (SH_RING - 1)    // tiles in flight beyond the one being computed
#define SH_LAZY 8.0f               // log2 of how far a tile's maximum may exceed the softmax reference before it moves
// wait until at most the 2 * (SH_AHEAD - 1) youngest direct loads of this wave are outstanding
__device__ __forceinline__ void sh_wait_landed()
{
    constexpr int n = 2 * (SH_AHEAD - 1);
    __builtin_amdgcn_s_waitcnt(0x0F70 | (n & 15) | ((n >> 4) << 14));     // vmcnt: bits 3:0 and 15:14
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
    __shared__ __attribute__((aligned(1024))) unsigned char s_k[SH_RING][8192];
    __shared__ __attribute__((aligned(1024))) unsigned char s_v[SH_RING][8192];
    __shared__ __attribute__((aligned(16))) float4 s_qm[8][8][64];    // upper half (dims 64..127) of the fp32 query master

    const int kh = blockIdx.x % L.n_kv_heads;          // consecutive workgroups (one per XCD) take different KV heads
    const PcShItem item = S.items[blockIdx.x / L.n_kv_heads];
    const PcShGroup gr = S.groups[item.group];
    const int g = L.n_q_heads / L.n_kv_heads;            // 1, 2, 4 or 8: a workgroup covers 8 / g blocks of 32 rows
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n = lane & 31, hh = lane >> 5;
    // A wave's 32 columns are 32 / g rows (calls) times the g heads of the KV head, head fastest: the lanes of
    // a wave then need the rotation rows of only 32 / g calls (for g = 8 an eighth of the table traffic of a
    // wave that held 32 rows of one head).  The workgroup covers 8 * 32 / g rows either way.
    const int rpw = 32 / g;
    const int row = rpw * wave + n / g;
    const int h = kh * g + n % g;
    const int ub = (rpw * wave) >> 5;                   // the 32-row block of the visibility masks this wave's rows lie in
    const bool row_ok = row < gr.n_rows;
    const int Rg = gr.row0 + (row_ok ? row : 0);         // the group's calls are consecutive one-row calls

    // query turned by its own position, scaled by softmax_scale * log2(e), fp32: x[ks][j] is dim
    // 16*ks + 8*hh + j (registers); its partner 64 dims up is kept in LDS (s_qm[wave][2*ks + j/4][lane],
    // read back once per message): the registers are needed for the MFMA fragments
    float x[4][8];
    {
        const uint16_t *qp = (const uint16_t *)L.q + ((int64_t)Rg * L.n_q_heads + h) * PC_D + 8 * hh;
        const float2 *rq = L.rot_q + (int64_t)Rg * (PC_D / 2) + 8 * hh;
        const float sc = row_ok ? L.scale_log2 : 0.f;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            const uint4 lo = ldg16(qp + 16 * ks), hi = ldg16(qp + 16 * ks + 64);
            const uint32_t lw[4] = {lo.x, lo.y, lo.z, lo.w}, hw[4] = {hi.x, hi.y, hi.z, hi.w};
            float yy[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const float a = ((j & 1) ? bf_hi(lw[j >> 1]) : bf_lo(lw[j >> 1])) * sc;
                const float b = ((j & 1) ? bf_hi(hw[j >> 1]) : bf_lo(hw[j >> 1])) * sc;
                const float2 cs = rq[16 * ks + j];
                x[ks][j] = a * cs.x - b * cs.y;
                yy[j] = a * cs.y + b * cs.x;
            }
            s_qm[wave][2 * ks][lane] = make_float4(yy[0], yy[1], yy[2], yy[3]);
            s_qm[wave][2 * ks + 1][lane] = make_float4(yy[4], yy[5], yy[6], yy[7]);
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

    unsigned k_off[8];                                   // byte offset of K fragment ks within a tile, for this lane
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) k_off[ks] = (unsigned)(krow * 256 + (((2 * ks + hh) ^ (krow & 15)) << 4));

    // Softmax state of this lane's column, as in the prefill kernel: probabilities are 2^(score - m_ref)
    // with a reference that starts at 0 and moves only when it has to (a tile's maximum more than
    // 2^SH_LAZY above it, or a row's first scores more than 2^SH_LAZY below it).  While no lane of the
    // wave has moved its reference the scores are not shifted at all.
    float m_ref = 0.f, thr_lo = -SH_LAZY, l_run = 0.f;
    bool shifted = false;                                // some lane of this wave has m_ref != 0
    f32x16 acc[4];
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[db][r] = 0.f;

    // Cursor of the REQUESTS over the group's union list (uniform over the workgroup): tiles are
    // requested in order, so it only moves forward; the descriptor of the segment after the
    // current one is loaded when the cursor enters a segment, several tiles before it is needed.
    const PcShSeg *segs = S.segs + gr.seg_off;
    struct SegD { int slot, len, tile0; unsigned vis; };
    // (scalar loads: they are counted apart from the direct loads, so waiting for a descriptor does
    // not drain the ring)
    typedef int i32x4 __attribute__((ext_vector_type(4)));
    const int ub_s = __builtin_amdgcn_readfirstlane(ub);
    auto load_seg = [&](int e) {
        const int ec = __builtin_amdgcn_readfirstlane(min(e, gr.n_seg - 1));
        const uintptr_t at = reinterpret_cast<uintptr_t>(segs + ec);
        const i32x4 w = *reinterpret_cast<const __attribute__((address_space(4))) i32x4 *>(at);
        SegD d;
        d.slot = w.x; d.len = w.y; d.tile0 = w.z;
        d.vis = *reinterpret_cast<const __attribute__((address_space(4))) unsigned *>(at + 16 + 4 * ub_s);
        return d;
    };
    int e = item.seg_begin;                              // the message that owns the first tile (found by the host)
    SegD sg = load_seg(e), sg_next = load_seg(e + 1);
    // a tile in flight: where it comes from is only needed for the request; what the compute step
    // needs travels in these three scalars
    struct TileD { int seg, valid; unsigned vis; };
    const unsigned wave_lds = __builtin_amdgcn_readfirstlane(wave) * 1024;
    const unsigned lds_k = (unsigned)(size_t)&s_k[0][0] + wave_lds, lds_v = (unsigned)(size_t)&s_v[0][0] + wave_lds;
    int64_t req_slot0 = 0;
    auto request = [&](int t) {                          // t in [tile_begin, tile_end): where the tile lives; the loads are issued apart
        while (t >= sg.tile0 + (sg.len + PC_TILE - 1) / PC_TILE) { ++e; sg = sg_next; sg_next = load_seg(e + 1); }
        const int key0 = (t - sg.tile0) * PC_TILE;
        req_slot0 = (int64_t)__builtin_amdgcn_readfirstlane(sg.slot) + key0;
        TileD d;
        d.seg = e; d.valid = min(PC_TILE, sg.len - key0); d.vis = sg.vis;
        return d;
    };
    auto issue_k = [&](int ring) { sh_dma16(kb + req_slot0 * 256, k_src_off, lds_k + ring * 8192); };
    auto issue_v = [&](int ring) { sh_dma16(vb + req_slot0 * 256, v_src_off, lds_v + ring * 8192); };

    bf16x8 qop[8];
    int cur_seg = -1;
    // turn this lane's row by -(start - base) of the message for its call; rows that do not list the
    // message keep whatever operands they have (their scores are masked)
    bool vis = false;
    auto turn = [&](int seg, unsigned vis_word) {
        cur_seg = seg;
        vis = row_ok && ((vis_word >> (row & 31)) & 1u);
        if (vis) {
            const float4 *rs = reinterpret_cast<const float4 *>(S.rot + ((int64_t)gr.rot_off + (int64_t)seg * gr.n_rows + row) * (PC_D / 2) + 8 * hh);
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                uint32_t lo[4], hi[4];
#pragma unroll
                for (int j4 = 0; j4 < 2; ++j4) {
                    const float4 c0 = rs[(16 * ks + 4 * j4) >> 1];          // (cos, sin) of pairs 4*j4, 4*j4 + 1
                    const float4 c1 = rs[((16 * ks + 4 * j4) >> 1) + 1];    // ... 4*j4 + 2, 4*j4 + 3
                    const float x0 = x[ks][4 * j4], x1 = x[ks][4 * j4 + 1], x2 = x[ks][4 * j4 + 2], x3 = x[ks][4 * j4 + 3];
                    const float4 yv = s_qm[wave][2 * ks + j4][lane];
                    lo[2 * j4] = pack_bf16(x0 * c0.x + yv.x * c0.y, x1 * c0.z + yv.y * c0.w);
                    hi[2 * j4] = pack_bf16(yv.x * c0.x - x0 * c0.y, yv.y * c0.z - x1 * c0.w);
                    lo[2 * j4 + 1] = pack_bf16(x2 * c1.x + yv.z * c1.y, x3 * c1.z + yv.w * c1.w);
                    hi[2 * j4 + 1] = pack_bf16(yv.z * c1.x - x2 * c1.y, yv.w * c1.z - x3 * c1.w);
                }
                qop[ks] = __builtin_bit_cast(bf16x8, make_uint4(lo[0], lo[1], lo[2], lo[3]));
                qop[ks + 4] = __builtin_bit_cast(bf16x8, make_uint4(hi[0], hi[1], hi[2], hi[3]));
            }
        }
    };
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) qop[ks] = __builtin_bit_cast(bf16x8, make_uint4(0, 0, 0, 0));

    auto compute = [&](int buf, int valid, int req_ring) {
        const unsigned char *kt = &s_k[buf][0], *vt = &s_v[buf][0];
        // all eight K fragments are requested up front; each is replaced by a V fragment as soon as its
        // MFMA has consumed it, so the P.V MFMAs find their operands in registers
        bf16x8 fr[8];
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) fr[ks] = *reinterpret_cast<const bf16x8 *>(kt + k_off[ks]);
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) asm volatile("" : "+v"(fr[ks]));      // (keeps the compiler from moving each read down to its MFMA)
        f32x16 s;
#pragma unroll
        for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            s = MFMA32(fr[ks], qop[ks], s);
            if (ks == 1) issue_k(req_ring);
            if (ks == 5) issue_v(req_ring);
            // V fragment f: d block f & 3, key step f >> 2; group 2*(f >> 2) + hh, dim 32*(f & 3) + n
            fr[ks] = *reinterpret_cast<const bf16x8 *>(vt + ((2 * (ks >> 2) + hh) * PC_D + 32 * (ks & 3) + n) * 16);
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
        if (valid < PC_TILE) {                           // ragged last tile of a message (uniform): keys past its end
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int key = 16 * (r >> 3) + 8 * hh + (r & 7);
                s[r] = (key < valid) ? s[r] : -INFINITY;
            }
        }
        {                                                // a row that does not list the message: every score to -inf
            const float m_eff = vis ? m_ref : INFINITY;
#pragma unroll
            for (int r = 0; r < 16; ++r) s[r] -= m_eff;
        }
        float mx = sh_max3(sh_max3(s[0], s[1], s[2]), s[3], s[4]);
        mx = sh_max3(sh_max3(mx, s[5], s[6]), s[7], s[8]);
        mx = sh_max3(sh_max3(mx, s[9], s[10]), s[11], s[12]);
        mx = sh_max3(sh_max3(mx, s[13], s[14]), s[15], s[15]);
        mx = sh_max_halves(mx);
        {
            const uint64_t above = __builtin_amdgcn_ballot_w64(mx > SH_LAZY);
            const uint64_t below = __builtin_amdgcn_ballot_w64(mx < thr_lo);
            const bool seen = mx > -INFINITY;
            const uint64_t need_mask = above | (below & __builtin_amdgcn_ballot_w64(seen));
            thr_lo = seen ? -INFINITY : thr_lo;
            if (__builtin_expect(need_mask != 0, 0)) {
                const bool need = (need_mask >> lane) & 1;
                const float shift = need ? mx : 0.f;
                // (moving down happens only at a row's first scores, with nothing accumulated: the factor is
                // irrelevant then, and 2^-shift could overflow into 0 * inf; it is taken as 1)
                const float alpha = sh_exp2(-fmaxf(shift, 0.f));
                l_run *= alpha;
#pragma unroll
                for (int db = 0; db < 4; ++db) acc[db] *= alpha;
                m_ref += shift;
#pragma unroll
                for (int r = 0; r < 16; ++r) s[r] -= shift;
                shifted = __builtin_amdgcn_ballot_w64(m_ref != 0.f) != 0;
            }
        }
        float ps = 0.f;
        uint32_t pk[8];
#pragma unroll
        for (int r = 0; r < 16; r += 2) {
            const float p0 = sh_exp2(s[r]), p1 = sh_exp2(s[r + 1]);
            ps += p0 + p1;
            pk[r >> 1] = pack_bf16(p0, p1);
        }
        l_run += ps;
        const bf16x8 p0 = __builtin_bit_cast(bf16x8, make_uint4(pk[0], pk[1], pk[2], pk[3]));
        const bf16x8 p1 = __builtin_bit_cast(bf16x8, make_uint4(pk[4], pk[5], pk[6], pk[7]));
#pragma unroll
        for (int f = 0; f < 8; ++f) acc[f & 3] = MFMA32(fr[f], (f >> 2) ? p1 : p0, acc[f & 3]);
    };

    // The walk.  Ring slot of tile t is (t - t0) mod SH_RING; SH_AHEAD tiles are in flight beyond the
    // one being computed.  Requests beyond the last tile repeat the last one, so that the number of
    // requests in flight is the same at every wait.
    const int t0 = item.tile_begin, t1 = item.tile_end;
    if (t0 < t1) {
        const int last = t1 - 1;
        TileD d[SH_AHEAD + 1];
#pragma unroll
        for (int i = 0; i < SH_AHEAD; ++i) { d[i] = request(min(t0 + i, last)); issue_k(i); issue_v(i); }
        sh_wait_landed();                                // the first tile has landed
        sh_barrier();
        for (int t = t0; t < t1; ++t) {
            const int ring = (t - t0) & (SH_RING - 1);
            // (the table loads of a turn go first: issued behind the new requests they would have to wait for them)
            if (d[0].seg != cur_seg) turn(d[0].seg, d[0].vis);
            // tile t + SH_AHEAD takes the slot of tile t - 1, which every wave left before the last barrier
            d[SH_AHEAD] = request(min(t + SH_AHEAD, last));
            compute(ring, d[0].valid, (ring + SH_AHEAD) & (SH_RING - 1));
            sh_wait_landed();                            // tile t + 1 has landed (the later ones may be in flight)
            sh_barrier();
#pragma unroll
            for (int i = 0; i < SH_AHEAD; ++i) d[i] = d[i + 1];
        }
        __builtin_amdgcn_s_waitcnt(0x0F70);              // drain the repeated requests
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
            L.lse[(int64_t)Rg * L.n_q_heads + h] = (l > 0.f) ? (m_ref + log2f(l)) * 0.6931471805599453f : -INFINITY;
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
            L.part_ml[(pr * L.n_q_heads + h) * 2] = (l > 0.f) ? m_ref : -INFINITY;
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
