// Gradient kernels (plain fp32 vector code; this path is not a hot one).
#include "pc_kernels.h"

// ----------------------------------------------------------------------------------
// Gradient of the attention, for both cache dtypes, in fp32 arithmetic (Sec. 2.4: in fine-tuning a position update is applied
// non-destructively, so gradients flow through it to the cached keys).  One wave per
// (query row, head), keys lane-strided as in the forward kernel.  With p_j = exp(s_j - LSE)
// from the forward's LSE and dp_j = dO . v_j:
//   Delta = sum_j p_j dp_j,   ds_j = p_j (dp_j - Delta),
//   dV_j += p_j dO,   dK~_j += scale ds_j qe,   dqe += scale ds_j K~_j
// where K~ is the stored key (turned to base + t) and qe the query turned for the segment;
// dqe is turned back per segment and once more by the row's own position at the end.
// d_k collects the gradient with respect to the STORED keys (pc_grad_keys_finalize turns
// it into the gradient with respect to the keys as they were appended).  Two kernels: this one, row-major,
// gives Delta and the gradient of the query; the key-major one below gives those of the keys and values.
// Plain fp32 vector code: this path is not a hot one.
// ----------------------------------------------------------------------------------
// element access for the two cache dtypes: fp32 as it is, bf16 widened; V of a bf16 cache is stored
// key-transposed in groups of 8 slots
template <typename T> __device__ __forceinline__ float bwd_ld(const T *p);
template <> __device__ __forceinline__ float bwd_ld<float>(const float *p) { return *p; }
template <> __device__ __forceinline__ float bwd_ld<uint16_t>(const uint16_t *p) { return __uint_as_float((uint32_t)*p << 16); }
template <typename T> __device__ __forceinline__ float bwd_v(const T *vbase, int64_t slot, int d, int D)
{
    if constexpr (sizeof(T) == 2) return bwd_ld(vbase + ((slot / PC_VGROUP) * D + d) * PC_VGROUP + (slot % PC_VGROUP));
    else return vbase[slot * D + d];
}

template <int D, typename T>
__global__ __launch_bounds__(64) void pc_attend_bwd_kernel(PcLaunch L, const int32_t *__restrict__ row_call,
                                                           const float *__restrict__ lse, const T *__restrict__ d_out,
                                                           float scale, float *__restrict__ d_q,
                                                           float *__restrict__ delta_out)
{
    constexpr int HALF = D / 2;
    __shared__ float s_qhat[D], s_qe[D], s_do[D], s_dqhat[D];
    __shared__ float s_red[64 * (D + 1)];
    const int R = blockIdx.x, h = blockIdx.y, lane = threadIdx.x;
    const PcCallDesc cd = L.calls[row_call[R]];
    const int r = R - cd.q_off;
    const int g = L.n_q_heads / L.n_kv_heads;
    const int kh = h / g;
    const int64_t rh = (int64_t)R * L.n_q_heads + h;
    const T *q = (const T *)L.q + rh * D;
    for (int i = lane; i < HALF; i += 64) {
        const float2 cs = L.rot_q[(int64_t)R * HALF + i];
        const float a = bwd_ld(q + i), b = bwd_ld(q + i + HALF);
        s_qhat[i] = a * cs.x - b * cs.y;
        s_qhat[i + HALF] = a * cs.y + b * cs.x;
    }
    for (int d = lane; d < D; d += 64) { s_do[d] = bwd_ld(d_out + rh * D + d); s_dqhat[d] = 0.f; }
    const float row_lse = lse[rh];
    float *dq = d_q + rh * D;
    if (!(row_lse > -INFINITY)) {                          // the row saw nothing: no gradient anywhere
        for (int d = lane; d < D; d += 64) dq[d] = 0.f;
        if (lane == 0) delta_out[rh] = 0.f;
        return;
    }
    __syncthreads();
    const T *kbase = (const T *)L.k_store + (int64_t)kh * L.slots * D;
    const T *vbase = (const T *)L.v_store + (int64_t)kh * L.slots * D;
    auto visible = [&](const PcSegment &sg, int e) {
        int n_vis = sg.len;
        if (cd.self_msg >= 0 && e == cd.n_seg - 1) {
            const int lim = cd.self_len - cd.n_q + r + 1;
            n_vis = lim < n_vis ? lim : n_vis;
        }
        return n_vis;
    };
    auto turn = [&](int e) {                               // s_qe = query turned by -(start - base) of segment e
        __syncthreads();
        for (int i = lane; i < HALF; i += 64) {
            const float2 cs = L.rot_seg[(int64_t)(cd.seg_off + e) * HALF + i];
            const float a = s_qhat[i], b = s_qhat[i + HALF];
            s_qe[i] = a * cs.x + b * cs.y;
            s_qe[i + HALF] = -a * cs.y + b * cs.x;
        }
        __syncthreads();
    };
    // pass 1: Delta
    float delta = 0.f;
    for (int e = 0; e < cd.n_seg; ++e) {
        const PcSegment sg = L.segs[cd.seg_off + e];
        const int n_vis = visible(sg, e);
        if (n_vis <= 0) continue;
        turn(e);
        for (int t = lane; t < n_vis; t += 64) {
            const int64_t slot = sg.slot_start + t;
            const T *kr = kbase + slot * D;
            float s = 0.f, dp = 0.f;
#pragma unroll 8
            for (int d = 0; d < D; ++d) { s = fmaf(s_qe[d], bwd_ld(kr + d), s); dp = fmaf(s_do[d], bwd_v(vbase, slot, d, D), dp); }
            delta += expf(s * scale - row_lse) * dp;
        }
    }
    for (int off = 32; off > 0; off >>= 1) delta += __shfl_xor(delta, off);
    if (lane == 0) delta_out[rh] = delta;                  // the key-major kernel needs it too
    // pass 2: the gradient of the query
    for (int e = 0; e < cd.n_seg; ++e) {
        const PcSegment sg = L.segs[cd.seg_off + e];
        const int n_vis = visible(sg, e);
        if (n_vis <= 0) continue;
        turn(e);
        float dqe[D];
#pragma unroll
        for (int d = 0; d < D; ++d) dqe[d] = 0.f;
        for (int t = lane; t < n_vis; t += 64) {
            const int64_t slot = sg.slot_start + t;
            const T *kr = kbase + slot * D;
            float s = 0.f, dp = 0.f;
#pragma unroll 8
            for (int d = 0; d < D; ++d) { s = fmaf(s_qe[d], bwd_ld(kr + d), s); dp = fmaf(s_do[d], bwd_v(vbase, slot, d, D), dp); }
            const float p = expf(s * scale - row_lse);
            const float ds = p * (dp - delta) * scale;
#pragma unroll 8
            for (int d = 0; d < D; ++d) dqe[d] = fmaf(ds, bwd_ld(kr + d), dqe[d]);
        }
        // sum the lanes' dqe, turn it back by +(start - base), add to the gradient of the position-turned query
        __syncthreads();
#pragma unroll
        for (int d = 0; d < D; ++d) s_red[lane * (D + 1) + d] = dqe[d];
        __syncthreads();
        for (int i = lane; i < HALF; i += 64) {
            float a = 0.f, b = 0.f;
            for (int j = 0; j < 64; ++j) { a += s_red[j * (D + 1) + i]; b += s_red[j * (D + 1) + i + HALF]; }
            const float2 cs = L.rot_seg[(int64_t)(cd.seg_off + e) * HALF + i];
            s_dqhat[i] += a * cs.x - b * cs.y;
            s_dqhat[i + HALF] += a * cs.y + b * cs.x;
        }
    }
    __syncthreads();
    for (int i = lane; i < HALF; i += 64) {                // back through the row's own position
        const float2 cs = L.rot_q[(int64_t)R * HALF + i];
        const float a = s_dqhat[i], b = s_dqhat[i + HALF];
        dq[i] = a * cs.x + b * cs.y;
        dq[i + HALF] = -a * cs.y + b * cs.x;
    }
}

// Key-major half of the gradient: a block owns 16 tokens of one gathered segment (one placement of a message
// in one call) and one KV head, four lanes per token with D/4 dims each, and walks the call's query rows and
// the g heads of the group: the sums over rows and heads stay in registers, and a token's gradient meets
// those of its other placements (other calls, repeated listings) in d_k, d_v through one float atomic per
// element at the end.
template <int D, typename T>
__global__ __launch_bounds__(64) void pc_attend_bwd_kv_kernel(PcLaunch L, int n_calls, const float *__restrict__ lse,
                                                              const T *__restrict__ d_out, const float *__restrict__ delta,
                                                              float scale, float *__restrict__ d_k, float *__restrict__ d_v)
{
    constexpr int HALF = D / 2, Q = D / 4;
    __shared__ float s_qe[D], s_do[D];
    const int seg = blockIdx.x, chunk = blockIdx.y, kh = blockIdx.z, tid = threadIdx.x;   // (segments on x: no 65535 limit)
    // the call that owns this segment (segments are laid out call by call)
    int lo = 0, hi = n_calls - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (L.calls[mid].seg_off <= seg) lo = mid; else hi = mid - 1;
    }
    const PcCallDesc cd = L.calls[lo];
    const int e = seg - cd.seg_off;
    if (e >= cd.n_seg) return;                             // (a call without segments in front of this index)
    const PcSegment sg = L.segs[seg];
    const int t = chunk * 16 + (tid >> 2), part = tid & 3;
    if (chunk * 16 >= sg.len) return;
    const bool t_ok = t < sg.len;
    const bool is_self = cd.self_msg >= 0 && e == cd.n_seg - 1;
    const int g = L.n_q_heads / L.n_kv_heads;
    const int64_t slot = sg.slot_start + (t_ok ? t : 0);
    const T *kbase = (const T *)L.k_store + (int64_t)kh * L.slots * D;
    const T *vbase = (const T *)L.v_store + (int64_t)kh * L.slots * D;
    float kq[Q], vq[Q], dk[Q], dv[Q];
#pragma unroll
    for (int d = 0; d < Q; ++d) {
        kq[d] = bwd_ld(kbase + slot * D + part * Q + d);
        vq[d] = bwd_v(vbase, slot, part * Q + d, D);
        dk[d] = 0.f; dv[d] = 0.f;
    }
    // rows that can see this block's tokens at all: in the new message a row sees tokens up to its own
    const int r_first = is_self ? max(0, chunk * 16 - (cd.self_len - cd.n_q)) : 0;
    for (int r = r_first; r < cd.n_q; ++r) {
        const int R = cd.q_off + r;
        const int n_vis = is_self ? min(sg.len, cd.self_len - cd.n_q + r + 1) : sg.len;
        for (int j = 0; j < g; ++j) {
            const int h = kh * g + j;
            const int64_t rh = (int64_t)R * L.n_q_heads + h;
            __syncthreads();
            if (tid < HALF) {                              // the query of (row, head) turned for this segment
                const T *q = (const T *)L.q + rh * D;
                const float2 cq = L.rot_q[(int64_t)R * HALF + tid];
                const float a = bwd_ld(q + tid), b = bwd_ld(q + tid + HALF);
                const float qa = a * cq.x - b * cq.y, qb = a * cq.y + b * cq.x;
                const float2 cs = L.rot_seg[(int64_t)seg * HALF + tid];
                s_qe[tid] = qa * cs.x + qb * cs.y;
                s_qe[tid + HALF] = -qa * cs.y + qb * cs.x;
            }
            for (int d = tid; d < D; d += 64) s_do[d] = bwd_ld(d_out + rh * D + d);
            __syncthreads();
            const float row_lse = lse[rh];
            if (!(row_lse > -INFINITY)) continue;          // (uniform over the block)
            float sp = 0.f, dpp = 0.f;
#pragma unroll
            for (int d = 0; d < Q; ++d) { sp = fmaf(s_qe[part * Q + d], kq[d], sp); dpp = fmaf(s_do[part * Q + d], vq[d], dpp); }
            sp += __shfl_xor(sp, 1); sp += __shfl_xor(sp, 2);
            dpp += __shfl_xor(dpp, 1); dpp += __shfl_xor(dpp, 2);
            const float p = (t < n_vis) ? expf(sp * scale - row_lse) : 0.f;
            const float ds = p * (dpp - delta[rh]) * scale;
#pragma unroll
            for (int d = 0; d < Q; ++d) { dk[d] = fmaf(ds, s_qe[part * Q + d], dk[d]); dv[d] = fmaf(p, s_do[part * Q + d], dv[d]); }
        }
    }
    if (!t_ok) return;
    float *gk = d_k + (slot * L.n_kv_heads + kh) * D + part * Q;
    float *gv = d_v + (slot * L.n_kv_heads + kh) * D + part * Q;
#pragma unroll
    for (int d = 0; d < Q; ++d) { atomicAdd(gk + d, dk[d]); atomicAdd(gv + d, dv[d]); }
}

void pc_launch_attend_bwd(int dtype, const PcLaunch &L, const int32_t *row_call, int n_calls, int total_q, int total_seg,
                          int max_seg_len, int D, const float *lse, const void *d_out, float scale, float *delta,
                          float *d_q, float *d_k, float *d_v, hipStream_t st)
{
    if (total_q <= 0) return;
    dim3 grid(total_q, L.n_q_heads);
    dim3 grid_kv((unsigned)total_seg, (unsigned)((max_seg_len + 15) / 16), (unsigned)L.n_kv_heads);
    const bool kv = total_seg > 0 && max_seg_len > 0;
    if (dtype == 1) {
        const uint16_t *go = (const uint16_t *)d_out;
        if (D == 64) {
            pc_attend_bwd_kernel<64, uint16_t><<<grid, 64, 0, st>>>(L, row_call, lse, go, scale, d_q, delta);
            if (kv) pc_attend_bwd_kv_kernel<64, uint16_t><<<grid_kv, 64, 0, st>>>(L, n_calls, lse, go, delta, scale, d_k, d_v);
        } else {
            pc_attend_bwd_kernel<128, uint16_t><<<grid, 64, 0, st>>>(L, row_call, lse, go, scale, d_q, delta);
            if (kv) pc_attend_bwd_kv_kernel<128, uint16_t><<<grid_kv, 64, 0, st>>>(L, n_calls, lse, go, delta, scale, d_k, d_v);
        }
    } else {
        const float *go = (const float *)d_out;
        if (D == 64) {
            pc_attend_bwd_kernel<64, float><<<grid, 64, 0, st>>>(L, row_call, lse, go, scale, d_q, delta);
            if (kv) pc_attend_bwd_kv_kernel<64, float><<<grid_kv, 64, 0, st>>>(L, n_calls, lse, go, delta, scale, d_k, d_v);
        } else {
            pc_attend_bwd_kernel<128, float><<<grid, 64, 0, st>>>(L, row_call, lse, go, scale, d_q, delta);
            if (kv) pc_attend_bwd_kv_kernel<128, float><<<grid_kv, 64, 0, st>>>(L, n_calls, lse, go, delta, scale, d_k, d_v);
        }
    }
}

// d_k holds the gradient with respect to the stored keys K~_t = R(base + t) k_t; the gradient with
// respect to k_t is R(base + t)^T of it (Sec. 2.4 "Position Updates", transposed).  One thread per
// (token, KV head, rotation pair) of every listed message (blockIdx.y).
__global__ __launch_bounds__(256) void pc_grad_keys_finalize_kernel(const PcMsgEntry *__restrict__ msgs, int n_kv_heads, int D,
                                                                    const double *__restrict__ inv_freq, float *__restrict__ d_k)
{
    const PcMsgEntry m = msgs[blockIdx.y];
    const int half = D / 2;
    const int64_t n = (int64_t)m.len * n_kv_heads * half;
    for (int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x; idx < n; idx += (int64_t)gridDim.x * 256) {
        const int i = (int)(idx % half);
        const int kh = (int)((idx / half) % n_kv_heads);
        const int t = (int)(idx / ((int64_t)half * n_kv_heads));
        double sn, cs;
        sincos((double)(m.base_pos + t) * inv_freq[i], &sn, &cs);
        float *row = d_k + ((int64_t)(m.slot_start + t) * n_kv_heads + kh) * D;
        const float a = row[i], b = row[i + half];
        row[i] = a * (float)cs + b * (float)sn;
        row[i + half] = -a * (float)sn + b * (float)cs;
    }
}

void pc_launch_grad_keys_finalize(const PcMsgEntry *msgs, int n_msgs, int n_kv_heads, int D, const double *inv_freq,
                                  float *d_k, hipStream_t st)
{
    for (int first = 0; first < n_msgs; first += 65535) {              // grid.y is limited to 65535
        const int n = n_msgs - first < 65535 ? n_msgs - first : 65535;
        dim3 grid(16, (unsigned)n);
        pc_grad_keys_finalize_kernel<<<grid, 256, 0, st>>>(msgs + first, n_kv_heads, D, inv_freq, d_k);
    }
}
