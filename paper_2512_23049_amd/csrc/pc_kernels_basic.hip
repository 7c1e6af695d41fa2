// Cache append, plan builder, table expansion, split merge and the fp32 attention
// kernel.  gfx950 only.
#include "pc_kernels.h"

#include <hip/hip_bf16.h>

#include <algorithm>

// ----------------------------------------------------------------------------------
// K1: fused cache append (Sec. 2.4: new messages are appended at the end of the
// occupied part of the cache; the i-th token's key is turned to a position by RoPE).
// Stored form: the key of in-message token t is turned by t (delta-rotated form), so
// that placing the message at offset s later only needs the query turned by -s.
// bf16 caches: blockIdx.y == 0 is the K part (a block takes APP_TB consecutive tokens: its threads
// first share out the (token, frequency) rotations, one fp64 sincos each, into LDS, then each moves
// 16 bytes of the lower and of the upper half of a (token, KV head) row), blockIdx.y == 1 the V part
// (a thread transposes 8 tokens x 2 dims of one KV head).  k and v must be 16-byte aligned.
// fp32 caches (small reference configurations): one thread per (token, frequency pair) and per element.
// ----------------------------------------------------------------------------------
template <typename T> struct Pair2;
template <> struct Pair2<__hip_bfloat16> {
    using type = uint32_t;
    __device__ static float lo(uint32_t u) { return __uint_as_float(u << 16); }
    __device__ static float hi(uint32_t u) { return __uint_as_float(u & 0xFFFF0000u); }
    __device__ static uint32_t pack(float a, float b) {
        __hip_bfloat16 x = __float2bfloat16(a), y = __float2bfloat16(b);
        return (uint32_t)(*reinterpret_cast<uint16_t *>(&x)) |
               ((uint32_t)(*reinterpret_cast<uint16_t *>(&y)) << 16);
    }
};

#define APP_TB 4               // tokens per block step of the K part: 4 x 64 rotations = one sincos per thread

// K part: tokens [t0, t0 + APP_TB) of one message.  s_cs: APP_TB * 64 rotations.
__device__ __forceinline__ void append_bf16_k_block(
    const uint16_t *__restrict__ k, int len, int t0, int n_kv_heads, int D, int64_t slot_start, int64_t slots,
    const double *__restrict__ inv_freq, uint16_t *__restrict__ k_store, float2 *s_cs)
{
    const int half = D / 2;
    const int nt = min(APP_TB, len - t0);
    for (int e = threadIdx.x; e < nt * half; e += blockDim.x) {
        const int tt = e / half, i = e - tt * half;
        double s, c;
        sincos((double)(t0 + tt) * inv_freq[i], &s, &c);
        s_cs[tt * 64 + i] = make_float2((float)c, (float)s);
    }
    __syncthreads();
    const int chunks = half / 8;                         // 16-byte chunks in half a row
    const int tasks = nt * n_kv_heads * chunks;
    using P = Pair2<__hip_bfloat16>;
    for (int e = threadIdx.x; e < tasks; e += blockDim.x) {
        const int c8 = e % chunks;
        const int h = (e / chunks) % n_kv_heads;
        const int tt = e / (chunks * n_kv_heads);
        const int t = t0 + tt;
        const uint16_t *src = k + ((int64_t)t * n_kv_heads + h) * D + 8 * c8;
        uint4 lo = *reinterpret_cast<const uint4 *>(src);
        uint4 hi = *reinterpret_cast<const uint4 *>(src + half);
        uint32_t *lw = reinterpret_cast<uint32_t *>(&lo), *hw = reinterpret_cast<uint32_t *>(&hi);
        const float2 *cs = s_cs + tt * 64 + 8 * c8;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const float fc0 = cs[2 * u].x, fs0 = cs[2 * u].y, fc1 = cs[2 * u + 1].x, fs1 = cs[2 * u + 1].y;
            const float a0 = P::lo(lw[u]), a1 = P::hi(lw[u]), b0 = P::lo(hw[u]), b1 = P::hi(hw[u]);
            lw[u] = P::pack(a0 * fc0 - b0 * fs0, a1 * fc1 - b1 * fs1);
            hw[u] = P::pack(a0 * fs0 + b0 * fc0, a1 * fs1 + b1 * fc1);
        }
        uint16_t *dst = k_store + ((int64_t)h * slots + slot_start + t) * D + 8 * c8;
        *reinterpret_cast<uint4 *>(dst) = lo;
        *reinterpret_cast<uint4 *>(dst + half) = hi;
    }
    __syncthreads();                                     // s_cs is rewritten by the block's next step
}

// V part: thread tid = (token group tg, KV head h, dim pair d0): 8 tokens x 2 dims, zero padded behind
// the message's last token, written key-transposed ([H_kv][slots/8][D][8]) as two 16-byte stores.
__device__ __forceinline__ void append_bf16_v_thread(
    int64_t tid, const uint16_t *__restrict__ v, int len, int n_kv_heads, int D, int64_t slot_start, int64_t slots,
    uint16_t *__restrict__ v_store)
{
    const int dp = D / 2;
    const int n_groups = (len + PC_VGROUP - 1) / PC_VGROUP;
    if (tid >= (int64_t)n_groups * n_kv_heads * dp) return;
    const int d0 = 2 * (int)(tid % dp);
    const int h = (int)((tid / dp) % n_kv_heads);
    const int tg = (int)(tid / ((int64_t)dp * n_kv_heads));
    uint32_t in[PC_VGROUP];
#pragma unroll
    for (int j = 0; j < PC_VGROUP; ++j) {
        const int t = tg * PC_VGROUP + j;
        in[j] = (t < len) ? *reinterpret_cast<const uint32_t *>(v + ((int64_t)t * n_kv_heads + h) * D + d0) : 0u;
    }
    uint4 ev, od;
    uint32_t *ew = reinterpret_cast<uint32_t *>(&ev), *ow = reinterpret_cast<uint32_t *>(&od);
#pragma unroll
    for (int w = 0; w < 4; ++w) {                        // tokens 2w and 2w + 1 of the group
        ew[w] = (in[2 * w] & 0xFFFFu) | (in[2 * w + 1] << 16);
        ow[w] = (in[2 * w] >> 16) | (in[2 * w + 1] & 0xFFFF0000u);
    }
    uint16_t *dst = v_store + (((int64_t)h * (slots / PC_VGROUP) + slot_start / PC_VGROUP + tg) * D + d0) * PC_VGROUP;
    *reinterpret_cast<uint4 *>(dst) = ev;
    *reinterpret_cast<uint4 *>(dst + PC_VGROUP) = od;
}

__device__ __forceinline__ void append_f32_thread(
    int part, int64_t tid, const float *__restrict__ k, const float *__restrict__ v, int len, int n_kv_heads, int D,
    int64_t slot_start, int64_t slots, const double *__restrict__ inv_freq,
    float *__restrict__ k_store, float *__restrict__ v_store)
{
    const int half = D / 2;
    if (part == 0) {
        if (tid >= (int64_t)len * half) return;
        const int t = (int)(tid / half);
        const int i = (int)(tid % half);
        double s, c;
        sincos((double)t * inv_freq[i], &s, &c);
        const float fc = (float)c, fs = (float)s;
        for (int h = 0; h < n_kv_heads; ++h) {
            const float *src = k + ((int64_t)t * n_kv_heads + h) * D;
            const float a = src[i], b = src[i + half];
            float *dst = k_store + ((int64_t)h * slots + slot_start + t) * D;
            dst[i] = a * fc - b * fs;
            dst[i + half] = a * fs + b * fc;
        }
    } else {
        if (tid >= (int64_t)len * n_kv_heads * D) return;
        const int d = (int)(tid % D);
        const int h = (int)((tid / D) % n_kv_heads);
        const int t = (int)(tid / ((int64_t)D * n_kv_heads));
        v_store[((int64_t)h * slots + slot_start + t) * D + d] = v[tid];
    }
}

__global__ __launch_bounds__(256) void pc_append_bf16_kernel(
    const uint16_t *__restrict__ k, const uint16_t *__restrict__ v, int len, int n_kv_heads, int D,
    int64_t slot_start, int64_t slots, const double *__restrict__ inv_freq,
    uint16_t *__restrict__ k_store, uint16_t *__restrict__ v_store,
    PcMsgEntry *__restrict__ table, int msg_id)
{
    __shared__ float2 s_cs[APP_TB * 64];
    if (blockIdx.y == 0) {
        if (blockIdx.x == 0 && threadIdx.x == 0) { table[msg_id].slot_start = (int32_t)slot_start; table[msg_id].len = len; table[msg_id].base_pos = 0; }
        const int t0 = (int)blockIdx.x * APP_TB;
        if (t0 < len) append_bf16_k_block(k, len, t0, n_kv_heads, D, slot_start, slots, inv_freq, k_store, s_cs);
    } else {
        append_bf16_v_thread((int64_t)blockIdx.x * blockDim.x + threadIdx.x, v, len, n_kv_heads, D, slot_start, slots, v_store);
    }
}

__global__ __launch_bounds__(256) void pc_append_f32_kernel(
    const float *__restrict__ k, const float *__restrict__ v, int len, int n_kv_heads, int D,
    int64_t slot_start, int64_t slots, const double *__restrict__ inv_freq,
    float *__restrict__ k_store, float *__restrict__ v_store,
    PcMsgEntry *__restrict__ table, int msg_id)
{
    const int64_t tid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (blockIdx.y == 0 && tid == 0) { table[msg_id].slot_start = (int32_t)slot_start; table[msg_id].len = len; table[msg_id].base_pos = 0; }
    append_f32_thread((int)blockIdx.y, tid, k, v, len, n_kv_heads, D, slot_start, slots, inv_freq, k_store, v_store);
}

// Several messages in one launch (Sec. 2.4 "Parallel API Calls": the new messages of parallel
// calls arrive together): blockIdx.z names the message, the blocks of a (part, message) walk
// its threads with a grid stride.
template <typename T>
__global__ __launch_bounds__(256) void pc_append_batch_kernel(
    const PcAppendItem *__restrict__ items, int n_kv_heads, int D, int64_t slots,
    const double *__restrict__ inv_freq, T *__restrict__ k_store, T *__restrict__ v_store, PcMsgEntry *__restrict__ table)
{
    const PcAppendItem it = items[blockIdx.z];
    if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0) {
        table[it.msg].slot_start = it.slot_start; table[it.msg].len = it.len; table[it.msg].base_pos = 0;
    }
    if constexpr (sizeof(T) == 2) {
        __shared__ float2 s_cs[APP_TB * 64];
        if (blockIdx.y == 0) {
            for (int t0 = (int)blockIdx.x * APP_TB; t0 < it.len; t0 += (int)gridDim.x * APP_TB)
                append_bf16_k_block((const uint16_t *)it.k, it.len, t0, n_kv_heads, D, it.slot_start, slots, inv_freq, k_store, s_cs);
        } else {
            const int64_t total = (int64_t)((it.len + PC_VGROUP - 1) / PC_VGROUP) * n_kv_heads * (D / 2);
            for (int64_t tid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; tid < total; tid += (int64_t)gridDim.x * blockDim.x)
                append_bf16_v_thread(tid, (const uint16_t *)it.v, it.len, n_kv_heads, D, it.slot_start, slots, v_store);
        }
    } else {
        const int64_t total = blockIdx.y == 0 ? (int64_t)it.len * (D / 2) : (int64_t)it.len * n_kv_heads * D;
        for (int64_t tid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; tid < total; tid += (int64_t)gridDim.x * blockDim.x)
            append_f32_thread((int)blockIdx.y, tid, (const float *)it.k, (const float *)it.v, it.len, n_kv_heads, D,
                              it.slot_start, slots, inv_freq, k_store, v_store);
    }
}

void pc_launch_append_batch(int dtype, const PcAppendItem *items, int n_items, int max_len, int n_kv_heads, int D,
                            int64_t slots, const double *inv_freq, void *k_store, void *v_store, PcMsgEntry *table,
                            hipStream_t st)
{
    // enough blocks per (part, message) for the longest message at one pass, within reason
    // (bf16: the K part takes APP_TB tokens per block step, which is more blocks than the V part needs)
    const int64_t per = dtype == 1 ? ((int64_t)max_len + APP_TB - 1) / APP_TB : ((int64_t)max_len * n_kv_heads * D + 255) / 256;
    const unsigned bx = (unsigned)std::min<int64_t>(std::max<int64_t>(per, 1), 256);
    for (int first = 0; first < n_items; first += 65535) {            // grid.z is limited to 65535
        const int n = n_items - first < 65535 ? n_items - first : 65535;
        dim3 grid(bx, 2, (unsigned)n);
        if (dtype == 1)
            pc_append_batch_kernel<uint16_t><<<grid, 256, 0, st>>>(items + first, n_kv_heads, D, slots, inv_freq,
                                                                   (uint16_t *)k_store, (uint16_t *)v_store, table);
        else
            pc_append_batch_kernel<float><<<grid, 256, 0, st>>>(items + first, n_kv_heads, D, slots, inv_freq,
                                                                (float *)k_store, (float *)v_store, table);
    }
}

void pc_launch_append(int dtype, const void *k, const void *v, int len, int n_kv_heads, int D,
                      int64_t slot_start, int64_t slots, const double *inv_freq, void *k_store,
                      void *v_store, PcMsgEntry *table, int msg_id, hipStream_t st)
{
    if (dtype == 1) {
        const int64_t bk = ((int64_t)len + APP_TB - 1) / APP_TB;
        const int64_t bv = ((int64_t)((len + PC_VGROUP - 1) / PC_VGROUP) * n_kv_heads * (D / 2) + 255) / 256;
        dim3 grid((unsigned)(bk > bv ? bk : bv), 2);
        pc_append_bf16_kernel<<<grid, 256, 0, st>>>((const uint16_t *)k, (const uint16_t *)v, len, n_kv_heads, D,
                                                    slot_start, slots, inv_freq, (uint16_t *)k_store,
                                                    (uint16_t *)v_store, table, msg_id);
    } else {
        const int64_t nk = (int64_t)len * (D / 2);
        const int64_t nv = (int64_t)len * n_kv_heads * D;
        const int64_t n = nk > nv ? nk : nv;
        dim3 grid((unsigned)((n + 255) / 256), 2);
        pc_append_f32_kernel<<<grid, 256, 0, st>>>((const float *)k, (const float *)v, len, n_kv_heads, D,
                                                   slot_start, slots, inv_freq, (float *)k_store,
                                                   (float *)v_store, table, msg_id);
    }
}

// ----------------------------------------------------------------------------------
// Tokens appended to existing messages (Sec. 2.4: the tails of parallel decode calls
// grow one token per step, interleaved).  thread = (token j, KV head h, frequency pair
// i0 = 2*m): key turned to the item's position, value written into its 8-slot group.
// ----------------------------------------------------------------------------------
template <typename T>
__device__ __forceinline__ void append_token_thread(const PcTokenItem it, int j, int h, int i0, const T *__restrict__ k,
                                                    const T *__restrict__ v, int n_kv_heads, int D, int64_t slots,
                                                    const double *__restrict__ inv_freq, T *__restrict__ k_store,
                                                    T *__restrict__ v_store, PcMsgEntry *__restrict__ table)
{
    const int half = D / 2;
    if (h == 0 && i0 == 0) table[it.msg].len = it.new_len;      // every item of a message carries its final length
    double s0, c0, s1, c1;
    sincos((double)it.pos * inv_freq[i0], &s0, &c0);
    sincos((double)it.pos * inv_freq[i0 + 1], &s1, &c1);
    const float fc0 = (float)c0, fs0 = (float)s0, fc1 = (float)c1, fs1 = (float)s1;
    const T *ksrc = k + ((int64_t)j * n_kv_heads + h) * D;
    const T *vsrc = v + ((int64_t)j * n_kv_heads + h) * D;
    T *kdst = k_store + ((int64_t)h * slots + it.slot) * D;
    if constexpr (sizeof(T) == 2) {
        using P = Pair2<__hip_bfloat16>;
        const uint32_t lo = *reinterpret_cast<const uint32_t *>(ksrc + i0);
        const uint32_t hi = *reinterpret_cast<const uint32_t *>(ksrc + half + i0);
        const float a0 = P::lo(lo), a1 = P::hi(lo), b0 = P::lo(hi), b1 = P::hi(hi);
        *reinterpret_cast<uint32_t *>(kdst + i0) = P::pack(a0 * fc0 - b0 * fs0, a1 * fc1 - b1 * fs1);
        *reinterpret_cast<uint32_t *>(kdst + half + i0) = P::pack(a0 * fs0 + b0 * fc0, a1 * fs1 + b1 * fc1);
        // V: [H_kv][slots/8][D][8]; this thread moves dims i0, i0+1 and half+i0, half+i0+1
        T *vg = v_store + ((int64_t)h * (slots / PC_VGROUP) + it.slot / PC_VGROUP) * D * PC_VGROUP + (it.slot % PC_VGROUP);
        vg[(int64_t)i0 * PC_VGROUP] = vsrc[i0];
        vg[(int64_t)(i0 + 1) * PC_VGROUP] = vsrc[i0 + 1];
        vg[(int64_t)(half + i0) * PC_VGROUP] = vsrc[half + i0];
        vg[(int64_t)(half + i0 + 1) * PC_VGROUP] = vsrc[half + i0 + 1];
    } else {
        const float a0 = ksrc[i0], a1 = ksrc[i0 + 1], b0 = ksrc[half + i0], b1 = ksrc[half + i0 + 1];
        kdst[i0] = a0 * fc0 - b0 * fs0; kdst[i0 + 1] = a1 * fc1 - b1 * fs1;
        kdst[half + i0] = a0 * fs0 + b0 * fc0; kdst[half + i0 + 1] = a1 * fs1 + b1 * fc1;
        T *vdst = v_store + ((int64_t)h * slots + it.slot) * D;
        vdst[i0] = vsrc[i0]; vdst[i0 + 1] = vsrc[i0 + 1];
        vdst[half + i0] = vsrc[half + i0]; vdst[half + i0 + 1] = vsrc[half + i0 + 1];
    }
}

template <typename T>
__global__ __launch_bounds__(256) void pc_append_tokens_kernel(
    const PcTokenItem *__restrict__ items, int n, const T *__restrict__ k, const T *__restrict__ v,
    int n_kv_heads, int D, int64_t slots, const double *__restrict__ inv_freq,
    T *__restrict__ k_store, T *__restrict__ v_store, PcMsgEntry *__restrict__ table)
{
    const int per_row = D / 4;
    const int64_t tid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (tid >= (int64_t)n * n_kv_heads * per_row) return;
    const int j = (int)(tid / ((int64_t)per_row * n_kv_heads));
    append_token_thread<T>(items[j], j, (int)((tid / per_row) % n_kv_heads), 2 * (int)(tid % per_row), k, v, n_kv_heads, D, slots,
                           inv_freq, k_store, v_store, table);
}

// The same with the items passed by value (a decode step's one token per call: up to PC_TOKEN_PACK items fit the
// kernel's arguments, which saves staging them through pinned memory and a copy).
template <typename T>
__global__ __launch_bounds__(256) void pc_append_tokens_packed_kernel(
    const PcTokenPack pack, int n, const T *__restrict__ k, const T *__restrict__ v,
    int n_kv_heads, int D, int64_t slots, const double *__restrict__ inv_freq,
    T *__restrict__ k_store, T *__restrict__ v_store, PcMsgEntry *__restrict__ table)
{
    const int per_row = D / 4;
    const int64_t tid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (tid >= (int64_t)n * n_kv_heads * per_row) return;
    const int j = (int)(tid / ((int64_t)per_row * n_kv_heads));
    append_token_thread<T>(pack.it[j], j, (int)((tid / per_row) % n_kv_heads), 2 * (int)(tid % per_row), k, v, n_kv_heads, D, slots,
                           inv_freq, k_store, v_store, table);
}

void pc_launch_append_tokens_packed(int dtype, const PcTokenPack &pack, int n, const void *k, const void *v, int n_kv_heads,
                                    int D, int64_t slots, const double *inv_freq, void *k_store, void *v_store,
                                    PcMsgEntry *table, hipStream_t st)
{
    const int64_t total = (int64_t)n * n_kv_heads * (D / 4);
    const unsigned grid = (unsigned)((total + 255) / 256);
    if (grid == 0) return;
    if (dtype == 1)
        pc_append_tokens_packed_kernel<uint16_t><<<grid, 256, 0, st>>>(pack, n, (const uint16_t *)k, (const uint16_t *)v, n_kv_heads,
                                                                       D, slots, inv_freq, (uint16_t *)k_store,
                                                                       (uint16_t *)v_store, table);
    else
        pc_append_tokens_packed_kernel<float><<<grid, 256, 0, st>>>(pack, n, (const float *)k, (const float *)v, n_kv_heads, D,
                                                                    slots, inv_freq, (float *)k_store, (float *)v_store, table);
}

void pc_launch_append_tokens(int dtype, const PcTokenItem *items, int n, const void *k, const void *v, int n_kv_heads,
                             int D, int64_t slots, const double *inv_freq, void *k_store, void *v_store,
                             PcMsgEntry *table, hipStream_t st)
{
    const int64_t total = (int64_t)n * n_kv_heads * (D / 4);
    const unsigned grid = (unsigned)((total + 255) / 256);
    if (grid == 0) return;
    if (dtype == 1)
        pc_append_tokens_kernel<uint16_t><<<grid, 256, 0, st>>>(items, n, (const uint16_t *)k, (const uint16_t *)v, n_kv_heads,
                                                                D, slots, inv_freq, (uint16_t *)k_store,
                                                                (uint16_t *)v_store, table);
    else
        pc_append_tokens_kernel<float><<<grid, 256, 0, st>>>(items, n, (const float *)k, (const float *)v, n_kv_heads, D,
                                                             slots, inv_freq, (float *)k_store, (float *)v_store, table);
}

// ----------------------------------------------------------------------------------
// In-place position update of one cached message (Sec. 2.4 "Position Updates"): every
// stored key is turned by `delta` more positions, with a table of the D/2 rotations
// (cos, sin)(delta * theta_i) built once per block in fp64.  V is not touched.
// thread = (token t, KV head h, frequency pair i0 = 2*j): handles pairs i0 and i0+1.
// ----------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void pc_reposition_kernel(
    int len, int n_kv_heads, int D, int64_t slot_start, int64_t slots, int delta, int new_base,
    const double *__restrict__ inv_freq, T *__restrict__ k_store, PcMsgEntry *__restrict__ table, int msg_id)
{
    __shared__ float2 s_lut[64];
    const int half = D / 2;
    if ((int)threadIdx.x < half) {
        double s, c;
        sincos((double)delta * inv_freq[threadIdx.x], &s, &c);
        s_lut[threadIdx.x] = make_float2((float)c, (float)s);
    }
    __syncthreads();
    const int64_t tid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (tid == 0) table[msg_id].base_pos = new_base;
    const int per_row = half / 2;
    if (tid >= (int64_t)len * n_kv_heads * per_row) return;
    const int i0 = 2 * (int)(tid % per_row);
    const int h = (int)((tid / per_row) % n_kv_heads);
    const int t = (int)(tid / ((int64_t)per_row * n_kv_heads));
    const float2 r0 = s_lut[i0], r1 = s_lut[i0 + 1];
    T *row = k_store + ((int64_t)h * slots + slot_start + t) * D;
    if constexpr (sizeof(T) == 2) {
        using P = Pair2<__hip_bfloat16>;
        const uint32_t lo = *reinterpret_cast<const uint32_t *>(row + i0);
        const uint32_t hi = *reinterpret_cast<const uint32_t *>(row + half + i0);
        const float a0 = P::lo(lo), a1 = P::hi(lo), b0 = P::lo(hi), b1 = P::hi(hi);
        *reinterpret_cast<uint32_t *>(row + i0) = P::pack(a0 * r0.x - b0 * r0.y, a1 * r1.x - b1 * r1.y);
        *reinterpret_cast<uint32_t *>(row + half + i0) = P::pack(a0 * r0.y + b0 * r0.x, a1 * r1.y + b1 * r1.x);
    } else {
        const float a0 = row[i0], a1 = row[i0 + 1], b0 = row[half + i0], b1 = row[half + i0 + 1];
        row[i0] = a0 * r0.x - b0 * r0.y; row[i0 + 1] = a1 * r1.x - b1 * r1.y;
        row[half + i0] = a0 * r0.y + b0 * r0.x; row[half + i0 + 1] = a1 * r1.y + b1 * r1.x;
    }
}

void pc_launch_reposition(int dtype, int len, int n_kv_heads, int D, int64_t slot_start, int64_t slots, int delta,
                          int new_base, const double *inv_freq, void *k_store, PcMsgEntry *table, int msg_id,
                          hipStream_t st)
{
    const int64_t n = (int64_t)len * n_kv_heads * (D / 4);
    const unsigned grid = (unsigned)((n + 255) / 256);
    if (grid == 0) return;
    if (dtype == 1)
        pc_reposition_kernel<uint16_t><<<grid, 256, 0, st>>>(len, n_kv_heads, D, slot_start, slots, delta, new_base, inv_freq,
                                                             (uint16_t *)k_store, table, msg_id);
    else
        pc_reposition_kernel<float><<<grid, 256, 0, st>>>(len, n_kv_heads, D, slot_start, slots, delta, new_base, inv_freq,
                                                          (float *)k_store, table, msg_id);
}

// Batched form: blockIdx.y names the message, the blocks of a row of the grid walk its key rows
// with a grid stride.  A thread takes 16 bytes from each half of a key row per step (8 frequency
// pairs in bf16, 4 in fp32): the kernel is one read and one write of K and lives on wide accesses.
template <typename T>
__global__ __launch_bounds__(256) void pc_reposition_batch_kernel(
    const PcMoveItem *__restrict__ items, int n_kv_heads, int D, int64_t slots,
    const double *__restrict__ inv_freq, T *__restrict__ k_store, PcMsgEntry *__restrict__ table)
{
    __shared__ float2 s_lut[64];
    const PcMoveItem it = items[blockIdx.y];
    const int half = D / 2;
    constexpr int PER = 16 / (int)sizeof(T);             // frequency pairs per thread and step
    const int per_row = half / PER;
    const int64_t total = (int64_t)it.len * n_kv_heads * per_row;
    if ((int64_t)blockIdx.x * blockDim.x >= total) return;            // a short message needs fewer blocks than the grid has
    if ((int)threadIdx.x < half) {
        double s, c;
        sincos((double)it.delta * inv_freq[threadIdx.x], &s, &c);
        s_lut[threadIdx.x] = make_float2((float)c, (float)s);
    }
    __syncthreads();
    if (blockIdx.x == 0 && threadIdx.x == 0) table[it.msg].base_pos = it.new_base;
    for (int64_t tid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; tid < total; tid += (int64_t)gridDim.x * blockDim.x) {
        const int i0 = PER * (int)(tid % per_row);
        const int h = (int)((tid / per_row) % n_kv_heads);
        const int t = (int)(tid / ((int64_t)per_row * n_kv_heads));
        T *row = k_store + ((int64_t)h * slots + it.slot_start + t) * D;
        uint4 lo = *reinterpret_cast<const uint4 *>(row + i0);
        uint4 hi = *reinterpret_cast<const uint4 *>(row + half + i0);
        uint32_t *lw = reinterpret_cast<uint32_t *>(&lo), *hw = reinterpret_cast<uint32_t *>(&hi);
        if constexpr (sizeof(T) == 2) {
            using P = Pair2<__hip_bfloat16>;
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const float2 r0 = s_lut[i0 + 2 * u], r1 = s_lut[i0 + 2 * u + 1];
                const float a0 = P::lo(lw[u]), a1 = P::hi(lw[u]), b0 = P::lo(hw[u]), b1 = P::hi(hw[u]);
                lw[u] = P::pack(a0 * r0.x - b0 * r0.y, a1 * r1.x - b1 * r1.y);
                hw[u] = P::pack(a0 * r0.y + b0 * r0.x, a1 * r1.y + b1 * r1.x);
            }
        } else {
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const float2 r = s_lut[i0 + u];
                const float a = __uint_as_float(lw[u]), b_ = __uint_as_float(hw[u]);
                lw[u] = __float_as_uint(a * r.x - b_ * r.y);
                hw[u] = __float_as_uint(a * r.y + b_ * r.x);
            }
        }
        *reinterpret_cast<uint4 *>(row + i0) = lo;
        *reinterpret_cast<uint4 *>(row + half + i0) = hi;
    }
}

void pc_launch_reposition_batch(int dtype, const PcMoveItem *items, int n_items, int n_kv_heads, int D, int64_t slots,
                                const double *inv_freq, void *k_store, PcMsgEntry *table, hipStream_t st)
{
    for (int first = 0; first < n_items; first += 65535) {            // grid.y is limited to 65535
        const int n = n_items - first < 65535 ? n_items - first : 65535;
        dim3 grid(64, (unsigned)n);                      // up to 64 blocks of 256 threads per message
        if (dtype == 1)
            pc_reposition_batch_kernel<uint16_t><<<grid, 256, 0, st>>>(items + first, n_kv_heads, D, slots, inv_freq,
                                                                       (uint16_t *)k_store, table);
        else
            pc_reposition_batch_kernel<float><<<grid, 256, 0, st>>>(items + first, n_kv_heads, D, slots, inv_freq,
                                                                    (float *)k_store, table);
    }
}

// ----------------------------------------------------------------------------------
// K2: plan builder.  Blocks [0, n_calls): per call, look each listed message up in the
// device message table and scan lengths into the segment list (Sec. 2.4 "Dynamic
// Masking": what a call sees is computed on the fly from message membership; here in
// gather form).  Blocks [n_calls, ...): rotation tables (cos, sin)(p * theta_i) for
// every segment start and every query row, in fp64 rounded to fp32 (Sec. 2.4
// "Position Updates": a lookup table of rotations).
// ----------------------------------------------------------------------------------
// Blocks [tok_block0, ...) (a decode step only): the step's new tokens go into the cache in the same launch; the plan
// blocks never read what they write (the grown messages' new lengths travel with the calls from the host).
__global__ __launch_bounds__(256) void pc_build_plan_kernel(
    const PcCallDesc *__restrict__ calls, int n_calls, const int2 *__restrict__ sel,
    const int32_t *__restrict__ q_pos, PcMsgEntry *__restrict__ table,
    const double *__restrict__ inv_freq, int half, int total_seg, int total_q,
    PcSegment *__restrict__ segs, int32_t *__restrict__ seg_kvoff,
    float2 *__restrict__ rot_seg, float2 *__restrict__ rot_q, float2 *__restrict__ rot_qw, PcTile *__restrict__ tiles, PcTokenWork tok, int tok_block0)
{
    if ((int)blockIdx.x >= tok_block0) {
        const int per_row = tok.D / 4;
        const int64_t tid = (int64_t)((int)blockIdx.x - tok_block0) * 256 + threadIdx.x;
        if (tid >= (int64_t)tok.n * tok.n_kv_heads * per_row) return;
        const int j = (int)(tid / ((int64_t)per_row * tok.n_kv_heads));
        const int hh = (int)((tid / per_row) % tok.n_kv_heads), i0 = 2 * (int)(tid % per_row);
        if (tok.dtype == 1)
            append_token_thread<uint16_t>(tok.items[j], j, hh, i0, (const uint16_t *)tok.k, (const uint16_t *)tok.v, tok.n_kv_heads, tok.D,
                                          tok.slots, inv_freq, (uint16_t *)tok.k_store, (uint16_t *)tok.v_store, table);
        else
            append_token_thread<float>(tok.items[j], j, hh, i0, (const float *)tok.k, (const float *)tok.v, tok.n_kv_heads, tok.D,
                                       tok.slots, inv_freq, (float *)tok.k_store, (float *)tok.v_store, table);
        return;
    }
    __shared__ int s_len[256];
    __shared__ int s_tiles[256];
    __shared__ int s_carry[2];
    __shared__ int s_rot[257];                           // query rotation (position - stored base) of the chunk's segments
    // the call's segment list as the tile loop needs it, kept in LDS when it fits (it nearly always
    // does): the per-tile binary search then costs LDS latencies, not a chain of global loads
    constexpr int SEG_LDS = 1024;
    __shared__ int s_seg_tile[SEG_LDS], s_seg_slot[SEG_LDS], s_seg_len[SEG_LDS];
    __shared__ unsigned char s_seg_same[SEG_LDS];
    if ((int)blockIdx.x < n_calls) {
        const PcCallDesc cd = calls[blockIdx.x];
        if (threadIdx.x == 0) { s_carry[0] = 0; s_carry[1] = 0; s_rot[0] = 0; }
        __syncthreads();
        for (int base = 0; base < cd.n_seg; base += 256) {
            const int e = base + threadIdx.x;
            int len = 0, slot = 0, pos = 0, rot = 0;
            if (e < cd.n_seg) {
                int m, p;
                if (e < cd.n_sel) { const int2 s = sel[cd.sel_off + e]; m = s.x; p = s.y; }
                else { m = cd.self_msg; p = cd.self_start; }
                const PcMsgEntry me = table[m];
                // (the new message's length comes from the host: a decode step appends its token beside this kernel)
                len = e < cd.n_sel ? me.len : cd.self_len; slot = me.slot_start; pos = p; rot = p - me.base_pos;
            }
            s_rot[threadIdx.x + 1] = rot;                // s_rot[0]: last segment of the chunk before
            const int tiles = (len + PC_TILE - 1) / PC_TILE;
            s_len[threadIdx.x] = len;
            s_tiles[threadIdx.x] = tiles;
            __syncthreads();
            // Hillis-Steele inclusive scan over the 256 entries of this chunk
            for (int off = 1; off < 256; off <<= 1) {
                int a = 0, b = 0;
                if ((int)threadIdx.x >= off) { a = s_len[threadIdx.x - off]; b = s_tiles[threadIdx.x - off]; }
                __syncthreads();
                s_len[threadIdx.x] += a;
                s_tiles[threadIdx.x] += b;
                __syncthreads();
            }
            const int c_len = s_carry[0], c_tiles = s_carry[1];
            if (e < cd.n_seg) {
                PcSegment sg;
                sg.slot_start = slot; sg.len = len; sg.pos_start = pos;
                sg.tile_off = c_tiles + s_tiles[threadIdx.x] - tiles;
                sg.rot_pos = rot;
                sg.same_rot = (e > 0 && s_rot[threadIdx.x] == rot) ? 1 : 0;
                sg.pad[0] = sg.pad[1] = 0;
                segs[cd.seg_off + e] = sg;
                seg_kvoff[cd.seg_off + e] = c_len + s_len[threadIdx.x] - len;
                if (e < SEG_LDS) { s_seg_tile[e] = sg.tile_off; s_seg_slot[e] = slot; s_seg_len[e] = len; s_seg_same[e] = (unsigned char)sg.same_rot; }
            }
            __syncthreads();
            if (threadIdx.x == 255) { s_carry[0] = c_len + s_len[255]; s_carry[1] = c_tiles + s_tiles[255]; s_rot[0] = rot; }
            __syncthreads();
        }
        // tile table of this call: one entry per 32-key tile, in gathered order (the segment
        // entries written above by this block are visible after the barrier)
        const int n_tiles = s_carry[1];
        const PcSegment *sg = segs + cd.seg_off;
        const bool in_lds = cd.n_seg <= SEG_LDS;
        for (int t = threadIdx.x; t < n_tiles; t += 256) {
            int lo = 0, hi = cd.n_seg - 1;
            int g_tile, g_slot, g_len, g_same;
            if (in_lds) {
                while (lo < hi) {
                    const int mid = (lo + hi + 1) >> 1;
                    if (s_seg_tile[mid] <= t) lo = mid; else hi = mid - 1;
                }
                g_tile = s_seg_tile[lo]; g_slot = s_seg_slot[lo]; g_len = s_seg_len[lo]; g_same = s_seg_same[lo];
            } else {
                while (lo < hi) {
                    const int mid = (lo + hi + 1) >> 1;
                    if (sg[mid].tile_off <= t) lo = mid; else hi = mid - 1;
                }
                const PcSegment g = sg[lo];
                g_tile = g.tile_off; g_slot = g.slot_start; g_len = g.len; g_same = g.same_rot;
            }
            PcTile tl;
            tl.key0 = (t - g_tile) * PC_TILE;
            tl.slot0 = g_slot + tl.key0;
            tl.seg = lo;
            const int valid = g_len - tl.key0 < PC_TILE ? g_len - tl.key0 : PC_TILE;
            tl.valid_flags = valid | ((t == g_tile && !g_same) ? PC_TILE_FRESH : 0) |
                             ((cd.self_msg >= 0 && lo == cd.n_seg - 1) ? PC_TILE_SELF : 0);
            tiles[cd.tile_off + t] = tl;
        }
        return;
    }
    // rotation tables: entity = segment (position from the staged lists) or query row
    const int64_t tid = (int64_t)(blockIdx.x - n_calls) * 256 + threadIdx.x;
    const int64_t n_ent = (int64_t)total_seg + total_q;
    if (tid >= n_ent * half) return;
    const int ent = (int)(tid / half);
    const int i = (int)(tid % half);
    int pos;
    if (ent < total_seg) {
        // find the call that owns this segment (calls are few; segments are laid out call by call)
        int lo = 0, hi = n_calls - 1;
        while (lo < hi) {
            const int mid = (lo + hi + 1) >> 1;
            if (calls[mid].seg_off <= ent) lo = mid; else hi = mid - 1;
        }
        const PcCallDesc cd = calls[lo];
        const int e = ent - cd.seg_off;
        int m;
        if (e < cd.n_sel) { const int2 s = sel[cd.sel_off + e]; m = s.x; pos = s.y; }
        else { m = cd.self_msg; pos = cd.self_start; }
        pos -= table[m].base_pos;                        // the stored key of token t already sits at base_pos + t
    } else {
        pos = q_pos[ent - total_seg];
    }
    double s, c;
    sincos((double)pos * inv_freq[i], &s, &c);
    const float2 r = make_float2((float)c, (float)s);
    if (ent < total_seg) rot_seg[(int64_t)ent * half + i] = r;
    else {
        const int R = ent - total_seg;
        rot_q[(int64_t)R * half + i] = r;
        // the copy the bf16 prefill kernel reads: 16 bytes per lane, the lanes of consecutive rows side by side
        if (rot_qw) rot_qw[((int64_t)(R >> 5) * 1024 + (i >> 4) * 256 + ((i >> 1) & 3) * 64 + ((i >> 3) & 1) * 32 + (R & 31)) * 2 + (i & 1)] = r;
    }
}

void pc_launch_build_plan(const PcCallDesc *calls, int n_calls, const int2 *sel, const int32_t *q_pos,
                          PcMsgEntry *table, const double *inv_freq, int half, int total_seg,
                          int total_q, PcSegment *segs, int32_t *seg_kvoff, float2 *rot_seg,
                          float2 *rot_q, float2 *rot_qw, PcTile *tiles, const PcTokenWork &tok, hipStream_t st)
{
    const int64_t n_rot = ((int64_t)total_seg + total_q) * half;
    const unsigned plan_blocks = (unsigned)(n_calls + (n_rot + 255) / 256);
    const int64_t tok_threads = (int64_t)tok.n * tok.n_kv_heads * (tok.D / 4);
    const unsigned grid = plan_blocks + (unsigned)((tok_threads + 255) / 256);
    pc_build_plan_kernel<<<grid, 256, 0, st>>>(calls, n_calls, sel, q_pos, table, inv_freq, half, total_seg,
                                               total_q, segs, seg_kvoff, rot_seg, rot_q, rot_qw, tiles, tok, (int)plan_blocks);
}

// ----------------------------------------------------------------------------------
// Expanded gather table / position map of one call (the (m, j) metadata of Sec. 2.4 in
// gathered form): token i of the gathered sequence -> physical slot and logical position.
// ----------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void pc_expand_tables_kernel(
    const PcSegment *__restrict__ segs, const int32_t *__restrict__ seg_kvoff, int n_seg, int64_t n_kv,
    int32_t *__restrict__ kv_slot, int32_t *__restrict__ kv_pos)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n_kv) return;
    int lo = 0, hi = n_seg - 1;
    while (lo < hi) {                      // last segment whose first token is <= i and non-empty
        const int mid = (lo + hi + 1) >> 1;
        if (seg_kvoff[mid] <= i) lo = mid; else hi = mid - 1;
    }
    const PcSegment sg = segs[lo];
    const int t = (int)(i - seg_kvoff[lo]);
    kv_slot[i] = sg.slot_start + t;
    kv_pos[i] = sg.pos_start + t;
}

void pc_launch_expand_tables(const PcSegment *segs, const int32_t *seg_kvoff, int n_seg, int64_t n_kv,
                             int32_t *kv_slot, int32_t *kv_pos, hipStream_t st)
{
    if (n_kv <= 0) return;
    pc_expand_tables_kernel<<<(unsigned)((n_kv + 255) / 256), 256, 0, st>>>(segs, seg_kvoff, n_seg, n_kv,
                                                                           kv_slot, kv_pos);
}

// ----------------------------------------------------------------------------------
// K5: merge of KV splits.  Each split s of a row holds its own normalised output O_s
// (fp16), a running maximum m_s (scaled log2 domain) and a sum l_s; the result is
//   m = max m_s,  w_s = l_s 2^(m_s - m),  l = sum w_s,  O = sum w_s O_s / l
// in a fixed order (deterministic; no atomics).
// SL * 16 threads per (row, head): a thread = (one of SL equal parts of the splits, eight of the 128
// dimensions).  It folds its part in split order, four splits per round of loads (one 16-byte load
// per split); for SL = 4 (rows with many splits, a wave per (row, head)) the four parts are then
// combined pairwise across lanes.  The kernel is bound by the latency of its dependent loads, so
// there are few levels of them: the row's descriptor, then the sums and outputs of up to four
// splits together.
// ----------------------------------------------------------------------------------
template <int SL>
__global__ __launch_bounds__(256) void pc_merge_kernel(
    const PcMergeRow *__restrict__ merge_rows, const uint16_t *__restrict__ part_o,
    const float *__restrict__ part_ml, uint16_t *__restrict__ out, float *__restrict__ lse, int n_q_heads,
    int n_pairs)
{
    constexpr int D = 128;
    constexpr int TPP = 16 * SL;                         // threads per (row, head)
    const int pair = blockIdx.x * (256 / TPP) + (int)threadIdx.x / TPP;
    if (pair >= n_pairs) return;                         // (SL = 4: whole waves)
    const int sub = threadIdx.x & 15, sg = ((int)threadIdx.x % TPP) >> 4;
    const int h = pair % n_q_heads;
    const PcMergeRow mr = merge_rows[pair / n_q_heads];
    const int part = (mr.n_splits + SL - 1) / SL;
    const int s_begin = sg * part, s_end = min(s_begin + part, mr.n_splits);
    float m = -INFINITY, l = 0.f, o[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) o[j] = 0.f;
    for (int s0 = s_begin; s0 < s_end; s0 += 4) {
        float2 ml[4];
        uint4 v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            ml[u] = make_float2(-INFINITY, 0.f);
            v[u] = make_uint4(0, 0, 0, 0);
            if (s0 + u < s_end) {
                const int64_t pr = (int64_t)mr.part_row0 + (int64_t)(s0 + u) * mr.n_q;
                ml[u] = *reinterpret_cast<const float2 *>(part_ml + (pr * n_q_heads + h) * 2);
                v[u] = *reinterpret_cast<const uint4 *>(part_o + (pr * n_q_heads + h) * D + 8 * sub);
            }
        }
        float m_new = m;
#pragma unroll
        for (int u = 0; u < 4; ++u) m_new = fmaxf(m_new, ml[u].x);
        if (m_new == -INFINITY) continue;
        const float keep = (m > -INFINITY) ? exp2f(m - m_new) : 0.f;
        l *= keep;
#pragma unroll
        for (int j = 0; j < 8; ++j) o[j] *= keep;
        m = m_new;
#pragma unroll
        for (int u = 0; u < 4; ++u) {                    // in split order
            const float w = (ml[u].x > -INFINITY) ? ml[u].y * exp2f(ml[u].x - m) : 0.f;
            l += w;
            const uint32_t d[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                o[2 * j] += (float)__builtin_bit_cast(_Float16, (uint16_t)(d[j] & 0xFFFF)) * w;
                o[2 * j + 1] += (float)__builtin_bit_cast(_Float16, (uint16_t)(d[j] >> 16)) * w;
            }
        }
    }
    // parts 0+1 and 2+3, then the two halves; only the lanes of part 0 keep the result
#pragma unroll
    for (int mask = 16; mask < TPP; mask <<= 1) {
        const float m_o = __shfl_xor(m, mask), l_o = __shfl_xor(l, mask);
        const float m_c = fmaxf(m, m_o);
        const float w_own = (m > -INFINITY) ? exp2f(m - m_c) : 0.f;
        const float w_oth = (m_o > -INFINITY) ? exp2f(m_o - m_c) : 0.f;
        l = l * w_own + l_o * w_oth;
#pragma unroll
        for (int j = 0; j < 8; ++j) o[j] = o[j] * w_own + __shfl_xor(o[j], mask) * w_oth;
        m = m_c;
    }
    if (sg != 0) return;
    const float inv = (l > 0.f) ? 1.f / l : 0.f;
    uint32_t packed[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        __hip_bfloat16 b0 = __float2bfloat16(o[2 * j] * inv), b1 = __float2bfloat16(o[2 * j + 1] * inv);
        packed[j] = (uint32_t)*reinterpret_cast<uint16_t *>(&b0) | ((uint32_t)*reinterpret_cast<uint16_t *>(&b1) << 16);
    }
    *reinterpret_cast<uint4 *>(out + ((int64_t)mr.row * n_q_heads + h) * D + 8 * sub) = make_uint4(packed[0], packed[1], packed[2], packed[3]);
    if (lse && sub == 0)
        lse[(int64_t)mr.row * n_q_heads + h] = (l > 0.f) ? (m + log2f(l)) * 0.6931471805599453f : -INFINITY;
}

// only bf16 caches with D = 128 split their work (the fp32 kernel never does)
void pc_launch_merge(int dtype, const PcMergeRow *merge_rows, int n_merge_rows, int split_lanes, const uint16_t *part_o,
                     const float *part_ml, void *out, float *lse, int n_q_heads, int D, hipStream_t st)
{
    if (n_merge_rows <= 0 || dtype != 1 || D != 128) return;
    const int n_pairs = n_merge_rows * n_q_heads;
    if (split_lanes == 4)
        pc_merge_kernel<4><<<(n_pairs + 3) / 4, 256, 0, st>>>(merge_rows, part_o, part_ml, (uint16_t *)out, lse, n_q_heads, n_pairs);
    else
        pc_merge_kernel<1><<<(n_pairs + 15) / 16, 256, 0, st>>>(merge_rows, part_o, part_ml, (uint16_t *)out, lse, n_q_heads, n_pairs);
}

// ----------------------------------------------------------------------------------
// K6: fp32 attention, one wave per (query row, query head).  Plain vector arithmetic,
// meant for fp32 caches (small reference-precision configurations).
// For each segment the query is turned by (q_pos - segment start) and dotted with the
// stored keys; online softmax per lane over the keys that lane visits; lanes are
// combined at the end.
// ----------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(64) void pc_attend_f32_kernel(PcLaunch L, const int32_t *__restrict__ row_call)
{
    constexpr int HALF = D / 2;
    __shared__ float s_qhat[D];
    __shared__ float s_qe[D];
    __shared__ float s_red[64 * (D + 1)];
    const int R = blockIdx.x, h = blockIdx.y, lane = threadIdx.x;
    const PcCallDesc cd = L.calls[row_call[R]];
    const int r = R - cd.q_off;
    const int g = L.n_q_heads / L.n_kv_heads;
    const int kh = h / g;
    const float *q = (const float *)L.q + ((int64_t)R * L.n_q_heads + h) * D;
    for (int i = lane; i < HALF; i += 64) {
        const float2 cs = L.rot_q[(int64_t)R * HALF + i];
        const float a = q[i], b = q[i + HALF];
        s_qhat[i] = a * cs.x - b * cs.y;
        s_qhat[i + HALF] = a * cs.y + b * cs.x;
    }
    __syncthreads();
    const float *kbase = (const float *)L.k_store + (int64_t)kh * L.slots * D;
    const float *vbase = (const float *)L.v_store + (int64_t)kh * L.slots * D;
    float m = -INFINITY, l = 0.f;
    float acc[D];
#pragma unroll
    for (int d = 0; d < D; ++d) acc[d] = 0.f;
    for (int e = 0; e < cd.n_seg; ++e) {
        const PcSegment sg = L.segs[cd.seg_off + e];
        int n_vis = sg.len;
        if (cd.self_msg >= 0 && e == cd.n_seg - 1) {
            const int lim = cd.self_len - cd.n_q + r + 1;
            n_vis = lim < n_vis ? lim : n_vis;
        }
        if (n_vis <= 0) continue;
        __syncthreads();
        for (int i = lane; i < HALF; i += 64) {
            const float2 cs = L.rot_seg[(int64_t)(cd.seg_off + e) * HALF + i];
            const float a = s_qhat[i], b = s_qhat[i + HALF];
            s_qe[i] = a * cs.x + b * cs.y;              // turn by -pos_start
            s_qe[i + HALF] = -a * cs.y + b * cs.x;
        }
        __syncthreads();
        for (int t = lane; t < n_vis; t += 64) {
            const float *kr = kbase + (int64_t)(sg.slot_start + t) * D;
            float s = 0.f;
#pragma unroll 8
            for (int d = 0; d < D; ++d) s = fmaf(s_qe[d], kr[d], s);
            s *= L.scale_log2;
            const float mn = fmaxf(m, s);
            const float alpha = exp2f(m - mn);          // m = -inf -> 0
            const float p = exp2f(s - mn);
            l = l * alpha + p;
            const float *vr = vbase + (int64_t)(sg.slot_start + t) * D;
#pragma unroll
            for (int d = 0; d < D; ++d) acc[d] = fmaf(acc[d], alpha, p * vr[d]);
            m = mn;
        }
    }
    // combine the 64 lanes
    float mw = m;
    for (int off = 32; off > 0; off >>= 1) mw = fmaxf(mw, __shfl_xor(mw, off));
    const float w = (m > -INFINITY) ? exp2f(m - mw) : 0.f;
    float lw = l * w;
    for (int off = 32; off > 0; off >>= 1) lw += __shfl_xor(lw, off);
    __syncthreads();
#pragma unroll
    for (int d = 0; d < D; ++d) s_red[lane * (D + 1) + d] = acc[d] * w;
    __syncthreads();
    float *out = (float *)L.out + ((int64_t)R * L.n_q_heads + h) * D;
    for (int d = lane; d < D; d += 64) {
        float o = 0.f;
        for (int j = 0; j < 64; ++j) o += s_red[j * (D + 1) + d];
        out[d] = (lw > 0.f) ? o / lw : 0.f;
    }
    if (L.lse && lane == 0)
        L.lse[(int64_t)R * L.n_q_heads + h] = (lw > 0.f) ? (mw + log2f(lw)) * 0.6931471805599453f : -INFINITY;
}

void pc_launch_attend_f32(const PcLaunch &L, const int32_t *row_call, int total_q, int D, hipStream_t st)
{
    if (total_q <= 0) return;
    dim3 grid(total_q, L.n_q_heads);
    if (D == 64) pc_attend_f32_kernel<64><<<grid, 64, 0, st>>>(L, row_call);
    else pc_attend_f32_kernel<128><<<grid, 64, 0, st>>>(L, row_call);
}

// ----------------------------------------------------------------------------------------
// Zero the K or V rows of a span of slots that is taken again after a free.  The attention kernels
// read whole 32-key tiles: behind a message's last token the scores are masked (the prefill kernel
// adds -inf to them) and the V side meets probabilities that are exactly zero, both of which only
// work if what lies there is finite.  A span never used before is zero from the cache's creation;
// one that held another message is cleared here, before the new message's append kernel, on the
// same stream.  The K store and both V layouts keep a head's slots contiguous (bf16 V: groups of 8
// slots, and spans are multiples of 32), so a span is one run of bytes per KV head.
// ----------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void pc_zero_span_kernel(uint4 *__restrict__ store, int64_t head_stride16, int64_t start16,
                                                             int64_t n16)
{
    uint4 *p = store + (int64_t)blockIdx.y * head_stride16 + start16;
    const uint4 z = make_uint4(0, 0, 0, 0);
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (int64_t)gridDim.x * 256) p[i] = z;
}

void pc_launch_zero_span(int dtype, void *store, int64_t slots, int n_kv_heads, int D, int64_t slot_start, int64_t n_slots,
                           hipStream_t st)
{
    if (n_slots <= 0) return;
    const int64_t per_slot16 = (int64_t)D * (dtype == 1 ? 2 : 4) / 16;        // 16-byte pieces per slot and head
    const int64_t n16 = n_slots * per_slot16;
    dim3 grid((unsigned)std::min<int64_t>((n16 + 255) / 256, 1024), (unsigned)n_kv_heads);
    pc_zero_span_kernel<<<grid, 256, 0, st>>>((uint4 *)store, slots * per_slot16, slot_start * per_slot16, n16);
}

// ----------------------------------------------------------------------------------------
// K2g: gather.  A call with many query rows reads its keys and values from a copy of its own:
// the tokens of its parents in list order, one after the other (no padding between messages),
// padded IN FRONT to whole 32-key tiles, then the tokens of its new message.  A key is copied
// turned from its stored position base + t to the position start + t the call gives it (Sec. 2.4
// "Position Updates": the rotation by start - base, here into a copy, so that the cache keeps its
// position-independent form and other calls may place the same message elsewhere); values are
// copied into the cache's own group-of-8 layout.  The attention kernel then walks plain tiles:
// nothing to look up per tile, no turn of the queries per message, one ragged tile per part
// instead of one per message.  Padding rows are written as zeros.  The pass also leaves, per tile of the
// copy and KV head, the largest squared norm of the tile's keys (kg_norm), from which the attention kernel
// bounds the scores of the call before computing any.
// One block per (tile of the copy, KV head).  The first 32 threads find where the tile's tokens
// live (a search in the call's segment offsets); then thread = (key row, 8 low dims and their
// partners 64 up) for K, and thread = (group of 8 tokens, dim) twice for V: when the group's tokens
// sit in 8 consecutive slots (nearly always: messages are long runs of slots) two 16-byte reads and a
// shift, else eight 2-byte reads; one 16-byte write.
// ----------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void pc_gather_kernel(PcLaunch L, const PcGatherItem *__restrict__ items, int n_items,
                                                        const int32_t *__restrict__ seg_kvoff)
{
    __shared__ int s_slot[PC_TILE], s_seg[PC_TILE];
    __shared__ float s_norm[4];
    const int G = blockIdx.x, kh = blockIdx.y;
    int j = 0;
    while (j + 1 < n_items && items[j + 1].kg_tile0 <= G) ++j;           // few calls gather: a short scan
    const PcGatherItem it = items[j];
    const PcCallDesc cd = L.calls[it.call];
    const int t = G - it.kg_tile0;
    const int p_tiles = (it.n_par + PC_TILE - 1) / PC_TILE;
    if (threadIdx.x < PC_TILE) {
        const int r = threadIdx.x;
        int slot = -1, seg = 0;
        if (t < p_tiles) {
            const int i = PC_TILE * t + r - (p_tiles * PC_TILE - it.n_par);   // token of the parents' part (the padding comes first)
            if (i >= 0) {
                const int32_t *off = seg_kvoff + cd.seg_off;
                int lo = 0, hi = cd.n_sel - 1;
                while (lo < hi) {                          // last parent whose first token is <= i (empty ones share their successor's offset)
                    const int mid = (lo + hi + 1) >> 1;
                    if (off[mid] <= i) lo = mid; else hi = mid - 1;
                }
                seg = lo;
                slot = L.segs[cd.seg_off + lo].slot_start + (i - off[lo]);
            }
        } else {
            const int i = PC_TILE * (t - p_tiles) + r;     // token of the new message
            if (i < cd.self_len) { seg = cd.n_seg - 1; slot = L.segs[cd.seg_off + seg].slot_start + i; }
        }
        s_slot[r] = slot; s_seg[r] = seg;
    }
    __syncthreads();
    {
        const int r = threadIdx.x >> 3, c = threadIdx.x & 7;
        const int slot = s_slot[r];
        uint16_t *dst = (uint16_t *)L.k_gather + ((int64_t)kh * L.kg_slots + (int64_t)G * PC_TILE + r) * 128 + 8 * c;
        uint4 lo = make_uint4(0, 0, 0, 0), hi = lo;
        if (slot >= 0) {
            const uint16_t *src = (const uint16_t *)L.k_store + ((int64_t)kh * L.slots + slot) * 128 + 8 * c;
            lo = *reinterpret_cast<const uint4 *>(src);
            hi = *reinterpret_cast<const uint4 *>(src + 64);
            const float4 *rot = reinterpret_cast<const float4 *>(L.rot_seg + (int64_t)(cd.seg_off + s_seg[r]) * 64 + 8 * c);
            uint32_t *lw = reinterpret_cast<uint32_t *>(&lo), *hw = reinterpret_cast<uint32_t *>(&hi);
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const float4 cs = rot[u];                    // (cos, sin) of pairs 2u and 2u + 1
                using P = Pair2<__hip_bfloat16>;
                const float x0 = P::lo(lw[u]), x1 = P::hi(lw[u]), y0 = P::lo(hw[u]), y1 = P::hi(hw[u]);
                lw[u] = P::pack(x0 * cs.x - y0 * cs.y, x1 * cs.z - y1 * cs.w);
                hw[u] = P::pack(x0 * cs.y + y0 * cs.x, x1 * cs.w + y1 * cs.z);
            }
        }
        *reinterpret_cast<uint4 *>(dst) = lo;
        *reinterpret_cast<uint4 *>(dst + 64) = hi;
        // The largest squared norm of the tile's keys, as stored: with the norm of its queries the attention kernel
        // bounds every score of the tile before computing any (|q.k| <= |q| |k|).  Eight lanes hold a row.
        float ss = 0.f;
        {
            using P = Pair2<__hip_bfloat16>;
            const uint32_t *lw = reinterpret_cast<const uint32_t *>(&lo), *hw = reinterpret_cast<const uint32_t *>(&hi);
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const float a = P::lo(lw[u]), b = P::hi(lw[u]), e = P::lo(hw[u]), f = P::hi(hw[u]);
                ss += a * a + b * b + e * e + f * f;
            }
        }
        ss += __shfl_xor(ss, 1); ss += __shfl_xor(ss, 2); ss += __shfl_xor(ss, 4);
        ss = fmaxf(ss, __shfl_xor(ss, 8)); ss = fmaxf(ss, __shfl_xor(ss, 16)); ss = fmaxf(ss, __shfl_xor(ss, 32));
        if ((threadIdx.x & 63) == 0) s_norm[threadIdx.x >> 6] = ss;
    }
    __syncthreads();
    if (threadIdx.x == 0)
        L.kg_norm[(int64_t)kh * (L.kg_slots / PC_TILE) + G] = fmaxf(fmaxf(s_norm[0], s_norm[1]), fmaxf(s_norm[2], s_norm[3]));
    const uint16_t *vsrc = (const uint16_t *)L.v_store;
    uint16_t *vdst = (uint16_t *)L.v_gather;
#pragma unroll
    for (int rep = 0; rep < 2; ++rep) {
        const int idx = threadIdx.x + 256 * rep;
        const int q = idx >> 7, d = idx & 127;             // (q is the same for all lanes of a wave)
        int sl[PC_VGROUP];
        bool run = true;                                   // the group's 8 tokens sit in 8 consecutive slots of the cache
#pragma unroll
        for (int k = 0; k < PC_VGROUP; ++k) {
            sl[k] = s_slot[PC_VGROUP * q + k];
            run = run && sl[0] >= 0 && sl[k] == sl[0] + k;
        }
        uint32_t w[4] = {0u, 0u, 0u, 0u};
        if (run) {
            // two 16-byte reads (this dim of the source group the run starts in, and of the next one) and a shift by
            // the run's offset in its group, instead of eight 2-byte reads
            const int64_t at = (int64_t)kh * L.slots + sl[0];
            const int sh = (int)(at & 7);
            const uint16_t *g0 = vsrc + ((at >> 3) * 128 + d) * PC_VGROUP;
            const uint4 lo = *reinterpret_cast<const uint4 *>(g0);
            uint4 hi = make_uint4(0, 0, 0, 0);
            if (sh) hi = *reinterpret_cast<const uint4 *>(g0 + 128 * PC_VGROUP);
            const uint32_t x[9] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w, 0u};
            const unsigned bits = 16u * (unsigned)(sh & 1);
            switch (sh >> 1) {
            case 0:
#pragma unroll
                for (int j = 0; j < 4; ++j) w[j] = __builtin_amdgcn_alignbit(x[j + 1], x[j], bits);
                break;
            case 1:
#pragma unroll
                for (int j = 0; j < 4; ++j) w[j] = __builtin_amdgcn_alignbit(x[j + 2], x[j + 1], bits);
                break;
            case 2:
#pragma unroll
                for (int j = 0; j < 4; ++j) w[j] = __builtin_amdgcn_alignbit(x[j + 3], x[j + 2], bits);
                break;
            default:
#pragma unroll
                for (int j = 0; j < 4; ++j) w[j] = __builtin_amdgcn_alignbit(x[j + 4], x[j + 3], bits);
                break;
            }
        } else {
#pragma unroll
            for (int k = 0; k < PC_VGROUP; ++k) {
                uint32_t v = 0;
                if (sl[k] >= 0) {
                    const int64_t at = (int64_t)kh * L.slots + sl[k];
                    v = vsrc[((at >> 3) * 128 + d) * PC_VGROUP + (at & 7)];
                }
                w[k >> 1] |= v << (16 * (k & 1));
            }
        }
        const int64_t grp = (((int64_t)kh * L.kg_slots + (int64_t)G * PC_TILE) >> 3) + q;
        *reinterpret_cast<uint4 *>(vdst + (grp * 128 + d) * PC_VGROUP) = make_uint4(w[0], w[1], w[2], w[3]);
    }
}

void pc_launch_gather(const PcLaunch &L, const PcGatherItem *items, int n_items, int64_t n_tiles, const int32_t *seg_kvoff,
                      hipStream_t st)
{
    if (n_items <= 0 || n_tiles <= 0) return;
    dim3 grid((unsigned)n_tiles, (unsigned)L.n_kv_heads);
    pc_gather_kernel<<<grid, 256, 0, st>>>(L, items, n_items, seg_kvoff);
}
