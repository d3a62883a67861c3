// HIP kernels for gfx950 (MI355X): KV-cache append, the unified mixed-batch attention kernel
// (row-streaming body for generation rows, matrix-core body for prompt tiles) and the merge of
// split partial results.
#include <hip/hip_runtime.h>

#include "mpa_internal.h"

namespace mpa {

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

// fp32 -> bf16, round to nearest even (the hardware conversion of gfx950).
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi)
{
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    bf16x2 v = {static_cast<__bf16>(lo), static_cast<__bf16>(hi)};
    return __builtin_bit_cast(uint32_t, v);
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Sum over the 16 lanes of a DPP row (all 16 lanes receive the total).
template <int CTRL>
__device__ __forceinline__ float dpp_add(float x)
{
    int y = __builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xF, 0xF, true);
    return x + __int_as_float(y);
}
constexpr int kQuadPerm1032 = 0xB1;   // lane ^ 1
constexpr int kQuadPerm2301 = 0x4E;   // lane ^ 2
constexpr int kRowHalfMirror = 0x141; // 7 - lane within 8
constexpr int kRowMirror = 0x140;     // 15 - lane within 16

template <int LANES>
__device__ __forceinline__ float group_sum(float x)
{
    x = dpp_add<kQuadPerm1032>(x);
    x = dpp_add<kQuadPerm2301>(x);
    x = dpp_add<kRowHalfMirror>(x);
    if (LANES == 16) x = dpp_add<kRowMirror>(x);
    return x;
}

// ------------------------------------------------------------------------------------------
// KV append: one thread moves 16 bytes of K and 16 bytes of V.
// ------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256)
kv_append_kernel(const uint4 *__restrict__ k_new, const uint4 *__restrict__ v_new,
                 const int64_t *__restrict__ slot_map, int32_t T, int32_t H, int32_t vec_per_row,
                 uint4 *__restrict__ k_cache, uint4 *__restrict__ v_cache)
{
    const int64_t per_token = (int64_t)H * vec_per_row;
    const int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (gid >= (int64_t)T * per_token) return;
    const int32_t t = (int32_t)(gid / per_token);
    const int32_t rem = (int32_t)(gid - (int64_t)t * per_token);
    const int32_t h = rem / vec_per_row;
    const int32_t c = rem - h * vec_per_row;
    const int64_t slot = slot_map[t];
    if (slot < 0) return;
    const int64_t blk = slot / kBlockSize;
    const int32_t off = (int32_t)(slot - blk * kBlockSize);
    const int64_t dst = ((blk * H + h) * kBlockSize + off) * vec_per_row + c;
    k_cache[dst] = k_new[gid];
    v_cache[dst] = v_new[gid];
}

// ------------------------------------------------------------------------------------------
// Row-streaming body: one wavefront, one query row, one head, a contiguous range of KV blocks.
//
// A (block, head) tile of K is 16 tokens x D bf16, contiguous.  A 1 KiB load (16 B per lane)
// covers 64/LPR whole tokens (LPR = D/8 lanes per token): lane l holds elements
// (l % LPR)*8 .. +7 of token l / LPR.  The LPR lanes of a token reduce their partial dot
// products with DPP adds; each group of LPR lanes then runs its own online softmax over "its"
// tokens and accumulates p*v for its 8 elements, so the main loop has no traffic across
// groups.  The groups are combined once at the end.
// ------------------------------------------------------------------------------------------
template <int D>
struct RowCfg {
    static constexpr int LPR = D / 8;             // lanes per token row
    static constexpr int TPL = 64 / LPR;          // tokens per 1 KiB load
    static constexpr int NL = kBlockSize / TPL;   // loads per (block, head) tile
};

template <int D>
struct KvRegs {
    u32x4 k[RowCfg<D>::NL];
    u32x4 v[RowCfg<D>::NL];
};

template <int D>
__device__ __forceinline__ void issue_loads(KvRegs<D> &r, const uint16_t *__restrict__ k_cache,
                                            const uint16_t *__restrict__ v_cache, int32_t blk,
                                            int32_t H, int32_t head, int lane)
{
    const size_t tile = ((size_t)blk * H + head) * (kBlockSize * D);
    const u32x4 *kp = reinterpret_cast<const u32x4 *>(k_cache + tile) + lane;
    const u32x4 *vp = reinterpret_cast<const u32x4 *>(v_cache + tile) + lane;
#pragma unroll
    for (int i = 0; i < RowCfg<D>::NL; ++i) r.k[i] = __builtin_nontemporal_load(kp + i * 64);
#pragma unroll
    for (int i = 0; i < RowCfg<D>::NL; ++i) r.v[i] = __builtin_nontemporal_load(vp + i * 64);
}

template <int D, bool MASKED>
__device__ __forceinline__ void consume(const KvRegs<D> &r, const float (&qf)[8], float &m,
                                        float &l, float (&acc)[8], int32_t tok0, int32_t limit,
                                        int sub)
{
    using C = RowCfg<D>;
    float s[C::NL];
#pragma unroll
    for (int i = 0; i < C::NL; ++i) {
        const u32x4 w = r.k[i];
        float d = qf[0] * bf16_lo(w.x);
        d = fmaf(qf[1], bf16_hi(w.x), d);
        d = fmaf(qf[2], bf16_lo(w.y), d);
        d = fmaf(qf[3], bf16_hi(w.y), d);
        d = fmaf(qf[4], bf16_lo(w.z), d);
        d = fmaf(qf[5], bf16_hi(w.z), d);
        d = fmaf(qf[6], bf16_lo(w.w), d);
        d = fmaf(qf[7], bf16_hi(w.w), d);
        d = group_sum<C::LPR>(d);
        if (MASKED) {
            const bool valid = tok0 + i * C::TPL + sub < limit;
            d = valid ? d : -INFINITY;
        }
        s[i] = d;
    }
    float m_new = m;
#pragma unroll
    for (int i = 0; i < C::NL; ++i) m_new = fmaxf(m_new, s[i]);
    const float m_safe = (m_new == -INFINITY) ? 0.f : m_new;
    const float alpha = fast_exp2(m - m_safe);
    l *= alpha;
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] *= alpha;
#pragma unroll
    for (int i = 0; i < C::NL; ++i) {
        const float p = fast_exp2(s[i] - m_safe);
        l += p;
        u32x4 w = r.v[i];
        if (MASKED) {
            const bool valid = tok0 + i * C::TPL + sub < limit;
            if (!valid) w = u32x4{0u, 0u, 0u, 0u};
        }
        acc[0] = fmaf(p, bf16_lo(w.x), acc[0]);
        acc[1] = fmaf(p, bf16_hi(w.x), acc[1]);
        acc[2] = fmaf(p, bf16_lo(w.y), acc[2]);
        acc[3] = fmaf(p, bf16_hi(w.y), acc[3]);
        acc[4] = fmaf(p, bf16_lo(w.z), acc[4]);
        acc[5] = fmaf(p, bf16_hi(w.z), acc[5]);
        acc[6] = fmaf(p, bf16_lo(w.w), acc[6]);
        acc[7] = fmaf(p, bf16_hi(w.w), acc[7]);
    }
    m = m_new;
}

template <int D>
__device__ __forceinline__ void row_body(const AttnParams &p, const WorkItem &it, int head, int lane)
{
    using C = RowCfg<D>;
    const int H = p.heads;
    const int c = lane % C::LPR;
    const int sub = lane / C::LPR;

    float qf[8];
    {
        const uint4 w = *reinterpret_cast<const uint4 *>(p.q + ((size_t)it.q_row0 * H + head) * D + c * 8);
        const float sc = p.scale_log2e;
        qf[0] = bf16_lo(w.x) * sc; qf[1] = bf16_hi(w.x) * sc;
        qf[2] = bf16_lo(w.y) * sc; qf[3] = bf16_hi(w.y) * sc;
        qf[4] = bf16_lo(w.z) * sc; qf[5] = bf16_hi(w.z) * sc;
        qf[6] = bf16_lo(w.w) * sc; qf[7] = bf16_hi(w.w) * sc;
    }
    float m = -INFINITY, l = 0.f;
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};

    const int32_t limit = min(it.kv_end, it.q_pos0 + 1);   // keys [kv_begin, limit)
    const int32_t b0 = it.kv_begin / kBlockSize;
    const int32_t nblk = (limit - it.kv_begin + kBlockSize - 1) / kBlockSize;
    const int32_t *tab = p.block_table + (size_t)it.seq * p.table_stride + b0;

    for (int32_t g0 = 0; g0 < nblk; g0 += 64) {
        const int32_t n = min(64, nblk - g0);
        // 64 table entries at a time, one per lane, broadcast from registers as needed
        const int32_t mine = (lane < n) ? tab[g0 + lane] : 0;
        auto blk_of = [&](int j) { return __builtin_amdgcn_readlane(mine, j); };
        auto step = [&](const KvRegs<D> &r, int j) {
            const int32_t tok0 = it.kv_begin + (g0 + j) * kBlockSize;
            if (tok0 + kBlockSize <= limit) consume<D, false>(r, qf, m, l, acc, tok0, limit, sub);
            else consume<D, true>(r, qf, m, l, acc, tok0, limit, sub);
        };
        KvRegs<D> r0, r1;
        issue_loads<D>(r0, p.k_cache, p.v_cache, blk_of(0), H, head, lane);
        for (int j = 0; j < n; j += 2) {
            if (j + 1 < n) issue_loads<D>(r1, p.k_cache, p.v_cache, blk_of(j + 1), H, head, lane);
            step(r0, j);
            if (j + 1 < n) {
                if (j + 2 < n) issue_loads<D>(r0, p.k_cache, p.v_cache, blk_of(j + 2), H, head, lane);
                step(r1, j + 1);
            }
        }
    }

    // combine the 64/LPR token groups of the wavefront
    float m_all = m;
#pragma unroll
    for (int off = C::LPR; off < 64; off <<= 1) m_all = fmaxf(m_all, __shfl_xor(m_all, off));
    const float m_safe = (m_all == -INFINITY) ? 0.f : m_all;
    const float w = fast_exp2(m - m_safe);
    l *= w;
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] *= w;
#pragma unroll
    for (int off = C::LPR; off < 64; off <<= 1) {
        l += __shfl_xor(l, off);
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] += __shfl_xor(acc[e], off);
    }
    if (sub == 0) {
        if (it.part_row < 0) {
            const float inv = 1.f / l;
            uint4 o;
            o.x = pack_bf16(acc[0] * inv, acc[1] * inv);
            o.y = pack_bf16(acc[2] * inv, acc[3] * inv);
            o.z = pack_bf16(acc[4] * inv, acc[5] * inv);
            o.w = pack_bf16(acc[6] * inv, acc[7] * inv);
            *reinterpret_cast<uint4 *>(p.out + ((size_t)it.q_row0 * H + head) * D + c * 8) = o;
        } else {
            const size_t prow = (size_t)it.part_row * H + head;
            float4 *dst = reinterpret_cast<float4 *>(p.part_acc + prow * D + c * 8);
            dst[0] = make_float4(acc[0], acc[1], acc[2], acc[3]);
            dst[1] = make_float4(acc[4], acc[5], acc[6], acc[7]);
            if (c == 0) *reinterpret_cast<float2 *>(p.part_ml + prow * 2) = make_float2(m_all, l);
        }
    }
}

// ------------------------------------------------------------------------------------------
// Unified kernel: work-groups [0, n_tile_items*H) run prompt tiles, the rest run row items
// (one wavefront per head, kWaves consecutive heads per work-group).
// ------------------------------------------------------------------------------------------
template <int D>
__global__ void __launch_bounds__(kThreads)
attention_kernel(const AttnParams p)
{
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int H = p.heads;
    const int64_t n_tile_wg = (int64_t)p.n_tile_items * H;
    if ((int64_t)blockIdx.x < n_tile_wg) {
        // prompt tiles: matrix-core body (not reached while tiles are planned as row items)
        return;
    }
    const int hg = (H + kWaves - 1) / kWaves;
    const int64_t idx = (int64_t)blockIdx.x - n_tile_wg;
    const int32_t item = p.n_tile_items + (int32_t)(idx / hg);
    const int head = (int)(idx % hg) * kWaves + wave;
    if (head >= H) return;
    const WorkItem it = p.items[item];
    row_body<D>(p, it, head, lane);
}

// ------------------------------------------------------------------------------------------
// Merge: one wavefront per (merge row, head).
// ------------------------------------------------------------------------------------------
template <int D>
__global__ void __launch_bounds__(256)
merge_kernel(const AttnParams p)
{
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int H = p.heads;
    const int64_t unit = (int64_t)blockIdx.x * 4 + wave;
    if (unit >= (int64_t)p.n_merge * H) return;
    const int32_t r = (int32_t)(unit / H);
    const int head = (int)(unit % H);
    const MergeRow mr = p.merge[r];
    constexpr int EPL = D / 64;  // elements per lane
    float m_all = -INFINITY;
    for (int s = 0; s < mr.nsplit; ++s) {
        const size_t prow = ((size_t)mr.part_row + (size_t)s * mr.stride) * H + head;
        m_all = fmaxf(m_all, p.part_ml[prow * 2]);
    }
    float l = 0.f;
    float acc[EPL];
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[e] = 0.f;
    for (int s = 0; s < mr.nsplit; ++s) {
        const size_t prow = ((size_t)mr.part_row + (size_t)s * mr.stride) * H + head;
        const float2 ml = *reinterpret_cast<const float2 *>(p.part_ml + prow * 2);
        const float w = fast_exp2(ml.x - m_all);
        l = fmaf(ml.y, w, l);
        const float *a = p.part_acc + prow * D + lane * EPL;
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[e] = fmaf(a[e], w, acc[e]);
    }
    const float inv = 1.f / l;
    uint16_t *o = p.out + ((size_t)mr.out_row * H + head) * D + lane * EPL;
    if (EPL == 2) {
        *reinterpret_cast<uint32_t *>(o) = pack_bf16(acc[0] * inv, acc[EPL - 1] * inv);
    } else {
        *o = (uint16_t)(pack_bf16(acc[0] * inv, 0.f) & 0xFFFFu);
    }
}

}  // namespace

int launch_kv_append(const void *k_new, const void *v_new, const int64_t *slot_map, int32_t T,
                     int32_t H, int32_t D, void *k_cache, void *v_cache, void *stream)
{
    const int32_t vec_per_row = D / 8;
    const int64_t total = (int64_t)T * H * vec_per_row;
    if (total == 0) return 0;
    const int64_t blocks = (total + 255) / 256;
    hipLaunchKernelGGL(kv_append_kernel, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream,
                       (const uint4 *)k_new, (const uint4 *)v_new, slot_map, T, H, vec_per_row,
                       (uint4 *)k_cache, (uint4 *)v_cache);
    return (int)hipGetLastError();
}

int launch_attention(const AttnParams &p, int32_t D, void *stream)
{
    const int hg = (p.heads + kWaves - 1) / kWaves;
    const int64_t grid = (int64_t)p.n_tile_items * p.heads + (int64_t)p.n_row_items * hg;
    if (grid == 0) return 0;
    if (grid > 0x7FFFFFFF) return (int)hipErrorInvalidConfiguration;
    if (D == 128)
        hipLaunchKernelGGL(attention_kernel<128>, dim3((unsigned)grid), dim3(kThreads), 0, (hipStream_t)stream, p);
    else
        hipLaunchKernelGGL(attention_kernel<64>, dim3((unsigned)grid), dim3(kThreads), 0, (hipStream_t)stream, p);
    return (int)hipGetLastError();
}

int launch_merge(const AttnParams &p, int32_t D, void *stream)
{
    const int64_t units = (int64_t)p.n_merge * p.heads;
    if (units == 0) return 0;
    const int64_t grid = (units + 3) / 4;
    if (D == 128)
        hipLaunchKernelGGL(merge_kernel<128>, dim3((unsigned)grid), dim3(256), 0, (hipStream_t)stream, p);
    else
        hipLaunchKernelGGL(merge_kernel<64>, dim3((unsigned)grid), dim3(256), 0, (hipStream_t)stream, p);
    return (int)hipGetLastError();
}

}  // namespace mpa
