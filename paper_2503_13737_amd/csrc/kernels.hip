// HIP kernels for gfx950 (MI355X): KV-cache append, work-list upload (alone or sharing a launch
// with the append), block copies between cache pools, the unified mixed-batch attention kernel
// (row-streaming body for generation rows, matrix-core body for prompt tiles and for grouped
// generation rows) and the merge of split partial results.  Every kernel that touches K/V
// elements exists for both 16-bit storage types.
#include <cstring>
#include <mutex>
#include <type_traits>
#include <hip/hip_runtime.h>

#include "mpa_internal.h"

namespace mpa {

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

// The two 16-bit storage types.  lo/hi widen the halves of a 32-bit word, pack rounds two fp32
// results to nearest even for the output; weights2 / dot2 / mfma are the matrix-core body's
// conversion of two softmax weights, their sum, and the 32x32x16 product.
//
// kWeightCap: a lane's sum of 16 weights above this makes the body re-reference the row (see
// tile_compute).  kRefShift: the reference exponent is set this far below the row maximum, so the
// largest weight is 2^kRefShift right after re-referencing.
struct Bf16 {
    typedef __bf16 x2 __attribute__((ext_vector_type(2)));
    typedef __bf16 x8 __attribute__((ext_vector_type(8)));
    static constexpr float kWeightCap = 0x1p64f;
    static constexpr float kRefShift = 0.f;
    static __device__ __forceinline__ float lo(uint32_t w) { return __uint_as_float(w << 16); }
    static __device__ __forceinline__ float hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }
    static __device__ __forceinline__ uint32_t pack(float a, float b)
    {
        x2 v = {static_cast<__bf16>(a), static_cast<__bf16>(b)};
        return __builtin_bit_cast(uint32_t, v);
    }
    static __device__ __forceinline__ x2 weights2(float a, float b) { return x2{static_cast<__bf16>(a), static_cast<__bf16>(b)}; }
    static __device__ __forceinline__ x2 ones2() { return x2{static_cast<__bf16>(1.0f), static_cast<__bf16>(1.0f)}; }
    static __device__ __forceinline__ float dot2(x2 a, x2 b, float c) { return __builtin_amdgcn_fdot2_f32_bf16(a, b, c, false); }
    static __device__ __forceinline__ f32x16 mfma(x8 a, x8 b, f32x16 c)
    {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
    }
};

// IEEE half: 5 exponent bits, largest finite value 65504.  Weights are converted with the packed
// round-toward-zero instruction (one instruction per pair; the row sum is taken from the
// converted values, so numerator and denominator see the same rounding); it saturates at 65504
// instead of producing infinity, which the cap below 65504 still catches.  The reference sits 8
// binades below the row maximum: weights start at up to 2^8, have 7 binades of head room before
// the cap, and keep full precision down to 2^-22 of the maximum.
struct Fp16 {
    typedef _Float16 x2 __attribute__((ext_vector_type(2)));
    typedef _Float16 x8 __attribute__((ext_vector_type(8)));
    static constexpr float kWeightCap = 0x1p15f;
    static constexpr float kRefShift = 8.f;
    static __device__ __forceinline__ float lo(uint32_t w) { return (float)__builtin_bit_cast(_Float16, (uint16_t)(w & 0xFFFFu)); }
    static __device__ __forceinline__ float hi(uint32_t w) { return (float)__builtin_bit_cast(_Float16, (uint16_t)(w >> 16)); }
    static __device__ __forceinline__ uint32_t pack(float a, float b)
    {
        x2 v = {static_cast<_Float16>(a), static_cast<_Float16>(b)};
        return __builtin_bit_cast(uint32_t, v);
    }
    static __device__ __forceinline__ x2 weights2(float a, float b)
    {
        return __builtin_bit_cast(x2, __builtin_amdgcn_cvt_pkrtz(a, b));
    }
    static __device__ __forceinline__ x2 ones2() { return x2{(_Float16)1.0f, (_Float16)1.0f}; }
    static __device__ __forceinline__ float dot2(x2 a, x2 b, float c) { return __builtin_amdgcn_fdot2(a, b, c, false); }
    static __device__ __forceinline__ f32x16 mfma(x8 a, x8 b, f32x16 c)
    {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
    }
};

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

// Page j (16 tokens) of a sequence as one word (see kPage): table entry j >> shift, page j & mask.
__device__ __forceinline__ int32_t page_word(const int32_t *table_row, int32_t j, int32_t page_shift)
{
    return (table_row[j >> page_shift] << kPageBits) | (j & ((1 << page_shift) - 1));
}
// First element of that page for one K/V head in a cache laid out [blocks][heads][block_size][D].
template <int D>
__device__ __forceinline__ size_t page_offset(int32_t word, int32_t kv_heads, int32_t kv_head, int32_t page_shift)
{
    const size_t blk = (size_t)(word >> kPageBits);
    const size_t sub = (size_t)(word & ((1 << kPageBits) - 1));
    return (((blk * kv_heads + kv_head) << page_shift) + sub) * (size_t)(kPage * D);
}

// ------------------------------------------------------------------------------------------
// KV append: one thread moves 16 bytes of K and 16 bytes of V.
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ void append_body(int64_t gid, const uint4 *__restrict__ k_new, const uint4 *__restrict__ v_new,
                                            const int64_t *__restrict__ slot_map, int32_t T, int32_t H, int32_t vec_per_row,
                                            int32_t block_size, uint4 *__restrict__ k_cache, uint4 *__restrict__ v_cache)
{
    const int64_t per_token = (int64_t)H * vec_per_row;
    if (gid >= (int64_t)T * per_token) return;
    const int32_t t = (int32_t)(gid / per_token);
    const int32_t rem = (int32_t)(gid - (int64_t)t * per_token);
    const int32_t h = rem / vec_per_row;
    const int32_t c = rem - h * vec_per_row;
    const int64_t slot = slot_map[t];
    if (slot < 0) return;
    const int64_t blk = slot / block_size;
    const int32_t off = (int32_t)(slot - blk * block_size);
    const int64_t dst = ((blk * H + h) * block_size + off) * vec_per_row + c;
    k_cache[dst] = k_new[gid];
    v_cache[dst] = v_new[gid];
}

__global__ void __launch_bounds__(256)
kv_append_kernel(const uint4 *__restrict__ k_new, const uint4 *__restrict__ v_new,
                 const int64_t *__restrict__ slot_map, int32_t T, int32_t H, int32_t vec_per_row,
                 int32_t block_size, uint4 *__restrict__ k_cache, uint4 *__restrict__ v_cache)
{
    append_body((int64_t)blockIdx.x * 256 + threadIdx.x, k_new, v_new, slot_map, T, H, vec_per_row, block_size, k_cache, v_cache);
}

// ------------------------------------------------------------------------------------------
// Work-list upload: the few KiB the host planned go from pinned host memory (which the GPU reads
// directly) into the workspace.  A kernel in the launch queue instead of an asynchronous memory
// copy: the copy engine's hand-over to the next kernel costs more than the copy itself.  One
// work-group, 64 KiB in flight per round; when every thread has read its share it tells the host,
// through a word in the same pinned allocation, that the staging buffer may be refilled (an
// event recorded behind the kernel would put a barrier into the queue for the same news).
// ------------------------------------------------------------------------------------------
constexpr int kUploadThreads = 1024;
template <int THREADS>
__device__ __forceinline__ void upload_body(const u32x4 *__restrict__ src, u32x4 *__restrict__ dst, int64_t n,
                                            uint64_t *done_flag, uint64_t ticket)
{
    for (int64_t i0 = threadIdx.x; i0 < n; i0 += THREADS * 4) {
        u32x4 v[4];
#pragma unroll
        for (int k = 0; k < 4; ++k)
            if (i0 + k * THREADS < n) v[k] = src[i0 + k * THREADS];
#pragma unroll
        for (int k = 0; k < 4; ++k)
            if (i0 + k * THREADS < n) dst[i0 + k * THREADS] = v[k];
    }
    __syncthreads();   // every thread's stores are issued, so all its loads from src have returned
    if (threadIdx.x == 0) __hip_atomic_store(done_flag, ticket, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
}

__global__ void __launch_bounds__(kUploadThreads)
upload_kernel(const u32x4 *__restrict__ src, u32x4 *__restrict__ dst, int64_t n, uint64_t *done_flag, uint64_t ticket)
{
    upload_body<kUploadThreads>(src, dst, n, done_flag, ticket);
}

// The append of an iteration's K/V and the upload of its work list in one launch (neither needs
// the other; both must precede the attention kernel): work-group 0 uploads, the rest append.
__global__ void __launch_bounds__(256)
append_upload_kernel(const uint4 *__restrict__ k_new, const uint4 *__restrict__ v_new,
                     const int64_t *__restrict__ slot_map, int32_t T, int32_t H, int32_t vec_per_row,
                     int32_t block_size, uint4 *__restrict__ k_cache, uint4 *__restrict__ v_cache,
                     const u32x4 *__restrict__ list_src, u32x4 *__restrict__ list_dst, int64_t list_vecs,
                     uint64_t *done_flag, uint64_t ticket)
{
    if (blockIdx.x == 0) {
        upload_body<256>(list_src, list_dst, list_vecs, done_flag, ticket);
        return;
    }
    append_body(((int64_t)blockIdx.x - 1) * 256 + threadIdx.x, k_new, v_new, slot_map, T, H, vec_per_row, block_size, k_cache, v_cache);
}

// ------------------------------------------------------------------------------------------
// Block copy: work-group (x, i) moves 16 KiB of K and of V of pair i (1024 lanes x 16 bytes each,
// four per thread, all loads issued before the stores).
// ------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256)
copy_blocks_kernel(const u32x4 *__restrict__ src_k, const u32x4 *__restrict__ src_v, u32x4 *__restrict__ dst_k,
                   u32x4 *__restrict__ dst_v, const int64_t *__restrict__ pairs, int64_t vec_per_block)
{
    const int64_t src = pairs[2 * (int64_t)blockIdx.y], dst = pairs[2 * (int64_t)blockIdx.y + 1];
    if (src < 0 || dst < 0) return;
    const int64_t v0 = (int64_t)blockIdx.x * 1024 + threadIdx.x;
    const u32x4 *sk = src_k + src * vec_per_block, *sv = src_v + src * vec_per_block;
    u32x4 *dk = dst_k + dst * vec_per_block, *dv = dst_v + dst * vec_per_block;
    u32x4 k[4], v[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int64_t j = v0 + i * 256;
        if (j < vec_per_block) {
            k[i] = __builtin_nontemporal_load(sk + j);
            v[i] = __builtin_nontemporal_load(sv + j);
        }
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int64_t j = v0 + i * 256;
        if (j < vec_per_block) {
            __builtin_nontemporal_store(k[i], dk + j);
            __builtin_nontemporal_store(v[i], dv + j);
        }
    }
}

// ------------------------------------------------------------------------------------------
// Row-streaming body: one wavefront, one query row, one head, a contiguous range of KV blocks.
//
// A (page, head) tile of K is 16 tokens x D 16-bit elements, contiguous.  A 1 KiB load (16 B per lane)
// covers 64/LPR whole tokens (LPR = D/8 lanes per token): lane l holds elements
// (l % LPR)*8 .. +7 of token l / LPR.  The LPR lanes of a token reduce their partial dot
// products with DPP adds; each group of LPR lanes then runs its own online softmax over "its"
// tokens and accumulates p*v for its 8 elements, so the main loop has no traffic across
// groups.  The groups are combined once at the end.
// ------------------------------------------------------------------------------------------
constexpr int kRowSets = 3;   // register sets of a row-streaming wavefront (more were measured: no gain, narrow or wide)

template <int D>
struct RowCfg {
    static constexpr int LPR = D / 8;             // lanes per token row
    static constexpr int TPL = 64 / LPR;          // tokens per 1 KiB load
    static constexpr int NL = kPage / TPL;        // loads per page of one head
};

template <int D>
struct KvRegs {
    u32x4 k[RowCfg<D>::NL];
    u32x4 v[RowCfg<D>::NL];
};

template <int D>
__device__ __forceinline__ void issue_loads(KvRegs<D> &r, const uint16_t *__restrict__ k_cache,
                                            const uint16_t *__restrict__ v_cache, int32_t page,
                                            int32_t HK, int32_t kv_head, int32_t page_shift, int lane)
{
    const size_t tile = page_offset<D>(page, HK, kv_head, page_shift);
    const u32x4 *kp = reinterpret_cast<const u32x4 *>(k_cache + tile) + lane;
    const u32x4 *vp = reinterpret_cast<const u32x4 *>(v_cache + tile) + lane;
#pragma unroll
    for (int i = 0; i < RowCfg<D>::NL; ++i) r.k[i] = __builtin_nontemporal_load(kp + i * 64);
#pragma unroll
    for (int i = 0; i < RowCfg<D>::NL; ++i) r.v[i] = __builtin_nontemporal_load(vp + i * 64);
}

// The same loads for the page that holds the row's own position when this iteration's K/V is not
// in the cache yet (append inside the launch): the lanes of that token (in-page index `slot`) read
// their 16 bytes from the new rows nk / nv, every other lane from the cache as usual.
template <int D>
__device__ __forceinline__ void issue_loads_own(KvRegs<D> &r, const uint16_t *__restrict__ k_cache,
                                                const uint16_t *__restrict__ v_cache, int32_t page, int32_t HK,
                                                int32_t kv_head, int32_t page_shift, int lane, const u32x4 *nk,
                                                const u32x4 *nv, int slot)
{
    using C = RowCfg<D>;
    const size_t tile = page_offset<D>(page, HK, kv_head, page_shift);
    const u32x4 *kp = reinterpret_cast<const u32x4 *>(k_cache + tile) + lane;
    const u32x4 *vp = reinterpret_cast<const u32x4 *>(v_cache + tile) + lane;
    const int c = lane % C::LPR, sub = lane / C::LPR;
#pragma unroll
    for (int i = 0; i < C::NL; ++i) r.k[i] = __builtin_nontemporal_load(i * C::TPL + sub == slot ? nk + c : kp + i * 64);
#pragma unroll
    for (int i = 0; i < C::NL; ++i) r.v[i] = __builtin_nontemporal_load(i * C::TPL + sub == slot ? nv + c : vp + i * 64);
}

template <class E, int D, bool MASKED>
__device__ __forceinline__ void consume(const KvRegs<D> &r, const float (&qf)[8], float &m,
                                        float &l, float (&acc)[8], int32_t tok0, int32_t limit,
                                        int sub)
{
    using C = RowCfg<D>;
    float s[C::NL];
#pragma unroll
    for (int i = 0; i < C::NL; ++i) {
        const u32x4 w = r.k[i];
        float d = qf[0] * E::lo(w.x);
        d = fmaf(qf[1], E::hi(w.x), d);
        d = fmaf(qf[2], E::lo(w.y), d);
        d = fmaf(qf[3], E::hi(w.y), d);
        d = fmaf(qf[4], E::lo(w.z), d);
        d = fmaf(qf[5], E::hi(w.z), d);
        d = fmaf(qf[6], E::lo(w.w), d);
        d = fmaf(qf[7], E::hi(w.w), d);
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
        acc[0] = fmaf(p, E::lo(w.x), acc[0]);
        acc[1] = fmaf(p, E::hi(w.x), acc[1]);
        acc[2] = fmaf(p, E::lo(w.y), acc[2]);
        acc[3] = fmaf(p, E::hi(w.y), acc[3]);
        acc[4] = fmaf(p, E::lo(w.z), acc[4]);
        acc[5] = fmaf(p, E::hi(w.z), acc[5]);
        acc[6] = fmaf(p, E::lo(w.w), acc[6]);
        acc[7] = fmaf(p, E::hi(w.w), acc[7]);
    }
    m = m_new;
}

template <class E, int D, int NS, bool FUSED>
__device__ __forceinline__ void row_body(const AttnParams &p, const WorkItem &it, int head, int lane)
{
    using C = RowCfg<D>;
    const int H = p.heads;
    const int HK = p.kv_heads;
    const int kv_head = head / p.group;
    const int c = lane % C::LPR;
    const int sub = lane / C::LPR;

    float qf[8];
    {
        const uint4 w = *reinterpret_cast<const uint4 *>(p.q + ((size_t)it.q_row0 * H + head) * D + c * 8);
        const float sc = p.scale_log2e;
        qf[0] = E::lo(w.x) * sc; qf[1] = E::hi(w.x) * sc;
        qf[2] = E::lo(w.y) * sc; qf[3] = E::hi(w.y) * sc;
        qf[4] = E::lo(w.z) * sc; qf[5] = E::hi(w.z) * sc;
        qf[6] = E::lo(w.w) * sc; qf[7] = E::hi(w.w) * sc;
    }
    float m = -INFINITY, l = 0.f;
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};

    const int32_t limit = min(it.kv_end, it.q_pos0 + 1);   // keys [kv_begin, limit)
    const int32_t b0 = it.kv_begin / kPage;   // pages from here on ("blk" below is a page word)
    const int32_t nblk = (limit - it.kv_begin + kPage - 1) / kPage;
    const int32_t *tab = p.block_table + (size_t)it.seq * p.table_stride;
    const int32_t page_shift = p.page_shift;
    // Append inside the launch: the row's own token (position q_pos0, the last key of the range that
    // reaches it) is not in the cache yet; its K/V is row q_row0 of k_new / v_new.
    const bool own_new = FUSED && it.kv_end > it.q_pos0;
    const u32x4 *own_k = nullptr, *own_v = nullptr;
    if (own_new) {
        const size_t el = ((size_t)it.q_row0 * HK + kv_head) * D;
        own_k = reinterpret_cast<const u32x4 *>(p.k_new + el);
        own_v = reinterpret_cast<const u32x4 *>(p.v_new + el);
    }

    for (int32_t g0 = 0; g0 < nblk; g0 += 64) {
        const int32_t n = min(64, nblk - g0);
        // 64 pages at a time, one per lane, broadcast from registers as needed
        const int32_t mine = (lane < n) ? page_word(tab, b0 + g0 + lane, page_shift) : 0;
        auto blk_of = [&](int j) { return __builtin_amdgcn_readlane(mine, j); };
        auto step = [&](const KvRegs<D> &r, int j) {
            const int32_t tok0 = it.kv_begin + (g0 + j) * kPage;
            if (tok0 + kPage <= limit) consume<E, D, false>(r, qf, m, l, acc, tok0, limit, sub);
            else consume<E, D, true>(r, qf, m, l, acc, tok0, limit, sub);
        };
        // NS register sets rotate: NS-1 blocks (8 KiB each at D=128) are in flight while one is consumed
        KvRegs<D> r[NS];
        auto issue = [&](KvRegs<D> &rr, int jj) {   // page g0 + jj of the range
            if (own_new && g0 + jj == nblk - 1)
                issue_loads_own<D>(rr, p.k_cache, p.v_cache, blk_of(jj), HK, kv_head, page_shift, lane, own_k, own_v,
                                   it.q_pos0 % kPage);
            else
                issue_loads<D>(rr, p.k_cache, p.v_cache, blk_of(jj), HK, kv_head, page_shift, lane);
        };
#pragma unroll
        for (int s = 0; s < NS - 1; ++s)
            if (s < n) issue(r[s], s);
        for (int j = 0; j < n; j += NS) {
#pragma unroll
            for (int s = 0; s < NS; ++s) {
                if (j + s < n) {
                    if (j + s + NS - 1 < n) issue(r[(s + NS - 1) % NS], j + s + NS - 1);
                    step(r[s], j + s);
                }
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
            o.x = E::pack(acc[0] * inv, acc[1] * inv);
            o.y = E::pack(acc[2] * inv, acc[3] * inv);
            o.z = E::pack(acc[4] * inv, acc[5] * inv);
            o.w = E::pack(acc[6] * inv, acc[7] * inv);
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
// Matrix-core body: one work-group (4 wavefronts), one head, a tile of up to 128 query rows
// (32 per wavefront), a contiguous key range walked in steps of 64 keys.
//
// Per step the work-group holds K [64 keys][D] and V [64 keys][D] row-major in LDS, loaded
// straight from HBM, two buffers.  Each wavefront computes S^T = K Q^T with 32x32x16 bf16 MFMAs
// (A = K rows from LDS, B = Q^T from registers), so a lane owns ONE query row (lane % 32) and 32
// of the 64 keys: row sums (and, when needed, row maxima) are in-lane reductions plus one
// exchange with lane ^ 32.  The weights, packed to bf16 in the very registers they were produced
// in, are the B operand of O^T += V^T P^T (A = V through the transposing LDS read), whose result
// again has the query row on the lane, so the occasional rescale needs no cross-lane traffic.
//
// Register layouts of v_mfma_f32_32x32x16_bf16 (lane l, half = l / 32):
//   A: row l % 32, k = 8*half .. 8*half+7        B: column l % 32, k = 8*half .. 8*half+7
//   C: column l % 32, rows 8*(v/4) + 4*half + v%4 for v = 0..15
// ------------------------------------------------------------------------------------------
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

template <int D, int WAVES = kWaves>
struct TileCfg {
    static constexpr int KS = D / 16;                   // k-steps of K Q^T
    static constexpr int DB = D / 32;                   // 32-row blocks of O^T
    // K and V tiles sit in LDS row-major, [64 keys][D], rows unpadded (ROW bytes), because they are
    // written by direct-to-LDS loads that place a wavefront's 64 x 16 bytes contiguously.  Bank
    // conflicts are avoided by a swizzle instead: the 16-byte chunk c of row r is stored at chunk
    // position c ^ swz(r), applied on the global-address side of the load.
    //   K rows are read 16 bytes per lane, four consecutive lanes (= four consecutive rows, same c)
    //   per LDS cycle: swz_k(r) = r mod CPR keeps them on different banks.
    //   V rows are read by the transposing load, 16 lanes touching 4 rows x 32 bytes: swz_v(r) =
    //   VSW * (r mod 4) spreads those rows (and the neighbouring lane group's 32 bytes) over all banks.
    static constexpr int ROW = D * 2;
    static constexpr int TILE_BYTES = kKvTile * ROW;
    static constexpr int K_BYTES = TILE_BYTES;
    static constexpr int V_BYTES = TILE_BYTES;
    static constexpr int CPR = D / 8;                   // 16-byte chunks per key row
    static constexpr int RPL = 64 / CPR;                // key rows covered by one wavefront-wide load
    static constexpr int KPW = kKvTile / WAVES;         // key rows of a step that one wavefront loads
    static constexpr int NL = KPW / RPL;                // loads per wavefront per operand and step
    static_assert(NL >= 1 && KPW <= kPage, "a wavefront loads whole rows of one page");
    static constexpr int VSW = CPR / 4;                 // 4 for D = 128, 2 for D = 64
};

// Everything a wavefront needs to issue its share of the next step's loads from inside
// tile_compute.  Only gk/gv change from step to step, and they are wavefront-uniform, so the
// loads address memory as scalar base + per-lane 32-bit offset and the loop spends no vector
// arithmetic on them.
template <int D, int WAVES = kWaves>
struct TileNext {
    const char *gk, *gv;                  // the page (16 keys) that holds the wavefront's rows, in the K and V caches
    uint32_t koff[TileCfg<D, WAVES>::NL]; // this lane's byte offset inside the page for load i (K swizzle)
    uint32_t voff[TileCfg<D, WAVES>::NL]; // same with the V swizzle
    uint32_t lds_w;                       // LDS address of the wavefront's 16 rows in the K tile of buffer 0
    bool stream;                          // K/V of this item are read once (see load_to_lds_16)
    // Append inside the launch: rows of the tile from position `new_begin` of the sequence on are not in
    // the cache yet.  nk / nv: where the page that holds the wavefront's rows would start in k_new /
    // v_new (token rows there are new_extra bytes further apart than in a cache page).
    const char *nk, *nv;
    uint32_t new_extra;
};

// 16 bytes per lane from base + off (base wavefront-uniform, in scalar registers) straight into
// LDS at lds_dst + 16 * lane (lds_dst wavefront-uniform; the instruction takes it from M0).
// Written by hand because the compiler's selection of this instruction always forms a 64-bit
// address per lane.  It is invisible to the compiler's bookkeeping of outstanding memory
// operations: whoever needs the data waits for vmcnt(0) explicitly.  M0 is written and consumed
// inside the statement and named as clobbered; nothing else in these kernels uses M0 (LDS
// instructions of this architecture take none).
// `stream` (wavefront-uniform) marks data that is read once: the load then carries the
// non-temporal hint, as the loads of the row body do.  Measured on grouped generation rows: 8-10 %
// more bytes per second than without it (prompt tiles, whose K/V other tiles read again from cache,
// go without).
__device__ __forceinline__ void load_to_lds_16(const char *base, uint32_t off, uint32_t lds_dst, bool stream)
{
    if (stream)
        asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1 nt"
                     :
                     : "v"(off), "s"(base), "s"(lds_dst)
                     : "m0");
    else
        asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                     :
                     : "v"(off), "s"(base), "s"(lds_dst)
                     : "m0");
}
__device__ __forceinline__ void wait_loads_to_lds() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// Wavefront `wave` brings its KV block (keys wave*16 .. wave*16+15 of the 64-key tile, block base
// in n.gk / n.gv) of both operands into LDS buffer `bufi`: NL loads per operand, lane l of load i
// serving row i*RPL + l/CPR of the block at chunk position l % CPR (the swizzles are in
// n.koff / n.voff).  keys_valid counts the keys of the tile that lie inside the item's range:
// rows at or past it (all rows if !have_block) are not loaded; the V rows among them are zeroed
// instead (their scores are masked, but 0 * NaN would poison the PV product), the K rows may hold
// anything.  Nothing is waited for here.
// Rows from new_from on (tile row index; none by default) come from n.nk / n.nv instead.
template <int D, int WAVES = kWaves>
__device__ __forceinline__ void tile_load(const TileNext<D, WAVES> &n, uint32_t buf_off, bool have_block, int32_t keys_valid,
                                          int wave, int lane, int32_t new_from = 0x7FFFFFFF)
{
    using C = TileCfg<D, WAVES>;
    typedef __attribute__((address_space(3))) u32x4 lds_u32x4;
#pragma unroll
    for (int i = 0; i < C::NL; ++i) {
        const int row = wave * C::KPW + i * C::RPL + lane / C::CPR;   // row inside the tile
        const uint32_t dst = n.lds_w + buf_off + i * C::RPL * C::ROW;
        if (row < keys_valid && row >= new_from) {
            const uint32_t extra = (uint32_t)(row % kPage) * n.new_extra;
            load_to_lds_16(n.nk, n.koff[i] + extra, dst, false);
            load_to_lds_16(n.nv, n.voff[i] + extra, dst + C::K_BYTES, false);
        } else if (have_block && row < keys_valid) {
            load_to_lds_16(n.gk, n.koff[i], dst, n.stream);
            load_to_lds_16(n.gv, n.voff[i], dst + C::K_BYTES, n.stream);
        } else {
            *reinterpret_cast<lds_u32x4 *>(static_cast<uintptr_t>(dst + C::K_BYTES + lane * 16)) = u32x4{0u, 0u, 0u, 0u};
        }
    }
}

// The V operand is read with hand-placed instructions and waits.  The compiler makes every LDS read
// it knows about wait for all outstanding direct-to-LDS loads, which would stall each step half
// way through on the loads of the NEXT step (they target the other buffer and are published by
// the barrier at the end of the step).  An asm read is outside that rule; in exchange the waits
// for the reads themselves are ours: LDS reads return in order, so once at most N operations are
// outstanding, every read but the last N issued has landed.
template <int OFF>
__device__ __forceinline__ u32x2 lds_read_tr16(uint32_t addr)
{
    u32x2 r;
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(r) : "v"(addr), "n"(OFF));
    return r;
}

template <int DB>
struct VGroup {
    u32x2 lo[DB], hi[DB];   // keys base..base+3 (+4*half) and base+8.. of d = 32*db + col
};

// 16 keys (group G of the 64-key tile) of V^T for all DB row blocks: 2*DB reads in flight.
template <int D, int G, int BUFI>
__device__ __forceinline__ void v_issue(VGroup<TileCfg<D>::DB> &g, const uint32_t (&vaddr)[TileCfg<D>::DB])
{
    using C = TileCfg<D>;
    constexpr int BASE = BUFI * (C::K_BYTES + C::V_BYTES) + C::K_BYTES;   // V tile of buffer BUFI
    static_assert(BASE + (3 * 16 + 8) * C::ROW < 65536, "must fit the instruction's offset field");
#pragma unroll
    for (int db = 0; db < C::DB; ++db) {
        g.lo[db] = lds_read_tr16<BASE + G * 16 * C::ROW>(vaddr[db]);
        g.hi[db] = lds_read_tr16<BASE + (G * 16 + 8) * C::ROW>(vaddr[db]);
    }
}

// Waits until at most N LDS operations are outstanding; the registers of `g` are operands so
// that nothing using them can be scheduled above the wait.
template <int N>
__device__ __forceinline__ void v_wait(VGroup<4> &g)
{
    asm volatile("s_waitcnt lgkmcnt(%[n])"
                 : "+v"(g.lo[0]), "+v"(g.lo[1]), "+v"(g.lo[2]), "+v"(g.lo[3]), "+v"(g.hi[0]), "+v"(g.hi[1]),
                   "+v"(g.hi[2]), "+v"(g.hi[3])
                 : [n] "n"(N));
}
template <int N>
__device__ __forceinline__ void v_wait(VGroup<2> &g)
{
    asm volatile("s_waitcnt lgkmcnt(%[n])"
                 : "+v"(g.lo[0]), "+v"(g.lo[1]), "+v"(g.hi[0]), "+v"(g.hi[1])
                 : [n] "n"(N));
}

template <class E, int D>
__device__ __forceinline__ void pv_group(f32x16 (&o)[TileCfg<D>::DB], const VGroup<TileCfg<D>::DB> &g, typename E::x8 pf)
{
#pragma unroll
    for (int db = 0; db < TileCfg<D>::DB; ++db) {
        const u32x4 both = {g.lo[db].x, g.lo[db].y, g.hi[db].x, g.hi[db].y};
        o[db] = E::mfma(__builtin_bit_cast(typename E::x8, both), pf, o[db]);
    }
}

// K fragments are read the same way (hand-placed, waited for by count).
template <int OFF>
__device__ __forceinline__ u32x4 lds_read_b128(uint32_t addr)
{
    u32x4 r;
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(r) : "v"(addr), "n"(OFF));
    return r;
}
template <int N>
__device__ __forceinline__ void k_wait(u32x4 &f)
{
    asm volatile("s_waitcnt lgkmcnt(%[n])" : "+v"(f) : [n] "n"(N));
}

// One step of the matrix-core body for one wavefront: S^T = K Q^T over 64 keys, online softmax,
// O^T += V^T P^T, from LDS buffer BUFI.  `masked` steps (wavefront-uniform) apply the causal limit
// `pos` of the lane's row.  kaddr/vaddr are the lane's LDS addresses in buffer 0 (loop-invariant:
// the buffer and the key group enter as instruction offsets); with LOAD_NEXT the wavefront's
// share of the next step goes into the other buffer along the way.
//
// The 64 keys are handled as two halves of 32 whose phases overlap inside the wavefront, because
// a wavefront issues in order and a run of matrix instructions holds back the vector
// instructions written behind it: the weights of half 0 are computed between the QK
// instructions of half 1, those of half 1 between the PV instructions of half 0.
//
// Issue priority: a wavefront raises its priority from phase to phase of the step (0 for the
// first score product up to 3 for the last output product) and drops it again at the end.  Of the
// two wavefronts that share a SIMD the one further into its step then wins the issue slots, so the
// two fall out of phase with each other -- one runs matrix instructions while the other computes
// weights -- instead of both wanting the same pipe (measured: +5 to 6 % on prompt chunks; any
// two-level scheme does about as well, equal priority in both halves does nothing).
//
// Softmax reference: weights are 2^(c2*(s - m)) for a per-row reference m that is some earlier
// score of the row, not necessarily its maximum -- any reference gives the same result after
// the final division as long as nothing overflows, and one that was once the row's maximum
// cannot make the leading terms underflow.  So no maximum is taken in the common case: the
// weights are computed against the current m, and only if a lane's partial row sum comes out
// above 2^64 (or m is still unset) does the wavefront take the row maxima, raise m, rescale l
// and O, and recompute the weights of that half.
template <class E, int D, bool LOAD_NEXT, int BUFI, int WAVES = kWaves>
__device__ __forceinline__ void tile_compute(const uint32_t (&kaddr)[TileCfg<D>::KS],
                                             const uint32_t (&vaddr)[TileCfg<D>::DB],
                                             const typename E::x8 (&qf)[TileCfg<D>::KS], f32x16 (&o)[TileCfg<D>::DB],
                                             float &m, float &l, float c2, int32_t k0, int32_t pos, int half,
                                             bool masked, const TileNext<D, WAVES> &next)
{
    using C = TileCfg<D, WAVES>;
    typedef typename E::x2 ex2;
    typedef typename E::x8 ex8;
    constexpr int BUF = C::K_BYTES + C::V_BYTES;
    constexpr int KB0 = BUFI * BUF;                 // K tile of this buffer
    constexpr int PER = 2 * C::DB;                  // LDS reads per V group
    static_assert(KB0 + 32 * C::ROW < 65536 && 2 * C::KS <= 16, "offset field, outstanding-read counter");

    // Load i (of NL) of tile_load into the other LDS buffer, for a block that lies entirely
    // inside the item's key range.
    auto load_part = [&](int i) {
        const uint32_t dst = next.lds_w + (BUFI ^ 1) * BUF + i * C::RPL * C::ROW;
        load_to_lds_16(next.gk, next.koff[i], dst, false);     // (items that stream do not load from in here)
        load_to_lds_16(next.gv, next.voff[i], dst + C::K_BYTES, false);
    };
    auto mask_half = [&](f32x16 &sv, int kb) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int32_t key = k0 + kb * 32 + (v >> 2) * 8 + half * 4 + (v & 3);
            if (key > pos) sv[v] = -INFINITY;
        }
    };
    // Weights j (two scores) of one half: rounded to bf16 in the B-operand layout of the PV
    // product; their sum is taken from the rounded values (the very ones the product uses, so
    // numerator and denominator stay consistent).
    const ex2 ones = E::ones2();
    auto weight_pair = [&](const f32x16 &sv, ex8 (&pf)[2], float mc, float &sum, int j) {
        const ex2 pr = E::weights2(fast_exp2(fmaf(sv[2 * j], c2, -mc)), fast_exp2(fmaf(sv[2 * j + 1], c2, -mc)));
        pf[j >> 2][(2 * j) & 7] = pr[0];
        pf[j >> 2][(2 * j + 1) & 7] = pr[1];
        sum = E::dot2(pr, ones, sum);
    };
    // exponent of the weights' reference for a row whose reference score is mref
    auto ref_exp = [&](float mref) { return fmaf(mref, c2, -E::kRefShift); };
    // After the weights of a half: is the reference still good for every row of the wavefront?
    auto settle = [&](const f32x16 &sv, ex8 (&pf)[2], float sum_a, float sum_b) {
        float lh = sum_a + sum_b;
        const bool redo = !(lh <= E::kWeightCap) || m == -INFINITY;     // also catches inf and NaN
        if (__builtin_amdgcn_ballot_w64(redo) != 0) {
            float mt = sv[0];
#pragma unroll
            for (int v = 1; v < 16; ++v) mt = fmaxf(mt, sv[v]);
            {   // lane l <-> lane l ^ 32 without going through LDS
                const uint32_t mi = __float_as_uint(mt);
                auto sw = __builtin_amdgcn_permlane32_swap(mi, mi, false, false);
                mt = fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));
            }
            const float m_new = fmaxf(m, mt);
            const float m_fin = (m_new == -INFINITY) ? 0.f : m_new;   // row without a visible key so far
            const float alpha = fast_exp2((m - m_fin) * c2);
            l *= alpha;
#pragma unroll
            for (int db = 0; db < C::DB; ++db)
#pragma unroll
                for (int v = 0; v < 16; ++v) o[db][v] *= alpha;
            m = m_new;
            const float mc = ref_exp(m_fin);
            float ra = 0.f, rb = 0.f;
#pragma unroll
            for (int j = 0; j < 8; ++j) weight_pair(sv, pf, mc, (j & 1) ? rb : ra, j);
            lh = ra + rb;
        }
        l += lh;
    };

    // ---- K fragments of half 0 (those of half 1 follow once these registers are being consumed)
    u32x4 kf[2][C::KS];
#pragma unroll
    for (int ks = 0; ks < C::KS; ++ks) kf[0][ks] = lds_read_b128<KB0>(kaddr[ks]);

    // ---- S0 = K0 Q^T (keys 0..31), with the next step's loads between the instructions
    f32x16 s0, s1;
#pragma unroll
    for (int v = 0; v < 16; ++v) s0[v] = s1[v] = 0.f;
#pragma unroll
    for (int ks = 0; ks < C::KS; ++ks) {
        if (ks == 0) k_wait<C::KS - 1>(kf[0][0]);
        else if (ks == 1) k_wait<C::KS - 2>(kf[0][1]);
        else if (ks == 2) k_wait<C::KS - 3>(kf[0][2]);
        else if (ks == 3) k_wait<C::KS - 4>(kf[0][3]);
        else if (ks == 4) k_wait<(C::KS - 5 < 0 ? 0 : C::KS - 5)>(kf[0][4 % C::KS]);
        else if (ks == 5) k_wait<(C::KS - 6 < 0 ? 0 : C::KS - 6)>(kf[0][5 % C::KS]);
        else if (ks == 6) k_wait<(C::KS - 7 < 0 ? 0 : C::KS - 7)>(kf[0][6 % C::KS]);
        else k_wait<0>(kf[0][7 % C::KS]);
        s0 = E::mfma(__builtin_bit_cast(ex8, kf[0][ks]), qf[ks], s0);
        if (LOAD_NEXT && ks % (C::KS / C::NL) == 0) load_part(ks / (C::KS / C::NL));
    }
#pragma unroll
    for (int ks = 0; ks < C::KS; ++ks) kf[1][ks] = lds_read_b128<KB0 + 32 * C::ROW>(kaddr[ks]);
    VGroup<C::DB> g0, g1, g2, g3;
    v_issue<D, 0, BUFI>(g0, vaddr);
    if (masked) mask_half(s0, 0);

    // ---- S1 = K1 Q^T (keys 32..63) with the weights of half 0
    __builtin_amdgcn_s_setprio(1);
    k_wait<PER>(kf[1][C::KS - 1]);   // only the V reads may still be under way
    ex8 pf0[2], pf1[2];
    {
        const float mc = (m == -INFINITY) ? 0.f : ref_exp(m);
        float sum_a = 0.f, sum_b = 0.f;
#pragma unroll
        for (int ks = 0; ks < C::KS; ++ks) {
            s1 = E::mfma(__builtin_bit_cast(ex8, kf[1][ks]), qf[ks], s1);
#pragma unroll
            for (int j = ks * 8 / C::KS; j < (ks + 1) * 8 / C::KS; ++j) weight_pair(s0, pf0, mc, (j & 1) ? sum_b : sum_a, j);
        }
        v_issue<D, 1, BUFI>(g1, vaddr);
        settle(s0, pf0, sum_a, sum_b);
    }
    if (masked) mask_half(s1, 1);

    // ---- O^T += V0^T P0^T with the weights of half 1
    __builtin_amdgcn_s_setprio(2);
    {
        const float mc = (m == -INFINITY) ? 0.f : ref_exp(m);
        float sum_a = 0.f, sum_b = 0.f;
        v_wait<PER>(g0);
        pv_group<E, D>(o, g0, pf0[0]);
        v_issue<D, 2, BUFI>(g2, vaddr);
#pragma unroll
        for (int j = 0; j < 4; ++j) weight_pair(s1, pf1, mc, (j & 1) ? sum_b : sum_a, j);
        v_wait<PER>(g1);
        pv_group<E, D>(o, g1, pf0[1]);
        v_issue<D, 3, BUFI>(g3, vaddr);
#pragma unroll
        for (int j = 4; j < 8; ++j) weight_pair(s1, pf1, mc, (j & 1) ? sum_b : sum_a, j);
        settle(s1, pf1, sum_a, sum_b);
    }

    // ---- O^T += V1^T P1^T
    __builtin_amdgcn_s_setprio(3);
    v_wait<PER>(g2);
    pv_group<E, D>(o, g2, pf1[0]);
    v_wait<0>(g3);
    pv_group<E, D>(o, g3, pf1[1]);
    __builtin_amdgcn_s_setprio(0);
}

// Pacing of a team (see TeamRef): every kPaceEvery steps wavefront 0 publishes the work-group's
// progress and reads the team's; a member more than kPaceGap steps ahead of a running team mate
// that is still within kPaceFar steps (pacing keeps a bunch together, it does not wait for one
// that started later or fell far behind: the wait would cost more than the shared fetches save) pauses
// for one to three steps' time, the longer the further ahead it is -- a bounded pause, so a mate
// that never advances (not resident, or stuck behind us in a queue) costs time, not progress.
// The other wavefronts are held by the step's barrier.
constexpr int kPaceEvery = 4;
constexpr uint32_t kPaceGap = 6;
constexpr uint32_t kPaceFar = 14;

__device__ __forceinline__ uint32_t progress_load(const uint32_t *w)
{
    return __hip_atomic_load(w, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void progress_store(uint32_t *w, uint32_t v)
{
    __hip_atomic_store(w, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// `head` is the query head of a tile item (its rows are consecutive tokens), or the first query
// head of the group of a group item (its rows are the group's heads, all at the token q_row0):
// row r of the item is row (q_row0 * H + head) + r * rstride of q / out seen as [T * H, D], and
// likewise in the partial buffers.
// FUSED: the launch also appends (AttnParams::k_new); without it none of that code is compiled in.
template <class E, int D, int WAVES, bool FUSED>
__device__ __forceinline__ void tile_body(const AttnParams &p, const WorkItem &it, const TeamRef &team, int head,
                                          char *lds)
{
    using C = TileCfg<D, WAVES>;
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int half = lane >> 5;
    const int col = lane & 31;
    const int H = p.heads;
    const bool grouped = (it.kind & 0xFF) == kGroupItem;       // uniform
    const int rows = grouped ? p.group : it.q_rows;
    const int rstride = grouped ? 1 : H;
    const int kv_head = head / p.group;

    // this lane's query row
    const int r_tile = wave * 32 + col;
    const int r_eff = min(r_tile, rows - 1);
    const int32_t pos = grouped ? it.q_pos0 : it.q_pos0 + r_eff;
    typename E::x8 qf[C::KS];
    {
        const uint16_t *qrow = p.q + ((size_t)it.q_row0 * H + head + (size_t)r_eff * rstride) * D + half * 8;
#pragma unroll
        for (int ks = 0; ks < C::KS; ++ks) qf[ks] = *reinterpret_cast<const typename E::x8 *>(qrow + ks * 16);
    }
    const float c2 = p.scale_log2e;
    float m = -INFINITY, l = 0.f;
    f32x16 o[C::DB];
#pragma unroll
    for (int db = 0; db < C::DB; ++db)
#pragma unroll
        for (int v = 0; v < 16; ++v) o[db][v] = 0.f;

    const int32_t *tab = p.block_table + (size_t)it.seq * p.table_stride;
    // a wavefront without rows of its own only helps to load (its limits make every step inactive)
    const bool has_rows = wave * 32 < rows;
    const int32_t wave_first_pos = grouped ? it.q_pos0 : it.q_pos0 + min(wave * 32, rows - 1);
    const int32_t wave_last_pos = !has_rows ? -1 : grouped ? it.q_pos0 : it.q_pos0 + min(wave * 32 + 31, rows - 1);

    // Block-table entries of this wavefront's blocks for 64 steps at a time, one per lane.
    const int32_t nsteps = (it.kv_end - it.kv_begin + kKvTile - 1) / kKvTile;
    const int32_t npages_item = (it.kv_end - it.kv_begin + kPage - 1) / kPage;
    const int32_t page0 = it.kv_begin / kPage;
    auto load_entries = [&](int32_t step0) {   // page word of this wavefront's page in step step0 + lane
        const int32_t b = (step0 + lane) * (kKvTile / kPage) + wave * C::KPW / kPage;
        return (b < npages_item) ? page_word(tab, page0 + b, p.page_shift) : -1;
    };
    int32_t entries = load_entries(0);

    // (pacing exists for work-groups of four wavefronts only)
    uint32_t *const pace = (WAVES == kWaves && team.base >= 0) ? p.progress + team.base + (size_t)head * team.stride : nullptr;
    if (pace && threadIdx.x == 0) progress_store(pace + team.member, 0u);

    auto step_block = [&](int32_t step) {
        if ((step & 63) == 0 && step > 0) entries = load_entries(step);
        return __builtin_amdgcn_readlane(entries, step & 63);
    };
    // Loop-invariant addresses.  K: chunk 2*ks + half of row (kb*32 +) col sits at chunk position
    // (2*ks + half) ^ (col mod CPR).  V: the lane's source row inside a 16-key group is
    // 4*half + s16/4 (+8), which fixes its swizzle term; it supplies the address of d0 + 4*(s16%4) + 32*db.
    const uint32_t lds0 = static_cast<uint32_t>(reinterpret_cast<uintptr_t>(lds));
    uint32_t kaddr[C::KS], vaddr[C::DB];
#pragma unroll
    for (int ks = 0; ks < C::KS; ++ks)
        kaddr[ks] = lds0 + col * C::ROW + (((2 * ks + half) ^ (col & (C::CPR - 1))) * 16);
    {
        const int s16 = col & 15, d0 = (col >> 4) * 16;
        const int vswz = C::VSW * ((s16 >> 2) & 3);
        const int vchunk = (2 * d0) / 16 + ((s16 & 3) >> 1);
#pragma unroll
        for (int db = 0; db < C::DB; ++db)
            vaddr[db] = lds0 + (half * 4 + (s16 >> 2)) * C::ROW + 8 * (s16 & 1) + (((vchunk + 4 * db) ^ vswz) * 16);
    }
    TileNext<D, WAVES> next;
    {
        const int cpos = lane % C::CPR, r_in = lane / C::CPR;
#pragma unroll
        for (int i = 0; i < C::NL; ++i) {
            const int row = wave * C::KPW + i * C::RPL + r_in, row_b = row % kPage;   // in the tile, in its page
            next.koff[i] = row_b * C::ROW + ((cpos ^ (row & (C::CPR - 1))) * 16);
            next.voff[i] = row_b * C::ROW + ((cpos ^ (C::VSW * (row & 3))) * 16);
        }
        next.lds_w = __builtin_amdgcn_readfirstlane(lds0 + wave * C::KPW * C::ROW);
        next.gk = next.gv = nullptr;
        next.stream = grouped || (it.kind & kSoloTile) != 0;
        next.nk = next.nv = nullptr;
        next.new_extra = (uint32_t)(p.kv_heads * D * 2 - C::ROW);
    }
    // Append inside the launch: the keys from position new_begin of this sequence on -- the chunk's own
    // tokens, a generation row's own token -- are not in the cache yet and are loaded from k_new / v_new,
    // where position pos is row q_row0 + (pos - q_pos0).  A wavefront's rows of a tile lie in one page;
    // point_new aims nk / nv at where that page would start in the new rows (before their first row if
    // the page begins with old keys: those lanes do not load from there).
    const int32_t new_begin = !FUSED ? 0x7FFFFFFF : grouped ? it.q_pos0 : it.q_pos0 - (it.kind >> kTileRowShift);
    const int32_t wave_row0 = __builtin_amdgcn_readfirstlane(wave * C::KPW);
    auto point_new = [&](int32_t k0_tile) {
        const int64_t row = (int64_t)it.q_row0 + ((int64_t)k0_tile + (wave_row0 & ~(kPage - 1)) - it.q_pos0);
        const int64_t bytes = (row * p.kv_heads + kv_head) * (int64_t)(D * 2);
        const uint64_t ak = reinterpret_cast<uint64_t>(p.k_new) + (uint64_t)bytes, av = reinterpret_cast<uint64_t>(p.v_new) + (uint64_t)bytes;
        // (wavefront-uniform by construction; the intrinsic returns a signed int: widen its bits, not its value)
        auto uniform64 = [](uint64_t a) {
            const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((uint32_t)a);
            const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((uint32_t)(a >> 32));
            return ((uint64_t)hi << 32) | (uint64_t)lo;
        };
        next.nk = reinterpret_cast<const char *>(uniform64(ak));
        next.nv = reinterpret_cast<const char *>(uniform64(av));
    };
    // does the wavefront's share of the tile that starts at key k0_tile reach new keys?
    auto reaches_new = [&](int32_t k0_tile) { return FUSED && k0_tile + wave_row0 + C::KPW > new_begin; };

    // Pipeline: while step s is computed from LDS buffer s&1, the direct loads of step s+1 fill the
    // other buffer.  That buffer was last read in step s-1, which every wavefront has left, and the
    // barrier at the end of step s (which waits for this wavefront's loads first) publishes it.
    // The loop is written out for both buffers so that the buffer is an instruction offset.
    auto point_at = [&](int32_t blk) {   // the wavefront's block of the next load
        const size_t tile = page_offset<D>(blk < 0 ? 0 : blk, p.kv_heads, kv_head, p.page_shift);
        next.gk = reinterpret_cast<const char *>(p.k_cache + tile);
        next.gv = reinterpret_cast<const char *>(p.v_cache + tile);
    };
    constexpr uint32_t kBuf = C::K_BYTES + C::V_BYTES;
    if constexpr (WAVES == kWaves) {
        const int32_t blk0 = step_block(0);
        point_at(blk0);
        if (reaches_new(it.kv_begin)) {
            point_new(it.kv_begin);
            tile_load<D, WAVES>(next, 0, blk0 >= 0, it.kv_end - it.kv_begin, wave, lane, new_begin - it.kv_begin);
        } else {
            tile_load<D, WAVES>(next, 0, blk0 >= 0, it.kv_end - it.kv_begin, wave, lane);
        }
    } else {
        // ring: the tiles of the first kRingAhead steps
#pragma unroll
        for (int t = 0; t < kRingAhead; ++t) {
            if (t < nsteps) {
                const int32_t blk = step_block(t);
                point_at(blk);
                const int32_t k0_t = it.kv_begin + t * kKvTile;
                if (reaches_new(k0_t)) {
                    point_new(k0_t);
                    tile_load<D, WAVES>(next, t * kBuf, blk >= 0, it.kv_end - k0_t, wave, lane, new_begin - k0_t);
                } else {
                    tile_load<D, WAVES>(next, t * kBuf, blk >= 0, it.kv_end - k0_t, wave, lane);
                }
            }
        }
    }
    wait_loads_to_lds();
    // Everything the compiler loaded from memory for this item (Q fragments, table entries) is
    // consumed once here, so that its waits for those loads sit here and not at their first use
    // inside the step loop: there a vmcnt wait would also wait for the hand-issued loads of the
    // next step, which the compiler does not count, and serialise them with the products.
#pragma unroll
    for (int ks = 0; ks < C::KS; ++ks) asm volatile("" : "+v"(qf[ks]));
    asm volatile("" : "+v"(entries));
    __syncthreads();
    auto do_step = [&](int32_t step, auto bufi) {
        constexpr int BUFI = decltype(bufi)::value;
        const int32_t k0 = it.kv_begin + step * kKvTile;
        const bool more = step + 1 < nsteps;
        const int32_t blk_n = more ? step_block(step + 1) : -1;
        const int32_t keys_n = it.kv_end - (k0 + kKvTile);
        // otherwise every key of the step is above all rows of this wavefront
        const bool active = k0 <= wave_last_pos;
        const bool masked = k0 + kKvTile - 1 > wave_first_pos;
        const bool pace_now = pace && (step % kPaceEvery) == kPaceEvery - 1;   // uniform
        uint32_t mates = kNotRunning;
        if (pace_now && wave == 0) {
            if (lane == 0) progress_store(pace + team.member, (uint32_t)step + 1u);
            if (lane < team.size) mates = progress_load(pace + lane);
        }
        if (more) point_at(blk_n);
        const bool new_n = more && reaches_new(k0 + kKvTile);
        if (active && blk_n >= 0 && keys_n >= kKvTile && !next.stream && !new_n) {
            tile_compute<E, D, true, BUFI>(kaddr, vaddr, qf, o, m, l, c2, k0, pos, half, masked, next);
        } else {
            if (new_n) {
                point_new(k0 + kKvTile);
                tile_load<D, WAVES>(next, (BUFI ^ 1) * kBuf, blk_n >= 0, keys_n, wave, lane, new_begin - (k0 + kKvTile));
            } else if (more) {
                tile_load<D, WAVES>(next, (BUFI ^ 1) * kBuf, blk_n >= 0, keys_n, wave, lane);
            }
            if (active) tile_compute<E, D, false, BUFI>(kaddr, vaddr, qf, o, m, l, c2, k0, pos, half, masked, next);
        }
        wait_loads_to_lds();
        if (pace_now && wave == 0) {
            asm volatile("" : "+v"(mates));   // use it only here, where all loads have landed anyway
            const uint32_t mine = (uint32_t)step + 1u;
            const uint32_t ahead = (mates != kNotRunning && mates < mine && mates + kPaceFar >= mine) ? mine - mates : 0u;
            // pause in proportion to the lead: about one step's time (s_sleep counts in units of 64
            // cycles) for each kPaceGap/2 steps beyond the gap; straight-line code on purpose (a
            // loop here costs the register allocator of the whole kernel 20 registers)
            if (__builtin_amdgcn_ballot_w64(ahead > kPaceGap) != 0) __builtin_amdgcn_s_sleep(48);
            if (__builtin_amdgcn_ballot_w64(ahead > kPaceGap + kPaceGap / 2) != 0) __builtin_amdgcn_s_sleep(48);
            if (__builtin_amdgcn_ballot_w64(ahead > 2 * kPaceGap) != 0) __builtin_amdgcn_s_sleep(48);
        }
        __syncthreads();
    };
    if constexpr (WAVES == kWaves) {
        for (int32_t step = 0; step < nsteps; step += 2) {
            do_step(step, std::integral_constant<int, 0>());
            if (step + 1 < nsteps) do_step(step + 1, std::integral_constant<int, 1>());
        }
    } else {
        // Ring of kRingBufs tiles.  During step s the loads of step s + kRingAhead are issued (their
        // buffer held step s + kRingAhead - kRingBufs, which every wavefront left before the last
        // barrier); the wavefronts meet every kRingBarrier steps, after each has waited for its loads of
        // the steps up to the next meeting, so between two barriers they may be a step apart.  Buffers
        // are addressed through registers here (one loop body, the ring position is a scalar).
        constexpr int kLoadsPerStep = 2 * C::NL;
        const uint32_t lds_w0 = next.lds_w;
        uint32_t ring_s = 0, ring_t = (kRingAhead % kRingBufs) * kBuf;   // byte offsets of the tiles of steps s and s + kRingAhead
        for (int32_t step = 0; step < nsteps; ++step) {
            const int32_t k0 = it.kv_begin + step * kKvTile;
            const int32_t t = step + kRingAhead;
            const bool more = t < nsteps;
            const int32_t blk_t = more ? step_block(t) : -1;
            const int32_t keys_t = it.kv_end - (it.kv_begin + t * kKvTile);
            const bool active = k0 <= wave_last_pos;
            const bool masked = k0 + kKvTile - 1 > wave_first_pos;
            uint32_t ka[C::KS], va[C::DB];
#pragma unroll
            for (int ks = 0; ks < C::KS; ++ks) ka[ks] = kaddr[ks] + ring_s;
#pragma unroll
            for (int db = 0; db < C::DB; ++db) va[db] = vaddr[db] + ring_s;
            if (more) point_at(blk_t);
            const int32_t k0_t = it.kv_begin + t * kKvTile;
            const bool new_t = more && reaches_new(k0_t);
            if (active && more && blk_t >= 0 && keys_t >= kKvTile && !next.stream && !new_t) {
                next.lds_w = lds_w0 + ring_t - kBuf;   // tile_compute aims at "the other buffer" of buffer 0
                tile_compute<E, D, true, 0, WAVES>(ka, va, qf, o, m, l, c2, k0, pos, half, masked, next);
            } else {
                next.lds_w = lds_w0;
                if (new_t) {
                    point_new(k0_t);
                    tile_load<D, WAVES>(next, ring_t, blk_t >= 0, keys_t, wave, lane, new_begin - k0_t);
                } else if (more) {
                    tile_load<D, WAVES>(next, ring_t, blk_t >= 0, keys_t, wave, lane);
                }
                if (active) tile_compute<E, D, false, 0, WAVES>(ka, va, qf, o, m, l, c2, k0, pos, half, masked, next);
            }
            ring_s = ring_s + kBuf == kRingBufs * kBuf ? 0u : ring_s + kBuf;
            ring_t = ring_t + kBuf == kRingBufs * kBuf ? 0u : ring_t + kBuf;
            if (step % kRingBarrier == kRingBarrier - 1 && step + 1 < nsteps) {
                // Landed must be everything up to step + kRingBarrier; the loads of the steps behind that
                // may stay in flight -- counted on only while those steps are whole tiles (the last step
                // of a range may be a partial tile with fewer loads).
                if (step + kRingAhead < nsteps - 1)
                    asm volatile("s_waitcnt vmcnt(%0)" : : "n"(kLoadsPerStep * (kRingAhead - kRingBarrier)) : "memory");
                else
                    wait_loads_to_lds();
                __syncthreads();
            }
        }
    }

    if (pace && threadIdx.x == 0) progress_store(pace + team.member, kNotRunning);

    const float l_tot = l + __shfl_xor(l, 32);
    {
        // The lane's row and output addresses are worked out afresh from the thread index (made opaque,
        // so that nothing computed before the loop is kept alive through it for this).
        uint32_t tid = threadIdx.x;
        asm volatile("" : "+v"(tid));
        const int half = (tid >> 5) & 1;
        const int r_tile = (int)(tid >> 6) * 32 + (int)(tid & 31);
        int32_t kind = it.kind;
        asm volatile("" : "+s"(kind));
        const bool grouped = (kind & 0xFF) == kGroupItem;
        const int rows = grouped ? p.group : it.q_rows;
        const int rstride = grouped ? 1 : H;
        if (r_tile < rows) {
            if (it.part_row < 0) {
                const float inv = 1.f / l_tot;
                uint16_t *orow = p.out + ((size_t)it.q_row0 * H + head + (size_t)r_tile * rstride) * D;
#pragma unroll
                for (int db = 0; db < C::DB; ++db)
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        u32x2 w = {E::pack(o[db][4 * g] * inv, o[db][4 * g + 1] * inv),
                                   E::pack(o[db][4 * g + 2] * inv, o[db][4 * g + 3] * inv)};
                        *reinterpret_cast<u32x2 *>(orow + db * 32 + g * 8 + half * 4) = w;
                    }
            } else {
                const size_t prow = (size_t)it.part_row * H + head + (size_t)r_tile * rstride;
                float *arow = p.part_acc + prow * D;
#pragma unroll
                for (int db = 0; db < C::DB; ++db)
#pragma unroll
                    for (int g = 0; g < 4; ++g)
                        *reinterpret_cast<float4 *>(arow + db * 32 + g * 8 + half * 4) =
                            make_float4(o[db][4 * g], o[db][4 * g + 1], o[db][4 * g + 2], o[db][4 * g + 3]);
                if (half == 0) *reinterpret_cast<float2 *>(p.part_ml + prow * 2) = make_float2(fmaf(m, c2, -E::kRefShift), l_tot);
            }
        }
    }
}

// The item is the same for every lane: keep its fields in scalar registers.
__device__ __forceinline__ WorkItem load_item(const WorkItem *src)
{
    WorkItem it;
    it.seq = __builtin_amdgcn_readfirstlane(src->seq);
    it.q_row0 = __builtin_amdgcn_readfirstlane(src->q_row0);
    it.q_rows = __builtin_amdgcn_readfirstlane(src->q_rows);
    it.q_pos0 = __builtin_amdgcn_readfirstlane(src->q_pos0);
    it.kv_begin = __builtin_amdgcn_readfirstlane(src->kv_begin);
    it.kv_end = __builtin_amdgcn_readfirstlane(src->kv_end);
    it.part_row = __builtin_amdgcn_readfirstlane(src->part_row);
    it.kind = __builtin_amdgcn_readfirstlane(src->kind);
    return it;
}

// ------------------------------------------------------------------------------------------
// Unified kernel: the first n_tile_wgs work-groups walk the prompt tiles' units (a tile for one
// head), each taking every n_tile_wgs-th; then one work-group per group item (a generation row of
// grouped K/V heads, on the matrix-core body as well); the rest run row items (one wavefront per
// head, kWaves consecutive heads per work-group).
// ------------------------------------------------------------------------------------------
constexpr int kXcds = 8;   // accelerator dies of the chip, each with its own L2

template <class E, int D, int WAVES, bool FUSED>
__global__ void __launch_bounds__(WAVES * 64, 8 / WAVES)
attention_kernel(const AttnParams p)
{
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int H = p.heads;
    const int32_t n_tile_wg = p.n_tile_wgs;
    // K/V tiles of the matrix-core body (the kernel's LDS is allocated for every work-group alike):
    // two buffers for work-groups of four wavefronts, the ring for wide ones
    __shared__ __attribute__((aligned(16))) char lds[(WAVES == kWaves ? 2 : kRingBufs) * (TileCfg<D>::K_BYTES + TileCfg<D>::V_BYTES)];
    if ((int32_t)blockIdx.x < n_tile_wg) {
        // Tile units (item, head) are dealt round-robin to the tile work-groups.  With as many
        // work-groups as units each takes one; with fewer (mixed batches: part of the resident
        // slots, so that generation rows stream through the others from the start) each
        // walks its share, longest units first.
        // Launch order inside a run of tiles that read the same keys (see TeamRef: member, size):
        // eight heads at a time, the run's tiles of one head kXcds positions apart -- so the
        // tiles that share K/V run at the same time, on one XCD, whatever the number of
        // work-groups (in plain item order a run spans size * H units and its late members
        // find the K/V gone from L2: measured 2.1 x the K/V bytes from HBM on a 12-head layer).  The
        // heads left over when H is not a multiple of kXcds follow tile by tile, H mod kXcds positions
        // apart (their tiles land on 8 / gcd XCDs; padding them to eight positions instead, so that
        // they too share one XCD, unbalances the XCDs by more than the fetches saved are worth).
        const int32_t n_tile_units = p.n_tile_items * H;   // the launcher checks that this fits
        for (int32_t u = (int32_t)blockIdx.x; u < n_tile_units; u += n_tile_wg) {
            int32_t item = u / H, j;
            {
                const int32_t m = __builtin_amdgcn_readfirstlane(p.teams[item].member);
                const int32_t size = __builtin_amdgcn_readfirstlane(p.teams[item].size);
                const int32_t first = item - m, v = u - first * H;          // v in [0, size * H)
                const int32_t full = H / kXcds * kXcds * size;              // units of the whole groups of eight heads
                if (v < full) {
                    const int32_t block = v / (kXcds * size), within = v % (kXcds * size);
                    item = first + within / kXcds;
                    j = block * kXcds + within % kXcds;
                } else {
                    const int32_t r = H % kXcds, w = v - full;
                    item = first + w / r;
                    j = H - r + w % r;
                }
            }
            const WorkItem it = load_item(p.items + item);
            // Query heads that share a K/V head read the same K/V tiles: their units are placed
            // kXcds launch positions apart, i.e. on the same XCD (work-groups go to the XCDs in
            // turn), so that one L2 serves the group instead of one fetch from memory per head.
            // Position j of an item is head (j mod kXcds) * (H / kXcds) + j / kXcds.
            const int head = (p.group > 1 && H % kXcds == 0) ? (j % kXcds) * (H / kXcds) + j / kXcds : j;
            TeamRef team;
            team.base = __builtin_amdgcn_readfirstlane(p.teams[item].base);
            team.member = __builtin_amdgcn_readfirstlane(p.teams[item].member);
            team.size = __builtin_amdgcn_readfirstlane(p.teams[item].size);
            team.stride = __builtin_amdgcn_readfirstlane(p.teams[item].stride);
            tile_body<E, D, WAVES, FUSED>(p, it, team, head, lds);
            __syncthreads();   // the next unit's first loads overwrite the tile buffers
        }
        return;
    }
    if ((int32_t)blockIdx.x < n_tile_wg + p.n_group_items) {
        // a group item (a generation row of grouped K/V heads) names its K/V head; one work-group each
        const WorkItem it = load_item(p.items + p.n_tile_items + ((int32_t)blockIdx.x - n_tile_wg));
        const TeamRef team = {-1, 0, 1, 0};
        tile_body<E, D, WAVES, FUSED>(p, it, team, (it.kind >> 8) * p.group, lds);
        return;
    }
    const int hg = (H + WAVES - 1) / WAVES;
    int32_t idx = (int32_t)blockIdx.x - n_tile_wg - p.n_group_items;
    if (FUSED && idx < p.n_append_wgs) {
        // The iteration's append (see AttnParams::k_new): nothing in this launch reads these slots.  Ahead
        // of the rows in launch order, so that it runs beside them and not as a tail behind them.
        append_body((int64_t)idx * (WAVES * 64) + threadIdx.x, reinterpret_cast<const uint4 *>(p.k_new),
                    reinterpret_cast<const uint4 *>(p.v_new), p.slot_map, p.n_new, p.kv_heads, D / 8, p.block_size,
                    reinterpret_cast<uint4 *>(const_cast<uint16_t *>(p.k_cache)),
                    reinterpret_cast<uint4 *>(const_cast<uint16_t *>(p.v_cache)));
        return;
    }
    if (FUSED) idx -= p.n_append_wgs;
    const int32_t item = p.n_tile_items + p.n_group_items + idx / hg;
    const int head = (idx % hg) * WAVES + wave;
    if (head >= H) return;
    const WorkItem it = load_item(p.items + item);
    row_body<E, D, kRowSets, FUSED>(p, it, head, lane);
}

// ------------------------------------------------------------------------------------------
// Merge: one wavefront per (merge row, head).
// ------------------------------------------------------------------------------------------
template <class E, int D>
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
        *reinterpret_cast<uint32_t *>(o) = E::pack(acc[0] * inv, acc[EPL - 1] * inv);
    } else {
        *o = (uint16_t)(E::pack(acc[0] * inv, 0.f) & 0xFFFFu);
    }
}

// ------------------------------------------------------------------------------------------
// Scratch memory of the entry point that allocates nothing (mpa_mixed_paged_attention_static):
// what the other entry points take as the caller's workspace -- the work list and the partial
// results of split key ranges -- lives in this array instead.  Every GPU the library runs on holds
// its own copy, at its own address, until the process ends.  In host code the array's name is only
// a handle for hipGetSymbolAddress: kernels get the address that call returns.
// ------------------------------------------------------------------------------------------
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

// The work list reaches the scratch array as kernel arguments, kListChunkBytes at a time: no
// staging memory on either side, nothing for the host to keep alive after the launch call.
struct ListChunk {
    u32x4 v[kListChunkBytes / 16];
};
static_assert(sizeof(ListChunk) + 16 <= 4096, "kernel arguments are limited to 4 KiB");

__global__ void __launch_bounds__(256)
list_chunk_kernel(const ListChunk chunk, u32x4 *__restrict__ dst, int32_t n)
{
    if ((int32_t)threadIdx.x < n) dst[threadIdx.x] = chunk.v[threadIdx.x];
}
static_assert(kListChunkBytes / 16 <= 256, "one thread per 16 bytes");

}  // namespace

int static_scratch(void **ptr)
{
    constexpr int kMaxDevices = 64;
    static std::mutex mu;
    static void *ptrs[kMaxDevices] = {};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return (int)e;
    if (dev < 0 || dev >= kMaxDevices) return (int)hipErrorInvalidDevice;
    std::lock_guard<std::mutex> g(mu);
    if (!ptrs[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));   // the current device's copy of the array
        if (e != hipSuccess) return (int)e;
        if (!p) return (int)hipErrorInvalidSymbol;
        ptrs[dev] = p;
    }
    *ptr = ptrs[dev];
    return 0;
}

int launch_list_chunks(const void *host_src, void *dst, size_t bytes, void *stream)
{
    const char *src = static_cast<const char *>(host_src);
    char *d = static_cast<char *>(dst);
    for (size_t off = 0; off < bytes; off += kListChunkBytes) {
        const size_t n = bytes - off < (size_t)kListChunkBytes ? bytes - off : (size_t)kListChunkBytes;   // a multiple of 16
        ListChunk c;
        std::memcpy(c.v, src + off, n);
        hipLaunchKernelGGL(list_chunk_kernel, dim3(1), dim3(256), 0, (hipStream_t)stream, c,
                           reinterpret_cast<u32x4 *>(d + off), (int32_t)(n / 16));
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return (int)e;
    }
    return 0;
}

int launch_kv_append(const void *k_new, const void *v_new, const int64_t *slot_map, int32_t T,
                     int32_t H, int32_t D, int32_t block_size, void *k_cache, void *v_cache, void *stream)
{
    const int32_t vec_per_row = D / 8;
    const int64_t total = (int64_t)T * H * vec_per_row;
    if (total == 0) return 0;
    const int64_t blocks = (total + 255) / 256;
    hipLaunchKernelGGL(kv_append_kernel, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream,
                       (const uint4 *)k_new, (const uint4 *)v_new, slot_map, T, H, vec_per_row, block_size,
                       (uint4 *)k_cache, (uint4 *)v_cache);
    return (int)hipGetLastError();
}

int launch_upload(const void *pinned_src, void *dst, size_t bytes, uint64_t *pinned_flag, uint64_t ticket, void *stream)
{
    const int64_t n = (int64_t)(bytes / 16);
    hipLaunchKernelGGL(upload_kernel, dim3(1), dim3(kUploadThreads), 0, (hipStream_t)stream,
                       (const u32x4 *)pinned_src, (u32x4 *)dst, n, pinned_flag, ticket);
    return (int)hipGetLastError();
}

int launch_append_upload(const void *k_new, const void *v_new, const int64_t *slot_map, int32_t T, int32_t H, int32_t D,
                         int32_t block_size, void *k_cache, void *v_cache, const void *pinned_src, void *dst,
                         size_t bytes, uint64_t *pinned_flag, uint64_t ticket, void *stream)
{
    const int32_t vec_per_row = D / 8;
    const int64_t total = (int64_t)T * H * vec_per_row;
    const int64_t blocks = 1 + (total + 255) / 256;
    if (blocks > 0x7FFFFFFF) return (int)hipErrorInvalidConfiguration;
    hipLaunchKernelGGL(append_upload_kernel, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream,
                       (const uint4 *)k_new, (const uint4 *)v_new, slot_map, T, H, vec_per_row, block_size,
                       (uint4 *)k_cache, (uint4 *)v_cache, (const u32x4 *)pinned_src, (u32x4 *)dst, (int64_t)(bytes / 16),
                       pinned_flag, ticket);
    return (int)hipGetLastError();
}

int launch_copy_blocks(const void *src_k, const void *src_v, void *dst_k, void *dst_v, const int64_t *pairs,
                       int32_t n, int64_t block_bytes, void *stream)
{
    if (n == 0) return 0;
    const int64_t vec_per_block = block_bytes / 16;
    const int64_t gx = (vec_per_block + 1023) / 1024;
    if (gx > 0x7FFFFFFF || n > 65535) return (int)hipErrorInvalidConfiguration;
    hipLaunchKernelGGL(copy_blocks_kernel, dim3((unsigned)gx, (unsigned)n), dim3(256), 0, (hipStream_t)stream,
                       (const u32x4 *)src_k, (const u32x4 *)src_v, (u32x4 *)dst_k, (u32x4 *)dst_v, pairs, vec_per_block);
    return (int)hipGetLastError();
}

template <bool FUSED>
static void (*pick_kernel(bool wide, bool fp16, int32_t D))(const AttnParams)
{
    if (wide)
        return fp16 ? (D == 128 ? attention_kernel<Fp16, 128, kWideWaves, FUSED> : attention_kernel<Fp16, 64, kWideWaves, FUSED>)
                    : (D == 128 ? attention_kernel<Bf16, 128, kWideWaves, FUSED> : attention_kernel<Bf16, 64, kWideWaves, FUSED>);
    return fp16 ? (D == 128 ? attention_kernel<Fp16, 128, kWaves, FUSED> : attention_kernel<Fp16, 64, kWaves, FUSED>)
                : (D == 128 ? attention_kernel<Bf16, 128, kWaves, FUSED> : attention_kernel<Bf16, 64, kWaves, FUSED>);
}

int launch_attention(const AttnParams &params, int32_t D, bool fp16, void *stream)
{
    AttnParams p = params;
    const int waves = p.wide ? kWideWaves : kWaves;
    const int hg = (p.heads + waves - 1) / waves;
    const int64_t row_wgs = (int64_t)p.n_row_items * hg;
    // the append's work-groups: one thread per 16 bytes of K (and of V) of the new rows
    const int64_t append_wgs = p.k_new ? ((int64_t)p.n_new * p.kv_heads * (D / 8) + waves * 64 - 1) / (waves * 64) : 0;
    const int64_t grid = (int64_t)p.n_tile_wgs + p.n_group_items + row_wgs + append_wgs;
    if (grid == 0) return 0;
    const int64_t units = (int64_t)p.n_tile_items * p.heads + p.n_group_items;
    if (grid > 0x7FFFFFFF || units > 0x7FFFFFFF || row_wgs > 0x7FFFFFFF) return (int)hipErrorInvalidConfiguration;
    p.n_append_wgs = (int32_t)append_wgs;
    void (*kernel)(const AttnParams) = p.k_new ? pick_kernel<true>(p.wide != 0, fp16, D) : pick_kernel<false>(p.wide != 0, fp16, D);
    hipLaunchKernelGGL(kernel, dim3((unsigned)grid), dim3(waves * 64), 0, (hipStream_t)stream, p);
    return (int)hipGetLastError();
}

int launch_merge(const AttnParams &p, int32_t D, bool fp16, void *stream)
{
    const int64_t units = (int64_t)p.n_merge * p.heads;
    if (units == 0) return 0;
    const int64_t grid = (units + 3) / 4;
    void (*kernel)(const AttnParams) =
        fp16 ? (D == 128 ? merge_kernel<Fp16, 128> : merge_kernel<Fp16, 64>)
             : (D == 128 ? merge_kernel<Bf16, 128> : merge_kernel<Bf16, 64>);
    hipLaunchKernelGGL(kernel, dim3((unsigned)grid), dim3(256), 0, (hipStream_t)stream, p);
    return (int)hipGetLastError();
}

}  // namespace mpa
