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
// Matrix-core body: one work-group (4 wavefronts), one head, a tile of up to 128 query rows
// (32 per wavefront), a contiguous key range walked in steps of 64 keys.
//
// Per step the work-group stages K [64 keys][D] and V transposed [D][64 keys] in LDS.  Each
// wavefront computes S^T = K Q^T with 32x32x16 bf16 MFMAs (A = K rows from LDS, B = Q^T from
// registers), so a lane owns ONE query row (lane % 32) and 32 of the 64 keys: the row maximum
// and sum are in-lane reductions plus one exchange with lane ^ 32.  The exponentials, packed to
// bf16 in the very registers they were produced in, are the B operand of O^T += V^T P^T, whose
// result again has the query row on the lane, so the running rescale needs no cross-lane
// traffic either.
//
// Register layouts of v_mfma_f32_32x32x16_bf16 (lane l, half = l / 32):
//   A: row l % 32, k = 8*half .. 8*half+7        B: column l % 32, k = 8*half .. 8*half+7
//   C: column l % 32, rows 8*(v/4) + 4*half + v%4 for v = 0..15
// ------------------------------------------------------------------------------------------
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

template <int D>
struct TileCfg {
    static constexpr int KS = D / 16;                   // k-steps of K Q^T
    static constexpr int DB = D / 32;                   // 32-row blocks of O^T
    static constexpr int K_STRIDE = D * 2 + 16;         // bytes per key row of the K tile
    static constexpr int VT_STRIDE = kKvTile * 2 + 8;   // bytes per row of the V^T tile
    static constexpr int K_BYTES = kKvTile * K_STRIDE;
    static constexpr int VT_BYTES = D * VT_STRIDE;
    static constexpr int CPR = D / 8;                   // 16-byte chunks per key row
    static constexpr int KG = 64 / CPR;                 // key groups per wavefront (V loads)
    static constexpr int KPT = kBlockSize / KG;         // consecutive keys per thread (V loads)
    static constexpr int NL = KPT;                      // 16-byte loads per thread per operand
};

template <int D>
struct TileRegs {
    u32x4 k[TileCfg<D>::NL];
    u32x4 v[TileCfg<D>::NL];
};

// Wavefront `wave` fetches KV block (k0/16 + wave) of the step that starts at key k0.
template <int D>
__device__ __forceinline__ void tile_fetch(TileRegs<D> &r, const AttnParams &p, const int32_t *tab,
                                           int32_t k0, int32_t kv_end, int head, int wave, int lane)
{
    using C = TileCfg<D>;
    const int32_t kb0 = k0 + wave * kBlockSize;
    if (kb0 < kv_end) {
        const int32_t blk = __builtin_amdgcn_readfirstlane(tab[kb0 / kBlockSize]);
        const size_t tile = ((size_t)blk * p.heads + head) * (kBlockSize * D);
        const u32x4 *kp = reinterpret_cast<const u32x4 *>(p.k_cache + tile);
        const u32x4 *vp = reinterpret_cast<const u32x4 *>(p.v_cache + tile);
        const int c = lane % C::CPR, kg = lane / C::CPR;
#pragma unroll
        for (int i = 0; i < C::NL; ++i) r.k[i] = kp[i * 64 + lane];
#pragma unroll
        for (int i = 0; i < C::NL; ++i) {
            const int key = C::KPT * kg + i;
            u32x4 w = vp[key * C::CPR + c];
            // keys at or past kv_end may hold anything (also NaN): they must contribute exact zeros
            if (kb0 + key >= kv_end) w = u32x4{0u, 0u, 0u, 0u};
            r.v[i] = w;
        }
    } else {
#pragma unroll
        for (int i = 0; i < C::NL; ++i) {
            r.k[i] = u32x4{0u, 0u, 0u, 0u};
            r.v[i] = u32x4{0u, 0u, 0u, 0u};
        }
    }
}

template <int D>
__device__ __forceinline__ void tile_stage(const TileRegs<D> &r, char *lds_k, char *lds_vt, int wave, int lane)
{
    using C = TileCfg<D>;
    const int c = lane % C::CPR, kg = lane / C::CPR;
#pragma unroll
    for (int i = 0; i < C::NL; ++i) {
        const int j = i * 64 + lane;
        const int key = wave * kBlockSize + j / C::CPR;
        *reinterpret_cast<u32x4 *>(lds_k + key * C::K_STRIDE + (j % C::CPR) * 16) = r.k[i];
    }
    // transpose in registers: for each of this thread's 8 head-dim elements, the KPT keys
    const int col = (wave * kBlockSize + C::KPT * kg) * 2;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        auto elem = [&](int i) -> uint32_t {
            const uint32_t w = r.v[i][e >> 1];
            return (e & 1) ? (w >> 16) : (w & 0xFFFFu);
        };
        char *dst = lds_vt + (8 * c + e) * C::VT_STRIDE + col;
        if (C::KPT == 4) {
            u32x2 o = {elem(0) | (elem(1) << 16), elem(2) | (elem(3) << 16)};
            *reinterpret_cast<u32x2 *>(dst) = o;
        } else {
            *reinterpret_cast<uint32_t *>(dst) = elem(0) | (elem(1) << 16);
        }
    }
}

template <int D>
__device__ __forceinline__ void tile_body(const AttnParams &p, const WorkItem &it, int head, char *lds)
{
    using C = TileCfg<D>;
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int half = lane >> 5;
    const int col = lane & 31;
    const int H = p.heads;
    char *lds_k = lds;
    char *lds_vt = lds + C::K_BYTES;

    // this lane's query row
    const int r_tile = wave * 32 + col;
    const int r_eff = min(r_tile, it.q_rows - 1);
    const int32_t pos = it.q_pos0 + r_eff;
    bf16x8 qf[C::KS];
    {
        const uint16_t *qrow = p.q + ((size_t)(it.q_row0 + r_eff) * H + head) * D + half * 8;
#pragma unroll
        for (int ks = 0; ks < C::KS; ++ks) qf[ks] = *reinterpret_cast<const bf16x8 *>(qrow + ks * 16);
    }
    const float c2 = p.scale_log2e;
    float m = -INFINITY, l = 0.f;
    f32x16 o[C::DB];
#pragma unroll
    for (int db = 0; db < C::DB; ++db)
#pragma unroll
        for (int v = 0; v < 16; ++v) o[db][v] = 0.f;

    const int32_t *tab = p.block_table + (size_t)it.seq * p.table_stride;
    const int32_t wave_first_pos = it.q_pos0 + min(wave * 32, it.q_rows - 1);
    const int32_t wave_last_pos = it.q_pos0 + min(wave * 32 + 31, it.q_rows - 1);

    TileRegs<D> regs;
    tile_fetch<D>(regs, p, tab, it.kv_begin, it.kv_end, head, wave, lane);
    for (int32_t k0 = it.kv_begin; k0 < it.kv_end; k0 += kKvTile) {
        tile_stage<D>(regs, lds_k, lds_vt, wave, lane);
        __syncthreads();
        if (k0 + kKvTile < it.kv_end) tile_fetch<D>(regs, p, tab, k0 + kKvTile, it.kv_end, head, wave, lane);

        if (k0 <= wave_last_pos) {  // otherwise every key of the step is above all rows of this wavefront
            f32x16 s[2];
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int v = 0; v < 16; ++v) s[kb][v] = 0.f;
#pragma unroll
            for (int ks = 0; ks < C::KS; ++ks)
#pragma unroll
                for (int kb = 0; kb < 2; ++kb) {
                    const bf16x8 kf = *reinterpret_cast<const bf16x8 *>(
                        lds_k + (kb * 32 + col) * C::K_STRIDE + ks * 32 + half * 16);
                    s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks], s[kb], 0, 0, 0);
                }
            const bool masked = k0 + kKvTile - 1 > wave_first_pos;
            if (masked) {
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const int32_t key = k0 + kb * 32 + (v >> 2) * 8 + half * 4 + (v & 3);
                        if (key > pos) s[kb][v] = -INFINITY;
                    }
            }
            float mt = s[0][0];
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int v = 0; v < 16; ++v) mt = fmaxf(mt, s[kb][v]);
            mt = fmaxf(mt, __shfl_xor(mt, 32));
            const float m_new = fmaxf(m, mt);
            const float m_safe = (m_new == -INFINITY) ? 0.f : m_new;
            const float alpha = fast_exp2((m - m_safe) * c2);
            const float mc = m_safe * c2;
            m = m_new;
            float psum = 0.f;
            bf16x8 pf[2][2];
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const float pv = fast_exp2(fmaf(s[kb][v], c2, -mc));
                    psum += pv;
                    pf[kb][v >> 3][v & 7] = static_cast<__bf16>(pv);
                }
            l = fmaf(l, alpha, psum);
#pragma unroll
            for (int db = 0; db < C::DB; ++db)
#pragma unroll
                for (int v = 0; v < 16; ++v) o[db][v] *= alpha;
#pragma unroll
            for (int db = 0; db < C::DB; ++db)
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int st = 0; st < 2; ++st) {
                        const char *src = lds_vt + (db * 32 + col) * C::VT_STRIDE + (kb * 32 + st * 16 + half * 4) * 2;
                        const u32x2 lo = *reinterpret_cast<const u32x2 *>(src);
                        const u32x2 hi = *reinterpret_cast<const u32x2 *>(src + 16);
                        const u32x4 both = {lo.x, lo.y, hi.x, hi.y};
                        o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, both),
                                                                        pf[kb][st], o[db], 0, 0, 0);
                    }
        }
        __syncthreads();
    }

    const float l_tot = l + __shfl_xor(l, 32);
    if (r_tile < it.q_rows) {
        if (it.part_row < 0) {
            const float inv = 1.f / l_tot;
            uint16_t *orow = p.out + ((size_t)(it.q_row0 + r_tile) * H + head) * D;
#pragma unroll
            for (int db = 0; db < C::DB; ++db)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    u32x2 w = {pack_bf16(o[db][4 * g] * inv, o[db][4 * g + 1] * inv),
                               pack_bf16(o[db][4 * g + 2] * inv, o[db][4 * g + 3] * inv)};
                    *reinterpret_cast<u32x2 *>(orow + db * 32 + g * 8 + half * 4) = w;
                }
        } else {
            const size_t prow = (size_t)(it.part_row + r_tile) * H + head;
            float *arow = p.part_acc + prow * D;
#pragma unroll
            for (int db = 0; db < C::DB; ++db)
#pragma unroll
                for (int g = 0; g < 4; ++g)
                    *reinterpret_cast<float4 *>(arow + db * 32 + g * 8 + half * 4) =
                        make_float4(o[db][4 * g], o[db][4 * g + 1], o[db][4 * g + 2], o[db][4 * g + 3]);
            if (half == 0) *reinterpret_cast<float2 *>(p.part_ml + prow * 2) = make_float2(m * c2, l_tot);
        }
    }
}

// ------------------------------------------------------------------------------------------
// Unified kernel: work-groups [0, n_tile_items*H) run prompt tiles, the rest run row items
// (one wavefront per head, kWaves consecutive heads per work-group).
// ------------------------------------------------------------------------------------------
template <int D>
__global__ void __launch_bounds__(kThreads, 2)
attention_kernel(const AttnParams p)
{
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int H = p.heads;
    const int64_t n_tile_wg = (int64_t)p.n_tile_items * H;
    if ((int64_t)blockIdx.x < n_tile_wg) {
        __shared__ __attribute__((aligned(16))) char lds[TileCfg<D>::K_BYTES + TileCfg<D>::VT_BYTES];
        const int32_t item = (int32_t)(blockIdx.x / H);
        const int head = (int)(blockIdx.x % H);
        const WorkItem it = p.items[item];
        tile_body<D>(p, it, head, lds);
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
