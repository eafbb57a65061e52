// HIP kernels of libooco for gfx950 (CDNA4, wave64): split-KV decode attention, prefill-chunk
// attention, split merge and KV block copy.
//
// Common scheme (decode and prefill): scores are computed TRANSPOSED, S^T[token][query column]
// = K · Q^T, and the output as O^T[dim][query column] = V^T · P^T.  A "query column" is a query
// head of the GQA group (decode) or a query row (prefill).  With the MFMA operand/result lane
// layouts this keeps one query column in one lane column for the whole kernel:
//   * the fp32 result of the first MFMA is, register for register, the B operand of the second
//     one (after bf16 rounding) -- no cross-lane movement of P;
//   * the softmax statistics (max, sum) and the accumulator rescale are per lane column;
//   * K tiles [hd/8][16][8] and V tiles [hd][16] of the paged cache are already in A-operand
//     order, so they go from global memory straight into MFMA source registers.
// Softmax runs in base 2: scores are multiplied by scale*log2(e) and exponentiated with
// v_exp_f32.  Masked scores are set to -inf by select; V values of slots past the end of a
// sequence are zeroed by select (those slots may hold NaN/Inf).
#include "ooco_internal.h"

namespace ooco {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

#define OOCO_DEV __device__ __forceinline__

OOCO_DEV uint32_t pack2_bf16(float a, float b)
{
    bf16x2 v = {(__bf16)a, (__bf16)b};   // round to nearest even
    return __builtin_bit_cast(uint32_t, v);
}

OOCO_DEV float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

OOCO_DEV float xor_max(float v, int mask) { return fmaxf(v, __shfl_xor(v, mask, 64)); }
OOCO_DEV float xor_sum(float v, int mask) { return v + __shfl_xor(v, mask, 64); }

// ------------------------------------------------------------------------------------------
// Decode: one wave per (work item, kv head).  The wave walks KV blocks [blk_begin, blk_end) of
// one sequence.  Per 16-token block:
//   S^T[16 tok][16 heads] = K[16 tok][hd] · Q^T[hd][16 heads]      (hd/32 x v_mfma_f32_16x16x32_bf16)
//   O^T[hd][16 heads]    += V^T[hd][16 tok] · P^T[16 tok][16 heads] (hd/16 x v_mfma_f32_16x16x16_bf16)
// Head columns >= g (the GQA group size) carry zeros.  Lane l = 16*kq + col:
//   K operand, chunk c:  16 B at tile offset (64c + l)*16          (token col, dims 32c+8kq..+8)
//   S^T result reg r:    token 4kq + r, head col
//   V operand, group nb: 8 B at tile offset ((16nb + col)*16 + 4kq)*2   (dim 16nb+col, tokens 4kq..+4)
//   O^T result reg r:    dim 16nb + 4kq + r, head col
// NBI blocks are processed per softmax step, and the loads of the next step are issued before
// the arithmetic of the current one (two register sets).
template <int HD, int NBI>
__global__ __launch_bounds__(64) void decode_kernel(const AttnParams p)
{
    constexpr int KC = HD / 32;
    constexpr int NB = HD / 16;
    const int lane = threadIdx.x;
    const int col = lane & 15;
    const int kq = lane >> 4;
    const int item_idx = blockIdx.x / p.Hkv;
    const int kvh = blockIdx.x - item_idx * p.Hkv;
    const DecodeItem it = p.ditems[item_idx];
    const int g = p.g;
    const int head = kvh * g + col;
    const int nblk = it.blk_end - it.blk_begin;
    const int niter = (nblk + NBI - 1) / NBI;

    // Q as B operand: head col, dims 32c + 8kq .. +8
    u32x4 qb[KC];
    {
        const u32x4 *qp = reinterpret_cast<const u32x4 *>(p.q + ((int64_t)it.q_row * p.Hq + (col < g ? head : 0)) * HD);
#pragma unroll
        for (int c = 0; c < KC; ++c) {
            u32x4 t = qp[c * 4 + kq];
            qb[c] = (col < g) ? t : u32x4{0u, 0u, 0u, 0u};
        }
    }

    // rolling window of 64 physical block ids, one per lane
    const int32_t *table = p.block_tables + (int64_t)it.seq * p.max_blocks_per_seq + it.blk_begin;
    int wbase = 0;
    int idv = table[min(lane, nblk - 1)];
    int idn = table[min(64 + lane, nblk - 1)];

    const int64_t tile_elems = (int64_t)HD * kBlockSize;   // one (block, kv head) tile
    struct KV {
        u32x4 k[NBI][KC];
        u32x2 v[NBI][NB];
    };

    auto load = [&](KV &t, int iter) {
        const int j0 = iter * NBI;
        if (j0 - wbase >= 64) {
            wbase += 64;
            idv = idn;
            idn = table[min(wbase + 64 + lane, nblk - 1)];
        }
#pragma unroll
        for (int u = 0; u < NBI; ++u) {
            const int j = min(j0 + u, nblk - 1);
            const int pb = __builtin_amdgcn_readlane(idv, j - wbase);
            const int64_t off = ((int64_t)pb * p.Hkv + kvh) * tile_elems;
            const u32x4 *kp = reinterpret_cast<const u32x4 *>(p.k_cache + off);
            const u32x2 *vp = reinterpret_cast<const u32x2 *>(p.v_cache + off);
#pragma unroll
            for (int c = 0; c < KC; ++c) t.k[u][c] = kp[c * 64 + lane];
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) t.v[u][nb] = vp[(nb * 16 + col) * 4 + kq];
        }
    };

    f32x4 O[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) O[nb] = f32x4{0.f, 0.f, 0.f, 0.f};
    float m = -INFINITY, lsum = 0.f;

    auto compute = [&](KV &t, int iter) {
        f32x4 S[NBI];
#pragma unroll
        for (int u = 0; u < NBI; ++u) {
            S[u] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int c = 0; c < KC; ++c)
                S[u] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, t.k[u][c]),
                                                               __builtin_bit_cast(bf16x8, qb[c]), S[u], 0, 0, 0);
        }
        float mloc = -INFINITY;
#pragma unroll
        for (int u = 0; u < NBI; ++u) {
            const int j = iter * NBI + u;
            int nvalid = it.seq_len - (it.blk_begin + j) * kBlockSize;
            nvalid = (j < nblk) ? nvalid : 0;
            if (nvalid < kBlockSize) {   // wave-uniform: tail block of the sequence, or past the item
#pragma unroll
                for (int r = 0; r < 4; ++r) S[u][r] = (4 * kq + r < nvalid) ? S[u][r] * p.scale_log2e : -INFINITY;
                const uint32_t m0 = (4 * kq + 0 < nvalid ? 0x0000FFFFu : 0u) | (4 * kq + 1 < nvalid ? 0xFFFF0000u : 0u);
                const uint32_t m1 = (4 * kq + 2 < nvalid ? 0x0000FFFFu : 0u) | (4 * kq + 3 < nvalid ? 0xFFFF0000u : 0u);
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) {
                    t.v[u][nb][0] &= m0;
                    t.v[u][nb][1] &= m1;
                }
            } else {
#pragma unroll
                for (int r = 0; r < 4; ++r) S[u][r] *= p.scale_log2e;
            }
#pragma unroll
            for (int r = 0; r < 4; ++r) mloc = fmaxf(mloc, S[u][r]);
        }
        mloc = xor_max(mloc, 16);
        mloc = xor_max(mloc, 32);
        const float m_new = fmaxf(m, mloc);
        const float alpha = fast_exp2(m - m_new);
        const bool grow = m_new > m;
        m = m_new;
        float psum = 0.f;
        s16x4 P[NBI];
#pragma unroll
        for (int u = 0; u < NBI; ++u) {
            float e[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                e[r] = fast_exp2(S[u][r] - m_new);
                psum += e[r];
            }
            u32x2 pk = {pack2_bf16(e[0], e[1]), pack2_bf16(e[2], e[3])};
            P[u] = __builtin_bit_cast(s16x4, pk);
        }
        lsum = lsum * alpha + psum;
        if (__any(grow)) {
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                for (int r = 0; r < 4; ++r) O[nb][r] *= alpha;
        }
#pragma unroll
        for (int u = 0; u < NBI; ++u)
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
                O[nb] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(s16x4, t.v[u][nb]), P[u], O[nb], 0, 0, 0);
    };

    KV A, B;
    load(A, 0);
    int i = 0;
    for (; i + 1 < niter; i += 2) {
        load(B, i + 1);
        compute(A, i);
        if (i + 2 < niter) load(A, i + 2);
        compute(B, i + 1);
    }
    if (i < niter) compute(A, i);

    float ltot = xor_sum(lsum, 16);
    ltot = xor_sum(ltot, 32);
    if (col < g) {
        if (it.part < 0) {
            const float inv = 1.0f / ltot;
            uint16_t *op = p.out + ((int64_t)it.q_row * p.Hq + head) * HD + 4 * kq;
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                u32x2 w = {pack2_bf16(O[nb][0] * inv, O[nb][1] * inv), pack2_bf16(O[nb][2] * inv, O[nb][3] * inv)};
                *reinterpret_cast<u32x2 *>(op + nb * 16) = w;
            }
        } else {
            float *ap = p.part_acc + ((int64_t)it.part * p.Hq + head) * HD + 4 * kq;
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) *reinterpret_cast<f32x4 *>(ap + nb * 16) = O[nb];
            if (kq == 0) {
                float *mp = p.part_ml + ((int64_t)it.part * p.Hq + head) * 2;
                mp[0] = m;
                mp[1] = ltot;
            }
        }
    }
}

// ------------------------------------------------------------------------------------------
// Merge of split-KV partials: out = sum_s acc_s 2^(m_s-M) / sum_s l_s 2^(m_s-M), M = max_s m_s.
// One wave per (sequence, query head); lane owns hd/64 consecutive dims.  Parts are visited in
// order, so the result does not depend on launch timing.
template <int HD>
__global__ __launch_bounds__(64) void merge_kernel(const AttnParams p)
{
    constexpr int PER = HD / 64;
    const int lane = threadIdx.x;
    const int mi = blockIdx.x / p.Hq;
    const int head = blockIdx.x - mi * p.Hq;
    const MergeItem it = p.mitems[mi];
    float M = -INFINITY;
    for (int s = 0; s < it.nparts; ++s) M = fmaxf(M, p.part_ml[((int64_t)(it.part0 + s) * p.Hq + head) * 2]);
    float L = 0.f;
    float acc[PER];
#pragma unroll
    for (int d = 0; d < PER; ++d) acc[d] = 0.f;
    for (int s = 0; s < it.nparts; ++s) {
        const int64_t row = (int64_t)(it.part0 + s) * p.Hq + head;
        const float w = fast_exp2(p.part_ml[row * 2] - M);
        L += p.part_ml[row * 2 + 1] * w;
        const float *ap = p.part_acc + row * HD + lane * PER;
#pragma unroll
        for (int d = 0; d < PER; ++d) acc[d] += ap[d] * w;
    }
    const float inv = 1.0f / L;
    uint16_t *op = p.out + ((int64_t)it.q_row * p.Hq + head) * HD + lane * PER;
    if constexpr (PER == 2) {
        *reinterpret_cast<uint32_t *>(op) = pack2_bf16(acc[0] * inv, acc[1] * inv);
    } else {
        const uint32_t w = pack2_bf16(acc[0] * inv, 0.f);
        op[0] = (uint16_t)(w & 0xFFFFu);
    }
}

// ------------------------------------------------------------------------------------------
// Prefill chunk, simple form: one wave per (tile of 32 query rows, query head); K/V operands
// come straight from global memory (L2) in operand order, two KV blocks (32 tokens) per step:
//   S^T[32 tok][32 rows] = K · Q^T    (hd/16 x v_mfma_f32_32x32x16_bf16)
//   O^T[hd][32 rows]    += V^T · P^T  (hd/32 x 2 x v_mfma_f32_32x32x16_bf16)
// Lane l = 32*h + col.  MFMA row i of the K operand is fed with token (i with bits 2 and 3
// swapped) of its block, so that S^T register r of lane (col, h) is token 16(r/8) + 8h + r%8 of
// the pair: eight consecutive tokens per block, which is what one 16-byte V operand load holds.
template <int HD>
__global__ __launch_bounds__(64) void prefill_kernel(const AttnParams p)
{
    constexpr int KS = HD / 16;   // k-steps of QK
    constexpr int MB = HD / 32;   // 32-dim groups of the output
    const int lane = threadIdx.x;
    const int col = lane & 31;
    const int h = lane >> 5;
    const int tile_idx = blockIdx.x / p.Hq;
    const int head = blockIdx.x - tile_idx * p.Hq;
    const PrefillTile tl = p.ptiles[tile_idx];
    const int kvh = head / p.g;
    const int row = min(col, tl.rows - 1);
    const int pos = tl.pos0 + row;                       // this lane column's absolute position
    const int kv_end = tl.pos0 + tl.rows;                // keys visible to the tile: [0, kv_end)
    const int nblk = (kv_end + kBlockSize - 1) / kBlockSize;
    const int npair = (nblk + 1) / 2;

    u32x4 qb[KS];
    {
        const u32x4 *qp = reinterpret_cast<const u32x4 *>(p.q + ((int64_t)(tl.q_row0 + row) * p.Hq + head) * HD);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) qb[ks] = qp[2 * ks + h];
    }
    const int32_t *table = p.block_tables + (int64_t)tl.seq * p.max_blocks_per_seq;
    const int64_t tile_elems = (int64_t)HD * kBlockSize;
    // K operand row col -> block (col>>4) of the pair, slot with bits 2,3 of (col&15) swapped
    const int ku = col >> 4;
    const int kslot = (col & 3) | ((col & 4) << 1) | ((col & 8) >> 1);

    f32x16 O[MB];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int r = 0; r < 16; ++r) O[mb][r] = 0.f;
    float m = -INFINITY, lsum = 0.f;

    for (int pr = 0; pr < npair; ++pr) {
        const int b0 = 2 * pr, b1 = min(2 * pr + 1, nblk - 1);
        const int pb0 = table[b0], pb1 = table[b1];
        const int64_t offk = ((int64_t)(ku ? pb1 : pb0) * p.Hkv + kvh) * tile_elems;
        const u32x4 *kp = reinterpret_cast<const u32x4 *>(p.k_cache + offk);
        u32x4 kreg[KS];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) kreg[ks] = kp[(2 * ks + h) * 16 + kslot];
        u32x4 vreg[2][MB];
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const u32x4 *vp = reinterpret_cast<const u32x4 *>(p.v_cache + ((int64_t)(u ? pb1 : pb0) * p.Hkv + kvh) * tile_elems);
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) vreg[u][mb] = vp[(mb * 32 + col) * 2 + h];
        }
        f32x16 S;
#pragma unroll
        for (int r = 0; r < 16; ++r) S[r] = 0.f;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
            S = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, kreg[ks]),
                                                        __builtin_bit_cast(bf16x8, qb[ks]), S, 0, 0, 0);
        const int tok0 = pr * 32 + 8 * h;                // token of register 0; register r: +16(r/8) + r%8
        const bool need_mask = (pr * 32 + 31 > tl.pos0) || (pr * 32 + 31 >= tl.seq_len);   // wave-uniform
        if (need_mask) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int tok = tok0 + 16 * (r / 8) + (r % 8);
                S[r] = (tok <= pos) ? S[r] * p.scale_log2e : -INFINITY;
            }
            // V slots at or past seq_len may hold anything: zero them (their P is 0, but 0*NaN is NaN)
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const int t0 = tok0 + 16 * u;            // tokens t0 .. t0+7 in this lane's V registers
                const bool whole = (u == 1 && 2 * pr + 1 >= nblk);   // the pair's second block does not exist
#pragma unroll
                for (int w = 0; w < 4; ++w) {
                    const uint32_t mk = ((!whole && t0 + 2 * w < tl.seq_len) ? 0x0000FFFFu : 0u) |
                                        ((!whole && t0 + 2 * w + 1 < tl.seq_len) ? 0xFFFF0000u : 0u);
#pragma unroll
                    for (int mb = 0; mb < MB; ++mb) vreg[u][mb][w] &= mk;
                }
            }
        } else {
#pragma unroll
            for (int r = 0; r < 16; ++r) S[r] *= p.scale_log2e;
        }
        float mloc = S[0];
#pragma unroll
        for (int r = 1; r < 16; ++r) mloc = fmaxf(mloc, S[r]);
        mloc = xor_max(mloc, 32);
        const float m_new = fmaxf(m, mloc);
        const float alpha = fast_exp2(m - m_new);
        const bool grow = m_new > m;
        m = m_new;
        float psum = 0.f;
        u32x4 P[2];
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            float e[8];
#pragma unroll
            for (int r = 0; r < 8; ++r) {
                e[r] = fast_exp2(S[8 * u + r] - m_new);
                psum += e[r];
            }
            P[u] = u32x4{pack2_bf16(e[0], e[1]), pack2_bf16(e[2], e[3]), pack2_bf16(e[4], e[5]), pack2_bf16(e[6], e[7])};
        }
        lsum = lsum * alpha + psum;
        if (__any(grow)) {
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                for (int r = 0; r < 16; ++r) O[mb][r] *= alpha;
        }
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
                O[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, vreg[u][mb]),
                                                            __builtin_bit_cast(bf16x8, P[u]), O[mb], 0, 0, 0);
    }
    const float ltot = xor_sum(lsum, 32);
    if (col < tl.rows) {
        const float inv = 1.0f / ltot;
        uint16_t *op = p.out + ((int64_t)(tl.q_row0 + col) * p.Hq + head) * HD + 4 * h;
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                // registers 4*q4 .. 4*q4+3: dims 32mb + 8*q4 + 4h + 0..3
                u32x2 w = {pack2_bf16(O[mb][4 * q4] * inv, O[mb][4 * q4 + 1] * inv),
                           pack2_bf16(O[mb][4 * q4 + 2] * inv, O[mb][4 * q4 + 3] * inv)};
                *reinterpret_cast<u32x2 *>(op + mb * 32 + q4 * 8) = w;
            }
    }
}

// ------------------------------------------------------------------------------------------
// KV block copy: workgroup (pair, which pool, slice) moves a contiguous slice of one block with
// 16-byte loads and stores; all loads of a thread are issued before its stores.
constexpr int kCopyThreads = 256;
constexpr int kCopyVecPerThread = 4;   // 256 threads x 4 x 16 B = 16 KiB per workgroup

__global__ __launch_bounds__(kCopyThreads) void block_copy_kernel(const u32x4 *k_src, const u32x4 *v_src, u32x4 *k_dst,
                                                                  u32x4 *v_dst, const int64_t *src_ids,
                                                                  const int64_t *dst_ids, int64_t block_vecs,
                                                                  int slices)
{
    const int64_t pair = blockIdx.x / (2 * slices);
    const int rem = blockIdx.x - pair * (2 * slices);
    const int which = rem / slices;
    const int slice = rem - which * slices;
    const int64_t sb = src_ids[pair], db = dst_ids[pair];
    const u32x4 *src = (which ? v_src : k_src) + sb * block_vecs;
    u32x4 *dst = (which ? v_dst : k_dst) + db * block_vecs;
    const int64_t base = (int64_t)slice * kCopyThreads * kCopyVecPerThread + threadIdx.x;
    u32x4 r[kCopyVecPerThread];
#pragma unroll
    for (int i = 0; i < kCopyVecPerThread; ++i) {
        const int64_t idx = base + (int64_t)i * kCopyThreads;
        if (idx < block_vecs) r[i] = __builtin_nontemporal_load(src + idx);
    }
#pragma unroll
    for (int i = 0; i < kCopyVecPerThread; ++i) {
        const int64_t idx = base + (int64_t)i * kCopyThreads;
        if (idx < block_vecs) __builtin_nontemporal_store(r[i], dst + idx);
    }
}

// ------------------------------------------------------------------------------------------
hipError_t launch_decode(const AttnParams &p, hipStream_t s)
{
    if (p.n_ditems == 0) return hipSuccess;
    const dim3 grid((unsigned)((int64_t)p.n_ditems * p.Hkv)), block(64);
    if (p.hd == 128)
        hipLaunchKernelGGL((decode_kernel<128, 2>), grid, block, 0, s, p);
    else
        hipLaunchKernelGGL((decode_kernel<64, 2>), grid, block, 0, s, p);
    return hipGetLastError();
}

hipError_t launch_prefill(const AttnParams &p, hipStream_t s)
{
    if (p.n_ptiles == 0) return hipSuccess;
    const dim3 grid((unsigned)((int64_t)p.n_ptiles * p.Hq)), block(64);
    if (p.hd == 128)
        hipLaunchKernelGGL((prefill_kernel<128>), grid, block, 0, s, p);
    else
        hipLaunchKernelGGL((prefill_kernel<64>), grid, block, 0, s, p);
    return hipGetLastError();
}

hipError_t launch_merge(const AttnParams &p, hipStream_t s)
{
    if (p.n_mitems == 0) return hipSuccess;
    const dim3 grid((unsigned)((int64_t)p.n_mitems * p.Hq)), block(64);
    if (p.hd == 128)
        hipLaunchKernelGGL((merge_kernel<128>), grid, block, 0, s, p);
    else
        hipLaunchKernelGGL((merge_kernel<64>), grid, block, 0, s, p);
    return hipGetLastError();
}

hipError_t launch_block_copy(const void *k_src, const void *v_src, void *k_dst, void *v_dst, const int64_t *src_ids,
                             const int64_t *dst_ids, int64_t num_pairs, int64_t block_bytes, hipStream_t s)
{
    if (num_pairs == 0) return hipSuccess;
    const int64_t block_vecs = block_bytes / 16;
    const int per_wg = kCopyThreads * kCopyVecPerThread;
    const int slices = (int)((block_vecs + per_wg - 1) / per_wg);
    const dim3 grid((unsigned)(num_pairs * 2 * slices)), block(kCopyThreads);
    hipLaunchKernelGGL(block_copy_kernel, grid, block, 0, s, (const u32x4 *)k_src, (const u32x4 *)v_src, (u32x4 *)k_dst,
                       (u32x4 *)v_dst, src_ids, dst_ids, block_vecs, slices);
    return hipGetLastError();
}

}  // namespace ooco
