// HIP kernels of libooco for gfx950 (CDNA4, wave64): split-KV decode attention with its in-kernel
// merge, prefill-chunk attention and KV block copy.
//
// Common scheme (decode and prefill): scores are computed TRANSPOSED, S^T[token][query column]
// = K · Q^T, and the output as O^T[dim][query column] = V^T · P^T.  A "query column" is a query
// head of the GQA group (decode) or a query row (prefill).  With the MFMA operand/result lane
// layouts this keeps one query column in one lane column for the whole kernel:
//   * the fp32 result of the first MFMA is, register for register, the B operand of the second
//     one (after bf16 rounding) -- no cross-lane movement of P;
//   * the softmax statistics (max, sum) and the accumulator rescale are per lane column;
//   * K tiles [hd/8][16][8] and V tiles [hd][16] of the paged cache are already in A-operand
//     order, so they go from global memory straight into MFMA source registers (decode) or are
//     copied unchanged into LDS by direct global->LDS loads and read from there (prefill).
// Softmax runs in base 2: scores are multiplied by scale*log2(e) and exponentiated with
// v_exp_f32.  Masked scores are set to -inf by select; V values of slots past the end of a
// sequence are zeroed by select (those slots may hold NaN/Inf).
#include "ooco_internal.h"

#include <algorithm>

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

// max of three without the NaN-quieting moves that fmaxf would add (one v_max3_f32)
OOCO_DEV float max3(float a, float b, float c)
{
    float d;
    asm("v_max3_f32 %0, %1, %2, %3" : "=v"(d) : "v"(a), "v"(b), "v"(c));
    return d;
}

// max of two / with a floor of -1e30, as single instructions (no NaN-quieting moves)
OOCO_DEV float max2(float a, float b)
{
    float d;
    asm("v_max_f32_e32 %0, %1, %2" : "=v"(d) : "v"(a), "v"(b));
    return d;
}
OOCO_DEV float floor_m1e30(float a)
{
    float d;
    asm("v_max_f32_e32 %0, 0xf149f2ca, %1" : "=v"(d) : "v"(a));   // 0xf149f2ca = -1e30f
    return d;
}
// max of the 32 scores a lane holds for one step (two 16-register MFMA results), as one dependent chain of
// v_max3_f32 in two asm statements (an asm statement takes at most 30 operands)
OOCO_DEV float max32(const f32x16 &a, const f32x16 &b)
{
    float d, e;
    asm("v_max3_f32 %0, %1, %2, %3\n\t"
        "v_max3_f32 %0, %0, %4, %5\n\t"
        "v_max3_f32 %0, %0, %6, %7\n\t"
        "v_max3_f32 %0, %0, %8, %9\n\t"
        "v_max3_f32 %0, %0, %10, %11\n\t"
        "v_max3_f32 %0, %0, %12, %13\n\t"
        "v_max3_f32 %0, %0, %14, %15\n\t"
        "v_max3_f32 %0, %0, %16, %17"
        : "=&v"(d)
        : "v"(a[0]), "v"(b[0]), "v"(a[1]), "v"(b[1]), "v"(a[2]), "v"(b[2]), "v"(a[3]), "v"(b[3]), "v"(a[4]), "v"(b[4]),
          "v"(a[5]), "v"(b[5]), "v"(a[6]), "v"(b[6]), "v"(a[7]), "v"(b[7]), "v"(a[8]));
    asm("v_max3_f32 %0, %1, %2, %3\n\t"
        "v_max3_f32 %0, %0, %4, %5\n\t"
        "v_max3_f32 %0, %0, %6, %7\n\t"
        "v_max3_f32 %0, %0, %8, %9\n\t"
        "v_max3_f32 %0, %0, %10, %11\n\t"
        "v_max3_f32 %0, %0, %12, %13\n\t"
        "v_max3_f32 %0, %0, %14, %15\n\t"
        "v_max_f32_e32 %0, %0, %16"
        : "=&v"(e)
        : "v"(d), "v"(b[8]), "v"(a[9]), "v"(b[9]), "v"(a[10]), "v"(b[10]), "v"(a[11]), "v"(b[11]), "v"(a[12]), "v"(b[12]),
          "v"(a[13]), "v"(b[13]), "v"(a[14]), "v"(b[14]), "v"(a[15]), "v"(b[15]));
    return e;
}

// acc + lo + hi of a packed bf16 pair (one v_dot2c_f32_bf16 against the pair (1, 1))
OOCO_DEV float sum2_bf16(uint32_t pair, float acc)
{
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, pair), __builtin_bit_cast(bf16x2, 0x3F803F80u), acc,
                                           false);
}

// Device-scope (all XCDs) relaxed store / load of one float: the store writes through to memory,
// the load bypasses the non-coherent cache levels.
typedef float f32x2 __attribute__((ext_vector_type(2)));
OOCO_DEV void store_dev2(float *ptr, float a, float b)   // ptr is 8-byte aligned
{
    const f32x2 v = {a, b};
    __hip_atomic_store(reinterpret_cast<uint64_t *>(ptr), __builtin_bit_cast(uint64_t, v), __ATOMIC_RELAXED,
                       __HIP_MEMORY_SCOPE_AGENT);
}
// The same cache policy for a 16-byte store (a plain vector store with the device-scope bit: the ordering
// against the arrival counter comes from s_waitcnt, 16-byte atomicity is not needed).  Far fewer memory
// operations than 8-byte atomic stores, which matters for the 64 KiB partial results of a prefill part.
// (The s_nop covers the wait states a wide store needs before its data registers may be overwritten, which
// the compiler cannot see through the asm.)
OOCO_DEV void store_dev4(float *ptr, f32x4 v)   // ptr is 16-byte aligned
{
    asm volatile("global_store_dwordx4 %0, %1, off sc1\n\ts_nop 1" ::"v"(ptr), "v"(v) : "memory");
}
// Device-scope 16-byte loads of one part of a split prefill tile as one lane sees it: four loads (1 KiB apart)
// from each of MB pointers.  All loads and the wait for them sit in ONE asm statement, so that the compiler
// never sees a register it believes loaded while the data is still on its way.
#define OOCO_LD4(o, a) \
    "global_load_dwordx4 %" #o ", %" #a ", off sc1\n\t"
#define OOCO_LD4O(o, a, off) \
    "global_load_dwordx4 %" #o ", %" #a ", off offset:" #off " sc1\n\t"
OOCO_DEV void load_dev_part(f32x4 (&t)[16], const float *p0, const float *p1, const float *p2, const float *p3)
{
    asm volatile(OOCO_LD4(0, 16) OOCO_LD4O(1, 16, 1024) OOCO_LD4O(2, 16, 2048) OOCO_LD4O(3, 16, 3072)
                 OOCO_LD4(4, 17) OOCO_LD4O(5, 17, 1024) OOCO_LD4O(6, 17, 2048) OOCO_LD4O(7, 17, 3072)
                 OOCO_LD4(8, 18) OOCO_LD4O(9, 18, 1024) OOCO_LD4O(10, 18, 2048) OOCO_LD4O(11, 18, 3072)
                 OOCO_LD4(12, 19) OOCO_LD4O(13, 19, 1024) OOCO_LD4O(14, 19, 2048) OOCO_LD4O(15, 19, 3072)
                 "s_waitcnt vmcnt(0)"
                 : "=&v"(t[0]), "=&v"(t[1]), "=&v"(t[2]), "=&v"(t[3]), "=&v"(t[4]), "=&v"(t[5]), "=&v"(t[6]), "=&v"(t[7]),
                   "=&v"(t[8]), "=&v"(t[9]), "=&v"(t[10]), "=&v"(t[11]), "=&v"(t[12]), "=&v"(t[13]), "=&v"(t[14]), "=&v"(t[15])
                 : "v"(p0), "v"(p1), "v"(p2), "v"(p3)
                 : "memory");
}
OOCO_DEV void load_dev_part(f32x4 (&t)[8], const float *p0, const float *p1)
{
    asm volatile(OOCO_LD4(0, 8) OOCO_LD4O(1, 8, 1024) OOCO_LD4O(2, 8, 2048) OOCO_LD4O(3, 8, 3072)
                 OOCO_LD4(4, 9) OOCO_LD4O(5, 9, 1024) OOCO_LD4O(6, 9, 2048) OOCO_LD4O(7, 9, 3072)
                 "s_waitcnt vmcnt(0)"
                 : "=&v"(t[0]), "=&v"(t[1]), "=&v"(t[2]), "=&v"(t[3]), "=&v"(t[4]), "=&v"(t[5]), "=&v"(t[6]), "=&v"(t[7])
                 : "v"(p0), "v"(p1)
                 : "memory");
}
#undef OOCO_LD4
#undef OOCO_LD4O
OOCO_DEV f32x2 load_dev2(const float *ptr)
{
    const uint64_t u = __hip_atomic_load(reinterpret_cast<uint64_t *>(const_cast<float *>(ptr)), __ATOMIC_RELAXED,
                                         __HIP_MEMORY_SCOPE_AGENT);
    return __builtin_bit_cast(f32x2, u);
}


// ------------------------------------------------------------------------------------------
// Cross-lane reductions over the four 16-lane rows of a wave with the CDNA4 lane-swap
// instructions (VALU only, no LDS traffic): v_permlane16_swap exchanges the odd rows of its first
// operand with the even rows of the second, v_permlane32_swap the upper half of the first with
// the lower half of the second; fed with two copies of one value they return both partners of
// an xor-16 / xor-32 butterfly.  (Vector elements are copied to scalars before
// __builtin_bit_cast: a bit_cast applied directly to an element reference reads element 0.)
OOCO_DEV void swap16(float v, float &lo, float &hi)
{
    const unsigned u = __builtin_bit_cast(unsigned, v);
    const auto a = __builtin_amdgcn_permlane16_swap(u, u, false, false);
    const unsigned a0 = a[0], a1 = a[1];
    lo = __builtin_bit_cast(float, a0);
    hi = __builtin_bit_cast(float, a1);
}
OOCO_DEV void swap32(float v, float &lo, float &hi)
{
    const unsigned u = __builtin_bit_cast(unsigned, v);
    const auto a = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    const unsigned a0 = a[0], a1 = a[1];
    lo = __builtin_bit_cast(float, a0);
    hi = __builtin_bit_cast(float, a1);
}
OOCO_DEV float rows_max(float v)
{
    float x, y;
    swap16(v, x, y);
    swap32(fmaxf(x, y), x, y);
    return fmaxf(x, y);
}
OOCO_DEV float rows_sum(float v)
{
    float x, y;
    swap16(v, x, y);
    swap32(x + y, x, y);
    return x + y;
}

// ------------------------------------------------------------------------------------------
// Work lookup shared by both kernels: cum[] is non-decreasing with cum[0] = 0; returns the number
// of entries j in [1, n] with cum[j] <= x, i.e. the index i with cum[i] <= x < cum[i+1].
// All 64 lanes of the wave must call it with the same x.
template <class CumAt>
OOCO_DEV int count_le(CumAt cum_at, int n, int x, int lane)
{
    int cnt = 0;
    for (int base = 1; base <= n; base += 64) {
        const int idx = base + lane;
        const int v = idx <= n ? cum_at(idx) : 0x7FFFFFFF;
        const int c = __popcll(__ballot(v <= x));
        cnt += c;
        if (c < 64) break;
    }
    return cnt;
}

// ------------------------------------------------------------------------------------------
// Decode: one wave per (run k of the decode block line, kv head).  A wave walks the pieces of its
// run one after the other; a piece is a range of KV blocks of one sequence.  Per 16-token block:
//   S^T[16 tok][16 heads] = K[16 tok][hd] · Q^T[hd][16 heads]      (hd/32 x v_mfma_f32_16x16x32_bf16)
//   O^T[hd][16 heads]    += V^T[hd][16 tok] · P^T[16 tok][16 heads] (hd/16 x v_mfma_f32_16x16x16_bf16)
// Head columns >= g (the GQA group size) carry zeros.  Lane l = 16*kq + col:
//   K operand, chunk c:  16 B at tile offset (64c + l)*16          (token col, dims 32c+8kq..+8)
//   S^T result reg r:    token 4kq + r, head col
//   V operand, group nb: 8 B at tile offset ((16nb + col)*16 + 4kq)*2   (dim 16nb+col, tokens 4kq..+4)
//   O^T result reg r:    dim 16nb + 4kq + r, head col
// One K and one V register set: the K loads of block j+1 are issued right after the QK MFMAs of
// block j have consumed the K registers, the V loads of block j+1 right after the PV MFMAs, so a
// wave always has one block's tiles (8 KiB with head_dim 128) on their way; a few such waves per
// compute unit keep HBM busy, and no second register set is needed.
//
// A piece that covers its whole sequence normalises and stores bf16 output.  Any other piece
// stores (acc, m, l) in fp32 into partial slot k + seq, then bumps the arrival counter of
// (seq, kv head); the piece that arrives last merges all slots of the sequence in slot order
// (so the result does not depend on which piece is last) and resets the counter.
// One run of the decode line for one kv head, all its pieces, executed by one wave (see above).
// `at_stream_end()` is called once the last piece of the run has been streamed, before its epilogue.
template <int HD, int NBI, int MBATCH, class CumAt, class AtStreamEnd>
OOCO_DEV void decode_run(const AttnParams &p, CumAt cum_at, const RunLayout &L, int run, int kvh, int lane, uint64_t *trace,
                         bool &first_piece, AtStreamEnd at_stream_end)
{
    constexpr int KC = HD / 32;
    constexpr int NB = HD / 16;
    const int col = lane & 15;
    const int kq = lane >> 4;
    const int g = p.g;
    const int64_t tile_elems = (int64_t)HD * kBlockSize;   // one (block, kv head) tile
    const int head = kvh * g + col;
    int lo, hi;
    run_bounds(L, run, lo, hi);
    int seq = count_le(cum_at, p.num_seqs, lo, lane);
    int pos = lo;
    while (pos < hi) {
        seq = __builtin_amdgcn_readfirstlane(seq);
        int cs = cum_at(seq), ce = cum_at(seq + 1);
        while (ce <= pos) {   // sequences without decode blocks
            ++seq;
            cs = ce;
            ce = cum_at(seq + 1);
        }
        const int stop = min(hi, ce);
        // the sequence's blocks start piece_pad units into its stretch of the line
        const int first = cs + p.piece_pad;
        const int begin = max(pos, first);
        if (begin >= stop) {   // the run ends before the first block of this sequence
            if (trace && lane == 0) trace[2] = wall_clock64();
            pos = stop;
            continue;
        }
        const int blk_begin = begin - first;
        const int nblk = stop - begin;
        const bool whole = (begin == first) && (stop == ce);
        const int seq_len = p.seq_lens[seq];
        const int q_row = min(max(p.query_start_loc[seq], 0), p.total_q - 1);

        // Q as B operand: head col, dims 32c + 8kq .. +8
        u32x4 qb[KC];
        {
            const u32x4 *qp = reinterpret_cast<const u32x4 *>(p.q + ((int64_t)q_row * p.Hq + (col < g ? head : 0)) * HD);
#pragma unroll
            for (int c = 0; c < KC; ++c) {
                u32x4 t = qp[c * 4 + kq];
                qb[c] = (col < g) ? t : u32x4{0u, 0u, 0u, 0u};
            }
        }
        // rolling window of 64 physical block ids, one per lane
        const int32_t *table = p.block_tables + (int64_t)seq * p.max_blocks_per_seq + blk_begin;
        int wbase = 0;
        int idv = table[min(lane, nblk - 1)];
        int idn = table[min(64 + lane, nblk - 1)];

        u32x4 kreg[NBI][KC];
        u32x2 vreg[NBI][NB];
        int64_t offs[NBI];
        auto tile_off = [&](int j) -> int64_t {   // j is wave-uniform and non-decreasing
            if (j - wbase >= 64) {
                wbase += 64;
                idv = idn;
                idn = table[min(wbase + 64 + lane, nblk - 1)];
            }
            const int pb = __builtin_amdgcn_readlane(idv, j - wbase);
            return ((int64_t)pb * p.Hkv + kvh) * tile_elems;
        };
        // K and V tiles are read once per kv head and never again in this launch: they are loaded with the
        // non-temporal policy (`nt`), so that the stream does not push other data out of the caches on its way
        // through them.  Measured on MI355X: 64 sequences 115.7 -> 103.3 us, 512 sequences 1.149 -> 1.030 ms
        // (6.1 -> 6.8 TB/s).
        // Loads are issued unconditionally (steps past the end re-read the last block, an L2 hit)
        // so that every step has the same number of loads in flight and the waits before the
        // MFMAs can leave the younger loads outstanding.
        auto issue_k = [&](int step) {
#pragma unroll
            for (int u = 0; u < NBI; ++u) {
                offs[u] = tile_off(min(step * NBI + u, nblk - 1));
                const u32x4 *kp = reinterpret_cast<const u32x4 *>(p.k_cache + offs[u]);
#pragma unroll
                for (int c = 0; c < KC; ++c) kreg[u][c] = __builtin_nontemporal_load(&kp[c * 64 + lane]);
            }
        };
        auto issue_v = [&]() {
#pragma unroll
            for (int u = 0; u < NBI; ++u) {
                const u32x2 *vp = reinterpret_cast<const u32x2 *>(p.v_cache + offs[u]);
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) vreg[u][nb] = __builtin_nontemporal_load(&vp[(nb * 16 + col) * 4 + kq]);
            }
        };

        f32x4 O[NB];
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) O[nb] = f32x4{0.f, 0.f, 0.f, 0.f};
        float m = -INFINITY, lsum = 0.f;

        const int nstep = (nblk + NBI - 1) / NBI;
        issue_k(0);
        issue_v();
        if (trace && first_piece) {   // time at which the first K/V tiles of the wave have arrived
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            if (lane == 0) trace[1] = wall_clock64();
            first_piece = false;
        }
        for (int t = 0; t < nstep; ++t) {
            f32x4 S[NBI];
#pragma unroll
            for (int u = 0; u < NBI; ++u) {
                S[u] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int c = 0; c < KC; ++c)
                    S[u] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kreg[u][c]),
                                                                   __builtin_bit_cast(bf16x8, qb[c]), S[u], 0, 0, 0);
            }
            issue_k(min(t + 1, nstep - 1));
            float mloc = -INFINITY;
#pragma unroll
            for (int u = 0; u < NBI; ++u) {
                const int j = t * NBI + u;
                int nvalid = seq_len - (blk_begin + j) * kBlockSize;
                if (NBI > 1 && j >= nblk) nvalid = 0;
                if (nvalid < kBlockSize) {   // wave-uniform: tail block of the sequence, or past the piece
#pragma unroll
                    for (int r = 0; r < 4; ++r) S[u][r] = (4 * kq + r < nvalid) ? S[u][r] * p.scale_log2e : -INFINITY;
                    const uint32_t m0 = (4 * kq + 0 < nvalid ? 0x0000FFFFu : 0u) | (4 * kq + 1 < nvalid ? 0xFFFF0000u : 0u);
                    const uint32_t m1 = (4 * kq + 2 < nvalid ? 0x0000FFFFu : 0u) | (4 * kq + 3 < nvalid ? 0xFFFF0000u : 0u);
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb) {
                        vreg[u][nb][0] &= m0;
                        vreg[u][nb][1] &= m1;
                    }
                } else {
#pragma unroll
                    for (int r = 0; r < 4; ++r) S[u][r] *= p.scale_log2e;
                }
                mloc = fmaxf(mloc, fmaxf(fmaxf(S[u][0], S[u][1]), fmaxf(S[u][2], S[u][3])));
            }
            mloc = rows_max(mloc);
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
                for (int r = 0; r < 4; ++r) e[r] = fast_exp2(S[u][r] - m_new);
                psum += (e[0] + e[1]) + (e[2] + e[3]);
                const u32x2 pk = {pack2_bf16(e[0], e[1]), pack2_bf16(e[2], e[3])};
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
                    O[nb] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(s16x4, vreg[u][nb]), P[u],
                                                                      O[nb], 0, 0, 0);
            issue_v();
        }

        if (trace && stop == hi && lane == 0) trace[2] = wall_clock64();   // end of streaming
        if (stop == hi) at_stream_end();
        float ltot = rows_sum(lsum);
        bool store_out = whole;
        if (!whole) {
            // ---- partial result into slot run + seq, then arrival count.  Partials are written
            // and read with device-scope accesses (write-through / L2-bypassing), so that pieces
            // running on other XCDs see them without any whole-cache write-back or invalidate.
            if (col < g) {
                const int64_t row = (int64_t)(run + seq) * p.Hq + head;
                float *ap = p.part_acc + row * HD + 4 * kq;
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) store_dev4(ap + nb * 16, O[nb]);
                if (kq == 0) store_dev2(p.part_ml + row * 2, m, ltot);
            }
            const int first_run = run_of(L, first);
            const int nparts = run_of(L, (int64_t)ce - 1) - first_run + 1;
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // the partial has reached memory before the count
            int prev = 0;
            if (lane == 0)
                prev = __hip_atomic_fetch_add(p.counters + (int64_t)seq * p.Hkv + kvh, 1, __ATOMIC_RELAXED,
                                              __HIP_MEMORY_SCOPE_AGENT);
            prev = __builtin_amdgcn_readfirstlane(prev);
            if (prev == nparts - 1) {   // last piece of this (sequence, kv head): merge, in slot order
                // The 16 lane columns hold only g heads, so 16/g (at most 4) groups of columns merge
                // different parts side by side: column group pg takes the parts pg, pg + ngrp, ...
                // (three at a time so that their memory round trips overlap); the groups' results
                // are then folded into group 0 in a fixed order.  Which parts meet in which order
                // depends only on the plan, never on which piece arrived last.
                // (only for sequences cut into many parts: below that one group is as fast and loads less)
                const int ngrp = nparts <= 2 * 3 ? 1 : (g <= 4 ? 4 : (g <= 8 ? 2 : 1));
                const int pg = col / g, hc = col - pg * g;
                const bool member = pg < ngrp;
                const int hm = kvh * g + (member ? hc : 0);
                float M = -INFINITY;
                ltot = 0.f;
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) O[nb] = f32x4{0.f, 0.f, 0.f, 0.f};
                auto fold = [&](float m2, float l2, const f32x4 (&o2)[NB]) {   // (M, ltot, O) <- merged with (m2, l2, o2)
                    const float M_new = fmaxf(M, m2);
                    const float w_old = fast_exp2(M - M_new), w_new = fast_exp2(m2 - M_new);
                    M = M_new;
                    ltot = ltot * w_old + l2 * w_new;
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                        for (int r = 0; r < 4; ++r) O[nb][r] = O[nb][r] * w_old + o2[nb][r] * w_new;
                };
                // (MBATCH parts per round trip: three by default; one in the register-lean instantiation)
                const int per_grp = (nparts + ngrp - 1) / ngrp;
                for (int k0 = 0; k0 < per_grp; k0 += MBATCH) {
                    f32x2 ml[MBATCH];
                    f32x2 t[MBATCH][NB][2];
#pragma unroll
                    for (int b = 0; b < MBATCH; ++b) {
                        const int sidx = min((member ? pg : 0) + ngrp * (k0 + b), nparts - 1);
                        const int64_t row = (int64_t)(first_run + sidx + seq) * p.Hq + hm;
                        ml[b] = load_dev2(p.part_ml + row * 2);
                        const float *ap = p.part_acc + row * HD + 4 * kq;
#pragma unroll
                        for (int nb = 0; nb < NB; ++nb) {
                            t[b][nb][0] = load_dev2(ap + nb * 16);
                            t[b][nb][1] = load_dev2(ap + nb * 16 + 2);
                        }
                    }
#pragma unroll
                    for (int b = 0; b < MBATCH; ++b) {
                        if (member && pg + ngrp * (k0 + b) < nparts) {
                            f32x4 o2[NB];
#pragma unroll
                            for (int nb = 0; nb < NB; ++nb)
                                o2[nb] = f32x4{t[b][nb][0][0], t[b][nb][0][1], t[b][nb][1][0], t[b][nb][1][1]};
                            fold(ml[b][0], ml[b][1], o2);
                        }
                    }
                }
                // groups 1 .. ngrp-1 into group 0 (lane col < g reads lane col + j*g of its 16-lane row);
                // a group that had no part carries (-inf, 0, 0) and changes nothing
                for (int j = 1; j < ngrp && j < nparts; ++j) {
                    const int src = (lane & ~15) | min(j * g + hc, 15);
                    const float m2 = __shfl(M, src), l2 = __shfl(ltot, src);
                    f32x4 o2[NB];
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                        for (int r = 0; r < 4; ++r) o2[nb][r] = __shfl(O[nb][r], src);
                    if (pg == 0) fold(m2, l2, o2);
                }
                if (lane == 0)   // ready for the next call
                    __hip_atomic_store(p.counters + (int64_t)seq * p.Hkv + kvh, 0, __ATOMIC_RELAXED,
                                       __HIP_MEMORY_SCOPE_AGENT);
                store_out = true;
            }
        }
        if (store_out && col < g) {
            const float inv = 1.0f / ltot;
            uint16_t *op = p.out + ((int64_t)q_row * p.Hq + head) * HD + 4 * kq;
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                u32x2 w = {pack2_bf16(O[nb][0] * inv, O[nb][1] * inv), pack2_bf16(O[nb][2] * inv, O[nb][3] * inv)};
                *reinterpret_cast<u32x2 *>(op + nb * 16) = w;
            }
        }
        pos = stop;
        ++seq;
    }
}

template <int HD, int NBI, int MBATCH>
OOCO_DEV void decode_kernel_body(const KernArgs &a)
{
    const AttnParams &p = a.p;
    // What a wave needs before its first KV tile is on its way comes from a dozen places of the kernel
    // arguments; asked for one after the other, each at its point of use, they cost a wave ten dependent
    // round trips to the scalar cache.  Naming them here makes the compiler fetch them together.
    asm volatile("" ::"s"(p.q), "s"(p.k_cache), "s"(p.v_cache), "s"(p.block_tables), "s"(p.seq_lens),
                 "s"(p.query_start_loc), "s"(p.cum_dev), "s"(p.trace), "s"(p.queue), "s"(p.Hq), "s"(p.Hkv), "s"(p.g),
                 "s"(p.max_blocks_per_seq), "s"(p.num_seqs), "s"(p.total_q), "s"(p.dec_blocks), "s"(p.static_blocks),
                 "s"(p.static_runs), "s"(p.tail_runs), "s"(p.piece_pad), "s"(p.rotate_heads), "s"(p.scale_log2e),
                 "s"(p.queue_base), "s"(*reinterpret_cast<const uint64_t *>(&p.xcd_cw[0])),
                 "s"(*reinterpret_cast<const uint64_t *>(&p.xcd_cw[4])));
    const int lane = threadIdx.x;
    // Workgroups are handed to the XCDs round-robin and the kv heads of a block lie in adjacent
    // 4 KiB pieces of memory: rotating the head by the run index gives every XCD every kv head
    // in turn instead of pinning XCD x to head x.
    int run = blockIdx.x / p.Hkv;
    int kvh = p.rotate_heads ? (int)((blockIdx.x - run * p.Hkv + run) % p.Hkv) : (int)(blockIdx.x - run * p.Hkv);
    if (p.xcd_cw[kXcds - 1]) {
        // weighted runs: all kv heads of run v on XCD v % 8 (workgroup b runs on XCD b % 8)
        const int x = blockIdx.x % kXcds, t = blockIdx.x / kXcds;
        kvh = t % p.Hkv;
        run = kXcds * (t / p.Hkv) + x;
    }
    auto cum_at = [&](int idx) -> int { return p.cum_dev ? p.cum_dev[idx] : a.cum[idx]; };
    const RunLayout L = {p.dec_blocks, p.static_blocks, p.static_runs, p.tail_runs, p.xcd_cw};
    const unsigned tail_tasks = (unsigned)p.tail_runs * (unsigned)p.Hkv;

    uint64_t *trace = p.trace ? p.trace + (int64_t)blockIdx.x * 4 : nullptr;   // per-wave time stamps
    if (trace && lane == 0) trace[0] = wall_clock64();
    bool first_piece = true;

  for (;;) {   // the wave's own run first, then tail runs by ticket
    // The ticket for the next tail run is drawn when the last piece of this run has been streamed (whoever
    // is done first gets the next run) and looked at after that piece's epilogue, which covers the round
    // trip of the atomic.  (Every wave ends by drawing a ticket that tells it to stop; atomics on one address
    // are served one after the other, about 13 ns each on MI355X, which is why the tail only pays on long
    // kernels.)
    unsigned ticket = 0xFFFFFFFFu;
    bool drawn = false;
    auto draw = [&]() {
        if (lane == 0)
            ticket = __hip_atomic_fetch_add(p.queue, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) - p.queue_base;
        drawn = true;
    };
    decode_run<HD, NBI, MBATCH>(p, cum_at, L, run, kvh, lane, trace, first_piece, [&]() {
        if (tail_tasks) draw();
    });
    if (!tail_tasks) break;
    if (!drawn) draw();   // (a run that held no block)
    ticket = __builtin_amdgcn_readfirstlane(ticket);
    if (ticket >= tail_tasks) break;
    run = p.static_runs + (int)(ticket / (unsigned)p.Hkv);
    kvh = (int)(ticket % (unsigned)p.Hkv);
  }
    if (trace) {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        if (lane == 0) trace[3] = wall_clock64();
    }
}

template <int HD, int NBI>
__global__ __launch_bounds__(64, 2) void decode_kernel(const KernArgs a)
{
    decode_kernel_body<HD, NBI, 3>(a);
}

// The same kernel within 160 registers per wave (one KV block per step, one part per merge round trip), for
// batches whose prefill workgroups need the rest of the register file: a SIMD then holds one decode wave beside
// two prefill waves of 176 registers.
template <int HD>
__global__ __launch_bounds__(64, 3) void decode_kernel_lean(const KernArgs a)
{
    decode_kernel_body<HD, 1, 1>(a);
}

// ------------------------------------------------------------------------------------------
// Prefill chunk: one workgroup of four waves per (tile of query rows, kv head).  The 128 query
// columns of a workgroup are the (row, head) pairs of tile_rows = 128/g consecutive query rows
// and the g query heads that share the kv head (column c = row*g + head), 32 columns per wave,
// so every K/V tile fetched serves the whole GQA group.  KV is walked four blocks (64 tokens) per
// step through two LDS slots for K and two for V (64 KiB for hd 128), filled by direct
// global->LDS loads, one barrier per step.  Per wave and step, for each 32-token half:
//   S^T[32 tok][32 cols] = K · Q^T    (hd/16 x v_mfma_f32_32x32x16_bf16, K operand from LDS)
//   O^T[hd][32 cols]    += V^T · P^T  (hd/32 x 2 x v_mfma_f32_32x32x16_bf16, V operand from LDS)
// with one softmax update over the 64 scores of a column.  The loop is software pipelined: the
// score MFMAs of step st+1 are issued together with the softmax arithmetic of step st (two score
// register sets that swap roles every step), so that the matrix core works on the next scores
// while the vector ALU exponentiates the current ones; K therefore runs one step ahead of V:
// at the top of step st the loads of K[st+2] and V[st+1] are sent off.
// Lane l = 32*h + col.  MFMA row i of the K operand is fed with token (i with bits 2 and 3
// swapped) of its block, so that S^T register r of lane (col, h) is token 16(r/8) + 8h + r%8 of
// the half: eight consecutive tokens per block, which is what one 16-byte V operand holds.
// LDS (16-byte units, CH = 2*hd per tile): K tiles keep the cache order [hd/8][16 slots]; V tiles
// are stored [token half][dim] so that the 16 lanes of a quarter wave read 256 contiguous bytes
// (no bank conflicts).
// The SIMD's VALU issue port is shared with the matrix core (a 32x32x16 MFMA holds it for half of
// its 32 cycles), so the kernel is tuned for few vector instructions per MFMA: 64-token steps
// halve the per-step bookkeeping, maxima use v_max3, row sums v_dot2c on the packed weights,
// the causal mask runs only on steps that touch the diagonal; at the end of a sequence the unused V
// slots are zeroed once in LDS instead of masking operands.  Two workgroups fit a CU (<= 256 VGPRs,
// 64 KiB LDS each).
constexpr int kPfThreads = 256;   // threads of the four-wave workgroup (the eight-wave one has 512)
constexpr int kPfBlocks = 4;    // KV blocks per step

// Entry idx of the plan's array: from device memory if the plan did not fit the kernel arguments, else from the
// argument block.  The two loads must stay two loads: merged into one load through a selected pointer, the argument
// block would have to be addressable like memory, and the compiler would copy all 4 KiB of it into every lane's
// private memory (the empty asm keeps the arms of the branch apart).
OOCO_DEV int plan_entry(const KernArgs &a, int idx)
{
    if (a.p.cum_dev) return a.p.cum_dev[idx];
    int v = a.cum[idx];
    asm volatile("" : "+v"(v));
    return v;
}

// One workgroup's work on virtual block index `vb` (what blockIdx.x is in the stand-alone kernel): with the plan's
// tile list, entry vb / Hkv of the list -- a (tile, part of its keys) pair -- for kv head vb % Hkv; without it, unit
// vb / split = (tile, kv head), part vb % split of its keys.  `cum_at(i)` reads the prefill array of the plan.  All
// threads of the workgroup call it together; every return is workgroup-uniform.
// NW = waves per workgroup: 4 (128 query columns) or 8 (256 columns: the same K/V tiles in LDS serve twice as many
// columns, which halves the traffic from L2 into the compute unit per unit of matrix work).
// PIPE = false: no software pipeline across steps (the scores of a step are computed in that step, one score
// register set): fewer registers, so that two such waves and a decode wave share a SIMD; the overlap of matrix and
// vector work then comes from the two waves of a SIMD rather than from within one wave.
// `phases` (option "trace", prefill-only batches): receives four 16-bit times in units of 10 ns since `t_start`
// (saturating), lowest first: tile looked up, first K/V loads sent off, first tiles arrived, last step done.
template <int HD, int NW, bool PIPE, class CumAt>
OOCO_DEV void prefill_unit(const AttnParams &p, CumAt cum_at, const int vb, uint64_t *phases = nullptr,
                           const uint64_t t_start = 0)
{
    constexpr int THREADS = NW * 64;
    constexpr int COLS = NW * 32;      // query columns per workgroup
    constexpr int KS = HD / 16;        // k-steps of QK
    constexpr int MB = HD / 32;        // 32-dim groups of the output
    constexpr int CH = HD * 2;         // 16-byte chunks per (block, kv head) tile
    constexpr int STAGE = kPfBlocks * CH;               // chunks of one step's K (or V) tiles
    constexpr int NCP = STAGE / THREADS;                // chunks each thread moves per stage
    __shared__ u32x4 ldsK[2][STAGE];
    __shared__ u32x4 ldsV[2][STAGE];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int col = lane & 31;
    const int h = lane >> 5;
    const int g = p.g;
    uint64_t phase_bits = 0;   // (scalar; touched only when tracing)
    auto phase = [&](int k) {
        if (phases) {
            const uint64_t dt = (uint64_t)wall_clock64() - t_start;
            phase_bits |= (dt < 0xFFFFu ? dt : (uint64_t)0xFFFFu) << (16 * k);
        }
    };
    // workgroup -> (tile, kv head, part of the tile's keys, parts the tile has), and the partial-result slot of
    // part 0 of that (tile, kv head) with the distance between the slots of consecutive parts.  With the tile list
    // every tile has its own number of parts; without it vb = ((tile * Hkv) + kv head) * pf_split + part.
    int split, part, tile_idx, kvh, list_raw = 0;
    int slot0, slot_step;   // (at most kPrefillSplitUnits * kMaxPrefillSplit slots)
    if (p.pf_table) {
        const int entry = min(vb / p.Hkv, p.pf_table - 1);
        kvh = vb - (vb / p.Hkv) * p.Hkv;
        list_raw = cum_at(2 * p.num_pf + 1 + entry);
        const int list_e = __builtin_amdgcn_readfirstlane(list_raw);   // (the same in every lane)
        part = entry_part(list_e);
        split = entry_parts(list_e);
        tile_idx = 0;   // (looked up from the entry below)
        slot0 = (entry - part) * p.Hkv + kvh;
        slot_step = p.Hkv;
    } else {
        split = p.pf_split;
        const int unit = vb / split;
        part = vb - unit * split;
        tile_idx = unit / p.Hkv;
        kvh = unit - tile_idx * p.Hkv;
        slot0 = unit * split;
        slot_step = 1;
    }

    // tile -> (sequence, tile of the sequence); tiles of a sequence are taken last-first because
    // the later rows of a chunk see more keys and the hardware dispatches in index order
    int seq, q_row0, rows, pos0, seq_len;
    {
        int chunk, t;
        if (p.pf_table) {   // the plan lists the (tile, part) pairs one by one
            chunk = min(entry_chunk(list_raw), p.num_pf - 1);
            t = entry_tile(list_raw);
        } else {
            chunk = __builtin_amdgcn_readfirstlane(count_le(cum_at, p.num_pf, tile_idx, lane));
            t = (cum_at(chunk + 1) - 1) - tile_idx;       // reversed order inside the sequence
        }
        seq = min(max(cum_at(p.num_pf + 1 + chunk), 0), p.num_seqs - 1);
        const int q0 = p.query_start_loc[seq];
        const int q_len = p.query_start_loc[seq + 1] - q0;
        const int tile_rows = max(1, COLS / g);
        const int t0 = t * tile_rows;
        q_row0 = min(max(q0 + t0, 0), p.total_q - 1);
        rows = max(1, min(min(tile_rows, q_len - t0), p.total_q - q_row0));
        seq_len = p.seq_lens[seq];
        // keys beyond what the plan allotted to this sequence are never touched
        const int cap = p.max_blocks_per_seq * kBlockSize;
        pos0 = min(max(p.ctx_lens[seq] + t0, 0), cap - rows);
        seq_len = min(seq_len, cap);
        // all of these are the same in every lane: keep them in scalar registers
        seq = __builtin_amdgcn_readfirstlane(seq);
        q_row0 = __builtin_amdgcn_readfirstlane(q_row0);
        rows = __builtin_amdgcn_readfirstlane(rows);
        pos0 = __builtin_amdgcn_readfirstlane(pos0);
        seq_len = __builtin_amdgcn_readfirstlane(seq_len);
    }
    const uint16_t *const k_cache = p.k_cache, *const v_cache = p.v_cache;
    const int Hkv = p.Hkv;
    const float c_log2e = p.scale_log2e;
    const uint32_t ldsK_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void *)&ldsK[0][0];
    const uint32_t ldsV_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void *)&ldsV[0][0];
    // this lane's query column
    const int c = wave * 32 + col;
    const int c_row = c / g, c_head = c - c_row * g;
    const bool c_valid = c_row < rows;
    const int row = min(c_row, rows - 1);
    const int head = kvh * g + c_head;
    const int pos = pos0 + row;                          // this column's absolute position
    // the wave's columns span rows [w_row_lo, w_row_hi] (scalar)
    const int w_row_lo = min((wave * 32) / g, rows - 1), w_row_hi = min((wave * 32 + 31) / g, rows - 1);
    const int w_pos_lo = pos0 + w_row_lo, w_pos_hi = pos0 + w_row_hi;
    const int kv_end = pos0 + rows;                      // keys visible to the tile: [0, kv_end)
    const int nblk = (kv_end + kBlockSize - 1) / kBlockSize;
    const int nstep_all = (nblk + kPfBlocks - 1) / kPfBlocks;
    // this workgroup's share of the steps: [st_lo, nstep); a unit with fewer steps than parts has fewer parts
    const int nparts = min(split, nstep_all);
    if (part >= nparts) return;                          // (the whole workgroup leaves: no barrier is pending)
    const int st_lo = nstep_all * part / nparts;
    const int nstep = nstep_all * (part + 1) / nparts;

    phase(0);
    u32x4 qb[KS];
    {
        const u32x4 *qp = reinterpret_cast<const u32x4 *>(p.q + ((int64_t)(q_row0 + row) * p.Hq + head) * HD);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) qb[ks] = qp[2 * ks + h];
        // Passing the registers through an empty asm makes the compiler wait for these loads here,
        // before the loop, instead of counting them down inside it (which would also wait for the
        // global->LDS loads it does not know about).
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) asm volatile("" : "+v"(qb[ks]));
    }
    const int32_t *table = p.block_tables + (int64_t)seq * p.max_blocks_per_seq;
    const int64_t tile_elems = (int64_t)HD * kBlockSize;
    // K operand row col -> block (col>>4) of the half, slot with bits 2,3 of (col&15) swapped
    const int ku = col >> 4;
    const int kslot = (col & 3) | ((col & 4) << 1) | ((col & 8) >> 1);

    // One stage (the K or the V tiles of a step) goes from global memory straight into LDS
    // (global_load_lds_dwordx4: every lane gives a 16-byte global address, the wave's 64 pieces land
    // contiguously at the LDS address in M0).  Wave w moves the 64-chunk groups w, w+4, ...; chunk
    // cidx of the stage belongs to block cidx/CH of the step and comes from
    //   K: cache chunk cidx%CH   (same order as the cache)
    //   V: LDS position r = half*HD + dim  <-  cache chunk 2*dim + half
    // The instruction is issued through inline asm so that the waits stay under this code's
    // control.  (The block table is read through the constant address space: scalar loads, which
    // the waits on the vector-memory counter do not see.)
    typedef const __attribute__((address_space(4))) int32_t *const_i32_ptr;
    const const_i32_ptr ctable = (const_i32_ptr)(uintptr_t)table;
    auto block_id = [&](int b) -> int { return ctable[min(b, nblk - 1)]; };
    // (tile of kv head kvh of physical block pb) = cache + pb * blk_stride + kvh * tile_elems, in elements
    const uint16_t *const k_head = k_cache + (int64_t)kvh * tile_elems, *const v_head = v_cache + (int64_t)kvh * tile_elems;
    const uint32_t blk_stride = (uint32_t)Hkv * (uint32_t)tile_elems;
    auto issue = [&](bool is_v, int slot, const int (&pb)[kPfBlocks]) {   // pb: physical ids of the step's blocks
        static_assert(NCP == 4 || NCP == 2, "one asm statement per stage");
        const uint16_t *base[NCP];
        uint32_t voff[NCP], dst[NCP];
#pragma unroll
        for (int n = 0; n < NCP; ++n) {
            const int grp = wave + NW * n;                 // wave-uniform
            const int cidx = grp * 64 + lane;
            // block of the step (wave-uniform).  Four waves and at least 256 chunks per tile: a compile-time
            // constant, which keeps pb[] in registers without select chains.  Eight waves (256 chunks per tile):
            // waves 0..3 move the even blocks' tiles, waves 4..7 the odd ones (one select, no indexed array).
            int which, pbw;
            if constexpr (NW == 4) {
                which = CH >= 256 ? (4 * n * 64) / CH : (grp * 64) / CH;
                pbw = pb[which];
            } else {
                static_assert(NW != 8 || CH == 256, "eight-wave workgroups: head_dim 128");
                which = 2 * n + (wave >> 2);
                pbw = (wave >> 2) ? pb[2 * n + 1] : pb[2 * n];
            }
            const int r = cidx - which * CH;
            // scalar tile address + 32-bit lane offset (bytes)
            base[n] = (is_v ? v_head : k_head) + (uint64_t)(uint32_t)pbw * blk_stride;
            voff[n] = (uint32_t)(is_v ? 2 * (r % HD) + r / HD : r) * 16u;
            dst[n] = (is_v ? ldsV_base : ldsK_base) + (uint32_t)((slot * STAGE + grp * 64) * 16);
        }
        uint32_t saved_m0;   // M0 is restored: the compiler may keep a value of its own there
        if constexpr (NCP == 4)
            asm volatile("s_mov_b32 %0, m0\n\t"
                         "s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %5, %9\n\t"
                         "s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %6, %10\n\t"
                         "s_mov_b32 m0, %3\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %7, %11\n\t"
                         "s_mov_b32 m0, %4\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %8, %12\n\t"
                         "s_mov_b32 m0, %0"
                         : "=&s"(saved_m0)
                         : "s"(dst[0]), "s"(dst[1]), "s"(dst[2]), "s"(dst[3]), "v"(voff[0]), "v"(voff[1]), "v"(voff[2]),
                           "v"(voff[3]), "s"(base[0]), "s"(base[1]), "s"(base[2]), "s"(base[3])
                         : "memory");
        else
            asm volatile("s_mov_b32 %0, m0\n\t"
                         "s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %3, %5\n\t"
                         "s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %4, %6\n\t"
                         "s_mov_b32 m0, %0"
                         : "=&s"(saved_m0)
                         : "s"(dst[0]), "s"(dst[1]), "v"(voff[0]), "v"(voff[1]), "s"(base[0]), "s"(base[1])
                         : "memory");
    };

    f32x16 O[MB];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int r = 0; r < 16; ++r) O[mb][r] = 0.f;

    // scores of one step: S[hh] register r is token st*64 + 32hh + 8h + 16(r/8) + r%8
    auto qk = [&](f32x16 (&S)[2], int slot) {
#pragma unroll
        for (int hh = 0; hh < 2; ++hh)
#pragma unroll
            for (int r = 0; r < 16; ++r) S[hh][r] = 0.f;
        // the two token halves alternate, so that consecutive MFMAs never wait for each other's result
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
#pragma unroll
            for (int hh = 0; hh < 2; ++hh) {
                const u32x4 kop = ldsK[slot][(2 * hh + ku) * CH + (2 * ks + h) * 16 + kslot];
                S[hh] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, kop),
                                                            __builtin_bit_cast(bf16x8, qb[ks]), S[hh], 0, 0, 0);
            }
    };
    // causal mask of a step that touches the diagonal
    auto mask = [&](f32x16 (&S)[2], int st) {
        const int room = pos - (st * 64 + 8 * h);        // visible iff 32hh + 16(r/8) + r%8 <= room
#pragma unroll
        for (int hh = 0; hh < 2; ++hh)
#pragma unroll
            for (int r = 0; r < 16; ++r)
                S[hh][r] = (32 * hh + 16 * (r / 8) + (r % 8) <= room) ? S[hh][r] : -INFINITY;
    };
    float m = -INFINITY, lsum = 0.f;
    // online-softmax update with the raw scores of one step; P[2hh+u] holds the packed weights of
    // tokens 32hh + 16u + 8h + 0..7.  The softmax scale rides in the fma that feeds exp2 (scale > 0,
    // so the maximum can be taken before scaling).
    // The update comes in two halves so that the PV products of the first 32 tokens can run beside the
    // exponentials of the last 32: weights(S, P, q4, ...) turns the scores of tokens 16*q4 + 8h + 0..7 into P[q4].
    auto weights = [&](const f32x16 (&S)[2], u32x4 (&P)[4], int q4, float m_ref, float &psum) {
        float e[8];
#pragma unroll
        for (int r = 0; r < 8; ++r) e[r] = fast_exp2(__builtin_fmaf(S[q4 >> 1][8 * (q4 & 1) + r], c_log2e, -m_ref));
        P[q4] = u32x4{pack2_bf16(e[0], e[1]), pack2_bf16(e[2], e[3]), pack2_bf16(e[4], e[5]), pack2_bf16(e[6], e[7])};
        // the denominator sums the same rounded weights that enter the PV product
#pragma unroll
        for (int w = 0; w < 4; ++w) psum = sum2_bf16(P[q4][w], psum);
    };
    auto softmax_first = [&](const f32x16 (&S)[2], u32x4 (&P)[4], float &alpha, bool &grow, float &psum) {
        float mloc = max32(S[0], S[1]);
        {
            float x, y;
            swap32(mloc, x, y);
            mloc = max2(x, y) * c_log2e;
        }
        // (floored: a part of a split tile may start with steps that a column does not see at all; its maximum
        // then stays at the floor, its weights and sum at 0, instead of running into inf - inf)
        // The reference point m only has to stay within 2^8 of the true running maximum (weights up to 256 are
        // exact enough in bf16 and harmless in the fp32 sums; the final division cancels the reference), so it
        // moves, and the accumulators are rescaled, only when a step's maximum exceeds it by more than 8.
        const float m_cand = floor_m1e30(mloc);
        grow = m_cand > m + 8.0f;
        const float m_new = grow ? m_cand : m;
        alpha = fast_exp2(m - m_new);
        m = m_new;
        psum = 0.f;
        weights(S, P, 0, m, psum);
        weights(S, P, 1, m, psum);
    };
    auto softmax_second = [&](const f32x16 (&S)[2], u32x4 (&P)[4], float alpha, float psum) {
        weights(S, P, 2, m, psum);
        weights(S, P, 3, m, psum);
        lsum = lsum * alpha + psum;
    };
    // The MFMAs of tokens 0..31 (P[0], P[1]) are laid out beside the vector work that is still due when pv
    // starts (the second half of the softmax update), those of tokens 32..63 follow.
    auto pv = [&](const u32x4 (&P)[4], int slot) {
        const u32x4 *vp = &ldsV[slot][h * HD + col];
#pragma unroll
        for (int i = 0; i < 4 * MB; ++i) {
            const u32x4 vop = vp[(i / MB) * CH + 32 * (i % MB)];
            O[i % MB] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, vop),
                                                            __builtin_bit_cast(bf16x8, P[i / MB]), O[i % MB], 0, 0, 0);
        }
        // every operand is requested kAhead MFMAs before the MFMA that uses it
        constexpr int kAhead = 4;
        __builtin_amdgcn_sched_group_barrier(0x100, kAhead, 0);
#pragma unroll
        for (int i = 0; i < 4 * MB - kAhead; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            if (i < 2 * MB) __builtin_amdgcn_sched_group_barrier(0x002, 6, 0);   // (exponentials count as VALU here)
        }
        __builtin_amdgcn_sched_group_barrier(0x008, kAhead, 0);
    };
    // Last step of a sequence only (workgroup-uniform): V slots at or past seq_len may hold anything; their
    // weights are 0, but 0*NaN is NaN, so they are zeroed in LDS before anybody multiplies with them.
    auto scrub_v = [&](int slot, int st) {
#pragma unroll
        for (int n = 0; n < NCP; ++n) {
            const int cidx = n * THREADS + tid;              // chunk [block][token half][dim] of the stage
            const int blk = cidx / CH, half = (cidx % CH) / HD;
            const int t0 = st * 64 + 16 * blk + 8 * half;    // tokens t0 .. t0+7
            u32x4 mk;
#pragma unroll
            for (int w = 0; w < 4; ++w)
                mk[w] = (t0 + 2 * w < seq_len ? 0x0000FFFFu : 0u) | (t0 + 2 * w + 1 < seq_len ? 0xFFFF0000u : 0u);
            ldsV[slot][cidx] &= mk;
        }
        __syncthreads();
    };

    int ids1[kPfBlocks], ids2[kPfBlocks];   // block ids of the steps st+1 and st+2
    {
        int ids0[kPfBlocks];
#pragma unroll
        for (int b = 0; b < kPfBlocks; ++b) {
            ids0[b] = block_id(kPfBlocks * st_lo + b);
            ids1[b] = block_id(kPfBlocks * (st_lo + 1) + b);
            ids2[b] = block_id(kPfBlocks * (st_lo + 2) + b);
        }
        issue(false, st_lo & 1, ids0);
        issue(true, st_lo & 1, ids0);
        if (PIPE && st_lo + 1 < nstep) issue(false, (st_lo + 1) & 1, ids1);
    }
    phase(1);
    // One step.  Sc: scores of step st (computed during step st-1), Sn: receives those of step st+1.
    auto body = [&](f32x16 (&Sc)[2], f32x16 (&Sn)[2], int st) {
        // this wave's loads of K[st+1] and V[st] have landed, and after the barrier so have
        // everybody's; nobody reads K[st] or V[st-1] any more
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        if (st + 2 < nstep) issue(false, st & 1, ids2);
        if (st + 1 < nstep) issue(true, (st + 1) & 1, ids1);
        if (st * 64 + 64 > seq_len) scrub_v(st & 1, st);
#pragma unroll
        for (int b = 0; b < kPfBlocks; ++b) {
            ids1[b] = ids2[b];
            ids2[b] = block_id(kPfBlocks * (st + 3) + b);
        }
        // wave-uniform: some column of this wave sees keys of the step
        if (st * 64 > w_pos_hi) return;
        if (st * 64 + 63 > w_pos_lo) mask(Sc, st);   // the step touches the causal diagonal
        u32x4 P[4];
        float alpha, psum;
        bool grow;
        // One straight-line region for the scheduler.  The scores of step st+1 are computed even
        // when nothing will use them (last step of the tile, or no column of the wave sees that
        // step): the K slot then holds an older step's tiles, and the result is dropped.
        qk(Sn, (st + 1) & 1);
        softmax_first(Sc, P, alpha, grow, psum);
        // the weights of the first 32 tokens are due here, inside the region of the score MFMAs ...
        asm volatile("" : "+v"(P[0]));
        asm volatile("" : "+v"(P[1]));
        // ... and the region is laid out as 2*hd/16 x (MFMA, LDS read, a share of the vector work):
        // the maximum is found next to the first MFMAs, the exponentials next to the others
        __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
#pragma unroll
        for (int i = 0; i < KS / 2; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x002, 4, 0);
        }
#pragma unroll
        for (int i = KS / 2; i < 2 * KS; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x002, 4, 0);
            __builtin_amdgcn_sched_group_barrier(0x400, 2, 0);
        }
        if (__any(grow)) {
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                for (int r = 0; r < 16; ++r) O[mb][r] *= alpha;
        }
        // the second half of the update belongs to the region of the PV MFMAs: its scores pass through an empty
        // asm here so that nothing of it is moved up
        asm volatile("" : "+v"(Sc[1]));
        softmax_second(Sc, P, alpha, psum);
        pv(P, st & 1);
    };

    if constexpr (PIPE) {
        f32x16 SA[2], SB[2];
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        phase(2);
        qk(SA, st_lo & 1);
        for (int st = st_lo; st < nstep; st += 2) {
            body(SA, SB, st);
            if (st + 1 < nstep) body(SB, SA, st + 1);
        }
    } else {
        for (int st = st_lo; st < nstep; ++st) {
            // the loads of K[st] and V[st] have landed (everybody's, after the barrier); nobody reads the tiles of
            // step st-1 any more, so the loads of step st+1 may overwrite them
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __syncthreads();
            if (st + 1 < nstep) {
                issue(false, (st + 1) & 1, ids1);
                issue(true, (st + 1) & 1, ids1);
            }
            if (st * 64 + 64 > seq_len) scrub_v(st & 1, st);
#pragma unroll
            for (int b = 0; b < kPfBlocks; ++b) ids1[b] = block_id(kPfBlocks * (st + 2) + b);
            if (st * 64 > w_pos_hi) continue;   // wave-uniform: no column of this wave sees keys of the step
            f32x16 S[2];
            qk(S, st & 1);
            if (st * 64 + 63 > w_pos_lo) mask(S, st);
            u32x4 P[4];
            float alpha, psum;
            bool grow;
            softmax_first(S, P, alpha, grow, psum);
            if (__any(grow)) {
#pragma unroll
                for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                    for (int r = 0; r < 16; ++r) O[mb][r] *= alpha;
            }
            softmax_second(S, P, alpha, psum);
            const u32x4 *vp = &ldsV[st & 1][h * HD + col];
#pragma unroll
            for (int i = 0; i < 4 * MB; ++i) {
                const u32x4 vop = vp[(i / MB) * CH + 32 * (i % MB)];
                O[i % MB] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, vop),
                                                                __builtin_bit_cast(bf16x8, P[i / MB]), O[i % MB], 0, 0, 0);
            }
        }
    }
    phase(3);
    if (phases && tid == 0) *phases = phase_bits;
    float ltot;
    {
        float x, y;
        swap32(lsum, x, y);
        ltot = x + y;
    }
    if (nparts > 1) {
        // (one counter per (tile, kv head): the slot of its part 0 with the list, the unit's index without)
        const int counter_idx = p.pf_table ? slot0 : slot0 / split;
        // ---- partial result of this part, arrival count, merge by the part that arrives last (same
        // device-scope accesses as the decode kernel).  Lane (col, h) of wave w owns column c = 32w + col,
        // dims 32mb + 8q4 + 4h + 0..3.  m is the same in both lane halves; ltot already sums them.
        // layout of a part: [wave][mb][q4][lane][4 floats], so that every store and load instruction of a wave
        // covers 1 KiB of contiguous memory
        auto part_ptr = [&](int64_t j, int mb) -> float * {
            return p.pf_acc + ((((int64_t)(slot0 + (int)j * slot_step) * NW + wave) * MB + mb) * 4 * 64 + lane) * 4;
        };
        {
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4)
                    store_dev4(part_ptr(part, mb) + q4 * 256,
                               f32x4{O[mb][4 * q4], O[mb][4 * q4 + 1], O[mb][4 * q4 + 2], O[mb][4 * q4 + 3]});
            if (h == 0) store_dev2(p.pf_ml + ((int64_t)(slot0 + part * slot_step) * COLS + c) * 2, m, ltot);
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // this wave's partial has reached memory ...
        __syncthreads();                                    // ... and so have the other waves'
        __shared__ int arrived;
        if (tid == 0)
            arrived = __hip_atomic_fetch_add(p.pf_counters + counter_idx, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __syncthreads();
        if (arrived != nparts - 1) return;
        float M = -INFINITY;
        ltot = 0.f;
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int r = 0; r < 16; ++r) O[mb][r] = 0.f;
        for (int j = 0; j < nparts; ++j) {                  // in part order: the result does not depend on who is last
            const f32x2 ml = load_dev2(p.pf_ml + ((int64_t)(slot0 + j * slot_step) * COLS + c) * 2);
            f32x4 t[4 * MB];   // t[4*mb + q4] = this lane's dims 32mb + 8q4 + 4h + 0..3 of part j
            if constexpr (MB == 4)
                load_dev_part(t, part_ptr(j, 0), part_ptr(j, 1), part_ptr(j, 2), part_ptr(j, 3));
            else
                load_dev_part(t, part_ptr(j, 0), part_ptr(j, 1));
            const float M_new = fmaxf(M, ml[0]);
            const float w_old = fast_exp2(M - M_new), w_new = fast_exp2(ml[0] - M_new);
            M = M_new;
            ltot = ltot * w_old + ml[1] * w_new;
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4) {
#pragma unroll
                    for (int r = 0; r < 4; ++r) O[mb][4 * q4 + r] = O[mb][4 * q4 + r] * w_old + t[4 * mb + q4][r] * w_new;
                }
        }
        if (tid == 0)   // ready for the next call
            __hip_atomic_store(p.pf_counters + counter_idx, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    if (c_valid) {
        const float inv = 1.0f / ltot;
        uint16_t *op = p.out + ((int64_t)(q_row0 + row) * p.Hq + head) * HD + 4 * h;
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

template <int HD, int NW>
__global__ __launch_bounds__(NW * 64, 8 / NW) void prefill_kernel(const KernArgs a)
{
    const AttnParams &p = a.p;
    // option "trace" on a batch without decode work: per workgroup (start, XCD * 256 + compute unit id, times of
    // four phases since the start, end)
    uint64_t *const trace = (p.trace && p.static_runs == 0) ? p.trace + (int64_t)blockIdx.x * 4 : nullptr;
    const uint64_t t_start = trace ? wall_clock64() : 0;
    if (trace && threadIdx.x == 0) {
        trace[0] = t_start;
        trace[1] = (__builtin_amdgcn_s_getreg((31 << 11) | 20) & 7u) * 256u + ((__builtin_amdgcn_s_getreg((31 << 11) | 4) >> 8) & 255u);
        trace[2] = 0;   // (a workgroup that leaves before its first step stores no phases)
    }
    prefill_unit<HD, NW, true>(p, [&](int idx) -> int { return plan_entry(a, idx); }, (int)blockIdx.x,
                               trace ? trace + 2 : nullptr, t_start);
    if (trace) {
        __syncthreads();
        if (threadIdx.x == 0) trace[3] = wall_clock64();
    }
}

// Eight waves, 256 query columns, no software pipeline, at most 176 registers per wave: the prefill kernel of
// batches that also hold decode work (see decode_kernel_lean).
template <int HD>
__global__ __launch_bounds__(512, 1) __attribute__((amdgpu_num_vgpr(168))) void prefill_kernel_lean(const KernArgs a)
{
    const AttnParams &p = a.p;
    prefill_unit<HD, 8, false>(p, [&](int idx) -> int { return plan_entry(a, idx); }, (int)blockIdx.x);
}

// ------------------------------------------------------------------------------------------
// Mixed batches in ONE launch: a persistent grid of two 256-thread workgroups per compute unit in which a compute
// unit runs EITHER decode waves (eight per unit, each streaming runs of the decode line exactly as the decode
// kernel's waves do) OR prefill workgroups (two per unit, each working through (tile, kv head) units exactly as
// the prefill kernel's workgroups do).  Side by side on one unit the two kinds get into each other's way -- the
// decode waves lose their issue slots and the matrix pipe to prefill waves that keep both busy, the prefill
// workgroups lose half their register file -- and both kernels stretch; apart, the decode units keep HBM busy
// while the prefill units keep the matrix cores busy.
//   * Which unit does what: the first workgroup to arrive on a compute unit (identified by the hardware's XCD,
//     shader-engine and CU ids) claims it and draws the unit's rank within its XCD from a counter; the other
//     workgroup of the unit reads that rank.  Ranks below p.dec_cus decode, the others prefill, so every XCD (and
//     its L2) gets the same mix.
//   * Work is pulled from counters: decode waves draw (run, kv head) items, prefill workgroups draw units from
//     the list of their own XCD first (unit index = XCD mod 8, so the tiles that share keys meet in one L2, as
//     in the stand-alone kernel) and from the other XCDs' lists after that.
//   * A workgroup whose own kind of work has run out takes up the other kind once, then leaves: the split of the
//     units only has to be roughly right.
// Nothing waits for another workgroup except the bounded look at a claim in progress, so the grid drains whatever
// the placement.  The last workgroup to leave resets the claims and counters for the next launch (or replay).
// State (int32, zero between launches), at p.queue - kMixedStateInts + 1:
//   [0, 2048) claims: 0 free, 1 being claimed, rank + 2;  [2048, 2056) arrivals per XCD;
//   [2056, 2064) prefill units drawn per XCD;  [2064] decode items drawn;  [2065] workgroups that have left
constexpr int kMixedClaims = 2048;
constexpr int kMixedShareCus = 99;
template <int HD>
__global__ __launch_bounds__(kPfThreads, 2) void mixed_kernel(const KernArgs a)
{
    const AttnParams &p = a.p;
    __shared__ int sh_role, sh_item;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    int32_t *const state = reinterpret_cast<int32_t *>(p.queue) - (kMixedStateInts - 1);
    int32_t *const claims = state, *const xcd_arrivals = state + kMixedClaims, *const pf_drawn = state + kMixedClaims + 8;
    int32_t *const dec_drawn = state + kMixedClaims + 16, *const left = state + kMixedClaims + 17;
    const int n_cum = p.num_seqs + 1;   // the prefill array follows the decode array
    auto dcum_at = [&](int idx) -> int { return p.cum_dev ? p.cum_dev[idx] : a.cum[idx]; };
    auto pf_at = [&](int idx) -> int { return plan_entry(a, n_cum + idx); };
    const unsigned xcc = __builtin_amdgcn_s_getreg((31 << 11) | 20) & 7u;              // XCC_ID
    if (tid == 0) {
        const unsigned hw = __builtin_amdgcn_s_getreg((31 << 11) | 4);                 // HW_ID: CU, SH, SE ids in bits 8..15
        int32_t *const claim = claims + (xcc * 256u + ((hw >> 8) & 255u));
        int expected = 0, rank;
        const bool won = __hip_atomic_compare_exchange_strong(claim, &expected, 1, __ATOMIC_RELAXED, __ATOMIC_RELAXED,
                                                              __HIP_MEMORY_SCOPE_AGENT);
        if (won) {
            rank = __hip_atomic_fetch_add(xcd_arrivals + xcc, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(claim, rank + 2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        } else {
            // the claimant runs on this very compute unit and needs two more memory operations: a bounded look
            int v = expected;
            for (int spin = 0; v < 2 && spin < (1 << 16); ++spin) {
                __builtin_amdgcn_s_sleep(8);
                v = __hip_atomic_load(claim, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
            rank = v >= 2 ? v - 2 : 0;   // (never seen: decode)
        }
        // p.dec_cus == kMixedShareCus: every unit runs both kinds side by side (its first workgroup decodes, its
        // second prefills) -- the arrangement of the two separate kernels, inside one launch, kept for measurements
        sh_role = p.dec_cus == kMixedShareCus ? (won ? 0 : 1) : (rank < p.dec_cus ? 0 : 1);
    }
    __syncthreads();
    int role = sh_role;   // 0 = decode, 1 = prefill
    // option "trace": per workgroup (start, end of its first kind of work, end of its second kind, first role +
    // 256 * items of wave 0 in the first kind + 2^32 * items in the second) on the 100 MHz clock
    uint64_t *const trace = p.trace ? p.trace + (int64_t)blockIdx.x * 4 : nullptr;
    uint64_t n_first = 0, n_second = 0;   // (two scalars: an array indexed by the pass would live in scratch memory)
    if (trace && tid == 0) {
        trace[0] = wall_clock64();
        trace[3] = (uint64_t)role;
    }
    const int n_dec_items = p.static_runs * p.Hkv;
    const int n_vb = p.pf_table ? p.pf_table * p.Hkv : p.n_tiles * p.Hkv * p.pf_split;
    const RunLayout L = {p.dec_blocks, p.static_blocks, p.static_runs, 0, p.xcd_cw};
    for (int pass = 0; pass < 2; ++pass, role ^= 1) {
        if (role == 0) {
            bool first_piece = false;
            for (;;) {
                int item = 0;
                if (lane == 0) item = __hip_atomic_fetch_add(dec_drawn, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                item = __builtin_amdgcn_readfirstlane(item);
                if (item >= n_dec_items) break;
                const int run = item / p.Hkv;
                const int kvh = (item - run * p.Hkv + run) % p.Hkv;   // kv heads rotate over the runs
                decode_run<HD, (HD == 64 ? 2 : 1), 3>(p, dcum_at, L, run, kvh, lane, nullptr, first_piece, []() {});
                if (pass == 0) ++n_first; else ++n_second;
            }
        } else {
            for (;;) {
                __syncthreads();   // everybody is done with the last unit's LDS tiles and has read sh_item
                if (tid == 0) {
                    int vb = -1;
                    for (unsigned k = 0; k < 8 && vb < 0; ++k) {
                        const unsigned x = (xcc + k) & 7u;
                        const int count = (n_vb - (int)x + 7) / 8;   // units x, x + 8, ... below n_vb
                        // (a look before the draw keeps the counters of exhausted lists from running on)
                        if (__hip_atomic_load(pf_drawn + x, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >= count) continue;
                        const int j = __hip_atomic_fetch_add(pf_drawn + x, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        if (j < count) vb = 8 * j + (int)x;
                    }
                    sh_item = vb;
                }
                __syncthreads();
                const int vb = sh_item;
                if (vb < 0) break;
                prefill_unit<HD, 4, true>(p, pf_at, vb);
                if (pass == 0) ++n_first; else ++n_second;
            }
        }
        __syncthreads();   // the whole workgroup changes its kind of work together
        if (trace && tid == 0) trace[1 + pass] = wall_clock64();
    }
    if (trace && tid == 0) trace[3] += (n_first << 8) + (n_second << 32);
    // leave; the last workgroup out clears the state
    if (tid == 0) {
        const int gone = __hip_atomic_fetch_add(left, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        sh_item = gone == (int)gridDim.x - 1;
    }
    __syncthreads();
    if (sh_item) {
        for (int i = tid; i < kMixedStateInts - 1; i += kPfThreads)
            __hip_atomic_store(state + i, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

// ------------------------------------------------------------------------------------------
// KV block copy: workgroup (pair, which pool, slice) moves a contiguous slice of one block with
// 16-byte loads and stores; all loads of a thread are issued before its stores.
constexpr int kCopyThreads = 256;

template <int VPT, bool NT>
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
    const int64_t base = (int64_t)slice * kCopyThreads * VPT + threadIdx.x;
    u32x4 r[VPT];
#pragma unroll
    for (int i = 0; i < VPT; ++i) {
        const int64_t idx = base + (int64_t)i * kCopyThreads;
        if (idx < block_vecs) r[i] = NT ? __builtin_nontemporal_load(src + idx) : src[idx];
    }
#pragma unroll
    for (int i = 0; i < VPT; ++i) {
        const int64_t idx = base + (int64_t)i * kCopyThreads;
        if (idx < block_vecs) {
            if (NT)
                __builtin_nontemporal_store(r[i], dst + idx);
            else
                dst[idx] = r[i];
        }
    }
}

// ------------------------------------------------------------------------------------------
// KV append: the K and V vectors of the step's tokens go into their paged slots.  One workgroup of 256 threads per
// (sequence, KV block that the step's rows of that sequence touch): the rows of a block are written together, so
// that whole lines leave the compute unit -- K keeps [hd/8][16 slots][8]: the 16-byte pieces of up to 16 rows are
// contiguous per group of 8 dims; V keeps [dim][16 slots]: a thread gathers one (kv head, dim) element from all
// rows of the block and writes them side by side (two 16-byte stores when the step covers the whole block, 2-byte
// stores otherwise).
// Workgroup w -> (sequence, block) without a plan: sequence i owns the workgroup indices [G(i), G(i+1)) with
// G(i) = query_start_loc[i] / 16 + 2 i, which is at least as many as the blocks its q_len rows can touch
// (q_len / 16 + 2); the grid has total_q / 16 + 2 num_seqs + 1 workgroups and those beyond a sequence's last
// block leave at once.  Every workgroup finds its sequence with one 64-lane look at query_start_loc.
constexpr int kAppendThreads = 256;
__global__ __launch_bounds__(kAppendThreads) void kv_append_kernel(const uint16_t *k_new, const uint16_t *v_new,
                                                                   uint16_t *k_cache, uint16_t *v_cache,
                                                                   const int32_t *block_tables,
                                                                   const int32_t *query_start_loc, const int32_t *ctx_lens,
                                                                   int num_seqs, int total_q, int Hkv, int hd,
                                                                   int max_blocks_per_seq, int64_t num_blocks, int parts)
{
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    // `parts` workgroups share a (sequence, block) pair: each takes every parts-th slice of the K chunks and of the
    // V elements, so that a pair whose rows cover its block only partly (many narrow stores) does not end last
    const int w = blockIdx.x / parts;
    const int part = blockIdx.x - w * parts;
    auto g_at = [&](int idx) -> int { return query_start_loc[idx] / kBlockSize + 2 * idx; };
    int seq, q0, q_len, ctx;
    if (num_seqs <= 4 * 64) {
        // up to 256 sequences: the four 64-lane looks are independent loads (one memory round trip), where
        // count_le would wait for each before starting the next; the same round trip brings the lengths of all
        // sequences (lane l of look p holds query_start_loc[64p + l + 1] and ctx_lens[64p + l]), so that the found
        // sequence's own values are a lane read away instead of a second round trip
        int cnt = 0, qv[4], cv[4];
        const int qs0 = query_start_loc[0];   // (0 by the arrays' contract; read in the same round trip all the same)
#pragma unroll
        for (int pass = 0; pass < 4; ++pass) {
            const int idx = 1 + 64 * pass + lane;
            qv[pass] = idx <= num_seqs ? query_start_loc[idx] : 0x7FFFFFFF;
            cv[pass] = idx <= num_seqs ? ctx_lens[idx - 1] : 0;
        }
#pragma unroll
        for (int pass = 0; pass < 4; ++pass) {
            const int idx = 1 + 64 * pass + lane;
            const int v = idx <= num_seqs ? qv[pass] / kBlockSize + 2 * idx : 0x7FFFFFFF;
            cnt += __popcll(__ballot(v <= w));
        }
        seq = __builtin_amdgcn_readfirstlane(min(cnt, num_seqs - 1));
        // query_start_loc[seq + 1] and ctx_lens[seq] sit in lane seq % 64 of look seq / 64, query_start_loc[seq] in
        // the lane before
        auto pick = [&](const int (&r)[4], int i) -> int {   // value of flat index i (wave-uniform) of a 4 x 64 array
            const int p4 = i >> 6, l = i & 63;
            const int x = p4 == 0 ? r[0] : p4 == 1 ? r[1] : p4 == 2 ? r[2] : r[3];
            return __builtin_amdgcn_readlane(x, l);
        };
        const int q1 = pick(qv, seq);
        q0 = seq > 0 ? pick(qv, seq - 1) : qs0;
        q_len = q1 - q0;
        ctx = pick(cv, seq);
    } else {
        seq = count_le(g_at, num_seqs, w, lane);
        seq = __builtin_amdgcn_readfirstlane(min(seq, num_seqs - 1));
        q0 = query_start_loc[seq];
        q_len = query_start_loc[seq + 1] - q0;
        ctx = ctx_lens[seq];
    }
    if (q_len <= 0 || ctx < 0 || q0 < 0 || q0 + q_len > total_q) return;   // nothing to write / inconsistent arrays
    const int j = w - (q0 / kBlockSize + 2 * seq);          // which of the touched blocks
    const int bidx = ctx / kBlockSize + j;
    if (j < 0 || bidx > (ctx + q_len - 1) / kBlockSize) return;   // beyond the sequence's last touched block
    if (bidx >= max_blocks_per_seq) return;                 // beyond the block table: nothing is written
    // (the id is checked where the stores are, so that the loads of the new vectors do not wait for it)
    const int64_t blk_raw = block_tables[(int64_t)seq * max_blocks_per_seq + bidx];
    const bool blk_ok = blk_raw >= 0 && blk_raw < num_blocks;   // id outside the pool: nothing is written
    const int64_t blk = blk_ok ? blk_raw : 0;
    // rows t_lo .. t_lo + nrow - 1 of the sequence fall into this block, starting at slot slot0
    const int t_lo = max(0, bidx * kBlockSize - ctx);
    const int slot0 = ctx + t_lo - bidx * kBlockSize;
    const int nrow = min(kBlockSize - slot0, q_len - t_lo);
    const int row_elems = Hkv * hd;
    const int64_t row0 = (int64_t)(q0 + t_lo);
    // K: thread -> (row r = tid % 16, 16-byte chunk c = tid / 16 + 16 i): the 16 rows of a chunk are adjacent in
    // the cache, so a wave's stores cover 4 chunks x 256 contiguous bytes
    {
        const int chunks = row_elems / 8;
        const int r = tid & 15;
        if (r < nrow) {
            const u32x4 *src = reinterpret_cast<const u32x4 *>(k_new + (row0 + r) * row_elems);
            u32x4 *dst = reinterpret_cast<u32x4 *>(k_cache) + (int64_t)blk * chunks * kBlockSize + slot0 + r;
            constexpr int kSlice = kAppendThreads / 16;   // chunks a workgroup moves per pass
            for (int c0 = (tid >> 4) + kSlice * part; c0 < chunks; c0 += 2 * kSlice * parts) {
                u32x4 v[2];
#pragma unroll
                for (int i = 0; i < 2; ++i) {
                    const int c = c0 + i * kSlice * parts;
                    if (c < chunks) v[i] = src[c];
                }
#pragma unroll
                for (int i = 0; i < 2; ++i) {
                    const int c = c0 + i * kSlice * parts;
                    if (c < chunks && blk_ok) dst[(int64_t)c * kBlockSize] = v[i];
                }
            }
        }
    }
    // V: thread -> element e = (kv head, dim); cache row (blk * Hkv * hd + e) * 16, slots slot0 .. slot0 + nrow - 1
    {
        const uint16_t *src0 = v_new + row0 * row_elems;
        uint16_t *dst0 = v_cache + (int64_t)blk * row_elems * kBlockSize + slot0;
        for (int e = tid + kAppendThreads * part; e < row_elems; e += kAppendThreads * parts) {
            const uint16_t *src = src0 + e;
            uint16_t *dst = dst0 + (int64_t)e * kBlockSize;
            if (nrow == kBlockSize) {
                uint32_t x[8];
#pragma unroll
                for (int r = 0; r < 8; ++r)
                    x[r] = (uint32_t)src[(int64_t)(2 * r) * row_elems] | ((uint32_t)src[(int64_t)(2 * r + 1) * row_elems] << 16);
                u32x4 *d4 = reinterpret_cast<u32x4 *>(dst);
                if (blk_ok) {
                    d4[0] = u32x4{x[0], x[1], x[2], x[3]};
                    d4[1] = u32x4{x[4], x[5], x[6], x[7]};
                }
            } else {
                // all loads before the first store (one memory round trip instead of one per row); x[s] = value of
                // slot s of the block.  Quarters of the cache row (4 slots = 8 bytes) that the step covers whole are
                // written with one store each, the ragged ends slot by slot.
                uint16_t x[kBlockSize];
#pragma unroll
                for (int sl = 0; sl < kBlockSize; ++sl) {
                    const int r = sl - slot0;
                    x[sl] = (r >= 0 && r < nrow) ? src[(int64_t)r * row_elems] : (uint16_t)0;
                }
                uint16_t *row = dst - slot0;   // slot 0 of the cache row (32-byte aligned)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    if (!blk_ok) {
                    } else if (4 * q >= slot0 && 4 * q + 4 <= slot0 + nrow) {
                        *reinterpret_cast<u32x2 *>(row + 4 * q) =
                            u32x2{(uint32_t)x[4 * q] | ((uint32_t)x[4 * q + 1] << 16), (uint32_t)x[4 * q + 2] | ((uint32_t)x[4 * q + 3] << 16)};
                    } else {
#pragma unroll
                        for (int k = 0; k < 4; ++k) {
                            const int sl = 4 * q + k;
                            if (sl >= slot0 && sl < slot0 + nrow) row[sl] = x[sl];
                        }
                    }
                }
            }
        }
    }
}

hipError_t launch_kv_append(const void *k_new, const void *v_new, void *k_cache, void *v_cache, const int32_t *block_tables,
                            const int32_t *query_start_loc, const int32_t *ctx_lens, int num_seqs, int total_q, int Hkv,
                            int hd, int max_blocks_per_seq, int64_t num_blocks, int parts_opt, hipStream_t s)
{
    if (total_q <= 0 || num_seqs <= 0) return hipSuccess;
    const int parts = parts_opt > 0 ? std::min(parts_opt, 8) : std::max(1, std::min(2, Hkv * hd / (2 * kAppendThreads)));   // two for 8 kv heads x 128: measured best (1: 13.6 us, 2: 11.2, 4: 14.6 on 4,224 tokens)
    const unsigned grid = (unsigned)((total_q / kBlockSize + 2 * (int64_t)num_seqs + 1) * parts);
    hipLaunchKernelGGL(kv_append_kernel, dim3(grid), dim3(kAppendThreads), 0, s, (const uint16_t *)k_new,
                       (const uint16_t *)v_new, (uint16_t *)k_cache, (uint16_t *)v_cache, block_tables, query_start_loc,
                       ctx_lens, num_seqs, total_q, Hkv, hd, max_blocks_per_seq, num_blocks, parts);
    return hipGetLastError();
}


// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void fill_zero_kernel(int32_t *p, int64_t n)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) p[i] = 0;
}

hipError_t launch_fill_zero(int32_t *p, int64_t n, hipStream_t s)
{
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, p, n);
    return hipGetLastError();
}

hipError_t launch_decode(const KernArgs &a, hipStream_t s)
{
    if (a.p.static_runs <= 0 || a.p.dec_blocks <= 0) return hipSuccess;
    const dim3 grid((unsigned)((int64_t)a.p.static_runs * a.p.Hkv)), block(64);
    if (a.p.lean && a.p.hd == 128) {
        hipLaunchKernelGGL((decode_kernel_lean<128>), grid, block, 0, s, a);
        return hipGetLastError();
    }
    // KV blocks per softmax step: a wave keeps one step's tiles in flight, and 8 KiB per wave is what it takes
    // to saturate HBM with three waves per compute unit: one block for head_dim 128, two for head_dim 64
    // (measured: 56.9 % -> 72.2 % of the HBM peak on 256 sequences with head_dim 64; four blocks: 69.8 %)
    const int nbi = a.p.nbi ? a.p.nbi : (a.p.hd == 64 ? 2 : 1);
    if (a.p.hd == 128) {
        if (nbi == 2)
            hipLaunchKernelGGL((decode_kernel<128, 2>), grid, block, 0, s, a);
        else if (nbi == 4)
            hipLaunchKernelGGL((decode_kernel<128, 4>), grid, block, 0, s, a);
        else
            hipLaunchKernelGGL((decode_kernel<128, 1>), grid, block, 0, s, a);
    } else {
        if (nbi == 2)
            hipLaunchKernelGGL((decode_kernel<64, 2>), grid, block, 0, s, a);
        else if (nbi == 4)
            hipLaunchKernelGGL((decode_kernel<64, 4>), grid, block, 0, s, a);
        else
            hipLaunchKernelGGL((decode_kernel<64, 1>), grid, block, 0, s, a);
    }
    return hipGetLastError();
}

hipError_t launch_prefill(const KernArgs &a, hipStream_t s)
{
    if (a.p.n_tiles <= 0) return hipSuccess;
    const dim3 grid((unsigned)(a.p.pf_table ? (int64_t)a.p.pf_table * a.p.Hkv
                                            : (int64_t)a.p.n_tiles * a.p.Hkv * (a.p.pf_split > 0 ? a.p.pf_split : 1)));
    if (a.p.hd == 128 && a.p.pf_waves == 8 && a.p.lean)
        hipLaunchKernelGGL((prefill_kernel_lean<128>), grid, dim3(512), 0, s, a);
    else if (a.p.hd == 128 && a.p.pf_waves == 8)
        hipLaunchKernelGGL((prefill_kernel<128, 8>), grid, dim3(512), 0, s, a);
    else if (a.p.hd == 128)
        hipLaunchKernelGGL((prefill_kernel<128, 4>), grid, dim3(kPfThreads), 0, s, a);
    else
        hipLaunchKernelGGL((prefill_kernel<64, 4>), grid, dim3(kPfThreads), 0, s, a);
    return hipGetLastError();
}

hipError_t launch_mixed(const KernArgs &a, int num_cus, hipStream_t s)
{
    if (a.p.n_tiles <= 0 || a.p.static_runs <= 0) return hipErrorInvalidValue;
    const dim3 grid((unsigned)(2 * num_cus)), block(kPfThreads);
    if (a.p.hd == 128)
        hipLaunchKernelGGL((mixed_kernel<128>), grid, block, 0, s, a);
    else
        hipLaunchKernelGGL((mixed_kernel<64>), grid, block, 0, s, a);
    return hipGetLastError();
}

hipError_t launch_block_copy(const void *k_src, const void *v_src, void *k_dst, void *v_dst, const int64_t *src_ids,
                             const int64_t *dst_ids, int64_t num_pairs, int64_t block_bytes, int variant, hipStream_t s)
{
    if (num_pairs == 0) return hipSuccess;
    const int64_t block_vecs = block_bytes / 16;
    if (variant == 0) variant = 41;
    const int vpt = variant / 10;
    const int per_wg = kCopyThreads * vpt;
    const int slices = (int)((block_vecs + per_wg - 1) / per_wg);
    const dim3 grid((unsigned)(num_pairs * 2 * slices)), block(kCopyThreads);
#define OOCO_COPY(V, N)                                                                                              \
    hipLaunchKernelGGL((block_copy_kernel<V, N>), grid, block, 0, s, (const u32x4 *)k_src, (const u32x4 *)v_src,      \
                       (u32x4 *)k_dst, (u32x4 *)v_dst, src_ids, dst_ids, block_vecs, slices)
    switch (variant) {
    case 20: OOCO_COPY(2, false); break;
    case 21: OOCO_COPY(2, true); break;
    case 40: OOCO_COPY(4, false); break;
    case 80: OOCO_COPY(8, false); break;
    case 81: OOCO_COPY(8, true); break;
    case 10: OOCO_COPY(1, false); break;
    case 11: OOCO_COPY(1, true); break;
    default: OOCO_COPY(4, true); break;
    }
#undef OOCO_COPY
    return hipGetLastError();
}

}  // namespace ooco
