// Internal declarations shared by the host side (plan, ABI) and the kernel launchers of
// libooco.  Not part of the public ABI.
//
// Work decomposition (computed by every wave from a small cumulative array, no work lists):
//   decode  - the KV blocks of all decode sequences, laid end to end in sequence order, each
//             preceded by `piece_pad` empty units (the cost of starting a piece, in blocks), form one
//             line of `dec_blocks` units.  Its first `static_blocks` units are cut into
//             `static_runs` equal runs, one per launched wave and kv head; the rest into
//             `tail_runs` short runs that the waves fetch from a shared ticket counter when they
//             are done with their own run, so that faster waves (XCDs differ by several percent
//             in delivered bandwidth) end up streaming more blocks.  Where a run crosses sequence
//             boundaries it has several pieces.
//             cum[i] = number of line units before sequence i (cum[num_seqs] = dec_blocks).
//             A piece that does not cover its whole sequence writes a partial result into slot
//             (run index) + i; the last piece of a sequence to finish merges the slots (arrival
//             counter per sequence and kv head).
//   prefill - the P chunks (q_len > 1) are listed longest sequence first; cum[k] = number of query
//             tiles (tile_rows = 128 / (Hq/Hkv) rows each, all heads of a GQA group) before
//             chunk k of that list, cum[P+1+k] = its sequence index; one workgroup per
//             (tile, kv head), heavy tiles first.
//             When a batch has too few tiles to occupy the GPU, each (tile, kv head) is cut along
//             its keys into pf_split parts (one workgroup each) whose partial results are merged
//             by the part that finishes last, as for decode.
// The cumulative array travels inside the kernel arguments (no upload, no synchronisation) when
// the batch has at most kInlineSeqs sequences, else through a device buffer.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ooco {

constexpr int kBlockSize = 16;      // tokens per KV block (fixed by the cache layout)
constexpr int kPrefillCols = 128;   // (row, head) query columns per four-wave prefill workgroup (eight waves: 256)
constexpr int kInlineSeqs = 960;    // sequences whose cumulative array fits the kernel arguments
constexpr int kMaxPrefillSplit = 16; // parts a prefill tile's keys may be cut into
constexpr int kPrefillSplitUnits = 8192;   // (tile, kv head) pairs up to which the split is available
constexpr int kListEntries = 896;    // (tile, part) entries the plan's tile list may have (it lives in the kernel arguments)
constexpr int kSortedTiles = kListEntries;   // prefill tiles up to which the plan lists them one by one, most 64-key steps first
constexpr int kMixedStateInts = 4096;      // ints in front of (and including) the ticket counter that the mixed kernel keeps its claims and counters in

struct AttnParams {
    const uint16_t *q;
    const uint16_t *k_cache;
    const uint16_t *v_cache;
    const int32_t *block_tables;
    const int32_t *seq_lens;
    const int32_t *query_start_loc;
    const int32_t *ctx_lens;
    uint16_t *out;
    float *part_acc;            // [slots][Hq][hd]   un-normalised partial outputs
    float *part_ml;             // [slots][Hq][2]    (running max in log2 units, sum)
    int32_t *counters;          // [num_seqs][Hkv]   arrival counters, zero between calls
    const int32_t *cum_dev;     // cumulative array in device memory, or NULL (inline array used)
    uint64_t *trace;            // NULL, or [decode waves][4] time stamps (option "trace")
    int32_t Hq, Hkv, g, hd;
    int32_t max_blocks_per_seq;
    float scale_log2e;          // softmax scale * log2(e)
    int32_t num_seqs, total_q;
    int32_t dec_blocks, static_blocks, static_runs, tail_runs;   // decode run layout
    int32_t piece_pad;   // line units in front of every decode sequence's blocks (the cost of starting a piece)
    int32_t n_tiles;            // prefill: tiles per kv head
    int32_t pf_waves;           // prefill: waves per workgroup, 4 or 8 (a tile has 32 query columns per wave)
    int32_t num_pf;             // prefill: number of chunks (entries of the prefill array, see below)
    int32_t dec_cus;            // mixed kernel: compute units per XCD that run decode waves (the others run prefill tiles)
    int32_t nbi;                // tuning: KV blocks per softmax step of the decode kernel
    int16_t rotate_heads;       // tuning: kv head rotation across XCDs
    int16_t lean;               // mixed batches: the register-lean kernels (decode 128, prefill 8 waves x 192 registers)
    uint16_t xcd_cw[8];         // cumulative XCD weights of the static runs (RunLayout::cw); zeros = equal runs
    uint32_t queue_base;        // ticket value at which this launch's tail runs start
    uint32_t *queue;            // ticket counter for the tail runs (monotonic across launches)
    // prefill tiles split along the context (pf_split > 1): part j of unit u = (tile, kv head) writes
    // pf_acc[(u*pf_split + j)][128 columns][hd] and pf_ml[..][128][2]; pf_counters[u] counts arrivals
    float *pf_acc;
    float *pf_ml;
    int32_t *pf_counters;
    int32_t pf_split;
    // > 0: the prefill array continues with that many entries, one per (tile, part of its keys) in dispatch order
    // (see list_entry): the parts of all tiles ordered by their number of 64-key steps, the longest first, the parts
    // of one tile next to each other in part order.  Workgroup b works on entry b / Hkv for kv head b % Hkv; part j
    // of the tile whose part 0 is entry e0 writes partial slot (e0 + j) * Hkv + kv head, and pf_counters[e0 * Hkv +
    // kv head] counts the arrivals.  Every tile has its own number of parts (pf_split is the largest).
    int32_t pf_table;
};

// Entry of the tile list: chunk of the prefill array (10 bits), tile of the chunk (10 bits), part (6 bits), parts of
// the tile - 1 (6 bits).  A list exists only for batches of at most kSortedTiles tiles, so both indices fit.
__host__ __device__ inline int32_t list_entry(int chunk, int tile, int part, int parts)
{
    return (int32_t)((uint32_t)chunk | ((uint32_t)tile << 10) | ((uint32_t)part << 20) | ((uint32_t)(parts - 1) << 26));
}
__host__ __device__ inline int entry_chunk(int32_t e) { return (int)((uint32_t)e & 1023u); }
__host__ __device__ inline int entry_tile(int32_t e) { return (int)(((uint32_t)e >> 10) & 1023u); }
__host__ __device__ inline int entry_part(int32_t e) { return (int)(((uint32_t)e >> 20) & 63u); }
__host__ __device__ inline int entry_parts(int32_t e) { return (int)(((uint32_t)e >> 26) & 63u) + 1; }
static_assert(kSortedTiles <= 1024, "tile and chunk indices of a list entry have 10 bits");

struct KernArgs {
    AttnParams p;
    int32_t cum[kInlineSeqs + 1];
};
static_assert(sizeof(KernArgs) <= 4096, "kernel arguments must stay within 4 KiB");

// Launchers (ooco_kernels.hip).  `a.cum` must hold the decode resp. prefill cumulative array
// unless a.p.cum_dev is set.  Each returns the hipError_t of its launch.
hipError_t launch_decode(const KernArgs &a, hipStream_t s);
hipError_t launch_prefill(const KernArgs &a, hipStream_t s);
// One launch for a batch with both kinds of work: a.cum holds the decode array (num_seqs + 1 entries) followed by
// the prefill array (or a.p.cum_dev both, in that order); 2 * num_cus persistent workgroups.
hipError_t launch_mixed(const KernArgs &a, int num_cus, hipStream_t s);
// variant: tuning knob of the block-copy kernel (option "copy_variant"): 10 x 16-byte vectors per thread
// + 1 for non-temporal accesses; 0 = default
hipError_t launch_block_copy(const void *k_src, const void *v_src, void *k_dst, void *v_dst,
                             const int64_t *src_ids, const int64_t *dst_ids, int64_t num_pairs,
                             int64_t block_bytes, int variant, hipStream_t s);

// Pairs ordered by destination id (ooco_sort.hip): bytes of temporary storage for num_pairs, and the sort itself
// (dst_sorted / src_sorted: num_pairs int64 each; the low `bits` bits of the destination ids are the sort key).
hipError_t sort_pairs_temp_bytes(int64_t num_pairs, size_t *bytes);
hipError_t launch_sort_pairs(void *temp, size_t temp_bytes, const int64_t *dst_ids, int64_t *dst_sorted,
                             const int64_t *src_ids, int64_t *src_sorted, int64_t num_pairs, int bits, hipStream_t s);

hipError_t launch_kv_append(const void *k_new, const void *v_new, void *k_cache, void *v_cache, const int32_t *block_tables,
                            const int32_t *query_start_loc, const int32_t *ctx_lens, int num_seqs, int total_q, int Hkv,
                            int hd, int max_blocks_per_seq, int64_t num_blocks, int parts_opt, hipStream_t s);

// n int32 values at p become zero (a kernel, so that callers under stream capture record no memset node).
hipError_t launch_fill_zero(int32_t *p, int64_t n, hipStream_t s);

// Query rows of one prefill tile for a GQA group of g heads.
__host__ __device__ inline int32_t prefill_tile_rows(int32_t g, int32_t waves = 4)
{
    return 32 * waves / g > 0 ? 32 * waves / g : 1;
}

// n blocks cut into s equal runs, run k = [n*k/s, n*(k+1)/s): index of the run holding block x.
__host__ __device__ inline int32_t segment_of(int64_t x, int64_t s, int64_t n)
{
    return (int32_t)((((uint64_t)x + 1u) * (uint64_t)s - 1u) / (uint64_t)n);
}

// The two-level run layout of the decode line (host and device use the same functions).
// Static runs are equal by default.  With XCD weights (cw[kXcds-1] != 0; static_runs is then a
// multiple of kXcds) every group of kXcds consecutive runs shares its blocks in proportion to the
// weights: run 8p+k gets the share (cw[k] - cw[k-1]) / cw[7] of group p.  The decode kernel places
// run v on XCD v % kXcds, so a slower XCD can be given shorter runs.
constexpr int kXcds = 8;
// Default cost of starting a piece, in line units (= KV tiles of one kv head): measured on MI355X a wave
// needs about 3 us from one piece to the first tile of the next, the time it streams three 8 KiB tiles.
inline int default_piece_pad(int head_dim) { return 3 * 128 / head_dim; }
struct RunLayout {
    int32_t dec_blocks, static_blocks, static_runs, tail_runs;
    // cumulative weights of the runs of a group, kXcds values; all zero = equal runs.  (A pointer, not a copy: the
    // device reads the weights straight from the kernel arguments; a local copy indexed by a run-time value would
    // live in scratch memory.)
    const uint16_t *cw;
};
__host__ __device__ inline int32_t group_cut(const RunLayout &L, int32_t plo, int32_t phi, int32_t k)
{
    // first block of run k (0..kXcds) of the group that covers blocks [plo, phi)
    if (k <= 0) return plo;
    if (k >= kXcds) return phi;
    return plo + (int32_t)((int64_t)(phi - plo) * L.cw[k - 1] / L.cw[kXcds - 1]);
}
__host__ __device__ inline void run_bounds(const RunLayout &L, int32_t v, int32_t &lo, int32_t &hi)
{
    if (v < L.static_runs) {
        if (L.cw[kXcds - 1] == 0) {
            lo = (int32_t)((int64_t)L.static_blocks * v / L.static_runs);
            hi = (int32_t)((int64_t)L.static_blocks * (v + 1) / L.static_runs);
        } else {
            const int32_t groups = L.static_runs / kXcds, p = v / kXcds, k = v - p * kXcds;
            const int32_t plo = (int32_t)((int64_t)L.static_blocks * p / groups);
            const int32_t phi = (int32_t)((int64_t)L.static_blocks * (p + 1) / groups);
            lo = group_cut(L, plo, phi, k);
            hi = group_cut(L, plo, phi, k + 1);
        }
    } else {
        const int64_t t = v - L.static_runs, tb = L.dec_blocks - L.static_blocks;
        lo = L.static_blocks + (int32_t)(tb * t / L.tail_runs);
        hi = L.static_blocks + (int32_t)(tb * (t + 1) / L.tail_runs);
    }
}
__host__ __device__ inline int32_t run_of(const RunLayout &L, int64_t x)
{
    if (x >= L.static_blocks)
        return L.static_runs + segment_of(x - L.static_blocks, L.tail_runs, (int64_t)L.dec_blocks - L.static_blocks);
    if (L.cw[kXcds - 1] == 0) return segment_of(x, L.static_runs, L.static_blocks);
    const int32_t groups = L.static_runs / kXcds;
    const int32_t p = segment_of(x, groups, L.static_blocks);
    const int32_t plo = (int32_t)((int64_t)L.static_blocks * p / groups);
    const int32_t phi = (int32_t)((int64_t)L.static_blocks * (p + 1) / groups);
    int32_t k = 0;
    for (int32_t j = 1; j < kXcds; ++j) k += group_cut(L, plo, phi, j) <= x ? 1 : 0;
    return p * kXcds + k;
}

}  // namespace ooco
