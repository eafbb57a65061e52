// Host side of libooco: context, argument validation, the work-list planner and the C ABI.
#include "../../include/ooco.h"
#include "ooco_internal.h"

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

using namespace ooco;

namespace {

thread_local char g_create_error[512] = "";

constexpr size_t kDefaultWorkspace = 128ull << 20;
constexpr size_t kPlanInts = 1u << 21;       // staging for cumulative arrays of very large batches
constexpr size_t kCounterInts = 1u << 20;    // arrival counters: num_seqs * num_kv_heads must fit
constexpr size_t kTraceWaves = 1u << 16;     // decode waves the trace buffer can hold
constexpr int kProfSlots = 1024;             // profiled calls between two ooco_profile_read
constexpr int kProfEvents = 6;               // events per profiled call

// ooco_attn_mixed_static: everything the kernels need beyond the caller's tensors lives in one fixed device array
// (arrival counters at the front, partial results behind them); see include/ooco.h
constexpr size_t kStaticScratchBytes = 16u << 20;
constexpr size_t kStaticCounterInts = 1u << 16;
constexpr int kStaticMaxDevices = 64;

}  // namespace

// One copy per GPU, at an address of its own on each; zero when the code object is loaded.  In host code the
// name below is only a handle for hipGetSymbolAddress, never a device address.  (No `used` attribute: the
// compiler gives a static device variable that host code refers to an externally visible symbol, which is what
// the runtime looks up; marked `used` it stays a local symbol and the lookup aborts.)
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {
struct StaticDevice {
    void *ptr = nullptr;   // device address of `scratch` on this GPU
    int num_cus = 0;
};
std::mutex g_static_mu;
StaticDevice g_static_dev[kStaticMaxDevices];

// Address of this device's scratch array and its CU count, looked up once per device with that device current.
hipError_t static_device(StaticDevice &out, int &device)
{
    hipError_t e = hipGetDevice(&device);
    if (e != hipSuccess) return e;
    if (device < 0 || device >= kStaticMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_static_mu);
    StaticDevice &d = g_static_dev[device];
    if (!d.ptr) {
        void *ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!ptr) return hipErrorInvalidSymbol;
        int cus = 0;
        e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, device);
        if (e != hipSuccess) return e;
        d.num_cus = cus > 0 ? cus : 256;
        d.ptr = ptr;
    }
    out = d;
    return hipSuccess;
}
}  // namespace

namespace {
// Geometry and knobs the planner needs (no device state).
struct PlanGeometry {
    int Hq, Hkv, hd, BS, max_blocks_per_seq, num_cus;
    size_t ws_bytes;
    int64_t segments_opt;   // static runs; 0 = automatic
    int64_t tail_pct;       // share of the decode line handed out dynamically, in percent
    int64_t tail_blocks;    // KV blocks per dynamically fetched run
    int64_t pf_split_opt = 0;   // parts per prefill tile; 0 = automatic
    int64_t piece_pad = 0;      // line units charged for starting a piece (see build_plan)
    int64_t pf_waves_opt = 0;   // waves per prefill workgroup: 4, 8, or 0 = automatic
    int64_t lean_opt = 0;       // mixed batches: register-lean kernels (see HostPlan::lean)
    int64_t fused = 0;          // batches with both kinds of work run in the one-launch mixed kernel
    int64_t dec_cus_opt = 0;    // mixed kernel: compute units per XCD that decode; 0 = automatic
    int64_t pf_table_opt = 1;   // batches of at most kSortedTiles prefill tiles: tiles dispatched longest first across chunks
    uint16_t xcd_cw[kXcds] = {};   // cumulative XCD weights of the static runs; zeros = equal runs
};

// The compact plan: two cumulative arrays and a few scalars (see ooco_internal.h).
struct HostPlan {
    // (the two arrays live in storage the caller of build_plan provides, see PlanStorage)
    const int32_t *dcum = nullptr;   // [num_seqs+1] units of the decode line before each sequence (blocks + piece_pad per decode sequence)
    // prefill chunks, heaviest (most keys) first: pf[0..P] = query tiles before chunk k of that
    // order, pf[P+1+k] = sequence index of chunk k
    const int32_t *pf = nullptr;
    size_t pf_size = 0;              // 2 * num_pf + 1, + pf_table with the tile list
    int32_t pf_table = 0;            // > 0: pf goes on with that many (tile, part) entries in dispatch order (list_entry)
    int32_t num_pf = 0;
    int32_t dec_blocks = 0, static_blocks = 0, static_runs = 0, tail_runs = 0;   // in line units
    int32_t piece_pad = 0;
    int64_t kv_blocks = 0;       // KV blocks of all decode sequences
    uint16_t cw[kXcds] = {};     // XCD weights in force (RunLayout::cw)
    int32_t n_tiles = 0, total_q = 0, num_seqs = 0;
    int32_t pf_split = 1;        // parts a prefill tile's keys are cut into (with the tile list: the most any tile has)
    int64_t pf_slots = 0;        // partial-result slots of the split tiles per kv head (with the list: its leading entries that are parts)
    int32_t pf_waves = 4;        // waves per prefill workgroup (32 query columns each)
    // mixed batches (head_dim 128): the register-lean pair of kernels -- prefill workgroups of eight waves (176
    // registers, no software pipeline) and decode waves of 144 registers, four per compute unit -- so that a SIMD
    // holds two prefill waves and a decode wave at once
    int32_t lean = 0;
    int32_t dec_cus = 0;         // > 0: the batch runs in the mixed kernel with this many decoding compute units per XCD
    int64_t slots = 0;           // partial-result slots the decode kernel may touch
    // a batch with both kinds of work whose two kernels, one after the other, are estimated to take under 80 us: they
    // then run in sequence on the caller's stream (the fork and join of the second stream cost more than they gain)
    bool brief = false;
    int32_t nbi = 0;             // KV blocks per softmax step of the decode kernel that the plan asks for (0 = the kernel's default)
};

// XCD weights -> cumulative form; false if a weight is outside 1..255 or they differ by more than 4x.
bool xcd_weights_to_cw(const int32_t *w, uint16_t *cw)
{
    int32_t lo = 256, hi = 0, acc = 0;
    for (int k = 0; k < kXcds; ++k) {
        if (w[k] < 1 || w[k] > 255) return false;
        lo = std::min(lo, w[k]);
        hi = std::max(hi, w[k]);
        acc += w[k];
        cw[k] = (uint16_t)acc;
    }
    return hi <= 4 * lo;
}

size_t slot_bytes(const PlanGeometry &geo) { return (size_t)geo.Hq * (geo.hd + 2) * sizeof(float); }

// Where build_plan puts the plan's arrays: room for `seqs_cap` sequences, i.e. dcum [seqs_cap + 1],
// pf [2 * seqs_cap + 1 + kListEntries] and a work array order [seqs_cap].  build_plan itself allocates nothing.
struct PlanStorage {
    int32_t *dcum, *pf, *order;
    size_t seqs_cap;
};
PlanStorage carve_storage(int32_t *base, size_t seqs_cap)
{
    return PlanStorage{base, base + (seqs_cap + 1), base + (seqs_cap + 1) + (2 * seqs_cap + 1 + kListEntries), seqs_cap};
}
constexpr size_t storage_ints(size_t seqs_cap) { return (seqs_cap + 1) + (2 * seqs_cap + 1 + kListEntries) + seqs_cap; }

// Run layout of the decode block line (see ooco_internal.h): how many static runs, their XCD weights, the dynamic tail,
// the partial-result slots; fills out.static_runs / static_blocks / tail_runs / slots / cw / nbi.
// dec_blocks: units of the line (blocks + piece pads), kv_blocks: KV blocks of all decode sequences, dec_seqs: decode
// sequences that hold a block, lean: the batch runs the register-lean pair of kernels.
void plan_decode_runs(const PlanGeometry &geo, int num_seqs, int64_t dec_blocks, int64_t kv_blocks, int64_t dec_seqs, bool lean,
                      HostPlan &out)
{
    // static runs: by default three waves per CU (measured best on MI355X: enough loads in
    // flight to saturate HBM, few enough waves that start-up and partial results stay small)
    // and at least ~16 blocks of head_dim 128 per wave (a small batch is a chain of dependent blocks per wave:
    // one sequence of 512 blocks takes 27 us in 16 runs, 21 us in 32, 26 us in 64; eight sequences of 1121 blocks
    // 30 us in 36 runs, 25 us in 64)
    // (mixed kernel: eight decode waves on every decoding unit, one run each)
    int64_t wave_slots = lean ? std::max<int64_t>(1, (int64_t)geo.num_cus * 4 / geo.Hkv) : out.dec_cus == 99 ? std::max<int64_t>(1, (int64_t)geo.num_cus * 4 / geo.Hkv)
                               : out.dec_cus > 0 ? std::max<int64_t>(1, (int64_t)out.dec_cus * kXcds * 8 / geo.Hkv)
                                               : std::max<int64_t>(1, (int64_t)geo.num_cus * 3 / geo.Hkv);
    // A small batch (at most 36,864 (block, kv head) tiles of head_dim 128) cannot keep HBM busy anyway: what
    // counts is the length of every wave's chain of dependent steps.  Two blocks per step and at most half the
    // usual number of runs: one 8K-token sequence 21.0 -> 18.3 us, eight sequences (1121 blocks) 25.9 -> 21.4 us,
    // sixteen (2277 blocks) 35.2 -> 31.9 us; from 32 sequences (5296 blocks) on the usual layout is faster.
    // (between 24,576 and 36,864 tiles two thirds of the usual runs: 3814 blocks 49.2 -> 46.6 us; at 4739 blocks the
    // two layouts are level)
    // A batch of SHORT sequences (24 blocks = 384 tokens on average, or fewer) is a line of many short pieces, each
    // with its own start (query vectors, first tiles): four waves per compute unit hide those better than three, and
    // one block per step wastes no padded step.  512 sequences of 128 tokens 58.5 -> 50.9 us, 900 of 64 71.9 -> 62.0,
    // 2048 of 256 403 -> 382, 1024 of 384 285 -> 275; 4096 of 512 tokens are faster with three waves (1430 / 1449 us).
    const bool short_seqs = geo.hd == 128 && !lean && out.dec_cus == 0 && dec_seqs > 0 && kv_blocks <= 24 * dec_seqs;
    const bool small = geo.hd == 128 && !lean && out.dec_cus == 0 && !short_seqs && kv_blocks * geo.Hkv <= 36864;
    // (up to 16,384 tiles of them two blocks per step, and as many runs as sequences even if those hold fewer than 16
    // blocks: 32 sequences of 128 tokens 13.0 -> 10.2 us, 64 of 256 15.2 -> 13.2, 128 of 128 17.7 -> 14.8; 128 of 384
    // tokens, 24,576 tiles: 34.5 / 33.7 us)
    if (small) out.nbi = 2;
    if (short_seqs) out.nbi = kv_blocks * geo.Hkv <= 16384 ? 2 : 1;
    if (short_seqs && geo.segments_opt == 0) wave_slots = std::max<int64_t>(1, (int64_t)geo.num_cus * 4 / geo.Hkv);
    const int64_t min_blocks = 16 * 128 / geo.hd;
    if (small && geo.segments_opt == 0)
        wave_slots = std::max<int64_t>(1, kv_blocks * geo.Hkv <= 24576 ? wave_slots / 2 : wave_slots * 2 / 3);
    int64_t runs = geo.segments_opt > 0 ? geo.segments_opt
                                        : std::min<int64_t>(wave_slots, std::max<int64_t>((kv_blocks + min_blocks - 1) / min_blocks, short_seqs ? dec_seqs : 0));
    runs = std::max<int64_t>(1, std::min<int64_t>(runs, dec_blocks));
    for (;;) {
        // weighted runs come in groups of one run per XCD
        bool weighted = geo.xcd_cw[kXcds - 1] != 0 && runs >= kXcds && out.dec_cus == 0;
        if (weighted) runs -= runs % kXcds;
        // dynamic tail: only when a static run is much longer than a tail run
        int64_t tail_blk = 0, tails = 0;
        if (geo.tail_pct > 0 && geo.tail_blocks > 0 && dec_blocks / runs >= 4 * geo.tail_blocks && out.dec_cus == 0) {
            tail_blk = std::min<int64_t>(dec_blocks - runs, dec_blocks * std::min<int64_t>(geo.tail_pct, 90) / 100);
            tails = (tail_blk + geo.tail_blocks - 1) / geo.tail_blocks;
            if (tails == 0) tail_blk = 0;
        }
        // ... and only for runs long enough that no weight (they differ by at most 4x) empties one
        if (dec_blocks - tail_blk < 16 * runs) weighted = false;
        // partial slots: (run index) + seq < runs + tails + num_seqs; one run never splits a sequence
        const int64_t slots = (runs + tails > 1) ? runs + tails + num_seqs : 0;
        if ((size_t)slots * slot_bytes(geo) <= geo.ws_bytes || runs == 1) {
            if ((size_t)slots * slot_bytes(geo) > geo.ws_bytes) {   // a single run, no tail, needs no slots
                tail_blk = tails = 0;
            }
            out.static_runs = (int32_t)runs;
            for (int k = 0; k < kXcds; ++k) out.cw[k] = weighted ? geo.xcd_cw[k] : 0;
            out.static_blocks = (int32_t)(dec_blocks - tail_blk);
            out.tail_runs = (int32_t)tails;
            out.slots = (runs + tails > 1) ? runs + tails + num_seqs : 0;
            break;
        }
        runs = (runs + 1) / 2;
    }
}

// What build_plan knows of the batch's prefill part when it decides how the tiles' keys are cut into parts.
struct PrefillFacts {
    int64_t tiles, tile_steps, max_tile_steps;   // tiles per kv head, their 64-key steps in all, steps of the longest
    size_t n_order;                              // prefill chunks
    const int32_t *st;                           // with the tile list: steps of the listed tiles, in list order
    int pf_waves;
    int64_t dec_blocks, kv_blocks;               // decode part: units of its line, KV blocks
    double pf_pairs;                             // visible (query row, key) pairs of all chunks
};

// Prefill tiles cut along the context when there are too few of them to occupy the GPU, or when a few of them are far
// longer than the rest: chooses the parts of every tile, rewrites the tile list as (tile, part) entries, fills
// out.pf_split / pf_slots / pf_table / pf_size.  `tab` is the tile list inside the plan's prefill array.
void plan_prefill_parts(const PlanGeometry &geo, const PrefillFacts &f, int32_t *const tab, HostPlan &out)
{
    const int64_t tiles = f.tiles, tile_steps = f.tile_steps, max_tile_steps = f.max_tile_steps;
    const size_t n_order = f.n_order;
    const int32_t *const st = f.st;
    const int pf_waves = f.pf_waves;
    const int64_t dec_blocks = f.dec_blocks, kv_blocks = f.kv_blocks;
    const double pf_pairs = f.pf_pairs;
    const int BS = geo.BS;
    const int64_t units = tiles * geo.Hkv;
    int64_t split = 1;
    const size_t part_bytes = (size_t)(32 * pf_waves) * (geo.hd + 2) * sizeof(float);
    const size_t left = geo.ws_bytes - std::min(geo.ws_bytes, ((size_t)out.slots * slot_bytes(geo) + 255) / 256 * 256);
    const double cus = (double)geo.num_cus;
    // Estimated time in microseconds of a launch of w workgroups in all, the longest of them `longest` 64-key steps,
    // fitted to sweeps of 28 batches of equal chunks x 8 forced splits on MI355X (the choice is within 2.5 % of the best
    // forced split on every one of them, and better than any forced split on chunks of unequal contexts).  A workgroup's step takes 1.08 us while at most every other compute unit
    // holds a workgroup, 1.3 us with one workgroup on every unit, 1.95 us with two (the unit then completes a step
    // every 0.98 us, and further workgroups queue behind); the last workgroup of a tile merges the partial results
    // of its parts, which costs 2 us + 0.03 us per workgroup of the launch up to two per unit + 0.04 us for every
    // further one (their partial results then meet in memory at the same time).  The launch takes as long as its
    // average workgroup at the launch's occupancy or as its longest one beside what the others leave of a unit
    // (a chunk on a long context among chunks on short ones), whichever is more.
    auto step_us = [&](double r) {   // r = workgroups per compute unit
        if (r <= 0.5) return 1.08;
        if (r <= 1.0) return 1.08 + 0.44 * (r - 0.5);
        if (r <= 2.0) return 1.3 + 0.65 * (r - 1.0);
        return 0.975 * r;
    };
    // (the longest workgroup shares its unit with as many others as the launch has per unit, but no more than the
    // launch's work provides over its lifetime; a workgroup's start-up and epilogue, 2.5 us, come once per
    // workgroup that a unit holds at a time)
    // A compute unit holds ONE prefill workgroup, not two, when the workgroups have eight waves or when decode waves
    // share its registers (a batch with both kinds of work): such a workgroup counts as two, and beside decode
    // waves it never has a unit to itself.
    // (... a decode part, that is, which by its bytes lasts at least half as long as the prefill part by its FLOPs)
    const bool beside_decode = dec_blocks > 0 && !geo.fused &&
                               (double)kv_blocks * BS * 2.0 * geo.Hkv * geo.hd * 2.0 / 6.8e12 >= 0.5 * 4.0 * geo.Hq * geo.hd * pf_pairs / 1.05e15;
    const double wg_weight = beside_decode || pf_waves == 8 ? 2.0 : 1.0;
    const double all_steps = (double)tile_steps * geo.Hkv;   // 64-key steps of all workgroups together
    // w workgroups, w_big of them at least half as long as the longest one (`longest` steps), w_parts of them parts
    // of split tiles (which write partial results that the last of them merges)
    auto est = [&](double w, double w_big, double w_parts, double longest) {
        const bool merges = w_parts > 0.0;
        const double r = wg_weight * w / cus;
        const double beside = beside_decode ? 2.0 : std::min(std::min(r, 2.0), wg_weight * all_steps / (longest * cus));
        const double merge = merges ? 2.0 + 0.03 * std::min(w_parts, 2.0 * cus) + 0.04 * std::max(0.0, w_parts - 2.0 * cus) : 0.0;
        double average = all_steps / w * step_us(r);
        if (r > 2.0 && merges) {
            // more workgroups than fit at a time: the units work through them at full occupancy, and the long ones
            // go in rounds (up to four rounds count whole: the parts of a split tile are equally long, and 2.5
            // rounds of them take as long as 3; whole tiles of many lengths pack better than that)
            double rounds = wg_weight * w_big / (2.0 * cus);
            if (rounds <= 4.0) rounds = std::ceil(rounds - 1e-9);
            average = std::max(average, rounds * longest * 1.95);
        }
        return std::max(average, longest * step_us(beside)) + merge + 2.5 * std::ceil(std::min(r, 2.0));
    };
    // With the tile list every tile gets parts by its own number of steps: the longest tile k parts, the others as
    // many as keep their parts no longer than that tile's (a tile of a short chunk stays whole beside a long one).
    // Without it (more than kSortedTiles tiles, or a forced value) every tile gets the same number.
    auto parts_of = [&](int64_t s, int64_t k, bool by_steps) -> int64_t {
        if (!by_steps) return std::min(k, s);
        const int64_t longest = (max_tile_steps + k - 1) / k;
        return std::min((s + longest - 1) / longest, s);
    };
    auto entries_of = [&](int64_t k, bool by_steps, int64_t *big = nullptr, int64_t *split_ones = nullptr) -> int64_t {
        const int64_t longest = (max_tile_steps + k - 1) / k;
        int64_t e = 0, b = 0, sp = 0;
        for (int64_t i = 0; i < tiles; ++i) {
            const int64_t parts = parts_of(st[i], k, by_steps);
            e += parts;
            if (2 * ((st[i] + parts - 1) / parts) >= longest) b += parts;
            if (parts > 1) sp += parts;
        }
        if (big) *big = b;
        if (split_ones) *split_ones = sp;
        return e;
    };
    // what a list of e entries, e_parts of them parts of split tiles, must fit: the kernel arguments; the counters
    // and the workspace (the parts come first in the list, and an entry's index is its partial-result slot)
    auto list_fits = [&](int64_t e, int64_t e_parts) {
        return e <= kListEntries && 2 * n_order + 1 + (size_t)e <= (size_t)kInlineSeqs + 1 &&
               e_parts * geo.Hkv <= kPrefillSplitUnits && (size_t)e_parts * geo.Hkv * part_bytes <= left;
    };
    bool by_steps = false;
    if (units <= kPrefillSplitUnits) {
        if (geo.pf_split_opt > 0) {
            split = std::min<int64_t>(std::min<int64_t>(geo.pf_split_opt, kMaxPrefillSplit), max_tile_steps);
        } else if (out.pf_table) {
            by_steps = true;
            int64_t big = 0, split_ones = 0;
            (void)entries_of(1, true, &big);
            double best = est((double)units, (double)(big * geo.Hkv), 0.0, (double)max_tile_steps) * 0.97;   // a split must win 3 %
            // (a launch of two or more workgroups per unit whose longest tile is no longer than the units' average
            // load cannot gain from more workgroups)
            const bool full = wg_weight * (double)units >= 2.0 * cus && wg_weight * all_steps / cus * 0.975 >= (double)max_tile_steps * 1.95;
            for (int64_t k = 2; !full && k <= kMaxPrefillSplit && k <= max_tile_steps; ++k) {
                const int64_t e = entries_of(k, true, &big, &split_ones);
                if (!list_fits(e, split_ones)) break;
                const double t = est((double)(e * geo.Hkv), (double)(big * geo.Hkv), (double)(split_ones * geo.Hkv),
                                     (double)((max_tile_steps + k - 1) / k));
                if (t < best) {
                    best = t;
                    split = k;
                } else if (k >= split + 4) {
                    break;   // (four values in a row without a gain: the estimate only grows from here)
                }
            }
        } else {
            const double steps = (double)tile_steps / (double)tiles;   // (every tile the same number of parts)
            double best = est((double)units, (double)units, 0.0, (double)max_tile_steps) * 0.97;
            for (int64_t sp = 2; sp <= kMaxPrefillSplit && sp <= (int64_t)steps; ++sp) {
                const double t = est((double)(units * sp), (double)(units * sp), (double)(units * sp), (double)((max_tile_steps + sp - 1) / sp));
                if (t < best) {
                    best = t;
                    split = sp;
                }
            }
        }
    }
    int64_t forced_parts = 0;
    if (out.pf_table && split > 1 && !by_steps && !list_fits(entries_of(split, false, nullptr, &forced_parts), forced_parts)) {
        // a forced number of parts whose list would not fit: the same parts without the list (chunk by chunk)
        out.pf_size -= (size_t)out.pf_table;
        out.pf_table = 0;
    }
    if (!out.pf_table)
        while (split > 1 && (size_t)units * (size_t)split * part_bytes > left) --split;
    if (out.pf_table && split > 1) {
        // (tile, part) entries: first the parts of the split tiles, then the whole tiles, each by decreasing number of
        // steps; the parts of a tile stay together, in part order; ties keep the chunk order and, inside a chunk,
        // the later tile first.  Sorted as plain numbers.
        uint64_t keys[kListEntries];
        size_t e = 0;
        int64_t most = 1;
        for (int64_t i = 0; i < tiles; ++i) {
            const int64_t s_i = st[i], parts = parts_of(s_i, split, by_steps), per = (s_i + parts - 1) / parts;
            most = std::max(most, parts);
            for (int64_t j = 0; j < parts; ++j)
                keys[e++] = ((uint64_t)(parts == 1) << 52) | ((uint64_t)(0xFFFFF - per) << 32) | ((uint32_t)entry_chunk(tab[i]) << 22) |
                            ((uint32_t)(1023 - entry_tile(tab[i])) << 12) | ((uint32_t)j << 6) | (uint32_t)(parts - 1);
        }
        std::sort(keys, keys + e);
        for (size_t i = 0; i < e; ++i) {
            const uint32_t k = (uint32_t)keys[i];
            tab[i] = list_entry((int)(k >> 22), 1023 - (int)((k >> 12) & 1023u), (int)((k >> 6) & 63u), (int)(k & 63u) + 1);
        }
        out.pf_size += e - (size_t)out.pf_table;
        out.pf_table = (int32_t)e;
        split = most;
        for (size_t i = 0; i < e && entry_parts(tab[i]) > 1; ++i) ++out.pf_slots;   // (the parts come first)
    } else if (split > 1) {
        out.pf_slots = tiles * split;
    }
    out.pf_split = (int32_t)split;
    // A launch of at most two four-wave workgroups per compute unit is one round: the hardware gives workgroups w
    // and w + CUs the same unit, and two workgroups that share a unit each advance at half its rate.  The tile
    // list then pairs the tile with the most steps with the one with the fewest, and so on (the second half of
    // the list ascending), so that every unit gets about the same number of steps: on MI355X one chunk of 2048
    // rows on 1662 cached tokens 102.1 -> 99.6 us, two of 1024 rows 67.5 -> 65.1 us (option "prefill_sorted" = 2
    // keeps the plain descending order).
    if (out.pf_table && geo.pf_table_opt == 1 && split == 1 && out.pf_waves == 4 && geo.num_cus % geo.Hkv == 0) {
        const int64_t half = geo.num_cus / geo.Hkv;   // tile positions whose workgroups arrive first on their unit
        if (tiles > half && tiles <= 2 * half) std::reverse(tab + half, tab + tiles);
    }
}

// Validates the length arrays and builds the plan.  Pure host code, no allocation.
ooco_status build_plan(const PlanGeometry &geo, int num_seqs, const int32_t *h_seq_lens,
                       const int32_t *h_query_start_loc, const int32_t *h_ctx_lens, const PlanStorage &store,
                       HostPlan &out, char *err)
{
    auto bad = [&](ooco_status code, const char *fmt, ...) __attribute__((format(printf, 3, 4))) {
        va_list ap;
        va_start(ap, fmt);
        vsnprintf(err, 512, fmt, ap);
        va_end(ap);
        return code;
    };
    out = HostPlan();
    if (num_seqs < 0) return bad(OOCO_EINVAL, "ooco_plan: num_seqs=%d", num_seqs);
    if (num_seqs > 0 && (!h_seq_lens || !h_query_start_loc || !h_ctx_lens))
        return bad(OOCO_EINVAL, "ooco_plan: NULL length array");
    const int BS = geo.BS;
    if (num_seqs > 0 && h_query_start_loc[0] != 0)
        return bad(OOCO_ESHAPE, "ooco_plan: query_start_loc[0]=%d, expected 0", h_query_start_loc[0]);
    if ((size_t)num_seqs > store.seqs_cap)
        return bad(OOCO_ENOMEM, "ooco_plan: %d sequences exceed the plan storage (%zu)", num_seqs, store.seqs_cap);
    out.num_seqs = num_seqs;
    int32_t *const dcum = store.dcum, *const pf = store.pf, *const order = store.order;
    out.dcum = dcum;
    out.pf = pf;
    std::fill(dcum, dcum + num_seqs + 1, 0);
    // The decode line: every decode sequence contributes piece_pad units followed by one unit per KV block.  The
    // runs cut the line into equal lengths, so a run that starts several pieces streams correspondingly fewer
    // blocks (starting a piece costs a wave about as long as streaming three 8 KiB tiles).
    int64_t dec_blocks = 0, kv_blocks = 0, tiles = 0, tile_steps = 0, max_tile_steps = 1;
    int64_t dec_seqs = 0;    // decode sequences that hold at least one block
    double pf_pairs = 0.0;   // visible (query row, key) pairs of all prefill chunks
    const int64_t pad = geo.piece_pad;
    // Waves per prefill workgroup.  Eight waves share every K/V tile staged in LDS among 256 query columns instead
    // of 128, which halves the traffic from L2 into the compute units.  Measured on MI355X it is no faster (that
    // traffic is not what bounds the kernel) and its 220-register waves leave no room for decode waves beside
    // them, so four waves are the default; eight (head_dim 128 only) stay selectable.
    // The register-lean pair for batches with both kinds of work (lean_opt 2 = whenever the batch is mixed; 1 = when
    // it pays: every compute unit gets at least one eight-wave prefill workgroup -- counting the parts of 16 or more
    // 64-key steps that tiles on a long context can be cut into --, and the prefill part, by itself,
    // would take between 0.30 and 4 times as long as the decode part -- estimated from the batch's FLOPs and bytes
    // at 1.05 PFLOP/s and 6.8 TB/s).  Measured on MI355X, 32/8 heads, 128 decode sequences of 1.4 GB in all: beside
    // 2 x 2048 rows 319 -> 291 us, beside 8 x 512 rows 286 -> 270 us, but beside 4 x 512 rows 257 -> 263 us and beside
    // 1 x 512 rows 242 -> 266 us (alone the lean decode kernel is 3 % slower than the stand-alone one, which a short
    // prefill part does not repay; alone the lean prefill kernel is 5 % slower, so a batch that is nearly all prefill
    // keeps the stand-alone pair too); the long-context batch of 64/8 heads 1.75 -> 1.62 ms.
    bool lean = false;
    if (geo.lean_opt && geo.hd == 128 && !geo.fused && num_seqs > 0) {
        const int rows8 = prefill_tile_rows(geo.Hq / geo.Hkv, 8);
        int64_t n_dec = 0, tiles8 = 0, wgs8 = 0, dec_blk = 0;
        double pairs = 0.0;
        for (int i = 0; i < num_seqs; ++i) {
            const int64_t ql = (int64_t)h_query_start_loc[i + 1] - h_query_start_loc[i];
            n_dec += ql == 1;
            if (ql == 1) dec_blk += ((int64_t)h_seq_lens[i] + BS - 1) / BS;
            if (ql > 1) {
                const int64_t t8 = (ql + rows8 - 1) / rows8, parts = ((int64_t)h_seq_lens[i] + 63) / 64 / 16;
                tiles8 += t8;
                wgs8 += t8 * std::min<int64_t>(std::max<int64_t>(parts, 1), kMaxPrefillSplit);
                pairs += (double)ql * (double)h_ctx_lens[i] + (double)ql * (double)(ql + 1) / 2.0;
            }
        }
        const double t_pf = 4.0 * geo.Hq * geo.hd * pairs / 1.05e15;
        const double t_dec = (double)dec_blk * BS * 2.0 * geo.Hkv * geo.hd * 2.0 / 6.8e12;
        const bool pays = wgs8 * geo.Hkv >= (int64_t)geo.num_cus && t_pf >= 0.30 * t_dec && t_pf <= 4.0 * t_dec;
        lean = n_dec > 0 && tiles8 > 0 && (geo.lean_opt >= 2 || pays);
    }
    out.lean = lean;
    const int pf_waves = geo.hd == 128 && (geo.pf_waves_opt == 8 || lean) ? 8 : 4;
    out.pf_waves = pf_waves;
    const int tile_rows = prefill_tile_rows(geo.Hq / geo.Hkv, pf_waves);
    for (int i = 0; i < num_seqs; ++i) {
        const int64_t ql = (int64_t)h_query_start_loc[i + 1] - h_query_start_loc[i];
        if (ql < 0) return bad(OOCO_ESHAPE, "ooco_plan: query_start_loc decreases at sequence %d", i);
        if (h_ctx_lens[i] < 0 || h_seq_lens[i] < 0)
            return bad(OOCO_ESHAPE, "ooco_plan: negative length at sequence %d", i);
        if ((int64_t)h_ctx_lens[i] + ql != h_seq_lens[i])
            return bad(OOCO_ESHAPE, "ooco_plan: sequence %d has ctx_len %d + q_len %lld != seq_len %d", i,
                       h_ctx_lens[i], (long long)ql, h_seq_lens[i]);
        const int64_t nb = ((int64_t)h_seq_lens[i] + BS - 1) / BS;
        if (nb > geo.max_blocks_per_seq)
            return bad(OOCO_ESHAPE, "ooco_plan: sequence %d needs %lld blocks > max_blocks_per_seq %d", i,
                       (long long)nb, geo.max_blocks_per_seq);
        if (ql == 1) {
            dec_blocks += nb + pad;
            kv_blocks += nb;
            dec_seqs += nb > 0;
        }
        if (ql > 1) {
            pf_pairs += (double)ql * (double)h_ctx_lens[i] + (double)ql * (double)(ql + 1) / 2.0;
            tiles += (ql + tile_rows - 1) / tile_rows;
            for (int64_t t0 = 0; t0 < ql; t0 += tile_rows) {    // 64-key steps of every tile
                const int64_t nstep = ((int64_t)h_ctx_lens[i] + std::min<int64_t>(ql, t0 + tile_rows) + 63) / 64;
                tile_steps += nstep;
                max_tile_steps = std::max(max_tile_steps, nstep);
            }
        }
        if (dec_blocks > 0x7FFFFFFF / 2 || tiles > 0x7FFFFFFF / 128)
            return bad(OOCO_ESHAPE, "ooco_plan: batch too large");
        dcum[(size_t)i + 1] = (int32_t)dec_blocks;
    }
    out.total_q = num_seqs > 0 ? h_query_start_loc[num_seqs] : 0;
    out.dec_blocks = (int32_t)dec_blocks;
    out.kv_blocks = kv_blocks;
    out.piece_pad = (int32_t)pad;
    out.n_tiles = (int32_t)tiles;
    // prefill chunks in order of decreasing sequence length: workgroups are dispatched in index
    // order, so the long ones start first and the short ones fill the end
    size_t n_order = 0;
    for (int i = 0; i < num_seqs; ++i)
        if (h_query_start_loc[i + 1] - h_query_start_loc[i] > 1) order[n_order++] = i;
    // (equal lengths keep their batch order; std::sort with the index as tie-break needs no temporary buffer)
    std::sort(order, order + n_order, [&](int32_t x, int32_t y) {
        return h_seq_lens[x] != h_seq_lens[y] ? h_seq_lens[x] > h_seq_lens[y] : x < y;
    });
    out.num_pf = (int32_t)n_order;
    out.pf_size = 2 * n_order + 1;
    std::fill(pf, pf + out.pf_size, 0);
    for (size_t k = 0; k < n_order; ++k) {
        const int64_t ql = (int64_t)h_query_start_loc[order[k] + 1] - h_query_start_loc[order[k]];
        pf[k + 1] = pf[k] + (int32_t)((ql + tile_rows - 1) / tile_rows);
        pf[n_order + 1 + k] = order[k];
    }
    int32_t st[kSortedTiles];   // with the tile list: 64-key steps of the listed tiles, in list order
    auto steps_of = [&](int32_t e) -> int64_t {   // 64-key steps of the tile a list entry names
        const int i = order[entry_chunk(e)];
        const int64_t ql = (int64_t)h_query_start_loc[i + 1] - h_query_start_loc[i], t0 = (int64_t)entry_tile(e) * tile_rows;
        return ((int64_t)h_ctx_lens[i] + std::min<int64_t>(ql, t0 + tile_rows) + 63) / 64;
    };
    // A launch of few tiles is as long as its unluckiest compute unit is busy, and the hardware hands workgroups out
    // in index order to whichever unit has room: the tiles of ALL chunks go out by decreasing number of 64-key
    // steps (a chunk on a short context has fewer steps in its last tile than one on a long context in its first).
    // (only while the longer array still travels in the kernel arguments)
    if (geo.pf_table_opt && tiles > 0 && tiles <= kSortedTiles && 2 * n_order + 1 + (size_t)tiles <= (size_t)kInlineSeqs + 1) {
        // (ties keep the chunk order and, inside a chunk, the later tile first; sorted as plain numbers: steps
        // descending in the high half, chunk and descending tile below)
        int32_t *const tab = pf + out.pf_size;
        uint64_t keys[kSortedTiles];
        size_t n = 0;
        for (size_t k = 0; k < n_order; ++k)
            for (int32_t t = pf[k + 1] - pf[k] - 1; t >= 0; --t)
                keys[n++] = ((uint64_t)(0xFFFFF - steps_of(list_entry((int)k, t, 0, 1))) << 32) | (uint32_t)((k << 10) | (uint32_t)(1023 - t));
        std::sort(keys, keys + n);
        for (size_t i = 0; i < n; ++i) {
            tab[i] = list_entry((int)((uint32_t)keys[i] >> 10), 1023 - (int)((uint32_t)keys[i] & 1023u), 0, 1);
            st[i] = (int32_t)(0xFFFFF - (keys[i] >> 32));
        }
        out.pf_size += n;
        out.pf_table = (int32_t)n;
    }

    // ---- short mixed batches.  Measured on MI355X (32/8 heads): 1 x 64 rows + 4 decode sequences 50.7 us side by
    // side, 44.9 us in sequence; 1 x 128 + 8: 49.0 / 46.9; 2 x 128 + 32: 84.9 / 81.3; 4 x 128 + 64: 129.8 / 139.7 -- and
    // enqueueing the forked call costs the host 41 us against 8 us.  Estimate: each kernel's roofline time plus its
    // fixed cost (15 us decode, 12 us prefill).
    if (dec_blocks > 0 && tiles > 0) {
        const double t_dec = (double)kv_blocks * BS * 2.0 * geo.Hkv * geo.hd * 2.0 / 6.8e12 + 15e-6;
        const double t_pf = 4.0 * geo.Hq * geo.hd * pf_pairs / 1.05e15 + 12e-6;
        out.brief = t_dec + t_pf < 80e-6;
    }
    // ---- one launch for both kinds of work: how many compute units of every XCD decode.  The decode part is
    // bound by HBM and reaches its bandwidth from a part of the units; the prefill part is bound by the matrix
    // cores and takes as long as its share of the units makes it.  The prefill units are sized so that they
    // finish with the decode stream (estimated from rates measured on MI355X: 6.8 TB/s, and 1.05 PFLOP/s on all
    // units), leaving the decode side at least kMinDecCus units per XCD; whoever finishes first helps the other.
    const int cus_per_xcd = std::max(1, geo.num_cus / kXcds);
    if (geo.fused && pf_waves == 4 && dec_blocks > 0 && tiles > 0 && cus_per_xcd >= 4 && geo.num_cus % kXcds == 0) {
        constexpr int kMinDecCus = 10;
        const double t_dec = (double)kv_blocks * BS * 2.0 * geo.Hkv * geo.hd * 2.0 / 6.8e12;
        const double t_pf = 4.0 * geo.Hq * geo.hd * pf_pairs / 1.05e15;
        int pf_cus = (int)std::ceil(cus_per_xcd * t_pf / std::max(t_dec, 1e-9));
        pf_cus = std::max(1, std::min(pf_cus, cus_per_xcd - std::min(kMinDecCus, cus_per_xcd / 2)));
        int dec = cus_per_xcd - pf_cus;
        if (geo.dec_cus_opt > 0) dec = (int)std::min<int64_t>(geo.dec_cus_opt, cus_per_xcd - 1);
        if (geo.dec_cus_opt == 99) dec = 99;   // every unit runs both kinds (one workgroup each): for measurements
        out.dec_cus = dec;
    }
    // ---- run layout of the decode block line (see plan_decode_runs)
    if (dec_blocks > 0) plan_decode_runs(geo, num_seqs, dec_blocks, kv_blocks, dec_seqs, lean, out);
    // ---- prefill tiles cut along the context (see plan_prefill_parts)
    if (tiles > 0) {
        const PrefillFacts facts = {tiles, tile_steps, max_tile_steps, n_order, st, pf_waves, dec_blocks, kv_blocks, pf_pairs};
        plan_prefill_parts(geo, facts, store.pf + (2 * (size_t)out.num_pf + 1), out);
    }
    return OOCO_OK;
}

// Pieces of the decode line as the kernel walks them (host mirror of the device logic).
struct Piece {
    int32_t seq, blk_begin, blk_end, slot, run;
};
std::vector<Piece> enumerate_pieces(const HostPlan &pl)
{
    std::vector<Piece> v;
    const RunLayout L = {pl.dec_blocks, pl.static_blocks, pl.static_runs, pl.tail_runs, pl.cw};
    for (int32_t k = 0; k < pl.static_runs + pl.tail_runs; ++k) {
        int32_t lo, hi;
        run_bounds(L, k, lo, hi);
        int seq = 0;
        while (pl.dcum[(size_t)seq + 1] <= lo) ++seq;
        int64_t pos = lo;
        while (pos < hi) {
            while (pl.dcum[(size_t)seq + 1] <= pos) ++seq;
            const int64_t cs = pl.dcum[(size_t)seq], ce = pl.dcum[(size_t)seq + 1];
            const int64_t stop = std::min<int64_t>(hi, ce);
            const int64_t first = cs + pl.piece_pad, begin = std::max(pos, first);   // the blocks start at `first`
            if (begin < stop) {
                const bool whole = begin == first && stop == ce;
                v.push_back(Piece{seq, (int32_t)(begin - first), (int32_t)(stop - first), whole ? -1 : (int32_t)(k + seq),
                                  (int32_t)k});
            }
            pos = stop;
            ++seq;
        }
    }
    return v;
}
}  // namespace

struct ooco_ctx {
    int Hq = 0, Hkv = 0, g = 0, hd = 0, BS = 0;
    int64_t num_blocks = 0;
    int max_blocks_per_seq = 0;
    float scale = 0.f;
    int device = 0;
    int num_cus = 256;

    void *ws = nullptr;
    size_t ws_bytes = 0;
    bool own_ws = false;

    // streams that calls have put work on which uses the context's memory (workspace, counters, plan, sort buffer):
    // what ooco_ctx_destroy and ooco_trace_read wait for.  More than kMaxStreams different ones: the whole device.
    static constexpr int kMaxStreams = 4;
    hipStream_t used_streams[kMaxStreams] = {};
    int n_used_streams = 0;
    bool many_streams = false;
    hipStream_t last_stream = nullptr;
    void note_stream(hipStream_t st)
    {
        last_stream = st;
        for (int i = 0; i < n_used_streams; ++i)
            if (used_streams[i] == st) return;
        if (n_used_streams < kMaxStreams)
            used_streams[n_used_streams++] = st;
        else
            many_streams = true;
    }
    // Waits for everything the context has enqueued (its side stream is joined into the caller's stream by every call).
    hipError_t wait_for_own_work()
    {
        if (many_streams) return hipDeviceSynchronize();
        hipError_t first = hipSuccess;
        for (int i = 0; i < n_used_streams; ++i) {
            const hipError_t e = hipStreamSynchronize(used_streams[i]);
            if (first == hipSuccess) first = e;
        }
        return first;
    }

    int32_t *plan_h = nullptr;   // pinned host staging for batches beyond kInlineSeqs sequences
    int32_t *plan_d = nullptr;   // device copy of the two cumulative arrays
    int32_t *counters = nullptr; // arrival counters [kCounterInts], zero between calls
    hipEvent_t upload_done = nullptr;
    bool upload_pending = false;

    // current plan (its arrays live in plan_store)
    std::vector<int32_t> plan_store;
    HostPlan plan;
    bool plan_valid = false;
    bool plan_dirty = false;
    bool plan_one_shot = false;   // planned inside ooco_attn_mixed from device lengths
    bool plan_made = false;       // ctx->plan holds the numbers of the last plan made (current or used up)
    int64_t opt_plan_persistent = 0;   // an explicit plan serves every following call of the same shape

    // options
    int64_t opt_segments = 0;
    int64_t opt_tail_pct = 0;
    int64_t opt_tail_blocks = 8;
    uint32_t queue_base = 0;       // ticket value the next launch's tail runs start at
    int64_t opt_nbi = 0;
    int64_t opt_trace = 0;
    int64_t opt_rotate = 1;
    int64_t opt_pf_split = 0;
    int64_t opt_pf_table = 1;       // few prefill tiles: dispatched by decreasing number of steps across chunks
    int opt_copy_variant = 0;       // block copy: 10 x vectors per thread + non-temporal flag, 0 = default
    int64_t opt_decode_first = 1;   // mixed batches: enqueue the decode kernel before the prefill kernel
    int64_t opt_piece_pad = 0;   // set at creation: 3 tiles of head_dim 128
    int32_t *pf_counters = nullptr;   // [kPrefillSplitUnits] arrival counters of split prefill tiles, zero between calls
    uint16_t xcd_cw[kXcds] = {};   // option "xcd_weights"
    int64_t opt_overlap = 1;
    int64_t opt_copy_sort = 1;      // block copy: order the pairs by destination id on the device (0 never, 1 from kCopySortMin pairs, 2 always)
    void *sort_buf = nullptr;       // [2 * sort_cap int64 (sorted dst, sorted src)] + temporary storage of the sort
    int64_t sort_cap = 0;           // pairs the buffer holds
    size_t sort_temp_bytes = 0;
    int64_t opt_append_parts = 0;   // KV append: workgroups per (sequence, block) pair, 0 = automatic
    int64_t opt_lean = 1;           // mixed batches: the register-lean kernels (0 never, 1 automatic, 2 always)
    int64_t opt_pf_waves = 0;       // waves per prefill workgroup: 0 = automatic, 4, 8
    int64_t opt_fused = 0;          // mixed batches in one launch (mixed kernel) instead of two kernels on two streams
    int64_t opt_dec_cus = 0;        // mixed kernel: decoding compute units per XCD, 0 = automatic
    hipStream_t side_stream = nullptr;   // default priority; carries the prefill kernel of mixed batches
    hipEvent_t fork_ev = nullptr, join_ev = nullptr;
    uint64_t *trace_d = nullptr;   // [kTraceWaves][4] decode-wave time stamps
    int64_t trace_waves = 0;       // waves of the last traced call
    int64_t opt_profile = 0;

    // per-kernel timing (option "profile"): kProfEvents events per call (decode start/end, prefill start/end,
    // call start/end), each pair recorded on the stream its kernel runs on
    std::vector<hipEvent_t> prof_ev;
    int64_t prof_calls = 0;

    KernArgs kargs;                      // staging of the kernel arguments of the current call
    std::vector<int32_t> h_len_scratch;   // for the plan-less path
    mutable char err[512] = "";
};

namespace {

ooco_status fail(const ooco_ctx *ctx, ooco_status code, const char *fmt, ...)
{
    char *dst = ctx ? ctx->err : g_create_error;
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(dst, 512, fmt, ap);
    va_end(ap);
    return code;
}


}  // namespace

extern "C" {

ooco_status ooco_ctx_create(ooco_ctx **out, int num_q_heads, int num_kv_heads, int head_dim, int block_size,
                            int64_t num_blocks, int max_blocks_per_seq, float softmax_scale, void *workspace,
                            size_t workspace_bytes)
{
    if (!out) return fail(nullptr, OOCO_EINVAL, "ooco_ctx_create: out is NULL");
    *out = nullptr;
    if (num_q_heads <= 0 || num_kv_heads <= 0 || num_q_heads % num_kv_heads != 0)
        return fail(nullptr, OOCO_ESHAPE, "ooco_ctx_create: num_q_heads=%d must be a positive multiple of num_kv_heads=%d",
                    num_q_heads, num_kv_heads);
    if (num_q_heads / num_kv_heads > 16)
        return fail(nullptr, OOCO_ESHAPE, "ooco_ctx_create: GQA group size %d > 16 is not supported",
                    num_q_heads / num_kv_heads);
    if (head_dim != 64 && head_dim != 128)
        return fail(nullptr, OOCO_ESHAPE, "ooco_ctx_create: head_dim=%d (supported: 64, 128)", head_dim);
    if (block_size != kBlockSize)
        return fail(nullptr, OOCO_ESHAPE, "ooco_ctx_create: block_size=%d (supported: %d)", block_size, kBlockSize);
    if (num_blocks <= 0 || max_blocks_per_seq <= 0)
        return fail(nullptr, OOCO_EINVAL, "ooco_ctx_create: num_blocks and max_blocks_per_seq must be positive");
    if (workspace && workspace_bytes == 0)
        return fail(nullptr, OOCO_EINVAL, "ooco_ctx_create: caller workspace given with workspace_bytes == 0");
    if (workspace && (reinterpret_cast<uintptr_t>(workspace) & 255u))
        return fail(nullptr, OOCO_EINVAL, "ooco_ctx_create: workspace must be 256-byte aligned");

    ooco_ctx *c = new (std::nothrow) ooco_ctx();
    if (!c) return fail(nullptr, OOCO_ENOMEM, "ooco_ctx_create: out of host memory");
    c->Hq = num_q_heads;
    c->Hkv = num_kv_heads;
    c->g = num_q_heads / num_kv_heads;
    c->hd = head_dim;
    c->BS = block_size;
    c->num_blocks = num_blocks;
    c->max_blocks_per_seq = max_blocks_per_seq;
    c->scale = softmax_scale > 0.f ? softmax_scale : 1.0f / std::sqrt((float)head_dim);

    hipError_t e = hipGetDevice(&c->device);
    if (e == hipSuccess) {
        int cus = 0;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, c->device) == hipSuccess && cus > 0)
            c->num_cus = cus;
    }
    c->opt_piece_pad = default_piece_pad(head_dim);
    if (e == hipSuccess) {
        if (workspace) {
            c->ws = workspace;
            c->ws_bytes = workspace_bytes;
        } else {
            c->ws_bytes = workspace_bytes ? workspace_bytes : kDefaultWorkspace;
            e = hipMalloc(&c->ws, c->ws_bytes);
            c->own_ws = (e == hipSuccess);
        }
    }
    if (e == hipSuccess) e = hipHostMalloc((void **)&c->plan_h, kPlanInts * sizeof(int32_t), hipHostMallocDefault);
    if (e == hipSuccess) e = hipMalloc((void **)&c->plan_d, kPlanInts * sizeof(int32_t));
    if (e == hipSuccess) e = hipMalloc((void **)&c->counters, kCounterInts * sizeof(int32_t));
    if (e == hipSuccess) e = hipMemset(c->counters, 0, kCounterInts * sizeof(int32_t));
    if (e == hipSuccess) e = hipMalloc((void **)&c->pf_counters, kPrefillSplitUnits * sizeof(int32_t));
    if (e == hipSuccess) e = hipMemset(c->pf_counters, 0, kPrefillSplitUnits * sizeof(int32_t));
    if (e == hipSuccess) e = hipEventCreateWithFlags(&c->upload_done, hipEventDisableTiming);
    if (e == hipSuccess) e = hipStreamCreateWithFlags(&c->side_stream, hipStreamNonBlocking);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&c->fork_ev, hipEventDisableTiming);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&c->join_ev, hipEventDisableTiming);
    if (e != hipSuccess) {
        fail(nullptr, e == hipErrorOutOfMemory ? OOCO_ENOMEM : OOCO_EHIP, "ooco_ctx_create: %s", hipGetErrorString(e));
        ooco_status st = e == hipErrorOutOfMemory ? OOCO_ENOMEM : OOCO_EHIP;
        (void)hipGetLastError();
        if (c->upload_done) (void)hipEventDestroy(c->upload_done);
        if (c->fork_ev) (void)hipEventDestroy(c->fork_ev);
        if (c->join_ev) (void)hipEventDestroy(c->join_ev);
        if (c->side_stream) (void)hipStreamDestroy(c->side_stream);
        if (c->counters) (void)hipFree(c->counters);
        if (c->pf_counters) (void)hipFree(c->pf_counters);
        if (c->plan_d) (void)hipFree(c->plan_d);
        if (c->plan_h) (void)hipHostFree(c->plan_h);
        if (c->own_ws && c->ws) (void)hipFree(c->ws);
        delete c;
        return st;
    }
    *out = c;
    return OOCO_OK;
}

ooco_status ooco_ctx_destroy(ooco_ctx *ctx)
{
    if (!ctx) return OOCO_OK;
    if (ctx->upload_pending) (void)hipEventSynchronize(ctx->upload_done);
    (void)ctx->wait_for_own_work();
    if (ctx->side_stream) (void)hipStreamSynchronize(ctx->side_stream);
    if (ctx->upload_done) (void)hipEventDestroy(ctx->upload_done);
    if (ctx->fork_ev) (void)hipEventDestroy(ctx->fork_ev);
    if (ctx->join_ev) (void)hipEventDestroy(ctx->join_ev);
    if (ctx->side_stream) (void)hipStreamDestroy(ctx->side_stream);
    for (hipEvent_t x : ctx->prof_ev)
        if (x) (void)hipEventDestroy(x);
    if (ctx->trace_d) (void)hipFree(ctx->trace_d);
    if (ctx->sort_buf) (void)hipFree(ctx->sort_buf);
    if (ctx->counters) (void)hipFree(ctx->counters);
    if (ctx->pf_counters) (void)hipFree(ctx->pf_counters);
    if (ctx->plan_d) (void)hipFree(ctx->plan_d);
    if (ctx->plan_h) (void)hipHostFree(ctx->plan_h);
    if (ctx->own_ws && ctx->ws) (void)hipFree(ctx->ws);
    delete ctx;
    return OOCO_OK;
}

ooco_status ooco_trace_read(ooco_ctx *ctx, uint64_t *stamps, int64_t cap_waves, int64_t *waves)
{
    if (!ctx) return OOCO_EINVAL;
    if (!ctx->trace_d) return fail(ctx, OOCO_EINVAL, "ooco_trace_read: option \"trace\" was never enabled");
    hipError_t e = ctx->wait_for_own_work();
    const int64_t n = std::min<int64_t>(cap_waves, ctx->trace_waves);
    if (e == hipSuccess && stamps && n > 0)
        e = hipMemcpy(stamps, ctx->trace_d, (size_t)n * 4 * sizeof(uint64_t), hipMemcpyDeviceToHost);
    if (e != hipSuccess) return fail(ctx, OOCO_EHIP, "ooco_trace_read: %s", hipGetErrorString(e));
    if (waves) *waves = ctx->trace_waves;
    return OOCO_OK;
}

ooco_status ooco_profile_read_calls(ooco_ctx *ctx, double *per_call_ms, int64_t cap, double *ms_sum, int64_t *calls)
{
    if (!ctx) return OOCO_EINVAL;
    if (cap < 0 || (cap > 0 && !per_call_ms)) return fail(ctx, OOCO_EINVAL, "ooco_profile_read_calls: bad per-call buffer");
    double sum[3] = {0.0, 0.0, 0.0};
    for (int64_t c = 0; c < ctx->prof_calls; ++c) {
        hipEvent_t *ev = ctx->prof_ev.data() + kProfEvents * c;
        // wait for the call's last record on either stream
        hipError_t e = hipEventSynchronize(ev[5]);
        if (e == hipSuccess) e = hipEventSynchronize(ev[3]);
        if (e == hipSuccess) e = hipEventSynchronize(ev[1]);
        // (prefill start, prefill end), (decode start, decode end), (call start, call end)
        static const int pairs[3][2] = {{2, 3}, {0, 1}, {4, 5}};
        for (int k = 0; k < 3 && e == hipSuccess; ++k) {
            float ms = 0.f;
            e = hipEventElapsedTime(&ms, ev[pairs[k][0]], ev[pairs[k][1]]);
            sum[k] += ms;
            if (c < cap) per_call_ms[3 * c + k] = ms;
        }
        if (e != hipSuccess) return fail(ctx, OOCO_EHIP, "ooco_profile_read: %s", hipGetErrorString(e));
    }
    if (ms_sum) ms_sum[0] = sum[0], ms_sum[1] = sum[1], ms_sum[2] = sum[2];
    if (calls) *calls = ctx->prof_calls;
    ctx->prof_calls = 0;
    return OOCO_OK;
}

ooco_status ooco_profile_read(ooco_ctx *ctx, double *ms_sum, int64_t *calls)
{
    return ooco_profile_read_calls(ctx, nullptr, 0, ms_sum, calls);
}

const char *ooco_last_error(const ooco_ctx *ctx) { return ctx ? ctx->err : g_create_error; }

ooco_status ooco_set_option(ooco_ctx *ctx, const char *name, int64_t value)
{
    if (!ctx) return OOCO_EINVAL;
    if (!name) return fail(ctx, OOCO_EINVAL, "ooco_set_option: name is NULL");
    if (value < 0) return fail(ctx, OOCO_EINVAL, "ooco_set_option: %s must be >= 0", name);
    if (!strcmp(name, "decode_segments"))
        ctx->opt_segments = value;
    else if (!strcmp(name, "decode_tail_pct"))
        ctx->opt_tail_pct = value;
    else if (!strcmp(name, "decode_tail_blocks"))
        ctx->opt_tail_blocks = value;
    else if (!strcmp(name, "prefill_split"))
        ctx->opt_pf_split = value;
    else if (!strcmp(name, "prefill_sorted"))
        ctx->opt_pf_table = value;
    else if (!strcmp(name, "decode_first"))
        ctx->opt_decode_first = value;
    else if (!strcmp(name, "prefill_waves")) {
        if (value != 0 && value != 4 && value != 8)
            return fail(ctx, OOCO_EINVAL, "ooco_set_option: prefill_waves must be 0 (automatic), 4 or 8");
        ctx->opt_pf_waves = value;
    }
    else if (!strcmp(name, "mixed_lean"))
        ctx->opt_lean = value;
    else if (!strcmp(name, "mixed_fused"))
        ctx->opt_fused = value;
    else if (!strcmp(name, "mixed_dec_cus"))
        ctx->opt_dec_cus = value;
    else if (!strcmp(name, "decode_piece_pad")) {
        if (value > 64) return fail(ctx, OOCO_EINVAL, "ooco_set_option: decode_piece_pad must be 0..64");
        ctx->opt_piece_pad = value;
    }
    else if (!strcmp(name, "trace")) {
        if (value && !ctx->trace_d) {
            hipError_t e = hipMalloc((void **)&ctx->trace_d, kTraceWaves * 4 * sizeof(uint64_t));
            if (e != hipSuccess) return fail(ctx, OOCO_ENOMEM, "ooco_set_option: trace buffer: %s", hipGetErrorString(e));
        }
        ctx->opt_trace = value;
        return OOCO_OK;
    } else if (!strcmp(name, "copy_variant")) {
        static const int64_t known[] = {0, 10, 11, 20, 21, 40, 41, 80, 81};
        if (std::find(std::begin(known), std::end(known), value) == std::end(known))
            return fail(ctx, OOCO_EINVAL, "ooco_set_option: copy_variant must be one of 0, 10, 11, 20, 21, 40, 41, 80, 81");
        ctx->opt_copy_variant = (int)value;
        return OOCO_OK;
    } else if (!strcmp(name, "copy_sort")) {
        ctx->opt_copy_sort = value;
        return OOCO_OK;
    } else if (!strcmp(name, "append_parts")) {
        ctx->opt_append_parts = value;
        return OOCO_OK;
    } else if (!strcmp(name, "plan_persistent")) {
        ctx->opt_plan_persistent = value;
        return OOCO_OK;
    } else if (!strcmp(name, "overlap")) {
        ctx->opt_overlap = value;
        return OOCO_OK;
    } else if (!strcmp(name, "rotate_heads")) {
        ctx->opt_rotate = value;
        return OOCO_OK;
    } else if (!strcmp(name, "xcd_weights")) {
        // eight relative weights, one byte each, XCD 0 in the lowest byte; 0 = equal runs
        int32_t w[kXcds];
        for (int k = 0; k < kXcds; ++k) w[k] = (int32_t)(((uint64_t)value >> (8 * k)) & 0xFFu);
        if (value == 0)
            for (int k = 0; k < kXcds; ++k) ctx->xcd_cw[k] = 0;
        else if (!xcd_weights_to_cw(w, ctx->xcd_cw)) {
            for (int k = 0; k < kXcds; ++k) ctx->xcd_cw[k] = 0;
            return fail(ctx, OOCO_EINVAL, "ooco_set_option: xcd_weights needs eight bytes in 1..255 that differ by at most 4x");
        }
    } else if (!strcmp(name, "decode_nbi")) {
        ctx->opt_nbi = value;
        return OOCO_OK;
    } else if (!strcmp(name, "profile")) {
        ctx->opt_profile = value;
        ctx->prof_calls = 0;
        return OOCO_OK;   // does not invalidate the plan
    }
    else
        return fail(ctx, OOCO_EINVAL, "ooco_set_option: unknown option '%s'", name);
    ctx->plan_valid = false;
    return OOCO_OK;
}

ooco_status ooco_plan(ooco_ctx *ctx, int num_seqs, const int32_t *h_seq_lens, const int32_t *h_query_start_loc,
                      const int32_t *h_ctx_lens)
{
    if (!ctx) return OOCO_EINVAL;
    ctx->plan_valid = false;
    PlanGeometry geo;
    geo.Hq = ctx->Hq;
    geo.Hkv = ctx->Hkv;
    geo.hd = ctx->hd;
    geo.BS = ctx->BS;
    geo.max_blocks_per_seq = ctx->max_blocks_per_seq;
    geo.num_cus = ctx->num_cus;
    geo.ws_bytes = ctx->ws_bytes;
    geo.segments_opt = ctx->opt_segments;
    geo.tail_pct = ctx->opt_tail_pct;
    geo.tail_blocks = ctx->opt_tail_blocks;
    geo.pf_split_opt = ctx->opt_pf_split;
    geo.piece_pad = ctx->opt_piece_pad;
    geo.pf_waves_opt = ctx->opt_pf_waves;
    geo.lean_opt = ctx->opt_lean;
    geo.fused = ctx->opt_fused && ctx->opt_overlap;
    geo.dec_cus_opt = ctx->opt_dec_cus;
    geo.pf_table_opt = ctx->opt_pf_table;
    for (int k = 0; k < kXcds; ++k) geo.xcd_cw[k] = ctx->xcd_cw[k];
    const size_t cap = (size_t)std::max(num_seqs, 0);
    if (ctx->plan_store.size() < storage_ints(cap)) ctx->plan_store.resize(storage_ints(cap));
    ooco_status st = build_plan(geo, num_seqs, h_seq_lens, h_query_start_loc, h_ctx_lens,
                                carve_storage(ctx->plan_store.data(), cap), ctx->plan, ctx->err);
    if (st != OOCO_OK) return st;
    if ((size_t)num_seqs * ctx->Hkv > kCounterInts - kMixedStateInts || 3 * ((size_t)num_seqs + 1) + kListEntries > kPlanInts)
        return fail(ctx, OOCO_ENOMEM, "ooco_plan: %d sequences exceed the context's counter/plan buffers", num_seqs);
    ctx->plan_valid = true;
    ctx->plan_made = true;
    ctx->plan_dirty = true;
    ctx->plan_one_shot = false;
    return OOCO_OK;
}

ooco_status ooco_plan_dry_run(int num_q_heads, int num_kv_heads, int head_dim, int block_size, int max_blocks_per_seq,
                              int num_cus, size_t workspace_bytes, int64_t decode_segments, int64_t decode_tail_pct,
                              int64_t decode_tail_blocks, int num_seqs,
                              const int32_t *h_seq_lens, const int32_t *h_query_start_loc, const int32_t *h_ctx_lens,
                              int32_t *decode_pieces_out, int64_t decode_cap, int32_t *prefill_tiles_out,
                              int64_t prefill_cap, int64_t *counts, char *msg, size_t msg_cap,
                              const int32_t *xcd_weights, int64_t prefill_split, int64_t decode_piece_pad)
{
    char err[512] = "";
    ooco_status st = OOCO_OK;
    HostPlan pl;
    std::vector<int32_t> store;
    if (num_q_heads <= 0 || num_kv_heads <= 0 || num_q_heads % num_kv_heads || (head_dim != 64 && head_dim != 128) ||
        block_size != kBlockSize || max_blocks_per_seq <= 0 || num_cus <= 0 || decode_segments < 0 ||
        decode_tail_pct < 0 || decode_tail_blocks < 0 || prefill_split < 0 || decode_piece_pad > 64) {
        snprintf(err, sizeof err, "ooco_plan_dry_run: bad geometry");
        st = OOCO_ESHAPE;
    } else {
        PlanGeometry geo;
        geo.Hq = num_q_heads;
        geo.Hkv = num_kv_heads;
        geo.hd = head_dim;
        geo.BS = block_size;
        geo.max_blocks_per_seq = max_blocks_per_seq;
        geo.num_cus = num_cus;
        geo.ws_bytes = workspace_bytes;
        geo.segments_opt = decode_segments;
        geo.tail_pct = decode_tail_pct;
        geo.tail_blocks = decode_tail_blocks;
        geo.pf_split_opt = prefill_split;
        geo.lean_opt = 1;   // (the default of a context)
        geo.piece_pad = decode_piece_pad < 0 ? default_piece_pad(head_dim) : decode_piece_pad;
        if (xcd_weights && !xcd_weights_to_cw(xcd_weights, geo.xcd_cw)) {
            snprintf(err, sizeof err, "ooco_plan_dry_run: xcd_weights needs eight values in 1..255 that differ by at most 4x");
            st = OOCO_EINVAL;
        }
        if (st == OOCO_OK) {
            const size_t cap = (size_t)std::max(num_seqs, 0);
            store.resize(storage_ints(cap));
            st = build_plan(geo, num_seqs, h_seq_lens, h_query_start_loc, h_ctx_lens, carve_storage(store.data(), cap), pl, err);
        }
    }
    if (msg && msg_cap) snprintf(msg, msg_cap, "%s", err);
    if (st != OOCO_OK) return st;
    const std::vector<Piece> pieces = enumerate_pieces(pl);
    if (counts) {
        counts[0] = (int64_t)pieces.size();
        counts[1] = pl.n_tiles;
        counts[2] = pl.static_runs;
        counts[3] = pl.slots;
        counts[4] = pl.tail_runs;
        counts[5] = pl.pf_split;
    }
    if (decode_pieces_out)
        for (int64_t i = 0; i < std::min<int64_t>(decode_cap, (int64_t)pieces.size()); ++i) {
            const Piece &d = pieces[(size_t)i];
            int32_t *o = decode_pieces_out + 5 * i;
            o[0] = d.seq, o[1] = d.blk_begin, o[2] = d.blk_end, o[3] = d.slot, o[4] = d.run;
        }
    if (prefill_tiles_out) {
        // in dispatch order, derived from the plan's arrays the way the prefill kernel derives them
        const int tile_rows = prefill_tile_rows(num_q_heads / num_kv_heads, pl.pf_waves);
        const int32_t *const pf = pl.pf;
        const int P = pl.num_pf;
        // (with the tile list a tile is listed where its first part is dispatched)
        const int64_t n_list = pl.pf_table ? pl.pf_table : pl.n_tiles;
        int64_t idx = 0;
        for (int64_t pos = 0; pos < n_list && idx < prefill_cap; ++pos) {
            int k, t, parts;
            if (pl.pf_table) {
                const int32_t e = pf[2 * P + 1 + pos];
                if (entry_part(e) != 0) continue;
                k = entry_chunk(e);
                t = entry_tile(e);
                parts = entry_parts(e);
            } else {
                k = (int)(std::upper_bound(pf, pf + P + 1, (int32_t)pos) - pf) - 1;
                t = (pf[k + 1] - 1) - (int)pos;
                parts = pl.pf_split;
            }
            const int i = pf[P + 1 + k];
            const int q0 = h_query_start_loc[i], ql = h_query_start_loc[i + 1] - q0, t0 = t * tile_rows;
            int32_t *o = prefill_tiles_out + 5 * idx++;
            o[0] = i, o[1] = q0 + t0, o[2] = std::min(tile_rows, ql - t0), o[3] = h_ctx_lens[i] + t0;
            o[4] = (int32_t)std::min<int64_t>(parts, ((int64_t)o[3] + o[2] + 63) / 64);
        }
    }
    return OOCO_OK;
}

ooco_status ooco_plan_info(const ooco_ctx *ctx, int64_t *decode_waves, int64_t *prefill_tiles, int64_t *decode_blocks,
                           int64_t *workspace_used, int64_t *prefill_parts)
{
    if (!ctx) return OOCO_EINVAL;
    if (!ctx->plan_made) return fail(ctx, OOCO_EINVAL, "ooco_plan_info: no plan has been made");
    if (decode_waves) *decode_waves = ctx->plan.static_runs;
    if (prefill_tiles) *prefill_tiles = ctx->plan.n_tiles;
    if (decode_blocks) *decode_blocks = ctx->plan.kv_blocks;
    if (workspace_used) {
        size_t bytes = (size_t)ctx->plan.slots * (size_t)ctx->Hq * (ctx->hd + 2) * sizeof(float);
        if (ctx->plan.pf_split > 1)
            bytes = (bytes + 255) / 256 * 256 + (size_t)ctx->plan.pf_slots * ctx->Hkv * (size_t)(32 * ctx->plan.pf_waves) *
                                                    (ctx->hd + 2) * sizeof(float);
        *workspace_used = (int64_t)bytes;
    }
    if (prefill_parts) *prefill_parts = ctx->plan.n_tiles > 0 ? ctx->plan.pf_split : 1;
    return OOCO_OK;
}

ooco_status ooco_plan_kernels(const ooco_ctx *ctx, char *names, size_t cap)
{
    if (!ctx) return OOCO_EINVAL;
    if (!ctx->plan_made) return fail(ctx, OOCO_EINVAL, "ooco_plan_kernels: no plan has been made");
    if (!names || cap == 0) return fail(ctx, OOCO_EINVAL, "ooco_plan_kernels: no buffer");
    const HostPlan &pl = ctx->plan;
    const bool dec = pl.static_runs > 0, pf = pl.n_tiles > 0;
    const int nbi = ctx->opt_nbi ? (int)ctx->opt_nbi : pl.nbi ? pl.nbi : (ctx->hd == 64 ? 2 : 1);
    char d[64] = "", f[64] = "";
    if (dec && pf && pl.dec_cus > 0)
        snprintf(d, sizeof d, "mixed_kernel<%d>", ctx->hd);
    else {
        if (dec && pl.lean)
            snprintf(d, sizeof d, "decode_kernel_lean<%d>", ctx->hd);
        else if (dec)
            snprintf(d, sizeof d, "decode_kernel<%d, %d>", ctx->hd, nbi);
        if (pf && pl.lean && pl.pf_waves == 8)
            snprintf(f, sizeof f, "prefill_kernel_lean<%d>", ctx->hd);
        else if (pf)
            snprintf(f, sizeof f, "prefill_kernel<%d, %d>", ctx->hd, pl.pf_waves);
    }
    snprintf(names, cap, "%s%s%s", d, d[0] && f[0] ? ";" : "", f);
    return OOCO_OK;
}

ooco_status ooco_attn_mixed(ooco_ctx *ctx, const void *q, const void *k_cache, const void *v_cache,
                            const int32_t *block_tables, const int32_t *seq_lens, const int32_t *query_start_loc,
                            const int32_t *ctx_lens, void *out, int num_seqs, int total_q_tokens, void *stream)
{
    if (!ctx) return OOCO_EINVAL;
    if (num_seqs < 0 || total_q_tokens < 0)
        return fail(ctx, OOCO_EINVAL, "ooco_attn_mixed: negative size (num_seqs=%d, total_q_tokens=%d)", num_seqs,
                    total_q_tokens);
    if (num_seqs == 0 || total_q_tokens == 0) return OOCO_OK;
    if (!q || !k_cache || !v_cache || !block_tables || !seq_lens || !query_start_loc || !ctx_lens || !out)
        return fail(ctx, OOCO_EINVAL, "ooco_attn_mixed: NULL pointer argument");
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    ctx->note_stream(s);

    if (!ctx->plan_valid) {
        // No host plan for this batch: fetch the lengths and plan here (costs one stream sync).
        ctx->h_len_scratch.resize((size_t)3 * num_seqs + 1);
        int32_t *h_seq = ctx->h_len_scratch.data();
        int32_t *h_ctx = h_seq + num_seqs;
        int32_t *h_qsl = h_ctx + num_seqs;
        hipError_t e = hipMemcpyAsync(h_seq, seq_lens, sizeof(int32_t) * num_seqs, hipMemcpyDeviceToHost, s);
        if (e == hipSuccess) e = hipMemcpyAsync(h_ctx, ctx_lens, sizeof(int32_t) * num_seqs, hipMemcpyDeviceToHost, s);
        if (e == hipSuccess)
            e = hipMemcpyAsync(h_qsl, query_start_loc, sizeof(int32_t) * (num_seqs + 1), hipMemcpyDeviceToHost, s);
        if (e == hipSuccess) e = hipStreamSynchronize(s);
        if (e != hipSuccess) return fail(ctx, OOCO_EHIP, "ooco_attn_mixed: reading lengths: %s", hipGetErrorString(e));
        ooco_status st = ooco_plan(ctx, num_seqs, h_seq, h_qsl, h_ctx);
        if (st != OOCO_OK) return st;
        ctx->plan_one_shot = true;
    }
    const HostPlan &pl = ctx->plan;
    if (pl.num_seqs != num_seqs || pl.total_q != total_q_tokens) {
        if (ctx->plan_one_shot) {   // the plan made above from the device's lengths does not outlive this call
            ctx->plan_one_shot = false;
            ctx->plan_valid = false;
        }
        return fail(ctx, OOCO_ESHAPE, "ooco_attn_mixed: plan was made for %d sequences / %d query tokens, call has %d / %d",
                    pl.num_seqs, pl.total_q, num_seqs, total_q_tokens);
    }

    // The cumulative arrays ride in the kernel arguments; only very large batches need a copy.
    const size_t n_cum = (size_t)num_seqs + 1, n_pf = pl.pf_size;
    // (the mixed kernel, pl.dec_cus > 0, takes both arrays at once; the two separate kernels one each)
    const bool inline_cum = pl.dec_cus > 0 ? n_cum + n_pf <= (size_t)kInlineSeqs + 1
                                           : n_cum <= (size_t)kInlineSeqs + 1 && n_pf <= (size_t)kInlineSeqs + 1;
    if (!inline_cum && ctx->plan_dirty) {
        if (ctx->upload_pending) (void)hipEventSynchronize(ctx->upload_done);
        memcpy(ctx->plan_h, pl.dcum, n_cum * sizeof(int32_t));
        memcpy(ctx->plan_h + n_cum, pl.pf, n_pf * sizeof(int32_t));
        hipError_t e = hipMemcpyAsync(ctx->plan_d, ctx->plan_h, (n_cum + n_pf) * sizeof(int32_t), hipMemcpyHostToDevice, s);
        if (e == hipSuccess) e = hipEventRecord(ctx->upload_done, s);
        if (e != hipSuccess) return fail(ctx, OOCO_EHIP, "ooco_attn_mixed: plan upload: %s", hipGetErrorString(e));
        ctx->upload_pending = true;
    }
    ctx->plan_dirty = false;

    KernArgs &ka = ctx->kargs;
    AttnParams &p = ka.p;
    p.q = static_cast<const uint16_t *>(q);
    p.k_cache = static_cast<const uint16_t *>(k_cache);
    p.v_cache = static_cast<const uint16_t *>(v_cache);
    p.block_tables = block_tables;
    p.seq_lens = seq_lens;
    p.query_start_loc = query_start_loc;
    p.ctx_lens = ctx_lens;
    p.out = static_cast<uint16_t *>(out);
    p.part_acc = static_cast<float *>(ctx->ws);
    p.part_ml = p.part_acc + (size_t)pl.slots * ctx->Hq * ctx->hd;
    p.counters = ctx->counters;
    {
        const size_t dec_floats = ((size_t)pl.slots * ctx->Hq * (ctx->hd + 2) + 63) / 64 * 64;   // 256-byte aligned
        const size_t parts = (size_t)pl.pf_slots * ctx->Hkv;   // (what the planner checked against the workspace)
        p.pf_acc = static_cast<float *>(ctx->ws) + dec_floats;
        p.pf_ml = p.pf_acc + parts * (size_t)(32 * pl.pf_waves) * ctx->hd;
        p.pf_counters = ctx->pf_counters;
        p.pf_split = pl.pf_split;
        p.pf_table = pl.pf_table;
        // (what the kernels will address, once more against what the context owns: a plan that does not fit is an error of
        // this library, reported instead of launched)
        const size_t pf_end = (dec_floats + parts * (size_t)(32 * pl.pf_waves) * (ctx->hd + 2)) * sizeof(float);
        // (arrival counters: one per part-0 slot with the tile list, one per (tile, kv head) without it)
        const size_t pf_counters_used = pl.pf_table ? parts : (size_t)pl.n_tiles * ctx->Hkv;
        if ((pl.pf_split > 1 && (pf_end > ctx->ws_bytes || pf_counters_used > (size_t)kPrefillSplitUnits)) ||
            (size_t)pl.slots * ctx->Hq * (ctx->hd + 2) * sizeof(float) > ctx->ws_bytes)
            return fail(ctx, OOCO_EINVAL, "ooco_attn_mixed: internal error: the plan's partial results (%zu bytes) do not fit the workspace (%zu bytes)",
                        pf_end, ctx->ws_bytes);
    }
    // (the mixed kernel stamps once per workgroup, the decode kernel once per wave)
    // (a batch without decode work: once per prefill workgroup)
    const int64_t trace_rows = pl.dec_cus > 0 && pl.n_tiles > 0 ? 2 * (int64_t)ctx->num_cus
                               : pl.static_runs > 0           ? (int64_t)pl.static_runs * ctx->Hkv
                               : pl.pf_table                  ? (int64_t)pl.pf_table * ctx->Hkv
                                                              : (int64_t)pl.n_tiles * ctx->Hkv * pl.pf_split;
    const bool tracing = ctx->opt_trace && ctx->trace_d && (size_t)trace_rows <= kTraceWaves;
    p.trace = tracing ? ctx->trace_d : nullptr;
    if (tracing) ctx->trace_waves = trace_rows;
    p.Hq = ctx->Hq;
    p.Hkv = ctx->Hkv;
    p.g = ctx->g;
    p.hd = ctx->hd;
    p.max_blocks_per_seq = ctx->max_blocks_per_seq;
    p.scale_log2e = ctx->scale * 1.4426950408889634f;
    p.num_seqs = num_seqs;
    p.total_q = total_q_tokens;
    p.dec_blocks = pl.dec_blocks;
    p.piece_pad = pl.piece_pad;
    p.static_blocks = pl.static_blocks;
    p.static_runs = pl.static_runs;
    p.tail_runs = pl.tail_runs;
    p.queue = reinterpret_cast<uint32_t *>(ctx->counters + kCounterInts - 1);
    p.queue_base = ctx->queue_base;
    p.n_tiles = pl.n_tiles;
    p.num_pf = pl.num_pf;
    p.dec_cus = pl.dec_cus;
    p.pf_waves = pl.pf_waves;
    p.nbi = ctx->opt_nbi ? (int32_t)ctx->opt_nbi : pl.nbi;
    p.rotate_heads = (int16_t)(ctx->opt_rotate != 0);
    p.lean = (int16_t)pl.lean;
    for (int k = 0; k < kXcds; ++k) p.xcd_cw[k] = pl.cw[k];

    if (pl.tail_runs > 0) {
        // the ticket base of the dynamic tail is fixed when the call is enqueued: a replayed graph would hand out
        // tickets that lie beyond it and leave the tail runs undone
        hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
        if (hipStreamIsCapturing(s, &cs) == hipSuccess && cs != hipStreamCaptureStatusNone)
            return fail(ctx, OOCO_EINVAL, "ooco_attn_mixed: a plan with a dynamic tail (decode_tail_pct) cannot be captured into a graph");
    }
    hipEvent_t *ev = nullptr;
    hipError_t e = hipSuccess;
    if (ctx->opt_profile) {
        if (ctx->prof_calls >= kProfSlots)
            return fail(ctx, OOCO_EINVAL, "ooco_attn_mixed: more than %d profiled calls without ooco_profile_read",
                        kProfSlots);
        if (ctx->prof_ev.empty()) {
            ctx->prof_ev.assign((size_t)kProfEvents * kProfSlots, nullptr);
            for (auto &x : ctx->prof_ev)
                if (e == hipSuccess) e = hipEventCreate(&x);
            if (e != hipSuccess) return fail(ctx, OOCO_EHIP, "ooco_attn_mixed: %s", hipGetErrorString(e));
        }
        ev = ctx->prof_ev.data() + kProfEvents * ctx->prof_calls++;
    }
    // A mixed batch runs its two kernels side by side: the prefill kernel (matrix-core bound) goes to
    // the context's side stream, forked from and joined back into the caller's stream with events,
    // the decode kernel (HBM bound) stays on the caller's stream.  The decode kernel is enqueued first
    // (its three waves per compute unit take their places before the prefill workgroups fill the
    // register files; measured 1.5 % faster on a long-context mixed batch, no difference on a short one).
    // With per-kernel profiling on, the launch order and the streams stay exactly as they are without it:
    // every kernel is bracketed by two events on the stream it runs on (ev[0..1] decode, ev[2..3] prefill)
    // and the whole call by two on the caller's stream (ev[4..5]), so the times are those of the kernels
    // as they run in the step.
    const bool mixed = pl.n_tiles > 0 && pl.static_runs > 0;
    // ... or, by default, in ONE launch: the mixed kernel, whose compute units either decode or prefill (the plan
    // says how many do which).  Both arrays of the plan travel together (in the kernel arguments if they fit).
    const bool fused = mixed && pl.dec_cus > 0;
    const bool overlap = mixed && !fused && ctx->side_stream && (ctx->opt_overlap >= 2 || (ctx->opt_overlap == 1 && !pl.brief));
    hipStream_t ps = overlap ? ctx->side_stream : s;   // the stream of the prefill kernel
    auto mark = [&](int k, hipStream_t st) {
        if (ev && e == hipSuccess) e = hipEventRecord(ev[k], st);
    };
    auto run_prefill = [&]() {
        if (e == hipSuccess && pl.n_tiles > 0) {
            p.cum_dev = inline_cum ? nullptr : ctx->plan_d + n_cum;
            if (inline_cum) memcpy(ka.cum, pl.pf, n_pf * sizeof(int32_t));
        }
        mark(2, ps);
        if (e == hipSuccess && pl.n_tiles > 0) e = launch_prefill(ka, ps);
        mark(3, ps);
    };
    auto run_decode = [&]() {
        if (e == hipSuccess && pl.static_runs > 0) {
            p.cum_dev = inline_cum ? nullptr : ctx->plan_d;
            if (inline_cum) memcpy(ka.cum, pl.dcum, n_cum * sizeof(int32_t));
        }
        mark(0, s);
        if (e == hipSuccess && pl.static_runs > 0) {
            e = launch_decode(ka, s);
            // every wave draws one ticket per tail run it takes plus one that tells it to stop
            if (e == hipSuccess && pl.tail_runs > 0)
                ctx->queue_base += (uint32_t)pl.tail_runs * (uint32_t)ctx->Hkv + (uint32_t)pl.static_runs * (uint32_t)ctx->Hkv;
        }
        mark(1, s);
    };
    mark(4, s);
    if (fused) {
        p.cum_dev = inline_cum ? nullptr : ctx->plan_d;
        if (inline_cum) {
            memcpy(ka.cum, pl.dcum, n_cum * sizeof(int32_t));
            memcpy(ka.cum + n_cum, pl.pf, n_pf * sizeof(int32_t));
        }
        mark(0, s);
        mark(2, s);
        if (e == hipSuccess) e = launch_mixed(ka, ctx->num_cus, s);
        mark(1, s);
        mark(3, s);
    } else if (overlap) {
        // fork before anything else is enqueued, so that the side stream waits for nothing of this call
        if (e == hipSuccess) e = hipEventRecord(ctx->fork_ev, s);
        if (e == hipSuccess) e = hipStreamWaitEvent(ctx->side_stream, ctx->fork_ev, 0);
        if (ctx->opt_decode_first) {
            run_decode();
            run_prefill();
        } else {
            run_prefill();
            run_decode();
        }
        if (e == hipSuccess) e = hipEventRecord(ctx->join_ev, ctx->side_stream);
        if (e == hipSuccess) e = hipStreamWaitEvent(s, ctx->join_ev, 0);
    } else {
        run_prefill();
        run_decode();
    }
    mark(5, s);
    // A plan serves one call: the device length arrays are trusted to equal the planned host copies, and a caller
    // that advances the lengths between steps must plan again (option "plan_persistent" keeps an explicit plan).
    if (ctx->plan_one_shot || !ctx->opt_plan_persistent) {
        ctx->plan_one_shot = false;
        ctx->plan_valid = false;
    }
    if (e != hipSuccess) return fail(ctx, OOCO_EHIP, "ooco_attn_mixed: kernel launch: %s", hipGetErrorString(e));
    return OOCO_OK;
}

ooco_status ooco_attn_mixed_static(int num_q_heads, int num_kv_heads, int head_dim, int block_size, int max_blocks_per_seq,
                                   float softmax_scale, const int32_t *h_seq_lens, const int32_t *h_query_start_loc,
                                   const int32_t *h_ctx_lens, const void *q, const void *k_cache, const void *v_cache,
                                   const int32_t *block_tables, const int32_t *seq_lens, const int32_t *query_start_loc,
                                   const int32_t *ctx_lens, void *out, int num_seqs, int total_q_tokens, void *stream,
                                   char *msg, size_t msg_cap)
{
    char err[512] = "";
    auto bad = [&](ooco_status code, const char *fmt, ...) __attribute__((format(printf, 3, 4))) {
        va_list ap;
        va_start(ap, fmt);
        vsnprintf(err, sizeof err, fmt, ap);
        va_end(ap);
        if (msg && msg_cap) snprintf(msg, msg_cap, "%s", err);
        return code;
    };
    if (msg && msg_cap) msg[0] = 0;
    if (num_seqs < 0 || total_q_tokens < 0)
        return bad(OOCO_EINVAL, "ooco_attn_mixed_static: negative size (num_seqs=%d, total_q_tokens=%d)", num_seqs, total_q_tokens);
    if (num_q_heads <= 0 || num_kv_heads <= 0 || num_q_heads % num_kv_heads != 0 || num_q_heads / num_kv_heads > 16 ||
        (head_dim != 64 && head_dim != 128) || block_size != kBlockSize || max_blocks_per_seq <= 0)
        return bad(OOCO_ESHAPE, "ooco_attn_mixed_static: unsupported geometry (heads %d/%d, head_dim %d, block_size %d, "
                                "max_blocks_per_seq %d)", num_q_heads, num_kv_heads, head_dim, block_size, max_blocks_per_seq);
    if (num_seqs == 0 || total_q_tokens == 0) return OOCO_OK;
    if (!q || !k_cache || !v_cache || !block_tables || !seq_lens || !query_start_loc || !ctx_lens || !out || !h_seq_lens ||
        !h_query_start_loc || !h_ctx_lens)
        return bad(OOCO_EINVAL, "ooco_attn_mixed_static: NULL pointer argument");
    if (num_seqs > kInlineSeqs)
        return bad(OOCO_ENOMEM, "ooco_attn_mixed_static: %d sequences exceed the maximum of %d", num_seqs, kInlineSeqs);
    if ((size_t)num_seqs * (size_t)num_kv_heads > kStaticCounterInts)
        return bad(OOCO_ENOMEM, "ooco_attn_mixed_static: %d sequences x %d kv heads exceed the %zu arrival counters", num_seqs,
                   num_kv_heads, kStaticCounterInts);
    StaticDevice dev;
    int device = 0;
    hipError_t e = static_device(dev, device);
    if (e != hipSuccess) return bad(OOCO_EHIP, "ooco_attn_mixed_static: scratch array: %s", hipGetErrorString(e));

    // plan on the stack: default run layout, no dynamic tail, prefill tiles never split (their partial results
    // would not fit the fixed array); a partial-result area too small for the wanted runs lowers their number
    PlanGeometry geo;
    geo.Hq = num_q_heads;
    geo.Hkv = num_kv_heads;
    geo.hd = head_dim;
    geo.BS = block_size;
    geo.max_blocks_per_seq = max_blocks_per_seq;
    geo.num_cus = dev.num_cus;
    geo.ws_bytes = kStaticScratchBytes - kStaticCounterInts * sizeof(int32_t);
    geo.segments_opt = 0;
    geo.tail_pct = 0;
    geo.tail_blocks = 0;
    geo.pf_split_opt = 1;
    geo.piece_pad = default_piece_pad(head_dim);
    int32_t store[storage_ints(kInlineSeqs)];
    HostPlan pl;
    ooco_status st = build_plan(geo, num_seqs, h_seq_lens, h_query_start_loc, h_ctx_lens, carve_storage(store, kInlineSeqs), pl, err);
    if (st != OOCO_OK) {
        if (msg && msg_cap) snprintf(msg, msg_cap, "%s", err);
        return st;
    }
    if (pl.total_q != total_q_tokens)
        return bad(OOCO_ESHAPE, "ooco_attn_mixed_static: query_start_loc ends at %d, call has %d query tokens", pl.total_q,
                   total_q_tokens);
    if ((size_t)pl.slots * slot_bytes(geo) > geo.ws_bytes)
        return bad(OOCO_ENOMEM, "ooco_attn_mixed_static: partial results of %lld slots exceed the scratch array", (long long)pl.slots);
    if (pl.pf_split != 1 || pl.pf_slots != 0)   // (this entry point has no area for parts of prefill tiles)
        return bad(OOCO_EINVAL, "ooco_attn_mixed_static: internal error: the plan splits prefill tiles");

    KernArgs ka;
    memset(&ka, 0, sizeof ka);
    AttnParams &p = ka.p;
    int32_t *const counters = static_cast<int32_t *>(dev.ptr);
    float *const partials = reinterpret_cast<float *>(static_cast<unsigned char *>(dev.ptr) + kStaticCounterInts * sizeof(int32_t));
    p.q = static_cast<const uint16_t *>(q);
    p.k_cache = static_cast<const uint16_t *>(k_cache);
    p.v_cache = static_cast<const uint16_t *>(v_cache);
    p.block_tables = block_tables;
    p.seq_lens = seq_lens;
    p.query_start_loc = query_start_loc;
    p.ctx_lens = ctx_lens;
    p.out = static_cast<uint16_t *>(out);
    p.part_acc = partials;
    p.part_ml = partials + (size_t)pl.slots * num_q_heads * head_dim;
    p.counters = counters;
    p.cum_dev = nullptr;
    p.trace = nullptr;
    p.Hq = num_q_heads;
    p.Hkv = num_kv_heads;
    p.g = num_q_heads / num_kv_heads;
    p.hd = head_dim;
    p.max_blocks_per_seq = max_blocks_per_seq;
    p.scale_log2e = (softmax_scale > 0.f ? softmax_scale : 1.0f / std::sqrt((float)head_dim)) * 1.4426950408889634f;
    p.num_seqs = num_seqs;
    p.total_q = total_q_tokens;
    p.dec_blocks = pl.dec_blocks;
    p.piece_pad = pl.piece_pad;
    p.static_blocks = pl.static_blocks;
    p.static_runs = pl.static_runs;
    p.tail_runs = 0;
    p.queue = reinterpret_cast<uint32_t *>(counters + kStaticCounterInts - 1);   // (no tail runs: never touched)
    p.queue_base = 0;
    p.n_tiles = pl.n_tiles;
    p.num_pf = pl.num_pf;
    p.pf_waves = pl.pf_waves;
    p.nbi = pl.nbi;
    p.rotate_heads = 1;
    p.pf_acc = nullptr;
    p.pf_ml = nullptr;
    p.pf_counters = nullptr;
    p.pf_split = 1;
    p.pf_table = pl.pf_table;

    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    // The array keeps whatever the last call on this GPU left: the arrival counters this call will count in
    // start at zero (a small fill kernel, not a memset node, so that the call can be captured into a graph).
    if (pl.static_runs > 1) e = launch_fill_zero(counters, (int64_t)num_seqs * num_kv_heads, s);
    if (e == hipSuccess && pl.n_tiles > 0) {
        memcpy(ka.cum, pl.pf, pl.pf_size * sizeof(int32_t));
        e = launch_prefill(ka, s);
    }
    if (e == hipSuccess && pl.static_runs > 0) {
        memcpy(ka.cum, pl.dcum, ((size_t)num_seqs + 1) * sizeof(int32_t));
        e = launch_decode(ka, s);
    }
    if (e != hipSuccess) return bad(OOCO_EHIP, "ooco_attn_mixed_static: kernel launch: %s", hipGetErrorString(e));
    return OOCO_OK;
}

ooco_status ooco_kv_block_copy(ooco_ctx *ctx, const void *k_src, const void *v_src, void *k_dst, void *v_dst,
                               const int64_t *src_block_ids, const int64_t *dst_block_ids, int64_t num_pairs,
                               void *stream)
{
    if (!ctx) return OOCO_EINVAL;
    if (num_pairs < 0) return fail(ctx, OOCO_EINVAL, "ooco_kv_block_copy: num_pairs=%lld", (long long)num_pairs);
    if (num_pairs == 0) return OOCO_OK;
    if (!k_src || !v_src || !k_dst || !v_dst || !src_block_ids || !dst_block_ids)
        return fail(ctx, OOCO_EINVAL, "ooco_kv_block_copy: NULL pointer argument");
    if (num_pairs > (int64_t)1 << 26)
        return fail(ctx, OOCO_EINVAL, "ooco_kv_block_copy: num_pairs=%lld too large", (long long)num_pairs);
    const int64_t block_bytes = (int64_t)ctx->Hkv * ctx->BS * ctx->hd * 2;
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    ctx->note_stream(s);
    hipError_t e = hipSuccess;
    // Large copies take their pairs in order of destination id (sorted on the device into a buffer of the context,
    // which grows on demand -- never while the stream is being captured, a captured copy keeps the caller's order).
    constexpr int64_t kCopySortMin = 2048;
    if (ctx->opt_copy_sort >= 2 || (ctx->opt_copy_sort == 1 && num_pairs >= kCopySortMin)) {
        bool ready = num_pairs <= ctx->sort_cap;
        if (!ready) {
            hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
            const bool capturing = hipStreamIsCapturing(s, &cs) != hipSuccess || cs != hipStreamCaptureStatusNone;
            size_t temp = 0;
            if (!capturing && sort_pairs_temp_bytes(num_pairs, &temp) == hipSuccess) {
                // (work of earlier calls may still read the old buffer: wait for it before freeing)
                if (ctx->sort_buf) {
                    (void)hipStreamSynchronize(s);
                    (void)hipFree(ctx->sort_buf);
                    ctx->sort_buf = nullptr;
                    ctx->sort_cap = 0;
                }
                const size_t ids = ((size_t)num_pairs * 2 * sizeof(int64_t) + 255) / 256 * 256;
                if (hipMalloc(&ctx->sort_buf, ids + temp) == hipSuccess) {
                    ctx->sort_cap = num_pairs;
                    ctx->sort_temp_bytes = temp;
                    ready = true;
                } else {
                    (void)hipGetLastError();
                    ctx->sort_buf = nullptr;
                }
            }
        }
        if (ready) {
            int64_t *dst_sorted = static_cast<int64_t *>(ctx->sort_buf), *src_sorted = dst_sorted + ctx->sort_cap;
            void *temp = static_cast<unsigned char *>(ctx->sort_buf) + ((size_t)ctx->sort_cap * 2 * sizeof(int64_t) + 255) / 256 * 256;
            // (key = the low bits that number the blocks of this context's pool; the destination pool is that pool or
            // a smaller one)
            int bits = 1;
            while (bits < 32 && ((int64_t)1 << bits) < ctx->num_blocks) ++bits;
            e = launch_sort_pairs(temp, ctx->sort_temp_bytes, dst_block_ids, dst_sorted, src_block_ids, src_sorted, num_pairs,
                                  bits, s);
            if (e == hipSuccess) {
                src_block_ids = src_sorted;
                dst_block_ids = dst_sorted;
            } else {
                (void)hipGetLastError();   // the sort did not start: copy in the caller's order
                e = hipSuccess;
            }
        }
    }
    if (e == hipSuccess)
        e = launch_block_copy(k_src, v_src, k_dst, v_dst, src_block_ids, dst_block_ids, num_pairs, block_bytes,
                              ctx->opt_copy_variant, s);
    if (e != hipSuccess) return fail(ctx, OOCO_EHIP, "ooco_kv_block_copy: kernel launch: %s", hipGetErrorString(e));
    return OOCO_OK;
}

ooco_status ooco_kv_append(ooco_ctx *ctx, const void *k_new, const void *v_new, void *k_cache, void *v_cache,
                           const int32_t *block_tables, const int32_t *query_start_loc, const int32_t *ctx_lens,
                           int num_seqs, int total_q_tokens, void *stream)
{
    if (!ctx) return OOCO_EINVAL;
    if (num_seqs < 0 || total_q_tokens < 0)
        return fail(ctx, OOCO_EINVAL, "ooco_kv_append: num_seqs=%d total_q_tokens=%d", num_seqs, total_q_tokens);
    if (num_seqs == 0 || total_q_tokens == 0) return OOCO_OK;
    if (!k_new || !v_new || !k_cache || !v_cache || !block_tables || !query_start_loc || !ctx_lens)
        return fail(ctx, OOCO_EINVAL, "ooco_kv_append: NULL pointer argument");
    hipError_t e = launch_kv_append(k_new, v_new, k_cache, v_cache, block_tables, query_start_loc, ctx_lens, num_seqs,
                                    total_q_tokens, ctx->Hkv, ctx->hd, ctx->max_blocks_per_seq, ctx->num_blocks,
                                    (int)ctx->opt_append_parts, reinterpret_cast<hipStream_t>(stream));
    if (e != hipSuccess) return fail(ctx, OOCO_EHIP, "ooco_kv_append: kernel launch: %s", hipGetErrorString(e));
    return OOCO_OK;
}

}  // extern "C"
