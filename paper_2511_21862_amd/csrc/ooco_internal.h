// Internal declarations shared by the host side (plan, ABI) and the kernel launchers of
// libooco.  Not part of the public ABI.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ooco {

constexpr int kBlockSize = 16;     // tokens per KV block (fixed by the cache layout)
constexpr int kPrefillRows = 32;   // query rows per prefill tile of the simple kernel

// One decode work item: query row `q_row` of sequence `seq` against KV blocks
// [blk_begin, blk_end) of that sequence.  part < 0: the item covers the whole sequence and
// writes bf16 output directly; otherwise it writes partial (acc, m, l) number `part`.
struct DecodeItem {
    int32_t seq;
    int32_t q_row;
    int32_t blk_begin;
    int32_t blk_end;
    int32_t seq_len;
    int32_t part;
    int32_t pad0, pad1;
};

// One prefill tile: `rows` consecutive query rows starting at global row `q_row0`, whose first
// row sits at absolute position `pos0` of sequence `seq`.
struct PrefillTile {
    int32_t seq;
    int32_t q_row0;
    int32_t rows;
    int32_t pos0;
    int32_t seq_len;
    int32_t pad0, pad1, pad2;
};

// One decode sequence whose parts [part0, part0 + nparts) must be merged into row q_row.
struct MergeItem {
    int32_t q_row;
    int32_t part0;
    int32_t nparts;
    int32_t pad0;
};

struct AttnParams {
    const uint16_t *q;
    const uint16_t *k_cache;
    const uint16_t *v_cache;
    const int32_t *block_tables;
    uint16_t *out;
    float *part_acc;            // [parts][Hq][hd]
    float *part_ml;             // [parts][Hq][2]   (running max in log2 units, sum)
    const DecodeItem *ditems;
    const PrefillTile *ptiles;
    const MergeItem *mitems;
    int32_t Hq, Hkv, g, hd;
    int32_t max_blocks_per_seq;
    float scale_log2e;          // softmax scale * log2(e)
    int32_t n_ditems, n_ptiles, n_mitems;
};

// Launchers (ooco_kernels.hip).  Each returns the hipError_t of its launch.
hipError_t launch_decode(const AttnParams &p, hipStream_t s);
hipError_t launch_prefill(const AttnParams &p, hipStream_t s);
hipError_t launch_merge(const AttnParams &p, hipStream_t s);
hipError_t launch_block_copy(const void *k_src, const void *v_src, void *k_dst, void *v_dst,
                             const int64_t *src_ids, const int64_t *dst_ids, int64_t num_pairs,
                             int64_t block_bytes, hipStream_t s);

}  // namespace ooco
