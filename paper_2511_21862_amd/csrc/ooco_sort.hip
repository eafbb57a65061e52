// Device-side ordering of the (source, destination) block pairs of ooco_kv_block_copy by destination id.
// The copy kernel takes its pairs in array order and the hardware dispatches its workgroups in index order, so
// with sorted pairs the blocks written at any one time are neighbours in the destination pool; on MI355X that is
// worth more than the sort costs once a copy moves a few thousand blocks.  The sort itself is the library radix
// sort (hipCUB); nothing of the copy's semantics depends on it (pairs are independent, destination ids distinct).
#include "ooco_internal.h"

#include <hipcub/hipcub.hpp>

namespace ooco {

// Only the low `bits` bits of the ids take part (the caller passes the bit length of the pool size): whatever the
// ids, the result is a permutation of whole pairs, so a pool larger than announced costs locality, never correctness.
hipError_t sort_pairs_temp_bytes(int64_t num_pairs, size_t *bytes)
{
    *bytes = 0;
    return hipcub::DeviceRadixSort::SortPairs(nullptr, *bytes, (const uint64_t *)nullptr, (uint64_t *)nullptr,
                                              (const int64_t *)nullptr, (int64_t *)nullptr, (int)num_pairs, 0, 32,
                                              (hipStream_t) nullptr);
}

hipError_t launch_sort_pairs(void *temp, size_t temp_bytes, const int64_t *dst_ids, int64_t *dst_sorted,
                             const int64_t *src_ids, int64_t *src_sorted, int64_t num_pairs, int bits, hipStream_t s)
{
    return hipcub::DeviceRadixSort::SortPairs(temp, temp_bytes, reinterpret_cast<const uint64_t *>(dst_ids),
                                              reinterpret_cast<uint64_t *>(dst_sorted), src_ids, src_sorted, (int)num_pairs, 0,
                                              bits < 1 ? 1 : (bits > 32 ? 32 : bits), s);
}

}  // namespace ooco
