// Leaf hashing of the matrix commitments on the device (the top-level hash stays on the host).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace imm {
namespace k {

// One leaf: `bytes` (1 .. 2^20) raw bytes at a 4-byte aligned device address.
struct LeafDesc {
    const uint8_t* p;
    uint64_t bytes;
};

// digests[32 * i .. 32 * i + 32) = SHA-256 of leaf i, for i < count.  `leaves` and `digests` are
// device memory; `aligned16` says that every leaf starts at a multiple of 16 bytes.
hipError_t commit_leaves(hipStream_t stream, const LeafDesc* leaves, uint32_t count, bool aligned16, uint8_t* digests);

}  // namespace k
}  // namespace imm
