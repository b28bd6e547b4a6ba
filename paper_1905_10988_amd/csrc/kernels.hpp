// Host-visible launch interface between the C ABI layer and the kernel files.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace natcomp {

constexpr int kBlock = 256;  // lanes per workgroup (4 wavefronts)

struct NatEncodeArgs {
    const float* x; size_t x_stride;           // floats between workers
    uint64_t d;
    uint32_t k0, k1;                           // Philox key = (lo32(seed), hi32(seed))
    uint32_t first_worker;
    uint64_t index_offset;
    uint8_t* exp_out; size_t exp_stride;       // bytes between workers
    uint8_t* sign_out; size_t sign_stride;
};
struct NatDecodeArgs {
    const uint8_t* exp; const uint8_t* sign; uint64_t d; float* out;
};
struct NatAggregateArgs {
    const uint8_t* exp; size_t exp_stride; const uint8_t* sign; size_t sign_stride;
    uint32_t n; uint64_t d; float* out;
};

// `fast` promises the alignment the vector path needs (checked by the caller).
hipError_t launch_nat_encode(const NatEncodeArgs& a, uint32_t n, bool fast, hipStream_t stream);
hipError_t launch_nat_decode(const NatDecodeArgs& a, bool fast, hipStream_t stream);
hipError_t launch_nat_aggregate(const NatAggregateArgs& a, bool fast, hipStream_t stream);

}  // namespace natcomp
