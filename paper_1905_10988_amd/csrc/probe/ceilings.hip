// Bench-only kernels that measure what this GPU can do at most for the access shapes the
// libnatcomp kernels use: a streaming copy, a read-only sweep, a write-only fill, a copy with
// the 9:4 read:write mix of the n = 8 decode-and-sum, and the Philox-4x32-10 call rate.
// Built into libncprobe.so; not part of libnatcomp.so or of its C ABI.  bench.py reports the
// figures next to the library's kernels so that a fraction of the 8 TB/s peak can be read
// against what a plain copy reaches on the same box.
//
// Every kernel uses the shape of the library's vector paths: workgroups of 256 lanes, each
// lane issuing `kPerLane` 16-byte non-temporal accesses that are contiguous across the lanes.
#include "../device_common.hpp"

namespace {

using natcomp::u32x4;
constexpr int kLanes = 256;
constexpr int kPerLane = 2;
constexpr uint64_t kTile = (uint64_t)kLanes * kPerLane;  // 16-byte items per workgroup

__global__ __launch_bounds__(kLanes) void copy_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst,
                                                      uint64_t items) {
    const uint64_t i0 = (uint64_t)blockIdx.x * kTile + threadIdx.x;
    u32x4 v[kPerLane];
#pragma unroll
    for (int k = 0; k < kPerLane; ++k) {
        const uint64_t i = i0 + (uint64_t)k * kLanes;
        v[k] = u32x4{0u, 0u, 0u, 0u};
        if (i < items) v[k] = __builtin_nontemporal_load(src + i);
    }
#pragma unroll
    for (int k = 0; k < kPerLane; ++k) {
        const uint64_t i = i0 + (uint64_t)k * kLanes;
        if (i < items) __builtin_nontemporal_store(v[k], dst + i);
    }
}

// Reads everything, writes (almost) nothing: the xor of the tile leaves only if it hits one value.
__global__ __launch_bounds__(kLanes) void read_kernel(const u32x4* __restrict__ src, uint32_t* __restrict__ sink,
                                                      uint64_t items) {
    const uint64_t i0 = (uint64_t)blockIdx.x * kTile + threadIdx.x;
    u32x4 v[kPerLane];
#pragma unroll
    for (int k = 0; k < kPerLane; ++k) {
        const uint64_t i = i0 + (uint64_t)k * kLanes;
        v[k] = u32x4{0u, 0u, 0u, 0u};
        if (i < items) v[k] = __builtin_nontemporal_load(src + i);
    }
    uint32_t acc = 0;
#pragma unroll
    for (int k = 0; k < kPerLane; ++k) acc ^= v[k].x ^ v[k].y ^ v[k].z ^ v[k].w;
    if (acc == 0x9E3779B9u) sink[threadIdx.x] = acc;
}

__global__ __launch_bounds__(kLanes) void fill_kernel(u32x4* __restrict__ dst, uint64_t items, uint32_t value) {
    const uint64_t i0 = (uint64_t)blockIdx.x * kTile + threadIdx.x;
#pragma unroll
    for (int k = 0; k < kPerLane; ++k) {
        const uint64_t i = i0 + (uint64_t)k * kLanes;
        if (i < items) __builtin_nontemporal_store(u32x4{value, value, value, value}, dst + i);
    }
}

// 9 bytes read per 4 bytes written, the mix of the n = 8 C_nat decode-and-sum: per 16-byte
// item written, two 16-byte items and one 4-byte word are read.
__global__ __launch_bounds__(kLanes) void mix94_kernel(const u32x4* __restrict__ a, const u32x4* __restrict__ b,
                                                       const uint32_t* __restrict__ c, u32x4* __restrict__ dst,
                                                       uint64_t items) {
    const uint64_t i0 = (uint64_t)blockIdx.x * kTile + threadIdx.x;
    u32x4 va[kPerLane], vb[kPerLane];
    uint32_t vc[kPerLane];
#pragma unroll
    for (int k = 0; k < kPerLane; ++k) {
        const uint64_t i = i0 + (uint64_t)k * kLanes;
        va[k] = vb[k] = u32x4{0u, 0u, 0u, 0u};
        vc[k] = 0;
        if (i < items) {
            va[k] = __builtin_nontemporal_load(a + i);
            vb[k] = __builtin_nontemporal_load(b + i);
            vc[k] = __builtin_nontemporal_load(c + i);
        }
    }
#pragma unroll
    for (int k = 0; k < kPerLane; ++k) {
        const uint64_t i = i0 + (uint64_t)k * kLanes;
        if (i < items) __builtin_nontemporal_store(va[k] ^ vb[k] ^ vc[k], dst + i);
    }
}

// `calls` independent Philox-4x32-10 calls per lane, the library's own device function (two
// 32x32->64 multiplies and two three-way xors per round); nothing is read from memory.
__global__ __launch_bounds__(kLanes) void philox_kernel(uint32_t* __restrict__ sink, uint32_t calls, uint32_t k0,
                                                        uint32_t k1) {
    const uint32_t lane = blockIdx.x * kLanes + threadIdx.x;
    uint32_t acc = 0;
    for (uint32_t q = 0; q < calls; ++q) {
        uint32_t w[4];
        natcomp::philox4x32_10<true>(lane, q, 7u, 0u, k0, k1, w);
        acc ^= w[0] ^ w[1] ^ w[2] ^ w[3];
    }
    if (acc == 0x12345678u) sink[threadIdx.x] = acc;
}

inline unsigned tiles(uint64_t items) { return (unsigned)((items + kTile - 1) / kTile); }

}  // namespace

extern "C" {

// All pointers are device pointers, 16-byte aligned; `bytes` is rounded down to a multiple
// of 16 and must stay below 2^40.  Calls are asynchronous on `stream`; the return value is
// the hipError_t of the launch.
int ncp_copy(const void* src, void* dst, uint64_t bytes, void* stream) {
    const uint64_t items = bytes / 16;
    if (!items) return 0;
    copy_kernel<<<tiles(items), kLanes, 0, (hipStream_t)stream>>>((const u32x4*)src, (u32x4*)dst, items);
    return (int)hipGetLastError();
}
// sink: at least 1 KiB.
int ncp_read(const void* src, uint64_t bytes, void* sink, void* stream) {
    const uint64_t items = bytes / 16;
    if (!items) return 0;
    read_kernel<<<tiles(items), kLanes, 0, (hipStream_t)stream>>>((const u32x4*)src, (uint32_t*)sink, items);
    return (int)hipGetLastError();
}
int ncp_fill(void* dst, uint64_t bytes, void* stream) {
    const uint64_t items = bytes / 16;
    if (!items) return 0;
    fill_kernel<<<tiles(items), kLanes, 0, (hipStream_t)stream>>>((u32x4*)dst, items, 0x3C000000u);
    return (int)hipGetLastError();
}
// a, b: `bytes` each; c: bytes / 4; dst: `bytes`.  Moves 2.25 * bytes in and bytes out.
int ncp_mix94(const void* a, const void* b, const void* c, void* dst, uint64_t bytes, void* stream) {
    const uint64_t items = bytes / 16;
    if (!items) return 0;
    mix94_kernel<<<tiles(items), kLanes, 0, (hipStream_t)stream>>>((const u32x4*)a, (const u32x4*)b,
                                                                    (const uint32_t*)c, (u32x4*)dst, items);
    return (int)hipGetLastError();
}
// workgroups * 256 lanes, `calls` Philox calls each.  sink: at least 1 KiB.
int ncp_philox(void* sink, uint32_t workgroups, uint32_t calls, void* stream) {
    if (!workgroups) return 0;
    philox_kernel<<<workgroups, kLanes, 0, (hipStream_t)stream>>>((uint32_t*)sink, calls, 1u, 2u);
    return (int)hipGetLastError();
}

}  // extern "C"
