// Device-side building blocks shared by the libnatcomp kernels (gfx950 only):
// the Philox-4x32-10 random words keyed by (seed, worker, operator, element index)
// and small bit helpers.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace natcomp {

constexpr uint32_t kDomainNat = 0;     // C_nat stream
constexpr uint32_t kDomainDither = 1;  // D_nat stream
constexpr uint32_t kDomainNorm = 4;    // C_nat of the dithering norms
constexpr uint32_t kDomainMaster = 3;  // master-side C_nat stream (2 = index selection of the sparsifier)

constexpr uint32_t kPhiloxM0 = 0xD2511F53u, kPhiloxM1 = 0xCD9E8D57u;
constexpr uint32_t kPhiloxW0 = 0x9E3779B9u, kPhiloxW1 = 0xBB67AE85u;

// Native vector types (the streaming load/store builtins want these, not HIP's structs).
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// Streaming (non-temporal) global accesses: every byte is touched once, so nothing is
// worth keeping in the caches.
template <class T>
__device__ __forceinline__ T load_stream(const T* p) { return __builtin_nontemporal_load(p); }
template <class T>
__device__ __forceinline__ void store_stream(T* p, T v) { __builtin_nontemporal_store(v, p); }

// Three-input xor in one VALU op (v_bitop3_b32, truth table 0x96).
__device__ __forceinline__ uint32_t xor3(uint32_t a, uint32_t b, uint32_t c) {
    return __builtin_amdgcn_bitop3_b32(a, b, c, 0x96);
}

// Philox-4x32 with 10 rounds (Salmon et al., SC'11).  One round: with the 64-bit products
// P0 = M0*c0 and P1 = M1*c2, (c0,c1,c2,c3) <- (hi(P1)^c1^k0, lo(P1), hi(P0)^c3^k1, lo(P0)),
// then the key advances by the Weyl constants.  The keys are wave-uniform, so their
// schedule lives in scalar registers; each round costs two 32x32->64 multiplies
// (v_mad_u64_u32) and two three-way xors per lane.
// COMPLEMENT = true returns the bitwise complement of the four words at the cost of two
// extra VALU ops (the other two complements fold into the last round's scalar keys).
template <bool COMPLEMENT>
__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                              uint32_t k0, uint32_t k1, uint32_t out[4]) {
#pragma unroll
    for (int round = 0; round < 10; ++round) {
        const uint64_t p0 = (uint64_t)kPhiloxM0 * c0;
        const uint64_t p1 = (uint64_t)kPhiloxM1 * c2;
        uint32_t ka = k0, kb = k1;
        if (COMPLEMENT && round == 9) { ka = ~ka; kb = ~kb; }
        const uint32_t n0 = xor3((uint32_t)(p1 >> 32), c1, ka);
        const uint32_t n2 = xor3((uint32_t)(p0 >> 32), c3, kb);
        c1 = (uint32_t)p1;
        c3 = (uint32_t)p0;
        c0 = n0;
        c2 = n2;
        k0 += kPhiloxW0;
        k1 += kPhiloxW1;
    }
    out[0] = c0;
    out[1] = COMPLEMENT ? ~c1 : c1;
    out[2] = c2;
    out[3] = COMPLEMENT ? ~c3 : c3;
}

// The four words of call q: they belong to the global elements 4q .. 4q+3.
template <bool COMPLEMENT>
__device__ __forceinline__ void random_words4(uint64_t q, uint32_t worker, uint32_t domain, uint32_t k0,
                                              uint32_t k1, uint32_t out[4]) {
    philox4x32_10<COMPLEMENT>((uint32_t)q, (uint32_t)(q >> 32), worker, domain, k0, k1, out);
}

// The word of one global element (slow path: one full call per element).
__device__ __forceinline__ uint32_t random_word(uint64_t g, uint32_t worker, uint32_t domain, uint32_t k0,
                                                uint32_t k1) {
    uint32_t w[4];
    random_words4<false>(g >> 2, worker, domain, k0, k1, w);
    const uint32_t j = (uint32_t)g & 3u;
    return j == 0 ? w[0] : j == 1 ? w[1] : j == 2 ? w[2] : w[3];
}

// Unsigned saturating add (v_add_u32 ... clamp).
__device__ __forceinline__ uint32_t add_sat(uint32_t a, uint32_t b) { return __builtin_elementwise_add_sat(a, b); }

// (acc << 1) | (u >> 31): shifts the sign bit of u into acc (v_alignbit_b32).
__device__ __forceinline__ uint32_t push_sign(uint32_t acc, uint32_t u) {
    return __builtin_amdgcn_alignbit(acc, u, 31);
}

// Lane i receives v from lane i+N of its row of 16 lanes (DPP row_shl:N); lanes whose source
// falls outside the row receive 0.  All lanes of the wavefront must be active.
template <int N>
__device__ __forceinline__ uint32_t from_lane_plus(uint32_t v) {
    return __builtin_amdgcn_update_dpp(0u, v, 0x100 + N, 0xF, 0xF, true);
}

// Each lane holds a 4-bit value; the word returned in lanes with (lane mod 8) == 0 packs the
// nibbles of lanes lane .. lane+7, lowest lane in the lowest nibble.
__device__ __forceinline__ uint32_t gather_nibbles8(uint32_t nib) {
    uint32_t t = nib | (from_lane_plus<1>(nib) << 4);
    t |= from_lane_plus<2>(t) << 8;
    t |= from_lane_plus<4>(t) << 16;
    return t;
}

// Byte 3 of four registers packed into one word: result byte j = top byte of yj.
__device__ __forceinline__ uint32_t pack_top_bytes(uint32_t y0, uint32_t y1, uint32_t y2, uint32_t y3) {
    const uint32_t lo = __builtin_amdgcn_perm(y1, y0, 0x0c0c0703u);  // bytes: [y0.b3, y1.b3, 0, 0]
    const uint32_t hi = __builtin_amdgcn_perm(y3, y2, 0x07030c0cu);  // bytes: [0, 0, y2.b3, y3.b3]
    return lo | hi;
}

// (mask & a) | (~mask & b)  (v_bfi_b32).
constexpr uint32_t kExpMask = 0x7F800000u;
__device__ __forceinline__ uint32_t bitfield_insert(uint32_t mask, uint32_t a, uint32_t b) {
    return (a & mask) | (b & ~mask);
}

constexpr uint32_t kTileLanes = 256;  // lanes of the workgroups that use store_tile_transposed

__device__ __forceinline__ uint32_t f32_bits(float f) { return __float_as_uint(f); }
__device__ __forceinline__ float bits_f32(uint32_t u) { return __uint_as_float(u); }

// Writes the workgroup's tile of results: lane t put its 8 values into LDS slots 2t, 2t+1;
// now every lane stores slots t and t+256, i.e. 16 contiguous bytes per lane per instruction.
// `groups` = number of whole groups of 8 in the tile (the others are not stored here).
__device__ __forceinline__ void store_tile_transposed(u32x4* lds, const uint32_t v[8], bool have, uint32_t groups,
                                                      float* __restrict__ out_tile) {
    if (have) {
        lds[2 * threadIdx.x] = u32x4{v[0], v[1], v[2], v[3]};
        lds[2 * threadIdx.x + 1] = u32x4{v[4], v[5], v[6], v[7]};
    }
    __syncthreads();
    u32x4* __restrict__ o = reinterpret_cast<u32x4*>(out_tile);
    if (threadIdx.x < 2 * groups) store_stream(o + threadIdx.x, lds[threadIdx.x]);
    if (threadIdx.x + kTileLanes < 2 * groups) store_stream(o + threadIdx.x + kTileLanes, lds[threadIdx.x + kTileLanes]);
}

}  // namespace natcomp
