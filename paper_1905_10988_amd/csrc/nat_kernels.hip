// Natural compression C_nat on gfx950: encoder, decoder and the fused n-worker
// decode-and-sum (Sec. 2, Def. 1 and the binary32 derivation; Algorithm 1's master sum).
//
// All three kernels are HBM-bound streams: 5.125 bytes per encoded element,
// 8*1.125 + 4 bytes per summed element at n = 8.  What decides their speed is the shape of
// the memory instructions, so every global access of the vector paths is lane-contiguous:
//   encoder  a workgroup owns a tile of 1024 elements; lane t reads the two 16-byte quads
//            t and t+128 of the tile, draws one Philox call per quad, stores its four
//            exponent bytes as one word per quad; the four sign bits of 8 neighbouring
//            lanes are gathered with DPP row shifts into one word stored by every 8th lane;
//   decoder  lane t reads 8 exponent bytes and one sign byte, builds 8 floats, and the
//            workgroup transposes them through LDS so that each store instruction writes 16
//            contiguous bytes per lane;
//   aggregate  lane t owns 16 output elements: per worker one 16-byte exponent load and one
//            2-byte sign load, all workers of a chunk of 8 in flight before the first add;
//            the sums leave through the same kind of LDS transpose (planes that are only
//            8-byte aligned take an 8-elements-per-lane kernel of the same shape).
#include "device_common.hpp"
#include "kernels.hpp"

namespace natcomp {

constexpr int kEncBlock = 128;        // lanes per encoder workgroup
constexpr uint32_t kEncTile = 1024;   // elements per encoder workgroup (128 lanes x 2 quads)

// New exponent byte in the top byte of the result.  With u = (sign, e, m) and T = m * 2^9
// the rule is "exponent + 1 iff r < T".  Since T is a multiple of 2^9 this is
// (r >> 8) < 2m, i.e. 2m + (~r >> 8) carries out of 24 bits: adding the complemented
// word to u << 1 (exponent in the top byte, 2m below it) performs the comparison and the
// increment in one saturating add; saturation keeps exponent 255 at 255.
__device__ __forceinline__ uint32_t nat_round_top(uint32_t u, uint32_t r_complement) {
    return add_sat(u << 1, r_complement >> 8);
}

// Four elements -> their four new exponent bytes in one word.
__device__ __forceinline__ uint32_t nat_round_quad(u32x4 v, const uint32_t rc[4]) {
    return pack_top_bytes(nat_round_top(v.x, rc[0]), nat_round_top(v.y, rc[1]), nat_round_top(v.z, rc[2]),
                          nat_round_top(v.w, rc[3]));
}
// Sign bits of four elements, element 0 in bit 0.
__device__ __forceinline__ uint32_t sign_nibble(u32x4 v) {
    uint32_t s = v.w >> 31;
    s = push_sign(s, v.z);
    s = push_sign(s, v.y);
    return push_sign(s, v.x);
}

// One group of up to 8 elements starting at local index i0 (a multiple of 8), any
// alignment: scalar loads, one Philox call per run of elements sharing a counter.
__device__ __noinline__ void nat_encode_group_generic(const float* __restrict__ x, uint64_t d, uint64_t i0,
                                                      uint64_t index_offset, uint32_t worker, uint32_t k0,
                                                      uint32_t k1, uint8_t* __restrict__ exp_out,
                                                      uint8_t* __restrict__ sign_out) {
    uint32_t sign_byte = 0;
    uint64_t cached_q = ~0ull;
    uint32_t w[4] = {0, 0, 0, 0};
    for (int j = 0; j < 8; ++j) {
        const uint64_t i = i0 + j;
        if (i >= d) break;
        const uint32_t u = f32_bits(x[i]);
        const uint64_t g = index_offset + i;
        if ((g >> 2) != cached_q) {
            cached_q = g >> 2;
            random_words4<true>(cached_q, worker, kDomainNat, k0, k1, w);
        }
        const uint32_t sel = (uint32_t)g & 3u;
        const uint32_t rc = sel == 0 ? w[0] : sel == 1 ? w[1] : sel == 2 ? w[2] : w[3];
        exp_out[i] = (uint8_t)(nat_round_top(u, rc) >> 24);
        sign_byte |= (u >> 31) << j;
    }
    sign_out[i0 >> 3] = (uint8_t)sign_byte;
}

// Vector encoder.  Requires: x 16-byte aligned, exp_out and sign_out 4-byte aligned,
// index_offset a multiple of 4 (and the same for every worker's planes).  Elements
// [0, 32*floor(d/32)) go through the vector path; the last d mod 32 through the scalar one.
// A workgroup of 128 lanes owns 1024 elements: lane t takes quads t and t+128, and both
// 16-byte loads are issued before any arithmetic (measured best among 64..512 lanes and
// 1..4 quads per lane).
__global__ __launch_bounds__(kEncBlock) void nat_encode_kernel(NatEncodeArgs a) {
    const uint32_t w = blockIdx.y;
    const float* __restrict__ x = a.x + (size_t)w * a.x_stride;
    uint8_t* __restrict__ exp_out = a.exp_out + (size_t)w * a.exp_stride;
    uint8_t* __restrict__ sign_out = a.sign_out + (size_t)w * a.sign_stride;
    const uint32_t worker = a.first_worker + w;
    const uint64_t vec_quads = (a.d >> 5) << 3;  // quads inside whole 32-element groups
    const uint64_t q0 = (uint64_t)blockIdx.x * (kEncTile / 4) + threadIdx.x;
    const uint64_t qbase = a.index_offset >> 2;
    const u32x4* __restrict__ xv = reinterpret_cast<const u32x4*>(x);
    uint32_t* __restrict__ ev = reinterpret_cast<uint32_t*>(exp_out);
    uint32_t* __restrict__ sv = reinterpret_cast<uint32_t*>(sign_out);
    u32x4 v[2];
#pragma unroll
    for (int half = 0; half < 2; ++half) {
        const uint64_t q = q0 + half * kEncBlock;
        v[half] = u32x4{0u, 0u, 0u, 0u};
        if (q < vec_quads) v[half] = load_stream(xv + q);
    }
#pragma unroll
    for (int half = 0; half < 2; ++half) {
        const uint64_t q = q0 + half * kEncBlock;
        const bool in = q < vec_quads;  // uniform over each run of 8 lanes
        uint32_t rc[4];
        random_words4<true>(qbase + q, worker, kDomainNat, a.k0, a.k1, rc);
        const uint32_t exps = nat_round_quad(v[half], rc);
        const uint32_t packed = gather_nibbles8(sign_nibble(v[half]));  // every lane takes part
        if (in) store_stream(ev + q, exps);
        if (in && (threadIdx.x & 7) == 0) store_stream(sv + (q >> 3), packed);
    }
    // scalar tail: at most 31 elements, four groups of 8
    const uint64_t tail0 = vec_quads * 4;
    if (tail0 < a.d && blockIdx.x == gridDim.x - 1 && threadIdx.x < 4) {
        const uint64_t i0 = tail0 + threadIdx.x * 8;
        if (i0 < a.d) nat_encode_group_generic(x, a.d, i0, a.index_offset, worker, a.k0, a.k1, exp_out, sign_out);
    }
}

// Any alignment: one group of 8 elements per lane.
__global__ __launch_bounds__(kBlock) void nat_encode_generic_kernel(NatEncodeArgs a) {
    const uint32_t w = blockIdx.y;
    const uint64_t i0 = ((uint64_t)blockIdx.x * kBlock + threadIdx.x) * 8;
    if (i0 >= a.d) return;
    nat_encode_group_generic(a.x + (size_t)w * a.x_stride, a.d, i0, a.index_offset, a.first_worker + w, a.k0, a.k1,
                             a.exp_out + (size_t)w * a.exp_stride, a.sign_out + (size_t)w * a.sign_stride);
}

// Value of one coded element: sign and exponent from the planes, mantissa zero.
__device__ __forceinline__ uint32_t nat_value_bits(uint32_t exp_byte, uint32_t sign_bit) {
    return (sign_bit << 31) | (exp_byte << 23);
}

// Eight values from 8 exponent bytes (two words) and one sign byte.  Element j takes
// exponent byte j and sign bit j; v_bfi merges "byte moved to bits 23..30" with "sign bit
// moved to bit 31" (the lower sign bits that travel along land inside the exponent field,
// which the mask takes from the exponent word).
__device__ __forceinline__ void nat_decode8(u32x2 e, uint32_t sb, uint32_t v[8]) {
    v[0] = bitfield_insert(kExpMask, e.x << 23, sb << 31);
    v[1] = bitfield_insert(kExpMask, e.x << 15, sb << 30);
    v[2] = bitfield_insert(kExpMask, e.x << 7, sb << 29);
    v[3] = bitfield_insert(kExpMask, e.x >> 1, sb << 28);
    v[4] = bitfield_insert(kExpMask, e.y << 23, sb << 27);
    v[5] = bitfield_insert(kExpMask, e.y << 15, sb << 26);
    v[6] = bitfield_insert(kExpMask, e.y << 7, sb << 25);
    v[7] = bitfield_insert(kExpMask, e.y >> 1, sb << 24);
}

// Vector decoder.  Requires exp 8-byte aligned and out 16-byte aligned.
__global__ __launch_bounds__(kBlock) void nat_decode_kernel(NatDecodeArgs a) {
    __shared__ u32x4 lds[2 * kBlock];
    const uint64_t g0 = (uint64_t)blockIdx.x * kBlock;
    const uint64_t grp = g0 + threadIdx.x;
    const uint64_t full = a.d >> 3;  // whole groups of 8
    const bool have = grp < full;
    uint32_t v[8];
    if (have) {
        const u32x2 e = load_stream(reinterpret_cast<const u32x2*>(a.exp) + grp);
        const uint32_t sb = load_stream(a.sign + grp);
        nat_decode8(e, sb, v);
    }
    const uint32_t groups = full - g0 < kBlock ? (uint32_t)(full - g0) : (uint32_t)kBlock;
    store_tile_transposed(lds, v, have, full > g0 ? groups : 0u, a.out + g0 * 8);
    if (grp == full && (a.d & 7)) {  // the ragged last group
        const uint32_t sb = a.sign[grp];
        for (uint64_t i = grp * 8; i < a.d; ++i) a.out[i] = bits_f32(nat_value_bits(a.exp[i], (sb >> (i & 7)) & 1u));
    }
}

__global__ __launch_bounds__(kBlock) void nat_decode_generic_kernel(NatDecodeArgs a) {
    const uint64_t i0 = ((uint64_t)blockIdx.x * kBlock + threadIdx.x) * 8;
    if (i0 >= a.d) return;
    const uint32_t sb = a.sign[i0 >> 3];
    for (int j = 0; j < 8; ++j) {
        const uint64_t i = i0 + j;
        if (i >= a.d) break;
        a.out[i] = bits_f32(nat_value_bits(a.exp[i], (sb >> j) & 1u));
    }
}

// One element of the sum, any alignment: workers added left to right from worker 0's value.
__device__ __forceinline__ float nat_sum_one(const NatAggregateArgs& a, uint64_t i) {
    float acc = 0.0f;
    for (uint32_t w = 0; w < a.n; ++w) {
        const uint32_t eb = a.exp[(size_t)w * a.exp_stride + i];
        const uint32_t sg = (a.sign[(size_t)w * a.sign_stride + (i >> 3)] >> (i & 7)) & 1u;
        const float v = bits_f32(nat_value_bits(eb, sg));
        acc = (w == 0) ? v : acc + v;
    }
    return acc;
}

// NW workers starting at w0: all 2*NW loads are issued before the first add.
template <int NW>
__device__ __forceinline__ void nat_sum_chunk(const NatAggregateArgs& a, uint64_t grp, uint32_t w0, float acc[8]) {
    u32x2 e[NW];
    uint32_t sb[NW];
#pragma unroll
    for (int k = 0; k < NW; ++k) {
        const size_t w = w0 + k;
        e[k] = load_stream(reinterpret_cast<const u32x2*>(a.exp + w * a.exp_stride) + grp);
        sb[k] = load_stream(a.sign + w * a.sign_stride + grp);
    }
#pragma unroll
    for (int k = 0; k < NW; ++k) {
        uint32_t v[8];
        nat_decode8(e[k], sb[k], v);
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[j] += bits_f32(v[j]);
    }
}

// Runs BODY<NW>(w0) over the workers in chunks of up to 8, in the order w = 0, 1, ..., n-1.
#define NATCOMP_FOR_WORKER_CHUNKS(n, CALL)                        \
    do {                                                          \
        uint32_t w0 = 0;                                          \
        for (; w0 + 8 <= (n); w0 += 8) { CALL(8); }               \
        switch ((n) - w0) {                                       \
            case 1: CALL(1); break;                               \
            case 2: CALL(2); break;                               \
            case 3: CALL(3); break;                               \
            case 4: CALL(4); break;                               \
            case 5: CALL(5); break;                               \
            case 6: CALL(6); break;                               \
            case 7: CALL(7); break;                               \
            default: break;                                       \
        }                                                         \
    } while (0)

// Fused decode-and-sum over n workers, 8 output elements per lane.  Workers are taken in
// chunks of up to 8 whose loads are all issued before the first add, and added in the
// fixed order w = 0, 1, ..., n-1 starting from worker 0's value.
// Requires every worker's exponent plane 8-byte aligned and out 16-byte aligned.
__global__ __launch_bounds__(kBlock) void nat_aggregate8_kernel(NatAggregateArgs a) {
    __shared__ u32x4 lds[2 * kBlock];
    const uint64_t g0 = (uint64_t)blockIdx.x * kBlock;
    const uint64_t grp = g0 + threadIdx.x;
    const uint64_t full = a.d >> 3;
    const bool have = grp < full;
    uint32_t bits[8];
    if (have) {
        // -0.0 is the identity of binary32 addition (x + -0.0 == x bit for bit, signed zeros
        // included), so starting there equals starting from worker 0's value.
        float acc[8] = {-0.0f, -0.0f, -0.0f, -0.0f, -0.0f, -0.0f, -0.0f, -0.0f};
#define NATCOMP_CALL(NW) nat_sum_chunk<NW>(a, grp, w0, acc)
        NATCOMP_FOR_WORKER_CHUNKS(a.n, NATCOMP_CALL);
#undef NATCOMP_CALL
#pragma unroll
        for (int j = 0; j < 8; ++j) bits[j] = f32_bits(acc[j]);
    }
    const uint32_t groups = full - g0 < kBlock ? (uint32_t)(full - g0) : (uint32_t)kBlock;
    store_tile_transposed(lds, bits, have, full > g0 ? groups : 0u, a.out + g0 * 8);
    if (grp == full && (a.d & 7)) {
        for (uint64_t i = grp * 8; i < a.d; ++i) a.out[i] = nat_sum_one(a, i);
    }
}

// NW workers starting at w0 for the lane's group of 16 elements: per worker one 16-byte
// exponent load and one 2-byte sign load, all issued before the first add.
template <int NW>
__device__ __forceinline__ void nat_sum_chunk16(const NatAggregateArgs& a, uint64_t grp, uint32_t w0, float acc[16]) {
    u32x4 e[NW];
    uint32_t sb[NW];
#pragma unroll
    for (int k = 0; k < NW; ++k) {
        const size_t w = w0 + k;
        e[k] = load_stream(reinterpret_cast<const u32x4*>(a.exp + w * a.exp_stride) + grp);
        sb[k] = load_stream(reinterpret_cast<const uint16_t*>(a.sign + w * a.sign_stride) + grp);
    }
#pragma unroll
    for (int k = 0; k < NW; ++k) {
        uint32_t v[8];
        nat_decode8(u32x2{e[k].x, e[k].y}, sb[k], v);
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[j] += bits_f32(v[j]);
        nat_decode8(u32x2{e[k].z, e[k].w}, sb[k] >> 8, v);
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[8 + j] += bits_f32(v[j]);
    }
}

// The same sum with 16 output elements per lane (a tile of 4096 per workgroup): wider loads,
// half as many of them.  Requires every worker's exponent plane 16-byte aligned, every sign
// plane 2-byte aligned and out 16-byte aligned.  Lane t puts its four result quads into LDS
// slots 4t .. 4t+3; every store instruction then writes slots t + 256 m, 16 contiguous bytes
// per lane.
__global__ __launch_bounds__(kBlock) void nat_aggregate_kernel(NatAggregateArgs a) {
    __shared__ u32x4 lds[4 * kBlock];
    const uint64_t g0 = (uint64_t)blockIdx.x * kBlock;
    const uint64_t grp = g0 + threadIdx.x;
    const uint64_t full = a.d >> 4;  // whole groups of 16
    if (grp < full) {
        float acc[16];
#pragma unroll
        for (int j = 0; j < 16; ++j) acc[j] = -0.0f;  // the identity of binary32 addition
#define NATCOMP_CALL(NW) nat_sum_chunk16<NW>(a, grp, w0, acc)
        NATCOMP_FOR_WORKER_CHUNKS(a.n, NATCOMP_CALL);
#undef NATCOMP_CALL
#pragma unroll
        for (int q = 0; q < 4; ++q)
            lds[4 * threadIdx.x + q] = u32x4{f32_bits(acc[4 * q]), f32_bits(acc[4 * q + 1]), f32_bits(acc[4 * q + 2]),
                                             f32_bits(acc[4 * q + 3])};
    }
    __syncthreads();
    const uint32_t groups = full > g0 ? (full - g0 < kBlock ? (uint32_t)(full - g0) : (uint32_t)kBlock) : 0u;
    u32x4* __restrict__ o = reinterpret_cast<u32x4*>(a.out + g0 * 16);
#pragma unroll
    for (int m = 0; m < 4; ++m) {
        const uint32_t slot = threadIdx.x + m * kBlock;
        if (slot < 4 * groups) store_stream(o + slot, lds[slot]);
    }
    if (grp == full && (a.d & 15)) {  // the ragged last group
        for (uint64_t i = grp * 16; i < a.d; ++i) a.out[i] = nat_sum_one(a, i);
    }
}

// Master step of Algorithm 1 with C_M = C_nat: the same sum, then natural compression of the
// sum with the master's own stream (domain 3, keyed by the master id), so 1.125 bytes leave per
// element instead of 4.  Requires the aggregate kernel's alignment, exp_out 8-byte aligned and
// index_offset a multiple of 4.
__global__ __launch_bounds__(kBlock) void nat_master_kernel(NatAggregateArgs a, NatMasterArgs m) {
    const uint64_t grp = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
    const uint64_t full = a.d >> 3;
    if (grp < full) {
        float acc[8] = {-0.0f, -0.0f, -0.0f, -0.0f, -0.0f, -0.0f, -0.0f, -0.0f};
        uint32_t w0 = 0;
        for (; w0 + 8 <= a.n; w0 += 8) nat_sum_chunk<8>(a, grp, w0, acc);
        for (; w0 + 2 <= a.n; w0 += 2) nat_sum_chunk<2>(a, grp, w0, acc);
        if (w0 < a.n) nat_sum_chunk<1>(a, grp, w0, acc);
        uint32_t r0[4], r1[4];
        const uint64_t q = (m.index_offset >> 2) + 2 * grp;
        random_words4<true>(q, m.master, kDomainMaster, m.k0, m.k1, r0);
        random_words4<true>(q + 1, m.master, kDomainMaster, m.k0, m.k1, r1);
        uint32_t u[8], sb;
#pragma unroll
        for (int j = 0; j < 8; ++j) u[j] = f32_bits(acc[j]);
        sb = u[7] >> 31;
#pragma unroll
        for (int j = 6; j >= 0; --j) sb = push_sign(sb, u[j]);
        u32x2 e;
        e.x = pack_top_bytes(nat_round_top(u[0], r0[0]), nat_round_top(u[1], r0[1]), nat_round_top(u[2], r0[2]),
                             nat_round_top(u[3], r0[3]));
        e.y = pack_top_bytes(nat_round_top(u[4], r1[0]), nat_round_top(u[5], r1[1]), nat_round_top(u[6], r1[2]),
                             nat_round_top(u[7], r1[3]));
        store_stream(reinterpret_cast<u32x2*>(m.exp_out) + grp, e);
        store_stream(m.sign_out + grp, (uint8_t)sb);
    } else if (grp == full && (a.d & 7)) {
        uint32_t sb = 0;
        for (uint64_t i = grp * 8; i < a.d; ++i) {
            const uint32_t u = f32_bits(nat_sum_one(a, i));
            const uint32_t r = random_word(m.index_offset + i, m.master, kDomainMaster, m.k0, m.k1);
            m.exp_out[i] = (uint8_t)(nat_round_top(u, ~r) >> 24);
            sb |= (u >> 31) << (i & 7);
        }
        m.sign_out[grp] = (uint8_t)sb;
    }
}

__global__ __launch_bounds__(kBlock) void nat_master_generic_kernel(NatAggregateArgs a, NatMasterArgs m) {
    const uint64_t i0 = ((uint64_t)blockIdx.x * kBlock + threadIdx.x) * 8;
    if (i0 >= a.d) return;
    uint32_t sb = 0;
    for (int j = 0; j < 8; ++j) {
        const uint64_t i = i0 + j;
        if (i >= a.d) break;
        const uint32_t u = f32_bits(nat_sum_one(a, i));
        const uint32_t r = random_word(m.index_offset + i, m.master, kDomainMaster, m.k0, m.k1);
        m.exp_out[i] = (uint8_t)(nat_round_top(u, ~r) >> 24);
        sb |= (u >> 31) << j;
    }
    m.sign_out[i0 >> 3] = (uint8_t)sb;
}

__global__ __launch_bounds__(kBlock) void nat_aggregate_generic_kernel(NatAggregateArgs a) {
    const uint64_t i0 = ((uint64_t)blockIdx.x * kBlock + threadIdx.x) * 8;
    for (int j = 0; j < 8; ++j) {
        const uint64_t i = i0 + j;
        if (i >= a.d) break;
        a.out[i] = nat_sum_one(a, i);
    }
}

// One lane per group of 8 elements; the grid always covers the ragged last group too.
static inline dim3 grid_for_groups(uint64_t d, uint32_t y) {
    const uint64_t groups = d / 8 + 1;
    return dim3((unsigned)((groups + kBlock - 1) / kBlock), y, 1);
}

hipError_t launch_nat_encode(const NatEncodeArgs& a, uint32_t n, bool fast, hipStream_t stream) {
    if (fast) {
        const dim3 grid((unsigned)((a.d + kEncTile - 1) / kEncTile), n, 1);
        nat_encode_kernel<<<grid, kEncBlock, 0, stream>>>(a);
    } else {
        nat_encode_generic_kernel<<<grid_for_groups(a.d, n), kBlock, 0, stream>>>(a);
    }
    return hipGetLastError();
}

hipError_t launch_nat_decode(const NatDecodeArgs& a, bool fast, hipStream_t stream) {
    const dim3 grid = grid_for_groups(a.d, 1);
    if (fast) nat_decode_kernel<<<grid, kBlock, 0, stream>>>(a);
    else nat_decode_generic_kernel<<<grid, kBlock, 0, stream>>>(a);
    return hipGetLastError();
}

hipError_t launch_nat_aggregate(const NatAggregateArgs& a, int width, hipStream_t stream) {
    const dim3 grid = grid_for_groups(a.d, 1);
    if (width == 16) {  // one lane per group of 16 elements, the ragged last group included
        const uint64_t groups = a.d / 16 + 1;
        nat_aggregate_kernel<<<(unsigned)((groups + kBlock - 1) / kBlock), kBlock, 0, stream>>>(a);
    } else if (width == 8) {
        nat_aggregate8_kernel<<<grid, kBlock, 0, stream>>>(a);
    } else {
        nat_aggregate_generic_kernel<<<grid, kBlock, 0, stream>>>(a);
    }
    return hipGetLastError();
}

hipError_t launch_nat_master(const NatAggregateArgs& a, const NatMasterArgs& m, bool fast, hipStream_t stream) {
    const dim3 grid = grid_for_groups(a.d, 1);
    if (fast) nat_master_kernel<<<grid, kBlock, 0, stream>>>(a, m);
    else nat_master_generic_kernel<<<grid, kBlock, 0, stream>>>(a, m);
    return hipGetLastError();
}

}  // namespace natcomp
