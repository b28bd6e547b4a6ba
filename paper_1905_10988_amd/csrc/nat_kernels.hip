// Natural compression C_nat on gfx950: encoder, decoder and the fused n-worker
// decode-and-sum (Sec. 2, Def. 1 and the binary32 derivation; Algorithm 1's master sum).
//
// Work split: one lane owns 8 consecutive elements.  It reads them with two 16-byte
// loads, draws its 8 random words with two Philox calls, and writes 8 exponent bytes as
// one 8-byte store plus one sign byte, so a wavefront reads 2 KiB and writes 512 + 64
// contiguous bytes; no cross-lane traffic is needed.  The kernels are HBM-bound:
// 5.125 bytes per encoded element, 8*1.125 + 4 bytes per summed element at n = 8.
#include "device_common.hpp"
#include "kernels.hpp"

namespace natcomp {

// New exponent byte in the top byte of the result.  With u = (sign, e, m) and T = m * 2^9
// the rule is "exponent + 1 iff r < T".  Since T is a multiple of 2^9 this is
// (r >> 8) < 2m, i.e. 2m + (~r >> 8) carries out of 24 bits: adding the complemented
// word to u << 1 (exponent in the top byte, 2m below it) performs the comparison and the
// increment in one saturating add; saturation keeps exponent 255 at 255.
__device__ __forceinline__ uint32_t nat_round_top(uint32_t u, uint32_t r_complement) {
    return add_sat(u << 1, r_complement >> 8);
}

// One group of up to 8 elements starting at local index i0, any alignment: scalar loads,
// one Philox call per run of elements sharing a counter.
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

template <bool FAST>
__global__ __launch_bounds__(kBlock) void nat_encode_kernel(NatEncodeArgs a) {
    const uint32_t w = blockIdx.y;
    const float* __restrict__ x = a.x + (size_t)w * a.x_stride;
    uint8_t* __restrict__ exp_out = a.exp_out + (size_t)w * a.exp_stride;
    uint8_t* __restrict__ sign_out = a.sign_out + (size_t)w * a.sign_stride;
    const uint32_t worker = a.first_worker + w;
    const uint64_t grp = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
    const uint64_t i0 = grp * 8;
    if (i0 >= a.d) return;
    if (FAST && i0 + 8 <= a.d) {
        const u32x4* __restrict__ xv = reinterpret_cast<const u32x4*>(x);
        const u32x4 v0 = load_stream(xv + 2 * grp);
        const u32x4 v1 = load_stream(xv + 2 * grp + 1);
        const uint64_t q = (a.index_offset + i0) >> 2;  // index_offset is a multiple of 4 here
        uint32_t r0[4], r1[4];
        random_words4<true>(q, worker, kDomainNat, a.k0, a.k1, r0);
        random_words4<true>(q + 1, worker, kDomainNat, a.k0, a.k1, r1);
        const uint32_t y0 = nat_round_top(v0.x, r0[0]), y1 = nat_round_top(v0.y, r0[1]);
        const uint32_t y2 = nat_round_top(v0.z, r0[2]), y3 = nat_round_top(v0.w, r0[3]);
        const uint32_t y4 = nat_round_top(v1.x, r1[0]), y5 = nat_round_top(v1.y, r1[1]);
        const uint32_t y6 = nat_round_top(v1.z, r1[2]), y7 = nat_round_top(v1.w, r1[3]);
        uint32_t sg = v1.w >> 31;
        sg = push_sign(sg, v1.z); sg = push_sign(sg, v1.y); sg = push_sign(sg, v1.x);
        sg = push_sign(sg, v0.w); sg = push_sign(sg, v0.z); sg = push_sign(sg, v0.y);
        sg = push_sign(sg, v0.x);
        u32x2 packed;
        packed.x = pack_top_bytes(y0, y1, y2, y3);
        packed.y = pack_top_bytes(y4, y5, y6, y7);
        store_stream(reinterpret_cast<u32x2*>(exp_out) + grp, packed);
        store_stream(sign_out + grp, (uint8_t)sg);
    } else {
        nat_encode_group_generic(x, a.d, i0, a.index_offset, worker, a.k0, a.k1, exp_out, sign_out);
    }
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

template <bool FAST>
__global__ __launch_bounds__(kBlock) void nat_decode_kernel(NatDecodeArgs a) {
    const uint64_t grp = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
    const uint64_t i0 = grp * 8;
    if (i0 >= a.d) return;
    if (FAST && i0 + 8 <= a.d) {
        const u32x2 e = load_stream(reinterpret_cast<const u32x2*>(a.exp) + grp);
        const uint32_t sb = load_stream(a.sign + grp);
        uint32_t v[8];
        nat_decode8(e, sb, v);
        u32x4* __restrict__ o = reinterpret_cast<u32x4*>(a.out) + 2 * grp;
        store_stream(o, u32x4{v[0], v[1], v[2], v[3]});
        store_stream(o + 1, u32x4{v[4], v[5], v[6], v[7]});
    } else {
        const uint32_t sb = a.sign[i0 >> 3];
        for (int j = 0; j < 8; ++j) {
            const uint64_t i = i0 + j;
            if (i >= a.d) break;
            a.out[i] = bits_f32(nat_value_bits(a.exp[i], (sb >> j) & 1u));
        }
    }
}

// Fused decode-and-sum over n workers, 8 output elements per lane.  Workers are taken in
// chunks of up to 8 whose loads are all issued before the first add, and added in the
// fixed order w = 0, 1, ..., n-1 starting from worker 0's value.
template <bool FAST>
__global__ __launch_bounds__(kBlock) void nat_aggregate_kernel(NatAggregateArgs a) {
    const uint64_t grp = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
    const uint64_t i0 = grp * 8;
    if (i0 >= a.d) return;
    if (FAST && i0 + 8 <= a.d) {
        float acc[8];
        for (uint32_t w0 = 0; w0 < a.n; w0 += 8) {
            u32x2 e[8];
            uint32_t sb[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                if (w0 + k < a.n) {
                    const size_t w = w0 + k;
                    e[k] = load_stream(reinterpret_cast<const u32x2*>(a.exp + w * a.exp_stride) + grp);
                    sb[k] = load_stream(a.sign + w * a.sign_stride + grp);
                }
            }
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                if (w0 + k < a.n) {
                    uint32_t v[8];
                    nat_decode8(e[k], sb[k], v);
                    if (w0 + k == 0) {
#pragma unroll
                        for (int j = 0; j < 8; ++j) acc[j] = bits_f32(v[j]);
                    } else {
#pragma unroll
                        for (int j = 0; j < 8; ++j) acc[j] += bits_f32(v[j]);
                    }
                }
            }
        }
        u32x4* __restrict__ o = reinterpret_cast<u32x4*>(a.out) + 2 * grp;
        store_stream(o, u32x4{f32_bits(acc[0]), f32_bits(acc[1]), f32_bits(acc[2]), f32_bits(acc[3])});
        store_stream(o + 1, u32x4{f32_bits(acc[4]), f32_bits(acc[5]), f32_bits(acc[6]), f32_bits(acc[7])});
    } else {
        for (int j = 0; j < 8; ++j) {
            const uint64_t i = i0 + j;
            if (i >= a.d) break;
            float acc = 0.0f;
            for (uint32_t w = 0; w < a.n; ++w) {
                const uint32_t eb = a.exp[(size_t)w * a.exp_stride + i];
                const uint32_t sg = (a.sign[(size_t)w * a.sign_stride + (i >> 3)] >> (i & 7)) & 1u;
                const float v = bits_f32(nat_value_bits(eb, sg));
                acc = (w == 0) ? v : acc + v;
            }
            a.out[i] = acc;
        }
    }
}

static inline dim3 grid_for_groups(uint64_t d, uint32_t y) {
    const uint64_t groups = (d + 7) / 8;
    return dim3((unsigned)((groups + kBlock - 1) / kBlock), y, 1);
}

hipError_t launch_nat_encode(const NatEncodeArgs& a, uint32_t n, bool fast, hipStream_t stream) {
    const dim3 grid = grid_for_groups(a.d, n);
    if (fast) nat_encode_kernel<true><<<grid, kBlock, 0, stream>>>(a);
    else nat_encode_kernel<false><<<grid, kBlock, 0, stream>>>(a);
    return hipGetLastError();
}

hipError_t launch_nat_decode(const NatDecodeArgs& a, bool fast, hipStream_t stream) {
    const dim3 grid = grid_for_groups(a.d, 1);
    if (fast) nat_decode_kernel<true><<<grid, kBlock, 0, stream>>>(a);
    else nat_decode_kernel<false><<<grid, kBlock, 0, stream>>>(a);
    return hipGetLastError();
}

hipError_t launch_nat_aggregate(const NatAggregateArgs& a, bool fast, hipStream_t stream) {
    const dim3 grid = grid_for_groups(a.d, 1);
    if (fast) nat_aggregate_kernel<true><<<grid, kBlock, 0, stream>>>(a);
    else nat_aggregate_kernel<false><<<grid, kBlock, 0, stream>>>(a);
    return hipGetLastError();
}

}  // namespace natcomp
