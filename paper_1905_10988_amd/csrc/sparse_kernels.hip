// Random sparsification composed with natural compression, C_nat o S^k (formal definition
// of S^q in the appendix on sparsification; composition theorem of Sec. 2), and the dense
// scatter-sum of n sparse messages (Algorithm 1's master sum).
//
// The k kept coordinates of a worker are pi(0..k-1) for a keyed permutation pi of [0, d):
// a 4-round alternating Feistel network on ceil(log2 d) bits with cycle walking, round keys = the four
// words of one Philox call (counter (0, 0, worker, 2)).  Every j is independent, so the
// selection is a plain parallel map.  One lane owns 8 consecutive j: it writes 8 indices,
// 8 exponent bytes and one whole sign byte.
#include "device_common.hpp"
#include "kernels.hpp"

namespace natcomp {

constexpr uint32_t kDomainSparse = 2;

__device__ __forceinline__ uint32_t feistel_round_fn(uint32_t r, uint32_t key) {
    uint32_t t = r * 0x9E3779B1u + key;
    t ^= t >> 16; t *= 0x85EBCA6Bu;
    t ^= t >> 13; t *= 0xC2B2AE35u;
    t ^= t >> 16;
    return t;
}

// One application of the network to a b-bit value: high part A (floor(b/2) bits), low part B;
// A ^= F(B,k0), B ^= F(A,k1), A ^= F(B,k2), B ^= F(A,k3), each truncated to its part's width.
__device__ __forceinline__ uint32_t feistel_apply(uint32_t v, uint32_t bits_b, uint32_t mask_a, uint32_t mask_b,
                                                  const uint32_t rk[4]) {
    uint32_t A = (v >> bits_b) & mask_a, B = v & mask_b;
    A ^= feistel_round_fn(B, rk[0]) & mask_a;
    B ^= feistel_round_fn(A, rk[1]) & mask_b;
    A ^= feistel_round_fn(B, rk[2]) & mask_a;
    B ^= feistel_round_fn(A, rk[3]) & mask_b;
    return (A << bits_b) | B;   // b <= 32 and A < 2^(b - bits_b): no overflow
}

// New exponent byte (top byte of the result) of u for the complemented random word rc:
// the same carry trick as the dense encoder.
__device__ __forceinline__ uint32_t nat_round_top_s(uint32_t u, uint32_t rc) { return add_sat(u << 1, rc >> 8); }

__global__ __launch_bounds__(kBlock) void sparse_nat_encode_kernel(SparseEncodeArgs a) {
    const uint32_t w = blockIdx.y;
    const float* __restrict__ x = a.x + (size_t)w * a.x_stride;
    uint32_t* __restrict__ idx_out = a.idx_out + (size_t)w * a.idx_stride;
    uint8_t* __restrict__ exp_out = a.exp_out + (size_t)w * a.exp_stride;
    uint8_t* __restrict__ sign_out = a.sign_out + (size_t)w * a.sign_stride;
    const uint32_t worker = a.first_worker + w;
    const uint64_t j0 = ((uint64_t)blockIdx.x * kBlock + threadIdx.x) * 8;
    if (j0 >= a.k) return;
    const uint32_t count = a.k - j0 < 8 ? (uint32_t)(a.k - j0) : 8u;
    uint32_t rk[4];
    philox4x32_10<false>(0u, 0u, worker, kDomainSparse, a.k0, a.k1, rk);
    // Cycle walking (apply the network until the value is below d) takes a different number of
    // rounds for every j.  The lane walks its 8 values as one queue, so a wavefront waits for the
    // slowest lane's total, not for the slowest single walk 8 times over; finished indices go
    // through an LDS column because a register array cannot be indexed by the queue position.
    __shared__ uint32_t walked[8][kBlock];
    {
        const uint32_t bits_b = a.bits - a.bits / 2;
        const uint32_t mask_a = (1u << (a.bits / 2)) - 1u, mask_b = (uint32_t)((1ull << bits_b) - 1ull);
        uint32_t t = 0;
        uint32_t v = (uint32_t)j0;           // d <= 2^32 and j < d: every value fits 32 bits
        while (t < count) {
            v = feistel_apply(v, bits_b, mask_a, mask_b, rk);
            if ((uint64_t)v < a.d) {
                walked[t][threadIdx.x] = v;
                ++t;
                v = (uint32_t)(j0 + t);
            }
        }
    }
    uint32_t idx[8];
    float xv[8];
#pragma unroll
    for (int t = 0; t < 8; ++t) idx[t] = (uint32_t)t < count ? walked[t][threadIdx.x] : 0u;
#pragma unroll
    for (int t = 0; t < 8; ++t) xv[t] = x[idx[t]];  // idx 0 for the padding lanes: always in range
    uint32_t top[8], sb = 0;
#pragma unroll
    for (int t = 0; t < 8; ++t) {
        const uint32_t u = f32_bits(a.scale * xv[t]);
        uint32_t rc[4];
        random_words4<true>((uint64_t)(idx[t] >> 2), worker, kDomainNat, a.k0, a.k1, rc);
        const uint32_t sel = idx[t] & 3u;
        const uint32_t r = sel == 0 ? rc[0] : sel == 1 ? rc[1] : sel == 2 ? rc[2] : rc[3];
        top[t] = nat_round_top_s(u, r);
        sb |= ((uint32_t)t < count ? (u >> 31) : 0u) << t;
    }
    if (count == 8 && a.vec) {
        u32x4* __restrict__ io = reinterpret_cast<u32x4*>(idx_out + j0);
        store_stream(io, u32x4{idx[0], idx[1], idx[2], idx[3]});
        store_stream(io + 1, u32x4{idx[4], idx[5], idx[6], idx[7]});
        u32x2 e;
        e.x = pack_top_bytes(top[0], top[1], top[2], top[3]);
        e.y = pack_top_bytes(top[4], top[5], top[6], top[7]);
        store_stream(reinterpret_cast<u32x2*>(exp_out + j0), e);
    } else {
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            if ((uint32_t)t < count) { idx_out[j0 + t] = idx[t]; exp_out[j0 + t] = (uint8_t)(top[t] >> 24); }
        }
    }
    sign_out[j0 >> 3] = (uint8_t)sb;
}

// out[0..d) = 0, 16 bytes per lane and two stores per lane; the last d mod 4 floats by one lane.
__global__ __launch_bounds__(kBlock) void fill_zero_kernel(float* __restrict__ out, uint64_t d) {
    const uint64_t quads = d >> 2;
    const uint64_t q0 = (uint64_t)blockIdx.x * (2 * kBlock) + threadIdx.x;
    u32x4* __restrict__ o = reinterpret_cast<u32x4*>(out);
    const u32x4 z = u32x4{0u, 0u, 0u, 0u};
    if (q0 < quads) store_stream(o + q0, z);
    if (q0 + kBlock < quads) store_stream(o + q0 + kBlock, z);
    if (blockIdx.x == 0 && threadIdx.x < (d & 3)) out[quads * 4 + threadIdx.x] = 0.0f;
}
__global__ __launch_bounds__(kBlock) void fill_zero_scalar_kernel(float* __restrict__ out, uint64_t d) {
    const uint64_t i = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i < d) out[i] = 0.0f;
}

// One worker's message added into the dense vector.  A worker's indices are distinct, so
// plain read-modify-write is race-free inside one launch; launches on the stream follow one
// another in worker order, which fixes the order of the binary32 additions.
__global__ __launch_bounds__(kBlock) void sparse_nat_scatter_kernel(SparseScatterArgs a) {
    const uint64_t j = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
    if (j >= a.k) return;
    const uint32_t i = load_stream(a.idx + j);
    const uint32_t e = load_stream(a.exp + j);
    const uint32_t sg = (a.sign[j >> 3] >> (j & 7)) & 1u;
    if (i < a.d) a.out[i] += bits_f32((sg << 31) | (e << 23));
}

hipError_t launch_sparse_nat_encode(const SparseEncodeArgs& a, uint32_t n, hipStream_t stream) {
    const uint64_t groups = (a.k + 7) / 8;
    const dim3 grid((unsigned)((groups + kBlock - 1) / kBlock), n, 1);
    sparse_nat_encode_kernel<<<grid, kBlock, 0, stream>>>(a);
    return hipGetLastError();
}

hipError_t launch_sparse_nat_aggregate(const uint32_t* idx, size_t idx_stride, const uint8_t* exp, size_t exp_stride,
                                       const uint8_t* sign, size_t sign_stride, uint32_t n, uint64_t k, uint64_t d,
                                       float* out, bool out_aligned, hipStream_t stream) {
    if (out_aligned) {
        const uint64_t quads = d / 4 + 1;
        fill_zero_kernel<<<(unsigned)((quads + 2 * kBlock - 1) / (2 * kBlock)), kBlock, 0, stream>>>(out, d);
    } else {
        fill_zero_scalar_kernel<<<(unsigned)((d + kBlock - 1) / kBlock), kBlock, 0, stream>>>(out, d);
    }
    hipError_t e = hipGetLastError();
    for (uint32_t w = 0; w < n && e == hipSuccess; ++w) {
        SparseScatterArgs a{idx + (size_t)w * idx_stride, exp + (size_t)w * exp_stride, sign + (size_t)w * sign_stride,
                            k, d, out};
        sparse_nat_scatter_kernel<<<(unsigned)((k + kBlock - 1) / kBlock), kBlock, 0, stream>>>(a);
        e = hipGetLastError();
    }
    return e;
}

}  // namespace natcomp
