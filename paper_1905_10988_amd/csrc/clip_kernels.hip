// The clipped 8-bit representation of C_nat and the integer aggregator (experimental setup,
// paragraph "Implementation optimization"; appendix "Natural Compression and Dithering Allow
// for Fast Aggregation").
//
// A byte is sign << 7 | zero << 6 | (clip(exponent of C_nat(x), -50, 10) + 50).  The
// aggregator restores every byte as the 64-bit integer +-2^field (units of 2^-50, one
// non-zero bit), adds the n workers as integers and applies C_nat again to the integer sum
// (Algorithm 1, master side), so only an exponent byte and a sign bit per element travel back.
#include "device_common.hpp"
#include "kernels.hpp"

namespace natcomp {

constexpr int kClipEncBlock = 128;        // lanes per encoder workgroup, 2 quads per lane
constexpr uint32_t kClipEncTile = 1024;   // elements per encoder workgroup
constexpr uint32_t kClipBias = 127 - 50;  // exponent field of 2^-50: field f stands for exponent field f + 77

// Byte of one element in the top byte of the result (the low 24 bits are not meaningful):
// u = bits of x, rc = complement of its random word.  t holds the exponent field e of
// C_nat(x) in its top byte (255 absorbing).  The clip is two saturating operations on that
// byte: adding 255 - 137 caps e at 137 (2^10), subtracting 255 - 137 + 77 floors it at 77
// (2^-50) and leaves field = clip(e, 77, 137) - 77; neither touches the low 24 bits except
// to fill or clear them on saturation.
__device__ __forceinline__ uint32_t clip_byte_top(uint32_t u, uint32_t rc) {
    const uint32_t t = add_sat(u << 1, rc >> 8);
    const uint32_t capped = add_sat(t, (255u - (kClipBias + 60u)) << 24);
    const uint32_t field = __builtin_elementwise_sub_sat(capped, (255u - 60u) << 24);
    const uint32_t body = t < (1u << 24) ? 0x40000000u : field;  // exponent field 0: C_nat(x) = 0
    return bitfield_insert(0x80000000u, u, body);
}
__device__ __forceinline__ uint32_t clip_byte(uint32_t u, uint32_t rc) { return clip_byte_top(u, rc) >> 24; }

// Vector encoder: x 16-byte aligned, code_out 4-byte aligned, index_offset a multiple of 4,
// strides keeping that for every worker.  Lane t of a workgroup takes quads t and t + 128 of
// the tile; both loads are issued before the arithmetic.  The last d mod 4 elements go one
// by one.
__global__ __launch_bounds__(kClipEncBlock) void clip_encode_kernel(ClipEncodeArgs a) {
    const uint32_t w = blockIdx.y;
    const float* __restrict__ x = a.x + (size_t)w * a.x_stride;
    uint8_t* __restrict__ code = a.code_out + (size_t)w * a.code_stride;
    const uint32_t worker = a.first_worker + w;
    const uint64_t quads = a.d >> 2;
    const uint64_t q0 = (uint64_t)blockIdx.x * (kClipEncTile / 4) + threadIdx.x;
    const u32x4* __restrict__ xv = reinterpret_cast<const u32x4*>(x);
    uint32_t* __restrict__ cv = reinterpret_cast<uint32_t*>(code);
    u32x4 v[2];
#pragma unroll
    for (int half = 0; half < 2; ++half) {
        const uint64_t q = q0 + half * kClipEncBlock;
        v[half] = u32x4{0u, 0u, 0u, 0u};
        if (q < quads) v[half] = load_stream(xv + q);
    }
#pragma unroll
    for (int half = 0; half < 2; ++half) {
        const uint64_t q = q0 + half * kClipEncBlock;
        uint32_t rc[4];
        random_words4<true>((a.index_offset >> 2) + q, worker, kDomainNat, a.k0, a.k1, rc);
        const uint32_t bytes = pack_top_bytes(clip_byte_top(v[half].x, rc[0]), clip_byte_top(v[half].y, rc[1]),
                                              clip_byte_top(v[half].z, rc[2]), clip_byte_top(v[half].w, rc[3]));
        if (q < quads) store_stream(cv + q, bytes);
    }
    if (blockIdx.x == gridDim.x - 1 && threadIdx.x == 0) {
        for (uint64_t i = quads * 4; i < a.d; ++i) {
            const uint32_t r = random_word(a.index_offset + i, worker, kDomainNat, a.k0, a.k1);
            code[i] = (uint8_t)clip_byte(f32_bits(x[i]), ~r);
        }
    }
}

// Any alignment: 8 consecutive elements per lane, one at a time.
__global__ __launch_bounds__(kBlock) void clip_encode_generic_kernel(ClipEncodeArgs a) {
    const uint32_t w = blockIdx.y;
    const uint64_t i0 = ((uint64_t)blockIdx.x * kBlock + threadIdx.x) * 8;
    for (uint64_t i = i0; i < i0 + 8 && i < a.d; ++i) {
        const uint32_t r = random_word(a.index_offset + i, a.first_worker + w, kDomainNat, a.k0, a.k1);
        a.code_out[(size_t)w * a.code_stride + i] = (uint8_t)clip_byte(f32_bits(a.x[(size_t)w * a.x_stride + i]), ~r);
    }
}

// binary32 bits of one byte: sign and 2^(field - 50), or a signed zero.
__device__ __forceinline__ uint32_t clip_value_bits(uint32_t byte) {
    const uint32_t mag = (byte & 0x40u) ? 0u : ((byte & 63u) + kClipBias) << 23;
    return mag | ((byte & 0x80u) << 24);
}

// Vector decoder (code 8-byte aligned, out 16-byte aligned): 8 elements per lane, results
// leave through the LDS transpose.
__global__ __launch_bounds__(kBlock) void clip_decode_kernel(const uint8_t* __restrict__ code, uint64_t d,
                                                             float* __restrict__ out) {
    __shared__ u32x4 lds[2 * kBlock];
    const uint64_t g0 = (uint64_t)blockIdx.x * kBlock;
    const uint64_t grp = g0 + threadIdx.x;
    const uint64_t full = d >> 3;
    const bool have = grp < full;
    uint32_t v[8];
    if (have) {
        const u32x2 c = load_stream(reinterpret_cast<const u32x2*>(code) + grp);
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] = clip_value_bits(((j < 4 ? c.x : c.y) >> (8 * (j & 3))) & 255u);
    }
    const uint32_t groups = full - g0 < kBlock ? (uint32_t)(full - g0) : (uint32_t)kBlock;
    store_tile_transposed(lds, v, have, full > g0 ? groups : 0u, out + g0 * 8);
    if (grp == full) {
        for (uint64_t i = grp * 8; i < d; ++i) out[i] = bits_f32(clip_value_bits(code[i]));
    }
}

__global__ __launch_bounds__(kBlock) void clip_decode_generic_kernel(const uint8_t* __restrict__ code, uint64_t d,
                                                                     float* __restrict__ out) {
    const uint64_t i0 = ((uint64_t)blockIdx.x * kBlock + threadIdx.x) * 8;
    for (uint64_t i = i0; i < i0 + 8 && i < d; ++i) out[i] = bits_f32(clip_value_bits(code[i]));
}

// ------------------------------------------------------------------------ integer aggregation
// +-2^field as a 64-bit integer (two's complement), 0 when the zero flag is set.
__device__ __forceinline__ uint64_t clip_units(uint32_t byte) {
    const uint64_t mag = (uint64_t)(((byte >> 6) & 1u) ^ 1u) << (byte & 63u);
    return (byte & 0x80u) ? 0ull - mag : mag;
}

// The same through a table in LDS: entry b is the 64-bit integer byte b stands for, so an
// addend costs one byte-select-and-shift, one 8-byte LDS read and one 64-bit add.  (Built in
// registers it is two sign-extracting field reads, two three-way logic operations and a 64-bit
// shift before the add: this kernel is bound by VALU work, not by HBM.)
__device__ __forceinline__ void clip_table_fill(uint64_t* table) {
    table[threadIdx.x] = clip_units(threadIdx.x);  // kBlock = 256 lanes: one entry each
    __syncthreads();
}
__device__ __forceinline__ uint64_t clip_units_at(const uint64_t* table, uint32_t word, int j) {
    return table[(word >> (8 * j)) & 255u];
}

// C_nat of the integer sum: exponent field of the result (0 for a zero sum).  With
// 2^k <= |S| < 2^(k+1) the exponent goes up iff r < floor((|S| - 2^k) / 2^k * 2^32): the 32
// bits that follow the leading one.
__device__ __forceinline__ uint32_t clip_round_sum(uint64_t total, uint32_t r) {
    const uint64_t mag = (total >> 63) ? 0ull - total : total;
    if (mag == 0) return 0u;
    const uint32_t lz = (uint32_t)__clzll((long long)mag);
    const uint64_t top = mag << lz;                             // leading one at bit 63
    const uint32_t threshold = (uint32_t)((top << 1) >> 32);
    return (63u - lz) + kClipBias + (r < threshold ? 1u : 0u);
}

__device__ __forceinline__ uint64_t clip_sum_one(const ClipAggregateArgs& a, uint64_t i) {
    uint64_t total = 0;
    for (uint32_t w = 0; w < a.n; ++w) total += clip_units(a.code[(size_t)w * a.code_stride + i]);
    return total;
}

// NW workers starting at w0; all loads issued before the first add.
template <int NW>
__device__ __forceinline__ void clip_sum_chunk(const ClipAggregateArgs& a, const uint64_t* table, uint64_t grp,
                                               uint32_t w0, uint64_t acc[8]) {
    u32x2 c[NW];
#pragma unroll
    for (int k = 0; k < NW; ++k)
        c[k] = load_stream(reinterpret_cast<const u32x2*>(a.code + (size_t)(w0 + k) * a.code_stride) + grp);
#pragma unroll
    for (int k = 0; k < NW; ++k) {
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[j] += clip_units_at(table, j < 4 ? c[k].x : c[k].y, j & 3);
    }
}

// Vector aggregator: code planes 8-byte aligned with strides that keep it, exp_out 8-byte
// aligned, sum_out (if given) 16-byte aligned, index_offset a multiple of 4.  One lane owns
// 8 consecutive elements; the ragged last group goes element by element.
__global__ __launch_bounds__(kBlock) void clip_aggregate_kernel(ClipAggregateArgs a) {
    __shared__ uint64_t table[kBlock];
    static_assert(kBlock == 256, "one table entry per lane");
    clip_table_fill(table);
    const uint64_t grp = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
    const uint64_t full = a.d >> 3;
    if (grp < full) {
        uint64_t acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
        uint32_t w0 = 0;
        for (; w0 + 8 <= a.n; w0 += 8) clip_sum_chunk<8>(a, table, grp, w0, acc);
        for (; w0 + 2 <= a.n; w0 += 2) clip_sum_chunk<2>(a, table, grp, w0, acc);
        if (w0 < a.n) clip_sum_chunk<1>(a, table, grp, w0, acc);
        if (a.sum_out) {
            typedef uint64_t u64x2 __attribute__((ext_vector_type(2)));
            u64x2* __restrict__ so = reinterpret_cast<u64x2*>(a.sum_out + grp * 8);
#pragma unroll
            for (int j = 0; j < 4; ++j) store_stream(so + j, u64x2{acc[2 * j], acc[2 * j + 1]});
        }
        if (a.exp_out) {
            uint32_t r[8];
            const uint64_t q = (a.index_offset >> 2) + 2 * grp;
            random_words4<false>(q, a.master, kDomainMaster, a.k0, a.k1, r);
            random_words4<false>(q + 1, a.master, kDomainMaster, a.k0, a.k1, r + 4);
            uint32_t e[8], sb = 0;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                e[j] = clip_round_sum(acc[j], r[j]);
                sb |= (uint32_t)(acc[j] >> 63) << j;
            }
            u32x2 ev;
            ev.x = e[0] | (e[1] << 8) | (e[2] << 16) | (e[3] << 24);
            ev.y = e[4] | (e[5] << 8) | (e[6] << 16) | (e[7] << 24);
            store_stream(reinterpret_cast<u32x2*>(a.exp_out) + grp, ev);
            store_stream(a.sign_out + grp, (uint8_t)sb);
        }
    } else if (grp == full && (a.d & 7)) {
        uint32_t sb = 0;
        for (uint64_t i = grp * 8; i < a.d; ++i) {
            const uint64_t total = clip_sum_one(a, i);
            if (a.sum_out) a.sum_out[i] = (int64_t)total;
            if (a.exp_out) {
                const uint32_t r = random_word(a.index_offset + i, a.master, kDomainMaster, a.k0, a.k1);
                a.exp_out[i] = (uint8_t)clip_round_sum(total, r);
                sb |= (uint32_t)(total >> 63) << (i & 7);
            }
        }
        if (a.exp_out) a.sign_out[grp] = (uint8_t)sb;
    }
}

// Any alignment: one lane per group of 8 elements, element by element.
__global__ __launch_bounds__(kBlock) void clip_aggregate_generic_kernel(ClipAggregateArgs a) {
    const uint64_t i0 = ((uint64_t)blockIdx.x * kBlock + threadIdx.x) * 8;
    if (i0 >= a.d) return;
    uint32_t sb = 0;
    for (int j = 0; j < 8; ++j) {
        const uint64_t i = i0 + j;
        if (i >= a.d) break;
        const uint64_t total = clip_sum_one(a, i);
        if (a.sum_out) a.sum_out[i] = (int64_t)total;
        if (a.exp_out) {
            const uint32_t r = random_word(a.index_offset + i, a.master, kDomainMaster, a.k0, a.k1);
            a.exp_out[i] = (uint8_t)clip_round_sum(total, r);
            sb |= (uint32_t)(total >> 63) << j;
        }
    }
    if (a.exp_out) a.sign_out[i0 >> 3] = (uint8_t)sb;
}

// ------------------------------------------------------------------------ launchers
hipError_t launch_clip_encode(const ClipEncodeArgs& a, uint32_t n, bool fast, hipStream_t stream) {
    if (fast) {
        const dim3 grid((unsigned)((a.d + kClipEncTile - 1) / kClipEncTile), n, 1);
        clip_encode_kernel<<<grid, kClipEncBlock, 0, stream>>>(a);
    } else {
        const dim3 grid((unsigned)((a.d + 8 * kBlock - 1) / (8 * kBlock)), n, 1);
        clip_encode_generic_kernel<<<grid, kBlock, 0, stream>>>(a);
    }
    return hipGetLastError();
}

hipError_t launch_clip_decode(const uint8_t* code, uint64_t d, float* out, bool fast, hipStream_t stream) {
    if (fast) {
        const uint64_t groups = d / 8 + 1;  // the grid covers the ragged last group too
        clip_decode_kernel<<<(unsigned)((groups + kBlock - 1) / kBlock), kBlock, 0, stream>>>(code, d, out);
    } else {
        clip_decode_generic_kernel<<<(unsigned)((d + 8 * kBlock - 1) / (8 * kBlock)), kBlock, 0, stream>>>(code, d, out);
    }
    return hipGetLastError();
}

hipError_t launch_clip_aggregate(const ClipAggregateArgs& a, bool fast, hipStream_t stream) {
    const uint64_t groups = a.d / 8 + 1;
    const unsigned grid = (unsigned)((groups + kBlock - 1) / kBlock);
    if (fast) clip_aggregate_kernel<<<grid, kBlock, 0, stream>>>(a);
    else clip_aggregate_generic_kernel<<<grid, kBlock, 0, stream>>>(a);
    return hipGetLastError();
}

}  // namespace natcomp
