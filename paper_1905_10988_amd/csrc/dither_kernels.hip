// Natural dithering D_nat^{p,s} on gfx950 (Sec. 3, Def. 3 with the level set
// 0, 2^(1-s), ..., 1/2, 1): segment norms, encoder, and the decoder fused with the
// n-worker sum (Algorithm 1's master sum; n = 1 is the plain decoder).
//
// As in the C_nat kernels one lane owns 8 consecutive elements, so it produces whole
// bytes of every plane by itself (4 bytes of nibble codes or 8 code bytes, 1 sign byte).
// Two encoders:
//   - fixed buckets of <= 8192 elements: one workgroup per bucket keeps the bucket in
//     registers, reduces the norm through LDS and encodes in the same pass, so x is read
//     once (4 + 0.5 or 0.625 bytes per element);
//   - any other segment description: partial norms per 2048-element chunk, one
//     wavefront per segment finishes the norm in a fixed order (no float atomics), and an
//     encode pass reads x a second time.
#include "device_common.hpp"
#include "kernels.hpp"

namespace natcomp {

// ------------------------------------------------------------------------ segments
__device__ __forceinline__ uint32_t seg_find(const Segs& sg, uint64_t i) {
    if (sg.offsets) {
        uint32_t lo = 0, hi = sg.num_segments;  // offsets[lo] <= i < offsets[hi]
        while (hi - lo > 1) {
            const uint32_t mid = (lo + hi) >> 1;
            if (sg.offsets[mid] <= i) lo = mid; else hi = mid;
        }
        return lo;
    }
    return sg.bucket ? (uint32_t)(i / sg.bucket) : 0u;
}
__device__ __forceinline__ uint64_t seg_begin(const Segs& sg, uint32_t s) {
    if (sg.offsets) return sg.offsets[s];
    return sg.bucket ? (uint64_t)s * sg.bucket : 0ull;
}
__device__ __forceinline__ uint64_t seg_end(const Segs& sg, uint32_t s) {
    if (sg.offsets) return sg.offsets[s + 1];
    if (!sg.bucket) return sg.d;
    const uint64_t e = ((uint64_t)s + 1) * sg.bucket;
    return e < sg.d ? e : sg.d;
}
__device__ __forceinline__ uint32_t seg_count(const Segs& sg) {
    if (sg.offsets) return sg.num_segments;
    return sg.bucket ? (uint32_t)((sg.d + sg.bucket - 1) / sg.bucket) : 1u;
}

// ------------------------------------------------------------------------ norms
// Accumulator of one p-norm: a double sum (p = 1, 2) or a float maximum (p = inf).
// v_max_f32 ignores NaN operands, like the comparison loop of a scalar reference.
struct NormAcc {
    double sum; float mx;
};
__device__ __forceinline__ NormAcc norm_zero() { return NormAcc{0.0, 0.0f}; }
__device__ __forceinline__ void norm_add(NormAcc& a, float x, int pnorm) {
    if (pnorm == kNormInf) a.mx = fmaxf(a.mx, fabsf(x));
    else if (pnorm == kNormL1) a.sum += (double)fabsf(x);
    else a.sum += (double)x * (double)x;
}
__device__ __forceinline__ NormAcc norm_merge(NormAcc a, NormAcc b, int pnorm) {
    if (pnorm == kNormInf) a.mx = fmaxf(a.mx, b.mx); else a.sum += b.sum;
    return a;
}
// Butterfly over the 64 lanes: every lane ends with the same bits.
__device__ __forceinline__ NormAcc norm_wave_reduce(NormAcc a, int pnorm) {
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) {
        NormAcc o;
        o.sum = __shfl_xor(a.sum, m, 64);
        o.mx = __shfl_xor(a.mx, m, 64);
        a = norm_merge(a, o, pnorm);
    }
    return a;
}
// Reduce over the workgroup in a fixed order; all lanes get the result.  `scratch` holds
// one slot per wavefront; the two barriers make it reusable right after the call.
template <int BLOCK>
__device__ __forceinline__ NormAcc norm_block_reduce(NormAcc a, int pnorm, NormAcc* scratch) {
    a = norm_wave_reduce(a, pnorm);
    constexpr int kWaves = BLOCK / 64;
    if (kWaves == 1) return a;
    const int wave = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) scratch[wave] = a;
    __syncthreads();
    NormAcc r = scratch[0];
#pragma unroll
    for (int w = 1; w < kWaves; ++w) r = norm_merge(r, scratch[w], pnorm);
    __syncthreads();
    return r;
}
__device__ __forceinline__ float norm_value(NormAcc a, int pnorm) {
    if (pnorm == kNormInf) return a.mx;
    if (pnorm == kNormL1) return (float)a.sum;
    return (float)sqrt(a.sum);
}
// Reciprocal the encoder multiplies by; a norm below the smallest normal number (zero
// included) makes the whole segment code to zeros (Def. 3: D(0) = 0).
__device__ __forceinline__ float inv_of_norm(float norm) {
    return (norm >= 1.17549435e-38f) ? 1.0f / norm : 0.0f;
}

// ------------------------------------------------------------------------ level of one element
// Parameters that depend on s only.
struct LevelParams {
    uint32_t s;
    int32_t e_min;        // 128 - s: smallest exponent field of y in the geometric region
    uint32_t regular_lo;  // (128 - s) << 23: bits of the lowest non-zero level 2^(1-s)
    float low_scale;      // 2^(s+31): y * low_scale = threshold of the linear region (s <= 95)
};
__device__ __forceinline__ LevelParams level_params(uint32_t s) {
    LevelParams p;
    p.s = s;
    p.e_min = 128 - (int32_t)s;
    p.regular_lo = (uint32_t)(128 - s) << 23;
    p.low_scale = (s <= 95) ? bits_f32((uint32_t)(127 + s + 31) << 23) : 0.0f;
    return p;
}

// Level code of y = fl(|x| * inv) given the COMPLEMENT rc of the element's random word r.
// y = 2^-k (1 + m): for y >= 2^(1-s) the code is s - k, plus one with probability m
// (r < m 2^9); below 2^(1-s) it is 1 with probability y 2^(s-1) (r < floor(y 2^(s+31)))
// and 0 otherwise; y >= 1 gives s.
//
// SMALL_S (s <= 95), branch-free: adding the 23 complemented top bits of r to y's bits
// carries into the exponent field exactly when r < m 2^9; the exponent, rebased and
// clamped to [0, s-1], is the code minus one in the geometric region and 0 below it.  The
// last unit is "geometric region, or r < T" where T = floor(y 2^(s+31)) comes from one
// multiply and a truncating conversion: one add-with-carry of T + rc + [geometric].
template <bool SMALL_S>
__device__ __forceinline__ uint32_t dither_level(float x, float inv, uint32_t rc, const LevelParams& lp) {
    const float y = fabsf(x) * inv;
    const uint32_t yb = f32_bits(y);
    if (SMALL_S) {
        const uint32_t bumped = yb + (rc >> 9);
        const int32_t rebased = (int32_t)(bumped >> 23) - lp.e_min;
        const uint32_t cm1 = (uint32_t)min(max(rebased, 0), (int32_t)lp.s - 1);  // v_med3_i32
        uint32_t T;
        asm("v_cvt_u32_f32 %0, %1" : "=v"(T) : "v"(y * lp.low_scale));  // truncates; saturates out of range
        const uint32_t geometric = (yb >= lp.regular_lo) ? 1u : 0u;
        const uint32_t plus = (uint32_t)(((uint64_t)T + rc + geometric) >> 32);
        return cm1 + plus;
    } else {
        const uint32_t ybm = yb & 0x7FFFFFFFu;
        const uint32_t r = ~rc;
        const uint32_t e_y = ybm >> 23, m = ybm & 0x7FFFFFu;
        if (ybm >= 0x3F800000u) return lp.s;
        if (e_y == 0) return 0;
        if ((int32_t)e_y >= lp.e_min) return e_y - (127u - lp.s) + (r < (m << 9) ? 1u : 0u);
        const uint32_t sh = 127u - lp.s - e_y;  // threshold = (2^31 | m 2^8) >> sh
        const uint32_t T = sh >= 32 ? 0u : ((0x80000000u | (m << 8)) >> sh);
        return r < T ? 1u : 0u;
    }
}

// ------------------------------------------------------------------------ packing of 8 codes
// Writes the planes of the group of (up to) 8 elements starting at element i0 (a multiple of
// 8 in plane coordinates).  `count` < 8 only for the last group of the vector.
template <int FMT, bool FAST>
__device__ __forceinline__ void store_codes8(const uint32_t c[8], const uint32_t u[8], uint64_t i0, uint32_t count,
                                             uint8_t* __restrict__ code_out, uint8_t* __restrict__ sign_out) {
    uint32_t sb = u[7] >> 31;
#pragma unroll
    for (int j = 6; j >= 0; --j) sb = push_sign(sb, u[j]);
    if (FMT == kFmtByte) {
        u32x2 w;
        w.x = c[0] | (c[1] << 8) | (c[2] << 16) | (c[3] << 24);
        w.y = c[4] | (c[5] << 8) | (c[6] << 16) | (c[7] << 24);
        if (FAST && count == 8) {
            store_stream(reinterpret_cast<u32x2*>(code_out + i0), w);
        } else {
            for (uint32_t j = 0; j < count; ++j) code_out[i0 + j] = (uint8_t)c[j];
        }
        sign_out[i0 >> 3] = (uint8_t)sb;
    } else {
        uint32_t w = 0;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const uint32_t nib = (FMT == kFmtFused) ? (c[j] | ((u[j] >> 28) & 8u)) : c[j];
            w |= nib << (4 * j);
        }
        if (FAST && count == 8) {
            store_stream(reinterpret_cast<uint32_t*>(code_out + (i0 >> 1)), w);
        } else {
            const uint32_t nbytes = (count + 1) >> 1;
            for (uint32_t b = 0; b < nbytes; ++b) code_out[(i0 >> 1) + b] = (uint8_t)(w >> (8 * b));
        }
        if (FMT == kFmtNibble) sign_out[i0 >> 3] = (uint8_t)sb;
    }
}

// Loads the group's bits (zeros past `count`), FAST: two 16-byte loads.
template <bool FAST>
__device__ __forceinline__ void load8(const float* __restrict__ x, uint64_t i0, uint32_t count, uint32_t u[8]) {
    if (FAST && count == 8) {
        const u32x4* p = reinterpret_cast<const u32x4*>(x + i0);
        const u32x4 a = load_stream(p), b = load_stream(p + 1);
        u[0] = a.x; u[1] = a.y; u[2] = a.z; u[3] = a.w;
        u[4] = b.x; u[5] = b.y; u[6] = b.z; u[7] = b.w;
    } else {
#pragma unroll
        for (int j = 0; j < 8; ++j) u[j] = (uint32_t)j < count ? f32_bits(x[i0 + j]) : 0u;
    }
}

// Complemented random words of the 8 elements with global indices g0 .. g0+7.
template <bool FAST>
__device__ __forceinline__ void words8(uint64_t g0, uint32_t worker, uint32_t k0, uint32_t k1, uint32_t rc[8]) {
    if (FAST) {  // g0 is a multiple of 4: two whole calls
        random_words4<true>(g0 >> 2, worker, kDomainDither, k0, k1, rc);
        random_words4<true>((g0 >> 2) + 1, worker, kDomainDither, k0, k1, rc + 4);
    } else {     // three calls cover any alignment
        uint32_t w[12];
        random_words4<true>(g0 >> 2, worker, kDomainDither, k0, k1, w);
        random_words4<true>((g0 >> 2) + 1, worker, kDomainDither, k0, k1, w + 4);
        random_words4<true>((g0 >> 2) + 2, worker, kDomainDither, k0, k1, w + 8);
        const uint32_t o = (uint32_t)g0 & 3u;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const uint32_t a = w[j], b = w[j + 1], c = w[j + 2], d = w[j + 3];
            rc[j] = o == 0 ? a : o == 1 ? b : o == 2 ? c : d;
        }
    }
}

template <int FMT, bool FAST>
__device__ __forceinline__ void encode_group(const DitherEncodeArgs& a, const uint32_t u[8], const float inv[8],
                                             uint64_t i0, uint32_t count) {
    uint32_t rc[8], c[8];
    words8<FAST>(a.index_offset + i0, a.worker, a.k0, a.k1, rc);
    const LevelParams lp = level_params(a.s);
    if (a.s <= 95) {
#pragma unroll
        for (int j = 0; j < 8; ++j) c[j] = dither_level<true>(bits_f32(u[j]), inv[j], rc[j], lp);
    } else {
#pragma unroll
        for (int j = 0; j < 8; ++j) c[j] = dither_level<false>(bits_f32(u[j]), inv[j], rc[j], lp);
    }
    store_codes8<FMT, FAST>(c, u, i0, count, a.code_out, a.sign_out);
}

// ------------------------------------------------------------------------ one-pass bucket encoder
template <int BLOCK, int FMT, bool FAST>
__global__ __launch_bounds__(BLOCK) void dither_bucket_encode_kernel(DitherEncodeArgs a) {
    __shared__ NormAcc scratch[BLOCK / 64];
    const uint64_t begin = (uint64_t)blockIdx.x * a.segs.bucket;
    const uint64_t rest = a.segs.d - begin;
    const uint32_t len = rest < a.segs.bucket ? (uint32_t)rest : a.segs.bucket;
    const uint32_t l0 = threadIdx.x * 8;
    const uint32_t count = l0 >= len ? 0u : (len - l0 < 8 ? len - l0 : 8u);
    uint32_t u[8];
    load8<FAST>(a.x, begin + l0, count, u);
    NormAcc acc = norm_zero();
#pragma unroll
    for (int j = 0; j < 8; ++j) norm_add(acc, bits_f32(u[j]), a.pnorm);  // padding zeros add nothing
    acc = norm_block_reduce<BLOCK>(acc, a.pnorm, scratch);
    const float norm = norm_value(acc, a.pnorm);
    if (threadIdx.x == 0) a.norms_out[blockIdx.x] = norm;
    if (count == 0) return;
    const float iv = inv_of_norm(norm);
    const float inv[8] = {iv, iv, iv, iv, iv, iv, iv, iv};
    encode_group<FMT, FAST>(a, u, inv, begin + l0, count);
}

// ------------------------------------------------------------------------ two-pass path
// Pass 1: partial norm of every (segment, chunk) intersection.  The piece of the segment
// that continues into a chunk from the left goes to first_partial[chunk]; a segment that
// starts inside the chunk puts its first piece into head_partial[segment].
template <bool FAST>
__global__ __launch_bounds__(kBlock) void dither_partial_kernel(DitherEncodeArgs a) {
    __shared__ NormAcc scratch[kBlock / 64];
    const Segs& sg = a.segs;
    const uint64_t cb = (uint64_t)blockIdx.x * kChunk;
    const uint64_t ce = cb + kChunk < sg.d ? cb + kChunk : sg.d;
    const uint32_t s0 = seg_find(sg, cb);
    const uint32_t nseg = seg_count(sg);
    if (seg_end(sg, s0) >= ce) {  // the whole chunk lies in one segment
        const uint64_t i0 = cb + (uint64_t)threadIdx.x * 8;
        const uint32_t count = i0 >= ce ? 0u : (ce - i0 < 8 ? (uint32_t)(ce - i0) : 8u);
        uint32_t u[8];
        load8<FAST>(a.x, i0, count, u);
        NormAcc acc = norm_zero();
#pragma unroll
        for (int j = 0; j < 8; ++j) norm_add(acc, bits_f32(u[j]), a.pnorm);
        acc = norm_block_reduce<kBlock>(acc, a.pnorm, scratch);
        if (threadIdx.x == 0) {
            const double v = a.pnorm == kNormInf ? (double)acc.mx : acc.sum;
            if (seg_begin(sg, s0) >= cb) a.head_partial[s0] = v; else a.first_partial[blockIdx.x] = v;
        }
        return;
    }
    for (uint32_t s = s0; s < nseg; ++s) {  // block-uniform loop over the segments that touch the chunk
        const uint64_t sb = seg_begin(sg, s), se = seg_end(sg, s);
        if (sb >= ce) break;
        const uint64_t b = sb > cb ? sb : cb, e = se < ce ? se : ce;
        if (e <= b) continue;  // empty segment
        NormAcc acc = norm_zero();
        for (uint64_t i = b + threadIdx.x; i < e; i += kBlock) norm_add(acc, a.x[i], a.pnorm);
        acc = norm_block_reduce<kBlock>(acc, a.pnorm, scratch);
        if (threadIdx.x == 0) {
            const double v = a.pnorm == kNormInf ? (double)acc.mx : acc.sum;
            if (sb >= cb) a.head_partial[s] = v; else a.first_partial[blockIdx.x] = v;
        }
    }
}

// Pass 2: one wavefront per segment adds the segment's partials in a fixed order.
__global__ __launch_bounds__(64) void dither_finalize_kernel(DitherEncodeArgs a) {
    const Segs& sg = a.segs;
    const uint32_t s = blockIdx.x;
    const uint64_t b = seg_begin(sg, s), e = seg_end(sg, s);
    NormAcc acc = norm_zero();
    if (e > b) {
        const uint64_t c_head = b / kChunk, c_last = (e - 1) / kChunk;
        // the piece in the chunk where the segment starts is in head_partial
        if (threadIdx.x == 0) {
            const double v = a.head_partial[s];
            if (a.pnorm == kNormInf) acc.mx = (float)v; else acc.sum = v;
        }
        for (uint64_t c = c_head + 1 + threadIdx.x; c <= c_last; c += 64) {
            const double v = a.first_partial[c];
            NormAcc o = norm_zero();
            if (a.pnorm == kNormInf) o.mx = (float)v; else o.sum = v;
            acc = norm_merge(acc, o, a.pnorm);
        }
    }
    acc = norm_wave_reduce(acc, a.pnorm);
    if (threadIdx.x == 0) {
        const float norm = norm_value(acc, a.pnorm);
        a.norms_out[s] = norm;
        a.inv_norm[s] = inv_of_norm(norm);
    }
}

// Pass 3: encode with the finished norms.
template <int FMT, bool FAST>
__global__ __launch_bounds__(kBlock) void dither_segment_encode_kernel(DitherEncodeArgs a) {
    const Segs& sg = a.segs;
    const uint64_t cb = (uint64_t)blockIdx.x * kChunk;
    const uint64_t ce = cb + kChunk < sg.d ? cb + kChunk : sg.d;
    const uint64_t i0 = cb + (uint64_t)threadIdx.x * 8;
    if (i0 >= ce) return;
    const uint32_t count = ce - i0 < 8 ? (uint32_t)(ce - i0) : 8u;
    uint32_t u[8];
    load8<FAST>(a.x, i0, count, u);
    float inv[8];
    const uint32_t s0 = seg_find(sg, cb);
    if (seg_end(sg, s0) >= ce) {
        const float iv = a.inv_norm[s0];
#pragma unroll
        for (int j = 0; j < 8; ++j) inv[j] = iv;
    } else {
        const uint32_t last = seg_count(sg) - 1;
        uint32_t s = seg_find(sg, i0);
        uint64_t se = seg_end(sg, s);
        float iv = a.inv_norm[s];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            if ((uint32_t)j < count) {
                while (i0 + j >= se && s < last) { ++s; se = seg_end(sg, s); iv = a.inv_norm[s]; }
            }
            inv[j] = iv;
        }
    }
    encode_group<FMT, FAST>(a, u, inv, i0, count);
}

// ------------------------------------------------------------------------ decode and sum
// Value bits of (norm, code c, sign): sign | fl(norm * 2^(c-s)), a signed zero for c = 0.
__device__ __forceinline__ float dither_value(float norm, uint32_t s, uint32_t c, uint32_t sign_bit) {
    const float level = bits_f32((127u + c - s) << 23);  // 2^(c-s), normal for 1 <= c <= s <= 127
    const float mag = c ? norm * level : 0.0f;
    return bits_f32(f32_bits(mag) | (sign_bit << 31));
}

// Table-driven fast path for the two nibble formats when a whole chunk lies in one segment:
// for up to 16 workers at a time the workgroup tabulates in LDS the 16 possible values of a
// nibble (fused format: sign included) and each element costs one bit-field extract, one
// LDS read and one add per worker.
template <int FMT, bool FAST>
__global__ __launch_bounds__(kBlock) void dither_aggregate_kernel(DitherAggregateArgs a) {
    __shared__ float table[16 * 16];
    const Segs& sg = a.segs;
    const uint64_t cb = (uint64_t)blockIdx.x * kChunk;
    const uint64_t ce = cb + kChunk < sg.d ? cb + kChunk : sg.d;
    const uint64_t i0 = cb + (uint64_t)threadIdx.x * 8;
    const uint32_t count = i0 >= ce ? 0u : (ce - i0 < 8 ? (uint32_t)(ce - i0) : 8u);
    const uint32_t s0 = seg_find(sg, cb);
    const bool one_segment = seg_end(sg, s0) >= ce;
    float acc[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] = 0.0f;

    if (FMT != kFmtByte && one_segment) {
        for (uint32_t w0 = 0; w0 < a.n; w0 += 16) {
            const uint32_t nw = a.n - w0 < 16 ? a.n - w0 : 16u;
            {   // tabulate: entry (w, nibble)
                const uint32_t w = threadIdx.x >> 4, nib = threadIdx.x & 15u;
                if (w < nw) {
                    const float norm = a.norms[(size_t)(w0 + w) * a.norm_stride + s0];
                    table[threadIdx.x] = (FMT == kFmtFused) ? dither_value(norm, a.s, nib & 7u, nib >> 3)
                                                           : dither_value(norm, a.s, nib, 0u);
                }
            }
            __syncthreads();
            if (count) {
                for (uint32_t w = 0; w < nw; w += 8) {
                    uint32_t cw[8], sb[8];
#pragma unroll
                    for (int k = 0; k < 8; ++k) {
                        if (w + k < nw) {
                            const size_t ww = w0 + w + k;
                            const uint8_t* cp = a.code + ww * a.code_stride + (i0 >> 1);
                            if (FAST && count == 8) {
                                cw[k] = load_stream(reinterpret_cast<const uint32_t*>(cp));
                            } else {
                                cw[k] = 0;
                                for (uint32_t b = 0; b < (count + 1) >> 1; ++b) cw[k] |= (uint32_t)cp[b] << (8 * b);
                            }
                            if (FMT == kFmtNibble) sb[k] = a.sign[ww * a.sign_stride + (i0 >> 3)];
                        }
                    }
#pragma unroll
                    for (int k = 0; k < 8; ++k) {
                        if (w + k < nw) {
                            const float* row = table + (w + k) * 16;
#pragma unroll
                            for (int j = 0; j < 8; ++j) {
                                float v = row[(cw[k] >> (4 * j)) & 15u];
                                if (FMT == kFmtNibble) v = bits_f32(f32_bits(v) | ((sb[k] << (31 - j)) & 0x80000000u));
                                acc[j] = (w0 + w + k == 0) ? v : acc[j] + v;
                            }
                        }
                    }
                }
            }
            __syncthreads();
        }
    } else if (count) {
        // any layout: walk the segments element by element
        uint32_t seg[8];
        {
            const uint32_t last = seg_count(sg) - 1;
            uint32_t s = seg_find(sg, i0);
            uint64_t se = seg_end(sg, s);
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                if ((uint32_t)j < count) {
                    while (i0 + j >= se && s < last) { ++s; se = seg_end(sg, s); }
                }
                seg[j] = s;
            }
        }
        for (uint32_t w = 0; w < a.n; ++w) {
            const uint8_t* cp = a.code + (size_t)w * a.code_stride;
            const uint32_t sbyte = (FMT == kFmtFused) ? 0u : a.sign[(size_t)w * a.sign_stride + (i0 >> 3)];
            const float* nr = a.norms + (size_t)w * a.norm_stride;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                if ((uint32_t)j < count) {
                    uint32_t c, sgn;
                    if (FMT == kFmtByte) {
                        c = cp[i0 + j]; sgn = (sbyte >> j) & 1u;
                    } else {
                        const uint32_t nib = (cp[(i0 + j) >> 1] >> (4 * (j & 1))) & 15u;
                        if (FMT == kFmtFused) { c = nib & 7u; sgn = nib >> 3; } else { c = nib; sgn = (sbyte >> j) & 1u; }
                    }
                    const float v = dither_value(nr[seg[j]], a.s, c, sgn);
                    acc[j] = (w == 0) ? v : acc[j] + v;
                }
            }
        }
    }
    if (count == 8 && FAST) {
        u32x4* o = reinterpret_cast<u32x4*>(a.out + i0);
        store_stream(o, u32x4{f32_bits(acc[0]), f32_bits(acc[1]), f32_bits(acc[2]), f32_bits(acc[3])});
        store_stream(o + 1, u32x4{f32_bits(acc[4]), f32_bits(acc[5]), f32_bits(acc[6]), f32_bits(acc[7])});
    } else {
#pragma unroll
        for (int j = 0; j < 8; ++j) if ((uint32_t)j < count) a.out[i0 + j] = acc[j];
    }
}

// ------------------------------------------------------------------------ launchers
template <int BLOCK, bool FAST>
static hipError_t launch_bucket(const DitherEncodeArgs& a, unsigned grid, hipStream_t st) {
    switch (a.fmt) {
        case kFmtFused: dither_bucket_encode_kernel<BLOCK, kFmtFused, FAST><<<grid, BLOCK, 0, st>>>(a); break;
        case kFmtNibble: dither_bucket_encode_kernel<BLOCK, kFmtNibble, FAST><<<grid, BLOCK, 0, st>>>(a); break;
        default: dither_bucket_encode_kernel<BLOCK, kFmtByte, FAST><<<grid, BLOCK, 0, st>>>(a); break;
    }
    return hipGetLastError();
}

hipError_t launch_dither_bucket_encode(const DitherEncodeArgs& a, bool fast, hipStream_t stream) {
    const unsigned grid = (unsigned)((a.segs.d + a.segs.bucket - 1) / a.segs.bucket);
    const uint32_t lanes = (a.segs.bucket + 7) / 8;
    if (lanes <= 256) return fast ? launch_bucket<256, true>(a, grid, stream) : launch_bucket<256, false>(a, grid, stream);
    if (lanes <= 512) return fast ? launch_bucket<512, true>(a, grid, stream) : launch_bucket<512, false>(a, grid, stream);
    return fast ? launch_bucket<1024, true>(a, grid, stream) : launch_bucket<1024, false>(a, grid, stream);
}

template <bool FAST>
static hipError_t launch_segment(const DitherEncodeArgs& a, hipStream_t st) {
    const unsigned chunks = (unsigned)((a.segs.d + kChunk - 1) / kChunk);
    const unsigned nseg = (unsigned)(a.segs.offsets ? a.segs.num_segments
                                     : a.segs.bucket ? (a.segs.d + a.segs.bucket - 1) / a.segs.bucket : 1);
    dither_partial_kernel<FAST><<<chunks, kBlock, 0, st>>>(a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    dither_finalize_kernel<<<nseg, 64, 0, st>>>(a);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    switch (a.fmt) {
        case kFmtFused: dither_segment_encode_kernel<kFmtFused, FAST><<<chunks, kBlock, 0, st>>>(a); break;
        case kFmtNibble: dither_segment_encode_kernel<kFmtNibble, FAST><<<chunks, kBlock, 0, st>>>(a); break;
        default: dither_segment_encode_kernel<kFmtByte, FAST><<<chunks, kBlock, 0, st>>>(a); break;
    }
    return hipGetLastError();
}

hipError_t launch_dither_segment_encode(const DitherEncodeArgs& a, bool fast, hipStream_t stream) {
    return fast ? launch_segment<true>(a, stream) : launch_segment<false>(a, stream);
}

template <bool FAST>
static hipError_t launch_agg(const DitherAggregateArgs& a, hipStream_t st) {
    const unsigned chunks = (unsigned)((a.segs.d + kChunk - 1) / kChunk);
    switch (a.fmt) {
        case kFmtFused: dither_aggregate_kernel<kFmtFused, FAST><<<chunks, kBlock, 0, st>>>(a); break;
        case kFmtNibble: dither_aggregate_kernel<kFmtNibble, FAST><<<chunks, kBlock, 0, st>>>(a); break;
        default: dither_aggregate_kernel<kFmtByte, FAST><<<chunks, kBlock, 0, st>>>(a); break;
    }
    return hipGetLastError();
}

hipError_t launch_dither_aggregate(const DitherAggregateArgs& a, bool fast, hipStream_t stream) {
    return fast ? launch_agg<true>(a, stream) : launch_agg<false>(a, stream);
}

}  // namespace natcomp
