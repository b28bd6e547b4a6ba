// Natural dithering D_nat^{p,s} on gfx950 (Sec. 3, Def. 3 with the level set
// 0, 2^(1-s), ..., 1/2, 1): segment norms, encoder, and the decoder fused with the
// n-worker sum (Algorithm 1's master sum; n = 1 is the plain decoder).
//
// Vector paths use the access shapes of the C_nat kernels: 16-byte lane-contiguous loads
// (one quad = 4 elements = one Philox call per load), code halves and sign nibbles gathered
// across neighbouring lanes with DPP row shifts so that stores are whole words, float
// results transposed through LDS.  The scalar paths (any alignment, ragged tails, chunks
// that straddle segment boundaries) let one lane own 8 consecutive elements, so it produces
// whole bytes of every plane by itself.
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
// The segment of a wavefront-uniform position together with what the kernels need next: its
// bounds and, if aux is given, aux[segment] (a norm or its reciprocal).  With segment offsets
// the binary search runs on the scalar unit: every step is a scalar load through the scalar data
// cache (the offsets and aux arrays are only read by the kernels that search them), counted by
// lgkmcnt, so the search neither waits for the kernel's vector loads in flight nor needs LDS or a
// barrier.  (A search by the whole workgroup, lane t testing segment t and publishing through
// LDS, costs the same in the norm pass and 1.3 us of 25.9 more in the config-3 decoder; the same
// binary search with vector loads waits for the data loads at every step: 22.3 us for a norm
// pass of 19.0.)  i must be wavefront-uniform.
struct SegHit {
    uint32_t s;
    float aux;
    uint64_t begin, end;
};
__device__ __forceinline__ uint64_t scalar_load_u64(const uint64_t* base, uint32_t k) {
    uint64_t v;
    asm volatile("s_load_dwordx2 %0, %1, %2\n\ts_waitcnt lgkmcnt(0)" : "=s"(v) : "s"(base), "s"(k * 8u));
    return v;
}
__device__ __forceinline__ float scalar_load_f32(const float* base, uint32_t k) {
    float v;
    asm volatile("s_load_dword %0, %1, %2\n\ts_waitcnt lgkmcnt(0)" : "=s"(v) : "s"(base), "s"(k * 4u));
    return v;
}
__device__ __forceinline__ SegHit seg_find_hit(const Segs& sg, uint64_t i, const float* __restrict__ aux) {
    SegHit h;
    if (sg.offsets && sg.num_segments < (1u << 29)) {  // (byte offsets of the scalar loads fit 32 bits)
        uint32_t lo = 0, hi = sg.num_segments;  // offsets[lo] <= i < offsets[hi]
        while (hi - lo > 1) {
            const uint32_t mid = (lo + hi) >> 1;
            if (scalar_load_u64(sg.offsets, mid) <= i) lo = mid; else hi = mid;
        }
        h.s = lo;
        h.begin = scalar_load_u64(sg.offsets, lo);
        h.end = scalar_load_u64(sg.offsets, lo + 1);
        h.aux = aux ? scalar_load_f32(aux, lo) : 0.0f;
        return h;
    }
    h.s = seg_find(sg, i);
    if (sg.offsets) {
        h.begin = sg.offsets[h.s];
        h.end = sg.offsets[h.s + 1];
    } else {
        h.begin = sg.bucket ? (uint64_t)h.s * sg.bucket : 0ull;
        h.end = sg.bucket && h.begin + sg.bucket < sg.d ? h.begin + sg.bucket : sg.d;
    }
    h.aux = aux ? aux[h.s] : 0.0f;
    return h;
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
__device__ __forceinline__ uint32_t seg_count(const Segs& sg) { return sg.count; }

// Segment boundaries inside one chunk, staged in LDS.  Segment s0 holds the chunk's first
// element cb; lane t looks at the begin of segment s0 + 1 + t and, if it lies before the
// chunk's end ce, writes its chunk-local position to bnd[t] (ascending; empty segments repeat
// a position).  Returns how many were staged; kBlock means "kBlock or more", and the caller
// falls back to searching the offsets in global memory.  All lanes must call (barrier inside).
// The segment of chunk-local position l is then s0 + #{t : bnd[t] <= l}.
__device__ __forceinline__ uint32_t stage_boundaries(const Segs& sg, uint64_t cb, uint64_t ce, uint32_t s0,
                                                     uint32_t* bnd) {
    const uint32_t s = s0 + 1 + threadIdx.x;
    bool in = false;
    if (s < seg_count(sg)) {
        const uint64_t b = seg_begin(sg, s);
        if (b < ce) { bnd[threadIdx.x] = (uint32_t)(b - cb); in = true; }
    }
    return (uint32_t)__syncthreads_count(in);
}
// A lane's position in the staged boundaries: idx = number of boundaries at or before the
// lane's current element (its segment is s0 + idx), next = position of the following one.
struct SegCursor {
    uint32_t idx, next;
};
__device__ __forceinline__ SegCursor cursor_at(const uint32_t* bnd, uint32_t nb, uint32_t l) {
    uint32_t lo = 0, hi = nb;
    while (lo < hi) {
        const uint32_t mid = (lo + hi) >> 1;
        if (bnd[mid] <= l) lo = mid + 1; else hi = mid;
    }
    return SegCursor{lo, lo < nb ? bnd[lo] : 0xFFFFFFFFu};
}
// Moves the cursor forward to position l; true if the segment changed.
__device__ __forceinline__ bool cursor_advance(SegCursor& c, const uint32_t* bnd, uint32_t nb, uint32_t l) {
    bool moved = false;
    while (l >= c.next) {
        ++c.idx;
        c.next = c.idx < nb ? bnd[c.idx] : 0xFFFFFFFFu;
        moved = true;
    }
    return moved;
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
    else a.sum = __builtin_fma((double)x, (double)x, a.sum);  // (the square of a binary32 value is exact in double)
}
__device__ __forceinline__ NormAcc norm_merge(NormAcc a, NormAcc b, int pnorm) {
    if (pnorm == kNormInf) a.mx = fmaxf(a.mx, b.mx); else a.sum += b.sum;
    return a;
}
// Butterfly over the 64 lanes: every lane ends with the same bits.
__device__ __forceinline__ NormAcc norm_wave_reduce(NormAcc a, int pnorm) {
    if (pnorm == kNormInf) {
#pragma unroll
        for (int m = 32; m >= 1; m >>= 1) a.mx = fmaxf(a.mx, __shfl_xor(a.mx, m, 64));
    } else {
#pragma unroll
        for (int m = 32; m >= 1; m >>= 1) a.sum += __shfl_xor(a.sum, m, 64);
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
    int32_t e_base;       // 127 - s: exponent field of 2^-s, one below that of the lowest non-zero level
    int32_t e_max;        // 127: exponent field of y = 1, the top level
    float half_lowest;    // 2^-s (s <= 95)
    uint32_t standard;    // 1: standard dithering (levels j/s) instead of the natural level set
    float s_float;        // s as a float (standard dithering)
};
__device__ __forceinline__ LevelParams level_params(uint32_t s, uint32_t standard) {
    LevelParams p;
    p.s = s;
    p.standard = standard;
    p.s_float = (float)s;
    p.e_base = 127 - (int32_t)s;
    p.e_max = 127;
    p.half_lowest = (s <= 95 && !standard) ? bits_f32((uint32_t)(127 - s) << 23) : 0.0f;
    return p;
}

// Level code of y = fl(|x| * inv) given the COMPLEMENT rc of the element's random word r, of
// which the top 23 bits r23 decide.  y = 2^-k (1 + m): for y >= 2^(1-s) the code is s - k, plus
// one with probability m (r23 < m 2^23); below 2^(1-s) it is 1 with probability y 2^(s-1) taken
// to 23 bits (r23 < round(y 2^(s+22)), ties to even) and 0 otherwise; y >= 1 gives s.
//
// SMALL_S (s <= 95), branch-free.  Below the lowest level, z = fl(y/2 + 2^-s) -- one fused
// multiply-add -- lies in [2^-s, 2^(1-s)] and its mantissa field is exactly that 23-bit
// threshold, so both regions become one rule on w = max(y, z) (z <= y from 2^(1-s) on): adding
// the 23 complemented top bits of r to w's bits carries into the exponent field exactly when
// r23 is below w's mantissa, and the exponent field, clamped to [127-s, 127] and rebased, is
// the code.
template <bool SMALL_S>
__device__ __forceinline__ uint32_t dither_level(float x, float inv, uint32_t rc, const LevelParams& lp) {
    const float y = fabsf(x) * inv;
    if (SMALL_S) {
        const float w = fmaxf(y, __builtin_fmaf(y, 0.5f, lp.half_lowest));
        const uint32_t bumped = f32_bits(w) + (rc >> 9);
        int32_t e_clamped;
        asm("v_med3_i32 %0, %1, %2, %3" : "=v"(e_clamped) : "v"(bumped >> 23), "v"(lp.e_base), "v"(lp.e_max));
        return (uint32_t)(e_clamped - lp.e_base);
    } else {
        const uint32_t ybm = f32_bits(y) & 0x7FFFFFFFu;
        const uint32_t r23 = ~rc >> 9;
        const uint32_t e_y = ybm >> 23, m = ybm & 0x7FFFFFu;
        if (ybm >= 0x3F800000u) return lp.s;
        if (e_y + lp.s >= 128u) return e_y - (127u - lp.s) + (r23 < m ? 1u : 0u);
        // y 2^(s+22) = M / 2^sh with M the 24-bit significand (no hidden bit for a subnormal y)
        const uint32_t M = e_y ? (0x800000u | m) : m;
        const uint32_t sh = 128u - lp.s - (e_y ? e_y : 1u);
        uint32_t T;
        if (sh == 0) {
            T = M;
        } else if (sh > 25) {
            T = 0;
        } else {
            const uint32_t q = M >> sh, rem = M & ((1u << sh) - 1u), half = 1u << (sh - 1);
            T = q + ((rem > half || (rem == half && (q & 1u))) ? 1u : 0u);
        }
        return r23 < T ? 1u : 0u;
    }
}

// Standard dithering (Def. 3 with the linear partition l = j/s, the QSGD / TernGrad operator,
// kept as the comparison operator of the empirical-variance study): t = fl(y s) lies between
// the levels floor(t)/s and (floor(t)+1)/s and goes up with probability t - floor(t), compared
// as floor(frac 2^32) against the random word; y >= 1 (or a NaN) is the top level s.
__device__ __forceinline__ uint32_t dither_level_standard(float x, float inv, uint32_t rc, const LevelParams& lp) {
    const float y = fabsf(x) * inv;
    const float t = y * lp.s_float;
    if (!(t < lp.s_float)) return lp.s;
    const float fl = floorf(t);
    const float frac = t - fl;  // exact
    uint32_t T;
    asm("v_cvt_u32_f32 %0, %1" : "=v"(T) : "v"(frac * 4294967296.0f));  // exact: frac < 1 has 24 bits
    uint32_t unused;
    const bool below = __builtin_uadd_overflow(T, rc, &unused);  // r < T
    return (uint32_t)fl + (below ? 1u : 0u);
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

// The dithering stream: one Philox call per 8 consecutive elements, counter (g/8, worker, 1).
// Elements 0..3 of the group share (a, b) = (w0, w1), elements 4..7 (a, b) = (w2, w3); the four
// elements of such a half take a, b, a<<16 | b>>16 and b<<16 | a>>16: each a rearrangement of
// 32 distinct bits of the call's output, so uniform by itself, which is all that unbiasedness
// and the second-moment bound of the operator need (they are sums over coordinates).
// Complementing commutes with the rearrangement, so the kernels draw complemented calls.
__device__ __forceinline__ void dither_half_words(uint32_t a, uint32_t b, uint32_t rc[4]) {
    rc[0] = a;
    rc[1] = b;
    rc[2] = __builtin_amdgcn_alignbit(a, b, 16);
    rc[3] = __builtin_amdgcn_alignbit(b, a, 16);
}
// Complemented words of the 8 elements of group `call` (global elements 8 call .. 8 call + 7).
__device__ __forceinline__ void dither_group_words(uint64_t call, uint32_t worker, uint32_t k0, uint32_t k1,
                                                   uint32_t rc[8]) {
    uint32_t w[4];
    philox4x32_10<true>((uint32_t)call, (uint32_t)(call >> 32), worker, kDomainDither, k0, k1, w);
    dither_half_words(w[0], w[1], rc);
    dither_half_words(w[2], w[3], rc + 4);
}
// Complemented words of the quad with global quad index gq (global elements 4 gq .. 4 gq + 3).
__device__ __forceinline__ void dither_quad_words(uint64_t gq, uint32_t worker, uint32_t k0, uint32_t k1,
                                                  uint32_t rc[4]) {
    uint32_t w[4];
    philox4x32_10<true>((uint32_t)(gq >> 1), (uint32_t)(gq >> 33), worker, kDomainDither, k0, k1, w);
    const bool upper = gq & 1u;
    dither_half_words(upper ? w[2] : w[0], upper ? w[3] : w[1], rc);
}
// The same for two quads per lane at one call per lane.  Contract: all 64 lanes call; lane l and
// lane l ^ 1 hold the two quads of one group, in both rounds (global quad indices gq_a and gq_b
// of the lane: gq_x even in even lanes, and lane l ^ 1 holds gq_x ^ 1).  Even lanes then draw the
// call of round a, odd lanes the call of round b, and adjacent lanes exchange halves.
__device__ __forceinline__ void dither_quad_words_two_rounds(uint64_t gq_a, uint64_t gq_b, uint32_t worker,
                                                             uint32_t k0, uint32_t k1, uint32_t rc_a[4],
                                                             uint32_t rc_b[4]) {
    const bool odd = gq_a & 1u;
    const uint64_t call = (odd ? gq_b : gq_a) >> 1;
    uint32_t w[4], o[4];
    philox4x32_10<true>((uint32_t)call, (uint32_t)(call >> 32), worker, kDomainDither, k0, k1, w);
#pragma unroll
    for (int i = 0; i < 4; ++i) o[i] = __builtin_amdgcn_update_dpp(0u, w[i], 0xB1, 0xF, 0xF, true);  // lane l ^ 1's word
    dither_half_words(odd ? o[2] : w[0], odd ? o[3] : w[1], rc_a);  // round a: the even lane's call
    dither_half_words(odd ? w[2] : o[0], odd ? w[3] : o[1], rc_b);  // round b: the odd lane's call
}

// Complemented random words of the 8 elements with global indices g0 .. g0+7.
template <bool FAST>
__device__ __forceinline__ void words8(uint64_t g0, uint32_t worker, uint32_t k0, uint32_t k1, uint32_t rc[8]) {
    const uint32_t o = (uint32_t)g0 & 7u;
    if (FAST && o == 0) {  // one whole group
        dither_group_words(g0 >> 3, worker, k0, k1, rc);
        return;
    }
    uint32_t w[16];  // two groups cover any alignment
    dither_group_words(g0 >> 3, worker, k0, k1, w);
    dither_group_words((g0 >> 3) + 1, worker, k0, k1, w + 8);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        uint32_t r = w[j];
#pragma unroll
        for (int sh = 1; sh < 8; ++sh) r = o == (uint32_t)sh ? w[j + sh] : r;
        rc[j] = r;
    }
}

template <int FMT, bool FAST>
__device__ __forceinline__ void encode_group(const DitherEncodeArgs& a, const uint32_t u[8], const float inv[8],
                                             uint64_t i0, uint32_t count) {
    uint32_t rc[8], c[8];
    words8<FAST>(a.index_offset + i0, a.worker, a.k0, a.k1, rc);
    const LevelParams lp = level_params(a.s, a.standard);
    if (a.standard) {
#pragma unroll
        for (int j = 0; j < 8; ++j) c[j] = dither_level_standard(bits_f32(u[j]), inv[j], rc[j], lp);
    } else if (a.s <= 95) {
#pragma unroll
        for (int j = 0; j < 8; ++j) c[j] = dither_level<true>(bits_f32(u[j]), inv[j], rc[j], lp);
    } else {
#pragma unroll
        for (int j = 0; j < 8; ++j) c[j] = dither_level<false>(bits_f32(u[j]), inv[j], rc[j], lp);
    }
    store_codes8<FMT, FAST>(c, u, i0, count, a.code_out, a.sign_out);
}

// ------------------------------------------------------------------------ vector (quad) encode
// Level codes of one quad; inv[j] is the reciprocal norm of element j's segment.
__device__ __forceinline__ void levels4(u32x4 v, const float inv[4], const uint32_t rc[4], const LevelParams& lp,
                                        uint32_t c[4]) {
    if (lp.standard) {
        c[0] = dither_level_standard(bits_f32(v.x), inv[0], rc[0], lp);
        c[1] = dither_level_standard(bits_f32(v.y), inv[1], rc[1], lp);
        c[2] = dither_level_standard(bits_f32(v.z), inv[2], rc[2], lp);
        c[3] = dither_level_standard(bits_f32(v.w), inv[3], rc[3], lp);
    } else if (lp.s <= 95) {
        c[0] = dither_level<true>(bits_f32(v.x), inv[0], rc[0], lp);
        c[1] = dither_level<true>(bits_f32(v.y), inv[1], rc[1], lp);
        c[2] = dither_level<true>(bits_f32(v.z), inv[2], rc[2], lp);
        c[3] = dither_level<true>(bits_f32(v.w), inv[3], rc[3], lp);
    } else {
        c[0] = dither_level<false>(bits_f32(v.x), inv[0], rc[0], lp);
        c[1] = dither_level<false>(bits_f32(v.y), inv[1], rc[1], lp);
        c[2] = dither_level<false>(bits_f32(v.z), inv[2], rc[2], lp);
        c[3] = dither_level<false>(bits_f32(v.w), inv[3], rc[3], lp);
    }
}
__device__ __forceinline__ uint32_t sign_nibble4(u32x4 v) {
    uint32_t sg = v.w >> 31;
    sg = push_sign(sg, v.z);
    sg = push_sign(sg, v.y);
    return push_sign(sg, v.x);
}

// Encodes quad q of the workgroup's tile and stores its codes; code_base / sign_base point
// at the tile's first code / sign word (workgroup-uniform, so q stays a 32-bit offset) and
// rc holds the complemented random words of its four elements.  Must be called by all 64 lanes
// of a wavefront with consecutive q (lane l holds q0 + l, q0 a multiple of 8); `in` says
// whether the lane's quad exists and is the same for each run of 8 lanes.  Stores: nibble formats, one word of
// 8 codes from every even lane; byte format, one word of 4 codes from every lane; sign
// planes, one word of 32 sign bits from every 8th lane.
template <int FMT>
__device__ __forceinline__ void encode_store_quad(const DitherEncodeArgs& a, const LevelParams& lp, u32x4 v,
                                                  const float inv[4], uint32_t* __restrict__ code_base,
                                                  uint32_t* __restrict__ sign_base, uint32_t q, const uint32_t rc[4],
                                                  bool in) {
    uint32_t c[4];
    levels4(v, inv, rc, lp, c);
    if (FMT == kFmtByte) {
        const uint32_t w = c[0] | (c[1] << 8) | (c[2] << 16) | (c[3] << 24);
        if (in) store_stream(code_base + q, w);
    } else {
        uint32_t h = c[0] | (c[1] << 4) | (c[2] << 8) | (c[3] << 12);
        if (FMT == kFmtFused)  // sign bit of element j to bit 4j+3
            h |= ((v.x >> 28) & 0x8u) | ((v.y >> 24) & 0x80u) | ((v.z >> 20) & 0x800u) | ((v.w >> 16) & 0x8000u);
        const uint32_t w = h | (from_lane_plus<1>(h) << 16);
        if (in && (threadIdx.x & 1) == 0) store_stream(code_base + (q >> 1), w);
    }
    if (FMT != kFmtFused) {
        const uint32_t packed = gather_nibbles8(sign_nibble4(v));
        if (in && (threadIdx.x & 7) == 0) store_stream(sign_base + (q >> 3), packed);
    }
}

// Words of the lane's quads q_a and q_b (tile-local; q_global is the tile's first quad in the
// random stream).  When q_global is even -- lanes then hold the two quads of a group side by
// side -- one call per lane serves both rounds; otherwise every quad draws the call it lies in.
__device__ __forceinline__ void tile_quad_words(const DitherEncodeArgs& a, uint64_t q_global, uint32_t q_a, uint32_t q_b,
                                                uint32_t rc_a[4], uint32_t rc_b[4]) {
    if ((q_global & 1u) == 0) {  // wave-uniform
        dither_quad_words_two_rounds(q_global + q_a, q_global + q_b, a.worker, a.k0, a.k1, rc_a, rc_b);
    } else {
        dither_quad_words(q_global + q_a, a.worker, a.k0, a.k1, rc_a);
        dither_quad_words(q_global + q_b, a.worker, a.k0, a.k1, rc_b);
    }
}

template <int P>
__device__ __forceinline__ void norm_add4_p(NormAcc& acc, u32x4 v) {
    norm_add(acc, bits_f32(v.x), P);
    norm_add(acc, bits_f32(v.y), P);
    norm_add(acc, bits_f32(v.z), P);
    norm_add(acc, bits_f32(v.w), P);
}
// Accumulates N quads; the switch on p is taken once, not per element.
template <int N>
__device__ __forceinline__ void norm_add_quads(NormAcc& acc, const u32x4 (&v)[N], int pnorm) {
    if (pnorm == kNormInf) {
#pragma unroll
        for (int k = 0; k < N; ++k) norm_add4_p<kNormInf>(acc, v[k]);
    } else if (pnorm == kNormL1) {
#pragma unroll
        for (int k = 0; k < N; ++k) norm_add4_p<kNormL1>(acc, v[k]);
    } else {
#pragma unroll
        for (int k = 0; k < N; ++k) norm_add4_p<kNormL2>(acc, v[k]);
    }
}

// One-pass bucket encoder, vector path: bucket a multiple of 32 and at most 8192 elements,
// x 16-byte aligned, code_out and sign_out 4-byte aligned, index_offset a multiple of 4.
// One workgroup of 256 lanes per bucket; lane t owns quads t, t+256, ... (QPL of them),
// all loaded before the norm is reduced, then encoded from registers.
// (The register budget is capped for 6 wavefronts per SIMD: left alone, the scheduler
// interleaves the QPL Philox chains and the kernel ends up with 2 wavefronts per SIMD.)
template <int QPL, int FMT>
__global__ __launch_bounds__(kBlock) __attribute__((amdgpu_waves_per_eu(6, 8)))
void dither_bucket_encode_vec_kernel(DitherEncodeArgs a) {
    __shared__ NormAcc scratch[kBlock / 64];
    const uint64_t begin = (uint64_t)blockIdx.x * a.segs.bucket;
    const uint64_t rest = a.segs.d - begin;
    const uint32_t len = rest < a.segs.bucket ? (uint32_t)rest : a.segs.bucket;
    const uint32_t vec_quads = (len >> 5) << 3;  // quads inside whole groups of 32 elements
    const u32x4* __restrict__ xv = reinterpret_cast<const u32x4*>(a.x + begin);
    u32x4 v[QPL];
#pragma unroll
    for (int k = 0; k < QPL; ++k) {
        const uint32_t q = threadIdx.x + k * kBlock;
        v[k] = u32x4{0u, 0u, 0u, 0u};
        if (q < vec_quads) v[k] = load_stream(xv + q);
    }
    NormAcc acc = norm_zero();
    norm_add_quads(acc, v, a.pnorm);
    const uint32_t tail0 = vec_quads * 4;  // the last bucket may end with up to 31 more elements
    if (tail0 + threadIdx.x < len) norm_add(acc, a.x[begin + tail0 + threadIdx.x], a.pnorm);
    acc = norm_block_reduce<kBlock>(acc, a.pnorm, scratch);
    const float norm = norm_value(acc, a.pnorm);
    if (threadIdx.x == 0) a.norms_out[blockIdx.x] = norm;
    const float iv = inv_of_norm(norm);
    const float iv4[4] = {iv, iv, iv, iv};
    const LevelParams lp = level_params(a.s, a.standard);
    const uint64_t q_global = (a.index_offset + begin) >> 2;
    uint32_t* __restrict__ code_base = reinterpret_cast<uint32_t*>(a.code_out + (FMT == kFmtByte ? begin : begin >> 1));
    uint32_t* __restrict__ sign_base = reinterpret_cast<uint32_t*>(a.sign_out + (begin >> 3));
    if (QPL == 1) {
        uint32_t rc[4];
        dither_quad_words(q_global + threadIdx.x, a.worker, a.k0, a.k1, rc);
        encode_store_quad<FMT>(a, lp, v[0], iv4, code_base, sign_base, threadIdx.x, rc, threadIdx.x < vec_quads);
    } else {
#pragma unroll
        for (int k = 0; k + 1 < QPL; k += 2) {
            const uint32_t q = threadIdx.x + k * kBlock;
            if (k * kBlock < vec_quads) {  // block-uniform: skip rounds no lane takes part in
                uint32_t rc_a[4], rc_b[4];
                tile_quad_words(a, q_global, q, q + kBlock, rc_a, rc_b);
                encode_store_quad<FMT>(a, lp, v[k], iv4, code_base, sign_base, q, rc_a, q < vec_quads);
                __builtin_amdgcn_sched_barrier(0);  // one quad at a time keeps the register count low
                if ((k + 1) * kBlock < vec_quads)
                    encode_store_quad<FMT>(a, lp, v[k + 1], iv4, code_base, sign_base, q + kBlock, rc_b,
                                           q + kBlock < vec_quads);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    if (tail0 < len && threadIdx.x < 4 && tail0 + threadIdx.x * 8 < len) {
        const uint32_t l0 = tail0 + threadIdx.x * 8;
        const uint32_t count = len - l0 < 8 ? len - l0 : 8u;
        uint32_t u[8];
        load8<false>(a.x, begin + l0, count, u);
        const float inv[8] = {iv, iv, iv, iv, iv, iv, iv, iv};
        encode_group<FMT, false>(a, u, inv, begin + l0, count);
    }
}

// ------------------------------------------------------------------------ one-pass bucket encoder
// One bucket by a whole workgroup, lane t owning elements 8t .. 8t+7 of it (BLOCK * 8 >= bucket).
// All lanes of the workgroup must call; `scratch` has one slot per wavefront.
template <int BLOCK, int FMT, bool FAST>
__device__ __forceinline__ void bucket_encode_by_workgroup(const DitherEncodeArgs& a, uint64_t bucket_index,
                                                           NormAcc* scratch) {
    const uint64_t begin = bucket_index * a.segs.bucket;
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
    if (threadIdx.x == 0) a.norms_out[bucket_index] = norm;
    if (count == 0) return;
    const float iv = inv_of_norm(norm);
    const float inv[8] = {iv, iv, iv, iv, iv, iv, iv, iv};
    encode_group<FMT, FAST>(a, u, inv, begin + l0, count);
}
template <int BLOCK, int FMT, bool FAST>
__global__ __launch_bounds__(BLOCK) void dither_bucket_encode_kernel(DitherEncodeArgs a) {
    __shared__ NormAcc scratch[BLOCK / 64];
    bucket_encode_by_workgroup<BLOCK, FMT, FAST>(a, blockIdx.x, scratch);
}

// One-pass encoder for buckets of 32 .. 2048 elements that are a multiple of 32, vector path
// (same alignment as the kernel above).  A workgroup takes 256 / L whole buckets; a bucket of
// W = bucket / 4 quads belongs to L consecutive lanes of one wavefront (8 <= L <= 64, a power of
// two with QPL * L >= W; buckets above 2048 are better served by the one-bucket-per-workgroup
// kernel above), lane r of them holding quads r, r + L, ... of the bucket (those below W), so
// every load instruction reads runs of up to 16 L contiguous bytes and every aligned group of 8
// lanes holds 8 consecutive quads (what the packed stores need).  The norm is reduced inside the bucket's
// lanes with xor-butterfly steps (no LDS, no barrier); the square root and the reciprocal are
// computed once per lane for its QPL quads.  The tiles hold the `full_buckets` whole buckets; a
// ragged last bucket is encoded by the last workgroup after its tile, lane by lane.
template <int QPL, int FMT>
__global__ __launch_bounds__(kBlock) __attribute__((amdgpu_waves_per_eu(6, 8)))
void dither_multi_bucket_encode_kernel(DitherEncodeArgs a, uint32_t log2_l, uint64_t full_buckets) {
    __shared__ NormAcc scratch[kBlock / 64];
    const uint32_t lanes = 1u << log2_l;                   // L
    const uint32_t quads = a.segs.bucket >> 2;             // W <= QPL * L
    const uint32_t b_local = threadIdx.x >> log2_l;        // bucket of this lane inside the tile
    const uint32_t r = threadIdx.x & (lanes - 1u);
    const uint32_t q_first = b_local * quads + r;          // tile-local quad of k = 0
    const uint64_t tile_quad0 = ((uint64_t)blockIdx.x << (8 - log2_l)) * quads;
    const uint64_t bucket_index = ((uint64_t)blockIdx.x << (8 - log2_l)) + b_local;
    const bool have = bucket_index < full_buckets;         // the same for all lanes of a bucket
    const u32x4* __restrict__ xv = reinterpret_cast<const u32x4*>(a.x) + tile_quad0;
    u32x4 v[QPL];
    bool in[QPL];                                          // W is a multiple of 8: the same for 8 aligned lanes
#pragma unroll
    for (int k = 0; k < QPL; ++k) {
        v[k] = u32x4{0u, 0u, 0u, 0u};
        in[k] = have && r + k * lanes < quads;
        if (in[k]) v[k] = load_stream(xv + q_first + k * lanes);
    }
    NormAcc acc = norm_zero();
    norm_add_quads(acc, v, a.pnorm);
    if (a.pnorm == kNormInf) {  // constant masks (cheap lane exchanges); steps 8, 16, 32 only for wider buckets
#pragma unroll
        for (int m = 1; m < 64; m <<= 1)
            if (m < 8 || (uint32_t)m < lanes) acc.mx = fmaxf(acc.mx, __shfl_xor(acc.mx, m, 64));
    } else {
#pragma unroll
        for (int m = 1; m < 64; m <<= 1)
            if (m < 8 || (uint32_t)m < lanes) acc.sum += __shfl_xor(acc.sum, m, 64);
    }
    const float norm = norm_value(acc, a.pnorm);
    if (have && r == 0) a.norms_out[bucket_index] = norm;
    const float iv = inv_of_norm(norm);
    const float iv4[4] = {iv, iv, iv, iv};
    const LevelParams lp = level_params(a.s, a.standard);
    const uint64_t tile_elem0 = tile_quad0 * 4;
    const uint64_t q_global = (a.index_offset >> 2) + tile_quad0;
    uint32_t* __restrict__ code_base =
        reinterpret_cast<uint32_t*>(a.code_out + (FMT == kFmtByte ? tile_elem0 : tile_elem0 >> 1));
    uint32_t* __restrict__ sign_base = reinterpret_cast<uint32_t*>(a.sign_out + (tile_elem0 >> 3));
    if (QPL == 1) {
        uint32_t rc[4];
        dither_quad_words(q_global + q_first, a.worker, a.k0, a.k1, rc);
        encode_store_quad<FMT>(a, lp, v[0], iv4, code_base, sign_base, q_first, rc, in[0]);
    } else {
#pragma unroll
        for (int k = 0; k + 1 < QPL; k += 2) {
            const uint32_t q = q_first + k * lanes;
            uint32_t rc_a[4], rc_b[4];
            tile_quad_words(a, q_global, q, q + lanes, rc_a, rc_b);
            encode_store_quad<FMT>(a, lp, v[k], iv4, code_base, sign_base, q, rc_a, in[k]);
            __builtin_amdgcn_sched_barrier(0);  // one quad at a time keeps the register count low
            encode_store_quad<FMT>(a, lp, v[k + 1], iv4, code_base, sign_base, q + lanes, rc_b, in[k + 1]);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    // the ragged last bucket (fewer than `bucket` <= 2048 elements) is the last workgroup's second job
    if (blockIdx.x == gridDim.x - 1 && full_buckets * a.segs.bucket < a.segs.d)
        bucket_encode_by_workgroup<kBlock, FMT, false>(a, full_buckets, scratch);
}

// Adds to acc the lane's elements that fall into the chunk-local piece [lb, le); the lane
// holds quads t, t + kBlock, ... of the chunk.  Rows of quads the piece does not reach are
// skipped (a workgroup-uniform test).
template <int P, int N>
__device__ __forceinline__ void piece_accumulate(NormAcc& acc, const u32x4 (&v)[N], uint32_t lb, uint32_t le) {
    const uint32_t span = le - lb;
#pragma unroll
    for (int k = 0; k < N; ++k) {
        const uint32_t row0 = (uint32_t)k * kBlock * 4;
        if (row0 < le && row0 + kBlock * 4 > lb) {
            const uint32_t l0 = row0 + threadIdx.x * 4;
            u32x4 m;  // zeros outside the piece add nothing
            m.x = (l0 + 0 - lb < span) ? v[k].x : 0u;
            m.y = (l0 + 1 - lb < span) ? v[k].y : 0u;
            m.z = (l0 + 2 - lb < span) ? v[k].z : 0u;
            m.w = (l0 + 3 - lb < span) ? v[k].w : 0u;
            norm_add4_p<P>(acc, m);
        }
    }
}

// ------------------------------------------------------------------------ two-pass path
// Pass 1: partial norm of every (segment, chunk) intersection, chunks of kNormChunk
// elements.  The piece of the segment that continues into a chunk from the left goes to
// first_partial[chunk]; a segment that starts inside the chunk puts its first piece into
// head_partial[segment].  FAST: lane t holds quads t, t+256, ... of the chunk, all loaded
// before the segment search; a chunk that straddles segments is reduced piece by piece from
// the same registers.
// The pieces of the segments s0, s0 + 1, ... that touch the chunk [cb, ce), each read from x
// and reduced by the whole workgroup (any alignment; also a vector chunk with too many
// boundaries to stage, which reads x again).
__device__ __forceinline__ void partial_by_segments(const DitherEncodeArgs& a, uint64_t cb, uint64_t ce, uint32_t s0,
                                                    NormAcc* scratch) {
    const Segs& sg = a.segs;
    const uint32_t nseg = seg_count(sg);
    for (uint32_t s = s0; s < nseg; ++s) {  // block-uniform loop
        const uint64_t sb = seg_begin(sg, s), se = seg_end(sg, s);
        if (sb >= ce) break;
        const uint64_t b = sb > cb ? sb : cb, e = se < ce ? se : ce;
        if (e <= b) continue;  // empty segment
        NormAcc acc = norm_zero();
        for (uint64_t i = b + threadIdx.x; i < e; i += kBlock) norm_add(acc, a.x[i], a.pnorm);
        acc = norm_block_reduce<kBlock>(acc, a.pnorm, scratch);
        if (threadIdx.x == 0) {
            const double r = a.pnorm == kNormInf ? (double)acc.mx : acc.sum;
            if (sb >= cb) a.head_partial[s] = r; else a.first_partial[blockIdx.x] = r;
        }
    }
}

template <bool FAST>
__global__ __launch_bounds__(kBlock) void dither_partial_kernel(DitherEncodeArgs a) {
    __shared__ NormAcc scratch[kBlock / 64];
    __shared__ uint32_t bnd[kBlock];
    __shared__ double piece_part[kBlock * (kBlock / 64)];  // [piece][wavefront]
    constexpr int kQuads = kNormChunk / 4 / kBlock;  // quads per lane
    const Segs& sg = a.segs;
    const uint64_t cb = (uint64_t)blockIdx.x * kNormChunk;
    const uint64_t ce = cb + kNormChunk < sg.d ? cb + kNormChunk : sg.d;
    if (!FAST || (ce - cb) != kNormChunk) {  // the ragged last chunk, or no alignment
        partial_by_segments(a, cb, ce, seg_find(sg, cb), scratch);
        return;
    }
    // A whole chunk: unconditional vector loads, all issued before the segment search.
    u32x4 v[kQuads];
    const u32x4* __restrict__ xv = reinterpret_cast<const u32x4*>(a.x + cb) + threadIdx.x;
#pragma unroll
    for (int k = 0; k < kQuads; ++k) v[k] = load_stream(xv + k * kBlock);
    const SegHit hit = seg_find_hit(sg, cb, nullptr);
    const uint32_t s0 = hit.s;
    // keep the loaded values opaque up to here, so that nothing is computed from them (and held
    // in registers) ahead of the search
#pragma unroll
    for (int k = 0; k < kQuads; ++k) asm volatile("" : "+v"(v[k]));
    if (hit.end >= ce) {  // the whole chunk lies in one segment
        NormAcc acc = norm_zero();
        norm_add_quads(acc, v, a.pnorm);
        acc = norm_block_reduce<kBlock>(acc, a.pnorm, scratch);
        if (threadIdx.x == 0) {
            const double r = a.pnorm == kNormInf ? (double)acc.mx : acc.sum;
            if (hit.begin >= cb) a.head_partial[s0] = r; else a.first_partial[blockIdx.x] = r;
        }
        return;
    }
    // pieces from the staged boundaries: no global loads and one barrier for all pieces
    const uint32_t nb = stage_boundaries(sg, cb, ce, s0, bnd);
    if (nb >= (uint32_t)kBlock) {
        partial_by_segments(a, cb, ce, s0, scratch);
        return;
    }
    constexpr int kWaves = kBlock / 64;
    for (uint32_t p = 0; p <= nb; ++p) {
        const uint32_t lb = p ? bnd[p - 1] : 0u, le = p < nb ? bnd[p] : (uint32_t)kNormChunk;
        if (le == lb) continue;  // empty segment
#pragma unroll
        for (int k = 0; k < kQuads; ++k) asm volatile("" : "+v"(v[k]));  // nothing hoisted out of the loop
        NormAcc acc = norm_zero();
        if (a.pnorm == kNormInf) piece_accumulate<kNormInf>(acc, v, lb, le);
        else if (a.pnorm == kNormL1) piece_accumulate<kNormL1>(acc, v, lb, le);
        else piece_accumulate<kNormL2>(acc, v, lb, le);
        acc = norm_wave_reduce(acc, a.pnorm);
        if ((threadIdx.x & 63) == 0)
            piece_part[p * kWaves + (threadIdx.x >> 6)] = a.pnorm == kNormInf ? (double)acc.mx : acc.sum;
    }
    __syncthreads();
    const uint32_t p = threadIdx.x;  // nb < kBlock: one piece per lane
    if (p <= nb) {
        const uint32_t lb = p ? bnd[p - 1] : 0u, le = p < nb ? bnd[p] : (uint32_t)kNormChunk;
        if (le != lb) {
            double r = piece_part[p * kWaves];
#pragma unroll
            for (int w = 1; w < kWaves; ++w) {
                const double o = piece_part[p * kWaves + w];
                r = a.pnorm == kNormInf ? fmax(r, o) : r + o;
            }
            if (p == 0 && hit.begin < cb) a.first_partial[blockIdx.x] = r;
            else a.head_partial[s0 + p] = r;
        }
    }
}

// Pass 2: one workgroup per segment adds the segment's partials in a fixed order.
__global__ __launch_bounds__(kBlock) void dither_finalize_kernel(DitherEncodeArgs a) {
    __shared__ NormAcc scratch[kBlock / 64];
    const Segs& sg = a.segs;
    const uint32_t s = blockIdx.x;
    const uint64_t b = seg_begin(sg, s), e = seg_end(sg, s);
    NormAcc acc = norm_zero();
    if (e > b) {
        const uint64_t c_head = b / kNormChunk, c_last = (e - 1) / kNormChunk;
        // the piece in the chunk where the segment starts is in head_partial
        if (threadIdx.x == 0) {
            const double r = a.head_partial[s];
            if (a.pnorm == kNormInf) acc.mx = (float)r; else acc.sum = r;
        }
        for (uint64_t c = c_head + 1 + threadIdx.x; c <= c_last; c += kBlock) {
            const double r = a.first_partial[c];
            NormAcc o = norm_zero();
            if (a.pnorm == kNormInf) o.mx = (float)r; else o.sum = r;
            acc = norm_merge(acc, o, a.pnorm);
        }
    }
    acc = norm_block_reduce<kBlock>(acc, a.pnorm, scratch);
    const float norm = norm_value(acc, a.pnorm);  // the same bits in every lane
    const float inv = inv_of_norm(norm);
    if (threadIdx.x == 0) {
        a.norms_out[s] = norm;
        a.inv_norm[s] = inv;
    }
    if (a.chunk_segment && e > b) {  // the encode chunks whose first element lies in this segment
        const uint64_t c0 = (b + kChunk - 1) / kChunk, c1 = (e - 1) / kChunk;
        for (uint64_t c = c0 + threadIdx.x; c <= c1; c += kBlock) a.chunk_segment[c] = ChunkSegment{e, s, inv};
    }
}

// Pass 3: encode with the finished norms.  A chunk that lies in one segment takes the
// vector path (FAST: alignment as for the one-pass kernel); a chunk that straddles segment
// boundaries, and the ragged end of the vector, go lane-by-lane in groups of 8.
template <int FMT, bool FAST>
__global__ __launch_bounds__(kBlock) void dither_segment_encode_kernel(DitherEncodeArgs a) {
    __shared__ uint32_t bnd[kBlock];
    const Segs& sg = a.segs;
    const uint64_t cb = (uint64_t)blockIdx.x * kChunk;
    const uint64_t ce = cb + kChunk < sg.d ? cb + kChunk : sg.d;
    const uint32_t len = (uint32_t)(ce - cb);
    const uint32_t vec_quads = (len >> 5) << 3;
    u32x4 v[2];
    if (FAST) {  // the loads do not depend on the segment: issue them before the search
        const u32x4* __restrict__ xv = reinterpret_cast<const u32x4*>(a.x + cb);
#pragma unroll
        for (int k = 0; k < 2; ++k) {
            const uint32_t q = threadIdx.x + k * kBlock;
            v[k] = u32x4{0u, 0u, 0u, 0u};
            if (q < vec_quads) v[k] = load_stream(xv + q);
        }
    }
    SegHit hit;
    if (a.chunk_segment) {  // segment offsets: the norm pass left one record per chunk
        const ChunkSegment rec = a.chunk_segment[blockIdx.x];
        // (offsets that do not cover [0, d) leave records unwritten: keep the index in range)
        hit = SegHit{min(rec.segment, sg.num_segments - 1), rec.inv_norm, 0ull, rec.end};
    } else {
        hit = seg_find_hit(sg, cb, a.inv_norm);  // arithmetic on the bucket size
    }
    const uint32_t s0 = hit.s;
    const bool one_segment = hit.end >= ce;  // block-uniform
    uint32_t scalar_from = 0;                         // chunk-local element where the scalar part starts
    uint32_t nb = one_segment ? 0u : (uint32_t)kBlock;  // staged boundaries (kBlock: not staged)
    if (FAST) {
        if (!one_segment) nb = stage_boundaries(sg, cb, ce, s0, bnd);
        if (nb < (uint32_t)kBlock) {
            const LevelParams lp = level_params(a.s, a.standard);
            const uint64_t q_global = (a.index_offset + cb) >> 2;
            uint32_t* __restrict__ code_base =
                reinterpret_cast<uint32_t*>(a.code_out + (FMT == kFmtByte ? cb : cb >> 1));
            uint32_t* __restrict__ sign_base = reinterpret_cast<uint32_t*>(a.sign_out + (cb >> 3));
            uint32_t rc[2][4];
            tile_quad_words(a, q_global, threadIdx.x, threadIdx.x + kBlock, rc[0], rc[1]);
            if (one_segment) {
                const float iv = hit.aux;
                const float iv4[4] = {iv, iv, iv, iv};
#pragma unroll
                for (int k = 0; k < 2; ++k) {
                    const uint32_t q = threadIdx.x + k * kBlock;
                    if (k * kBlock < vec_quads)
                        encode_store_quad<FMT>(a, lp, v[k], iv4, code_base, sign_base, q, rc[k], q < vec_quads);
                }
            } else {  // each element takes the reciprocal norm of its own segment
#pragma unroll
                for (int k = 0; k < 2; ++k) {
                    const uint32_t q = threadIdx.x + k * kBlock;
                    if (k * kBlock < vec_quads) {
                        SegCursor cur = cursor_at(bnd, nb, q * 4);
                        float iv = a.inv_norm[s0 + cur.idx];
                        float iv4[4];
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            if (cursor_advance(cur, bnd, nb, q * 4 + j)) iv = a.inv_norm[s0 + cur.idx];
                            iv4[j] = iv;
                        }
                        encode_store_quad<FMT>(a, lp, v[k], iv4, code_base, sign_base, q, rc[k], q < vec_quads);
                    }
                }
            }
            scalar_from = vec_quads * 4;
            if (scalar_from >= len) return;
        }
    }
    const uint64_t i0 = cb + scalar_from + (uint64_t)threadIdx.x * 8;
    if (i0 >= ce) return;
    const uint32_t count = ce - i0 < 8 ? (uint32_t)(ce - i0) : 8u;
    uint32_t u[8];
    load8<false>(a.x, i0, count, u);
    float inv[8];
    if (one_segment) {
        const float iv = hit.aux;
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
    encode_group<FMT, false>(a, u, inv, i0, count);
}

// ------------------------------------------------------------------------ decode and sum
// Norm of (worker row, segment): a binary32 value, or (norm8) the exponent byte of a norm that
// natural compression rounded to a power of two, 2^(e-127) with e = 0 standing for 0.  Times a
// level 2^(c-s) that is the exponent sum e + c - s; the decoders keep the one multiply, which
// costs the same as an integer add and also covers results below the normal range.
__device__ __forceinline__ float load_norm(const DitherAggregateArgs& a, size_t index) {
    if (a.norm8) return bits_f32((uint32_t)reinterpret_cast<const uint8_t*>(a.norms)[index] << 23);
    return a.norms[index];
}

// Value bits of (norm, code c, sign): sign | fl(norm * 2^(c-s)), a signed zero for c = 0.
__device__ __forceinline__ float dither_value(float norm, uint32_t s, uint32_t c, uint32_t sign_bit,
                                              uint32_t standard) {
    // natural: 2^(c-s), normal for 1 <= c <= s <= 127; standard: fl(c / s)
    const float level = standard ? (float)c / (float)s : bits_f32((127u + c - s) << 23);
    const float mag = c ? norm * level : 0.0f;
    return bits_f32(f32_bits(mag) | (sign_bit << 31));
}

// Code words (8 nibbles) and sign bytes of the lane's group for NW workers starting at w.
template <int FMT, int NW>
__device__ __forceinline__ void dither_load_codes(const DitherAggregateArgs& a, uint64_t grp, size_t w,
                                                  uint32_t cw[NW], uint32_t sb[NW]) {
#pragma unroll
    for (int k = 0; k < NW; ++k) {
        cw[k] = load_stream(reinterpret_cast<const uint32_t*>(a.code + (w + k) * a.code_stride) + grp);
        sb[k] = (FMT == kFmtNibble) ? (uint32_t)load_stream(a.sign + (w + k) * a.sign_stride + grp) : 0u;
    }
}
// Each of the lane's 8 elements looks its value up in the workers' 16-entry tables and adds it.
// `rows` is the lane's table of table-worker 0 and row_stride the distance to the next worker's.
template <int FMT, int NW>
__device__ __forceinline__ void dither_add_codes(const float* rows, uint32_t row_stride, uint32_t w_table,
                                                 const uint32_t cw[NW], const uint32_t sb[NW], float acc[8]) {
#pragma unroll
    for (int k = 0; k < NW; ++k) {
        const float* row = rows + (w_table + k) * row_stride;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            float v = row[(cw[k] >> (4 * j)) & 15u];
            if (FMT == kFmtNibble) v = bits_f32(f32_bits(v) | ((sb[k] << (31 - j)) & 0x80000000u));
            acc[j] += v;
        }
    }
}
template <int FMT, int NW>
__device__ __forceinline__ void dither_sum_chunk(const DitherAggregateArgs& a, const float* rows, uint32_t row_stride,
                                                 uint64_t grp, uint32_t w_table, size_t w_global, float acc[8]) {
    uint32_t cw[NW], sb[NW];
    dither_load_codes<FMT, NW>(a, grp, w_global, cw, sb);
    dither_add_codes<FMT, NW>(rows, row_stride, w_table, cw, sb, acc);
}

// NW workers of the lane's group decoded arithmetically with the norms of segment seg.
template <int FMT, int NW>
__device__ __forceinline__ void dither_sum_chunk_arith(const DitherAggregateArgs& a, uint64_t grp, size_t w0,
                                                       uint32_t seg, float acc[8]) {
    uint32_t cw[NW], sb[NW];
    float norm[NW];
    dither_load_codes<FMT, NW>(a, grp, w0, cw, sb);
#pragma unroll
    for (int k = 0; k < NW; ++k) norm[k] = load_norm(a, (w0 + k) * a.norm_stride + seg);
#pragma unroll
    for (int k = 0; k < NW; ++k) {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const uint32_t nib = (cw[k] >> (4 * j)) & 15u;
            const uint32_t c = (FMT == kFmtFused) ? (nib & 7u) : nib;
            const uint32_t sgn = (FMT == kFmtFused) ? (nib >> 3) : ((sb[k] >> j) & 1u);
            acc[j] += dither_value(norm[k], a.s, c, sgn, a.standard);
        }
    }
}

// One element of the sum by plain arithmetic (any layout and alignment).
template <int FMT>
__device__ __forceinline__ float dither_sum_one(const DitherAggregateArgs& a, uint64_t i, uint32_t seg) {
    float acc = -0.0f;  // identity of binary32 addition: the sum starts from worker 0's value
    for (uint32_t w = 0; w < a.n; ++w) {
        const uint8_t* cp = a.code + (size_t)w * a.code_stride;
        uint32_t c, sgn;
        if (FMT == kFmtByte) {
            c = cp[i];
            sgn = (a.sign[(size_t)w * a.sign_stride + (i >> 3)] >> (i & 7)) & 1u;
        } else {
            const uint32_t nib = (cp[i >> 1] >> (4 * (i & 1))) & 15u;
            if (FMT == kFmtFused) { c = nib & 7u; sgn = nib >> 3; }
            else { c = nib; sgn = (a.sign[(size_t)w * a.sign_stride + (i >> 3)] >> (i & 7)) & 1u; }
        }
        acc += dither_value(load_norm(a, (size_t)w * a.norm_stride + seg), a.s, c, sgn, a.standard);
    }
    return acc;
}

// Decode (n = 1) and fused decode-and-sum.  One lane owns 8 consecutive output elements;
// results leave through the LDS transpose (VEC: out 16-byte aligned, code planes 4-byte
// aligned with 4-byte-multiple strides).  Nibble formats use tables: for up to 16 workers at a
// time the workgroup tabulates in LDS the 16 values a nibble can decode to (fused format: sign
// included), so an element costs one bit-field extract, one LDS read and one add per worker.
// TABLE = 256 floats: one table per worker, for chunks that lie inside one segment.
// TABLE = 4096 floats: power-of-two buckets of 64..1024 elements (a.log2_bucket), one table per
// (worker, bucket of the chunk); a lane's 8 elements share a bucket.  Everything else (byte
// codes, chunks that straddle other segment boundaries) is decoded arithmetically:
// norm * 2^(c-s).
template <int FMT, bool VEC, int TABLE>
__global__ __launch_bounds__(kBlock) void dither_aggregate_kernel(DitherAggregateArgs a) {
    __shared__ float table[TABLE];
    __shared__ u32x4 tile[2 * kBlock];
    __shared__ uint32_t bnd[kBlock];
    const Segs& sg = a.segs;
    const uint64_t cb = (uint64_t)blockIdx.x * kChunk;
    const uint64_t ce = cb + kChunk < sg.d ? cb + kChunk : sg.d;
    const uint64_t grp = (cb >> 3) + threadIdx.x;
    const uint64_t i0 = grp * 8;
    const uint32_t count = i0 >= ce ? 0u : (ce - i0 < 8 ? (uint32_t)(ce - i0) : 8u);
    // The first (up to 8) workers' codes do not depend on the segment: load them before the
    // table is built, so the two global round trips overlap.
    constexpr bool kTables = VEC && FMT != kFmtByte;
    constexpr bool kMulti = TABLE > 256;
    const uint32_t n_first = a.n >= 8 ? 8u : (a.n == 1 ? 1u : 0u);  // 2..7 workers: no preload
    uint32_t cw0[8] = {0u, 0u, 0u, 0u, 0u, 0u, 0u, 0u}, sb0[8] = {0u, 0u, 0u, 0u, 0u, 0u, 0u, 0u};
    if (kTables && count == 8) {
        if (n_first == 8) dither_load_codes<FMT, 8>(a, grp, 0, cw0, sb0);
        else if (n_first == 1) dither_load_codes<FMT, 1>(a, grp, 0, cw0, sb0);
    }
    SegHit hit{0u, 0.0f, 0ull, 0ull};
    if (!kMulti) hit = seg_find_hit(sg, cb, nullptr);  // (scalar loads: the preload stays in flight)
    uint32_t s0, log2_nbk = 0, lane_bucket = 0, nseg = 0;
    uint64_t s0_begin = 0;
    bool one_segment;
    if (kMulti) {  // the chunk holds 2^log2_nbk whole buckets, the first of index s0
        log2_nbk = 11u - a.log2_bucket;  // kChunk = 2^11
        s0 = blockIdx.x << log2_nbk;
        lane_bucket = (threadIdx.x * 8u) >> a.log2_bucket;
        nseg = seg_count(sg);
        one_segment = true;  // (for the table path: every lane's elements have a table)
    } else {
        s0 = hit.s;
        s0_begin = hit.begin;
        one_segment = hit.end >= ce;
    }
    const uint32_t nbk = 1u << log2_nbk;
    const uint32_t rounds_of = (kMulti && nbk > 16u) ? (uint32_t)(TABLE / 16) >> log2_nbk : 16u;  // workers per table round
    const float* rows = table + lane_bucket * 16u;
    const uint32_t row_stride = nbk * 16u;
    float acc[8] = {-0.0f, -0.0f, -0.0f, -0.0f, -0.0f, -0.0f, -0.0f, -0.0f};

    if (kTables && one_segment) {
        for (uint32_t w0 = 0; w0 < a.n; w0 += rounds_of) {
            const uint32_t nw = a.n - w0 < rounds_of ? a.n - w0 : rounds_of;
            // tabulate: entry ((worker, bucket), nibble)
            for (uint32_t e = threadIdx.x; e < (nw << (4u + log2_nbk)); e += kBlock) {
                const uint32_t w = e >> (4u + log2_nbk), seg = s0 + ((e >> 4) & (nbk - 1u)), nib = e & 15u;
                const float norm = (!kMulti || seg < nseg) ? load_norm(a, (size_t)(w0 + w) * a.norm_stride + seg) : 0.0f;
                table[e] = (FMT == kFmtFused) ? dither_value(norm, a.s, nib & 7u, nib >> 3, a.standard)
                                              : dither_value(norm, a.s, nib, 0u, a.standard);
            }
            __syncthreads();
            if (count == 8) {
                uint32_t w = 0;
                if (w0 == 0) {  // the preloaded workers
                    // keep the code words opaque up to here: otherwise all 64 table addresses are
                    // computed ahead of the barrier and the kernel loses half its wavefronts
#pragma unroll
                    for (int k = 0; k < 8; ++k) asm volatile("" : "+v"(cw0[k]), "+v"(sb0[k]));
                    if (n_first == 8) dither_add_codes<FMT, 8>(rows, row_stride, 0, cw0, sb0, acc);
                    else if (n_first == 1) dither_add_codes<FMT, 1>(rows, row_stride, 0, cw0, sb0, acc);
                    w = n_first;
                }
                for (; w + 8 <= nw; w += 8) dither_sum_chunk<FMT, 8>(a, rows, row_stride, grp, w, w0 + w, acc);
                for (; w + 2 <= nw; w += 2) dither_sum_chunk<FMT, 2>(a, rows, row_stride, grp, w, w0 + w, acc);
                if (w < nw) dither_sum_chunk<FMT, 1>(a, rows, row_stride, grp, w, w0 + w, acc);
            }
            __syncthreads();
        }
        if (count > 0 && count < 8) {  // the ragged last group of the vector
#pragma unroll
            for (int j = 0; j < 8; ++j)
                if ((uint32_t)j < count) acc[j] = dither_sum_one<FMT>(a, i0 + j, s0 + lane_bucket);
        }
    } else if (kTables && !sg.offsets && (sg.bucket & 7u) == 0 && sg.bucket <= (1u << 20)) {
        // buckets that are a multiple of 8 (not a power of two, or too small for tables): the lane's 8
        // elements share one bucket, whose index follows from the position; codes still come as words
        const uint32_t seg = s0 + ((uint32_t)(cb - s0_begin) + threadIdx.x * 8u) / sg.bucket;
        if (count == 8) {
            uint32_t w = 0;
            for (; w + 2 <= a.n; w += 2) dither_sum_chunk_arith<FMT, 2>(a, grp, w, seg, acc);  // (4 at a time would cost the table path its occupancy)
            for (; w < a.n; ++w) dither_sum_chunk_arith<FMT, 1>(a, grp, w, seg, acc);
        } else if (count) {
#pragma unroll
            for (int j = 0; j < 8; ++j) if ((uint32_t)j < count) acc[j] = dither_sum_one<FMT>(a, i0 + j, seg);
        }
    } else {
        const uint32_t nb = one_segment ? 0u : stage_boundaries(sg, cb, ce, s0, bnd);  // block-uniform
        if (count && nb < (uint32_t)kBlock) {
            const uint32_t l0 = threadIdx.x * 8;
            SegCursor cur = cursor_at(bnd, nb, l0);
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                if ((uint32_t)j < count) {
                    cursor_advance(cur, bnd, nb, l0 + j);
                    acc[j] = dither_sum_one<FMT>(a, i0 + j, s0 + cur.idx);
                }
            }
        } else if (count) {  // too many boundaries to stage: search the offsets
            const uint32_t last = seg_count(sg) - 1;
            uint32_t s = seg_find(sg, i0);
            uint64_t se = seg_end(sg, s);
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                if ((uint32_t)j < count) {
                    while (i0 + j >= se && s < last) { ++s; se = seg_end(sg, s); }
                    acc[j] = dither_sum_one<FMT>(a, i0 + j, s);
                }
            }
        }
    }
    if (VEC) {
        uint32_t bits[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) bits[j] = f32_bits(acc[j]);
        const uint32_t groups = (uint32_t)((ce - cb) >> 3);  // whole groups of 8 in this chunk
        store_tile_transposed(tile, bits, count == 8, groups, a.out + cb);
        if (count > 0 && count < 8) {
#pragma unroll
            for (int j = 0; j < 8; ++j) if ((uint32_t)j < count) a.out[i0 + j] = acc[j];
        }
    } else {
#pragma unroll
        for (int j = 0; j < 8; ++j) if ((uint32_t)j < count) a.out[i0 + j] = acc[j];
    }
}

// Plain decoder (n = 1) for the nibble formats, vector path: the lean special case of the
// aggregate kernel.  The lane's 8 codes are loaded first; the 16 values a nibble can stand for
// in this chunk's segment are kept one per lane and looked up with lane permutes; chunks that
// straddle segments (and the ragged end) decode arithmetically.  Results leave through the LDS
// transpose.
template <int FMT>
__global__ __launch_bounds__(kBlock) void dither_decode_kernel(DitherAggregateArgs a) {
    __shared__ u32x4 tile[2 * kBlock];
    __shared__ uint32_t bnd[kBlock];
    const Segs& sg = a.segs;
    const uint64_t cb = (uint64_t)blockIdx.x * kChunk;
    const uint64_t ce = cb + kChunk < sg.d ? cb + kChunk : sg.d;
    const uint32_t grp_local = threadIdx.x;
    const uint32_t l0 = grp_local * 8;
    const uint32_t len = (uint32_t)(ce - cb);
    const uint32_t count = l0 >= len ? 0u : (len - l0 < 8 ? len - l0 : 8u);
    const uint32_t* __restrict__ code_base = reinterpret_cast<const uint32_t*>(a.code + (cb >> 1));
    const uint8_t* __restrict__ sign_base = a.sign + (cb >> 3);
    uint32_t cw = 0, sb = 0;
    if (count == 8) {
        cw = load_stream(code_base + grp_local);
        if (FMT == kFmtNibble) sb = load_stream(sign_base + grp_local);
    }
    const SegHit hit = seg_find_hit(sg, cb, a.norm8 ? nullptr : a.norms);  // (scalar loads: the code loads stay in flight)
    const uint32_t s0 = hit.s;
    const bool one_segment = hit.end >= ce;
    uint32_t bits[8];
    if (one_segment) {
        // The 16 values a nibble can stand for live one per lane (lane l holds the value of nibble
        // l mod 16) and are looked up with a lane permute: no table in memory and no barrier.
        const uint32_t nib_of_lane = threadIdx.x & 15u;
        const float norm = a.norm8 ? load_norm(a, s0) : hit.aux;
        const uint32_t value_of_lane =
            f32_bits((FMT == kFmtFused) ? dither_value(norm, a.s, nib_of_lane & 7u, nib_of_lane >> 3, a.standard)
                                        : dither_value(norm, a.s, nib_of_lane, 0u, a.standard));
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            uint32_t v = (uint32_t)__builtin_amdgcn_ds_bpermute((int)(((cw >> (4 * j)) & 15u) << 2), (int)value_of_lane);
            if (FMT == kFmtNibble) v |= (sb << (31 - j)) & 0x80000000u;
            bits[j] = v;
        }
    } else if (!sg.offsets && (sg.bucket & 7u) == 0 && sg.bucket <= (1u << 20)) {
        // buckets that are a multiple of 8: the lane's 8 elements share one bucket, whose index
        // follows from the position alone (no search, so the norm load is not behind a barrier)
        const uint32_t seg = s0 + ((uint32_t)(cb - hit.begin) + l0) / sg.bucket;
        const float norm = load_norm(a, seg < seg_count(sg) ? seg : s0);  // (lanes past the end: any valid index)
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const uint32_t nib = (cw >> (4 * j)) & 15u;
            const uint32_t c = (FMT == kFmtFused) ? (nib & 7u) : nib;
            const uint32_t sgn = (FMT == kFmtFused) ? (nib >> 3) : ((sb >> j) & 1u);
            bits[j] = f32_bits(dither_value(norm, a.s, c, sgn, a.standard));
        }
    } else {
        const uint32_t nb = stage_boundaries(sg, cb, ce, s0, bnd);  // block-uniform branch
        SegCursor cur;
        if (nb < (uint32_t)kBlock) cur = cursor_at(bnd, nb, l0);
        else cur = SegCursor{count ? seg_find(sg, cb + l0) - s0 : 0u, 0u};
        float norm = load_norm(a, s0 + cur.idx);
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            if (nb < (uint32_t)kBlock) {
                if (cursor_advance(cur, bnd, nb, l0 + j)) norm = load_norm(a, s0 + cur.idx);
            } else if (count) {
                const uint32_t last = seg_count(sg) - 1;
                while (cb + l0 + j >= seg_end(sg, s0 + cur.idx) && s0 + cur.idx < last) {
                    ++cur.idx;
                    norm = load_norm(a, s0 + cur.idx);
                }
            }
            const uint32_t nib = (cw >> (4 * j)) & 15u;
            const uint32_t c = (FMT == kFmtFused) ? (nib & 7u) : nib;
            const uint32_t sgn = (FMT == kFmtFused) ? (nib >> 3) : ((sb >> j) & 1u);
            bits[j] = f32_bits(dither_value(norm, a.s, c, sgn, a.standard));
        }
    }
    store_tile_transposed(tile, bits, count == 8, len >> 3, a.out + cb);
    if (count > 0 && count < 8) {  // the ragged last group of the vector
        const uint32_t last = seg_count(sg) - 1;
        uint32_t s = seg_find(sg, cb + l0);
        for (uint32_t j = 0; j < count; ++j) {
            const uint64_t i = cb + l0 + j;
            while (i >= seg_end(sg, s) && s < last) ++s;
            a.out[i] = dither_sum_one<FMT>(a, i, s);
        }
    }
}

// ------------------------------------------------------------------------ compressed norm
// C_nat of every norm (Sec. 3: general dithering with C = C_nat sends the norm as a power of
// two): the exponent byte and the power of two it stands for.  Norms are non-negative, so
// no sign is kept; norm s draws word s of its own stream (domain 4).
__global__ __launch_bounds__(kBlock) void norm_compress_kernel(const float* __restrict__ norms, uint64_t count,
                                                               uint32_t k0, uint32_t k1, uint32_t worker,
                                                               uint8_t* __restrict__ exp_out,
                                                               float* __restrict__ q_out) {
    const uint64_t s = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
    if (s >= count) return;
    const uint32_t u = f32_bits(norms[s]) & 0x7FFFFFFFu;
    const uint32_t r = random_word(s, worker, kDomainNorm, k0, k1);
    const uint32_t e = add_sat(u << 1, (~r) >> 8) >> 24;  // exponent + [r < m 2^9], 255 absorbing
    exp_out[s] = (uint8_t)e;
    q_out[s] = bits_f32(e << 23);
}

hipError_t launch_norm_compress(const float* norms, uint64_t count, uint32_t k0, uint32_t k1, uint32_t worker,
                                uint8_t* exp_out, float* q_out, hipStream_t stream) {
    norm_compress_kernel<<<(unsigned)((count + kBlock - 1) / kBlock), kBlock, 0, stream>>>(norms, count, k0, k1, worker,
                                                                                          exp_out, q_out);
    return hipGetLastError();
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

template <int QPL>
static hipError_t launch_bucket_vec(const DitherEncodeArgs& a, unsigned grid, hipStream_t st) {
    switch (a.fmt) {
        case kFmtFused: dither_bucket_encode_vec_kernel<QPL, kFmtFused><<<grid, kBlock, 0, st>>>(a); break;
        case kFmtNibble: dither_bucket_encode_vec_kernel<QPL, kFmtNibble><<<grid, kBlock, 0, st>>>(a); break;
        default: dither_bucket_encode_vec_kernel<QPL, kFmtByte><<<grid, kBlock, 0, st>>>(a); break;
    }
    return hipGetLastError();
}

template <int QPL>
static void launch_multi(const DitherEncodeArgs& a, uint32_t log2_l, uint64_t full, unsigned tiles, hipStream_t st) {
    switch (a.fmt) {
        case kFmtFused: dither_multi_bucket_encode_kernel<QPL, kFmtFused><<<tiles, kBlock, 0, st>>>(a, log2_l, full); break;
        case kFmtNibble: dither_multi_bucket_encode_kernel<QPL, kFmtNibble><<<tiles, kBlock, 0, st>>>(a, log2_l, full); break;
        default: dither_multi_bucket_encode_kernel<QPL, kFmtByte><<<tiles, kBlock, 0, st>>>(a, log2_l, full); break;
    }
}

hipError_t launch_dither_bucket_encode(const DitherEncodeArgs& a, bool fast, hipStream_t stream) {
    const unsigned grid = (unsigned)((a.segs.d + a.segs.bucket - 1) / a.segs.bucket);
    const uint32_t bucket = a.segs.bucket;
    if (fast && bucket >= 32 && bucket <= 2048 && (bucket & 31) == 0) {
        // QPL quads per lane, L lanes per bucket with QPL * L = the power of two at or above bucket / 4
        const uint32_t quads = bucket / 4;
        uint32_t pow2 = 8;
        while (pow2 < quads) pow2 <<= 1;
        // measured best: runs of at least 256 contiguous bytes per load where the bucket allows it
        const int qpl = pow2 <= 8 ? 1 : pow2 <= 32 ? 2 : pow2 <= 128 ? 4 : 8;
        uint32_t log2_l = 0;
        while (((uint32_t)qpl << log2_l) < pow2) ++log2_l;
        const uint64_t full = a.segs.d / bucket;
        const uint64_t per_tile = (uint64_t)kBlock >> log2_l;  // buckets per workgroup
        uint64_t tiles = (full + per_tile - 1) / per_tile;
        if (tiles == 0) tiles = 1;  // a vector shorter than one bucket: only the ragged bucket
        switch (qpl) {
            case 1: launch_multi<1>(a, log2_l, full, (unsigned)tiles, stream); break;
            case 2: launch_multi<2>(a, log2_l, full, (unsigned)tiles, stream); break;
            case 4: launch_multi<4>(a, log2_l, full, (unsigned)tiles, stream); break;
            default: launch_multi<8>(a, log2_l, full, (unsigned)tiles, stream); break;
        }
        return hipGetLastError();
    }
    if (fast && (a.segs.bucket & 31) == 0) {  // vector path: 256 lanes, QPL quads per lane
        const uint32_t quads = a.segs.bucket / 4;
        if (quads <= 256) return launch_bucket_vec<1>(a, grid, stream);
        if (quads <= 512) return launch_bucket_vec<2>(a, grid, stream);
        if (quads <= 1024) return launch_bucket_vec<4>(a, grid, stream);
        return launch_bucket_vec<8>(a, grid, stream);
    }
    const uint32_t lanes = (a.segs.bucket + 7) / 8;
    if (lanes <= 256) return fast ? launch_bucket<256, true>(a, grid, stream) : launch_bucket<256, false>(a, grid, stream);
    if (lanes <= 512) return fast ? launch_bucket<512, true>(a, grid, stream) : launch_bucket<512, false>(a, grid, stream);
    return fast ? launch_bucket<1024, true>(a, grid, stream) : launch_bucket<1024, false>(a, grid, stream);
}

template <bool FAST>
static hipError_t launch_segment(const DitherEncodeArgs& a, hipStream_t st) {
    const unsigned chunks = (unsigned)((a.segs.d + kChunk - 1) / kChunk);
    const unsigned norm_chunks = (unsigned)((a.segs.d + kNormChunk - 1) / kNormChunk);
    const unsigned nseg = (unsigned)(a.segs.offsets ? a.segs.num_segments
                                     : a.segs.bucket ? (a.segs.d + a.segs.bucket - 1) / a.segs.bucket : 1);
    dither_partial_kernel<FAST><<<norm_chunks, kBlock, 0, st>>>(a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    dither_finalize_kernel<<<nseg, kBlock, 0, st>>>(a);
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
    if (FAST && a.n == 1 && a.fmt != kFmtByte) {  // plain decoder
        if (a.fmt == kFmtFused) dither_decode_kernel<kFmtFused><<<chunks, kBlock, 0, st>>>(a);
        else dither_decode_kernel<kFmtNibble><<<chunks, kBlock, 0, st>>>(a);
        return hipGetLastError();
    }
    const uint32_t bucket = a.segs.bucket;
    if (FAST && a.fmt != kFmtByte && !a.segs.offsets && bucket >= 64 && bucket <= 1024 && (bucket & (bucket - 1)) == 0) {
        DitherAggregateArgs b = a;  // several whole buckets per chunk: tables per (worker, bucket)
        b.log2_bucket = 6;
        while ((1u << b.log2_bucket) < bucket) ++b.log2_bucket;
        if (a.fmt == kFmtFused) dither_aggregate_kernel<kFmtFused, FAST, 4096><<<chunks, kBlock, 0, st>>>(b);
        else dither_aggregate_kernel<kFmtNibble, FAST, 4096><<<chunks, kBlock, 0, st>>>(b);
        return hipGetLastError();
    }
    switch (a.fmt) {
        case kFmtFused: dither_aggregate_kernel<kFmtFused, FAST, 256><<<chunks, kBlock, 0, st>>>(a); break;
        case kFmtNibble: dither_aggregate_kernel<kFmtNibble, FAST, 256><<<chunks, kBlock, 0, st>>>(a); break;
        default: dither_aggregate_kernel<kFmtByte, FAST, 256><<<chunks, kBlock, 0, st>>>(a); break;
    }
    return hipGetLastError();
}

hipError_t launch_dither_aggregate(const DitherAggregateArgs& a, bool fast, hipStream_t stream) {
    return fast ? launch_agg<true>(a, stream) : launch_agg<false>(a, stream);
}

}  // namespace natcomp
