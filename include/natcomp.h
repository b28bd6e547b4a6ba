/*
 * natcomp.h -- C ABI of libnatcomp: natural compression C_nat and natural dithering
 * D_nat^{p,s} of fp32 gradient vectors on one MI355X (gfx950), after
 * "Natural Compression for Distributed Deep Learning" (arXiv 1905.10988).
 *
 * Conventions that hold for every entry point unless its comment says otherwise:
 *   - Pointers marked DEVICE point to HIP device memory owned by the caller; the
 *     library never allocates, frees or keeps them.  Pointers marked HOST are read
 *     during the call only.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls
 *     enqueue their kernels on it and return without waiting.
 *   - The return value reports argument errors (nothing was enqueued) and launch
 *     failures.  No exception crosses this boundary.  d = 0 is accepted and does nothing.
 *   - Inputs are never modified; an output may not overlap an input or another output.
 *   - Randomness: element i of a call uses the 32-bit word of global index
 *     g = index_offset + i of the stream (seed, worker, operator): output word (g mod 4)
 *     of Philox-4x32-10 with key = (lo32(seed), hi32(seed)) and counter =
 *     (lo32(g/4), hi32(g/4), worker, domain), domain 0 for C_nat, 2 for the sparsifier's
 *     index selection, 3 for the master's C_nat and 4 for compressed norms.
 *     The dithering operators (domain 1) draw one call per 8 elements instead: counter
 *     (lo32(g/8), hi32(g/8), worker, 1); with (a, b) = output words (0, 1) for g mod 8 < 4 and
 *     (2, 3) otherwise, the element's word is a, b, a<<16 | b>>16 or b<<16 | a>>16 for
 *     g mod 4 = 0, 1, 2, 3: each a rearrangement of 32 distinct bits of the call's output, so
 *     uniform by itself (neighbouring elements are not independent; unbiasedness and the
 *     variance bound of the operators are statements about single coordinates).
 *     Results therefore do not depend on how a vector is split into calls or launches.
 *
 * Plane layouts (little-endian bit order inside a byte):
 *   sign plane      bit (i mod 8) of byte i/8 is the sign bit of element i; ceil(d/8) bytes,
 *                   unused high bits of the last byte are written as zero.
 *   exponent plane  byte i is the 8-bit exponent field of C_nat(x_i); d bytes.
 *   level codes     c = 0 is the level 0 and c in 1..s is the level 2^(c-s).  With
 *                   b = ceil(log2(s+1)) bits per code:
 *                     b <= 3: fused nibbles (sign << 3) | c, element i in byte i/2, low nibble
 *                             for even i; no sign plane;
 *                     b == 4: nibble plane of codes (same order) + sign plane;
 *                     b >= 5: one byte per code + sign plane.
 *                   Planes are indexed by the element's position in the call's vector.
 *
 * Sizes: a call takes at most d = 2^34 elements (NC_ERR_INVALID beyond: one launch holds fewer
 * than 2^32 lanes); the sparse entry points take d <= 2^32 (32-bit indices).  A launch the
 * device rejects (for example one workgroup per bucket with hundreds of millions of tiny
 * buckets) is reported as NC_ERR_LAUNCH; nothing has run in that case.
 */
#ifndef NATCOMP_H
#define NATCOMP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    NC_OK = 0,
    NC_ERR_NULL = 1,        /* a required pointer is NULL */
    NC_ERR_INVALID = 2,     /* n = 0, s outside its range, bad strides or segment description, d beyond the
                               maximum (d = 0 is not an error: the call returns NC_OK and does nothing) */
    NC_ERR_UNSUPPORTED = 3, /* p is not 1, 2 or INFINITY */
    NC_ERR_WORKSPACE = 4,   /* workspace missing or too small */
    NC_ERR_LAUNCH = 5       /* the HIP runtime refused a launch */
} nc_status;

/* Human-readable name of a status code (static storage). */
const char *nc_status_string(nc_status st);

/* ----------------------------------------------------------------------------------------
 * Sizes (pure host functions).
 * -------------------------------------------------------------------------------------- */
size_t nc_nat_exp_bytes(uint64_t d);                   /* d */
size_t nc_sign_bytes(uint64_t d);                      /* ceil(d/8) */
size_t nc_dither_code_bytes(uint64_t d, uint32_t s);   /* ceil(d/2) for s <= 15, else d; 0 if s is outside 1..255 */
size_t nc_dither_sign_bytes(uint64_t d, uint32_t s);   /* 0 for s <= 7, else ceil(d/8) */
/* Suggested distance between the planes of consecutive workers: bytes rounded up to 256. */
size_t nc_plane_stride(size_t bytes);
/* Number of segments a description yields (see nc_dither_encode). */
uint64_t nc_segment_count(uint64_t d, uint32_t num_segments, uint32_t bucket, int have_offsets);
/* Bytes of DEVICE scratch nc_dither_encode needs for this description (0 when none). */
size_t nc_dither_workspace_bytes(uint64_t d, uint32_t num_segments, uint32_t bucket, int have_offsets);

/* ----------------------------------------------------------------------------------------
 * Natural compression (Sec. 2, Def. 1; binary32 realisation in "From 32 to 9 bits").
 *
 * Each x_i = (-1)^sign 2^(e-127) (1+m) is rounded to 2^(e+1-127) with probability m and to
 * 2^(e-127) otherwise, by comparing the random word r with the mantissa: up iff
 * r < m * 2^32 (m as a fraction), an integer comparison on the bit pattern; no
 * floating-point operation touches the value.  Zeros and exact powers of two are
 * unchanged; subnormals go to 0 or 2^-126; exponent 255 (Inf, NaN) stays 255 and values
 * in (2^127, 2^128) may round to it.  Output: exponent plane + sign plane.
 *
 *   x         DEVICE, d floats.
 *   exp_out   DEVICE, nc_nat_exp_bytes(d) bytes.     sign_out  DEVICE, nc_sign_bytes(d) bytes.
 * Fastest when x is 16-byte aligned, exp_out and sign_out 4-byte aligned and index_offset a multiple
 * of 4; any alignment and offset is accepted.
 * -------------------------------------------------------------------------------------- */
nc_status nc_nat_encode(const float *x, uint64_t d, uint64_t seed, uint32_t worker,
                        uint64_t index_offset, uint8_t *exp_out, uint8_t *sign_out, void *stream);

/* The same for n workers in one launch: worker w (stream id first_worker + w) reads
 * x + w*x_stride (stride in floats) and writes exp_out + w*exp_stride and
 * sign_out + w*sign_stride (strides in bytes).  Equal to n calls of nc_nat_encode. */
nc_status nc_nat_encode_batch(const float *x, size_t x_stride, uint32_t n, uint64_t d, uint64_t seed,
                              uint32_t first_worker, uint64_t index_offset, uint8_t *exp_out,
                              size_t exp_stride, uint8_t *sign_out, size_t sign_stride, void *stream);

/* Decoder: out_i has the stored sign and exponent and a zero mantissa ("computation-free",
 * Sec. 2).  exp, sign DEVICE planes of d elements; out DEVICE, d floats. */
nc_status nc_nat_decode(const uint8_t *exp, const uint8_t *sign, uint64_t d, float *out, void *stream);

/* ----------------------------------------------------------------------------------------
 * Natural dithering D_nat^{p,s} (Sec. 3, Def. 3 with levels 0, 2^(1-s), ..., 1/2, 1 and the
 * norm sent uncompressed).
 *
 * The vector is cut into segments and each is normalised by its own p-norm (the paper
 * normalises the whole vector: that is the single-segment case).  Segments are given by
 *   seg_offsets != NULL: DEVICE array of num_segments+1 ascending uint64, first 0, last d
 *                        (empty segments allowed); bucket ignored;
 *   seg_offsets == NULL, bucket > 0: consecutive buckets of `bucket` elements (last shorter);
 *   seg_offsets == NULL, bucket == 0: one segment.
 * Per element: y = fl(|x_i| * fl(1/norm)) in binary32; y between adjacent levels
 * l_low <= y <= l_high goes to l_high with probability (y - l_low)/(l_high - l_low), decided
 * by an integer comparison of the top 23 bits r23 of the random word with a 23-bit threshold
 * built from y's bits: for y = 2^-k (1 + m/2^23) >= 2^(1-s) the threshold is m (exact); below
 * the lowest level 2^(1-s) it is y 2^(s+22) rounded to the nearest integer, ties to even
 * (within 2^-24 of the exact probability; for s <= 126 the mantissa field of
 * fl(y/2 + 2^-s)); y >= 1 is the level 1.  A segment whose norm is below 2^-126 (zero
 * included) codes to zeros.
 *
 *   p           1, 2 or INFINITY.               s  number of levels, 1..127.
 *   norms_out   DEVICE, one float per segment: the p-norm (sum accumulated in double,
 *               rounded once to binary32; the maximum for p = INFINITY is exact).
 *   code_out    DEVICE, nc_dither_code_bytes(d, s).
 *   sign_out    DEVICE, nc_dither_sign_bytes(d, s); may be NULL when that is 0.
 *   workspace   DEVICE scratch of at least nc_dither_workspace_bytes(...) bytes, 8-byte
 *               aligned; may be NULL when that is 0.  Contents need not be initialised.
 * -------------------------------------------------------------------------------------- */
nc_status nc_dither_encode(const float *x, uint64_t d, const uint64_t *seg_offsets, uint32_t num_segments,
                           uint32_t bucket, float p, uint32_t s, uint64_t seed, uint32_t worker,
                           uint64_t index_offset, float *norms_out, uint8_t *code_out, uint8_t *sign_out,
                           void *workspace, size_t workspace_bytes, void *stream);

/* nc_dither_encode for callers that cannot allocate device memory or pass a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments (without the workspace), same kernels and bit-identical outputs; the scratch
 * memory is a static device array of nc_static_scratch_bytes() = 4 MiB that every GPU the
 * library runs on holds until the process ends.  The call allocates nothing and frees nothing.
 *   - nc_static_scratch_init() looks up the array's address on the current device (the HIP
 *     runtime places the array in device memory at that moment, once per device and process).
 *     Call it at set-up, with the device current, before a region that must not touch the
 *     allocator (a graph capture, say); otherwise the first nc_dither_encode_static call on a
 *     device does the same.  NC_OK, or NC_ERR_LAUNCH if the runtime cannot resolve the address.
 *   - A description whose nc_dither_workspace_bytes(...) exceeds nc_static_scratch_bytes()
 *     is rejected with NC_ERR_WORKSPACE and nothing is enqueued (use nc_dither_encode then):
 *     with segment offsets this allows about d <= 2.5e8 with up to 65,536 segments;
 *     descriptions that need no workspace (fixed buckets of at most 8192 elements that are a
 *     multiple of 8) are never rejected for size.
 *   - All calls on one GPU share that GPU's array: calls that may run concurrently (different
 *     streams, different host threads) race on it and must be serialised by the caller.  The
 *     array keeps the previous call's contents; the kernels rewrite every slot they read.
 *   - NC_ERR_LAUNCH if the runtime cannot resolve the array's address. */
size_t nc_static_scratch_bytes(void);
nc_status nc_static_scratch_init(void);
nc_status nc_dither_encode_static(const float *x, uint64_t d, const uint64_t *seg_offsets, uint32_t num_segments,
                                  uint32_t bucket, float p, uint32_t s, uint64_t seed, uint32_t worker,
                                  uint64_t index_offset, float *norms_out, uint8_t *code_out, uint8_t *sign_out,
                                  void *stream);

/* Decoder: out_i = sign * fl(norm_segment * 2^(c-s)), a signed zero for c = 0 (multiplying by
 * the level is an exponent addition, Sec. 3 and the fast-aggregation remark). */
nc_status nc_dither_decode(const float *norms, const uint8_t *code, const uint8_t *sign, uint64_t d,
                           const uint64_t *seg_offsets, uint32_t num_segments, uint32_t bucket, uint32_t s,
                           float *out, void *stream);

/* Standard dithering D_sta^{p,s} (Def. 3 with the linear partition l = j/s and the norm sent
 * uncompressed: the operator of QSGD and TernGrad), the comparison operator of the paper's
 * empirical-variance study.  Same arguments, segments, planes and code formats as
 * nc_dither_encode / nc_dither_decode (random words: the same stream, domain 1), with
 * 1 <= s <= 255 and level code c in 0..s standing for c/s:
 *   t = fl(y s) with y = fl(|x| fl(1/norm)); c = floor(t) + [r < floor((t - floor(t)) 2^32)];
 *   t >= s gives c = s.  Decoded value: sign * fl(norm * fl(c / s)). */
nc_status nc_dither_sta_encode(const float *x, uint64_t d, const uint64_t *seg_offsets, uint32_t num_segments,
                               uint32_t bucket, float p, uint32_t s, uint64_t seed, uint32_t worker,
                               uint64_t index_offset, float *norms_out, uint8_t *code_out, uint8_t *sign_out,
                               void *workspace, size_t workspace_bytes, void *stream);
nc_status nc_dither_sta_decode(const float *norms, const uint8_t *code, const uint8_t *sign, uint64_t d,
                               const uint64_t *seg_offsets, uint32_t num_segments, uint32_t bucket, uint32_t s,
                               float *out, void *stream);

/* Naturally compressed norms (Sec. 3: general dithering with C = C_nat on the norm, 8 bits per
 * norm; multiplying a level by such a norm is an exponent addition, at the price of a factor
 * 9/8 in the second moment).  Each non-negative norms[s] is rounded by C_nat with word s of a
 * stream of its own (domain 4): exp_out[s] is its exponent byte and norms_q_out[s] the power of
 * two it stands for, ready to be passed as `norms` to nc_dither_decode / nc_aggregate_sum.  The
 * encoder keeps normalising by the exact norm, as Def. 3 prescribes.
 *   norms, norms_q_out DEVICE count floats (may be the same array);  exp_out DEVICE count bytes. */
nc_status nc_norm_compress(const float *norms, uint64_t count, uint64_t seed, uint32_t worker,
                           uint8_t *exp_out, float *norms_q_out, void *stream);

/* Decoding straight from the 8-bit norms: norm_exp[s] is the exponent byte nc_norm_compress
 * wrote (the norm 2^(e-127), e = 0 meaning 0), so the wire carries one byte per norm and the
 * product norm * 2^(c-s) is the exponent sum e + c - s (Sec. 3 and the appendix on fast
 * aggregation).  Same result, bit for bit, as nc_dither_decode with the power-of-two floats.
 * For the sum over workers use nc_aggregate_sum with kind = NC_KIND_DITHER_NORM8: `norms`
 * then points at the exponent bytes (cast to const float *) and norm_stride counts bytes. */
nc_status nc_dither_decode_norm8(const uint8_t *norm_exp, const uint8_t *code, const uint8_t *sign, uint64_t d,
                                 const uint64_t *seg_offsets, uint32_t num_segments, uint32_t bucket,
                                 uint32_t s, float *out, void *stream);

/* ----------------------------------------------------------------------------------------
 * Master-side aggregation (Algorithm 1: Delta = sum over workers of the decompressed
 * updates).  One fused kernel decodes the n code streams and adds them in binary32 in the
 * fixed order ((v_0 + v_1) + v_2) + ... ; the result is the sum, not the mean.
 *
 * The descriptor is a HOST struct.  Worker w's planes start at code + w*code_stride,
 * sign + w*sign_stride (bytes) and norms + w*norm_stride (floats).
 *   kind = NC_KIND_NAT:    code is the exponent plane; norms, s and the segment fields unused.
 *   kind = NC_KIND_DITHER: code/sign/norms as written by nc_dither_encode with the same s and
 *                          segment description; sign may be NULL when s <= 7.
 *   kind = NC_KIND_DITHER_STA: the same for nc_dither_sta_encode.
 *   kind = NC_KIND_DITHER_NORM8: as NC_KIND_DITHER with 8-bit norms (see nc_dither_decode_norm8).
 * out: DEVICE, d floats.  Fastest when strides are multiples of 16 and planes 16-byte aligned.
 * -------------------------------------------------------------------------------------- */
enum { NC_KIND_NAT = 0, NC_KIND_DITHER = 1, NC_KIND_DITHER_STA = 2, NC_KIND_DITHER_NORM8 = 3 };

typedef struct {
    int32_t kind;
    uint32_t n;                 /* number of workers, >= 1 */
    uint64_t d;
    uint32_t s;                 /* D_nat only */
    uint32_t bucket;            /* D_nat only */
    const uint8_t *code;   size_t code_stride;
    const uint8_t *sign;   size_t sign_stride;
    const float *norms;    size_t norm_stride;      /* D_nat only */
    const uint64_t *seg_offsets; uint32_t num_segments; uint32_t reserved; /* D_nat only */
} nc_agg_desc;

nc_status nc_aggregate_sum(const nc_agg_desc *desc, float *out, void *stream);

/* Master step of Algorithm 1 with compression on the master too (bidirectional compression,
 * Sec. 4): g = C_M(sum over workers of the decompressed updates) with C_M = C_nat.  One fused
 * kernel sums the n C_nat streams as nc_aggregate_sum does (binary32, worker order) and
 * naturally compresses the sum; the fp32 sum is never written.  The master's random words come
 * from a stream of their own: domain 3, with `master` in the counter field the workers use for
 * their id, element i at global index index_offset + i.
 *   desc     HOST, kind = NC_KIND_NAT.
 *   exp_out  DEVICE, nc_nat_exp_bytes(d) bytes;  sign_out  DEVICE, nc_sign_bytes(d) bytes. */
nc_status nc_master_nat(const nc_agg_desc *desc, uint64_t seed, uint32_t master, uint64_t index_offset,
                        uint8_t *exp_out, uint8_t *sign_out, void *stream);

/* ----------------------------------------------------------------------------------------
 * The 8-bit representation and the integer aggregator of the in-network aggregation
 * prototype (experimental setup, paragraph "Implementation optimization"; appendix "Natural
 * Compression and Dithering Allow for Fast Aggregation").
 *
 * One byte per element: bit 7 = sign of x, bit 6 = 1 marks C_nat(x) = 0, bits 5..0 = field =
 * clip(exponent of C_nat(x), -50, 10) + 50 (0 when bit 6 is set).  The clip clamps: magnitudes
 * below 2^-50 become 2^-50, above 2^10 (Inf, NaN) become 2^10.  The random words are those of
 * nc_nat_encode (same seed, worker, index_offset: the byte is the clipped form of that call's
 * exponent and sign).
 *
 * nc_nat_clip_encode: n workers' vectors in one launch.
 *   x            DEVICE, worker w at x + w * x_stride (floats), d elements each.
 *   code_out     DEVICE, worker w at code_out + w * code_stride (bytes), d bytes each.
 *   first_worker worker id of w = 0 (ids are consecutive); strides are ignored for n = 1.
 *   Vector path: x 16-byte and code_out 4-byte aligned, strides multiples of 4, index_offset a
 *   multiple of 4; anything else takes a slower kernel with the same result.
 * nc_nat_clip_decode: out[i] = +-2^(field - 50) or a signed zero (DEVICE, d floats).
 * nc_clip_aggregate_int: every byte is restored as the 64-bit integer +-2^field (units of
 *   2^-50; fields 61..63, which the encoder never writes, are taken literally), the n workers
 *   are added as integers (exact for n <= 7 and in any case modulo 2^64), and the sum S is
 *   compressed with C_nat from the master's stream (domain 3, `master` in the worker field,
 *   element i at index_offset + i): for 2^k <= |S| < 2^(k+1) the exponent is k + 1 iff
 *   r < floor((|S| - 2^k) / 2^k * 2^32), else k.
 *   code       DEVICE, worker w at code + w * code_stride.
 *   sum_out    DEVICE, d int64 (units of 2^-50), or NULL.
 *   exp_out    DEVICE, d bytes: binary32 exponent field of the compressed sum (k - 50 + 127,
 *              plus one when rounded up; 0 for S = 0), decodable with nc_nat_decode;
 *   sign_out   DEVICE, nc_sign_bytes(d) bytes: bit set for S < 0.  exp_out and sign_out are
 *              both given or both NULL; at least one of sum_out / exp_out must be given.
 * Errors: NC_ERR_NULL for missing pointers, NC_ERR_INVALID for n = 0, strides below d, d above
 * the library maximum or a sum_out that is not 8-byte aligned.  All calls are asynchronous on
 * `stream`; buffers stay owned by the caller.
 * -------------------------------------------------------------------------------------- */
nc_status nc_nat_clip_encode(const float *x, size_t x_stride, uint32_t n, uint64_t d, uint64_t seed,
                             uint32_t first_worker, uint64_t index_offset, uint8_t *code_out,
                             size_t code_stride, void *stream);
nc_status nc_nat_clip_decode(const uint8_t *code, uint64_t d, float *out, void *stream);
nc_status nc_clip_aggregate_int(const uint8_t *code, size_t code_stride, uint32_t n, uint64_t d, uint64_t seed,
                                uint32_t master, uint64_t index_offset, int64_t *sum_out, uint8_t *exp_out,
                                uint8_t *sign_out, void *stream);

/* ----------------------------------------------------------------------------------------
 * Random sparsification composed with natural compression, C_nat o S^k (formal definition
 * of S^q in the appendix on sparsification: S^q(x) = (d/q) xi o x with exactly q kept
 * coordinates; C_nat o S^q is in B(9d/8q - 1) by the composition theorem of Sec. 2).
 *
 * The k kept coordinates of a worker are pi(0), ..., pi(k-1) for a keyed pseudo-random
 * permutation pi of [0, d): a 4-round alternating Feistel network on b = ceil(log2 d) >= 2
 * bits (high part A of floor(b/2) bits, low part B: A ^= F(B,k0), B ^= F(A,k1), A ^= F(B,k2),
 * B ^= F(A,k3), each truncated to its part) with cycle walking; the round keys are the four
 * words of the Philox call with counter (0, 0, worker, 2) and key = seed, and
 * F(R, key): t = R*0x9E3779B1 + key; t ^= t>>16; t *= 0x85EBCA6B; t ^= t>>13; t *= 0xC2B2AE35;
 * t ^= t>>16.
 * Entry j of the message: idx_out[j] = i = pi(j); exponent byte j and sign bit j are
 * C_nat(fl(scale * x[i])) with the random word of dense position i in the C_nat stream
 * (so k = d, scale = 1 reproduces nc_nat_encode).  scale = d/k makes the operator unbiased.
 *
 *   x DEVICE d floats (1 <= d <= 2^32, 1 <= k <= d);  idx_out DEVICE k uint32;
 *   exp_out DEVICE k bytes;  sign_out DEVICE ceil(k/8) bytes.
 * The batch form encodes n workers in one launch (strides in elements of each array).
 * -------------------------------------------------------------------------------------- */
nc_status nc_sparse_nat_encode(const float *x, uint64_t d, uint64_t k, float scale, uint64_t seed,
                               uint32_t worker, uint32_t *idx_out, uint8_t *exp_out, uint8_t *sign_out,
                               void *stream);
nc_status nc_sparse_nat_encode_batch(const float *x, size_t x_stride, uint32_t n, uint64_t d, uint64_t k,
                                     float scale, uint64_t seed, uint32_t first_worker, uint32_t *idx_out,
                                     size_t idx_stride, uint8_t *exp_out, size_t exp_stride, uint8_t *sign_out,
                                     size_t sign_stride, void *stream);

/* Master's sum of n sparse messages (Algorithm 1): out[0..d) is zero-filled, then worker
 * w = 0, 1, ..., n-1 adds its k decoded values at its indices, in binary32 and in this
 * order (one launch per worker, so the result is reproducible).  Indices >= d are ignored;
 * a worker's indices must be distinct.  out DEVICE d floats. */
nc_status nc_sparse_nat_aggregate(const uint32_t *idx, size_t idx_stride, const uint8_t *exp, size_t exp_stride,
                                  const uint8_t *sign, size_t sign_stride, uint32_t n, uint64_t k, uint64_t d,
                                  float *out, void *stream);

/* The same sum (Algorithm 1's master sum of sparse messages), bit for bit, for large d: the
 * n*k entries are first sorted by output position inside a caller workspace (two counting
 * sorts: at most 256 coarse bins, then tiles of 8192 positions), then every tile of out is
 * built in on-chip memory, worker by worker in worker order, and written once, zeros included.
 * The per-worker scatter of nc_sparse_nat_aggregate moves a whole cache line in and out of HBM
 * for every 4-byte addition; this form moves about 50 bytes per entry and 4 bytes per output
 * element.
 *   workspace DEVICE, 16-byte aligned, at least nc_sparse_aggregate_workspace_bytes(n, k, d)
 *   bytes (16*n*k for the sorted entries plus a few per cent for counters; 0 is returned for
 *   arguments the call rejects); its contents need no initialisation and mean nothing
 *   afterwards; calls that share a workspace must not overlap.
 * Limits beyond those of nc_sparse_nat_aggregate: n <= 65535 and n*k < 2^32 (NC_ERR_INVALID);
 * NC_ERR_WORKSPACE for a missing, misaligned or short workspace.  Indices >= d are ignored; a
 * worker's indices must be distinct. */
size_t nc_sparse_aggregate_workspace_bytes(uint32_t n, uint64_t k, uint64_t d);
nc_status nc_sparse_nat_aggregate_ws(const uint32_t *idx, size_t idx_stride, const uint8_t *exp, size_t exp_stride,
                                     const uint8_t *sign, size_t sign_stride, uint32_t n, uint64_t k, uint64_t d,
                                     float *out, void *workspace, size_t workspace_bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* NATCOMP_H */
