// C ABI of libnatcomp: argument validation, alignment-based path selection and kernel
// launches.  Declarations and the meaning of every argument are in include/natcomp.h.
#include "../../include/natcomp.h"

#include <hip/hip_runtime.h>
#include <math.h>

#include <atomic>

#include "kernels.hpp"

using namespace natcomp;

namespace {

// A launch may hold at most 2^32 - 1 lanes; the vector kernels give a lane 4 to 32 elements.
constexpr uint64_t kMaxD = 1ull << 34;

// Scratch memory of nc_dither_encode_static: one array per GPU, held until the process ends.
// The name is a host-side stand-in; the device address comes from hipGetSymbolAddress, once
// per device, and only that address is ever passed to a kernel.
constexpr size_t kStaticScratchBytes = (size_t)4 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
std::atomic<void*> g_scratch_address[kMaxDevices];

// Address of `scratch` on the current device (nullptr if the runtime cannot tell).
void* static_scratch_address() {
    int device = -1;
    if (hipGetDevice(&device) != hipSuccess || device < 0 || device >= kMaxDevices) return nullptr;
    void* p = g_scratch_address[device].load(std::memory_order_acquire);
    if (!p) {
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return nullptr;
        g_scratch_address[device].store(p, std::memory_order_release);  // every thread finds the same address
    }
    return p;
}

inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }
inline nc_status from_hip(hipError_t e) { return e == hipSuccess ? NC_OK : NC_ERR_LAUNCH; }
inline uint32_t code_width(uint32_t s) { uint32_t b = 0; while ((1u << b) < s + 1) ++b; return b; }
inline bool valid_s(uint32_t s) { return s >= 1 && s <= 127; }       // natural levels: all normal numbers
inline bool valid_s_size(uint32_t s) { return s >= 1 && s <= 255; }  // codes 0..s fit one byte

}  // namespace

extern "C" {

const char* nc_status_string(nc_status st) {
    switch (st) {
        case NC_OK: return "NC_OK";
        case NC_ERR_NULL: return "NC_ERR_NULL";
        case NC_ERR_INVALID: return "NC_ERR_INVALID";
        case NC_ERR_UNSUPPORTED: return "NC_ERR_UNSUPPORTED";
        case NC_ERR_WORKSPACE: return "NC_ERR_WORKSPACE";
        case NC_ERR_LAUNCH: return "NC_ERR_LAUNCH";
    }
    return "NC_ERR_?";
}

size_t nc_nat_exp_bytes(uint64_t d) { return (size_t)d; }
size_t nc_sign_bytes(uint64_t d) { return (size_t)((d + 7) / 8); }
size_t nc_dither_code_bytes(uint64_t d, uint32_t s) {
    if (!valid_s_size(s)) return 0;
    return code_width(s) <= 4 ? (size_t)((d + 1) / 2) : (size_t)d;
}
size_t nc_dither_sign_bytes(uint64_t d, uint32_t s) {
    if (!valid_s_size(s)) return 0;
    return code_width(s) <= 3 ? 0 : (size_t)((d + 7) / 8);
}
size_t nc_plane_stride(size_t bytes) { return (bytes + 255) & ~(size_t)255; }

uint64_t nc_segment_count(uint64_t d, uint32_t num_segments, uint32_t bucket, int have_offsets) {
    if (have_offsets) return num_segments;
    if (bucket) return (d + bucket - 1) / bucket;
    return 1;
}

nc_status nc_nat_encode_batch(const float* x, size_t x_stride, uint32_t n, uint64_t d, uint64_t seed,
                              uint32_t first_worker, uint64_t index_offset, uint8_t* exp_out, size_t exp_stride,
                              uint8_t* sign_out, size_t sign_stride, void* stream) {
    if (n == 0 || d > kMaxD || n > 65535) return NC_ERR_INVALID;
    if (d == 0) return NC_OK;
    if (!x || !exp_out || !sign_out) return NC_ERR_NULL;
    if (n > 1 && (x_stride < d || exp_stride < nc_nat_exp_bytes(d) || sign_stride < nc_sign_bytes(d)))
        return NC_ERR_INVALID;
    NatEncodeArgs a;
    a.x = x; a.x_stride = x_stride; a.d = d;
    a.k0 = (uint32_t)seed; a.k1 = (uint32_t)(seed >> 32);
    a.first_worker = first_worker; a.index_offset = index_offset;
    a.exp_out = exp_out; a.exp_stride = exp_stride; a.sign_out = sign_out; a.sign_stride = sign_stride;
    const bool fast = aligned(x, 16) && aligned(exp_out, 4) && aligned(sign_out, 4) && (index_offset & 3) == 0 &&
                      (n == 1 || ((x_stride & 3) == 0 && (exp_stride & 3) == 0 && (sign_stride & 3) == 0));
    return from_hip(launch_nat_encode(a, n, fast, (hipStream_t)stream));
}

nc_status nc_nat_encode(const float* x, uint64_t d, uint64_t seed, uint32_t worker, uint64_t index_offset,
                        uint8_t* exp_out, uint8_t* sign_out, void* stream) {
    return nc_nat_encode_batch(x, 0, 1, d, seed, worker, index_offset, exp_out, 0, sign_out, 0, stream);
}

nc_status nc_nat_decode(const uint8_t* exp, const uint8_t* sign, uint64_t d, float* out, void* stream) {
    if (d > kMaxD) return NC_ERR_INVALID;
    if (d == 0) return NC_OK;
    if (!exp || !sign || !out) return NC_ERR_NULL;
    NatDecodeArgs a{exp, sign, d, out};
    const bool fast = aligned(exp, 8) && aligned(out, 16);
    return from_hip(launch_nat_decode(a, fast, (hipStream_t)stream));
}

// Segment description checks shared by the dithering entry points.
static nc_status check_segments(uint64_t d, const uint64_t* seg_offsets, uint32_t num_segments, uint32_t bucket,
                                Segs* out) {
    if (seg_offsets) {
        if (num_segments == 0 || num_segments >= (1u << 31)) return NC_ERR_INVALID;
    } else if (bucket) {
        if ((d + bucket - 1) / bucket >= (1ull << 31)) return NC_ERR_INVALID;
    }
    out->offsets = seg_offsets;
    out->num_segments = seg_offsets ? num_segments : 0;
    out->bucket = seg_offsets ? 0 : bucket;
    out->d = d;
    out->count = (uint32_t)nc_segment_count(d, num_segments, bucket, seg_offsets != nullptr);
    return NC_OK;
}
static inline bool one_pass_bucket(const uint64_t* seg_offsets, uint32_t bucket) {
    return !seg_offsets && bucket >= 8 && bucket <= kMaxOnePassBucket && (bucket & 7) == 0;
}
static inline int format_of(uint32_t s) {
    const uint32_t b = code_width(s);
    return b <= 3 ? kFmtFused : b == 4 ? kFmtNibble : kFmtByte;
}
static inline size_t align8(size_t v) { return (v + 7) & ~(size_t)7; }

size_t nc_dither_workspace_bytes(uint64_t d, uint32_t num_segments, uint32_t bucket, int have_offsets) {
    if (d == 0) return 0;
    if (!have_offsets && one_pass_bucket(nullptr, bucket)) return 0;
    const uint64_t nseg = nc_segment_count(d, num_segments, bucket, have_offsets);
    const uint64_t chunks = (d + kNormChunk - 1) / kNormChunk;
    const uint64_t code_chunks = have_offsets ? (d + kChunk - 1) / kChunk : 0;
    return (size_t)(8 * chunks + 8 * nseg + align8(4 * nseg) + sizeof(ChunkSegment) * code_chunks);
}

static nc_status dither_encode(uint32_t standard, const float* x, uint64_t d, const uint64_t* seg_offsets,
                               uint32_t num_segments, uint32_t bucket, float p, uint32_t s, uint64_t seed,
                               uint32_t worker, uint64_t index_offset, float* norms_out, uint8_t* code_out,
                               uint8_t* sign_out, void* workspace, size_t workspace_bytes, void* stream,
                               bool static_scratch = false) {
    if (!(standard ? valid_s_size(s) : valid_s(s)) || d > kMaxD) return NC_ERR_INVALID;
    int pnorm;
    if (p == 1.0f) pnorm = kNormL1;
    else if (p == 2.0f) pnorm = kNormL2;
    else if (isinf(p) && p > 0) pnorm = kNormInf;
    else return NC_ERR_UNSUPPORTED;
    if (d == 0) return NC_OK;
    if (!x || !norms_out || !code_out) return NC_ERR_NULL;
    const int fmt = format_of(s);
    if (fmt != kFmtFused && !sign_out) return NC_ERR_NULL;
    DitherEncodeArgs a{};
    nc_status st = check_segments(d, seg_offsets, num_segments, bucket, &a.segs);
    if (st != NC_OK) return st;
    a.x = x; a.pnorm = pnorm; a.s = s; a.fmt = fmt; a.standard = standard;
    a.k0 = (uint32_t)seed; a.k1 = (uint32_t)(seed >> 32); a.worker = worker; a.index_offset = index_offset;
    a.norms_out = norms_out; a.code_out = code_out; a.sign_out = sign_out;
    const bool fast = aligned(x, 16) && (index_offset & 3) == 0 && aligned(code_out, fmt == kFmtByte ? 8 : 4) &&
                      (fmt == kFmtFused || aligned(sign_out, 4));
    if (one_pass_bucket(seg_offsets, bucket))
        return from_hip(launch_dither_bucket_encode(a, fast, (hipStream_t)stream));
    const size_t need = nc_dither_workspace_bytes(d, num_segments, bucket, seg_offsets != nullptr);
    if (static_scratch) {  // the library's own array instead of a caller workspace
        if (need > kStaticScratchBytes) return NC_ERR_WORKSPACE;
        workspace = static_scratch_address();
        if (!workspace) return NC_ERR_LAUNCH;
        workspace_bytes = kStaticScratchBytes;
    }
    if (!workspace || workspace_bytes < need || !aligned(workspace, 8)) return NC_ERR_WORKSPACE;
    const uint64_t nseg = nc_segment_count(d, num_segments, bucket, seg_offsets != nullptr);
    const uint64_t chunks = (d + kNormChunk - 1) / kNormChunk;
    a.first_partial = static_cast<double*>(workspace);
    a.head_partial = a.first_partial + chunks;
    a.inv_norm = reinterpret_cast<float*>(a.head_partial + nseg);
    a.chunk_segment = seg_offsets ? reinterpret_cast<ChunkSegment*>(static_cast<char*>(workspace) + 8 * chunks +
                                                                    8 * nseg + align8(4 * nseg))
                                  : nullptr;
    return from_hip(launch_dither_segment_encode(a, fast, (hipStream_t)stream));
}

nc_status nc_dither_encode(const float* x, uint64_t d, const uint64_t* seg_offsets, uint32_t num_segments,
                           uint32_t bucket, float p, uint32_t s, uint64_t seed, uint32_t worker,
                           uint64_t index_offset, float* norms_out, uint8_t* code_out, uint8_t* sign_out,
                           void* workspace, size_t workspace_bytes, void* stream) {
    return dither_encode(0, x, d, seg_offsets, num_segments, bucket, p, s, seed, worker, index_offset, norms_out,
                         code_out, sign_out, workspace, workspace_bytes, stream);
}

size_t nc_static_scratch_bytes(void) { return kStaticScratchBytes; }

nc_status nc_static_scratch_init(void) { return static_scratch_address() ? NC_OK : NC_ERR_LAUNCH; }

nc_status nc_dither_encode_static(const float* x, uint64_t d, const uint64_t* seg_offsets, uint32_t num_segments,
                                  uint32_t bucket, float p, uint32_t s, uint64_t seed, uint32_t worker,
                                  uint64_t index_offset, float* norms_out, uint8_t* code_out, uint8_t* sign_out,
                                  void* stream) {
    return dither_encode(0, x, d, seg_offsets, num_segments, bucket, p, s, seed, worker, index_offset, norms_out,
                         code_out, sign_out, nullptr, 0, stream, /*static_scratch=*/true);
}

nc_status nc_dither_sta_encode(const float* x, uint64_t d, const uint64_t* seg_offsets, uint32_t num_segments,
                               uint32_t bucket, float p, uint32_t s, uint64_t seed, uint32_t worker,
                               uint64_t index_offset, float* norms_out, uint8_t* code_out, uint8_t* sign_out,
                               void* workspace, size_t workspace_bytes, void* stream) {
    return dither_encode(1, x, d, seg_offsets, num_segments, bucket, p, s, seed, worker, index_offset, norms_out,
                         code_out, sign_out, workspace, workspace_bytes, stream);
}

static nc_status dither_aggregate(uint32_t standard, uint32_t norm8, const float* norms, size_t norm_stride, const uint8_t* code, size_t code_stride,
                                  const uint8_t* sign, size_t sign_stride, uint32_t n, uint64_t d,
                                  const uint64_t* seg_offsets, uint32_t num_segments, uint32_t bucket, uint32_t s,
                                  float* out, void* stream) {
    if (!(standard ? valid_s_size(s) : valid_s(s)) || d > kMaxD || n == 0) return NC_ERR_INVALID;
    if (d == 0) return NC_OK;
    if (!norms || !code || !out) return NC_ERR_NULL;
    const int fmt = format_of(s);
    if (fmt != kFmtFused && !sign) return NC_ERR_NULL;
    DitherAggregateArgs a{};
    nc_status st = check_segments(d, seg_offsets, num_segments, bucket, &a.segs);
    if (st != NC_OK) return st;
    if (n > 1) {
        if (code_stride < nc_dither_code_bytes(d, s) || (fmt != kFmtFused && sign_stride < nc_dither_sign_bytes(d, s)) ||
            norm_stride < nc_segment_count(d, num_segments, bucket, seg_offsets != nullptr))
            return NC_ERR_INVALID;
    }
    a.norms = norms; a.norm_stride = norm_stride; a.code = code; a.code_stride = code_stride;
    a.sign = sign; a.sign_stride = sign_stride; a.n = n; a.s = s; a.fmt = fmt; a.standard = standard; a.out = out;
    a.norm8 = norm8;
    const bool fast = aligned(code, 4) && aligned(out, 16) && (n == 1 || (code_stride & 3) == 0);
    return from_hip(launch_dither_aggregate(a, fast, (hipStream_t)stream));
}

nc_status nc_dither_decode(const float* norms, const uint8_t* code, const uint8_t* sign, uint64_t d,
                           const uint64_t* seg_offsets, uint32_t num_segments, uint32_t bucket, uint32_t s,
                           float* out, void* stream) {
    return dither_aggregate(0, 0, norms, 0, code, 0, sign, 0, 1, d, seg_offsets, num_segments, bucket, s, out, stream);
}

nc_status nc_dither_decode_norm8(const uint8_t* norm_exp, const uint8_t* code, const uint8_t* sign, uint64_t d,
                                 const uint64_t* seg_offsets, uint32_t num_segments, uint32_t bucket, uint32_t s,
                                 float* out, void* stream) {
    return dither_aggregate(0, 1, reinterpret_cast<const float*>(norm_exp), 0, code, 0, sign, 0, 1, d, seg_offsets,
                            num_segments, bucket, s, out, stream);
}

nc_status nc_dither_sta_decode(const float* norms, const uint8_t* code, const uint8_t* sign, uint64_t d,
                               const uint64_t* seg_offsets, uint32_t num_segments, uint32_t bucket, uint32_t s,
                               float* out, void* stream) {
    return dither_aggregate(1, 0, norms, 0, code, 0, sign, 0, 1, d, seg_offsets, num_segments, bucket, s, out, stream);
}

nc_status nc_sparse_nat_encode_batch(const float* x, size_t x_stride, uint32_t n, uint64_t d, uint64_t k, float scale,
                                     uint64_t seed, uint32_t first_worker, uint32_t* idx_out, size_t idx_stride,
                                     uint8_t* exp_out, size_t exp_stride, uint8_t* sign_out, size_t sign_stride,
                                     void* stream) {
    if (n == 0 || n > 65535 || d == 0 || d > (1ull << 32) || k == 0 || k > d) return NC_ERR_INVALID;
    if (!x || !idx_out || !exp_out || !sign_out) return NC_ERR_NULL;
    if (n > 1 && (x_stride < d || idx_stride < k || exp_stride < k || sign_stride < (k + 7) / 8)) return NC_ERR_INVALID;
    SparseEncodeArgs a{};
    a.x = x; a.x_stride = x_stride; a.d = d; a.k = k; a.scale = scale;
    a.bits = 2;
    while (a.bits < 32 && (1ull << a.bits) < d) ++a.bits;
    a.k0 = (uint32_t)seed; a.k1 = (uint32_t)(seed >> 32); a.first_worker = first_worker;
    a.idx_out = idx_out; a.idx_stride = idx_stride; a.exp_out = exp_out; a.exp_stride = exp_stride;
    a.sign_out = sign_out; a.sign_stride = sign_stride;
    a.vec = aligned(idx_out, 16) && aligned(exp_out, 8) && (n == 1 || ((idx_stride & 3) == 0 && (exp_stride & 7) == 0));
    return from_hip(launch_sparse_nat_encode(a, n, (hipStream_t)stream));
}

nc_status nc_sparse_nat_encode(const float* x, uint64_t d, uint64_t k, float scale, uint64_t seed, uint32_t worker,
                               uint32_t* idx_out, uint8_t* exp_out, uint8_t* sign_out, void* stream) {
    return nc_sparse_nat_encode_batch(x, 0, 1, d, k, scale, seed, worker, idx_out, 0, exp_out, 0, sign_out, 0, stream);
}

nc_status nc_sparse_nat_aggregate(const uint32_t* idx, size_t idx_stride, const uint8_t* exp, size_t exp_stride,
                                  const uint8_t* sign, size_t sign_stride, uint32_t n, uint64_t k, uint64_t d,
                                  float* out, void* stream) {
    if (n == 0 || d == 0 || d > (1ull << 32) || k == 0 || k > d) return NC_ERR_INVALID;
    if (!idx || !exp || !sign || !out) return NC_ERR_NULL;
    if (n > 1 && (idx_stride < k || exp_stride < k || sign_stride < (k + 7) / 8)) return NC_ERR_INVALID;
    return from_hip(launch_sparse_nat_aggregate(idx, idx_stride, exp, exp_stride, sign, sign_stride, n, k, d, out,
                                                aligned(out, 16), (hipStream_t)stream));
}

static bool sparse_partition_ok(uint32_t n, uint64_t k, uint64_t d) {
    return n >= 1 && n <= 65535 && d >= 1 && d <= (1ull << 32) && k >= 1 && k <= d && (uint64_t)n * k < (1ull << 32);
}

size_t nc_sparse_aggregate_workspace_bytes(uint32_t n, uint64_t k, uint64_t d) {
    if (!sparse_partition_ok(n, k, d)) return 0;
    return (size_t)sparse_partition_plan(n, k, d).bytes;
}

nc_status nc_sparse_nat_aggregate_ws(const uint32_t* idx, size_t idx_stride, const uint8_t* exp, size_t exp_stride,
                                     const uint8_t* sign, size_t sign_stride, uint32_t n, uint64_t k, uint64_t d,
                                     float* out, void* workspace, size_t workspace_bytes, void* stream) {
    if (!sparse_partition_ok(n, k, d)) return NC_ERR_INVALID;
    if (!idx || !exp || !sign || !out) return NC_ERR_NULL;
    if (n > 1 && (idx_stride < k || exp_stride < k || sign_stride < (k + 7) / 8)) return NC_ERR_INVALID;
    if (!workspace || !aligned(workspace, 16) || workspace_bytes < sparse_partition_plan(n, k, d).bytes)
        return NC_ERR_WORKSPACE;
    return from_hip(launch_sparse_nat_aggregate_partitioned(idx, idx_stride, exp, exp_stride, sign, sign_stride, n, k, d,
                                                            out, aligned(out, 16), workspace, (hipStream_t)stream));
}

nc_status nc_norm_compress(const float* norms, uint64_t count, uint64_t seed, uint32_t worker, uint8_t* exp_out,
                           float* norms_q_out, void* stream) {
    if (count >= (1ull << 31) * kBlock) return NC_ERR_INVALID;
    if (count == 0) return NC_OK;
    if (!norms || !exp_out || !norms_q_out) return NC_ERR_NULL;
    return from_hip(launch_norm_compress(norms, count, (uint32_t)seed, (uint32_t)(seed >> 32), worker, exp_out,
                                         norms_q_out, (hipStream_t)stream));
}

nc_status nc_master_nat(const nc_agg_desc* desc, uint64_t seed, uint32_t master, uint64_t index_offset,
                        uint8_t* exp_out, uint8_t* sign_out, void* stream) {
    if (!desc) return NC_ERR_NULL;
    if (desc->n == 0 || desc->d > kMaxD || desc->kind != NC_KIND_NAT) return NC_ERR_INVALID;
    if (desc->d == 0) return NC_OK;
    if (!desc->code || !desc->sign || !exp_out || !sign_out) return NC_ERR_NULL;
    if (desc->n > 1 && (desc->code_stride < nc_nat_exp_bytes(desc->d) || desc->sign_stride < nc_sign_bytes(desc->d)))
        return NC_ERR_INVALID;
    NatAggregateArgs a{desc->code, desc->code_stride, desc->sign, desc->sign_stride, desc->n, desc->d, nullptr};
    NatMasterArgs m{(uint32_t)seed, (uint32_t)(seed >> 32), master, index_offset, exp_out, sign_out};
    const bool fast = aligned(desc->code, 8) && (desc->n == 1 || (desc->code_stride & 7) == 0) && aligned(exp_out, 8) &&
                      (index_offset & 3) == 0;
    return from_hip(launch_nat_master(a, m, fast, (hipStream_t)stream));
}

nc_status nc_nat_clip_encode(const float* x, size_t x_stride, uint32_t n, uint64_t d, uint64_t seed,
                             uint32_t first_worker, uint64_t index_offset, uint8_t* code_out, size_t code_stride,
                             void* stream) {
    if (n == 0 || d > kMaxD || n > 65535) return NC_ERR_INVALID;
    if (d == 0) return NC_OK;
    if (!x || !code_out) return NC_ERR_NULL;
    if (n > 1 && (x_stride < d || code_stride < d)) return NC_ERR_INVALID;
    ClipEncodeArgs a{x, x_stride, d, (uint32_t)seed, (uint32_t)(seed >> 32), first_worker, index_offset, code_out,
                     code_stride};
    const bool fast = aligned(x, 16) && aligned(code_out, 4) && (index_offset & 3) == 0 &&
                      (n == 1 || ((x_stride & 3) == 0 && (code_stride & 3) == 0));
    return from_hip(launch_clip_encode(a, n, fast, (hipStream_t)stream));
}

nc_status nc_nat_clip_decode(const uint8_t* code, uint64_t d, float* out, void* stream) {
    if (d > kMaxD) return NC_ERR_INVALID;
    if (d == 0) return NC_OK;
    if (!code || !out) return NC_ERR_NULL;
    return from_hip(launch_clip_decode(code, d, out, aligned(code, 8) && aligned(out, 16), (hipStream_t)stream));
}

nc_status nc_clip_aggregate_int(const uint8_t* code, size_t code_stride, uint32_t n, uint64_t d, uint64_t seed,
                                uint32_t master, uint64_t index_offset, int64_t* sum_out, uint8_t* exp_out,
                                uint8_t* sign_out, void* stream) {
    if (n == 0 || d > kMaxD) return NC_ERR_INVALID;
    if (d == 0) return NC_OK;
    if (!code || (!sum_out && !exp_out) || (exp_out == nullptr) != (sign_out == nullptr)) return NC_ERR_NULL;
    if (n > 1 && code_stride < d) return NC_ERR_INVALID;
    if (sum_out && !aligned(sum_out, 8)) return NC_ERR_INVALID;
    ClipAggregateArgs a{code, code_stride, n, d, (uint32_t)seed, (uint32_t)(seed >> 32), master, index_offset,
                        sum_out, exp_out, sign_out};
    const bool fast = aligned(code, 8) && (n == 1 || (code_stride & 7) == 0) && (!exp_out || aligned(exp_out, 8)) &&
                      (!sum_out || aligned(sum_out, 16)) && (index_offset & 3) == 0;
    return from_hip(launch_clip_aggregate(a, fast, (hipStream_t)stream));
}

nc_status nc_aggregate_sum(const nc_agg_desc* desc, float* out, void* stream) {
    if (!desc) return NC_ERR_NULL;
    if (desc->n == 0 || desc->d > kMaxD) return NC_ERR_INVALID;
    if (desc->kind != NC_KIND_NAT && desc->kind != NC_KIND_DITHER && desc->kind != NC_KIND_DITHER_STA &&
        desc->kind != NC_KIND_DITHER_NORM8)
        return NC_ERR_INVALID;
    if (desc->d == 0) return NC_OK;
    if (!out || !desc->code) return NC_ERR_NULL;
    if (desc->kind == NC_KIND_NAT) {
        if (!desc->sign) return NC_ERR_NULL;
        if (desc->n > 1 && (desc->code_stride < nc_nat_exp_bytes(desc->d) || desc->sign_stride < nc_sign_bytes(desc->d)))
            return NC_ERR_INVALID;
        NatAggregateArgs a{desc->code, desc->code_stride, desc->sign, desc->sign_stride, desc->n, desc->d, out};
        const bool one = desc->n == 1;
        const bool w8 = aligned(desc->code, 8) && aligned(out, 16) && (one || (desc->code_stride & 7) == 0);
        const bool w16 = w8 && aligned(desc->code, 16) && aligned(desc->sign, 2) &&
                         (one || ((desc->code_stride & 15) == 0 && (desc->sign_stride & 1) == 0));
        return from_hip(launch_nat_aggregate(a, w16 ? 16 : w8 ? 8 : 0, (hipStream_t)stream));
    }
    return dither_aggregate(desc->kind == NC_KIND_DITHER_STA ? 1u : 0u, desc->kind == NC_KIND_DITHER_NORM8 ? 1u : 0u, desc->norms, desc->norm_stride, desc->code, desc->code_stride, desc->sign,
                            desc->sign_stride, desc->n, desc->d, desc->seg_offsets, desc->num_segments, desc->bucket,
                            desc->s, out, stream);
}

}  // extern "C"
