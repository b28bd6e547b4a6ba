// Host-visible launch interface between the C ABI layer and the kernel files.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace natcomp {

constexpr int kBlock = 256;  // lanes per workgroup (4 wavefronts)

struct NatEncodeArgs {
    const float* x; size_t x_stride;           // floats between workers
    uint64_t d;
    uint32_t k0, k1;                           // Philox key = (lo32(seed), hi32(seed))
    uint32_t first_worker;
    uint64_t index_offset;
    uint8_t* exp_out; size_t exp_stride;       // bytes between workers
    uint8_t* sign_out; size_t sign_stride;
};
struct NatDecodeArgs {
    const uint8_t* exp; const uint8_t* sign; uint64_t d; float* out;
};
struct NatAggregateArgs {
    const uint8_t* exp; size_t exp_stride; const uint8_t* sign; size_t sign_stride;
    uint32_t n; uint64_t d; float* out;
};

// Segment description shared by the dithering kernels: explicit offsets (num_segments+1
// ascending values), or a fixed bucket length, or (both absent) one segment.
struct Segs {
    const uint64_t* offsets; uint32_t num_segments; uint32_t bucket; uint64_t d;
    uint32_t count;   // number of segments whichever way they are described (set by the host)
};

enum { kNormL1 = 1, kNormL2 = 2, kNormInf = 3 };
// Code formats by bits per level code: fused nibble (sign<<3)|c, nibble + sign plane, byte + sign plane.
enum { kFmtFused = 0, kFmtNibble = 1, kFmtByte = 2 };

constexpr uint32_t kChunk = 2048;          // elements per workgroup in the chunked kernels (256 lanes x 8)
constexpr uint32_t kNormChunk = 8192;      // elements per workgroup in the partial-norm pass (256 lanes x 8 quads)
constexpr uint32_t kMaxOnePassBucket = 8192;  // largest bucket one workgroup keeps in registers

// What the encode pass needs to know about the segment that holds a chunk's first element
// (segment-offset mode: written by the norm-finishing pass, one record per kChunk elements).
struct ChunkSegment {
    uint64_t end;      // one past the segment's last element
    uint32_t segment;  // its index
    float inv_norm;    // reciprocal of its norm (0 for a norm below the smallest normal number)
};
struct DitherEncodeArgs {
    const float* x; Segs segs;
    int pnorm; uint32_t s; int fmt; uint32_t standard;   // standard = 1: levels j/s instead of 2^(j-s)
    uint32_t k0, k1, worker; uint64_t index_offset;
    float* norms_out; uint8_t* code_out; uint8_t* sign_out;
    double* first_partial;   // one per norm chunk (two-pass path only)
    double* head_partial;    // one per segment    (two-pass path only)
    float* inv_norm;         // one per segment    (two-pass path only)
    ChunkSegment* chunk_segment;  // one per kChunk elements (two-pass path with segment offsets only)
};
struct DitherAggregateArgs {
    const float* norms; size_t norm_stride; const uint8_t* code; size_t code_stride;
    const uint8_t* sign; size_t sign_stride;
    uint32_t n; Segs segs; uint32_t s; int fmt; uint32_t standard; float* out;
    uint32_t log2_bucket;   // set by the launcher for the kernel with per-bucket tables
    uint32_t norm8;         // 1: `norms` points at exponent bytes (norms rounded to powers of two)
};

// One-pass encoder for fixed buckets of at most kMaxOnePassBucket elements (a multiple of 8).
hipError_t launch_dither_bucket_encode(const DitherEncodeArgs& a, bool fast, hipStream_t stream);
// Two-pass encoder for any segment description: partial norms, per-segment finish, encode.
hipError_t launch_dither_segment_encode(const DitherEncodeArgs& a, bool fast, hipStream_t stream);
// Decode (n = 1) and fused decode-and-sum (n > 1) of dithering codes.
hipError_t launch_dither_aggregate(const DitherAggregateArgs& a, bool fast, hipStream_t stream);

struct SparseEncodeArgs {
    const float* x; size_t x_stride;
    uint64_t d, k; uint32_t bits;              // bits of the Feistel network: smallest b >= 2 with 2^b >= d
    float scale;
    uint32_t k0, k1, first_worker;
    uint32_t* idx_out; size_t idx_stride;      // elements between workers
    uint8_t* exp_out; size_t exp_stride;
    uint8_t* sign_out; size_t sign_stride;
    bool vec;                                  // idx_out 16-byte and exp_out 8-byte aligned for every worker
};
struct SparseScatterArgs {
    const uint32_t* idx; const uint8_t* exp; const uint8_t* sign; uint64_t k, d; float* out;
};
// The partitioned form of the scatter-sum: entries sorted by output position in a workspace,
// then one workgroup per tile of 2^kSparseTileShift output positions.
constexpr uint32_t kSparseTileShift = 13;
struct SparsePiece {   // one chunk of the coarse-sorted lists: its bin and entries [begin, end)
    uint32_t bin, begin, end, pad;
};
struct SparsePartitionArgs {
    const uint32_t* idx; size_t idx_stride; const uint8_t* exp; size_t exp_stride; const uint8_t* sign; size_t sign_stride;
    uint32_t n; uint64_t k, d; uint32_t coarse_shift, coarse_bins;
    uint32_t chunks1;        // chunks of the n messages (worker by worker)
    uint32_t* coarse_count;  // entries per coarse bin
    uint32_t* tile_count; uint32_t* tile_base;  // per tile: entries, start in the tile-sorted lists
    uint32_t* hist1;         // [coarse bin][message chunk]: counts, then running offsets
    uint32_t* hist2;         // [chunk of the coarse-sorted lists][tile of its bin]: the same
    SparsePiece* pieces;     // one per chunk of the coarse-sorted lists
    uint32_t* total_chunks;  // how many of them there are
    uint32_t* idx1; uint32_t* meta1;   // the entries sorted by coarse bin
    uint32_t* idx2; uint32_t* meta2;   // the entries sorted by tile
    float* out;
};
struct SparsePartitionPlan {
    uint32_t coarse_shift, coarse_bins, tile_bins;
    uint64_t tile_slots, tiles, entries, chunks1, chunks2;
    uint64_t off_coarse_count, off_tile_count, off_tile_base, off_hist1, off_hist2, off_pieces, off_lists, list_bytes, bytes;
};
SparsePartitionPlan sparse_partition_plan(uint32_t n, uint64_t k, uint64_t d);
hipError_t launch_sparse_nat_aggregate_partitioned(const uint32_t* idx, size_t idx_stride, const uint8_t* exp,
                                                   size_t exp_stride, const uint8_t* sign, size_t sign_stride,
                                                   uint32_t n, uint64_t k, uint64_t d, float* out, bool out_aligned,
                                                   void* workspace, hipStream_t stream);
hipError_t launch_sparse_nat_encode(const SparseEncodeArgs& a, uint32_t n, hipStream_t stream);
// Zero-fills out[0..d) and adds the n messages, one launch per worker in worker order.
hipError_t launch_sparse_nat_aggregate(const uint32_t* idx, size_t idx_stride, const uint8_t* exp, size_t exp_stride,
                                       const uint8_t* sign, size_t sign_stride, uint32_t n, uint64_t k, uint64_t d,
                                       float* out, bool out_aligned, hipStream_t stream);

hipError_t launch_norm_compress(const float* norms, uint64_t count, uint32_t k0, uint32_t k1, uint32_t worker,
                                uint8_t* exp_out, float* q_out, hipStream_t stream);

struct NatMasterArgs {
    uint32_t k0, k1, master; uint64_t index_offset; uint8_t* exp_out; uint8_t* sign_out;
};
hipError_t launch_nat_master(const NatAggregateArgs& a, const NatMasterArgs& m, bool fast, hipStream_t stream);

// Clipped 8-bit representation (one byte per element) and the integer aggregator.
struct ClipEncodeArgs {
    const float* x; size_t x_stride; uint64_t d;
    uint32_t k0, k1, first_worker; uint64_t index_offset;
    uint8_t* code_out; size_t code_stride;
};
struct ClipAggregateArgs {
    const uint8_t* code; size_t code_stride; uint32_t n; uint64_t d;
    uint32_t k0, k1, master; uint64_t index_offset;
    int64_t* sum_out;                       // may be null
    uint8_t* exp_out; uint8_t* sign_out;    // both null or both set
};
hipError_t launch_clip_encode(const ClipEncodeArgs& a, uint32_t n, bool fast, hipStream_t stream);
hipError_t launch_clip_decode(const uint8_t* code, uint64_t d, float* out, bool fast, hipStream_t stream);
hipError_t launch_clip_aggregate(const ClipAggregateArgs& a, bool fast, hipStream_t stream);

// `fast` promises the alignment the vector path needs (checked by the caller).
hipError_t launch_nat_encode(const NatEncodeArgs& a, uint32_t n, bool fast, hipStream_t stream);
hipError_t launch_nat_decode(const NatDecodeArgs& a, bool fast, hipStream_t stream);
// width: elements per lane the planes' alignment allows (16, 8) or 0 for any alignment.
hipError_t launch_nat_aggregate(const NatAggregateArgs& a, int width, hipStream_t stream);

}  // namespace natcomp
