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

// ------------------------------------------------------------------------ partitioned sum
// The same sum with every cache line of the dense vector written once.  The one-launch-per-worker
// scatter above pays a whole line read and written for each 4-byte addition; here the n*k
// entries are first sorted by output position, in two counting sorts so that every pass writes
// runs of about a line (coarse bins of 2^coarse_shift positions, at most 256 of them, then the
// tiles of 2^kSparseTileShift positions inside each bin), and one workgroup per tile then builds
// its piece of the sum in LDS and stores it, zeros included.
// An entry travels as two words: its index and meta = exponent byte | sign << 8 | worker << 9
// (so meta << 23 is the binary32 value).  The sorted lists keep no order inside a bin: a tile's
// workgroup adds its entries worker by worker, one barrier per worker, which is the order of the
// scatter path; a worker's indices are distinct, so the additions of one round touch different
// words.
// Each sort is count -> prefix sums -> move, with no global atomics (thousands of workgroups
// adding to the same 160 counters serialise): a workgroup takes a chunk of kSparseChunk
// entries, leaves its histogram in a matrix, a small kernel turns every matrix column (one
// bin, all chunks) into running offsets, and the moving pass sorts its chunk in LDS so that
// what it writes to a bin is one contiguous run.
constexpr uint32_t kSparseChunk = 8192;   // entries per workgroup in the counting and moving passes
constexpr uint32_t kPerLane = kSparseChunk / kBlock;   // counting passes: 256 lanes x 32 entries
constexpr int kMoveLanes = 1024;                         // moving passes: 1024 lanes x 8 entries (four words
constexpr uint32_t kMovePerLane = kSparseChunk / kMoveLanes;  // per entry stay in registers across the sort)
constexpr uint32_t kSparseTile = 1u << kSparseTileShift;
constexpr uint32_t kMaxTileBins = 2048;   // tiles per coarse bin at d = 2^32

// Exclusive prefix sum over the workgroup (LANES lanes); *total gets the sum.  `lds`: LANES/64 words.
template <int LANES = kBlock>
__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t v, uint32_t* lds, uint32_t* total) {
    const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
    uint32_t incl = v;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const uint32_t t = __shfl_up(incl, o, 64);
        if (lane >= (uint32_t)o) incl += t;
    }
    __syncthreads();  // (lds may still be read from an earlier call)
    if (lane == 63u) lds[wave] = incl;
    __syncthreads();
    uint32_t before = 0, all = 0;
#pragma unroll
    for (uint32_t w = 0; w < LANES / 64; ++w) {
        const uint32_t t = lds[w];
        before += w < wave ? t : 0u;
        all += t;
    }
    *total = all;
    return before + incl - v;
}

// A chunk's words: the lane's entries are first + threadIdx.x + kBlock * r; bit r of the returned
// mask says that entry exists.  A whole chunk is loaded without a test between the loads.
template <int LANES, uint32_t PER>
__device__ __forceinline__ uint32_t load_chunk_words(const uint32_t* __restrict__ src, uint64_t first, uint64_t end,
                                                     uint32_t (&v)[PER]) {
    static_assert(LANES * PER == kSparseChunk, "a chunk per workgroup");
    if (first + kSparseChunk <= end) {
#pragma unroll
        for (uint32_t r = 0; r < PER; ++r) v[r] = load_stream(src + first + threadIdx.x + LANES * r);
        return PER == 32 ? 0xFFFFFFFFu : (1u << PER) - 1u;
    }
    uint32_t have = 0u;
#pragma unroll
    for (uint32_t r = 0; r < PER; ++r) {
        const uint64_t j = first + threadIdx.x + LANES * r;
        v[r] = 0u;
        if (j < end) { v[r] = src[j]; have |= 1u << r; }
    }
    return have;
}

// Histogram of the chunk's bins in LDS (hist: nbins words, zeroed here).  BIN(index) -> bin.
template <class BinOf>
__device__ __forceinline__ void chunk_histogram(const uint32_t (&i)[kPerLane], uint32_t have, uint32_t nbins,
                                                uint32_t* hist, BinOf bin_of) {
    for (uint32_t b = threadIdx.x; b < nbins; b += kBlock) hist[b] = 0u;
    __syncthreads();
#pragma unroll
    for (uint32_t r = 0; r < kPerLane; ++r)
        if ((have >> r) & 1u) atomicAdd(&hist[bin_of(i[r])], 1u);
    __syncthreads();
}

// The chunk sorted by bin in LDS and written out as one run per bin: run_base(bin) is where this
// chunk's run of the bin starts in the output lists.  hist, lstart, delta: nbins words each;
// buf: kSparseChunk entries (index in the low word, meta in the high word).  Workgroups of
// kMoveLanes lanes; lanes own bins t*per_lane .. t*per_lane + per_lane - 1 for the prefix sums
// (per_lane = nbins / kMoveLanes, at least 1).  (Entries written straight from the lanes that
// hold them, 4 bytes here and 4 bytes there, take twice as long as the runs out of LDS.)
template <class BinOf, class RunBase>
__device__ __forceinline__ void chunk_sort_and_write(const uint32_t (&i)[kMovePerLane], const uint32_t (&meta)[kMovePerLane],
                                                     uint32_t have, uint32_t nbins, uint32_t* hist, uint32_t* lstart,
                                                     uint32_t* delta, uint64_t* buf, uint32_t* scan_lds, BinOf bin_of,
                                                     RunBase run_base, uint32_t* __restrict__ out_idx,
                                                     uint32_t* __restrict__ out_meta) {
    for (uint32_t b = threadIdx.x; b < nbins; b += kMoveLanes) hist[b] = 0u;
    __syncthreads();
    uint32_t rank[kMovePerLane];
#pragma unroll
    for (uint32_t r = 0; r < kMovePerLane; ++r) {
        rank[r] = 0u;
        if ((have >> r) & 1u) rank[r] = atomicAdd(&hist[bin_of(i[r])], 1u);
    }
    const uint32_t per_lane = nbins > (uint32_t)kMoveLanes ? nbins / kMoveLanes : 1u;
    const uint32_t b0 = threadIdx.x * per_lane;
    __syncthreads();
    uint32_t own = 0;
    if (b0 < nbins)
        for (uint32_t q = 0; q < per_lane; ++q) own += hist[b0 + q];
    uint32_t total;
    uint32_t start = block_exclusive_scan<kMoveLanes>(own, scan_lds, &total);
    if (b0 < nbins) {
        for (uint32_t q = 0; q < per_lane; ++q) {
            const uint32_t c = hist[b0 + q];
            lstart[b0 + q] = start;
            delta[b0 + q] = c ? run_base(b0 + q) - start : 0u;
            start += c;
        }
    }
    __syncthreads();
#pragma unroll
    for (uint32_t r = 0; r < kMovePerLane; ++r)
        if ((have >> r) & 1u) buf[lstart[bin_of(i[r])] + rank[r]] = ((uint64_t)meta[r] << 32) | i[r];
    __syncthreads();
#pragma unroll
    for (uint32_t r = 0; r < kMovePerLane; ++r) {
        const uint32_t q = threadIdx.x + kMoveLanes * r;
        if (q < total) {
            const uint64_t e = buf[q];
            const uint32_t v = (uint32_t)e;
            const uint32_t dst = delta[bin_of(v)] + q;
            out_idx[dst] = v;
            out_meta[dst] = (uint32_t)(e >> 32);
        }
    }
}

// Pass 1: the chunk's entries per coarse bin -> hist1[bin][chunk] (indices >= d are dropped
// here and in pass 3).  Chunks are numbered worker by worker.
__global__ __launch_bounds__(kBlock) void sparse_count_coarse_kernel(SparsePartitionArgs a) {
    __shared__ uint32_t hist[kBlock];
    const uint32_t* __restrict__ idx = a.idx + (size_t)blockIdx.y * a.idx_stride;
    uint32_t i[kPerLane];
    uint32_t have = load_chunk_words<kBlock>(idx, (uint64_t)blockIdx.x * kSparseChunk, a.k, i);
#pragma unroll
    for (uint32_t r = 0; r < kPerLane; ++r)
        if ((uint64_t)i[r] >= a.d) have &= ~(1u << r);
    const uint32_t shift = a.coarse_shift;
    chunk_histogram(i, have, a.coarse_bins, hist, [shift](uint32_t v) { return v >> shift; });
    const uint32_t chunk = blockIdx.y * gridDim.x + blockIdx.x;
    if (threadIdx.x < a.coarse_bins) a.hist1[(size_t)threadIdx.x * a.chunks1 + chunk] = hist[threadIdx.x];
}

// Pass 2: one workgroup per coarse bin turns its row of hist1 into running offsets (exclusive,
// in place) and leaves the bin's total.
__global__ __launch_bounds__(kBlock) void sparse_scan_coarse_kernel(SparsePartitionArgs a) {
    __shared__ uint32_t scan_lds[kBlock / 64];
    uint32_t* __restrict__ row = a.hist1 + (size_t)blockIdx.x * a.chunks1;
    constexpr uint32_t kEach = 8;
    uint32_t carry = 0;
    for (uint32_t c0 = 0; c0 < a.chunks1; c0 += kBlock * kEach) {
        uint32_t v[kEach], own = 0;
        const uint32_t first = c0 + threadIdx.x * kEach;
#pragma unroll
        for (uint32_t q = 0; q < kEach; ++q) {
            v[q] = first + q < a.chunks1 ? row[first + q] : 0u;
            own += v[q];
        }
        uint32_t total;
        uint32_t at = carry + block_exclusive_scan(own, scan_lds, &total);
#pragma unroll
        for (uint32_t q = 0; q < kEach; ++q) {
            if (first + q < a.chunks1) row[first + q] = at;
            at += v[q];
        }
        carry += total;
    }
    if (threadIdx.x == 0) a.coarse_count[blockIdx.x] = carry;
}

// Pass 3: entries moved into their coarse bins.  A bin's base is the prefix sum of the bins'
// totals (every workgroup computes them itself: at most 256 words).
__global__ __launch_bounds__(kMoveLanes) void sparse_move_coarse_kernel(SparsePartitionArgs a) {
    __shared__ uint32_t hist[kBlock], lstart[kBlock], delta[kBlock], base[kBlock];
    __shared__ uint64_t buf[kSparseChunk];
    __shared__ uint32_t scan_lds[kMoveLanes / 64];
    const uint32_t w = blockIdx.y;
    const uint32_t* __restrict__ idx = a.idx + (size_t)w * a.idx_stride;
    const uint8_t* __restrict__ exp = a.exp + (size_t)w * a.exp_stride;
    const uint8_t* __restrict__ sign = a.sign + (size_t)w * a.sign_stride;
    const uint64_t j0 = (uint64_t)blockIdx.x * kSparseChunk;
    const uint32_t chunk = blockIdx.y * gridDim.x + blockIdx.x;
    // where this chunk's runs start: the bin's base plus the chunk's running offset in the bin
    const uint32_t bin_total = threadIdx.x < a.coarse_bins ? a.coarse_count[threadIdx.x] : 0u;
    const uint32_t offset = threadIdx.x < a.coarse_bins ? a.hist1[(size_t)threadIdx.x * a.chunks1 + chunk] : 0u;
    uint32_t i[kMovePerLane], meta[kMovePerLane];
    uint32_t have = load_chunk_words<kMoveLanes>(idx, j0, a.k, i);
    if (j0 + kSparseChunk <= a.k) {  // a whole chunk: no test between the loads
#pragma unroll
        for (uint32_t r = 0; r < kMovePerLane; ++r) {
            const uint64_t j = j0 + threadIdx.x + kMoveLanes * r;
            meta[r] = (uint32_t)load_stream(exp + j) | ((uint32_t)sign[j >> 3] << 16) | ((uint32_t)(j & 7) << 24);
        }
    } else {
#pragma unroll
        for (uint32_t r = 0; r < kMovePerLane; ++r) {
            const uint64_t j = j0 + threadIdx.x + kMoveLanes * r;
            meta[r] = 0u;
            if ((have >> r) & 1u) meta[r] = (uint32_t)exp[j] | ((uint32_t)sign[j >> 3] << 16) | ((uint32_t)(j & 7) << 24);
        }
    }
#pragma unroll
    for (uint32_t r = 0; r < kMovePerLane; ++r) {  // exponent | sign << 8 | worker << 9
        const uint32_t sg = (meta[r] >> (16u + (meta[r] >> 24))) & 1u;
        meta[r] = (meta[r] & 0xFFu) | (sg << 8) | (w << 9);
        if ((uint64_t)i[r] >= a.d) have &= ~(1u << r);
    }
    uint32_t all;
    const uint32_t bin_base = block_exclusive_scan<kMoveLanes>(bin_total, scan_lds, &all);
    if (threadIdx.x < kBlock) base[threadIdx.x] = bin_base + offset;
    const uint32_t shift = a.coarse_shift;
    chunk_sort_and_write(i, meta, have, a.coarse_bins, hist, lstart, delta, buf, scan_lds,
                         [shift](uint32_t v) { return v >> shift; }, [&](uint32_t b) { return base[b]; }, a.idx1, a.meta1);
}

// Which piece of the coarse-sorted list a workgroup of pass 4 takes: chunks of kSparseChunk
// entries that do not cross a bin's end, numbered bin by bin (pass 6 takes the same pieces from
// the descriptors that pass 5 leaves).  False past the last chunk (the grid is sized for the worst
// case; workgroup-uniform).
struct CoarsePiece {
    uint32_t bin, bin_base, begin, end, first_chunk;  // first_chunk: number of the bin's first chunk
};
template <int LANES>
__device__ __forceinline__ bool coarse_piece(const SparsePartitionArgs& a, uint32_t chunk, uint32_t* scan_lds,
                                             CoarsePiece* slot, CoarsePiece& out) {
    const uint32_t cnt = threadIdx.x < a.coarse_bins ? a.coarse_count[threadIdx.x] : 0u;
    const uint32_t chunks = (cnt + kSparseChunk - 1) / kSparseChunk;
    uint32_t total_chunks, total;
    const uint32_t chunk_base = block_exclusive_scan<LANES>(chunks, scan_lds, &total_chunks);
    const uint32_t entry_base = block_exclusive_scan<LANES>(cnt, scan_lds, &total);
    if (chunk >= total_chunks) return false;
    if (chunk_base <= chunk && chunk < chunk_base + chunks) {
        const uint32_t c = chunk - chunk_base;
        const uint32_t b = entry_base + c * kSparseChunk;
        const uint32_t e = entry_base + cnt;
        *slot = CoarsePiece{threadIdx.x, entry_base, b, e - b > kSparseChunk ? b + kSparseChunk : e, chunk_base};
    }
    __syncthreads();
    out = *slot;
    return true;
}

// Pass 4: the chunk's entries per tile of its coarse bin -> hist2[chunk][tile].
__global__ __launch_bounds__(kBlock) void sparse_count_tiles_kernel(SparsePartitionArgs a) {
    __shared__ uint32_t hist[kMaxTileBins];
    __shared__ uint32_t scan_lds[kBlock / 64];
    __shared__ CoarsePiece slot;
    CoarsePiece pc;
    if (!coarse_piece<kBlock>(a, blockIdx.x, scan_lds, &slot, pc)) return;
    const uint32_t tile_bins = 1u << (a.coarse_shift - kSparseTileShift);
    uint32_t i[kPerLane];
    const uint32_t have = load_chunk_words<kBlock>(a.idx1, pc.begin, pc.end, i);
    chunk_histogram(i, have, tile_bins, hist, [tile_bins](uint32_t v) { return (v >> kSparseTileShift) & (tile_bins - 1u); });
    uint32_t* __restrict__ row = a.hist2 + (size_t)blockIdx.x * tile_bins;
    for (uint32_t t = threadIdx.x; t < tile_bins; t += kBlock) row[t] = hist[t];
}

// Pass 5: one workgroup per coarse bin: for every tile, running offsets over the bin's chunks
// (in place in hist2), the tile's count, and its base in the tile-sorted lists.
__global__ __launch_bounds__(kBlock) void sparse_scan_tiles_kernel(SparsePartitionArgs a) {
    __shared__ uint32_t scan_lds[kBlock / 64];
    __shared__ CoarsePiece slot;
    const uint32_t tile_bins = 1u << (a.coarse_shift - kSparseTileShift);
    // this bin's base, number of chunks and first chunk, from the same prefix sums as coarse_piece
    const uint32_t cnt = threadIdx.x < a.coarse_bins ? a.coarse_count[threadIdx.x] : 0u;
    const uint32_t chunks = (cnt + kSparseChunk - 1) / kSparseChunk;
    uint32_t total_chunks, total;
    const uint32_t chunk_base = block_exclusive_scan(chunks, scan_lds, &total_chunks);
    const uint32_t entry_base = block_exclusive_scan(cnt, scan_lds, &total);
    if (threadIdx.x == blockIdx.x) slot = CoarsePiece{threadIdx.x, entry_base, chunks, cnt, chunk_base};
    __syncthreads();
    const CoarsePiece pc = slot;  // begin = number of chunks, end = entries of the bin
    const uint32_t per_lane = tile_bins > (uint32_t)kBlock ? tile_bins / kBlock : 1u;
    const uint32_t t0 = threadIdx.x * per_lane;
    const size_t bin_tiles = (size_t)blockIdx.x * tile_bins;
    uint32_t own = 0;
    uint32_t counts[kMaxTileBins / kBlock];
#pragma unroll
    for (uint32_t q = 0; q < kMaxTileBins / kBlock; ++q) {
        counts[q] = 0u;
        if (q < per_lane && t0 + q < tile_bins) {
            uint32_t run = 0;
            for (uint32_t c = 0; c < pc.begin; ++c) {
                uint32_t* cell = a.hist2 + (size_t)(pc.first_chunk + c) * tile_bins + t0 + q;
                const uint32_t v = *cell;
                *cell = run;
                run += v;
            }
            counts[q] = run;
            own += run;
        }
    }
    uint32_t all;
    uint32_t at = pc.bin_base + block_exclusive_scan(own, scan_lds, &all);
#pragma unroll
    for (uint32_t q = 0; q < kMaxTileBins / kBlock; ++q) {
        if (q < per_lane && t0 + q < tile_bins) {
            a.tile_count[bin_tiles + t0 + q] = counts[q];
            a.tile_base[bin_tiles + t0 + q] = at;
            at += counts[q];
        }
    }
    // what pass 6 needs to know about each of this bin's chunks, so that it starts with one load
    for (uint32_t c = threadIdx.x; c < pc.begin; c += kBlock) {
        const uint32_t b = pc.bin_base + c * kSparseChunk, e = pc.bin_base + pc.end;
        a.pieces[pc.first_chunk + c] = SparsePiece{blockIdx.x, b, e - b > kSparseChunk ? b + kSparseChunk : e, 0u};
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) *a.total_chunks = total_chunks;
}

// Pass 6: entries moved into their tiles.  MAX_BINS: 256 (two workgroups fit a CU's LDS) or
// kMaxTileBins (d beyond 2^29).
template <uint32_t MAX_BINS>
__global__ __launch_bounds__(kMoveLanes) void sparse_move_tiles_kernel(SparsePartitionArgs a) {
    __shared__ uint32_t hist[MAX_BINS], lstart[MAX_BINS], delta[MAX_BINS];
    __shared__ uint64_t buf[kSparseChunk];
    __shared__ uint32_t scan_lds[kMoveLanes / 64];
    if (blockIdx.x >= *a.total_chunks) return;  // (the grid is sized for the worst case)
    const SparsePiece pc = a.pieces[blockIdx.x];
    const uint32_t tile_bins = 1u << (a.coarse_shift - kSparseTileShift);
    // where this chunk's run of each tile starts, for the tiles whose prefix sums the lane owns
    constexpr uint32_t kOwn = kMaxTileBins / kMoveLanes;
    const uint32_t per_lane = tile_bins > (uint32_t)kMoveLanes ? tile_bins / kMoveLanes : 1u;
    const uint32_t t0 = threadIdx.x * per_lane;
    const uint32_t* __restrict__ offsets = a.hist2 + (size_t)blockIdx.x * tile_bins;
    const uint32_t* __restrict__ bases = a.tile_base + (size_t)pc.bin * tile_bins;
    uint32_t run[kOwn];
#pragma unroll
    for (uint32_t q = 0; q < kOwn; ++q) {
        const uint32_t t = t0 + q < tile_bins ? t0 + q : 0u;  // (lanes without a tile: any valid one)
        run[q] = bases[t] + offsets[t];
    }
    uint32_t i[kMovePerLane], meta[kMovePerLane];
    const uint32_t have = load_chunk_words<kMoveLanes>(a.idx1, pc.begin, pc.end, i);
    load_chunk_words<kMoveLanes>(a.meta1, pc.begin, pc.end, meta);
    static_assert(kOwn == 2, "run_base below picks one of two");
    chunk_sort_and_write(i, meta, have, tile_bins, hist, lstart, delta, buf, scan_lds,
                         [tile_bins](uint32_t v) { return (v >> kSparseTileShift) & (tile_bins - 1u); },
                         [&](uint32_t t) { return t == t0 ? run[0] : run[1]; }, a.idx2, a.meta2);
}

// Pass 7: one workgroup per tile of the dense vector.  The tile starts as +0.0 (the scatter
// path's zero fill); the workers' entries are added in worker order; the tile leaves once.
template <bool VEC>
__global__ __launch_bounds__(kBlock) void sparse_tile_sum_kernel(SparsePartitionArgs a) {
    __shared__ __attribute__((aligned(16))) float tile[kSparseTile];
    constexpr uint32_t kHeld = 4;  // entries a lane keeps in registers
    const uint32_t cnt = a.tile_count[blockIdx.x];
    const uint32_t base = a.tile_base[blockIdx.x];
    const bool held = cnt <= kHeld * kBlock;  // workgroup-uniform
    uint32_t i[kHeld], meta[kHeld];
#pragma unroll
    for (uint32_t r = 0; r < kHeld; ++r) {
        const uint32_t e = threadIdx.x + kBlock * r;
        i[r] = 0u;
        meta[r] = 0xFFFFFFFFu;  // no worker has this number (n <= 65535)
        if (held && e < cnt) { i[r] = a.idx2[base + e]; meta[r] = a.meta2[base + e]; }
    }
    u32x4* t4 = reinterpret_cast<u32x4*>(tile);
#pragma unroll
    for (uint32_t r = 0; r < kSparseTile / 4 / kBlock; ++r) t4[threadIdx.x + kBlock * r] = u32x4{0u, 0u, 0u, 0u};
    __syncthreads();
    if (cnt) {
        for (uint32_t w = 0; w < a.n; ++w) {
            if (held) {
#pragma unroll
                for (uint32_t r = 0; r < kHeld; ++r)
                    if ((meta[r] >> 9) == w) tile[i[r] & (kSparseTile - 1u)] += bits_f32(meta[r] << 23);
            } else {  // a crowded tile: the list is read once per worker
                for (uint32_t e = threadIdx.x; e < cnt; e += kBlock) {
                    const uint32_t m = a.meta2[base + e];
                    if ((m >> 9) == w) tile[a.idx2[base + e] & (kSparseTile - 1u)] += bits_f32(m << 23);
                }
            }
            __syncthreads();
        }
    }
    const uint64_t p0 = (uint64_t)blockIdx.x << kSparseTileShift;
#pragma unroll
    for (uint32_t r = 0; r < kSparseTile / 4 / kBlock; ++r) {
        const uint32_t q = threadIdx.x + kBlock * r;
        const uint64_t p = p0 + 4ull * q;
        if (VEC && p + 4 <= a.d) {
            store_stream(reinterpret_cast<u32x4*>(a.out + p), t4[q]);
        } else {
            for (uint32_t c = 0; c < 4; ++c)
                if (p + c < a.d) a.out[p + c] = tile[4 * q + c];
        }
    }
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

SparsePartitionPlan sparse_partition_plan(uint32_t n, uint64_t k, uint64_t d) {
    SparsePartitionPlan p{};
    uint32_t shift = kSparseTileShift;
    while ((((d + (1ull << shift) - 1) >> shift)) > 256ull) ++shift;  // at most 256 coarse bins
    p.coarse_shift = shift;
    p.coarse_bins = (uint32_t)((d + (1ull << shift) - 1) >> shift);
    p.tile_bins = 1u << (shift - kSparseTileShift);
    p.tile_slots = (uint64_t)p.coarse_bins * p.tile_bins;
    p.tiles = (d + kSparseTile - 1) >> kSparseTileShift;
    p.entries = (uint64_t)n * k;
    p.chunks1 = (uint64_t)n * ((k + kSparseChunk - 1) / kSparseChunk);
    p.chunks2 = p.entries / kSparseChunk + p.coarse_bins;  // upper bound: one ragged chunk per bin
    auto up = [](uint64_t b) { return (b + 255) & ~255ull; };
    p.off_coarse_count = 0;
    p.off_tile_count = up(4 * 257);   // (the word after the 256 counts: chunks of the coarse-sorted lists)
    p.off_tile_base = p.off_tile_count + up(4 * p.tile_slots);
    p.off_hist1 = p.off_tile_base + up(4 * p.tile_slots);
    p.off_hist2 = p.off_hist1 + up(4 * p.coarse_bins * p.chunks1);
    p.off_pieces = p.off_hist2 + up(4 * p.chunks2 * p.tile_bins);
    p.off_lists = p.off_pieces + up(16 * p.chunks2);
    p.list_bytes = up(4 * p.entries);
    p.bytes = p.off_lists + 4 * p.list_bytes;
    return p;
}

hipError_t launch_sparse_nat_aggregate_partitioned(const uint32_t* idx, size_t idx_stride, const uint8_t* exp,
                                                   size_t exp_stride, const uint8_t* sign, size_t sign_stride,
                                                   uint32_t n, uint64_t k, uint64_t d, float* out, bool out_aligned,
                                                   void* workspace, hipStream_t stream) {
    const SparsePartitionPlan p = sparse_partition_plan(n, k, d);
    uint8_t* ws = static_cast<uint8_t*>(workspace);
    auto words = [ws](uint64_t off) { return reinterpret_cast<uint32_t*>(ws + off); };
    SparsePartitionArgs a{};
    a.idx = idx; a.idx_stride = idx_stride; a.exp = exp; a.exp_stride = exp_stride; a.sign = sign; a.sign_stride = sign_stride;
    a.n = n; a.k = k; a.d = d; a.coarse_shift = p.coarse_shift; a.coarse_bins = p.coarse_bins; a.chunks1 = (uint32_t)p.chunks1;
    a.coarse_count = words(p.off_coarse_count);
    a.tile_count = words(p.off_tile_count);
    a.tile_base = words(p.off_tile_base);
    a.hist1 = words(p.off_hist1);
    a.hist2 = words(p.off_hist2);
    a.pieces = reinterpret_cast<SparsePiece*>(ws + p.off_pieces);
    a.total_chunks = words(p.off_coarse_count) + 256;
    a.idx1 = words(p.off_lists);
    a.meta1 = words(p.off_lists + p.list_bytes);
    a.idx2 = words(p.off_lists + 2 * p.list_bytes);
    a.meta2 = words(p.off_lists + 3 * p.list_bytes);
    a.out = out;
    const dim3 by_message((unsigned)((k + kSparseChunk - 1) / kSparseChunk), n, 1);
    hipError_t e;
    sparse_count_coarse_kernel<<<by_message, kBlock, 0, stream>>>(a);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    sparse_scan_coarse_kernel<<<p.coarse_bins, kBlock, 0, stream>>>(a);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    sparse_move_coarse_kernel<<<by_message, kMoveLanes, 0, stream>>>(a);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    sparse_count_tiles_kernel<<<(unsigned)p.chunks2, kBlock, 0, stream>>>(a);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    sparse_scan_tiles_kernel<<<p.coarse_bins, kBlock, 0, stream>>>(a);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    if (p.tile_bins <= 256) sparse_move_tiles_kernel<256><<<(unsigned)p.chunks2, kMoveLanes, 0, stream>>>(a);
    else sparse_move_tiles_kernel<kMaxTileBins><<<(unsigned)p.chunks2, kMoveLanes, 0, stream>>>(a);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    if (out_aligned) sparse_tile_sum_kernel<true><<<(unsigned)p.tiles, kBlock, 0, stream>>>(a);
    else sparse_tile_sum_kernel<false><<<(unsigned)p.tiles, kBlock, 0, stream>>>(a);
    return hipGetLastError();
}

}  // namespace natcomp
