// Bloom index kernels: build (Sec. 4.1), item-major export and the stand-alone mask export.
//
// Index layout in HBM ("rotated" / bit-sliced, Sec. 4.1, blocked for 128-byte lines):
//   word(tile, row, w) = bloom[(tile * m_bits + row) * 16 + w],  tile = item / 1024,
//   w = (item % 1024) / 64, bit (item % 64) of that word = bit `row` of the item's signature.
// One row segment of a tile is 16 words = 128 bytes; a filter that sets r signature bits
// touches r such lines per tile.
#pragma once
#include "st_device.h"

namespace st {

// One workgroup per 1024-item tile.  The tile's block of the index -- m rows of 128 bytes -- is
// assembled in LDS (in slabs of kBuildSlabRows rows where m is larger): every thread hashes the
// ids of its items once per slab (k positions each, Sec. 4.1), sets the item's bit in the rows the
// positions name with LDS atomic ORs, and the finished rows go out as one contiguous, coalesced
// copy.  Hash work is therefore independent of m up to the slab size, and HBM sees the feature
// lists once and the index once.
constexpr int kBuildThreads = 256;
constexpr int kBuildSlabRows = 1024;  // 128 KB of LDS

__global__ __launch_bounds__(kBuildThreads) void bloom_build_kernel(const int64_t* __restrict__ feat_offsets,
                                                                    const uint64_t* __restrict__ feat_ids,
                                                                    int64_t n_items, int32_t m_bits,
                                                                    int32_t k_hashes, uint64_t* __restrict__ bloom)
{
    extern __shared__ __attribute__((aligned(16))) uint32_t s_bits[];  // [rows][32]: the 16 words of a row as 32-bit halves
    const int tid = threadIdx.x;
    const int64_t tile = blockIdx.x;
    const int64_t item0 = tile * kTileItems;
    const bool pow2 = (m_bits & (m_bits - 1)) == 0;
    for (int slab0 = 0; slab0 < m_bits; slab0 += kBuildSlabRows) {
        const int rows = min(kBuildSlabRows, m_bits - slab0);
        for (int i = tid; i < rows * 8; i += kBuildThreads) reinterpret_cast<int4*>(s_bits)[i] = make_int4(0, 0, 0, 0);
        __syncthreads();
        for (int it = tid; it < kTileItems; it += kBuildThreads) {
            const int64_t item = item0 + it;
            if (item >= n_items) break;
            const int64_t f_end = feat_offsets[item + 1];
            const uint32_t bit = 1u << (it & 31);
            for (int64_t e = feat_offsets[item]; e < f_end; ++e) {
                const uint64_t f = feat_ids[e];
                for (int j = 0; j < k_hashes; ++j) {
                    const uint64_t h = splitmix64(f ^ (uint64_t)j);
                    const int r = (int)(pow2 ? (h & (uint64_t)(m_bits - 1)) : (h % (uint64_t)m_bits)) - slab0;
                    if (r >= 0 && r < rows) atomicOr(&s_bits[r * 32 + (it >> 5)], bit);
                }
            }
        }
        __syncthreads();
        int4* dst = reinterpret_cast<int4*>(bloom + (tile * (int64_t)m_bits + slab0) * kTileWords);
        for (int i = tid; i < rows * 8; i += kBuildThreads) dst[i] = reinterpret_cast<const int4*>(s_bits)[i];
        __syncthreads();
    }
}

// Item-major signatures for parity checks: out[item][word j] gathers bit `row` from 64 rows.
__global__ __launch_bounds__(256) void bloom_export_kernel(const uint64_t* __restrict__ bloom,
                                                           int64_t n_items, int32_t m_bits,
                                                           uint64_t* __restrict__ out)
{
    const int64_t item = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (item >= n_items) return;
    const int64_t tile = item >> 10;
    const int w = (int)((item & 1023) >> 6);
    const int bit = (int)(item & 63);
    const uint64_t* base = bloom + (tile * (int64_t)m_bits) * kTileWords + w;
    const int n_slabs = (m_bits + 63) >> 6;
    for (int slab = 0; slab < n_slabs; ++slab) {
        uint64_t sig = 0;
        for (int b = 0; b < 64; ++b) {
            const int row = slab * 64 + b;
            if (row < m_bits) sig |= ((base[(int64_t)row * kTileWords] >> bit) & 1ULL) << b;
        }
        out[item * n_slabs + slab] = sig;
    }
}

// Mask word of one filter: AND of the rows its signature sets, limited to real items.
__device__ inline uint64_t bloom_mask_word(const uint64_t* __restrict__ bloom, int32_t m_bits,
                                           int64_t gw, int64_t n_items,
                                           const int32_t* __restrict__ rows, int n_rows)
{
    const int64_t first = gw * 64;
    if (first >= n_items) return 0;
    const int64_t left = n_items - first;
    uint64_t mask = left >= 64 ? ~0ULL : ((1ULL << left) - 1ULL);
    const uint64_t* base = bloom + ((gw >> 4) * (int64_t)m_bits) * kTileWords + (gw & 15);
    // four independent loads at a time, so that their latencies overlap
    int r = 0;
    for (; r + 4 <= n_rows; r += 4) {
        const uint64_t a = base[(int64_t)rows[r] * kTileWords], b = base[(int64_t)rows[r + 1] * kTileWords];
        const uint64_t c = base[(int64_t)rows[r + 2] * kTileWords], e = base[(int64_t)rows[r + 3] * kTileWords];
        mask &= (a & b) & (c & e);
    }
    for (; r < n_rows; ++r) mask &= base[(int64_t)rows[r] * kTileWords];
    return mask;
}

// dev_mask[f][w] for every filter f and word w (Eq. 4, 64 items per AND).
__global__ __launch_bounds__(256) void bloom_mask_kernel(const uint64_t* __restrict__ bloom,
                                                         int32_t m_bits, int64_t n_items,
                                                         int64_t n_words,
                                                         const int32_t* __restrict__ row_off,
                                                         const int32_t* __restrict__ rows,
                                                         int32_t n_filters,
                                                         uint64_t* __restrict__ out)
{
    const int64_t gw = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int f = blockIdx.y;
    if (gw >= n_words || f >= n_filters) return;
    const int r0 = row_off[f], r1 = row_off[f + 1];
    out[(int64_t)f * n_words + gw] = bloom_mask_word(bloom, m_bits, gw, n_items, rows + r0, r1 - r0);
}

// Boolean filter expressions over per-feature Bloom results (Sec. 4: a query is a conjunction of
// OR-groups of feature = value terms, possibly negated; Sec. 4.3: the per-feature results and the
// operators sit in an operation array that is run in order on a stack).  One thread per 64-item
// word and expression: a leaf pushes the AND of the k signature rows of its feature, NOT / AND /
// OR work on the top of the stack, which lives in LDS (one column per thread, so the dynamic
// depth costs no register indexing).  The host has checked every program: depth <= kExprDepth,
// no pop from an empty stack, one result left.
//   code[i]       operator of entry i (0 leaf, 1 and, 2 or, 3 not)
//   leaf_rows     k_hashes rows per entry (read for leaves only), entry-major
//   prog_off      [n_exprs + 1] entries of each expression; an empty one passes every item
//   out_tile_rows > 0: the result becomes row e of a bit-sliced index of that many rows in the
//                 layout above (the scan kernels read it like a Bloom index whose "signature bit"
//                 e is the whole expression); 0: plain [n_exprs][n_words] masks (Sec. 4.3: 1 bit
//                 per item)
constexpr int kExprDepth = 16;
constexpr int kExprOps = 256;    // entries of one program, at most
constexpr int kExprHashes = 16;  // rows of a leaf, at most

// One program on one 64-item word: s_code / s_rows hold the program (LDS), base points at word w
// of row 0 of the word's tile, column tid of s_stack (NT columns, one per thread) is this thread's stack.  Returns the raw
// result (all ones for the empty program); the caller masks the bits that are not items.
template <int NT>
__device__ inline uint64_t expr_eval_word(const int32_t* s_code, const int32_t* s_rows, int n_ops, int k_hashes,
                                          const uint64_t* __restrict__ base, uint64_t (*s_stack)[NT], int tid)
{
    int top = 0;
    for (int i = 0; i < n_ops; ++i) {
        const int op = s_code[i];
        if (op == 0) {
            // four rows at a time, so that their latencies overlap (a short leaf repeats its last row)
            uint64_t w = ~0ULL;
            const int32_t* rows = s_rows + i * k_hashes;
            for (int j = 0; j < k_hashes; j += 4) {
                const int j1 = j + 1 < k_hashes ? j + 1 : k_hashes - 1, j2 = j + 2 < k_hashes ? j + 2 : k_hashes - 1,
                          j3 = j + 3 < k_hashes ? j + 3 : k_hashes - 1;
                const uint64_t a = base[(int64_t)rows[j] * kTileWords], b = base[(int64_t)rows[j1] * kTileWords];
                const uint64_t c = base[(int64_t)rows[j2] * kTileWords], e = base[(int64_t)rows[j3] * kTileWords];
                w &= (a & b) & (c & e);
            }
            s_stack[top++][tid] = w;
        } else if (op == 3) {
            s_stack[top - 1][tid] = ~s_stack[top - 1][tid];
        } else {
            const uint64_t rhs = s_stack[--top][tid];
            const uint64_t lhs = s_stack[top - 1][tid];
            s_stack[top - 1][tid] = op == 1 ? (lhs & rhs) : (lhs | rhs);
        }
    }
    return n_ops > 0 ? s_stack[0][tid] : ~0ULL;
}

__global__ __launch_bounds__(256) void bloom_expr_kernel(const uint64_t* __restrict__ bloom, int32_t m_bits,
                                                         int32_t k_hashes, int64_t n_items, int64_t n_words,
                                                         const int32_t* __restrict__ prog_off,
                                                         const int32_t* __restrict__ code,
                                                         const int32_t* __restrict__ leaf_rows,
                                                         int32_t out_tile_rows, uint64_t* __restrict__ out)
{
    __shared__ uint64_t s_stack[kExprDepth][256];
    __shared__ int32_t s_code[kExprOps];
    __shared__ int32_t s_rows[kExprOps * kExprHashes];
    const int tid = threadIdx.x;
    const int64_t gw = (int64_t)blockIdx.x * 256 + tid;
    const int e = blockIdx.y;
    // the workgroup's program, fetched once (the tables may sit in pinned host memory: one round
    // trip for the whole workgroup instead of one per entry)
    const int i0 = prog_off[e], n_ops = prog_off[e + 1] - i0;
    for (int i = tid; i < n_ops; i += 256) s_code[i] = code[i0 + i];
    for (int i = tid; i < n_ops * k_hashes; i += 256) s_rows[i] = leaf_rows[(int64_t)i0 * k_hashes + i];
    __syncthreads();
    if (gw >= n_words) return;  // (no barrier below: a thread's stack column is its own)
    const int64_t first = gw * 64;
    const int64_t left = n_items - first;
    const uint64_t valid = left >= 64 ? ~0ULL : (left > 0 ? ((1ULL << left) - 1ULL) : 0ULL);
    const uint64_t* base = bloom + ((gw >> 4) * (int64_t)m_bits) * kTileWords + (gw & 15);
    const uint64_t raw = expr_eval_word(s_code, s_rows, n_ops, k_hashes, base, s_stack, tid);
    // bits past the last item stay 0, also under a NOT
    const uint64_t res = raw & valid;
    if (out_tile_rows > 0)
        out[((gw >> 4) * (int64_t)out_tile_rows + e) * kTileWords + (gw & 15)] = res;
    else
        out[(int64_t)e * n_words + gw] = res;
}

}  // namespace st
