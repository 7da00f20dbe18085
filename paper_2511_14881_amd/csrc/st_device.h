// Device-side helpers shared by the kernels of the filtered int8 top-K library (gfx950).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace st {

constexpr int kTileItems = 1024;            // items per Bloom tile block
constexpr int kTileWords = kTileItems / 64; // 64-bit mask words per tile (one 128-byte row segment)
constexpr int kWave = 64;

// splitmix64 output function: add the golden-ratio increment, then mix (hash family of the
// Bloom index, h_j(f) = splitmix64(f ^ j) mod m; paper Sec. 4.1 leaves the family open).
__host__ __device__ inline uint64_t splitmix64(uint64_t x)
{
    uint64_t z = x + 0x9E3779B97F4A7C15ULL;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
    return z ^ (z >> 31);
}

__host__ __device__ inline uint32_t bloom_bit(uint64_t f, int j, uint32_t m)
{
    return (uint32_t)(splitmix64(f ^ (uint64_t)j) % (uint64_t)m);
}

// Sort key: larger key = better candidate.  High half is the fp32 score mapped to an
// unsigned integer that preserves order, low half is ~id so that equal scores rank the
// lower item id first.  -0.0 is folded onto +0.0 (they compare equal as floats).
__device__ inline uint32_t score_bits(float s)
{
    s = s + 0.0f;
    uint32_t u = __float_as_uint(s);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ inline float bits_score(uint32_t k)
{
    uint32_t u = (k & 0x80000000u) ? (k & 0x7FFFFFFFu) : ~k;
    return __uint_as_float(u);
}
__device__ inline uint64_t make_key(float score, uint32_t item)
{
    return ((uint64_t)score_bits(score) << 32) | (uint64_t)(0xFFFFFFFFu - item);
}
__device__ inline uint32_t key_item(uint64_t key) { return 0xFFFFFFFFu - (uint32_t)key; }
__device__ inline float key_score(uint64_t key) { return bits_score((uint32_t)(key >> 32)); }

// ((float)dot * s_q) * s_i with both products rounded separately.
__device__ inline float rescale(int dot, float s_q, float s_i)
{
    float a = __fmul_rn((float)dot, s_q);
    return __fmul_rn(a, s_i);
}

// 16 int8 x 16 int8 -> int32 accumulate (four v_dot4_i32_i8).
__device__ inline int dot16(const int4& a, const int4& b, int acc)
{
    acc = __builtin_amdgcn_sdot4(a.x, b.x, acc, false);
    acc = __builtin_amdgcn_sdot4(a.y, b.y, acc, false);
    acc = __builtin_amdgcn_sdot4(a.z, b.z, acc, false);
    acc = __builtin_amdgcn_sdot4(a.w, b.w, acc, false);
    return acc;
}

// int8 dot product of two d-byte rows, d % 16 == 0, both 16-byte aligned.
__device__ inline int dot_rows(const int8_t* a, const int8_t* b, int d)
{
    const int4* pa = reinterpret_cast<const int4*>(a);
    const int4* pb = reinterpret_cast<const int4*>(b);
    int acc = 0;
    for (int c = 0; c < (d >> 4); ++c) acc = dot16(pa[c], pb[c], acc);
    return acc;
}

// Lanes of the wavefront for which the predicate holds (the compiler folds the comparison that
// produced the predicate into this, which it does not do for the int-taking __ballot).
__device__ inline uint64_t ballot(bool pred) { return __builtin_amdgcn_ballot_w64(pred); }

__device__ inline int lane_id() { return (int)(threadIdx.x & 63); }

// ---- cross-lane steps with data-parallel register moves.  A shuffle (__shfl*) goes through the
// LDS pipe and a chain of six dependent ones costs well over a thousand cycles; a move that reads
// another lane's register directly costs a few.  The hardware offers them inside rows of 16 lanes
// (shift right by n: lane l reads lane l - n) and as broadcasts of a row's last lane into the rows
// after it, which is all a scan or a reduction over the wavefront needs.

// Value of lane l - N for the lanes whose source lies in their own row of 16; 0 for the others.
template <int N>
__device__ inline uint32_t row_shr(uint32_t v)
{
    static_assert(N >= 1 && N <= 15, "shift within a row of 16 lanes");
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x110 + N, 0xF, 0xF, false);
}
// Lane 15 of rows 0 and 2 into every lane of rows 1 and 3 (0 elsewhere); lane 31 into rows 2 and 3.
__device__ inline uint32_t row_bcast15(uint32_t v) { return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x142, 0xA, 0xF, false); }
__device__ inline uint32_t row_bcast31(uint32_t v) { return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x143, 0xC, 0xF, false); }

// Inclusive prefix sum over the wavefront (lane l: sum of lanes 0 .. l).
__device__ inline uint32_t wave_scan_add(uint32_t v)
{
    v += row_shr<1>(v);
    v += row_shr<2>(v);
    v += row_shr<4>(v);
    v += row_shr<8>(v);
    v += row_bcast15(v);
    v += row_bcast31(v);
    return v;
}
// Maximum over the wavefront, delivered in lane 63 (overlapping windows do no harm to a maximum;
// lanes without a source take 0).
__device__ inline uint32_t wave_max_u32(uint32_t v)
{
    uint32_t o;
    o = row_shr<1>(v); v = o > v ? o : v;
    o = row_shr<2>(v); v = o > v ? o : v;
    o = row_shr<4>(v); v = o > v ? o : v;
    o = row_shr<8>(v); v = o > v ? o : v;
    o = row_bcast15(v); v = o > v ? o : v;
    o = row_bcast31(v); v = o > v ? o : v;
    return v;
}
// Maximum of a 64-bit value over the wavefront, delivered in lane 63.
__device__ inline uint64_t wave_max_u64(uint64_t v)
{
#define ST_MAX64_STEP(MOVE)                                                      \
    {                                                                            \
        const uint64_t o = ((uint64_t)MOVE((uint32_t)(v >> 32)) << 32) | MOVE((uint32_t)v); \
        v = o > v ? o : v;                                                       \
    }
    ST_MAX64_STEP(row_shr<1>)
    ST_MAX64_STEP(row_shr<2>)
    ST_MAX64_STEP(row_shr<4>)
    ST_MAX64_STEP(row_shr<8>)
    ST_MAX64_STEP(row_bcast15)
    ST_MAX64_STEP(row_bcast31)
#undef ST_MAX64_STEP
    return v;
}
// Bitwise OR over the wavefront, delivered in lane 63.
__device__ inline uint32_t wave_or_u32(uint32_t v)
{
    v |= row_shr<1>(v);
    v |= row_shr<2>(v);
    v |= row_shr<4>(v);
    v |= row_shr<8>(v);
    v |= row_bcast15(v);
    v |= row_bcast31(v);
    return v;
}
// A value of lane `src` (the same in every lane) for all lanes.
__device__ inline uint32_t lane_value(uint32_t v, int src) { return (uint32_t)__builtin_amdgcn_readlane((int)v, src); }

}  // namespace st
