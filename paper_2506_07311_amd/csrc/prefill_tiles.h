// Pieces shared by the matrix-core prefill kernels (internal header): tile geometry in LDS, the swizzle, the
// launch plan, and the tile fetch that lets the load unit write K/V rows straight into LDS.
#pragma once

#include "common.h"

namespace pa {
namespace prefill {

typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef mfma_f32x16 f32x16;

constexpr int kBM = 128;              // rows per workgroup of the 32-rows-per-wave kernel
constexpr int kBN = 64;               // keys per tile
constexpr int kThreads = 256;
constexpr int kPreciseKeys = 256;     // contexts up to this length use two-term bf16 weights
constexpr int kRow = 256;             // bytes per K or V row in LDS (unpadded, pieces swizzled)
constexpr int kTileBytes = kBN * kRow;   // K part of a tile buffer; the V part follows
constexpr int kBufBytes = 2 * kTileBytes;

// 16-byte piece L of LDS row r is stored at piece L ^ swz(r).
__device__ __forceinline__ int swz(int r) { return ((r & 3) << 2) | ((r >> 2) & 3); }
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

// ---------------------------------------------------------------------------------------------------
// Tile fetch.  Wave w issues, for i < 4, one load-to-LDS instruction for K and one for V that fill rows
// 16*i + 4*w .. +3 of the tile: lane l brings the 16-byte piece that belongs at position l%16 of row
// 16*i + 4*w + l/16.  UNIFORM (page size >= 16): the four rows of an instruction lie in one page, so the page
// id is a scalar load and the page base scalar arithmetic; page ids are fetched one tile earlier than the rows.
// ---------------------------------------------------------------------------------------------------
typedef __attribute__((address_space(3))) void lds_void;
typedef __attribute__((address_space(1))) const void glb_void;

// How the launch cuts the work: head packing and the context split.
struct PrefillPlan {
    int32_t log2_pack;    // query heads of one KV head packed into a row tile (1 << log2_pack divides the group size)
    int32_t chunk;        // context tokens per workgroup (multiple of 64 and of the page size when nsplit > 1)
    int32_t nsplit;       // chunks along the grid; > 1: partials go to part_o / part_lse for the merge kernel
    int32_t skip_small;   // 1: sequences with q_len * G <= 16 are computed by the decode kernel, not here
    float* part_o;        // [total_q, Hq, nsplit, head_dim]
    float* part_lse;      // [total_q, Hq, nsplit]
    ModArgs mods;         // mask / score hooks (used by the instantiations that have them)
};

struct PageIds {
    int32_t p0, p1, p2, p3;
};

template <bool UNIFORM>
__device__ __forceinline__ void load_ids(PageIds& p, const CacheView& cache, const int32_t* table, int32_t t0,
                                         int32_t row, int32_t last_key)
{
    const int32_t key = UNIFORM ? t0 : t0 + row;
    p.p0 = table[min(key, last_key) >> cache.log2_page];
    p.p1 = table[min(key + 16, last_key) >> cache.log2_page];
    p.p2 = table[min(key + 32, last_key) >> cache.log2_page];
    p.p3 = table[min(key + 48, last_key) >> cache.log2_page];
    if (UNIFORM) {
        p.p0 = __builtin_amdgcn_readfirstlane(p.p0);
        p.p1 = __builtin_amdgcn_readfirstlane(p.p1);
        p.p2 = __builtin_amdgcn_readfirstlane(p.p2);
        p.p3 = __builtin_amdgcn_readfirstlane(p.p3);
    }
}

// K row and V row of `key` (clamped to a live slot) in page `page` -> LDS rows at `dst` (K) and dst + kTileBytes (V).
template <bool UNIFORM>
__device__ __forceinline__ void fetch_rows(char* dst, const CacheView& cache, int32_t page, int32_t key,
                                           int32_t last_key, uint32_t lane_off)
{
    const int32_t slot = min(key, last_key) & (cache.page_size - 1);
    if (UNIFORM) {
        // scalar page base + 32-bit lane offset: the loads take the scalar-base form and a row group costs a handful
        // of 32-bit vector operations instead of 64-bit multiply-adds per lane
        int64_t page_off = (int64_t)page * cache.page_stride * 2;
        asm volatile("" : "+s"(page_off));                 // stays in scalar registers
        const uint32_t off32 = (uint32_t)slot * (uint32_t)(cache.token_stride * 2) + lane_off;
        const char* kp = reinterpret_cast<const char*>(cache.k) + page_off;
        const char* vp = reinterpret_cast<const char*>(cache.v) + page_off;
        __builtin_amdgcn_global_load_lds((glb_void*)(kp + off32), (lds_void*)dst, 16, 0, 0);
        __builtin_amdgcn_global_load_lds((glb_void*)(vp + off32), (lds_void*)(dst + kTileBytes), 16, 0, 0);
        return;
    }
    const int64_t off = ((int64_t)page * cache.page_stride + (int64_t)slot * cache.token_stride) * 2 + lane_off;
    __builtin_amdgcn_global_load_lds((glb_void*)(reinterpret_cast<const char*>(cache.k) + off), (lds_void*)dst, 16, 0, 0);
    __builtin_amdgcn_global_load_lds((glb_void*)(reinterpret_cast<const char*>(cache.v) + off),
                                     (lds_void*)(dst + kTileBytes), 16, 0, 0);
}

// dst = buffer + 4*w*kRow (this wave's first row); row = 4*w + lane/16 (this lane's row within a 16-row group).
template <bool UNIFORM>
__device__ __forceinline__ void fetch_tile(char* dst, const PageIds& p, const CacheView& cache, int32_t t0, int32_t row,
                                           int32_t last_key, uint32_t lane_off)
{
    fetch_rows<UNIFORM>(dst, cache, p.p0, t0 + row, last_key, lane_off);
    fetch_rows<UNIFORM>(dst + 16 * kRow, cache, p.p1, t0 + row + 16, last_key, lane_off);
    fetch_rows<UNIFORM>(dst + 32 * kRow, cache, p.p2, t0 + row + 32, last_key, lane_off);
    fetch_rows<UNIFORM>(dst + 48 * kRow, cache, p.p3, t0 + row + 48, last_key, lane_off);
}


// max over the two lanes that share a row (lane and lane ^ 32) without an LDS round trip
__device__ __forceinline__ float pair_max(float x)
{
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

// Online softmax keeps a REFERENCE exponent (log2 domain) that may trail the true running max; the reference is
// raised when the 16 weights a lane computes for a half tile sum to more than this (fp16 operands end at 65504).
constexpr float kWeightSumMax = 16384.f;

}  // namespace prefill
}  // namespace pa
