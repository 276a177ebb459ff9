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

// 16 bytes per lane from global memory straight into LDS (lane i lands at lds_addr + 16 i; lds_addr wave-uniform),
// written as ONE OPAQUE STATEMENT.  Issued through the compiler's builtin, a load that writes LDS is booked as an
// access that may complete out of order with LDS reads, and while one is in flight -- here: for the whole tile --
// every wait for an LDS read becomes a wait for ALL of them, which drains the operand pipeline of the matrix
// instructions (reads kept four ahead) at every step.  The compiler does not look inside this statement, so its
// LDS waits count exactly; the loads are waited for by hand (wait_tile_loads) in front of the barrier that
// publishes a tile.  Two forms: scalar 64-bit base + 32-bit lane offset, and a 64-bit lane address.
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"   // m0 is written on purpose: it carries the LDS address of the load
// lds = wave-uniform LDS byte address, lds_imm = compile-time constant added to it
__device__ __forceinline__ void load_to_lds16(uint32_t lds, int lds_imm, const char* base, uint32_t off)
{
    asm volatile("s_add_u32 m0, %0, %3\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :
                 : "s"(lds), "v"(off), "s"(base), "n"(lds_imm)
                 : "memory", "m0", "scc");
}
__device__ __forceinline__ void load_to_lds16(uint32_t lds, int lds_imm, const char* addr)
{
    asm volatile("s_add_u32 m0, %0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"
                 :
                 : "s"(lds), "v"(addr), "n"(lds_imm)
                 : "memory", "m0", "scc");
}
#pragma clang diagnostic pop
// LDS byte address of a (wave-uniform) pointer into a __shared__ array, as a scalar
__device__ __forceinline__ uint32_t lds_address(const char* p)
{
    return __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(__attribute__((address_space(3))) const char*)p);
}
// This wave's loads to LDS have landed (to be followed by the workgroup barrier).  The wait is the compiler's own
// instruction, not text: it also tells the compiler's bookkeeping that none of ITS loads is pending any more
// (otherwise the query fragments loaded in front of the tile loop would be waited for again inside the loop, with
// counts that the tile loads in flight turn into waits for the next tile).
__device__ __forceinline__ void wait_tile_loads()
{
    __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0), the other counters left alone
}

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

// K row and V row of `key` (clamped to a live slot) in page `page` -> LDS rows at lds + IMM (K) and kTileBytes further (V).
template <bool UNIFORM, int IMM>
__device__ __forceinline__ void fetch_rows(uint32_t lds, const CacheView& cache, int32_t page, int32_t key,
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
        load_to_lds16(lds, IMM, kp, off32);
        load_to_lds16(lds, IMM + kTileBytes, vp, off32);
        return;
    }
    const int64_t off = ((int64_t)page * cache.page_stride + (int64_t)slot * cache.token_stride) * 2 + lane_off;
    load_to_lds16(lds, IMM, reinterpret_cast<const char*>(cache.k) + off);
    load_to_lds16(lds, IMM + kTileBytes, reinterpret_cast<const char*>(cache.v) + off);
}

// lds = LDS address of buffer + 4*w*kRow (this wave's first row); row = 4*w + lane/16 (this lane's row within a
// 16-row group).
template <bool UNIFORM>
__device__ __forceinline__ void fetch_tile(uint32_t lds, const PageIds& p, const CacheView& cache, int32_t t0, int32_t row,
                                           int32_t last_key, uint32_t lane_off)
{
    fetch_rows<UNIFORM, 0>(lds, cache, p.p0, t0 + row, last_key, lane_off);
    fetch_rows<UNIFORM, 16 * kRow>(lds, cache, p.p1, t0 + row + 16, last_key, lane_off);
    fetch_rows<UNIFORM, 32 * kRow>(lds, cache, p.p2, t0 + row + 32, last_key, lane_off);
    fetch_rows<UNIFORM, 48 * kRow>(lds, cache, p.p3, t0 + row + 48, last_key, lane_off);
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
