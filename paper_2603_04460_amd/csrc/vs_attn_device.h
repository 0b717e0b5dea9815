// Device code shared by the two attention kernels of libvsprefill (sparse vertical-slash and dense causal):
// MFMA fragment types, the LDS tile layout that both stage K / V with, the launch parameters and the
// mask / staging primitives.
#pragma once
#include <hip/hip_runtime.h>
#include <limits.h>
#include <math.h>
#include <stdint.h>

#include "vs_common.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4t __attribute__((__vector_size__(4 * sizeof(__bf16))));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kD = 128;
// A tile is staged with loads that write LDS directly: one wavefront instruction deposits its 64 16-byte pieces
// back to back, which makes 4 rows of 256 B a contiguous 1 KB group.  Groups are 64 B apart and the pieces are rotated
// inside a group so that fragment reads spread over all banks:
//   K (16-byte reads, 16 rows at one chunk c): chunk c of row r sits at 64 (c / 4) + 16 ((c + r) % 4) of its row
//   V (transposing reads, 4 rows x 64 B):      byte x of row r sits at 64 ((x / 64 + r) % 4) + x % 64 of its row
constexpr int kGroupBytes = 4 * 256 + 64;      // four rows and the gap to the next group
constexpr int kTileBytes = 8 * kGroupBytes;    // one 32-key tile of K or V
constexpr int kSlotBytes = 2 * kTileBytes;     // one LDS slot: a K tile, then the V tile of the same keys
constexpr int kSlots = 6;                      // ring of three stages of two tiles
constexpr uint64_t kAll63 = 0x7fffffffffffffffull;
constexpr float kRescaleThreshold = 8.0f;      // log2 units: stale maxima up to 2^8 are tolerated

struct AttnParams {
    const uint16_t* q;
    const uint16_t* k;
    const uint16_t* v;
    uint16_t* o;
    float* lse;
    int q_heads, kv_heads, group, hc, n, tiles, index_per_q;   // n: keys per head
    int nq, pos0;                   // query rows per head; row r is position pos0 + r (pos0 + nq <= n)
    int gran;                       // slash granularity: 1 (element-exact) or 32 (per 32-row block)
    float scale, c;                 // c = scale * log2(e)
    const int32_t* idx_v;
    const int32_t* cnt_v;
    int cap_v;
    // prepared once per call from the index lists (one set per index head):
    const uint32_t* vbit;           // bit j set iff column j selected
    int vw;                         // words per head of vbit
    const int32_t* dlist;           // block diagonals, ascending: delta is listed iff a selected offset crosses key block
                                    // (first row block of the tile - delta) for some 32-row block of a query tile
    const unsigned long long* wlist;  // per listed diagonal and 32-row block r < 4: selected offsets 32 (delta + r) - 31 ..
                                    // 32 (delta + r) + 31 at bits 0..62
    int dcap;                       // entries per head of dlist (wlist: 4 dcap)
    const int32_t* ndiag;           // per head and 32-row block q: number of listed diagonals <= q
    const int32_t* ncol32;          // per head and 32-row block q: number of listed columns <= 32 q + 31
    int nq32;                       // entries per head of ndiag and ncol32
    const int32_t* vfirst;          // per head: position of the first non-negative entry of the column list
    unsigned long long* tile_counter;
    unsigned int* work_counter;     // persistent launch: next unit of every KV head's queue (zero at launch); null: one unit per workgroup
    int work_total;                 // units of work (query tiles x KV heads x head chunks)
};

__device__ __forceinline__ float half_swap_max(float x) {
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

__device__ __forceinline__ float half_swap_sum(float x) {
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ uint64_t uniform64(uint64_t x) {
    const uint32_t lo = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(x));
    const uint32_t hi = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(x >> 32));
    return (static_cast<uint64_t>(hi) << 32) | lo;
}

// Keep-bits of one lane of a 32x32 S^T tile.  Lane (q, h) holds, in accumulator element E = 4a + c, key kj = 8a + 4h + c
// of query q; the result has that element's keep-bit at position 27 - 8a - c.
// w: selected offsets dlt-31 .. dlt+31 at bits 0..62 (key kj of row q is offset bit 31 + q - kj); cz: the causal ones
// among them; fw: keys kept for every causal row of the block; xw: keys dropped for every row.
// sh = q + 4 - 4h and ysh = 4 - 4h are per-lane constants.
__device__ __forceinline__ uint32_t lane_keep_bits(uint64_t w, uint64_t cz, uint32_t fw, uint32_t xw, int sh, int ysh) {
    const uint32_t x = static_cast<uint32_t>(w >> sh), cx = static_cast<uint32_t>(cz >> sh);
    const uint32_t yf = __builtin_bitreverse32(fw) >> ysh;  // bit 27 - 8a - c = key 8a + 4h + c
    const uint32_t yx = __builtin_bitreverse32(xw) >> ysh;
    return (x | (yf & cx)) & ~yx;
}

// Four elements (one group a) at a time: the keep-bits spread over a word each (written out: from the C form the compiler
// makes and + compare + select), then a bitwise select that stays visible to the compiler, which must space it from the
// matrix instruction that produced acc.
template <int A>
__device__ __forceinline__ void mask_elements(f32x16& acc, uint32_t keep, uint32_t dead_bits) {
    uint32_t m0, m1, m2, m3;
    asm("v_bfe_i32 %0, %4, %5, 1\n\tv_bfe_i32 %1, %4, %6, 1\n\tv_bfe_i32 %2, %4, %7, 1\n\tv_bfe_i32 %3, %4, %8, 1"
        : "=&v"(m0), "=&v"(m1), "=&v"(m2), "=&v"(m3)
        : "v"(keep), "n"(27 - 8 * A), "n"(26 - 8 * A), "n"(25 - 8 * A), "n"(24 - 8 * A));
    acc[4 * A] = __uint_as_float((m0 & __float_as_uint(acc[4 * A])) | (~m0 & dead_bits));
    acc[4 * A + 1] = __uint_as_float((m1 & __float_as_uint(acc[4 * A + 1])) | (~m1 & dead_bits));
    acc[4 * A + 2] = __uint_as_float((m2 & __float_as_uint(acc[4 * A + 2])) | (~m2 & dead_bits));
    acc[4 * A + 3] = __uint_as_float((m3 & __float_as_uint(acc[4 * A + 3])) | (~m3 & dead_bits));
    if constexpr (A + 1 < 4) mask_elements<A + 1>(acc, keep, dead_bits);
}

// 16 bytes per lane from global memory straight into LDS: lane L's piece lands at lds_base + 16 L (lds_base is
// wave-uniform).  Written as an instruction rather than through the builtin: the compiler orders every later LDS read
// behind a builtin load it cannot tell apart (a full vmcnt wait in the middle of the pipeline); here the kernel itself
// waits (vmcnt) before the barrier that publishes a stage.
__device__ __forceinline__ void lds_load16(const void* gsrc, const void* lds_base) {
    const uint32_t base = static_cast<uint32_t>(reinterpret_cast<uintptr_t>(
        (const __attribute__((address_space(3))) void*)lds_base));
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" : : "s"(base), "v"(gsrc) : "memory", "m0");
}

// the same with a wave-uniform base pointer and a 32-bit per-lane byte offset: no address arithmetic per lane
__device__ __forceinline__ void lds_load16s(uint32_t voff, const void* sbase, const void* lds_base) {
    const uint32_t base = static_cast<uint32_t>(reinterpret_cast<uintptr_t>(
        (const __attribute__((address_space(3))) void*)lds_base));
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" : : "s"(base), "v"(voff), "s"(sbase) : "memory", "m0");
}

// chunk: nq query rows at positions pos0 .. pos0 + nq - 1 against n keys
int check_chunk(int64_t nq, int64_t n, int64_t pos0) {
    if (nq <= 0 || pos0 < 0 || pos0 + nq > n) return VS_ERR_INVALID_ARG;
    return VS_OK;
}

int check_qkv(const void* q, const void* k, const void* v, int q_heads, int kv_heads, int64_t n, float scale, void* o) {
    if (!q || !k || !v || !o) return VS_ERR_INVALID_ARG;
    if (!vs::aligned16(q) || !vs::aligned16(k) || !vs::aligned16(v) || !vs::aligned16(o)) return VS_ERR_INVALID_ARG;
    if (q_heads <= 0 || kv_heads <= 0 || n <= 0) return VS_ERR_INVALID_ARG;
    if (!(scale > 0.f) || !isfinite(scale)) return VS_ERR_INVALID_ARG;
    if (q_heads % kv_heads != 0) return VS_ERR_UNSUPPORTED;
    if (n > VS_MAX_SEQ) return VS_ERR_UNSUPPORTED;
    return VS_OK;
}

int heads_per_workgroup(int group, bool index_per_q) {
    if (index_per_q) return 1;
    if (group % 4 == 0) return 4;
    if (group % 2 == 0) return 2;
    return 1;
}

}  // namespace
