// VSIndexer forward (Sec. "VSIndexer Design": X = concat(K, V), Z = act(X W_U + b_U),
// A_v = softmax(Z W_V + b_V), A_s = softmax(Z W_S + b_S), softmax over the n positions).
//
// The up-projection is the only dense contraction (n x 256 x d_h per head) and runs on the matrix
// cores as U^T = W_U^T X^T with v_mfma_f32_32x32x16_bf16.  X is bf16 already; the fp32 W_U is split
// into two bf16 terms (hi + lo, 16 significant bits together) so that the product keeps fp32 class
// accuracy with two MFMA passes.  With hidden units on the M axis a lane holds 16 hidden units of ONE
// token, so activation and both down-projections finish in registers; no Z tensor exists.
//
// Workgroups are persistent: 8 wavefronts, each keeping the W_U fragments of ITS 32 hidden units in
// registers for the whole kernel (256 units per workgroup; wider layers are split over workgroups
// and their partial logits added afterwards), while 128-token tiles of X stream through a double
// buffer in LDS, read from HBM exactly once.  Per tile every wavefront adds its units' share of the
// two logits; the shares meet in LDS and wavefronts 0 and 1 write the logits together with the tile's
// (max, sum of exp) for the softmax over all positions, which a second kernel finishes in place.
// The wavefronts of a workgroup meet at a barrier per tile and therefore run in phase: left to
// itself, every SIMD would alternate between a stretch of matrix instructions and a stretch of
// activation arithmetic.  The four 32-token blocks of a tile are software-pipelined instead: the
// matrix products of block j + 1 are interleaved, instruction by instruction, with the activation
// of block j.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include <type_traits>
#include <utility>

#include "vs_common.h"
#include "vs_wave.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kThreads = 512;
constexpr int kWaves = kThreads / 64;
constexpr int kUnitsPerWg = 32 * kWaves;   // 256
constexpr int kTokTile = 128;              // tokens per step: four MFMA column blocks of 32
constexpr int kBlocks = kTokTile / 32;
constexpr int kXPitch = 512;               // bytes per token row in LDS: K | V in bf16; 16-byte chunk c of row r sits at chunk
                                           // position c ^ (r % 16), so that 16 consecutive rows read at one chunk hit 16 bank groups
constexpr int kXBufs = 2;                  // token tiles: one being read, one in flight from HBM
constexpr int kMaxDh = 1024;
constexpr size_t kXBytes = static_cast<size_t>(kTokTile) * kXPitch;
constexpr size_t kVecOff = kXBufs * kXBytes;                            // b_U, W_V, W_S of the workgroup's units
constexpr size_t kRedOff = kVecOff + 3 * kUnitsPerWg * 4;          // two parities x wavefronts x tokens x (v, s)
constexpr size_t kSmemBytes = kRedOff + 2 * kWaves * kTokTile * 8;

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f) {
    uint32_t u = __float_as_uint(f);
    u += 0x7fffu + ((u >> 16) & 1u);
    return static_cast<uint16_t>(u >> 16);
}

// W_U [256, d_h] fp32 -> hi, lo [d_h, 256] bf16 (k contiguous): w ~= hi + lo
__global__ void split_weights_kernel(const float* __restrict__ W_U, int d_h, uint16_t* __restrict__ hi, uint16_t* __restrict__ lo) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;   // over d_h * 256, u fastest for coalesced reads
    if (i >= d_h * 256) return;
    const int u = i % d_h, k = i / d_h;
    const float w = W_U[static_cast<size_t>(k) * d_h + u];
    const uint16_t h = f32_to_bf16_rne(w);
    const float rem = w - __uint_as_float(static_cast<uint32_t>(h) << 16);
    hi[static_cast<size_t>(u) * 256 + k] = h;
    lo[static_cast<size_t>(u) * 256 + k] = f32_to_bf16_rne(rem);
}

// 16 bytes per lane from global memory straight into LDS: lane L's piece lands at lds_base + 16 L (lds_base is
// wave-uniform).  The loads complete in the background; the kernel waits (vmcnt) before the barrier that publishes a tile.
__device__ __forceinline__ void lds_load16(const void* gsrc, const void* lds_base) {
    const uint32_t base = static_cast<uint32_t>(reinterpret_cast<uintptr_t>(
        (const __attribute__((address_space(3))) void*)lds_base));
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" : : "s"(base), "v"(gsrc) : "memory", "m0");
}

__device__ __forceinline__ float half_swap_sum(float x) {
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// GELU (erf form) = x Phi(x) with the normal distribution function written as a logistic function of an odd polynomial,
// Phi(x) = 1 / (1 + exp(-x P(x^2))), P of degree 4 fitted (minimax over |x| <= 8, own fit) so that x Phi(x) is within
// 3.1e-6 of the exact value everywhere; beyond the fitted range the leading coefficient keeps the argument growing with
// the right sign, so Phi saturates at 0 / 1 as it should.  Far inside the 1e-3 relative bar of the scores (256 hidden
// units with |W| < 1 move a logit by less than 4e-4 even if every error had the same sign) and 8 vector instructions +
// 2 transcendentals, half of what a rational erf costs.  (A table of Phi in LDS with linear interpolation was measured
// slower still: its gathers conflict on the banks.)  The coefficients below carry the factor -log2(e) of the exp2.
__device__ __forceinline__ float gelu_logistic(float x) {
    constexpr float kL = -1.4426950408889634f;
    const float x2 = x * x;
    float p = fmaf(kL * 2.2394289190536126e-06f, x2, kL * -6.118309274724009e-05f);
    p = fmaf(p, x2, kL * -0.00024962059614273813f);
    p = fmaf(p, x2, kL * 0.07293742830114522f);
    p = fmaf(p, x2, kL * 1.5956563098014116f);
    return x * __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(x * p));
}

// f(integral_constant<int, 0>) ... f(integral_constant<int, N - 1>): a loop whose counter is a constant in every iteration
// by construction (an unrolling pragma is a request; when it is not honoured, register arrays indexed by the counter go
// to scratch memory)
template <int... I, typename F>
__device__ __forceinline__ void static_for_impl(std::integer_sequence<int, I...>, F&& f) {
    (f(std::integral_constant<int, I>{}), ...);
}
template <int N, typename F>
__device__ __forceinline__ void static_for(F&& f) {
    static_for_impl(std::make_integer_sequence<int, N>{}, static_cast<F&&>(f));
}

struct IndexerParams {
    const uint16_t* kx;
    const uint16_t* vx;
    int heads, n, d_h;
    const uint16_t* w_hi;
    const uint16_t* w_lo;
    const float* b_U;
    const float* W_V;
    const float* W_S;
    float b_V, b_S;
    float* out_v;                   // logits: a_v / a_s (one slice of hidden units) or the slices' partial sums
    float* out_s;
    size_t slice_stride;            // elements between the partial-logit arrays of consecutive slices (0: one slice)
    float2* part;                   // per (head, direction, 64-token block): (max, sum of exp) of its logits; null with several slices
    int tiles_per_head;             // 128-token tiles
    int parts_per_head;             // 64-token statistics blocks
    int nslices, lanes;             // slices of 256 hidden units; workgroups per slice (a multiple of 8)
};

template <int ACT>
__global__ __launch_bounds__(kThreads) void indexer_logits_kernel(const IndexerParams p) {
    extern __shared__ __align__(16) unsigned char smem[];
    float* const sbU = reinterpret_cast<float*>(smem + kVecOff);
    float* const sWV = sbU + kUnitsPerWg;
    float* const sWS = sWV + kUnitsPerWg;
    float2* const red = reinterpret_cast<float2*>(smem + kRedOff);

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int col = lane & 31, hh = lane >> 5;
    // Workgroup id -> (slice of hidden units, lane of the tile loop).  Consecutive ids go to consecutive XCDs, so the slices
    // that work on the same tiles are given ids that are multiples of 8 apart: they run on one XCD at about the same time
    // and all but the first find the tile in that XCD's L2.
    const int xcd_slot = blockIdx.x & 7, id_hi = blockIdx.x >> 3;
    const int slice = id_hi % p.nslices;
    const int tile_lane = (id_hi / p.nslices) * 8 + xcd_slot;
    const int u_base = slice * kUnitsPerWg;                 // first hidden unit of the workgroup
    const int units_here = min(kUnitsPerWg, p.d_h - u_base);
    const int nact = units_here / 32;                       // wavefronts with units (d_h is a multiple of 64)
    const bool active = wave < nact;
    const int n = p.n;

    for (int i = tid; i < kUnitsPerWg; i += kThreads) {
        const bool ok = i < units_here;
        sbU[i] = ok ? p.b_U[u_base + i] : 0.f;
        sWV[i] = ok ? p.W_V[u_base + i] : 0.f;
        sWS[i] = ok ? p.W_S[u_base + i] : 0.f;
    }
    // W_U^T fragments of this wavefront's 32 units: A operand, lane = unit row, features 16 kk + 8 hh .. + 7
    bf16x8 whi[16], wlo[16];
    if (active) {
        const size_t row = static_cast<size_t>(u_base + 32 * wave + col) * 256 + 8 * hh;
#pragma unroll
        for (int kk = 0; kk < 16; ++kk) {
            whi[kk] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(p.w_hi + row + 16 * kk));
            wlo[kk] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(p.w_lo + row + 16 * kk));
        }
    }
    float* const out_v = p.out_v + static_cast<size_t>(slice) * p.slice_stride;
    float* const out_s = p.out_s + static_cast<size_t>(slice) * p.slice_stride;

    // tiles of 64 tokens, never across heads; workgroup b takes tiles b, b + gridDim.x, ...
    const long long total_tiles = static_cast<long long>(p.heads) * p.tiles_per_head;
    // Staging: a wavefront instruction deposits 1 KB = two token rows; wavefront w moves rows 16 w .. 16 w + 15 of a tile
    // with eight instructions.  Lane L fills chunk position L % 32 of its row, i.e. it fetches that row's chunk
    // (L % 32) ^ (row % 16) (chunks 0-15: K, 16-31: V).
    const int st_pos = lane & 31;
    auto load_tile = [&](long long t, int buf) __attribute__((always_inline)) {
        const int head = static_cast<int>(t / p.tiles_per_head);
        const int tok0 = static_cast<int>(t % p.tiles_per_head) * kTokTile;
#pragma unroll
        for (int i = 0; i < kTokTile / (2 * kWaves); ++i) {
            const int row0 = (kTokTile / kWaves) * wave + 2 * i;
            const int row = row0 + hh;
            const int chunk = st_pos ^ (row & 15);
            const int tok = min(tok0 + row, n - 1);
            const uint16_t* src = (chunk < 16 ? p.kx : p.vx) + (static_cast<size_t>(head) * n + tok) * 128 + 8 * (chunk & 15);
            lds_load16(src, smem + buf * kXBytes + row0 * kXPitch);
        }
    };
    long long tile = tile_lane;
    const long long stride = p.lanes;
    if (tile < total_tiles) load_tile(tile, 0);
    __builtin_amdgcn_s_waitcnt(0x0F70);                      // the first tile (and the weight fragments) have arrived
    __syncthreads();
    const int sw16 = (col & 15) << 4;                        // byte swizzle of this lane's token rows
    int par = 0;
    for (; tile < total_tiles; tile += stride, par ^= 1) {
        const int buf = par;
        // the other buffer held the tile of the previous step: free since the barrier that ended it
        if (tile + stride < total_tiles) load_tile(tile + stride, buf ^ 1);
        const unsigned char* xt = smem + buf * kXBytes;
        if (active) {
            // Block j: tokens 32 j + col.  The accumulator starts from the bias; lane (token col, hh) holds hidden units
            // 32 wave + 8 a + 4 hh + c.  X^T fragments (B operand: lane = token column, features 16 kk + 8 hh .. + 7) come from
            // LDS a few steps ahead of the products that use them.
            //
            // fused(jn, accn, j, accc): the 32 matrix instructions of block jn, each followed by a piece of the activation
            // of block j, written out in issue order with scheduling barriers between the pieces.  A wavefront issues in
            // order and a matrix instruction waits at issue until the matrix core takes it (32 clocks apart), so vector
            // work that follows a run of matrix instructions in the program starts only when the run is through; both
            // wavefronts of a SIMD belong to this workgroup and meet at the tile's barrier, so they do not cover for each
            // other either.  (The declarative form, scheduling-group barriers, left the matrix instructions in one run.)
            // The activation of a block is cut into stages of four independent elements (one group), so that no
            // instruction waits for its predecessor; pure arithmetic is pinned with empty asm statements, or the
            // compiler moves it to its use.
            constexpr int kLook = 2;
            constexpr int kStages = 7;                       // stages of one group's activation (SiLU)
            constexpr int kGrp = 4;                          // elements per group
            constexpr int kPieces = (16 / kGrp) * kStages;
            auto fused = [&](int jn, f32x16& accn, int j, const f32x16& accc, auto mfma_tag, auto act_tag) __attribute__((always_inline)) {
                constexpr bool MFMA = decltype(mfma_tag)::value, ACTV = decltype(act_tag)::value;
                uint4 xq[kLook];
                auto xread = [&](int kk) __attribute__((always_inline)) -> uint4 {
                    return *reinterpret_cast<const uint4*>(xt + (32 * jn + col) * kXPitch + (((2 * kk + hh) << 4) ^ sw16));
                };
                if constexpr (MFMA) {
#pragma unroll
                    for (int a = 0; a < 4; ++a) {
                        const float4 bu = *reinterpret_cast<const float4*>(sbU + 32 * wave + 8 * a + 4 * hh);
                        accn[4 * a] = bu.x;
                        accn[4 * a + 1] = bu.y;
                        accn[4 * a + 2] = bu.z;
                        accn[4 * a + 3] = bu.w;
                    }
#pragma unroll
                    for (int kk = 0; kk < kLook; ++kk) xq[kk] = xread(kk);
                }
                float t[kGrp], lvp[kGrp], lsp[kGrp];
#pragma unroll
                for (int c = 0; c < kGrp; ++c) lvp[c] = lsp[c] = 0.f;
                float wv_[kGrp], ws_[kGrp];
                // piece pc: stage pc % kStages of group g = pc / kStages: accumulator elements 4 g + c, hidden units 32 wave + 8 g + 4 hh + c;
                // the two logit sums are kept per element slot c (no chain of dependent additions) and added at the end
                auto piece = [&](auto pc_tag) __attribute__((always_inline)) {
                    constexpr int pc = decltype(pc_tag)::value;
                    constexpr int g = pc / kStages, st = pc % kStages;
                    if (st == 0) {
                        const int u = 32 * wave + 8 * ((kGrp * g) >> 2) + 4 * hh + ((kGrp * g) & 3);
#pragma unroll
                        for (int c = 0; c < kGrp; ++c) {
                            wv_[c] = sWV[u + c];
                            ws_[c] = sWS[u + c];
                        }
                    }
#pragma unroll
                    for (int c = 0; c < kGrp; ++c) {
                        const float x = accc[kGrp * g + c];
                        constexpr float kL = -1.4426950408889634f;
                        // SiLU: x / (1 + 2^(-log2(e) x))
                        if (st == 0) t[c] = kL * x;
                        if (st == 1) t[c] = __builtin_amdgcn_exp2f(t[c]);
                        if (st == 2) t[c] = 1.f + t[c];
                        if (st == 3) t[c] = __builtin_amdgcn_rcpf(t[c]);
                        if (st == 4) t[c] = x * t[c];
                        if (st == 5) lvp[c] = fmaf(t[c], wv_[c], lvp[c]);
                        if (st == 6) lsp[c] = fmaf(t[c], ws_[c], lsp[c]);
                        if (st < kStages - 2) asm volatile("" : "+v"(t[c]));
                        else if (st == kStages - 2) asm volatile("" : "+v"(lvp[c]));
                        else asm volatile("" : "+v"(lsp[c]));
                    }
                };
                static_for<32>([&](auto i_tag) __attribute__((always_inline)) {
                    constexpr int i = decltype(i_tag)::value;
                    if constexpr (MFMA) {
                        constexpr int kk = i >> 1;
                        const bf16x8 xb = __builtin_bit_cast(bf16x8, xq[kk % kLook]);
                        accn = __builtin_amdgcn_mfma_f32_32x32x16_bf16((i & 1) ? wlo[kk] : whi[kk], xb, accn, 0, 0, 0);
                        if constexpr ((i & 1) && kk + kLook < 16) xq[kk % kLook] = xread(kk + kLook);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                    if constexpr (ACTV) {
                        // pieces [i kPieces / 32, (i + 1) kPieces / 32)
                        constexpr int lo = (i * kPieces) / 32, hi = ((i + 1) * kPieces) / 32;
                        static_for<hi - lo>([&](auto q_tag) __attribute__((always_inline)) {
                            piece(std::integral_constant<int, lo + decltype(q_tag)::value>{});
                        });
                        if constexpr (MFMA) __builtin_amdgcn_sched_barrier(0);
                    }
                });
                if constexpr (ACTV) {
                    // both halves of the wavefront hold the same sums afterwards and write the same value
                    float lv = 0.f, ls = 0.f;
#pragma unroll
                    for (int c = 0; c < kGrp; ++c) {
                        lv += lvp[c];
                        ls += lsp[c];
                    }
                    red[(par * kWaves + wave) * kTokTile + 32 * j + col] = make_float2(half_swap_sum(lv), half_swap_sum(ls));
                }
            };
            if constexpr (ACT == 0) {
                using T = std::true_type;
                using F = std::false_type;
                f32x16 acc[2];
                fused(0, acc[0], 0, acc[0], T{}, F{});
#pragma unroll
                for (int j = 0; j < kBlocks; ++j) {
                    if (j + 1 < kBlocks) fused(j + 1, acc[(j + 1) & 1], j, acc[j & 1], T{}, T{});
                    else fused(0, acc[0], j, acc[j & 1], F{}, T{});
                }
            } else {
                // GELU: its vector work (84 clocks per element against 59 for SiLU) outweighs the matrix work of a block, the
                // kernel runs at the vector pipe's pace either way, and the fixed order above only takes freedom from the
                // compiler (measured 5 % slower): blocks as plain code, matrix products of block j + 1 before the activation
                // of block j.
                auto mfma_block = [&](int j, f32x16& acc) __attribute__((always_inline)) {
#pragma unroll
                    for (int a = 0; a < 4; ++a) {
                        const float4 bu = *reinterpret_cast<const float4*>(sbU + 32 * wave + 8 * a + 4 * hh);
                        acc[4 * a] = bu.x;
                        acc[4 * a + 1] = bu.y;
                        acc[4 * a + 2] = bu.z;
                        acc[4 * a + 3] = bu.w;
                    }
                    constexpr int kAhead = 4;
                    uint4 xq[kAhead];
                    auto xread = [&](int kk) __attribute__((always_inline)) -> uint4 {
                        return *reinterpret_cast<const uint4*>(xt + (32 * j + col) * kXPitch + (((2 * kk + hh) << 4) ^ sw16));
                    };
#pragma unroll
                    for (int kk = 0; kk < kAhead; ++kk) xq[kk] = xread(kk);
#pragma unroll
                    for (int kk = 0; kk < 16; ++kk) {
                        const bf16x8 xb = __builtin_bit_cast(bf16x8, xq[kk % kAhead]);
                        if (kk + kAhead < 16) xq[kk % kAhead] = xread(kk + kAhead);
                        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(whi[kk], xb, acc, 0, 0, 0);
                        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wlo[kk], xb, acc, 0, 0, 0);
                    }
                };
                auto act_block = [&](int j, const f32x16& acc) __attribute__((always_inline)) {
                    float lv = 0.f, ls = 0.f;
#pragma unroll
                    for (int a = 0; a < 4; ++a) {
                        const float4 wv = *reinterpret_cast<const float4*>(sWV + 32 * wave + 8 * a + 4 * hh);
                        const float4 ws = *reinterpret_cast<const float4*>(sWS + 32 * wave + 8 * a + 4 * hh);
                        const float wv_[4] = {wv.x, wv.y, wv.z, wv.w}, ws_[4] = {ws.x, ws.y, ws.z, ws.w};
#pragma unroll
                        for (int c = 0; c < 4; ++c) {
                            const float z = gelu_logistic(acc[4 * a + c]);
                            lv = fmaf(z, wv_[c], lv);
                            ls = fmaf(z, ws_[c], ls);
                        }
                    }
                    // both halves of the wavefront hold the same sums afterwards and write the same value
                    red[(par * kWaves + wave) * kTokTile + 32 * j + col] = make_float2(half_swap_sum(lv), half_swap_sum(ls));
                };
                f32x16 acc[2];
                mfma_block(0, acc[0]);
#pragma unroll
                for (int j = 0; j < kBlocks; ++j) {
                    if (j + 1 < kBlocks) mfma_block(j + 1, acc[(j + 1) & 1]);
                    act_block(j, acc[j & 1]);
                }
            }
        }
        __builtin_amdgcn_s_waitcnt(0x0F70);                  // this wavefront's pieces of the next tile have landed
        __syncthreads();
        if (wave < kTokTile / 64) {
            // 64 tokens of the tile per wavefront: add the wavefronts' shares, write the logits, fold the softmax statistics
            const int head = static_cast<int>(tile / p.tiles_per_head);
            const int tile_in_head = static_cast<int>(tile % p.tiles_per_head);
            const int tt = 64 * wave + lane;
            const int tok = tile_in_head * kTokTile + tt;
            float v = 0.f, s2 = 0.f;
            for (int w = 0; w < nact; ++w) {
                const float2 r = red[(par * kWaves + w) * kTokTile + tt];
                v += r.x;
                s2 += r.y;
            }
            if (slice == 0) {                               // the scalar output biases enter once
                v += p.b_V;
                s2 += p.b_S;
            }
            const bool ok = tok < n;
            if (ok) {
                out_v[static_cast<size_t>(head) * n + tok] = v;
                out_s[static_cast<size_t>(head) * n + tok] = s2;
            }
            if (p.part) {
                // (this stretch delays the two wavefronts that run it, and through the tile's barrier all eight: the
                // reductions stay on the vector ALU)
                const float mv = wave_max(ok ? v : -INFINITY), ms = wave_max(ok ? s2 : -INFINITY);
                const float ev = wave_sum(ok ? expf(v - mv) : 0.f), es = wave_sum(ok ? expf(s2 - ms) : 0.f);
                const int pt = (kTokTile / 64) * tile_in_head + wave;           // statistics per 64 tokens
                if (lane == 0 && pt < p.parts_per_head) {
                    p.part[(static_cast<size_t>(head) * 2 + 0) * p.parts_per_head + pt] = make_float2(mv, ev);
                    p.part[(static_cast<size_t>(head) * 2 + 1) * p.parts_per_head + pt] = make_float2(ms, es);
                }
            }
        }
    }
}

// Several slices of hidden units: logits = sum of the slices' partial logits, written to the output arrays together with
// the (max, sum of exp) of every 64-token block.  One wavefront per block.
__global__ __launch_bounds__(64) void combine_slices_kernel(const float* __restrict__ part_v, const float* __restrict__ part_s,
                                                            size_t slice_stride, int nslices, int n, float* __restrict__ a_v,
                                                            float* __restrict__ a_s, float2* __restrict__ part, int parts_per_head) {
    const int head = blockIdx.y, tile = blockIdx.x, dir = blockIdx.z, lane = threadIdx.x;
    const int tok = tile * 64 + lane;
    const bool ok = tok < n;
    const float* src = (dir == 0 ? part_v : part_s) + static_cast<size_t>(head) * n + tok;
    float x = 0.f;
    if (ok)
        for (int s = 0; s < nslices; ++s) x += src[static_cast<size_t>(s) * slice_stride];
    if (ok) (dir == 0 ? a_v : a_s)[static_cast<size_t>(head) * n + tok] = x;
    float m = ok ? x : -INFINITY;
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) m = fmaxf(m, __shfl_xor(m, d));
    float e = ok ? expf(x - m) : 0.f;
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) e += __shfl_xor(e, d);
    if (lane == 0) part[(static_cast<size_t>(head) * 2 + dir) * parts_per_head + tile] = make_float2(m, e);
}

// Second stage of the softmax over the n positions of one (head, direction): every workgroup folds the per-block
// (max, sum) pairs into the global pair (a few hundred values, cheaper than another launch) and normalises its own
// 1024 logits in place.
__global__ __launch_bounds__(256) void softmax_finish_kernel(float* a_v, float* a_s, int n, const float2* __restrict__ part, int nblk) {
    __shared__ float red[8];
    const int g = blockIdx.y, dir = blockIdx.z;
    const float2* pp = part + (static_cast<size_t>(g) * 2 + dir) * nblk;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    float m = -INFINITY;
    for (int i = tid; i < nblk; i += 256) m = fmaxf(m, pp[i].x);
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) m = fmaxf(m, __shfl_xor(m, d));
    if (lane == 0) red[wave] = m;
    __syncthreads();
    m = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    float e = 0.f;
    for (int i = tid; i < nblk; i += 256) {
        const float2 q = pp[i];
        if (q.x > -INFINITY) e += q.y * expf(q.x - m);
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) e += __shfl_xor(e, d);
    if (lane == 0) red[4 + wave] = e;
    __syncthreads();
    const float inv = 1.f / (red[4] + red[5] + red[6] + red[7]);
    float* x = (dir == 0 ? a_v : a_s) + static_cast<size_t>(g) * n;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int i = blockIdx.x * 1024 + 256 * u + tid;
        if (i < n) x[i] = expf(x[i] - m) * inv;
    }
}

struct IndexerWs {
    size_t hi_off, lo_off, part_off, plog_off, total;
    size_t slice_stride;            // elements per slice of partial logits (one direction)
    int tiles_per_head, parts_per_head, nslices;
};

IndexerWs indexer_ws_layout(int kv_heads, int64_t n, int d_h) {
    IndexerWs w;
    w.hi_off = 0;
    w.lo_off = vs::round_up(static_cast<size_t>(d_h) * 256 * 2, 256);
    w.part_off = 2 * w.lo_off;
    w.tiles_per_head = static_cast<int>((n + kTokTile - 1) / kTokTile);
    w.parts_per_head = static_cast<int>((n + 63) / 64);
    w.nslices = (d_h + kUnitsPerWg - 1) / kUnitsPerWg;
    w.plog_off = w.part_off + vs::round_up(static_cast<size_t>(kv_heads) * 2 * w.parts_per_head * sizeof(float2), 256);
    w.slice_stride = w.nslices > 1 ? vs::round_up(static_cast<size_t>(kv_heads) * n, 64) : 0;
    w.total = w.plog_off + (w.nslices > 1 ? 2 * static_cast<size_t>(w.nslices) * w.slice_stride * 4 : 0);
    return w;
}

bool dh_supported(int d_h) { return d_h >= 64 && d_h <= kMaxDh && d_h % 64 == 0; }

}  // namespace

extern "C" {

size_t vs_index_score_workspace(int kv_heads, int64_t n, int d_h) {
    if (kv_heads <= 0 || n <= 0 || !dh_supported(d_h)) return 0;
    return indexer_ws_layout(kv_heads, n, d_h).total;
}

int vs_index_score(const void* k_bf16, const void* v_bf16, int kv_heads, int64_t n, const vs_indexer_t* w, float* a_v,
                   float* a_s, void* ws, size_t ws_bytes, void* stream) {
    if (!k_bf16 || !v_bf16 || !w || !a_v || !a_s) return VS_ERR_INVALID_ARG;
    if (!w->W_U || !w->b_U || !w->W_V || !w->W_S) return VS_ERR_INVALID_ARG;
    if (!vs::aligned16(k_bf16) || !vs::aligned16(v_bf16)) return VS_ERR_INVALID_ARG;
    if (kv_heads <= 0 || n <= 0) return VS_ERR_INVALID_ARG;
    if (w->act != 0 && w->act != 1) return VS_ERR_INVALID_ARG;
    if (!dh_supported(w->d_h) || n > VS_MAX_SEQ || kv_heads > 65535) return VS_ERR_UNSUPPORTED;
    const IndexerWs lay = indexer_ws_layout(kv_heads, n, w->d_h);
    if (!ws || ws_bytes < lay.total) return VS_ERR_WORKSPACE;
    if (!vs::aligned16(ws)) return VS_ERR_INVALID_ARG;
    hipStream_t st = static_cast<hipStream_t>(stream);
    uint16_t* hi = reinterpret_cast<uint16_t*>(static_cast<unsigned char*>(ws) + lay.hi_off);
    uint16_t* lo = reinterpret_cast<uint16_t*>(static_cast<unsigned char*>(ws) + lay.lo_off);

    static vs::PerDeviceOnce once;
    static int cus_of[vs::kMaxDevices];
    int dev = 0;
    const int rc_once = once.run(&dev, [](int d) -> int {
        VS_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&indexer_logits_kernel<0>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(kSmemBytes)));
        VS_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&indexer_logits_kernel<1>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(kSmemBytes)));
        int cus = 0;
        VS_HIP(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, d));
        cus_of[d] = cus > 0 ? cus : 256;
        return VS_OK;
    });
    if (rc_once != VS_OK) return rc_once;
    hipLaunchKernelGGL(split_weights_kernel, dim3((w->d_h * 256 + 255) / 256), dim3(256), 0, st, w->W_U, w->d_h, hi, lo);
    VS_LAUNCH_CHECK();
    unsigned char* base = static_cast<unsigned char*>(ws);
    float2* part = reinterpret_cast<float2*>(base + lay.part_off);
    IndexerParams p{};
    p.kx = static_cast<const uint16_t*>(k_bf16);
    p.vx = static_cast<const uint16_t*>(v_bf16);
    p.heads = kv_heads;
    p.n = static_cast<int>(n);
    p.d_h = w->d_h;
    p.w_hi = hi;
    p.w_lo = lo;
    p.b_U = w->b_U;
    p.W_V = w->W_V;
    p.W_S = w->W_S;
    p.b_V = w->b_V;
    p.b_S = w->b_S;
    p.tiles_per_head = lay.tiles_per_head;
    p.parts_per_head = lay.parts_per_head;
    float* plog_v = reinterpret_cast<float*>(base + lay.plog_off);
    float* plog_s = plog_v + static_cast<size_t>(lay.nslices) * lay.slice_stride;
    if (lay.nslices == 1) {
        p.out_v = a_v;
        p.out_s = a_s;
        p.slice_stride = 0;
        p.part = part;
    } else {
        p.out_v = plog_v;
        p.out_s = plog_s;
        p.slice_stride = lay.slice_stride;
        p.part = nullptr;
    }
    // persistent workgroups of 8 wavefronts, one per compute unit, shared out over the slices of 256 hidden units
    const long long total_tiles = static_cast<long long>(kv_heads) * lay.tiles_per_head;
    long long lanes = (cus_of[dev] / lay.nslices) & ~7;
    if (lanes < 8) lanes = 8;
    const long long need = (total_tiles + 7) & ~7ll;
    if (lanes > need) lanes = need;
    p.nslices = lay.nslices;
    p.lanes = static_cast<int>(lanes);
    const dim3 grid(static_cast<unsigned>(lanes * lay.nslices));
    if (w->act == 0) hipLaunchKernelGGL(indexer_logits_kernel<0>, grid, dim3(kThreads), kSmemBytes, st, p);
    else hipLaunchKernelGGL(indexer_logits_kernel<1>, grid, dim3(kThreads), kSmemBytes, st, p);
    VS_LAUNCH_CHECK();
    if (lay.nslices > 1) {
        hipLaunchKernelGGL(combine_slices_kernel, dim3(lay.parts_per_head, kv_heads, 2), dim3(64), 0, st, plog_v, plog_s,
                           lay.slice_stride, lay.nslices, static_cast<int>(n), a_v, a_s, part, lay.parts_per_head);
        VS_LAUNCH_CHECK();
    }
    hipLaunchKernelGGL(softmax_finish_kernel, dim3(static_cast<unsigned>((n + 1023) / 1024), kv_heads, 2), dim3(256), 0, st, a_v,
                       a_s, static_cast<int>(n), part, lay.parts_per_head);
    VS_LAUNCH_CHECK();
    return VS_OK;
}

}  // extern "C"
