// VSIndexer forward (Sec. "VSIndexer Design": X = concat(K, V), Z = act(X W_U + b_U),
// A_v = softmax(Z W_V + b_V), A_s = softmax(Z W_S + b_S), softmax over the n positions).
//
// The up-projection is the only dense contraction (n x 256 x d_h per head) and runs on the matrix
// cores as U^T = W_U^T X^T with v_mfma_f32_32x32x16_bf16.  X is bf16 already; the fp32 W_U is split
// once into two bf16 terms (hi + lo, 16 significant bits together) so that the product keeps fp32
// class accuracy with two MFMA passes.  With hidden units on the M axis a lane holds 16 hidden
// units of ONE token, so activation and both down-projections finish in registers and X is read
// from HBM exactly once; no Z tensor exists.  Logits go to the output arrays and a second kernel
// normalises them in place.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include "vs_common.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kThreads = 256;
constexpr int kTokensPerWg = 256;          // 4 wavefronts x 2 blocks of 32 tokens
constexpr int kChunkU = 64;                // hidden units staged in LDS at a time
constexpr int kWRowBytes = 512 + 32;       // 256 bf16 + pad (conflict-free 16-byte fragment reads)
constexpr int kMaxDh = 1024;
constexpr size_t kSmemBytes = 2 * kChunkU * kWRowBytes + 3 * kMaxDh * 4;

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

__device__ __forceinline__ float half_swap_sum(float x) {
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// erf by the rational approximation 7.1.26 of Abramowitz & Stegun, erf(y) = 1 - (a1 t + ... + a5 t^5) exp(-y^2),
// t = 1 / (1 + p y), y >= 0, absolute error below 1.5e-7: far inside the 1e-3 relative bar of the scores (the GELU
// output inherits at most 0.5 |x| * 1.5e-7) and about half the instructions of the library erff.
__device__ __forceinline__ float erf_as(float x) {
    const float y = fabsf(x);
    const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f, y, 1.f));
    float poly = fmaf(1.061405429f, t, -1.453152027f);
    poly = fmaf(poly, t, 1.421413741f);
    poly = fmaf(poly, t, -0.284496736f);
    poly = fmaf(poly, t, 0.254829592f);
    poly *= t;
    const float e = __builtin_amdgcn_exp2f(-1.4426950408889634f * y * y);
    return copysignf(fmaf(-poly, e, 1.f), x);
}

template <int ACT>
__device__ __forceinline__ float activate(float x) {
    if (ACT == 0) return x * __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(-1.4426950408889634f * x));
    return 0.5f * x * (1.f + erf_as(x * 0.70710678118654752f));
}

template <int ACT>
__global__ __launch_bounds__(kThreads) void indexer_logits_kernel(const uint16_t* __restrict__ kx, const uint16_t* __restrict__ vx,
                                                                  int n, int d_h, const uint16_t* __restrict__ w_hi,
                                                                  const uint16_t* __restrict__ w_lo, const float* __restrict__ b_U,
                                                                  const float* __restrict__ W_V, const float* __restrict__ W_S,
                                                                  float b_V, float b_S, float* __restrict__ logit_v,
                                                                  float* __restrict__ logit_s, float2* __restrict__ part,
                                                                  int nblk) {
    extern __shared__ __align__(16) unsigned char smem[];
    unsigned char* const whi = smem;
    unsigned char* const wlo = smem + kChunkU * kWRowBytes;
    float* const sbU = reinterpret_cast<float*>(smem + 2 * kChunkU * kWRowBytes);
    float* const sWV = sbU + d_h;
    float* const sWS = sWV + d_h;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int col = lane & 31, hh = lane >> 5;
    const int g = blockIdx.y;
    float* const red = reinterpret_cast<float*>(smem);     // 4 wavefronts x (max_v, sum_v, max_s, sum_s); over the weight chunk, after its last use

    for (int u = tid; u < d_h; u += kThreads) {
        sbU[u] = b_U[u];
        sWV[u] = W_V[u];
        sWS[u] = W_S[u];
    }
    const int blk = blockIdx.x;
    const int tok0 = blk * kTokensPerWg + 64 * wave;

    // X^T fragments: lane holds token col, features 16 kk + 8 hh .. + 7 (kk < 8: K, kk >= 8: V)
    bf16x8 xf[2][16];
#pragma unroll
    for (int tb = 0; tb < 2; ++tb) {
        const int tok = tok0 + 32 * tb + col;
        const size_t row = (static_cast<size_t>(g) * n + min(tok, n - 1)) * 128 + 8 * hh;
#pragma unroll
        for (int kk = 0; kk < 16; ++kk) {
            uint4 raw = make_uint4(0, 0, 0, 0);
            if (tok < n) raw = *reinterpret_cast<const uint4*>((kk < 8 ? kx : vx) + row + 16 * (kk & 7));
            xf[tb][kk] = __builtin_bit_cast(bf16x8, raw);
        }
    }
    float lv[2] = {0.f, 0.f}, ls[2] = {0.f, 0.f};

    for (int u0 = 0; u0 < d_h; u0 += kChunkU) {
        __syncthreads();                                   // previous chunk fully consumed
        for (int i = tid; i < kChunkU * 32; i += kThreads) {   // 32 16-byte pieces per hidden unit
            const int r = i >> 5, c = i & 31;
            const size_t src = static_cast<size_t>(u0 + r) * 256 + c * 8;
            *reinterpret_cast<uint4*>(whi + r * kWRowBytes + c * 16) = *reinterpret_cast<const uint4*>(w_hi + src);
            *reinterpret_cast<uint4*>(wlo + r * kWRowBytes + c * 16) = *reinterpret_cast<const uint4*>(w_lo + src);
        }
        __syncthreads();
#pragma unroll
        for (int ub = 0; ub < kChunkU / 32; ++ub) {
            f32x16 acc[2];
#pragma unroll
            for (int tb = 0; tb < 2; ++tb)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[tb][e] = 0.f;
#pragma unroll
            for (int kk = 0; kk < 16; ++kk) {
                const int off = (32 * ub + col) * kWRowBytes + kk * 32 + hh * 16;
                const bf16x8 ah = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(whi + off));
                const bf16x8 al = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(wlo + off));
#pragma unroll
                for (int tb = 0; tb < 2; ++tb) {
                    acc[tb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, xf[tb][kk], acc[tb], 0, 0, 0);
                    acc[tb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al, xf[tb][kk], acc[tb], 0, 0, 0);
                }
            }
            // lane holds hidden units u0 + 32 ub + 8 a + 4 hh + c of token `col`
#pragma unroll
            for (int a = 0; a < 4; ++a) {
                const int ub0 = u0 + 32 * ub + 8 * a + 4 * hh;
                const float4 bu = *reinterpret_cast<const float4*>(sbU + ub0);
                const float4 wv = *reinterpret_cast<const float4*>(sWV + ub0);
                const float4 ws = *reinterpret_cast<const float4*>(sWS + ub0);
                const float bu_[4] = {bu.x, bu.y, bu.z, bu.w}, wv_[4] = {wv.x, wv.y, wv.z, wv.w}, ws_[4] = {ws.x, ws.y, ws.z, ws.w};
#pragma unroll
                for (int tb = 0; tb < 2; ++tb)
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        const float z = activate<ACT>(acc[tb][4 * a + c] + bu_[c]);
                        lv[tb] = fmaf(z, wv_[c], lv[tb]);
                        ls[tb] = fmaf(z, ws_[c], ls[tb]);
                    }
            }
        }
    }
    // logits out; (max, sum of exp) of the block's tokens per direction for the softmax over all positions
    float mv = -INFINITY, ms = -INFINITY, v2[2], s2[2];
#pragma unroll
    for (int tb = 0; tb < 2; ++tb) {
        v2[tb] = half_swap_sum(lv[tb]) + b_V;
        s2[tb] = half_swap_sum(ls[tb]) + b_S;
        const int tok = tok0 + 32 * tb + col;
        if (tok < n) {
            if (hh == 0) {
                logit_v[static_cast<size_t>(g) * n + tok] = v2[tb];
                logit_s[static_cast<size_t>(g) * n + tok] = s2[tb];
            }
            mv = fmaxf(mv, v2[tb]);
            ms = fmaxf(ms, s2[tb]);
        }
    }
#pragma unroll
    for (int d = 16; d >= 1; d >>= 1) {                     // both halves hold the same 32 tokens
        mv = fmaxf(mv, __shfl_xor(mv, d));
        ms = fmaxf(ms, __shfl_xor(ms, d));
    }
    float ev = 0.f, es = 0.f;
#pragma unroll
    for (int tb = 0; tb < 2; ++tb) {
        if (tok0 + 32 * tb + col < n) {
            ev += expf(v2[tb] - mv);
            es += expf(s2[tb] - ms);
        }
    }
#pragma unroll
    for (int d = 16; d >= 1; d >>= 1) {
        ev += __shfl_xor(ev, d);
        es += __shfl_xor(es, d);
    }
    __syncthreads();                                        // every wavefront is done with the weight chunk
    if (lane == 0) {
        red[4 * wave] = mv;
        red[4 * wave + 1] = ev;
        red[4 * wave + 2] = ms;
        red[4 * wave + 3] = es;
    }
    __syncthreads();
    if (tid < 2) {                                          // thread 0: vertical, thread 1: slash
        float m = -INFINITY, e = 0.f;
        for (int w = 0; w < 4; ++w) m = fmaxf(m, red[4 * w + 2 * tid]);
        for (int w = 0; w < 4; ++w) {
            const float mw = red[4 * w + 2 * tid];
            if (mw > -INFINITY) e += red[4 * w + 2 * tid + 1] * expf(mw - m);
        }
        part[(static_cast<size_t>(g) * 2 + tid) * nblk + blk] = make_float2(m, e);
    }
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
    size_t hi_off, lo_off, part_off, total;
    int nblk;
};

IndexerWs indexer_ws_layout(int kv_heads, int64_t n, int d_h) {
    IndexerWs w;
    w.hi_off = 0;
    w.lo_off = vs::round_up(static_cast<size_t>(d_h) * 256 * 2, 256);
    w.part_off = 2 * w.lo_off;
    w.nblk = static_cast<int>((n + kTokensPerWg - 1) / kTokensPerWg);
    w.total = w.part_off + vs::round_up(static_cast<size_t>(kv_heads) * 2 * w.nblk * sizeof(float2), 256);
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
    const int rc_once = once.run(nullptr, [](int) -> int {
        VS_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&indexer_logits_kernel<0>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(kSmemBytes)));
        VS_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&indexer_logits_kernel<1>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(kSmemBytes)));
        return VS_OK;
    });
    if (rc_once != VS_OK) return rc_once;
    hipLaunchKernelGGL(split_weights_kernel, dim3((w->d_h * 256 + 255) / 256), dim3(256), 0, st, w->W_U, w->d_h, hi, lo);
    VS_LAUNCH_CHECK();
    float2* part = reinterpret_cast<float2*>(static_cast<unsigned char*>(ws) + lay.part_off);
    // one workgroup per block of 256 tokens
    const dim3 grid(static_cast<unsigned>(lay.nblk), kv_heads);
    // LDS: one 64-unit chunk of both weight halves + the three per-unit vectors; two workgroups per CU up to d_h = 1024
    const size_t smem = 2 * kChunkU * kWRowBytes + 3 * static_cast<size_t>(w->d_h) * 4;
    const uint16_t* kx = static_cast<const uint16_t*>(k_bf16);
    const uint16_t* vx = static_cast<const uint16_t*>(v_bf16);
    if (w->act == 0)
        hipLaunchKernelGGL(indexer_logits_kernel<0>, grid, dim3(kThreads), smem, st, kx, vx, static_cast<int>(n), w->d_h,
                           hi, lo, w->b_U, w->W_V, w->W_S, w->b_V, w->b_S, a_v, a_s, part, lay.nblk);
    else
        hipLaunchKernelGGL(indexer_logits_kernel<1>, grid, dim3(kThreads), smem, st, kx, vx, static_cast<int>(n), w->d_h,
                           hi, lo, w->b_U, w->W_V, w->W_S, w->b_V, w->b_S, a_v, a_s, part, lay.nblk);
    VS_LAUNCH_CHECK();
    hipLaunchKernelGGL(softmax_finish_kernel, dim3(static_cast<unsigned>((n + 1023) / 1024), kv_heads, 2), dim3(256), 0, st, a_v,
                       a_s, static_cast<int>(n), part, lay.nblk);
    VS_LAUNCH_CHECK();
    return VS_OK;
}

}  // extern "C"
