// Distillation step of the VSIndexer (Sec. "Vertical-Slash Aggregation for Distillation Training", paragraph "Loss
// function design"): loss L = KL(A^_v || A_v) + KL(A^_s || A_s) between the indexer's two score vectors and the
// aggregated attention of the frozen model (vs_aggregate's outputs), and the gradient of L with respect to the
// indexer's parameters W_U, b_U, W_V, W_S.  The optimizer is the caller's.
//
//   1. forward: the inference kernels (vs_index_score) give A^_v, A^_s;
//   2. per (head, direction): KL = sum_t A^_t (ln A^_t - ln max(A_t, eps)) and the gradient with respect to the logits,
//      g_t = A^_t ((ln A^_t - ln A_t) - KL) / heads  (fp64 sums: this kernel is a few passes over n values);
//   3. backward through the two-layer net with the hidden activations recomputed on the matrix cores.  Here the
//      up-projection runs as U = X W_U (tokens on the M axis, hidden units on the N axis), so that a lane holds 16 TOKENS
//      of ONE hidden unit: the token sums dW_V[u] = sum_t g_v z_u, dW_S, db_U are in-lane, and the pre-activation
//      gradients, rounded to two bf16 terms, are already the B operand of the second contraction
//      dW_U^T[c, u] = sum_t X[t, c] dpre[t, u], whose A operand X^T comes from LDS through the transposing read.
//      Every workgroup owns 128 hidden units (one 32-unit slice per wavefront, W_U fragments resident in registers) and a
//      strided set of 32-token blocks; its partial sums go to the workspace and a last kernel adds them up in a fixed
//      order (no float atomics: the step is deterministic).
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include "vs_common.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4t __attribute__((__vector_size__(4 * sizeof(__bf16))));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

constexpr int kThreads = 256;
constexpr int kUnitsPerWg = 128;               // 4 wavefronts x 32 hidden units
constexpr int kTokTile = 32;
constexpr int kXPitch = 512 + 16;              // bytes per token row of the X tile in LDS (K then V, bf16)
constexpr int kKlThreads = 1024;

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f) {
    uint32_t u = __float_as_uint(f);
    u += 0x7fffu + ((u >> 16) & 1u);
    return static_cast<uint16_t>(u >> 16);
}

// W_U [256, d_h] fp32 -> hi, lo [d_h, 256] bf16 (k contiguous): w ~= hi + lo
__global__ void train_split_kernel(const float* __restrict__ W_U, int d_h, uint16_t* __restrict__ hi, uint16_t* __restrict__ lo) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= d_h * 256) return;
    const int u = i % d_h, k = i / d_h;
    const float w = W_U[static_cast<size_t>(k) * d_h + u];
    const uint16_t h = f32_to_bf16_rne(w);
    hi[static_cast<size_t>(u) * 256 + k] = h;
    lo[static_cast<size_t>(u) * 256 + k] = f32_to_bf16_rne(w - __uint_as_float(static_cast<uint32_t>(h) << 16));
}

__device__ __forceinline__ double block_sum(double x, double* red) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) x += __shfl_xor(x, d);
    __syncthreads();
    if (lane == 0) red[wave] = x;
    __syncthreads();
    double s = 0.0;
    for (int w = 0; w < kKlThreads / 64; ++w) s += red[w];
    return s;
}

// One workgroup per (head, direction): KL and the gradient with respect to the logits.
__global__ __launch_bounds__(kKlThreads) void train_kl_kernel(const float* __restrict__ p_v, const float* __restrict__ p_s,
                                                               const float* __restrict__ t_v, const float* __restrict__ t_s, int n,
                                                               int heads, float eps, float* __restrict__ g_v,
                                                               float* __restrict__ g_s, double* __restrict__ kl) {
    __shared__ double red[kKlThreads / 64];
    const int h = blockIdx.x, dir = blockIdx.y;
    const float* __restrict__ p = (dir == 0 ? p_v : p_s) + static_cast<size_t>(h) * n;
    const float* __restrict__ q = (dir == 0 ? t_v : t_s) + static_cast<size_t>(h) * n;
    float* __restrict__ g = (dir == 0 ? g_v : g_s) + static_cast<size_t>(h) * n;
    double acc = 0.0;
    for (int t = threadIdx.x; t < n; t += kKlThreads) {
        const float pt = p[t];
        if (pt > 0.f) acc += static_cast<double>(pt) * (log(static_cast<double>(pt)) - log(static_cast<double>(fmaxf(q[t], eps))));
    }
    const double total = block_sum(acc, red);
    if (threadIdx.x == 0) kl[h * 2 + dir] = total;
    const double inv_heads = 1.0 / heads;
    for (int t = threadIdx.x; t < n; t += kKlThreads) {
        const float pt = p[t];
        double gt = 0.0;
        if (pt > 0.f)
            gt = static_cast<double>(pt) * (log(static_cast<double>(pt)) - log(static_cast<double>(fmaxf(q[t], eps))) - total) * inv_heads;
        g[t] = static_cast<float>(gt);
    }
}

__global__ void train_loss_kernel(const double* __restrict__ kl, int heads, float* __restrict__ loss) {
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        double s = 0.0;
        for (int i = 0; i < 2 * heads; ++i) s += kl[i];
        *loss = static_cast<float>(s / heads);
    }
}

// erf by the rational approximation 7.1.26 of Abramowitz & Stegun (absolute error below 1.5e-7); also returns
// exp(-y^2), which the GELU slope needs
__device__ __forceinline__ float erf_exp(float y_signed, float& e_out) {
    const float y = fabsf(y_signed);
    const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f, y, 1.f));
    float poly = fmaf(1.061405429f, t, -1.453152027f);
    poly = fmaf(poly, t, 1.421413741f);
    poly = fmaf(poly, t, -0.284496736f);
    poly = fmaf(poly, t, 0.254829592f);
    poly *= t;
    const float e = __builtin_amdgcn_exp2f(-1.4426950408889634f * y * y);
    e_out = e;
    return copysignf(fmaf(-poly, e, 1.f), y_signed);
}

// activation and its derivative
template <int ACT>
__device__ __forceinline__ void act_slope(float x, float& z, float& slope) {
    if (ACT == 0) {                                         // SiLU: x s, s + x s (1 - s)
        const float s = __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(-1.4426950408889634f * x));
        z = x * s;
        slope = fmaf(z, 1.f - s, s);
    } else {                                                // GELU: x Phi(x), Phi(x) + x phi(x)
        float e;
        const float Phi = 0.5f * (1.f + erf_exp(x * 0.70710678118654752f, e));
        z = x * Phi;
        slope = fmaf(x * 0.3989422804014327f, e, Phi);      // phi(x) = exp(-x^2 / 2) / sqrt(2 pi)
    }
}

struct TrainParams {
    const uint16_t* kx;
    const uint16_t* vx;
    int heads, n, d_h;
    const uint16_t* w_hi;
    const uint16_t* w_lo;
    const float* b_U;
    const float* W_V;
    const float* W_S;
    const float* g_v;
    const float* g_s;
    float* part_wu;                 // [chunks][256][d_h]
    float* part_vec;                // [chunks][3][d_h]: dW_V, dW_S, db_U
    int chunks;
};

template <int ACT>
__global__ __launch_bounds__(kThreads) void train_backward_kernel(const TrainParams p) {
    __shared__ __align__(16) unsigned char xt[kTokTile * kXPitch];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int col = lane & 31, hh = lane >> 5;
    const int chunk = blockIdx.x;
    const int u = blockIdx.y * kUnitsPerWg + 32 * wave + col;      // this lane's hidden unit
    const bool active = 32 * wave + blockIdx.y * kUnitsPerWg < p.d_h;   // the wavefront's slice exists (d_h is a multiple of 64)
    const int n = p.n;

    // W_U fragments of this lane's unit: B operand of U = X W_U (lane = unit column, 8 consecutive features)
    bf16x8 whi[16], wlo[16];
    float bu = 0.f, wv = 0.f, ws = 0.f;
    if (active) {
#pragma unroll
        for (int kk = 0; kk < 16; ++kk) {
            const size_t src = static_cast<size_t>(u) * 256 + 16 * kk + 8 * hh;
            whi[kk] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(p.w_hi + src));
            wlo[kk] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(p.w_lo + src));
        }
        bu = p.b_U[u];
        wv = p.W_V[u];
        ws = p.W_S[u];
    }
    f32x16 dwu[8];                                          // dW_U^T tile: lane (unit, hh), element 4a+c: feature 32 cb + 8a + 4hh + c
#pragma unroll
    for (int cb = 0; cb < 8; ++cb)
#pragma unroll
        for (int e = 0; e < 16; ++e) dwu[cb][e] = 0.f;
    float s_wv = 0.f, s_ws = 0.f, s_bu = 0.f;

    const int blocks_per_head = (n + kTokTile - 1) / kTokTile;
    const long long total_blocks = static_cast<long long>(p.heads) * blocks_per_head;
    typedef __attribute__((address_space(3))) bf16x4t* lds_tr_t;
    for (long long blk = chunk; blk < total_blocks; blk += p.chunks) {
        const int head = static_cast<int>(blk / blocks_per_head);
        const int tok0 = static_cast<int>(blk % blocks_per_head) * kTokTile;
        // ---- stage the X tile (32 tokens x [K | V]) in LDS: thread t copies 64 bytes of row t / 8 ----
        __syncthreads();                                    // the previous tile is consumed
        {
            const int r = tid >> 3, piece = tid & 7;        // piece: 64 bytes = 32 features; pieces 0-3 K, 4-7 V
            const int tok = min(tok0 + r, n - 1);
            const uint16_t* src = (piece < 4 ? p.kx : p.vx) + (static_cast<size_t>(head) * n + tok) * 128 + 32 * (piece & 3);
            const uint4* s4 = reinterpret_cast<const uint4*>(src);
            uint4* d4 = reinterpret_cast<uint4*>(xt + r * kXPitch + 64 * piece);
#pragma unroll
            for (int i = 0; i < 4; ++i) d4[i] = s4[i];
        }
        __syncthreads();
        if (!active) continue;
        // ---- pre-activations: acc[token, unit] = X W_U, lane (unit, hh) holds tokens 8a + 4hh + c ----
        f32x16 acc;
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[e] = 0.f;
#pragma unroll
        for (int kk = 0; kk < 16; ++kk) {
            // A operand: lane = token row `col`, features 16 kk + 8 hh .. + 7
            const bf16x8 xa = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(xt + col * kXPitch + 32 * kk + 16 * hh));
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xa, whi[kk], acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xa, wlo[kk], acc, 0, 0, 0);
        }
        // ---- this lane's 16 tokens: logit gradients, activation, slope ----
        bf16x8 dhi[2], dlo[2];
#pragma unroll
        for (int a = 0; a < 4; ++a) {
            const int t0 = tok0 + 8 * a + 4 * hh;
            float gv[4], gs[4];
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const bool ok = t0 + c < n;
                const size_t at = static_cast<size_t>(head) * n + min(t0 + c, n - 1);
                gv[c] = ok ? p.g_v[at] : 0.f;
                gs[c] = ok ? p.g_s[at] : 0.f;
            }
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                float z, slope;
                act_slope<ACT>(acc[4 * a + c] + bu, z, slope);
                s_wv = fmaf(gv[c], z, s_wv);
                s_ws = fmaf(gs[c], z, s_ws);
                const float dpre = fmaf(gv[c], wv, gs[c] * ws) * slope;
                s_bu += dpre;
                const uint16_t hbits = f32_to_bf16_rne(dpre);
                const uint16_t lbits = f32_to_bf16_rne(dpre - __uint_as_float(static_cast<uint32_t>(hbits) << 16));
                const int e = 4 * a + c;                    // B operand of k-step e / 8, k index e % 8
                dhi[e >> 3][e & 7] = __builtin_bit_cast(__bf16, hbits);
                dlo[e >> 3][e & 7] = __builtin_bit_cast(__bf16, lbits);
            }
        }
        // ---- dW_U^T[c, u] += sum_t X[t, c] dpre[t, u]: A = X^T through the transposing read ----
        // k-step j, lane (m, hh): k index i <-> token 16 j + 8 (i / 4) + 4 hh + i % 4 (the order of the accumulator elements)
#pragma unroll
        for (int cb = 0; cb < 8; ++cb)
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                // 16 lanes read 4 token rows x 16 features: lane i addresses (row i / 4, 4 features at 4 (i % 4)) and receives
                // feature i of the 4 rows
                const int li = lane & 15, half16 = (lane >> 4) & 1;
                const unsigned char* a0 = xt + (16 * j + 4 * hh + (li >> 2)) * kXPitch + 2 * (32 * cb + 16 * half16 + 4 * (li & 3));
                const bf16x4t lo4 = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_tr_t)(a0));
                const bf16x4t hi4 = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_tr_t)(a0 + 8 * kXPitch));
                bf16x8 xa;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    xa[e] = lo4[e];
                    xa[4 + e] = hi4[e];
                }
                dwu[cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xa, dhi[j], dwu[cb], 0, 0, 0);
                dwu[cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xa, dlo[j], dwu[cb], 0, 0, 0);
            }
    }
    if (!active) return;
    // ---- partial sums of this workgroup ----
    float* const pw = p.part_wu + static_cast<size_t>(chunk) * 256 * p.d_h;
#pragma unroll
    for (int cb = 0; cb < 8; ++cb)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const int c = 32 * cb + 8 * (e >> 2) + 4 * hh + (e & 3);
            pw[static_cast<size_t>(c) * p.d_h + u] = dwu[cb][e];
        }
    auto half_sum = [](float x) -> float {
        auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
        return __uint_as_float(r[0]) + __uint_as_float(r[1]);
    };
    s_wv = half_sum(s_wv);
    s_ws = half_sum(s_ws);
    s_bu = half_sum(s_bu);
    if (hh == 0) {
        float* const pv = p.part_vec + static_cast<size_t>(chunk) * 3 * p.d_h;
        pv[u] = s_wv;
        pv[p.d_h + u] = s_ws;
        pv[2 * p.d_h + u] = s_bu;
    }
}

// out[i] = sum over chunks of part[chunk * stride + i], i < count, in chunk order, fp64 accumulation
__global__ void train_reduce_kernel(const float* __restrict__ part, int chunks, size_t stride, size_t count, float* __restrict__ out) {
    const size_t i = static_cast<size_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (i >= count) return;
    double s = 0.0;
    for (int c = 0; c < chunks; ++c) s += static_cast<double>(part[static_cast<size_t>(c) * stride + i]);
    out[i] = static_cast<float>(s);
}

struct TrainWs {
    size_t fwd_off, fwd_bytes, pv_off, ps_off, gv_off, gs_off, kl_off, hi_off, lo_off, pwu_off, pvec_off, total;
    int chunks;
};

bool dh_ok(int d_h) { return d_h >= 64 && d_h <= 1024 && d_h % 64 == 0; }

TrainWs train_ws_layout(int kv_heads, int64_t n, int d_h) {
    TrainWs w;
    const size_t rows = static_cast<size_t>(kv_heads) * n;
    const long long blocks = static_cast<long long>(kv_heads) * ((n + kTokTile - 1) / kTokTile);
    w.chunks = static_cast<int>(blocks < 256 ? blocks : 256);
    w.fwd_off = 0;
    w.fwd_bytes = vs::round_up(vs_index_score_workspace(kv_heads, n, d_h), 256);
    w.pv_off = w.fwd_off + w.fwd_bytes;
    w.ps_off = w.pv_off + vs::round_up(rows * 4, 256);
    w.gv_off = w.ps_off + vs::round_up(rows * 4, 256);
    w.gs_off = w.gv_off + vs::round_up(rows * 4, 256);
    w.kl_off = w.gs_off + vs::round_up(rows * 4, 256);
    w.hi_off = w.kl_off + vs::round_up(static_cast<size_t>(kv_heads) * 2 * 8, 256);
    w.lo_off = w.hi_off + vs::round_up(static_cast<size_t>(d_h) * 256 * 2, 256);
    w.pwu_off = w.lo_off + vs::round_up(static_cast<size_t>(d_h) * 256 * 2, 256);
    w.pvec_off = w.pwu_off + vs::round_up(static_cast<size_t>(w.chunks) * 256 * d_h * 4, 256);
    w.total = w.pvec_off + vs::round_up(static_cast<size_t>(w.chunks) * 3 * d_h * 4, 256);
    return w;
}

}  // namespace

extern "C" {

size_t vs_index_train_workspace(int kv_heads, int64_t n, int d_h) {
    if (kv_heads <= 0 || n <= 0 || n > VS_MAX_SEQ || !dh_ok(d_h)) return 0;
    return train_ws_layout(kv_heads, n, d_h).total;
}

int vs_index_train_step(const void* k_bf16, const void* v_bf16, int kv_heads, int64_t n, const vs_indexer_t* w, const float* t_v,
                        const float* t_s, float eps, float* loss, float* dW_U, float* db_U, float* dW_V, float* dW_S, void* ws,
                        size_t ws_bytes, void* stream) {
    if (!k_bf16 || !v_bf16 || !w || !t_v || !t_s || !loss || !dW_U || !db_U || !dW_V || !dW_S) return VS_ERR_INVALID_ARG;
    if (!w->W_U || !w->b_U || !w->W_V || !w->W_S) return VS_ERR_INVALID_ARG;
    if (!vs::aligned16(k_bf16) || !vs::aligned16(v_bf16)) return VS_ERR_INVALID_ARG;
    if (kv_heads <= 0 || n <= 0 || !(eps > 0.f)) return VS_ERR_INVALID_ARG;
    if (w->act != 0 && w->act != 1) return VS_ERR_INVALID_ARG;
    if (!dh_ok(w->d_h) || n > VS_MAX_SEQ || kv_heads > 65535) return VS_ERR_UNSUPPORTED;
    const TrainWs lay = train_ws_layout(kv_heads, n, w->d_h);
    if (!ws || ws_bytes < lay.total) return VS_ERR_WORKSPACE;
    if (!vs::aligned16(ws)) return VS_ERR_INVALID_ARG;
    hipStream_t st = static_cast<hipStream_t>(stream);
    unsigned char* base = static_cast<unsigned char*>(ws);
    float* p_v = reinterpret_cast<float*>(base + lay.pv_off);
    float* p_s = reinterpret_cast<float*>(base + lay.ps_off);
    float* g_v = reinterpret_cast<float*>(base + lay.gv_off);
    float* g_s = reinterpret_cast<float*>(base + lay.gs_off);
    double* kl = reinterpret_cast<double*>(base + lay.kl_off);
    uint16_t* hi = reinterpret_cast<uint16_t*>(base + lay.hi_off);
    uint16_t* lo = reinterpret_cast<uint16_t*>(base + lay.lo_off);

    // 1. forward (the inference kernels)
    int rc = vs_index_score(k_bf16, v_bf16, kv_heads, n, w, p_v, p_s, base + lay.fwd_off, lay.fwd_bytes, stream);
    if (rc != VS_OK) return rc;
    // 2. loss and logit gradients
    hipLaunchKernelGGL(train_kl_kernel, dim3(kv_heads, 2), dim3(kKlThreads), 0, st, p_v, p_s, t_v, t_s, static_cast<int>(n), kv_heads,
                       eps, g_v, g_s, kl);
    VS_LAUNCH_CHECK();
    hipLaunchKernelGGL(train_loss_kernel, dim3(1), dim3(64), 0, st, kl, kv_heads, loss);
    VS_LAUNCH_CHECK();
    // 3. backward
    hipLaunchKernelGGL(train_split_kernel, dim3((w->d_h * 256 + 255) / 256), dim3(256), 0, st, w->W_U, w->d_h, hi, lo);
    VS_LAUNCH_CHECK();
    TrainParams p{};
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
    p.g_v = g_v;
    p.g_s = g_s;
    p.part_wu = reinterpret_cast<float*>(base + lay.pwu_off);
    p.part_vec = reinterpret_cast<float*>(base + lay.pvec_off);
    p.chunks = lay.chunks;
    const dim3 grid(lay.chunks, (w->d_h + kUnitsPerWg - 1) / kUnitsPerWg);
    if (w->act == 0) hipLaunchKernelGGL(train_backward_kernel<0>, grid, dim3(kThreads), 0, st, p);
    else hipLaunchKernelGGL(train_backward_kernel<1>, grid, dim3(kThreads), 0, st, p);
    VS_LAUNCH_CHECK();
    const size_t nwu = static_cast<size_t>(256) * w->d_h;
    hipLaunchKernelGGL(train_reduce_kernel, dim3(static_cast<unsigned>((nwu + 255) / 256)), dim3(256), 0, st, p.part_wu, lay.chunks, nwu,
                       nwu, dW_U);
    VS_LAUNCH_CHECK();
    float* const outs[3] = {dW_V, dW_S, db_U};              // the order of a partial's three vectors
    const size_t dh = static_cast<size_t>(w->d_h);
    for (int i = 0; i < 3; ++i) {
        hipLaunchKernelGGL(train_reduce_kernel, dim3(static_cast<unsigned>((dh + 255) / 256)), dim3(256), 0, st, p.part_vec + i * dh,
                           lay.chunks, 3 * dh, dh, outs[i]);
        VS_LAUNCH_CHECK();
    }
    return VS_OK;
}

}  // extern "C"
