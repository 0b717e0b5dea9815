// Vertical-slash aggregation of the dense causal attention map (Sec. "Obtaining Ground Truth" of the paper) and
// Attention Recall of a vertical-slash mask (Eq. R(S)) for gfx950.
//
// The n x n probability matrix A = softmax(Q K^T / sqrt(d)) (causal) is never stored.  Two sweeps over the score tiles:
//   1. row sweep:    lse2[i] = log2 sum_j 2^(c s_ij), c = scale * log2(e): the normaliser of every row
//   2. column sweep: A[i,j] = 2^(c s_ij - lse2[i]) is recomputed tile by tile and added to its column sum A_v[j], to its
//                    diagonal sum A_s[i-j] and, where the mask keeps (i,j), to the recall.
// Both sweeps are the same kernel with the operands exchanged.  A workgroup (8 wavefronts) keeps 256 rows of the
// RESIDENT operand in registers (32 rows per wavefront, as the B operand of v_mfma_f32_32x32x16_bf16) and streams 32-row
// tiles of the other operand through LDS (A operand).  A lane then holds the scores of ONE resident row against 16
// streamed rows, so the reduction over the streamed index is in-lane:
//   row sweep:    resident = queries, streamed = keys 0 .. diagonal  -> per-lane online max / sum over keys
//   column sweep: resident = keys,    streamed = queries diagonal .. n-1 -> per-lane sum over queries = column sum, kept
//                 in a register for the whole sweep and written once.
// Diagonal sums: element (streamed row r, resident key kq) of a tile belongs to offset o = i - j.  Inside a tile the 16
// accumulator registers of a lane are 16 different rows r of ONE key; register e is rotated by its row number across the
// 32 lanes of its half-wave (ds_bpermute), after which lane l holds, in every register, an element with kq - r = l
// (mod 32), i.e. of diagonal -l or 32 - l.  A plain sum and a sum weighted with a precomputed 0/1 "wrapped" factor
// separate the two, so a tile costs 16 lane permutes and ONE LDS float atomic per lane (63 distinct offsets), instead of
// one atomic per element.  The atomics go to a 512-entry ring in LDS indexed by o mod 512.  The offsets a workgroup can
// still touch form a window of 319 consecutive values that advances by 64 per stage, so the 64 offsets that fall out of
// the window are flushed to global memory (one float atomic each) after every stage.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include "vs_common.h"
#include "vs_device.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kD = 128;
constexpr int kThreads = 512;
constexpr int kWaves = kThreads / 64;
constexpr int kGroupRows = 32 * kWaves;        // resident rows per workgroup
constexpr int kRowBytes = 272;                 // streamed row: 256 B + 16 B pad, conflict-free for the 16-byte fragment reads
constexpr int kTileBytes = 32 * kRowBytes;
constexpr int kRingTiles = 6;                  // three stages of two tiles
constexpr int kNormOff = kRingTiles * kTileBytes;           // per streamed row of the ring: its normaliser (column sweep)
constexpr int kDiagOff = kNormOff + kRingTiles * 32 * 4;
constexpr int kDiagRing = 512;                 // residues of the offset ring
constexpr int kSmemBytes = kDiagOff + kDiagRing * 4;
constexpr uint64_t kAll63 = 0x7fffffffffffffffull;

struct SweepParams {
    const uint16_t* q;              // [q_heads, n, 128]
    const uint16_t* k;              // [kv_heads, n, 128]
    float* lse2;                    // [q_heads, n]: written by the row sweep, read by the column sweep
    float* a_v;                     // [out_heads, n], zeroed before the column sweep
    float* a_s;
    float* recall;                  // [out_heads] or null
    int q_heads, kv_heads, group, n;
    int reduce_group;               // 1: outputs are per KV head (mean over the group's query heads)
    float c;                        // scale * log2(e)
    float log2_norm;                // log2(n) (+ log2(group) when reducing): folded into the exponent
    const uint32_t* sbit;           // recall only; per index head: bit (o + 64) set iff offset o selected
    const uint32_t* vbit;           // recall only; per index head: bit j set iff column j selected
    int sw, vw, index_per_q;
};

__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ float half_swap_sum(float x) {
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// COLUMNS == false: row sweep (resident queries, streamed keys).  COLUMNS == true: column sweep.
template <bool COLUMNS, bool RECALL>
__global__ __launch_bounds__(kThreads) void vs_sweep_kernel(const SweepParams p) {
    __shared__ __align__(16) unsigned char smem[kSmemBytes];
    float* const norm_ring = reinterpret_cast<float*>(smem + kNormOff);
    float* const diag = reinterpret_cast<float*>(smem + kDiagOff);

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int qi = lane & 31, hh = lane >> 5;
    const int n = p.n;
    const float NEG_INF = -INFINITY;

    // ---- which 256 resident rows of which query head; longest sweeps first ----
    const int h = blockIdx.x % p.q_heads;
    const int ngroups = (n + kGroupRows - 1) / kGroupRows;
    const int grp = COLUMNS ? blockIdx.x / p.q_heads : ngroups - 1 - blockIdx.x / p.q_heads;
    const int g = h / p.group;
    const int r0_wg = kGroupRows * grp;
    const int my_r0 = r0_wg + 32 * wave;
    const uint16_t* __restrict__ res_base = COLUMNS ? p.k + static_cast<size_t>(g) * n * kD : p.q + static_cast<size_t>(h) * n * kD;
    const uint16_t* __restrict__ str_base = COLUMNS ? p.q + static_cast<size_t>(h) * n * kD : p.k + static_cast<size_t>(g) * n * kD;
    const float* __restrict__ lse2 = p.lse2 + static_cast<size_t>(h) * n;

    // ---- resident fragments: B operand; lane holds resident row qi, d = 16 kk + 8 hh .. +7 ----
    bf16x8 rf[8];
    {
        const uint16_t* src = res_base + static_cast<size_t>(min(my_r0 + qi, n - 1)) * kD + 8 * hh;
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) rf[kk] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(src + 16 * kk));
    }

    // ---- streamed tiles: keys 0 .. last resident row (rows), queries first resident row .. n-1 (columns) ----
    const int t_begin = COLUMNS ? r0_wg >> 5 : 0;
    const int t_end = COLUMNS ? (n + 31) >> 5 : (min(r0_wg + kGroupRows, n) + 31) >> 5;
    const int nstages = (t_end - t_begin + 1) >> 1;

    if (COLUMNS) {
        for (int s = tid; s < kDiagRing; s += kThreads) diag[s] = 0.f;
    }

    // ---- staging: thread moves 16-byte chunk (tid & 15) of row (tid >> 4) of each of the two tiles of a stage ----
    const int st_row = tid >> 4, st_chunk = tid & 15;
    u32x4 sreg[2];
    float nreg = 0.f;
    // rows past the sequence and the padding tile of an odd count read row 0: such tiles are skipped or masked, and an
    // unpredicated load keeps the number of loads in flight independent of the path
    auto load_stage = [&](int st) __attribute__((always_inline)) {
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int t = t_begin + 2 * st + u;
            int row = 32 * t + st_row;
            if (t >= t_end || row >= n) row = 0;
            sreg[u] = *reinterpret_cast<const u32x4*>(str_base + static_cast<size_t>(row) * kD + st_chunk * 8);
        }
        if (COLUMNS && tid < 64) {
            // normaliser of streamed query row: 2^(c s - lse2 - log2_norm) is the entry of A / (n * heads averaged);
            // +inf for rows that do not exist makes their entries zero
            const int t = t_begin + 2 * st + (tid >> 5);
            const int row = 32 * t + (tid & 31);
            nreg = (t < t_end && row < n) ? lse2[row] + p.log2_norm : INFINITY;
        }
    };
    auto store_stage = [&](int buf) __attribute__((always_inline)) {
#pragma unroll
        for (int u = 0; u < 2; ++u)
            *reinterpret_cast<u32x4*>(smem + (2 * buf + u) * kTileBytes + st_row * kRowBytes + st_chunk * 16) = sreg[u];
        if (COLUMNS && tid < 64) norm_ring[64 * buf + tid] = nreg;
    };
    const int a_off = qi * kRowBytes + hh * 16;              // A fragment: lane holds streamed row qi, d = 16 kk + 8 hh ..
    auto read_a = [&](int slot, bf16x8 (&af)[8]) __attribute__((always_inline)) {
        const unsigned char* at = smem + slot * kTileBytes + a_off;
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) af[kk] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(at + kk * 32));
    };

    // ---- per-lane state ----
    float m_run = NEG_INF, l_run = 0.f;                      // row sweep: running max (log2 domain) and sum of this lane's keys
    float col_sum = 0.f, rec_sum = 0.f;                      // column sweep
    // recall: the resident key of this lane is a selected column -> every causal entry of the column is kept
    const int ih = p.index_per_q ? h : g;
    uint32_t col_keep = 0u;
    const uint32_t* __restrict__ sbit = nullptr;
    if (RECALL) {
        sbit = p.sbit + static_cast<size_t>(ih) * p.sw;
        const int key = my_r0 + qi;
        if (key < n && ((p.vbit[static_cast<size_t>(ih) * p.vw + (key >> 5)] >> (key & 31)) & 1u)) col_keep = 0xffffffffu;
    }

    // diagonal sums: source lane of the rotation of register e (row 8a + 4hh + c of the tile) and its "wrapped" factor
    int rot_src[16];
    float rot_wrap[16];
    if (COLUMNS) {
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const int x = qi + 4 * hh + 8 * (e >> 2) + (e & 3);      // key this lane receives = x mod 32
            rot_src[e] = 4 * (32 * hh + (x & 31));
            rot_wrap[e] = x >= 32 ? 1.f : 0.f;                       // wrapped: diagonal 32 - qi, else -qi
        }
    }

    // One 32 x 32 tile of scores: acc element E = 4a + c of lane (qi, hh) is (streamed row 8a + 4hh + c, resident row qi).
    auto tile = [&](int t, int slot, const f32x16& acc, uint64_t win) __attribute__((always_inline)) {
        const int s0 = 32 * t;                               // first streamed row of the tile
        if (!COLUMNS) {
            // keys s0 .. s0+31 against query my_r0 + qi: causal where key <= query
            float x[16];
            const bool diag_tile = s0 + 31 > my_r0;
            const int lim = my_r0 + qi - s0 - 4 * hh;        // element (a, c) is causal iff 8a + c <= lim
            float mt = NEG_INF;
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                x[e] = acc[e] * p.c;
                if (diag_tile && 8 * (e >> 2) + (e & 3) > lim) x[e] = NEG_INF;
                mt = fmaxf(mt, x[e]);
            }
            if (mt > m_run) {
                l_run *= __builtin_amdgcn_exp2f(m_run - mt);  // m_run = -inf: l_run is 0 and stays 0
                m_run = mt;
            }
            if (m_run > NEG_INF) {
#pragma unroll
                for (int e = 0; e < 16; ++e) l_run += __builtin_amdgcn_exp2f(x[e] - m_run);
            }
        } else {
            // queries s0 .. s0+31 against key my_r0 + qi: causal where query >= key
            const float* nr = norm_ring + 32 * slot + 4 * hh;
            const bool diag_tile = s0 < my_r0 + 32;
            const int lim = my_r0 + qi - s0 - 4 * hh;        // element (a, c) is causal iff 8a + c >= lim
            uint32_t keep = 0u;
            if (RECALL) keep = static_cast<uint32_t>(win >> (31 - qi + 4 * hh)) | col_keep;   // bit 8a + c: (i, j) kept by the mask
            float psum = 0.f, rsum = 0.f, dsum = 0.f, dwrap = 0.f;
#pragma unroll
            for (int a = 0; a < 4; ++a) {
                const f32x4 nv = *reinterpret_cast<const f32x4*>(nr + 8 * a);
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    float pr = __builtin_amdgcn_exp2f(acc[4 * a + c] * p.c - nv[c]);
                    if (diag_tile && 8 * a + c < lim) pr = 0.f;
                    psum += pr;
                    if (RECALL) {                            // adds pr where the keep-bit is set: bit spread over a word, and, add
                        uint32_t m;
                        asm("v_bfe_i32 %0, %1, %2, 1" : "=v"(m) : "v"(keep), "n"(8 * a + c));
                        rsum += __uint_as_float(__float_as_uint(pr) & m);
                    }
                    const float rot = __int_as_float(__builtin_amdgcn_ds_bpermute(rot_src[4 * a + c], __float_as_int(pr)));
                    dsum += rot;
                    dwrap = fmaf(rot, rot_wrap[4 * a + c], dwrap);
                }
            }
            col_sum += psum;
            rec_sum += rsum;
            // both halves hold rows of the same two diagonals; lanes 0..31 then add diagonal -qi, lanes 32..63 add 32 - qi
            dsum = half_swap_sum(dsum);
            dwrap = half_swap_sum(dwrap);
            atomicAdd(diag + ((s0 - my_r0 + 32 * hh - qi) & (kDiagRing - 1)), hh ? dwrap : dsum - dwrap);
        }
    };

    // ---- pipeline: step s computes stage s from LDS, prefetches the fragments of stage s+1 and refills the buffer of
    //      stage s-1 with stage s+2, whose global loads were issued at the top of the step ----
#pragma unroll
    for (int st = 0; st < 2; ++st) {
        if (st < nstages) {
            load_stage(st);
            store_stage(st);
        }
    }
    __syncthreads();
    int buf = 0;
    for (int st = 0; st < nstages; ++st) {
        if (st > 0) __syncthreads();
        const int buf1 = buf == 2 ? 0 : buf + 1, buf2 = buf1 == 2 ? 0 : buf1 + 1;
        if (COLUMNS && st > 0 && tid < 64) {
            // offsets below 64 st - 255 can no longer be touched: flush the 64 that became final with the last stage
            const int o = 64 * (st - 1) - (kGroupRows - 1) + tid;
            if (o >= 0 && o < n) {
                const int s = o & (kDiagRing - 1);
                const float v = diag[s];
                diag[s] = 0.f;
                if (v != 0.f) unsafeAtomicAdd(p.a_s + static_cast<size_t>(p.reduce_group ? g : h) * n + o, v);
            }
        }
        const bool more = st + 2 < nstages;
        load_stage(st + 2);
        const int t0 = t_begin + 2 * st, t1 = t0 + 1;
        // a tile is live for this wavefront if any of its entries is causal
        const bool live0 = my_r0 < n && (COLUMNS ? 32 * t0 + 31 >= my_r0 : 32 * t0 <= my_r0 + 31);
        const bool live1 = t1 < t_end && my_r0 < n && (COLUMNS ? 32 * t1 + 31 >= my_r0 : 32 * t1 <= my_r0 + 31);
        uint64_t win0 = 0ull, win1 = 0ull;
        if (RECALL) {
            // selected offsets dlt-31 .. dlt+31 of a tile at bits 0..62, dlt = first query - first key
            if (live0) win0 = window64(sbit, 32 * t0 - my_r0 + 33) & kAll63;
            if (live1) win1 = window64(sbit, 32 * t1 - my_r0 + 33) & kAll63;
        }
        if (live0 || live1) {
            bf16x8 a0[8], a1[8];
            f32x16 s0, s1;
#pragma unroll
            for (int e = 0; e < 16; ++e) s0[e] = s1[e] = 0.f;
            if (live0) read_a(2 * buf, a0);
            if (live1) read_a(2 * buf + 1, a1);
            if (live0 && live1) {
#pragma unroll
                for (int kk = 0; kk < 8; ++kk) {             // two independent accumulation chains
                    s0 = mfma32(a0[kk], rf[kk], s0);
                    s1 = mfma32(a1[kk], rf[kk], s1);
                }
            } else if (live0) {
#pragma unroll
                for (int kk = 0; kk < 8; ++kk) s0 = mfma32(a0[kk], rf[kk], s0);
            } else {
#pragma unroll
                for (int kk = 0; kk < 8; ++kk) s1 = mfma32(a1[kk], rf[kk], s1);
            }
            if (live0) tile(t0, 2 * buf, s0, win0);
            if (live1) tile(t1, 2 * buf + 1, s1, win1);
        }
        if (more) store_stage(buf2);
        buf = buf1;
    }

    // ---- results ----
    if (!COLUMNS) {
        // the two halves of the wavefront hold disjoint keys of the same query: merge (max, sum) pairs
        const auto mo = __builtin_amdgcn_permlane32_swap(__float_as_uint(m_run), __float_as_uint(m_run), false, false);
        const auto lo = __builtin_amdgcn_permlane32_swap(__float_as_uint(l_run), __float_as_uint(l_run), false, false);
        const float m_a = __uint_as_float(mo[0]), m_b = __uint_as_float(mo[1]);
        const float l_a = __uint_as_float(lo[0]), l_b = __uint_as_float(lo[1]);
        const float m2 = fmaxf(m_a, m_b);
        float l2 = 0.f;
        if (m_a > NEG_INF) l2 += l_a * __builtin_amdgcn_exp2f(m_a - m2);
        if (m_b > NEG_INF) l2 += l_b * __builtin_amdgcn_exp2f(m_b - m2);
        const int row = my_r0 + qi;
        if (row < n && hh == 0) p.lse2[static_cast<size_t>(h) * n + row] = m2 + __log2f(l2);
    } else {
        __syncthreads();
        // what is still in the ring: the last 319 offsets the workgroup touched
        if (tid < kGroupRows + 64) {
            const int o = 64 * (nstages - 1) - (kGroupRows - 1) + tid;
            if (o >= 0 && o < n) {
                const int s = o & (kDiagRing - 1);
                const float v = diag[s];
                if (v != 0.f) unsafeAtomicAdd(p.a_s + static_cast<size_t>(p.reduce_group ? g : h) * n + o, v);
            }
        }
        const int out_head = p.reduce_group ? g : h;
        const float cs = half_swap_sum(col_sum);
        const int key = my_r0 + qi;
        if (key < n && hh == 0) {
            if (p.reduce_group) unsafeAtomicAdd(p.a_v + static_cast<size_t>(out_head) * n + key, cs);
            else p.a_v[static_cast<size_t>(out_head) * n + key] = cs;
        }
        if (RECALL) {
            float r = rec_sum;
#pragma unroll
            for (int d = 32; d >= 1; d >>= 1) r += __shfl_xor(r, d);
            if (lane == 0 && r != 0.f) unsafeAtomicAdd(p.recall + out_head, r);
        }
    }
}

__global__ void fill_float_kernel(float* p, size_t count, float value) {
    const size_t i = static_cast<size_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (i < count) p[i] = value;
}

// natural-log row normalisers (as written by the dense attention call) -> log2 domain
__global__ void lse_to_log2_kernel(const float* lse, float* lse2, size_t count) {
    const size_t i = static_cast<size_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (i < count) lse2[i] = lse[i] * 1.4426950408889634f;
}

struct AggWs {
    size_t lse_off, sbit_off, vbit_off, total;
    int sw, vw;
};

AggWs agg_ws_layout(int q_heads, int index_heads, int64_t n) {
    AggWs w;
    w.sw = static_cast<int>(vs::round_up(static_cast<size_t>(n + 64 + 160 + 31) / 32, 4));
    w.vw = static_cast<int>(vs::round_up(static_cast<size_t>((n + 31) / 32 + 4), 4));
    w.lse_off = 0;
    w.sbit_off = vs::round_up(static_cast<size_t>(q_heads) * n * 4, 256);
    w.vbit_off = w.sbit_off + static_cast<size_t>(index_heads) * w.sw * 4;
    w.total = vs::round_up(w.vbit_off + static_cast<size_t>(index_heads) * w.vw * 4, 256);
    return w;
}

}  // namespace

extern "C" {

size_t vs_aggregate_workspace(int q_heads, int kv_heads, int index_heads, int64_t n) {
    if (q_heads <= 0 || kv_heads <= 0 || index_heads < 0 || n <= 0 || n > VS_MAX_SEQ) return 0;
    return agg_ws_layout(q_heads, index_heads, n).total;
}

int vs_aggregate(const void* q, const void* k, int q_heads, int kv_heads, int64_t n, float scale, const float* lse,
                 int out_heads, float* a_v, float* a_s, const int32_t* idx_v, const int32_t* cnt_v, int cap_v,
                 const int32_t* idx_s, const int32_t* cnt_s, int cap_s, int index_heads, float* recall, void* ws,
                 size_t ws_bytes, void* stream) {
    if (!q || !k || !a_v || !a_s) return VS_ERR_INVALID_ARG;
    if (!vs::aligned16(q) || !vs::aligned16(k) || !vs::aligned16(a_v) || !vs::aligned16(a_s)) return VS_ERR_INVALID_ARG;
    if (q_heads <= 0 || kv_heads <= 0 || n <= 0) return VS_ERR_INVALID_ARG;
    if (!(scale > 0.f) || !isfinite(scale)) return VS_ERR_INVALID_ARG;
    if (q_heads % kv_heads != 0) return VS_ERR_UNSUPPORTED;
    if (n > VS_MAX_SEQ) return VS_ERR_UNSUPPORTED;
    if (out_heads != q_heads && out_heads != kv_heads) return VS_ERR_UNSUPPORTED;
    const bool want_recall = recall != nullptr;
    if (want_recall) {
        if (!idx_v || !cnt_v || !idx_s || !cnt_s || cap_v <= 0 || cap_s <= 0) return VS_ERR_INVALID_ARG;
        if (index_heads != kv_heads && index_heads != q_heads) return VS_ERR_UNSUPPORTED;
    } else {
        index_heads = 0;
    }
    const AggWs w = agg_ws_layout(q_heads, index_heads, n);
    if (!ws || ws_bytes < w.total) return VS_ERR_WORKSPACE;
    if (!vs::aligned16(ws)) return VS_ERR_INVALID_ARG;
    hipStream_t st = static_cast<hipStream_t>(stream);
    unsigned char* base = static_cast<unsigned char*>(ws);

    SweepParams p{};
    p.q = static_cast<const uint16_t*>(q);
    p.k = static_cast<const uint16_t*>(k);
    p.lse2 = reinterpret_cast<float*>(base + w.lse_off);
    p.a_v = a_v;
    p.a_s = a_s;
    p.recall = recall;
    p.q_heads = q_heads;
    p.kv_heads = kv_heads;
    p.group = q_heads / kv_heads;
    p.n = static_cast<int>(n);
    p.reduce_group = (out_heads != q_heads) ? 1 : 0;
    p.c = scale * 1.4426950408889634f;
    p.log2_norm = log2f(static_cast<float>(n)) + (p.reduce_group ? log2f(static_cast<float>(p.group)) : 0.f);
    p.index_per_q = (want_recall && index_heads == q_heads && q_heads != kv_heads) ? 1 : 0;

    // outputs are accumulated with atomics
    const size_t out_count = static_cast<size_t>(out_heads) * n;
    hipLaunchKernelGGL(fill_float_kernel, dim3(static_cast<unsigned>((out_count + 255) / 256)), dim3(256), 0, st, a_v, out_count, 0.f);
    VS_LAUNCH_CHECK();
    hipLaunchKernelGGL(fill_float_kernel, dim3(static_cast<unsigned>((out_count + 255) / 256)), dim3(256), 0, st, a_s, out_count, 0.f);
    VS_LAUNCH_CHECK();
    if (want_recall) {
        hipLaunchKernelGGL(fill_float_kernel, dim3(static_cast<unsigned>((out_heads + 255) / 256)), dim3(256), 0, st, recall,
                           static_cast<size_t>(out_heads), 0.f);
        VS_LAUNCH_CHECK();
        uint32_t* sbit = reinterpret_cast<uint32_t*>(base + w.sbit_off);
        uint32_t* vbit = reinterpret_cast<uint32_t*>(base + w.vbit_off);
        const size_t words = (w.total - w.sbit_off) / 4;
        hipLaunchKernelGGL(fill_zero_kernel, dim3(static_cast<unsigned>((words + 255) / 256)), dim3(256), 0, st, sbit, words);
        VS_LAUNCH_CHECK();
        hipLaunchKernelGGL(set_bits_kernel, dim3((cap_s + 255) / 256, index_heads), dim3(256), 0, st, idx_s, cnt_s, cap_s,
                           static_cast<int>(n), sbit, w.sw, 64);
        VS_LAUNCH_CHECK();
        hipLaunchKernelGGL(set_bits_kernel, dim3((cap_v + 255) / 256, index_heads), dim3(256), 0, st, idx_v, cnt_v, cap_v,
                           static_cast<int>(n), vbit, w.vw, 0);
        VS_LAUNCH_CHECK();
        p.sbit = sbit;
        p.vbit = vbit;
        p.sw = w.sw;
        p.vw = w.vw;
    }
    const int64_t blocks = static_cast<int64_t>(q_heads) * ((n + kGroupRows - 1) / kGroupRows);
    if (blocks > 0x7fffffffLL) return VS_ERR_UNSUPPORTED;
    const size_t rows = static_cast<size_t>(q_heads) * n;
    if (lse) {
        hipLaunchKernelGGL(lse_to_log2_kernel, dim3(static_cast<unsigned>((rows + 255) / 256)), dim3(256), 0, st, lse, p.lse2, rows);
    } else {
        hipLaunchKernelGGL((vs_sweep_kernel<false, false>), dim3(static_cast<unsigned>(blocks)), dim3(kThreads), 0, st, p);
    }
    VS_LAUNCH_CHECK();
    if (want_recall) hipLaunchKernelGGL((vs_sweep_kernel<true, true>), dim3(static_cast<unsigned>(blocks)), dim3(kThreads), 0, st, p);
    else hipLaunchKernelGGL((vs_sweep_kernel<true, false>), dim3(static_cast<unsigned>(blocks)), dim3(kThreads), 0, st, p);
    VS_LAUNCH_CHECK();
    return VS_OK;
}

}  // extern "C"
