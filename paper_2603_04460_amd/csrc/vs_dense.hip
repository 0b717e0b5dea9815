// Dense causal attention for gfx950 on the layout of the sparse kernel (bf16 Q / K / V, head dimension 128, GQA).
//
// Four wavefronts per workgroup, one per SIMD, each owning TWO 32-row blocks of the workgroup's 8 (hc query heads of
// the KV group times 8 / hc consecutive 32-row sub-blocks).  Every K / V fragment read from LDS feeds two matrix
// instructions, one per row block, which halves the LDS reads per flop against one row block per wavefront.  The
// arithmetic per row block (S^T = K Q^T, joint softmax over a stage of two 32-key tiles with a lazily updated
// maximum, O^T = V^T P^T) and the LDS tile layout are those of the sparse kernel.
//
// A SIMD issues about one vector instruction per 4-5 clocks whichever wavefront it comes from (an exponential
// takes 16), while a 32x32x16 matrix instruction occupies the matrix core for 32: the softmax of a stage costs
// more issue time than its matrix products cost matrix time, so the kernel is bound by the instruction stream
// and is written to keep that stream short and free of waits.  With one wavefront per SIMD the overlap of the
// softmax with the matrix core comes from inside the wavefront: the two row blocks run half a stage apart and
// each slot is written out in issue order, matrix and vector instructions alternating.
//   slot X(i): matrix: scores of block 0 for stage i, then P V of block 0 for stage i-1;  vector: softmax of block 1, stage i-1
//   slot Y(i): matrix: scores of block 1 for stage i, then P V of block 1 for stage i-1;  vector: softmax of block 0, stage i
// V fragments of stage i-1 are read at the start of X(i), K fragments of stage i+1 in Y(i) after the scores of
// block 1; one barrier per stage, in Y(i), publishes stage i+1 and frees the buffer of stage i-1 for stage i+2.
//
// Built with -mllvm -amdgpu-mfma-vgpr-form: score accumulators are then written to the vector registers the softmax
// reads them from (the default puts every accumulator of a 512-register kernel in the accumulation registers and
// copies element by element).
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include <type_traits>

#include "vs_attn_device.h"

namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;
constexpr size_t kSmemBytes = kSlots * kSlotBytes;

__global__ __launch_bounds__(kThreads) void vs_dense_kernel(const AttnParams p) {
    extern __shared__ __align__(16) unsigned char smem[];
    unsigned char* const kvbuf = smem;
    const float NEG_INF = -INFINITY;
    const int bid = blockIdx.x;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int qi = lane & 31, hh = lane >> 5;
    const int rest = bid / p.kv_heads;
    const int g = bid % p.kv_heads;
    const int hchunks = p.group / p.hc;
    const int hchunk = rest % hchunks;
    const int tile = p.tiles - 1 - rest / hchunks;          // longest tiles first
    const int BQ = 256 / p.hc;
    const int i0 = p.pos0 + tile * BQ;                      // positions are absolute; the tile grid starts at the chunk
    const int n = p.n;                                      // keys
    const int n_pos = p.pos0 + p.nq;                        // positions that exist
    const int i_last = min(i0 + BQ, n_pos) - 1;

    int my_head[2], my_i0[2];
    bool my_rows[2];
#pragma unroll
    for (int rb = 0; rb < 2; ++rb) {
        const int w = 2 * wave + rb;
        my_head[rb] = g * p.group + hchunk * p.hc + w % p.hc;
        my_i0[rb] = i0 + 32 * (w / p.hc);
        my_rows[rb] = my_i0[rb] < n_pos;
    }
    const uint16_t* __restrict__ kbase = p.k + static_cast<size_t>(g) * n * kD;
    const uint16_t* __restrict__ vbase = p.v + static_cast<size_t>(g) * n * kD;

    bf16x8 qf[2][8];
#pragma unroll
    for (int rb = 0; rb < 2; ++rb) {
        const int row = my_i0[rb] + qi;
        const uint16_t* src = p.q + (static_cast<size_t>(my_head[rb]) * p.nq + (min(row, n_pos - 1) - p.pos0)) * kD + 8 * hh;
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) {
            uint4 raw = make_uint4(0, 0, 0, 0);
            if (row < n_pos) raw = *reinterpret_cast<const uint4*>(src + 16 * kk);
            qf[rb][kk] = __builtin_bit_cast(bf16x8, raw);
        }
    }
    f32x16 oacc[2][4];
    float m_run[2], l_run[2];
#pragma unroll
    for (int rb = 0; rb < 2; ++rb) {
        m_run[rb] = NEG_INF;
        l_run[rb] = 0.f;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int e = 0; e < 16; ++e) oacc[rb][db][e] = 0.f;
    }

    // staging: wavefront w fills groups w and w + 4 of a tile (rows 4 w + L / 16 and 16 more)
    const int st_row = tid >> 4;
    const int st_rho = (lane >> 4) & 3;
    const int st_ck = 4 * ((lane >> 2) & 3) + (((lane & 3) - st_rho) & 3);
    const int st_cv = 4 * ((((lane >> 2) & 3) - st_rho) & 3) + (lane & 3);
    const int nblk = i_last / 32 + 1;
    const int nst = (nblk + 1) >> 1;
    // per-thread byte offsets of its four pieces of a stage (tile u, row half h), relative to the stage's first row
    uint32_t voff_k[2][2], voff_v[2][2];
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            voff_k[u][h] = static_cast<uint32_t>(((32 * u + st_row + 16 * h) * kD + st_ck * 8) * 2);
            voff_v[u][h] = static_cast<uint32_t>(((32 * u + st_row + 16 * h) * kD + st_cv * 8) * 2);
        }
    auto load_stage = [&](int st) __attribute__((always_inline)) {
        const int buf = st % 3;
        if (2 * st + 1 < nblk && 64 * st + 63 < n) {
            // every row of the stage exists: uniform base + per-thread offset, no address arithmetic per load
            const uint16_t* ks = kbase + static_cast<size_t>(64 * st) * kD;
            const uint16_t* vs_ = vbase + static_cast<size_t>(64 * st) * kD;
#pragma unroll
            for (int u = 0; u < 2; ++u)
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    unsigned char* dst = kvbuf + (2 * buf + u) * kSlotBytes + (wave + 4 * h) * kGroupBytes;
                    lds_load16s(voff_k[u][h], ks, dst);
                    lds_load16s(voff_v[u][h], vs_, dst + kTileBytes);
                }
            return;
        }
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int t = 2 * st + u;
                int row = 32 * t + st_row + 16 * h;
                if (t >= nblk || row >= n) row = 0;          // masked anyway: no predicate on the load
                unsigned char* dst = kvbuf + (2 * buf + u) * kSlotBytes + (wave + 4 * h) * kGroupBytes;
                const size_t off = static_cast<size_t>(row) * kD;
                lds_load16(kbase + off + st_ck * 8, dst);
                lds_load16(vbase + off + st_cv * 8, dst + kTileBytes);
            }
    };
    const int li = lane & 15, dsel = (lane >> 4) & 1;
    const int k_row = (qi >> 2) * kGroupBytes + (qi & 3) * 256;
    const int k_off0 = k_row + 16 * ((hh + qi) & 3), k_off2 = k_row + 16 * ((hh + qi + 2) & 3);
    const int v_rho = (li >> 2) & 3;
    const int v_lane = kTileBytes + hh * kGroupBytes + v_rho * 256 + 32 * dsel + 8 * (li & 3);
    int v_off[4];
#pragma unroll
    for (int sgr = 0; sgr < 4; ++sgr) v_off[sgr] = v_lane + 64 * ((sgr + v_rho) & 3);
    typedef __attribute__((address_space(3))) bf16x4t* lds_ptr_t;
    auto read_k = [&](int slot, bf16x8 (&kf)[8]) __attribute__((always_inline)) {
        const unsigned char* kt = kvbuf + slot * kSlotBytes;
#pragma unroll
        for (int kk = 0; kk < 8; ++kk)
            kf[kk] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(kt + ((kk & 1) ? k_off2 : k_off0) + 64 * (kk >> 1)));
    };

    bf16x8 kf[2][8], vf[2][8], pb[2][2][2];
    f32x16 sc[2][2];
    const uint32_t lds0 = static_cast<uint32_t>(reinterpret_cast<uintptr_t>((const __attribute__((address_space(3))) void*)kvbuf));

    // causal mask of tile t for row block rb (only the tiles on and past the diagonal need it)
    auto mask_tile = [&](f32x16& acc, int t, int rb) __attribute__((always_inline)) {
        const int dlt = my_i0[rb] - 32 * t;
        if (dlt >= 31 && my_rows[rb]) return;
        const uint64_t w = (dlt < -31 || !my_rows[rb] || t >= nblk) ? 0ull : (dlt >= 31 ? kAll63 : ((kAll63 << (31 - dlt)) & kAll63));
        mask_elements<0>(acc, lane_keep_bits(w, w, 0u, 0u, qi + 4 - 4 * hh, 4 - 4 * hh), __float_as_uint(NEG_INF));
    };
    // One slot, written out in issue order: pieces are separated by scheduling barriers, so the matrix instructions
    // and the vector work alternate as listed.  MR: the row block whose matrix products are issued; VR = 1 - MR: the
    // row block whose softmax runs.  sq: stage whose scores are computed (HAS_Q); sq - 1: stage whose P V is
    // accumulated (HAS_P); sv: stage whose scores go through the softmax (HAS_S).
#define VS_FENCE() __builtin_amdgcn_sched_barrier(0)
    auto slot = [&](auto mr_tag, auto has_q, auto has_p, auto has_s, auto masked, int sq, int sv) __attribute__((always_inline)) {
        constexpr int MR = decltype(mr_tag)::value, VR = 1 - MR;
        constexpr bool HAS_Q = decltype(has_q)::value, HAS_P = decltype(has_p)::value, HAS_S = decltype(has_s)::value;
        constexpr bool MASKED = decltype(masked)::value;
        auto qmfma = [&](int kk, int u) __attribute__((always_inline)) {
            if (kk == 0) {
                f32x16 zero;
#pragma unroll
                for (int e = 0; e < 16; ++e) zero[e] = 0.f;
                sc[MR][u] = mfma32(kf[u][0], qf[MR][0], zero);
            } else {
                sc[MR][u] = mfma32(kf[u][kk], qf[MR][kk], sc[MR][u]);
            }
        };
        auto pmfma = [&](int idx) __attribute__((always_inline)) {
            const int u = idx >> 3, t = (idx >> 2) & 1, db = idx & 3;
            oacc[MR][db] = mfma32(vf[u][2 * db + t], pb[MR][u][t], oacc[MR][db]);
        };
        // vbase[sgr] / kbase_[par]: per-lane LDS addresses of the stage, everything else is an immediate offset
        auto vread = [&](int u, int j, const uint32_t (&vbase)[4]) __attribute__((always_inline)) {
            const uint32_t a0 = vbase[j >> 1] + u * kSlotBytes + 4 * (j & 1) * kGroupBytes;
            const bf16x4t lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_ptr_t)(a0));
            const bf16x4t hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_ptr_t)(a0 + 2 * kGroupBytes));
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                vf[u][j][e] = lo[e];
                vf[u][j][4 + e] = hi[e];
            }
        };
        auto kread = [&](int u, int kk, const uint32_t (&kb)[2]) __attribute__((always_inline)) {
            typedef const __attribute__((address_space(3))) uint4* lds_u4_t;
            kf[u][kk] = __builtin_bit_cast(bf16x8, *(lds_u4_t)(kb[kk & 1] + u * kSlotBytes + 64 * (kk >> 1)));
        };
        if constexpr (MR == 1) {
            // stage sq+1 has arrived (this wavefront's part; the barrier publishes all of it) and every wavefront
            // has left stage sq-1 behind: its buffer takes stage sq+2
            __builtin_amdgcn_s_waitcnt(0x0F70);
            __syncthreads();
            if (sq + 2 < nst) load_stage(sq + 2);
            VS_FENCE();
        }
        // ---- part 1: first matrix instructions | V fragments (X slot) | row maximum ----
        float mx0 = NEG_INF, mx1 = NEG_INF;
        float mxc[4];
        if constexpr (HAS_S && MASKED) {
            mask_tile(sc[VR][0], 2 * sv, VR);
            mask_tile(sc[VR][1], 2 * sv + 1, VR);
            VS_FENCE();
        }
        uint32_t vbase[4];                                   // V fragments of stage sq - 1
        if constexpr (MR == 0 && HAS_P) {
            const uint32_t sbase = lds0 + 2 * ((sq + 2) % 3) * kSlotBytes;
#pragma unroll
            for (int sgr = 0; sgr < 4; ++sgr) {
                vbase[sgr] = sbase + v_off[sgr];
                asm volatile("" : "+v"(vbase[sgr]));
            }
        }
#pragma unroll
        for (int j = 0; j < 6; ++j) {
            if constexpr (HAS_Q) qmfma(j >> 1, j & 1);
            VS_FENCE();
            if constexpr (MR == 0 && HAS_P) {
                // V fragments of stage sq-1: 16 fragments over 6 pieces
#pragma unroll
                for (int f = 3 * j; f < min(3 * j + 3, 16); ++f) vread(f >> 3, f & 7, vbase);
            }
            if constexpr (HAS_S) {
                // row maximum: four independent chains (two per tile) of three-input maxima, one link of each per piece
                if (j < 4) {
#pragma unroll
                    for (int ch = 0; ch < 4; ++ch) {
                        const f32x16& a = sc[VR][ch >> 1];
                        const int b0 = 8 * (ch & 1);
                        if (j == 0) mxc[ch] = fmaxf(fmaxf(a[b0], a[b0 + 1]), a[b0 + 2]);
                        if (j == 1) mxc[ch] = fmaxf(fmaxf(mxc[ch], a[b0 + 3]), a[b0 + 4]);
                        if (j == 2) mxc[ch] = fmaxf(fmaxf(mxc[ch], a[b0 + 5]), a[b0 + 6]);
                        if (j == 3) mxc[ch] = fmaxf(mxc[ch], a[b0 + 7]);
                    }
                }
                if (j == 4) {
                    mx0 = fmaxf(mxc[0], mxc[1]);
                    mx1 = fmaxf(mxc[2], mxc[3]);
                }
            }
            VS_FENCE();
        }
        if constexpr (HAS_S) {
            const float m_new = fmaxf(m_run[VR], half_swap_max(fmaxf(mx0, mx1)));
            if (__ballot((m_new - m_run[VR]) * p.c > kRescaleThreshold)) {
                const float alpha = (m_new == NEG_INF) ? 1.f : __builtin_amdgcn_exp2f((m_run[VR] - m_new) * p.c);
#pragma unroll
                for (int db = 0; db < 4; ++db)
#pragma unroll
                    for (int e = 0; e < 16; ++e) oacc[VR][db][e] *= alpha;
                l_run[VR] *= alpha;
                m_run[VR] = m_new;
            }
        }
        // ---- part 2: remaining matrix instructions | K fragments (Y slot) | exponentials ----
        const float mc = (!HAS_S || m_run[VR] == NEG_INF) ? 0.f : m_run[VR] * p.c;
        float lsum = 0.f;
        // Softmax elements as a three-deep pipeline: step k scales element k, takes the exponential of element k-1 and adds
        // element k-2 to the row sum (packing a finished pair): no instruction uses the result of its predecessor.
        float tq[3] = {0.f, 0.f, 0.f};                       // values in flight, indexed by element mod 3
        int estep = 0;
        auto expstep = [&]() __attribute__((always_inline)) {
            if constexpr (HAS_S) {
                const int k = estep;
                if (k < 32) {
                    float t = fmaf(sc[VR][k >> 4][k & 15], p.c, -mc);
                    asm volatile("" : "+v"(t));
                    tq[k % 3] = t;
                }
                if (k >= 1 && k <= 32) {
                    float x = tq[(k - 1) % 3];
                    x = __builtin_amdgcn_exp2f(x);
                    asm volatile("" : "+v"(x));              // keeps the arithmetic at this place
                    tq[(k - 1) % 3] = x;
                }
                if (k >= 2 && k <= 33) {
                    const int idx = k - 2, u = idx >> 4, e = idx & 15;
                    const float x = tq[idx % 3];
                    lsum += x;
                    asm volatile("" : "+v"(lsum));
                    sc[VR][u][e] = x;
                    if (e & 1) {
                        const f32x2 two = {sc[VR][u][e - 1], sc[VR][u][e]};
                        const bf16x2 r = __builtin_convertvector(two, bf16x2);
                        uint32_t packed = __builtin_bit_cast(uint32_t, r);
                        asm volatile("" : "+v"(packed));
                        const bf16x2 r2 = __builtin_bit_cast(bf16x2, packed);
                        pb[VR][u][e >> 3][(e & 7) - 1] = r2[0];
                        pb[VR][u][e >> 3][e & 7] = r2[1];
                    }
                }
                ++estep;
            }
        };
        // 34 steps over the 26 matrix instructions of this part
        auto expsteps_upto = [&](int target) __attribute__((always_inline)) {
            while (estep < target) expstep();
        };
        uint32_t kb[2];                                      // K fragments of stage sq + 1 (past the last stage: a stale slot, never used)
        if constexpr (MR == 1 && HAS_Q) {
            const uint32_t sbase = lds0 + 2 * ((sq + 1) % 3) * kSlotBytes;
            kb[0] = sbase + k_off0;
            kb[1] = sbase + k_off2;
            asm volatile("" : "+v"(kb[0]), "+v"(kb[1]));
        }
#pragma unroll
        for (int j = 6; j < 16; ++j) {                       // 10 more score products
            if constexpr (HAS_Q) qmfma(j >> 1, j & 1);
            VS_FENCE();
            if constexpr (HAS_S) expsteps_upto(((j - 6 + 1) * 34 + 25) / 26);
            VS_FENCE();
        }
#pragma unroll
        for (int j = 0; j < 16; ++j) {                       // 16 P V products
            if constexpr (HAS_P) pmfma(j);
            VS_FENCE();
            if constexpr (MR == 1 && HAS_Q) {
                kread(j >> 3, j & 7, kb);
            }
            if constexpr (HAS_S) expsteps_upto(((10 + j + 1) * 34 + 25) / 26);
            VS_FENCE();
        }
        if constexpr (HAS_S) {
            expsteps_upto(34);
            l_run[VR] += lsum;
        }
        VS_FENCE();
    };
#undef VS_FENCE

    __builtin_amdgcn_s_waitcnt(0x0F70);
    load_stage(0);
    if (nst > 1) load_stage(1);
    __builtin_amdgcn_s_waitcnt(0x0F70);
    __syncthreads();
    read_k(0, kf[0]);
    read_k(1, kf[1]);
    using T = std::true_type;
    using F = std::false_type;
    using R0 = std::integral_constant<int, 0>;
    using R1 = std::integral_constant<int, 1>;
    // stages whose two tiles lie below the diagonal for both row blocks need no mask
    const int nfree = (my_rows[0] && my_rows[1]) ? min(my_i0[0], my_i0[1]) / 64 : 0;
    slot(R0{}, T{}, F{}, F{}, T{}, 0, 0);                    // X(0): scores of block 0
    slot(R1{}, T{}, F{}, T{}, T{}, 0, 0);                    // Y(0): scores of block 1; softmax of block 0
    int i = 1;
    for (; i < min(nst, nfree); ++i) {
        slot(R0{}, T{}, T{}, T{}, F{}, i, i - 1);
        slot(R1{}, T{}, T{}, T{}, F{}, i, i);
    }
    for (; i < nst; ++i) {
        slot(R0{}, T{}, T{}, T{}, T{}, i, i - 1);
        slot(R1{}, T{}, T{}, T{}, T{}, i, i);
    }
    slot(R0{}, F{}, T{}, T{}, T{}, nst, nst - 1);            // X(nst): P V of block 0; softmax of block 1
    slot(R1{}, F{}, T{}, F{}, T{}, nst, nst);                // Y(nst): P V of block 1

#pragma unroll
    for (int rb = 0; rb < 2; ++rb) {
        const float l_tot = half_swap_sum(l_run[rb]);
        const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
        const int row = my_i0[rb] + qi;
        if (row < n_pos) {
            uint16_t* dst = p.o + (static_cast<size_t>(my_head[rb]) * p.nq + (row - p.pos0)) * kD;
#pragma unroll
            for (int db = 0; db < 4; ++db)
#pragma unroll
                for (int a = 0; a < 4; ++a) {
                    const f32x2 x01 = {oacc[rb][db][4 * a] * inv, oacc[rb][db][4 * a + 1] * inv};
                    const f32x2 x23 = {oacc[rb][db][4 * a + 2] * inv, oacc[rb][db][4 * a + 3] * inv};
                    const bf16x2 y01 = __builtin_convertvector(x01, bf16x2);
                    const bf16x2 y23 = __builtin_convertvector(x23, bf16x2);
                    uint2 out;
                    out.x = __builtin_bit_cast(uint32_t, y01);
                    out.y = __builtin_bit_cast(uint32_t, y23);
                    *reinterpret_cast<uint2*>(dst + 32 * db + 8 * a + 4 * hh) = out;
                }
            if (p.lse && hh == 0)
                p.lse[static_cast<size_t>(my_head[rb]) * p.nq + (row - p.pos0)] = l_tot > 0.f ? m_run[rb] * p.scale + __logf(l_tot) : NEG_INF;
        }
    }
}

int launch_dense(AttnParams& p, hipStream_t stream) {
    static vs::PerDeviceOnce once;
    const int rc_once = once.run(nullptr, [](int) -> int {
        VS_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&vs_dense_kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                                   static_cast<int>(kSmemBytes)));
        return VS_OK;
    });
    if (rc_once != VS_OK) return rc_once;
    const int BQ = 256 / p.hc;
    p.tiles = (p.nq + BQ - 1) / BQ;
    // one workgroup per (query tile, KV head, chunk of the group's heads), longest tiles first; workgroups are dealt
    // to the 8 XCDs round-robin, so KV head = block % kv_heads keeps a head's K / V in one XCD's L2
    const long long blocks = static_cast<long long>(p.kv_heads) * (p.group / p.hc) * p.tiles;
    if (blocks > 0x7fffffffLL) return VS_ERR_UNSUPPORTED;
    p.work_total = static_cast<int>(blocks);
    hipLaunchKernelGGL(vs_dense_kernel, dim3(static_cast<unsigned>(blocks)), dim3(kThreads), kSmemBytes, stream, p);
    VS_LAUNCH_CHECK();
    return VS_OK;
}

}  // namespace

extern "C" {

int vs_dense_prefill_chunk(const void* q, const void* k, const void* v, int q_heads, int kv_heads, int64_t n_q, int64_t n_kv,
                           int64_t pos0, float scale, void* o_bf16, float* lse, void* stream) {
    int rc = check_qkv(q, k, v, q_heads, kv_heads, n_kv, scale, o_bf16);
    if (rc != VS_OK) return rc;
    rc = check_chunk(n_q, n_kv, pos0);
    if (rc != VS_OK) return rc;
    AttnParams p{};
    p.q = static_cast<const uint16_t*>(q);
    p.k = static_cast<const uint16_t*>(k);
    p.v = static_cast<const uint16_t*>(v);
    p.o = static_cast<uint16_t*>(o_bf16);
    p.lse = lse;
    p.q_heads = q_heads;
    p.kv_heads = kv_heads;
    p.group = q_heads / kv_heads;
    p.index_per_q = 0;
    p.hc = heads_per_workgroup(p.group, false);
    p.n = static_cast<int>(n_kv);
    p.nq = static_cast<int>(n_q);
    p.pos0 = static_cast<int>(pos0);
    p.scale = scale;
    p.c = scale * 1.4426950408889634f;
    p.tile_counter = nullptr;
    return launch_dense(p, static_cast<hipStream_t>(stream));
}

int vs_dense_prefill(const void* q, const void* k, const void* v, int q_heads, int kv_heads, int64_t n, float scale,
                     void* o_bf16, float* lse, void* stream) {
    return vs_dense_prefill_chunk(q, k, v, q_heads, kv_heads, n, n, 0, scale, o_bf16, lse, stream);
}

}  // extern "C"
