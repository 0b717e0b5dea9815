// Budget rule and TopK (Sec. "Adaptive Sparse Index Selection": k_d is the fewest top-ranked scores
// whose mass reaches tau_d, I_d = TopK(A_d, k_d)), one workgroup per (head, direction).
//
// Non-negative fp32 scores order like their bit patterns, so the k-th ranked score is found by a
// most-significant-digit radix descent (12 + 12 + 8 bits) over LDS histograms that carry, per
// bucket, the element count and the INTEGER mass floor(score * 2^40).  Integer masses make every
// partial sum exact and order-independent, so the threshold crossing is the same whatever order
// the wavefronts add in.  Ties at the crossing value are taken in ascending index order.  The
// selected set, united with the forced leading indices, is then written in ascending order by
// three coalesced sweeps that use wave ballots for ranks (no atomics on the output path).
//
// Long sequences with a workspace: the same descent split over many workgroups (one per 8192-score chunk of a problem),
// one kernel per radix pass.  A chunk's histogram is built in LDS and added to the problem's histogram in the workspace
// with integer atomics (exact, so the sums do not depend on the order); every workgroup of the next kernel scans that
// histogram for the crossing bucket.  The emission gets its chunk's position from the per-chunk counts of a sweep of
// its own.  A problem whose selection exceeds the capacity is redone by the single-workgroup kernel.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include "vs_common.h"

namespace {

constexpr int kSelThreads = 1024;
constexpr int kWaves = kSelThreads / 64;
constexpr int kMaxBuckets = 4096;
typedef unsigned long long u64;

struct SelParams {
    const float* a[2];
    int32_t* idx[2];
    int32_t* cnt[2];
    int32_t* status;
    int n, mode;
    double tau[2];
    int kfix[2], nforced[2], cap[2];
};

struct SelShared {
    u64 hist_mass[kMaxBuckets];
    uint32_t hist_cnt[kMaxBuckets];
    u64 wave_m[kWaves];
    uint32_t wave_c[kWaves];
    uint32_t wave_eq[kWaves], wave_eqf[kWaves], wave_in[kWaves];   // emission: ties, forced ties, entries in without a tie
    // result of the bucket search
    uint32_t sel_bucket, eq_c;
    u64 above_m, eq_m;
    uint32_t above_c;
    int status;
};

__device__ __forceinline__ uint32_t score_key(float x, int& st) {
    if (!(x >= 0.f)) {            // NaN or negative
        st |= VS_STATUS_BAD_SCORE;
        return 0u;
    }
    return x == 0.f ? 0u : __float_as_uint(x);
}

__device__ __forceinline__ u64 key_mass(uint32_t key, int& st) {
    double xd = static_cast<double>(__uint_as_float(key));
    if (xd > 1.0) {
        xd = 1.0;
        st |= VS_STATUS_SATURATED;
    }
    return static_cast<u64>(xd * 1099511627776.0);   // exact power-of-two scaling, truncation
}

// Selection state of one (head, direction): elements with key > vstar are in; of those with
// key == vstar the first `ties` in index order are in.  none: nothing is selected by rank.
struct Pick {
    uint32_t vstar;
    uint32_t ties;
    bool none;
};

// redo: null, or per problem (head * 2 + dir) non-zero where this kernel has work
__global__ __launch_bounds__(kSelThreads) void select_kernel(const SelParams p, const int32_t* redo) {
    __shared__ SelShared sh;
    const int head = blockIdx.x, dir = blockIdx.y;
    if (redo && redo[head * 2 + dir] == 0) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = p.n;
    const float* __restrict__ a = p.a[dir] + static_cast<size_t>(head) * n;
    const int nforced = min(p.nforced[dir], n);
    const int cap = p.cap[dir];
    int st = 0;
    if (tid == 0) sh.status = 0;

    // radix descent.  by_count: rank target is a count (krem) instead of a mass (trem).  tau >= 0 (first descent of the
    // threshold rule): the first pass sees every element, so its histogram also gives the total mass; the target
    // ceil(tau * total) is taken from it instead of from a sweep of its own.  first: the first pass also collects the
    // status bits of the scores.
    auto descend = [&](bool by_count, bool skip_forced, u64 trem, uint32_t krem, double tau, bool first) -> Pick {
        Pick pk{0u, 0u, false};
        if (tau < 0.0 && (by_count ? krem == 0 : trem == 0)) {
            pk.none = true;
            return pk;
        }
        uint32_t prefix = 0, pmask = 0;
        const int shifts[3] = {20, 8, 0};
        const int widths[3] = {12, 12, 8};
        for (int pass = 0; pass < 3; ++pass) {
            const int shf = shifts[pass], nb = 1 << widths[pass];
            for (int b = tid; b < nb; b += kSelThreads) {
                sh.hist_mass[b] = 0;
                sh.hist_cnt[b] = 0;
            }
            __syncthreads();
            const bool collect = first && pass == 0;
            for (int i = tid; i < n; i += kSelThreads) {
                if (skip_forced && i < nforced) continue;
                int dummy = 0;
                const uint32_t key = score_key(a[i], collect ? st : dummy);
                if ((key & pmask) != prefix) continue;
                const uint32_t b = (key >> shf) & (nb - 1);
                atomicAdd(&sh.hist_cnt[b], 1u);
                if (!by_count) atomicAdd(&sh.hist_mass[b], key_mass(key, collect ? st : dummy));
                else if (collect) (void)key_mass(key, st);
            }
            __syncthreads();
            // buckets in descending order; thread owns `per` consecutive ones
            const int per = nb >= kSelThreads ? nb / kSelThreads : 1;
            u64 m_loc[4] = {0, 0, 0, 0};
            uint32_t c_loc[4] = {0, 0, 0, 0};
            u64 msum = 0;
            uint32_t csum = 0;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int rb = tid * per + j;
                if (j < per && rb < nb) {
                    m_loc[j] = sh.hist_mass[nb - 1 - rb];
                    c_loc[j] = sh.hist_cnt[nb - 1 - rb];
                    msum += m_loc[j];
                    csum += c_loc[j];
                }
            }
            // exclusive prefix over threads of (mass, count)
            u64 mi = msum;
            uint32_t ci = csum;
#pragma unroll
            for (int d = 1; d < 64; d <<= 1) {
                const u64 my = __shfl_up(mi, d);
                const uint32_t cy = __shfl_up(ci, d);
                if (lane >= d) {
                    mi += my;
                    ci += cy;
                }
            }
            if (lane == 63) {
                sh.wave_m[wave] = mi;
                sh.wave_c[wave] = ci;
            }
            __syncthreads();
            u64 mbase = 0;
            uint32_t cbase = 0;
            for (int w = 0; w < wave; ++w) {
                mbase += sh.wave_m[w];
                cbase += sh.wave_c[w];
            }
            if (pass == 0 && tau >= 0.0) {
                u64 total = 0;
                for (int w = 0; w < kWaves; ++w) total += sh.wave_m[w];
                trem = static_cast<u64>(ceil(tau * static_cast<double>(total)));
                if (trem == 0) {                              // uniform: every thread sees the same total
                    pk.none = true;
                    __syncthreads();
                    return pk;
                }
                if (trem > total) {
                    // Totals above 2^53 are rounded when they become a double, so ceil(tau * total) can exceed the total
                    // itself (tau = 1, more than 2^13 saturated scores): the mass is then never reached and the rule
                    // keeps every element.  Crossing value 0 with every tie taken says exactly that.
                    pk.vstar = 0u;
                    pk.ties = 0xffffffffu;
                    __syncthreads();
                    return pk;
                }
            }
            u64 mrun = mbase + mi - msum;
            uint32_t crun = cbase + ci - csum;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int rb = tid * per + j;
                if (j < per && rb < nb) {
                    const bool hit = by_count ? (crun < krem && crun + c_loc[j] >= krem)
                                              : (mrun < trem && mrun + m_loc[j] >= trem);
                    if (hit) {
                        sh.sel_bucket = nb - 1 - rb;
                        sh.above_m = mrun;
                        sh.above_c = crun;
                        sh.eq_m = m_loc[j];
                        sh.eq_c = c_loc[j];
                    }
                    mrun += m_loc[j];
                    crun += c_loc[j];
                }
            }
            __syncthreads();
            prefix |= sh.sel_bucket << shf;
            pmask |= static_cast<uint32_t>(nb - 1) << shf;
            trem -= by_count ? 0 : sh.above_m;
            krem -= by_count ? sh.above_c : 0;
            __syncthreads();
        }
        pk.vstar = prefix;
        if (by_count) {
            pk.ties = krem;
        } else {
            const u64 wstar = sh.eq_m / sh.eq_c;               // every tie has the same mass
            pk.ties = static_cast<uint32_t>((trem + wstar - 1) / wstar);
        }
        return pk;
    };

    // ---- total mass, threshold ----
    Pick pk;
    if (p.mode == 0) {
        pk = descend(false, false, 0, 0u, p.tau[dir], true);
    } else {
        const uint32_t kfix = static_cast<uint32_t>(min(p.kfix[dir], n));
        if (kfix == 0) {                                     // nothing ranked in: the status bits still need their sweep
            for (int i = tid; i < n; i += kSelThreads) {
                const uint32_t key = score_key(a[i], st);
                (void)key_mass(key, st);
            }
        }
        pk = descend(true, false, 0, kfix, -1.0, true);
    }

    // ---- ordered emission: each wavefront owns a contiguous range, ranks come from ballots ----
    const int per_wave = ((n + kWaves - 1) / kWaves + 63) & ~63;
    const int w_lo = min(wave * per_wave, n), w_hi = min(w_lo + per_wave, n);
    const u64 lt_mask = (1ull << lane) - 1ull;
    int32_t* __restrict__ out = p.idx[dir] + static_cast<size_t>(head) * cap;

    bool skip_forced = false;
    for (int attempt = 0; attempt < 2; ++attempt) {
        // sweep 1: per wavefront, the ties, the ties among the forced entries, and the entries that are in whatever the
        // ties decide (forced, or ranked above the crossing value).  Ties are taken in index order and the forced entries
        // are the lowest indices, so the number of selected entries of a wavefront follows from these three counts.
        uint32_t eqc = 0, eqf = 0, inc = 0;
        for (int base = w_lo; base < w_hi; base += 64) {
            const int i = base + lane;
            bool eq = false, in = false, forced = false;
            if (i < w_hi) {
                int dummy = 0;
                const uint32_t key = score_key(a[i], dummy);
                forced = i < nforced;
                const bool ranked = !pk.none && !(skip_forced && forced);
                eq = ranked && key == pk.vstar;
                in = forced || (ranked && key > pk.vstar);
            }
            eqc += __popcll(__ballot(eq));
            eqf += __popcll(__ballot(eq && forced));
            inc += __popcll(__ballot(in));
        }
        if (lane == 0) {
            sh.wave_eq[wave] = eqc;
            sh.wave_eqf[wave] = eqf;
            sh.wave_in[wave] = inc;
        }
        __syncthreads();
        uint32_t tie_base = 0, pos = 0, total = 0;
        {
            uint32_t ties_before = 0;
            for (int w = 0; w < kWaves; ++w) {
                const uint32_t e = sh.wave_eq[w], ef = sh.wave_eqf[w];
                // free ties of wavefront w that are taken: its forced ties come first and are already counted as in
                const uint32_t room = pk.ties > ties_before + ef ? pk.ties - ties_before - ef : 0u;
                const uint32_t sel = sh.wave_in[w] + min(room, e - ef);
                if (w < wave) pos += sel;
                if (w == wave) tie_base = ties_before;
                total += sel;
                ties_before += e;
            }
        }
        __syncthreads();
        auto selected = [&](int i, uint32_t& tie_run) -> bool {
            bool in = false, eq = false;
            if (i < w_hi) {
                const bool forced = i < nforced;
                int dummy = 0;
                const uint32_t key = score_key(a[i], dummy);
                const bool ranked = !pk.none && !(skip_forced && forced);
                eq = ranked && key == pk.vstar;
                in = forced || (ranked && key > pk.vstar);
            }
            const u64 eb = __ballot(eq);
            if (eq && tie_run + __popcll(eb & lt_mask) < pk.ties) in = true;
            tie_run += __popcll(eb);
            return in;
        };
        uint32_t tie_run = tie_base;
        if (total > static_cast<uint32_t>(cap) && attempt == 0) {
            // keep the forced entries and the best-ranked others: count-ranked pick over the rest
            st |= VS_STATUS_OVERFLOW;
            skip_forced = true;
            pk = descend(true, true, 0, static_cast<uint32_t>(cap - nforced), -1.0, false);
            continue;
        }
        // sweep 2: write
        tie_run = tie_base;
        for (int base = w_lo; base < w_hi; base += 64) {
            const bool in = selected(base + lane, tie_run);
            const u64 sb = __ballot(in);
            if (in) out[pos + __popcll(sb & lt_mask)] = base + lane;
            pos += __popcll(sb);
        }
        if (tid == 0) p.cnt[dir][head] = static_cast<int32_t>(total);
        break;
    }
    if (st) atomicOr(&sh.status, st);
    __syncthreads();
    if (tid == 0 && p.status && sh.status) atomicOr(p.status + head, sh.status);
}

// ---- the same selection over many workgroups ----
constexpr int kChunk = 8192;                   // scores per workgroup
constexpr int kChunkThreads = 512;
constexpr int kChunkWaves = kChunkThreads / 64;
constexpr int kMinSplitN = 32768;              // shorter problems stay with one workgroup (fewer launches)

// descent state of one problem after a pass (written by the workgroup of chunk 0, read by the next kernel)
struct SelState {
    u64 trem, eq_m;
    uint32_t prefix, pmask, krem, eq_c;
    uint32_t none, all, vstar, ties;
};

struct SplitParams {
    SelParams s;
    int chunks;
    u64* hist_m[3];                 // [problems][4096 | 4096 | 256]
    uint32_t* hist_c[3];
    SelState* state;                // [problems][4]
    uint32_t* chunk_cnt;            // [problems][chunks][3]: in, ties, forced ties
    int32_t* redo;                  // [problems]
};

// Where bucket b of an nb-bucket histogram (nb = R * R) sits in the workspace: transposed, so that neighbouring buckets,
// which the scores of one problem crowd into, are R entries apart.  Atomics of many workgroups on one cache line are
// served one after the other (~12 ns each); spread out they go to different lines.  The scan, whose thread t owns the
// buckets 8 t .. 8 t + 7 from the top, then reads a few lines per wavefront instruction instead of 64.
__device__ __forceinline__ int bucket_slot(int b, int nb) {
    const int r = nb == 4096 ? 64 : 16, sh = nb == 4096 ? 6 : 4;
    return ((b & (r - 1)) << sh) | (b >> sh);
}

struct ScanShared {
    u64 wave_m[kChunkWaves];
    uint32_t wave_c[kChunkWaves];
    uint32_t sel_bucket, eq_c, above_c;
    u64 above_m, eq_m;
};

// One pass of the descent on a finished histogram of nb buckets: the bucket in which the running (mass | count), taken
// over the buckets in descending order, reaches the target.  All kChunkThreads threads call it; the arithmetic is that of
// the single-workgroup kernel.
__device__ __forceinline__ void scan_pass(ScanShared& sc, const u64* __restrict__ hm, const uint32_t* __restrict__ hc, int nb,
                                          int shf, bool by_count, double tau, SelState& st) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int per = nb >= kChunkThreads ? nb / kChunkThreads : 1;      // 8 or 1
    constexpr int kPer = 4096 / kChunkThreads;
    u64 m_loc[kPer];
    uint32_t c_loc[kPer];
    u64 msum = 0;
    uint32_t csum = 0;
#pragma unroll
    for (int j = 0; j < kPer; ++j) {
        const int rb = tid * per + j;
        m_loc[j] = 0;
        c_loc[j] = 0;
        if (j < per && rb < nb) {
            m_loc[j] = hm[bucket_slot(nb - 1 - rb, nb)];
            c_loc[j] = hc[bucket_slot(nb - 1 - rb, nb)];
            msum += m_loc[j];
            csum += c_loc[j];
        }
    }
    u64 mi = msum;
    uint32_t ci = csum;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const u64 my = __shfl_up(mi, d);
        const uint32_t cy = __shfl_up(ci, d);
        if (lane >= d) {
            mi += my;
            ci += cy;
        }
    }
    __syncthreads();                                         // (the shared words may still be read from the previous pass)
    if (lane == 63) {
        sc.wave_m[wave] = mi;
        sc.wave_c[wave] = ci;
    }
    __syncthreads();
    u64 mbase = 0;
    uint32_t cbase = 0;
    for (int w = 0; w < wave; ++w) {
        mbase += sc.wave_m[w];
        cbase += sc.wave_c[w];
    }
    if (shf == 20 && tau >= 0.0) {
        u64 total = 0;
        for (int w = 0; w < kChunkWaves; ++w) total += sc.wave_m[w];
        st.trem = static_cast<u64>(ceil(tau * static_cast<double>(total)));
        if (st.trem == 0) {
            st.none = 1u;
            return;
        }
        if (st.trem > total) {                               // see the single-workgroup kernel: the rule keeps every element
            st.all = 1u;
            st.vstar = 0u;
            st.ties = 0xffffffffu;
            return;
        }
    }
    u64 mrun = mbase + mi - msum;
    uint32_t crun = cbase + ci - csum;
#pragma unroll
    for (int j = 0; j < kPer; ++j) {
        const int rb = tid * per + j;
        if (j < per && rb < nb) {
            const bool hit = by_count ? (crun < st.krem && crun + c_loc[j] >= st.krem) : (mrun < st.trem && mrun + m_loc[j] >= st.trem);
            if (hit) {
                sc.sel_bucket = nb - 1 - rb;
                sc.above_m = mrun;
                sc.above_c = crun;
                sc.eq_m = m_loc[j];
                sc.eq_c = c_loc[j];
            }
            mrun += m_loc[j];
            crun += c_loc[j];
        }
    }
    __syncthreads();
    st.prefix |= sc.sel_bucket << shf;
    st.pmask |= static_cast<uint32_t>(nb - 1) << shf;
    if (by_count) st.krem -= sc.above_c;
    else st.trem -= sc.above_m;
    st.eq_m = sc.eq_m;
    st.eq_c = sc.eq_c;
}

// PASS 0..2: histogram of this chunk's scores at digit PASS (after the scan of the previous digit's histogram);
// PASS 3: scan of the last histogram, then this chunk's counts for the emission.
template <int PASS>
__global__ __launch_bounds__(kChunkThreads) void split_pass_kernel(const SplitParams q) {
    __shared__ u64 h_m[PASS < 2 ? 4096 : 256];
    __shared__ uint32_t h_c[PASS < 2 ? 4096 : 256];
    __shared__ ScanShared sc;
    __shared__ uint32_t cnt3[3];
    const SelParams& p = q.s;
    const int chunk = blockIdx.x, head = blockIdx.y, dir = blockIdx.z;
    const int pr = head * 2 + dir;
    const int tid = threadIdx.x;
    const int n = p.n;
    const float* __restrict__ a = p.a[dir] + static_cast<size_t>(head) * n;
    const bool by_count = p.mode != 0;
    const int lo = chunk * kChunk, hi = min(lo + kChunk, n);
    constexpr int shifts[3] = {20, 8, 0};
    constexpr int nbs[3] = {4096, 4096, 256};

    SelState st{};
    if (PASS == 1) {
        st.krem = static_cast<uint32_t>(min(p.kfix[dir], n));
        if (by_count && st.krem == 0) st.none = 1u;
        else scan_pass(sc, q.hist_m[0] + static_cast<size_t>(pr) * 4096, q.hist_c[0] + static_cast<size_t>(pr) * 4096, 4096, 20,
                       by_count, by_count ? -1.0 : p.tau[dir], st);
    } else if (PASS >= 2) {
        st = q.state[pr * 4 + PASS - 1];
        if (!st.none && !st.all) {
            const int pp = PASS - 1;
            scan_pass(sc, q.hist_m[pp] + static_cast<size_t>(pr) * 4096, q.hist_c[pp] + static_cast<size_t>(pr) * 4096, nbs[pp],
                      shifts[pp], by_count, -1.0, st);
        }
    }
    if (PASS == 3 && !st.none && !st.all) {
        st.vstar = st.prefix;
        if (by_count) {
            st.ties = st.krem;
        } else {
            const u64 wstar = st.eq_m / st.eq_c;             // every tie has the same mass
            st.ties = static_cast<uint32_t>((st.trem + wstar - 1) / wstar);
        }
    }
    if (PASS >= 1 && chunk == 0 && tid == 0) q.state[pr * 4 + PASS] = st;

    if constexpr (PASS < 3) {
        if (PASS > 0 && (st.none || st.all)) return;          // uniform over the workgroup
        constexpr int nb = nbs[PASS], shf = shifts[PASS];
        for (int b = tid; b < nb; b += kChunkThreads) {
            h_m[b] = 0;
            h_c[b] = 0;
        }
        __syncthreads();
        int stbits = 0, matched = 0;
        for (int i = lo + tid; i < hi; i += kChunkThreads) {
            int dummy = 0;
            const uint32_t key = score_key(a[i], PASS == 0 ? stbits : dummy);
            if ((key & st.pmask) != st.prefix) continue;
            matched = 1;
            const uint32_t b = (key >> shf) & (nb - 1);
            atomicAdd(&h_c[b], 1u);
            if (!by_count) atomicAdd(&h_m[b], key_mass(key, PASS == 0 ? stbits : dummy));
            else if (PASS == 0) (void)key_mass(key, stbits);
        }
        if (PASS == 0 && stbits && p.status) atomicOr(p.status + head, stbits);
        if (PASS > 0 && !__syncthreads_or(matched)) return;   // nothing of this chunk under the prefix (the usual case)
        __syncthreads();
        u64* gm = q.hist_m[PASS] + static_cast<size_t>(pr) * 4096;
        uint32_t* gc = q.hist_c[PASS] + static_cast<size_t>(pr) * 4096;
        for (int b = tid; b < nb; b += kChunkThreads) {
            const uint32_t c = h_c[b];
            if (c) {
                atomicAdd(&gc[bucket_slot(b, nb)], c);
                if (!by_count) atomicAdd(&gm[bucket_slot(b, nb)], h_m[b]);
            }
        }
    } else {
        // counts of this chunk for the emission: entries that are in whatever the ties decide, ties, forced ties
        if (tid < 3) cnt3[tid] = 0;
        __syncthreads();
        const int nforced = min(p.nforced[dir], n);
        uint32_t inc = 0, eqc = 0, eqf = 0;
        for (int i = lo + tid; i < hi; i += kChunkThreads) {
            int dummy = 0;
            const uint32_t key = score_key(a[i], dummy);
            const bool forced = i < nforced;
            const bool ranked = !st.none;
            const bool eq = ranked && key == st.vstar;
            inc += (forced || (ranked && key > st.vstar)) ? 1u : 0u;
            eqc += eq ? 1u : 0u;
            eqf += (eq && forced) ? 1u : 0u;
        }
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) {
            inc += __shfl_xor(inc, d);
            eqc += __shfl_xor(eqc, d);
            eqf += __shfl_xor(eqf, d);
        }
        if ((tid & 63) == 0) {
            atomicAdd(&cnt3[0], inc);
            atomicAdd(&cnt3[1], eqc);
            atomicAdd(&cnt3[2], eqf);
        }
        __syncthreads();
        if (tid < 3) q.chunk_cnt[(static_cast<size_t>(pr) * q.chunks + chunk) * 3 + tid] = cnt3[tid];
    }
}

// Ordered emission of one chunk: its first output position and its first tie rank follow from the counts of the chunks
// before it; inside the chunk each wavefront owns a contiguous range, as in the single-workgroup kernel.
__global__ __launch_bounds__(kChunkThreads) void split_emit_kernel(const SplitParams q) {
    __shared__ uint32_t c_in[256], c_eq[256], c_ef[256];
    __shared__ uint32_t w_in[kChunkWaves], w_eq[kChunkWaves], w_ef[kChunkWaves];
    const SelParams& p = q.s;
    const int chunk = blockIdx.x, head = blockIdx.y, dir = blockIdx.z;
    const int pr = head * 2 + dir;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = p.n;
    const float* __restrict__ a = p.a[dir] + static_cast<size_t>(head) * n;
    const int nforced = min(p.nforced[dir], n);
    const int cap = p.cap[dir];
    const SelState st = q.state[pr * 4 + 3];
    if (tid < q.chunks) {
        const uint32_t* c = q.chunk_cnt + (static_cast<size_t>(pr) * q.chunks + tid) * 3;
        c_in[tid] = c[0];
        c_eq[tid] = c[1];
        c_ef[tid] = c[2];
    }
    __syncthreads();
    uint32_t pos = 0, tie_base = 0, total = 0, ties_before = 0;
    for (int c = 0; c < q.chunks; ++c) {
        const uint32_t e = c_eq[c], ef = c_ef[c];
        const uint32_t room = st.ties > ties_before + ef ? st.ties - ties_before - ef : 0u;
        const uint32_t sel = c_in[c] + min(room, e - ef);
        if (c < chunk) pos += sel;
        if (c == chunk) tie_base = ties_before;
        total += sel;
        ties_before += e;
    }
    if (total > static_cast<uint32_t>(cap)) {                // the single-workgroup kernel redoes this problem
        if (chunk == 0 && tid == 0) q.redo[pr] = 1;
        return;
    }
    if (chunk == 0 && tid == 0) p.cnt[dir][head] = static_cast<int32_t>(total);
    const int lo = chunk * kChunk, hi = min(lo + kChunk, n);
    const int per_wave = kChunk / kChunkWaves;
    const int w_lo = min(lo + wave * per_wave, hi), w_hi = min(w_lo + per_wave, hi);
    const u64 lt_mask = (1ull << lane) - 1ull;
    auto classify = [&](int i, bool& eq, bool& in, bool& forced) {
        eq = in = forced = false;
        if (i < w_hi) {
            int dummy = 0;
            const uint32_t key = score_key(a[i], dummy);
            forced = i < nforced;
            const bool ranked = !st.none;
            eq = ranked && key == st.vstar;
            in = forced || (ranked && key > st.vstar);
        }
    };
    uint32_t eqc = 0, eqf = 0, inc = 0;
    for (int base = w_lo; base < w_hi; base += 64) {
        bool eq, in, forced;
        classify(base + lane, eq, in, forced);
        eqc += __popcll(__ballot(eq));
        eqf += __popcll(__ballot(eq && forced));
        inc += __popcll(__ballot(in));
    }
    if (lane == 0) {
        w_eq[wave] = eqc;
        w_ef[wave] = eqf;
        w_in[wave] = inc;
    }
    __syncthreads();
    uint32_t tb = tie_base;
    for (int w = 0; w < wave; ++w) {
        const uint32_t e = w_eq[w], ef = w_ef[w];
        const uint32_t room = st.ties > tb + ef ? st.ties - tb - ef : 0u;
        pos += w_in[w] + min(room, e - ef);
        tb += e;
    }
    int32_t* __restrict__ out = p.idx[dir] + static_cast<size_t>(head) * cap;
    uint32_t tie_run = tb;
    for (int base = w_lo; base < w_hi; base += 64) {
        bool eq, in, forced;
        classify(base + lane, eq, in, forced);
        const u64 eb = __ballot(eq);
        if (eq && tie_run + __popcll(eb & lt_mask) < st.ties) in = true;
        tie_run += __popcll(eb);
        const u64 sb = __ballot(in);
        if (in) out[pos + __popcll(sb & lt_mask)] = base + lane;
        pos += __popcll(sb);
    }
}

__global__ void zero_words_kernel(uint32_t* w, size_t count, int32_t* status, int heads) {
    const size_t i = static_cast<size_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (i < count) w[i] = 0u;
    if (status && i < static_cast<size_t>(heads)) status[i] = 0;
}

struct SplitLayout {
    size_t hist_m[3], hist_c[3], state, chunk_cnt, redo, zero_bytes, total;
    int chunks;
};

SplitLayout split_layout(int heads, int64_t n) {
    SplitLayout w{};
    const size_t pr = static_cast<size_t>(heads) * 2;
    w.chunks = static_cast<int>((n + kChunk - 1) / kChunk);
    size_t off = 0;
    for (int i = 0; i < 3; ++i) {
        w.hist_m[i] = off;
        off += pr * 4096 * sizeof(u64);
    }
    for (int i = 0; i < 3; ++i) {
        w.hist_c[i] = off;
        off += pr * 4096 * sizeof(uint32_t);
    }
    w.redo = off;
    off = vs::round_up(off + pr * sizeof(int32_t), 256);
    w.zero_bytes = off;                                      // everything up to here starts at zero
    w.state = off;
    off = vs::round_up(off + pr * 4 * sizeof(SelState), 256);
    w.chunk_cnt = off;
    off = vs::round_up(off + pr * w.chunks * 3 * sizeof(uint32_t), 256);
    w.total = off;
    return w;
}

__global__ void zero_status_kernel(int32_t* status, int heads) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < heads) status[i] = 0;
}

}  // namespace

extern "C" {

size_t vs_select_budget_workspace(int heads, int64_t n) {
    if (heads <= 0 || n < kMinSplitN || n > VS_MAX_SEQ) return 0;   // one workgroup per problem: everything lives in LDS
    return split_layout(heads, n).total;
}

int vs_select_budget(const float* a_v, const float* a_s, int heads, int64_t n, const vs_budget_t* b, int32_t* idx_v,
                     int32_t* cnt_v, int32_t* idx_s, int32_t* cnt_s, int32_t* status, void* ws, size_t ws_bytes,
                     void* stream) {
    if (!a_v || !a_s || !b || !idx_v || !cnt_v || !idx_s || !cnt_s) return VS_ERR_INVALID_ARG;
    if (heads <= 0 || n <= 0) return VS_ERR_INVALID_ARG;
    if (n > VS_MAX_SEQ || heads > 65535) return VS_ERR_UNSUPPORTED;
    if (b->mode != 0 && b->mode != 1) return VS_ERR_INVALID_ARG;
    if (b->mode == 0 && !(b->tau_v >= 0.0 && b->tau_v <= 1.0 && b->tau_s >= 0.0 && b->tau_s <= 1.0)) return VS_ERR_INVALID_ARG;
    if (b->mode == 1 && (b->k_v < 0 || b->k_s < 0)) return VS_ERR_INVALID_ARG;
    if (b->n_sink < 0) return VS_ERR_INVALID_ARG;
    if (b->cap_v <= 0 || b->cap_s <= 0) return VS_ERR_CAPACITY;
    const int64_t forced_v = b->n_sink < n ? b->n_sink : n;
    const int64_t local = b->n_local < 1 ? 1 : b->n_local;
    const int64_t forced_s = local < n ? local : n;
    if (forced_v > b->cap_v || forced_s > b->cap_s) return VS_ERR_CAPACITY;

    SelParams p{};
    p.a[0] = a_v;
    p.a[1] = a_s;
    p.idx[0] = idx_v;
    p.idx[1] = idx_s;
    p.cnt[0] = cnt_v;
    p.cnt[1] = cnt_s;
    p.status = status;
    p.n = static_cast<int>(n);
    p.mode = b->mode;
    p.tau[0] = b->tau_v;
    p.tau[1] = b->tau_s;
    p.kfix[0] = b->k_v;
    p.kfix[1] = b->k_s;
    p.nforced[0] = static_cast<int>(forced_v);
    p.nforced[1] = static_cast<int>(forced_s);
    p.cap[0] = b->cap_v;
    p.cap[1] = b->cap_s;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (ws && n >= kMinSplitN) {
        const SplitLayout w = split_layout(heads, n);
        if (ws_bytes < w.total) return VS_ERR_WORKSPACE;
        if (!vs::aligned16(ws)) return VS_ERR_INVALID_ARG;
        unsigned char* base = static_cast<unsigned char*>(ws);
        SplitParams q{};
        q.s = p;
        q.chunks = w.chunks;
        for (int i = 0; i < 3; ++i) {
            q.hist_m[i] = reinterpret_cast<u64*>(base + w.hist_m[i]);
            q.hist_c[i] = reinterpret_cast<uint32_t*>(base + w.hist_c[i]);
        }
        q.state = reinterpret_cast<SelState*>(base + w.state);
        q.chunk_cnt = reinterpret_cast<uint32_t*>(base + w.chunk_cnt);
        q.redo = reinterpret_cast<int32_t*>(base + w.redo);
        const size_t words = w.zero_bytes / 4;                  // (more words than heads: the status words ride along)
        hipLaunchKernelGGL(zero_words_kernel, dim3(static_cast<unsigned>((words + 255) / 256)), dim3(256), 0, st,
                           reinterpret_cast<uint32_t*>(base), words, status, heads);
        VS_LAUNCH_CHECK();
        const dim3 grid(w.chunks, heads, 2);
        hipLaunchKernelGGL(split_pass_kernel<0>, grid, dim3(kChunkThreads), 0, st, q);
        VS_LAUNCH_CHECK();
        hipLaunchKernelGGL(split_pass_kernel<1>, grid, dim3(kChunkThreads), 0, st, q);
        VS_LAUNCH_CHECK();
        hipLaunchKernelGGL(split_pass_kernel<2>, grid, dim3(kChunkThreads), 0, st, q);
        VS_LAUNCH_CHECK();
        hipLaunchKernelGGL(split_pass_kernel<3>, grid, dim3(kChunkThreads), 0, st, q);
        VS_LAUNCH_CHECK();
        hipLaunchKernelGGL(split_emit_kernel, grid, dim3(kChunkThreads), 0, st, q);
        VS_LAUNCH_CHECK();
        hipLaunchKernelGGL(select_kernel, dim3(heads, 2), dim3(kSelThreads), 0, st, p, static_cast<const int32_t*>(q.redo));
        VS_LAUNCH_CHECK();
        return VS_OK;
    }
    if (status) {
        hipLaunchKernelGGL(zero_status_kernel, dim3((heads + 255) / 256), dim3(256), 0, st, status, heads);
        VS_LAUNCH_CHECK();
    }
    hipLaunchKernelGGL(select_kernel, dim3(heads, 2), dim3(kSelThreads), 0, st, p, static_cast<const int32_t*>(nullptr));
    VS_LAUNCH_CHECK();
    return VS_OK;
}

}  // extern "C"
