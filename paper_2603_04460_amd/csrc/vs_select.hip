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

__global__ __launch_bounds__(kSelThreads) void select_kernel(const SelParams p) {
    __shared__ SelShared sh;
    const int head = blockIdx.x, dir = blockIdx.y;
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

__global__ void zero_status_kernel(int32_t* status, int heads) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < heads) status[i] = 0;
}

}  // namespace

extern "C" {

size_t vs_select_budget_workspace(int heads, int64_t n) {
    (void)heads;
    (void)n;
    return 0;   // histograms and ranks live in LDS
}

int vs_select_budget(const float* a_v, const float* a_s, int heads, int64_t n, const vs_budget_t* b, int32_t* idx_v,
                     int32_t* cnt_v, int32_t* idx_s, int32_t* cnt_s, int32_t* status, void* ws, size_t ws_bytes,
                     void* stream) {
    (void)ws;
    (void)ws_bytes;
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
    if (status) {
        hipLaunchKernelGGL(zero_status_kernel, dim3((heads + 255) / 256), dim3(256), 0, st, status, heads);
        VS_LAUNCH_CHECK();
    }
    hipLaunchKernelGGL(select_kernel, dim3(heads, 2), dim3(kSelThreads), 0, st, p);
    VS_LAUNCH_CHECK();
    return VS_OK;
}

}  // extern "C"
