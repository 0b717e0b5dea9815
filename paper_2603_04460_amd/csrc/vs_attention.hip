// Causal vertical-slash sparse attention for gfx950.
//
// One workgroup (4 wavefronts, one per SIMD) owns a query tile of one KV head: 4 row blocks of 32
// query rows, arranged as hc query heads of the KV group times 4/hc consecutive 32-row sub-blocks
// (hc = 4 for the 4:1 GQA layers: a 32-row tile of all four heads).  K / V tiles are staged once in
// LDS for all four row blocks.  Each wavefront owns one row block.  A workgroup stays under 80 KB of
// LDS and 256 registers per lane, so that TWO workgroups share a compute unit: per unit of work the
// set-up (index merge, lists) is a chain of memory round trips and barriers during which a workgroup
// issues little, and the other workgroup's tile loop runs meanwhile; in steady state the two
// wavefronts of a SIMD (one per workgroup) overlap softmax and matrix instructions.
//
// Scores are computed transposed, S^T = K Q^T, with v_mfma_f32_32x32x16_bf16: a lane then holds
// 16 keys of ONE query, which makes the row maximum a 16-way in-lane reduction plus one
// half-wave swap, and makes the S^T accumulator directly usable as the B operand (P^T) of the
// second product O^T = V^T P^T.  V^T fragments come from LDS through the transposing read.
//
// Sparse path (Sec. "Fused attention kernel implementation" of the paper: indices read per query
// tile, merged on the fly, keys fetched on demand).  The slash part of the mask is shift-invariant: a
// selected offset o crosses key block b for the 32-row block t exactly when it crosses block b + 1
// for t + 1.  So one small kernel prepares, once per call and index head, the ascending list of
// "block diagonals" delta = t - b that any selected offset crosses, with the 63-bit window of the
// offset bitmap that belongs to each (it depends on delta only), plus the column bitmap.  Per query
// tile the workgroup then
//   1. lists the key blocks first_block(tile) - delta, delta <= first_block(tile): the merged
//      contiguous key ranges of the slash part; each comes with its window and its column word,
//   2. takes the leading entries of the sorted column list that are causal for the tile: the gather
//      list.  A key that is both a selected column and reached by a selected offset belongs to the
//      gather list only: the block tiles drop the listed columns (the deduplication),
//   3. streams the listed blocks (coalesced rows) and the gathered columns (row gathers) through
//      LDS and runs online-softmax attention on them.  The exact element mask of a block tile,
//          live(i, j) = j <= i and offset i-j selected and column j not selected,
//      is the 63-bit window and the 32-bit column word, both wave-uniform (SGPRs).  Each lane shifts
//      the window by its own query row, which leaves the keep-bits of its 16 accumulator elements in
//      one register; an element then costs a bit-field extract and a bitwise select.  Tiles whose
//      window is all ones and whose column word is empty skip the mask, row blocks whose window is
//      empty skip the tile.  A gathered tile needs a mask (column <= row) only in the one or two
//      stages that straddle the row block's first row.
//
// Staging: K / V rows go from global memory straight into LDS (global_load_lds_dwordx4: no staging registers, no LDS
// store instructions).  Two stage buffers: the loads of stage s+1 are issued at the top of step s, after its barrier,
// into the buffer that stage s-1 has just left; each wavefront waits for its own loads (vmcnt) before the barrier that
// opens step s+1, which publishes them.  Loads are never predicated: rows that do not exist read another row, whose
// scores are masked.
#include <hip/hip_runtime.h>
#include <limits.h>
#include <math.h>
#include <stdint.h>

#include <mutex>
#include <type_traits>

#include "vs_attn_device.h"
#include "vs_device.h"

namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;
constexpr int kRing = 4;                       // ring of two stages of two tiles
constexpr int kListCap = 128;                  // block list: kListCap / nsub entries per pass
constexpr int kLdsBudget = 80 * 1024;          // per workgroup: two of them share the 160 KB of a compute unit
// LDS: ring | tile records per (sub-block, listed block) | scratch | gather list (entries per pass)
constexpr int kGatherCap = 2432;
constexpr int kRecPad = 4;                     // dead records after a sub-block's last listed block (a step looks one stage ahead)
constexpr size_t kListRecOff = kRing * kSlotBytes;           // 16-byte tile record per (sub-block, listed block)
constexpr size_t kScratchOff = kListRecOff + (kListCap + 4 * kRecPad) * 16;
constexpr size_t kGatherOff = kScratchOff + 128;
constexpr size_t kLdsBytes = kGatherOff + kGatherCap * 4;
static_assert(kLdsBytes <= kLdsBudget, "two workgroups per compute unit");
static_assert(kGatherCap % 64 == 0, "whole stages");

// (the second launch bound caps the registers at 256 per lane, i.e. two wavefronts per SIMD: without it the compiler
// takes accumulation registers for its spills and only one workgroup fits a compute unit)
__global__ __launch_bounds__(kThreads, 2) void vs_attention_kernel(const AttnParams p) {
    extern __shared__ __align__(16) unsigned char smem[];
    unsigned char* const kvbuf = smem;
    uint4* const list_rec = reinterpret_cast<uint4*>(smem + kListRecOff);
    int* const wtot = reinterpret_cast<int*>(smem + kScratchOff);
    int* const glist = reinterpret_cast<int*>(smem + kGatherOff);

    const float NEG_INF = -INFINITY;

    // ---- which unit of work: (query tile, KV head, chunk of the group's query heads) ----
    // Persistent launch: two workgroups per compute unit take units from counters in the workspace until none is
    // left.  With one workgroup per unit the hardware dispatcher left a compute unit idle for ~20 us between two
    // large workgroups (measured with 160 KB / 512 threads: 23 % of the kernel at 128k).  There is
    // one queue of units per KV head.  A workgroup starts in the queue of head (its XCD number) % kv_heads, so an XCD's
    // L2 mostly sees one head's K / V, and moves on to the next queue when its own is empty, so that heads with a
    // larger budget do not become the critical path.  Every wavefront leaves the loop at the same point.  (Without
    // counters, more than 32 KV heads: one workgroup per unit, heads rotated over the XCDs.)
    int bid = blockIdx.x;
    int queue = 0;
    // statistics of this workgroup over all its units, added to the workspace counters once, at the end: one atomic per
    // unit on the same three words from every workgroup of the chip serialises in the memory system (measured: a floor
    // of 75 ns per unit of work, 2.4 ms at 128k, whatever the unit's size)
    unsigned int tiles_done = 0, staged_gather = 0, staged_block = 0;
    const int units_per_head = p.work_total / p.kv_heads;
    if (p.work_counter) {
        queue = static_cast<int>(__builtin_amdgcn_s_getreg((20) | (0 << 6) | (3 << 11)) & 0xf) % p.kv_heads;   // XCC_ID
        bid = -1;
    }
    for (;;) {
    if (p.work_counter) {
        __syncthreads();                                     // LDS and the slots below are free again
        if (threadIdx.x == 0) {
            int q = queue, unit = -1;
            for (int t = 0; t < p.kv_heads; ++t) {
                const int u = static_cast<int>(atomicAdd(p.work_counter + q, 1u));
                if (u < units_per_head) {
                    unit = u;
                    break;
                }
                q = q + 1 == p.kv_heads ? 0 : q + 1;
            }
            wtot[31] = unit;
            wtot[30] = q;
        }
        __syncthreads();
        queue = __builtin_amdgcn_readfirstlane(wtot[30]);
        const int unit = __builtin_amdgcn_readfirstlane(wtot[31]);
        if (unit < 0) break;
        bid = unit * p.kv_heads;                             // rest = unit; the head comes from the queue
    }
    if (bid >= p.work_total) break;
    // The thread number is made opaque once per unit: every per-thread constant below is then recomputed per unit
    // instead of being carried (and spilled) across the register-hungry loops of the previous unit.
    int tid = threadIdx.x;
    asm volatile("" : "+v"(tid));
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int qi = lane & 31, hh = lane >> 5;
    const int rest = bid / p.kv_heads;
    const int g = p.work_counter ? queue : (bid + rest) % p.kv_heads;
    const int hchunks = p.group / p.hc;
    const int hchunk = rest % hchunks;
    const int tile = p.tiles - 1 - rest / hchunks;          // longest tiles first
    const int BQ = 32 * kWaves / p.hc;
    const int nsub = BQ >> 5;
    const int i0 = p.pos0 + tile * BQ;                      // positions are absolute; the tile grid starts at the chunk
    const int n = p.n;                                      // keys
    const int n_pos = p.pos0 + p.nq;                        // positions that exist
    const int i_last = min(i0 + BQ, n_pos) - 1;

    // this wavefront's row block: 32 rows of one query head
    const int my_head = g * p.group + hchunk * p.hc + wave % p.hc;
    const int my_i0 = i0 + 32 * (wave / p.hc);
    const bool my_rows = my_i0 < n_pos;
    const int ih = p.index_per_q ? my_head : g;
    const uint32_t* __restrict__ vbit = p.vbit + static_cast<size_t>(ih) * p.vw;

    const uint16_t* __restrict__ kbase = p.k + static_cast<size_t>(g) * n * kD;
    const uint16_t* __restrict__ vbase = p.v + static_cast<size_t>(g) * n * kD;

    // ---- Q fragments: B operand of S^T = K Q^T; lane holds query qi, d = 16 kk + 8 hh .. +7 ----
    bf16x8 qf[8];
    {
        const int row = my_i0 + qi;
        const uint16_t* src = p.q + (static_cast<size_t>(my_head) * p.nq + (min(row, n_pos - 1) - p.pos0)) * kD + 8 * hh;
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) {
            uint4 raw = make_uint4(0, 0, 0, 0);
            if (row < n_pos) raw = *reinterpret_cast<const uint4*>(src + 16 * kk);
            qf[kk] = __builtin_bit_cast(bf16x8, raw);
        }
    }

    f32x16 oacc[4];
    float m_run = NEG_INF, l_run = 0.f;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int e = 0; e < 16; ++e) oacc[db][e] = 0.f;

    // ---- staging: a stage is two 32-key tiles; a thread moves one 16-byte chunk of rows st_row and st_row + 16 of K and V of each ----
    const int st_row = tid >> 4;
    // thread (wavefront w, lane L) fills piece L of groups w and w + 4 of a tile: rows 4w + L/16 (= st_row) and 16 more;
    // which 16-byte chunk of the row that piece holds follows from the rotations above
    typedef const __attribute__((address_space(1))) void* gptr_t;
    typedef __attribute__((address_space(3))) void* lptr_t;
    const int st_rho = (lane >> 4) & 3;
    const int st_ck = 4 * ((lane >> 2) & 3) + (((lane & 3) - st_rho) & 3);          // K chunk of this piece
    const int st_cv = 4 * ((((lane >> 2) & 3) - st_rho) & 3) + (lane & 3);          // V chunk of this piece
    // buf: which of the two stage buffers.  The loads complete in the background (vmcnt).
    // The head's K / V base is wave-uniform; a thread adds a 32-bit byte offset: row * 256 + its chunk (n <= 2^20 rows).
    const uint32_t st_bk = static_cast<uint32_t>(st_ck * 16), st_bv = static_cast<uint32_t>(st_cv * 16);
    auto load_stage = [&](const int (&rows)[2][2], int buf) __attribute__((always_inline)) {
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                unsigned char* dst = kvbuf + (2 * buf + u) * kSlotBytes + (wave + kWaves * h) * kGroupBytes;
                const uint32_t off = static_cast<uint32_t>(rows[u][h]) << 8;
                lds_load16s(off + st_bk, kbase, dst);
                lds_load16s(off + st_bv, vbase, dst + kTileBytes);
            }
    };

    // ---- pieces of one (row block, 32-key tile) unit ----
    const int li = lane & 15, dsel = (lane >> 4) & 1;
    // K fragment kk: chunk 2 kk + hh of row qi -> 64 (kk / 2) + 16 ((2 kk + hh + qi) % 4): two per-lane bases (kk even / odd)
    const int k_row = (qi >> 2) * kGroupBytes + (qi & 3) * 256;
    const int k_off0 = k_row + 16 * ((hh + qi) & 3), k_off2 = k_row + 16 * ((hh + qi + 2) & 3);
    // V fragment j: rows 4 hh + li / 4 + 16 (j % 2) (+ 8), bytes 64 (j / 2) + 32 dsel + 8 (li % 4) .. + 7
    const int v_rho = (li >> 2) & 3;
    const int v_lane = kTileBytes + hh * kGroupBytes + v_rho * 256 + 32 * dsel + 8 * (li & 3);
    int v_off[4];
#pragma unroll
    for (int sgr = 0; sgr < 4; ++sgr) v_off[sgr] = v_lane + 64 * ((sgr + v_rho) & 3);
    typedef __attribute__((address_space(3))) bf16x4t* lds_ptr_t;
    // slot: which of the four tile slots (wave-uniform)
    auto read_k = [&](int slot, bf16x8 (&kf)[8]) __attribute__((always_inline)) {
        const unsigned char* kt = kvbuf + slot * kSlotBytes;
#pragma unroll
        for (int kk = 0; kk < 8; ++kk)
            kf[kk] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(kt + ((kk & 1) ? k_off2 : k_off0) + 64 * (kk >> 1)));
    };
    // transposing LDS read: within 16 lanes, lane i addresses row i/4, 4 columns at 4 (i%4); it receives column i of
    // those 4 rows, i.e. 4 consecutive keys of one d
    auto read_v = [&](int slot, bf16x8 (&vf)[8]) __attribute__((always_inline)) {
        const unsigned char* va = kvbuf + slot * kSlotBytes;
#pragma unroll
        for (int j = 0; j < 8; ++j) {                      // j = 2 db + t16: d block db, keys 16 t16 ..
            const unsigned char* a0 = va + v_off[j >> 1] + 4 * (j & 1) * kGroupBytes;
            const bf16x4t lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_ptr_t)(a0));
            const bf16x4t hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_ptr_t)(a0 + 2 * kGroupBytes));
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                vf[j][e] = lo[e];
                vf[j][4 + e] = hi[e];
            }
        }
    };
    auto tile_max = [&](const f32x16& acc) __attribute__((always_inline)) -> float {
        float mx = fmaxf(fmaxf(acc[0], acc[1]), acc[2]);
#pragma unroll
        for (int e = 3; e < 15; e += 2) mx = fmaxf(fmaxf(mx, acc[e]), acc[e + 1]);
        return fmaxf(mx, acc[15]);
    };
    auto rescale = [&](float m_new) __attribute__((always_inline)) {
        const float alpha = (m_new == NEG_INF) ? 1.f : __builtin_amdgcn_exp2f((m_run - m_new) * p.c);
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int e = 0; e < 16; ++e) oacc[db][e] *= alpha;
        l_run *= alpha;
        m_run = m_new;
    };
    // p = exp2(c s - c m) for elements [E0, E1) of acc, row sum into lsum
    auto exp_part = [&](f32x16& acc, int e0, int e1, float mc, float& lsum) __attribute__((always_inline)) {
#pragma unroll
        for (int e = e0; e < e1; ++e) {
            acc[e] = __builtin_amdgcn_exp2f(fmaf(acc[e], p.c, -mc));
            lsum += acc[e];
        }
    };
    auto pack_p = [&](const f32x16& acc, bf16x8 (&pb)[2]) __attribute__((always_inline)) {
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int e = 0; e < 8; e += 2) {
                const f32x2 two = {acc[8 * t + e], acc[8 * t + e + 1]};
                const bf16x2 r = __builtin_convertvector(two, bf16x2);
                pb[t][e] = r[0];
                pb[t][e + 1] = r[1];
            }
    };

    // per-wavefront description of a tile: live (anything kept for this row block), need (a mask is required)
    struct TileInfo {
        bool live, need;
        const uint4* rec;        // contiguous tile: its record in LDS
        const int* cols;         // gathered tile: its 32 column numbers in LDS
    };
    const int bcap = kListCap / nsub;                        // listed blocks per round
    const int my_sub = wave / p.hc;
    // Tile record of a listed block for one 32-row sub-block, made once per unit by the thread that lists the block, so
    // that a step of the tile loop reads one flag word (scalar instructions cost this loop as much as vector ones):
    //   x, y: 64-bit window wz; lane (q, h) keeps key kj iff bit 31 + q - kj of wz is set and bit kj of kw (word z) is:
    //         element-exact mode: wz = selected offsets dlt-31 .. dlt+31, kw = columns not listed
    //         tile-granular mode: wz = causal offsets, kw = keys that some row of the block reaches through a selected
    //         offset, listed columns taken out
    //   w: bit 0 live, bit 1 a mask is needed, bits 2..: the key block (so that one word per tile tells a step all it
    //      needs for the staging loads and the tests; the rest is read only where a mask is applied)
    // sub_i0: first row of the sub-block; b: key block; w: the offset window prepared with the diagonal list; xw: the block's
    // column word
    auto make_record = [&](int sub_i0, int b, uint64_t w, uint32_t xw) __attribute__((always_inline)) -> uint4 {
        const int dlt = sub_i0 - 32 * b;                     // offset of (row 0, key 0) of the 32x32 tile
        uint64_t wz = w;
        uint32_t kw = ~xw;
        bool live = w != 0ull, need = w != kAll63 || xw != 0u;
        if (p.gran == 32) {
            // Tile-granular slash: key kj is kept for every causal row of this 32-row block if ANY of its rows reaches it
            // through a selected offset, i.e. if the window has a bit in [31 - kj, 62 - kj].
            // x bit s = OR of window bits s .. s+len-1, len = rows of this block that exist (32 except at the end of
            // the sequence): doubling up to the largest power of two pw <= len, then two overlapping windows
            const int len = max(1, min(32, n_pos - sub_i0));
            uint64_t x = w;
            int pw = 1;
            while (2 * pw <= len) {
                x |= x >> pw;
                pw *= 2;
            }
            x |= x >> (len - pw);
            wz = dlt >= 31 ? kAll63 : (dlt < -31 ? 0ull : ((kAll63 << (31 - dlt)) & kAll63));   // offsets >= 0
            kw = __builtin_bitreverse32(static_cast<uint32_t>(x)) & ~xw;
            live = kw != 0u && wz != 0ull;
            need = !(kw == 0xffffffffu && wz == kAll63);
        }
        if (dlt < -31 || sub_i0 >= n_pos) live = false;      // every key lies after every row / padding rows
        return make_uint4(static_cast<uint32_t>(wz), static_cast<uint32_t>(wz >> 32), kw,
                          (live ? 1u : 0u) | (need ? 2u : 0u) | (static_cast<uint32_t>(b) << 2));
    };
    const int rcap = bcap + kRecPad;                         // records per sub-block
    const uint4* const my_rec = list_rec + my_sub * rcap;
    // t: position in the block list; d: word w of its record
    auto block_info = [&](int t, uint32_t d) __attribute__((always_inline)) -> TileInfo {
        const uint32_t fl = static_cast<uint32_t>(__builtin_amdgcn_readfirstlane(d));
        return TileInfo{(fl & 1u) != 0u, (fl & 2u) != 0u, my_rec + t, nullptr};
    };
    auto gather_info = [&](const int* cols) __attribute__((always_inline)) -> TileInfo {
        TileInfo ti{false, false, nullptr, cols};
        const int cmin = cols[0], cmax = cols[31];           // ascending, INT_MAX padding
        ti.live = my_rows && cmin <= my_i0 + 31;
        ti.need = cmax > my_i0;
        return ti;
    };
    auto apply_mask = [&](f32x16& acc, const TileInfo& ti, auto gather_tag) __attribute__((always_inline)) {
        if (!ti.need) return;
        if constexpr (decltype(gather_tag)::value) {
            const int row = my_i0 + qi;
#pragma unroll
            for (int a = 0; a < 4; ++a) {
                const int4 c4 = *reinterpret_cast<const int4*>(ti.cols + 8 * a + 4 * hh);
                if (c4.x > row) acc[4 * a] = NEG_INF;
                if (c4.y > row) acc[4 * a + 1] = NEG_INF;
                if (c4.z > row) acc[4 * a + 2] = NEG_INF;
                if (c4.w > row) acc[4 * a + 3] = NEG_INF;
            }
        } else {
            const uint4 r = *ti.rec;                         // one broadcast read
            const uint64_t wz = (static_cast<uint64_t>(r.y) << 32) | r.x;
            const uint32_t keep = static_cast<uint32_t>(wz >> (qi + 4 - 4 * hh)) & (__builtin_bitreverse32(r.z) >> (4 - 4 * hh));
            mask_elements<0>(acc, keep, __float_as_uint(NEG_INF));
        }
    };

    // ---- pipeline over the tiles of one phase ----
    // GATHER == false: tile t is the key block of record t;  GATHER == true: tile t is glist[32 t .. 32 t + 31].
    // A stage is two tiles (64 keys).  Two stages live in LDS: step s computes on stage s and refills the buffer of
    // stage s-1 with stage s+1, whose global loads are started at the top of the step.  One barrier per step.  The two
    // tiles of a stage go through one softmax (one row maximum, one rescale decision) and their matrix products are
    // issued as independent chains.
    // nfull: leading stages in which this wavefront's row block keeps every key of both tiles (no mask, nothing to skip)
    // primed: stage 0 of this phase was requested by the previous phase's last step (into the buffer it had free);
    // chain: this (block) phase is followed by a gather phase whose list is ready, so its last step requests that phase's
    // stage 0 and the pipeline does not drain between the two.
    int buf = 0;                                             // buffer of the current stage; the next stage goes to the other one
    auto run_phase = [&](int ntiles, auto gather_tag, int nfull, bool primed, bool chain) __attribute__((always_inline)) {
        constexpr bool GATHER = decltype(gather_tag)::value;
        if (ntiles == 0) return;
        const int nstages = (ntiles + 1) >> 1;
        if (GATHER) staged_gather += static_cast<unsigned int>(ntiles);   // 32-key tiles this workgroup stages in LDS
        else staged_block += static_cast<unsigned int>(ntiles);
        // Descriptor words of the two tiles of stage st (block phase): one LDS instruction; the records are padded with dead
        // entries, so a stage past the list reads as "not live, block 0".
        auto stage_desc = [&](int st, uint32_t (&d)[2]) __attribute__((always_inline)) {
            d[0] = d[1] = 0u;
            if constexpr (!GATHER) {
                d[0] = my_rec[2 * st].w;
                d[1] = my_rec[2 * st + 1].w;
            }
        };
        // rows past the sequence and tiles past the list read another row instead: their scores are masked, so the loads
        // need no predicate
        auto stage_rows = [&](int st, const uint32_t (&d)[2], int (&rows)[2][2]) __attribute__((always_inline)) {
#pragma unroll
            for (int u = 0; u < 2; ++u)
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const int r = st_row + 16 * h;
                    if (GATHER) rows[u][h] = min(glist[32 * (2 * st + u) + r], n - 1);   // padded with INT_MAX to a whole stage
                    else rows[u][h] = min(static_cast<int>(d[u] >> 2) * 32 + r, n - 1);
                }
        };
        auto info = [&](int t, uint32_t d) __attribute__((always_inline)) -> TileInfo {
            if (GATHER) {
                if (t >= ntiles) return TileInfo{false, false, nullptr, nullptr};
                return gather_info(glist + 32 * t);
            }
            return block_info(t, d);
        };
        // Every vector memory load issued so far (the Q fragments) is waited for here, once.  Left pending, the first
        // use of Q inside the loop would wait for "all loads", including the staging loads issued just before it.
        __builtin_amdgcn_s_waitcnt(0x0F70);                  // vmcnt(0), other counters untouched
        int rows[2][2];
        uint32_t d0[2];
        stage_desc(0, d0);
        if (!primed) {
            stage_rows(0, d0, rows);
            load_stage(rows, buf);
            __builtin_amdgcn_s_waitcnt(0x0F70);              // the barrier publishes only what has arrived
        }
        __syncthreads();
        nfull = min(nfull, nstages);
        TileInfo a{false, false, nullptr, nullptr}, b = a;
        if (nfull == 0) {
            a = info(0, d0[0]);
            b = info(1, d0[1]);
        }
        auto pv = [&](const bf16x8 (&pk)[2], const bf16x8 (&vf)[8]) __attribute__((always_inline)) {
#pragma unroll
            for (int t = 0; t < 2; ++t)                      // the four d-blocks in turn: consecutive MFMAs are independent
#pragma unroll
                for (int db = 0; db < 4; ++db) oacc[db] = mfma32(vf[2 * db + t], pk[t], oacc[db]);
        };
        // one step
        // FULL: both tiles are kept whole by this row block: no tile descriptions, no masks, no tests
        auto step = [&](int st, auto mode_tag) __attribute__((always_inline)) {
            constexpr int MODE = decltype(mode_tag)::value;
            constexpr bool FULL = MODE == 0;
            if (st > 0) {
                __builtin_amdgcn_s_waitcnt(0x0F70);          // this wavefront's part of stage st has arrived
                __syncthreads();
            }
            const int buf1 = buf ^ 1;
            // list / bitmap words of the next stage are requested before the staging loads: the memory counters retire
            // in order, so waiting for them does not wait for the (younger) staging loads
            TileInfo na{false, false, nullptr, nullptr}, nb = na;
            uint32_t d[2];
            stage_desc(st + 1, d);
            if constexpr (!FULL) {
                na = info(2 * st + 2, d[0]);
                nb = info(2 * st + 3, d[1]);
            }
            const bool more = st + 1 < nstages;
            if (more) {                                      // into the buffer of stage st-1, free since the barrier
                stage_rows(st + 1, d, rows);
                load_stage(rows, buf1);
            } else if (!GATHER && chain) {                   // first stage of the gather phase that follows
#pragma unroll
                for (int u = 0; u < 2; ++u)
#pragma unroll
                    for (int h = 0; h < 2; ++h) rows[u][h] = min(glist[32 * u + st_row + 16 * h], n - 1);
                load_stage(rows, buf1);
            }
            if constexpr (MODE != 2) {
                // Both tiles live: one straight-line piece in a fixed order (the scheduling barriers keep the compiler from
                // moving LDS reads across them: left alone it either hoists all of them, which does not fit the registers,
                // or issues them one at a time in front of their use).  The K fragments of both tiles are read first, the
                // two score chains are interleaved, the V fragments of both tiles are requested as soon as the K fragments
                // are dead (they take their registers) and arrive during the softmax.
                bf16x8 k0[8], k1[8], v0[8], v1[8], p0[2], p1[2];
                f32x16 s0, s1, zero;
#pragma unroll
                for (int e = 0; e < 16; ++e) zero[e] = 0.f;
                read_k(2 * buf, k0);
                read_k(2 * buf + 1, k1);
                tiles_done += 2;
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int kk = 0; kk < 8; ++kk) {
                    s0 = mfma32(k0[kk], qf[kk], kk == 0 ? zero : s0);
                    s1 = mfma32(k1[kk], qf[kk], kk == 0 ? zero : s1);
                }
                __builtin_amdgcn_sched_barrier(0);
                read_v(2 * buf, v0);
                read_v(2 * buf + 1, v1);
                __builtin_amdgcn_sched_barrier(0);
                if constexpr (!FULL) {
                    apply_mask(s0, a, gather_tag);
                    apply_mask(s1, b, gather_tag);
                }
                const float mx = fmaxf(tile_max(s0), tile_max(s1));
                const float m_new = fmaxf(m_run, half_swap_max(mx));
                if (__ballot((m_new - m_run) * p.c > kRescaleThreshold)) rescale(m_new);   // false when both are -inf
                const float mc = (m_run == NEG_INF) ? 0.f : m_run * p.c;
                float lsum = 0.f;
                exp_part(s0, 0, 16, mc, lsum);
                pack_p(s0, p0);
                exp_part(s1, 0, 16, mc, lsum);
                pack_p(s1, p1);
                l_run += lsum;
                pv(p0, v0);
                pv(p1, v1);
            } else {
            // scores of the two tiles: defined only where the tile is live (every later use is under the same test), so
            // that no registers are cleared for tiles that are skipped
            bf16x8 k0[8], k1[8], vf[8], p0[2], p1[2];       // (local to the step: nothing is carried round the loop)
            f32x16 s0, s1, zero;
#pragma unroll
            for (int e = 0; e < 16; ++e) zero[e] = 0.f;
            // one chain after the other; the second tile's fragments are requested before the first chain starts
            const bool alive = a.live, blive = b.live;
            if (alive) read_k(2 * buf, k0);
            if (blive) read_k(2 * buf + 1, k1);
            if (alive) {
                ++tiles_done;
#pragma unroll
                for (int kk = 0; kk < 8; ++kk) s0 = mfma32(k0[kk], qf[kk], kk == 0 ? zero : s0);
            }
            if (blive) {
                ++tiles_done;
#pragma unroll
                for (int kk = 0; kk < 8; ++kk) s1 = mfma32(k1[kk], qf[kk], kk == 0 ? zero : s1);
            }
            if (alive || blive) {
                float mx = NEG_INF;
                if (alive) {
                    apply_mask(s0, a, gather_tag);
                    mx = tile_max(s0);
                }
                if (blive) {
                    apply_mask(s1, b, gather_tag);
                    mx = fmaxf(mx, tile_max(s1));
                }
                const float m_new = fmaxf(m_run, half_swap_max(mx));
                if (__ballot((m_new - m_run) * p.c > kRescaleThreshold)) rescale(m_new);   // false when both are -inf
                const float mc = (m_run == NEG_INF) ? 0.f : m_run * p.c;
                float lsum = 0.f;
                if (alive) {
                    exp_part(s0, 0, 16, mc, lsum);
                    pack_p(s0, p0);
                }
                if (blive) {
                    exp_part(s1, 0, 16, mc, lsum);
                    pack_p(s1, p1);
                }
                l_run += lsum;
                if (alive) {
                    read_v(2 * buf, vf);
                    pv(p0, vf);
                }
                if (blive) {
                    read_v(2 * buf + 1, vf);
                    pv(p1, vf);
                }
            }
            }
            a = na;
            b = nb;
            buf = buf1;
        };
        int st = 0;
        for (; st < nfull; ++st) step(st, std::integral_constant<int, 0>{});
        if (st > 0 && st < nstages) {
            stage_desc(st, d0);
            a = info(2 * st, d0[0]);
            b = info(2 * st + 1, d0[1]);
        }
        while (st < nstages) {
            if (a.live && b.live) {
                do {
                    step(st, std::integral_constant<int, 1>{});
                    ++st;
                } while (st < nstages && a.live && b.live);
            } else {
                step(st, std::integral_constant<int, 2>{});
                ++st;
            }
        }
        if (!(!GATHER && chain)) {
            __syncthreads();                                 // the ring and the list are reused by the next phase
            buf = 0;
        }
    };

    // ---- phases ----
    {
        const int qb0 = i0 >> 5;                             // first 32-row block of the tile
        const int32_t* __restrict__ iv = p.idx_v + static_cast<size_t>(ih) * p.cap_v;
        const int32_t* __restrict__ ncol = p.ncol32 + static_cast<size_t>(ih) * p.nq32;
        const int32_t* __restrict__ dl = p.dlist + static_cast<size_t>(ih) * p.dcap;
        const unsigned long long* __restrict__ wl = p.wlist + static_cast<size_t>(ih) * p.dcap * 4;
        // slash part: the listed block diagonals <= qb0;  vertical part: the listed columns <= i_last (negative entries,
        // a prefix of the ascending list, are skipped)
        const int ndiag = p.ndiag[static_cast<size_t>(ih) * p.nq32 + qb0];
        const int ncand = ncol[i_last >> 5];
        int cursor = min(p.vfirst[ih], ncand);
        // columns before this row block's first row: every row of the block keeps them (no mask in their stages)
        const int nbefore = (my_rows && my_i0 >= 32) ? __builtin_amdgcn_readfirstlane(ncol[(my_i0 >> 5) - 1]) : 0;
        // One round of the gather list: the next kGatherCap causal columns, copied as they are (ascending), padded with
        // INT_MAX to a whole stage.  Returns the number of columns; sets first to the list position of the round's start.
        int first = 0;
        auto gather_round = [&]() -> int {
            const int count = min(ncand - cursor, kGatherCap);
            for (int t = tid; t < count; t += kThreads) glist[t] = iv[cursor + t];
            const int padded = (count + 63) & ~63;
            for (int t = count + tid; t < padded; t += kThreads) glist[t] = INT_MAX;
            first = cursor;
            cursor += count;
            __syncthreads();
            return count;
        };
        // 1. slash part: key blocks qb0 - delta in the order of the diagonal list (nearest block first), in rounds of bcap
        //    blocks.  Each listed block gets its column word and, per 32-row sub-block of the tile, its offset window.
        //    The first round of the gather list is copied with the first block round (one barrier for both).
        int gcount = -1;
        bool chained = false;
        for (int rbase = 0; rbase < ndiag; rbase += bcap) {
            const int count = min(bcap, ndiag - rbase);
            if (tid < count) {                               // bcap < kThreads: one entry per thread
                const int e = tid;
                const int b = qb0 - dl[rbase + e];
                const uint32_t xw = vbit[b];
                for (int r = 0; r < nsub; ++r)
                    list_rec[r * rcap + e] = make_record(i0 + 32 * r, b, wl[static_cast<size_t>(rbase + e) * 4 + r], xw);
            } else if (tid < count + kRecPad) {
                for (int r = 0; r < nsub; ++r) list_rec[r * rcap + tid] = make_uint4(0u, 0u, 0u, 0u);
            }
            if (gcount < 0) gcount = gather_round();         // ends with a barrier
            else __syncthreads();
            chained = rbase + bcap >= ndiag && gcount > 0;   // last block round, and a gather phase follows
            run_phase(count, std::false_type{}, 0, false, chained);
        }
        // 2. vertical part: the causal columns, gathered row by row
        if (gcount < 0) gcount = gather_round();
        while (true) {
            const int nfull = max(0, min(nbefore - first, gcount)) >> 6;
            run_phase((gcount + 31) >> 5, std::true_type{}, nfull, chained, false);
            chained = false;
            if (cursor >= ncand) break;
            gcount = gather_round();
        }
    }

    // ---- epilogue: O = O^T / l in bf16; lse = m * scale + ln(l) ----
    // A lane holds 8-byte pieces of one output row; stored directly they would be 64 scattered pieces per instruction.
    // The row block goes through the wavefront's own 8.5 KB of the (now idle) ring instead: written as held, read back
    // 16 bytes per lane, so that 16 lanes store one whole 256-byte row and an instruction stores four rows.
    {
        const float l_tot = half_swap_sum(l_run);
        const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
        constexpr int kPitch = 256 + 16;                     // row pitch in LDS: 16-byte aligned, spreads the rows over the banks
        static_assert(32 * kPitch <= kTileBytes && kWaves * kTileBytes <= kRing * kSlotBytes, "staging area of the epilogue");
        unsigned char* const stage = kvbuf + wave * kTileBytes;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int a = 0; a < 4; ++a) {
                const f32x2 x01 = {oacc[db][4 * a] * inv, oacc[db][4 * a + 1] * inv};
                const f32x2 x23 = {oacc[db][4 * a + 2] * inv, oacc[db][4 * a + 3] * inv};
                const bf16x2 y01 = __builtin_convertvector(x01, bf16x2);
                const bf16x2 y23 = __builtin_convertvector(x23, bf16x2);
                uint2 out;
                out.x = __builtin_bit_cast(uint32_t, y01);
                out.y = __builtin_bit_cast(uint32_t, y23);
                *reinterpret_cast<uint2*>(stage + qi * kPitch + 2 * (32 * db + 8 * a + 4 * hh)) = out;
            }
        // (only this wavefront touches its staging area: no barrier, the compiler orders the LDS accesses)
        const int srow = lane >> 4, schunk = lane & 15;
        uint16_t* const obase = p.o + (static_cast<size_t>(my_head) * p.nq + (my_i0 - p.pos0)) * kD;
#pragma unroll
        for (int it = 0; it < 8; ++it) {
            const int r = 4 * it + srow;
            const uint4 piece = *reinterpret_cast<const uint4*>(stage + r * kPitch + 16 * schunk);
            if (my_i0 + r < n_pos) *reinterpret_cast<uint4*>(obase + static_cast<size_t>(r) * kD + 8 * schunk) = piece;
        }
        const int row = my_i0 + qi;
        if (row < n_pos && p.lse && hh == 0)
            p.lse[static_cast<size_t>(my_head) * p.nq + (row - p.pos0)] = l_tot > 0.f ? m_run * p.scale + __logf(l_tot) : NEG_INF;
    }
    if (!p.work_counter) break;
    }
    if (p.tile_counter && (threadIdx.x & 63) == 0 && tiles_done) atomicAdd(p.tile_counter, static_cast<unsigned long long>(tiles_done));
    if (p.tile_counter && threadIdx.x == 0) {
        if (staged_gather) atomicAdd(p.tile_counter + 1, static_cast<unsigned long long>(staged_gather));
        if (staged_block) atomicAdd(p.tile_counter + 2, static_cast<unsigned long long>(staged_block));
    }
}

// ---- once per call: index lists -> bitmaps, block-diagonal list, per-block counts ----
// One workgroup per index head.  The head's offset bitmap, then its column bitmap, is built in LDS (bit atomics stay on
// chip) and written out with plain stores; everything derived from the offsets is read back from LDS.
constexpr int kPrepThreads = 1024;
struct PrepParams {
    const int32_t* idx_v;
    const int32_t* cnt_v;
    int cap_v;
    const int32_t* idx_s;
    const int32_t* cnt_s;
    int cap_s;
    int n, nsub, nblk;
    int shift;                      // pos0 % 32: row blocks start at positions 32 t + shift
    uint32_t* sbit;                 // per head: bit (o + 64) set iff offset o selected (64-bit zero guard in front, zero tail)
    uint32_t* vbit;
    int sw, vw;
    int32_t* dlist;
    unsigned long long* wlist;
    int dcap;
    int32_t* ndiag;
    int32_t* ncol32;
    int nq32;
    int32_t* vfirst;
    uint32_t* counters;             // tile counter and the work queues' counters at the head of the workspace, zeroed here
    int ncounters;
};

__global__ __launch_bounds__(kPrepThreads) void vs_prepare_kernel(const PrepParams p) {
    extern __shared__ __align__(16) uint32_t bm[];           // max(sw, vw) words, then 32 words of scan scratch
    const int ih = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    uint32_t* const scan = bm + max(p.sw, p.vw);
    if (ih == 0)
        for (int i = tid; i < p.ncounters; i += kPrepThreads) p.counters[i] = 0u;
    // offsets
    for (int w = tid; w < p.sw; w += kPrepThreads) bm[w] = 0u;
    __syncthreads();
    const int cs = min(p.cnt_s[ih], p.cap_s);
    for (int t = tid; t < cs; t += kPrepThreads) {
        const int e = p.idx_s[static_cast<size_t>(ih) * p.cap_s + t];
        if (e >= 0 && e < p.n) atomicOr(&bm[(e + 64) >> 5], 1u << ((e + 64) & 31));
    }
    __syncthreads();
    uint32_t* const sbit = p.sbit + static_cast<size_t>(ih) * p.sw;
    for (int w = tid; w < p.sw; w += kPrepThreads) sbit[w] = bm[w];
    // Block diagonals.  A query tile whose first row block starts at position 32 qb + shift looks, for diagonal delta, at
    // key block qb - delta; its 32-row block r < nsub then sees that block through the offsets 32 (delta + r) + shift - 31
    // .. + 31.  Candidate c stands for delta = c + dmin.  A thread owns a run of consecutive candidates; an exclusive
    // scan of the per-thread counts gives the list positions.
    const int nsub = p.nsub;
    const int dmin = -(nsub - 1) - (p.shift > 0 ? 1 : 0);
    const int ncand = p.nblk - dmin;
    const int per = (ncand + kPrepThreads - 1) / kPrepThreads;
    const int c0 = min(tid * per, ncand), c1 = min(c0 + per, ncand);
    auto window = [&](int t) -> uint64_t {                   // offsets 32 t + shift - 31 .. 32 t + shift + 31 at bits 0..62
        return 32 * t + p.shift + 31 < 0 ? 0ull : (window64(bm, 32 * t + p.shift + 33) & kAll63);
    };
    auto crossed = [&](int delta) -> bool {
        uint64_t any = 0ull;
        for (int r = 0; r < nsub; ++r) any |= window(delta + r);
        return any != 0ull;
    };
    int mine = 0;
    for (int c = c0; c < c1; ++c) mine += crossed(c + dmin) ? 1 : 0;
    int incl = mine;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const int y = __shfl_up(incl, d);
        if (lane >= d) incl += y;
    }
    if (lane == 63) scan[wave] = incl;
    __syncthreads();
    int pos = incl - mine;
    for (int i = 0; i < wave; ++i) pos += scan[i];
    int32_t* const dl = p.dlist + static_cast<size_t>(ih) * p.dcap;
    unsigned long long* const wl = p.wlist + static_cast<size_t>(ih) * p.dcap * 4;
    int32_t* const nd = p.ndiag + static_cast<size_t>(ih) * p.nq32;
    for (int c = c0; c < c1; ++c) {
        const int delta = c + dmin;
        if (crossed(delta)) {
            dl[pos] = delta;
            for (int r = 0; r < 4; ++r) wl[static_cast<size_t>(pos) * 4 + r] = r < nsub ? window(delta + r) : 0ull;
            ++pos;
        }
        if (delta >= 0 && delta < p.nq32) nd[delta] = pos;  // listed diagonals <= delta
    }
    __syncthreads();
    // columns
    for (int w = tid; w < p.vw; w += kPrepThreads) bm[w] = 0u;
    __syncthreads();
    const int cv = min(p.cnt_v[ih], p.cap_v);
    const int32_t* const iv = p.idx_v + static_cast<size_t>(ih) * p.cap_v;
    for (int t = tid; t < cv; t += kPrepThreads) {
        const int e = iv[t];
        if (e >= 0 && e < p.n) atomicOr(&bm[e >> 5], 1u << (e & 31));
    }
    __syncthreads();
    uint32_t* const vbit = p.vbit + static_cast<size_t>(ih) * p.vw;
    for (int w = tid; w < p.vw; w += kPrepThreads) vbit[w] = bm[w];
    // ncol32[q] = entries of the ascending list that are <= min(32 q + 31, n - 1);  vfirst = entries that are < 0
    for (int q = tid; q <= p.nq32; q += kPrepThreads) {
        const int limit = q < p.nq32 ? min(32 * q + 31, p.n - 1) : -1;
        int lo = 0, hi = cv;
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (iv[mid] <= limit) lo = mid + 1; else hi = mid;
        }
        if (q < p.nq32) p.ncol32[static_cast<size_t>(ih) * p.nq32 + q] = lo;
        else p.vfirst[ih] = lo;
    }
}

struct SparseWs {
    size_t counter_off, sbit_off, vbit_off, ncol_off, ndiag_off, vfirst_off, dlist_off, wlist_off, total;
    int sw, vw, nq32, dcap;
};

SparseWs sparse_ws_layout(int kv_heads, int index_heads, int64_t n) {
    SparseWs w;
    const int64_t nblk = (n + 31) / 32;
    const size_t ih = static_cast<size_t>(index_heads);
    w.sw = static_cast<int>(vs::round_up(static_cast<size_t>(n + 64 + 320 + 31) / 32, 4));
    w.vw = static_cast<int>(vs::round_up(static_cast<size_t>(nblk + 4), 4));
    w.nq32 = static_cast<int>(nblk);
    w.dcap = static_cast<int>(nblk + 4);
    w.counter_off = 0;                                      // three 8-byte tile counters, then from byte 64 one counter per KV head
    w.sbit_off = vs::round_up(64 + static_cast<size_t>(kv_heads) * 4, 256);
    w.vbit_off = w.sbit_off + ih * w.sw * 4;
    w.ncol_off = vs::round_up(w.vbit_off + ih * w.vw * 4, 256);
    w.ndiag_off = vs::round_up(w.ncol_off + ih * w.nq32 * 4, 256);
    w.vfirst_off = vs::round_up(w.ndiag_off + ih * w.nq32 * 4, 256);
    w.dlist_off = vs::round_up(w.vfirst_off + ih * 4, 256);
    w.wlist_off = vs::round_up(w.dlist_off + ih * w.dcap * 4, 256);
    w.total = vs::round_up(w.wlist_off + ih * w.dcap * 4 * 8, 256);
    return w;
}

// Scratch of the entry point that allocates nothing: one copy per GPU, held until the process ends.  In host code the
// array's name is only a handle; its device address comes from hipGetSymbolAddress (device_info below).
constexpr size_t kStaticScratchBytes = VS_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

// Device-dependent launch facts, looked up once per device (and thread-safe).
struct DeviceInfo {
    int cus = 0;
    unsigned char* scratch_ptr = nullptr;                    // this device's copy of `scratch`
};
int device_info(DeviceInfo& out) {
    constexpr int kMaxDevices = 64;
    static std::mutex mu;
    static DeviceInfo cache[kMaxDevices];
    static bool attr_set[kMaxDevices] = {};
    int dev = 0;
    VS_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return VS_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> lock(mu);
    if (!attr_set[dev]) {
        VS_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&vs_attention_kernel),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(kLdsBytes)));
        VS_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&vs_prepare_kernel),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));
        int cus = 0;
        VS_HIP(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
        cache[dev].cus = cus > 0 ? cus : 256;
        void* sp = nullptr;
        VS_HIP(hipGetSymbolAddress(&sp, HIP_SYMBOL(scratch)));   // the current device's copy
        if (!sp) return VS_ERR_HIP;
        cache[dev].scratch_ptr = static_cast<unsigned char*>(sp);
        attr_set[dev] = true;
    }
    out = cache[dev];
    return VS_OK;
}

int launch_attention(AttnParams& p, hipStream_t stream) {
    DeviceInfo info;
    const int rc = device_info(info);
    if (rc != VS_OK) return rc;
    const int BQ = 32 * kWaves / p.hc;
    p.tiles = (p.nq + BQ - 1) / BQ;
    const long long blocks = static_cast<long long>(p.kv_heads) * (p.group / p.hc) * p.tiles;
    if (blocks > 0x7fffffffLL) return VS_ERR_UNSUPPORTED;
    p.work_total = static_cast<int>(blocks);
    long long launch = blocks;
    if (p.work_counter) launch = blocks < 2 * info.cus ? blocks : 2 * info.cus;   // two workgroups per compute unit
    hipLaunchKernelGGL(vs_attention_kernel, dim3(static_cast<unsigned>(launch)), dim3(kThreads), kLdsBytes, stream, p);
    VS_LAUNCH_CHECK();
    return VS_OK;
}

// Runs the whole sparse call on a workspace that is known to be large enough.
int sparse_prefill_on(unsigned char* base, const SparseWs& w, const void* q, const void* k, const void* v, int q_heads,
                      int kv_heads, int64_t nq, int64_t n, int64_t pos0, float scale, const int32_t* idx_v, const int32_t* cnt_v, int cap_v,
                      const int32_t* idx_s, const int32_t* cnt_s, int cap_s, int index_heads, int slash_granularity,
                      void* o_bf16, float* lse, hipStream_t st) {
    AttnParams p{};
    p.q = static_cast<const uint16_t*>(q);
    p.k = static_cast<const uint16_t*>(k);
    p.v = static_cast<const uint16_t*>(v);
    p.o = static_cast<uint16_t*>(o_bf16);
    p.lse = lse;
    p.q_heads = q_heads;
    p.kv_heads = kv_heads;
    p.group = q_heads / kv_heads;
    p.index_per_q = (index_heads == q_heads && q_heads != kv_heads) ? 1 : 0;
    p.hc = heads_per_workgroup(p.group, p.index_per_q != 0);
    p.gran = slash_granularity;
    p.n = static_cast<int>(n);
    p.nq = static_cast<int>(nq);
    p.pos0 = static_cast<int>(pos0);
    p.scale = scale;
    p.c = scale * 1.4426950408889634f;
    p.idx_v = idx_v;
    p.cnt_v = cnt_v;
    p.cap_v = cap_v;
    p.vbit = reinterpret_cast<const uint32_t*>(base + w.vbit_off);
    p.vw = w.vw;
    p.dlist = reinterpret_cast<const int32_t*>(base + w.dlist_off);
    p.wlist = reinterpret_cast<const unsigned long long*>(base + w.wlist_off);
    p.dcap = w.dcap;
    p.ndiag = reinterpret_cast<const int32_t*>(base + w.ndiag_off);
    p.ncol32 = reinterpret_cast<const int32_t*>(base + w.ncol_off);
    p.nq32 = w.nq32;
    p.vfirst = reinterpret_cast<const int32_t*>(base + w.vfirst_off);
    p.tile_counter = reinterpret_cast<unsigned long long*>(base + w.counter_off);
    // one queue counter per KV head from byte 64 of the counter block (zeroed by the preparation kernel)
    p.work_counter = reinterpret_cast<unsigned int*>(base + w.counter_off + 64);

    DeviceInfo info;
    int rc = device_info(info);
    if (rc != VS_OK) return rc;
    PrepParams pp{};
    pp.idx_v = idx_v;
    pp.cnt_v = cnt_v;
    pp.cap_v = cap_v;
    pp.idx_s = idx_s;
    pp.cnt_s = cnt_s;
    pp.cap_s = cap_s;
    pp.n = p.n;
    pp.nsub = kWaves / p.hc;
    pp.nblk = w.nq32;
    pp.shift = static_cast<int>(pos0 % 32);
    pp.sbit = reinterpret_cast<uint32_t*>(base + w.sbit_off);
    pp.vbit = reinterpret_cast<uint32_t*>(base + w.vbit_off);
    pp.sw = w.sw;
    pp.vw = w.vw;
    pp.dlist = reinterpret_cast<int32_t*>(base + w.dlist_off);
    pp.wlist = reinterpret_cast<unsigned long long*>(base + w.wlist_off);
    pp.dcap = w.dcap;
    pp.ndiag = reinterpret_cast<int32_t*>(base + w.ndiag_off);
    pp.ncol32 = reinterpret_cast<int32_t*>(base + w.ncol_off);
    pp.nq32 = w.nq32;
    pp.vfirst = reinterpret_cast<int32_t*>(base + w.vfirst_off);
    pp.counters = reinterpret_cast<uint32_t*>(base + w.counter_off);
    pp.ncounters = 16 + kv_heads;
    const size_t prep_lds = (static_cast<size_t>(w.sw > w.vw ? w.sw : w.vw) + 32) * 4;
    if (prep_lds > 160 * 1024) return VS_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(vs_prepare_kernel, dim3(index_heads), dim3(kPrepThreads), prep_lds, st, pp);
    VS_LAUNCH_CHECK();
    return launch_attention(p, st);
}

}  // namespace

extern "C" {

size_t vs_sparse_prefill_workspace(int q_heads, int kv_heads, int index_heads, int64_t n) {
    if (q_heads <= 0 || kv_heads <= 0 || n <= 0 || n > VS_MAX_SEQ) return 0;
    if (index_heads != q_heads && index_heads != kv_heads) return 0;
    return sparse_ws_layout(kv_heads, index_heads, n).total;
}

int vs_sparse_prefill(const void* q, const void* k, const void* v, int q_heads, int kv_heads, int64_t n, float scale,
                      const int32_t* idx_v, const int32_t* cnt_v, int cap_v, const int32_t* idx_s, const int32_t* cnt_s,
                      int cap_s, int index_heads, void* o_bf16, float* lse, void* ws, size_t ws_bytes, void* stream) {
    return vs_sparse_prefill_chunk(q, k, v, q_heads, kv_heads, n, n, 0, scale, idx_v, cnt_v, cap_v, idx_s, cnt_s, cap_s,
                                   index_heads, 1, o_bf16, lse, ws, ws_bytes, stream);
}

int vs_sparse_prefill_tiled(const void* q, const void* k, const void* v, int q_heads, int kv_heads, int64_t n, float scale,
                            const int32_t* idx_v, const int32_t* cnt_v, int cap_v, const int32_t* idx_s,
                            const int32_t* cnt_s, int cap_s, int index_heads, int slash_granularity, void* o_bf16,
                            float* lse, void* ws, size_t ws_bytes, void* stream) {
    return vs_sparse_prefill_chunk(q, k, v, q_heads, kv_heads, n, n, 0, scale, idx_v, cnt_v, cap_v, idx_s, cnt_s, cap_s,
                                   index_heads, slash_granularity, o_bf16, lse, ws, ws_bytes, stream);
}

int vs_sparse_prefill_chunk(const void* q, const void* k, const void* v, int q_heads, int kv_heads, int64_t n_q, int64_t n_kv,
                            int64_t pos0, float scale, const int32_t* idx_v, const int32_t* cnt_v, int cap_v,
                            const int32_t* idx_s, const int32_t* cnt_s, int cap_s, int index_heads, int slash_granularity,
                            void* o_bf16, float* lse, void* ws, size_t ws_bytes, void* stream) {
    int rc = check_qkv(q, k, v, q_heads, kv_heads, n_kv, scale, o_bf16);
    if (rc != VS_OK) return rc;
    rc = check_chunk(n_q, n_kv, pos0);
    if (rc != VS_OK) return rc;
    if (slash_granularity != 1 && slash_granularity != 32) return VS_ERR_UNSUPPORTED;
    if (slash_granularity == 32 && pos0 % 32 != 0) return VS_ERR_UNSUPPORTED;   // aligned 32-position blocks
    if (!idx_v || !cnt_v || !idx_s || !cnt_s || cap_v <= 0 || cap_s <= 0) return VS_ERR_INVALID_ARG;
    if (index_heads != q_heads && index_heads != kv_heads) return VS_ERR_INVALID_ARG;
    const SparseWs w = sparse_ws_layout(kv_heads, index_heads, n_kv);
    if (!ws || ws_bytes < w.total) return VS_ERR_WORKSPACE;
    if (!vs::aligned16(ws)) return VS_ERR_INVALID_ARG;
    return sparse_prefill_on(static_cast<unsigned char*>(ws), w, q, k, v, q_heads, kv_heads, n_q, n_kv, pos0, scale, idx_v,
                             cnt_v, cap_v, idx_s, cnt_s, cap_s, index_heads, slash_granularity, o_bf16, lse,
                             static_cast<hipStream_t>(stream));
}

int vs_sparse_prefill_static(const void* q, const void* k, const void* v, int q_heads, int kv_heads, int64_t n, float scale,
                             const int32_t* idx_v, const int32_t* cnt_v, int cap_v, const int32_t* idx_s,
                             const int32_t* cnt_s, int cap_s, int index_heads, void* o_bf16, float* lse, void* stream) {
    int rc = check_qkv(q, k, v, q_heads, kv_heads, n, scale, o_bf16);
    if (rc != VS_OK) return rc;
    if (!idx_v || !cnt_v || !idx_s || !cnt_s || cap_v <= 0 || cap_s <= 0) return VS_ERR_INVALID_ARG;
    if (index_heads != q_heads && index_heads != kv_heads) return VS_ERR_INVALID_ARG;
    const SparseWs w = sparse_ws_layout(kv_heads, index_heads, n);
    if (w.total > kStaticScratchBytes) return VS_ERR_STATIC_LIMIT;
    DeviceInfo info;
    rc = device_info(info);
    if (rc != VS_OK) return rc;
    // every structure the kernels read is rewritten by the preparation kernel of this call (counters included), so what
    // the previous call left in the array does not matter
    return sparse_prefill_on(info.scratch_ptr, w, q, k, v, q_heads, kv_heads, n, n, 0, scale, idx_v, cnt_v, cap_v, idx_s, cnt_s,
                             cap_s, index_heads, 1, o_bf16, lse, static_cast<hipStream_t>(stream));
}

int vs_sparse_prefill_tiles(const void* ws, size_t ws_bytes, void* stream, int64_t* executed_tiles_host) {
    if (!executed_tiles_host) return VS_ERR_INVALID_ARG;
    int64_t c[3] = {0, 0, 0};
    const int rc = vs_sparse_prefill_counters(ws, ws_bytes, stream, c);
    if (rc == VS_OK) *executed_tiles_host = c[0];
    return rc;
}

int vs_sparse_prefill_counters(const void* ws, size_t ws_bytes, void* stream, int64_t* counters_host) {
    if (!ws || ws_bytes < 256 || !counters_host) return VS_ERR_INVALID_ARG;
    hipStream_t st = static_cast<hipStream_t>(stream);
    VS_HIP(hipStreamSynchronize(st));
    unsigned long long c[3] = {0, 0, 0};
    VS_HIP(hipMemcpy(c, ws, sizeof(c), hipMemcpyDeviceToHost));
    for (int i = 0; i < 3; ++i) counters_host[i] = static_cast<int64_t>(c[i]);
    return VS_OK;
}

}  // extern "C"
