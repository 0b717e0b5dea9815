// CPU oracle for the vertical-slash sparse-prefill path.  TEST INFRASTRUCTURE ONLY.
//
// Everything here is the plain definition from the paper, evaluated in fp64 with
// straightforward loops.  Nothing in this file is shared with the GPU library and the
// product path never calls it: only the test-suite, the smoke check and the benchmark's
// CPU-baseline leg load this object.  There is no tiling, fusion or reordering beyond
// what the cited definition states; threads only split independent rows / heads.
//
//   vso_rope_*            rotary embedding, block-diagonal 2x2 rotations (Appendix,
//                         "RoPE Matrix Representation")
//   vso_index_score       VSIndexer forward (Sec. "VSIndexer Design", Eqs. X, Z, A_v, A_s)
//   vso_select            cumulative-threshold budget and TopK (Sec. "Adaptive Sparse
//                         Index Selection", Eqs. k_d, I_d) with the integer mass rule
//   vso_sparse_attention  masked softmax attention (Sec. "Sparse Attention Formulation",
//                         Eqs. M_S, A-hat) with the vertical-slash mask (Sec.
//                         "Linear-Complexity Mask Construction", Eq. M_S) plus causality
//   vso_dense_attention   scaled dot-product attention (Sec. "Attention Computation",
//                         Eqs. P, A, O) under the causal mask
//   vso_vs_aggregate      column and diagonal sums of the causal attention matrix
//                         (Sec. "Obtaining Ground Truth") and vso_recall (Eq. R(S))
//   vso_index_train       distillation loss L = KL(A^_v || A_v) + KL(A^_s || A_s) (Sec. "Vertical-Slash
//                         Aggregation for Distillation Training", paragraph "Loss function design") and
//                         its gradient with respect to the indexer's parameters, by the chain rule
//
// Parity pins live in tests/ (brute force on tiny inputs, closed forms, hand-worked masks,
// library special cases).  No function here is "parity unpinned".
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <functional>
#include <limits>
#include <thread>
#include <vector>

namespace {

double bf16_to_f64(uint16_t b) {
    uint32_t u = static_cast<uint32_t>(b) << 16;
    float f;
    std::memcpy(&f, &u, 4);
    return static_cast<double>(f);
}

// fp64 -> bf16, round to nearest even, done in one rounding step from the double.
uint16_t f64_to_bf16(double x) {
    if (std::isnan(x)) return 0x7fc0;
    double ax = std::fabs(x);
    uint16_t sign = std::signbit(x) ? 0x8000 : 0;
    if (ax == 0.0) return sign;
    if (std::isinf(x)) return sign | 0x7f80;
    double r;
    if (ax < std::ldexp(1.0, -126)) {
        // subnormal range of bf16: spacing 2^-133
        r = std::nearbyint(ax * std::ldexp(1.0, 133)) * std::ldexp(1.0, -133);
    } else {
        int e;
        double m = std::frexp(ax, &e);                       // ax = m * 2^e, m in [0.5,1)
        double scaled = std::nearbyint(m * 256.0);           // 8 significant bits, ties-to-even
        r = std::ldexp(scaled, e - 8);
    }
    if (r >= std::ldexp(1.0, 128)) return sign | 0x7f80;
    float f = static_cast<float>(r);                          // exact: r has <= 8 significant bits
    uint32_t u;
    std::memcpy(&u, &f, 4);
    return sign | static_cast<uint16_t>(u >> 16);
}

void parallel_for(int64_t count, int threads, const std::function<void(int64_t)>& body) {
    if (threads <= 0) threads = static_cast<int>(std::thread::hardware_concurrency());
    if (threads < 1) threads = 1;
    if (threads > count) threads = static_cast<int>(std::max<int64_t>(count, 1));
    if (threads == 1) {
        for (int64_t i = 0; i < count; ++i) body(i);
        return;
    }
    std::vector<std::thread> pool;
    for (int t = 0; t < threads; ++t) {
        pool.emplace_back([=, &body]() {
            for (int64_t i = t; i < count; i += threads) body(i);
        });
    }
    for (auto& th : pool) th.join();
}

// Rotation of one vector of length d at position t.  Plane p couples elements (a,b):
// pairing 0 -> (2p, 2p+1) as in the appendix matrix; pairing 1 -> (p, p + d/2).
void rope_vec(double* x, int d, double t, double base, int pairing) {
    for (int p = 0; p < d / 2; ++p) {
        double theta = std::pow(base, -2.0 * p / d);
        double phi = t * theta;
        double c = std::cos(phi), s = std::sin(phi);
        int a = pairing == 0 ? 2 * p : p;
        int b = pairing == 0 ? 2 * p + 1 : p + d / 2;
        double xa = x[a], xb = x[b];
        x[a] = xa * c - xb * s;
        x[b] = xa * s + xb * c;
    }
}

double activation(double x, int act) {
    if (act == 0) return x / (1.0 + std::exp(-x));                    // SiLU
    return 0.5 * x * (1.0 + std::erf(x / std::sqrt(2.0)));            // GELU, exact erf form
}

// Row i of the masked attention for one query head.  `live(j)` says whether key j is kept.
// Returns the number of live keys.  out: d doubles; lse: log-sum-exp of the kept logits.
template <class Live>
int64_t attention_row(const uint16_t* q_row, const uint16_t* k_head, const uint16_t* v_head,
                      int64_t i, int d, double scale, Live live, double* out, double* lse) {
    std::vector<double> q(d);
    for (int c = 0; c < d; ++c) q[c] = bf16_to_f64(q_row[c]);
    std::vector<int64_t> keys;
    std::vector<double> s;
    for (int64_t j = 0; j <= i; ++j) {
        if (!live(j)) continue;
        double acc = 0.0;
        const uint16_t* kr = k_head + j * d;
        for (int c = 0; c < d; ++c) acc += q[c] * bf16_to_f64(kr[c]);
        keys.push_back(j);
        s.push_back(acc * scale);
    }
    for (int c = 0; c < d; ++c) out[c] = 0.0;
    if (keys.empty()) {
        if (lse) *lse = -std::numeric_limits<double>::infinity();
        return 0;
    }
    double m = *std::max_element(s.begin(), s.end());
    double z = 0.0;
    for (double& e : s) { e = std::exp(e - m); z += e; }
    for (size_t t = 0; t < keys.size(); ++t) {
        double p = s[t] / z;
        const uint16_t* vr = v_head + keys[t] * d;
        for (int c = 0; c < d; ++c) out[c] += p * bf16_to_f64(vr[c]);
    }
    if (lse) *lse = m + std::log(z);
    return static_cast<int64_t>(keys.size());
}

}  // namespace

extern "C" {

const char* vso_version() { return "vs-oracle 1 (fp64, definitions only)"; }

uint16_t vso_f64_to_bf16(double x) { return f64_to_bf16(x); }
double vso_bf16_to_f64(uint16_t b) { return bf16_to_f64(b); }

// x: [heads, n, d] fp64, rotated in place; token at row r has position pos0 + r.
int vso_rope_f64(double* x, int heads, int64_t n, int d, int64_t pos0, double theta_base, int pairing) {
    if (!x || heads <= 0 || n < 0 || d <= 0 || d % 2 || pairing < 0 || pairing > 1) return -1;
    for (int h = 0; h < heads; ++h)
        for (int64_t r = 0; r < n; ++r)
            rope_vec(x + (static_cast<int64_t>(h) * n + r) * d, d, static_cast<double>(pos0 + r), theta_base, pairing);
    return 0;
}

// Same on bf16 storage: widen exactly, rotate in fp64, round once to bf16 (nearest even).
int vso_rope_bf16(uint16_t* x, int heads, int64_t n, int d, int64_t pos0, double theta_base, int pairing, int threads) {
    if (!x || heads <= 0 || n < 0 || d <= 0 || d % 2 || pairing < 0 || pairing > 1) return -1;
    parallel_for(static_cast<int64_t>(heads) * n, threads, [&](int64_t row) {
        std::vector<double> buf(d);
        uint16_t* p = x + row * d;
        for (int c = 0; c < d; ++c) buf[c] = bf16_to_f64(p[c]);
        rope_vec(buf.data(), d, static_cast<double>(pos0 + row % n), theta_base, pairing);
        for (int c = 0; c < d; ++c) p[c] = f64_to_bf16(buf[c]);
    });
    return 0;
}

// VSIndexer forward.  k, v: [kv_heads, n, d] bf16.  W_U: [2d, d_h] row-major fp32, b_U: [d_h],
// W_V, W_S: [d_h].  act: 0 SiLU, 1 GELU(erf).  a_v, a_s: [kv_heads, n] fp64 probabilities
// (softmax over the n positions of each head).  logits_v/logits_s optional, same shape.
int vso_index_score(const uint16_t* k, const uint16_t* v, int kv_heads, int64_t n, int d,
                    const float* W_U, const float* b_U, const float* W_V, const float* W_S,
                    float b_V, float b_S, int d_h, int act,
                    double* a_v, double* a_s, double* logits_v, double* logits_s, int threads) {
    if (!k || !v || !W_U || !b_U || !W_V || !W_S || !a_v || !a_s) return -1;
    if (kv_heads <= 0 || n <= 0 || d <= 0 || d_h <= 0 || act < 0 || act > 1) return -1;
    std::vector<double> lv(static_cast<size_t>(kv_heads) * n), ls(static_cast<size_t>(kv_heads) * n);
    parallel_for(static_cast<int64_t>(kv_heads) * n, threads, [&](int64_t row) {
        std::vector<double> x(2 * d);
        for (int c = 0; c < d; ++c) {
            x[c] = bf16_to_f64(k[row * d + c]);
            x[d + c] = bf16_to_f64(v[row * d + c]);
        }
        double sv = static_cast<double>(b_V), ss = static_cast<double>(b_S);
        for (int u = 0; u < d_h; ++u) {
            double pre = static_cast<double>(b_U[u]);
            for (int c = 0; c < 2 * d; ++c) pre += x[c] * static_cast<double>(W_U[static_cast<int64_t>(c) * d_h + u]);
            double z = activation(pre, act);
            sv += z * static_cast<double>(W_V[u]);
            ss += z * static_cast<double>(W_S[u]);
        }
        lv[row] = sv;
        ls[row] = ss;
    });
    for (int h = 0; h < kv_heads; ++h) {
        for (int dir = 0; dir < 2; ++dir) {
            const double* l = (dir == 0 ? lv.data() : ls.data()) + static_cast<int64_t>(h) * n;
            double* a = (dir == 0 ? a_v : a_s) + static_cast<int64_t>(h) * n;
            double m = *std::max_element(l, l + n);
            double z = 0.0;
            for (int64_t t = 0; t < n; ++t) z += std::exp(l[t] - m);
            for (int64_t t = 0; t < n; ++t) a[t] = std::exp(l[t] - m) / z;
        }
    }
    if (logits_v) std::copy(lv.begin(), lv.end(), logits_v);
    if (logits_s) std::copy(ls.begin(), ls.end(), logits_s);
    return 0;
}

// Budget + TopK for one direction, all heads.  scores: [heads, n] fp32.
//   mode 0: cumulative threshold tau.  Integer rule: w_i = floor(s_i * 2^40) (s_i clamped to
//           [0,1], NaN -> 0), S = sum w_i, T = ceil(tau * S); rank by (score descending,
//           index ascending); k = fewest leading elements whose w-sum reaches T (k = n if never).
//   mode 1: k = min(k_fixed, n), same ranking.
// Then the forced indices 0..n_forced-1 are united with the pick and the result is written
// ascending.  If the union exceeds cap: forced entries stay, the best-ranked others fill the
// rest, status bit 1 is set.  status bits: 1 overflow, 2 NaN/negative score seen, 4 score > 1.
// k_out (optional): the k of the rule before forcing / capping.
int vso_select(const float* scores, int heads, int64_t n, int mode, double tau, int64_t k_fixed,
               int64_t n_forced, int64_t cap, int32_t* idx, int32_t* cnt, int32_t* status, int64_t* k_out) {
    if (!scores || !idx || !cnt || heads <= 0 || n <= 0 || cap <= 0) return -1;
    if (mode == 0 && !(tau >= 0.0 && tau <= 1.0)) return -1;
    if (mode == 1 && k_fixed < 0) return -1;
    if (mode != 0 && mode != 1) return -1;
    if (n_forced < 0) n_forced = 0;
    if (n_forced > n) n_forced = n;
    if (n_forced > cap) return -2;
    const double two40 = std::ldexp(1.0, 40);
    for (int h = 0; h < heads; ++h) {
        const float* s = scores + static_cast<int64_t>(h) * n;
        int32_t st = 0;
        std::vector<float> val(n);
        std::vector<uint64_t> w(n);
        for (int64_t i = 0; i < n; ++i) {
            float x = s[i];
            if (std::isnan(x) || x < 0.0f) { x = 0.0f; st |= 2; }
            if (x == 0.0f) x = 0.0f;                              // -0 -> +0
            val[i] = x;
            double xd = static_cast<double>(x);
            if (xd > 1.0) { xd = 1.0; st |= 4; }
            w[i] = static_cast<uint64_t>(std::floor(xd * two40));
        }
        std::vector<int64_t> order(n);
        for (int64_t i = 0; i < n; ++i) order[i] = i;
        std::stable_sort(order.begin(), order.end(), [&](int64_t a, int64_t b) { return val[a] > val[b]; });
        int64_t k;
        if (mode == 1) {
            k = std::min<int64_t>(k_fixed, n);
        } else {
            uint64_t S = 0;
            for (int64_t i = 0; i < n; ++i) S += w[i];
            uint64_t T = static_cast<uint64_t>(std::ceil(tau * static_cast<double>(S)));
            uint64_t acc = 0;
            k = 0;
            while (acc < T && k < n) { acc += w[order[k]]; ++k; }
            if (acc < T) k = n;
        }
        if (k_out) k_out[h] = k;
        std::vector<char> keep(n, 0);
        for (int64_t i = 0; i < n_forced; ++i) keep[i] = 1;
        int64_t total = n_forced;
        for (int64_t r = 0; r < k; ++r) {
            int64_t e = order[r];
            if (keep[e]) continue;
            if (total >= cap) { st |= 1; break; }
            keep[e] = 1;
            ++total;
        }
        int32_t* out = idx + static_cast<int64_t>(h) * cap;
        int64_t c = 0;
        for (int64_t i = 0; i < n; ++i) if (keep[i]) out[c++] = static_cast<int32_t>(i);
        cnt[h] = static_cast<int32_t>(c);
        if (status) status[h] = st;
    }
    return 0;
}

// Vertical-slash sparse attention.  q: [q_heads, n_q, d], k, v: [kv_heads, n, d] bf16.
// Chunked prefill: the n_q query rows are the positions pos0 .. pos0 + n_q - 1 of a sequence whose keys 0 .. n - 1 are
// present (pos0 + n_q <= n); n_q <= 0 means the whole sequence (n_q = n, pos0 = 0).  The mask speaks of absolute
// positions: the query at position i keeps key j iff j <= i and (j in I_v or i - j in I_s).
// Query head h reads KV head h / (q_heads / kv_heads); its index lists come from index head
// h (index_heads == q_heads) or from its KV head (index_heads == kv_heads).
// Kept set of position i: { j : 0 <= j <= i and ( j in I_v or i - j in I_s ) }, each key once.
// granularity g > 1 selects the tile-granular slash variant: positions are grouped in aligned blocks of g (position i
// belongs to g*floor(i/g) .. g*floor(i/g)+g-1, clipped to the positions that exist, i.e. < pos0 + n_q) and key j <= i is
// kept if it is a selected column or ANY position i' of the block of i has i' - j in I_s.  g = 1 is the mask equation.
// rows: optional list of LOCAL row numbers (n_rows of them, each in [0, n_q)); NULL -> all n_q rows in order.
// out: [q_heads, n_rows, d] fp64; lse: [q_heads, n_rows] or NULL; live: [q_heads, n_rows] or NULL.
int vso_sparse_attention(const uint16_t* q, const uint16_t* k, const uint16_t* v,
                         int q_heads, int kv_heads, int64_t n, int d, double scale,
                         const int32_t* idx_v, const int32_t* cnt_v, int64_t cap_v,
                         const int32_t* idx_s, const int32_t* cnt_s, int64_t cap_s, int index_heads,
                         int64_t granularity,
                         const int64_t* rows, int64_t n_rows, int64_t n_q, int64_t pos0,
                         double* out, double* lse, int64_t* live, int threads) {
    if (!q || !k || !v || !idx_v || !cnt_v || !idx_s || !cnt_s || !out) return -1;
    if (q_heads <= 0 || kv_heads <= 0 || q_heads % kv_heads || n <= 0 || d <= 0) return -1;
    if (index_heads != q_heads && index_heads != kv_heads) return -1;
    if (granularity < 1) return -1;
    if (n_q <= 0) { n_q = n; pos0 = 0; }
    if (pos0 < 0 || pos0 + n_q > n) return -1;
    if (!rows) n_rows = n_q;
    const int group = q_heads / kv_heads;
    const int64_t n_pos = pos0 + n_q;                         // positions that exist
    // membership tables per index head
    std::vector<std::vector<char>> in_v(index_heads, std::vector<char>(n, 0)), in_s(index_heads, std::vector<char>(n, 0));
    for (int ih = 0; ih < index_heads; ++ih) {
        for (int32_t t = 0; t < cnt_v[ih]; ++t) {
            int32_t c = idx_v[static_cast<int64_t>(ih) * cap_v + t];
            if (c < 0 || c >= n) return -3;
            in_v[ih][c] = 1;
        }
        for (int32_t t = 0; t < cnt_s[ih]; ++t) {
            int32_t o = idx_s[static_cast<int64_t>(ih) * cap_s + t];
            if (o < 0 || o >= n) return -3;
            in_s[ih][o] = 1;
        }
    }
    if (rows)
        for (int64_t r = 0; r < n_rows; ++r)
            if (rows[r] < 0 || rows[r] >= n_q) return -4;
    parallel_for(static_cast<int64_t>(q_heads) * n_rows, threads, [&](int64_t item) {
        int h = static_cast<int>(item / n_rows);
        int64_t r = item % n_rows;
        int64_t local = rows ? rows[r] : r;
        int64_t i = pos0 + local;                             // absolute position of the query
        int g = h / group;
        int ih = index_heads == q_heads ? h : g;
        const std::vector<char>& cv = in_v[ih];
        const std::vector<char>& cs = in_s[ih];
        double l;
        int64_t c = attention_row(q + (static_cast<int64_t>(h) * n_q + local) * d, k + static_cast<int64_t>(g) * n * d,
                                  v + static_cast<int64_t>(g) * n * d, i, d, scale,
                                  [&](int64_t j) {
                                      if (cv[j]) return true;
                                      const int64_t first = granularity * (i / granularity);
                                      for (int64_t r2 = first; r2 < first + granularity && r2 < n_pos; ++r2)
                                          if (r2 - j >= 0 && cs[r2 - j]) return true;
                                      return false;
                                  },
                                  out + item * d, &l);
        if (lse) lse[item] = l;
        if (live) live[item] = c;
    });
    return 0;
}

// Dense causal attention; chunk arguments (n_q, pos0, local rows) as for vso_sparse_attention.
int vso_dense_attention(const uint16_t* q, const uint16_t* k, const uint16_t* v,
                        int q_heads, int kv_heads, int64_t n, int d, double scale,
                        const int64_t* rows, int64_t n_rows, int64_t n_q, int64_t pos0, double* out, double* lse, int threads) {
    if (!q || !k || !v || !out) return -1;
    if (q_heads <= 0 || kv_heads <= 0 || q_heads % kv_heads || n <= 0 || d <= 0) return -1;
    if (n_q <= 0) { n_q = n; pos0 = 0; }
    if (pos0 < 0 || pos0 + n_q > n) return -1;
    if (!rows) n_rows = n_q;
    if (rows)
        for (int64_t r = 0; r < n_rows; ++r)
            if (rows[r] < 0 || rows[r] >= n_q) return -4;
    const int group = q_heads / kv_heads;
    parallel_for(static_cast<int64_t>(q_heads) * n_rows, threads, [&](int64_t item) {
        int h = static_cast<int>(item / n_rows);
        int64_t r = item % n_rows;
        int64_t local = rows ? rows[r] : r;
        int g = h / group;
        double l;
        attention_row(q + (static_cast<int64_t>(h) * n_q + local) * d, k + static_cast<int64_t>(g) * n * d,
                      v + static_cast<int64_t>(g) * n * d, pos0 + local, d, scale, [](int64_t) { return true; },
                      out + item * d, &l);
        if (lse) lse[item] = l;
    });
    return 0;
}

// Column sums A_v[j] = sum_i A[i,j] and diagonal sums A_s[o] = sum_i A[i,i-o] of the causal
// attention matrix of ONE head (q, k: [n, d] bf16), both divided by n.  Optionally also the
// recall of a vertical-slash mask: (1/n) sum_i sum_{j kept} A[i,j].
int vso_vs_aggregate(const uint16_t* q, const uint16_t* k, int64_t n, int d, double scale,
                     double* a_v, double* a_s,
                     const int32_t* idx_v, int64_t cnt_v, const int32_t* idx_s, int64_t cnt_s, double* recall) {
    if (!q || !k || !a_v || !a_s || n <= 0 || d <= 0) return -1;
    std::vector<char> cv(n, 0), cs(n, 0);
    if (recall) {
        for (int64_t t = 0; t < cnt_v; ++t) cv[idx_v[t]] = 1;
        for (int64_t t = 0; t < cnt_s; ++t) cs[idx_s[t]] = 1;
        *recall = 0.0;
    }
    for (int64_t j = 0; j < n; ++j) a_v[j] = a_s[j] = 0.0;
    std::vector<double> s(n);
    for (int64_t i = 0; i < n; ++i) {
        double m = -std::numeric_limits<double>::infinity();
        for (int64_t j = 0; j <= i; ++j) {
            double acc = 0.0;
            for (int c = 0; c < d; ++c) acc += bf16_to_f64(q[i * d + c]) * bf16_to_f64(k[j * d + c]);
            s[j] = acc * scale;
            m = std::max(m, s[j]);
        }
        double z = 0.0;
        for (int64_t j = 0; j <= i; ++j) { s[j] = std::exp(s[j] - m); z += s[j]; }
        for (int64_t j = 0; j <= i; ++j) {
            double a = s[j] / z;
            a_v[j] += a;
            a_s[i - j] += a;
            if (recall && (cv[j] || cs[i - j])) *recall += a;
        }
    }
    for (int64_t j = 0; j < n; ++j) { a_v[j] /= n; a_s[j] /= n; }
    if (recall) *recall /= n;
    return 0;
}

// Distillation loss of the VSIndexer and its gradient (paragraph "Loss function design").
// Forward as vso_index_score: A^_d = softmax over the n positions of the logits of direction d, per KV head.
// Loss, as the paper prints it (prediction first):  KL(A^ || A) = sum_t A^_t (ln A^_t - ln max(A_t, eps)),
//   L = (1 / kv_heads) * sum over heads of [ KL(A^_v || A_v) + KL(A^_s || A_s) ].
// eps floors the target (a target of exactly zero would make the term infinite).  Terms with A^_t = 0 contribute 0.
// Gradient by the chain rule, every quantity in fp64:
//   dL/dlogit_d[t] = A^_d[t] * ( (ln A^_d[t] - ln A_d[t]) - KL_d ) / kv_heads
//   z = act(pre), pre = x W_U + b_U;  dz_u = g_v W_V[u] + g_s W_S[u];  dpre_u = dz_u act'(pre_u)
//   dW_V[u] = sum_t g_v[t] z_u(t), dW_S likewise;  db_U[u] = sum_t dpre_u(t);  dW_U[c,u] = sum_t x_t[c] dpre_u(t)
// (sums over the tokens of every head; the scalar output biases get zero gradient: they cancel in the softmax).
// targets t_v, t_s: [kv_heads, n] fp64.  Outputs: loss (1), dW_U [2d, d_h], db_U, dW_V, dW_S [d_h] fp64;
// glogit_v / glogit_s optional [kv_heads, n].
int vso_index_train(const uint16_t* k, const uint16_t* v, int kv_heads, int64_t n, int d,
                    const float* W_U, const float* b_U, const float* W_V, const float* W_S, float b_V, float b_S,
                    int d_h, int act, const double* t_v, const double* t_s, double eps,
                    double* loss, double* dW_U, double* db_U, double* dW_V, double* dW_S,
                    double* glogit_v, double* glogit_s) {
    if (!k || !v || !W_U || !b_U || !W_V || !W_S || !t_v || !t_s || !loss || !dW_U || !db_U || !dW_V || !dW_S) return -1;
    if (kv_heads <= 0 || n <= 0 || d <= 0 || d_h <= 0 || act < 0 || act > 1 || !(eps > 0.0)) return -1;
    const int64_t rows = static_cast<int64_t>(kv_heads) * n;
    std::vector<double> a_v(rows), a_s(rows);
    int rc = vso_index_score(k, v, kv_heads, n, d, W_U, b_U, W_V, W_S, b_V, b_S, d_h, act, a_v.data(), a_s.data(), nullptr,
                             nullptr, 1);
    if (rc != 0) return rc;
    std::vector<double> g_v(rows, 0.0), g_s(rows, 0.0);
    double total = 0.0;
    for (int h = 0; h < kv_heads; ++h)
        for (int dir = 0; dir < 2; ++dir) {
            const double* p = (dir == 0 ? a_v.data() : a_s.data()) + static_cast<int64_t>(h) * n;
            const double* q = (dir == 0 ? t_v : t_s) + static_cast<int64_t>(h) * n;
            double* g = (dir == 0 ? g_v.data() : g_s.data()) + static_cast<int64_t>(h) * n;
            std::vector<double> diff(n, 0.0);
            double kl = 0.0;
            for (int64_t t = 0; t < n; ++t) {
                if (p[t] > 0.0) {
                    diff[t] = std::log(p[t]) - std::log(std::max(q[t], eps));
                    kl += p[t] * diff[t];
                }
            }
            for (int64_t t = 0; t < n; ++t) g[t] = p[t] * (diff[t] - kl) / kv_heads;
            total += kl;
        }
    *loss = total / kv_heads;
    for (int64_t i = 0; i < static_cast<int64_t>(2) * d * d_h; ++i) dW_U[i] = 0.0;
    for (int u = 0; u < d_h; ++u) db_U[u] = dW_V[u] = dW_S[u] = 0.0;
    std::vector<double> x(2 * d);
    for (int64_t row = 0; row < rows; ++row) {
        for (int c = 0; c < d; ++c) {
            x[c] = bf16_to_f64(k[row * d + c]);
            x[d + c] = bf16_to_f64(v[row * d + c]);
        }
        for (int u = 0; u < d_h; ++u) {
            double pre = static_cast<double>(b_U[u]);
            for (int c = 0; c < 2 * d; ++c) pre += x[c] * static_cast<double>(W_U[static_cast<int64_t>(c) * d_h + u]);
            double z = activation(pre, act);
            double slope;
            if (act == 0) {                                   // SiLU: s + x s (1 - s), s = sigmoid(x)
                double sg = 1.0 / (1.0 + std::exp(-pre));
                slope = sg + pre * sg * (1.0 - sg);
            } else {                                          // GELU: Phi(x) + x phi(x)
                double Phi = 0.5 * (1.0 + std::erf(pre / std::sqrt(2.0)));
                double phi = std::exp(-0.5 * pre * pre) / std::sqrt(2.0 * 3.14159265358979323846);
                slope = Phi + pre * phi;
            }
            dW_V[u] += g_v[row] * z;
            dW_S[u] += g_s[row] * z;
            double dpre = (g_v[row] * static_cast<double>(W_V[u]) + g_s[row] * static_cast<double>(W_S[u])) * slope;
            db_U[u] += dpre;
            for (int c = 0; c < 2 * d; ++c) dW_U[static_cast<int64_t>(c) * d_h + u] += x[c] * dpre;
        }
    }
    if (glogit_v) std::copy(g_v.begin(), g_v.end(), glogit_v);
    if (glogit_s) std::copy(g_s.begin(), g_s.end(), glogit_s);
    return 0;
}

}  // extern "C"
