// Runs every entry point of the fp64 oracle once on small deterministic inputs.  Built together with
// oracle/vs_oracle.cpp under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only): any out-of-bounds access,
// use of uninitialised stack, signed overflow or misaligned access in the oracle aborts the run.
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <vector>

extern "C" {
uint16_t vso_f64_to_bf16(double x);
int vso_rope_bf16(uint16_t* x, int heads, int64_t n, int d, int64_t pos0, double theta_base, int pairing, int threads);
int vso_index_score(const uint16_t* k, const uint16_t* v, int kv_heads, int64_t n, int d, const float* W_U, const float* b_U,
                    const float* W_V, const float* W_S, float b_V, float b_S, int d_h, int act, double* a_v, double* a_s,
                    double* logits_v, double* logits_s, int threads);
int vso_select(const float* scores, int heads, int64_t n, int mode, double tau, int64_t k_fixed, int64_t n_forced, int64_t cap,
               int32_t* idx, int32_t* cnt, int32_t* status, int64_t* k_out);
int vso_sparse_attention(const uint16_t* q, const uint16_t* k, const uint16_t* v, int q_heads, int kv_heads, int64_t n, int d,
                         double scale, const int32_t* idx_v, const int32_t* cnt_v, int64_t cap_v, const int32_t* idx_s,
                         const int32_t* cnt_s, int64_t cap_s, int index_heads, int64_t granularity, const int64_t* rows,
                         int64_t n_rows, int64_t n_q, int64_t pos0, double* out, double* lse, int64_t* live, int threads);
int vso_dense_attention(const uint16_t* q, const uint16_t* k, const uint16_t* v, int q_heads, int kv_heads, int64_t n, int d,
                        double scale, const int64_t* rows, int64_t n_rows, int64_t n_q, int64_t pos0, double* out, double* lse,
                        int threads);
int vso_vs_aggregate(const uint16_t* q, const uint16_t* k, int64_t n, int d, double scale, double* a_v, double* a_s,
                     const int32_t* idx_v, int64_t cnt_v, const int32_t* idx_s, int64_t cnt_s, double* recall);
}

static uint64_t state = 88172645463325252ull;
static double unit() {                                      // xorshift64, values in (-1, 1)
    state ^= state << 13;
    state ^= state >> 7;
    state ^= state << 17;
    return static_cast<double>(state >> 11) / 4503599627370496.0 - 1.0;
}

#define CHECK(x) do { if (!(x)) { std::fprintf(stderr, "check failed: %s (line %d)\n", #x, __LINE__); return 1; } } while (0)

int main() {
    const int hq = 4, hk = 2, d = 16, d_h = 8;
    const int64_t n = 37;
    std::vector<uint16_t> q(hq * n * d), k(hk * n * d), v(hk * n * d);
    for (auto& x : q) x = vso_f64_to_bf16(unit());
    for (auto& x : k) x = vso_f64_to_bf16(unit());
    for (auto& x : v) x = vso_f64_to_bf16(unit());
    CHECK(vso_rope_bf16(q.data(), hq, n, d, 5, 1e4, 0, 2) == 0);
    CHECK(vso_rope_bf16(k.data(), hk, n, d, 5, 1e4, 1, 1) == 0);

    std::vector<float> W_U(2 * d * d_h), b_U(d_h), W_V(d_h), W_S(d_h);
    for (auto& x : W_U) x = static_cast<float>(unit());
    for (auto& x : b_U) x = static_cast<float>(unit());
    for (auto& x : W_V) x = static_cast<float>(unit());
    for (auto& x : W_S) x = static_cast<float>(unit());
    std::vector<double> a_v(hk * n), a_s(hk * n), lv(hk * n), ls(hk * n);
    for (int act = 0; act < 2; ++act)
        CHECK(vso_index_score(k.data(), v.data(), hk, n, d, W_U.data(), b_U.data(), W_V.data(), W_S.data(), 0.5f, -0.5f, d_h, act,
                              a_v.data(), a_s.data(), lv.data(), ls.data(), 3) == 0);

    std::vector<float> sc(hk * n);
    for (int64_t i = 0; i < hk * n; ++i) sc[i] = static_cast<float>(a_v[i]);
    sc[3] = NAN;
    sc[4] = -1.f;
    sc[5] = 2.f;
    const int64_t cap = 9;
    std::vector<int32_t> idx_v(hk * cap), cnt_v(hk), st(hk), idx_s(hk * cap), cnt_s(hk);
    std::vector<int64_t> kk(hk);
    CHECK(vso_select(sc.data(), hk, n, 0, 0.9, 0, 2, cap, idx_v.data(), cnt_v.data(), st.data(), kk.data()) == 0);
    CHECK(vso_select(sc.data(), hk, n, 1, 0.0, 5, 3, cap, idx_s.data(), cnt_s.data(), st.data(), nullptr) == 0);
    CHECK(vso_select(sc.data(), hk, n, 0, 1.0, 0, 0, n, std::vector<int32_t>(hk * n).data(), cnt_s.data(), nullptr, nullptr) == 0);
    CHECK(vso_select(sc.data(), hk, n, 1, 0.0, 5, 3, cap, idx_s.data(), cnt_s.data(), st.data(), nullptr) == 0);

    const int64_t rows[3] = {0, 17, n - 1};
    std::vector<double> out(hq * n * d), lse(hq * n);
    std::vector<int64_t> live(hq * n);
    for (int64_t g : {1, 4, 32}) {
        CHECK(vso_sparse_attention(q.data(), k.data(), v.data(), hq, hk, n, d, 0.25, idx_v.data(), cnt_v.data(), cap, idx_s.data(),
                                   cnt_s.data(), cap, hk, g, nullptr, 0, 0, 0, out.data(), lse.data(), live.data(), 2) == 0);
        CHECK(vso_sparse_attention(q.data(), k.data(), v.data(), hq, hk, n, d, 0.25, idx_v.data(), cnt_v.data(), cap, idx_s.data(),
                                   cnt_s.data(), cap, hk, g, rows, 3, 0, 0, out.data(), lse.data(), nullptr, 1) == 0);
    }
    // a chunk: 10 query rows at positions n - 10 .. n - 1 (the first 10 rows of each head of q serve as the chunk's queries);
    // a chunk that would run past the keys is refused
    const int64_t crow[2] = {0, 9};
    CHECK(vso_sparse_attention(q.data(), k.data(), v.data(), hq, hk, n, d, 0.25, idx_v.data(), cnt_v.data(), cap, idx_s.data(),
                               cnt_s.data(), cap, hk, 4, crow, 2, 10, n - 10, out.data(), lse.data(), live.data(), 2) == 0);
    CHECK(vso_sparse_attention(q.data(), k.data(), v.data(), hq, hk, n, d, 0.25, idx_v.data(), cnt_v.data(), cap, idx_s.data(),
                               cnt_s.data(), cap, hk, 1, nullptr, 0, 10, n - 9, out.data(), lse.data(), live.data(), 2) == -1);
    CHECK(vso_dense_attention(q.data(), k.data(), v.data(), hq, hk, n, d, 0.25, nullptr, 0, 0, 0, out.data(), lse.data(), 2) == 0);
    CHECK(vso_dense_attention(q.data(), k.data(), v.data(), hq, hk, n, d, 0.25, rows, 3, 0, 0, out.data(), nullptr, 1) == 0);
    CHECK(vso_dense_attention(q.data(), k.data(), v.data(), hq, hk, n, d, 0.25, nullptr, 0, 10, n - 10, out.data(), lse.data(), 1) == 0);
    double rec = 0.0;
    CHECK(vso_vs_aggregate(q.data(), k.data(), n, d, 0.25, a_v.data(), a_s.data(), idx_v.data(), cnt_v[0], idx_s.data(), cnt_s[0],
                           &rec) == 0);
    CHECK(rec > 0.0 && rec <= 1.0 + 1e-12);
    std::puts("oracle sanitizer run ok");
    return 0;
}
