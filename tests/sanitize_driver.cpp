// Host-only driver for the sanitizer leg: the batch planner (planner.cpp) and the float64 oracle
// (oracle/lora_oracle.c) built with -fsanitize=address,undefined and run over seeded random batches.
// tests/test_sanitizers.py compiles and runs it; it exits non-zero on any failed check, and the
// sanitizers abort on any invalid access or undefined operation inside the two libraries.
//
// What is checked besides memory safety: the planner's unique tables against a re-derivation written
// here (stable grouping by adapter), the exactly-once cover of the shrink and expand tile lists and of
// the fused forward's adapter stages, the status codes of invalid descriptors; the oracle against an
// exact integer evaluation of  y = x W + s (x A_a) B_a  on small integer inputs (every product and sum
// is exact in float64, so the comparison is for equality).
#include <algorithm>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <map>
#include <set>
#include <utility>
#include <vector>

#include "../include/lora_abi.h"

extern "C" {
int oracle_token_adapter(int32_t T, int32_t S, const int32_t* seg_indptr, const int32_t* seg_adapter, int32_t* tok);
void oracle_shrink(int32_t T, int32_t K, const int32_t* tok, const int32_t* rank, const double* scale, const double* x,
                   const double* const* A, int apply_scale, double* v, int32_t R, const int32_t* rows, int32_t n_rows);
void oracle_expand(int32_t T, int32_t K, int32_t N, const int32_t* tok, const int32_t* rank, const double* scale,
                   const double* x, const double* const* A, const double* const* B, const double* y_in, double* y_out,
                   const int32_t* rows, int32_t n_rows);
void oracle_expand_fast(int32_t T, int32_t K, int32_t N, const int32_t* tok, const int32_t* rank, const double* scale,
                        const double* x, const double* const* A, const double* const* B, const double* y_in,
                        double* y_out, const int32_t* rows, int32_t n_rows, int32_t max_rank);
void oracle_base(int32_t T, int32_t K, int32_t N, const double* x, const double* W, double* y, const int32_t* rows,
                 int32_t n_rows);
void oracle_forward(int32_t T, int32_t K, int32_t N, const int32_t* tok, const int32_t* rank, const double* scale,
                    const double* x, const double* W, const double* const* A, const double* const* B, double* y,
                    const int32_t* rows, int32_t n_rows, int32_t max_rank);
}

static uint64_t g_state = 0x2411091500000001ull;
static uint32_t rnd()
{
    g_state = g_state * 6364136223846793005ull + 1442695040888963407ull;
    return (uint32_t)(g_state >> 33);
}
static int rnd_in(int lo, int hi) { return lo + (int)(rnd() % (uint32_t)(hi - lo + 1)); }

#define REQUIRE(cond)                                                                      \
    do {                                                                                   \
        if (!(cond)) {                                                                     \
            std::fprintf(stderr, "check failed at %s:%d: %s\n", __FILE__, __LINE__, #cond); \
            std::exit(3);                                                                  \
        }                                                                                  \
    } while (0)

struct batch {
    std::vector<int32_t> indptr, seg_adapter, rank;
    std::vector<float> scale;
    int32_t T = 0, K = 0, N = 0, dtype = LORA_BF16, variant = LORA_VARIANT_AUTO;
    lora_batch_desc desc() const
    {
        lora_batch_desc d{};
        d.num_tokens = T;
        d.num_segments = (int32_t)seg_adapter.size();
        d.seg_indptr = indptr.data();
        d.seg_adapter = seg_adapter.data();
        d.num_adapters = (int32_t)rank.size();
        d.adapter_rank = rank.data();
        d.adapter_scale = scale.data();
        d.k = K; d.n = N; d.dtype = dtype; d.variant = variant;
        return d;
    }
};

static batch random_batch(int flavour)
{
    batch b;
    const int n_a = rnd_in(1, flavour == 2 ? 300 : 12);
    static const int aligned[] = {8, 16, 24, 32, 40, 64, 96, 128};
    static const int any[] = {0, 1, 3, 8, 12, 16, 64, 130, 200, 256};
    for (int a = 0; a < n_a; ++a) {
        b.rank.push_back(flavour == 1 ? any[rnd() % 10] : aligned[rnd() % (flavour == 2 ? 4 : 8)]);
        b.scale.push_back((float)rnd_in(-4, 8) * 0.25f);
    }
    const int S = rnd_in(0, flavour == 2 ? 400 : 30);
    const int max_len = flavour == 2 ? 2 : (flavour == 3 ? 700 : 40);
    b.indptr.push_back(0);
    for (int s = 0; s < S; ++s) {
        b.seg_adapter.push_back(rnd() % 5 == 0 ? -1 : rnd_in(0, n_a - 1));
        b.indptr.push_back(b.indptr.back() + (rnd() % 6 == 0 ? 0 : rnd_in(1, max_len)));
    }
    b.T = b.indptr.back();
    b.K = flavour == 1 ? rnd_in(1, 300) : 8 * rnd_in(1, flavour == 3 ? 640 : 80);
    b.N = flavour == 1 ? rnd_in(1, 300) : rnd_in(1, 3000);
    b.dtype = (flavour == 1 && rnd() % 2) ? LORA_F32 : LORA_BF16;
    b.variant = (int32_t)(rnd() % 3);
    return b;
}

static void check_plan(const batch& b)
{
    const lora_batch_desc d = b.desc();
    lora_plan* p = nullptr;
    REQUIRE(lora_plan_create(&d, &p) == LORA_OK && p);
    int32_t R = 0;
    size_t v_bytes = 0, ws_bytes = 0;
    REQUIRE(lora_plan_query(p, &R, &v_bytes, &ws_bytes) == LORA_OK);
    lora_plan_view v{};
    REQUIRE(lora_plan_export(p, &v) == LORA_OK);
    REQUIRE(v.num_tokens == b.T && R >= 8 && R % 8 == 0);
    REQUIRE(v_bytes == (size_t)v.v_parts * (size_t)b.T * (size_t)R * 4 && ws_bytes >= v_bytes);

    // the unique tables, re-derived: adapter of every token, stable grouping by adapter id
    std::vector<int32_t> tok((size_t)b.T, -1);
    for (size_t s = 0; s < b.seg_adapter.size(); ++s)
        for (int32_t t = b.indptr[s]; t < b.indptr[s + 1]; ++t) {
            const int32_t a = b.seg_adapter[s];
            tok[t] = (a >= 0 && b.rank[a] > 0) ? a : -1;
        }
    std::vector<int32_t> perm;
    for (int32_t t = 0; t < b.T; ++t)
        if (tok[t] >= 0) perm.push_back(t);
    std::stable_sort(perm.begin(), perm.end(), [&](int32_t x, int32_t y) { return tok[x] < tok[y]; });
    REQUIRE(v.num_active == (int32_t)perm.size());
    for (int32_t t = 0; t < b.T; ++t) REQUIRE(v.token_adapter[t] == tok[t]);
    for (size_t i = 0; i < perm.size(); ++i) REQUIRE(v.perm[i] == perm[i]);
    int32_t g = 0;
    for (size_t i = 0; i < perm.size(); ++i)
        if (i == 0 || tok[perm[i]] != tok[perm[i - 1]]) {
            REQUIRE(g < v.num_groups && v.group_adapter[g] == tok[perm[i]] && v.group_offset[g] == (int32_t)i);
            ++g;
        }
    REQUIRE(g == v.num_groups && v.group_offset[g] == (int32_t)perm.size());

    REQUIRE(v.shrink_kernel_family == LORA_VARIANT_TILED || v.kernel_family != LORA_VARIANT_TILED);
    if (v.shrink_kernel_family == LORA_VARIANT_TILED) {
        // exactly-once cover: shrink tiles over (token, rank index) per K part, expand tiles over (token, feature);
        // a plan whose shrink alone is tiled has no expand tiles
        const int32_t P = v.v_parts;
        REQUIRE(P == 1 || P == 2 || P == 4 || P == 8);
        // K parts per adapter (bits 12..15 of a shrink tile's shape): the same on every tile of the adapter, <= P
        std::map<int32_t, int32_t> parts_of;
        for (int32_t i = 0; i < v.num_shrink_tiles; ++i) {
            const lora_tile& t = v.shrink_tiles[i];
            const int32_t parts = (t.shape >> 12) & 15;
            REQUIRE(parts >= 1 && parts <= P && ((t.shape >> 8) & 15) < parts);
            REQUIRE(parts_of.emplace(t.adapter, parts).first->second == parts);
        }
        for (int part = 0; part < P; ++part) {
            std::vector<std::vector<int32_t>> canvas(perm.size());
            for (size_t i = 0; i < perm.size(); ++i) canvas[i].assign((size_t)b.rank[tok[perm[i]]], 0);
            for (int32_t i = 0; i < v.num_shrink_tiles; ++i) {
                const lora_tile& t = v.shrink_tiles[i];
                if (((t.shape >> 8) & 15) != part) continue;
                REQUIRE(t.row0 >= 0 && t.nrows > 0 && t.row0 + t.nrows <= (int32_t)perm.size());
                REQUIRE(t.c0 >= 0 && t.cn > 0 && t.c0 + t.cn <= b.rank[t.adapter]);
                for (int32_t r = t.row0; r < t.row0 + t.nrows; ++r) {
                    REQUIRE(tok[perm[r]] == t.adapter);
                    for (int32_t c = t.c0; c < t.c0 + t.cn; ++c) canvas[r][c] += 1;
                }
            }
            for (size_t i = 0; i < perm.size(); ++i)
                for (int32_t c : canvas[i]) REQUIRE(c == (part < parts_of.at(tok[perm[i]]) ? 1 : 0));
        }
        if (v.kernel_family != LORA_VARIANT_TILED) REQUIRE(v.num_expand_tiles == 0);
        std::vector<std::vector<int32_t>> canvas(perm.size(), std::vector<int32_t>((size_t)b.N, 0));
        for (int32_t i = 0; i < v.num_expand_tiles; ++i) {
            const lora_tile& t = v.expand_tiles[i];
            REQUIRE(t.row0 >= 0 && t.nrows > 0 && t.row0 + t.nrows <= (int32_t)perm.size());
            REQUIRE(t.c0 >= 0 && t.cn > 0 && t.c0 + t.cn <= b.N);
            for (int32_t r = t.row0; r < t.row0 + t.nrows; ++r) {
                REQUIRE(tok[perm[r]] == t.adapter);
                for (int32_t c = t.c0; c < t.c0 + t.cn; ++c) canvas[r][c] += 1;
            }
        }
        for (auto& row : canvas)
            for (int32_t c : row) REQUIRE(c == (v.kernel_family == LORA_VARIANT_TILED ? 1 : 0));
    } else {
        REQUIRE(v.num_shrink_tiles == 0 && v.num_expand_tiles == 0);
    }
    if (v.num_gemm_rows > 0) {
        // fused forward: the row order is a permutation; every 256-row tile lists each (adapter present, block of 32
        // of its 2 r columns) exactly once
        REQUIRE(v.num_gemm_rows == b.T && v.num_gemm_tiles == (b.T + 255) / 256);
        std::vector<int> seen((size_t)b.T, 0);
        for (int32_t i = 0; i < b.T; ++i) {
            REQUIRE(v.gemm_order[i] >= 0 && v.gemm_order[i] < b.T);
            seen[v.gemm_order[i]] += 1;
        }
        for (int s : seen) REQUIRE(s == 1);
        REQUIRE(v.gemm_stage_offset[0] == 0);
        for (int32_t tile = 0; tile < v.num_gemm_tiles; ++tile) {
            std::set<std::pair<int32_t, int32_t>> want, got;
            for (int32_t i = tile * 256; i < std::min(b.T, tile * 256 + 256); ++i) {
                const int32_t a = tok[v.gemm_order[i]];
                if (a < 0) continue;
                for (int32_t jb = 0; jb * 64 < 2 * b.rank[a]; ++jb) want.insert({a, jb});
            }
            REQUIRE(v.gemm_stage_offset[tile + 1] >= v.gemm_stage_offset[tile]);
            for (int32_t i = v.gemm_stage_offset[tile]; i < v.gemm_stage_offset[tile + 1]; ++i)
                REQUIRE(got.insert({v.gemm_stage[i] & 0xffffff, v.gemm_stage[i] >> 24}).second);
            REQUIRE(got == want);
        }
    }
    // equal descriptors give equal plans
    lora_plan* q = nullptr;
    REQUIRE(lora_plan_create(&d, &q) == LORA_OK);
    lora_plan_view w{};
    REQUIRE(lora_plan_export(q, &w) == LORA_OK);
    REQUIRE(w.num_shrink_tiles == v.num_shrink_tiles && w.num_expand_tiles == v.num_expand_tiles);
    for (int32_t i = 0; i < v.num_shrink_tiles; ++i) {
        const lora_tile &x = v.shrink_tiles[i], &y = w.shrink_tiles[i];
        REQUIRE(x.adapter == y.adapter && x.row0 == y.row0 && x.nrows == y.nrows && x.c0 == y.c0 && x.cn == y.cn &&
                x.shape == y.shape);
    }
    lora_plan_destroy(q);
    lora_plan_destroy(p);
}

// Mixture mode: the plan of the tokens' own branches plus the removal of the merged adapter over all other tokens.
static void check_mixture(const batch& b)
{
    if (b.rank.empty()) return;
    const int32_t m = (int32_t)(rnd() % b.rank.size());
    lora_batch_desc d = b.desc();
    d.merged_adapter_plus1 = m + 1;
    lora_plan* p = nullptr;
    REQUIRE(lora_plan_create(&d, &p) == LORA_OK && p);
    lora_plan_view v{};
    REQUIRE(lora_plan_export(p, &v) == LORA_OK);
    size_t v_bytes = 0, ws_bytes = 0;
    int32_t R = 0;
    REQUIRE(lora_plan_query(p, &R, &v_bytes, &ws_bytes) == LORA_OK);
    if (b.rank[m] == 0) {
        REQUIRE(v.merged_adapter == -1 && v.num_unmerge == 0);
    } else {
        REQUIRE(v.merged_adapter == m);
        std::vector<int32_t> want;
        for (size_t s = 0; s < b.seg_adapter.size(); ++s)
            for (int32_t t = b.indptr[s]; t < b.indptr[s + 1]; ++t) {
                if (b.seg_adapter[s] != m) want.push_back(t);
                REQUIRE(v.token_adapter[t] != m);
            }
        REQUIRE(v.num_unmerge == (int32_t)want.size());
        for (size_t i = 0; i < want.size(); ++i) REQUIRE(v.unmerge_perm[i] == want[i]);
        REQUIRE(v.unmerge_v_offset % 256 == 0 && v.unmerge_v_offset >= (size_t)v.v_parts * (size_t)b.T * (size_t)R * 4);
        REQUIRE(v_bytes == v.unmerge_v_offset + (size_t)v.unmerge_v_parts * (size_t)b.T * (size_t)v.unmerge_v_row_stride * 4);
        REQUIRE(ws_bytes >= v_bytes);
        for (int32_t i = 0; i < v.num_unmerge_shrink_tiles; ++i) {
            const lora_tile& t = v.unmerge_shrink_tiles[i];
            REQUIRE(t.adapter == m && t.row0 >= 0 && t.nrows > 0 && t.row0 + t.nrows <= v.num_unmerge);
            REQUIRE(t.c0 >= 0 && t.cn > 0 && t.c0 + t.cn <= b.rank[m]);
        }
        for (int32_t i = 0; i < v.num_unmerge_expand_tiles; ++i) {
            const lora_tile& t = v.unmerge_expand_tiles[i];
            REQUIRE(t.adapter == m && t.row0 >= 0 && t.nrows > 0 && t.row0 + t.nrows <= v.num_unmerge);
            REQUIRE(t.c0 >= 0 && t.cn > 0 && t.c0 + t.cn <= b.N);
        }
        // marked stages only in tiles that hold a token of the removal, and then all of the merged adapter's blocks
        for (int32_t tile = 0; tile < v.num_gemm_tiles; ++tile) {
            bool needs = false;
            for (int32_t q = tile * 256; q < std::min((tile + 1) * 256, b.T); ++q) {
                const int32_t t = v.gemm_order[q];
                REQUIRE(t >= 0 && t < b.T);
                needs = needs || std::binary_search(want.begin(), want.end(), t);
            }
            int32_t marked = 0;
            for (int32_t i = v.gemm_stage_offset[tile]; i < v.gemm_stage_offset[tile + 1]; ++i)
                if (v.gemm_stage[i] & (1 << 23)) {
                    REQUIRE((v.gemm_stage[i] & 0x7fffff) == m && (v.gemm_stage[i] >> 24) == marked);
                    ++marked;
                }
            REQUIRE(marked == (needs ? (2 * b.rank[m] + 63) / 64 : 0));
        }
    }
    lora_plan_destroy(p);
}

static void check_errors()
{
    batch b = random_batch(0);
    lora_plan* p = nullptr;
    lora_batch_desc d = b.desc();
    REQUIRE(lora_plan_create(nullptr, &p) == LORA_ERR_INVALID_ARG);
    REQUIRE(lora_plan_create(&d, nullptr) == LORA_ERR_INVALID_ARG);
    d = b.desc(); d.k = 0;
    REQUIRE(lora_plan_create(&d, &p) == LORA_ERR_INVALID_ARG && p == nullptr);
    d = b.desc(); d.num_tokens += 1;
    REQUIRE(lora_plan_create(&d, &p) == LORA_ERR_INVALID_ARG);
    d = b.desc(); d.dtype = 7;
    REQUIRE(lora_plan_create(&d, &p) == LORA_ERR_INVALID_ARG);
    d = b.desc(); d.seg_indptr = nullptr;
    REQUIRE(lora_plan_create(&d, &p) == LORA_ERR_INVALID_ARG);
    batch c = b;
    c.rank[0] = LORA_MAX_RANK + 1;
    d = c.desc();
    REQUIRE(lora_plan_create(&d, &p) == LORA_ERR_INVALID_ARG);
    if (!b.seg_adapter.empty()) {
        c = b;
        c.seg_adapter[0] = (int32_t)b.rank.size();
        d = c.desc();
        REQUIRE(lora_plan_create(&d, &p) == LORA_ERR_INVALID_ARG);
    }
    REQUIRE(lora_plan_query(nullptr, nullptr, nullptr, nullptr) == LORA_ERR_INVALID_ARG);
    lora_plan_destroy(nullptr);
    for (int s = 0; s < 7; ++s) REQUIRE(lora_status_str((lora_status)s) != nullptr);
}

// y = x W + s (x A_a) B_a in exact integer arithmetic against every oracle entry point
static void check_oracle(int round)
{
    const int T = rnd_in(1, 9), K = rnd_in(1, 7), N = rnd_in(1, 6), n_a = rnd_in(1, 4);
    std::vector<int32_t> rank(n_a), indptr{0}, seg_ad;
    std::vector<double> scale(n_a);
    int max_rank = 0;
    for (int a = 0; a < n_a; ++a) {
        rank[a] = rnd_in(0, 3);
        scale[a] = rnd_in(-3, 3);
        max_rank = std::max(max_rank, (int)rank[a]);
    }
    while (indptr.back() < T) {
        seg_ad.push_back(rnd_in(-1, n_a - 1));
        indptr.push_back(std::min(T, indptr.back() + rnd_in(0, 3)));
    }
    const int S = (int)seg_ad.size();
    auto ints = [&](size_t n) { std::vector<double> v(n); for (auto& e : v) e = rnd_in(-4, 4); return v; };
    std::vector<double> x = ints((size_t)T * K), W = ints((size_t)K * N);
    std::vector<std::vector<double>> A(n_a), B(n_a);
    std::vector<const double*> Ap(n_a), Bp(n_a);
    for (int a = 0; a < n_a; ++a) {
        A[a] = ints((size_t)K * rank[a] + 1);       // +1: never an empty vector's null data()
        B[a] = ints((size_t)rank[a] * N + 1);
        Ap[a] = A[a].data();
        Bp[a] = B[a].data();
    }
    std::vector<int32_t> tok(T);
    REQUIRE(oracle_token_adapter(T, S, indptr.data(), seg_ad.data(), tok.data()) == 0);
    const int R = std::max(1, max_rank);
    std::vector<double> v((size_t)T * R, -1.0), y((size_t)T * N), yb((size_t)T * N), ye((size_t)T * N), yf((size_t)T * N);
    oracle_shrink(T, K, tok.data(), rank.data(), scale.data(), x.data(), Ap.data(), 1, v.data(), R, nullptr, 0);
    oracle_base(T, K, N, x.data(), W.data(), yb.data(), nullptr, 0);
    oracle_expand(T, K, N, tok.data(), rank.data(), scale.data(), x.data(), Ap.data(), Bp.data(), yb.data(), ye.data(), nullptr, 0);
    oracle_expand_fast(T, K, N, tok.data(), rank.data(), scale.data(), x.data(), Ap.data(), Bp.data(), yb.data(), yf.data(), nullptr, 0, max_rank);
    oracle_forward(T, K, N, tok.data(), rank.data(), scale.data(), x.data(), W.data(), Ap.data(), Bp.data(), y.data(), nullptr, 0, max_rank);
    for (int t = 0; t < T; ++t) {
        int a = -1;
        for (int s = 0; s < S; ++s)
            if (indptr[s] <= t && t < indptr[s + 1]) a = seg_ad[s];
        REQUIRE(tok[t] == a);
        const int r = (a >= 0) ? rank[a] : 0;
        std::vector<long long> vj(R, 0);
        for (int j = 0; j < r; ++j)
            for (int k = 0; k < K; ++k) vj[j] += (long long)x[(size_t)t * K + k] * (long long)A[a][(size_t)k * r + j];
        for (int j = 0; j < R; ++j) REQUIRE(v[(size_t)t * R + j] == (double)(j < r ? (long long)scale[a] * vj[j] : 0));
        for (int n = 0; n < N; ++n) {
            long long base = 0, delta = 0;
            for (int k = 0; k < K; ++k) base += (long long)x[(size_t)t * K + k] * (long long)W[(size_t)k * N + n];
            for (int j = 0; j < r; ++j) delta += vj[j] * (long long)B[a][(size_t)j * N + n];
            const double want = (double)(base + (r ? (long long)scale[a] * delta : 0));
            REQUIRE(yb[(size_t)t * N + n] == (double)base);
            REQUIRE(y[(size_t)t * N + n] == want && ye[(size_t)t * N + n] == want && yf[(size_t)t * N + n] == want);
        }
    }
    // row selection: the last and the first token only
    const int32_t rows[2] = {T - 1, 0};
    std::vector<double> ys((size_t)2 * N);
    oracle_forward(T, K, N, tok.data(), rank.data(), scale.data(), x.data(), W.data(), Ap.data(), Bp.data(), ys.data(), rows, 2, max_rank);
    for (int n = 0; n < N; ++n) REQUIRE(ys[n] == y[(size_t)(T - 1) * N + n] && ys[(size_t)N + n] == y[n]);
    (void)round;
}

int main()
{
    int32_t tuning[32];
    lora_tuning_get(tuning, 32);
    lora_tuning_set(tuning, 32);
    for (int i = 0; i < 220; ++i) check_plan(random_batch(i % 4));
    for (int i = 0; i < 120; ++i) check_mixture(random_batch(i % 4));
    {   // no segments, no tokens
        batch b;
        b.indptr = {0}; b.rank = {8}; b.scale = {1.f}; b.K = 64; b.N = 64;
        check_plan(b);
    }
    check_errors();
    for (int i = 0; i < 200; ++i) check_oracle(i);
    std::puts("sanitize_driver: ok");
    return 0;
}
