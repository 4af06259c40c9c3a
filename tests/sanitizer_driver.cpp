// Host-side checks meant to run under AddressSanitizer and UndefinedBehaviorSanitizer (built and run by
// tests/test_sanitizer_build.py; plain C++, no HIP, no GPU).  Linked with the host planner (ttc_plan.cpp,
// ttc_cache.cpp) and, as the checker, the C oracle.
//
//  * planner: plans for a spread of problems (every data type, leading dimensions, odd and size-1
//    extents, 1 to 6 indices), the complete candidate list, and for sampled candidates the host replay
//    of the kernels' index arithmetic (ttc_debug_emulate_map), whose element map must be the oracle's;
//  * plan store: store / look-up round trip, a damaged line, a missing file;
//  * refusals: every error path of ttc_plan_create_ex;
//  * oracle: all eight data types on small tensors, slabs of 1, 3 and 4 threads bit-identical, the
//    identity permutation equal to the scalar statement written out.
// Any sanitizer report aborts the program; every mismatch prints a line and makes the exit status 1.
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <string>
#include <vector>

#include "ttc.h"
#include "ttc_aux.h"

extern "C" int ttc_oracle_transpose_ld(int dtype, int ndim, const int64_t* sizes, const int* perm,
                                       const int64_t* lda, const int64_t* ldb, const void* alpha,
                                       const void* beta, const void* A, void* B, int nthreads);

static int g_failures = 0;
#define EXPECT(cond, ...) do { if (!(cond)) { ++g_failures; std::printf("FAIL %s:%d: ", __FILE__, __LINE__); std::printf(__VA_ARGS__); std::printf("\n"); } } while (0)

struct Case {
    int dtype, ndim;
    int64_t sizes[6];
    int perm[6];
    int64_t lda[6], ldb[6];       // lda[0] == 0: dense
    double alpha, beta;
};

static const Case kCases[] = {
    {TTC_F32, 2, {37, 19}, {1, 0}, {0}, {0}, 1.0, 0.0},
    {TTC_F32, 3, {70, 33, 45}, {2, 0, 1}, {0}, {0}, 1.5, 0.0},
    {TTC_F32, 3, {96, 20, 31}, {0, 2, 1}, {0}, {0}, 1.0, 0.0},
    {TTC_F64, 4, {9, 8, 7, 11}, {3, 2, 1, 0}, {0}, {0}, 0.75, 1.25},
    {TTC_C64, 4, {8, 20, 12, 6}, {3, 1, 0, 2}, {0}, {0}, 0.5, 1.0},
    {TTC_C128, 3, {5, 17, 9}, {1, 2, 0}, {0}, {0}, 1.0, 0.0},
    {TTC_F32, 6, {4, 5, 3, 6, 2, 7}, {5, 3, 1, 0, 4, 2}, {0}, {0}, 2.0, -1.0},
    {TTC_F32, 5, {6, 1, 5, 1, 9}, {4, 3, 2, 1, 0}, {0}, {0}, 1.0, 0.0},          // size-1 extents
    {TTC_F32, 1, {5000}, {0}, {0}, {0}, 1.0, 0.0},
    {TTC_F64_F32, 3, {37, 9, 21}, {2, 1, 0}, {40, 9, 23}, {21, 11, 37}, 0.75, 1.25},   // sub-tensors
    {TTC_F32_F64, 3, {12, 7, 10}, {1, 0, 2}, {12, 9, 10}, {8, 12, 11}, 1.0, 0.0},
    {TTC_C64_C128, 2, {33, 14}, {1, 0}, {35, 14}, {14, 40}, 1.0, 0.0},
    {TTC_C128_C64, 3, {6, 10, 4}, {2, 0, 1}, {0}, {0}, 1.0, 0.5},
    {TTC_F32, 4, {24, 20, 6, 5}, {1, 0, 3, 2}, {0}, {0}, 1.0, 0.0},
};

static int64_t prod(const int64_t* v, int n) { int64_t p = 1; for (int i = 0; i < n; ++i) p *= v[i]; return p; }

// The element map of a problem, as the oracle moves a tensor that holds its own linear offsets
// (double precision: exact for every offset that occurs here).
static std::vector<double> oracle_map(const Case& c, int64_t span_a, int64_t span_b)
{
    std::vector<double> A((size_t)span_a), B((size_t)span_b, -1.0);
    for (int64_t i = 0; i < span_a; ++i) A[(size_t)i] = (double)i;
    const double one = 1.0, zero = 0.0;
    const int rc = ttc_oracle_transpose_ld(TTC_F64, c.ndim, c.sizes, c.perm, c.lda[0] ? c.lda : nullptr,
                                           c.ldb[0] ? c.ldb : nullptr, &one, &zero, A.data(), B.data(), 1);
    EXPECT(rc == 0, "oracle refused a valid problem (%d)", rc);
    return B;
}

static void check_planner()
{
    const std::string store = std::string(std::getenv("TMPDIR") ? std::getenv("TMPDIR") : "/tmp") + "/ttc_sanitizer_plans.txt";
    std::remove(store.c_str());
    for (const Case& c : kCases) {
        float af[2] = {(float)c.alpha, 0.f}, bf[2] = {(float)c.beta, 0.f};
        double ad[2] = {c.alpha, 0.0}, bd[2] = {c.beta, 0.0};
        const bool wide = !(c.dtype == TTC_F32 || c.dtype == TTC_C64);
        const void* al = wide ? (const void*)ad : (const void*)af;
        const void* be = wide ? (const void*)bd : (const void*)bf;
        ttc_plan_t p = ttc_plan_create_ex(c.dtype, c.ndim, c.sizes, c.perm, c.lda[0] ? c.lda : nullptr,
                                          c.ldb[0] ? c.ldb : nullptr, al, be);
        EXPECT(p != nullptr, "plan refused: status %d", ttc_last_status());
        if (!p) continue;
        ttc_plan_info_t info;
        EXPECT(ttc_plan_get_info(p, &info) == TTC_OK, "get_info");
        EXPECT(info.elements == prod(c.sizes, c.ndim), "elements");
        const std::vector<double> want = oracle_map(c, info.span_a, info.span_b);
        const int n = ttc_plan_candidate_count(p);
        EXPECT(n >= 1, "candidate count %d", n);
        std::vector<int64_t> got((size_t)info.span_b);
        const int step = n > 40 ? n / 40 : 1;
        for (int k = 0; k < n; k += step) {
            EXPECT(ttc_plan_select_candidate(p, k) == TTC_OK, "select %d", k);
            const int st = ttc_debug_emulate_map(p, got.data());
            EXPECT(st == TTC_OK, "replay of candidate %d of case dtype %d ndim %d: status %d", k, c.dtype, c.ndim, st);
            if (st != TTC_OK) continue;
            int64_t bad = 0;
            for (int64_t o = 0; o < info.span_b; ++o) bad += ((double)got[(size_t)o] != want[(size_t)o]);
            EXPECT(bad == 0, "candidate %d: %lld elements land elsewhere than the oracle puts them", k, (long long)bad);
        }
        // plan store round trip on the last candidate looked at
        ttc_plan_info_t before;
        ttc_plan_get_info(p, &before);
        EXPECT(ttc_plan_cache_store(p, store.c_str()) == TTC_OK, "store");
        EXPECT(ttc_plan_select_candidate(p, 0) == TTC_OK, "select 0");
        EXPECT(ttc_plan_cache_lookup(p, store.c_str()) == TTC_OK, "look-up after store");
        ttc_plan_info_t after;
        ttc_plan_get_info(p, &after);
        EXPECT(after.candidate_index == before.candidate_index, "look-up selected %d, stored %d", after.candidate_index, before.candidate_index);
        EXPECT(ttc_plan_cache_lookup(p, "/nonexistent/dir/plans.txt") == TTC_ERR_NOT_FOUND, "missing file");
        ttc_plan_destroy(p);
    }
    {   // a damaged line for a known problem is "not found" and leaves the plan alone
        const Case& c = kCases[0];
        ttc_plan_t p = ttc_plan_create(c.dtype, c.ndim, c.sizes, c.perm, nullptr, nullptr);
        const std::string bad = store + ".bad";
        std::FILE* f = std::fopen(bad.c_str(), "w");
        if (f) { std::fputs("ttc4 gfx950 0 1 2 37 19 1 0 1 37 19 1 | 1 2 x 4 | 0 0 99 12\n", f); std::fclose(f); }
        ttc_plan_info_t a, b;
        ttc_plan_get_info(p, &a);
        EXPECT(ttc_plan_cache_lookup(p, bad.c_str()) == TTC_ERR_NOT_FOUND, "damaged line accepted");
        ttc_plan_get_info(p, &b);
        EXPECT(a.candidate_index == b.candidate_index && a.nt_a == b.nt_a && a.xcd_remap == b.xcd_remap, "plan changed by a refused entry");
        ttc_plan_destroy(p);
        std::remove(bad.c_str());
    }
    std::remove(store.c_str());
}

static void check_refusals()
{
    const int64_t s3[3] = {4, 5, 6};
    const int p3[3] = {2, 0, 1}, twice[3] = {0, 0, 1}, range[3] = {0, 1, 3};
    const int64_t zero[3] = {4, 0, 6}, small_ld[3] = {3, 5, 6};
    EXPECT(!ttc_plan_create(TTC_F32, 3, nullptr, p3, nullptr, nullptr) && ttc_last_status() == TTC_ERR_NULL_POINTER, "null sizes");
    EXPECT(!ttc_plan_create(TTC_F32, 0, s3, p3, nullptr, nullptr) && ttc_last_status() == TTC_ERR_INVALID_VALUE, "ndim 0");
    EXPECT(!ttc_plan_create(TTC_F32, 7, s3, p3, nullptr, nullptr) && ttc_last_status() == TTC_ERR_INVALID_VALUE, "ndim 7");
    EXPECT(!ttc_plan_create(99, 3, s3, p3, nullptr, nullptr) && ttc_last_status() == TTC_ERR_UNSUPPORTED_DTYPE, "dtype");
    EXPECT(!ttc_plan_create(TTC_F32, 3, s3, twice, nullptr, nullptr) && ttc_last_status() == TTC_ERR_INVALID_PERM, "repeated index");
    EXPECT(!ttc_plan_create(TTC_F32, 3, s3, range, nullptr, nullptr) && ttc_last_status() == TTC_ERR_INVALID_PERM, "index out of range");
    EXPECT(!ttc_plan_create(TTC_F32, 3, zero, p3, nullptr, nullptr) && ttc_last_status() == TTC_ERR_INVALID_VALUE, "extent 0");
    EXPECT(!ttc_plan_create_ex(TTC_F32, 3, s3, p3, small_ld, nullptr, nullptr, nullptr) && ttc_last_status() == TTC_ERR_INVALID_VALUE, "lda below extent");
    const int64_t huge[3] = {INT64_MAX / 4, 8, 8};
    EXPECT(!ttc_plan_create(TTC_F32, 3, huge, p3, nullptr, nullptr) && ttc_last_status() == TTC_ERR_OVERFLOW, "overflow");
    EXPECT(ttc_plan_destroy(nullptr) == TTC_OK, "destroy(NULL)");
    EXPECT(ttc_plan_get_info(nullptr, nullptr) == TTC_ERR_NULL_POINTER, "get_info(NULL)");
    EXPECT(ttc_plan_candidate_count(nullptr) < 0, "count(NULL)");
}

// deterministic values in [-1, 1)
static double draw(uint64_t* state)
{
    *state = *state * 6364136223846793005ull + 1442695040888963407ull;
    return (double)((*state >> 11) & ((1ull << 53) - 1)) / (double)(1ull << 52) - 1.0;
}

static void check_oracle()
{
    const int64_t sizes[4] = {7, 5, 6, 3};
    const int perm[4] = {2, 0, 3, 1};
    const int64_t n = prod(sizes, 4);
    for (int dtype = 0; dtype < 8; ++dtype) {
        const bool cplx = (dtype == TTC_C64 || dtype == TTC_C128 || dtype == TTC_C64_C128 || dtype == TTC_C128_C64);
        const bool a32 = (dtype == TTC_F32 || dtype == TTC_C64 || dtype == TTC_F32_F64 || dtype == TTC_C64_C128);
        const bool b32 = (dtype == TTC_F32 || dtype == TTC_C64 || dtype == TTC_F64_F32 || dtype == TTC_C128_C64);
        const bool s32 = (dtype == TTC_F32 || dtype == TTC_C64);
        const int comps = cplx ? 2 : 1;
        uint64_t st = 1603 + (uint64_t)dtype;
        std::vector<float> Af((size_t)(n * comps)), Bf((size_t)(n * comps));
        std::vector<double> Ad((size_t)(n * comps)), Bd((size_t)(n * comps));
        for (int64_t i = 0; i < n * comps; ++i) { Ad[(size_t)i] = draw(&st); Af[(size_t)i] = (float)Ad[(size_t)i]; }
        for (int64_t i = 0; i < n * comps; ++i) { Bd[(size_t)i] = draw(&st); Bf[(size_t)i] = (float)Bd[(size_t)i]; }
        float alf[2] = {0.75f, cplx ? -0.5f : 0.f}, bef[2] = {1.25f, cplx ? 0.25f : 0.f};
        double ald[2] = {0.75, cplx ? -0.5 : 0.0}, bed[2] = {1.25, cplx ? 0.25 : 0.0};
        std::vector<unsigned char> ref;
        for (int threads : {1, 3, 4}) {
            std::vector<float> bf = Bf;
            std::vector<double> bd = Bd;
            const int rc = ttc_oracle_transpose_ld(dtype, 4, sizes, perm, nullptr, nullptr, s32 ? (const void*)alf : (const void*)ald,
                                                   s32 ? (const void*)bef : (const void*)bed, a32 ? (const void*)Af.data() : (const void*)Ad.data(),
                                                   b32 ? (void*)bf.data() : (void*)bd.data(), threads);
            EXPECT(rc == 0, "oracle dtype %d: %d", dtype, rc);
            const unsigned char* out = b32 ? (const unsigned char*)bf.data() : (const unsigned char*)bd.data();
            const size_t bytes = (size_t)(n * comps) * (b32 ? 4 : 8);
            if (threads == 1) ref.assign(out, out + bytes);
            else EXPECT(std::memcmp(ref.data(), out, bytes) == 0, "oracle dtype %d: %d threads differ from 1", dtype, threads);
        }
    }
    {   // identity permutation = the scalar statement on flat arrays
        const int64_t s1[2] = {11, 13};
        const int id[2] = {0, 1};
        uint64_t st = 7;
        std::vector<float> A(143), B(143), want(143);
        for (float& x : A) x = (float)draw(&st);
        for (float& x : B) x = (float)draw(&st);
        const float al = 1.5f, be = -0.25f;
        for (int i = 0; i < 143; ++i) want[(size_t)i] = std::fmaf(al, A[(size_t)i], be * B[(size_t)i]);
        EXPECT(ttc_oracle_transpose_ld(TTC_F32, 2, s1, id, nullptr, nullptr, &al, &be, A.data(), B.data(), 2) == 0, "identity");
        EXPECT(std::memcmp(B.data(), want.data(), 143 * sizeof(float)) == 0, "identity is not axpby");
    }
}

int main()
{
    check_refusals();
    check_oracle();
    check_planner();
    if (g_failures) { std::printf("%d failure(s)\n", g_failures); return 1; }
    std::printf("sanitizer driver ok\n");
    return 0;
}
