// Exercises the host side of the C ABI (validation, bundle classification, Strassen schedule, tail split, model,
// automatic choice, inspection calls, error paths) on host-only plans.  Built together with tc_host.cpp under
// AddressSanitizer and UndefinedBehaviorSanitizer by tests/test_host_sanitizers.py; any report makes it fail.
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <string>
#include <vector>

#include "strassen_tc.h"

static int failures = 0;
#define CHECK(cond)                                                        \
    do {                                                                   \
        if (!(cond)) {                                                     \
            std::fprintf(stderr, "%s:%d: %s\n", __FILE__, __LINE__, #cond); \
            ++failures;                                                    \
        }                                                                  \
    } while (0)

struct Desc {
    std::vector<int64_t> len, stride;
    std::string idx;
    tc_tensor_desc_t d() const { return tc_tensor_desc_t{(int)idx.size(), len.data(), stride.data(), idx.data()}; }
};

static Desc col_major(const char* idx, std::vector<int64_t> len) {
    Desc t;
    t.idx = idx;
    t.len = len;
    int64_t s = 1;
    for (int64_t n : len) {
        t.stride.push_back(s);
        s *= n > 0 ? n : 1;
    }
    return t;
}

static void walk(const Desc& A, const Desc& B, const Desc& C, int level, int variant, tc_options_t opts) {
    opts.host_only = 1;
    tc_plan_t* p = nullptr;
    tc_tensor_desc_t a = A.d(), b = B.d(), c = C.d();
    int rc = tc_plan_ex(&p, &a, &b, &c, level, variant, &opts, nullptr);
    CHECK(rc == TC_OK && p);
    if (rc != TC_OK) return;
    tc_plan_info_t info;
    CHECK(tc_plan_info(p, &info) == TC_OK);
    for (int i = -1; i <= info.n_products; ++i) {
        tc_product_t e;
        const int r = tc_plan_schedule(p, i, &e);
        CHECK((r == TC_OK) == (i >= 0 && i < info.n_products));
    }
    for (int i = -1; i <= info.n_launches; ++i) {
        tc_launch_info_t L;
        const int r = tc_plan_launch(p, i, &L);
        CHECK((r == TC_OK) == (i >= 0 && i < info.n_launches));
    }
    tc_model_time_t t;
    CHECK(tc_plan_predict(p, nullptr, &t) == TC_OK && t.total >= 0);
    tc_model_params_t mp;
    CHECK(tc_model_defaults(&mp) == TC_OK);
    mp.units = 100;
    CHECK(tc_plan_predict(p, &mp, &t) == TC_OK);
    (void)tc_plan_workspace_bytes(p);
    for (int which = -1; which <= 12; ++which) {
        const int64_t n = tc_plan_vector(p, which, nullptr, 0);
        CHECK((n >= 0) == (which >= 0 && which < 12));
        int64_t buf[4];
        if (n >= 0) CHECK(tc_plan_vector(p, which, buf, 4) == TC_ERR_STATE);  // host-only plans hold no device vectors
    }
    double x = 0;
    CHECK(tc_contract(p, 1.0, &x, &x, 1.0, &x, nullptr, nullptr) == TC_ERR_STATE);
    CHECK(tc_destroy(p) == TC_OK);
}

int main() {
    tc_options_t none;
    std::memset(&none, 0, sizeof none);
    const int levels[] = {0, 1, 2, TC_LEVEL_AUTO};
    const int variants[] = {TC_VARIANT_NAIVE, TC_VARIANT_AB, TC_VARIANT_ABC, TC_VARIANT_HYBRID, TC_VARIANT_AUTO};
    // plain matrices of many shapes, including ones shorter than 2^L, odd ones, and ones with a tail of tiles
    const int64_t shapes[][3] = {{1, 1, 1}, {3, 64, 5}, {20, 64, 64}, {300, 275, 190}, {1000, 3000, 520}, {4096, 4096, 4096},
                                 {10001, 10001, 10001}, {16384, 16384, 256}, {9216, 96, 4096}, {36864, 2304, 36864}};
    for (auto& s : shapes)
        for (int L : levels)
            for (int v : variants) {
                Desc A = col_major("ik", {s[0], s[2]}), B = col_major("kj", {s[2], s[1]}), C = col_major("ij", {s[0], s[1]});
                walk(A, B, C, L, v, none);
                tc_options_t o = none;
                o.tail_split = -1;
                walk(A, B, C, L, v, o);
                o.tail_split = 3;
                o.no_merge = 1;
                o.bs_block = 4;
                walk(A, B, C, L, v, o);
                if (L == 0) {
                    o = none;
                    o.split_k = -1;
                    walk(A, B, C, L, v, o);
                    o.split_k = 4;
                    walk(A, B, C, L, v, o);
                }
            }
    // tensor-shaped contractions: the benchmark index strings at reduced and at full lengths, empty bundles
    {
        Desc A = col_major("aebf", {16, 16, 16, 16}), B = col_major("dfce", {16, 16, 16, 16}), C = col_major("abcd", {16, 16, 16, 16});
        for (int L : levels) walk(A, B, C, L, TC_VARIANT_ABC, none);
        Desc A5 = col_major("agbch", {24, 96, 24, 24, 96}), B5 = col_major("hdgef", {96, 24, 96, 24, 24}), C5 = col_major("abcdef", {24, 24, 24, 24, 24, 24});
        for (int L : levels)
            for (int v : variants) walk(A5, B5, C5, L, v, none);
        Desc Av = col_major("k", {1000}), Bv = col_major("k", {1000}), Cs = col_major("", {});
        walk(Av, Bv, Cs, 2, TC_VARIANT_ABC, none);
        Desc Ao = col_major("i", {37}), Bo = col_major("j", {41}), Co = col_major("ij", {37, 41});
        walk(Ao, Bo, Co, 1, TC_VARIANT_AB, none);
        Desc Az = col_major("ik", {9, 0}), Bz = col_major("kj", {0, 8}), Cz = col_major("ij", {9, 8});
        walk(Az, Bz, Cz, 1, TC_VARIANT_NAIVE, none);
        Desc Ae = col_major("ik", {0, 5}), Be = col_major("kj", {5, 8}), Ce = col_major("ij", {0, 8});
        walk(Ae, Be, Ce, 2, TC_VARIANT_HYBRID, none);
    }
    // error paths
    {
        Desc A = col_major("ik", {4, 5}), B = col_major("kj", {5, 6}), C = col_major("ij", {4, 6});
        tc_tensor_desc_t a = A.d(), b = B.d(), c = C.d();
        tc_plan_t* p = reinterpret_cast<tc_plan_t*>(&a);
        tc_options_t o = none;
        o.host_only = 1;
        CHECK(tc_plan_ex(nullptr, &a, &b, &c, 0, TC_VARIANT_ABC, &o, nullptr) == TC_ERR_NULL);
        CHECK(tc_plan_ex(&p, nullptr, &b, &c, 0, TC_VARIANT_ABC, &o, nullptr) == TC_ERR_NULL && p == nullptr);
        CHECK(tc_plan_ex(&p, &a, &b, &c, 3, TC_VARIANT_ABC, &o, nullptr) == TC_ERR_LEVEL);
        CHECK(tc_plan_ex(&p, &a, &b, &c, 0, 9, &o, nullptr) == TC_ERR_VARIANT);
        CHECK(tc_plan_ex(&p, &a, &b, &c, 5, TC_VARIANT_AUTO, &o, nullptr) == TC_ERR_LEVEL);
        o.split_k = 9;
        CHECK(tc_plan_ex(&p, &a, &b, &c, 0, TC_VARIANT_ABC, &o, nullptr) == TC_ERR_STATE);
        o.split_k = 0;
        o.tail_split = 1;
        CHECK(tc_plan_ex(&p, &a, &b, &c, 0, TC_VARIANT_ABC, &o, nullptr) == TC_ERR_STATE);
        o.tail_split = 0;
        Desc Cbad = C;
        Cbad.stride[1] = 3;  // columns overlap
        tc_tensor_desc_t cb = Cbad.d();
        CHECK(tc_plan_ex(&p, &a, &b, &cb, 0, TC_VARIANT_ABC, &o, nullptr) == TC_ERR_STRIDE);
        Desc Cil = col_major("ij", {2, 3});
        Cil.stride = {3, 2};  // interleaved but free of overlap
        Desc Ai = col_major("ik", {2, 5}), Bi = col_major("kj", {5, 3});
        tc_tensor_desc_t ai = Ai.d(), bi = Bi.d(), ci = Cil.d();
        CHECK(tc_plan_ex(&p, &ai, &bi, &ci, 0, TC_VARIANT_ABC, &o, nullptr) == TC_OK);
        tc_destroy(p);
        Desc Bl = col_major("kl", {5, 6});
        tc_tensor_desc_t bl = Bl.d();
        CHECK(tc_plan_ex(&p, &a, &bl, &c, 0, TC_VARIANT_ABC, &o, nullptr) == TC_ERR_LABEL);
        Desc Bn = col_major("kj", {7, 6});
        tc_tensor_desc_t bn = Bn.d();
        CHECK(tc_plan_ex(&p, &a, &bn, &c, 0, TC_VARIANT_ABC, &o, nullptr) == TC_ERR_LENGTH);
        tc_tensor_desc_t many = a;
        many.ndim = TC_MAX_NDIM + 1;
        CHECK(tc_plan_ex(&p, &many, &b, &c, 0, TC_VARIANT_ABC, &o, nullptr) == TC_ERR_NDIM);
        CHECK(tc_plan_info(nullptr, nullptr) == TC_ERR_NULL);
        CHECK(tc_plan_workspace_bytes(nullptr) == 0);
        CHECK(tc_destroy(nullptr) == TC_OK);
        for (int s = 1; s >= -14; --s) CHECK(tc_strerror(s) != nullptr);
        // without host_only the stubbed device calls fail: the error must come back as a status, nothing may leak
        CHECK(tc_plan(&p, &a, &b, &c, 1, TC_VARIANT_ABC, nullptr) == TC_ERR_HIP && p == nullptr);
    }
    if (failures) {
        std::fprintf(stderr, "%d checks failed\n", failures);
        return 1;
    }
    std::puts("planner driver: all checks passed");
    return 0;
}
