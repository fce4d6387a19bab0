// CPU parity run of libdgs' kernels (test infrastructure).  The library's .hip sources are
// compiled as plain C++ against the host emulation in hip/hip_runtime.h and driven through
// the C ABI exactly like on the GPU, with "device" buffers that are heap blocks of exactly the
// documented size; every result is compared bit for bit with the CPU oracle.  Built with
// AddressSanitizer + UndefinedBehaviorSanitizer by tests/test_sanitizers.py: any access
// outside a buffer, in the kernels or in the host code, stops the run.  Parts are shrunk
// (-DDGS_SEG_TILES=16) so that small layouts exercise the multi-part paths: joins by several
// workgroups, the gather by the last one, re-collection after a failed prediction, the chain
// kernels, zero fills, dense requests.
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <string>
#include <vector>

#include "../../include/dgs.h"

extern "C" {
int dgs_oracle_nnz(const uint64_t *, uint32_t, double, uint64_t *, uint64_t *);
int dgs_oracle_worker_step(const float *, float *, const uint64_t *, uint32_t, float, float, double, uint32_t *,
                           float *, uint64_t *);
int dgs_oracle_server_push(float *, float *, uint32_t, uint64_t, const uint32_t *, const float *, uint64_t);
int dgs_oracle_server_pull(float *, const uint64_t *, uint32_t, double, uint32_t *, float *, uint64_t *);
int dgs_oracle_server_push_model(float *, uint64_t, const uint32_t *, const float *, uint64_t);
int dgs_oracle_server_pull_sent(const float *, float *, const uint64_t *, uint32_t, double, uint32_t *, float *,
                                uint64_t *);
int dgs_oracle_server_pull_all(float *, uint64_t, uint32_t *, float *, uint64_t, uint64_t *);
int dgs_oracle_apply_sparse(float *, uint64_t, const uint32_t *, const float *, uint64_t, float);
int dgs_oracle_wire_bytes(const uint64_t *, uint32_t, double, uint64_t *);
int dgs_oracle_encode(const uint64_t *, uint32_t, double, const uint32_t *, const float *, uint8_t *);
int dgs_oracle_wire_bytes16(const uint64_t *, uint32_t, double, uint64_t *);
int dgs_oracle_encode16(const uint64_t *, uint32_t, double, const uint32_t *, const float *, uint8_t *);
int dgs_oracle_decode16(const uint64_t *, uint32_t, double, const uint8_t *, uint32_t *, float *);
}

#define CHECK(c)                                                                             \
    do {                                                                                     \
        if (!(c)) {                                                                          \
            fprintf(stderr, "%s:%d: [%s] check failed: %s\n", __FILE__, __LINE__, g_what.c_str(), #c); \
            exit(1);                                                                         \
        }                                                                                    \
    } while (0)

static std::string g_what;

struct Rng {
    uint64_t s;
    explicit Rng(uint64_t seed) : s(seed * 0x9E3779B97F4A7C15ull + 12345) {}
    uint32_t u32() { s = s * 6364136223846793005ull + 1442695040888963407ull; return (uint32_t)(s >> 32); }
    double uni() { return (u32() + 0.5) / 4294967296.0; }
    float gauss() { return (float)(std::sqrt(-2.0 * std::log(uni())) * std::cos(6.283185307179586 * uni())); }
};

// exact-size heap block aligned to 256 bytes (the alignment the workspace needs); ASan guards both ends
template <class T> struct Buf {
    T *p = nullptr;
    size_t n = 0;
    explicit Buf(size_t count = 0) { reset(count); }
    void reset(size_t count)
    {
        free(p);
        n = count;
        p = nullptr;
        if (posix_memalign((void **)&p, 256, (count ? count : 1) * sizeof(T)) != 0) abort();
        memset(p, 0, (count ? count : 1) * sizeof(T));
    }
    ~Buf() { free(p); }
    Buf(const Buf &) = delete;
    Buf &operator=(const Buf &) = delete;
};

struct Layout {
    std::vector<uint64_t> off;
    uint32_t J;
    uint64_t n;
    explicit Layout(const std::vector<uint64_t> &sizes)
    {
        off.push_back(0);
        for (auto s : sizes) off.push_back(off.back() + s);
        J = (uint32_t)sizes.size();
        n = off.back();
    }
    uint64_t K(double rho) const
    {
        uint64_t k = 0;
        CHECK(dgs_oracle_nnz(off.data(), J, rho, nullptr, &k) == 0);
        return k;
    }
};

struct Ctx {
    dgs_ctx *c = nullptr;
    Buf<unsigned char> ws;
    Ctx(const Layout &L, uint32_t W)
    {
        const size_t bytes = dgs_workspace_bytes(L.off.data(), L.J, W);
        CHECK(bytes != 0);
        ws.reset(bytes);
        memset(ws.p, 0xA5, bytes);      // the library must not rely on a cleared workspace
        CHECK(dgs_create(&c, L.off.data(), L.J, W, ws.p, bytes, nullptr) == DGS_OK);
    }
    ~Ctx() { dgs_destroy(c); }
    dgs_stats stats()
    {
        dgs_stats s;
        CHECK(dgs_get_stats(c, &s) == DGS_OK);
        return s;
    }
};

static void fill_grad(const Layout &L, Rng &r, float *g, float scale, int flavour)
{
    for (uint32_t j = 0; j < L.J; ++j) {
        const float sj = scale * std::pow(10.0f, -1.0f - 3.0f * (float)((j * 7) % 5) / 5.0f);
        for (uint64_t i = L.off[j]; i < L.off[j + 1]; ++i) {
            float v = r.gauss() * sj;
            if (flavour == 1) v = std::round(v / sj * 2.0f) * sj;               // few levels: massive ties
            if (flavour == 2 && (r.u32() & 15u) != 0) v = 0.0f;                  // mostly exact zeros
            if (flavour == 3) v = 1.5f;                                          // one value everywhere
            if (flavour == 4) v = 0.0f;                                          // nothing at all
            if (flavour == 5 && (r.u32() % 2000u) != 0) v = 0.0f;                // fewer nonzeros than k
            if (flavour == 6) v = (float)((int)(r.u32() % 2001u) - 1000) * 1e-45f;   // subnormals
            if (flavour == 7) {                                                  // infinities and NaNs
                const uint32_t q = r.u32() % 1001u;
                if (q < 140) v = INFINITY;
                else if (q == 999) v = NAN;
            }
            g[i] = v;
        }
    }
}

static void expect_same(const uint32_t *gi, const float *gv, const uint32_t *wi, const float *wv, uint64_t K)
{
    for (uint64_t e = 0; e < K; ++e) {
        if (gi[e] != wi[e] || memcmp(&gv[e], &wv[e], 4) != 0) {
            fprintf(stderr, "[%s] entry %llu of %llu: got (%u, %g) want (%u, %g)\n", g_what.c_str(),
                    (unsigned long long)e, (unsigned long long)K, gi[e], gv[e], wi[e], wv[e]);
            exit(1);
        }
    }
}

static void expect_same_f(const float *a, const float *b, uint64_t n, const char *which)
{
    if (memcmp(a, b, n * 4) != 0) {
        for (uint64_t i = 0; i < n; ++i)
            if (memcmp(&a[i], &b[i], 4) != 0) {
                fprintf(stderr, "[%s] %s differs at %llu: got %g want %g\n", g_what.c_str(), which,
                        (unsigned long long)i, a[i], b[i]);
                exit(1);
            }
    }
}

struct Opts {
    int force_exact = 0, seg_mode = 0, repair = 1, margin = -1;
    int misalign = 0;      // floats by which grad and state are shifted off their 16-byte alignment
};

static void set_opts(Ctx &c, const Opts &o)
{
    CHECK(dgs_set_option(c.c, DGS_OPT_FORCE_EXACT, o.force_exact) == DGS_OK);
    CHECK(dgs_set_option(c.c, DGS_OPT_SEGMENTED, o.seg_mode) == DGS_OK);
    CHECK(dgs_set_option(c.c, DGS_OPT_REPAIR_ROUND, o.repair) == DGS_OK);
    if (o.margin >= 0) CHECK(dgs_set_option(c.c, DGS_OPT_MARGIN_PCT, o.margin) == DGS_OK);
}

// worker steps + push + pull on one context, every message against the oracle
static dgs_stats worker_server(const char *name, const std::vector<uint64_t> &sizes, double rho_up, double rho_down,
                               float lr, float m, bool residual, const std::vector<float> &scales, int flavour,
                               const Opts &o, uint64_t seed)
{
    g_what = name;
    Layout L(sizes);
    Rng r(seed);
    Ctx c(L, 1);
    set_opts(c, o);
    const uint64_t Ku = L.K(rho_up), Kd = L.K(rho_down);
    const int mis = o.misalign;
    Buf<float> g_store(L.n + mis), s_store(L.n + mis), s_ref(L.n), model_gpu(L.n), model_ref(L.n), d_gpu(L.n), d_ref(L.n);
    struct View { float *p; } g{g_store.p + mis}, s_gpu{s_store.p + mis};
    Buf<uint32_t> gi(Ku), wi(Ku), pi(Kd), qi(Kd);
    Buf<float> gv(Ku), wv(Ku), pv(Kd), qv(Kd);
    CHECK(dgs_server_attach(c.c, d_gpu.p) == DGS_OK);
    for (size_t t = 0; t < scales.size(); ++t) {
        g_what = std::string(name) + " step " + std::to_string(t);
        fill_grad(L, r, g.p, scales[t], flavour);
        uint64_t k1 = 0, k2 = 0;
        CHECK(dgs_oracle_worker_step(g.p, s_ref.p, L.off.data(), L.J, lr, m, rho_up, wi.p, wv.p, &k1) == 0);
        CHECK(dgs_worker_step(c.c, g.p, residual ? nullptr : s_gpu.p, residual ? s_gpu.p : nullptr, lr, m, rho_up,
                              gi.p, gv.p, &k2) == DGS_OK);
        CHECK(k1 == Ku && k2 == Ku);
        expect_same(gi.p, gv.p, wi.p, wv.p, Ku);
        expect_same_f(s_gpu.p, s_ref.p, L.n, "worker state");
        CHECK(dgs_oracle_server_push(model_ref.p, d_ref.p, 1, L.n, wi.p, wv.p, Ku) == 0);
        CHECK(dgs_server_push(c.c, model_gpu.p, 0, gi.p, gv.p, Ku) == DGS_OK);
        CHECK(dgs_oracle_server_pull(d_ref.p, L.off.data(), L.J, rho_down, qi.p, qv.p, &k1) == 0);
        CHECK(dgs_server_pull(c.c, 0, rho_down, pi.p, pv.p, &k2) == DGS_OK);
        CHECK(k1 == Kd && k2 == Kd);
        expect_same(pi.p, pv.p, qi.p, qv.p, Kd);
        expect_same_f(d_gpu.p, d_ref.p, L.n, "difference row");
        expect_same_f(model_gpu.p, model_ref.p, L.n, "model");
    }
    const dgs_stats st = c.stats();
    CHECK(st.internal_errors == 0);
    printf("%-44s ok: exact %llu, chain %llu, repaired %llu, fallback %llu\n", name, (unsigned long long)st.exact_calls,
           (unsigned long long)st.segmented_tensors, (unsigned long long)st.repaired_tensors,
           (unsigned long long)st.fallback_tensors);
    fflush(stdout);
    return st;
}

// the printed server form (model + sent_k) with two workers, pulls at another density
static void printed_form(const char *name, const std::vector<uint64_t> &sizes, double rho_up, double rho_down,
                         int events, const Opts &o, uint64_t seed)
{
    g_what = name;
    Layout L(sizes);
    Rng r(seed);
    const uint32_t W = 2;
    Ctx c(L, W);
    set_opts(c, o);
    const uint64_t Ku = L.K(rho_up), Kd = L.K(rho_down);
    Buf<float> g(L.n), s_ref(L.n), model_gpu(L.n), model_ref(L.n), sent_gpu(W * L.n), sent_ref(W * L.n);
    Buf<uint32_t> wi(Ku), pi(Kd), qi(Kd);
    Buf<float> wv(Ku), pv(Kd), qv(Kd);
    CHECK(dgs_server_attach_sent(c.c, sent_gpu.p) == DGS_OK);
    for (int e = 0; e < events; ++e) {
        g_what = std::string(name) + " event " + std::to_string(e);
        fill_grad(L, r, g.p, e == 3 ? 1e-3f : 1.0f, 0);
        uint64_t k1 = 0, k2 = 0;
        CHECK(dgs_oracle_worker_step(g.p, s_ref.p, L.off.data(), L.J, 1.0f, 0.9f, rho_up, wi.p, wv.p, &k1) == 0);
        const uint32_t w = (uint32_t)(e % 3 == 2 ? 0 : e % 2);
        CHECK(dgs_oracle_server_push_model(model_ref.p, L.n, wi.p, wv.p, Ku) == 0);
        CHECK(dgs_server_push_model(c.c, model_gpu.p, wi.p, wv.p, Ku) == DGS_OK);
        CHECK(dgs_oracle_server_pull_sent(model_ref.p, sent_ref.p + w * L.n, L.off.data(), L.J, rho_down, qi.p, qv.p,
                                          &k1) == 0);
        CHECK(dgs_server_pull_sent(c.c, model_gpu.p, w, rho_down, pi.p, pv.p, &k2) == DGS_OK);
        CHECK(k1 == Kd && k2 == Kd);
        expect_same(pi.p, pv.p, qi.p, qv.p, Kd);
        expect_same_f(sent_gpu.p, sent_ref.p, W * L.n, "sent rows");
    }
    CHECK(c.stats().internal_errors == 0);
    printf("%-44s ok\n", name);
    fflush(stdout);
}

static void helpers_and_static(uint64_t seed)
{
    g_what = "helpers";
    const std::vector<uint64_t> sizes = {70001, 5, 20000, 2048};
    Layout L(sizes);
    Rng r(seed);
    const double rho = 0.01;
    const uint64_t K = L.K(rho);
    Buf<float> g(L.n), s_ref(L.n), s_gpu(L.n), theta(L.n), theta_ref(L.n), row(L.n), row_ref(L.n);
    Buf<uint32_t> wi(K), gi(K), di(K), ai(L.n), bi(L.n);
    Buf<float> wv(K), gv(K), dv(K), av(L.n), bv(L.n);
    fill_grad(L, r, g.p, 1.0f, 0);
    for (uint64_t i = 0; i < L.n; ++i) s_ref.p[i] = s_gpu.p[i] = 0.3f * r.gauss();
    uint64_t k1 = 0, k2 = 0;
    CHECK(dgs_oracle_worker_step(g.p, s_ref.p, L.off.data(), L.J, 0.5f, 0.9f, rho, wi.p, wv.p, &k1) == 0);
    // the entry point that allocates nothing (twice: the second call must not see the first)
    for (int rep = 0; rep < 2; ++rep) {
        Buf<float> s2(L.n);
        for (uint64_t i = 0; i < L.n; ++i) s2.p[i] = s_gpu.p[i];
        CHECK(dgs_worker_step_static(L.off.data(), L.J, g.p, s2.p, nullptr, 0.5f, 0.9f, rho, gi.p, gv.p, &k2, nullptr) == DGS_OK);
        CHECK(k2 == K);
        expect_same(gi.p, gv.p, wi.p, wv.p, K);
        expect_same_f(s2.p, s_ref.p, L.n, "state after the static call");
    }
    Ctx c(L, 1);
    // wire form
    uint64_t wb = 0, wb2 = 0;
    CHECK(dgs_wire_bytes(c.c, rho, &wb) == DGS_OK);
    CHECK(dgs_oracle_wire_bytes(L.off.data(), L.J, rho, &wb2) == 0 && wb == wb2);
    Buf<uint8_t> wire(wb), wire_ref(wb);
    CHECK(dgs_oracle_encode(L.off.data(), L.J, rho, wi.p, wv.p, wire_ref.p) == 0);
    CHECK(dgs_encode(c.c, rho, wi.p, wv.p, wire.p) == DGS_OK);
    CHECK(memcmp(wire.p, wire_ref.p, wb) == 0);
    CHECK(dgs_decode(c.c, rho, wire.p, di.p, dv.p) == DGS_OK);
    expect_same(di.p, dv.p, wi.p, wv.p, K);
    {   // the same with bfloat16 values (exact-size buffers: the value area is half as long)
        uint64_t hb = 0, hb2 = 0;
        CHECK(dgs_set_option(c.c, DGS_OPT_WIRE_VALUE_BITS, 16) == DGS_OK);
        CHECK(dgs_wire_bytes(c.c, rho, &hb) == DGS_OK);
        CHECK(dgs_oracle_wire_bytes16(L.off.data(), L.J, rho, &hb2) == 0 && hb == hb2 && hb < wb);
        Buf<uint8_t> h(hb), h_ref(hb);
        Buf<uint32_t> qi(K), ri(K);
        Buf<float> qv(K), rv(K);
        CHECK(dgs_oracle_encode16(L.off.data(), L.J, rho, wi.p, wv.p, h_ref.p) == 0);
        CHECK(dgs_encode(c.c, rho, wi.p, wv.p, h.p) == DGS_OK);
        CHECK(memcmp(h.p, h_ref.p, hb) == 0);
        CHECK(dgs_oracle_decode16(L.off.data(), L.J, rho, h_ref.p, ri.p, rv.p) == 0);
        CHECK(dgs_decode(c.c, rho, h.p, qi.p, qv.p) == DGS_OK);
        expect_same(qi.p, qv.p, ri.p, rv.p, K);
        CHECK(dgs_set_option(c.c, DGS_OPT_WIRE_VALUE_BITS, 32) == DGS_OK);
    }
    // apply with a sign, an out-of-range index is skipped
    for (uint64_t i = 0; i < L.n; ++i) theta.p[i] = theta_ref.p[i] = r.gauss();
    CHECK(dgs_oracle_apply_sparse(theta_ref.p, L.n, wi.p, wv.p, K - 1, -1.0f) == 0);
    di.p[K - 1] = (uint32_t)L.n + 3;
    CHECK(dgs_apply_sparse(c.c, theta.p, di.p, dv.p, K, -1.0f) == DGS_OK);
    expect_same_f(theta.p, theta_ref.p, L.n, "theta");
    // pull without secondary compression
    CHECK(dgs_server_attach(c.c, row.p) == DGS_OK);
    CHECK(dgs_server_push(c.c, nullptr, 0, wi.p, wv.p, K) == DGS_OK);
    CHECK(dgs_oracle_server_push(nullptr, row_ref.p, 1, L.n, wi.p, wv.p, K) == 0);
    CHECK(dgs_server_pull_all(c.c, 0, ai.p, av.p, 3, &k2) == DGS_ECAPACITY && k2 == K);
    CHECK(dgs_server_pull_all(c.c, 0, ai.p, av.p, L.n, &k2) == DGS_OK);
    CHECK(dgs_oracle_server_pull_all(row_ref.p, L.n, bi.p, bv.p, L.n, &k1) == 0 && k1 == k2);
    expect_same(ai.p, av.p, bi.p, bv.p, k1);
    expect_same_f(row.p, row_ref.p, L.n, "row after pull_all");
    CHECK(c.stats().internal_errors == 0);
    printf("%-44s ok\n", "static entry point, wire form, apply, pull_all");
    fflush(stdout);
}

// Randomised layouts, densities, options, server forms and gradient-scale jumps (which make
// predictions fail): `soak <first seed> <count>`.
static void soak(uint64_t seed)
{
    Rng r(seed * 7919 + 13);
    std::vector<uint64_t> sizes;
    const uint32_t J = 1 + r.u32() % 6;
    uint64_t total = 0;
    for (uint32_t j = 0; j < J; ++j) {
        static const uint64_t pool[] = {1, 3, 64, 1000, 8192, 8193, 9408, 12345, 20000, 40001, 65536, 65537, 70001, 100003, 150000};
        uint64_t n = pool[r.u32() % (sizeof pool / sizeof pool[0])];
        if (total + n > 330000) n = 1 + r.u32() % 3000;
        sizes.push_back(n);
        total += n;
    }
    static const double rhos[] = {0.0005, 0.001, 0.002, 0.004, 0.01, 0.03, 0.05, 0.3, 1.0};
    const double rho_up = rhos[r.u32() % 9], rho_down = rhos[r.u32() % 9];
    Opts o;
    {
        const uint32_t pick = r.u32() % 6;       // mostly predicted; two-pass and sampled now and then
        o.force_exact = pick == 0 ? 1 : (pick == 1 ? 2 : 0);
    }
    o.seg_mode = (int)(r.u32() % 3);
    o.repair = (r.u32() % 4) != 0;
    o.margin = (r.u32() % 3) == 0 ? (int)(r.u32() % 120) : -1;
    o.misalign = (r.u32() % 6) == 0 ? 1 + (int)(r.u32() % 3) : 0;
    const bool residual = (r.u32() % 3) == 0;
    const float m = residual ? 0.0f : (r.u32() % 2 ? 0.9f : 0.5f);
    std::vector<float> scales;
    const uint32_t steps = 3 + r.u32() % 4;
    for (uint32_t t = 0; t < steps; ++t) {
        static const float jumps[] = {1, 1, 1, 1, 1e3f, 1e-3f, 1e-6f, 30.0f};
        scales.push_back(jumps[r.u32() % 8]);
    }
    const int flavour = (r.u32() % 4) == 0 ? (int)(r.u32() % 3) : 0;
    char name[160];
    snprintf(name, sizeof name, "soak %llu: J=%u n=%llu up=%g down=%g ex=%d seg=%d rep=%d res=%d fl=%d", (unsigned long long)seed,
             J, (unsigned long long)total, rho_up, rho_down, o.force_exact, o.seg_mode, o.repair, (int)residual, flavour);
    if ((r.u32() % 4) == 0 && !residual)
        printed_form(name, sizes, rho_up, rho_down, (int)steps, o, seed);
    else
        worker_server(name, sizes, rho_up, rho_down, r.u32() % 2 ? 1.0f : 0.3f, m, residual, scales, flavour, o, seed);
}

int main(int argc, char **argv)
{
    if (argc > 3 && std::string(argv[1]) == "soak") {
        const uint64_t first = strtoull(argv[2], nullptr, 10), count = strtoull(argv[3], nullptr, 10);
        for (uint64_t sd = first; sd < first + count; ++sd) soak(sd);
        return 0;
    }
    const bool quick = argc > 1 && std::string(argv[1]) == "quick";
    if (argc > 1 && std::string(argv[1]) == "flat") {
        // one flat tensor of 2^20 elements at density 0.01, as the smallest benchmark configuration
        Opts o;
        worker_server("flat 2^20", {1u << 20}, 0.01, 0.01, 1.0f, 0.9f, false, {1, 1, 1}, 0, o, 20);
        return 0;
    }
    if (argc > 1 && std::string(argv[1]) == "rounds") {
        // join groups of more tiles than a workgroup has lanes (build with the default DGS_GROUP_TILES):
        // several rounds per group, the second tensor starting inside a tile of the first
        Opts o;
        worker_server("groups of several rounds", {1500017, 64, 2300000}, 0.001, 0.002, 1.0f, 0.9f, false, {1, 1, 1, 30, 30},
                      0, o, 29);
        // one workgroup's join that ends with more candidates than it can select from, all of
        // them collected (LDS list plus global tail): trimmed in place
        Opts nr;
        nr.repair = 0;
        const dgs_stats st = worker_server("scale triples, one group's list trimmed", {1200000, 64}, 0.001, 0.001, 1.0f, 0.0f,
                                           true, {1, 1, 1, 3, 3}, 0, nr, 34);
        CHECK(st.repaired_tensors >= 1 && st.fallback_tensors == 0);
        // the same where what remains (about 2 k entries) is itself longer than the LDS list and
        // ends in the global scratch it is read from
        const dgs_stats st2 = worker_server("one group's list trimmed into LDS and scratch", {4000000, 64}, 0.0025, 0.0025,
                                            1.0f, 0.0f, true, {1, 1, 2}, 0, nr, 35);
        CHECK(st2.repaired_tensors >= 1 && st2.fallback_tensors == 0);
        return 0;
    }
    const std::vector<uint64_t> ragged = {1, 7, 64, 1000, 8192, 8193, 9408, 3, 100003, 20000, 70001, 17, 65537, 12345};
    const std::vector<uint64_t> two = {150000, 64, 66000};
    Opts def, exact, always, never, norepair;
    exact.force_exact = 1;
    always.seg_mode = 1;
    never.seg_mode = 2;
    norepair.repair = 0;
    const std::vector<float> steady = {1, 1, 1, 1};
    const std::vector<float> jumps = {1, 1, 1e3f, 1e3f, 1e-6f, 1e-6f, 1, 1};

    worker_server("ragged, predicted", ragged, 0.004, 0.004, 0.5f, 0.9f, false, steady, 0, def, 1);
    worker_server("scale jumps, residual mode (re-collection)", two, 0.002, 0.004, 1.0f, 0.0f, true, jumps, 0, def, 2);
    worker_server("scale jumps, chain for every large tensor", two, 0.002, 0.002, 1.0f, 0.0f, true, jumps, 0, always, 3);
    {
        // a scale that grows three- and fourfold: every candidate is collected, but the lists of
        // the large tensors outgrow one workgroup and are trimmed against their own histogram
        // inside the launch -- with the re-collecting roles switched off, where such a tensor
        // would otherwise fall back to the single-workgroup selection
        const std::vector<float> grows = {1, 1, 1, 3, 1, 1, 4, 4};
        const dgs_stats st = worker_server("scale grows, lists trimmed (no re-collecting roles)", {300000, 64, 150000}, 0.002,
                                           0.002, 1.0f, 0.9f, false, grows, 0, norepair, 33);
        CHECK(st.repaired_tensors >= 1 && st.fallback_tensors == 0);
        if (!quick) worker_server("scale grows, lists trimmed", {300000, 64, 150000}, 0.002, 0.002, 1.0f, 0.0f, true, grows, 0, def, 32);
    }
    if (!quick) {
        worker_server("ragged, exact path", ragged, 0.01, 0.002, 0.5f, 0.9f, false, {1, 1}, 0, exact, 4);
        Opts sampled;
        sampled.force_exact = 2;
        worker_server("ragged, sampled estimate on every call", ragged, 0.004, 0.002, 0.5f, 0.9f, false, {1, 1, 1e3f, 1e-6f, 1}, 0,
                      sampled, 30);
        worker_server("mostly zeros, sampled estimate", two, 0.001, 0.02, 1.0f, 0.9f, false, steady, 2, sampled, 31);
        worker_server("scale jumps, no re-collecting roles", two, 0.002, 0.004, 1.0f, 0.0f, true, jumps, 0, norepair, 5);
        worker_server("massive ties", two, 0.003, 0.003, 1.0f, 0.9f, false, steady, 1, def, 6);
        worker_server("massive ties, chain", two, 0.003, 0.003, 1.0f, 0.9f, false, steady, 1, always, 7);
        worker_server("mostly zeros (zero fill on the pull)", two, 0.001, 0.02, 1.0f, 0.9f, false, steady, 2, def, 8);
        worker_server("mostly zeros, chain", two, 0.001, 0.02, 1.0f, 0.9f, false, steady, 2, always, 9);
        worker_server("long lists (beyond the LDS list)", {300000, 9000}, 0.03, 0.03, 1.0f, 0.9f, false, {1, 1, 1}, 0, never, 10);
        worker_server("one value everywhere", {70000, 100, 9000}, 0.002, 0.002, 1.0f, 0.5f, false, {1, 1, 1}, 3, def, 21);
        worker_server("one value everywhere, exact path", {70000, 100, 9000}, 0.002, 0.002, 1.0f, 0.5f, false, {1, 1}, 3, exact, 22);
        worker_server("all zero", {70000, 100, 9000}, 0.002, 0.002, 1.0f, 0.5f, false, {1, 1, 1}, 4, def, 23);
        worker_server("fewer nonzeros than k", {70000, 100, 9000}, 0.002, 0.002, 1.0f, 0.5f, false, {1, 1, 1}, 5, def, 24);
        worker_server("subnormals", {70000, 100, 9000}, 0.002, 0.002, 1.0f, 0.5f, false, {1, 1, 1}, 6, def, 25);
        worker_server("infinities and NaNs", {70000, 100, 9000}, 0.002, 0.002, 1.0f, 0.5f, false, {1}, 7, def, 26);
        Opts mis1;
        mis1.misalign = 1;
        worker_server("buffers off their 16-byte alignment", {20000, 5, 40001}, 0.01, 0.01, 1.0f, 0.9f, false, {1, 1, 1}, 0, mis1, 27);
        worker_server("threshold collapse, momentum 0", {200000, 64}, 0.001, 0.001, 1.0f, 0.0f, true, {1, 1, 1e-6f, 1e-6f, 1, 1}, 0, def, 28);
        worker_server("dense request 0.05", ragged, 0.05, 0.05, 0.5f, 0.9f, false, {1, 1}, 0, def, 11);
        worker_server("dense request 1.0", two, 1.0, 1.0, 0.5f, 0.9f, false, {1, 1}, 0, def, 12);
        worker_server("dense request, ties", two, 0.5, 0.05, 1.0f, 0.9f, false, {1, 1}, 1, def, 13);
        printed_form("printed server form", two, 0.002, 0.004, 6, def, 14);
        printed_form("printed server form, chain", two, 0.002, 0.004, 5, always, 15);
    }
    helpers_and_static(16);
    puts("emulated kernels: all scenarios match the oracle");
    return 0;
}
