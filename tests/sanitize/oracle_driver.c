/*
 * Sanitizer driver for the CPU oracle (test infrastructure).  Built by
 * tests/test_sanitizers.py together with oracle/dgs_oracle.c under
 * -fsanitize=address,undefined; every buffer handed to the oracle is a heap block of
 * exactly the documented size, so any access outside it, any misuse of the heap and any
 * undefined arithmetic inside the oracle stops the run.  On top of that the driver checks
 * what must hold for every input: message size, ascending order, per-tensor counts, the
 * sent/kept split of the state (Algorithm 3, Eq. 12), what a push and a pull leave
 * behind (Algorithm 2, Eq. 1, Eq. 6), and the round trip of the wire form.
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

uint64_t dgs_oracle_k(double density, uint64_t n);
int dgs_oracle_nnz(const uint64_t *, uint32_t, double, uint64_t *, uint64_t *);
int dgs_oracle_topk(const float *, uint64_t, uint64_t, uint32_t *);
int dgs_oracle_topk_bruteforce(const float *, uint32_t, uint32_t, uint32_t *);
int dgs_oracle_worker_step(const float *, float *, const uint64_t *, uint32_t, float, float, double,
                           uint32_t *, float *, uint64_t *);
int dgs_oracle_server_push(float *, float *, uint32_t, uint64_t, const uint32_t *, const float *, uint64_t);
int dgs_oracle_server_pull(float *, const uint64_t *, uint32_t, double, uint32_t *, float *, uint64_t *);
int dgs_oracle_server_push_model(float *, uint64_t, const uint32_t *, const float *, uint64_t);
int dgs_oracle_server_pull_sent(const float *, float *, const uint64_t *, uint32_t, double, uint32_t *,
                                float *, uint64_t *);
int dgs_oracle_server_pull_all(float *, uint64_t, uint32_t *, float *, uint64_t, uint64_t *);
int dgs_oracle_server_pull_all_sent(const float *, float *, uint64_t, uint32_t *, float *, uint64_t,
                                    uint64_t *);
int dgs_oracle_apply_sparse(float *, uint64_t, const uint32_t *, const float *, uint64_t, float);
int dgs_oracle_wire_bytes(const uint64_t *, uint32_t, double, uint64_t *);
int dgs_oracle_encode(const uint64_t *, uint32_t, double, const uint32_t *, const float *, uint8_t *);
int dgs_oracle_decode(const uint64_t *, uint32_t, double, const uint8_t *, uint32_t *, float *);

static uint64_t rng_state = 0x9E3779B97F4A7C15ull;
static uint32_t rnd(void)
{
    rng_state = rng_state * 6364136223846793005ull + 1442695040888963407ull;
    return (uint32_t)(rng_state >> 33);
}
/* values with ties, zeros of both signs, subnormals and large magnitudes mixed in */
static float rnd_value(int flavour)
{
    uint32_t r = rnd();
    switch (flavour) {
    case 0: return (float)((int)(r % 17) - 8);                       /* small integers: many ties */
    case 1: return ((r & 7) == 0) ? 0.0f : ((r & 7) == 1 ? -0.0f : (float)(r >> 8) * 1e-6f - 8.0f);
    case 2: return ldexpf((float)((int)(r % 2001) - 1000), -149 + (int)((r >> 12) % 30));   /* around subnormal */
    default: return ((float)(r >> 8) / 8388608.0f - 1.0f) * ldexpf(1.0f, (int)((r >> 3) % 40) - 20);
    }
}

static uint32_t key_of(float x)
{
    uint32_t b;
    memcpy(&b, &x, 4);
    return b & 0x7FFFFFFFu;
}

#define CHECK(c) do { if (!(c)) { fprintf(stderr, "%s:%d: check failed: %s\n", __FILE__, __LINE__, #c); exit(1); } } while (0)
static void *xmalloc(size_t n) { void *p = malloc(n ? n : 1); CHECK(p); return p; }

static void check_message(const uint64_t *off, uint32_t J, double rho, const uint32_t *idx, uint64_t nnz)
{
    uint64_t o = 0, e;
    uint32_t j;
    for (j = 0; j < J; ++j) {
        uint64_t kj = dgs_oracle_k(rho, off[j + 1] - off[j]);
        for (e = 0; e < kj; ++e, ++o) {
            CHECK(o < nnz);
            CHECK(idx[o] >= off[j] && idx[o] < off[j + 1]);
            if (e) CHECK(idx[o] > idx[o - 1]);
        }
    }
    CHECK(o == nnz);
}

static void run_layout(const uint64_t *off, uint32_t J, double rho, int flavour)
{
    const uint64_t n = off[J];
    const uint32_t W = 3;
    uint64_t K = 0, nnz = 0, e, i, wb = 0;
    uint64_t *kj = xmalloc(J * sizeof *kj);
    CHECK(dgs_oracle_nnz(off, J, rho, kj, &K) == 0);
    float *g = xmalloc(n * 4), *s = xmalloc(n * 4), *s0 = xmalloc(n * 4);
    uint32_t *idx = xmalloc(K * 4);
    float *val = xmalloc(K * 4);
    for (i = 0; i < n; ++i) { g[i] = rnd_value(flavour); s[i] = rnd_value((flavour + 1) & 3) * 0.5f; }
    memcpy(s0, s, n * 4);
    const float lr = 0.75f, m = 0.9f;
    CHECK(dgs_oracle_worker_step(g, s, off, J, lr, m, rho, idx, val, &nnz) == 0);
    CHECK(nnz == K);
    check_message(off, J, rho, idx, nnz);
    /* sent: val = a, state = m a; kept: state = a (Eq. 12 with the state stored as m u) */
    for (e = 0, i = 0; i < n; ++i) {
        float a = fmaf(lr, g[i], s0[i]);
        if (e < nnz && idx[e] == i) {
            CHECK(memcmp(&val[e], &a, 4) == 0);
            float ma = m * a;
            CHECK(memcmp(&s[i], &ma, 4) == 0);
            ++e;
        } else {
            CHECK(memcmp(&s[i], &a, 4) == 0);
        }
    }
    /* per tensor: no kept entry outranks a sent one */
    {
        uint32_t j;
        uint64_t o = 0;
        for (j = 0; j < J; ++j) {
            uint32_t tmin = 0xFFFFFFFFu, kmax = 0;
            uint64_t q = o;
            for (e = 0; e < kj[j]; ++e) { uint32_t kk = key_of(val[o + e]); if (kk < tmin) tmin = kk; }
            for (i = off[j]; i < off[j + 1]; ++i) {
                if (q < o + kj[j] && idx[q] == i) { ++q; continue; }
                uint32_t kk = key_of(fmaf(lr, g[i], s0[i]));
                if (kk > kmax) kmax = kk;
            }
            CHECK(kmax <= tmin);
            o += kj[j];
        }
    }
    /* brute force agrees on the first tensor when it is small */
    if (off[1] <= 2000) {
        uint32_t nn = (uint32_t)off[1], kk = (uint32_t)kj[0];
        float *a = xmalloc(nn * 4);
        uint32_t *b1 = xmalloc(kk * 4), *b2 = xmalloc(kk * 4);
        for (i = 0; i < nn; ++i) a[i] = fmaf(lr, g[i], s0[i]);
        CHECK(dgs_oracle_topk_bruteforce(a, nn, kk, b1) == 0);
        CHECK(dgs_oracle_topk(a, nn, kk, b2) == 0);
        CHECK(memcmp(b1, b2, kk * 4) == 0 && memcmp(b1, idx, kk * 4) == 0);
        free(a); free(b1); free(b2);
    }
    /* wire form round trip */
    CHECK(dgs_oracle_wire_bytes(off, J, rho, &wb) == 0);
    {
        uint8_t *wire = xmalloc(wb);
        uint32_t *di = xmalloc(K * 4);
        float *dv = xmalloc(K * 4);
        CHECK(dgs_oracle_encode(off, J, rho, idx, val, wire) == 0);
        CHECK(dgs_oracle_decode(off, J, rho, wire, di, dv) == 0);
        CHECK(memcmp(di, idx, K * 4) == 0 && memcmp(dv, val, K * 4) == 0);
        free(wire); free(di); free(dv);
    }
    /* server, difference rows: push then pull of worker 1, twice */
    {
        float *model = xmalloc(n * 4), *diff = xmalloc((size_t)W * n * 4), *theta = xmalloc(n * 4);
        uint32_t *pi = xmalloc(K * 4);
        float *pv = xmalloc(K * 4);
        memset(model, 0, n * 4);
        memset(diff, 0, (size_t)W * n * 4);
        memset(theta, 0, n * 4);
        CHECK(dgs_oracle_server_push(model, diff, W, n, idx, val, nnz) == 0);
        CHECK(dgs_oracle_server_push(NULL, diff, W, n, idx, val, 0) == 0);     /* empty message, no model */
        for (int rep = 0; rep < 2; ++rep) {
            uint64_t pn = 0;
            CHECK(dgs_oracle_server_pull(diff + n, off, J, rho, pi, pv, &pn) == 0);
            CHECK(pn == K);
            check_message(off, J, rho, pi, pn);
            for (e = 0; e < pn; ++e) { uint32_t z; memcpy(&z, &diff[n + pi[e]], 4); CHECK(z == 0); }
            CHECK(dgs_oracle_apply_sparse(theta, n, pi, pv, pn, 1.0f) == 0);
        }
        /* theta_1 + D_1 == model on exact data (Eq. 5); on all data: rows 0 and 2 still equal the model */
        CHECK(memcmp(diff, model, n * 4) == 0 && memcmp(diff + 2 * n, model, n * 4) == 0);
        if (flavour == 0) for (i = 0; i < n; ++i) CHECK(theta[i] + diff[n + i] == model[i]);
        /* no secondary compression: capacity refused, then granted */
        {
            uint64_t cnt = 0, cnt2 = 0;
            uint32_t *ai = xmalloc(n * 4);
            float *av = xmalloc(n * 4);
            int rc = dgs_oracle_server_pull_all(diff, n, ai, av, 0, &cnt);
            CHECK((rc != 0) == (cnt > 0));
            CHECK(dgs_oracle_server_pull_all(diff, n, ai, av, cnt, &cnt2) == 0 && cnt2 == cnt);
            for (i = 0; i < n; ++i) CHECK(diff[i] == 0.0f);
            free(ai); free(av);
        }
        /* printed form: model + sent_k */
        {
            float *sent = xmalloc(n * 4);
            uint64_t pn = 0, cnt = 0;
            memset(sent, 0, n * 4);
            CHECK(dgs_oracle_server_push_model(model, n, idx, val, nnz) == 0);
            CHECK(dgs_oracle_server_pull_sent(model, sent, off, J, rho, pi, pv, &pn) == 0);
            CHECK(pn == K);
            check_message(off, J, rho, pi, pn);
            uint32_t *ai = xmalloc(n * 4);
            float *av = xmalloc(n * 4);
            CHECK(dgs_oracle_server_pull_all_sent(model, sent, n, ai, av, n, &cnt) == 0);
            CHECK(cnt <= n);
            free(ai); free(av); free(sent);
        }
        free(model); free(diff); free(theta); free(pi); free(pv);
    }
    free(kj); free(g); free(s); free(s0); free(idx); free(val);
}

int main(void)
{
    /* ragged, tiny and border cases; the shapes of the benchmark layouts at reduced size */
    static const uint64_t sizes[][8] = {
        {1, 0}, {1, 1, 1, 0}, {7, 64, 1, 1000, 0}, {1024, 1023, 1025, 0}, {4096, 3, 9408, 64, 64, 0},
        {1000, 2048, 512, 512, 36864, 0}, {65537, 5, 0}, {30522, 768, 2304, 0}, {15625, 15625, 15625, 15625, 0},
    };
    static const double rhos[] = {1e-4, 1e-3, 0.004, 0.01, 0.25, 0.5, 1.0};
    for (size_t L = 0; L < sizeof sizes / sizeof sizes[0]; ++L) {
        uint64_t off[9] = {0};
        uint32_t J = 0;
        while (J < 8 && sizes[L][J]) { off[J + 1] = off[J] + sizes[L][J]; ++J; }
        for (size_t r = 0; r < sizeof rhos / sizeof rhos[0]; ++r)
            for (int flavour = 0; flavour < 4; ++flavour) run_layout(off, J, rhos[r], flavour);
    }
    /* argument errors are reported, not acted on */
    {
        uint64_t off[2] = {0, 10}, K = 0;
        float a[10] = {0};
        uint32_t out[10];
        CHECK(dgs_oracle_nnz(off, 1, 0.0, NULL, &K) != 0);
        CHECK(dgs_oracle_nnz(off, 1, 1.5, NULL, &K) != 0);
        CHECK(dgs_oracle_topk(a, 10, 11, out) != 0);
        CHECK(dgs_oracle_topk_bruteforce(a, 10, 11, out) != 0);
        uint32_t bad = 10;
        float one = 1.0f;
        CHECK(dgs_oracle_apply_sparse(a, 10, &bad, &one, 1, 1.0f) != 0);
        CHECK(dgs_oracle_server_push_model(a, 10, &bad, &one, 1) != 0);
    }
    puts("oracle sanitizer driver: ok");
    return 0;
}
