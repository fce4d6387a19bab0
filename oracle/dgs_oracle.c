/*
 * dgs_oracle.c -- plain, slow, single-threaded CPU statement of what the DGS
 * hot path computes.
 *
 * THIS IS TEST INFRASTRUCTURE.  Only tests, the smoke check and the benchmark's
 * CPU-baseline leg may call it.  It shares no code with the HIP library and the
 * product path never falls back to it.
 *
 * What it follows (arXiv 1910.10929, "Gradient Sparsification for Asynchronous
 * Distributed Training"):
 *   - worker update with sparsification-aware momentum: Algorithm 3, Eq. 11, Eq. 12;
 *     with momentum 0 it is the residual scheme of Algorithm 1;
 *   - server: Algorithm 2 with secondary compression, Eq. 1, Eq. 3, Eq. 6;
 *   - encode() / decode(): the paper asks for coordinate format only; the byte layout of
 *     dgs_oracle_encode is this library's own (PARITY UNPINNED with respect to the paper,
 *     pinned to its own statement), see there.
 *
 * Readings fixed where the paper is silent (all listed in the design notes):
 *   - "thr <- R% of |x|" is the k-th largest magnitude of tensor j with
 *     k = ceil(density * n_j) in IEEE double, density = 1 - R/100;
 *   - exactly k entries per tensor are selected; among equal magnitudes the
 *     lower index wins; magnitude is compared as the 31-bit integer
 *     bits(x) & 0x7FFFFFFF (so NaN > Inf > finite, -0 == +0);
 *   - the accumulate step is one fused multiply-add in fp32:
 *     a = fmaf(lr, grad, state); denormals are kept;
 *   - the worker state is stored as s = m * u (u = the paper's velocity):
 *     sent entries keep u = a  <=> s = m * a (one fp32 multiply),
 *     unsent entries get u = a / m  <=> s = a.  With m = 0 this is Algorithm 1's
 *     residual (sent -> 0, unsent -> a);
 *   - the server keeps, per worker k, D_k = M - v_k (the part of the accumulated
 *     update M not yet sent to k).  A push subtracts the decoded update from the
 *     model and from every D_w (Eq. 1, Eq. 3); a pull sends the top-k of D_k and
 *     zeroes what it sent (Eq. 6: v_k += G  <=>  D_k -= G).  The printed form (global
 *     model and v_k per worker) is given as well, see dgs_oracle_server_pull_sent.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ORACLE_OK = 0, ORACLE_EINVAL = -1, ORACLE_ENOMEM = -2 };

static uint32_t mag_key(float x)
{
    uint32_t b;
    memcpy(&b, &x, sizeof b);
    return b & 0x7FFFFFFFu;
}

/* k = ceil(density * n), IEEE double (reading of "R% of"). */
uint64_t dgs_oracle_k(double density, uint64_t n)
{
    return (uint64_t)ceil(density * (double)n);
}

static int cmp_key_desc(const void *pa, const void *pb)
{
    uint32_t a = *(const uint32_t *)pa, b = *(const uint32_t *)pb;
    return (a < b) - (a > b);
}

/*
 * Definition of the per-tensor selection (Algorithm 1/3 inner loop, Algorithm 2
 * secondary compression): mark the k entries of a[0..n) with the largest
 * magnitude; ties at the k-th magnitude go to the lowest indices.
 * Written as: sort all magnitudes, read off the k-th largest T, then walk the
 * tensor in index order taking everything above T and the first r entries equal
 * to T, r = k - #{> T}.
 */
static int select_topk(const float *a, uint64_t n, uint64_t k, uint8_t *sel)
{
    uint64_t i, gt = 0, r;
    uint32_t T;
    uint32_t *keys;
    memset(sel, 0, n);
    if (k == 0) return ORACLE_OK;
    if (k > n) return ORACLE_EINVAL;
    keys = (uint32_t *)malloc(n * sizeof *keys);
    if (!keys) return ORACLE_ENOMEM;
    for (i = 0; i < n; ++i) keys[i] = mag_key(a[i]);
    qsort(keys, n, sizeof *keys, cmp_key_desc);
    T = keys[k - 1];
    while (gt < n && keys[gt] > T) ++gt;
    free(keys);
    r = k - gt;
    for (i = 0; i < n; ++i) {
        uint32_t key = mag_key(a[i]);
        if (key > T) sel[i] = 1;
        else if (key == T && r > 0) { sel[i] = 1; --r; }
    }
    return ORACLE_OK;
}

/*
 * Brute-force statement of the same selection, for tiny inputs: sort (magnitude,
 * index) pairs by magnitude descending then index ascending and keep the first
 * k.  idx_out receives the k positions in ascending order.
 */
typedef struct { uint32_t key; uint32_t idx; } pair_t;

static int cmp_pair(const void *pa, const void *pb)
{
    const pair_t *a = (const pair_t *)pa, *b = (const pair_t *)pb;
    if (a->key != b->key) return (a->key < b->key) - (a->key > b->key);
    return (a->idx > b->idx) - (a->idx < b->idx);
}

static int cmp_u32_asc(const void *pa, const void *pb)
{
    uint32_t a = *(const uint32_t *)pa, b = *(const uint32_t *)pb;
    return (a > b) - (a < b);
}

int dgs_oracle_topk_bruteforce(const float *a, uint32_t n, uint32_t k, uint32_t *idx_out)
{
    uint32_t i;
    pair_t *p;
    if (k > n) return ORACLE_EINVAL;
    p = (pair_t *)malloc((size_t)(n ? n : 1) * sizeof *p);
    if (!p) return ORACLE_ENOMEM;
    for (i = 0; i < n; ++i) { p[i].key = mag_key(a[i]); p[i].idx = i; }
    qsort(p, n, sizeof *p, cmp_pair);
    for (i = 0; i < k; ++i) idx_out[i] = p[i].idx;
    qsort(idx_out, k, sizeof *idx_out, cmp_u32_asc);
    free(p);
    return ORACLE_OK;
}

/* Same selection through the production definition, positions ascending. */
int dgs_oracle_topk(const float *a, uint64_t n, uint64_t k, uint32_t *idx_out)
{
    uint8_t *sel = (uint8_t *)malloc(n ? n : 1);
    uint64_t i, o = 0;
    int rc;
    if (!sel) return ORACLE_ENOMEM;
    rc = select_topk(a, n, k, sel);
    if (rc == ORACLE_OK)
        for (i = 0; i < n; ++i)
            if (sel[i]) idx_out[o++] = (uint32_t)i;
    free(sel);
    return rc;
}

/* Sum over tensors of k_j; k_per_tensor (J entries) may be NULL. */
int dgs_oracle_nnz(const uint64_t *offsets, uint32_t J, double density,
                   uint64_t *k_per_tensor, uint64_t *K_out)
{
    uint32_t j;
    uint64_t K = 0;
    if (!(density > 0.0) || density > 1.0) return ORACLE_EINVAL;
    for (j = 0; j < J; ++j) {
        uint64_t kj = dgs_oracle_k(density, offsets[j + 1] - offsets[j]);
        if (k_per_tensor) k_per_tensor[j] = kj;
        K += kj;
    }
    *K_out = K;
    return ORACLE_OK;
}

/*
 * One worker iteration after the backward pass (Algorithm 3 steps "u <- m u +
 * eta grad" through "send encode(g)"; Algorithm 1 when m == 0).
 *   grad   n floats, read only
 *   state  n floats, in/out: s = m * u (velocity form) or the residual v (m == 0)
 *   idx,val  outputs, capacity >= sum_j k_j; pairs in ascending flat index,
 *            tensor after tensor; val is the accumulated value a_i that is sent
 */
int dgs_oracle_worker_step(const float *grad, float *state, const uint64_t *offsets,
                           uint32_t J, float lr, float m, double density,
                           uint32_t *idx, float *val, uint64_t *nnz)
{
    uint64_t n = offsets[J], i, o = 0;
    uint32_t j;
    float *a;
    uint8_t *sel;
    int rc = ORACLE_OK;
    if (!(density > 0.0) || density > 1.0) return ORACLE_EINVAL;
    a = (float *)malloc((n ? n : 1) * sizeof *a);
    sel = (uint8_t *)malloc(n ? n : 1);
    if (!a || !sel) { free(a); free(sel); return ORACLE_ENOMEM; }

    /* accumulate: a = m*u + eta*grad  (state already holds m*u) */
    for (i = 0; i < n; ++i) a[i] = fmaf(lr, grad[i], state[i]);

    for (j = 0; j < J && rc == ORACLE_OK; ++j) {
        uint64_t b = offsets[j], nj = offsets[j + 1] - b;
        uint64_t kj = dgs_oracle_k(density, nj);
        rc = select_topk(a + b, nj, kj, sel + b);
    }
    if (rc == ORACLE_OK) {
        for (i = 0; i < n; ++i) {
            if (sel[i]) {
                idx[o] = (uint32_t)i;          /* encode(): coordinate format */
                val[o] = a[i];                 /* g = u (.) Mask              */
                ++o;
                state[i] = m * a[i];           /* sent: u stays a  => s = m a */
            } else {
                state[i] = a[i];               /* unsent: u = a/m  => s = a   */
            }
        }
        *nnz = o;
    }
    free(a);
    free(sel);
    return rc;
}

/*
 * Server receives one decoded update (Algorithm 2 "M <- M - decode(g)"; Eq. 1).
 * model (n floats) tracks theta_0 + M; diff holds W rows of n floats, row w =
 * D_w = M - v_w, so every row moves with M (Eq. 3).
 */
int dgs_oracle_server_push(float *model, float *diff, uint32_t W, uint64_t n,
                           const uint32_t *idx, const float *val, uint64_t nnz)
{
    uint64_t e;
    uint32_t w;
    for (e = 0; e < nnz; ++e) {
        uint64_t i = idx[e];
        if (i >= n) return ORACLE_EINVAL;
        if (model) model[i] = model[i] - val[e];
        for (w = 0; w < W; ++w) diff[(uint64_t)w * n + i] = diff[(uint64_t)w * n + i] - val[e];
    }
    return ORACLE_OK;
}

/*
 * Server answers worker k with secondary compression (Algorithm 2 inner loop,
 * Eq. 6): G = top-k_j per tensor of D_k; v_k += G, i.e. sent entries of D_k
 * become +0.  diff_k points at row k.
 */
int dgs_oracle_server_pull(float *diff_k, const uint64_t *offsets, uint32_t J,
                           double density, uint32_t *idx, float *val, uint64_t *nnz)
{
    uint64_t n = offsets[J], i, o = 0;
    uint32_t j;
    uint8_t *sel;
    int rc = ORACLE_OK;
    if (!(density > 0.0) || density > 1.0) return ORACLE_EINVAL;
    sel = (uint8_t *)malloc(n ? n : 1);
    if (!sel) return ORACLE_ENOMEM;
    for (j = 0; j < J && rc == ORACLE_OK; ++j) {
        uint64_t b = offsets[j], nj = offsets[j + 1] - b;
        rc = select_topk(diff_k + b, nj, dgs_oracle_k(density, nj), sel + b);
    }
    if (rc == ORACLE_OK) {
        for (i = 0; i < n; ++i) {
            if (sel[i]) {
                idx[o] = (uint32_t)i;
                val[o] = diff_k[i];
                ++o;
                diff_k[i] = 0.0f;
            }
        }
        *nnz = o;
    }
    free(sel);
    return rc;
}

/*
 * The same server step with the state Algorithm 2 prints: one global model
 * (theta_0 + M) and sent_k = theta_0 + v_k per worker.
 *   push:  M <- M - decode(g)  (Eq. 1) touches the model only;
 *   pull:  G <- M - v_k (dense, one fp32 subtraction per element), per tensor keep the
 *          k_j largest magnitudes of G (the threshold loop), send them, then
 *          v_k <- v_k + G on what was sent (Eq. 6; Eq. 4 fixes the sign).
 */
int dgs_oracle_server_push_model(float *model, uint64_t n, const uint32_t *idx, const float *val,
                                 uint64_t nnz)
{
    uint64_t e;
    for (e = 0; e < nnz; ++e) {
        if (idx[e] >= n) return ORACLE_EINVAL;
        model[idx[e]] = model[idx[e]] - val[e];
    }
    return ORACLE_OK;
}

int dgs_oracle_server_pull_sent(const float *model, float *sent_k, const uint64_t *offsets, uint32_t J,
                                double density, uint32_t *idx, float *val, uint64_t *nnz)
{
    uint64_t n = offsets[J], i, o = 0;
    uint32_t j;
    uint8_t *sel;
    float *G;
    int rc = ORACLE_OK;
    if (!(density > 0.0) || density > 1.0) return ORACLE_EINVAL;
    sel = (uint8_t *)malloc(n ? n : 1);
    G = (float *)malloc((n ? n : 1) * sizeof(float));
    if (!sel || !G) { free(sel); free(G); return ORACLE_ENOMEM; }
    for (i = 0; i < n; ++i) G[i] = model[i] - sent_k[i];
    for (j = 0; j < J && rc == ORACLE_OK; ++j) {
        uint64_t b = offsets[j], nj = offsets[j + 1] - b;
        rc = select_topk(G + b, nj, dgs_oracle_k(density, nj), sel + b);
    }
    if (rc == ORACLE_OK) {
        for (i = 0; i < n; ++i) {
            if (sel[i]) {
                idx[o] = (uint32_t)i;
                val[o] = G[i];
                ++o;
                sent_k[i] = sent_k[i] + G[i];
            }
        }
        *nnz = o;
    }
    free(sel);
    free(G);
    return rc;
}

/*
 * Server answers worker k WITHOUT secondary compression (Algorithm 2 with the
 * switch off; Eq. 3-4): G = D_k in coordinate format, i.e. every entry whose
 * magnitude key is nonzero, ascending; afterwards D_k == 0 (v_k = M).
 * Returns ORACLE_EINVAL if more than `capacity` pairs would be produced.
 */
int dgs_oracle_server_pull_all(float *diff_k, uint64_t n, uint32_t *idx, float *val,
                               uint64_t capacity, uint64_t *nnz)
{
    uint64_t i, o = 0;
    for (i = 0; i < n; ++i)
        if (mag_key(diff_k[i]) != 0) ++o;
    if (o > capacity) { *nnz = o; return ORACLE_EINVAL; }
    o = 0;
    for (i = 0; i < n; ++i) {
        if (mag_key(diff_k[i]) != 0) {
            idx[o] = (uint32_t)i;
            val[o] = diff_k[i];
            ++o;
            diff_k[i] = 0.0f;
        }
    }
    *nnz = o;
    return ORACLE_OK;
}

/*
 * The same on the state Algorithm 2 prints (global model and sent_k = theta_0 + v_k):
 * G = M - v_k (Eq. 3, one fp32 subtraction per element), every entry with a nonzero
 * magnitude key is sent, then v_k <- v_k + G on those (Eq. 6).  In fp32 v_k + (M - v_k)
 * need not reproduce M bit for bit; the printed update is what is computed.
 */
int dgs_oracle_server_pull_all_sent(const float *model, float *sent_k, uint64_t n, uint32_t *idx,
                                    float *val, uint64_t capacity, uint64_t *nnz)
{
    uint64_t i, o = 0;
    for (i = 0; i < n; ++i)
        if (mag_key(model[i] - sent_k[i]) != 0) ++o;
    if (o > capacity) { *nnz = o; return ORACLE_EINVAL; }
    o = 0;
    for (i = 0; i < n; ++i) {
        float g = model[i] - sent_k[i];
        if (mag_key(g) != 0) {
            idx[o] = (uint32_t)i;
            val[o] = g;
            ++o;
            sent_k[i] = sent_k[i] + g;
        }
    }
    *nnz = o;
    return ORACLE_OK;
}

/* Worker applies a decoded message: theta[idx] += sign * val (Eq. 5 with sign = +1). */
int dgs_oracle_apply_sparse(float *dst, uint64_t n, const uint32_t *idx, const float *val,
                            uint64_t nnz, float sign)
{
    uint64_t e;
    for (e = 0; e < nnz; ++e) {
        if (idx[e] >= n) return ORACLE_EINVAL;
        dst[idx[e]] = fmaf(sign, val[e], dst[idx[e]]);
    }
    return ORACLE_OK;
}

/*
 * Wire form of one message: encode() / decode() of Algorithms 1-3.  The paper only says
 * that encode() packs the nonzero entries into coordinate format; the (idx, val) pairs
 * above already are that.  The byte layout below is this library's own -- PARITY UNPINNED
 * with respect to the paper: the pins fix it to the statement given here (a byte string
 * worked out by hand, a big-integer construction, the round trip), not to anything printed
 * in the paper.
 *
 * A message for (layout, density) holds exactly k_j = ceil(density * n_j) entries of every
 * tensor j, ascending, tensor after tensor (K = sum k_j); both ends know the layout and the
 * density, so there is no header:
 *   bytes [0, 4K)   the K values, fp32 little-endian, in message order (bit-exact);
 *   then for j = 0 .. J-1 the index block of tensor j: its k_j local indices idx - off_j,
 *   b_j bits each with b_j = number of bits of n_j - 1 (at least 1); entry e holds bits
 *   [e b_j, (e + 1) b_j) of the block, least significant bit first; bit i of the block is
 *   bit i mod 8 of its byte i / 8; the block is padded with zero bits to a multiple of 4
 *   bytes.
 */
static uint32_t index_bits(uint64_t nj)
{
    uint32_t b = 0;
    uint64_t top = nj - 1;
    while (top) { ++b; top >>= 1; }
    return b ? b : 1;
}

int dgs_oracle_wire_bytes(const uint64_t *offsets, uint32_t J, double density, uint64_t *bytes_out)
{
    uint32_t j;
    uint64_t bytes = 0;
    if (!(density > 0.0) || density > 1.0) return ORACLE_EINVAL;
    for (j = 0; j < J; ++j) {
        uint64_t nj = offsets[j + 1] - offsets[j];
        uint64_t kj = dgs_oracle_k(density, nj);
        bytes += 4 * kj;                                       /* values */
        bytes += 4 * ((kj * index_bits(nj) + 31) / 32);        /* index block */
    }
    *bytes_out = bytes;
    return ORACLE_OK;
}

int dgs_oracle_encode(const uint64_t *offsets, uint32_t J, double density, const uint32_t *idx,
                      const float *val, uint8_t *wire)
{
    uint32_t j, t;
    uint64_t K = 0, e, o = 0, base, total;
    if (dgs_oracle_wire_bytes(offsets, J, density, &total) != ORACLE_OK) return ORACLE_EINVAL;
    for (j = 0; j < J; ++j) K += dgs_oracle_k(density, offsets[j + 1] - offsets[j]);
    memset(wire, 0, total);
    for (e = 0; e < K; ++e) {                                   /* values, byte by byte */
        uint32_t bits;
        memcpy(&bits, &val[e], sizeof bits);
        for (t = 0; t < 4; ++t) wire[4 * e + t] = (uint8_t)(bits >> (8 * t));
    }
    base = 4 * K;                                               /* first byte of the current index block */
    for (j = 0; j < J; ++j) {
        uint64_t nj = offsets[j + 1] - offsets[j];
        uint64_t kj = dgs_oracle_k(density, nj);
        uint32_t b = index_bits(nj);
        for (e = 0; e < kj; ++e, ++o) {
            uint64_t local;
            if (idx[o] < offsets[j] || idx[o] >= offsets[j + 1]) return ORACLE_EINVAL;
            if (e > 0 && idx[o] <= idx[o - 1]) return ORACLE_EINVAL;
            local = idx[o] - offsets[j];
            for (t = 0; t < b; ++t) {                           /* bit by bit */
                uint64_t pos = e * b + t;
                if ((local >> t) & 1u) wire[base + pos / 8] |= (uint8_t)(1u << (pos % 8));
            }
        }
        base += 4 * ((kj * b + 31) / 32);
    }
    return ORACLE_OK;
}

/*
 * The same wire form with 16-bit values (PARITY UNPINNED with respect to the paper, which names
 * the combination with quantisation as future work, Section 6; pinned to this statement of it).
 * Every value travels as a bfloat16: the binary32 number cut to its upper 16 bits (sign, 8
 * exponent bits, 7 fraction bits), rounded to the nearest such number, halfway cases to the one
 * whose last kept bit is 0; a value beyond the largest finite bfloat16 becomes infinity; a NaN
 * stays a NaN (quiet).  Layout: K values of 2 bytes (little endian), padded with zero bytes to
 * a multiple of 4, then the index blocks exactly as in the 32-bit form.
 */
static uint16_t bf16_nearest_even(float x)
{
    uint32_t bits, kept, rest;
    memcpy(&bits, &x, sizeof bits);
    if ((bits & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((bits >> 16) | 0x0040u);   /* NaN, made quiet */
    kept = bits >> 16;                 /* candidate below (in magnitude) */
    rest = bits & 0xFFFFu;             /* what is cut off, in units of 2^-16 of the kept step */
    if (rest > 0x8000u) kept += 1;                       /* nearer to the candidate above */
    else if (rest == 0x8000u && (kept & 1u)) kept += 1;  /* halfway: to the even one */
    return (uint16_t)kept;             /* a carry out of the fraction moves to the next exponent, up to infinity */
}

int dgs_oracle_wire_bytes16(const uint64_t *offsets, uint32_t J, double density, uint64_t *bytes_out)
{
    uint32_t j;
    uint64_t K = 0, bytes = 0;
    if (!(density > 0.0) || density > 1.0) return ORACLE_EINVAL;
    for (j = 0; j < J; ++j) {
        uint64_t nj = offsets[j + 1] - offsets[j];
        uint64_t kj = dgs_oracle_k(density, nj);
        K += kj;
        bytes += 4 * ((kj * index_bits(nj) + 31) / 32);
    }
    *bytes_out = 4 * ((2 * K + 3) / 4) + bytes;
    return ORACLE_OK;
}

int dgs_oracle_encode16(const uint64_t *offsets, uint32_t J, double density, const uint32_t *idx,
                        const float *val, uint8_t *wire)
{
    uint32_t j, t;
    uint64_t K = 0, e, o = 0, base, total;
    if (dgs_oracle_wire_bytes16(offsets, J, density, &total) != ORACLE_OK) return ORACLE_EINVAL;
    for (j = 0; j < J; ++j) K += dgs_oracle_k(density, offsets[j + 1] - offsets[j]);
    memset(wire, 0, total);
    for (e = 0; e < K; ++e) {
        uint16_t h = bf16_nearest_even(val[e]);
        wire[2 * e] = (uint8_t)(h & 0xFFu);
        wire[2 * e + 1] = (uint8_t)(h >> 8);
    }
    base = 4 * ((2 * K + 3) / 4);
    for (j = 0; j < J; ++j) {
        uint64_t nj = offsets[j + 1] - offsets[j];
        uint64_t kj = dgs_oracle_k(density, nj);
        uint32_t b = index_bits(nj);
        for (e = 0; e < kj; ++e, ++o) {
            uint64_t local;
            if (idx[o] < offsets[j] || idx[o] >= offsets[j + 1]) return ORACLE_EINVAL;
            if (e > 0 && idx[o] <= idx[o - 1]) return ORACLE_EINVAL;
            local = idx[o] - offsets[j];
            for (t = 0; t < b; ++t) {
                uint64_t pos = e * b + t;
                if ((local >> t) & 1u) wire[base + pos / 8] |= (uint8_t)(1u << (pos % 8));
            }
        }
        base += 4 * ((kj * b + 31) / 32);
    }
    return ORACLE_OK;
}

int dgs_oracle_decode16(const uint64_t *offsets, uint32_t J, double density, const uint8_t *wire,
                        uint32_t *idx, float *val)
{
    uint32_t j, t;
    uint64_t K = 0, e, o = 0, base;
    if (!(density > 0.0) || density > 1.0) return ORACLE_EINVAL;
    for (j = 0; j < J; ++j) K += dgs_oracle_k(density, offsets[j + 1] - offsets[j]);
    for (e = 0; e < K; ++e) {          /* a bfloat16 is the upper half of a binary32: exact */
        uint32_t bits = ((uint32_t)wire[2 * e] | ((uint32_t)wire[2 * e + 1] << 8)) << 16;
        memcpy(&val[e], &bits, sizeof bits);
    }
    base = 4 * ((2 * K + 3) / 4);
    for (j = 0; j < J; ++j) {
        uint64_t nj = offsets[j + 1] - offsets[j];
        uint64_t kj = dgs_oracle_k(density, nj);
        uint32_t b = index_bits(nj);
        for (e = 0; e < kj; ++e, ++o) {
            uint64_t local = 0;
            for (t = 0; t < b; ++t) {
                uint64_t pos = e * b + t;
                if ((wire[base + pos / 8] >> (pos % 8)) & 1u) local |= (uint64_t)1 << t;
            }
            if (local >= nj) return ORACLE_EINVAL;
            idx[o] = (uint32_t)(offsets[j] + local);
        }
        base += 4 * ((kj * b + 31) / 32);
    }
    return ORACLE_OK;
}

int dgs_oracle_decode(const uint64_t *offsets, uint32_t J, double density, const uint8_t *wire,
                      uint32_t *idx, float *val)
{
    uint32_t j, t;
    uint64_t K = 0, e, o = 0, base;
    if (!(density > 0.0) || density > 1.0) return ORACLE_EINVAL;
    for (j = 0; j < J; ++j) K += dgs_oracle_k(density, offsets[j + 1] - offsets[j]);
    for (e = 0; e < K; ++e) {
        uint32_t bits = 0;
        for (t = 0; t < 4; ++t) bits |= (uint32_t)wire[4 * e + t] << (8 * t);
        memcpy(&val[e], &bits, sizeof bits);
    }
    base = 4 * K;
    for (j = 0; j < J; ++j) {
        uint64_t nj = offsets[j + 1] - offsets[j];
        uint64_t kj = dgs_oracle_k(density, nj);
        uint32_t b = index_bits(nj);
        for (e = 0; e < kj; ++e, ++o) {
            uint64_t local = 0;
            for (t = 0; t < b; ++t) {
                uint64_t pos = e * b + t;
                if ((wire[base + pos / 8] >> (pos % 8)) & 1u) local |= (uint64_t)1 << t;
            }
            if (local >= nj) return ORACLE_EINVAL;
            idx[o] = (uint32_t)(offsets[j] + local);
        }
        base += 4 * ((kj * b + 31) / 32);
    }
    return ORACLE_OK;
}
