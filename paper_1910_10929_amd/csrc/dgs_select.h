// Exact per-tensor selection on ordered entries: sources, window / radix passes, ordered
// emission ("encode()" of Algorithms 1-3) with the state fix-up of Eq. 12 / Eq. 6, and the
// threshold hints.  Shared by the single-workgroup selection and the segmented chain.
#pragma once
#include "dgs_wave.h"

namespace dgs {

// ---------------------------------------------------------------------------
// select
// ---------------------------------------------------------------------------

// The value the selection ranks at flat index ix, read from the buffers themselves
// (dense sources, zero fill): the state / difference row, or model - sent_k.
template <int OP>
__device__ __forceinline__ float row_value(const float *state, const float *model, uint32_t ix)
{
    return (OP == SEL_PULL_V) ? (model[ix] - state[ix]) : state[ix];
}

// What a sent entry leaves behind: worker m * a (Eq. 12, state stored as m u); pull on a
// difference row +0 (Eq. 6 as D_k -= G); pull on model - sent_k: sent_k += G (Eq. 6).
template <int OP>
__device__ __forceinline__ void fix_sent(float *state, uint32_t ix, float val, float m)
{
    if (OP == SEL_WORKER) store_scattered(&state[ix], m * val);
    else if (OP == SEL_PULL) store_scattered(&state[ix], 0.0f);
    else store_scattered(&state[ix], state[ix] + val);
}

// An index that came out of a candidate list is used as an address: one outside the buffer
// (a corrupted list) is counted as an internal error and never dereferenced.
__device__ __forceinline__ bool index_ok(const SelectArgs &A, uint32_t ix)
{
    if (ix < A.n) return true;
    atomicAdd(&A.stats->internal_errors, 1ull);
    return false;
}

template <int OP>
struct SrcDense {          // the tensor itself: position p <-> element off + p
    static constexpr bool AGG = false;
    const float *base;
    const float *model;
    uint32_t off;
    __device__ __forceinline__ uint32_t bits(uint32_t p) const
    {
        return __float_as_uint(row_value<OP>(base, model, off + p));
    }
    __device__ __forceinline__ uint32_t index(uint32_t p) const { return off + p; }
};

struct SrcDenseLds {       // a small tensor staged in LDS: position p <-> element off + p
    static constexpr bool AGG = false;
    const uint32_t *v;
    uint32_t off;
    __device__ __forceinline__ uint32_t bits(uint32_t p) const { return v[p]; }
    __device__ __forceinline__ uint32_t index(uint32_t p) const { return off + p; }
};

struct SrcList {           // ordered candidates (index, value bits)
    static constexpr bool AGG = true;   // candidates share their top key bits: merge per wavefront
    const uint2 *list;
    __device__ __forceinline__ uint32_t bits(uint32_t p) const { return list[p].y; }
    __device__ __forceinline__ uint32_t index(uint32_t p) const { return list[p].x; }
};

struct SrcSplit {          // a list whose first SEL_LDS_LIST entries are in LDS, the rest in global scratch
    static constexpr bool AGG = true;
    const uint2 *llist;
    const uint2 *glist;
    __device__ __forceinline__ uint2 get(uint32_t p) const { return (p < SEL_LDS_LIST) ? llist[p] : glist[p]; }
    __device__ __forceinline__ uint32_t bits(uint32_t p) const { return get(p).y; }
    __device__ __forceinline__ uint32_t index(uint32_t p) const { return get(p).x; }
};

struct SelShared {
    uint32_t h[2048];
    uint32_t wsum[SEL_WAVES];
    uint32_t rowsum[64];
    int res[6];
    uint32_t kmin;
};

// Count into an LDS histogram.  With AGG (all 64 lanes must call this together), the
// lanes that hit the same bin as the first valid lane are merged into one atomic --
// candidate keys mostly share their top bits -- and the others add on their own.
template <bool AGG>
__device__ __forceinline__ void hist_add(uint32_t *h, uint32_t bin, bool valid)
{
    if (!AGG) {
        if (valid) atomicAdd(&h[bin], 1u);
        return;
    }
    const uint64_t todo = ballot64(valid);
    if (todo == 0) return;
    const int leader = __ffsll((unsigned long long)todo) - 1;
    const uint32_t b0 = (uint32_t)__builtin_amdgcn_readlane((int)bin, leader);
    const uint64_t same = ballot64(valid && bin == b0);
    if ((int)lane_id() == leader) atomicAdd(&h[b0], (uint32_t)__popcll(same));
    else if (valid && bin != b0) atomicAdd(&h[bin], 1u);
}

// Window histogram of candidate keys: bucket (key >> 11) - win_base, everything at or
// below the base in bucket 0, everything beyond the window in bucket 2047.
__device__ __forceinline__ void window_count(uint32_t *h, uint32_t win_base, uint32_t key)
{
    const uint32_t hi = key >> 11;
    const uint32_t w = (hi > win_base) ? (hi - win_base) : 0u;
    atomicAdd(&h[min(w, 2047u)], 1u);
}

// Next threshold when fewer candidates (c) than the hinted rank R were collected, all at
// or above `kmin`: the lowest q of them span `width` keys; the same density is assumed
// below kmin (it is higher in fact, so this errs towards more candidates), with half as
// much again for safety, and never below half of the smallest candidate key.
__device__ __forceinline__ uint32_t hint_extrapolated(uint32_t kmin, uint32_t c, uint32_t R, uint32_t q,
                                                      uint32_t width)
{
    const float delta = 1.5f * (float)(R - c) * (float)width / (float)max(q, 1u);
    uint32_t tn = (delta < (float)kmin) ? (kmin - (uint32_t)delta) : 1u;
    if (kmin < 0x7F800000u) {
        const uint32_t half = __float_as_uint(__uint_as_float(kmin) * 0.5f) & 0x7FFFFFFFu;
        tn = max(tn, half);
    }
    return max(tn, 1u);
}

// Exact selection over `cN` ordered entries of `src`; emits the k winners in
// order and applies the state fix-up.  If R != 0 and R <= cN, also finds the
// 21-bit key prefix of the entry of rank R: *tau_next = its lower edge (>= 1)
// and *expect = how many entries lie at or above that edge; otherwise both 0.
// Candidate lists come with a window: win_base = first bucket (key >> 11), 0xFFFFFFFF for
// other sources; win_min = 1 if entries may lie below the base (bucket 0 is then mixed and
// cannot hold a result), else 0; win_ready: S.h already holds the window histogram of the
// entries (window_count); kmin = smallest key of the list.
template <int OP, int ITEMS, class Src>
__device__ __forceinline__ void select_emit(const Src src, const uint32_t cN, const uint32_t k,
                                            const uint32_t R, const uint32_t Eq, const uint32_t win_base,
                                            const uint32_t win_min, const bool win_ready, const uint32_t kmin,
                                            SelShared &S, const SelectArgs &A, const uint32_t outoff,
                                            uint32_t *tau_next, uint32_t *expect, uint32_t *q_e,
                                            uint32_t *t_out)
{
    const uint32_t tid = threadIdx.x;
    const bool measurable = (R != 0) && (cN >= R);
    *tau_next = 0;
    *expect = 0;
    *q_e = 0;

    uint32_t pfx = 0;        // key prefix of the k-th entry, `lowbits` bits still unresolved
    uint32_t r2 = 0;         // its rank among the entries sharing that prefix
    uint32_t lowbits = 10;
    bool have_prefix = false;

    // ---- candidate lists: every key is >= the collection threshold, and the k-th key
    //      normally lies within a factor ~1.4 of it, or close to the previous call's.  One
    //      pass over a window of 2047 buckets of key >> 11 (bucket 2047 = everything
    //      beyond) resolves 20 key bits at once.  A window that was placed by those hints
    //      and missed the k-th key is tried once more from the smallest key of the list.
    if (Src::AGG && win_base != 0xFFFFFFFFu) {
        uint32_t base = win_base, bmin = win_min;
        bool counted = win_ready;
        for (int attempt = 0; attempt < 2; ++attempt) {
            if (!counted) {   // otherwise the caller has counted the entries while it built the list
                for (uint32_t b = tid; b < 2048; b += SEL_THREADS) S.h[b] = 0;
                __syncthreads();
                for (uint32_t pb = 0; pb < cN; pb += 4 * SEL_THREADS) {
                    uint32_t kk[4];
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const uint32_t p = pb + i * SEL_THREADS + tid;
                        kk[i] = (p < cN) ? (src.bits(p) & 0x7FFFFFFFu) : 0u;
                    }
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        if (pb + i * SEL_THREADS + tid < cN) window_count(S.h, base, kk[i]);
                }
            }
            // third rank: the drift quantile if R is among the candidates; otherwise the entry
            // below which the lowest quarter of the candidates lies (for the extrapolated hint)
            const uint32_t qlow = max(cN / 4u, min(cN, 16u));
            const uint32_t third = measurable ? ((Eq <= cN) ? Eq : 0u) : ((R != 0) ? (cN - qlow + 1u) : 0u);
            find_ranks<2048, SEL_WAVES>(S.h, k, measurable ? R : k, third, S.rowsum, S.res);
            const int bk = S.res[0], bR = S.res[2], bE = S.res[4];
            const uint32_t rk = (uint32_t)S.res[1], rR = (uint32_t)S.res[3];
            const int lo = (int)bmin;
            if (bk >= lo && bk < 2047 && bR >= lo && bR < 2047) {
                have_prefix = true;
                pfx = base + (uint32_t)bk;
                r2 = rk;
                lowbits = 11;
                if (measurable) {
                    const uint32_t edge = (base + (uint32_t)bR) << 11;
                    *tau_next = edge ? edge : 1u;
                    *expect = R - rR + S.h[bR];
                    if (bE >= lo && bE < 2047) *q_e = (base + (uint32_t)bE) << 11;
                } else if (R != 0 && bE >= lo && bE < 2047) {
                    const uint32_t top = (base + (uint32_t)bE + 1u) << 11;   // the lowest quarter ends below it
                    *tau_next = hint_extrapolated(max(kmin, 1u), cN, R, qlow, top - min(kmin, top - 1u));
                    *expect = R;
                }
            }
            __syncthreads();
            if (have_prefix || base == (kmin >> 11)) break;
            base = kmin >> 11;
            bmin = 0;
            counted = false;
        }
    }

    if (!have_prefix) {
        // ---- pass 1: key bits [30:20]
        for (uint32_t b = tid; b < 2048; b += SEL_THREADS) S.h[b] = 0;
        __syncthreads();
        for (uint32_t pb = 0; pb < cN; pb += 4 * SEL_THREADS) {
            uint32_t kk[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const uint32_t p = pb + i * SEL_THREADS + tid;
                kk[i] = (p < cN) ? (src.bits(p) & 0x7FFFFFFFu) : 0u;
            }
#pragma unroll
            for (int i = 0; i < 4; ++i)
                hist_add<Src::AGG>(S.h, kk[i] >> 20, pb + i * SEL_THREADS + tid < cN);
        }
        find_ranks<2048, SEL_WAVES>(S.h, k, measurable ? R : k, 0u, S.rowsum, S.res);
        const int b1 = S.res[0];
        const uint32_t r1 = (uint32_t)S.res[1];
        const int c1 = S.res[2];
        const uint32_t q1 = (uint32_t)S.res[3];
        __syncthreads();
        if (b1 < 0 || c1 < 0) {   // cannot happen for cN >= k
            if (tid == 0) atomicAdd(&A.stats->internal_errors, 1ull);
            return;
        }

        // ---- pass 2: key bits [19:10] inside bucket b1 (and inside c1 for the hint)
        const bool two = measurable && (c1 != b1);
        for (uint32_t b = tid; b < 2048; b += SEL_THREADS) S.h[b] = 0;
        __syncthreads();
        for (uint32_t pb = 0; pb < cN; pb += 4 * SEL_THREADS) {
            uint32_t kk[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const uint32_t p = pb + i * SEL_THREADS + tid;
                kk[i] = (p < cN) ? (src.bits(p) & 0x7FFFFFFFu) : 0xFFFFFFFFu;   // top bits match no bucket
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int top = (int)(kk[i] >> 20);
                if (top == b1) atomicAdd(&S.h[(kk[i] >> 10) & 1023u], 1u);
                else if (two && top == c1) atomicAdd(&S.h[1024u + ((kk[i] >> 10) & 1023u)], 1u);
            }
        }
        find_ranks<1024, SEL_WAVES>(S.h, r1, (measurable && !two) ? q1 : r1, 0u, S.rowsum, S.res);
        const int b2 = S.res[0];
        r2 = (uint32_t)S.res[1];
        int c2 = S.res[2];
        uint32_t q2 = (uint32_t)S.res[3];
        __syncthreads();
        if (two) {
            find_ranks<1024, SEL_WAVES>(S.h + 1024, q1, 0u, 0u, S.rowsum, S.res);
            c2 = S.res[0];
            q2 = (uint32_t)S.res[1];
            __syncthreads();
        }
        if (measurable && c2 >= 0) {
            const uint32_t edge = ((uint32_t)c1 << 20) | ((uint32_t)c2 << 10);
            *tau_next = edge ? edge : 1u;
            *expect = R - q2 + S.h[(two ? 1024 : 0) + c2];
        }
        if (b2 < 0) {
            if (tid == 0) atomicAdd(&A.stats->internal_errors, 1ull);
            return;
        }
        pfx = ((uint32_t)b1 << 10) | (uint32_t)b2;
        lowbits = 10;
        __syncthreads();
    }

    // ---- last pass: the low key bits among the entries sharing the prefix
    const uint32_t lowmask = (1u << lowbits) - 1u;
    for (uint32_t b = tid; b < 2048; b += SEL_THREADS) S.h[b] = 0;
    __syncthreads();
    for (uint32_t pb = 0; pb < cN; pb += 4 * SEL_THREADS) {
        uint32_t kk[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint32_t p = pb + i * SEL_THREADS + tid;
            kk[i] = (p < cN) ? (src.bits(p) & 0x7FFFFFFFu) : 0xFFFFFFFFu;
        }
#pragma unroll
        for (int i = 0; i < 4; ++i)
            if ((kk[i] >> lowbits) == pfx) atomicAdd(&S.h[kk[i] & lowmask], 1u);
    }
    find_ranks<2048, SEL_WAVES>(S.h, r2, 0u, 0u, S.rowsum, S.res);
    const int b3 = S.res[0];
    const uint32_t rT = (uint32_t)S.res[1];   // how many entries equal to T are taken (lowest index first)
    __syncthreads();
    if (b3 < 0) {
        if (tid == 0) atomicAdd(&A.stats->internal_errors, 1ull);
        return;
    }
    const uint32_t T = (pfx << lowbits) | (uint32_t)b3;
    *t_out = T;

    // ---- ordered emission
    uint32_t run_sel = 0, run_eq = 0;
    constexpr uint32_t CHUNK = SEL_THREADS * ITEMS;
    for (uint32_t cb = 0; cb < cN; cb += CHUNK) {
        const uint32_t p0 = cb + tid * ITEMS;
        uint32_t vb[ITEMS];
        uint32_t g = 0, q = 0;
#pragma unroll
        for (int i = 0; i < ITEMS; ++i) {
            const uint32_t p = p0 + i;
            vb[i] = (p < cN) ? src.bits(p) : 0u;
        }
#pragma unroll
        for (int i = 0; i < ITEMS; ++i) {
            const uint32_t p = p0 + i;
            const uint32_t key = vb[i] & 0x7FFFFFFFu;
            if (p < cN) {
                g += (key > T);
                q += (key == T);
            }
        }
        uint32_t total;
        const uint32_t before = block_excl_scan<SEL_WAVES>(g | (q << 16), S.wsum, total);
        const uint32_t g_before = before & 0xFFFFu, q_before = before >> 16;
        const uint32_t G = total & 0xFFFFu, Q = total >> 16;
        const uint32_t rem = (rT > run_eq) ? (rT - run_eq) : 0u;   // ties still to take
        uint32_t pos = run_sel + g_before + min(q_before, rem);
        uint32_t eq_seen = q_before;
        if (g | q) {
            // which of this thread's entries are sent, and where they go
            uint32_t ix[ITEMS], at[ITEMS];
#pragma unroll
            for (int i = 0; i < ITEMS; ++i) {
                const uint32_t p = p0 + i;
                const uint32_t key = vb[i] & 0x7FFFFFFFu;
                bool sel = (p < cN) && key > T;
                if (p < cN && key == T) {
                    sel = eq_seen < rem;
                    ++eq_seen;
                }
                at[i] = 0xFFFFFFFFu;
                ix[i] = 0;
                if (sel) {
                    if (pos < k) {
                        ix[i] = src.index(p);
                        if (index_ok(A, ix[i])) at[i] = pos;
                    }
                    ++pos;
                }
            }
            // sent_k += G reads the row: all of this thread's reads are issued before the first
            // is needed (one memory round trip instead of one per entry)
            float old[ITEMS];
            if (OP == SEL_PULL_V) {
#pragma unroll
                for (int i = 0; i < ITEMS; ++i) old[i] = (at[i] != 0xFFFFFFFFu) ? A.state[ix[i]] : 0.0f;
            }
#pragma unroll
            for (int i = 0; i < ITEMS; ++i) {
                if (at[i] != 0xFFFFFFFFu) {
                    const float v = __uint_as_float(vb[i]);
                    A.out_idx[outoff + at[i]] = ix[i];
                    A.out_val[outoff + at[i]] = v;
                    if (OP == SEL_WORKER) store_scattered(&A.state[ix[i]], A.m * v);
                    else if (OP == SEL_PULL) store_scattered(&A.state[ix[i]], 0.0f);
                    else store_scattered(&A.state[ix[i]], old[i] + v);
                }
            }
        }
        run_sel += G + min(Q, rem);
        run_eq += Q;
    }
    if (run_sel != k && tid == 0) atomicAdd(&A.stats->internal_errors, 1ull);
}

// Rank (from the top) whose key becomes the next predicted threshold, and how the
// drift since the current threshold was set is measured.
//   c: candidates collected at the current threshold; E: candidates that threshold was
//   expected to collect when it was set (0 = unknown); `drift`: the two are comparable.
// Worker: sent entries stay large (they keep m * a) and unsent ones keep growing, so
// the keys of the tail move from step to step.  If the tail grew (c >= E), *Eq = E asks
// for the key of rank E among the present candidates: the old threshold's quantile has
// moved there, and the next threshold is scaled by the same ratio (hint_scaled).  If it
// shrank, the quantile lies below every candidate and cannot be read off: the rank is
// widened by the ratio of the counts instead.
template <int OP>
__device__ __forceinline__ uint32_t hint_rank(const TensorDesc &td, const PlanEntry &pe, bool drift,
                                              uint32_t c, uint32_t E, float m, uint32_t *Eq)
{
    *Eq = 0;
    // a pull, or a worker without momentum: sent entries vanish, so even with nothing new
    // before the next call k entries must remain above the hinted key (about 2k)
    uint32_t R = (OP != SEL_WORKER || m == 0.0f) ? pe.k2_pull : pe.k2;
    if (OP == SEL_WORKER && drift && E != 0) {
        if (c >= E) {
            *Eq = E;
        } else {
            const float d = fmaxf((float)c / (float)E, 0.5f);
            R = (uint32_t)((float)R / d);
        }
    }
    const uint32_t rmin = max(1u, pe.k / 4u);
    return min(max(R, rmin), td.n);
}

// Threshold for the next step: the key `edge` of the hinted rank, moved by half of the
// relative shift that the previous threshold's quantile showed (q_e / tau_cur, between 1
// and 2).  Half: growth usually slows down, and a threshold that is too high costs a
// dense re-selection while one that is too low only costs extra candidates.
__device__ __forceinline__ uint32_t hint_scaled(uint32_t edge, uint32_t q_e, uint32_t tau_cur)
{
    if (q_e <= tau_cur || tau_cur < 0x00800000u || q_e >= 0x7F800000u) return edge;   // no growth / not normal
    const float f = 1.0f + 0.5f * (fminf(__uint_as_float(q_e) / __uint_as_float(tau_cur), 2.0f) - 1.0f);
    const float x = __uint_as_float(edge) * f;
    const uint32_t t = __float_as_uint(x) & 0x7FFFFFFFu;
    return (t > edge && t < 0x7F800000u) ? t : edge;
}

// Next threshold when rank R was not among the candidates: relax the current one by a
// quarter, but not below half of the smallest candidate key (all of them already pass).
__device__ __forceinline__ uint32_t hint_relaxed(uint32_t tau_cur, uint32_t kmin)
{
    const float f = __uint_as_float(tau_cur & 0x7FFFFFFFu) * 0.75f;
    uint32_t tn = __float_as_uint(f) & 0x7FFFFFFFu;
    if (!(tau_cur > 1u) || tn == 0) tn = 1;
    if (kmin != 0xFFFFFFFFu && kmin < 0x7F800000u) {
        const uint32_t half = __float_as_uint(__uint_as_float(kmin) * 0.5f) & 0x7FFFFFFFu;
        if (half > tn) tn = half;
    }
    return tn;
}

// Fewer candidates than k although every nonzero key was collected: the message is
// completed with the tensor's lowest-index zero-key entries.  With z = k - c zeros to
// add and candidate i (in index order) at x_i, the zeros below x_i number x_i - off - i;
// the P candidates for which that is < z lie inside the leading run [off, off + z + P),
// which is sent whole (z zeros and P candidates); the other candidates follow.
template <int OP, class Src>
__device__ __forceinline__ void zero_fill_emit(const Src src, const uint32_t c, const TensorDesc &td,
                                               const PlanEntry &pe, const SelectArgs &A, uint32_t *wsum)
{
    const uint32_t tid = threadIdx.x;
    const uint32_t z = pe.k - c;
    uint32_t mine = 0;
    for (uint32_t p = tid; p < c; p += SEL_THREADS) mine += ((src.index(p) - td.off - p) < z) ? 1u : 0u;
    const uint32_t P = block_sum(mine, wsum, SEL_WAVES);
    const uint32_t X = z + P;
    for (uint32_t q = tid; q < X; q += SEL_THREADS) {
        const uint32_t ix = td.off + q;
        const float v = row_value<OP>(A.state, A.model, ix);
        A.out_idx[pe.outoff + q] = ix;
        A.out_val[pe.outoff + q] = v;
        fix_sent<OP>(A.state, ix, v, A.m);
    }
    for (uint32_t p = P + tid; p < c; p += SEL_THREADS) {
        const uint32_t ix = src.index(p);
        const float v = __uint_as_float(src.bits(p));
        A.out_idx[pe.outoff + z + p] = ix;
        A.out_val[pe.outoff + z + p] = v;
        if (index_ok(A, ix)) fix_sent<OP>(A.state, ix, v, A.m);
    }
}

// Minimum over the 64 lanes of a wavefront (DPP, same pattern as the scan);
// the result is valid in lane 63.
__device__ __forceinline__ uint32_t wave_min_to_last(uint32_t v)
{
    int x = (int)v;
    const int id = (int)0xFFFFFFFFu;
#define DGS_MIN_STEP(ctrl, rmask)                                                             \
    x = (int)min((uint32_t)x, (uint32_t)__builtin_amdgcn_update_dpp(id, x, ctrl, rmask, 0xf, false))
    DGS_MIN_STEP(0x111, 0xf);
    DGS_MIN_STEP(0x112, 0xf);
    DGS_MIN_STEP(0x114, 0xf);
    DGS_MIN_STEP(0x118, 0xf);
    DGS_MIN_STEP(0x142, 0xa);
    DGS_MIN_STEP(0x143, 0xc);
#undef DGS_MIN_STEP
    return (uint32_t)x;
}

// Ordered-list entry: LDS while it fits, global scratch beyond (an ordinary cached store: the
// list is read back by this workgroup; see release_dev() for the one case where another
// workgroup writes to the same place later in the launch).
__device__ __forceinline__ void put_entry(uint2 *llist, uint2 *glist, uint32_t pos, uint2 e)
{
    if (pos < SEL_LDS_LIST) {
        llist[pos] = e;
    } else {
        glist[pos] = e;
        // keeps the two stores apart: merged into one store through a generic pointer they
        // would take the slow flat path into LDS
        asm volatile("" ::: "memory");
    }
}

}  // namespace dgs
