// gfx950 (CDNA4, wave64) kernels of libdgs.
//
// Streaming pass  : one wavefront per 1024-element tile, 16-byte loads, fused
//                   accumulate (Algorithm 3, "u <- m u + eta grad") + magnitude key +
//                   either candidate collection against a per-tensor threshold or
//                   a 12-bit LDS histogram of the keys.
// Pick            : per tensor, histogram -> threshold bucket.
// Select          : per tensor, one workgroup: exact k-th key by 3 radix passes
//                   (11+10+10 bits) over the ordered candidates (or over the tensor
//                   itself), then ordered emission ("encode()" of Algorithm 1-3)
//                   and the state fix-up of Eq. 12.
// Push / apply    : atomic-free sparse scatter (Algorithm 2, "M <- M - decode(g)").
#include <hip/hip_runtime.h>
#include "dgs_device.h"

namespace dgs {

typedef float f32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ uint32_t lane_id() { return threadIdx.x & 63u; }

__device__ __forceinline__ uint32_t mbcnt64(uint64_t mask)
{
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32),
                                     __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
}

__device__ __forceinline__ uint64_t ballot64(bool p) { return __builtin_amdgcn_ballot_w64(p); }

__device__ __forceinline__ uint32_t uniform(uint32_t v) { return __builtin_amdgcn_readfirstlane(v); }

// ---------------------------------------------------------------------------
// streaming pass
// ---------------------------------------------------------------------------

template <int MODE>
__device__ __forceinline__ void flush_hist(uint32_t *lhist, uint32_t *ghist, int cur)
{
    if (MODE != MODE_HIST) return;
    __syncthreads();
    if (cur >= 0) {
        for (uint32_t b = threadIdx.x; b < HBINS; b += STREAM_THREADS) {
            uint32_t v = lhist[b];
            if (v) {
                atomicAdd(&ghist[(size_t)cur * HBINS + b], v);
                lhist[b] = 0;
            }
        }
    }
    __syncthreads();
}

template <int OP, int MODE, bool VEC>
__device__ __forceinline__ void process_tile(const StreamArgs &A, uint32_t t, uint32_t *lhist, int cur)
{
    const uint32_t lane = lane_id();
    const uint32_t base = t * TILE;
    const bool full = (base + TILE <= A.n);

    float a[4][4];
    if (VEC && full) {
        f32x4 s[4];
        if (OP == OP_FMA) {
            f32x4 g[4];
#pragma unroll
            for (int r = 0; r < 4; ++r)
                g[r] = __builtin_nontemporal_load((const f32x4 *)(A.grad + base + r * 256 + lane * 4));
#pragma unroll
            for (int r = 0; r < 4; ++r)
                s[r] = *(const f32x4 *)(A.state + base + r * 256 + lane * 4);
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                f32x4 o;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    a[r][j] = __builtin_fmaf(A.lr, g[r][j], s[r][j]);
                    o[j] = a[r][j];
                }
                *(f32x4 *)(A.state + base + r * 256 + lane * 4) = o;
            }
        } else {
#pragma unroll
            for (int r = 0; r < 4; ++r)
                s[r] = *(const f32x4 *)(A.state + base + r * 256 + lane * 4);
#pragma unroll
            for (int r = 0; r < 4; ++r)
#pragma unroll
                for (int j = 0; j < 4; ++j) a[r][j] = s[r][j];
        }
    } else {
#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const uint32_t e = base + r * 256 + lane * 4 + j;
                float v = 0.0f;
                if (e < A.n) {
                    if (OP == OP_FMA) {
                        v = __builtin_fmaf(A.lr, A.grad[e], A.state[e]);
                        A.state[e] = v;
                    } else {
                        v = A.state[e];
                    }
                }
                a[r][j] = v;
            }
    }
    if (MODE == MODE_PLAIN) return;

    // which tensors does this tile touch?
    const uint2 d = A.tile_desc[t];
    const uint32_t tA = uniform(d.x), tB = uniform(d.y);
    const bool straddle = (tA != tB);
    const TensorDesc dA = A.tdesc[tA];
    const uint32_t endA = uniform(dA.off + dA.n);
    uint32_t begB = 0xFFFFFFFFu;
    uint32_t bigB = 0;
    if (straddle) {
        const TensorDesc dB = A.tdesc[tB];
        begB = uniform(dB.off);
        bigB = uniform(dB.big);
    }
    const uint32_t bigA = uniform(dA.big);

    if (MODE == MODE_COLLECT) {
        const uint32_t tauA = uniform(A.tau[tA]);
        const uint32_t tauB = straddle ? uniform(A.tau[tB]) : TAU_NEVER;
        uint2 *myslots = A.slots + (size_t)t * CAPT;
        uint32_t run = 0, runA = 0;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const uint32_t e0 = base + r * 256 + lane * 4;
            bool f[4];
            uint64_t mk[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const uint32_t e = e0 + j;
                const uint32_t key = __float_as_uint(a[r][j]) & 0x7FFFFFFFu;
                uint32_t thr = tauA;
                if (straddle) thr = (e < endA) ? tauA : ((e >= begB) ? tauB : TAU_NEVER);
                f[j] = (key >= thr) && (full || e < A.n);
                mk[j] = ballot64(f[j]);
            }
            const uint64_t any = mk[0] | mk[1] | mk[2] | mk[3];
            if (any != 0) {
                uint32_t p = run + mbcnt64(mk[0]) + mbcnt64(mk[1]) + mbcnt64(mk[2]) + mbcnt64(mk[3]);
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    if (f[j]) {
                        if (p < CAPT) myslots[p] = make_uint2(e0 + j, __float_as_uint(a[r][j]));
                        ++p;
                    }
                }
                run += (uint32_t)(__popcll(mk[0]) + __popcll(mk[1]) + __popcll(mk[2]) + __popcll(mk[3]));
                if (straddle) {
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        runA += (uint32_t)__popcll(ballot64(f[j] && (e0 + j < endA)));
                }
            }
        }
        if (!straddle) runA = run;
        if (lane == 0)
            A.tile_cnt[t] = (run > CAPT) ? CNT_OVERFLOW : (runA | ((run - runA) << 16));
    } else {  // MODE_HIST
#pragma unroll
        for (int r = 0; r < 4; ++r) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const uint32_t e = base + r * 256 + lane * 4 + j;
                if (!(full || e < A.n)) continue;
                int tt = -1;
                if (e < endA) {
                    if (bigA) tt = (int)tA;
                } else if (e >= begB) {
                    if (bigB) tt = (int)tB;
                }
                if (tt < 0) continue;
                const uint32_t bin = (__float_as_uint(a[r][j]) & 0x7FFFFFFFu) >> HSHIFT;
                if (tt == cur) atomicAdd(&lhist[bin], 1u);
                else atomicAdd(&A.ghist[(size_t)tt * HBINS + bin], 1u);
            }
        }
    }
}

template <int OP, int MODE, bool VEC>
__global__ __launch_bounds__(STREAM_THREADS) void k_stream(const StreamArgs A)
{
    __shared__ uint32_t lhist[MODE == MODE_HIST ? HBINS : 1];
    const uint32_t wave = threadIdx.x >> 6;
    const uint32_t q0 = blockIdx.x * A.quads_per_block;
    const uint32_t q1 = min(q0 + A.quads_per_block, A.nquads);
    int cur = -1;
    if (MODE == MODE_HIST) {
        for (uint32_t b = threadIdx.x; b < HBINS; b += STREAM_THREADS) lhist[b] = 0;
        __syncthreads();
    }
    for (uint32_t q = q0; q < q1; ++q) {
        if (MODE == MODE_HIST) {
            // the LDS histogram belongs to the big tensor the quad starts in
            const uint32_t ft = A.tile_desc[q * WAVES_PER_BLOCK].x;
            const int qt = A.tdesc[ft].big ? (int)ft : -1;
            if (qt != cur) {
                flush_hist<MODE>(lhist, A.ghist, cur);
                cur = qt;
            }
        }
        const uint32_t t = q * WAVES_PER_BLOCK + wave;
        if (t < A.ntiles) process_tile<OP, MODE, VEC>(A, t, lhist, cur);
    }
    flush_hist<MODE>(lhist, A.ghist, cur);
}

template <int OP, int MODE>
static void launch_stream_t(bool vec, const StreamArgs &a, uint32_t blocks, hipStream_t st)
{
    if (vec) hipLaunchKernelGGL((k_stream<OP, MODE, true>), dim3(blocks), dim3(STREAM_THREADS), 0, st, a);
    else hipLaunchKernelGGL((k_stream<OP, MODE, false>), dim3(blocks), dim3(STREAM_THREADS), 0, st, a);
}

void launch_stream(int op, int mode, bool vec, const StreamArgs &a, uint32_t blocks, void *stream)
{
    hipStream_t st = (hipStream_t)stream;
    if (blocks == 0) return;
    if (op == OP_FMA) {
        if (mode == MODE_PLAIN) launch_stream_t<OP_FMA, MODE_PLAIN>(vec, a, blocks, st);
        else if (mode == MODE_COLLECT) launch_stream_t<OP_FMA, MODE_COLLECT>(vec, a, blocks, st);
        else launch_stream_t<OP_FMA, MODE_HIST>(vec, a, blocks, st);
    } else {
        if (mode == MODE_COLLECT) launch_stream_t<OP_IDENT, MODE_COLLECT>(vec, a, blocks, st);
        else if (mode == MODE_HIST) launch_stream_t<OP_IDENT, MODE_HIST>(vec, a, blocks, st);
    }
}

// ---------------------------------------------------------------------------
// workgroup helpers for pick / select (SEL_THREADS threads unless stated)
// ---------------------------------------------------------------------------

__device__ __forceinline__ uint32_t wave_incl_scan(uint32_t v)
{
    const uint32_t lane = lane_id();
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        uint32_t t = __shfl_up(v, d, 64);
        if (lane >= (uint32_t)d) v += t;
    }
    return v;
}

// Exclusive scan over the workgroup in thread order; `total` is the workgroup sum.
// wsum: LDS scratch of NW words.  Contains two barriers.
template <int NW>
__device__ __forceinline__ uint32_t block_excl_scan(uint32_t v, uint32_t *wsum, uint32_t &total)
{
    const uint32_t wave = threadIdx.x >> 6;
    const uint32_t incl = wave_incl_scan(v);
    __syncthreads();
    if (lane_id() == 63) wsum[wave] = incl;
    __syncthreads();
    uint32_t before = 0, tot = 0;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
        const uint32_t x = wsum[w];
        if ((uint32_t)w < wave) before += x;
        tot += x;
    }
    total = tot;
    return before + incl - v;
}

// In an LDS histogram h[NB] (NB = NT * BPT), find the bucket holding the key of
// rank R counted from the top (R >= 1), and the rank inside that bucket.
// res[0] = bucket (or -1 if R exceeds the histogram total), res[1] = rank inside.
template <int NB, int NT, int NW>
__device__ __forceinline__ void find_rank(const uint32_t *h, uint32_t R, uint32_t *wsum, int *res)
{
    constexpr int BPT = NB / NT;
    static_assert(BPT * NT == NB, "bins must divide evenly");
    const int hi = NB - 1 - (int)threadIdx.x * BPT;   // thread 0 owns the top bins
    uint32_t sum = 0;
#pragma unroll
    for (int i = 0; i < BPT; ++i) sum += h[hi - i];
    if (threadIdx.x == 0) { res[0] = -1; res[1] = 0; }
    uint32_t total;
    const uint32_t excl = block_excl_scan<NW>(sum, wsum, total);   // keys in higher bins
    if (excl < R && R <= excl + sum) {
        uint32_t acc = excl;
#pragma unroll
        for (int i = 0; i < BPT; ++i) {
            const uint32_t c = h[hi - i];
            if (acc + c >= R) { res[0] = hi - i; res[1] = (int)(R - acc); break; }
            acc += c;
        }
    }
    __syncthreads();
}

// ---------------------------------------------------------------------------
// pick: streaming-pass histogram -> candidate threshold (non-predicted path)
// ---------------------------------------------------------------------------

__global__ __launch_bounds__(256) void k_pick(const TensorDesc *tdesc, const PlanEntry *plan,
                                              uint32_t *ghist, uint32_t *tau, DevStats *stats)
{
    const uint32_t j = blockIdx.x;
    if (!tdesc[j].big) return;
    __shared__ uint32_t h[HBINS];
    __shared__ uint32_t wsum[4];
    __shared__ int res[2];
    uint32_t *g = ghist + (size_t)j * HBINS;
    for (uint32_t b = threadIdx.x; b < HBINS; b += 256) {
        h[b] = g[b];
        g[b] = 0;   // leave the histogram clean for the next use
    }
    __syncthreads();
    const PlanEntry pe = plan[j];
    find_rank<HBINS, 256, 4>(h, pe.k2, wsum, res);
    int b2 = res[0];
    __syncthreads();
    find_rank<HBINS, 256, 4>(h, pe.k, wsum, res);
    int b1 = res[0];
    if (threadIdx.x == 0) {
        uint32_t t;
        if (b2 < 0 || b1 < 0) {
            atomicAdd(&stats->internal_errors, 1ull);
            t = 1;
        } else if (b2 > 0) {
            t = (uint32_t)b2 << HSHIFT;
        } else if (b1 > 0) {
            t = 1u << HSHIFT;
        } else {
            t = 1;   // the k-th key is tiny or zero: collect every nonzero
        }
        tau[j] = t;
    }
}

void launch_pick(const TensorDesc *tdesc, const PlanEntry *plan, uint32_t *ghist, uint32_t *tau,
                 DevStats *stats, uint32_t J, void *stream)
{
    hipLaunchKernelGGL(k_pick, dim3(J), dim3(256), 0, (hipStream_t)stream, tdesc, plan, ghist, tau, stats);
}

// ---------------------------------------------------------------------------
// select
// ---------------------------------------------------------------------------

struct SrcDense {          // the tensor itself: position p <-> element off + p
    const float *base;
    uint32_t off;
    __device__ __forceinline__ uint32_t bits(uint32_t p) const { return __float_as_uint(base[off + p]); }
    __device__ __forceinline__ uint32_t index(uint32_t p) const { return off + p; }
};

struct SrcList {           // ordered candidates (index, value bits)
    const uint2 *list;
    __device__ __forceinline__ uint32_t bits(uint32_t p) const { return list[p].y; }
    __device__ __forceinline__ uint32_t index(uint32_t p) const { return list[p].x; }
};

struct SelShared {
    uint32_t h[2048];
    uint32_t wsum[SEL_WAVES];
    int res[2];
    uint32_t bcast[4];
};

// Exact selection over `cN` ordered entries of `src`; emits the k winners in
// order, applies the state fix-up, returns the next threshold hint through
// *tau_next (0 if rank k2 was not measurable).
template <int OP, int ITEMS, class Src>
__device__ __forceinline__ void select_emit(const Src src, const uint32_t cN, const uint32_t k,
                                            const uint32_t k2, SelShared &S, const SelectArgs &A,
                                            const uint32_t outoff, uint32_t *tau_next)
{
    const uint32_t tid = threadIdx.x;
    const bool measurable = (cN >= k2);

    // ---- pass 1: key bits [30:20]
    for (uint32_t b = tid; b < 2048; b += SEL_THREADS) S.h[b] = 0;
    __syncthreads();
    {
        uint32_t p = tid;
        for (; p + 3 * SEL_THREADS < cN; p += 4 * SEL_THREADS) {
            uint32_t k0 = src.bits(p), k1 = src.bits(p + SEL_THREADS), k2_ = src.bits(p + 2 * SEL_THREADS),
                     k3 = src.bits(p + 3 * SEL_THREADS);
            atomicAdd(&S.h[(k0 & 0x7FFFFFFFu) >> 20], 1u);
            atomicAdd(&S.h[(k1 & 0x7FFFFFFFu) >> 20], 1u);
            atomicAdd(&S.h[(k2_ & 0x7FFFFFFFu) >> 20], 1u);
            atomicAdd(&S.h[(k3 & 0x7FFFFFFFu) >> 20], 1u);
        }
        for (; p < cN; p += SEL_THREADS) atomicAdd(&S.h[(src.bits(p) & 0x7FFFFFFFu) >> 20], 1u);
    }
    __syncthreads();
    find_rank<2048, SEL_THREADS, SEL_WAVES>(S.h, k, S.wsum, S.res);
    const int b1 = S.res[0];
    const uint32_t r1 = (uint32_t)S.res[1];
    __syncthreads();
    int c1 = b1;
    uint32_t q1 = 0;
    if (measurable) {
        find_rank<2048, SEL_THREADS, SEL_WAVES>(S.h, k2, S.wsum, S.res);
        c1 = S.res[0];
        q1 = (uint32_t)S.res[1];
        __syncthreads();
    }
    if (b1 < 0 || c1 < 0) {   // cannot happen for cN >= k
        if (tid == 0) atomicAdd(&A.stats->internal_errors, 1ull);
        *tau_next = 0;
        return;
    }

    // ---- pass 2: key bits [19:10] inside bucket b1 (and inside c1 for the hint)
    for (uint32_t b = tid; b < 2048; b += SEL_THREADS) S.h[b] = 0;
    __syncthreads();
    {
        const bool two = measurable && (c1 != b1);
        uint32_t p = tid;
        for (; p + 3 * SEL_THREADS < cN; p += 4 * SEL_THREADS) {
            uint32_t kk[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) kk[i] = src.bits(p + i * SEL_THREADS) & 0x7FFFFFFFu;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int top = (int)(kk[i] >> 20);
                if (top == b1) atomicAdd(&S.h[(kk[i] >> 10) & 1023u], 1u);
                else if (two && top == c1) atomicAdd(&S.h[1024u + ((kk[i] >> 10) & 1023u)], 1u);
            }
        }
        for (; p < cN; p += SEL_THREADS) {
            const uint32_t key = src.bits(p) & 0x7FFFFFFFu;
            const int top = (int)(key >> 20);
            if (top == b1) atomicAdd(&S.h[(key >> 10) & 1023u], 1u);
            else if (two && top == c1) atomicAdd(&S.h[1024u + ((key >> 10) & 1023u)], 1u);
        }
    }
    __syncthreads();
    find_rank<1024, SEL_THREADS, SEL_WAVES>(S.h, r1, S.wsum, S.res);
    const int b2 = S.res[0];
    const uint32_t r2 = (uint32_t)S.res[1];
    __syncthreads();
    uint32_t hint = 0;
    if (measurable) {
        find_rank<1024, SEL_THREADS, SEL_WAVES>(S.h + ((c1 != b1) ? 1024 : 0), q1, S.wsum, S.res);
        const int c2 = S.res[0];
        __syncthreads();
        if (c2 >= 0) hint = ((uint32_t)c1 << 20) | ((uint32_t)c2 << 10);
        if (hint == 0) hint = 1;
    }
    *tau_next = hint;
    if (b2 < 0) {
        if (tid == 0) atomicAdd(&A.stats->internal_errors, 1ull);
        return;
    }

    // ---- pass 3: key bits [9:0] inside (b1, b2)
    const uint32_t pfx = ((uint32_t)b1 << 10) | (uint32_t)b2;
    for (uint32_t b = tid; b < 1024; b += SEL_THREADS) S.h[b] = 0;
    __syncthreads();
    {
        uint32_t p = tid;
        for (; p + 3 * SEL_THREADS < cN; p += 4 * SEL_THREADS) {
            uint32_t kk[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) kk[i] = src.bits(p + i * SEL_THREADS) & 0x7FFFFFFFu;
#pragma unroll
            for (int i = 0; i < 4; ++i)
                if ((kk[i] >> 10) == pfx) atomicAdd(&S.h[kk[i] & 1023u], 1u);
        }
        for (; p < cN; p += SEL_THREADS) {
            const uint32_t key = src.bits(p) & 0x7FFFFFFFu;
            if ((key >> 10) == pfx) atomicAdd(&S.h[key & 1023u], 1u);
        }
    }
    __syncthreads();
    find_rank<1024, SEL_THREADS, SEL_WAVES>(S.h, r2, S.wsum, S.res);
    const int b3 = S.res[0];
    const uint32_t rT = (uint32_t)S.res[1];   // how many entries equal to T are taken (lowest index first)
    __syncthreads();
    if (b3 < 0) {
        if (tid == 0) atomicAdd(&A.stats->internal_errors, 1ull);
        return;
    }
    const uint32_t T = (pfx << 10) | (uint32_t)b3;

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
#pragma unroll
            for (int i = 0; i < ITEMS; ++i) {
                const uint32_t p = p0 + i;
                if (p >= cN) break;
                const uint32_t key = vb[i] & 0x7FFFFFFFu;
                bool sel = key > T;
                if (key == T) {
                    sel = eq_seen < rem;
                    ++eq_seen;
                }
                if (sel) {
                    const uint32_t ix = src.index(p);
                    if (pos < k) {
                        A.out_idx[outoff + pos] = ix;
                        A.out_val[outoff + pos] = __uint_as_float(vb[i]);
                        A.state[ix] = (OP == SEL_WORKER) ? (A.m * __uint_as_float(vb[i])) : 0.0f;
                    }
                    ++pos;
                }
            }
        }
        run_sel += G + min(Q, rem);
        run_eq += Q;
    }
    if (run_sel != k && tid == 0) atomicAdd(&A.stats->internal_errors, 1ull);
}

template <int OP>
__global__ __launch_bounds__(SEL_THREADS) void k_select(const SelectArgs A)
{
    __shared__ SelShared S;
    __shared__ uint2 llist[SEL_LDS_LIST];
    const uint32_t j = blockIdx.x;
    const uint32_t tid = threadIdx.x;
    const TensorDesc td = A.tdesc[j];
    const PlanEntry pe = A.plan[j];
    const uint32_t tlo = td.off / TILE;
    const uint32_t thi = (td.off + td.n - 1) / TILE;
    const bool head_shared = (td.off % TILE) != 0;   // first tile starts inside an earlier tensor
    bool dense = (!td.big) || A.force_dense;
    uint32_t c = 0;
    uint32_t tau_next = 0;
    const uint32_t tau_cur = td.big ? A.tau[j] : TAU_NEVER;

    const uint32_t ntl = thi - tlo + 1;
    const uint32_t per = (ntl + SEL_THREADS - 1) / SEL_THREADS;
    const uint32_t my_lo = min(tlo + tid * per, thi + 1);
    const uint32_t my_hi = min(my_lo + per, thi + 1);

    if (!dense) {
        // candidates of this tensor, tile by tile
        uint32_t mine = 0, ovf = 0;
        for (uint32_t t = my_lo; t < my_hi; ++t) {
            const uint32_t w = A.tile_cnt[t];
            if (w == CNT_OVERFLOW) ovf = 1;
            else mine += (t == tlo && head_shared) ? (w >> 16) : (w & 0xFFFFu);
        }
        uint32_t total;
        const uint32_t before = block_excl_scan<SEL_WAVES>(mine, S.wsum, total);
        const uint32_t any_ovf = __syncthreads_or((int)ovf);
        c = total;   // < 2^30: n < 2^32 and at most a quarter of a tile are candidates
        if (any_ovf || c < pe.k) {
            dense = true;
            if (tid == 0) {
                atomicAdd(&A.stats->fallback_tensors, 1ull);
                atomicAdd(&A.stats->fallback_elems, (unsigned long long)td.n);
            }
        } else {
            // gather into index order
            uint2 *dst = (c <= SEL_LDS_LIST) ? llist : (A.ord + (size_t)(tlo + j) * CAPT);
            uint32_t pos = before;
            for (uint32_t t = my_lo; t < my_hi; ++t) {
                const uint32_t w = A.tile_cnt[t];
                const bool hs = (t == tlo && head_shared);
                const uint32_t cnt = hs ? (w >> 16) : (w & 0xFFFFu);
                const uint32_t start = hs ? (w & 0xFFFFu) : 0u;
                const uint2 *sl = A.slots + (size_t)t * CAPT + start;
                for (uint32_t i = 0; i < cnt; ++i) dst[pos + i] = sl[i];
                pos += cnt;
            }
            if (tid == 0) atomicAdd(&A.stats->candidates, (unsigned long long)c);
            __threadfence_block();
            __syncthreads();
        }
    }

    if (dense) {
        SrcDense src{A.state, td.off};
        select_emit<OP, 8>(src, td.n, pe.k, pe.k2, S, A, pe.outoff, &tau_next);
    } else if (c <= SEL_LDS_LIST) {
        SrcList src{llist};
        select_emit<OP, 4>(src, c, pe.k, pe.k2, S, A, pe.outoff, &tau_next);
    } else {
        SrcList src{A.ord + (size_t)(tlo + j) * CAPT};
        select_emit<OP, 8>(src, c, pe.k, pe.k2, S, A, pe.outoff, &tau_next);
    }

    if (td.big && A.write_hint && tid == 0) {
        uint32_t t = tau_next;
        if (t == 0) {
            // rank k2 was not among the candidates: relax the current threshold by a quarter
            float f = __uint_as_float(tau_cur & 0x7FFFFFFFu) * 0.75f;
            t = __float_as_uint(f) & 0x7FFFFFFFu;
            if (!(tau_cur > 1u) || t == 0) t = 1;
        }
        if (t >= 0x7F800000u) t = 0x7F7FFFFFu;   // keep the hint finite
        A.tau[j] = t;
    }
}

void launch_select(int op, const SelectArgs &a, uint32_t J, void *stream)
{
    hipStream_t st = (hipStream_t)stream;
    if (op == SEL_WORKER) hipLaunchKernelGGL(k_select<SEL_WORKER>, dim3(J), dim3(SEL_THREADS), 0, st, a);
    else hipLaunchKernelGGL(k_select<SEL_PULL>, dim3(J), dim3(SEL_THREADS), 0, st, a);
}

// ---------------------------------------------------------------------------
// sparse scatter: push, apply, validation
// ---------------------------------------------------------------------------

// blockIdx.y selects the destination buffer (model first, then the difference
// rows), so a wavefront walks ascending indices of one buffer.  Indices are
// unique within a message, and calls are ordered on one stream: no atomics.
__global__ __launch_bounds__(256) void k_push(float *model, float *diff, uint32_t n,
                                              const uint32_t *idx, const float *val, uint32_t nnz,
                                              uint32_t first_buf)
{
    const uint32_t e = blockIdx.x * 256 + threadIdx.x;
    if (e >= nnz) return;
    const uint32_t b = blockIdx.y + first_buf;
    float *dst = (b == 0) ? model : diff + (size_t)(b - 1) * n;
    const uint32_t i = idx[e];
    if (i < n) dst[i] = dst[i] - val[e];
}

void launch_push(float *model, float *diff, uint32_t W, uint32_t n, const uint32_t *idx,
                 const float *val, uint32_t nnz, void *stream)
{
    if (nnz == 0) return;
    const uint32_t first = model ? 0u : 1u;
    const uint32_t bufs = W + 1 - first;
    if (bufs == 0) return;
    // gridDim.y is limited to 65535: loop over slabs of buffers
    for (uint32_t b0 = 0; b0 < bufs; b0 += 32768) {
        const uint32_t nb = (bufs - b0 < 32768u) ? (bufs - b0) : 32768u;
        hipLaunchKernelGGL(k_push, dim3((nnz + 255) / 256, nb), dim3(256), 0, (hipStream_t)stream,
                           model, diff, n, idx, val, nnz, first + b0);
    }
}

__global__ __launch_bounds__(256) void k_validate_idx(const uint32_t *idx, uint32_t nnz, uint32_t n,
                                                      uint32_t *flag)
{
    const uint32_t e = blockIdx.x * 256 + threadIdx.x;
    if (e >= nnz) return;
    const uint32_t i = idx[e];
    bool bad = (i >= n);
    if (e > 0 && idx[e - 1] >= i) bad = true;
    if (bad) atomicOr(flag, 1u);
}

void launch_validate_idx(const uint32_t *idx, uint32_t nnz, uint32_t n, uint32_t *flag, void *stream)
{
    if (nnz == 0) return;
    hipLaunchKernelGGL(k_validate_idx, dim3((nnz + 255) / 256), dim3(256), 0, (hipStream_t)stream,
                       idx, nnz, n, flag);
}

__global__ __launch_bounds__(256) void k_apply(float *dst, const uint32_t *idx, const float *val,
                                               uint32_t nnz, float sign)
{
    const uint32_t e = blockIdx.x * 256 + threadIdx.x;
    if (e >= nnz) return;
    const uint32_t i = idx[e];
    dst[i] = __builtin_fmaf(sign, val[e], dst[i]);
}

void launch_apply(float *dst, const uint32_t *idx, const float *val, uint32_t nnz, float sign,
                  void *stream)
{
    if (nnz == 0) return;
    hipLaunchKernelGGL(k_apply, dim3((nnz + 255) / 256), dim3(256), 0, (hipStream_t)stream, dst, idx,
                       val, nnz, sign);
}

__global__ __launch_bounds__(256) void k_fill_u32(uint32_t *p, uint32_t v, size_t count)
{
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * 256;
    for (; i < count; i += stride) p[i] = v;
}

void launch_fill_u32(uint32_t *p, uint32_t v, size_t count, void *stream)
{
    if (count == 0) return;
    size_t blocks = (count + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(k_fill_u32, dim3((uint32_t)blocks), dim3(256), 0, (hipStream_t)stream, p, v, count);
}

// ---------------------------------------------------------------------------
// pull without secondary compression: every nonzero of one difference row
// ---------------------------------------------------------------------------

__device__ __forceinline__ void load_tile_guarded(const float *row, uint32_t base, uint32_t n,
                                                  float (&a)[4][4])
{
    const uint32_t lane = lane_id();
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint32_t e = base + r * 256 + lane * 4 + j;
            a[r][j] = (e < n) ? row[e] : 0.0f;
        }
}

__global__ __launch_bounds__(STREAM_THREADS) void k_pull_all_count(const float *row, uint32_t n,
                                                                   uint32_t ntiles, uint32_t *tile_cnt)
{
    const uint32_t t = blockIdx.x * WAVES_PER_BLOCK + (threadIdx.x >> 6);
    if (t >= ntiles) return;
    float a[4][4];
    load_tile_guarded(row, t * TILE, n, a);
    uint32_t cnt = 0;
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int j = 0; j < 4; ++j)
            cnt += (uint32_t)__popcll(ballot64((__float_as_uint(a[r][j]) & 0x7FFFFFFFu) != 0));
    if (lane_id() == 0) tile_cnt[t] = cnt;
}

// single workgroup: in-place exclusive scan of tile_cnt, total to *total
__global__ __launch_bounds__(1024) void k_pull_all_scan(uint32_t *tile_cnt, uint32_t ntiles, uint32_t *total)
{
    __shared__ uint32_t wsum[16];
    const uint32_t per = (ntiles + 1023) / 1024;
    const uint32_t lo = min(threadIdx.x * per, ntiles), hi = min(lo + per, ntiles);
    uint32_t sum = 0;
    for (uint32_t t = lo; t < hi; ++t) sum += tile_cnt[t];
    uint32_t tot;
    uint32_t pos = block_excl_scan<16>(sum, wsum, tot);
    for (uint32_t t = lo; t < hi; ++t) {
        const uint32_t c = tile_cnt[t];
        tile_cnt[t] = pos;
        pos += c;
    }
    if (threadIdx.x == 0) *total = tot;
}

__global__ __launch_bounds__(STREAM_THREADS) void k_pull_all_emit(float *row, uint32_t n, uint32_t ntiles,
                                                                  const uint32_t *tile_pos,
                                                                  uint32_t *out_idx, float *out_val)
{
    const uint32_t t = blockIdx.x * WAVES_PER_BLOCK + (threadIdx.x >> 6);
    if (t >= ntiles) return;
    const uint32_t lane = lane_id();
    const uint32_t base = t * TILE;
    float a[4][4];
    load_tile_guarded(row, base, n, a);
    uint32_t run = tile_pos[t];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        bool f[4];
        uint64_t mk[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            f[j] = (__float_as_uint(a[r][j]) & 0x7FFFFFFFu) != 0;
            mk[j] = ballot64(f[j]);
        }
        if ((mk[0] | mk[1] | mk[2] | mk[3]) != 0) {
            uint32_t p = run + mbcnt64(mk[0]) + mbcnt64(mk[1]) + mbcnt64(mk[2]) + mbcnt64(mk[3]);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if (f[j]) {
                    const uint32_t e = base + r * 256 + lane * 4 + j;
                    out_idx[p] = e;
                    out_val[p] = a[r][j];
                    row[e] = 0.0f;
                    ++p;
                }
            }
            run += (uint32_t)(__popcll(mk[0]) + __popcll(mk[1]) + __popcll(mk[2]) + __popcll(mk[3]));
        }
    }
}

void launch_pull_all_count(const float *row, uint32_t n, uint32_t ntiles, uint32_t *tile_cnt, void *stream)
{
    hipLaunchKernelGGL(k_pull_all_count, dim3((ntiles + WAVES_PER_BLOCK - 1) / WAVES_PER_BLOCK),
                       dim3(STREAM_THREADS), 0, (hipStream_t)stream, row, n, ntiles, tile_cnt);
}

void launch_pull_all_scan(uint32_t *tile_cnt, uint32_t ntiles, uint32_t *total, void *stream)
{
    hipLaunchKernelGGL(k_pull_all_scan, dim3(1), dim3(1024), 0, (hipStream_t)stream, tile_cnt, ntiles, total);
}

void launch_pull_all_emit(float *row, uint32_t n, uint32_t ntiles, const uint32_t *tile_pos,
                          uint32_t *out_idx, float *out_val, void *stream)
{
    hipLaunchKernelGGL(k_pull_all_emit, dim3((ntiles + WAVES_PER_BLOCK - 1) / WAVES_PER_BLOCK),
                       dim3(STREAM_THREADS), 0, (hipStream_t)stream, row, n, ntiles, tile_pos, out_idx,
                       out_val);
}

}  // namespace dgs
