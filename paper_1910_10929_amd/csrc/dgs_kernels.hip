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
#include <hip/hip_ext.h>
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

// Isolated 4-byte store into a large buffer that a later streaming pass will sweep
// (state fix-ups, pull zero-writes, the push scatter).  Non-temporal: plain stores
// leave partially written lines behind in the cache hierarchy, and 1e5 of them were
// measured to slow the NEXT streaming pass over a 4 GB buffer by 130 us (6 %);
// non-temporal ones by 15 us.
__device__ __forceinline__ void store_scattered(float *p, float v) { __builtin_nontemporal_store(v, p); }

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

// Which tensors does a span [first, last] of the flat buffer touch?  Binary search
// in the tensor offsets (uniform addresses: scalar loads that stay in the scalar
// cache), so that no per-tile table has to be fetched from HBM.
//   x = tensor of `first` (bit 31: that tensor is big), y = tensor of `last` (bit 31: big),
//   z = end of the leading tensor part (0xFFFFFFFF when the span lies inside one tensor),
//   w = begin of the trailing tensor part (0xFFFFFFFF when there is none)
__device__ __forceinline__ uint32_t find_tensor(const uint32_t *__restrict__ toff, uint32_t lo,
                                                uint32_t hi, uint32_t e)
{
    // largest j in [lo, hi) with toff[j] <= e
    while (hi - lo > 1) {
        const uint32_t mid = (lo + hi) >> 1;
        if (toff[mid] <= e) lo = mid;
        else hi = mid;
    }
    return lo;
}

__device__ __forceinline__ uint4 span_desc(const uint32_t *__restrict__ toff, uint32_t J,
                                           uint32_t first, uint32_t last)
{
    const uint32_t tA = find_tensor(toff, 0, J, first);
    const uint32_t offA = toff[tA], endA = toff[tA + 1];
    uint4 d;
    d.x = tA | ((endA - offA > SMALL_N) ? 0x80000000u : 0u);
    if (last < endA) {
        d.y = d.x;
        d.z = 0xFFFFFFFFu;
        d.w = 0xFFFFFFFFu;
    } else {
        const uint32_t tB = find_tensor(toff, tA + 1, J, last);
        const uint32_t offB = toff[tB], endB = toff[tB + 1];
        d.y = tB | ((endB - offB > SMALL_N) ? 0x80000000u : 0u);
        d.z = endA;
        d.w = offB;
    }
    return d;
}

// What follows the accumulate for one tile whose 16 values per lane are in `a`:
// candidate collection against the per-tensor thresholds, or the key histogram.
template <int MODE>
__device__ __forceinline__ void tile_tail(const StreamArgs &A, const uint32_t *__restrict__ tau, uint32_t t,
                                          const uint4 d, const float (&a)[4][4], uint32_t *lhist, int cur,
                                          uint2 *stage, int only)
{
    const uint32_t lane = lane_id();
    const uint32_t base = t * TILE;
    const bool full = (base + TILE <= A.n);
    const uint32_t tA = d.x & 0x7FFFFFFFu, tB = d.y & 0x7FFFFFFFu;
    const uint32_t endA = d.z, begB = d.w;
    const bool straddle = (endA != 0xFFFFFFFFu);

    if (MODE == MODE_COLLECT) {
        const uint32_t tauA = tau[tA];
        const uint32_t tauB = (begB != 0xFFFFFFFFu) ? tau[tB] : TAU_NEVER;
        uint2 *myheads = A.heads + (size_t)t * HEAD;
        uint2 *myslots = A.slots + (size_t)t * CAPT;
        uint32_t run = 0, runA = 0;
        const bool simple = full && !straddle;     // wave-uniform: one tensor, no ragged end
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const uint32_t e0 = base + r * 256 + lane * 4;
            bool f[4];
            uint64_t mk[4];
            if (simple) {
                // two VALU operations per element: clear the sign, compare into a lane mask
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    f[j] = (__float_as_uint(a[r][j]) & 0x7FFFFFFFu) >= tauA;
                    mk[j] = ballot64(f[j]);
                }
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const uint32_t e = e0 + j;
                    const uint32_t key = __float_as_uint(a[r][j]) & 0x7FFFFFFFu;
                    uint32_t thr = tauA;
                    if (straddle) thr = (e < endA) ? tauA : ((e >= begB) ? tauB : TAU_NEVER);
                    f[j] = (key >= thr) && (full || e < A.n);
                    mk[j] = ballot64(f[j]);
                }
            }
            const uint64_t any = mk[0] | mk[1] | mk[2] | mk[3];
            if (any != 0) {
                uint32_t p = run + mbcnt64(mk[0]) + mbcnt64(mk[1]) + mbcnt64(mk[2]) + mbcnt64(mk[3]);
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    if (f[j]) {
                        const uint2 ent = make_uint2(e0 + j, __float_as_uint(a[r][j]));
                        if (p < STAGE) stage[p] = ent;
                        else if (p < CAPT) myslots[p] = ent;
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
        // The staged candidates leave as whole 64-byte lines (8 entries; the head line
        // always, also when empty): a full-line store needs no fill from memory, while
        // scattered 8-byte stores into cold lines were measured to cost the pass 15 %.
        __builtin_amdgcn_wave_barrier();
        const uint32_t nst = min(run, STAGE);
        if (lane < HEAD) myheads[lane] = (lane < nst) ? stage[lane] : make_uint2(0u, 0u);
        if (nst > HEAD) {   // wave-uniform and rare: the spill lines of a crowded tile
            const uint32_t nlines = (nst + HEAD - 1u) / HEAD;
            if (lane >= HEAD && lane < nlines * HEAD)
                myslots[lane] = (lane < nst) ? stage[lane] : make_uint2(0u, 0u);
        }
        if (!straddle) runA = run;
        if (lane == 0)
            A.tile_cnt[t] = (run > CAPT) ? CNT_OVERFLOW : (runA | ((run - runA) << 16));
    } else {  // MODE_HIST
        const bool bigA = (d.x >> 31) != 0, bigB = (d.y >> 31) != 0;
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
                if (tt < 0 || (only >= 0 && tt != only)) continue;
                const uint32_t key = __float_as_uint(a[r][j]) & 0x7FFFFFFFu;
                if (key == 0) continue;            // zeros (often the bulk of a difference row) are implied
                const uint32_t bin = key >> HSHIFT;
                if (tt == cur) atomicAdd(&lhist[bin], 1u);
                else atomicAdd(&A.ghist[(size_t)tt * HBINS + bin], 1u);
            }
        }
    }
}

template <int OP, int MODE, bool VEC>
__device__ __forceinline__ void process_tile(const StreamArgs &A, const uint32_t *__restrict__ toff,
                                             const uint32_t *__restrict__ tau, uint32_t t,
                                             uint32_t *lhist, int cur, uint2 *stage, int only = -1)
{
    const uint32_t lane = lane_id();
    const uint32_t base = t * TILE;
    const bool full = (base + TILE <= A.n);
    float a[4][4];
    uint4 d = make_uint4(0, 0, 0xFFFFFFFFu, 0xFFFFFFFFu);

    if (VEC && full) {
        // Issue the tile's vector loads first; the scalar search for the tensors touched by
        // the tile then runs while they are in flight.
        f32x4 g[4], s[4];
        if (OP == OP_FMA) {
#pragma unroll
            for (int r = 0; r < 4; ++r)
                g[r] = __builtin_nontemporal_load((const f32x4 *)(A.grad + base + r * 256 + lane * 4));
        }
        if (OP == OP_SUB) {
#pragma unroll
            for (int r = 0; r < 4; ++r) g[r] = *(const f32x4 *)(A.grad + base + r * 256 + lane * 4);
        }
#pragma unroll
        for (int r = 0; r < 4; ++r)
            s[r] = *(const f32x4 *)(A.state + base + r * 256 + lane * 4);
        if (MODE != MODE_PLAIN) d = span_desc(toff, A.J, base, base + TILE - 1u);
#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                a[r][j] = (OP == OP_FMA) ? __builtin_fmaf(A.lr, g[r][j], s[r][j])
                                         : ((OP == OP_SUB) ? (g[r][j] - s[r][j]) : s[r][j]);
        if (MODE != MODE_PLAIN) tile_tail<MODE>(A, tau, t, d, a, lhist, cur, stage, only);
        // The state goes out last: this wave never has to wait for the stores to be
        // acknowledged (the memory counter it would wait on also counts stores).
        if (OP == OP_FMA) {
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                f32x4 o;
#pragma unroll
                for (int j = 0; j < 4; ++j) o[j] = a[r][j];
                *(f32x4 *)(A.state + base + r * 256 + lane * 4) = o;
            }
        }
        return;
    }

    // ragged last tile, or buffers that are only 4-byte aligned
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
                } else if (OP == OP_SUB) {
                    v = A.grad[e] - A.state[e];
                } else {
                    v = A.state[e];
                }
            }
            a[r][j] = v;
        }
    if (MODE == MODE_PLAIN) return;
    d = span_desc(toff, A.J, base, min(base + TILE, A.n) - 1u);
    tile_tail<MODE>(A, tau, t, d, a, lhist, cur, stage, only);
}

template <int OP, int MODE, bool VEC>
__global__ __launch_bounds__(STREAM_THREADS) void k_stream(const StreamArgs A,
                                                           const uint32_t *__restrict__ toff,
                                                           const uint32_t *__restrict__ tau)
{
    __shared__ uint32_t lhist[MODE == MODE_HIST ? HBINS : 1];
    __shared__ uint2 stage_all[MODE == MODE_COLLECT ? WAVES_PER_BLOCK * STAGE : 1];
    const uint32_t wave = uniform(threadIdx.x >> 6);
    uint2 *stage = stage_all + (MODE == MODE_COLLECT ? wave * STAGE : 0u);
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
            const uint32_t qfirst = q * WAVES_PER_BLOCK * TILE;
            const uint32_t fx = span_desc(toff, A.J, qfirst, qfirst).x;
            const int qt = (fx >> 31) ? (int)(fx & 0x7FFFFFFFu) : -1;
            if (qt != cur) {
                flush_hist<MODE>(lhist, A.ghist, cur);
                cur = qt;
            }
        }
        const uint32_t t = q * WAVES_PER_BLOCK + wave;
        if (t < A.ntiles) process_tile<OP, MODE, VEC>(A, toff, tau, t, lhist, cur, stage);
    }
    flush_hist<MODE>(lhist, A.ghist, cur);
}

// Plain launch, or a launch whose begin and / or end is stamped into an event.
template <class K, class... Args>
static void launch_k(K kernel, dim3 grid, dim3 block, hipStream_t st, void *ev0, void *ev1, Args... args)
{
    if (ev0 || ev1)
        hipExtLaunchKernelGGL(kernel, grid, block, 0, st, (hipEvent_t)ev0, (hipEvent_t)ev1, 0, args...);
    else
        hipLaunchKernelGGL(kernel, grid, block, 0, st, args...);
}

template <int OP, int MODE>
static void launch_stream_t(bool vec, const StreamArgs &a, uint32_t blocks, hipStream_t st, void *ev0,
                            void *ev1)
{
    if (vec)
        launch_k(k_stream<OP, MODE, true>, dim3(blocks), dim3(STREAM_THREADS), st, ev0, ev1, a,
                 a.toff, a.tau);
    else
        launch_k(k_stream<OP, MODE, false>, dim3(blocks), dim3(STREAM_THREADS), st, ev0, ev1, a,
                 a.toff, a.tau);
}

void launch_stream(int op, int mode, bool vec, const StreamArgs &a, uint32_t blocks, void *stream,
                   void *ev0, void *ev1)
{
    hipStream_t st = (hipStream_t)stream;
    if (blocks == 0) return;
    if (op == OP_FMA) {
        if (mode == MODE_PLAIN) launch_stream_t<OP_FMA, MODE_PLAIN>(vec, a, blocks, st, ev0, ev1);
        else if (mode == MODE_COLLECT) launch_stream_t<OP_FMA, MODE_COLLECT>(vec, a, blocks, st, ev0, ev1);
        else launch_stream_t<OP_FMA, MODE_HIST>(vec, a, blocks, st, ev0, ev1);
    } else if (op == OP_SUB) {
        if (mode == MODE_COLLECT) launch_stream_t<OP_SUB, MODE_COLLECT>(vec, a, blocks, st, ev0, ev1);
        else if (mode == MODE_HIST) launch_stream_t<OP_SUB, MODE_HIST>(vec, a, blocks, st, ev0, ev1);
    } else {
        if (mode == MODE_COLLECT) launch_stream_t<OP_IDENT, MODE_COLLECT>(vec, a, blocks, st, ev0, ev1);
        else if (mode == MODE_HIST) launch_stream_t<OP_IDENT, MODE_HIST>(vec, a, blocks, st, ev0, ev1);
    }
}

// ---------------------------------------------------------------------------
// workgroup helpers for pick / select
// ---------------------------------------------------------------------------

// Inclusive prefix sum over the 64 lanes of a wavefront, in registers (DPP):
// four shifts inside each row of 16 lanes, then two row broadcasts.
__device__ __forceinline__ uint32_t wave_incl_scan(uint32_t v)
{
    int x = (int)v;
    x += __builtin_amdgcn_update_dpp(0, x, 0x111, 0xf, 0xf, false);   // row_shr:1
    x += __builtin_amdgcn_update_dpp(0, x, 0x112, 0xf, 0xf, false);   // row_shr:2
    x += __builtin_amdgcn_update_dpp(0, x, 0x114, 0xf, 0xf, false);   // row_shr:4
    x += __builtin_amdgcn_update_dpp(0, x, 0x118, 0xf, 0xf, false);   // row_shr:8
    x += __builtin_amdgcn_update_dpp(0, x, 0x142, 0xa, 0xf, false);   // row_bcast:15 into rows 1, 3
    x += __builtin_amdgcn_update_dpp(0, x, 0x143, 0xc, 0xf, false);   // row_bcast:31 into rows 2, 3
    return (uint32_t)x;
}

__device__ __forceinline__ uint32_t wave_sum(uint32_t v)
{
    return (uint32_t)__builtin_amdgcn_readlane((int)wave_incl_scan(v), 63);
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

// Workgroup sum.  wsum: LDS scratch of nw words.  Contains two barriers.
__device__ __forceinline__ uint32_t block_sum(uint32_t v, uint32_t *wsum, int nw)
{
    const uint32_t s = wave_sum(v);
    __syncthreads();
    if (lane_id() == 0) wsum[threadIdx.x >> 6] = s;
    __syncthreads();
    uint32_t tot = 0;
    for (int w = 0; w < nw; ++w) tot += wsum[w];
    return tot;
}

// In an LDS histogram h[NB] (NB a multiple of 64, at most 4096), find for each of
// three ranks R[0..2] (counted from the top bin, >= 1) the bin holding it and the
// rank inside that bin:  res[2 i] = bin, res[2 i + 1] = rank in the bin; bin -1 if the
// rank exceeds the histogram total (or is 0).  Every wavefront sums rows of 64 bins,
// then up to three wavefronts each scan the row sums and the row their rank lands in.
// Barriers: one on entry (h complete), one in the middle, one on exit.
template <int NB, int NW>
__device__ __forceinline__ void find_ranks(const uint32_t *h, uint32_t R0, uint32_t R1, uint32_t R2,
                                           uint32_t *rowsum, int *res)
{
    constexpr int ROWS = NB / 64;
    constexpr int SEARCHERS = NW < 3 ? NW : 3;
    static_assert(ROWS * 64 == NB && ROWS <= 64, "histogram shape");
    const uint32_t lane = lane_id();
    const uint32_t wave = threadIdx.x >> 6;
    __syncthreads();
    for (int r = (int)wave; r < ROWS; r += NW) {
        const uint32_t s = wave_sum(h[r * 64 + lane]);
        if (lane == 0) rowsum[r] = s;
    }
    __syncthreads();
    if (wave < (uint32_t)SEARCHERS) {
        // lane l looks at row ROWS-1-l: the top row first
        const uint32_t rs = (lane < (uint32_t)ROWS) ? rowsum[ROWS - 1 - lane] : 0u;
        const uint32_t rincl = wave_incl_scan(rs);
        for (int which = (int)wave; which < 3; which += SEARCHERS) {
            const uint32_t R = which == 0 ? R0 : (which == 1 ? R1 : R2);
            int bin = -1;
            uint32_t rin = 0;
            const uint64_t hit = ballot64(lane < (uint32_t)ROWS && rincl >= R);
            if (hit != 0 && R != 0) {
                const int rl = __ffsll((unsigned long long)hit) - 1;          // first row reaching R
                const uint32_t above = (uint32_t)__builtin_amdgcn_readlane((int)(rincl - rs), rl);
                const int row = ROWS - 1 - rl;
                const uint32_t Rr = R - above;                                 // rank inside the row
                const uint32_t v = h[row * 64 + (63 - lane)];                  // top bin first
                const uint32_t vincl = wave_incl_scan(v);
                const uint64_t hit2 = ballot64(vincl >= Rr);
                const int bl = __ffsll((unsigned long long)hit2) - 1;
                const uint32_t above2 = (uint32_t)__builtin_amdgcn_readlane((int)(vincl - v), bl);
                bin = row * 64 + 63 - bl;
                rin = Rr - above2;
            }
            if (lane == 0) {
                res[2 * which] = bin;
                res[2 * which + 1] = (int)rin;
            }
        }
    }
    __syncthreads();
}

// ---------------------------------------------------------------------------
// pick: streaming-pass histogram -> candidate threshold (non-predicted path)
// ---------------------------------------------------------------------------

__global__ __launch_bounds__(256) void k_pick(const TensorDesc *tdesc, const PlanEntry *plan,
                                              uint32_t *ghist, uint32_t *tau, uint32_t *tprev,
                                              DevStats *stats, const SegState *only_pending,
                                              const uint32_t *pending)
{
    const uint32_t j = blockIdx.x;
    if (!tdesc[j].big) return;
    if (only_pending && (*pending == 0 || only_pending[j].status != SEG_PENDING)) return;
    __shared__ uint32_t h[HBINS];
    __shared__ uint32_t rowsum[64];
    __shared__ int res[6];
    uint32_t *g = ghist + (size_t)j * HBINS;
    for (uint32_t b = threadIdx.x; b < HBINS; b += 256) {
        h[b] = g[b];
        g[b] = 0;   // leave the histogram clean for the next use
    }
    const PlanEntry pe = plan[j];
    find_ranks<HBINS, 4>(h, pe.k2, pe.k, 0u, rowsum, res);
    if (threadIdx.x == 0) {
        const int b2 = res[0], b1 = res[2];
        // the histogram holds the nonzero keys only: a rank beyond its total means
        // "fewer nonzeros than that", and every nonzero is collected
        uint32_t t;
        if (b2 < 0 && b1 < 0) {
            t = 1;
        } else if (b2 < 0) {
            t = (b1 > 0) ? (1u << HSHIFT) : 1u;
        } else if (b2 > 0) {
            t = (uint32_t)b2 << HSHIFT;
        } else if (b1 > 0) {
            t = 1u << HSHIFT;
        } else {
            t = 1;   // the k-th key is tiny or zero: collect every nonzero
        }
        tau[j] = t;
        // where the k-th key lies (middle of its bucket): anchors the window histogram of
        // the segmented selection
        tprev[j] = (b1 >= 0) ? (((uint32_t)b1 << HSHIFT) + (1u << (HSHIFT - 1))) : 0u;
    }
}

void launch_pick(const TensorDesc *tdesc, const PlanEntry *plan, uint32_t *ghist, uint32_t *tau,
                 uint32_t *tprev, DevStats *stats, uint32_t J, void *stream, const SegState *only_pending,
                 const uint32_t *pending)
{
    hipLaunchKernelGGL(k_pick, dim3(J), dim3(256), 0, (hipStream_t)stream, tdesc, plan, ghist, tau, tprev,
                       stats, only_pending, pending);
}

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
                        fix_sent<OP>(A.state, ix, __uint_as_float(vb[i]), A.m);
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
template <int OP>
__device__ __forceinline__ void zero_fill_emit(const SrcList src, const uint32_t c, const TensorDesc &td,
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
        fix_sent<OP>(A.state, ix, v, A.m);
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

// Ordered-list entry: LDS while it fits, global scratch beyond.
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

constexpr uint32_t SEL_ROWS = 12;                                  // rows of 16 tiles per wavefront and batch
constexpr uint32_t SEL_WAVE_TILES = SEL_ROWS * 16;                 // 192
constexpr uint32_t SEL_BATCH_TILES = SEL_WAVES * SEL_WAVE_TILES;   // 3072

// One workgroup per tensor.  Big tensors: join the per-tile candidate slots into
// one ordered list (LDS; lists that outgrow it continue in global scratch), then
// select on the list; if the list is short or a tile overflowed, select densely
// from the state buffer.  Small tensors always select densely.
//
// The join: a batch of tiles is dealt out to the wavefronts in equal runs of whole
// rows (16 consecutive tiles).  A wavefront fetches the counts of its run, one tile
// per lane, and the first line of every tile (its first 8 candidates), 4 lanes per
// tile and a row per load, before the counts are known.  Counts are handed to the
// tiles' lanes by lane permutation and scanned row by row in registers; one exchange
// of the wavefronts' totals through LDS gives every tile its list position, and the
// lanes drop their two entries into place.  Tiles with more than 8 candidates, and a
// first tile shared with the previous tensor, take a per-tile loop.
template <int OP>
__global__ __launch_bounds__(SEL_THREADS) void k_select(const SelectArgs A,
                                                        const uint32_t *__restrict__ tile_cnt,
                                                        const uint2 *__restrict__ heads,
                                                        const uint2 *__restrict__ slots)
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
    if (j == 0 && tid == 0 && A.pending) *A.pending = 0;   // every reader of this call has finished
    if (pe.seg) {
        // planned for the segmented kernels; only a tensor they handed over is taken here
        const uint32_t status = A.segstate[j].status;
        if (status == SEG_FALLBACK) dense = true;
        else if (status != SEG_ZEROFILL) return;
    }
    bool zerofill = false;
    uint32_t c = 0;
    uint32_t kmin = 0xFFFFFFFFu;                     // smallest candidate key
    const uint32_t tau_cur = td.big ? A.tau[j] : TAU_NEVER;
    const uint32_t hint2_cur = (td.big && A.write_hint) ? A.hint2[j] : 0u;
    // every candidate key is >= the collection threshold: the window histogram starts there,
    // and the join counts the entries into it as it places them
    // (or 1024 buckets below the k-th key of the previous call, if that lies higher)
    const uint32_t tprev_cur = td.big ? A.tprev[j] : 0u;
    const uint32_t win_join = max(tau_cur >> 11, max(tprev_cur >> 11, 1024u) - 1024u);
    uint2 *glist = A.ord + (size_t)(tlo + j) * CAPT;   // this tensor's ordered list in global scratch
    if (tid == 0) S.kmin = 0xFFFFFFFFu;

    if (!dense) {
        for (uint32_t b = tid; b < 2048; b += SEL_THREADS) S.h[b] = 0;   // complete before the join's barrier
        const uint32_t ntl = thi - tlo + 1;
        const uint32_t lane = lane_id(), wave = tid >> 6;
        const uint32_t qw = lane >> 2, sub = lane & 3u;
        uint32_t ovf = 0;
        auto join_batch = [&](const uint32_t cb) __attribute__((always_inline)) {
            const uint32_t nb = min(ntl - cb, SEL_BATCH_TILES);
            const uint32_t rows = (nb + 16 * SEL_WAVES - 1) / (16 * SEL_WAVES);   // per wavefront, 1..SEL_ROWS
            const uint32_t w0 = cb + wave * rows * 16;                            // first tile of this wavefront's run
            // counts of the run, one tile per lane and load
            uint32_t w[SEL_ROWS / 4];
#pragma unroll
            for (uint32_t u = 0; u < SEL_ROWS / 4; ++u) {
                const uint32_t sl = u * 64 + lane;
                w[u] = (sl < rows * 16 && w0 + sl < ntl) ? tile_cnt[tlo + w0 + sl] : 0u;
            }
            // first line of every tile of the run
            uint4 pf[SEL_ROWS];
#pragma unroll
            for (uint32_t it = 0; it < SEL_ROWS; ++it) {
                const uint32_t tl = w0 + it * 16 + qw;
                pf[it] = make_uint4(0, 0, 0, 0);
                if (it < rows && tl < ntl) pf[it] = ((const uint4 *)(heads + (size_t)(tlo + tl) * HEAD))[sub];
            }
            // a first tile shared with the previous tensor: that tensor's candidates come first
            uint32_t start0 = 0;
            if (head_shared && w0 == 0) {
                const uint32_t ww = (uint32_t)__builtin_amdgcn_readfirstlane((int)w[0]);
                if (ww != CNT_OVERFLOW) {
                    start0 = ww & 0xFFFFu;
                    if (lane == 0) w[0] = ww >> 16;
                }
            }
#pragma unroll
            for (uint32_t u = 0; u < SEL_ROWS / 4; ++u) {
                if (w[u] == CNT_OVERFLOW) { ovf = 1; w[u] = 0; }
                else if (!(head_shared && w0 == 0 && u == 0 && lane == 0)) w[u] &= 0xFFFFu;
            }
            // positions inside the run: the counts go to the tiles' lanes, rows are scanned in turn
            // (per tile: count in the low half, position in the high half -- a run holds at
            // most 192 * CAPT entries)
            uint32_t cp[SEL_ROWS];
            uint32_t run = 0;
#pragma unroll
            for (uint32_t it = 0; it < SEL_ROWS; ++it) {
                cp[it] = 0;
                if (it < rows) {                                                  // uniform
                    const uint32_t n_t = (uint32_t)__builtin_amdgcn_ds_bpermute(
                        (int)((((it & 3u) * 16u) + qw) * 4u), (int)w[it >> 2]);
                    const uint32_t incl = wave_incl_scan(sub == 0 ? n_t : 0u);    // over the row's tiles
                    cp[it] = n_t | ((run + incl - n_t) << 16);
                    run += (uint32_t)__builtin_amdgcn_readlane((int)incl, 63);
                }
            }
            if (lane == 0) S.wsum[wave] = run;
            __syncthreads();
            uint32_t before = 0, tot = 0;
#pragma unroll
            for (uint32_t x = 0; x < SEL_WAVES; ++x) {
                const uint32_t v = S.wsum[x];
                if (x < wave) before += v;
                tot += v;
            }
            const uint32_t base = c + before;
            c += tot;
            // entries into place
#pragma unroll
            for (uint32_t it = 0; it < SEL_ROWS; ++it) {
                const uint32_t tl = w0 + it * 16 + qw;
                const uint32_t n_t = cp[it] & 0xFFFFu;
                if (n_t == 0) continue;
                const uint32_t start = (tl == 0) ? start0 : 0u;
                const uint32_t pos = base + (cp[it] >> 16);
                uint32_t i0 = 0;
                if (start == 0) {
                    if (2 * sub < n_t) {
                        put_entry(llist, glist, pos + 2 * sub, make_uint2(pf[it].x, pf[it].y));
                        kmin = min(kmin, pf[it].y & 0x7FFFFFFFu);
                        window_count(S.h, win_join, pf[it].y & 0x7FFFFFFFu);
                    }
                    if (2 * sub + 1 < n_t) {
                        put_entry(llist, glist, pos + 2 * sub + 1, make_uint2(pf[it].z, pf[it].w));
                        kmin = min(kmin, pf[it].w & 0x7FFFFFFFu);
                        window_count(S.h, win_join, pf[it].w & 0x7FFFFFFFu);
                    }
                    i0 = HEAD;
                }
                if (i0 < n_t) {
                    // the rest of a crowded tile: the four lanes interleave, each with four
                    // independent loads at a time (entry q of the tile: heads for q < HEAD,
                    // slots beyond)
                    const uint2 *hd = heads + (size_t)(tlo + tl) * HEAD;
                    const uint2 *sl = slots + (size_t)(tlo + tl) * CAPT;
                    for (uint32_t i = i0 + sub; i < n_t; i += 16) {
                        uint2 e[4];
#pragma unroll
                        for (uint32_t v = 0; v < 4; ++v) {
                            const uint32_t q = start + i + 4 * v;
                            e[v] = (i + 4 * v < n_t) ? ((q < HEAD) ? hd[q] : sl[q]) : make_uint2(0, 0);
                        }
#pragma unroll
                        for (uint32_t v = 0; v < 4; ++v) {
                            if (i + 4 * v < n_t) {
                                put_entry(llist, glist, pos + i + 4 * v, e[v]);
                                kmin = min(kmin, e[v].y & 0x7FFFFFFFu);
                                window_count(S.h, win_join, e[v].y & 0x7FFFFFFFu);
                            }
                        }
                    }
                }
            }
        };
        // the first batch (up to 3072 tiles: all there is, as a rule) stands outside the loop, so
        // that what the loop keeps in registers across its rounds does not weigh on it
        join_batch(0);
        for (uint32_t cb = SEL_BATCH_TILES; cb < ntl; cb += SEL_BATCH_TILES) {
            __syncthreads();   // wsum is reused
            join_batch(cb);
        }
        kmin = wave_min_to_last(kmin);
        if (lane_id() == 63) atomicMin(&S.kmin, kmin);
        const bool any_ovf = __syncthreads_or((int)ovf) != 0;   // also orders the list writes
        kmin = S.kmin;
        if (!any_ovf && c < pe.k && tau_cur <= 1u) zerofill = true;   // every nonzero is already here
        else if (any_ovf || c < pe.k) dense = true;
        if (!dense && c > SEL_LDS_LIST) {
            // the list outgrew LDS: complete the global copy
            for (uint32_t p = tid; p < SEL_LDS_LIST; p += SEL_THREADS) glist[p] = llist[p];
            __syncthreads();
        }
        if (tid == 0) {
            if (dense) {
                atomicAdd(&A.stats->fallback_tensors, 1ull);
                atomicAdd(&A.stats->fallback_elems, (unsigned long long)td.n);
            } else {
                atomicAdd(&A.stats->candidates, (unsigned long long)c);
            }
        }
    }

    if (zerofill) {
        if (c <= SEL_LDS_LIST) zero_fill_emit<OP>(SrcList{llist}, c, td, pe, A, S.wsum);
        else zero_fill_emit<OP>(SrcList{glist}, c, td, pe, A, S.wsum);
        if (A.write_hint && tid == 0) {
            A.tau[j] = 1u;
            A.hint2[j] = 0u;
            A.tprev[j] = 0u;
        }
        return;
    }

    // ---- rank whose key becomes the next predicted threshold
    uint32_t R = 0, Eq = 0;
    if (td.big && A.write_hint)
        R = hint_rank<OP>(td, pe, !dense && !A.exact_mode, c, hint2_cur, A.m, &Eq);

    uint32_t tau_next = 0, expect = 0, q_e = 0, t_k = 0;
    // the join's histogram stands if no candidate lies below the threshold (none can)
    const bool win_ready = (kmin != 0xFFFFFFFFu) && (kmin >> 11) >= (tau_cur >> 11);
    const uint32_t win_base = (kmin == 0xFFFFFFFFu) ? 0xFFFFFFFFu : (win_ready ? win_join : (kmin >> 11));
    const uint32_t win_min = (win_ready && win_join > (kmin >> 11)) ? 1u : 0u;   // entries below the window
    if (dense) {
        if (td.n <= 2 * SEL_LDS_LIST) {
            uint32_t *lv = (uint32_t *)llist;
            __syncthreads();
            for (uint32_t p = tid; p < td.n; p += SEL_THREADS)
                lv[p] = __float_as_uint(row_value<OP>(A.state, A.model, td.off + p));
            __syncthreads();
            SrcDenseLds src{lv, td.off};
            select_emit<OP, 4>(src, td.n, pe.k, R, 0u, 0xFFFFFFFFu, 0u, false, 0xFFFFFFFFu, S, A, pe.outoff,
                               &tau_next, &expect, &q_e, &t_k);
        } else {
            SrcDense<OP> src{A.state, A.model, td.off};
            select_emit<OP, 8>(src, td.n, pe.k, R, 0u, 0xFFFFFFFFu, 0u, false, 0xFFFFFFFFu, S, A, pe.outoff,
                               &tau_next, &expect, &q_e, &t_k);
        }
    } else if (c <= SEL_LDS_LIST) {
        SrcList src{llist};
        select_emit<OP, 4>(src, c, pe.k, R, Eq, win_base, win_min, win_ready, kmin, S, A, pe.outoff,
                           &tau_next, &expect, &q_e, &t_k);
    } else {
        SrcList src{glist};
        select_emit<OP, 8>(src, c, pe.k, R, Eq, win_base, win_min, win_ready, kmin, S, A, pe.outoff,
                           &tau_next, &expect, &q_e, &t_k);
    }

    if (td.big && A.write_hint && tid == 0) {
        uint32_t tn = tau_next;
        if (tn == 0) {
            tn = hint_relaxed(tau_cur, dense ? 0xFFFFFFFFu : kmin);
            expect = 0;
        } else if (q_e != 0) {
            tn = hint_scaled(tn, q_e, tau_cur);
        }
        if (tn >= 0x7F800000u) tn = 0x7F7FFFFFu;   // keep the hint finite
        A.tau[j] = tn;
        A.hint2[j] = expect;
        A.tprev[j] = t_k;
    }
}


// ---------------------------------------------------------------------------
// segmented selection: one workgroup per segment of SEG_TILES tiles
// ---------------------------------------------------------------------------
//
//   join    per segment : compact the tiles' candidates into one ordered list and
//                         count them into the tensor's window histogram
//                         (key >> 12, counted from the collection threshold)
//   window  per tensor  : histogram -> 19-bit prefix of the k-th key, next threshold
//   prefix  per segment : count entries above the prefix, append those sharing it
//                         to the tensor's prefix list
//   rank    per tensor  : low 12 bits of the k-th key among the prefix list, then the
//                         output position and the tie budget of every segment
//   emit    per segment : ordered emission ("encode()") and the state fix-up
//
// A tensor the chain cannot resolve (fewer candidates than k, an overflowed tile,
// the k-th key beyond the window, a prefix list that outgrows PFX_CAP) is marked
// SEG_FALLBACK and selected from the state buffer by k_select afterwards.

// First bin (key >> SEG_LOWBITS) of a tensor's window histogram.  Candidates start at
// the collection threshold; when that lies far below the k-th key of the previous
// selection on this stream (a relaxed hint), the window is centred on that key instead,
// so that it reaches half an octave to either side of it.  Keys below the window are
// counted into bin 0, which then holds no usable rank.
__device__ __forceinline__ uint32_t seg_window_base(uint32_t tau_cur, uint32_t t_prev)
{
    const uint32_t b_tau = tau_cur >> SEG_LOWBITS;
    const uint32_t b_prev = t_prev >> SEG_LOWBITS;
    const uint32_t b_mid = (b_prev > SEG_WBINS / 2) ? (b_prev - SEG_WBINS / 2) : 0u;
    return max(b_tau, b_mid);
}

// The entries one segment contributes: its compacted candidate list, or (dense
// requests) the tensor's own elements inside the segment, in index order.
struct SegSource {
    const uint2 *list;
    const float *state;
    const float *model;
    uint32_t first;   // dense: first element
    uint32_t count;
    bool dense;
    __device__ __forceinline__ uint2 get(uint32_t e) const
    {
        if (!dense) return list[e];
        const uint32_t ix = first + e;
        const float v = model ? (model[ix] - state[ix]) : state[ix];
        return make_uint2(ix, __float_as_uint(v));
    }
};

__device__ __forceinline__ SegSource seg_source(const SegArgs &A, const TensorDesc &td, const SegDesc &sd,
                                                uint32_t seg, bool dense)
{
    SegSource S;
    S.list = A.ord + (size_t)(sd.tile0 + sd.j) * CAPT;
    S.state = A.state;
    S.model = A.model;
    S.dense = dense;
    if (dense) {
        const uint64_t lo = max((uint64_t)td.off, (uint64_t)sd.tile0 * TILE);
        const uint64_t hi = min((uint64_t)td.off + td.n, ((uint64_t)sd.tile0 + sd.ntiles) * TILE);
        S.first = (uint32_t)lo;
        S.count = (uint32_t)(hi - lo);
    } else {
        S.first = 0;
        S.count = A.segcnt[seg];
    }
    return S;
}

__global__ __launch_bounds__(SEG_THREADS) void k_seg_join(const SegArgs A)
{
    __shared__ uint32_t h[SEG_WBINS];
    __shared__ uint32_t tpos[SEG_TILES];
    __shared__ uint32_t tstart[SEG_TILES];
    __shared__ uint32_t wsum[SEG_THREADS / 64];
    if (A.round != 0 && *A.pending == 0) return;
    const SegDesc sd = A.segtab[blockIdx.x];
    if (!A.plan[sd.j].seg) return;
    if (A.round != 0 && A.segstate[sd.j].status != SEG_PENDING) return;
    const TensorDesc td = A.tdesc[sd.j];
    const uint32_t tid = threadIdx.x;
    for (uint32_t b = tid; b < SEG_WBINS; b += SEG_THREADS) h[b] = 0;
    if (A.dense) {
        // dense request: count the segment's own elements at or above this call's threshold
        const SegSource S = seg_source(A, td, sd, blockIdx.x, true);
        const uint32_t tau_d = A.tau[sd.j];
        const uint32_t base_d = seg_window_base(tau_d, A.tprev[sd.j]);
        uint32_t mine = 0;
        __syncthreads();
        for (uint32_t e = tid; e < S.count; e += SEG_THREADS) {
            const uint32_t key = S.get(e).y & 0x7FFFFFFFu;
            if (key >= tau_d) {
                const uint32_t hi12 = key >> SEG_LOWBITS;
                const uint32_t w = (hi12 > base_d) ? (hi12 - base_d) : 0u;
                atomicAdd(&h[min(w, SEG_WBINS - 1u)], 1u);
                ++mine;
            }
        }
        const uint32_t tot = block_sum(mine, wsum, SEG_THREADS / 64);
        uint32_t *ghd = A.whist + (size_t)sd.j * HBINS;
        for (uint32_t b = tid; b < SEG_WBINS; b += SEG_THREADS) {
            const uint32_t v = h[b];
            if (v) atomicAdd(&ghd[b], v);
        }
        if (tid == 0) A.segcnt[blockIdx.x] = tot;
        return;
    }
    const uint32_t tlo = td.off / TILE;
    const bool head_shared = (td.off % TILE) != 0;

    // this tensor's candidates in every tile of the segment: count and first slot
    uint32_t cnt = 0, start = 0;
    int ovf = 0;
    if (tid < sd.ntiles) {
        uint32_t ww = A.tile_cnt[sd.tile0 + tid];
        if (ww == CNT_OVERFLOW) { ovf = 1; ww = 0; }
        const bool hs = head_shared && (sd.tile0 + tid == tlo);
        cnt = hs ? (ww >> 16) : (ww & 0xFFFFu);
        start = hs ? (ww & 0xFFFFu) : 0u;
    }
    uint32_t cs;
    const uint32_t pos = block_excl_scan<SEG_THREADS / 64>(cnt, wsum, cs);
    tpos[tid] = (tid < sd.ntiles) ? pos : cs;
    tstart[tid] = start;
    const bool any_ovf = __syncthreads_or(ovf) != 0;

    uint2 *dst = A.ord + (size_t)(sd.tile0 + sd.j) * CAPT;
    const uint32_t win_base = seg_window_base(A.tau[sd.j], A.tprev[sd.j]);
    // entry e of the segment: tile = last one whose first position is <= e
    for (uint32_t eb = 0; eb < cs; eb += 4 * SEG_THREADS) {
        uint2 ent[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const uint32_t e = eb + u * SEG_THREADS + tid;
            ent[u] = make_uint2(0, 0);
            if (e < cs) {
                uint32_t lo = 0, hi = sd.ntiles;
                while (hi - lo > 1) {
                    const uint32_t mid = (lo + hi) >> 1;
                    if (tpos[mid] <= e) lo = mid;
                    else hi = mid;
                }
                const uint32_t q = tstart[lo] + (e - tpos[lo]);
                const size_t t = (size_t)sd.tile0 + lo;
                ent[u] = (q < HEAD) ? A.heads[t * HEAD + q] : A.slots[t * CAPT + q];
            }
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const uint32_t e = eb + u * SEG_THREADS + tid;
            if (e < cs) {
                dst[e] = ent[u];
                const uint32_t hi12 = (ent[u].y & 0x7FFFFFFFu) >> SEG_LOWBITS;
                const uint32_t w = (hi12 > win_base) ? (hi12 - win_base) : 0u;
                atomicAdd(&h[min(w, SEG_WBINS - 1u)], 1u);
            }
        }
    }
    __syncthreads();
    uint32_t *gh = A.whist + (size_t)sd.j * HBINS;
    for (uint32_t b = tid; b < SEG_WBINS; b += SEG_THREADS) {
        const uint32_t v = h[b];
        if (v) atomicAdd(&gh[b], v);
    }
    if (tid == 0) {
        A.segcnt[blockIdx.x] = cs;
        if (any_ovf) atomicOr(&A.segstate[sd.j].ovf, 1u);
    }
}

template <int OP>
__global__ __launch_bounds__(SEG_THREADS) void k_seg_window(const SegArgs A)
{
    __shared__ uint32_t h[SEG_WBINS];
    __shared__ uint32_t rowsum[64];
    __shared__ int res[6];
    __shared__ uint32_t wsum[SEG_THREADS / 64];
    __shared__ uint32_t lowest;
    if (A.round != 0 && *A.pending == 0) return;
    const uint32_t j = blockIdx.x;
    const PlanEntry pe = A.plan[j];
    if (!pe.seg) return;
    if (A.round != 0 && A.segstate[j].status != SEG_PENDING) return;
    const TensorDesc td = A.tdesc[j];
    const uint32_t tid = threadIdx.x;
    uint32_t *gh = A.whist + (size_t)j * HBINS;
    uint32_t mine = 0, mylow = 0xFFFFFFFFu;
    if (tid == 0) lowest = 0xFFFFFFFFu;
    for (uint32_t b = tid; b < SEG_WBINS; b += SEG_THREADS) {
        const uint32_t v = gh[b];
        h[b] = v;
        gh[b] = 0;   // clean for the next use
        mine += v;
        if (v && mylow == 0xFFFFFFFFu) mylow = b;
    }
    const uint32_t c = block_sum(mine, wsum, SEG_THREADS / 64);
    if (mylow != 0xFFFFFFFFu) atomicMin(&lowest, mylow);
    const uint32_t tau_cur = A.tau[j];
    const uint32_t win_base = seg_window_base(tau_cur, A.tprev[j]);
    const int bin_min = (win_base > (tau_cur >> SEG_LOWBITS)) ? 1 : 0;   // bin 0 mixes in lower keys
    uint32_t R = 0, Eq = 0;
    if (A.write_hint) R = hint_rank<OP>(td, pe, !A.exact_mode, c, A.hint2[j], A.m, &Eq);
    const bool measurable = (R != 0) && (c >= R);
    const uint32_t qlow = max(c / 4u, min(c, 16u));
    const uint32_t third = measurable ? Eq : ((R != 0 && c != 0) ? (c - qlow + 1u) : 0u);
    find_ranks<SEG_WBINS, SEG_THREADS / 64>(h, pe.k, measurable ? R : pe.k, third, rowsum, res);
    if (tid == 0) {
        SegState *st = &A.segstate[j];
        const int bk = res[0], bR = res[2];
        const bool all = (pe.k == td.n);   // everything is sent: no threshold to find
        const bool ok = all || ((st->ovf == 0) && (c >= pe.k) && bk >= bin_min && bk < (int)SEG_WBINS - 1);
        // fewer candidates than k with every nonzero collected: k_select completes with zeros
        // (from the candidate lists, which a dense request does not have)
        const bool zf = !A.dense && !all && (st->ovf == 0) && (c < pe.k) && (tau_cur <= 1u);
        st->ovf = 0;
        st->pfxcount = 0;
        st->pfx = win_base + (uint32_t)max(bk, 0);
        st->r2 = (uint32_t)res[1];
        st->T = 0;
        // a failed first attempt is collected again by the repair round; a failed repair
        // (e.g. one value filling a whole histogram bucket) is left to k_select
        const bool again = (A.round == 0) && A.repair && !A.dense;   // the second collection needs candidate lists
        const uint32_t bad = again ? SEG_PENDING : SEG_FALLBACK;
        st->status = all ? (uint32_t)SEG_ALL : (ok ? (SEG_ACTIVE + A.round) : (zf ? SEG_ZEROFILL : bad));
        if (!ok && !zf) {
            if (again) {
                atomicAdd(A.pending, 1u);
            } else {
                atomicAdd(&A.stats->fallback_tensors, 1ull);
                atomicAdd(&A.stats->fallback_elems, (unsigned long long)td.n);
            }
        } else if (ok) {
            atomicAdd(&A.stats->candidates, (unsigned long long)c);
            atomicAdd(&A.stats->segmented_tensors, 1ull);
            if (A.round != 0) atomicAdd(&A.stats->repaired_tensors, 1ull);
            if (A.write_hint) {
                uint32_t tn = 0, expect = 0;
                if (measurable && bR >= bin_min && bR < (int)SEG_WBINS - 1) {
                    const uint32_t edge = (win_base + (uint32_t)bR) << SEG_LOWBITS;
                    tn = edge ? edge : 1u;
                    expect = R - (uint32_t)res[3] + h[bR];
                    const int bE = res[4];
                    if (bE >= bin_min && bE < (int)SEG_WBINS - 1)
                        tn = hint_scaled(tn, (win_base + (uint32_t)bE) << SEG_LOWBITS, tau_cur);
                }
                if (tn == 0 && !measurable && R != 0 && lowest != 0xFFFFFFFFu && (int)lowest >= bin_min &&
                    res[4] >= (int)lowest && res[4] < (int)SEG_WBINS - 1) {
                    const uint32_t kmin = max((win_base + lowest) << SEG_LOWBITS, tau_cur);
                    tn = hint_extrapolated(kmin, c, R, qlow, ((uint32_t)res[4] - lowest + 1u) << SEG_LOWBITS);
                    expect = R;
                }
                if (tn == 0) {
                    const uint32_t kmin = (lowest == 0xFFFFFFFFu || (int)lowest < bin_min) ? 0xFFFFFFFFu
                                                                 : max((win_base + lowest) << SEG_LOWBITS, tau_cur);
                    tn = hint_relaxed(tau_cur, kmin);
                    expect = 0;
                }
                if (tn >= 0x7F800000u) tn = 0x7F7FFFFFu;
                A.tau[j] = tn;
                A.hint2[j] = expect;
            }
        }
    }
}

constexpr uint32_t PFX_STAGE = 1024;   // entries sharing the prefix that one segment can stage in LDS

__global__ __launch_bounds__(SEG_THREADS) void k_seg_prefix(const SegArgs A)
{
    __shared__ uint32_t wsum[SEG_THREADS / 64];
    __shared__ uint2 stage[PFX_STAGE];
    __shared__ uint32_t nstage, base;
    const SegDesc sd = A.segtab[blockIdx.x];
    if (A.round != 0 && *A.pending == 0) return;
    if (!A.plan[sd.j].seg) return;
    SegState *st = &A.segstate[sd.j];
    const uint32_t status = st->status;
    const SegSource src = seg_source(A, A.tdesc[sd.j], sd, blockIdx.x, A.dense != 0);
    const uint32_t cs = src.count;
    const uint32_t tid = threadIdx.x;
    if (A.round != 0 && status == SEG_COUNT) {
        // the k-th key T is known (the prefix list had overflowed): count this segment's
        // entries above T and equal to T
        const uint32_t T = st->T;
        uint32_t g = 0, q = 0;
        for (uint32_t e = tid; e < cs; e += SEG_THREADS) {
            const uint32_t key = src.get(e).y & 0x7FFFFFFFu;
            g += (key > T) ? 1u : 0u;
            q += (key == T) ? 1u : 0u;
        }
        const uint32_t G = block_sum(g, wsum, SEG_THREADS / 64);
        const uint32_t Q = block_sum(q, wsum, SEG_THREADS / 64);
        if (tid == 0) {
            A.segG1[blockIdx.x] = G;
            A.segQ[blockIdx.x] = Q;
        }
        return;
    }
    if (status != SEG_ACTIVE + A.round) return;
    const uint32_t pfx = st->pfx;
    uint4 *plist = A.pfxlist + (size_t)A.tdesc[sd.j].pfx_slot * PFX_CAP;
    uint32_t *glow = A.whist + (size_t)sd.j * HBINS;   // low key bits of the entries sharing the prefix
    if (tid == 0) nstage = 0;
    __syncthreads();
    uint32_t g1 = 0;
    for (uint32_t eb = 0; eb < cs; eb += 4 * SEG_THREADS) {
        uint2 ent[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const uint32_t e = eb + u * SEG_THREADS + tid;
            ent[u] = (e < cs) ? src.get(e) : make_uint2(0, 0);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const uint32_t e = eb + u * SEG_THREADS + tid;
            if (e < cs) {
                const uint32_t hi12 = (ent[u].y & 0x7FFFFFFFu) >> SEG_LOWBITS;
                if (hi12 > pfx) {
                    ++g1;
                } else if (hi12 == pfx) {
                    atomicAdd(&glow[ent[u].y & (SEG_LBINS - 1u)], 1u);
                    const uint32_t p = atomicAdd(&nstage, 1u);
                    if (p < PFX_STAGE) stage[p] = ent[u];
                }
            }
        }
    }
    const uint32_t G1 = block_sum(g1, wsum, SEG_THREADS / 64);   // its barriers also complete `stage`
    const uint32_t ns = nstage;
    if (tid == 0) {
        A.segG1[blockIdx.x] = G1;
        // one reservation per segment in the tensor's prefix list; a segment that could not
        // stage all of its entries pushes the count past the capacity, which the ranking
        // kernel turns into a fallback
        if (ns) base = atomicAdd(&st->pfxcount, ns > PFX_STAGE ? PFX_CAP + 1u : ns);
    }
    __syncthreads();
    if (ns && ns <= PFX_STAGE) {
        const uint32_t b0 = base;
        for (uint32_t i = tid; i < ns; i += SEG_THREADS)
            if (b0 + i < PFX_CAP) plist[b0 + i] = make_uint4(stage[i].x, stage[i].y, sd.sidx, 0u);
    }
}

constexpr uint32_t RANK_THREADS = 1024;

__global__ __launch_bounds__(RANK_THREADS) void k_seg_rank(const SegArgs A)
{
    __shared__ uint32_t h[SEG_LBINS];
    __shared__ uint32_t sG[SEG_MAX_PER_TENSOR];
    __shared__ uint32_t sQ[SEG_MAX_PER_TENSOR];
    __shared__ uint32_t rowsum[64];
    __shared__ int res[6];
    __shared__ uint32_t wsum[RANK_THREADS / 64];
    if (A.round != 0 && *A.pending == 0) return;
    const uint32_t j = blockIdx.x;
    const PlanEntry pe = A.plan[j];
    if (!pe.seg) return;
    SegState *st = &A.segstate[j];
    const uint32_t status = st->status;
    // SEG_COUNT (repair round only): the k-th key is known, the prefix kernel has just
    // counted every segment against it
    const bool counted = (A.round != 0) && (status == SEG_COUNT);
    if (status != SEG_ACTIVE + A.round && !counted) return;
    const TensorDesc td = A.tdesc[j];
    const uint32_t tid = threadIdx.x;
    const uint32_t m = st->pfxcount;
    const uint32_t r2 = st->r2, pfx = st->pfx;
    uint32_t T, rT;   // the k-th key; entries equal to it that are taken, lowest index first
    for (uint32_t s = tid; s < td.nseg; s += RANK_THREADS) { sG[s] = 0; sQ[s] = 0; }
    if (counted) {
        T = st->T;
        rT = r2;
        for (uint32_t s = tid; s < td.nseg; s += RANK_THREADS) sQ[s] = A.segQ[td.seg_first + s];
        __syncthreads();
    } else {
        // low key bits of the entries sharing the prefix: counted by the prefix kernel
        uint32_t *gl = A.whist + (size_t)j * HBINS;
        for (uint32_t b = tid; b < SEG_LBINS; b += RANK_THREADS) {
            h[b] = gl[b];
            gl[b] = 0;   // clean for the next use
        }
        find_ranks<SEG_LBINS, RANK_THREADS / 64>(h, r2, 0u, 0u, rowsum, res);
        const int b3 = res[0];
        if (b3 < 0) {   // the rank exceeds what the prefix kernel counted: cannot happen
            if (tid == 0) {
                st->status = SEG_FALLBACK;
                atomicAdd(&A.stats->fallback_tensors, 1ull);
                atomicAdd(&A.stats->fallback_elems, (unsigned long long)td.n);
                atomicAdd(&A.stats->internal_errors, 1ull);
            }
            return;
        }
        T = (pfx << SEG_LOWBITS) | (uint32_t)b3;
        rT = (uint32_t)res[1];
        if (m > PFX_CAP) {
            // too many entries share the prefix for the list: the repair round counts every
            // segment against T instead (a second overflow cannot happen there)
            if (tid == 0) {
                st->T = T;
                st->r2 = rT;
                A.tprev[j] = T;
                if (A.round == 0 && A.repair) {
                    st->status = SEG_COUNT;
                    atomicAdd(A.pending, 1u);
                } else {
                    st->status = SEG_FALLBACK;
                    atomicAdd(&A.stats->fallback_tensors, 1ull);
                    atomicAdd(&A.stats->fallback_elems, (unsigned long long)td.n);
                }
            }
            return;
        }
        const uint4 *plist = A.pfxlist + (size_t)td.pfx_slot * PFX_CAP;
        for (uint32_t p = tid; p < m; p += RANK_THREADS) {
            const uint4 e = plist[p];
            const uint32_t low = e.y & (SEG_LBINS - 1u);
            if (low > (uint32_t)b3) atomicAdd(&sG[e.z], 1u);
            else if (low == (uint32_t)b3) atomicAdd(&sQ[e.z], 1u);
        }
        __syncthreads();
    }
    // segments in order: ties are taken lowest index first, i.e. earlier segments first
    uint32_t carry_q = 0, carry_o = 0;
    for (uint32_t sb = 0; sb < td.nseg; sb += RANK_THREADS) {
        const uint32_t s = sb + tid;
        const bool in = s < td.nseg;
        const uint32_t G = in ? (A.segG1[td.seg_first + s] + sG[s]) : 0u;
        const uint32_t Q = in ? sQ[s] : 0u;
        uint32_t totq, toto;
        const uint32_t qb = carry_q + block_excl_scan<RANK_THREADS / 64>(Q, wsum, totq);
        const uint32_t take = min(Q, (rT > qb) ? (rT - qb) : 0u);
        const uint32_t ob = carry_o + block_excl_scan<RANK_THREADS / 64>(G + take, wsum, toto);
        if (in) A.segOut[td.seg_first + s] = make_uint2(ob, take);
        carry_q += totq;
        carry_o += toto;
    }
    if (tid == 0) {
        st->T = T;
        A.tprev[j] = T;
        if (counted) {
            st->status = SEG_ACTIVE + A.round;
            atomicAdd(&A.stats->repaired_tensors, 1ull);
        }
        if (carry_o != pe.k) atomicAdd(&A.stats->internal_errors, 1ull);
    }
}

template <int OP>
__global__ __launch_bounds__(SEG_THREADS) void k_seg_emit(const SegArgs A)
{
    __shared__ uint32_t wsum[SEG_THREADS / 64];
    const SegDesc sd = A.segtab[blockIdx.x];
    if (A.round != 0 && *A.pending == 0) return;
    const PlanEntry pe = A.plan[sd.j];
    if (!pe.seg) return;
    const SegState *st = &A.segstate[sd.j];
    const uint32_t status = st->status;
    const TensorDesc td = A.tdesc[sd.j];
    const uint32_t tid = threadIdx.x;
    if (A.round == 0 && status == SEG_ALL) {
        // k_j = n_j: every element of the segment is sent, at its own position
        const SegSource all = seg_source(A, td, sd, blockIdx.x, true);
        for (uint32_t e = tid; e < all.count; e += SEG_THREADS) {
            const uint2 ent = all.get(e);
            const uint32_t pos = ent.x - td.off;
            A.out_idx[pe.outoff + pos] = ent.x;
            A.out_val[pe.outoff + pos] = __uint_as_float(ent.y);
            fix_sent<OP>(A.state, ent.x, __uint_as_float(ent.y), A.m);
        }
        return;
    }
    if (status != SEG_ACTIVE + A.round) return;
    const uint32_t T = st->T;
    const uint32_t seg = td.seg_first + sd.sidx;
    const uint2 so = A.segOut[seg];
    const SegSource src = seg_source(A, td, sd, seg, A.dense != 0);
    const uint32_t cs = src.count;
    constexpr uint32_t ITEMS = 4;
    uint32_t run_sel = so.x, run_eq = 0;
    const uint32_t rT = so.y;
    for (uint32_t cb = 0; cb < cs; cb += SEG_THREADS * ITEMS) {
        const uint32_t p0 = cb + tid * ITEMS;
        uint2 v[ITEMS];
        uint32_t g = 0, q = 0;
#pragma unroll
        for (uint32_t i = 0; i < ITEMS; ++i) v[i] = (p0 + i < cs) ? src.get(p0 + i) : make_uint2(0, 0);
#pragma unroll
        for (uint32_t i = 0; i < ITEMS; ++i) {
            const uint32_t key = v[i].y & 0x7FFFFFFFu;
            if (p0 + i < cs) {
                g += (key > T);
                q += (key == T);
            }
        }
        uint32_t total;
        const uint32_t before = block_excl_scan<SEG_THREADS / 64>(g | (q << 16), wsum, total);
        const uint32_t g_before = before & 0xFFFFu, q_before = before >> 16;
        const uint32_t G = total & 0xFFFFu, Q = total >> 16;
        const uint32_t rem = (rT > run_eq) ? (rT - run_eq) : 0u;
        uint32_t pos = run_sel + g_before + min(q_before, rem);
        uint32_t eq_seen = q_before;
        if (g | q) {
#pragma unroll
            for (uint32_t i = 0; i < ITEMS; ++i) {
                if (p0 + i >= cs) break;
                const uint32_t key = v[i].y & 0x7FFFFFFFu;
                bool sel = key > T;
                if (key == T) {
                    sel = eq_seen < rem;
                    ++eq_seen;
                }
                if (sel) {
                    if (pos < pe.k) {
                        A.out_idx[pe.outoff + pos] = v[i].x;
                        A.out_val[pe.outoff + pos] = __uint_as_float(v[i].y);
                        fix_sent<OP>(A.state, v[i].x, __uint_as_float(v[i].y), A.m);
                    }
                    ++pos;
                }
            }
        }
        run_sel += G + min(Q, rem);
        run_eq += Q;
    }
}

// Repair round: the streaming pass again, read-only, over the segments of the tensors
// left SEG_PENDING -- a histogram pass (MODE_HIST, counting the segment's own tensor
// only) and, after k_pick, a collecting pass (MODE_COLLECT) with the fresh threshold.
// A border tile shared with a neighbouring tensor is rewritten whole; the neighbour's
// candidates in it are no longer needed by then (its selection is complete, or it is
// pending too and rewrites the same values).
template <int OP, int MODE, bool VEC>
__global__ __launch_bounds__(STREAM_THREADS) void k_seg_restream(const StreamArgs A, const SegArgs G,
                                                                const uint32_t *__restrict__ toff,
                                                                const uint32_t *__restrict__ tau)
{
    __shared__ uint32_t lhist[MODE == MODE_HIST ? HBINS : 1];
    __shared__ uint2 stage_all[MODE == MODE_COLLECT ? WAVES_PER_BLOCK * STAGE : 1];
    if (*G.pending == 0) return;
    const SegDesc sd = G.segtab[blockIdx.x];
    if (!G.plan[sd.j].seg || G.segstate[sd.j].status != SEG_PENDING) return;
    if (MODE == MODE_HIST) {
        for (uint32_t b = threadIdx.x; b < HBINS; b += STREAM_THREADS) lhist[b] = 0;
        __syncthreads();
    }
    const uint32_t wave = uniform(threadIdx.x >> 6);
    uint2 *stage = stage_all + (MODE == MODE_COLLECT ? wave * STAGE : 0u);
    for (uint32_t i = wave; i < sd.ntiles; i += WAVES_PER_BLOCK)
        process_tile<OP, MODE, VEC>(A, toff, tau, sd.tile0 + i, lhist, (int)sd.j, stage, (int)sd.j);
    flush_hist<MODE>(lhist, A.ghist, (int)sd.j);
}

template <int OP>
static void launch_seg_recollect_t(const StreamArgs &a, bool vec, const SegArgs &g, hipStream_t st)
{
    const dim3 grid(g.nseg_total), block(STREAM_THREADS);
    if (vec) hipLaunchKernelGGL((k_seg_restream<OP, MODE_HIST, true>), grid, block, 0, st, a, g, a.toff, a.tau);
    else hipLaunchKernelGGL((k_seg_restream<OP, MODE_HIST, false>), grid, block, 0, st, a, g, a.toff, a.tau);
    launch_pick(g.tdesc, g.plan, a.ghist, g.tau, g.tprev, g.stats, g.J, st, g.segstate, g.pending);
    if (vec) hipLaunchKernelGGL((k_seg_restream<OP, MODE_COLLECT, true>), grid, block, 0, st, a, g, a.toff, a.tau);
    else hipLaunchKernelGGL((k_seg_restream<OP, MODE_COLLECT, false>), grid, block, 0, st, a, g, a.toff, a.tau);
}

// op: OP_IDENT (the values are in `state`) or OP_SUB (model - state)
void launch_seg_recollect(int op, const StreamArgs &a, bool vec, const SegArgs &g, void *stream)
{
    if (g.nseg_total == 0) return;
    if (op == OP_SUB) launch_seg_recollect_t<OP_SUB>(a, vec, g, (hipStream_t)stream);
    else launch_seg_recollect_t<OP_IDENT>(a, vec, g, (hipStream_t)stream);
}

void launch_segmented(int op, const SegArgs &a, void *stream, void *ev0, void *ev1)
{
    hipStream_t st = (hipStream_t)stream;
    if (a.nseg_total == 0) return;
    launch_k(k_seg_join, dim3(a.nseg_total), dim3(SEG_THREADS), st, ev0, nullptr, a);
    if (op == SEL_WORKER)
        launch_k(k_seg_window<SEL_WORKER>, dim3(a.J), dim3(SEG_THREADS), st, nullptr, nullptr, a);
    else   // both kinds of pull share the hint policy
        launch_k(k_seg_window<SEL_PULL>, dim3(a.J), dim3(SEG_THREADS), st, nullptr, nullptr, a);
    launch_k(k_seg_prefix, dim3(a.nseg_total), dim3(SEG_THREADS), st, nullptr, nullptr, a);
    launch_k(k_seg_rank, dim3(a.J), dim3(RANK_THREADS), st, nullptr, nullptr, a);
    if (op == SEL_WORKER)
        launch_k(k_seg_emit<SEL_WORKER>, dim3(a.nseg_total), dim3(SEG_THREADS), st, nullptr, ev1, a);
    else if (op == SEL_PULL)
        launch_k(k_seg_emit<SEL_PULL>, dim3(a.nseg_total), dim3(SEG_THREADS), st, nullptr, ev1, a);
    else
        launch_k(k_seg_emit<SEL_PULL_V>, dim3(a.nseg_total), dim3(SEG_THREADS), st, nullptr, ev1, a);
}

void launch_select(int op, const SelectArgs &a, uint32_t J, void *stream, void *ev0, void *ev1)
{
    hipStream_t st = (hipStream_t)stream;
    if (op == SEL_WORKER)
        launch_k(k_select<SEL_WORKER>, dim3(J), dim3(SEL_THREADS), st, ev0, ev1, a, a.tile_cnt, a.heads,
                 a.slots);
    else if (op == SEL_PULL)
        launch_k(k_select<SEL_PULL>, dim3(J), dim3(SEL_THREADS), st, ev0, ev1, a, a.tile_cnt, a.heads, a.slots);
    else
        launch_k(k_select<SEL_PULL_V>, dim3(J), dim3(SEL_THREADS), st, ev0, ev1, a, a.tile_cnt, a.heads, a.slots);
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
    if (i < n) store_scattered(&dst[i], dst[i] - val[e]);
}

void launch_push(float *model, float *diff, uint32_t W, uint32_t n, const uint32_t *idx,
                 const float *val, uint32_t nnz, void *stream, void *ev0, void *ev1)
{
    if (nnz == 0) return;
    const uint32_t first = model ? 0u : 1u;
    const uint32_t bufs = W + 1 - first;
    if (bufs == 0) return;
    // gridDim.y is limited to 65535: loop over slabs of buffers
    for (uint32_t b0 = 0; b0 < bufs; b0 += 32768) {
        const uint32_t nb = (bufs - b0 < 32768u) ? (bufs - b0) : 32768u;
        // events time the first slab only (one slab unless there are more than 32768 buffers)
        launch_k(k_push, dim3((nnz + 255) / 256, nb), dim3(256), (hipStream_t)stream,
                 b0 == 0 ? ev0 : nullptr, b0 == 0 ? ev1 : nullptr, model, diff, n, idx, val, nnz,
                 first + b0);
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

// ---------------------------------------------------------------------------
// wire form of a message: fp32 values, then per tensor its local indices bit-packed
// ---------------------------------------------------------------------------

// Last tensor whose `field` (ascending over the tensors) is <= x.
template <uint32_t PlanEntry::*FIELD>
__device__ __forceinline__ uint32_t plan_search(const PlanEntry *plan, uint32_t J, uint32_t x)
{
    uint32_t lo = 0, hi = J;                 // invariant: plan[lo].FIELD <= x, answer in [lo, hi)
    while (hi - lo > 1) {
        const uint32_t mid = (lo + hi) >> 1;
        if (plan[mid].*FIELD <= x) lo = mid; else hi = mid;
    }
    return lo;                               // offsets increase strictly: every tensor has k_j >= 1
}

// One thread per value (copied) and per 32-bit word of the index area: the word gathers the
// pieces of the entries that overlap it (entry e of tensor j covers bits [e b_j, (e + 1) b_j)
// of the tensor's block).  Out-of-tensor indices are masked to b_j bits and, with `flag`, reported.
__global__ __launch_bounds__(256) void k_wire_pack(const TensorDesc *tdesc, const PlanEntry *plan, uint32_t J,
                                                   uint32_t K, uint32_t words, const uint32_t *idx,
                                                   const float *val, uint32_t *wire, uint32_t *flag)
{
    const uint64_t t = (uint64_t)blockIdx.x * 256 + threadIdx.x;
    if (t < K) {
        wire[t] = __float_as_uint(val[t]);
        return;
    }
    if (t >= (uint64_t)K + words) return;
    const uint32_t w = (uint32_t)(t - K);
    const uint32_t j = plan_search<&PlanEntry::wire_off>(plan, J, w);
    const PlanEntry pe = plan[j];
    const TensorDesc td = tdesc[j];
    const uint32_t b = pe.wire_bits;
    const uint64_t bit0 = (uint64_t)(w - pe.wire_off) * 32u;           // first bit of this word in the block
    const uint64_t e0 = bit0 / b;
    if (e0 >= pe.k) { wire[t] = 0; return; }                           // cannot happen: blocks end with their last entry
    const uint64_t e1 = min((uint64_t)pe.k - 1u, (bit0 + 31u) / b);
    const uint32_t mask = (b >= 32u) ? 0xFFFFFFFFu : ((1u << b) - 1u);
    uint32_t word = 0;
    bool bad = false;
    for (uint64_t e = e0; e <= e1; ++e) {
        const uint32_t local = idx[pe.outoff + e] - td.off;
        bad |= local >= td.n;
        const uint64_t pos = e * b;
        const uint32_t piece = local & mask;
        word |= (pos >= bit0) ? (piece << (uint32_t)(pos - bit0)) : (piece >> (uint32_t)(bit0 - pos));
    }
    wire[t] = word;
    if (bad && flag) atomicOr(flag, 1u);
}

// One thread per entry: value copied, local index cut out of one or two words of its block.
__global__ __launch_bounds__(256) void k_wire_unpack(const TensorDesc *tdesc, const PlanEntry *plan, uint32_t J,
                                                     uint32_t K, const uint32_t *wire, uint32_t *idx,
                                                     float *val, uint32_t *flag)
{
    const uint64_t t = (uint64_t)blockIdx.x * 256 + threadIdx.x;
    if (t >= K) return;
    val[t] = __uint_as_float(wire[t]);
    const uint32_t j = plan_search<&PlanEntry::outoff>(plan, J, (uint32_t)t);
    const PlanEntry pe = plan[j];
    const TensorDesc td = tdesc[j];
    const uint32_t b = pe.wire_bits;
    const uint64_t pos = (uint64_t)((uint32_t)t - pe.outoff) * b;
    const uint32_t *block = wire + K + pe.wire_off;
    const uint32_t w = (uint32_t)(pos >> 5), sh = (uint32_t)(pos & 31u);
    uint64_t x = block[w];
    if (sh + b > 32u) x |= (uint64_t)block[w + 1] << 32;              // an entry that crosses ends inside the block
    const uint32_t mask = (b >= 32u) ? 0xFFFFFFFFu : ((1u << b) - 1u);
    const uint32_t local = (uint32_t)(x >> sh) & mask;
    idx[t] = td.off + local;
    if (local >= td.n && flag) atomicOr(flag, 1u);
}

void launch_wire_pack(const TensorDesc *tdesc, const PlanEntry *plan, uint32_t J, uint32_t K, uint32_t words,
                      const uint32_t *idx, const float *val, uint32_t *wire, uint32_t *flag, void *stream,
                      void *ev0, void *ev1)
{
    const uint64_t threads = (uint64_t)K + words;
    if (threads == 0) return;
    launch_k(k_wire_pack, dim3((uint32_t)((threads + 255) / 256)), dim3(256), (hipStream_t)stream, ev0, ev1,
             tdesc, plan, J, K, words, idx, val, wire, flag);
}

void launch_wire_unpack(const TensorDesc *tdesc, const PlanEntry *plan, uint32_t J, uint32_t K,
                        const uint32_t *wire, uint32_t *idx, float *val, uint32_t *flag, void *stream,
                        void *ev0, void *ev1)
{
    if (K == 0) return;
    launch_k(k_wire_unpack, dim3((K + 255) / 256), dim3(256), (hipStream_t)stream, ev0, ev1, tdesc, plan, J, K,
             wire, idx, val, flag);
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
// pull without secondary compression: every nonzero of one difference row, or of
// model - sent_k when a model is given (the server state as Algorithm 2 prints it)
// ---------------------------------------------------------------------------

__device__ __forceinline__ void load_tile_guarded(const float *row, const float *model, uint32_t base,
                                                  uint32_t n, float (&a)[4][4])
{
    const uint32_t lane = lane_id();
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint32_t e = base + r * 256 + lane * 4 + j;
            a[r][j] = (e < n) ? (model ? model[e] - row[e] : row[e]) : 0.0f;
        }
}

__global__ __launch_bounds__(STREAM_THREADS) void k_pull_all_count(const float *row, const float *model,
                                                                   uint32_t n, uint32_t ntiles,
                                                                   uint32_t *tile_cnt)
{
    const uint32_t t = blockIdx.x * WAVES_PER_BLOCK + (threadIdx.x >> 6);
    if (t >= ntiles) return;
    float a[4][4];
    load_tile_guarded(row, model, t * TILE, n, a);
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

// What is sent leaves the row as +0 (D_k -= G), or is added to it (sent_k += G, Eq. 6).
__global__ __launch_bounds__(STREAM_THREADS) void k_pull_all_emit(float *row, const float *model, uint32_t n,
                                                                  uint32_t ntiles, const uint32_t *tile_pos,
                                                                  uint32_t *out_idx, float *out_val)
{
    const uint32_t t = blockIdx.x * WAVES_PER_BLOCK + (threadIdx.x >> 6);
    if (t >= ntiles) return;
    const uint32_t lane = lane_id();
    const uint32_t base = t * TILE;
    float a[4][4];
    load_tile_guarded(row, model, base, n, a);
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
                    store_scattered(&row[e], model ? row[e] + a[r][j] : 0.0f);
                    ++p;
                }
            }
            run += (uint32_t)(__popcll(mk[0]) + __popcll(mk[1]) + __popcll(mk[2]) + __popcll(mk[3]));
        }
    }
}

void launch_pull_all_count(const float *row, const float *model, uint32_t n, uint32_t ntiles,
                           uint32_t *tile_cnt, void *stream)
{
    hipLaunchKernelGGL(k_pull_all_count, dim3((ntiles + WAVES_PER_BLOCK - 1) / WAVES_PER_BLOCK),
                       dim3(STREAM_THREADS), 0, (hipStream_t)stream, row, model, n, ntiles, tile_cnt);
}

void launch_pull_all_scan(uint32_t *tile_cnt, uint32_t ntiles, uint32_t *total, void *stream)
{
    hipLaunchKernelGGL(k_pull_all_scan, dim3(1), dim3(1024), 0, (hipStream_t)stream, tile_cnt, ntiles, total);
}

void launch_pull_all_emit(float *row, const float *model, uint32_t n, uint32_t ntiles,
                          const uint32_t *tile_pos, uint32_t *out_idx, float *out_val, void *stream)
{
    hipLaunchKernelGGL(k_pull_all_emit, dim3((ntiles + WAVES_PER_BLOCK - 1) / WAVES_PER_BLOCK),
                       dim3(STREAM_THREADS), 0, (hipStream_t)stream, row, model, n, ntiles, tile_pos, out_idx,
                       out_val);
}

}  // namespace dgs
