// One tile (1024 consecutive elements) of the streaming pass, as one wavefront processes it:
// loads, fused accumulate (Algorithm 3, "u <- m u + eta grad"), magnitude keys, and either
// candidate collection against the per-tensor thresholds or the LDS histogram of the keys.
// Shared by the full pass (k_stream) and the per-segment re-collection (k_seg_restream).
#pragma once
#include "dgs_wave.h"

namespace dgs {

// ---------------------------------------------------------------------------
// streaming pass
// ---------------------------------------------------------------------------

template <int MODE>
__device__ __forceinline__ void flush_hist(uint32_t *lhist, uint32_t *ghist, int cur)
{
    if (MODE != MODE_HIST && MODE != MODE_SAMPLE) return;
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
    } else {  // MODE_HIST, MODE_SAMPLE
        const bool bigA = (d.x >> 31) != 0, bigB = (d.y >> 31) != 0;
        uint32_t zeroA = 0, zeroB = 0;     // MODE_SAMPLE: zero keys of the two tensors, added once per tile
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
                if (key == 0) {
                    // zeros (often the bulk of a difference row) are implied; a sample counts
                    // them, so that the counters of a tensor add up to what was sampled of it
                    if (MODE == MODE_SAMPLE) {
                        if (e < endA) ++zeroA;
                        else ++zeroB;
                    }
                    continue;
                }
                const uint32_t bin = key >> HSHIFT;
                if (tt == cur) atomicAdd(&lhist[bin], 1u);
                else atomicAdd(&A.ghist[(size_t)tt * HBINS + bin], 1u);
            }
        }
        if (MODE == MODE_SAMPLE) {
            zeroA = wave_sum(zeroA);
            zeroB = wave_sum(zeroB);
            if (lane == 0) {
                if (zeroA) {
                    if ((int)tA == cur) atomicAdd(&lhist[0], zeroA);
                    else atomicAdd(&A.ghist[(size_t)tA * HBINS], zeroA);
                }
                if (zeroB) {
                    if ((int)tB == cur) atomicAdd(&lhist[0], zeroB);
                    else atomicAdd(&A.ghist[(size_t)tB * HBINS], zeroB);
                }
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
        // Non-temporal like the gradient: a pass that allocates what it streams in the
        // last-level cache pushes out the dirty lines earlier kernels left there and waits for
        // their write-back.  Measured: a cold 433 MB server row takes 131 us with plain loads
        // and 66 us with non-temporal ones; the worker pass over 1e9 parameters 2255 us against
        // 2165 us; buffers small enough to stay cached (102 MB) lose nothing.
#pragma unroll
        for (int r = 0; r < 4; ++r)
            s[r] = __builtin_nontemporal_load((const f32x4 *)(A.state + base + r * 256 + lane * 4));
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
        if (OP == OP_FMA && MODE != MODE_SAMPLE) {
            // How the state goes back (measured on the accumulate pass, 25.6M / 1e9 parameters):
            // plain write-back stores 47.3 / 2131 us; device-scope write-through 45.3 / 2035 us;
            // non-temporal 48.8 / 1951 us.  Write-through for buffers that fit the last-level
            // cache, non-temporal beyond.
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                f32x4 o;
#pragma unroll
                for (int j = 0; j < 4; ++j) o[j] = a[r][j];
                float *dst = A.state + base + r * 256 + lane * 4;
                if (A.store_mode == STORE_NT) __builtin_nontemporal_store(o, (f32x4 *)dst);
                else if (A.store_mode == STORE_WT) store_through16(A.state + uniform(base), (r * 256 + lane * 4) * 4u, o);
                else *(f32x4 *)dst = o;
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
                    if (MODE != MODE_SAMPLE) A.state[e] = v;
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

}  // namespace dgs
