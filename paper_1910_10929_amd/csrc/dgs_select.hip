// Pick (histogram -> candidate threshold) and the selection kernel of libdgs: per tensor the
// exact k-th largest magnitude with the lowest-index tie rule ("thr <- R% of |x|" in
// Algorithms 1-3), the ordered emission ("encode()"), the state fix-up (Eq. 12 / Eq. 6) and
// the next threshold hint -- all tensors in one launch.
#include "dgs_select.h"

namespace dgs {

// ---------------------------------------------------------------------------
// pick: key histogram (bits [30:19], nonzero keys only) -> candidate threshold
// ---------------------------------------------------------------------------

// h: HBINS counters in LDS.  Thread 0 receives the threshold whose candidates number at
// least pe.k2 (or every nonzero when there are fewer), and the middle of the bucket that holds
// the k-th key (anchors the window histograms).  Contains find_ranks' three barriers.
template <int NW>
__device__ __forceinline__ void pick_from_hist(const uint32_t *h, const PlanEntry &pe, uint32_t *rowsum, int *res,
                                               uint32_t &tau_out, uint32_t &tprev_out)
{
    find_ranks<HBINS, NW>(h, pe.k2, pe.k, 0u, rowsum, res);
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
    tau_out = t;
    tprev_out = (b1 >= 0) ? (((uint32_t)b1 << HSHIFT) + (1u << (HSHIFT - 1))) : 0u;
}

// sample != 0: the histogram is that of a sample of the tensor, zero keys included (its total is
// the number of sampled elements).  The ranks shrink with the sampled share; the candidate rank
// aims at 2 k instead of the plan's and gets two standard deviations of slack on top, since a
// threshold that lets too few through costs a second collection and one that lets a few more
// through costs nothing.  A tensor that was sampled completely keeps the plan's ranks.
__global__ __launch_bounds__(256) void k_pick(const TensorDesc *tdesc, const PlanEntry *plan,
                                              uint32_t *ghist, uint32_t *tau, uint32_t *tprev,
                                              DevStats *stats, uint32_t sample)
{
    const uint32_t j = blockIdx.x;
    if (!tdesc[j].big) return;
    __shared__ uint32_t h[HBINS];
    __shared__ uint32_t rowsum[64];
    __shared__ int res[6];
    __shared__ uint32_t wsum[4];
    uint32_t *g = ghist + (size_t)j * HBINS;
    uint32_t mine = 0;
    for (uint32_t b = threadIdx.x; b < HBINS; b += 256) {
        const uint32_t v = g[b];
        h[b] = v;
        mine += v;
        g[b] = 0;   // leave the histogram clean for the next use
    }
    PlanEntry pe = plan[j];
    if (sample) {
        const uint32_t total = block_sum(mine, wsum, 4);
        // from here on the histogram is that of the nonzero keys, as in a full pass (bucket 0 held
        // the zeros; keys below 2^19, denormals of about 1e-39, go with them)
        if (threadIdx.x == 0) h[0] = 0;
        __syncthreads();
        const uint32_t n = tdesc[j].n;
        if (total < n) {
            const double share = (double)total / (double)n;
            const double want = share * (double)min(2u * pe.k, n);
            const uint32_t k2s = (uint32_t)ceil(want + 2.0 * sqrt(want)) + 1u;
            pe.k2 = max(1u, min(k2s, total));
            pe.k = max(1u, min((uint32_t)ceil(share * (double)pe.k), pe.k2));
        }
    }
    uint32_t t, tp;
    pick_from_hist<4>(h, pe, rowsum, res, t, tp);
    if (sample) {
        // A sample that holds fewer nonzeros than the scaled k says nothing about where the k-th
        // key lies, except that it cannot be far above the smallest nonzero seen: that bucket
        // anchors the window histograms then (a full pass knows the bucket itself).
        __shared__ uint32_t lowbin;
        if (threadIdx.x == 0) lowbin = 0xFFFFFFFFu;
        __syncthreads();
        uint32_t mine_low = 0xFFFFFFFFu;
        for (uint32_t b = 1 + threadIdx.x; b < HBINS; b += 256)
            if (h[b] != 0) { mine_low = b; break; }
        if (mine_low != 0xFFFFFFFFu) atomicMin(&lowbin, mine_low);
        __syncthreads();
        if (tp == 0 && lowbin != 0xFFFFFFFFu) tp = (lowbin << HSHIFT) + (1u << (HSHIFT - 1));
    }
    if (threadIdx.x == 0) {
        tau[j] = t;
        tprev[j] = tp;
    }
}

void launch_pick(const TensorDesc *tdesc, const PlanEntry *plan, uint32_t *ghist, uint32_t *tau,
                 uint32_t *tprev, DevStats *stats, uint32_t J, bool sample, void *stream)
{
    hipLaunchKernelGGL(k_pick, dim3(J), dim3(256), 0, (hipStream_t)stream, tdesc, plan, ghist, tau, tprev,
                       stats, sample ? 1u : 0u);
}

// ---------------------------------------------------------------------------
// the selection kernel
// ---------------------------------------------------------------------------
//
// Grid: block b < G is the JOIN of join group b (1024 threads; a group is a tensor, or up to
// GROUP_TILES tiles of one).  With the re-collecting roles enabled, nb = ceil(P / bgroup)
// RE-HISTOGRAM blocks follow (P: the number of parts), then as many RE-COLLECTION blocks; block
// b of a role looks after parts b, b + nb, b + 2 nb, ... in turn, so the parts of one tensor
// lie in different blocks.  These blocks act on tensors of several parts whose prediction
// failed, and pass over everything else.
//
//   JOIN      compacts the candidates the streaming pass left in the part's tiles into one
//             ordered list.  The workgroup that arrives last for a tensor (the only one, for a
//             tensor of one part) gathers the parts' lists and SELECTS: exact k-th key, ordered
//             emission, state fix-up, next hint.  A tensor planned for the chain kernels only
//             gets its key window resolved here.  Lists that are complete but beyond one
//             workgroup's reach are trimmed on the way (threshold from their own histogram).
//             If the prediction failed otherwise (fewer candidates than k, an overflowed tile)
//             the tensor is left pending: a tensor of one part is collected again on the spot,
//             for the others the verdict releases the waiting roles.
//   RE-HISTOGRAM  every part counts the keys of its own elements; the last one derives a fresh
//             threshold and publishes it.
//   RE-COLLECTION every part compacts its elements at or above that threshold straight from
//             the buffers into its list; the last one selects as above.  What still fails then
//             (one value filling the tensor, say) is selected from the buffers by that one
//             workgroup -- slow, never wrong.
//
// Waiting is only ever for blocks with a lower index, which the hardware dispatches first,
// and every wait is bounded (A.spin_limit polls).

constexpr uint32_t B_GROUP_MAX = 8;   // most parts one re-collecting workgroup looks after

struct PartShared {
    SelShared S;
    uint32_t pbase[SEG_MAX_PER_TENSOR + 1];   // first list position of every part of the tensor
    uint32_t pofs[SEG_MAX_PER_TENSOR];        // where every part's global list starts (entries into ord)
    uint32_t wtot[SEL_WAVES];
    uint32_t vbuf[B_GROUP_MAX];               // verdicts of the tensors of a re-collecting workgroup's parts
    uint32_t tile_pos[SEL_THREADS];           // JOIN: list position and count of every tile of the round
    uint32_t tile_n[SEL_THREADS];             //       (bit 31: the tile's entries are fetched one by one)
    uint32_t start0;                          //       entries of the previous tensor in a shared first tile
    uint32_t crowd_slot[SEL_THREADS];         //       the round's crowded tiles (which lane has them)
    uint32_t bc;
};

// Entry e of a crowded or border tile: heads for q < HEAD, slots beyond.
__device__ __forceinline__ uint2 tile_entry(const uint2 *hd, const uint2 *sl, uint32_t q)
{
    return (q < HEAD) ? hd[q] : sl[q];
}

// What a tile's counter word says about tensor td's candidates in tile t: how many, and after
// how many of the previous tensor's (a first tile shared with it).  An overflowed tile, or a
// count beyond the slots (a corrupted word), sets ovf and counts as empty.
__device__ __forceinline__ void tile_counts(uint32_t w, uint32_t t, uint32_t tlo, bool head_shared, uint32_t &n_t,
                                            uint32_t &start, int &ovf)
{
    n_t = 0;
    start = 0;
    if (w == CNT_OVERFLOW) {
        ovf = 1;
    } else if (head_shared && t == tlo) {
        start = w & 0xFFFFu;      // the previous tensor's candidates come first in this tile
        n_t = w >> 16;
    } else {
        n_t = w & 0xFFFFu;
    }
    if (start + n_t > CAPT) {
        ovf = 1;
        n_t = 0;
        start = 0;
    }
}

// JOIN of a run of tiles: the candidates of tensor j in tiles [sd.tile0, sd.tile0 + sd.ntiles),
// in index order, through `put(position, entry)`.  Returns the count; `ovf` is set if a tile had
// overflowed its slots.  Rounds of SEL_THREADS tiles.  Every lane takes one tile's count; a
// workgroup scan of the counts gives every tile its list position.  The tiles' first lines (8
// candidates, 64 bytes) are fetched as the contiguous stretch they are -- four lanes per line,
// four lines per lane -- and put in place with the positions read back from LDS; crowded tiles
// and a first tile shared with the previous tensor go to a worklist that the wavefronts then
// copy entry by entry.
struct NoTileHook {
    __device__ __forceinline__ void operator()(uint32_t, uint32_t) const {}
};

// (`at_tile(tile index within the run, list position)` is called once for every tile.)
template <class Put, class AtTile = NoTileHook>
__device__ __forceinline__ uint32_t join_part(const SelectArgs &A, const TensorDesc &td, const SegDesc &sd,
                                              PartShared &P, bool &ovf_out, Put put, AtTile at_tile = AtTile())
{
    const uint32_t tid = threadIdx.x, wave = tid >> 6, lane = tid & 63u;
    const uint32_t tlo = td.off / TILE;
    const bool head_shared = (td.off % TILE) != 0;
    uint32_t base = 0;
    int ovf = 0;
    for (uint32_t r0 = 0; r0 < sd.ntiles; r0 += SEL_THREADS) {
        // lines of this wavefront's 64 tiles: load v covers tiles 16 v .. 16 v + 15
        uint4 pf[4];
#pragma unroll
        for (uint32_t v = 0; v < 4; ++v) {
            const uint32_t tl = r0 + wave * 64u + v * 16u + (lane >> 2);
            pf[v] = (tl < sd.ntiles) ? ((const uint4 *)(A.heads + (size_t)(sd.tile0 + tl) * HEAD))[lane & 3u]
                                     : make_uint4(0, 0, 0, 0);
        }
        const uint32_t t = sd.tile0 + r0 + tid;
        const uint32_t w = (r0 + tid < sd.ntiles) ? A.tile_cnt[t] : 0u;
        uint32_t n_t, start;
        tile_counts(w, t, tlo, head_shared, n_t, start, ovf);
        // one scan for both: list positions (low 19 bits: at most 2^18 candidates a round) and the
        // number of crowded tiles (the bits above)
        const bool crowded = n_t != 0 && (start != 0 || n_t > HEAD);
        uint32_t total;
        const uint32_t excl = block_excl_scan<SEL_WAVES>(n_t | (crowded ? 1u << 19 : 0u), P.S.wsum, total);
        const uint32_t pos = base + (excl & 0x7FFFFu);
        const uint32_t nc = total >> 19, round_n = total & 0x7FFFFu;
        P.tile_pos[tid] = pos;
        P.tile_n[tid] = n_t | (crowded ? 0x80000000u : 0u);
        if (crowded) P.crowd_slot[excl >> 19] = tid;
        if (head_shared && t == tlo) P.start0 = start;      // (the tensor's first tile, shared with the one before)
        if (r0 + tid < sd.ntiles) at_tile(r0 + tid, pos);
        __syncthreads();
#pragma unroll
        for (uint32_t v = 0; v < 4; ++v) {
            const uint32_t slot = wave * 64u + v * 16u + (lane >> 2);
            const uint32_t nv = P.tile_n[slot], p = P.tile_pos[slot], e0 = 2u * (lane & 3u);
            const uint32_t n = (nv >> 31) ? 0u : nv;
            if (e0 < n) put(p + e0, make_uint2(pf[v].x, pf[v].y));
            if (e0 + 1 < n) put(p + e0 + 1, make_uint2(pf[v].z, pf[v].w));
        }
        if (nc != 0 && nc <= 2 * SEL_WAVES) {
            // a few crowded tiles: a wavefront copies one at a time
            for (uint32_t q = wave; q < nc; q += SEL_WAVES) {
                const uint32_t slot = P.crowd_slot[q], tc = sd.tile0 + r0 + slot;
                const uint32_t n_c = P.tile_n[slot] & 0x7FFFFFFFu, pc = P.tile_pos[slot];
                const uint32_t st0 = (head_shared && tc == tlo) ? P.start0 : 0u;
                const uint2 *hd = A.heads + (size_t)tc * HEAD;
                const uint2 *sl = A.slots + (size_t)tc * CAPT;
                for (uint32_t i = lane; i < n_c; i += 64) put(pc + i, tile_entry(hd, sl, st0 + i));
            }
        } else if (nc != 0) {
            // many crowded tiles: every list position of the round finds its tile (the last one
            // that starts at or before it) and, if that tile is crowded, fetches its own entry
            constexpr uint32_t CU = 4;      // entries per thread in flight
            for (uint32_t q0 = 0; q0 < round_n; q0 += CU * SEL_THREADS) {
                uint2 e[CU];
                bool take[CU];
#pragma unroll
                for (uint32_t u = 0; u < CU; ++u) {
                    const uint32_t q = base + q0 + u * SEL_THREADS + tid;
                    take[u] = false;
                    e[u] = make_uint2(0, 0);
                    if (q0 + u * SEL_THREADS + tid < round_n) {
                        uint32_t lo = 0, hi = SEL_THREADS;
                        while (hi - lo > 1) {
                            const uint32_t mid = (lo + hi) >> 1;
                            if (P.tile_pos[mid] <= q) lo = mid;
                            else hi = mid;
                        }
                        if (P.tile_n[lo] >> 31) {
                            const uint32_t tc = sd.tile0 + r0 + lo;
                            const uint32_t st0 = (head_shared && tc == tlo) ? P.start0 : 0u;
                            take[u] = true;
                            e[u] = tile_entry(A.heads + (size_t)tc * HEAD, A.slots + (size_t)tc * CAPT,
                                              st0 + (q - P.tile_pos[lo]));
                        }
                    }
                }
#pragma unroll
                for (uint32_t u = 0; u < CU; ++u)
                    if (take[u]) put(base + q0 + u * SEL_THREADS + tid, e[u]);
            }
        }
        base += round_n;
        // (the next round rewrites the positions behind the two barriers of its scan)
    }
    ovf_out = __syncthreads_or(ovf) != 0;
    return base;
}

// Elements of tensor j inside the part, as rows of 256 consecutive elements per wavefront
// (4 per lane): the wavefronts take the part's tiles in equal consecutive runs, so that the
// order of wavefronts is the order of indices.
struct DenseRun {
    uint32_t t0, t1;     // this wavefront's tiles [t0, t1) of the flat buffer
    uint32_t lo, hi;     // the tensor's elements [lo, hi)
};

__device__ __forceinline__ DenseRun dense_run(const TensorDesc &td, const SegDesc &sd)
{
    const uint32_t wave = threadIdx.x >> 6;
    const uint32_t per = (sd.ntiles + SEL_WAVES - 1) / SEL_WAVES;
    DenseRun r;
    r.t0 = sd.tile0 + min(wave * per, sd.ntiles);
    r.t1 = sd.tile0 + min((wave + 1) * per, sd.ntiles);
    r.lo = td.off;
    r.hi = td.off + td.n;
    return r;
}

// The four consecutive elements e0 .. e0 + 3 (e0 a multiple of 4) of the ranked row as bit
// patterns, and which of them belong to the tensor [lo, hi): one 16-byte load per buffer where
// the quad lies inside the tensor and the buffers are 16-byte aligned (`vec`), element by
// element at a tensor border or off alignment.
template <int OP>
__device__ __forceinline__ uint32_t quad_bits(const SelectArgs &A, uint32_t e0, uint32_t lo, uint32_t hi, bool vec,
                                              uint32_t (&bits)[4])
{
    if (vec && e0 >= lo && e0 + 3u < hi) {
        f32x4 v = *(const f32x4 *)(A.state + e0);
        if (OP == SEL_PULL_V) v = *(const f32x4 *)(A.model + e0) - v;      // one fp32 subtraction per element
        bits[0] = __float_as_uint(v.x);
        bits[1] = __float_as_uint(v.y);
        bits[2] = __float_as_uint(v.z);
        bits[3] = __float_as_uint(v.w);
        return 0xFu;
    }
    uint32_t in = 0;
#pragma unroll
    for (int x = 0; x < 4; ++x) {
        const uint32_t e = e0 + x;
        const bool ok = e >= lo && e < hi;
        bits[x] = ok ? __float_as_uint(row_value<OP>(A.state, A.model, e)) : 0u;
        in |= ok ? (1u << x) : 0u;
    }
    return in;
}

__device__ __forceinline__ bool rows_aligned(const SelectArgs &A)
{
    return (((uintptr_t)A.state | (uintptr_t)A.model) & 15u) == 0;   // (a null model counts as aligned)
}

// RE-HISTOGRAM of one part: key bits [30:19] of the tensor's nonzero elements in the part,
// into lh (HBINS counters in LDS, zeroed here).  Ends with a barrier.
template <int OP>
__device__ __forceinline__ void dense_hist(const SelectArgs &A, const TensorDesc &td, const SegDesc &sd, uint32_t *lh)
{
    for (uint32_t b = threadIdx.x; b < HBINS; b += SEL_THREADS) lh[b] = 0;
    __syncthreads();
    const DenseRun r = dense_run(td, sd);
    const uint32_t lane = lane_id();
    const bool vec = rows_aligned(A);
    // two tiles per turn, all of their loads issued before the first counter is touched (the odd
    // last turn reads its one tile twice and counts it once)
    for (uint32_t t = r.t0; t < r.t1; t += 2) {
        const bool two = t + 1 < r.t1;
        uint32_t bits[2][4][4];
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int row = 0; row < 4; ++row)
                quad_bits<OP>(A, (u && two ? t + 1 : t) * TILE + row * 256 + lane * 4, r.lo, r.hi, vec, bits[u][row]);
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int row = 0; row < 4; ++row)
#pragma unroll
                for (int x = 0; x < 4; ++x) {
                    const uint32_t key = bits[u][row][x] & 0x7FFFFFFFu;      // elements outside the tensor read as 0
                    if (key != 0 && (u == 0 || two)) atomicAdd(&lh[key >> HSHIFT], 1u);
                }
    }
    __syncthreads();
}

// RE-COLLECTION of one part: the tensor's elements in the part with key >= tau, in index
// order, through `put(position, entry)`; nothing is written when there are more than `cap`.
// Two passes over the part (count, then place).  Returns the count.
template <int OP, class Put>
__device__ __forceinline__ uint32_t dense_compact(const SelectArgs &A, const TensorDesc &td, const SegDesc &sd,
                                                  uint32_t tau, uint32_t cap, PartShared &P, Put put)
{
    const DenseRun r = dense_run(td, sd);
    const uint32_t lane = lane_id(), wave = threadIdx.x >> 6;
    const bool vec = rows_aligned(A);
    uint32_t mine = 0;
    for (uint32_t t = r.t0; t < r.t1; t += 2) {      // two tiles in flight, as in dense_hist
        const bool two = t + 1 < r.t1;
        uint32_t bits[2][4][4], in[2][4];
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int row = 0; row < 4; ++row)
                in[u][row] = quad_bits<OP>(A, (u && two ? t + 1 : t) * TILE + row * 256 + lane * 4, r.lo, r.hi, vec,
                                           bits[u][row]);
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int row = 0; row < 4; ++row)
#pragma unroll
                for (int x = 0; x < 4; ++x)
                    if ((u == 0 || two) && ((in[u][row] >> x) & 1u) && (bits[u][row][x] & 0x7FFFFFFFu) >= tau) ++mine;
    }
    const uint32_t wsum_ = wave_sum(mine);
    __syncthreads();
    if (lane == 0) P.wtot[wave] = wsum_;
    __syncthreads();
    uint32_t before = 0, total = 0;
#pragma unroll
    for (uint32_t x = 0; x < SEL_WAVES; ++x) {
        const uint32_t v = P.wtot[x];
        if (x < wave) before += v;
        total += v;
    }
    if (total > cap) return total;
    uint32_t run = before;
    for (uint32_t t = r.t0; t < r.t1; ++t) {
        uint32_t tbits[4][4], tin[4];
#pragma unroll
        for (int row = 0; row < 4; ++row) tin[row] = quad_bits<OP>(A, t * TILE + row * 256 + lane * 4, r.lo, r.hi, vec, tbits[row]);
#pragma unroll
        for (int row = 0; row < 4; ++row) {
            const uint32_t e0 = t * TILE + row * 256 + lane * 4;
            const uint32_t (&bits)[4] = tbits[row];
            bool f[4];
            uint64_t mk[4];
            const uint32_t in = tin[row];
#pragma unroll
            for (int x = 0; x < 4; ++x) {
                f[x] = ((in >> x) & 1u) && (bits[x] & 0x7FFFFFFFu) >= tau;
                mk[x] = ballot64(f[x]);
            }
            if ((mk[0] | mk[1] | mk[2] | mk[3]) != 0) {
                uint32_t p = run + mbcnt64(mk[0]) + mbcnt64(mk[1]) + mbcnt64(mk[2]) + mbcnt64(mk[3]);
#pragma unroll
                for (int x = 0; x < 4; ++x) {
                    if (f[x]) {
                        put(p, make_uint2(e0 + x, bits[x]));
                        ++p;
                    }
                }
                run += (uint32_t)(__popcll(mk[0]) + __popcll(mk[1]) + __popcll(mk[2]) + __popcll(mk[3]));
            }
        }
    }
    // the two passes must have seen the same elements
    if (lane == 0 && run - before != wsum_) atomicAdd(&A.stats->internal_errors, 1ull);
    return total;
}

// Dense request on a tensor that takes the chain: how many of the part's elements reach the
// threshold, counted into the tensor's window histogram (LDS h, SEG_WBINS bins).
template <int OP>
__device__ __forceinline__ uint32_t dense_window_count(const SelectArgs &A, const TensorDesc &td, const SegDesc &sd,
                                                       uint32_t tau, uint32_t win_base, uint32_t *h, uint32_t *wsum)
{
    const uint64_t lo = max((uint64_t)td.off, (uint64_t)sd.tile0 * TILE);
    const uint64_t hi = min((uint64_t)td.off + td.n, ((uint64_t)sd.tile0 + sd.ntiles) * TILE);
    uint32_t mine = 0;
    for (uint64_t e = lo + threadIdx.x; e < hi; e += SEL_THREADS) {
        const uint32_t key = __float_as_uint(row_value<OP>(A.state, A.model, (uint32_t)e)) & 0x7FFFFFFFu;
        if (key >= tau) {
            const uint32_t hi12 = key >> SEG_LOWBITS;
            const uint32_t w = (hi12 > win_base) ? (hi12 - win_base) : 0u;
            atomicAdd(&h[min(w, SEG_WBINS - 1u)], 1u);
            ++mine;
        }
    }
    return block_sum(mine, wsum, SEL_WAVES);
}

// First bin (key >> SEG_LOWBITS) of the window histogram of a tensor that takes the chain.
// Candidates start at the collection threshold; when that lies far below the k-th key of the
// previous selection on this stream (a relaxed hint), the window is centred on that key
// instead, so that it reaches half an octave to either side of it.  Keys below the window are
// counted into bin 0, which then holds no usable rank.
__device__ __forceinline__ uint32_t seg_window_base(uint32_t tau_cur, uint32_t t_prev)
{
    const uint32_t b_tau = tau_cur >> SEG_LOWBITS;
    const uint32_t b_prev = t_prev >> SEG_LOWBITS;
    const uint32_t b_mid = (b_prev > SEG_WBINS / 2) ? (b_prev - SEG_WBINS / 2) : 0u;
    return max(b_tau, b_mid);
}

// The last part of a tensor that takes the chain: the tensor's window histogram (global, c
// candidates in all) -> the 19-bit prefix of the k-th key, its rank among the entries sharing
// it, and the next hint.  Returns the tensor's status (SEG_ACTIVE, SEG_ALL, or 0 = failed);
// thread 0 writes segstate / hints.  h: SEG_WBINS words of LDS.
template <int OP>
__device__ __forceinline__ uint32_t window_step(const SelectArgs &A, const TensorDesc &td, const PlanEntry &pe,
                                                uint32_t j, uint32_t c, bool ovf, uint32_t tau_cur, uint32_t tprev_cur,
                                                bool exact_mode, PartShared &P)
{
    const uint32_t tid = threadIdx.x;
    uint32_t *h = P.S.h;
    uint32_t *gh = A.ghist + (size_t)j * HBINS;
    uint32_t mylow = 0xFFFFFFFFu;
    if (tid == 0) P.S.kmin = 0xFFFFFFFFu;
    __syncthreads();
    for (uint32_t b = tid; b < SEG_WBINS; b += SEL_THREADS) {
        const uint32_t v = ld_dev(&gh[b]);
        h[b] = v;
        if (v) st_dev(&gh[b], 0u);   // clean for the next use
        if (v && mylow == 0xFFFFFFFFu) mylow = b;
    }
    if (mylow != 0xFFFFFFFFu) atomicMin(&P.S.kmin, mylow);
    const uint32_t win_base = seg_window_base(tau_cur, tprev_cur);
    const int bin_min = (win_base > (tau_cur >> SEG_LOWBITS)) ? 1 : 0;   // bin 0 mixes in lower keys
    uint32_t R = 0, Eq = 0;
    if (A.write_hint) R = hint_rank<OP>(td, pe, !exact_mode, c, A.hint2[j], A.m, &Eq);
    const bool measurable = (R != 0) && (c >= R);
    const uint32_t qlow = max(c / 4u, min(c, 16u));
    const uint32_t third = measurable ? Eq : ((R != 0 && c != 0) ? (c - qlow + 1u) : 0u);
    find_ranks<SEG_WBINS, SEL_WAVES>(h, pe.k, measurable ? R : pe.k, third, P.S.rowsum, P.S.res);
    const int bk = P.S.res[0], bR = P.S.res[2];
    const uint32_t lowest = P.S.kmin;
    const bool all = (pe.k == td.n);   // everything is sent: no threshold to find
    const bool ok = all || (!ovf && (c >= pe.k) && bk >= bin_min && bk < (int)SEG_WBINS - 1);
    if (tid == 0 && ok) {
        SegState *st = &A.segstate[j];
        st->pfxcount = 0;
        st->pfx = win_base + (uint32_t)max(bk, 0);
        st->r2 = (uint32_t)P.S.res[1];
        st->T = 0;
        atomicAdd(&A.stats->candidates, (unsigned long long)c);
        atomicAdd(&A.stats->segmented_tensors, 1ull);
        if (A.write_hint) {
            uint32_t tn = 0, expect = 0;
            if (measurable && bR >= bin_min && bR < (int)SEG_WBINS - 1) {
                const uint32_t edge = (win_base + (uint32_t)bR) << SEG_LOWBITS;
                tn = edge ? edge : 1u;
                expect = R - (uint32_t)P.S.res[3] + h[bR];
                const int bE = P.S.res[4];
                if (bE >= bin_min && bE < (int)SEG_WBINS - 1)
                    tn = hint_scaled(tn, (win_base + (uint32_t)bE) << SEG_LOWBITS, tau_cur);
            }
            if (tn == 0 && !measurable && R != 0 && lowest != 0xFFFFFFFFu && (int)lowest >= bin_min &&
                P.S.res[4] >= (int)lowest && P.S.res[4] < (int)SEG_WBINS - 1) {
                const uint32_t kmin = max((win_base + lowest) << SEG_LOWBITS, tau_cur);
                tn = hint_extrapolated(kmin, c, R, qlow, ((uint32_t)P.S.res[4] - lowest + 1u) << SEG_LOWBITS);
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
    __syncthreads();
    return all ? (uint32_t)SEG_ALL : (ok ? (uint32_t)SEG_ACTIVE : 0u);
}

// Selection of a whole tensor straight from the buffers by this one workgroup: small tensors,
// dense requests on tensors outside the chain, and whatever the re-collection could not
// resolve.  Exact for any data; slow on large tensors.
template <int OP>
__device__ __forceinline__ void dense_select(const SelectArgs &A, const TensorDesc &td, const PlanEntry &pe, uint32_t j,
                                             uint32_t tau_cur, PartShared &P, uint2 *llist)
{
    const uint32_t tid = threadIdx.x;
    uint32_t R = 0, Eq = 0;
    if (td.big && A.write_hint) R = hint_rank<OP>(td, pe, false, 0u, 0u, A.m, &Eq);
    uint32_t tau_next = 0, expect = 0, q_e = 0, t_k = 0;
    if (td.n <= 2 * SEL_LDS_LIST) {
        uint32_t *lv = (uint32_t *)llist;
        __syncthreads();
        for (uint32_t p = tid; p < td.n; p += SEL_THREADS)
            lv[p] = __float_as_uint(row_value<OP>(A.state, A.model, td.off + p));
        __syncthreads();
        SrcDenseLds src{lv, td.off};
        select_emit<OP, 4>(src, td.n, pe.k, R, 0u, 0xFFFFFFFFu, 0u, false, 0xFFFFFFFFu, P.S, A, pe.outoff,
                           &tau_next, &expect, &q_e, &t_k);
    } else {
        SrcDense<OP> src{A.state, A.model, td.off};
        select_emit<OP, 8>(src, td.n, pe.k, R, 0u, 0xFFFFFFFFu, 0u, false, 0xFFFFFFFFu, P.S, A, pe.outoff,
                           &tau_next, &expect, &q_e, &t_k);
    }
    if (td.big && A.write_hint && tid == 0) {
        uint32_t tn = tau_next;
        if (tn == 0) {
            tn = hint_relaxed(tau_cur, 0xFFFFFFFFu);
            expect = 0;
        }
        if (tn >= 0x7F800000u) tn = 0x7F7FFFFFu;
        A.tau[j] = tn;
        A.hint2[j] = expect;
        A.tprev[j] = t_k;
    }
}

// The tensor's candidates are in `llist` (first SEL_LDS_LIST) and `glist` (beyond): exact
// selection, emission, fix-up and the next hint.  win_*: the window histogram in P.S.h counted
// while the list was built (single-part tensors), see select_emit.
template <int OP>
__device__ __forceinline__ void list_select(const SelectArgs &A, const TensorDesc &td, const PlanEntry &pe, uint32_t j,
                                            uint32_t c, uint32_t kmin, uint32_t tau_cur, uint32_t hint2_cur,
                                            uint32_t win_join, bool win_counted, bool exact_mode, PartShared &P,
                                            uint2 *llist, uint2 *glist)
{
    const uint32_t tid = threadIdx.x;
    uint32_t R = 0, Eq = 0;
    if (A.write_hint) R = hint_rank<OP>(td, pe, !exact_mode, c, hint2_cur, A.m, &Eq);
    uint32_t tau_next = 0, expect = 0, q_e = 0, t_k = 0;
    // the window placed by the hints serves if no candidate lies below the threshold (none can);
    // a histogram counted on the way then stands as it is
    const bool anchored = (win_join != 0xFFFFFFFFu) && (kmin != 0xFFFFFFFFu) && (kmin >> 11) >= (tau_cur >> 11);
    const bool win_ready = win_counted && anchored;
    const uint32_t win_base = (kmin == 0xFFFFFFFFu) ? 0xFFFFFFFFu : (anchored ? win_join : (kmin >> 11));
    const uint32_t win_min = (anchored && win_join > (kmin >> 11)) ? 1u : 0u;   // entries below the window
    if (c <= SEL_LDS_LIST) {
        SrcList src{llist};
        select_emit<OP, 4>(src, c, pe.k, R, Eq, win_base, win_min, win_ready, kmin, P.S, A, pe.outoff,
                           &tau_next, &expect, &q_e, &t_k);
    } else {
        SrcSplit src{llist, glist};     // the list outgrew LDS: its tail is read from global scratch
        select_emit<OP, 8>(src, c, pe.k, R, Eq, win_base, win_min, win_ready, kmin, P.S, A, pe.outoff,
                           &tau_next, &expect, &q_e, &t_k);
    }
    if (A.write_hint && tid == 0) {
        uint32_t tn = tau_next;
        if (tn == 0) {
            tn = hint_relaxed(tau_cur, kmin);
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

// The candidates of a tensor of several parts, addressed by list position through the parts'
// global lists (pbase: first position of every part, in LDS).
struct SrcParts {
    static constexpr bool AGG = true;
    const uint2 *ord;
    const uint32_t *pbase;     // LDS: first list position of every part
    const uint32_t *pofs;      // LDS: where every part's list starts in ord
    uint32_t nseg;
    __device__ __forceinline__ uint2 get(uint32_t p) const
    {
        uint32_t lo = 0, hi = nseg;       // last part whose first position is <= p
        while (hi - lo > 1) {
            const uint32_t mid = (lo + hi) >> 1;
            if (pbase[mid] <= p) lo = mid;
            else hi = mid;
        }
        return ld_dev(&ord[(size_t)pofs[lo] + (p - pbase[lo])]);
    }
    __device__ __forceinline__ uint32_t bits(uint32_t p) const { return get(p).y; }
    __device__ __forceinline__ uint32_t index(uint32_t p) const { return get(p).x; }
};

// TRIM: a candidate list that is complete but too long for one workgroup is cut down to what a
// fresh collection would have found.  The list's own key histogram (bits [30:20]) gives the
// threshold -- the lower edge of the bucket that holds rank pe.k2 -- and the entries at or above
// it are moved up in list order into llist / glist.  No second pass over the tensor.  Returns the
// new count, or 0 (nothing moved) if that is still beyond list_max; tau is raised to the new
// threshold.  A success is published to `verdict` before the entries are moved.
//   In place: an entry never moves to a later position, and every turn has read its entries
//   before it writes any, so both an LDS list and the tail that spills into the first unit's
//   global list are only ever written where they have been read.
template <class Src>
__device__ __forceinline__ uint32_t trim_list(const SelectArgs &A, const Src &src, uint32_t c, uint32_t list_max,
                                              const PlanEntry &pe, uint32_t *verdict, PartShared &P, uint2 *llist,
                                              uint2 *glist, uint32_t &tau)
{
    const uint32_t tid = threadIdx.x;
    constexpr uint32_t GU = 8;      // entries per thread in flight
    for (uint32_t b = tid; b < 2048; b += SEL_THREADS) P.S.h[b] = 0;
    __syncthreads();
    for (uint32_t q0 = 0; q0 < c; q0 += GU * SEL_THREADS) {
        uint32_t key[GU];
#pragma unroll
        for (uint32_t u = 0; u < GU; ++u) {
            const uint32_t q = q0 + u * SEL_THREADS + tid;
            key[u] = (q < c) ? (src.bits(q) & 0x7FFFFFFFu) : 0u;
        }
#pragma unroll
        for (uint32_t u = 0; u < GU; ++u)
            if (key[u] != 0) atomicAdd(&P.S.h[key[u] >> 20], 1u);
    }
    find_ranks<2048, SEL_WAVES>(P.S.h, pe.k2, pe.k, 0u, P.S.rowsum, P.S.res);
    const int b2 = P.S.res[0];
    // (rank k2 beyond the nonzero keys of the list: nothing to cut, the count below says so)
    const uint32_t t = max((b2 > 0) ? ((uint32_t)b2 << 20) : 1u, tau);    // nothing below tau is in the list
    uint32_t reach = 0;      // entries at or above t: whole buckets, by construction
    for (uint32_t b = tid; b < 2048; b += SEL_THREADS)
        if (b >= (t >> 20)) reach += P.S.h[b];
    __syncthreads();
    const uint32_t c2 = block_sum(reach, P.S.wsum, SEL_WAVES);
    __syncthreads();
    if (c2 < pe.k || c2 > list_max) return 0u;
    if (verdict && tid == 0) st_dev(verdict, 0x100u | (uint32_t)SEG_DONE);
    uint32_t run = 0;
    for (uint32_t q0 = 0; q0 < c; q0 += GU * SEL_THREADS) {      // GU consecutive entries per thread
        uint2 e[GU];
        uint32_t keep = 0;
#pragma unroll
        for (uint32_t u = 0; u < GU; ++u) {
            const uint32_t q = q0 + tid * GU + u;
            e[u] = (q < c) ? src.get(q) : make_uint2(0, 0);
        }
#pragma unroll
        for (uint32_t u = 0; u < GU; ++u) {
            const uint32_t q = q0 + tid * GU + u;
            if (q < c && (e[u].y & 0x7FFFFFFFu) >= t) keep |= 1u << u;
        }
        uint32_t tot;
        uint32_t pos = run + block_excl_scan<SEL_WAVES>((uint32_t)__popcll((unsigned long long)keep), P.S.wsum, tot);
#pragma unroll
        for (uint32_t u = 0; u < GU; ++u) {
            if ((keep >> u) & 1u) {
                if (pos < c2) put_entry(llist, glist, pos, e[u]);
                ++pos;
            }
        }
        run += tot;
    }
    wait_mem();
    __syncthreads();
    if (tid == 0 && run != c2) atomicAdd(&A.stats->internal_errors, 1ull);      // the two passes disagree
    tau = t;
    return c2;
}

// What the workgroup that completes a tensor's candidate lists does with them (`round` 0: the
// streaming pass's candidates, 1: re-collected with a fresh threshold).  Returns the tensor's
// status: SEG_DONE, SEG_ACTIVE / SEG_ALL (the chain kernels go on), or SEG_PENDING (round 0
// only: collect again).
//   multi: the lists are global lists of several units -- the tensor's parts (by_parts: counts
//   in segcnt) or its join groups (counts in grpcnt) -- and are gathered here; otherwise the
//   one list is in llist / glist (or, for a tensor that takes the chain, in its global list
//   only) with count c0, overflow ovf0, smallest key (or a lower bound of it) kmin0, and --
//   win_counted -- the window histogram counted on the way.
//   verdict: where the outcome is published for the re-collecting workgroups of the launch
//   (null: nobody waits); a success is published as soon as it is certain, before the work.
//   tau_cur, tprev_cur: the threshold the lists were collected with and the anchor of the window
//   histograms (handed in: in round 1 they were published by another workgroup of this launch).
template <int OP>
__device__ __forceinline__ uint32_t tensor_select(const SelectArgs &A, const TensorDesc &td, const PlanEntry &pe,
                                                  uint32_t j, int round, bool multi, bool by_parts, uint32_t c0,
                                                  bool ovf0, uint32_t kmin0, uint32_t tau_cur, uint32_t tprev_cur,
                                                  uint32_t win_join, bool win_counted, uint32_t *verdict,
                                                  PartShared &P, uint2 *llist)
{
    const uint32_t tid = threadIdx.x;
    const uint32_t tlo = td.off / TILE;
    uint2 *glist = A.ord + (size_t)(tlo + j) * CAPT;      // = the first part's list
    const bool exact_mode = A.exact_mode || round != 0;
    const uint32_t hint2_cur = A.write_hint ? A.hint2[j] : 0u;
    const uint32_t nunits = by_parts ? td.nseg : td.ngrp;
    const SegDesc *units = by_parts ? A.segtab + td.seg_first : A.grptab + td.grp_first;
    const uint32_t *ucnt = by_parts ? A.segcnt + td.seg_first : A.grpcnt + td.grp_first;
    const bool have_pbase = nunits <= SEG_MAX_PER_TENSOR;
    // The longest list this workgroup selects from.  A tensor of several parts is gathered in
    // place: what does not fit the LDS list goes to the first part's global list, which must
    // end before the second part's begins.
    const uint32_t list_max = multi ? max(SEL_LDS_LIST, min(SEL_LIST_HARD, units[0].ntiles * CAPT))
                                    : SEL_LIST_HARD;
    uint32_t c = c0, kmin = kmin0;
    bool ovf = ovf0;
    if (multi) {
        // counts of the units -> list positions
        uint32_t o = 0;
        c = 0;
        for (uint32_t s0 = 0; s0 < nunits; s0 += SEL_THREADS) {
            const uint32_t s = s0 + tid;
            uint32_t cnt = (s < nunits) ? ld_dev(&ucnt[s]) : 0u;
            if (cnt >> 31) o = 1;
            cnt &= 0x7FFFFFFFu;
            uint32_t tot;
            const uint32_t ex = block_excl_scan<SEL_WAVES>(cnt, P.S.wsum, tot);
            if (s < nunits && have_pbase) {
                P.pbase[s] = c + ex;
                // (a part of a tensor that takes the chain lies where its group's join put it)
                P.pofs[s] = (by_parts && pe.seg) ? ld_dev(&A.segstart[td.seg_first + s])
                                                 : (units[s].tile0 + j) * CAPT;   // below 2^32: n < 2^32
            }
            c += tot;
        }
        if (tid == 0 && have_pbase) P.pbase[nunits] = c;
        ovf = __syncthreads_or((int)o) != 0;
    }
    uint32_t status = 0;
    bool early = false;      // the verdict went out before the work
    // every nonzero is in the lists (a dense request has no lists: it falls back instead)
    const bool zerofill = !A.dense && !ovf && c < pe.k && tau_cur <= 1u && (!multi || have_pbase);
    if (pe.seg) status = window_step<OP>(A, td, pe, j, c, ovf, tau_cur, tprev_cur, exact_mode, P);
    if (status == 0 && zerofill) {
        // the message is completed with the tensor's lowest-index zeros
        early = true;
        if (verdict && tid == 0) st_dev(verdict, 0x100u | (uint32_t)SEG_DONE);
        if (multi) {
            zero_fill_emit<OP>(SrcParts{A.ord, P.pbase, P.pofs, nunits}, c, td, pe, A, P.S.wsum);
        } else if (pe.seg) {
            zero_fill_emit<OP>(SrcList{glist}, c, td, pe, A, P.S.wsum);
        } else if (c > SEL_LDS_LIST) {
            zero_fill_emit<OP>(SrcSplit{llist, glist}, c, td, pe, A, P.S.wsum);
        } else {
            zero_fill_emit<OP>(SrcList{llist}, c, td, pe, A, P.S.wsum);
        }
        if (A.write_hint && tid == 0) {
            A.tau[j] = 1u;
            A.hint2[j] = 0u;
            A.tprev[j] = 0u;
        }
        if (tid == 0) atomicAdd(&A.stats->candidates, (unsigned long long)c);
        status = SEG_DONE;
    } else if (!pe.seg && !ovf && c >= pe.k && c <= list_max && (!multi || have_pbase)) {
        early = true;
        if (verdict && tid == 0) st_dev(verdict, 0x100u | (uint32_t)SEG_DONE);
        if (multi) {
            // gather the parts' lists into one (positions beyond the LDS list land in the first
            // part's global list: on dead space, or on the very entry that is being moved)
            const bool count_win = (win_join != 0xFFFFFFFFu);   // the hinted window is counted on the way
            for (uint32_t b = tid; b < 2048; b += SEL_THREADS) P.S.h[b] = 0;
            if (tid == 0) P.S.kmin = 0xFFFFFFFFu;
            __syncthreads();
            const SrcParts src{A.ord, P.pbase, P.pofs, nunits};
            uint32_t km = 0xFFFFFFFFu;
            constexpr uint32_t GU = 8;      // entries per thread in flight
            for (uint32_t q0 = 0; q0 < c; q0 += GU * SEL_THREADS) {
                uint2 e[GU];
#pragma unroll
                for (uint32_t u = 0; u < GU; ++u) {
                    const uint32_t q = q0 + u * SEL_THREADS + tid;
                    e[u] = (q < c) ? src.get(q) : make_uint2(0, 0);
                }
#pragma unroll
                for (uint32_t u = 0; u < GU; ++u) {
                    const uint32_t q = q0 + u * SEL_THREADS + tid;
                    if (q < c) {
                        put_entry(llist, glist, q, e[u]);
                        km = min(km, e[u].y & 0x7FFFFFFFu);
                        if (count_win) window_count(P.S.h, win_join, e[u].y & 0x7FFFFFFFu);
                    }
                }
            }
            km = wave_min_to_last(km);
            if (lane_id() == 63) atomicMin(&P.S.kmin, km);
            wait_mem();
            __syncthreads();
            kmin = P.S.kmin;
        }
        list_select<OP>(A, td, pe, j, c, kmin, tau_cur, hint2_cur, win_join,
                        multi ? (win_join != 0xFFFFFFFFu) : win_counted, exact_mode, P, llist, glist);
        if (tid == 0) atomicAdd(&A.stats->candidates, (unsigned long long)c);
        status = SEG_DONE;
    }
    if (status == 0 && !pe.seg && !ovf && (!multi || have_pbase) && c >= pe.k && c > list_max) {
        // Every candidate is in the lists, there are only too many of them for one workgroup
        // (the threshold has fallen behind a scale that grew): trimmed on the spot.
        uint32_t tau_new = tau_cur;
        const uint32_t c2 = multi ? trim_list(A, SrcParts{A.ord, P.pbase, P.pofs, nunits}, c, list_max, pe, verdict, P,
                                              llist, glist, tau_new)
                                  : trim_list(A, SrcSplit{llist, glist}, c, list_max, pe, verdict, P, llist, glist, tau_new);
        if (c2 != 0) {
            early = true;
            if (tid == 0) {
                atomicAdd(&A.stats->candidates, (unsigned long long)c2);
                if (round == 0) atomicAdd(&A.stats->repaired_tensors, 1ull);
            }
            // (smallest key unknown: the threshold is a lower bound of it, and the window is
            // counted from the list)
            list_select<OP>(A, td, pe, j, c2, tau_new, tau_new, hint2_cur, 0xFFFFFFFFu, false, true, P, llist, glist);
            status = SEG_DONE;
        }
    }
    if (status == 0) status = (round == 0 && A.repair) ? (uint32_t)SEG_PENDING : (uint32_t)SEG_FALLBACK;
    if (status == SEG_FALLBACK) {
        if (tid == 0) {
            atomicAdd(&A.stats->fallback_tensors, 1ull);
            atomicAdd(&A.stats->fallback_elems, (unsigned long long)td.n);
        }
        dense_select<OP>(A, td, pe, j, tau_cur, P, llist);
        status = SEG_DONE;
    } else if (round != 0 && tid == 0) {
        atomicAdd(&A.stats->repaired_tensors, 1ull);
    }
    if (tid == 0) A.segstate[j].status = status;
    if (verdict && !early) {
        wait_mem();
        __syncthreads();
        if (tid < 64) {
            // A rejected join may have spilled list entries with cached stores into the very
            // lists that other workgroups now fill again: written back before they start, so
            // that no older copy in this L2 shadows theirs.
            if (status == SEG_PENDING) release_dev();
            if (tid == 0) st_dev(verdict, 0x100u | status);
        }
    }
    return status;
}

// RE-HISTOGRAM (role 1) or RE-COLLECTION (role 2) of one part of a tensor that the JOIN left
// pending (the caller has seen that verdict).
template <int OP>
__device__ __forceinline__ void recollect_part(const SelectArgs &A, uint32_t role, uint32_t part, PartShared &P,
                                               uint2 *llist)
{
    const uint32_t tid = threadIdx.x;
    const SegDesc sd = A.segtab[part];
    const uint32_t j = sd.j;
    const TensorDesc td = A.tdesc[j];
    const PlanEntry pe = A.plan[j];
    const bool multi = td.nseg > 1;
    SegState *st = &A.segstate[j];
    uint2 *plist = A.ord + (size_t)(sd.tile0 + j) * CAPT;       // this part's list
    const uint32_t part_cap = sd.ntiles * CAPT;
    if (!multi) return;
    uint32_t *gh = A.ghist + (size_t)j * HBINS;
    if (role == 1) {
        uint32_t *lh = (uint32_t *)llist;
        dense_hist<OP>(A, td, sd, lh);
        for (uint32_t b = tid; b < HBINS; b += SEL_THREADS) {
            const uint32_t v = lh[b];
            if (v) atomicAdd(&gh[b], v);
        }
        if (!arrive_last(&st->arrive[1], td.nseg, &P.bc)) return;
        for (uint32_t b = tid; b < HBINS; b += SEL_THREADS) {
            const uint32_t v = ld_dev(&gh[b]);
            lh[b] = v;
            if (v) st_dev(&gh[b], 0u);
        }
        uint32_t tau_new = 0, tprev_new = 0;
        pick_from_hist<SEL_WAVES>(lh, pe, P.S.rowsum, P.S.res, tau_new, tprev_new);
        if (tid == 0) {
            st_dev(&A.tau[j], tau_new);
            st_dev(&A.tprev[j], tprev_new);
        }
        wait_mem();
        __syncthreads();
        if (tid == 0) st_dev(&st->tau_ready, 1u);
        return;
    }
    const uint32_t ready = wait_word(&st->tau_ready, A.spin_limit, &P.bc);
    if (tid == 0) {
        if (ready == 0) atomicAdd(&A.stats->internal_errors, 1ull);
        reader_done(&st->seen[1], td.nseg, 1u, &st->tau_ready);
    }
    if (ready == 0) return;
    const uint32_t tau_new = ld_dev(&A.tau[j]);
    const uint32_t tprev_new = ld_dev(&A.tprev[j]);
    const uint32_t win2 = seg_window_base(tau_new, tprev_new);
    for (uint32_t b = tid; b < 2048; b += SEL_THREADS) P.S.h[b] = 0;
    __syncthreads();
    uint32_t c2;
    if (pe.seg) {
        c2 = dense_compact<OP>(A, td, sd, tau_new, part_cap, P, [&](uint32_t pos, uint2 e) {
            st_dev(&plist[pos], e);
            const uint32_t hi12 = (e.y & 0x7FFFFFFFu) >> SEG_LOWBITS;
            const uint32_t w = (hi12 > win2) ? (hi12 - win2) : 0u;
            atomicAdd(&P.S.h[min(w, SEG_WBINS - 1u)], 1u);
        });
        __syncthreads();
        if (c2 <= part_cap) {
            for (uint32_t b = tid; b < SEG_WBINS; b += SEL_THREADS) {
                const uint32_t v = P.S.h[b];
                if (v) atomicAdd(&gh[b], v);
            }
        }
    } else {
        c2 = dense_compact<OP>(A, td, sd, tau_new, part_cap, P, [&](uint32_t pos, uint2 e) { st_dev(&plist[pos], e); });
    }
    if (tid == 0) {
        st_dev(&A.segcnt[part], min(c2, 0x7FFFFFFFu) | (c2 > part_cap ? 0x80000000u : 0u));
        if (pe.seg) st_dev(&A.segstart[part], (sd.tile0 + j) * CAPT);      // the part's own place again
    }
    if (!arrive_last(&st->arrive[2], td.nseg, &P.bc)) return;
    tensor_select<OP>(A, td, pe, j, 1, true, true, 0u, false, 0xFFFFFFFFu, tau_new, tprev_new, 0xFFFFFFFFu, false,
                      nullptr, P, llist);
}

template <int OP>
__global__ __launch_bounds__(SEL_THREADS) void k_select(const SelectArgs A)
{
    __shared__ PartShared P;
    __shared__ uint2 llist[SEL_LDS_LIST];
    const uint32_t tid = threadIdx.x;
    if (blockIdx.x >= A.ngroups) {
        // RE-HISTOGRAM / RE-COLLECTION: this workgroup looks after up to B_GROUP parts, nb apart,
        // so that the parts of one failed tensor are spread over as many workgroups as there are
        const uint32_t nb = (A.nparts + A.bgroup - 1) / A.bgroup;
        const uint32_t b = blockIdx.x - A.ngroups;
        const uint32_t role = (b < nb) ? 1u : 2u;
        const uint32_t first = (role == 1) ? b : b - nb;
        // the verdicts of the tensors these parts belong to: lane i waits for part i's tensor and
        // signs off for that part
        if (tid < B_GROUP_MAX) P.vbuf[tid] = 0;
        __syncthreads();
        const uint32_t mypart = first + tid * nb;
        if (tid < A.bgroup && mypart < A.nparts) {
            const SegDesc sd = A.segtab[mypart];
            if (A.tdesc[sd.j].nseg > 1) {
                SegState *st = &A.segstate[sd.j];
                uint32_t v = 0;
                for (uint32_t spin = 0; spin < A.spin_limit; ++spin) {
                    v = ld_dev(&st->verdict);
                    if (v != 0) break;
                    __builtin_amdgcn_s_sleep(4);
                }
                if (v == 0) atomicAdd(&A.stats->internal_errors, 1ull);   // gave up waiting
                reader_done(&st->seen[0], 2u * A.tdesc[sd.j].nseg, 1u, &st->verdict);
                P.vbuf[tid] = v;
            }
        }
        __syncthreads();
        for (uint32_t i = 0; i < A.bgroup; ++i)
            if ((P.vbuf[i] & 0xFFu) == SEG_PENDING) recollect_part<OP>(A, role, first + i * nb, P, llist);
        return;
    }
    const SegDesc sd = A.grptab[blockIdx.x];      // this workgroup's join group
    const uint32_t j = sd.j;
    const TensorDesc td = A.tdesc[j];
    const PlanEntry pe = A.plan[j];
    const bool multi = td.ngrp > 1;               // the groups' lists go to the last group to arrive
    const bool has_parts = td.nseg > 1;           // a failed prediction is collected again part by part
    const uint32_t part = td.seg_first;           // (the part, where the tensor has only one)
    SegState *st = &A.segstate[j];
    uint2 *plist = A.ord + (size_t)(sd.tile0 + j) * CAPT;       // this group's list
    const uint32_t part_cap = sd.ntiles * CAPT;
    const bool chain_dense = A.dense && pe.seg;                  // the chain reads the tensor itself

    {
        // ------------------------------------------------------------------ JOIN
        if (!td.big || (A.dense && !pe.seg)) {
            if (sd.sidx != 0) return;
            if (tid == 0) st->status = SEG_DONE;
            dense_select<OP>(A, td, pe, j, td.big ? A.tau[j] : TAU_NEVER, P, llist);
            return;
        }
        const uint32_t tau_cur = A.tau[j];
        const uint32_t tprev_cur = A.tprev[j];
        uint32_t cs = 0, kmin = 0xFFFFFFFFu;
        bool ovf = false;
        // window of the single-workgroup selection: starts at the collection threshold or, when
        // that lies far below (a relaxed hint), 1024 buckets under the previous k-th key
        const uint32_t win_join = max(tau_cur >> 11, max(tprev_cur >> 11, 1024u) - 1024u);
        const uint32_t win_seg = seg_window_base(tau_cur, tprev_cur);
        uint32_t *verdict = (has_parts && A.repair) ? &st->verdict : nullptr;
        uint32_t status;
        if (pe.seg) {
            // a tensor that takes the chain: the group's candidates in one list, with every part's
            // start and count noted for the chain kernels, and the group's window histogram
            const uint32_t p0 = td.seg_first + sd.sidx * A.gparts;
            const uint32_t p1 = min(p0 + A.gparts, td.seg_first + td.nseg);
            uint32_t *gh = A.ghist + (size_t)j * HBINS;
            if (chain_dense) {
                for (uint32_t p = p0; p < p1; ++p) {       // no lists: the parts' elements are counted
                    const SegDesc ps = A.segtab[p];
                    for (uint32_t b = tid; b < 2048; b += SEL_THREADS) P.S.h[b] = 0;
                    __syncthreads();
                    const uint32_t cp = dense_window_count<OP>(A, td, ps, tau_cur, win_seg, P.S.h, P.S.wsum);
                    __syncthreads();
                    for (uint32_t b = tid; b < SEG_WBINS; b += SEL_THREADS) {
                        const uint32_t v = P.S.h[b];
                        if (v) atomicAdd(&gh[b], v);
                    }
                    if (tid == 0) st_dev(&A.segcnt[p], cp);
                    cs += cp;
                    __syncthreads();
                }
            } else {
                for (uint32_t b = tid; b < 2048; b += SEL_THREADS) P.S.h[b] = 0;
                __syncthreads();
                const uint32_t ptiles = A.segtab[p0].ntiles;         // tiles per part (the tensor's last part may have fewer)
                const uint32_t gbase = (sd.tile0 + j) * CAPT;        // below 2^32: n < 2^32
                cs = join_part(
                    A, td, sd, P, ovf,
                    [&](uint32_t pos, uint2 e) {
                        st_dev(&plist[pos], e);          // read by the chain kernels, and by a zero fill
                        const uint32_t hi12 = (e.y & 0x7FFFFFFFu) >> SEG_LOWBITS;
                        const uint32_t w = (hi12 > win_seg) ? (hi12 - win_seg) : 0u;
                        atomicAdd(&P.S.h[min(w, SEG_WBINS - 1u)], 1u);
                    },
                    [&](uint32_t tl, uint32_t pos) {
                        if (tl % ptiles == 0) P.pbase[tl / ptiles] = pos;
                    });
                for (uint32_t b = tid; b < SEG_WBINS; b += SEL_THREADS) {
                    const uint32_t v = P.S.h[b];
                    if (v) atomicAdd(&gh[b], v);
                }
                const uint32_t np = p1 - p0;
                if (tid < np) {
                    const uint32_t start = P.pbase[tid], end = (tid + 1 < np) ? P.pbase[tid + 1] : cs;
                    st_dev(&A.segstart[p0 + tid], gbase + start);
                    st_dev(&A.segcnt[p0 + tid], (end - start) | (ovf ? 0x80000000u : 0u));
                }
                __syncthreads();
            }
            if (multi) {
                if (!arrive_last(&st->arrive[0], td.ngrp, &P.bc)) return;
            } else {
                wait_mem();       // counts and histogram are read back below
                __syncthreads();
            }
            status = tensor_select<OP>(A, td, pe, j, 0, has_parts, true, cs, ovf, kmin, tau_cur, tprev_cur, win_join,
                                       true, verdict, P, llist);
        } else if (multi) {
            cs = join_part(A, td, sd, P, ovf, [&](uint32_t pos, uint2 e) { st_dev(&plist[pos], e); });
            if (tid == 0) st_dev(&A.grpcnt[blockIdx.x], cs | (ovf ? 0x80000000u : 0u));
            if (!arrive_last(&st->arrive[0], td.ngrp, &P.bc)) return;
            status = tensor_select<OP>(A, td, pe, j, 0, true, false, cs, ovf, kmin, tau_cur, tprev_cur, win_join, true,
                                       verdict, P, llist);
        } else {
            for (uint32_t b = tid; b < 2048; b += SEL_THREADS) P.S.h[b] = 0;
            if (tid == 0) P.S.kmin = 0xFFFFFFFFu;
            __syncthreads();
            uint2 *glist = plist;
            cs = join_part(A, td, sd, P, ovf, [&](uint32_t pos, uint2 e) {
                put_entry(llist, glist, pos, e);
                kmin = min(kmin, e.y & 0x7FFFFFFFu);
                window_count(P.S.h, win_join, e.y & 0x7FFFFFFFu);
            });
            kmin = wave_min_to_last(kmin);
            if (lane_id() == 63) atomicMin(&P.S.kmin, kmin);
            wait_mem();
            __syncthreads();
            kmin = P.S.kmin;
            status = tensor_select<OP>(A, td, pe, j, 0, false, false, cs, ovf, kmin, tau_cur, tprev_cur, win_join, true,
                                       verdict, P, llist);
        }
        if (has_parts) return;        // the re-collecting workgroups have the verdict
        if (status != SEG_PENDING) return;
        // ---- a tensor of one part whose prediction failed: collect again on the spot
        uint32_t *lh = (uint32_t *)llist;
        dense_hist<OP>(A, td, sd, lh);
        uint32_t tau_new = 0, tprev_new = 0;
        pick_from_hist<SEL_WAVES>(lh, pe, P.S.rowsum, P.S.res, tau_new, tprev_new);
        if (tid == 0) {
            A.tau[j] = tau_new;
            A.tprev[j] = tprev_new;
            P.bc = tau_new;
        }
        __syncthreads();
        tau_new = P.bc;
        for (uint32_t b = tid; b < 2048; b += SEL_THREADS) P.S.h[b] = 0;
        __syncthreads();
        const uint32_t win2 = seg_window_base(tau_new, tprev_new);
        const uint32_t cap = pe.seg ? part_cap : min(part_cap, SEL_LIST_HARD);
        uint32_t c2;
        if (pe.seg) {
            c2 = dense_compact<OP>(A, td, sd, tau_new, cap, P, [&](uint32_t pos, uint2 e) {
                st_dev(&plist[pos], e);
                const uint32_t hi12 = (e.y & 0x7FFFFFFFu) >> SEG_LOWBITS;
                const uint32_t w = (hi12 > win2) ? (hi12 - win2) : 0u;
                atomicAdd(&P.S.h[min(w, SEG_WBINS - 1u)], 1u);
            });
            __syncthreads();
            if (c2 <= cap) {
                uint32_t *gh = A.ghist + (size_t)j * HBINS;
                for (uint32_t b = tid; b < SEG_WBINS; b += SEL_THREADS) {
                    const uint32_t v = P.S.h[b];
                    if (v) atomicAdd(&gh[b], v);
                }
                if (tid == 0) st_dev(&A.segcnt[part], c2);
            }
        } else {
            uint2 *glist = plist;
            c2 = dense_compact<OP>(A, td, sd, tau_new, cap, P, [&](uint32_t pos, uint2 e) { put_entry(llist, glist, pos, e); });
        }
        wait_mem();
        __syncthreads();
        // kmin unknown (0 keeps the window honest: it is counted again from the list)
        tensor_select<OP>(A, td, pe, j, 1, false, true, c2, c2 > cap, tau_new, tau_new, tprev_new, 0xFFFFFFFFu, false,
                          nullptr, P, llist);
        return;
    }

}

void launch_select(int op, const SelectArgs &a, void *stream, void *ev0, void *ev1)
{
    hipStream_t st = (hipStream_t)stream;
    if (a.ngroups == 0) return;
    const uint32_t nb = (a.nparts + a.bgroup - 1) / a.bgroup;
    const dim3 grid(a.ngroups + (a.repair ? 2u * nb : 0u)), block(SEL_THREADS);
    if (op == SEL_WORKER) launch_k(k_select<SEL_WORKER>, grid, block, st, ev0, ev1, a);
    else if (op == SEL_PULL) launch_k(k_select<SEL_PULL>, grid, block, st, ev0, ev1, a);
    else launch_k(k_select<SEL_PULL_V>, grid, block, st, ev0, ev1, a);
}

}  // namespace dgs
