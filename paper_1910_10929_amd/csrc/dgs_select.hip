// Pick (histogram -> candidate threshold) and the single-workgroup selection of libdgs.
#include "dgs_select.h"

namespace dgs {

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

constexpr uint32_t SEL_ROWS = 12;                                  // rows of 16 tiles per wavefront and batch
constexpr uint32_t SEL_CNT_LOADS = (SEL_ROWS + 3) / 4;             // count loads per lane, 64 tiles each
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
    // The join counts the entries into the window histogram as it places them.  Every candidate
    // key is >= the collection threshold, so the window starts there -- or, when that lies far
    // below (a relaxed hint), 1024 buckets under the k-th key of the previous call.
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
            uint32_t w[SEL_CNT_LOADS];
#pragma unroll
            for (uint32_t u = 0; u < SEL_CNT_LOADS; ++u) {
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
            for (uint32_t u = 0; u < SEL_CNT_LOADS; ++u) {
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

}  // namespace dgs
