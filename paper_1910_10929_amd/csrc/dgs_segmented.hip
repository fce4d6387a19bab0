// Multi-workgroup ("segmented") selection of libdgs, for very large tensors and for
// candidate lists that outgrow one workgroup.
#include "dgs_select.h"
#include "dgs_tile.h"

namespace dgs {

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

}  // namespace dgs
