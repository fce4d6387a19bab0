// The chain: what follows the selection kernel for tensors whose candidate lists are too long
// for one workgroup (and for dense requests, where the "list" of a part is the tensor's own
// elements).  The selection kernel has left, per tensor, the 19-bit prefix of the k-th key and
// its rank among the entries sharing that prefix; here
//   prefix  per part   : counts the entries above the prefix, appends those sharing it to the
//                        tensor's prefix list and counts their low 12 bits; the part that
//                        arrives last for a tensor RANKS: exact k-th key, tie budget, and every
//                        part's output position
//   emit    per part   : ordered emission ("encode()" of Algorithms 1-3) and the state fix-up
//                        (Eq. 12 / Eq. 6).
#include "dgs_select.h"

namespace dgs {

// The entries one part contributes: its compacted candidate list, or (dense requests) the
// tensor's own elements inside the part, in index order.
struct PartSource {
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

__device__ __forceinline__ PartSource part_source(const SelectArgs &A, const TensorDesc &td, const SegDesc &sd,
                                                  uint32_t part, bool dense)
{
    PartSource S;
    S.list = A.ord + (dense ? 0u : A.segstart[part]);
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
        S.count = A.segcnt[part] & 0x7FFFFFFFu;
    }
    return S;
}

constexpr uint32_t PFX_STAGE = 1024;   // entries sharing the prefix that one part can stage in LDS

struct ChainShared {
    uint32_t h[SEG_LBINS];
    uint32_t sG[SEG_MAX_PER_TENSOR];
    uint32_t sQ[SEG_MAX_PER_TENSOR];
    uint32_t rowsum[64];
    int res[6];
    uint32_t wsum[SEL_WAVES];
    uint2 stage[PFX_STAGE];
    uint32_t nstage, base, bc;
};

__global__ __launch_bounds__(SEL_THREADS) void k_chain_prefix(const SelectArgs A)
{
    __shared__ ChainShared C;
    const uint32_t part = blockIdx.x;
    const SegDesc sd = A.segtab[part];
    const uint32_t j = sd.j;
    const PlanEntry pe = A.plan[j];
    if (!pe.seg) return;
    SegState *st = &A.segstate[j];
    if (st->status != SEG_ACTIVE) return;
    const TensorDesc td = A.tdesc[j];
    const PartSource src = part_source(A, td, sd, part, A.dense != 0);
    const uint32_t cs = src.count;
    const uint32_t tid = threadIdx.x;
    const uint32_t pfx = st->pfx;
    uint4 *plist = A.pfxlist + (size_t)td.pfx_slot * PFX_CAP;
    uint32_t *glow = A.ghist + (size_t)j * HBINS;   // low key bits of the entries sharing the prefix
    if (tid == 0) C.nstage = 0;
    __syncthreads();
    uint32_t g1 = 0;
    for (uint32_t eb = 0; eb < cs; eb += 4 * SEL_THREADS) {
        uint2 ent[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const uint32_t e = eb + u * SEL_THREADS + tid;
            ent[u] = (e < cs) ? src.get(e) : make_uint2(0, 0);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const uint32_t e = eb + u * SEL_THREADS + tid;
            if (e < cs) {
                const uint32_t hi12 = (ent[u].y & 0x7FFFFFFFu) >> SEG_LOWBITS;
                if (hi12 > pfx) {
                    ++g1;
                } else if (hi12 == pfx) {
                    atomicAdd(&glow[ent[u].y & (SEG_LBINS - 1u)], 1u);
                    const uint32_t p = atomicAdd(&C.nstage, 1u);
                    if (p < PFX_STAGE) C.stage[p] = ent[u];
                }
            }
        }
    }
    const uint32_t G1 = block_sum(g1, C.wsum, SEL_WAVES);   // its barriers also complete `stage`
    const uint32_t ns = C.nstage;
    if (tid == 0) {
        st_dev(&A.segG1[part], G1);
        // one reservation per part in the tensor's prefix list; a part that could not stage all
        // of its entries pushes the count past the capacity, and the ranking counts instead
        if (ns) C.base = __hip_atomic_fetch_add(&st->pfxcount, ns > PFX_STAGE ? PFX_CAP + 1u : ns,
                                                __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __syncthreads();
    if (ns && ns <= PFX_STAGE) {
        const uint32_t b0 = C.base;
        for (uint32_t i = tid; i < ns; i += SEL_THREADS)
            if (b0 + i < PFX_CAP) {
                // (index, value bits) and (part, 0) as two 8-byte device-scope stores
                uint2 *dst = (uint2 *)&plist[b0 + i];
                st_dev(&dst[0], C.stage[i]);
                st_dev(&dst[1], make_uint2(sd.sidx, 0u));
            }
    }
    if (!arrive_last(&st->arrive[3], td.nseg, &C.bc)) return;

    // ------------------------------------------------------------------ RANK (last part)
    const uint32_t m = ld_dev(&st->pfxcount);
    const uint32_t r2 = st->r2;
    for (uint32_t s = tid; s < td.nseg; s += SEL_THREADS) { C.sG[s] = 0; C.sQ[s] = 0; }
    for (uint32_t b = tid; b < SEG_LBINS; b += SEL_THREADS) {
        const uint32_t v = ld_dev(&glow[b]);
        C.h[b] = v;
        if (v) st_dev(&glow[b], 0u);   // clean for the next use
    }
    find_ranks<SEG_LBINS, SEL_WAVES>(C.h, r2, 0u, 0u, C.rowsum, C.res);
    const int b3 = C.res[0];
    if (b3 < 0) {   // the rank exceeds what the parts counted: cannot happen
        if (tid == 0) {
            st->status = SEG_FALLBACK;
            atomicAdd(&A.stats->internal_errors, 1ull);
        }
        return;
    }
    const uint32_t T = (pfx << SEG_LOWBITS) | (uint32_t)b3;
    const uint32_t rT = (uint32_t)C.res[1];   // entries equal to T that are taken, lowest index first
    __syncthreads();
    if (m <= PFX_CAP) {
        for (uint32_t p = tid; p < m; p += SEL_THREADS) {
            const uint2 *srcp = (const uint2 *)&plist[p];
            const uint2 e = ld_dev(&srcp[0]);
            const uint32_t seg = ld_dev(&srcp[1]).x;
            const uint32_t low = e.y & (SEG_LBINS - 1u);
            if (seg >= td.nseg) continue;      // (a corrupted list entry)
            if (low > (uint32_t)b3) atomicAdd(&C.sG[seg], 1u);
            else if (low == (uint32_t)b3) atomicAdd(&C.sQ[seg], 1u);
        }
        __syncthreads();
    } else {
        // too many entries share the prefix for the list (massive ties): count every part
        // against T here -- slow, reached by degenerate data only
        for (uint32_t s = 0; s < td.nseg; ++s) {
            const SegDesc ps = A.segtab[td.seg_first + s];
            PartSource q = part_source(A, td, ps, td.seg_first + s, A.dense != 0);
            if (!q.dense) q.count = ld_dev(&A.segcnt[td.seg_first + s]) & 0x7FFFFFFFu;
            uint32_t g = 0, qq = 0;
            for (uint32_t e = tid; e < q.count; e += SEL_THREADS) {
                const uint2 ent = q.dense ? q.get(e) : ld_dev(&q.list[e]);
                const uint32_t key = ent.y & 0x7FFFFFFFu;
                if ((key >> SEG_LOWBITS) == pfx) {
                    g += (key > T) ? 1u : 0u;
                    qq += (key == T) ? 1u : 0u;
                }
            }
            const uint32_t Gs = block_sum(g, C.wsum, SEL_WAVES);
            const uint32_t Qs = block_sum(qq, C.wsum, SEL_WAVES);
            if (tid == 0) { C.sG[s] = Gs; C.sQ[s] = Qs; }
        }
        __syncthreads();
    }
    // parts in order: ties are taken lowest index first, i.e. earlier parts first
    uint32_t carry_q = 0, carry_o = 0;
    for (uint32_t sb = 0; sb < td.nseg; sb += SEL_THREADS) {
        const uint32_t s = sb + tid;
        const bool in = s < td.nseg;
        const uint32_t G = in ? (ld_dev(&A.segG1[td.seg_first + s]) + C.sG[s]) : 0u;
        const uint32_t Q = in ? C.sQ[s] : 0u;
        uint32_t totq, toto;
        const uint32_t qb = carry_q + block_excl_scan<SEL_WAVES>(Q, C.wsum, totq);
        const uint32_t take = min(Q, (rT > qb) ? (rT - qb) : 0u);
        const uint32_t ob = carry_o + block_excl_scan<SEL_WAVES>(G + take, C.wsum, toto);
        if (in) A.segOut[td.seg_first + s] = make_uint2(ob, take);
        carry_q += totq;
        carry_o += toto;
    }
    if (tid == 0) {
        st->T = T;
        st->pfxcount = 0;
        A.tprev[j] = T;
        if (carry_o != pe.k) atomicAdd(&A.stats->internal_errors, 1ull);
    }
}

template <int OP>
__global__ __launch_bounds__(SEG_THREADS) void k_chain_emit(const SelectArgs A)
{
    __shared__ uint32_t wsum[SEG_THREADS / 64];
    const uint32_t part = blockIdx.x;
    const SegDesc sd = A.segtab[part];
    const PlanEntry pe = A.plan[sd.j];
    if (!pe.seg) return;
    const SegState *st = &A.segstate[sd.j];
    const uint32_t status = st->status;
    const TensorDesc td = A.tdesc[sd.j];
    const uint32_t tid = threadIdx.x;
    if (status == SEG_ALL) {
        // k_j = n_j: every element of the part is sent, at its own position
        const PartSource all = part_source(A, td, sd, part, true);
        for (uint32_t e = tid; e < all.count; e += SEG_THREADS) {
            const uint2 ent = all.get(e);
            const uint32_t pos = ent.x - td.off;
            A.out_idx[pe.outoff + pos] = ent.x;
            A.out_val[pe.outoff + pos] = __uint_as_float(ent.y);
            fix_sent<OP>(A.state, ent.x, __uint_as_float(ent.y), A.m);
        }
        return;
    }
    if (status != SEG_ACTIVE) return;
    const uint32_t T = st->T;
    const uint2 so = A.segOut[part];
    const PartSource src = part_source(A, td, sd, part, A.dense != 0);
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
                        if (index_ok(A, v[i].x)) fix_sent<OP>(A.state, v[i].x, __uint_as_float(v[i].y), A.m);
                    }
                    ++pos;
                }
            }
        }
        run_sel += G + min(Q, rem);
        run_eq += Q;
    }
}

void launch_chain(int op, const SelectArgs &a, void *stream, void *ev0, void *ev1)
{
    hipStream_t st = (hipStream_t)stream;
    if (a.nparts == 0) return;
    launch_k(k_chain_prefix, dim3(a.nparts), dim3(SEL_THREADS), st, ev0, nullptr, a);
    if (op == SEL_WORKER)
        launch_k(k_chain_emit<SEL_WORKER>, dim3(a.nparts), dim3(SEG_THREADS), st, nullptr, ev1, a);
    else if (op == SEL_PULL)
        launch_k(k_chain_emit<SEL_PULL>, dim3(a.nparts), dim3(SEG_THREADS), st, nullptr, ev1, a);
    else
        launch_k(k_chain_emit<SEL_PULL_V>, dim3(a.nparts), dim3(SEG_THREADS), st, nullptr, ev1, a);
}

}  // namespace dgs
