// Host side of libdgs: argument checks, the launch plan, workspace carve-up and
// kernel sequencing.  All arithmetic of the method runs in the kernels.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "../../include/dgs.h"
#include "dgs_device.h"

#ifndef DGS_SAMPLE_WGS_PER_CU
#define DGS_SAMPLE_WGS_PER_CU 4u      // workgroups of the sampling pass per compute unit
#endif

using namespace dgs;

namespace {

constexpr uint32_t NPLAN = 8;          // densities cached per context
constexpr size_t ALIGN = 256;
constexpr uint32_t MAX_PROF = 4096;

size_t align_up(size_t x) { return (x + ALIGN - 1) / ALIGN * ALIGN; }

struct Layout {          // byte offsets inside the workspace
    size_t tile_desc, tdesc, plans, tau, hint2, tprev, ghist, tile_cnt, heads, slots, ord, stats, flag;
    size_t qlist, segtab, grptab, grpcnt, segstart, segcnt, segG1, segOut, segstate, pfxlist, total;
};

bool check_offsets(const uint64_t *offsets, uint32_t J)
{
    if (!offsets || J == 0) return false;
    if (offsets[0] != 0) return false;
    for (uint32_t j = 0; j < J; ++j)
        if (offsets[j + 1] <= offsets[j]) return false;
    if (offsets[J] >= (1ull << 32)) return false;
    return true;
}

// Parts of tensor [off, off + n): its tiles cut into equal runs of `scale` x SEG_TILES tiles
// (longer runs for a tensor that would otherwise have more than SEG_MAX_PER_TENSOR parts).
// Every tensor has at least one part.  `scale` grows with the layout (layout_scale) so that
// the selection launch stays at a few workgroups per compute unit.
uint32_t part_tiles(uint64_t off, uint64_t n, uint32_t scale)
{
    const uint64_t nt = (off + n - 1) / TILE - off / TILE + 1;
    uint64_t per = (uint64_t)SEG_TILES * scale;
    if ((nt + per - 1) / per > SEG_MAX_PER_TENSOR)
        per = ((nt + SEG_MAX_PER_TENSOR - 1) / SEG_MAX_PER_TENSOR + SEG_TILES - 1) / SEG_TILES * SEG_TILES;
    return (uint32_t)per;
}

uint32_t tensor_segments(uint64_t off, uint64_t n, uint32_t scale)
{
    const uint64_t nt = (off + n - 1) / TILE - off / TILE + 1;
    const uint64_t per = part_tiles(off, n, scale);
    return (uint32_t)((nt + per - 1) / per);
}

uint32_t layout_scale(const uint64_t *offsets, uint32_t J)
{
    const uint64_t ntiles = (offsets[J] + TILE - 1) / TILE;
    const uint64_t target = 512ull * SEG_TILES;      // tiles that give about 512 parts
    const uint64_t s = (ntiles + target - 1) / target;
    return (uint32_t)(s < 1 ? 1 : (s > 64 ? 64 : s));
}

Layout make_layout(const uint64_t *offsets, uint32_t J, uint32_t W)
{
    const uint64_t n = offsets[J];
    const size_t ntiles = (size_t)((n + TILE - 1) / TILE);
    size_t nseg_total = 0, ncap = 0;
    const uint32_t scale = layout_scale(offsets, J);
    for (uint32_t j = 0; j < J; ++j) {
        const uint32_t ns = tensor_segments(offsets[j], offsets[j + 1] - offsets[j], scale);
        nseg_total += ns;
        ncap += (offsets[j + 1] - offsets[j] >= SEG_MIN_N) ? 1 : 0;
    }
    Layout L;
    size_t o = 0;
    L.tile_desc = o; o = align_up(o + ((size_t)J + 1) * sizeof(uint32_t));   // tensor offsets
    L.tdesc = o;     o = align_up(o + (size_t)J * sizeof(TensorDesc));
    L.plans = o;     o = align_up(o + (size_t)NPLAN * J * sizeof(PlanEntry));
    L.tau = o;       o = align_up(o + (size_t)(W + 1) * J * sizeof(uint32_t));
    L.hint2 = o;     o = align_up(o + (size_t)(W + 1) * J * sizeof(uint32_t));
    L.tprev = o;     o = align_up(o + (size_t)(W + 1) * J * sizeof(uint32_t));
    L.ghist = o;     o = align_up(o + (size_t)J * HBINS * sizeof(uint32_t));
    L.tile_cnt = o;  o = align_up(o + (ntiles + 4) * sizeof(uint32_t));
    L.heads = o;     o = align_up(o + ntiles * HEAD * sizeof(uint2));
    L.slots = o;     o = align_up(o + ntiles * CAPT * sizeof(uint2));
    L.ord = o;       o = align_up(o + (ntiles + J) * CAPT * sizeof(uint2));
    L.stats = o;     o = align_up(o + sizeof(DevStats));
    L.flag = o;      o = align_up(o + 64);
    L.qlist = o;     o = align_up(o + (ntiles + 4) * sizeof(uint32_t));
    L.segtab = o;    o = align_up(o + (nseg_total + 1) * sizeof(SegDesc));
    L.grptab = o;    o = align_up(o + (nseg_total + 1) * sizeof(SegDesc));      // groups <= parts
    L.grpcnt = o;    o = align_up(o + (nseg_total + 1) * sizeof(uint32_t));
    L.segstart = o;  o = align_up(o + (nseg_total + 1) * sizeof(uint32_t));
    L.segcnt = o;    o = align_up(o + (nseg_total + 1) * sizeof(uint32_t));
    L.segG1 = o;     o = align_up(o + (nseg_total + 1) * sizeof(uint32_t));
    L.segOut = o;    o = align_up(o + (nseg_total + 1) * sizeof(uint2));
    L.segstate = o;  o = align_up(o + (size_t)J * sizeof(SegState));
    L.pfxlist = o;   o = align_up(o + (ncap * PFX_CAP + 1) * sizeof(uint4));
    L.total = o;
    return L;
}

struct PlanSlot {
    bool valid = false;
    bool captured = false;             // used while the stream was being captured: never evicted
    double density = 0.0;
    int margin = 0;
    int seg_mode = 0;
    uint32_t nseg_active = 0;          // tensors planned as segmented
    uint64_t K = 0;
    uint64_t wire_words = 0;           // 32-bit words of the wire form's index area
    uint64_t last_use = 0;
};

struct ProfClass {
    std::vector<hipEvent_t> start, stop;
    uint32_t used = 0;
};

uint32_t isqrt_u32(uint32_t x) { return (uint32_t)std::floor(std::sqrt((double)x)); }

// Host-side array of a context: owned (heap) for contexts made by dgs_create, borrowed from
// the caller's stack for the entry point that must not allocate.
template <class T>
struct HostArr {
    T *p = nullptr;
    std::vector<T> own;
    T &operator[](size_t i) const { return p[i]; }
    template <class It> void assign(It first, It last) { own.assign(first, last); p = own.data(); }
    void assign(size_t count, T v) { own.assign(count, v); p = own.data(); }
    void borrow(T *q) { p = q; }
};

}  // namespace

struct dgs_ctx {
    hipStream_t stream = nullptr;
    uint32_t J = 0, W = 0, n = 0, ntiles = 0, nquads = 0;
    int cus = 256;
    HostArr<uint64_t> offsets;
    char *ws = nullptr;
    Layout L{};
    // device views
    uint32_t *toff = nullptr;
    TensorDesc *tdesc = nullptr;
    PlanEntry *plans = nullptr;
    uint32_t *tau = nullptr;
    uint32_t *hint2 = nullptr;
    uint32_t *tprev = nullptr;
    uint32_t *ghist = nullptr;
    uint32_t *tile_cnt = nullptr;
    uint2 *heads = nullptr;
    uint2 *slots = nullptr;
    uint2 *ord = nullptr;
    DevStats *stats = nullptr;
    uint32_t *flag = nullptr;
    uint32_t *qlist = nullptr;         // the tiles that a sampling pass visits
    uint32_t nqlist = 0;               // 0: no sampling on this context
    SegDesc *segtab = nullptr;
    SegDesc *grptab = nullptr;
    uint32_t *grpcnt = nullptr, *segstart = nullptr;
    uint32_t ngroups = 0, gparts = 1;  // join groups; parts per group
    uint32_t bgroup = 8;               // parts per re-collecting workgroup (about 2048 tiles)
    uint32_t *segcnt = nullptr, *segG1 = nullptr;
    uint2 *segOut = nullptr;
    SegState *segstate = nullptr;
    uint4 *pfxlist = nullptr;
    uint32_t nseg_total = 0;
    HostArr<uint32_t> nseg;            // per tensor: parts (at least one)
    float *diff = nullptr;
    float *sent = nullptr;             // W rows: what each worker has been sent (model - sent_k form)
    // plan cache
    PlanSlot plan_slot[NPLAN];
    PlanEntry *plan_stage = nullptr;   // pinned host, NPLAN * J
    uint64_t tick = 0;
    // which density each hint set was produced for (0 = none yet)
    HostArr<double> hint_density;      // W + 1 entries; entry 0 = worker
    bool no_alloc = false;             // tables go up as kernel arguments, nothing is allocated or copied
    // options
    bool force_exact = false, profile = false, validate = false;
    bool force_sample = false;         // never predict, estimate from a sample on every call
    int margin_pct = 50;
    int seg_mode = SEG_MODE_AUTO;
    bool repair_round = true;
    uint32_t spin_limit = 1u << 20;    // polls before a waiting workgroup of the selection gives up
    uint32_t stream_quads = 0;         // 0 = automatic
    uint32_t wire_value_bits = 32;     // wire form: fp32 values, or 16 = bfloat16
    // host counters
    uint64_t calls_worker = 0, calls_pull = 0, calls_push = 0, exact_calls = 0;
    ProfClass prof[DGS_PROF_KINDS];
};

namespace {

// Event pair for one timed kernel launch (null events when profiling is off or full).
struct ProfSlot {
    dgs_ctx *c;
    int kind;
    hipEvent_t ev0 = nullptr, ev1 = nullptr;
    ProfSlot(dgs_ctx *ctx, int k) : c(ctx), kind(k)
    {
        if (!c->profile) return;
        ProfClass &p = c->prof[kind];
        if (p.used >= MAX_PROF) return;
        if (p.used >= p.start.size()) {
            hipEvent_t a, b;
            if (hipEventCreate(&a) != hipSuccess) return;
            if (hipEventCreate(&b) != hipSuccess) { (void)hipEventDestroy(a); return; }
            p.start.push_back(a);
            p.stop.push_back(b);
        }
        ev0 = p.start[p.used];
        ev1 = p.stop[p.used];
    }
    void launched() { if (ev0) ++c->prof[kind].used; }
};

// k_j = ceil(density * n_j) in IEEE double; k2 = rank that sets the next predicted threshold.
// Which tensors take the chain kernels behind the selection: those of at least SEG_MIN_N
// elements whose hinted candidate list is longer than one workgroup selects from
// (SEL_LIST_MAX), and, for a dense request, all of that size (one workgroup would crawl
// through the tensor itself).
void fill_plan(const dgs_ctx *c, double density, int margin_pct, PlanEntry *out, uint64_t *K_out,
               uint32_t *nseg_active, uint64_t *wire_words_out)
{
    {
        const uint64_t list_limit = SEL_LIST_MAX;
        uint64_t K = 0, words = 0;
        uint32_t active = 0;
        for (uint32_t j = 0; j < c->J; ++j) {
            const uint64_t nj = c->offsets[j + 1] - c->offsets[j];
            uint64_t k = (uint64_t)std::ceil(density * (double)nj);
            if (k < 1) k = 1;
            if (k > nj) k = nj;
            uint64_t k2 = k + (k * (uint64_t)margin_pct) / 100 + 4ull * isqrt_u32((uint32_t)k) + 16;
            if (k2 > nj) k2 = nj;
            out[j].k = (uint32_t)k;
            out[j].k2 = (uint32_t)k2;
            out[j].outoff = (uint32_t)K;
            uint64_t k2p = 2 * k + 4ull * isqrt_u32((uint32_t)k) + 16;
            if (k2p > nj) k2p = nj;
            out[j].k2_pull = (uint32_t)k2p;
            bool seg = false;
            if (nj >= SEG_MIN_N && c->seg_mode != SEG_MODE_NEVER) {
                if (density > DENSE_DENSITY)
                    seg = true;   // dense request: the chain reads the tensor itself, one workgroup would crawl
                else
                    seg = c->seg_mode == SEG_MODE_ALWAYS || (k2 > k2p ? k2 : k2p) > list_limit;
            }
            out[j].seg = seg ? 1u : 0u;
            // wire form: local indices of b bits each, the tensor's block padded to whole words
            uint32_t b = 0;
            for (uint64_t top = nj - 1; top; top >>= 1) ++b;
            if (b == 0) b = 1;
            out[j].wire_off = (uint32_t)words;      // fits: words <= K, checked by the caller
            out[j].wire_bits = b;
            out[j].pad2 = 0;
            words += (k * b + 31) / 32;
            active += seg ? 1u : 0u;
            K += k;
        }
        *nseg_active = active;
        *K_out = K;
        *wire_words_out = words;
    }
}

int upload(dgs_ctx *c, void *dst, const void *src, size_t bytes);

// Returns the cache slot holding the plan for `density`, uploading it if new.  A slot used
// while the stream was being captured is never evicted afterwards (the captured graph holds
// its device address), and a plan that would have to be uploaded during capture is refused.
int get_plan(dgs_ctx *c, double density, uint32_t *slot_out, uint64_t *K_out)
{
    ++c->tick;
    bool capturing = false;
    if (!c->no_alloc) {
        hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
        if (hipStreamIsCapturing(c->stream, &cs) == hipSuccess) capturing = (cs != hipStreamCaptureStatusNone);
        else (void)hipGetLastError();
    }
    for (uint32_t s = 0; s < NPLAN; ++s) {
        PlanSlot &p = c->plan_slot[s];
        if (p.valid && p.density == density && p.margin == c->margin_pct && p.seg_mode == c->seg_mode) {
            p.last_use = c->tick;
            if (capturing) p.captured = true;
            *slot_out = s;
            *K_out = p.K;
            return DGS_OK;
        }
    }
    if (capturing) return DGS_ENOTSUP;   // first use of a density: call it once outside the capture
    uint32_t victim = NPLAN;
    bool reuse = true;
    for (uint32_t s = 0; s < NPLAN; ++s) {
        if (!c->plan_slot[s].valid) { victim = s; reuse = false; break; }
        if (c->plan_slot[s].captured) continue;
        if (victim == NPLAN || c->plan_slot[s].last_use < c->plan_slot[victim].last_use) victim = s;
    }
    if (victim == NPLAN) return DGS_ENOTSUP;   // every slot belongs to a captured graph
    if (reuse) {
        // the staging area of this slot may still feed an earlier upload
        if (hipStreamSynchronize(c->stream) != hipSuccess) return DGS_EHIP;
    }
    PlanEntry *stage = c->plan_stage + (size_t)victim * c->J;
    uint64_t K = 0, wire_words = 0;
    uint32_t active = 0;
    fill_plan(c, density, c->margin_pct, stage, &K, &active, &wire_words);
    if (K >= (1ull << 32)) return DGS_EINVAL;
    const int rc = upload(c, c->plans + (size_t)victim * c->J, stage, (size_t)c->J * sizeof(PlanEntry));
    if (rc != DGS_OK) return rc;
    PlanSlot &p = c->plan_slot[victim];
    p.valid = true;
    p.captured = false;
    p.density = density;
    p.margin = c->margin_pct;
    p.seg_mode = c->seg_mode;
    p.nseg_active = active;
    p.K = K;
    p.wire_words = wire_words;
    p.last_use = c->tick;
    *slot_out = victim;
    *K_out = K;
    return DGS_OK;
}

bool aligned16(const void *p) { return ((uintptr_t)p & 15u) == 0; }
bool aligned4(const void *p) { return ((uintptr_t)p & 3u) == 0; }

uint32_t stream_blocks(const dgs_ctx *c, int mode, uint32_t *qpb_out)
{
    uint32_t qpb;
    if (mode == MODE_HIST) {
        // long contiguous spans per workgroup keep the number of histogram flushes small
        const uint32_t target = (uint32_t)c->cus * 8u;
        qpb = (c->nquads + target - 1) / target;
    } else {
        qpb = c->stream_quads ? c->stream_quads : 1u;
    }
    if (qpb == 0) qpb = 1;
    *qpb_out = qpb;
    return (c->nquads + qpb - 1) / qpb;
}

// The selection pipeline shared by the worker step and the pull.
//   op_stream: OP_FMA (worker: grad + state) or OP_IDENT (pull: a difference row)
int run_selection(dgs_ctx *c, int op_stream, int op_select, const float *grad, float *state, float lr,
                  float m, double density, uint32_t hint_set, uint32_t *idx_out, float *val_out,
                  uint64_t *nnz_out, int prof_stream, int prof_select, int prof_seg)
{
    uint32_t slot;
    uint64_t K;
    int rc = get_plan(c, density, &slot, &K);
    if (rc != DGS_OK) return rc;
    if (nnz_out) *nnz_out = K;

    const bool vec = aligned16(state) && (op_stream == OP_IDENT || aligned16(grad));
    // the read-only pass that sees the same values again (second pass of the non-predicted path,
    // repair round): the worker's are in `state` by then, a model - sent_k pull recomputes them
    const int op_again = (op_stream == OP_SUB) ? OP_SUB : OP_IDENT;
    const bool dense_req = density > DENSE_DENSITY;
    const bool exact = !dense_req && (c->force_exact || c->force_sample || c->hint_density[hint_set] != density);
    uint32_t *tau = c->tau + (size_t)hint_set * c->J;
    const PlanEntry *plan = c->plans + (size_t)slot * c->J;

    StreamArgs sa{};
    sa.grad = grad;
    sa.state = state;
    sa.toff = c->toff;
    sa.J = c->J;
    sa.tau = tau;
    sa.tile_cnt = c->tile_cnt;
    sa.heads = c->heads;
    sa.slots = c->slots;
    sa.ghist = c->ghist;
    sa.n = c->n;
    sa.ntiles = c->ntiles;
    sa.nquads = c->nquads;
    sa.lr = lr;
    // the state goes back write-through while it fits the last-level cache, non-temporal beyond
    sa.store_mode = ((size_t)c->n * sizeof(float) > (192u << 20)) ? STORE_NT : STORE_WT;

    const bool have_seg = c->plan_slot[slot].nseg_active != 0;
    uint32_t *tprev = c->tprev + (size_t)hint_set * c->J;
    if (dense_req && have_seg) {
        // dense request with large tensors: the accumulate pass also histograms the keys, and
        // k_pick turns that into a lower bound of each k-th key; the chain then reads the
        // tensors themselves
        ProfSlot ps(c, prof_stream);
        const uint32_t blocks = stream_blocks(c, MODE_HIST, &sa.quads_per_block);
        launch_stream(op_stream, MODE_HIST, vec, sa, blocks, c->stream, ps.ev0, ps.ev1);
        ps.launched();
        launch_pick(c->tdesc, plan, c->ghist, tau, tprev, c->stats, c->J, false, c->stream);
    } else if (dense_req) {
        if (op_stream == OP_FMA) {
            ProfSlot ps(c, prof_stream);
            const uint32_t blocks = stream_blocks(c, MODE_PLAIN, &sa.quads_per_block);
            launch_stream(OP_FMA, MODE_PLAIN, vec, sa, blocks, c->stream, ps.ev0, ps.ev1);
            ps.launched();
        }
    } else if (exact && !c->force_exact && c->nqlist != 0) {
        // No usable prediction: a histogram of a sample of the buffer gives the thresholds (k_pick
        // scales the ranks), and the call goes on as a predicted one; where the estimate lets too
        // few candidates through, the selection launch collects that tensor again.
        ++c->exact_calls;
        ProfSlot ps(c, DGS_PROF_EXACT_EXTRA);
        StreamArgs sb = sa;
        sb.tile_list = c->qlist;
        sb.nlist = c->nqlist;
        sb.nquads = (c->nqlist + WAVES_PER_BLOCK - 1) / WAVES_PER_BLOCK;
        // a few workgroups per compute unit: enough loads in flight, but every workgroup ends with a
        // flush of its LDS histogram into the tensors' counters, and those atomics meet on a few
        // hundred addresses (at 1e9 parameters: 119 us with two per unit, 90 with four, 101 with eight)
        const uint32_t wgs = (uint32_t)c->cus * DGS_SAMPLE_WGS_PER_CU;
        sb.quads_per_block = std::max<uint32_t>(1u, (sb.nquads + wgs - 1u) / wgs);
        launch_stream(op_stream, MODE_SAMPLE, vec, sb, (sb.nquads + sb.quads_per_block - 1u) / sb.quads_per_block,
                      c->stream, ps.ev0, ps.ev1);
        ps.launched();
        launch_pick(c->tdesc, plan, c->ghist, tau, tprev, c->stats, c->J, true, c->stream);
        ProfSlot pc(c, prof_stream);
        const uint32_t blocks = stream_blocks(c, MODE_COLLECT, &sa.quads_per_block);
        launch_stream(op_stream, MODE_COLLECT, vec, sa, blocks, c->stream, pc.ev0, pc.ev1);
        pc.launched();
    } else if (exact) {
        ++c->exact_calls;
        {
            ProfSlot ps(c, prof_stream);
            const uint32_t blocks = stream_blocks(c, MODE_HIST, &sa.quads_per_block);
            launch_stream(op_stream, MODE_HIST, vec, sa, blocks, c->stream, ps.ev0, ps.ev1);
            ps.launched();
        }
        {
            launch_pick(c->tdesc, plan, c->ghist, tau, tprev, c->stats, c->J, false, c->stream);
            ProfSlot ps(c, DGS_PROF_EXACT_EXTRA);
            StreamArgs sb = sa;
            if (op_again == OP_IDENT) sb.grad = nullptr;
            const uint32_t blocks = stream_blocks(c, MODE_COLLECT, &sb.quads_per_block);
            launch_stream(op_again, MODE_COLLECT, op_again == OP_IDENT ? aligned16(state) : vec, sb, blocks,
                          c->stream, ps.ev0, ps.ev1);
            ps.launched();
        }
    } else {
        ProfSlot ps(c, prof_stream);
        const uint32_t blocks = stream_blocks(c, MODE_COLLECT, &sa.quads_per_block);
        launch_stream(op_stream, MODE_COLLECT, vec, sa, blocks, c->stream, ps.ev0, ps.ev1);
        ps.launched();
    }

    SelectArgs se{};
    se.state = state;
    se.model = (op_stream == OP_SUB) ? grad : nullptr;
    se.tdesc = c->tdesc;
    se.plan = plan;
    se.segtab = c->segtab;
    se.grptab = c->grptab;
    se.grpcnt = c->grpcnt;
    se.segstart = c->segstart;
    se.ngroups = c->ngroups;
    se.gparts = c->gparts;
    se.bgroup = c->bgroup;
    se.tau = tau;
    se.tile_cnt = c->tile_cnt;
    se.heads = c->heads;
    se.slots = c->slots;
    se.ord = c->ord;
    se.hint2 = c->hint2 + (size_t)hint_set * c->J;
    se.tprev = tprev;
    se.ghist = c->ghist;
    se.segstate = c->segstate;
    se.segcnt = c->segcnt;
    se.segG1 = c->segG1;
    se.segOut = c->segOut;
    se.pfxlist = c->pfxlist;
    se.out_idx = idx_out;
    se.out_val = val_out;
    se.stats = c->stats;
    se.toff = c->toff;
    se.m = m;
    se.n = c->n;
    se.ntiles = c->ntiles;
    se.J = c->J;
    se.nparts = c->nseg_total;
    se.dense = dense_req ? 1u : 0u;
    se.write_hint = dense_req ? 0u : 1u;
    se.exact_mode = exact ? 1u : 0u;
    se.repair = (c->repair_round && !dense_req) ? 1u : 0u;   // a dense request has no lists to collect again
    se.spin_limit = c->spin_limit;
    {
        ProfSlot ps(c, prof_select);
        launch_select(op_select, se, c->stream, ps.ev0, ps.ev1);
        ps.launched();
    }
    if (have_seg) {
        ProfSlot ps(c, prof_seg);
        launch_chain(op_select, se, c->stream, ps.ev0, ps.ev1);
        ps.launched();
    }
    if (!dense_req) c->hint_density[hint_set] = density;
    else if (have_seg) c->hint_density[hint_set] = 0.0;   // k_pick has overwritten this stream's hints
    if (hipGetLastError() != hipSuccess) return DGS_EHIP;
    return DGS_OK;
}

// Point the context's device views into its workspace.
void carve_workspace(dgs_ctx *c, void *workspace, const Layout &L)
{
    c->ws = (char *)workspace;
    c->L = L;
    c->toff = (uint32_t *)(c->ws + L.tile_desc);
    c->tdesc = (TensorDesc *)(c->ws + L.tdesc);
    c->plans = (PlanEntry *)(c->ws + L.plans);
    c->tau = (uint32_t *)(c->ws + L.tau);
    c->hint2 = (uint32_t *)(c->ws + L.hint2);
    c->tprev = (uint32_t *)(c->ws + L.tprev);
    c->ghist = (uint32_t *)(c->ws + L.ghist);
    c->tile_cnt = (uint32_t *)(c->ws + L.tile_cnt);
    c->heads = (uint2 *)(c->ws + L.heads);
    c->slots = (uint2 *)(c->ws + L.slots);
    c->ord = (uint2 *)(c->ws + L.ord);
    c->stats = (DevStats *)(c->ws + L.stats);
    c->flag = (uint32_t *)(c->ws + L.flag);
    c->qlist = (uint32_t *)(c->ws + L.qlist);
    c->segtab = (SegDesc *)(c->ws + L.segtab);
    c->grptab = (SegDesc *)(c->ws + L.grptab);
    c->grpcnt = (uint32_t *)(c->ws + L.grpcnt);
    c->segstart = (uint32_t *)(c->ws + L.segstart);
    c->segcnt = (uint32_t *)(c->ws + L.segcnt);
    c->segG1 = (uint32_t *)(c->ws + L.segG1);
    c->segOut = (uint2 *)(c->ws + L.segOut);
    c->segstate = (SegState *)(c->ws + L.segstate);
    c->pfxlist = (uint4 *)(c->ws + L.pfxlist);
}

// Tensor, segment and initial-threshold tables of a layout, into host arrays of J,
// (W + 1) J, J + 1 and (sum of tensor_segments) entries; fills c->nseg and c->nseg_total.
void fill_tables(dgs_ctx *c, TensorDesc *td, uint32_t *tau0, uint32_t *toff, SegDesc *segs, SegDesc *groups)
{
    const uint32_t J = c->J, W = c->W;
    uint32_t pfx_slots = 0, nsegs = 0;
    const uint32_t scale = layout_scale(&c->offsets[0], J);
    for (uint32_t j = 0; j < J; ++j) {
        td[j].off = (uint32_t)c->offsets[j];
        td[j].n = (uint32_t)(c->offsets[j + 1] - c->offsets[j]);
        td[j].big = td[j].n > SMALL_N ? 1u : 0u;
        td[j].grp_first = td[j].ngrp = 0;
        const uint32_t ns = tensor_segments(c->offsets[j], c->offsets[j + 1] - c->offsets[j], scale);
        const uint32_t per = part_tiles(c->offsets[j], c->offsets[j + 1] - c->offsets[j], scale);
        td[j].seg_first = nsegs;
        td[j].nseg = ns;
        td[j].pfx_slot = (td[j].n >= SEG_MIN_N) ? pfx_slots++ : 0u;
        c->nseg[j] = ns;
        const uint32_t tlo = td[j].off / TILE, thi = (td[j].off + td[j].n - 1) / TILE;
        for (uint32_t sidx = 0; sidx < ns; ++sidx) {
            SegDesc d;
            d.j = j;
            d.tile0 = tlo + sidx * per;
            d.ntiles = (thi + 1 - d.tile0 < per) ? (thi + 1 - d.tile0) : per;
            d.sidx = sidx;
            segs[nsegs++] = d;
        }
        for (uint32_t w = 0; w <= W; ++w) tau0[(size_t)w * J + j] = td[j].big ? 1u : TAU_NEVER;
    }
    for (uint32_t j = 0; j <= J; ++j) toff[j] = (uint32_t)c->offsets[j];
    c->nseg_total = nsegs;
    // re-collecting workgroups: both roles together about as many as the compute units that the
    // tensors' selecting workgroups (at most one per tensor) leave free, each looking after at
    // most 8 consecutive parts
    const uint32_t busy = std::min<uint32_t>(J, (uint32_t)c->cus / 2u);
    const uint32_t per_role = std::max<uint32_t>(16u, ((uint32_t)c->cus - busy) / 2u);
    c->bgroup = std::min<uint32_t>(8u, std::max<uint32_t>(1u, (nsegs + per_role - 1u) / per_role));
    // Join groups: runs of `gparts` consecutive parts (about GROUP_TILES tiles).  The launch takes
    // the groups of the tensors with several groups first: those tensors end with a gather and
    // a selection by the last group to arrive, the critical path of the launch.
    const uint32_t gparts = std::max<uint32_t>(1u, GROUP_TILES / (SEG_TILES * scale));
    c->gparts = gparts;
    uint32_t g = 0;
    for (uint32_t pass = 0; pass < 2; ++pass)
        for (uint32_t j = 0; j < J; ++j) {
            const uint32_t ng = (td[j].nseg + gparts - 1) / gparts;
            if ((pass == 0) != (ng > 1)) continue;
            td[j].grp_first = g;
            td[j].ngrp = ng;
            for (uint32_t gi = 0; gi < ng; ++gi) {
                const SegDesc &first = segs[td[j].seg_first + gi * gparts];
                const SegDesc &last = segs[td[j].seg_first + std::min(td[j].nseg, (gi + 1) * gparts) - 1];
                SegDesc d;
                d.j = j;
                d.tile0 = first.tile0;
                d.ntiles = last.tile0 + last.ntiles - first.tile0;
                d.sidx = gi;
                groups[g++] = d;
            }
        }
    c->ngroups = g;
}

// Host -> device: a copy on the stream, or -- for the context that must not allocate or copy
// -- kernels that carry the bytes as their arguments.
int upload(dgs_ctx *c, void *dst, const void *src, size_t bytes)
{
    if (bytes == 0) return DGS_OK;
    if (c->no_alloc) {
        launch_put_words((uint32_t *)dst, (const uint32_t *)src, bytes / 4, c->stream);
        return DGS_OK;
    }
    return hipMemcpyAsync(dst, src, bytes, hipMemcpyHostToDevice, c->stream) == hipSuccess ? DGS_OK : DGS_EHIP;
}

// Tables up, counters cleared: what a context's workspace holds before its first call.
int upload_tables(dgs_ctx *c, const TensorDesc *td, const uint32_t *tau0, const uint32_t *toff, const SegDesc *segs,
                  const SegDesc *groups)
{
    const uint32_t J = c->J, W = c->W;
    int rc = upload(c, c->toff, toff, ((size_t)J + 1) * sizeof(uint32_t));
    if (rc == DGS_OK) rc = upload(c, c->tdesc, td, (size_t)J * sizeof(TensorDesc));
    if (rc == DGS_OK) rc = upload(c, c->tau, tau0, (size_t)(W + 1) * J * sizeof(uint32_t));
    if (rc == DGS_OK) rc = upload(c, c->segtab, segs, (size_t)c->nseg_total * sizeof(SegDesc));
    if (rc == DGS_OK) rc = upload(c, c->grptab, groups, (size_t)c->ngroups * sizeof(SegDesc));
    if (rc != DGS_OK) return rc;
    launch_fill_u32(c->hint2, 0u, (size_t)(W + 1) * J, c->stream);
    launch_fill_u32(c->tprev, 0u, (size_t)(W + 1) * J, c->stream);
    launch_fill_u32(c->ghist, 0u, (size_t)J * HBINS, c->stream);
    launch_fill_u32(c->tile_cnt, 0u, (size_t)c->ntiles + 4, c->stream);
    launch_fill_u32((uint32_t *)c->stats, 0u, sizeof(DevStats) / 4, c->stream);
    launch_fill_u32(c->flag, 0u, 16, c->stream);
    launch_fill_u32((uint32_t *)c->segstate, 0u, (size_t)J * sizeof(SegState) / 4, c->stream);
    return hipGetLastError() == hipSuccess ? DGS_OK : DGS_EHIP;
}

// DGS_OPT_VALIDATE: indices strictly ascending and inside [0, n), checked on the device
// before anything is modified (waits for the stream).
int validate_message(dgs_ctx *c, const uint32_t *idx, uint64_t nnz)
{
    launch_fill_u32(c->flag, 0u, 1, c->stream);
    launch_validate_idx(idx, (uint32_t)nnz, c->n, c->flag, c->stream);
    uint32_t bad = 0;
    if (hipMemcpyAsync(&bad, c->flag, 4, hipMemcpyDeviceToHost, c->stream) != hipSuccess) return DGS_EHIP;
    if (hipStreamSynchronize(c->stream) != hipSuccess) return DGS_EHIP;
    return bad ? DGS_EINVAL : DGS_OK;
}

}  // namespace

extern "C" {

size_t dgs_workspace_bytes(const uint64_t *offsets, uint32_t J, uint32_t W)
{
    if (!check_offsets(offsets, J)) return 0;
    return make_layout(offsets, J, W).total;
}

int dgs_create(dgs_ctx **out, const uint64_t *offsets, uint32_t J, uint32_t W, void *workspace,
               size_t workspace_bytes, void *hip_stream)
{
    if (!out) return DGS_EINVAL;
    *out = nullptr;
    if (!check_offsets(offsets, J) || !workspace) return DGS_EINVAL;
    if (((uintptr_t)workspace & (ALIGN - 1)) != 0) return DGS_EINVAL;
    const Layout L = make_layout(offsets, J, W);
    if (workspace_bytes < L.total) return DGS_ENOMEM;

    dgs_ctx *c = new (std::nothrow) dgs_ctx();
    if (!c) return DGS_ENOMEM;
    c->stream = (hipStream_t)hip_stream;
    c->J = J;
    c->W = W;
    c->n = (uint32_t)offsets[J];
    c->ntiles = (c->n + TILE - 1) / TILE;
    c->nquads = (c->ntiles + WAVES_PER_BLOCK - 1) / WAVES_PER_BLOCK;
    c->offsets.assign(offsets, offsets + J + 1);
    carve_workspace(c, workspace, L);
    c->hint_density.assign((size_t)W + 1, 0.0);

    int dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess &&
        prop.multiProcessorCount > 0)
        c->cus = prop.multiProcessorCount;
    const char *env = std::getenv("DGS_FORCE_EXACT");
    if (env && env[0] == '1') c->force_exact = true;
    env = std::getenv("DGS_SEGMENTED");
    if (env && env[0] >= '0' && env[0] <= '2') c->seg_mode = env[0] - '0';
    env = std::getenv("DGS_STREAM_QUADS");
    if (env) c->stream_quads = (uint32_t)std::strtoul(env, nullptr, 10);

    // host-side plan: tensor and tile descriptors
    uint32_t nseg_total = 0;
    for (uint32_t j = 0; j < J; ++j)
        nseg_total += tensor_segments(offsets[j], offsets[j + 1] - offsets[j], layout_scale(offsets, J));
    std::vector<TensorDesc> td(J);
    std::vector<uint32_t> tau0((size_t)(W + 1) * J);
    std::vector<SegDesc> segs(nseg_total + 1);
    std::vector<uint32_t> toff(J + 1);
    std::vector<SegDesc> groups(nseg_total + 1);
    c->nseg.assign(J, 0u);
    fill_tables(c, td.data(), tau0.data(), toff.data(), segs.data(), groups.data());

    // What a sampling pass visits: every 16th tile of the buffer, and every tile of the tensors of
    // at most 64 tiles, whose ranks are too small to estimate from a sixteenth.
    std::vector<uint32_t> qlist;
    {
        std::vector<uint8_t> mark(c->ntiles, 0);
        for (uint32_t t = 0; t < c->ntiles; t += 16) mark[t] = 1;
        for (uint32_t j = 0; j < J; ++j) {
            if (!td[j].big) continue;
            const uint32_t tlo = td[j].off / TILE, thi = (td[j].off + td[j].n - 1) / TILE;
            if (thi - tlo + 1 > 64) continue;
            for (uint32_t t = tlo; t <= thi; ++t) mark[t] = 1;
        }
        for (uint32_t t = 0; t < c->ntiles; ++t)
            if (mark[t]) qlist.push_back(t);
    }
    c->nqlist = (uint32_t)qlist.size();
    bool ok = true;
    ok = ok && upload(c, c->qlist, qlist.data(), qlist.size() * sizeof(uint32_t)) == DGS_OK;
    ok = ok && hipHostMalloc((void **)&c->plan_stage, (size_t)NPLAN * J * sizeof(PlanEntry), hipHostMallocDefault) == hipSuccess;
    ok = ok && upload_tables(c, td.data(), tau0.data(), toff.data(), segs.data(), groups.data()) == DGS_OK;
    ok = ok && hipStreamSynchronize(c->stream) == hipSuccess;
    ok = ok && hipGetLastError() == hipSuccess;
    if (!ok) {
        if (c->plan_stage) (void)hipHostFree(c->plan_stage);
        delete c;
        return DGS_EHIP;
    }
    *out = c;
    return DGS_OK;
}

int dgs_destroy(dgs_ctx *c)
{
    if (!c) return DGS_EINVAL;
    (void)hipStreamSynchronize(c->stream);
    for (auto &p : c->prof) {
        for (auto e : p.start) (void)hipEventDestroy(e);
        for (auto e : p.stop) (void)hipEventDestroy(e);
    }
    if (c->plan_stage) (void)hipHostFree(c->plan_stage);
    delete c;
    return DGS_OK;
}

int dgs_nnz(const dgs_ctx *c, double density, uint64_t *K_out)
{
    if (!c || !K_out) return DGS_EINVAL;
    if (!(density > 0.0) || density > 1.0) return DGS_EINVAL;
    uint64_t K = 0;
    for (uint32_t j = 0; j < c->J; ++j) {
        const uint64_t nj = c->offsets[j + 1] - c->offsets[j];
        uint64_t k = (uint64_t)std::ceil(density * (double)nj);
        if (k < 1) k = 1;
        if (k > nj) k = nj;
        K += k;
    }
    *K_out = K;
    return DGS_OK;
}

int dgs_worker_step(dgs_ctx *c, const float *grad, float *momentum, float *residual, float lr, float m,
                    double density, uint32_t *idx_out, float *val_out, uint64_t *nnz_out)
{
    if (!c || !grad || !idx_out || !val_out) return DGS_EINVAL;
    if (!momentum && !residual) return DGS_EINVAL;
    if (momentum && residual) return DGS_ENOTSUP;
    if (!(density > 0.0) || density > 1.0) return DGS_EINVAL;
    if (!(m >= 0.0f) || !(m < 1.0f)) return DGS_EINVAL;
    if (residual && m != 0.0f) return DGS_EINVAL;
    if (!std::isfinite(lr)) return DGS_EINVAL;
    float *state = momentum ? momentum : residual;
    if (!aligned4(grad) || !aligned4(state) || !aligned4(idx_out) || !aligned4(val_out)) return DGS_EINVAL;
    ++c->calls_worker;
    return run_selection(c, OP_FMA, SEL_WORKER, grad, state, lr, m, density, 0, idx_out, val_out, nnz_out,
                         DGS_PROF_WORKER_STREAM, DGS_PROF_WORKER_SELECT, DGS_PROF_WORKER_SEGMENTED);
}

// ---------------------------------------------------------------------------
// the entry point that allocates nothing
// ---------------------------------------------------------------------------

namespace {

// Scratch of dgs_worker_step_static: in place of the caller-allocated workspace of a context.
// One copy per GPU, held until the process ends.
static __device__ __align__(256) unsigned char scratch[DGS_STATIC_SCRATCH_BYTES];

constexpr int STATIC_MAX_DEVICES = 64;
constexpr uint32_t STATIC_MAX_SEGS = 1024;
void *g_scratch_ptr[STATIC_MAX_DEVICES];   // device address of `scratch`, per device (0 = not asked yet)
std::mutex g_scratch_mutex;

// Device address of this GPU's copy of `scratch`, resolved once per device with that device
// current.  The array's name is only a host-side handle: everything on the host uses the
// address returned here.
int static_scratch(void **out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= STATIC_MAX_DEVICES) return DGS_EHIP;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
            (void)hipGetLastError();
            return DGS_EHIP;
        }
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return DGS_OK;
}

}  // namespace

int dgs_worker_step_static(const uint64_t *offsets, uint32_t J, const float *grad, float *momentum,
                           float *residual, float lr, float m, double density, uint32_t *idx_out,
                           float *val_out, uint64_t *nnz_out, void *hip_stream)
{
    if (!check_offsets(offsets, J) || !grad || !idx_out || !val_out) return DGS_EINVAL;
    if (!momentum && !residual) return DGS_EINVAL;
    if (momentum && residual) return DGS_ENOTSUP;
    if (!(density > 0.0) || density > 1.0) return DGS_EINVAL;
    if (!(m >= 0.0f) || !(m < 1.0f)) return DGS_EINVAL;
    if (residual && m != 0.0f) return DGS_EINVAL;
    if (!std::isfinite(lr)) return DGS_EINVAL;
    float *state = momentum ? momentum : residual;
    if (!aligned4(grad) || !aligned4(state) || !aligned4(idx_out) || !aligned4(val_out)) return DGS_EINVAL;
    // limits: the tables live on this call's stack, the workspace in the static array
    if (J > DGS_STATIC_MAX_TENSORS) return DGS_ECAPACITY;
    const Layout L = make_layout(offsets, J, 0);
    if (L.total > DGS_STATIC_SCRATCH_BYTES) return DGS_ECAPACITY;
    uint32_t nseg_total = 0;
    for (uint32_t j = 0; j < J; ++j)
        nseg_total += tensor_segments(offsets[j], offsets[j + 1] - offsets[j], layout_scale(offsets, J));
    if (nseg_total > STATIC_MAX_SEGS) return DGS_ECAPACITY;
    void *ws = nullptr;
    int rc = static_scratch(&ws);
    if (rc != DGS_OK) return rc;

    // a context that lives on this stack: no heap, no pinned memory, no events
    uint64_t offs[DGS_STATIC_MAX_TENSORS + 1];
    uint32_t nseg[DGS_STATIC_MAX_TENSORS];
    double hint_density[1] = {0.0};
    TensorDesc td[DGS_STATIC_MAX_TENSORS];
    uint32_t tau0[DGS_STATIC_MAX_TENSORS], toff[DGS_STATIC_MAX_TENSORS + 1];
    SegDesc segs[STATIC_MAX_SEGS + 1];
    SegDesc groups[STATIC_MAX_SEGS + 1];
    PlanEntry plan[DGS_STATIC_MAX_TENSORS];
    for (uint32_t j = 0; j <= J; ++j) offs[j] = offsets[j];
    dgs_ctx c;
    c.no_alloc = true;
    c.stream = (hipStream_t)hip_stream;
    c.J = J;
    c.W = 0;
    c.n = (uint32_t)offsets[J];
    c.ntiles = (c.n + TILE - 1) / TILE;
    c.nquads = (c.ntiles + WAVES_PER_BLOCK - 1) / WAVES_PER_BLOCK;
    c.offsets.borrow(offs);
    c.nseg.borrow(nseg);
    c.hint_density.borrow(hint_density);
    c.plan_stage = plan;               // one density per call: only the first cache slot is used
    carve_workspace(&c, ws, L);
    fill_tables(&c, td, tau0, toff, segs, groups);
    // every call starts from a clean workspace (the array keeps the previous call's contents);
    // with no threshold hints the step takes the two-pass path
    rc = upload_tables(&c, td, tau0, toff, segs, groups);
    if (rc != DGS_OK) return rc;
    return run_selection(&c, OP_FMA, SEL_WORKER, grad, state, lr, m, density, 0, idx_out, val_out, nnz_out,
                         DGS_PROF_WORKER_STREAM, DGS_PROF_WORKER_SELECT, DGS_PROF_WORKER_SEGMENTED);
}

int dgs_server_attach(dgs_ctx *c, float *diff)
{
    if (!c || !diff || c->W == 0) return DGS_EINVAL;
    if (!aligned4(diff)) return DGS_EINVAL;
    c->diff = diff;
    return DGS_OK;
}

int dgs_server_push(dgs_ctx *c, float *model, uint32_t worker_id, const uint32_t *idx, const float *val,
                    uint64_t nnz)
{
    if (!c || !c->diff) return DGS_EINVAL;
    if (worker_id >= c->W) return DGS_EINVAL;
    if (nnz > c->n) return DGS_EINVAL;
    if (nnz && (!idx || !val)) return DGS_EINVAL;
    if (model && !aligned4(model)) return DGS_EINVAL;
    if (c->validate && nnz) {
        const int rc = validate_message(c, idx, nnz);
        if (rc != DGS_OK) return rc;
    }
    ++c->calls_push;
    {
        ProfSlot ps(c, DGS_PROF_PUSH);
        launch_push(model, c->diff, c->W, c->n, idx, val, (uint32_t)nnz, c->stream, ps.ev0, ps.ev1);
        if (nnz && c->W + (model ? 1u : 0u) > 0) ps.launched();
    }
    if (hipGetLastError() != hipSuccess) return DGS_EHIP;
    return DGS_OK;
}

int dgs_server_pull(dgs_ctx *c, uint32_t worker_id, double density, uint32_t *idx_out, float *val_out,
                    uint64_t *nnz_out)
{
    if (!c || !c->diff || !idx_out || !val_out) return DGS_EINVAL;
    if (worker_id >= c->W) return DGS_EINVAL;
    if (!(density > 0.0) || density > 1.0) return DGS_EINVAL;
    if (!aligned4(idx_out) || !aligned4(val_out)) return DGS_EINVAL;
    float *row = c->diff + (size_t)worker_id * c->n;
    ++c->calls_pull;
    return run_selection(c, OP_IDENT, SEL_PULL, nullptr, row, 0.0f, 0.0f, density, 1 + worker_id, idx_out,
                         val_out, nnz_out, DGS_PROF_PULL_STREAM, DGS_PROF_PULL_SELECT, DGS_PROF_PULL_SEGMENTED);
}

int dgs_server_attach_sent(dgs_ctx *c, float *sent)
{
    if (!c || !sent || c->W == 0) return DGS_EINVAL;
    if (!aligned4(sent)) return DGS_EINVAL;
    c->sent = sent;
    return DGS_OK;
}

int dgs_server_push_model(dgs_ctx *c, float *model, const uint32_t *idx, const float *val, uint64_t nnz)
{
    if (!c || !model) return DGS_EINVAL;
    if (nnz > c->n) return DGS_EINVAL;
    if (nnz && (!idx || !val)) return DGS_EINVAL;
    if (!aligned4(model)) return DGS_EINVAL;
    if (c->validate && nnz) {
        const int rc = validate_message(c, idx, nnz);
        if (rc != DGS_OK) return rc;
    }
    ++c->calls_push;
    {
        ProfSlot ps(c, DGS_PROF_PUSH);
        launch_push(model, nullptr, 0, c->n, idx, val, (uint32_t)nnz, c->stream, ps.ev0, ps.ev1);
        if (nnz) ps.launched();
    }
    if (hipGetLastError() != hipSuccess) return DGS_EHIP;
    return DGS_OK;
}

int dgs_server_pull_sent(dgs_ctx *c, const float *model, uint32_t worker_id, double density,
                         uint32_t *idx_out, float *val_out, uint64_t *nnz_out)
{
    if (!c || !c->sent || !model || !idx_out || !val_out) return DGS_EINVAL;
    if (worker_id >= c->W) return DGS_EINVAL;
    if (!(density > 0.0) || density > 1.0) return DGS_EINVAL;
    if (!aligned4(model) || !aligned4(idx_out) || !aligned4(val_out)) return DGS_EINVAL;
    float *row = c->sent + (size_t)worker_id * c->n;
    ++c->calls_pull;
    return run_selection(c, OP_SUB, SEL_PULL_V, model, row, 0.0f, 0.0f, density, 1 + worker_id, idx_out,
                         val_out, nnz_out, DGS_PROF_PULL_STREAM, DGS_PROF_PULL_SELECT, DGS_PROF_PULL_SEGMENTED);
}

namespace {

// Every nonzero of `row` (model == nullptr) or of model - row; waits for the count.
int pull_all(dgs_ctx *c, float *row, const float *model, uint32_t *idx_out, float *val_out, uint64_t capacity,
             uint64_t *nnz_out)
{
    uint32_t *total = c->flag + 4;
    launch_pull_all_count(row, model, c->n, c->ntiles, c->tile_cnt, c->stream);
    launch_pull_all_scan(c->tile_cnt, c->ntiles, total, c->stream);
    uint32_t cnt = 0;
    if (hipMemcpyAsync(&cnt, total, 4, hipMemcpyDeviceToHost, c->stream) != hipSuccess) return DGS_EHIP;
    if (hipStreamSynchronize(c->stream) != hipSuccess) return DGS_EHIP;
    *nnz_out = cnt;
    if (cnt > capacity) return DGS_ECAPACITY;
    if (cnt) launch_pull_all_emit(row, model, c->n, c->ntiles, c->tile_cnt, idx_out, val_out, c->stream);
    ++c->calls_pull;
    if (hipGetLastError() != hipSuccess) return DGS_EHIP;
    return DGS_OK;
}

}  // namespace

int dgs_server_pull_all(dgs_ctx *c, uint32_t worker_id, uint32_t *idx_out, float *val_out,
                        uint64_t capacity, uint64_t *nnz_out)
{
    if (!c || !c->diff || !nnz_out) return DGS_EINVAL;
    if (worker_id >= c->W) return DGS_EINVAL;
    if (capacity && (!idx_out || !val_out)) return DGS_EINVAL;
    return pull_all(c, c->diff + (size_t)worker_id * c->n, nullptr, idx_out, val_out, capacity, nnz_out);
}

int dgs_server_pull_all_sent(dgs_ctx *c, const float *model, uint32_t worker_id, uint32_t *idx_out,
                             float *val_out, uint64_t capacity, uint64_t *nnz_out)
{
    if (!c || !c->sent || !model || !nnz_out) return DGS_EINVAL;
    if (worker_id >= c->W || !aligned4(model)) return DGS_EINVAL;
    if (capacity && (!idx_out || !val_out)) return DGS_EINVAL;
    return pull_all(c, c->sent + (size_t)worker_id * c->n, model, idx_out, val_out, capacity, nnz_out);
}

int dgs_apply_sparse(dgs_ctx *c, float *dst, const uint32_t *idx, const float *val, uint64_t nnz, float sign)
{
    if (!c || !dst) return DGS_EINVAL;
    if (nnz > c->n) return DGS_EINVAL;
    if (nnz && (!idx || !val)) return DGS_EINVAL;
    if (!aligned4(dst)) return DGS_EINVAL;
    if (c->validate && nnz) {
        const int rc = validate_message(c, idx, nnz);
        if (rc != DGS_OK) return rc;
    }
    launch_apply(dst, c->n, idx, val, (uint32_t)nnz, sign, c->stream);
    if (hipGetLastError() != hipSuccess) return DGS_EHIP;
    return DGS_OK;
}

int dgs_wire_bytes(dgs_ctx *c, double density, uint64_t *bytes_out)
{
    if (!c || !bytes_out || !(density > 0.0) || density > 1.0) return DGS_EINVAL;
    uint32_t slot;
    uint64_t K;
    const int rc = get_plan(c, density, &slot, &K);
    if (rc != DGS_OK) return rc;
    const uint64_t vw = (c->wire_value_bits == 16) ? (K + 1) / 2 : K;
    *bytes_out = 4ull * (vw + c->plan_slot[slot].wire_words);
    return DGS_OK;
}

namespace {

// Reads the device flag the validating kernels set (synchronises).
int read_flag(dgs_ctx *c, uint32_t *out)
{
    if (hipMemcpyAsync(out, c->flag, sizeof(uint32_t), hipMemcpyDeviceToHost, c->stream) != hipSuccess)
        return DGS_EHIP;
    if (hipStreamSynchronize(c->stream) != hipSuccess) return DGS_EHIP;
    return DGS_OK;
}

}  // namespace

int dgs_encode(dgs_ctx *c, double density, const uint32_t *idx, const float *val, void *wire)
{
    if (!c || !idx || !val || !wire || !(density > 0.0) || density > 1.0) return DGS_EINVAL;
    if (!aligned4(idx) || !aligned4(val) || !aligned4(wire)) return DGS_EINVAL;
    uint32_t slot;
    uint64_t K;
    const int rc = get_plan(c, density, &slot, &K);
    if (rc != DGS_OK) return rc;
    const uint64_t words = c->plan_slot[slot].wire_words;
    if (K + words >= (1ull << 32)) return DGS_EINVAL;      // (the value area is at most K words)
    if (c->validate) launch_fill_u32(c->flag, 0u, 1, c->stream);
    ProfSlot ps(c, DGS_PROF_ENCODE);
    launch_wire_pack(c->tdesc, c->plans + (size_t)slot * c->J, c->J, (uint32_t)K, (uint32_t)words,
                     c->wire_value_bits, idx, val, (uint32_t *)wire, c->validate ? c->flag : nullptr, c->stream, ps.ev0, ps.ev1);
    ps.launched();
    if (hipGetLastError() != hipSuccess) return DGS_EHIP;
    if (c->validate) {
        uint32_t bad = 0;
        const int rf = read_flag(c, &bad);
        if (rf != DGS_OK) return rf;
        if (bad) return DGS_EINVAL;
    }
    return DGS_OK;
}

int dgs_decode(dgs_ctx *c, double density, const void *wire, uint32_t *idx_out, float *val_out)
{
    if (!c || !idx_out || !val_out || !wire || !(density > 0.0) || density > 1.0) return DGS_EINVAL;
    if (!aligned4(idx_out) || !aligned4(val_out) || !aligned4(wire)) return DGS_EINVAL;
    uint32_t slot;
    uint64_t K;
    const int rc = get_plan(c, density, &slot, &K);
    if (rc != DGS_OK) return rc;
    if (c->validate) launch_fill_u32(c->flag, 0u, 1, c->stream);
    ProfSlot ps(c, DGS_PROF_DECODE);
    launch_wire_unpack(c->tdesc, c->plans + (size_t)slot * c->J, c->J, (uint32_t)K, c->wire_value_bits,
                       (const uint32_t *)wire, idx_out, val_out, c->validate ? c->flag : nullptr, c->stream, ps.ev0, ps.ev1);
    ps.launched();
    if (hipGetLastError() != hipSuccess) return DGS_EHIP;
    if (c->validate) {
        uint32_t bad = 0;
        const int rf = read_flag(c, &bad);
        if (rf != DGS_OK) return rf;
        if (bad) return DGS_EINVAL;
    }
    return DGS_OK;
}

int dgs_set_option(dgs_ctx *c, int option, int64_t value)
{
    if (!c) return DGS_EINVAL;
    switch (option) {
    case DGS_OPT_FORCE_EXACT:
        if (value < 0 || value > 2) return DGS_EINVAL;
        c->force_exact = value == 1;
        c->force_sample = value == 2;
        return DGS_OK;
    case DGS_OPT_PROFILE: c->profile = value != 0; return DGS_OK;
    case DGS_OPT_VALIDATE: c->validate = value != 0; return DGS_OK;
    case DGS_OPT_MARGIN_PCT:
        if (value < 0 || value > 1000) return DGS_EINVAL;
        c->margin_pct = (int)value;
        return DGS_OK;
    case DGS_OPT_SEGMENTED:
        if (value < 0 || value > 2) return DGS_EINVAL;
        c->seg_mode = (int)value;
        return DGS_OK;
    case DGS_OPT_REPAIR_ROUND: c->repair_round = value != 0; return DGS_OK;
    case DGS_OPT_WIRE_VALUE_BITS:
        if (value != 32 && value != 16) return DGS_EINVAL;
        c->wire_value_bits = (uint32_t)value;
        return DGS_OK;
    case DGS_OPT_SPIN_LIMIT:
        if (value < 1 || value > (1ll << 30)) return DGS_EINVAL;
        c->spin_limit = (uint32_t)value;
        return DGS_OK;
    case DGS_OPT_STREAM_QUADS:
        if (value < 0 || value > (1 << 20)) return DGS_EINVAL;
        c->stream_quads = (uint32_t)value;
        return DGS_OK;
    default: return DGS_EINVAL;
    }
}

int dgs_get_stats(dgs_ctx *c, dgs_stats *out)
{
    if (!c || !out) return DGS_EINVAL;
    DevStats d;
    if (hipMemcpyAsync(&d, c->stats, sizeof d, hipMemcpyDeviceToHost, c->stream) != hipSuccess) return DGS_EHIP;
    if (hipStreamSynchronize(c->stream) != hipSuccess) return DGS_EHIP;
    out->calls_worker = c->calls_worker;
    out->calls_pull = c->calls_pull;
    out->calls_push = c->calls_push;
    out->exact_calls = c->exact_calls;
    out->fallback_tensors = d.fallback_tensors;
    out->fallback_elems = d.fallback_elems;
    out->candidates = d.candidates;
    out->internal_errors = d.internal_errors;
    out->segmented_tensors = d.segmented_tensors;
    out->repaired_tensors = d.repaired_tensors;
    return DGS_OK;
}

int dgs_profile_read(dgs_ctx *c, int kind, uint64_t *launches, double *total_ms)
{
    if (!c || kind < 0 || kind >= DGS_PROF_KINDS || !launches || !total_ms) return DGS_EINVAL;
    if (hipStreamSynchronize(c->stream) != hipSuccess) return DGS_EHIP;
    ProfClass &p = c->prof[kind];
    double sum = 0.0;
    for (uint32_t i = 0; i < p.used; ++i) {
        float ms = 0.0f;
        if (hipEventElapsedTime(&ms, p.start[i], p.stop[i]) != hipSuccess) return DGS_EHIP;
        sum += ms;
    }
    *launches = p.used;
    *total_ms = sum;
    p.used = 0;
    return DGS_OK;
}

const char *dgs_strerror(int code)
{
    switch (code) {
    case DGS_OK: return "ok";
    case DGS_EINVAL: return "invalid argument";
    case DGS_ENOMEM: return "workspace too small or host allocation failed";
    case DGS_ENOTSUP: return "not supported";
    case DGS_ECAPACITY: return "output capacity exceeded";
    case DGS_EHIP: return "HIP runtime error";
    default: return "unknown error";
    }
}

}  // extern "C"
