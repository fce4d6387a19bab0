// Definitions shared by the host-side plan and the gfx950 kernels of libdgs.
#pragma once
#include <stdint.h>
#include <stddef.h>

namespace dgs {

// A tile is the unit one wavefront streams: 1024 consecutive elements of the
// flat buffer, tile t = [1024 t, 1024 t + 1024), regardless of tensor borders.
constexpr uint32_t TILE = 1024;
// Candidate slots reserved per tile.  A tile that would need more marks itself
// overflowed and its tensors are re-selected densely.
constexpr uint32_t CAPT = 256;
// The first HEAD candidates of every tile live in one 64-byte line of a dense
// array (tile t at heads[HEAD * t]), so that the selection kernel fetches a
// tensor's candidates with contiguous loads; candidate p >= HEAD of a crowded
// tile goes to slots[CAPT * t + p].
constexpr uint32_t HEAD = 8;
// Candidates of a tile that the streaming wavefront stages in LDS and writes out as
// whole 64-byte lines (later ones are stored one by one).
constexpr uint32_t STAGE = 64;
constexpr uint32_t WAVES_PER_BLOCK = 4;            // one "quad" = 4 tiles = 4096 elements
constexpr uint32_t STREAM_THREADS = 64 * WAVES_PER_BLOCK;
// Tensors up to this size are selected directly from the state buffer by one
// workgroup; larger ones ("big") go through candidate collection.
constexpr uint32_t SMALL_N = 8192;
// Threshold value that no 31-bit magnitude key reaches.
constexpr uint32_t TAU_NEVER = 0x80000000u;
constexpr uint32_t CNT_OVERFLOW = 0xFFFFFFFFu;
// Histogram of the streaming pass: key bits [30:19] (exponent + 4 mantissa bits).
constexpr uint32_t HBITS = 12;
constexpr uint32_t HBINS = 1u << HBITS;
constexpr uint32_t HSHIFT = 31 - HBITS;
// Selection workgroup.
constexpr uint32_t SEL_THREADS = 1024;
constexpr uint32_t SEL_WAVES = SEL_THREADS / 64;
constexpr uint32_t SEL_LDS_LIST = 16384;           // candidates kept in LDS (128 KB); longer lists continue in global scratch
constexpr uint32_t SEL_LIST_MAX = 24576;           // longest candidate list one workgroup is planned for
constexpr uint32_t SEL_LIST_HARD = 65536;          // longest it accepts when a tail has grown beyond the plan
// Above this density candidates stop paying off; such requests select densely.
constexpr double DENSE_DENSITY = 1.0 / 32.0;

// Parts.  Every tensor is cut into parts of up to SEG_TILES tiles, one workgroup each: a part
// joins its tiles' candidates into one ordered list, and the workgroup that arrives last for a
// tensor selects from the parts' lists.  Tensors whose candidate lists outgrow one workgroup
// (or whose request is dense) continue through the chain kernels, one workgroup per part.
#ifndef DGS_SEG_TILES          // (a CPU test build shrinks the parts so that small layouts have several)
#define DGS_SEG_TILES 256
#endif
constexpr uint32_t SEG_TILES = DGS_SEG_TILES;
// Join groups.  The candidates of consecutive parts of a tensor, up to about GROUP_TILES tiles,
// are joined by one workgroup: a tensor of one group is selected by that workgroup straight
// from LDS with no hand-over, larger tensors hand their groups' lists to the last to arrive.
#ifndef DGS_GROUP_TILES
#define DGS_GROUP_TILES 4096
#endif
constexpr uint32_t GROUP_TILES = DGS_GROUP_TILES;
constexpr uint32_t SEG_THREADS = 256;
constexpr uint32_t SEG_MIN_N = 65536;              // smaller tensors never take the chain
constexpr uint32_t SEG_AUTO_N = 1u << 22;          // (kept for the plan: tensors this large always may)
constexpr uint32_t SEG_LOWBITS = 12;               // key bits resolved by the second level
constexpr uint32_t SEG_WBINS = 2048;               // window of key >> SEG_LOWBITS above the threshold
constexpr uint32_t SEG_LBINS = 1u << SEG_LOWBITS;
constexpr uint32_t PFX_CAP = 8192;                 // candidates sharing the k-th key's prefix, per tensor
constexpr uint32_t SEG_MAX_PER_TENSOR = 512;       // parts per tensor whose list positions fit the selection's LDS
// Status of a tensor inside one selection call.
//   SEG_IDLE      nothing decided yet
//   SEG_DONE      selected and emitted
//   SEG_ACTIVE    the chain kernels finish it (prefix of the k-th key known)
//   SEG_ALL       k_j = n_j: the chain's emission sends every element
//   SEG_PENDING   the prediction failed: the parts collect again with a fresh threshold
//   SEG_FALLBACK  left to the dense single-workgroup selection
enum SegStatus { SEG_IDLE = 0, SEG_DONE = 1, SEG_FALLBACK = 2, SEG_PENDING = 4, SEG_ALL = 6, SEG_ACTIVE = 8 };
enum SegMode { SEG_MODE_AUTO = 0, SEG_MODE_ALWAYS = 1, SEG_MODE_NEVER = 2 };

struct TensorDesc {
    uint32_t off;        // first element
    uint32_t n;          // elements
    uint32_t big;        // n > SMALL_N
    uint32_t seg_first;  // first entry of this tensor in the segment table
    uint32_t nseg;       // segments (0: the tensor never goes segmented)
    uint32_t pfx_slot;   // which PFX_CAP-sized block of the prefix list belongs to it
    uint32_t grp_first;  // first entry of this tensor in the group table
    uint32_t ngrp;       // its join groups (>= 1)
};

struct PlanEntry {
    uint32_t k;       // ceil(density * n_j)
    uint32_t k2;      // rank whose key becomes the next predicted threshold (>= k, <= n_j)
    uint32_t outoff;  // sum of k over earlier tensors
    uint32_t k2_pull; // same for a pull, whose sent entries vanish: about 2k (<= n_j)
    uint32_t seg;     // 1: segmented selection at this density
    uint32_t wire_off;   // wire form: first 32-bit word of the tensor's index block (after the values)
    uint32_t wire_bits;  // wire form: bits per local index = bit length of n_j - 1 (>= 1)
    uint32_t pad2;
};

struct SegDesc {
    uint32_t j;       // tensor
    uint32_t tile0;   // first tile (of the flat buffer) of the segment
    uint32_t ntiles;  // tiles in the segment (<= SEG_TILES)
    uint32_t sidx;    // index of the segment within its tensor
};

struct SegState {        // per tensor, rewritten by every selection
    uint32_t status;     // SegStatus
    uint32_t pfx;        // key >> SEG_LOWBITS of the k-th entry
    uint32_t r2;         // its rank among the entries sharing that prefix
    uint32_t T;          // the k-th key
    uint32_t pfxcount;   // entries appended to the prefix list
    uint32_t pad0, pad1, pad2;
    // Hand-over between the workgroups of one launch (all zero between launches):
    uint32_t arrive[4];  // parts that have finished: [0] join, [1] re-histogram, [2] re-collection, [3] chain prefix
    uint32_t verdict;    // 0 = not decided; else 0x100 | SegStatus, written by the last joining part
    uint32_t tau_ready;  // 1: the fresh threshold of a pending tensor is in place
    uint32_t seen[2];    // readers of verdict / tau_ready that have passed (the last one clears)
};

struct DevStats {
    unsigned long long fallback_tensors;
    unsigned long long fallback_elems;
    unsigned long long candidates;
    unsigned long long internal_errors;
    unsigned long long segmented_tensors;
    unsigned long long repaired_tensors;
};

// OP_FMA: a = fmaf(lr, grad, state), state <- a (worker);  OP_IDENT: a = state (pull on a
// difference row);  OP_SUB: a = grad - state, nothing stored (pull on model - sent_k).
enum StreamOp { OP_FMA = 0, OP_IDENT = 1, OP_SUB = 2 };
// MODE_SAMPLE: the histogram of a sample of the buffer (the tiles in tile_list, zero keys counted
// too so that a tensor's counters add up to its sampled elements), nothing stored.
enum StreamMode { MODE_PLAIN = 0, MODE_COLLECT = 1, MODE_HIST = 2, MODE_SAMPLE = 3 };
enum StoreMode { STORE_PLAIN = 0, STORE_WT = 1, STORE_NT = 2 };
// What happens to a sent entry: SEL_WORKER state <- m * val;  SEL_PULL state <- +0;
// SEL_PULL_V state <- state + val (the values themselves are model - state).
enum SelectOp { SEL_WORKER = 0, SEL_PULL = 1, SEL_PULL_V = 2 };

struct StreamArgs {
    const float *grad;            // OP_FMA only
    float *state;                 // OP_FMA: in/out.  OP_IDENT: read only.
    const uint32_t *toff;         // J + 1 tensor offsets (elements)
    const uint32_t *tau;          // per tensor: candidate threshold (TAU_NEVER for small tensors)
    uint32_t *tile_cnt;           // per tile: low 16 = candidates of the leading tensor part, high 16 = trailing part
    uint2 *heads;                 // per tile HEAD x (index, value bits): candidates 0 .. HEAD-1
    uint2 *slots;                 // per tile CAPT x (index, value bits): candidates HEAD .. CAPT-1
    uint32_t *ghist;              // per tensor HBINS counters
    uint32_t n, ntiles, nquads, quads_per_block, J;
    const uint32_t *tile_list;    // MODE_SAMPLE: the tiles to visit, nlist of them, four per "quad"
    uint32_t nlist;               //   (nquads = ceil(nlist / 4))
    float lr;
    uint32_t store_mode;          // OP_FMA: how the state is written back (StoreMode)
};

struct SelectArgs {
    float *state;                 // worker state, difference row, or sent_k row
    const float *model;           // SEL_PULL_V only: values are model - state
    const TensorDesc *tdesc;
    const PlanEntry *plan;
    const SegDesc *segtab;        // the parts, tensor after tensor
    const SegDesc *grptab;        // the join groups in launch order (tensors of several groups first)
    uint32_t *tau;                // hints of this stream, updated
    uint32_t *tile_cnt;
    uint2 *heads;
    uint2 *slots;
    uint2 *ord;                   // ordered candidates of a part start at CAPT * (tile0 + j)
    uint32_t *hint2;              // per tensor: candidates expected at the hinted threshold (0 = unknown)
    uint32_t *tprev;              // per tensor: k-th key of the previous selection on this stream (0 = unknown)
    uint32_t *ghist;              // per tensor HBINS counters, all zero between uses
    SegState *segstate;
    uint32_t *segcnt;             // per part: candidates (bit 31: a tile of the part overflowed)
    uint32_t *grpcnt;             // per join group: the same, for the lists joined by groups
    uint32_t *segstart;           // per part of a tensor that takes the chain: where its list starts in ord
    uint32_t *segG1;              // per part: candidates with a larger key prefix than the k-th
    uint2 *segOut;                // per part: (output position within the tensor, ties to take)
    uint4 *pfxlist;               // per tensor PFX_CAP x (index, value bits, part, 0)
    uint32_t *out_idx;
    float *out_val;
    DevStats *stats;
    const uint32_t *toff;         // J + 1 tensor offsets
    float m;                      // SEL_WORKER: sent entries keep m * a
    uint32_t n, ntiles, J, nparts;
    uint32_t ngroups, gparts;     // join groups; parts per group
    uint32_t dense;               // dense request: no candidate lists; tensors with parts take the chain
                                  // reading their own elements, the others select from the state buffer
    uint32_t write_hint;
    uint32_t exact_mode;          // the threshold came from this call's histogram
    uint32_t repair;              // the launch carries the re-collecting workgroups
    uint32_t spin_limit;          // polls before a waiting workgroup gives up
    uint32_t bgroup;              // parts looked after by one re-collecting workgroup
};

// Host-callable launchers (defined next to the kernels).
// ev0 / ev1: optional hipEvent_t recorded at the begin / end of the kernel (both or neither).
void launch_stream(int op, int mode, bool vec, const StreamArgs &a, uint32_t blocks, void *stream,
                   void *ev0, void *ev1);
void launch_pick(const TensorDesc *tdesc, const PlanEntry *plan, uint32_t *ghist, uint32_t *tau,
                 uint32_t *tprev, DevStats *stats, uint32_t J, bool sample, void *stream);
// The selection: one launch for every tensor (join, exact k-th key, ordered emission, state
// fix-up, next hint; failed predictions are collected again inside the same launch).
void launch_select(int op, const SelectArgs &a, void *stream, void *ev0, void *ev1);
// What remains for tensors left SEG_ACTIVE / SEG_ALL (very long candidate lists, dense requests).
void launch_chain(int op, const SelectArgs &a, void *stream, void *ev0, void *ev1);
void launch_push(float *model, float *diff, uint32_t W, uint32_t n, const uint32_t *idx,
                 const float *val, uint32_t nnz, void *stream, void *ev0, void *ev1);
void launch_validate_idx(const uint32_t *idx, uint32_t nnz, uint32_t n, uint32_t *flag, void *stream);
void launch_wire_pack(const TensorDesc *tdesc, const PlanEntry *plan, uint32_t J, uint32_t K, uint32_t words,
                      uint32_t value_bits, const uint32_t *idx, const float *val, uint32_t *wire, uint32_t *flag,
                      void *stream, void *ev0, void *ev1);
void launch_wire_unpack(const TensorDesc *tdesc, const PlanEntry *plan, uint32_t J, uint32_t K,
                        uint32_t value_bits, const uint32_t *wire, uint32_t *idx, float *val, uint32_t *flag,
                        void *stream, void *ev0, void *ev1);
void launch_apply(float *dst, uint32_t n, const uint32_t *idx, const float *val, uint32_t nnz, float sign,
                  void *stream);
void launch_fill_u32(uint32_t *p, uint32_t v, size_t count, void *stream);
// Host words -> device through kernel arguments (for the entry point that must not copy).
void launch_put_words(uint32_t *dst, const uint32_t *src_host, size_t words, void *stream);
void launch_pull_all_count(const float *row, const float *model, uint32_t n, uint32_t ntiles,
                           uint32_t *tile_cnt, void *stream);
void launch_pull_all_scan(uint32_t *tile_cnt, uint32_t ntiles, uint32_t *total, void *stream);
void launch_pull_all_emit(float *row, const float *model, uint32_t n, uint32_t ntiles,
                          const uint32_t *tile_pos, uint32_t *out_idx, float *out_val, void *stream);

}  // namespace dgs
