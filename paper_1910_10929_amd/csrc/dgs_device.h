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
constexpr uint32_t SEL_LDS_LIST = 8192;            // candidates kept in LDS (64 KB)
// Above this density candidates stop paying off; such requests select densely.
constexpr double DENSE_DENSITY = 1.0 / 32.0;

struct TensorDesc {
    uint32_t off;   // first element
    uint32_t n;     // elements
    uint32_t big;   // n > SMALL_N
    uint32_t pad;
};

struct PlanEntry {
    uint32_t k;       // ceil(density * n_j)
    uint32_t k2;      // rank whose key becomes the next predicted threshold (>= k, <= n_j)
    uint32_t outoff;  // sum of k over earlier tensors
    uint32_t k2_pull; // same for a pull, whose sent entries vanish: about 2k (<= n_j)
};

struct DevStats {
    unsigned long long fallback_tensors;
    unsigned long long fallback_elems;
    unsigned long long candidates;
    unsigned long long internal_errors;
};

enum StreamOp { OP_FMA = 0, OP_IDENT = 1 };
enum StreamMode { MODE_PLAIN = 0, MODE_COLLECT = 1, MODE_HIST = 2 };
enum SelectOp { SEL_WORKER = 0, SEL_PULL = 1 };

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
    float lr;
};

struct SelectArgs {
    float *state;                 // worker state or difference row
    const TensorDesc *tdesc;
    const PlanEntry *plan;
    uint32_t *tau;                // hints of this stream, updated
    const uint32_t *tile_cnt;
    const uint2 *heads;
    const uint2 *slots;
    uint2 *ord;                   // ordered candidates of tensor j start at CAPT * (first tile + j)
    uint32_t *hint2;              // per tensor: candidates expected at the hinted threshold (0 = unknown)
    uint32_t *out_idx;
    float *out_val;
    DevStats *stats;
    float m;                      // SEL_WORKER: sent entries keep m * a
    uint32_t force_dense;         // select every tensor straight from `state`
    uint32_t write_hint;
    uint32_t exact_mode;          // the threshold came from this step's histogram
};

// Host-callable launchers (defined next to the kernels).
// ev0 / ev1: optional hipEvent_t recorded at the begin / end of the kernel (both or neither).
void launch_stream(int op, int mode, bool vec, const StreamArgs &a, uint32_t blocks, void *stream,
                   void *ev0, void *ev1);
void launch_pick(const TensorDesc *tdesc, const PlanEntry *plan, uint32_t *ghist, uint32_t *tau,
                 DevStats *stats, uint32_t J, void *stream);
void launch_select(int op, const SelectArgs &a, uint32_t J, void *stream, void *ev0, void *ev1);
void launch_push(float *model, float *diff, uint32_t W, uint32_t n, const uint32_t *idx,
                 const float *val, uint32_t nnz, void *stream, void *ev0, void *ev1);
void launch_validate_idx(const uint32_t *idx, uint32_t nnz, uint32_t n, uint32_t *flag, void *stream);
void launch_apply(float *dst, const uint32_t *idx, const float *val, uint32_t nnz, float sign,
                  void *stream);
void launch_fill_u32(uint32_t *p, uint32_t v, size_t count, void *stream);
void launch_pull_all_count(const float *row, uint32_t n, uint32_t ntiles, uint32_t *tile_cnt, void *stream);
void launch_pull_all_scan(uint32_t *tile_cnt, uint32_t ntiles, uint32_t *total, void *stream);
void launch_pull_all_emit(float *row, uint32_t n, uint32_t ntiles, const uint32_t *tile_pos,
                          uint32_t *out_idx, float *out_val, void *stream);

}  // namespace dgs
