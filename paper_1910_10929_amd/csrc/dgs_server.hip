// Server-side scatter (Algorithm 2, "M <- M - decode(g)"), worker apply, index validation,
// the wire form of a message, and the pull without secondary compression.
#include "dgs_wave.h"

namespace dgs {

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

// An index outside [0, n) is skipped, as in k_push: a corrupted message must not write
// outside the destination.
__global__ __launch_bounds__(256) void k_apply(float *dst, uint32_t n, const uint32_t *idx, const float *val,
                                               uint32_t nnz, float sign)
{
    const uint32_t e = blockIdx.x * 256 + threadIdx.x;
    if (e >= nnz) return;
    const uint32_t i = idx[e];
    if (i < n) dst[i] = __builtin_fmaf(sign, val[e], dst[i]);
}

void launch_apply(float *dst, uint32_t n, const uint32_t *idx, const float *val, uint32_t nnz, float sign,
                  void *stream)
{
    if (nnz == 0) return;
    hipLaunchKernelGGL(k_apply, dim3((nnz + 255) / 256), dim3(256), 0, (hipStream_t)stream, dst, n, idx,
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

// binary32 -> bfloat16 (its upper half), to nearest, halfway cases to the even one; beyond the
// largest finite bfloat16 the carry runs into the exponent and gives infinity; NaN stays NaN.
__device__ __forceinline__ uint32_t to_bf16(float x)
{
    const uint32_t b = __float_as_uint(x);
    if ((b << 1) > 0xFF000000u) return (b >> 16) | 0x40u;
    return (b + 0x7FFFu + ((b >> 16) & 1u)) >> 16;
}

// Words of the value area: one per fp32 value, or one per two bfloat16 values.
__host__ __device__ __forceinline__ uint32_t wire_value_words(uint32_t K, uint32_t value_bits)
{
    return value_bits == 16u ? (K + 1u) / 2u : K;
}

// One thread per word of the value area (a copied fp32 value, or two values rounded to bfloat16)
// and per 32-bit word of the index area: the word gathers the pieces of the entries that overlap
// it (entry e of tensor j covers bits [e b_j, (e + 1) b_j) of the tensor's block).  Out-of-tensor
// indices are masked to b_j bits and, with `flag`, reported.
__global__ __launch_bounds__(256) void k_wire_pack(const TensorDesc *tdesc, const PlanEntry *plan, uint32_t J,
                                                   uint32_t K, uint32_t words, uint32_t value_bits,
                                                   const uint32_t *idx, const float *val, uint32_t *wire,
                                                   uint32_t *flag)
{
    const uint64_t t = (uint64_t)blockIdx.x * 256 + threadIdx.x;
    const uint32_t vw = wire_value_words(K, value_bits);
    if (t < vw) {
        if (value_bits == 16u) {
            const uint32_t e = 2u * (uint32_t)t;
            wire[t] = to_bf16(val[e]) | ((e + 1u < K) ? (to_bf16(val[e + 1u]) << 16) : 0u);
        } else {
            wire[t] = __float_as_uint(val[t]);
        }
        return;
    }
    if (t >= (uint64_t)vw + words) return;
    const uint32_t w = (uint32_t)(t - vw);
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

// One thread per entry: value copied (a bfloat16 widened), local index cut out of one or two
// words of its block.
__global__ __launch_bounds__(256) void k_wire_unpack(const TensorDesc *tdesc, const PlanEntry *plan, uint32_t J,
                                                     uint32_t K, uint32_t value_bits, const uint32_t *wire,
                                                     uint32_t *idx, float *val, uint32_t *flag)
{
    const uint64_t t = (uint64_t)blockIdx.x * 256 + threadIdx.x;
    if (t >= K) return;
    if (value_bits == 16u) {
        const uint32_t w2 = wire[t >> 1];
        val[t] = __uint_as_float((t & 1u) ? (w2 & 0xFFFF0000u) : (w2 << 16));
    } else {
        val[t] = __uint_as_float(wire[t]);
    }
    const uint32_t j = plan_search<&PlanEntry::outoff>(plan, J, (uint32_t)t);
    const PlanEntry pe = plan[j];
    const TensorDesc td = tdesc[j];
    const uint32_t b = pe.wire_bits;
    const uint64_t pos = (uint64_t)((uint32_t)t - pe.outoff) * b;
    const uint32_t *block = wire + wire_value_words(K, value_bits) + pe.wire_off;
    const uint32_t w = (uint32_t)(pos >> 5), sh = (uint32_t)(pos & 31u);
    uint64_t x = block[w];
    if (sh + b > 32u) x |= (uint64_t)block[w + 1] << 32;              // an entry that crosses ends inside the block
    const uint32_t mask = (b >= 32u) ? 0xFFFFFFFFu : ((1u << b) - 1u);
    const uint32_t local = (uint32_t)(x >> sh) & mask;
    idx[t] = td.off + local;
    if (local >= td.n && flag) atomicOr(flag, 1u);
}

void launch_wire_pack(const TensorDesc *tdesc, const PlanEntry *plan, uint32_t J, uint32_t K, uint32_t words,
                      uint32_t value_bits, const uint32_t *idx, const float *val, uint32_t *wire, uint32_t *flag,
                      void *stream, void *ev0, void *ev1)
{
    const uint64_t threads = (uint64_t)wire_value_words(K, value_bits) + words;
    if (threads == 0) return;
    launch_k(k_wire_pack, dim3((uint32_t)((threads + 255) / 256)), dim3(256), (hipStream_t)stream, ev0, ev1,
             tdesc, plan, J, K, words, value_bits, idx, val, wire, flag);
}

void launch_wire_unpack(const TensorDesc *tdesc, const PlanEntry *plan, uint32_t J, uint32_t K,
                        uint32_t value_bits, const uint32_t *wire, uint32_t *idx, float *val, uint32_t *flag,
                        void *stream, void *ev0, void *ev1)
{
    if (K == 0) return;
    launch_k(k_wire_unpack, dim3((K + 255) / 256), dim3(256), (hipStream_t)stream, ev0, ev1, tdesc, plan, J, K,
             value_bits, wire, idx, val, flag);
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

// A small host table carried to the device inside kernel arguments (no copy engine, no
// staging buffer): PUT_WORDS 32-bit words per launch.
constexpr uint32_t PUT_WORDS = 768;
struct PutChunk { uint32_t w[PUT_WORDS]; };

__global__ __launch_bounds__(256) void k_put_words(uint32_t *dst, const PutChunk c, uint32_t count)
{
    for (uint32_t i = threadIdx.x; i < count; i += 256) dst[i] = c.w[i];
}

void launch_put_words(uint32_t *dst, const uint32_t *src_host, size_t words, void *stream)
{
    for (size_t o = 0; o < words; o += PUT_WORDS) {
        PutChunk c;
        const uint32_t cnt = (uint32_t)((words - o < PUT_WORDS) ? (words - o) : PUT_WORDS);
        for (uint32_t i = 0; i < cnt; ++i) c.w[i] = src_host[o + i];
        for (uint32_t i = cnt; i < PUT_WORDS; ++i) c.w[i] = 0;
        hipLaunchKernelGGL(k_put_words, dim3(1), dim3(256), 0, (hipStream_t)stream, dst + o, c, cnt);
    }
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
