// Streaming pass of libdgs: one wavefront per 1024-element tile, 16-byte loads, fused
// accumulate + magnitude key + candidate collection or key histogram.
#include "dgs_tile.h"

namespace dgs {

template <int OP, int MODE, bool VEC>
__global__ __launch_bounds__(STREAM_THREADS) void k_stream(const StreamArgs A,
                                                           const uint32_t *__restrict__ toff,
                                                           const uint32_t *__restrict__ tau)
{
    constexpr bool HISTO = (MODE == MODE_HIST || MODE == MODE_SAMPLE);
    __shared__ uint32_t lhist[HISTO ? HBINS : 1];
    __shared__ uint2 stage_all[MODE == MODE_COLLECT ? WAVES_PER_BLOCK * STAGE : 1];
    const uint32_t wave = uniform(threadIdx.x >> 6);
    uint2 *stage = stage_all + (MODE == MODE_COLLECT ? wave * STAGE : 0u);
    const uint32_t q0 = blockIdx.x * A.quads_per_block;
    const uint32_t q1 = min(q0 + A.quads_per_block, A.nquads);
    int cur = -1;
    if (HISTO) {
        for (uint32_t b = threadIdx.x; b < HBINS; b += STREAM_THREADS) lhist[b] = 0;
        __syncthreads();
    }
    for (uint32_t q = q0; q < q1; ++q) {
        // (a sampling pass takes its tiles from a list, four at a time: "quad" q = entries 4 q ..)
        const uint32_t t = (MODE == MODE_SAMPLE)
                               ? ((q * WAVES_PER_BLOCK + wave < A.nlist) ? A.tile_list[q * WAVES_PER_BLOCK + wave] : 0xFFFFFFFFu)
                               : q * WAVES_PER_BLOCK + wave;
        if (HISTO) {
            // the LDS histogram belongs to the big tensor the quad starts in
            const uint32_t qfirst = ((MODE == MODE_SAMPLE) ? A.tile_list[q * WAVES_PER_BLOCK] : q * WAVES_PER_BLOCK) * TILE;
            const uint32_t fx = span_desc(toff, A.J, qfirst, qfirst).x;
            const int qt = (fx >> 31) ? (int)(fx & 0x7FFFFFFFu) : -1;
            if (qt != cur) {
                flush_hist<MODE>(lhist, A.ghist, cur);
                cur = qt;
            }
        }
        if (t < A.ntiles) process_tile<OP, MODE, VEC>(A, toff, tau, t, lhist, cur, stage);
    }
    flush_hist<MODE>(lhist, A.ghist, cur);
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
        else if (mode == MODE_SAMPLE) launch_stream_t<OP_FMA, MODE_SAMPLE>(vec, a, blocks, st, ev0, ev1);
        else launch_stream_t<OP_FMA, MODE_HIST>(vec, a, blocks, st, ev0, ev1);
    } else if (op == OP_SUB) {
        if (mode == MODE_COLLECT) launch_stream_t<OP_SUB, MODE_COLLECT>(vec, a, blocks, st, ev0, ev1);
        else if (mode == MODE_HIST) launch_stream_t<OP_SUB, MODE_HIST>(vec, a, blocks, st, ev0, ev1);
        else if (mode == MODE_SAMPLE) launch_stream_t<OP_SUB, MODE_SAMPLE>(vec, a, blocks, st, ev0, ev1);
    } else {
        if (mode == MODE_COLLECT) launch_stream_t<OP_IDENT, MODE_COLLECT>(vec, a, blocks, st, ev0, ev1);
        else if (mode == MODE_HIST) launch_stream_t<OP_IDENT, MODE_HIST>(vec, a, blocks, st, ev0, ev1);
        else if (mode == MODE_SAMPLE) launch_stream_t<OP_IDENT, MODE_SAMPLE>(vec, a, blocks, st, ev0, ev1);
    }
}

}  // namespace dgs
