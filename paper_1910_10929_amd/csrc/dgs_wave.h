// Wavefront and workgroup helpers shared by the gfx950 (CDNA4, wave64) kernels of libdgs:
// lane primitives, DPP scans, workgroup scans, rank search in an LDS histogram, and the
// kernel launch wrapper that can stamp a dispatch into HIP events.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include "dgs_device.h"

namespace dgs {

typedef float f32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ uint32_t lane_id() { return threadIdx.x & 63u; }

__device__ __forceinline__ uint32_t mbcnt64(uint64_t mask)
{
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32),
                                     __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
}

__device__ __forceinline__ uint64_t ballot64(bool p) { return __builtin_amdgcn_ballot_w64(p); }

__device__ __forceinline__ uint32_t uniform(uint32_t v) { return __builtin_amdgcn_readfirstlane(v); }

// Isolated 4-byte store into a large buffer that a later streaming pass will sweep
// (state fix-ups, pull zero-writes, the push scatter).  Non-temporal: plain stores
// leave partially written lines behind in the cache hierarchy, and 1e5 of them were
// measured to slow the NEXT streaming pass over a 4 GB buffer by 130 us (6 %);
// non-temporal ones by 15 us.
__device__ __forceinline__ void store_scattered(float *p, float v) { __builtin_nontemporal_store(v, p); }

// ---------------------------------------------------------------------------
// hand-over between workgroups of one launch
// ---------------------------------------------------------------------------
// The L2 caches of the chip's eight dies (XCDs) are not coherent with each other, and a
// device-wide release fence writes back a die's whole L2 (measured: a streaming pass whose
// workgroups each fence runs 15 x longer).  So what one workgroup hands to another inside a
// launch goes through memory explicitly: written with device-scope stores (write-through),
// read with device-scope loads (never a stale line of the reader's L2), and the writer waits
// for its stores to be acknowledged before it signals through a device-scope atomic.
__device__ __forceinline__ void st_dev(uint32_t *p, uint32_t v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_dev(uint2 *p, uint2 v)
{
    __hip_atomic_store((unsigned long long *)p, ((unsigned long long)v.y << 32) | v.x, __ATOMIC_RELAXED,
                       __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ uint32_t ld_dev(const uint32_t *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ uint2 ld_dev(const uint2 *p)
{
    const unsigned long long x =
        __hip_atomic_load((const unsigned long long *)p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return make_uint2((uint32_t)x, (uint32_t)(x >> 32));
}
// 16-byte device-scope (write-through) store at base + byte_off; `base` must be wave-uniform
// and the 16 bytes must lie within 1 MB of it.
#ifdef DGS_HOST_EMULATION
__device__ __forceinline__ void store_through16(float *base, uint32_t byte_off, f32x4 v)
{
    *(f32x4 *)((char *)base + byte_off) = v;
}
#else
typedef unsigned u32x4_store __attribute__((__vector_size__(16)));
__device__ __forceinline__ void store_through16(float *base, uint32_t byte_off, f32x4 v)
{
    const __amdgpu_buffer_rsrc_t r = __builtin_amdgcn_make_buffer_rsrc(base, 0, 1 << 20, 0x00020000);
    u32x4_store u;
    __builtin_memcpy(&u, &v, 16);
    __builtin_amdgcn_raw_buffer_store_b128(u, r, (int)byte_off, 0, 16);   // aux 16: sc1 = device scope
}
#endif

// All vector memory operations of this wavefront (stores and atomics included) are complete.
#ifdef DGS_HOST_EMULATION   // CPU build of the kernels for sanitizer runs: no such instruction, nothing to wait for
__device__ __forceinline__ void wait_mem() {}
#else
__device__ __forceinline__ void wait_mem() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }
#endif

// Everything this compute-unit group's L2 holds dirty goes to memory (device-scope release).
// Expensive -- the whole L2 is walked -- and therefore only used where a prediction has failed.
#ifdef DGS_HOST_EMULATION
__device__ __forceinline__ void release_dev() {}
#else
__device__ __forceinline__ void release_dev() { __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent"); }
#endif

// The workgroup has finished its share of a per-tensor phase: after every wavefront's stores
// are acknowledged, one device-scope atomic counts it in.  Returns true in every thread of the
// workgroup that arrives last of `expected` (it then also clears the counter for the next
// launch).  `bc` is one word of LDS.  Contains two barriers.
__device__ __forceinline__ bool arrive_last(uint32_t *counter, uint32_t expected, uint32_t *bc)
{
    wait_mem();
    __syncthreads();
    if (threadIdx.x == 0) {
        const uint32_t old = __hip_atomic_fetch_add(counter, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const bool last = (old + 1u == expected);
        if (last) st_dev(counter, 0u);
        *bc = last ? 1u : 0u;
    }
    __syncthreads();
    return *bc != 0;
}

// Thread 0 polls a word another workgroup of this launch will set (device-scope loads, sleeping
// in between); the value is handed to the whole workgroup through `bc`.  Bounded: after
// `limit` polls it gives up and returns 0.  Only ever waits for workgroups with a lower block
// index, which the hardware has dispatched before this one.  Contains two barriers.
__device__ __forceinline__ uint32_t wait_word(const uint32_t *p, uint32_t limit, uint32_t *bc)
{
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t v = 0;
        for (uint32_t spin = 0; spin < limit; ++spin) {
            v = ld_dev(p);
            if (v != 0) break;
            __builtin_amdgcn_s_sleep(4);
        }
        *bc = v;
    }
    __syncthreads();
    return *bc;
}

// `count` readers of a hand-over word have passed; whoever completes the `readers` clears the
// word and the count for the next launch.  Call from one thread.
__device__ __forceinline__ void reader_done(uint32_t *seen, uint32_t readers, uint32_t count, uint32_t *word)
{
    const uint32_t old = __hip_atomic_fetch_add(seen, count, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (old + count == readers) {
        st_dev(word, 0u);
        st_dev(seen, 0u);
    }
}

// Plain launch, or a launch whose begin and / or end is stamped into an event.
template <class K, class... Args>
static void launch_k(K kernel, dim3 grid, dim3 block, hipStream_t st, void *ev0, void *ev1, Args... args)
{
    if (ev0 || ev1)
        hipExtLaunchKernelGGL(kernel, grid, block, 0, st, (hipEvent_t)ev0, (hipEvent_t)ev1, 0, args...);
    else
        hipLaunchKernelGGL(kernel, grid, block, 0, st, args...);
}

// ---------------------------------------------------------------------------
// workgroup helpers for pick / select
// ---------------------------------------------------------------------------

// Inclusive prefix sum over the 64 lanes of a wavefront, in registers (DPP):
// four shifts inside each row of 16 lanes, then two row broadcasts.
__device__ __forceinline__ uint32_t wave_incl_scan(uint32_t v)
{
    int x = (int)v;
    x += __builtin_amdgcn_update_dpp(0, x, 0x111, 0xf, 0xf, false);   // row_shr:1
    x += __builtin_amdgcn_update_dpp(0, x, 0x112, 0xf, 0xf, false);   // row_shr:2
    x += __builtin_amdgcn_update_dpp(0, x, 0x114, 0xf, 0xf, false);   // row_shr:4
    x += __builtin_amdgcn_update_dpp(0, x, 0x118, 0xf, 0xf, false);   // row_shr:8
    x += __builtin_amdgcn_update_dpp(0, x, 0x142, 0xa, 0xf, false);   // row_bcast:15 into rows 1, 3
    x += __builtin_amdgcn_update_dpp(0, x, 0x143, 0xc, 0xf, false);   // row_bcast:31 into rows 2, 3
    return (uint32_t)x;
}

__device__ __forceinline__ uint32_t wave_sum(uint32_t v)
{
    return (uint32_t)__builtin_amdgcn_readlane((int)wave_incl_scan(v), 63);
}

// Exclusive scan over the workgroup in thread order; `total` is the workgroup sum.
// wsum: LDS scratch of NW words.  Contains two barriers.
template <int NW>
__device__ __forceinline__ uint32_t block_excl_scan(uint32_t v, uint32_t *wsum, uint32_t &total)
{
    const uint32_t wave = threadIdx.x >> 6;
    const uint32_t incl = wave_incl_scan(v);
    __syncthreads();
    if (lane_id() == 63) wsum[wave] = incl;
    __syncthreads();
    uint32_t before = 0, tot = 0;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
        const uint32_t x = wsum[w];
        if ((uint32_t)w < wave) before += x;
        tot += x;
    }
    total = tot;
    return before + incl - v;
}

// Workgroup sum.  wsum: LDS scratch of nw words.  Contains two barriers.
__device__ __forceinline__ uint32_t block_sum(uint32_t v, uint32_t *wsum, int nw)
{
    const uint32_t s = wave_sum(v);
    __syncthreads();
    if (lane_id() == 0) wsum[threadIdx.x >> 6] = s;
    __syncthreads();
    uint32_t tot = 0;
    for (int w = 0; w < nw; ++w) tot += wsum[w];
    return tot;
}

// In an LDS histogram h[NB] (NB a multiple of 64, at most 4096), find for each of
// three ranks R[0..2] (counted from the top bin, >= 1) the bin holding it and the
// rank inside that bin:  res[2 i] = bin, res[2 i + 1] = rank in the bin; bin -1 if the
// rank exceeds the histogram total (or is 0).  Every wavefront sums rows of 64 bins,
// then up to three wavefronts each scan the row sums and the row their rank lands in.
// Barriers: one on entry (h complete), one in the middle, one on exit.
template <int NB, int NW>
__device__ __forceinline__ void find_ranks(const uint32_t *h, uint32_t R0, uint32_t R1, uint32_t R2,
                                           uint32_t *rowsum, int *res)
{
    constexpr int ROWS = NB / 64;
    constexpr int SEARCHERS = NW < 3 ? NW : 3;
    static_assert(ROWS * 64 == NB && ROWS <= 64, "histogram shape");
    const uint32_t lane = lane_id();
    const uint32_t wave = threadIdx.x >> 6;
    __syncthreads();
    for (int r = (int)wave; r < ROWS; r += NW) {
        const uint32_t s = wave_sum(h[r * 64 + lane]);
        if (lane == 0) rowsum[r] = s;
    }
    __syncthreads();
    if (wave < (uint32_t)SEARCHERS) {
        // lane l looks at row ROWS-1-l: the top row first
        const uint32_t rs = (lane < (uint32_t)ROWS) ? rowsum[ROWS - 1 - lane] : 0u;
        const uint32_t rincl = wave_incl_scan(rs);
        for (int which = (int)wave; which < 3; which += SEARCHERS) {
            const uint32_t R = which == 0 ? R0 : (which == 1 ? R1 : R2);
            int bin = -1;
            uint32_t rin = 0;
            const uint64_t hit = ballot64(lane < (uint32_t)ROWS && rincl >= R);
            if (hit != 0 && R != 0) {
                const int rl = __ffsll((unsigned long long)hit) - 1;          // first row reaching R
                const uint32_t above = (uint32_t)__builtin_amdgcn_readlane((int)(rincl - rs), rl);
                const int row = ROWS - 1 - rl;
                const uint32_t Rr = R - above;                                 // rank inside the row
                const uint32_t v = h[row * 64 + (63 - lane)];                  // top bin first
                const uint32_t vincl = wave_incl_scan(v);
                const uint64_t hit2 = ballot64(vincl >= Rr);
                const int bl = __ffsll((unsigned long long)hit2) - 1;
                const uint32_t above2 = (uint32_t)__builtin_amdgcn_readlane((int)(vincl - v), bl);
                bin = row * 64 + 63 - bl;
                rin = Rr - above2;
            }
            if (lane == 0) {
                res[2 * which] = bin;
                res[2 * which + 1] = (int)rin;
            }
        }
    }
    __syncthreads();
}

}  // namespace dgs
