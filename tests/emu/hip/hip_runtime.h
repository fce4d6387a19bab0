// Host emulation of the small part of HIP / gfx950 that libdgs uses, so that the library's
// kernels and host code compile as plain C++ and run on the CPU under AddressSanitizer and
// UndefinedBehaviorSanitizer (test infrastructure; see tests/emu/emu_driver.cpp).
//
// Model.  A launch runs its workgroups one after the other in block order (so a workgroup
// that waits for a word set by a lower block finds it set).  The threads of a workgroup are
// fibers; a thread runs until it reaches a synchronisation point -- a workgroup barrier or a
// wavefront-collective builtin (ballot, readlane, DPP, bpermute, wave barrier) -- where it
// blocks.  When no thread of the workgroup can run, the pending collectives are resolved per
// wavefront and call site among the lanes waiting there (the lanes that took the same branch:
// the hardware's exec mask), then barriers.  LDS (`__shared__`) is static storage, global
// memory is host memory, atomics are plain operations.  Cross-die cache effects are NOT
// modelled: this checks indexing, synchronisation structure and results, not memory ordering.
#pragma once
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <functional>
#include <vector>

#define DGS_HOST_EMULATION 1
#define __global__
#define __device__
#define __host__
// (plain inline: forcing everything into the three kernel bodies made the sanitizer build take minutes)
#define __forceinline__ inline
// LDS: static storage in a section of its own, so that the scheduler can fill all of it with
// garbage before every workgroup starts (the hardware gives a workgroup uninitialised LDS).
#define __shared__ static __attribute__((section("emu_lds")))
#define __launch_bounds__(...)
#define __align__(x) __attribute__((aligned(x)))
#define HIP_SYMBOL(x) (&(x))

struct uint2 { uint32_t x, y; };
struct __attribute__((aligned(16))) uint4 { uint32_t x, y, z, w; };
static inline uint2 make_uint2(uint32_t x, uint32_t y) { return uint2{x, y}; }
static inline uint4 make_uint4(uint32_t x, uint32_t y, uint32_t z, uint32_t w) { return uint4{x, y, z, w}; }
struct dim3 {
    uint32_t x, y, z;
    dim3(uint32_t x_ = 1, uint32_t y_ = 1, uint32_t z_ = 1) : x(x_), y(y_), z(z_) {}
};

typedef int hipError_t;
enum { hipSuccess = 0, hipErrorUnknown = 999 };
typedef void *hipStream_t;
typedef void *hipEvent_t;
enum hipMemcpyKind { hipMemcpyHostToDevice = 1, hipMemcpyDeviceToHost = 2, hipMemcpyDeviceToDevice = 3 };
enum hipStreamCaptureStatus { hipStreamCaptureStatusNone = 0, hipStreamCaptureStatusActive = 1 };
enum { hipHostMallocDefault = 0 };
struct hipDeviceProp_t { int multiProcessorCount; };

static inline hipError_t hipMemcpyAsync(void *d, const void *s, size_t n, hipMemcpyKind, hipStream_t) { memcpy(d, s, n); return hipSuccess; }
static inline hipError_t hipStreamSynchronize(hipStream_t) { return hipSuccess; }
static inline hipError_t hipHostMalloc(void **p, size_t n, unsigned) { *p = malloc(n ? n : 1); return *p ? hipSuccess : hipErrorUnknown; }
static inline hipError_t hipHostFree(void *p) { free(p); return hipSuccess; }
static inline hipError_t hipGetDevice(int *d) { *d = 0; return hipSuccess; }
static inline hipError_t hipGetDeviceProperties(hipDeviceProp_t *p, int) { p->multiProcessorCount = 4; return hipSuccess; }
static inline hipError_t hipGetLastError() { return hipSuccess; }
static inline hipError_t hipEventCreate(hipEvent_t *e) { *e = nullptr; return hipSuccess; }
static inline hipError_t hipEventDestroy(hipEvent_t) { return hipSuccess; }
static inline hipError_t hipEventElapsedTime(float *ms, hipEvent_t, hipEvent_t) { *ms = 0.0f; return hipSuccess; }
static inline hipError_t hipStreamIsCapturing(hipStream_t, hipStreamCaptureStatus *s) { *s = hipStreamCaptureStatusNone; return hipSuccess; }
template <class T> static inline hipError_t hipGetSymbolAddress(void **p, T *sym) { *p = (void *)sym; return hipSuccess; }

namespace emu {

struct Idx { uint32_t x, y, z; };

enum Op { OP_NONE, OP_BALLOT, OP_READLANE, OP_READFIRST, OP_DPP, OP_BPERMUTE, OP_WAVEBAR, OP_BARRIER, OP_BARRIER_OR };
enum State { RUNNABLE, BLOCKED, DONE };

struct Fiber {
    void *sp = nullptr;          // saved stack pointer while the fiber is not running
    char *stack = nullptr;
    State state = DONE;
    Op op = OP_NONE;
    const void *site = nullptr;
    uint64_t a = 0, b = 0, c = 0, d = 0;   // operands
    uint64_t result = 0;
    const void *fake_stack = nullptr;      // ASan fiber bookkeeping
};

struct Machine {
    std::vector<Fiber> fibers;
    void *sched_sp = nullptr;
    uint32_t current = 0, nthreads = 0;
    std::function<void()> body;
    static Machine &get() { static Machine m; return m; }
};

extern "C" void __sanitizer_start_switch_fiber(void **fake_stack_save, const void *bottom, size_t size) __attribute__((weak));
extern "C" void __sanitizer_finish_switch_fiber(void *fake_stack_save, const void **bottom_old, size_t *size_old) __attribute__((weak));

constexpr size_t STACK_BYTES = 256 * 1024;

}  // namespace emu

extern emu::Idx threadIdx, blockIdx, blockDim, gridDim;

namespace emu {

void to_scheduler();                 // block the current fiber (state already set) and run others
uint64_t collective(Op op, const void *site, uint64_t a, uint64_t b = 0, uint64_t c = 0, uint64_t d = 0);
void launch(dim3 grid, dim3 block, const std::function<void()> &body);

}  // namespace emu

// ---- workgroup / wavefront builtins
#define EMU_SITE __builtin_return_address(0)
__attribute__((noinline)) static void __syncthreads() { emu::collective(emu::OP_BARRIER, EMU_SITE, 0); }
__attribute__((noinline)) static int __syncthreads_or(int p) { return (int)emu::collective(emu::OP_BARRIER_OR, EMU_SITE, p != 0); }
__attribute__((noinline)) static uint64_t __builtin_amdgcn_ballot_w64(bool p) { return emu::collective(emu::OP_BALLOT, EMU_SITE, p); }
__attribute__((noinline)) static int __builtin_amdgcn_readlane(int v, int lane) { return (int)emu::collective(emu::OP_READLANE, EMU_SITE, (uint32_t)v, (uint32_t)lane); }
__attribute__((noinline)) static uint32_t __builtin_amdgcn_readfirstlane(uint32_t v) { return (uint32_t)emu::collective(emu::OP_READFIRST, EMU_SITE, v); }
__attribute__((noinline)) static int __builtin_amdgcn_update_dpp(int old, int src, int ctrl, int row_mask, int bank_mask, bool bound_ctrl)
{
    (void)bank_mask; (void)bound_ctrl;
    return (int)emu::collective(emu::OP_DPP, EMU_SITE, (uint32_t)old, (uint32_t)src, (uint32_t)ctrl, (uint32_t)row_mask);
}
__attribute__((noinline)) static int __builtin_amdgcn_ds_bpermute(int addr, int v) { return (int)emu::collective(emu::OP_BPERMUTE, EMU_SITE, (uint32_t)addr, (uint32_t)v); }
__attribute__((noinline)) static void __builtin_amdgcn_wave_barrier() { emu::collective(emu::OP_WAVEBAR, EMU_SITE, 0); }
static inline uint32_t __builtin_amdgcn_mbcnt_lo(uint32_t mask, uint32_t acc)
{
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t m = lane >= 32 ? 0xFFFFFFFFu : ((1u << lane) - 1u);
    return acc + (uint32_t)__builtin_popcount(mask & m);
}
static inline uint32_t __builtin_amdgcn_mbcnt_hi(uint32_t mask, uint32_t acc)
{
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t m = lane <= 32 ? 0u : ((1u << (lane - 32)) - 1u);
    return acc + (uint32_t)__builtin_popcount(mask & m);
}
static inline void __builtin_amdgcn_s_sleep(int) {}
#define __builtin_amdgcn_fence(...) ((void)0)

// ---- scalar helpers
static inline uint32_t __float_as_uint(float f) { uint32_t u; memcpy(&u, &f, 4); return u; }
static inline float __uint_as_float(uint32_t u) { float f; memcpy(&f, &u, 4); return f; }
static inline int __popcll(unsigned long long x) { return __builtin_popcountll(x); }
static inline int __ffsll(unsigned long long x) { return __builtin_ffsll((long long)x); }
using std::max;
using std::min;
static inline float fmaxf_(float a, float b) { return a > b ? a : b; }

// ---- atomics (one thread runs at a time)
template <class T> static inline T atomicAdd(T *p, T v) { T o = *p; *p = o + v; return o; }
template <class T> static inline T atomicMin(T *p, T v) { T o = *p; if (v < o) *p = v; return o; }
template <class T> static inline T atomicOr(T *p, T v) { T o = *p; *p = o | v; return o; }
// __hip_atomic_load / _store / _fetch_add are compiler builtins that also exist for the host.
#ifndef __HIP_MEMORY_SCOPE_AGENT
#define __HIP_MEMORY_SCOPE_AGENT 4
#endif

// ---- launches
template <class K, class... A>
static inline void hipLaunchKernelGGL(K kernel, dim3 grid, dim3 block, size_t, hipStream_t, A... args)
{
    emu::launch(grid, block, [=]() { kernel(args...); });
}
template <class K, class... A>
static inline void hipExtLaunchKernelGGL(K kernel, dim3 grid, dim3 block, size_t, hipStream_t, hipEvent_t, hipEvent_t, int,
                                         A... args)
{
    emu::launch(grid, block, [=]() { kernel(args...); });
}
