// Scheduler of the host emulation (see hip/hip_runtime.h).
#include <hip/hip_runtime.h>

emu::Idx threadIdx, blockIdx, blockDim, gridDim;

extern "C" char __start_emu_lds[] __attribute__((weak));
extern "C" char __stop_emu_lds[] __attribute__((weak));

namespace emu {

// Minimal stack switch (System V x86-64): callee-saved registers on the old stack, stack
// pointers exchanged.  (swapcontext would make a system call per switch.)
extern "C" void emu_stack_switch(void **save_sp, void *load_sp);
asm(R"(
    .text
    .globl emu_stack_switch
    .type emu_stack_switch,@function
emu_stack_switch:
    pushq %rbp
    pushq %rbx
    pushq %r12
    pushq %r13
    pushq %r14
    pushq %r15
    movq %rsp, (%rdi)
    movq %rsi, %rsp
    popq %r15
    popq %r14
    popq %r13
    popq %r12
    popq %rbx
    popq %rbp
    ret
    .size emu_stack_switch, .-emu_stack_switch
)");

static void switch_to(void **from_sp, void *to_sp, void **fake_save, const void *to_bottom, size_t to_size)
{
    if (__sanitizer_start_switch_fiber) __sanitizer_start_switch_fiber(fake_save, to_bottom, to_size);
    emu_stack_switch(from_sp, to_sp);
}

static const void *g_sched_bottom = nullptr;
static size_t g_sched_size = 0;

static void fiber_entry()
{
    Machine &m = Machine::get();
    if (__sanitizer_finish_switch_fiber) __sanitizer_finish_switch_fiber(nullptr, &g_sched_bottom, &g_sched_size);
    m.body();
    Fiber &f = m.fibers[m.current];
    f.state = DONE;
    // leave for good: tell ASan this fiber's fake stack can go
    if (__sanitizer_start_switch_fiber) __sanitizer_start_switch_fiber(nullptr, g_sched_bottom, g_sched_size);
    void *dead = nullptr;
    emu_stack_switch(&dead, m.sched_sp);
    abort();   // never resumed
}

void to_scheduler()
{
    Machine &m = Machine::get();
    Fiber &f = m.fibers[m.current];
    void *fake = nullptr;
    switch_to(&f.sp, m.sched_sp, &fake, g_sched_bottom, g_sched_size);
    if (__sanitizer_finish_switch_fiber) __sanitizer_finish_switch_fiber(fake, &g_sched_bottom, &g_sched_size);
}

uint64_t collective(Op op, const void *site, uint64_t a, uint64_t b, uint64_t c, uint64_t d)
{
    Machine &m = Machine::get();
    Fiber &f = m.fibers[m.current];
    f.state = BLOCKED;
    f.op = op;
    f.site = site;
    f.a = a; f.b = b; f.c = c; f.d = d;
    to_scheduler();
    return f.result;
}

static void resolve_wave_group(Machine &m, uint32_t wave, const void *site, Op op)
{
    const uint32_t lo = wave * 64, hi = std::min<uint32_t>(lo + 64, m.nthreads);
    bool in[64] = {false};
    for (uint32_t t = lo; t < hi; ++t) {
        Fiber &f = m.fibers[t];
        in[t - lo] = (f.state == BLOCKED && f.site == site && f.op == op);
    }
    uint64_t ballot = 0;
    int first = -1;
    for (int l = 0; l < 64; ++l) {
        if (!in[l]) continue;
        if (first < 0) first = l;
        if (op == OP_BALLOT && m.fibers[lo + l].a) ballot |= 1ull << l;
    }
    for (int l = 0; l < 64; ++l) {
        if (!in[l]) continue;
        Fiber &f = m.fibers[lo + l];
        switch (op) {
        case OP_BALLOT: f.result = ballot; break;
        case OP_READFIRST: f.result = m.fibers[lo + first].a; break;
        case OP_READLANE: {
            const uint32_t s = (uint32_t)f.b & 63u;
            f.result = in[s] ? m.fibers[lo + s].a : 0u;
            break;
        }
        case OP_BPERMUTE: {
            const uint32_t s = ((uint32_t)f.a >> 2) & 63u;
            f.result = in[s] ? m.fibers[lo + s].b : 0u;
            break;
        }
        case OP_DPP: {
            // a = old, b = src, c = dpp_ctrl, d = row_mask; bank mask 0xf, bound_ctrl off
            const uint32_t ctrl = (uint32_t)f.c, rmask = (uint32_t)f.d;
            const int row = l >> 4, pos = l & 15;
            uint64_t r = f.a;
            if ((rmask >> row) & 1u) {
                int src = -1;
                if (ctrl >= 0x111 && ctrl <= 0x11F) {            // row_shr:n
                    const int n = (int)(ctrl - 0x110);
                    if (pos - n >= 0) src = row * 16 + pos - n;
                } else if (ctrl == 0x142) {                      // row_bcast:15
                    if (row > 0) src = (row - 1) * 16 + 15;
                } else if (ctrl == 0x143) {                      // row_bcast:31
                    if (row >= 2) src = 31;
                } else {
                    fprintf(stderr, "emu: unsupported dpp_ctrl 0x%x\n", ctrl);
                    abort();
                }
                if (src >= 0 && in[src]) r = m.fibers[lo + src].b;
            }
            f.result = r;
            break;
        }
        default: f.result = 0; break;
        }
    }
    for (int l = 0; l < 64; ++l)
        if (in[l]) {
            m.fibers[lo + l].state = RUNNABLE;
            m.fibers[lo + l].op = OP_NONE;
        }
}

static void run_block(Machine &m)
{
    for (;;) {
        bool ran = false, live = false;
        for (uint32_t t = 0; t < m.nthreads; ++t) {
            Fiber &f = m.fibers[t];
            if (f.state != RUNNABLE) continue;
            ran = true;
            m.current = t;
            threadIdx = Idx{t, 0, 0};
            void *fake = nullptr;
            switch_to(&m.sched_sp, f.sp, &fake, f.stack, STACK_BYTES);
            if (__sanitizer_finish_switch_fiber) __sanitizer_finish_switch_fiber(fake, nullptr, nullptr);
        }
        for (uint32_t t = 0; t < m.nthreads; ++t) live |= (m.fibers[t].state != DONE);
        if (!live) return;
        if (ran) continue;
        // nobody can run: resolve wavefront collectives first
        bool resolved = false;
        const uint32_t nw = (m.nthreads + 63) / 64;
        for (uint32_t w = 0; w < nw; ++w) {
            for (uint32_t t = w * 64; t < std::min<uint32_t>(w * 64 + 64, m.nthreads); ++t) {
                Fiber &f = m.fibers[t];
                if (f.state == BLOCKED && f.op != OP_BARRIER && f.op != OP_BARRIER_OR) {
                    resolve_wave_group(m, w, f.site, f.op);
                    resolved = true;
                }
            }
        }
        if (resolved) continue;
        // then the workgroup barrier: every live thread must be waiting at one
        bool all = true, any_or = false;
        for (uint32_t t = 0; t < m.nthreads; ++t) {
            Fiber &f = m.fibers[t];
            if (f.state == DONE) continue;
            if (f.op != OP_BARRIER && f.op != OP_BARRIER_OR) all = false;
            if (f.op == OP_BARRIER_OR && f.a) any_or = true;
        }
        if (!all) {
            fprintf(stderr, "emu: deadlock in block %u\n", blockIdx.x);
            abort();
        }
        for (uint32_t t = 0; t < m.nthreads; ++t) {
            Fiber &f = m.fibers[t];
            if (f.state == DONE) continue;
            f.result = any_or;
            f.state = RUNNABLE;
            f.op = OP_NONE;
        }
    }
}

void launch(dim3 grid, dim3 block, const std::function<void()> &body)
{
    Machine &m = Machine::get();
    if (block.y != 1 || block.z != 1 || grid.z != 1) {
        fprintf(stderr, "emu: unsupported launch shape\n");
        abort();
    }
    m.nthreads = block.x;
    if (m.fibers.size() < m.nthreads) m.fibers.resize(m.nthreads);
    for (uint32_t t = 0; t < m.nthreads; ++t)
        if (!m.fibers[t].stack) m.fibers[t].stack = (char *)malloc(STACK_BYTES);
    m.body = body;
    blockDim = Idx{block.x, 1, 1};
    gridDim = Idx{grid.x, grid.y, 1};
    for (uint32_t by = 0; by < grid.y; ++by)
        for (uint32_t bx = 0; bx < grid.x; ++bx) {
            blockIdx = Idx{bx, by, 0};
            if (__start_emu_lds && __stop_emu_lds > __start_emu_lds)
                memset(__start_emu_lds, 0xCD, (size_t)(__stop_emu_lds - __start_emu_lds));   // LDS starts as garbage
            for (uint32_t t = 0; t < m.nthreads; ++t) {
                Fiber &f = m.fibers[t];
                // a fresh stack that "returns" into fiber_entry: six zeroed callee-saved registers, then
                // the entry address, placed so that the stack is 16-byte aligned at the entry's first push
                uintptr_t top = ((uintptr_t)f.stack + STACK_BYTES) & ~(uintptr_t)15;
                void **sp = (void **)(top - 8);
                *--sp = (void *)&fiber_entry;
                for (int i = 0; i < 6; ++i) *--sp = nullptr;
                f.sp = sp;
                f.state = RUNNABLE;
                f.op = OP_NONE;
            }
            run_block(m);
        }
}

}  // namespace emu
