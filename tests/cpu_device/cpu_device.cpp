// Test scaffolding (CPU only): runs "kernels" on the host.  A launch executes block after block; the threads of a
// block are fibers (ucontext) resumed round-robin, so that __syncthreads and wavefront shuffles (64 consecutive
// threads) behave as on the device: a thread that reaches one waits until its whole block / wavefront has.
#include <hip/hip_runtime.h>
#include <ucontext.h>

#include <cstdio>
#include <cstdlib>
#include <vector>

#if defined(__has_feature)
#if __has_feature(address_sanitizer)
#define GA_FIBERS_UNDER_ASAN 1
#include <sanitizer/common_interface_defs.h>
#endif
#endif

cpu_device::Index threadIdx, blockIdx;
dim3 blockDim, gridDim;

namespace cpu_device {
namespace {

constexpr size_t kStackBytes = 256 * 1024;
constexpr int kWave = 64;

struct Fiber {
    ucontext_t ctx;
    bool done;
};

ucontext_t g_scheduler;
std::vector<Fiber> g_fibers;
std::vector<char> g_stacks;
const std::function<void()>* g_body = nullptr;
uint32_t g_current = 0, g_threads = 0;
// block barrier
uint32_t g_arrived = 0, g_generation = 0;
uint64_t g_events = 0;   // barrier releases and thread exits: a round of the scheduler without any is a deadlock
// per wavefront: exchange buffer and two-phase barrier
std::vector<uint64_t> g_lane_bits;
std::vector<uint32_t> g_wave_arrived, g_wave_generation;

void switch_to(ucontext_t* from, ucontext_t* to, const void* to_stack, size_t to_size) {
#ifdef GA_FIBERS_UNDER_ASAN
    void* fake = nullptr;
    __sanitizer_start_switch_fiber(&fake, to_stack, to_size);
    swapcontext(from, to);
    __sanitizer_finish_switch_fiber(fake, nullptr, nullptr);
#else
    (void)to_stack; (void)to_size;
    swapcontext(from, to);
#endif
}

const void* g_main_stack = nullptr;
size_t g_main_stack_size = 0;

void yield() {
    Fiber& f = g_fibers[g_current];
    switch_to(&f.ctx, &g_scheduler, g_main_stack, g_main_stack_size);
}

void fiber_entry() {
#ifdef GA_FIBERS_UNDER_ASAN
    __sanitizer_finish_switch_fiber(nullptr, &g_main_stack, &g_main_stack_size);
#endif
    (*g_body)();
    g_fibers[g_current].done = true;
    yield();
    std::abort();   // a finished fiber is never resumed
}

uint32_t wave_size_of(uint32_t wave) {
    const uint32_t first = wave * kWave;
    return g_threads - first < (uint32_t)kWave ? g_threads - first : (uint32_t)kWave;
}

void sync_wave(uint32_t wave) {
    const uint32_t gen = g_wave_generation[wave];
    if (++g_wave_arrived[wave] == wave_size_of(wave)) {
        g_wave_arrived[wave] = 0;
        ++g_wave_generation[wave];
        ++g_events;
        return;
    }
    while (g_wave_generation[wave] == gen) yield();
}

}  // namespace

void sync_block() {
    const uint32_t gen = g_generation;
    if (++g_arrived == g_threads) {
        g_arrived = 0;
        ++g_generation;
        ++g_events;
        return;
    }
    while (g_generation == gen) yield();
}

uint64_t shuffle_xor_bits(uint64_t bits, int lane_mask) {
    const uint32_t me = g_current, wave = me / kWave;
    g_lane_bits[me] = bits;
    sync_wave(wave);
    uint32_t partner = (me % kWave) ^ (uint32_t)lane_mask;
    partner = wave * kWave + partner;
    const uint64_t got = partner < g_threads ? g_lane_bits[partner] : bits;
    sync_wave(wave);   // nobody overwrites its slot before every lane has read
    return got;
}

void launch(dim3 grid, dim3 block, const std::function<void()>& thread_body) {
    if (grid.y != 1 || grid.z != 1 || block.y != 1 || block.z != 1 || block.x == 0 || grid.x == 0) {
        std::fprintf(stderr, "cpu_device: only one-dimensional launches\n");
        std::abort();
    }
    g_threads = block.x;
    gridDim = grid;
    blockDim = block;
    g_body = &thread_body;
    if (g_fibers.size() < g_threads) {
        g_fibers.resize(g_threads);
        g_stacks.resize((size_t)g_threads * kStackBytes);
        g_lane_bits.resize(g_threads);
    }
    const uint32_t waves = (g_threads + kWave - 1) / kWave;
    g_wave_arrived.assign(waves, 0);
    g_wave_generation.assign(waves, 0);
    for (uint32_t b = 0; b < grid.x; ++b) {
        blockIdx = {b, 0, 0};
        g_arrived = 0;
        for (uint32_t t = 0; t < g_threads; ++t) {
            Fiber& f = g_fibers[t];
            f.done = false;
            getcontext(&f.ctx);
            f.ctx.uc_stack.ss_sp = g_stacks.data() + (size_t)t * kStackBytes;
            f.ctx.uc_stack.ss_size = kStackBytes;
            f.ctx.uc_link = nullptr;
            makecontext(&f.ctx, fiber_entry, 0);
        }
        uint32_t remaining = g_threads;
        while (remaining > 0) {
            const uint64_t events_before = g_events;
            for (uint32_t t = 0; t < g_threads; ++t) {
                Fiber& f = g_fibers[t];
                if (f.done) continue;
                g_current = t;
                threadIdx = {t, 0, 0};
                switch_to(&g_scheduler, &f.ctx, f.ctx.uc_stack.ss_sp, kStackBytes);
                if (f.done) {
                    --remaining;
                    ++g_events;
                }
            }
            if (g_events == events_before) {
                std::fprintf(stderr, "cpu_device: block %u: %u threads wait at a barrier or shuffle that the others never reach\n", b, remaining);
                std::abort();
            }
        }
    }
    g_body = nullptr;
}

}  // namespace cpu_device
