// Fiber scheduler and guarded allocator behind hip_emu.h (test scaffolding only).
#include "hip_emu.h"

#include <sys/mman.h>
#include <ucontext.h>
#include <unistd.h>

#include <cstdio>
#include <cstdlib>
#include <map>
#include <vector>

dim3 threadIdx, blockIdx, blockDim, gridDim;

namespace emu {

static const size_t kStack = 256 * 1024;
static ucontext_t g_main;
static std::vector<ucontext_t> g_ctx;
static std::vector<char *> g_stack;
static std::vector<char> g_done;
static int g_cur = -1;
static const std::function<void()> *g_body = nullptr;

static void trampoline() {
    (*g_body)();
    g_done[g_cur] = 1;
    swapcontext(&g_ctx[g_cur], &g_main);
}

void sync() { swapcontext(&g_ctx[g_cur], &g_main); }

void launch(dim3 grid, dim3 block, const std::function<void()> &body) {
    const unsigned nt = block.x * block.y * block.z;
    if (g_stack.size() < nt) {
        size_t old = g_stack.size();
        g_stack.resize(nt);
        for (size_t i = old; i < nt; i++) g_stack[i] = (char *)malloc(kStack);
    }
    g_ctx.resize(nt);
    g_done.assign(nt, 0);
    g_body = &body;
    gridDim = grid;
    blockDim = block;
    for (unsigned bz = 0; bz < grid.z; bz++)
        for (unsigned by = 0; by < grid.y; by++)
            for (unsigned bx = 0; bx < grid.x; bx++) {
                for (unsigned t = 0; t < nt; t++) {
                    getcontext(&g_ctx[t]);
                    g_ctx[t].uc_stack.ss_sp = g_stack[t];
                    g_ctx[t].uc_stack.ss_size = kStack;
                    g_ctx[t].uc_link = &g_main;
                    makecontext(&g_ctx[t], trampoline, 0);
                    g_done[t] = 0;
                }
                unsigned left = nt;
                while (left) {
                    for (unsigned t = 0; t < nt; t++) {
                        if (g_done[t]) continue;
                        g_cur = (int)t;
                        blockIdx = dim3(bx, by, bz);
                        threadIdx = dim3(t % block.x, (t / block.x) % block.y, t / (block.x * block.y));
                        swapcontext(&g_main, &g_ctx[t]);
                        if (g_done[t]) left--;
                    }
                }
            }
    g_cur = -1;
}

static std::map<void *, std::pair<void *, size_t>> g_maps;

void *guarded_alloc(size_t bytes) {
    const size_t page = (size_t)sysconf(_SC_PAGESIZE);
    size_t body = (bytes + page - 1) / page * page;
    if (body == 0) body = page;
    char *base = (char *)mmap(nullptr, body + 2 * page, PROT_READ | PROT_WRITE, MAP_PRIVATE | MAP_ANONYMOUS, -1, 0);
    if (base == (char *)MAP_FAILED) return nullptr;
    mprotect(base, page, PROT_NONE);
    mprotect(base + page + body, page, PROT_NONE);
    // end of the buffer flush against the trailing guard page (16-byte aligned)
    char *user = base + page + (body - ((bytes + 15) / 16 * 16));
    g_maps[user] = std::make_pair((void *)base, body + 2 * page);
    return user;
}

void guarded_free(void *p) {
    auto it = g_maps.find(p);
    if (it == g_maps.end()) return;
    munmap(it->second.first, it->second.second);
    g_maps.erase(it);
}

}  // namespace emu

// Matrix-core instruction v_mfma_i32_16x16x64_i8 for one wave of 64 fibers: lane l supplies 16 bytes of A (row l%16,
// k-group l/16) and of B (column l%16, k-group l/16) and receives D[4*(l/16)+r][l%16].  Every thread of the block must
// reach the call (the exchange uses the block barrier).
typedef int emu_v4i __attribute__((vector_size(16)));
emu_v4i emu_mfma_i32_16x16x64_i8(emu_v4i a, emu_v4i b, emu_v4i c) {
    static emu_v4i sa[1024], sb[1024];
    const unsigned tid = threadIdx.x + blockDim.x * (threadIdx.y + blockDim.y * threadIdx.z);
    sa[tid] = a;
    sb[tid] = b;
    emu::sync();
    const unsigned base = tid & ~63u, lane = tid & 63u, col = lane % 16, g = lane / 16;
    for (int r = 0; r < 4; r++) {
        const unsigned row = 4 * g + r;
        int sum = 0;
        for (unsigned kg = 0; kg < 4; kg++) {
            signed char ab[16], bb[16];
            memcpy(ab, &sa[base + kg * 16 + row], 16);
            memcpy(bb, &sb[base + kg * 16 + col], 16);
            for (int t = 0; t < 16; t++) sum += (int)ab[t] * (int)bb[t];
        }
        c[r] += sum;
    }
    emu::sync();
    return c;
}

extern "C" void *emu_alloc(size_t bytes) { return emu::guarded_alloc(bytes); }
extern "C" void emu_free(void *p) { emu::guarded_free(p); }
