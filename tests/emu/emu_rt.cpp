#include <hip/hip_runtime.h>
#include <sys/mman.h>
#include <sys/wait.h>
#include <unistd.h>
namespace emu {
thread_local dim3 t_threadIdx, t_blockIdx;
dim3 g_blockDim, g_gridDim;
int g_occupancy = 3, g_cus = 256;
BlockCtx *g_ctx = nullptr;
thread_local unsigned t_opcount = 0;

uint32_t exchange(uint32_t v, int src_lane, int ctrl, int xor_mask)
{
    const unsigned tid = t_threadIdx.x, wave = tid / 64, lane = tid % 64;
    const unsigned par = (t_opcount++) & 1u;
    uint32_t *buf = &g_ctx->xbuf[(wave * 2 + par) * 64];
    buf[lane] = v;
    g_ctx->wave_bar[wave]->arrive_and_wait();
    unsigned from;
    if (src_lane >= 0) from = (unsigned)src_lane;
    else if (ctrl >= 0) {
        if (ctrl <= 0xFF) from = (lane & ~3u) | ((ctrl >> (2 * (lane & 3))) & 3);
        else if (ctrl == 0x140) from = (lane & ~15u) | (15 - (lane & 15));
        else if (ctrl == 0x141) from = (lane & ~7u) | (7 - (lane & 7));
        else { fprintf(stderr, "emu: dpp ctrl %x not emulated\n", ctrl); abort(); }
    } else from = lane ^ (unsigned)xor_mask;
    return buf[from];
}

// One block: a thread per lane, barriers for the block and for each wave.
static void run_block(unsigned bx, unsigned by, unsigned nthreads, const std::function<void()> &fn)
{
    const unsigned nwaves = (nthreads + 63) / 64;
    BlockCtx ctx;
    ctx.block_bar = std::make_unique<std::barrier<>>(nthreads);
    for (unsigned w = 0; w < nwaves; ++w)
        ctx.wave_bar.push_back(std::make_unique<std::barrier<>>(std::min(64u, nthreads - 64 * w)));
    ctx.xbuf.assign(nwaves * 2 * 64, 0u);
    g_ctx = &ctx;
    std::vector<std::thread> th;
    th.reserve(nthreads);
    for (unsigned t = 0; t < nthreads; ++t)
        th.emplace_back([&, t]() {
            t_threadIdx = dim3(t, 0, 0);
            t_blockIdx = dim3(bx, by, 0);
            t_opcount = 0;
            fn();
            ctx.block_bar->arrive_and_drop();
            ctx.wave_bar[t / 64]->arrive_and_drop();
        });
    for (auto &x : th) x.join();
    g_ctx = nullptr;
}

// EMU_CONCURRENT_BLOCKS=K (K >= 1): the blocks of a launch run in an order shuffled by EMU_SEED, K at a time,
// each in a process of its own (fork), so that __shared__ variables (statics here) are per block as on the
// device while "device memory" is shared: the driver then allocates it with shared_alloc below.  Blocks finish
// and draw their tickets in any order and their atomics interleave, which the in-order mode cannot show.  What
// it still cannot show: the device's memory model (x86 orders stores more strongly than the GPU's caches do).
static int concurrent_blocks()
{
    const char *e = getenv("EMU_CONCURRENT_BLOCKS");
    return e ? atoi(e) : 0;
}

void *shared_alloc(size_t bytes)
{
    // the buffer ends at a page that is not mapped for access: an overrun past the end faults at once
    const size_t page = 4096, body = (bytes + page - 1) / page * page;
    char *base = (char *)mmap(nullptr, body + page, PROT_READ | PROT_WRITE, MAP_SHARED | MAP_ANONYMOUS, -1, 0);
    if (base == (char *)MAP_FAILED) { perror("mmap"); exit(3); }
    if (mprotect(base + body, page, PROT_NONE) != 0) { perror("mprotect"); exit(3); }
    return base + body - (bytes + 15) / 16 * 16;
}

void launch(dim3 grid, dim3 block, const std::function<void()> &fn)
{
    g_blockDim = block;
    g_gridDim = grid;
    if (block.y != 1 || block.z != 1 || grid.z != 1) { fprintf(stderr, "emu: shape not supported\n"); abort(); }
    const unsigned nthreads = block.x;
    const int conc = concurrent_blocks();
    if (conc <= 0) {
        for (unsigned by = 0; by < grid.y; ++by)
            for (unsigned bx = 0; bx < grid.x; ++bx) run_block(bx, by, nthreads, fn);
        return;
    }
    static uint64_t rng = 0;
    if (rng == 0) {
        const char *e = getenv("EMU_SEED");
        rng = 0x9E3779B97F4A7C15ull ^ (e ? strtoull(e, nullptr, 10) * 0xD1342543DE82EF95ull : 1ull);
    }
    auto next = [&]() { rng ^= rng << 13; rng ^= rng >> 7; rng ^= rng << 17; return rng; };
    std::vector<std::pair<unsigned, unsigned>> order;
    for (unsigned by = 0; by < grid.y; ++by)
        for (unsigned bx = 0; bx < grid.x; ++bx) order.emplace_back(bx, by);
    for (size_t i = order.size(); i > 1; --i) std::swap(order[i - 1], order[next() % i]);
    fflush(stdout);
    fflush(stderr);
    for (size_t i = 0; i < order.size(); i += (size_t)conc) {
        std::vector<pid_t> kids;
        for (size_t k = i; k < order.size() && k < i + (size_t)conc; ++k) {
            const pid_t pid = fork();
            if (pid < 0) { perror("fork"); abort(); }
            if (pid == 0) {
                run_block(order[k].first, order[k].second, nthreads, fn);
                _exit(0);
            }
            kids.push_back(pid);
        }
        for (pid_t pid : kids) {
            int status = 0;
            if (waitpid(pid, &status, 0) != pid || !WIFEXITED(status) || WEXITSTATUS(status) != 0) {
                fprintf(stderr, "emu: a block's process failed (status %d)\n", status);
                exit(4);
            }
        }
    }
}
}  // namespace emu
