#include <hip/hip_runtime.h>
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

void launch(dim3 grid, dim3 block, const std::function<void()> &fn)
{
    g_blockDim = block;
    g_gridDim = grid;
    if (block.y != 1 || block.z != 1 || grid.z != 1) { fprintf(stderr, "emu: shape not supported\n"); abort(); }
    const unsigned nthreads = block.x, nwaves = (nthreads + 63) / 64;
    for (unsigned by = 0; by < grid.y; ++by)
        for (unsigned bx = 0; bx < grid.x; ++bx) {
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
        }
    g_ctx = nullptr;
}
}  // namespace emu
