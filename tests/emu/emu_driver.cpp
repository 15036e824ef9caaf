// TEST INFRASTRUCTURE ONLY: drives the library's C ABI on the CPU emulation (host memory stands in
// for device memory) and writes everything it produced to files, for comparison with the oracle.
//   emu_driver <in.bin> <n> <dtype 0|1> <bits> <t_steps> <dist> <flags> <stride> <nbins> <cus> <outdir> [cands_per_round]
#include <hip/hip_runtime.h>

#include <string>
#include <vector>

#include "quantpipe.h"

namespace emu { extern int g_occupancy, g_cus; void *shared_alloc(size_t); }

static void dump(const std::string &dir, const char *name, const void *p, size_t bytes)
{
    FILE *f = fopen((dir + "/" + name).c_str(), "wb");
    if (!f || fwrite(p, 1, bytes, f) != bytes) { perror(name); exit(3); }
    fclose(f);
}

static bool g_shared = false;             // blocks run as processes: "device memory" must be shared between them
static void *alloc_exact(size_t bytes)   // 16-byte aligned; the sanitizer sees any overrun past `bytes` (rounded to 16)
{
    if (g_shared) return emu::shared_alloc(bytes);   // ends at an inaccessible page instead
    void *p = aligned_alloc(16, (bytes + 15) / 16 * 16);
    if (!p) exit(3);
    return p;
}
static void release(void *p)
{
    if (!g_shared) free(p);
}

int main(int argc, char **argv)
{
    if (argc != 12 && argc != 13) { fprintf(stderr, "usage: see source\n"); return 2; }
    const char *in = argv[1];
    const uint64_t n = strtoull(argv[2], nullptr, 10);
    const qp_dtype dtype = (qp_dtype)atoi(argv[3]);
    const uint32_t bits = (uint32_t)atoi(argv[4]);
    qp_search_cfg_t cfg;
    qp_default_search_cfg(&cfg);
    cfg.t_steps = (uint32_t)atoi(argv[5]);
    cfg.dist = (uint32_t)atoi(argv[6]);
    cfg.flags = (uint32_t)atoi(argv[7]);
    cfg.coarse_stride = (uint32_t)atoi(argv[8]);
    cfg.nbins = (uint32_t)atoi(argv[9]);
    emu::g_cus = atoi(argv[10]);
    const std::string out = argv[11];
    if (argc == 13) cfg.cands_per_round = (uint32_t)atoi(argv[12]);

    g_shared = getenv("EMU_CONCURRENT_BLOCKS") && atoi(getenv("EMU_CONCURRENT_BLOCKS")) > 0;
    const size_t esz = dtype == QP_BF16 ? 2 : 4;
    void *x = alloc_exact(n * esz);
    FILE *f = fopen(in, "rb");
    if (!f || fread(x, esz, n, f) != n) { perror("input"); return 3; }
    fclose(f);

    const size_t wsb = qp_workspace_bytes(n, &cfg), pkb = qp_packed_bytes(n, bits);
    void *ws = alloc_exact(wsb), *ws2 = alloc_exact(wsb);
    memset(ws, 0xC3, wsb);
    memset(ws2, 0x5A, wsb);
    void *packed = alloc_exact(pkb), *packed2 = alloc_exact(pkb);
    memset(packed, 0x77, pkb);
    memset(packed2, 0x11, pkb);
    float *y = (float *)alloc_exact(n * 4);

    qp_stats_t st;
    qp_search_result_t res;
    qp_qparams_t q;
    memset(&res, 0, sizeof res);
    memset(&q, 0, sizeof q);
    int rc_stats = qp_stats(x, n, dtype, cfg.nbins, ws, wsb, nullptr, &st);
    int rc_search = qp_dsaciq_search(x, n, dtype, &st, bits, &cfg, ws, wsb, nullptr, &res, &q);
    int rc_pack = -100, rc_unpack = -100, rc_compress = -100, same = -1;
    if (rc_search == QP_OK) {
        rc_pack = qp_quant_pack(x, n, dtype, &q, packed, pkb, nullptr);
        rc_unpack = qp_unpack_dequant(packed, pkb, &q, y, n, nullptr);
        qp_qparams_t &qout = *(qp_qparams_t *)alloc_exact(sizeof(qp_qparams_t));
        rc_compress = qp_compress_async(x, n, dtype, bits, &cfg, ws2, wsb, packed2, pkb, &qout, nullptr);
        if (rc_compress == QP_OK) {
            const char *a = (const char *)ws, *b = (const char *)ws2;
            same = memcmp(a + qp_ws_offset(QP_WS_STATS), b + qp_ws_offset(QP_WS_STATS), sizeof(qp_stats_t)) == 0 &&
                   memcmp(a + qp_ws_offset(QP_WS_QPARAMS), b + qp_ws_offset(QP_WS_QPARAMS), sizeof(qp_qparams_t)) == 0 &&
                   memcmp(&qout, &q, sizeof q) == 0 && memcmp(packed, packed2, pkb) == 0;
        }
    }
    dump(out, "stats.bin", &st, sizeof st);
    dump(out, "hist.bin", (const char *)ws + qp_ws_offset(QP_WS_HIST), (size_t)cfg.nbins * 4);
    dump(out, "result.bin", &res, sizeof res);
    dump(out, "qparams.bin", &q, sizeof q);
    dump(out, "scores.bin", (const char *)ws + qp_ws_offset(QP_WS_SCORES), ((size_t)cfg.t_steps + 1) * 8);
    // what the fused sender path left in its own workspace (its search may run a different kernel sequence)
    dump(out, "scores2.bin", (const char *)ws2 + qp_ws_offset(QP_WS_SCORES), ((size_t)cfg.t_steps + 1) * 8);
    dump(out, "result2.bin", (const char *)ws2 + qp_ws_offset(QP_WS_RESULT), sizeof res);
    dump(out, "packed.bin", packed, pkb);
    dump(out, "y.bin", y, n * 4);
    char line[256];
    snprintf(line, sizeof line, "%d %d %d %d %d %d\n", rc_stats, rc_search, rc_pack, rc_unpack, rc_compress, same);
    dump(out, "status.txt", line, strlen(line));
    release(x); release(ws); release(ws2); release(packed); release(packed2); release(y);
    return 0;
}
