// Step 4: unpack + dequantize (the receiving stage consumes fp32 again; Sec. 3).
// HBM-bound and write-dominated: k/8 bytes in, 4 bytes out per element.
//
// A lane produces one 16-byte store per step: four consecutive elements, i.e. one 4k-bit
// chunk of the code stream.  Consecutive lanes take consecutive chunks, so a wave64 writes
// 1 KB contiguous per store instruction.  The chunk is fetched with the narrowest aligned
// load that covers it (byte / halfword / dword / two dwords); for k = 3 and 6 a chunk may
// straddle two dwords, so both are read (neighbouring lanes share them, the loads coalesce
// in the vector cache) and joined with one funnel shift.  The stores are nontemporal: the
// output is written once and not read back by this kernel.  The loads are ordinary ones:
// neighbouring lanes and waves share the packed cache lines, and nontemporal loads of them
// measured up to 30 % slower.
#include "qp_common.hpp"

namespace qp {

// Two block shapes, chosen by the launcher from measurements with every stream cold (payloads rotating over more
// than twice the Infinity Cache): 256 lanes x 4 stores for tensors up to 2^24 elements, 512 lanes x 2 stores beyond
// (10 to 15 % faster on 77 M and 151 M elements, where a lane that fetches for four stores at a time leaves the
// write stream idle for longer; equal or slightly slower on 10 M elements) and for 6-bit codes at any size.
struct UpSmall { static constexpr int threads = 256, stores = 4; };
struct UpLarge { static constexpr int threads = 512, stores = 2; };

struct Deq {
    float lo, scale;
};

// the 4k-bit chunk number ci of the stream (k <= 8); ndw = dwords in the buffer
template <int K>
__device__ __forceinline__ uint32_t get_chunk(const uint32_t *__restrict__ p, uint64_t ci, uint64_t ndw)
{
    if constexpr (K == 2) return reinterpret_cast<const uint8_t *>(p)[ci];
    else if constexpr (K == 4) return reinterpret_cast<const uint16_t *>(p)[ci];
    else if constexpr (K == 8) return p[ci];
    else {
        const uint64_t bit = ci * (4 * K);
        const uint64_t d = bit >> 5;
        const uint32_t s = (uint32_t)bit & 31u;
        const uint32_t w0 = p[d];
        const uint32_t w1 = p[(d + 1 < ndw) ? d + 1 : d];   // never past the end; unused bits when it is clamped
        return __builtin_amdgcn_alignbit(w1, w0, s);          // ((w1:w0) >> s)[31:0]
    }
}

template <int K>
__device__ __forceinline__ float4 expand(const uint32_t *__restrict__ p, uint64_t ci, uint64_t ndw, Deq q)
{
    float c[4];
    if constexpr (K == 16) {
        const uint2 w = reinterpret_cast<const uint2 *>(p)[ci];
        c[0] = (float)(w.x & 0xffffu);
        c[1] = (float)(w.x >> 16);
        c[2] = (float)(w.y & 0xffffu);
        c[3] = (float)(w.y >> 16);
    } else {
        const uint32_t w = get_chunk<K>(p, ci, ndw);
        constexpr uint32_t m = (1u << K) - 1u;
        c[0] = (float)(w & m);
        c[1] = (float)((w >> K) & m);
        c[2] = (float)((w >> (2 * K)) & m);
        c[3] = (float)((w >> (3 * K)) & m);
    }
    return make_float4(dequant_level(c[0], q.scale, q.lo), dequant_level(c[1], q.scale, q.lo),
                       dequant_level(c[2], q.scale, q.lo), dequant_level(c[3], q.scale, q.lo));
}

template <int K, typename SHAPE>
__global__ __launch_bounds__(SHAPE::threads) void k_unpack_dequant(const uint32_t *__restrict__ packed, uint64_t ndw, Deq q,
                                                               const qp_qparams_t *__restrict__ qdev,
                                                               float *__restrict__ y, uint64_t n)
{
    constexpr int kUpThreads = SHAPE::threads, kUpStores = SHAPE::stores;   // 16-byte stores per lane
    constexpr int kUpTileChunks = kUpThreads * kUpStores;
    if (qdev) {
        q.lo = qdev->lo;
        q.scale = qdev->scale;
    }
    const uint32_t tid = threadIdx.x;
    const uint64_t nchunk = n / 4;   // whole chunks
    const uint64_t c0 = (uint64_t)blockIdx.x * kUpTileChunks;
    float4 *__restrict__ y4 = reinterpret_cast<float4 *>(y);
    if (c0 + kUpTileChunks <= nchunk) {
        float4 v[kUpStores];
#pragma unroll
        for (int u = 0; u < kUpStores; ++u) v[u] = expand<K>(packed, c0 + (uint64_t)u * kUpThreads + tid, ndw, q);
#pragma unroll
        for (int u = 0; u < kUpStores; ++u) {
            __builtin_nontemporal_store(f32x4{v[u].x, v[u].y, v[u].z, v[u].w},
                                        reinterpret_cast<f32x4 *>(y) + c0 + (uint64_t)u * kUpThreads + tid);
        }
    } else {
        for (uint64_t ci = c0 + tid; ci < nchunk; ci += kUpThreads) y4[ci] = expand<K>(packed, ci, ndw, q);
        // last n mod 4 elements: one lane, bit by bit out of the dwords that hold them
        if (c0 + kUpTileChunks > nchunk && c0 <= nchunk && tid == 0) {
            for (uint64_t i = nchunk * 4; i < n; ++i) {
                const uint64_t bit = i * K;
                const uint64_t d = bit >> 5;
                const uint32_t s = (uint32_t)bit & 31u;
                uint32_t w = packed[d] >> s;
                if (s + K > 32) w |= packed[d + 1] << (32 - s);
                const uint32_t c = w & ((1u << K) - 1u);
                y[i] = dequant_level((float)c, q.scale, q.lo);
            }
        }
    }
}

template <int K, typename SHAPE>
static hipError_t launch_shape(const void *packed, Deq q, const qp_qparams_t *qdev, float *y, uint64_t n, hipStream_t s)
{
    const uint64_t ndw = (n * K + 31) / 32;
    // one extra block when n is a multiple of the tile keeps the "last block takes the tail" rule simple
    const uint32_t blocks = (uint32_t)((n / 4) / (SHAPE::threads * SHAPE::stores) + 1);
    hipLaunchKernelGGL((k_unpack_dequant<K, SHAPE>), dim3(blocks), dim3(SHAPE::threads), 0, s,
                       static_cast<const uint32_t *>(packed), ndw, q, qdev, y, n);
    return hipGetLastError();
}

template <int K>
static hipError_t launch_k(const void *packed, Deq q, const qp_qparams_t *qdev, float *y, uint64_t n, hipStream_t s)
{
    if (n >= kLargeFormsMinN || K == 6) return launch_shape<K, UpLarge>(packed, q, qdev, y, n, s);
    return launch_shape<K, UpSmall>(packed, q, qdev, y, n, s);
}

hipError_t launch_unpack_dequant(const void *packed, uint32_t bits, const qp_qparams_t *hq, const qp_qparams_t *dq,
                                 float *y, uint64_t n, hipStream_t s)
{
    Deq q{0.f, 0.f};
    if (hq) {
        q.lo = hq->lo;
        q.scale = hq->scale;
    }
    switch (bits) {
        case 2: return launch_k<2>(packed, q, dq, y, n, s);
        case 3: return launch_k<3>(packed, q, dq, y, n, s);
        case 4: return launch_k<4>(packed, q, dq, y, n, s);
        case 6: return launch_k<6>(packed, q, dq, y, n, s);
        case 8: return launch_k<8>(packed, q, dq, y, n, s);
        case 16: return launch_k<16>(packed, q, dq, y, n, s);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace qp
