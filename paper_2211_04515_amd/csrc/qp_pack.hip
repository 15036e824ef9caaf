// Step 3: clip + uniform quantize + bit-pack (Sec. 3: ACIQ clipping, then PTQ with the
// chosen bitwidth).  HBM-bound: (4 + k/8) bytes per fp32 element, (2 + k/8) per bf16.
//
// One block of 256 lanes (four wave64s) owns a tile of 4096 (fp32) or 8192 (bf16) consecutive
// elements, 16 KB of input either way.
//   stage 1  each lane issues four coalesced 16-byte loads (lane i of a wave reads bytes
//            [16 i, 16 i + 16) of a 1 KB segment), quantizes the elements of each load and
//            merges the codes of four neighbours into one 4k-bit chunk, which it writes to LDS
//            at the chunk's position in the tile;
//   stage 2  the LDS tile is (k = 2,4,8,16) already the output byte stream, or (k = 3,6) an
//            array of 12/24-bit chunks that eight/four at a time squeeze into three dwords;
//            lanes read it back 16 bytes at a time and store 128-bit (k = 3,6: 96-bit)
//            words, consecutive lanes to consecutive addresses.  For k = 3,6 on tensors of 2^24
//            elements or more (RESTAGE) the three dwords go back to LDS first and leave as
//            128-bit words like the others: 8-10 % faster there (151 M bf16 elements: 64.9 ->
//            58.3 us at 3 bit, 71.2 -> 65.8 us at 6 bit), 2-4 % slower on a 9.7 M-element
//            tensor, where the extra barrier shows.
// So both the loads and the stores of a wave are contiguous, and the bit-packing is a
// cooperative transpose through LDS rather than per-lane strided access.  Loads and stores
// are nontemporal (the tensor and the payload are touched once); measured on MI355X that is
// worth about 10 % of HBM rate, and four loads per lane beat eight.
#include "qp_common.hpp"

namespace qp {

constexpr int kPkThreads = 256;
constexpr int kPkLoads = 4;                               // 16-byte loads per lane
// a load brings 4 fp32 or 8 bf16 elements, i.e. one or two chunks of 4 codes
template <int DT> struct PackTile {
    static constexpr int chunks_per_load = Vec16<DT>::kElems / 4;
    static constexpr int chunks = kPkThreads * kPkLoads * chunks_per_load;   // 1024 (fp32) / 2048 (bf16)
    static constexpr int elems = chunks * 4;                                  // 4096 / 8192 elements per tile
};

struct Grid4 {
    float lo, hi, inv_scale, L;
};

template <int K> struct PackLds {           // bytes of LDS per chunk
    static constexpr int per_chunk = (K == 2) ? 1 : (K == 3 || K == 4) ? 2 : (K == 6 || K == 8) ? 4 : 8;
};

// merge four codes (floats holding integers in [0, 2^K - 1]) and put the chunk in LDS
template <int K>
__device__ __forceinline__ void put_chunk(unsigned char *lds, uint32_t ci, const float (&r)[4])
{
    const uint32_t c0 = (uint32_t)r[0], c1 = (uint32_t)r[1], c2 = (uint32_t)r[2], c3 = (uint32_t)r[3];
    if constexpr (K == 16) {
        reinterpret_cast<uint2 *>(lds)[ci] = make_uint2(c0 | (c1 << 16), c2 | (c3 << 16));
    } else {
        const uint32_t chunk = c0 | (c1 << K) | (c2 << (2 * K)) | (c3 << (3 * K));
        if constexpr (K == 2) reinterpret_cast<uint8_t *>(lds)[ci] = (uint8_t)chunk;
        else if constexpr (K == 3 || K == 4) reinterpret_cast<uint16_t *>(lds)[ci] = (uint16_t)chunk;
        else reinterpret_cast<uint32_t *>(lds)[ci] = chunk;   // K = 6 (24 bits), K = 8
    }
}

// four 24-bit fields -> three dwords
__device__ __forceinline__ void squeeze24(uint32_t w0, uint32_t w1, uint32_t w2, uint32_t w3, uint32_t (&o)[3])
{
    o[0] = w0 | (w1 << 24);
    o[1] = (w1 >> 8) | (w2 << 16);
    o[2] = (w2 >> 16) | (w3 << 8);
}

// one group: K = 3, eight 12-bit chunks (one per 16-bit LDS slot); K = 6, four 24-bit chunks -> three dwords
template <int K> __device__ __forceinline__ void squeeze_group(const uint4 a, uint32_t (&o)[3])
{
    if constexpr (K == 3) {
        const uint32_t w0 = (a.x & 0xfffu) | ((a.x >> 16) << 12);
        const uint32_t w1 = (a.y & 0xfffu) | ((a.y >> 16) << 12);
        const uint32_t w2 = (a.z & 0xfffu) | ((a.z >> 16) << 12);
        const uint32_t w3 = (a.w & 0xfffu) | ((a.w >> 16) << 12);
        squeeze24(w0, w1, w2, w3, o);
    } else {
        squeeze24(a.x, a.y, a.z, a.w, o);
    }
}

template <int K, int DT, bool RESTAGE>
__global__ __launch_bounds__(kPkThreads) void k_quant_pack(const void *__restrict__ x, uint64_t n, Grid4 g,
                                                           const qp_qparams_t *__restrict__ qdev,
                                                           uint32_t *__restrict__ out, uint64_t ndw)
{
    constexpr int kPkTile = PackTile<DT>::elems;
    constexpr int CPL = PackTile<DT>::chunks_per_load;
    constexpr int E = Vec16<DT>::kElems;
    __shared__ __align__(16) unsigned char lds[PackTile<DT>::chunks * PackLds<K>::per_chunk];
    const uint32_t tid = threadIdx.x;
    if (qdev) {   // grid left in device memory by the search
        g.lo = qdev->lo;
        g.hi = qdev->hi;
        g.inv_scale = qdev->inv_scale;
    }
    const uint64_t e0 = (uint64_t)blockIdx.x * kPkTile;

    // ---- stage 1 ----
    if (e0 + kPkTile <= n) {
        float f[kPkLoads][E];
#pragma unroll
        for (int u = 0; u < kPkLoads; ++u)
            load16_stream<DT>(x, e0 / E + (uint64_t)u * kPkThreads + tid, f[u]);
#pragma unroll
        for (int u = 0; u < kPkLoads; ++u) {
#pragma unroll
            for (int h = 0; h < CPL; ++h) {
                float r[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) r[i] = quant_level(f[u][4 * h + i], g.lo, g.hi, g.inv_scale, g.L);
                put_chunk<K>(lds, ((uint32_t)u * kPkThreads + tid) * CPL + h, r);
            }
        }
    } else {   // last, partial tile: elements past the end count as code 0
#pragma unroll 1
        for (int u = 0; u < kPkLoads * CPL; ++u) {
            const uint32_t ci = (uint32_t)u * kPkThreads + tid;
            const uint64_t e = e0 + 4ull * ci;
            float r[4];
#pragma unroll
            for (int i = 0; i < 4; ++i)
                r[i] = (e + i < n) ? quant_level(Vec4<DT>::load1(x, e + i), g.lo, g.hi, g.inv_scale, g.L) : 0.0f;
            put_chunk<K>(lds, ci, r);
        }
    }
    __syncthreads();

    // ---- stage 2 ----
    constexpr uint32_t tile_dw = kPkTile * K / 32;           // dwords of output per tile
    const uint64_t d0 = (uint64_t)blockIdx.x * tile_dw;
    if constexpr ((K == 3 || K == 6) && !RESTAGE) {
        // groups of three dwords: K = 3 from eight 12-bit chunks, K = 6 from four 24-bit chunks
        constexpr uint32_t groups = tile_dw / 3;               // 128 (K = 3) or 256 (K = 6)
        for (uint32_t gi = tid; gi < groups; gi += kPkThreads) {
            uint32_t o[3];
            squeeze_group<K>(reinterpret_cast<const uint4 *>(lds)[gi], o);
            const uint64_t d = d0 + 3ull * gi;
            if (d + 3 <= ndw) {
                uint32_t *p = out + d;
                struct alignas(4) U3 { uint32_t a, b, c; };
                *reinterpret_cast<U3 *>(p) = U3{o[0], o[1], o[2]};
            } else {
#pragma unroll
                for (int i = 0; i < 3; ++i)
                    if (d + i < ndw) out[d + i] = o[i];
            }
        }
    } else {
        if constexpr (K == 3 || K == 6) {
            // A lane squeezes its one or two groups in registers; once every lane has read its chunks the dwords
            // go back to LDS, where they form the tile's output byte stream as for the other bitwidths.
            constexpr uint32_t groups = tile_dw / 3;           // 128 ... 512
            constexpr int GPL = (groups + kPkThreads - 1) / kPkThreads;
            uint32_t o[GPL][3];
#pragma unroll
            for (int i = 0; i < GPL; ++i) {
                const uint32_t gi = tid + (uint32_t)i * kPkThreads;
                if (gi < groups) squeeze_group<K>(reinterpret_cast<const uint4 *>(lds)[gi], o[i]);
            }
            __syncthreads();
#pragma unroll
            for (int i = 0; i < GPL; ++i) {
                const uint32_t gi = tid + (uint32_t)i * kPkThreads;
                if (gi < groups) {
                    uint32_t *w = reinterpret_cast<uint32_t *>(lds) + 3u * gi;
                    w[0] = o[i][0];
                    w[1] = o[i][1];
                    w[2] = o[i][2];
                }
            }
            __syncthreads();
        }
        constexpr uint32_t quads = tile_dw / 4;                // 16-byte words of output per tile
        for (uint32_t qi = tid; qi < quads; qi += kPkThreads) {
            const uint4 a = reinterpret_cast<const uint4 *>(lds)[qi];
            const uint64_t d = d0 + 4ull * qi;
            if (d + 4 <= ndw) {
                __builtin_nontemporal_store(u32x4{a.x, a.y, a.z, a.w}, reinterpret_cast<u32x4 *>(out) + d / 4);
            } else {
                const uint32_t o[4] = {a.x, a.y, a.z, a.w};
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    if (d + i < ndw) out[d + i] = o[i];
            }
        }
    }
}

template <int K, int DT, bool RESTAGE>
static hipError_t launch_form(const void *x, uint64_t n, Grid4 g, const qp_qparams_t *qdev, void *packed, hipStream_t s)
{
    const uint64_t ndw = (n * K + 31) / 32;
    const uint32_t blocks = ceil_div_u64(n, PackTile<DT>::elems);
    hipLaunchKernelGGL((k_quant_pack<K, DT, RESTAGE>), dim3(blocks), dim3(kPkThreads), 0, s, x, n, g, qdev,
                       static_cast<uint32_t *>(packed), ndw);
    return hipGetLastError();
}

template <int K>
static hipError_t launch_k(const void *x, uint64_t n, int dtype, Grid4 g, const qp_qparams_t *qdev, void *packed,
                           hipStream_t s)
{
    if constexpr (K == 3 || K == 6) {
        if (n >= kLargeFormsMinN)
            return dtype == QP_F32 ? launch_form<K, QP_F32, true>(x, n, g, qdev, packed, s)
                                   : launch_form<K, QP_BF16, true>(x, n, g, qdev, packed, s);
    }
    return dtype == QP_F32 ? launch_form<K, QP_F32, false>(x, n, g, qdev, packed, s)
                           : launch_form<K, QP_BF16, false>(x, n, g, qdev, packed, s);
}

hipError_t launch_quant_pack(const void *x, uint64_t n, int dtype, uint32_t bits, const qp_qparams_t *hq,
                             const qp_qparams_t *dq, void *packed, hipStream_t s)
{
    Grid4 g{0.f, 0.f, 0.f, (float)((1u << bits) - 1u)};
    if (hq) {
        g.lo = hq->lo;
        g.hi = hq->hi;
        g.inv_scale = hq->inv_scale;
    }
    switch (bits) {
        case 2: return launch_k<2>(x, n, dtype, g, dq, packed, s);
        case 3: return launch_k<3>(x, n, dtype, g, dq, packed, s);
        case 4: return launch_k<4>(x, n, dtype, g, dq, packed, s);
        case 6: return launch_k<6>(x, n, dtype, g, dq, packed, s);
        case 8: return launch_k<8>(x, n, dtype, g, dq, packed, s);
        case 16: return launch_k<16>(x, n, dtype, g, dq, packed, s);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace qp
