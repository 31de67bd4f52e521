// Streaming pre-passes of the large-token path: NF4 -> bf16 (optionally transposed) and bf16
// transposes, so that every product of the layer becomes a K-contiguous "NT" GEMM.  All of
// them are plain HBM streams over one operand (<= 2.6 bytes per NF4 element, 4 per bf16).
#include "loqt_internal.h"

namespace loqt {

namespace {

constexpr int TP = 72;  // LDS pitch (elements) of a 64 x 64 bf16 tile: 144 bytes, 16-byte aligned

// dst[c][r] = bf16( absmax * q[code[r][c]] ): one 64 x 64 tile (one NF4 block per row) per group
__global__ __launch_bounds__(256) void nf4_dequant_transpose_kernel(const uint8_t* __restrict__ codes,
                                                                    const float* __restrict__ absmax, int rows,
                                                                    int cols, int64_t ld_q,
                                                                    uint16_t* __restrict__ dst, int64_t ld_d) {
    __shared__ __attribute__((aligned(16))) uint16_t tile[64 * TP];  // [col][row]
    __shared__ float lut[16];
    const int t = threadIdx.x;
    if (t < 16) lut[t] = kNf4Levels[t];
    __syncthreads();
    const int tiles_c = (cols + 63) >> 6;
    const int r0 = (blockIdx.x / tiles_c) * 64, c0 = (blockIdx.x % tiles_c) * 64;
    {
        const int r = t >> 2, q = t & 3;  // row of the tile, quarter of its 64 codes
        uint2 w = make_uint2(0x77777777u, 0x77777777u);
        float m = 0.f;
        if (r0 + r < rows) {
            w = *reinterpret_cast<const uint2*>(codes + (int64_t)(r0 + r) * (ld_q >> 1) + (c0 >> 1) + q * 8);
            m = absmax[(int64_t)(r0 + r) * (ld_q >> 6) + (c0 >> 6)];
        }
        const uint32_t ww[2] = {w.x, w.y};
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const uint32_t word = ww[e >> 3];
            const int b = e & 7;
            const uint32_t c = (word >> (8 * (b >> 1) + ((b & 1) ? 0 : 4))) & 15u;
            tile[(q * 16 + e) * TP + r] = (uint16_t)(pack_bf16(m * lut[c], 0.f) & 0xffffu);
        }
    }
    __syncthreads();
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
        const int c = (t >> 3) + 32 * pass, ch = t & 7;
        if (c0 + c < cols) {
            const uint4 v = *reinterpret_cast<const uint4*>(&tile[c * TP + ch * 8]);
            uint16_t* d = dst + (int64_t)(c0 + c) * ld_d + r0 + ch * 8;
            if (r0 + ch * 8 + 8 <= rows) {
                *reinterpret_cast<uint4*>(d) = v;
            } else {
                const uint16_t* s = reinterpret_cast<const uint16_t*>(&v);
                for (int e = 0; e < 8; ++e)
                    if (r0 + ch * 8 + e < rows) d[e] = s[e];
            }
        }
    }
}

// dst[c][r] = src[r][c], bf16, 64 x 64 tiles
__global__ __launch_bounds__(256) void transpose_bf16_kernel(const uint16_t* __restrict__ src, int rows, int cols,
                                                             int64_t ld_s, uint16_t* __restrict__ dst,
                                                             int64_t ld_d) {
    __shared__ __attribute__((aligned(16))) uint16_t tile[64 * TP];  // [row][col]
    const int t = threadIdx.x;
    const int tiles_c = (cols + 63) >> 6;
    const int r0 = (blockIdx.x / tiles_c) * 64, c0 = (blockIdx.x % tiles_c) * 64;
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
        const int r = (t >> 3) + 32 * pass, ch = t & 7;
        uint4 v = make_uint4(0, 0, 0, 0);
        // the pitch is a multiple of 8, so a chunk that starts inside the row stays inside the pitch
        if (r0 + r < rows && c0 + ch * 8 < cols)
            v = *reinterpret_cast<const uint4*>(src + (int64_t)(r0 + r) * ld_s + c0 + ch * 8);
        *reinterpret_cast<uint4*>(&tile[r * TP + ch * 8]) = v;
    }
    __syncthreads();
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
        const int c = (t >> 3) + 32 * pass, ch = t & 7;
        if (c0 + c < cols) {
            uint16_t s[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) s[e] = tile[(ch * 8 + e) * TP + c];
            uint16_t* d = dst + (int64_t)(c0 + c) * ld_d + r0 + ch * 8;
            if (r0 + ch * 8 + 8 <= rows) {
                uint4 v;
                v.x = s[0] | ((uint32_t)s[1] << 16);
                v.y = s[2] | ((uint32_t)s[3] << 16);
                v.z = s[4] | ((uint32_t)s[5] << 16);
                v.w = s[6] | ((uint32_t)s[7] << 16);
                *reinterpret_cast<uint4*>(d) = v;
            } else {
                for (int e = 0; e < 8; ++e)
                    if (r0 + ch * 8 + e < rows) d[e] = s[e];
            }
        }
    }
}

}  // namespace

hipError_t launch_dequant_transpose(const uint8_t* codes, const float* absmax, int64_t rows, int64_t cols,
                                    int64_t ld_q, uint16_t* dst, int64_t ld_d, hipStream_t st) {
    TimedLaunch tl(SLOT_PREPASS, st);
    const int64_t blocks = ((rows + 63) / 64) * ((cols + 63) / 64);
    hipLaunchKernelGGL(nf4_dequant_transpose_kernel, dim3((unsigned)blocks), dim3(256), 0, st, codes, absmax,
                       (int)rows, (int)cols, ld_q, dst, ld_d);
    return hipGetLastError();
}

hipError_t launch_transpose_bf16(const uint16_t* src, int64_t rows, int64_t cols, int64_t ld_s, uint16_t* dst,
                                 int64_t ld_d, hipStream_t st) {
    TimedLaunch tl(SLOT_PREPASS, st);
    const int64_t blocks = ((rows + 63) / 64) * ((cols + 63) / 64);
    hipLaunchKernelGGL(transpose_bf16_kernel, dim3((unsigned)blocks), dim3(256), 0, st, src, (int)rows, (int)cols,
                       ld_s, dst, ld_d);
    return hipGetLastError();
}

}  // namespace loqt
