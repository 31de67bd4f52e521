// NF4 block codec kernels (paper sec. 5.1): stand-alone quantise and dequantise.
// Both are pure HBM streams: 4 + 0.5625 bytes per element for the encoder,
// 0.5625 + 2 (bf16) or 4 (fp32) for the decoder.
#include "loqt_internal.h"

namespace loqt {

// ---------------------------------------------------------------------------------------
// quantise: 8 lanes per block of 64, 8 consecutive elements per lane (two 16-byte loads,
// one 4-byte store).  The block maximum is a 3-step butterfly inside each group of 8 lanes.
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void nf4_quantize_kernel(const float* __restrict__ w, int64_t rows,
                                                           int cols, int64_t ld_w,
                                                           uint8_t* __restrict__ codes,
                                                           float* __restrict__ absmax, int64_t ld_q) {
    __shared__ Nf4EncTables enc;
    if (threadIdx.x < 64) nf4_enc_tables_fill(&enc, threadIdx.x);
    __syncthreads();
    const int nbr = (int)(ld_q >> 6);  // blocks per row, padding included
    const int64_t nblocks = rows * nbr;
    const int sub = threadIdx.x & 7;
    for (int64_t blk = (int64_t)blockIdx.x * 32 + (threadIdx.x >> 3); blk < nblocks;
         blk += (int64_t)gridDim.x * 32) {
        const int64_t row = blk / nbr;
        const int bcol = (int)(blk - row * nbr);
        const int j0 = bcol * 64 + sub * 8;
        const float* src = w + row * ld_w + j0;
        float v[8];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            float4 f = make_float4(0.f, 0.f, 0.f, 0.f);
            if (j0 + 4 * h < cols) f = *reinterpret_cast<const float4*>(src + 4 * h);
            v[4 * h + 0] = (j0 + 4 * h + 0 < cols) ? f.x : 0.f;
            v[4 * h + 1] = (j0 + 4 * h + 1 < cols) ? f.y : 0.f;
            v[4 * h + 2] = (j0 + 4 * h + 2 < cols) ? f.z : 0.f;
            v[4 * h + 3] = (j0 + 4 * h + 3 < cols) ? f.w : 0.f;
        }
        float m = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) m = fmaxf(m, fabsf(v[e]));
        m = fmaxf(m, __shfl_xor(m, 1));
        m = fmaxf(m, __shfl_xor(m, 2));
        m = fmaxf(m, __shfl_xor(m, 4));
        // elements past `cols` were read as 0 and encode to 7 like any zero
        Nf4BlockEncoder be;
        be.set(m);
        uint32_t c[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) c[e] = be.encode(&enc, v[e]);
        const uint32_t word = nf4_pack4(c[0], c[1], c[2], c[3]) | (nf4_pack4(c[4], c[5], c[6], c[7]) << 16);
        *reinterpret_cast<uint32_t*>(codes + row * (ld_q >> 1) + (j0 >> 1)) = word;
        if (sub == 0) absmax[row * nbr + bcol] = m;
    }
}

// ---------------------------------------------------------------------------------------
// dequantise: 8 elements (4 code bytes) per lane.
// ---------------------------------------------------------------------------------------
template <int OUT_BF16>
__global__ __launch_bounds__(256) void nf4_dequantize_kernel(const uint8_t* __restrict__ codes,
                                                             const float* __restrict__ absmax,
                                                             int64_t rows, int cols, int64_t ld_q,
                                                             void* __restrict__ out, int64_t ld_out) {
    __shared__ float lut[16];
    if (threadIdx.x < 16) lut[threadIdx.x] = kNf4Levels[threadIdx.x];
    __syncthreads();
    const int gpr = (cols + 7) >> 3;  // groups of 8 elements per row
    const int64_t ngroups = rows * gpr;
    for (int64_t g = (int64_t)blockIdx.x * 256 + threadIdx.x; g < ngroups;
         g += (int64_t)gridDim.x * 256) {
        const int64_t row = g / gpr;
        const int j0 = (int)(g - row * gpr) * 8;
        const uint32_t word = *reinterpret_cast<const uint32_t*>(codes + row * (ld_q >> 1) + (j0 >> 1));
        const float m = absmax[row * (ld_q >> 6) + (j0 >> 6)];
        float v[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const uint32_t c = (word >> (8 * (e >> 1) + ((e & 1) ? 0 : 4))) & 15u;
            v[e] = m * lut[c];
        }
        if (OUT_BF16) {
            uint16_t* dst = reinterpret_cast<uint16_t*>(out) + row * ld_out + j0;
            if (j0 + 8 <= cols) {
                uint4 o;
                o.x = pack_bf16(v[0], v[1]);
                o.y = pack_bf16(v[2], v[3]);
                o.z = pack_bf16(v[4], v[5]);
                o.w = pack_bf16(v[6], v[7]);
                *reinterpret_cast<uint4*>(dst) = o;
            } else {
                for (int e = 0; e < 8 && j0 + e < cols; ++e)
                    dst[e] = (uint16_t)(pack_bf16(v[e], 0.f) & 0xffffu);
            }
        } else {
            float* dst = reinterpret_cast<float*>(out) + row * ld_out + j0;
            if (j0 + 8 <= cols) {
                *reinterpret_cast<float4*>(dst) = make_float4(v[0], v[1], v[2], v[3]);
                *reinterpret_cast<float4*>(dst + 4) = make_float4(v[4], v[5], v[6], v[7]);
            } else {
                for (int e = 0; e < 8 && j0 + e < cols; ++e) dst[e] = v[e];
            }
        }
    }
}

// ---------------------------------------------------------------------------------------
// fp32 -> bf16 copy of a matrix (round to nearest even): 4 elements per lane.  ld_in % 4 == 0 and
// ld_out % 4 == 0, so a group of 4 never leaves its row's pitch; columns past `cols` are written as 0.
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void f32_to_bf16_kernel(const float* __restrict__ in, int64_t rows, int cols,
                                                          int64_t ld_in, uint16_t* __restrict__ out,
                                                          int64_t ld_out) {
    const int gpr = (cols + 3) >> 2;
    const int64_t ngroups = rows * gpr;
    for (int64_t g = (int64_t)blockIdx.x * 256 + threadIdx.x; g < ngroups; g += (int64_t)gridDim.x * 256) {
        const int64_t row = g / gpr;
        const int j0 = (int)(g - row * gpr) * 4;
        const float4 f = *reinterpret_cast<const float4*>(in + row * ld_in + j0);
        const float v1 = j0 + 1 < cols ? f.y : 0.f, v2 = j0 + 2 < cols ? f.z : 0.f, v3 = j0 + 3 < cols ? f.w : 0.f;
        *reinterpret_cast<uint2*>(out + row * ld_out + j0) = make_uint2(pack_bf16(f.x, v1), pack_bf16(v2, v3));
    }
}

// ---------------------------------------------------------------------------------------
// Adam on the trainable factor (paper Alg. 1 line 9: B <- B - rho(G^B), rho = Adam): bf16 parameter,
// fp32 moments, fp32 arithmetic, one rounding to bf16 at the end.  24 bytes per element with an fp32
// gradient: a pure HBM stream.
// ---------------------------------------------------------------------------------------
template <int G_BF16>
__global__ __launch_bounds__(256) void adam_kernel(uint16_t* __restrict__ B, int64_t ld_B, const void* __restrict__ g,
                                                   int64_t ld_g, float* __restrict__ m, float* __restrict__ v,
                                                   int64_t ld_mv, int64_t rows, int cols, float lr, float beta1,
                                                   float beta2, float eps, float bc1, float bc2) {
    const int64_t total = rows * cols;
    for (int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x; idx < total; idx += (int64_t)gridDim.x * 256) {
        const int64_t row = idx / cols;
        const int col = (int)(idx - row * cols);
        float grad;
        if (G_BF16) grad = __uint_as_float((uint32_t)reinterpret_cast<const uint16_t*>(g)[row * ld_g + col] << 16);
        else grad = reinterpret_cast<const float*>(g)[row * ld_g + col];
        const int64_t k = row * ld_mv + col;
        const float mn = beta1 * m[k] + (1.0f - beta1) * grad;
        const float vn = beta2 * v[k] + (1.0f - beta2) * grad * grad;
        m[k] = mn;
        v[k] = vn;
        const float upd = lr * (mn * bc1) / (sqrtf(vn * bc2) + eps);
        uint16_t* b = B + row * ld_B + col;
        const float bf = __uint_as_float((uint32_t)(*b) << 16);
        *b = (uint16_t)(pack_bf16(bf - upd, 0.f) & 0xffffu);
    }
}

static int grid_for(int64_t work_items, int per_block) {
    int64_t b = (work_items + per_block - 1) / per_block;
    const int64_t cap = 256 * 64;  // enough waves to saturate HBM; the kernels grid-stride
    if (b > cap) b = cap;
    if (b < 1) b = 1;
    return (int)b;
}

hipError_t launch_quantize(const float* w, int64_t rows, int64_t cols, int64_t ld_w, uint8_t* codes,
                           float* absmax, int64_t ld_q, hipStream_t st) {
    TimedLaunch tl(SLOT_QUANTIZE, st);
    const int64_t nblocks = rows * (ld_q >> 6);
    hipLaunchKernelGGL(nf4_quantize_kernel, dim3(grid_for(nblocks, 32)), dim3(256), 0, st, w, rows,
                       (int)cols, ld_w, codes, absmax, ld_q);
    return hipGetLastError();
}

hipError_t launch_dequantize(const uint8_t* codes, const float* absmax, int64_t rows, int64_t cols,
                             int64_t ld_q, void* out, int out_dtype, int64_t ld_out, hipStream_t st, int slot) {
    TimedLaunch tl(slot, st);
    const int64_t ngroups = rows * ((cols + 7) >> 3);
    const int grid = grid_for(ngroups, 256);
    if (out_dtype == LOQT_BF16)
        hipLaunchKernelGGL(nf4_dequantize_kernel<1>, dim3(grid), dim3(256), 0, st, codes, absmax, rows,
                           (int)cols, ld_q, out, ld_out);
    else
        hipLaunchKernelGGL(nf4_dequantize_kernel<0>, dim3(grid), dim3(256), 0, st, codes, absmax, rows,
                           (int)cols, ld_q, out, ld_out);
    return hipGetLastError();
}

hipError_t launch_adam(uint16_t* B, int64_t ld_B, const void* g, int g_dtype, int64_t ld_g, float* m, float* v,
                       int64_t ld_mv, int64_t rows, int64_t cols, float lr, float beta1, float beta2, float eps,
                       float bc1, float bc2, hipStream_t st) {
    TimedLaunch tl(SLOT_ADAM, st);
    const int grid = grid_for(rows * cols, 256);
    if (g_dtype == LOQT_BF16)
        hipLaunchKernelGGL(adam_kernel<1>, dim3(grid), dim3(256), 0, st, B, ld_B, g, ld_g, m, v, ld_mv, rows,
                           (int)cols, lr, beta1, beta2, eps, bc1, bc2);
    else
        hipLaunchKernelGGL(adam_kernel<0>, dim3(grid), dim3(256), 0, st, B, ld_B, g, ld_g, m, v, ld_mv, rows,
                           (int)cols, lr, beta1, beta2, eps, bc1, bc2);
    return hipGetLastError();
}

hipError_t launch_f32_to_bf16(const float* in, int64_t rows, int64_t cols, int64_t ld_in, uint16_t* out,
                              int64_t ld_out, hipStream_t st) {
    TimedLaunch tl(SLOT_PREPASS, st);
    const int64_t ngroups = rows * ((cols + 3) >> 2);
    hipLaunchKernelGGL(f32_to_bf16_kernel, dim3(grid_for(ngroups, 256)), dim3(256), 0, st, in, rows, (int)cols,
                       ld_in, out, ld_out);
    return hipGetLastError();
}

}  // namespace loqt
