// NF4 block codec kernels (paper sec. 5.1): stand-alone quantise and dequantise.
// Both are pure HBM streams: 4 + 0.5625 bytes per element for the encoder,
// 0.5625 + 2 (bf16) or 4 (fp32) for the decoder.
#include <string.h>

#include <mutex>

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
        uint32_t near = 0;
#pragma unroll
        for (int e = 0; e < 8; ++e) c[e] = be.encode_fast(&enc, v[e], near);
        if (__any(near)) {  // wave-uniform: some element sits within rounding of a decision point
#pragma unroll
            for (int e = 0; e < 8; ++e) c[e] = be.encode(&enc, v[e]);
        }
        const uint32_t word = nf4_pack4(c[0], c[1], c[2], c[3]) | (nf4_pack4(c[4], c[5], c[6], c[7]) << 16);
        *reinterpret_cast<uint32_t*>(codes + row * (ld_q >> 1) + (j0 >> 1)) = word;
        if (sub == 0) absmax[row * nbr + bcol] = m;
    }
}

// ---------------------------------------------------------------------------------------
// dequantise: 8 elements (4 code bytes) per lane.  (A form with 32 elements per lane -- one 16-byte code load, four
// 16-byte stores -- measured 40 % slower: its stores leave the wave as four quarter-filled lines each.)
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

// The same for several matrices in one launch (the deq(P) of the layers of a grouped merge): every work-group
// belongs to one matrix and walks it with that matrix's share of the grid.  Descriptors travel in the kernel
// argument block.
struct DequantGroupParams {
    int n;
    DequantGroupItem it[MERGE_GROUP_MAX];
    int block_end[MERGE_GROUP_MAX];
};
static_assert(sizeof(DequantGroupParams) <= 4096, "kernel arguments are limited to 4 KB");

__global__ __launch_bounds__(256) void nf4_dequantize_grouped_kernel(const DequantGroupParams g) {
    __shared__ float lut[16];
    if (threadIdx.x < 16) lut[threadIdx.x] = kNf4Levels[threadIdx.x];
    __syncthreads();
    int li = 0;
    while (li + 1 < g.n && (int)blockIdx.x >= g.block_end[li]) ++li;  // wave-uniform
    const int first = li ? g.block_end[li - 1] : 0, nblk = g.block_end[li] - first;
    const DequantGroupItem& it = g.it[li];
    const int cols = it.cols;
    const int gpr = (cols + 7) >> 3;
    const int64_t ngroups = it.rows * gpr;
    for (int64_t gi = (int64_t)((int)blockIdx.x - first) * 256 + threadIdx.x; gi < ngroups; gi += (int64_t)nblk * 256) {
        const int64_t row = gi / gpr;
        const int j0 = (int)(gi - row * gpr) * 8;
        const uint32_t word = *reinterpret_cast<const uint32_t*>(it.codes + row * (it.ld_q >> 1) + (j0 >> 1));
        const float m = it.absmax[row * (it.ld_q >> 6) + (j0 >> 6)];
        float v[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const uint32_t c = (word >> (8 * (e >> 1) + ((e & 1) ? 0 : 4))) & 15u;
            v[e] = m * lut[c];
        }
        uint16_t* dst = it.out + row * it.ld_out + j0;
        if (j0 + 8 <= cols) {
            uint4 o;
            o.x = pack_bf16(v[0], v[1]);
            o.y = pack_bf16(v[2], v[3]);
            o.z = pack_bf16(v[4], v[5]);
            o.w = pack_bf16(v[6], v[7]);
            *reinterpret_cast<uint4*>(dst) = o;
        } else {
            for (int e = 0; e < 8 && j0 + e < cols; ++e) dst[e] = (uint16_t)(pack_bf16(v[e], 0.f) & 0xffffu);
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

// ---------------------------------------------------------------------------------------
// Double quantisation of the block scales (paper sec. 2.4 says that the quantisation state is
// itself quantised again; it gives no format, the one used is stated in include/loqt.h):
// scales minus their mean, in blocks of 256 with one fp32 constant c1 = max |d| per block, each
// stored as an 8-bit float (1-4-3, bias 7, no infinities, largest value 448).
// ---------------------------------------------------------------------------------------
constexpr int DQ_BLOCK = 256;
constexpr int DQ_CHUNK = 4096;  // scales summed by one work-group of the mean's first stage

// fixed-order sum of the 256 per-thread values of a work-group (same result on every run)
__device__ __forceinline__ double block_sum_f64(double v, double* sh) {
    sh[threadIdx.x] = v;
    __syncthreads();
#pragma unroll
    for (int s = 128; s > 0; s >>= 1) {
        if ((int)threadIdx.x < s) sh[threadIdx.x] += sh[threadIdx.x + s];
        __syncthreads();
    }
    return sh[0];
}

__global__ __launch_bounds__(256) void dq_partial_sums_kernel(const float* __restrict__ a, int64_t n,
                                                              double* __restrict__ partial) {
    __shared__ double sh[256];
    const int64_t base = (int64_t)blockIdx.x * DQ_CHUNK;
    double acc = 0.0;
#pragma unroll
    for (int i = 0; i < DQ_CHUNK / 256; ++i) {
        const int64_t j = base + i * 256 + threadIdx.x;
        if (j < n) acc += (double)a[j];
    }
    const double tot = block_sum_f64(acc, sh);
    if (threadIdx.x == 0) partial[blockIdx.x] = tot;
}

__global__ __launch_bounds__(256) void dq_mean_kernel(const double* __restrict__ partial, int64_t nparts, int64_t n,
                                                      float* __restrict__ mean) {
    __shared__ double sh[256];
    double acc = 0.0;
    for (int64_t j = threadIdx.x; j < nparts; j += 256) acc += partial[j];
    const double tot = block_sum_f64(acc, sh);
    if (threadIdx.x == 0) *mean = (float)(tot / (double)n);
}

// fp32 -> E4M3 code, round to nearest even, |u| <= 448 by construction (saturates anyway)
__device__ __forceinline__ uint32_t e4m3_encode(float u) {
    const uint32_t bits = __float_as_uint(u);
    const uint32_t sign = (bits >> 24) & 0x80u;
    const float a = fabsf(u);
    uint32_t code;
    if (a < 0.03125f) {
        // below 2^-5 the representable values are the multiples of 2^-9 (subnormals and the first binade)
        code = (uint32_t)__float2int_rn(a * 512.0f);
    } else {
        const uint32_t ab = bits & 0x7fffffffu;
        const uint32_t r = ab + 0x7ffffu + ((ab >> 20) & 1u);  // round the 23-bit mantissa to 3 bits, ties to even
        code = (r >> 20) - (120u << 3);                        // exponent bias 127 -> 7
        if (code > 0x7eu) code = 0x7eu;
    }
    return code | sign;
}
__device__ __forceinline__ float e4m3_decode(uint32_t code) {
    const uint32_t e = (code >> 3) & 15u, m = code & 7u;
    const float mag = e == 0 ? (float)m * 0.001953125f : __uint_as_float(((e + 120u) << 23) | (m << 20));
    return (code & 0x80u) ? -mag : mag;
}

// one work-group per block of 256 scales
__global__ __launch_bounds__(256) void dq_compress_kernel(const float* __restrict__ a, int64_t n,
                                                          const float* __restrict__ mean_p, uint8_t* __restrict__ codes,
                                                          float* __restrict__ c1) {
    __shared__ float shm[4];
    const int64_t j = (int64_t)blockIdx.x * DQ_BLOCK + threadIdx.x;
    const float mean = *mean_p;
    const float d = j < n ? a[j] - mean : 0.f;
    float m = fabsf(d);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o));
    if ((threadIdx.x & 63) == 0) shm[threadIdx.x >> 6] = m;
    __syncthreads();
    const float c = fmaxf(fmaxf(shm[0], shm[1]), fmaxf(shm[2], shm[3]));
    if (threadIdx.x == 0) c1[blockIdx.x] = c;
    if (j < n) {
        uint32_t code = (__float_as_uint(d) >> 24) & 0x80u;  // block of equal scales: +-0
        if (c > 0.f) {
            const float t = d / c;  // correctly rounded division
            code = e4m3_encode(t * 448.0f);
        }
        codes[j] = (uint8_t)code;
    }
}

__global__ __launch_bounds__(256) void dq_expand_kernel(const uint8_t* __restrict__ codes, const float* __restrict__ c1,
                                                        const float* __restrict__ mean_p, int64_t n,
                                                        float* __restrict__ out) {
    const int64_t j = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (j >= n) return;
    const float v = e4m3_decode(codes[j]);
    float t = v * c1[j / DQ_BLOCK];
    t = t / 448.0f;
    out[j] = t + *mean_p;
}

hipError_t launch_dq_compress(const float* absmax, int64_t n, uint8_t* codes, float* c1, float* mean, double* partial,
                              hipStream_t st) {
    const int64_t nparts = (n + DQ_CHUNK - 1) / DQ_CHUNK;
    hipLaunchKernelGGL(dq_partial_sums_kernel, dim3((unsigned)nparts), dim3(256), 0, st, absmax, n, partial);
    hipLaunchKernelGGL(dq_mean_kernel, dim3(1), dim3(256), 0, st, partial, nparts, n, mean);
    hipLaunchKernelGGL(dq_compress_kernel, dim3((unsigned)((n + DQ_BLOCK - 1) / DQ_BLOCK)), dim3(256), 0, st, absmax, n,
                       mean, codes, c1);
    return hipGetLastError();
}
hipError_t launch_dq_expand(const uint8_t* codes, const float* c1, const float* mean, int64_t n, float* out,
                            hipStream_t st) {
    hipLaunchKernelGGL(dq_expand_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, codes, c1, mean, n, out);
    return hipGetLastError();
}
int64_t dq_partials(int64_t n) { return (n + DQ_CHUNK - 1) / DQ_CHUNK; }

// ---------------------------------------------------------------------------------------
// The same compression for callers that cannot allocate (HIP graph capture, serving loops): the
// partial sums of the mean live in a file-scope device array instead of a caller's workspace.
// Every GPU the library runs on holds its own copy of the array at its own address, so the device
// address is looked up once per device (with that device current) and kept; host code never uses
// the array's name for anything else.  All calls on one GPU share the array: calls that overlap on
// one GPU (two streams, two threads) race on it.  Nothing in it has to start at zero: each call
// writes every partial sum it later reads.
// ---------------------------------------------------------------------------------------
constexpr int64_t DQ_STATIC_MAX_N = (int64_t)1 << 25;  // 2^25 scales = 2^31 weights per call
constexpr size_t DQ_STATIC_BYTES = (size_t)(DQ_STATIC_MAX_N / DQ_CHUNK) * sizeof(double);  // 64 KB
static __device__ __align__(256) unsigned char scratch[DQ_STATIC_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void* g_scratch_ptr[kMaxDevices] = {};
}  // namespace

int64_t dq_static_max_n() { return DQ_STATIC_MAX_N; }

// device address of `scratch` on the current device (resolved on first use, then cached)
hipError_t dq_static_scratch(void** out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!ptr) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return hipSuccess;
}

hipError_t launch_dq_compress_static(const float* absmax, int64_t n, uint8_t* codes, float* c1, float* mean,
                                     hipStream_t st) {
    if (n > DQ_STATIC_MAX_N) return hipErrorInvalidValue;  // the caller checks first; never launch past the array
    void* ptr = nullptr;
    hipError_t e = dq_static_scratch(&ptr);
    if (e != hipSuccess) return e;
    return launch_dq_compress(absmax, n, codes, c1, mean, reinterpret_cast<double*>(ptr), st);
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

hipError_t launch_dequantize_grouped(const DequantGroupItem* items, int n, hipStream_t st, int slot) {
    if (n < 1 || n > MERGE_GROUP_MAX) return hipErrorInvalidValue;
    TimedLaunch tl(slot, st);
    DequantGroupParams g;
    memset(&g, 0, sizeof(g));
    g.n = n;
    int total = 0;
    for (int i = 0; i < n; ++i) {
        g.it[i] = items[i];
        total += grid_for(items[i].rows * ((items[i].cols + 7) >> 3), 256 * 4);  // about four groups of 8 per lane
        g.block_end[i] = total;
    }
    hipLaunchKernelGGL(nf4_dequantize_grouped_kernel, dim3((unsigned)total), dim3(256), 0, st, g);
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
