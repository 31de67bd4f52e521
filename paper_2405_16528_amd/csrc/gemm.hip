// bf16 MFMA GEMM for gfx950 with NF4 dequantisation fused into the operand staging.
//
//   C[M x N] = alpha * sum_seg  A_seg[M x K_seg] * B_seg[K_seg x N]        (fp32 accumulate)
//
// One kernel template serves every product of the LoQT layer (paper sec. 2.2 / 2.4, Alg. 1):
//   U  = s x B^T                 y  = x deq(W)^T + U deq(P)^T
//   Z  = s dy deq(P)             dx = dy deq(W) + Z B
//   dB = Z^T x (split over T)    merge: (deq(P) B)^T tile + deq(W) -> requantise
// Operands come in four storage kinds (bf16 or NF4, contiguous along K or along the row
// index); whatever the kind, a 64-deep K slice of the operand tile is brought to LDS as
// bf16 [row][k] with k contiguous, so the MFMA inner loop is the same for all of them.
// NF4 codes are expanded on the way from global memory to LDS: nibble -> 16-entry fp32
// table held in LDS -> times the block's absmax -> round to nearest even bf16.
//
// Work-group: 256 threads = 4 waves in a 2 x 2 grid, each wave owns (BM/2) x (BN/2) of C as
// 32x32 MFMA tiles (v_mfma_f32_32x32x16_bf16).  LDS holds two stages of (BM + BN) rows x 128
// bytes; 16-byte chunks of a row are XOR-swizzled so that both the fragment reads (32 rows,
// same chunk) and the staging writes are free of bank conflicts.
#include "loqt_internal.h"

namespace loqt {

namespace {

constexpr int BK = 64;         // K depth of one stage (= one NF4 block)
constexpr int ROW_BYTES = 128; // BK bf16

__device__ __forceinline__ int swz(int row) { return (row & 7) ^ ((row >> 3) & 1); }
__device__ __forceinline__ int lds_off(int row, int chunk) {
    return row * ROW_BYTES + ((chunk ^ swz(row)) << 4);
}

__device__ __forceinline__ uint32_t nib(uint32_t word, int e) {
    // element e (0..7) of a 4-byte group: byte e/2, even e in the high nibble
    return (word >> (8 * (e >> 1) + ((e & 1) ? 0 : 4))) & 15u;
}

// ---------------------------------------------------------------------------------------
// Tile staging: global -> registers (load), registers -> LDS as bf16 [row][k] (store).
// The two halves are separate so that the global loads of the next K slice are in flight
// while the MFMAs of the current one run.
// ---------------------------------------------------------------------------------------
template <int KIND, int BR>
struct Stager;

// bf16, rows x K, K contiguous: 16-byte chunks, 8 lanes cover one 128-byte row slice
template <int BR>
struct Stager<KC_BF16, BR> {
    static constexpr int NV = BR / 32;
    uint4 v[NV];
    int kleft;
    __device__ __forceinline__ void load(const Operand& op, int row0, int k0, int tid) {
        kleft = op.K - k0;
        const uint16_t* base = reinterpret_cast<const uint16_t*>(op.ptr);
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            const int c = tid + 256 * i, row = c >> 3, kc = c & 7;
            v[i] = make_uint4(0, 0, 0, 0);
            if (row0 + row < op.rows && kc * 8 < kleft)
                v[i] = *reinterpret_cast<const uint4*>(base + (int64_t)(row0 + row) * op.ld + k0 + kc * 8);
        }
    }
    __device__ __forceinline__ void store(char* tile, const float*, int tid) {
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            const int c = tid + 256 * i, row = c >> 3, kc = c & 7;
            uint4 o = v[i];
            if (kleft < BK) {  // K tail: zero the elements past the end
                const int nv = kleft - kc * 8;  // valid elements in this chunk
                uint32_t* w = reinterpret_cast<uint32_t*>(&o);
#pragma unroll
                for (int d = 0; d < 4; ++d) {
                    if (2 * d >= nv) w[d] = 0;
                    else if (2 * d + 1 >= nv) w[d] &= 0xffffu;
                }
            }
            *reinterpret_cast<uint4*>(tile + lds_off(row, kc)) = o;
        }
    }
};

// bf16, K x rows, rows contiguous: each thread takes a patch of KP k-values x 8 rows,
// transposes it in registers and writes 8 row pieces of KP consecutive k.
template <int BR>
struct Stager<RC_BF16, BR> {
    static constexpr int KP = BR / 32;  // 8 (BR 256) or 4 (BR 128)
    uint4 v[KP];
    __device__ __forceinline__ void load(const Operand& op, int row0, int k0, int tid) {
        const int rg = tid % (BR / 8), kg = tid / (BR / 8);
        const uint16_t* base = reinterpret_cast<const uint16_t*>(op.ptr);
        const int r = row0 + rg * 8;
#pragma unroll
        for (int j = 0; j < KP; ++j) {
            const int k = k0 + kg * KP + j;
            v[j] = make_uint4(0, 0, 0, 0);
            if (k < op.K && r < op.rows)
                v[j] = *reinterpret_cast<const uint4*>(base + (int64_t)k * op.ld + r);
        }
    }
    __device__ __forceinline__ void store(char* tile, const float*, int tid) {
        const int rg = tid % (BR / 8), kg = tid / (BR / 8);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            uint32_t o[KP / 2];
#pragma unroll
            for (int d = 0; d < KP / 2; ++d) {
                const uint32_t lo = reinterpret_cast<const uint32_t*>(&v[2 * d])[i >> 1];
                const uint32_t hi = reinterpret_cast<const uint32_t*>(&v[2 * d + 1])[i >> 1];
                o[d] = __builtin_amdgcn_perm(hi, lo, (i & 1) ? 0x07060302u : 0x05040100u);
            }
            const int row = rg * 8 + i;
            if constexpr (KP == 8) {
                *reinterpret_cast<uint4*>(tile + lds_off(row, kg)) = make_uint4(o[0], o[1], o[2], o[3]);
            } else {
                *reinterpret_cast<uint2*>(tile + lds_off(row, kg >> 1) + (kg & 1) * 8) = make_uint2(o[0], o[1]);
            }
        }
    }
};

// NF4, rows x K, K contiguous: a 16-byte unit is 32 codes of one row, all with one absmax
template <int BR>
struct Stager<KC_NF4, BR> {
    static constexpr int NU = BR / 128;
    uint4 v[NU];
    float am[NU];
    int kleft;
    __device__ __forceinline__ void load(const Operand& op, int row0, int k0, int tid) {
        kleft = op.K - k0;
        const uint8_t* base = reinterpret_cast<const uint8_t*>(op.ptr);
#pragma unroll
        for (int i = 0; i < NU; ++i) {
            const int u = tid + 256 * i, row = u >> 1, half = u & 1;
            v[i] = make_uint4(0x77777777u, 0x77777777u, 0x77777777u, 0x77777777u);
            am[i] = 0.f;
            if (row0 + row < op.rows) {
                const int64_t r = row0 + row;
                v[i] = *reinterpret_cast<const uint4*>(base + r * (op.ld >> 1) + (k0 >> 1) + half * 16);
                am[i] = op.absmax[r * (op.ld >> 6) + (k0 >> 6)];
            }
        }
    }
    __device__ __forceinline__ void store(char* tile, const float* lut, int tid) {
#pragma unroll
        for (int i = 0; i < NU; ++i) {
            const int u = tid + 256 * i, row = u >> 1, half = u & 1;
            const uint32_t* w = reinterpret_cast<const uint32_t*>(&v[i]);
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                float f[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    f[e] = lut[nib(w[d], e)] * am[i];
                    if (kleft < BK && half * 32 + d * 8 + e >= kleft) f[e] = 0.f;
                }
                *reinterpret_cast<uint4*>(tile + lds_off(row, half * 4 + d)) =
                    make_uint4(pack_bf16(f[0], f[1]), pack_bf16(f[2], f[3]), pack_bf16(f[4], f[5]),
                               pack_bf16(f[6], f[7]));
            }
        }
    }
};

// NF4, K x rows, rows contiguous: a patch of KP k-values x 8 rows (one 4-byte group of codes
// per k); every k has its own absmax (blocks run along the row index).
template <int BR>
struct Stager<RC_NF4, BR> {
    static constexpr int KP = BR / 32;
    uint32_t c[KP];
    float am[KP];
    __device__ __forceinline__ void load(const Operand& op, int row0, int k0, int tid) {
        const int rg = tid % (BR / 8), kg = tid / (BR / 8);
        const uint8_t* base = reinterpret_cast<const uint8_t*>(op.ptr);
        const int r = row0 + rg * 8;
#pragma unroll
        for (int j = 0; j < KP; ++j) {
            const int k = k0 + kg * KP + j;
            c[j] = 0x77777777u;
            am[j] = 0.f;
            if (k < op.K && r < op.rows) {
                c[j] = *reinterpret_cast<const uint32_t*>(base + (int64_t)k * (op.ld >> 1) + (r >> 1));
                am[j] = op.absmax[(int64_t)k * (op.ld >> 6) + (r >> 6)];
            }
        }
    }
    __device__ __forceinline__ void store(char* tile, const float* lut, int tid) {
        const int rg = tid % (BR / 8), kg = tid / (BR / 8);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            uint32_t o[KP / 2];
#pragma unroll
            for (int d = 0; d < KP / 2; ++d)
                o[d] = pack_bf16(lut[nib(c[2 * d], i)] * am[2 * d], lut[nib(c[2 * d + 1], i)] * am[2 * d + 1]);
            const int row = rg * 8 + i;
            if constexpr (KP == 8) {
                *reinterpret_cast<uint4*>(tile + lds_off(row, kg)) = make_uint4(o[0], o[1], o[2], o[3]);
            } else {
                *reinterpret_cast<uint2*>(tile + lds_off(row, kg >> 1) + (kg & 1) * 8) = make_uint2(o[0], o[1]);
            }
        }
    }
};

template <int BR>
struct Stager<OP_NONE, BR> {
    __device__ __forceinline__ void load(const Operand&, int, int, int) {}
    __device__ __forceinline__ void store(char*, const float*, int) {}
};

// ---------------------------------------------------------------------------------------
// the kernel
// ---------------------------------------------------------------------------------------
template <int BM, int BN, int AK, int BK0, int BK1, int EPI>
__global__ __launch_bounds__(256) void loqt_gemm_kernel(const GemmParams p) {
    constexpr int TM = BM / 64, TN = BN / 64;  // 32x32 tiles per wave
    constexpr int STAGE = (BM + BN) * ROW_BYTES;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    float* lut = reinterpret_cast<float*>(smem + 2 * STAGE);

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;

    if (tid < 16) lut[tid] = kNf4Levels[tid];

    // tile coordinates: consecutive work-groups walk down M inside a band of N tiles
    const int tiles_m = (p.M + BM - 1) / BM;
    const int tm = blockIdx.x % tiles_m, tn = blockIdx.x / tiles_m;
    const int m0 = tm * BM, n0 = tn * BN;

    const int nkt0 = (p.A[0].K + BK - 1) / BK;
    const int nkt1 = (BK1 == OP_NONE) ? 0 : (p.A[1].K + BK - 1) / BK;
    int kt_begin = 0, kt_end = nkt0 + nkt1;
    if (EPI == EPI_F32_SPLITK) {
        const int per = (kt_end + p.splits - 1) / p.splits;
        kt_begin = blockIdx.y * per;
        kt_end = min(kt_end, kt_begin + per);
    }

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    Stager<AK, BM> sa;
    Stager<BK0, BN> sb0;
    Stager<BK1, BN> sb1;

    auto load_tile = [&](int kt) {
        if (BK1 != OP_NONE && kt >= nkt0) {
            const int k0 = (kt - nkt0) * BK;
            sa.load(p.A[1], m0, k0, tid);
            sb1.load(p.B[1], n0, k0, tid);
        } else {
            const int k0 = kt * BK;
            sa.load(p.A[0], m0, k0, tid);
            sb0.load(p.B[0], n0, k0, tid);
        }
    };
    auto store_tile = [&](int kt, char* stage) {
        sa.store(stage, lut, tid);
        if (BK1 != OP_NONE && kt >= nkt0) sb1.store(stage + BM * ROW_BYTES, lut, tid);
        else sb0.store(stage + BM * ROW_BYTES, lut, tid);
    };

    // per-lane fragment offsets: row (lane & 31), 16-byte chunk 2*ks + (lane >> 5)
    const int frow = lane & 31;
    const int fsw = (lane >> 5) ^ swz(frow);
    const int a_off = (wm * (BM / 2) + frow) * ROW_BYTES;
    const int b_off = BM * ROW_BYTES + (wn * (BN / 2) + frow) * ROW_BYTES;

    __syncthreads();  // lut visible
    if (kt_begin < kt_end) {
        load_tile(kt_begin);
        store_tile(kt_begin, smem);
    }
    __syncthreads();

    for (int kt = kt_begin; kt < kt_end; ++kt) {
        char* cur = smem + ((kt - kt_begin) & 1) * STAGE;
        char* nxt = smem + (((kt - kt_begin) & 1) ^ 1) * STAGE;
        const bool more = kt + 1 < kt_end;
        if (more) load_tile(kt + 1);

#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            const int coff = ((2 * ks) ^ fsw) << 4;
            bf16x8 af[TM], bfr[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i)
                af[i] = *reinterpret_cast<const bf16x8*>(cur + a_off + i * 32 * ROW_BYTES + coff);
#pragma unroll
            for (int j = 0; j < TN; ++j)
                bfr[j] = *reinterpret_cast<const bf16x8*>(cur + b_off + j * 32 * ROW_BYTES + coff);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
        }

        if (more) store_tile(kt + 1, nxt);
        __syncthreads();
    }

    // ------------------------------------------------------------------ epilogues
    // accumulator layout of a 32x32 tile: lane holds column (lane & 31); register 4*i + j
    // is row 8*i + 4*(lane >> 5) + j.
    const int h = lane >> 5;
    if (EPI == EPI_BF16 || EPI == EPI_F32_SPLITK) {
#pragma unroll
        for (int ti = 0; ti < TM; ++ti)
#pragma unroll
            for (int tj = 0; tj < TN; ++tj) {
                const int n = n0 + wn * (BN / 2) + tj * 32 + frow;
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int m = m0 + wm * (BM / 2) + ti * 32 + 8 * (e >> 2) + 4 * h + (e & 3);
                    if (m < p.M && n < p.N) {
                        const float val = p.alpha * acc[ti][tj][e];
                        if (EPI == EPI_BF16) {
                            reinterpret_cast<uint16_t*>(p.C)[(int64_t)m * p.ldc + n] =
                                (uint16_t)(pack_bf16(val, 0.f) & 0xffffu);
                        } else {
                            reinterpret_cast<float*>(p.C)[((int64_t)blockIdx.y * p.M + m) * p.N + n] = val;
                        }
                    }
                }
            }
    } else {
        // merge: rows of the tile run along `in` (the block direction of W), columns are
        // rows of W.  A 64-block of W row n lives in two vertically adjacent 32x32 tiles of
        // one wave: 32 values in this lane, 32 in lane ^ 32.
        Nf4EncTables* enc = reinterpret_cast<Nf4EncTables*>(smem);  // the stages are free now
        if (tid < 64) nf4_enc_tables_fill(enc, tid);
        __syncthreads();
        const int64_t ldb = p.w_ld >> 1, lda = p.w_ld >> 6;
#pragma unroll
        for (int tj = 0; tj < TN; ++tj) {
            const int n = n0 + wn * (BN / 2) + tj * 32 + frow;
            const bool nvalid = n < p.N;
#pragma unroll
            for (int b = 0; b < TM / 2; ++b) {
                const int mb = m0 + wm * (BM / 2) + b * 64;  // first `in` index of the block
                const bool live = nvalid && mb < p.w_ld;
                float am_old = 0.f;
                if (live) am_old = p.w_absmax[n * lda + (mb >> 6)];
                uint32_t cw[8];
                float v[32];
#pragma unroll
                for (int q = 0; q < 8; ++q) {  // q = 4*tt + i: tile tt of the pair, row group i
                    const int mq = mb + (q >> 2) * 32 + 8 * (q & 3) + 4 * h;
                    cw[q] = 0x7777u;
                    if (live) cw[q] = *reinterpret_cast<const uint16_t*>(p.w_codes + n * ldb + (mq >> 1));
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        float val = __builtin_fmaf(p.alpha, acc[2 * b + (q >> 2)][tj][4 * (q & 3) + j],
                                                   am_old * lut[nib(cw[q], j)]);
                        if (mq + j >= p.w_cols) val = 0.f;
                        v[4 * q + j] = val;
                    }
                }
                float amax = 0.f;
#pragma unroll
                for (int e = 0; e < 32; ++e) amax = fmaxf(amax, fabsf(v[e]));
                amax = fmaxf(amax, __shfl_xor(amax, 32));
                Nf4BlockEncoder be;
                be.set(amax);
#pragma unroll
                for (int q = 0; q < 8; ++q) {
                    const int mq = mb + (q >> 2) * 32 + 8 * (q & 3) + 4 * h;
                    // zeros (an all-zero block, columns past the end) encode to 7 by themselves
                    const uint32_t word = nf4_pack4(be.encode(enc, v[4 * q + 0]), be.encode(enc, v[4 * q + 1]),
                                                    be.encode(enc, v[4 * q + 2]), be.encode(enc, v[4 * q + 3]));
                    if (live) *reinterpret_cast<uint16_t*>(p.out_codes + n * ldb + (mq >> 1)) = (uint16_t)word;
                }
                if (live && h == 0) p.out_absmax[n * lda + (mb >> 6)] = amax;
            }
        }
    }
}

// dB = (accumulate ? dB : 0) + sum over splits of the fp32 partials, then to the output dtype
__global__ __launch_bounds__(256) void reduce_db_kernel(const float* __restrict__ partials, int splits,
                                                        int64_t M, int N, int64_t ldp, void* __restrict__ dB,
                                                        int dB_bf16, int64_t ld_dB, int accumulate) {
    const int64_t total = M * N;
    for (int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x; idx < total;
         idx += (int64_t)gridDim.x * 256) {
        const int64_t m = idx / N;
        const int n = (int)(idx - m * N);
        float s = 0.f;
        for (int k = 0; k < splits; ++k) s += partials[((int64_t)k * M + m) * ldp + n];
        if (dB_bf16) {
            uint16_t* d = reinterpret_cast<uint16_t*>(dB) + m * ld_dB + n;
            if (accumulate) s += __uint_as_float((uint32_t)(*d) << 16);
            *d = (uint16_t)(pack_bf16(s, 0.f) & 0xffffu);
        } else {
            float* d = reinterpret_cast<float*>(dB) + m * ld_dB + n;
            if (accumulate) s += *d;
            *d = s;
        }
    }
}

// The same sum four columns per thread (16-byte loads and stores); N, ldp and ld_dB multiples of 4, pointers
// aligned to match.  The order of the additions per element is the same as above.
__global__ __launch_bounds__(256) void reduce_db4_kernel(const float* __restrict__ partials, int splits,
                                                         int64_t M, int N4, int64_t ldp, void* __restrict__ dB,
                                                         int dB_bf16, int64_t ld_dB, int accumulate) {
    const int64_t total = M * N4;
    for (int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x; idx < total;
         idx += (int64_t)gridDim.x * 256) {
        const int64_t m = idx / N4;
        const int n = (int)(idx - m * N4) * 4;
        float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
        for (int k = 0; k < splits; ++k) {
            const float4 v = *reinterpret_cast<const float4*>(partials + ((int64_t)k * M + m) * ldp + n);
            s.x += v.x, s.y += v.y, s.z += v.z, s.w += v.w;
        }
        if (dB_bf16) {
            uint2* d = reinterpret_cast<uint2*>(reinterpret_cast<uint16_t*>(dB) + m * ld_dB + n);
            if (accumulate) {
                const uint2 o = *d;
                s.x += __uint_as_float(o.x << 16), s.y += __uint_as_float(o.x & 0xffff0000u);
                s.z += __uint_as_float(o.y << 16), s.w += __uint_as_float(o.y & 0xffff0000u);
            }
            *d = make_uint2(pack_bf16(s.x, s.y), pack_bf16(s.z, s.w));
        } else {
            float4* d = reinterpret_cast<float4*>(reinterpret_cast<float*>(dB) + m * ld_dB + n);
            if (accumulate) {
                const float4 o = *d;
                s.x += o.x, s.y += o.y, s.z += o.z, s.w += o.w;
            }
            *d = s;
        }
    }
}

// the kernel's LDS size has to be raised above the default once per process (first launch, or loqt_prepare)
template <int BM, int BN, int AK, int BK0, int BK1, int EPI>
hipError_t ensure_attr_one() {
    constexpr int smem = 2 * (BM + BN) * ROW_BYTES + 64;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(loqt_gemm_kernel<BM, BN, AK, BK0, BK1, EPI>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, smem);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    return hipSuccess;
}

template <int BM, int BN, int AK, int BK0, int BK1, int EPI>
hipError_t launch_one(const GemmParams& p, hipStream_t st) {
    auto kern = loqt_gemm_kernel<BM, BN, AK, BK0, BK1, EPI>;
    constexpr int smem = 2 * (BM + BN) * ROW_BYTES + 64;
    hipError_t e0 = ensure_attr_one<BM, BN, AK, BK0, BK1, EPI>();
    if (e0 != hipSuccess) return e0;
    const int tiles = ((p.M + BM - 1) / BM) * ((p.N + BN - 1) / BN);
    dim3 grid(tiles, EPI == EPI_F32_SPLITK ? p.splits : 1);
    hipLaunchKernelGGL(kern, grid, dim3(256), smem, st, p);
    return hipGetLastError();
}

// Big tiles when they still fill the 256 compute units, small tiles otherwise.
bool use_big_tiles(int M, int N) {
    const int64_t t = (int64_t)((M + 255) / 256) * ((N + 255) / 256);
    return t >= 192;
}

}  // namespace

hipError_t prepare_fused_kernels() {
    hipError_t e;
#define LOQT_PREP(...)                                 \
    if ((e = ensure_attr_one<__VA_ARGS__>()) != hipSuccess) return e
    LOQT_PREP(128, 128, KC_BF16, KC_BF16, OP_NONE, EPI_BF16);
    LOQT_PREP(256, 256, KC_BF16, KC_NF4, KC_NF4, EPI_BF16);
    LOQT_PREP(128, 128, KC_BF16, KC_NF4, KC_NF4, EPI_BF16);
    LOQT_PREP(128, 128, KC_BF16, RC_NF4, OP_NONE, EPI_BF16);
    LOQT_PREP(256, 256, KC_BF16, RC_NF4, RC_BF16, EPI_BF16);
    LOQT_PREP(128, 128, KC_BF16, RC_NF4, RC_BF16, EPI_BF16);
    LOQT_PREP(128, 128, RC_BF16, RC_BF16, OP_NONE, EPI_F32_SPLITK);
    LOQT_PREP(128, 128, RC_BF16, KC_NF4, OP_NONE, EPI_MERGE);
#undef LOQT_PREP
    return hipSuccess;
}

int gemm_db_splits(int64_t T, int64_t r, int64_t in) {
    // enough work-groups for 256 compute units at two groups per unit, at least 512 deep
    const int64_t tiles = ((r + 127) / 128) * ((in + 127) / 128);
    int64_t s = (768 + tiles - 1) / tiles;
    const int64_t max_s = (T + 511) / 512;
    if (s > max_s) s = max_s;
    if (s < 1) s = 1;
    if (s > 32) s = 32;
    return (int)s;
}

hipError_t launch_gemm(GemmId id, const GemmParams& p, hipStream_t st) {
    const bool big = use_big_tiles(p.M, p.N);
    switch (id) {
        case GEMM_U: {
            TimedLaunch tl(SLOT_GEMM_U, st);
            return launch_one<128, 128, KC_BF16, KC_BF16, OP_NONE, EPI_BF16>(p, st);
        }
        case GEMM_Y: {
            TimedLaunch tl(SLOT_GEMM_Y, st);
            return big ? launch_one<256, 256, KC_BF16, KC_NF4, KC_NF4, EPI_BF16>(p, st)
                       : launch_one<128, 128, KC_BF16, KC_NF4, KC_NF4, EPI_BF16>(p, st);
        }
        case GEMM_Z: {
            TimedLaunch tl(SLOT_GEMM_Z, st);
            return launch_one<128, 128, KC_BF16, RC_NF4, OP_NONE, EPI_BF16>(p, st);
        }
        case GEMM_DX: {
            TimedLaunch tl(SLOT_GEMM_DX, st);
            return big ? launch_one<256, 256, KC_BF16, RC_NF4, RC_BF16, EPI_BF16>(p, st)
                       : launch_one<128, 128, KC_BF16, RC_NF4, RC_BF16, EPI_BF16>(p, st);
        }
        case GEMM_DB: {
            TimedLaunch tl(SLOT_GEMM_DB, st);
            return launch_one<128, 128, RC_BF16, RC_BF16, OP_NONE, EPI_F32_SPLITK>(p, st);
        }
        case GEMM_MERGE: {
            TimedLaunch tl(SLOT_MERGE, st);
            return launch_one<128, 128, RC_BF16, KC_NF4, OP_NONE, EPI_MERGE>(p, st);
        }
    }
    return hipErrorInvalidValue;
}

hipError_t launch_reduce_db(const float* partials, int splits, int64_t M, int64_t N, int64_t ldp, void* dB,
                            int dB_dtype, int64_t ld_dB, int accumulate, hipStream_t st, bool timed) {
    // (untimed when it runs inside another timed launch)
    TimedLaunch tl(timed ? SLOT_REDUCE_DB : -1, st);
    const bool bf16 = dB_dtype == LOQT_BF16;
    if (N % 4 == 0 && ldp % 4 == 0 && ld_dB % 4 == 0 && (reinterpret_cast<uintptr_t>(partials) & 15) == 0 &&
        (reinterpret_cast<uintptr_t>(dB) & (bf16 ? 7 : 15)) == 0) {
        int64_t blocks4 = (M * (N / 4) + 255) / 256;
        if (blocks4 > 256 * 16) blocks4 = 256 * 16;
        hipLaunchKernelGGL(reduce_db4_kernel, dim3((int)blocks4), dim3(256), 0, st, partials, splits, M, (int)(N / 4),
                           ldp, dB, bf16 ? 1 : 0, ld_dB, accumulate);
        return hipGetLastError();
    }
    int64_t blocks = (M * N + 255) / 256;
    if (blocks > 256 * 32) blocks = 256 * 32;
    hipLaunchKernelGGL(reduce_db_kernel, dim3((int)blocks), dim3(256), 0, st, partials, splits, M, (int)N,
                       ldp, dB, dB_dtype == LOQT_BF16 ? 1 : 0, ld_dB, accumulate);
    return hipGetLastError();
}

}  // namespace loqt
