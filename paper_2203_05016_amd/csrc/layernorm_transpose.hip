// LayerNorm-side transposition for the Shfl-BW kernels on gfx950 (CDNA4).
//
// The sparse kernels read and write their dense matrices row-wise, so they
// want activations batch-innermost: X[K features][N tokens].  A LayerNorm
// produces them feature-innermost, x[N][K]; Section 4.3 (discussion of the
// activation layout) folds the transposition into that LayerNorm.  This
// kernel is that step: per token it normalises over the K features (mean,
// biased variance, eps, then gamma and beta), or just copies when asked to,
// and writes the result transposed.
//
// A workgroup (8 wavefronts) owns 64 tokens and a range of the features.
// Phase A: each wavefront takes 8 tokens and sums x - p and (x - p)^2 over
// all K features in one sweep, p being the token's first feature (a pivot
// near the data keeps the fp32 variance free of cancellation); 16 row loads
// are in flight per lane.  Workgroups that share tokens repeat this sweep;
// all but the first read it from the L2.  Phase B: 64-feature blocks of the
// workgroup's range are loaded up to four blocks ahead (16 bytes per lane),
// normalised in fp32, written transposed into an LDS tile and stored as 64
// rows of 128 bytes.  It is bound by HBM: 2*N*K bytes read and 2*N*K written.
//
// When a block of 64 (or 32) tokens with all its features fits the LDS, a
// second kernel keeps it there instead: every activation is read from HBM
// once, the statistics come from the same loads, and the transposed rows are
// gathered from LDS columns (row pitch chosen so that the 8 token rows a
// lane reads fall into different banks).
#include <hip/hip_runtime.h>

#include <cstdint>
#include <string>

#include "shflbw.h"
#include "shflbw_internal.h"

namespace shflbw {
namespace {

typedef unsigned short ln_ushort8 __attribute__((ext_vector_type(8)));

constexpr int LN_TOK = 64;       // tokens per workgroup
constexpr int LN_WAVES = 8;
constexpr int LN_FB = 64;        // features per block in phase B
constexpr int LN_PITCH = LN_TOK + 8;   // LDS row pitch of the transposed tile (16-bit units)
constexpr int LN_AHEAD = 4;      // feature blocks loaded ahead

struct LnArgs {
    const uint16_t* x;      // [N][K], leading dimension ldx
    const uint16_t* gamma;  // [K] or nullptr
    const uint16_t* beta;   // [K] or nullptr
    uint16_t* out;          // [K][N], leading dimension ldo
    long ldx, ldo, N;
    int K;
    float eps;
    int normalize;
    int blocks_per_wg;      // 64-feature blocks one workgroup transposes (grid.y covers K)
};

template <bool BF>
__device__ __forceinline__ float ln_widen(uint16_t v)
{
    if constexpr (BF) return __builtin_bit_cast(float, (unsigned)v << 16);
    else return (float)__builtin_bit_cast(_Float16, v);
}
template <bool BF>
__device__ __forceinline__ uint16_t ln_narrow(float f)
{
    if constexpr (BF) return __builtin_bit_cast(uint16_t, (__bf16)f);
    else return __builtin_bit_cast(uint16_t, (_Float16)f);
}

template <bool BF>
__global__ __launch_bounds__(64 * LN_WAVES) void layernorm_transpose_kernel(LnArgs a)
{
    __shared__ float stat_mean[LN_TOK], stat_rstd[LN_TOK];
    __shared__ __attribute__((aligned(16))) uint16_t tile[LN_FB * LN_PITCH];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const long n0 = (long)blockIdx.x * LN_TOK;
    const int K = a.K;

    // phase B's first blocks are requested now, so that they travel while phase A runs
    // load: thread -> token tid/8, 8 features at (tid%8)*8 of the block;
    // store: thread -> feature row tid/8 of the block, 8 tokens at (tid%8)*8
    const int ltok = tid >> 3, lchunk = tid & 7;
    const int nblocks_all = (K + LN_FB - 1) / LN_FB;
    const int bbeg = blockIdx.y * a.blocks_per_wg;
    int bend = bbeg + a.blocks_per_wg;
    bend = bend < nblocks_all ? bend : nblocks_all;
    const long ntok = n0 + ltok;
    auto load_block = [&](int b, ln_ushort8& v) __attribute__((always_inline)) {
        const int k = b * LN_FB + lchunk * 8;
        v = ln_ushort8{0, 0, 0, 0, 0, 0, 0, 0};
        if (b < bend && k < K && ntok < a.N) v = *reinterpret_cast<const ln_ushort8*>(a.x + ntok * a.ldx + k);
    };
    ln_ushort8 ring[LN_AHEAD];
#pragma unroll
    for (int u = 0; u < LN_AHEAD; ++u) load_block(bbeg + u, ring[u]);

    // ---------------------------------------------------------------- phase A
    if (a.normalize) {
        constexpr int TPW = LN_TOK / LN_WAVES;   // tokens per wavefront
        float s1[TPW], s2[TPW], pivot[TPW];
#pragma unroll
        for (int t = 0; t < TPW; ++t) { s1[t] = 0.f; s2[t] = 0.f; pivot[t] = 0.f; }
        for (int kc0 = 0; kc0 < K; kc0 += 2 * 64 * 8) {
            ln_ushort8 v[TPW][2];
#pragma unroll
            for (int t = 0; t < TPW; ++t) {
                const long n = n0 + wave * TPW + t;
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const int kc = kc0 + h * 512 + lane * 8;
                    v[t][h] = ln_ushort8{0, 0, 0, 0, 0, 0, 0, 0};
                    if (n < a.N && kc < K) v[t][h] = *reinterpret_cast<const ln_ushort8*>(a.x + n * a.ldx + kc);
                }
            }
            if (kc0 == 0) {
                // the token's first feature, which lane 0 has just loaded
#pragma unroll
                for (int t = 0; t < TPW; ++t)
                    pivot[t] = __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(
                        __builtin_bit_cast(int, ln_widen<BF>(v[t][0][0]))));
            }
#pragma unroll
            for (int t = 0; t < TPW; ++t) {
                const long n = n0 + wave * TPW + t;
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const int kc = kc0 + h * 512 + lane * 8;
                    if (n < a.N && kc < K) {
#pragma unroll
                        for (int e = 0; e < 8; ++e) {
                            const float d = ln_widen<BF>(v[t][h][e]) - pivot[t];
                            s1[t] += d;
                            s2[t] += d * d;
                        }
                    }
                }
            }
        }
#pragma unroll
        for (int t = 0; t < TPW; ++t) {
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) {
                s1[t] += __shfl_xor(s1[t], off, 64);
                s2[t] += __shfl_xor(s2[t], off, 64);
            }
        }
        if (lane == 0) {
#pragma unroll
            for (int t = 0; t < TPW; ++t) {
                const float m = s1[t] / (float)K;              // mean of x - pivot
                float var = s2[t] / (float)K - m * m;
                var = var > 0.f ? var : 0.f;
                stat_mean[wave * TPW + t] = pivot[t] + m;
                stat_rstd[wave * TPW + t] = 1.0f / __builtin_sqrtf(var + a.eps);
            }
        }
    } else if (tid < LN_TOK) {
        stat_mean[tid] = 0.f;
        stat_rstd[tid] = 1.f;
    }
    __syncthreads();

    // ---------------------------------------------------------------- phase B
    const float mean = stat_mean[ltok], rstd = stat_rstd[ltok];

    for (int b0 = bbeg; b0 < bend; b0 += LN_AHEAD) {
#pragma unroll
        for (int u = 0; u < LN_AHEAD; ++u) {
            const int b = b0 + u;
            if (b < bend) {   // uniform
                const int k = b * LN_FB + lchunk * 8;
                float g[8], bt[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) { g[e] = 1.f; bt[e] = 0.f; }
                if (a.normalize && k < K) {
                    if (a.gamma) {
                        const ln_ushort8 gv = *reinterpret_cast<const ln_ushort8*>(a.gamma + k);
#pragma unroll
                        for (int e = 0; e < 8; ++e) g[e] = ln_widen<BF>(gv[e]);
                    }
                    if (a.beta) {
                        const ln_ushort8 bv = *reinterpret_cast<const ln_ushort8*>(a.beta + k);
#pragma unroll
                        for (int e = 0; e < 8; ++e) bt[e] = ln_widen<BF>(bv[e]);
                    }
                }
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    uint16_t o = ring[u][e];
                    if (a.normalize)
                        o = ln_narrow<BF>((ln_widen<BF>(o) - mean) * rstd * g[e] + bt[e]);
                    tile[(lchunk * 8 + e) * LN_PITCH + ltok] = o;
                }
                load_block(b + LN_AHEAD, ring[u]);
                __syncthreads();
                {
                    const int kr = ltok;   // the same split of the thread index, now feature row / token chunk
                    const long kk = (long)b * LN_FB + kr, n = n0 + lchunk * 8;
                    if (kk < K && n < a.N)
                        *reinterpret_cast<ln_ushort8*>(a.out + kk * a.ldo + n) =
                            *reinterpret_cast<const ln_ushort8*>(tile + kr * LN_PITCH + lchunk * 8);
                }
                __syncthreads();
            }
        }
    }
}

// ---------------------------------------------------------------- LDS-resident variant
// TOK tokens x K features (pitch P halves, P/2 = 1 mod 64) + statistics + gamma/beta in fp32.
template <bool BF, int TOK>
__global__ __launch_bounds__(64 * LN_WAVES) void layernorm_transpose_resident_kernel(LnArgs a, int P)
{
    extern __shared__ __attribute__((aligned(16))) char ln_smem[];
    uint16_t* xs = reinterpret_cast<uint16_t*>(ln_smem);                       // [TOK][P]
    float* st_mean = reinterpret_cast<float*>(ln_smem + (size_t)TOK * P * 2);   // [TOK]
    float* st_rstd = st_mean + TOK;                                             // [TOK]
    float* gam = st_rstd + TOK;                                                 // [K]
    float* bet = gam + a.K;                                                     // [K]
    constexpr int TPW = TOK / LN_WAVES;   // tokens per wavefront
    constexpr int CH = TOK / 8;           // 16-byte token chunks per output row
    constexpr int FW = 64 / CH;           // features one wavefront stores per pass

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const long n0 = (long)blockIdx.x * TOK;
    const int K = a.K;

    for (int k = tid; k < K; k += 64 * LN_WAVES) {
        gam[k] = (a.normalize && a.gamma) ? ln_widen<BF>(a.gamma[k]) : 1.f;
        bet[k] = (a.normalize && a.beta) ? ln_widen<BF>(a.beta[k]) : 0.f;
    }

    // ---- load the block once: LDS copy and, from the same registers, the statistics
    float s1[TPW], s2[TPW], pivot[TPW];
#pragma unroll
    for (int t = 0; t < TPW; ++t) { s1[t] = 0.f; s2[t] = 0.f; pivot[t] = 0.f; }
    for (int kc0 = 0; kc0 < K; kc0 += 2 * 64 * 8) {
        ln_ushort8 v[TPW][2];
#pragma unroll
        for (int t = 0; t < TPW; ++t) {
            const long n = n0 + wave * TPW + t;
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int kc = kc0 + h * 512 + lane * 8;
                v[t][h] = ln_ushort8{0, 0, 0, 0, 0, 0, 0, 0};
                if (n < a.N && kc < K) v[t][h] = *reinterpret_cast<const ln_ushort8*>(a.x + n * a.ldx + kc);
            }
        }
        if (kc0 == 0) {
#pragma unroll
            for (int t = 0; t < TPW; ++t)
                pivot[t] = __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(
                    __builtin_bit_cast(int, ln_widen<BF>(v[t][0][0]))));
        }
#pragma unroll
        for (int t = 0; t < TPW; ++t) {
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int kc = kc0 + h * 512 + lane * 8;
                if (kc < K) {
                    unsigned* dst = reinterpret_cast<unsigned*>(xs + (wave * TPW + t) * P + kc);   // 4-byte aligned
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        dst[e] = (unsigned)v[t][h][2 * e] | ((unsigned)v[t][h][2 * e + 1] << 16);
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const float d = ln_widen<BF>(v[t][h][e]) - pivot[t];
                        s1[t] += d;
                        s2[t] += d * d;
                    }
                }
            }
        }
    }
    if (a.normalize) {
#pragma unroll
        for (int t = 0; t < TPW; ++t) {
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) {
                s1[t] += __shfl_xor(s1[t], off, 64);
                s2[t] += __shfl_xor(s2[t], off, 64);
            }
        }
    }
    if (lane == 0) {
#pragma unroll
        for (int t = 0; t < TPW; ++t) {
            const float m = s1[t] / (float)K;
            float var = s2[t] / (float)K - m * m;
            var = var > 0.f ? var : 0.f;
            st_mean[wave * TPW + t] = a.normalize ? pivot[t] + m : 0.f;
            st_rstd[wave * TPW + t] = a.normalize ? 1.0f / __builtin_sqrtf(var + a.eps) : 1.f;
        }
    }
    __syncthreads();

    // ---- transposed rows: a wavefront stores FW feature rows x TOK tokens per pass;
    // lane -> feature lane/CH of the pass, tokens (lane%CH)*8 .. +7
    const int kk = lane / CH, tchunk = lane % CH;
    float mean[8], rstd[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) { mean[e] = st_mean[tchunk * 8 + e]; rstd[e] = st_rstd[tchunk * 8 + e]; }
    const long n = n0 + tchunk * 8;
    for (int kb = wave * FW; kb < K; kb += LN_WAVES * FW) {
        const int k = kb + kk;
        if (k < K && n < a.N) {
            const float g = gam[k], b = bet[k];
            ln_ushort8 o;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const uint16_t raw = xs[(tchunk * 8 + e) * P + k];
                o[e] = a.normalize ? ln_narrow<BF>((ln_widen<BF>(raw) - mean[e]) * rstd[e] * g + b) : raw;
            }
            __builtin_nontemporal_store(o, reinterpret_cast<ln_ushort8*>(a.out + (long)k * a.ldo + n));
        }
    }
}

}  // namespace
}  // namespace shflbw

extern "C" int shflbw_layernorm_transpose(const void* x, int64_t ldx, const void* gamma,
                                          const void* beta, float eps, int normalize, void* out,
                                          int64_t ldo, int64_t N, int K, shflbw_dtype dtype,
                                          void* stream)
{
    using namespace shflbw;
    if (dtype != SHFLBW_F16 && dtype != SHFLBW_BF16)
        return fail(SHFLBW_ERR_BAD_DTYPE, "dtype must be SHFLBW_F16 or SHFLBW_BF16");
    if (N < 0 || K <= 0) return fail(SHFLBW_ERR_BAD_SHAPE, "N < 0 or K <= 0");
    if (N == 0) return SHFLBW_OK;
    if (!x || !out) return fail(SHFLBW_ERR_NULL_ARG, "x and out must not be NULL");
    if (ldx < K || ldo < N) return fail(SHFLBW_ERR_BAD_SHAPE, "leading dimension too small");
    if (K % 8 || N % 8 || ldx % 8 || ldo % 8 || reinterpret_cast<uintptr_t>(x) % 16 ||
        reinterpret_cast<uintptr_t>(out) % 16 || (gamma && reinterpret_cast<uintptr_t>(gamma) % 16) ||
        (beta && reinterpret_cast<uintptr_t>(beta) % 16))
        return fail(SHFLBW_ERR_BAD_SHAPE,
                    "K, N and the leading dimensions must be multiples of 8 and all bases 16-byte aligned");
    if (normalize && !(eps >= 0.f)) return fail(SHFLBW_ERR_BAD_SHAPE, "eps must be >= 0");
    const int64_t wgs = (N + LN_TOK - 1) / LN_TOK;
    if (wgs > 0x7fffffffLL) return fail(SHFLBW_ERR_BAD_SHAPE, "grid too large");
    LnArgs a;
    a.x = static_cast<const uint16_t*>(x);
    a.gamma = static_cast<const uint16_t*>(gamma);
    a.beta = static_cast<const uint16_t*>(beta);
    a.out = static_cast<uint16_t*>(out);
    a.ldx = (long)ldx; a.ldo = (long)ldo; a.N = (long)N; a.K = K; a.eps = eps;
    a.normalize = normalize ? 1 : 0;
    hipStream_t st = static_cast<hipStream_t>(stream);
    // LDS-resident variant when a block of tokens with all its features fits: 64 tokens per
    // workgroup, or 32 when that fills the chip better or is all that fits
    auto resident_bytes = [&](int tok, int& pitch) {
        int pad = 2;
        while (((K + pad) / 2) % 64 != 1) pad += 2;     // 8 rows apart -> 8 banks apart
        pitch = K + pad;
        return (size_t)tok * pitch * 2 + 2 * (size_t)tok * 4 + 2 * (size_t)K * 4;
    };
    const size_t lds_cap = 160 * 1024 - 256;
    int pitch = 0;
    int tok = 0;
    if (resident_bytes(64, pitch) <= lds_cap && (N + 63) / 64 >= 256) tok = 64;
    else if (resident_bytes(32, pitch) <= lds_cap) tok = 32;
    if (tok) {
        const size_t bytes = resident_bytes(tok, pitch);
        const int64_t rwgs = (N + tok - 1) / tok;
        if (rwgs > 0x7fffffffLL) return fail(SHFLBW_ERR_BAD_SHAPE, "grid too large");
        const void* fn = dtype == SHFLBW_BF16
            ? (tok == 64 ? (const void*)&layernorm_transpose_resident_kernel<true, 64>
                         : (const void*)&layernorm_transpose_resident_kernel<true, 32>)
            : (tok == 64 ? (const void*)&layernorm_transpose_resident_kernel<false, 64>
                         : (const void*)&layernorm_transpose_resident_kernel<false, 32>);
        // the attribute is raised once per kernel and device
        static thread_local int raised_on[4] = {-1, -1, -1, -1};
        const int which = (dtype == SHFLBW_BF16 ? 2 : 0) + (tok == 64 ? 1 : 0);
        int dev = 0;
        hipError_t ea = hipGetDevice(&dev);
        if (ea != hipSuccess) return fail(SHFLBW_ERR_HIP, std::string("hipGetDevice: ") + hipGetErrorString(ea));
        if (raised_on[which] != dev) {
            ea = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
            if (ea != hipSuccess) return fail(SHFLBW_ERR_HIP, std::string("hipFuncSetAttribute: ") + hipGetErrorString(ea));
            raised_on[which] = dev;
        }
        const dim3 grid((unsigned)rwgs), block(64 * LN_WAVES);
        if (dtype == SHFLBW_BF16) {
            if (tok == 64) hipLaunchKernelGGL((layernorm_transpose_resident_kernel<true, 64>), grid, block, bytes, st, a, pitch);
            else hipLaunchKernelGGL((layernorm_transpose_resident_kernel<true, 32>), grid, block, bytes, st, a, pitch);
        } else {
            if (tok == 64) hipLaunchKernelGGL((layernorm_transpose_resident_kernel<false, 64>), grid, block, bytes, st, a, pitch);
            else hipLaunchKernelGGL((layernorm_transpose_resident_kernel<false, 32>), grid, block, bytes, st, a, pitch);
        }
        hipError_t el = hipGetLastError();
        if (el != hipSuccess) return fail(SHFLBW_ERR_HIP, std::string("kernel launch: ") + hipGetErrorString(el));
        return SHFLBW_OK;
    }
    // split the features over grid.y until there are about two workgroups per CU
    const int nblocks = (K + LN_FB - 1) / LN_FB;
    int split = 1;
    while (wgs * split < 512 && split * 2 <= nblocks && split < 16) split *= 2;
    a.blocks_per_wg = (nblocks + split - 1) / split;
    const unsigned gy = (unsigned)((nblocks + a.blocks_per_wg - 1) / a.blocks_per_wg);
    if (dtype == SHFLBW_BF16)
        hipLaunchKernelGGL(layernorm_transpose_kernel<true>, dim3((unsigned)wgs, gy), dim3(64 * LN_WAVES), 0, st, a);
    else
        hipLaunchKernelGGL(layernorm_transpose_kernel<false>, dim3((unsigned)wgs, gy), dim3(64 * LN_WAVES), 0, st, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(SHFLBW_ERR_HIP, std::string("kernel launch: ") + hipGetErrorString(e));
    return SHFLBW_OK;
}
