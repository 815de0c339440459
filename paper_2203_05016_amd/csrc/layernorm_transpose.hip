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
#include <hip/hip_runtime.h>

#include <cstdint>
#include <string>

#include "shflbw.h"
#include "shflbw_internal.h"

namespace shflbw {
namespace {

typedef _Float16 ln_half8 __attribute__((ext_vector_type(8)));
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
    // split the features over grid.y until there are about two workgroups per CU
    const int nblocks = (K + LN_FB - 1) / LN_FB;
    int split = 1;
    while (wgs * split < 512 && split * 2 <= nblocks && split < 16) split *= 2;
    a.blocks_per_wg = (nblocks + split - 1) / split;
    const unsigned gy = (unsigned)((nblocks + a.blocks_per_wg - 1) / a.blocks_per_wg);
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (dtype == SHFLBW_BF16)
        hipLaunchKernelGGL(layernorm_transpose_kernel<true>, dim3((unsigned)wgs, gy), dim3(64 * LN_WAVES), 0, st, a);
    else
        hipLaunchKernelGGL(layernorm_transpose_kernel<false>, dim3((unsigned)wgs, gy), dim3(64 * LN_WAVES), 0, st, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(SHFLBW_ERR_HIP, std::string("kernel launch: ") + hipGetErrorString(e));
    return SHFLBW_OK;
}
