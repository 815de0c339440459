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
// When a block of 32 (or 64) tokens with all its features fits the LDS, a
// second kernel keeps it there instead: every activation is read from HBM
// once, the statistics come from the same loads (sixteen wavefronts, two or four
// tokens each),
// and the transposed rows are gathered from LDS columns, two neighbouring
// features per lane (row pitch chosen so that the 64 four-byte reads of a
// wavefront fall into 64 different banks).
#include <hip/hip_runtime.h>

#include <cstdint>
#include <string>
#include <type_traits>

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

template <bool BF, bool NORM>
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
    if (NORM) {
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
                if (NORM) {
                    float g[8], bt[8];
#pragma unroll
                    for (int e = 0; e < 8; ++e) { g[e] = 1.f; bt[e] = 0.f; }
                    if (k < K) {
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
                    for (int e = 0; e < 8; ++e)
                        tile[(lchunk * 8 + e) * LN_PITCH + ltok] =
                            ln_narrow<BF>((ln_widen<BF>(ring[u][e]) - mean) * rstd * g[e] + bt[e]);
                } else {
#pragma unroll
                    for (int e = 0; e < 8; ++e) tile[(lchunk * 8 + e) * LN_PITCH + ltok] = ring[u][e];
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
// TOK tokens x K features (pitch P halves) + statistics + gamma/beta in fp32.  A lane of
// the store phase takes two neighbouring features of 8 tokens: 8 four-byte LDS reads
// for two 16-byte stores.  The 64 lanes of a wavefront read, per token, 64/CH feature
// pairs for each of CH token chunks; with P/2 = 64/CH/8 (mod 8) the chunks' rows start
// 64/CH banks apart, so the 64 words fall into 64 different banks.
// lo = low half of w + c, hi = high half of w + c, in fp32.  For float16 the widening
// rides on the mixed-precision multiply-add (x * 1 + c, rounded once: the same bits as
// a conversion followed by an addition), which halves the instructions.
template <bool BF>
__device__ __forceinline__ void ln_add_pair(unsigned w, float c, float& lo, float& hi)
{
    if constexpr (BF) {
        lo = __builtin_bit_cast(float, w << 16) + c;
        hi = __builtin_bit_cast(float, w & 0xffff0000u) + c;
    } else {
        asm("v_fma_mix_f32 %0, %1, 1.0, %2 op_sel_hi:[1,0,0]" : "=v"(lo) : "v"(w), "v"(c));
        asm("v_fma_mix_f32 %0, %1, 1.0, %2 op_sel:[1,0,0] op_sel_hi:[1,0,0]" : "=v"(hi) : "v"(w), "v"(c));
    }
}

template <bool BF, int TOK, bool NORM>
__global__ __launch_bounds__(1024) void layernorm_transpose_resident_kernel(LnArgs a, int P)
{
    extern __shared__ __attribute__((aligned(16))) char ln_smem[];
    uint16_t* xs = reinterpret_cast<uint16_t*>(ln_smem);                       // [TOK][P]
    float* st_mean = reinterpret_cast<float*>(ln_smem + (size_t)TOK * P * 2);   // [TOK]
    float* st_rstd = st_mean + TOK;                                             // [TOK]
    float* gam = st_rstd + TOK;                                                 // [K]
    float* bet = gam + a.K;                                                     // [K]
    constexpr int WAVES = 16;
    constexpr int TPW = TOK / WAVES;     // tokens per wavefront: 2 or 4
    constexpr int CH = TOK / 8;           // 16-byte token chunks per output row
    constexpr int FP = 64 / CH;           // feature pairs one wavefront stores per pass
    constexpr bool WIDE = (TOK == 32);    // its pitch keeps every row 8-byte aligned

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const long n0 = (long)blockIdx.x * TOK;
    const int K = a.K;

    if (NORM) {
        for (int k = tid; k < K; k += 64 * WAVES) {
            gam[k] = a.gamma ? ln_widen<BF>(a.gamma[k]) : 1.f;
            bet[k] = a.beta ? ln_widen<BF>(a.beta[k]) : 0.f;
        }
    }

    // ---- load the block once: LDS copy and, from the same registers, the statistics
    float s1[TPW], s2[TPW], pivot[TPW];
#pragma unroll
    for (int t = 0; t < TPW; ++t) { s1[t] = 0.f; s2[t] = 0.f; pivot[t] = 0.f; }
    const bool all_tokens = n0 + TOK <= a.N;
    // one sweep of 1024 features; FULL = every token and feature of it exists
    auto sweep = [&](int kc0, auto full_tag) __attribute__((always_inline)) {
        constexpr bool FULL = decltype(full_tag)::value;
        ln_ushort8 v[TPW][2];
#pragma unroll
        for (int t = 0; t < TPW; ++t) {
            const long n = n0 + wave * TPW + t;
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int kc = kc0 + h * 512 + lane * 8;
                if (FULL) {
                    v[t][h] = *reinterpret_cast<const ln_ushort8*>(a.x + n * a.ldx + kc);
                } else {
                    v[t][h] = ln_ushort8{0, 0, 0, 0, 0, 0, 0, 0};
                    if (n < a.N && kc < K) v[t][h] = *reinterpret_cast<const ln_ushort8*>(a.x + n * a.ldx + kc);
                }
            }
        }
        if (NORM && kc0 == 0) {
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
                if (FULL || kc < K) {
                    unsigned w[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        w[e] = (unsigned)v[t][h][2 * e] | ((unsigned)v[t][h][2 * e + 1] << 16);
                    uint16_t* row = xs + (wave * TPW + t) * P + kc;
                    if (WIDE) {
                        uint2* dst = reinterpret_cast<uint2*>(row);
                        dst[0] = uint2{w[0], w[1]};
                        dst[1] = uint2{w[2], w[3]};
                    } else {
                        unsigned* dst = reinterpret_cast<unsigned*>(row);
#pragma unroll
                        for (int e = 0; e < 4; ++e) dst[e] = w[e];
                    }
                    if (NORM) {
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            float d0, d1;
                            ln_add_pair<BF>(w[e], -pivot[t], d0, d1);
                            s1[t] += d0;
                            s2[t] += d0 * d0;
                            s1[t] += d1;
                            s2[t] += d1 * d1;
                        }
                    }
                }
            }
        }
    };
    for (int kc0 = 0; kc0 < K; kc0 += 2 * 64 * 8) {
        if (all_tokens && kc0 + 2 * 64 * 8 <= K) sweep(kc0, std::true_type{});
        else sweep(kc0, std::false_type{});
    }
    if (NORM) {
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
                const float m = s1[t] / (float)K;
                float var = s2[t] / (float)K - m * m;
                var = var > 0.f ? var : 0.f;
                st_mean[wave * TPW + t] = pivot[t] + m;
                st_rstd[wave * TPW + t] = 1.0f / __builtin_sqrtf(var + a.eps);
            }
        }
    }
    __syncthreads();

    // ---- transposed rows: a wavefront stores 2*FP feature rows x TOK tokens per pass;
    // lane -> features 2*(lane/CH), +1 of the pass, tokens (lane%CH)*8 .. +7
    const int kk2 = lane / CH, tchunk = lane % CH;
    float mean[8], rstd[8];
    if (NORM) {
#pragma unroll
        for (int e = 0; e < 8; ++e) { mean[e] = st_mean[tchunk * 8 + e]; rstd[e] = st_rstd[tchunk * 8 + e]; }
    }
    const long n = n0 + tchunk * 8;
    const unsigned* xw = reinterpret_cast<const unsigned*>(xs) + tchunk * 8 * (P / 2);
    const int Q = P / 2;
    if (n < a.N) {
#pragma unroll 2
        for (int kb = wave * 2 * FP; kb < K; kb += WAVES * 2 * FP) {
            const int k = kb + 2 * kk2;      // K is even: the pair exists or does not
            if (k < K) {
                unsigned w[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) w[e] = xw[e * Q + (k >> 1)];
                ln_ushort8 o0, o1;
                if (NORM) {
                    const float2 g = *reinterpret_cast<const float2*>(gam + k);
                    const float2 b = *reinterpret_cast<const float2*>(bet + k);
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        float lo, hi;
                        ln_add_pair<BF>(w[e], -mean[e], lo, hi);
                        o0[e] = ln_narrow<BF>(lo * rstd[e] * g.x + b.x);
                        o1[e] = ln_narrow<BF>(hi * rstd[e] * g.y + b.y);
                    }
                } else {
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        o0[e] = (uint16_t)(w[e] & 0xffffu);
                        o1[e] = (uint16_t)(w[e] >> 16);
                    }
                }
                uint16_t* dst = a.out + (long)k * a.ldo + n;
                __builtin_nontemporal_store(o0, reinterpret_cast<ln_ushort8*>(dst));
                __builtin_nontemporal_store(o1, reinterpret_cast<ln_ushort8*>(dst + a.ldo));
            }
        }
    }
}

// ---------------------------------------------------------------- register-resident variant
// For feature counts whose token blocks no longer fit the LDS: a workgroup of sixteen
// wavefronts keeps 4096 features of its 32 tokens in registers (two tokens per wavefront,
// 64 registers per lane), takes the statistics from there, and passes them through the
// LDS in slices of 1024 features, double-buffered so that one barrier per slice suffices;
// the transposed store of a slice is the LDS-resident kernel's.  Up to 4096 features
// (PARTS = 1) every activation is read from HBM once.  Wider rows (PARTS = 2 .. 4, up to
// 16384 features) are swept in parts of 4096 for the statistics; the last part stays in
// registers and goes out first, the others are read again (2 - 1/PARTS reads per
// activation; the streaming kernel reads a row once per workgroup that shares its
// tokens, and 16-token blocks, whose 32-byte row segments halve the write rate, measured
// 187 us against 112 on 8192 x 8192).
template <bool BF, bool NORM, int PARTS>
__global__ __launch_bounds__(1024) void layernorm_transpose_register_kernel(LnArgs a)
{
    constexpr int TOK = 32, WAVES = 16, TPW = 2, KH = 4096, SL = 1024, NSL = KH / SL;
    constexpr int CH = TOK / 8, FP = 64 / CH;
    constexpr int P = SL + 4, Q = P / 2;   // Q = 2 (mod 8): see the LDS-resident kernel
    extern __shared__ __attribute__((aligned(16))) char ln_smem[];
    uint16_t* xs = reinterpret_cast<uint16_t*>(ln_smem);                          // [2][TOK][P]
    float* st_mean = reinterpret_cast<float*>(ln_smem + (size_t)2 * TOK * P * 2);  // [TOK]
    float* st_rstd = st_mean + TOK;                                                // [TOK]

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const long n0 = (long)blockIdx.x * TOK;
    const int K = a.K;
    const bool full = n0 + TOK <= a.N && K == KH * PARTS;

    // chunk j of a token's part: features part*4096 + j*512 + lane*8 .. +7
    ln_ushort8 v[TPW][2 * NSL];
    float s1[TPW], s2[TPW], pivot[TPW];
#pragma unroll
    for (int t = 0; t < TPW; ++t) { s1[t] = 0.f; s2[t] = 0.f; pivot[t] = 0.f; }
    auto fetch_as = [&](int part, auto full_tag, auto stats_tag) __attribute__((always_inline)) {
        constexpr bool FULL = decltype(full_tag)::value, STATS = decltype(stats_tag)::value;
        const int kh = part * KH;
#pragma unroll
        for (int t = 0; t < TPW; ++t) {
            const long n = n0 + wave * TPW + t;
#pragma unroll
            for (int j = 0; j < 2 * NSL; ++j) {
                const int kc = kh + j * 512 + lane * 8;
                if (FULL) {
                    v[t][j] = *reinterpret_cast<const ln_ushort8*>(a.x + n * a.ldx + kc);
                } else {
                    v[t][j] = ln_ushort8{0, 0, 0, 0, 0, 0, 0, 0};
                    if (n < a.N && kc < K) v[t][j] = *reinterpret_cast<const ln_ushort8*>(a.x + n * a.ldx + kc);
                }
            }
        }
        if (STATS) {
#pragma unroll
            for (int t = 0; t < TPW; ++t) {
                if (part == 0)
                    pivot[t] = __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(
                        __builtin_bit_cast(int, ln_widen<BF>(v[t][0][0]))));
#pragma unroll
                for (int j = 0; j < 2 * NSL; ++j) {
                    if (FULL || kh + j * 512 + lane * 8 < K) {
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const unsigned w = (unsigned)v[t][j][2 * e] | ((unsigned)v[t][j][2 * e + 1] << 16);
                            float d0, d1;
                            ln_add_pair<BF>(w, -pivot[t], d0, d1);
                            s1[t] += d0;
                            s2[t] += d0 * d0;
                            s1[t] += d1;
                            s2[t] += d1 * d1;
                        }
                    }
                }
            }
        }
    };
    auto fetch = [&](int part, auto stats_tag) __attribute__((always_inline)) {
        if (full) fetch_as(part, std::true_type{}, stats_tag);
        else fetch_as(part, std::false_type{}, stats_tag);
    };

    const int kk2 = lane / CH, tchunk = lane % CH;
    const long n = n0 + tchunk * 8;
    float mean[8], rstd[8];
    // 1.0 twice in the 16-bit format, for an absent gamma
    const unsigned one2 = BF ? 0x3f803f80u : 0x3c003c00u;
    // the part held in registers, slice by slice through the LDS, out as transposed rows
    auto emit = [&](int part) __attribute__((always_inline)) {
        const int kh = part * KH;
        auto stage = [&](int sl) __attribute__((always_inline)) {
#pragma unroll
            for (int t = 0; t < TPW; ++t) {
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const ln_ushort8& c = v[t][2 * sl + h];
                    uint2* dst = reinterpret_cast<uint2*>(xs + ((sl & 1) * TOK + wave * TPW + t) * P + h * 512 + lane * 8);
                    dst[0] = uint2{(unsigned)c[0] | ((unsigned)c[1] << 16), (unsigned)c[2] | ((unsigned)c[3] << 16)};
                    dst[1] = uint2{(unsigned)c[4] | ((unsigned)c[5] << 16), (unsigned)c[6] | ((unsigned)c[7] << 16)};
                }
            }
        };
        // buffer 0's last readers passed the barrier that closed the slice before
        stage(0);
        __syncthreads();
#pragma unroll
        for (int sl = 0; sl < NSL; ++sl) {
            // whole slices every time (a slice beyond K holds zeros and stores nothing), so
            // that every wavefront meets every barrier
            if (sl + 1 < NSL) stage(sl + 1);
            const unsigned* xw = reinterpret_cast<const unsigned*>(xs + (sl & 1) * TOK * P) + tchunk * 8 * Q;
#pragma unroll
            for (int pass = 0; pass < SL / (WAVES * 2 * FP); ++pass) {
                const int kl = (pass * WAVES + wave) * 2 * FP + 2 * kk2;   // feature inside the slice
                const int k = kh + sl * SL + kl;
                if (k < K && n < a.N) {
                    unsigned w[8];
#pragma unroll
                    for (int e = 0; e < 8; ++e) w[e] = xw[e * Q + (kl >> 1)];
                    ln_ushort8 o0, o1;
                    if (NORM) {
                        const unsigned gw = a.gamma ? *reinterpret_cast<const unsigned*>(a.gamma + k) : one2;
                        const unsigned bw = a.beta ? *reinterpret_cast<const unsigned*>(a.beta + k) : 0u;
                        float g0, g1, b0, b1;
                        ln_add_pair<BF>(gw, 0.f, g0, g1);
                        ln_add_pair<BF>(bw, 0.f, b0, b1);
#pragma unroll
                        for (int e = 0; e < 8; ++e) {
                            float lo, hi;
                            ln_add_pair<BF>(w[e], -mean[e], lo, hi);
                            o0[e] = ln_narrow<BF>(lo * rstd[e] * g0 + b0);
                            o1[e] = ln_narrow<BF>(hi * rstd[e] * g1 + b1);
                        }
                    } else {
#pragma unroll
                        for (int e = 0; e < 8; ++e) {
                            o0[e] = (uint16_t)(w[e] & 0xffffu);
                            o1[e] = (uint16_t)(w[e] >> 16);
                        }
                    }
                    uint16_t* dst = a.out + (long)k * a.ldo + n;
                    __builtin_nontemporal_store(o0, reinterpret_cast<ln_ushort8*>(dst));
                    __builtin_nontemporal_store(o1, reinterpret_cast<ln_ushort8*>(dst + a.ldo));
                }
            }
            __syncthreads();
        }
    };

    if (!NORM) {
        // nothing to wait for: each part goes out as it comes in
#pragma unroll
        for (int part = 0; part < PARTS; ++part) {
            fetch(part, std::false_type{});
            emit(part);
        }
        return;
    }
#pragma unroll
    for (int part = 0; part < PARTS; ++part) fetch(part, std::true_type{});
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
            const float m = s1[t] / (float)K;
            float var = s2[t] / (float)K - m * m;
            var = var > 0.f ? var : 0.f;
            st_mean[wave * TPW + t] = pivot[t] + m;
            st_rstd[wave * TPW + t] = 1.0f / __builtin_sqrtf(var + a.eps);
        }
    }
    __syncthreads();
#pragma unroll
    for (int e = 0; e < 8; ++e) { mean[e] = st_mean[tchunk * 8 + e]; rstd[e] = st_rstd[tchunk * 8 + e]; }
    emit(PARTS - 1);   // the part the sweep left in the registers
#pragma unroll
    for (int part = 0; part < PARTS - 1; ++part) {
        fetch(part, std::false_type{});
        emit(part);
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
    // LDS-resident variant when a block of tokens with all its features fits
    auto resident_bytes = [&](int tok, int& pitch) {
        const int want = tok == 32 ? 2 : 1;             // (pitch / 2) mod 8, see the kernel
        int pad = 0;
        while (((K + pad) / 2) % 8 != want) pad += 2;
        pitch = K + pad;
        return (size_t)tok * pitch * 2 + 2 * (size_t)tok * 4 + 2 * (size_t)K * 4;
    };
    const size_t lds_cap = 160 * 1024 - 256;
    int pitch = 0;
    int tok = 0;
    // Blocks of 32 tokens (64-byte row segments, two workgroups per CU) are faster while input
    // and output together stay well inside the 256 MB memory-side cache, where the halves of a
    // line still meet; beyond that the 128-byte segments of 64-token blocks win (measured:
    // 26 against 27 us at 134 MB, 53 against 44 us at 201 MB).
    const bool big = 4.0 * (double)N * (double)K > 160e6;
    if (big && resident_bytes(64, pitch) <= lds_cap) tok = 64;
    else if (resident_bytes(32, pitch) <= lds_cap) tok = 32;
    if (tok) {
        const size_t bytes = resident_bytes(tok, pitch);
        const int64_t rwgs = (N + tok - 1) / tok;
        if (rwgs > 0x7fffffffLL) return fail(SHFLBW_ERR_BAD_SHAPE, "grid too large");
        typedef void (*resident_fn)(LnArgs, int);
        static const resident_fn table[8] = {
            &layernorm_transpose_resident_kernel<false, 32, false>, &layernorm_transpose_resident_kernel<false, 32, true>,
            &layernorm_transpose_resident_kernel<false, 64, false>, &layernorm_transpose_resident_kernel<false, 64, true>,
            &layernorm_transpose_resident_kernel<true, 32, false>,  &layernorm_transpose_resident_kernel<true, 32, true>,
            &layernorm_transpose_resident_kernel<true, 64, false>,  &layernorm_transpose_resident_kernel<true, 64, true>};
        const int which = (dtype == SHFLBW_BF16 ? 4 : 0) + (tok == 64 ? 2 : 0) + (a.normalize ? 1 : 0);
        const resident_fn fn = table[which];
        // the attribute is raised once per kernel and device
        static thread_local int raised_on[8] = {-1, -1, -1, -1, -1, -1, -1, -1};
        int dev = 0;
        hipError_t ea = hipGetDevice(&dev);
        if (ea != hipSuccess) return fail(SHFLBW_ERR_HIP, std::string("hipGetDevice: ") + hipGetErrorString(ea));
        if (raised_on[which] != dev) {
            ea = hipFuncSetAttribute(reinterpret_cast<const void*>(fn), hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
            if (ea != hipSuccess) return fail(SHFLBW_ERR_HIP, std::string("hipFuncSetAttribute: ") + hipGetErrorString(ea));
            raised_on[which] = dev;
        }
        hipLaunchKernelGGL(fn, dim3((unsigned)rwgs), dim3(1024), bytes, st, a, pitch);
        hipError_t el = hipGetLastError();
        if (el != hipSuccess) return fail(SHFLBW_ERR_HIP, std::string("kernel launch: ") + hipGetErrorString(el));
        return SHFLBW_OK;
    }
    if (K <= 16384) {
        // too wide for the LDS, narrow enough to go through the registers of sixteen wavefronts
        // in at most four parts
        typedef void (*register_fn)(LnArgs);
#define SHFLBW_LN_REG(P) \
    &layernorm_transpose_register_kernel<false, false, P>, &layernorm_transpose_register_kernel<false, true, P>, \
    &layernorm_transpose_register_kernel<true, false, P>, &layernorm_transpose_register_kernel<true, true, P>
        static const register_fn rtable[16] = {SHFLBW_LN_REG(1), SHFLBW_LN_REG(2), SHFLBW_LN_REG(3), SHFLBW_LN_REG(4)};
#undef SHFLBW_LN_REG
        const int parts = (K + 4095) / 4096;
        const int which = (parts - 1) * 4 + (dtype == SHFLBW_BF16 ? 2 : 0) + (a.normalize ? 1 : 0);
        const register_fn fn = rtable[which];
        const size_t bytes = (size_t)2 * 32 * (1024 + 4) * 2 + 2 * 32 * 4;
        const int64_t rwgs = (N + 31) / 32;
        if (rwgs > 0x7fffffffLL) return fail(SHFLBW_ERR_BAD_SHAPE, "grid too large");
        static thread_local int raised_reg[16] = {-1, -1, -1, -1, -1, -1, -1, -1, -1, -1, -1, -1, -1, -1, -1, -1};
        int dev = 0;
        hipError_t ea = hipGetDevice(&dev);
        if (ea != hipSuccess) return fail(SHFLBW_ERR_HIP, std::string("hipGetDevice: ") + hipGetErrorString(ea));
        if (raised_reg[which] != dev) {
            ea = hipFuncSetAttribute(reinterpret_cast<const void*>(fn), hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
            if (ea != hipSuccess) return fail(SHFLBW_ERR_HIP, std::string("hipFuncSetAttribute: ") + hipGetErrorString(ea));
            raised_reg[which] = dev;
        }
        hipLaunchKernelGGL(fn, dim3((unsigned)rwgs), dim3(1024), bytes, st, a);
        hipError_t el = hipGetLastError();
        if (el != hipSuccess) return fail(SHFLBW_ERR_HIP, std::string("kernel launch: ") + hipGetErrorString(el));
        return SHFLBW_OK;
    }
    // split the features over grid.y until there are about two workgroups per CU
    const int nblocks = (K + LN_FB - 1) / LN_FB;
    int split = 1;
    // every workgroup that shares a token block repeats the block's statistics sweep, so a
    // normalising launch stops splitting at one workgroup per CU
    while (wgs * split < (a.normalize ? 256 : 512) && split * 2 <= nblocks && split < 16) split *= 2;
    a.blocks_per_wg = (nblocks + split - 1) / split;
    const unsigned gy = (unsigned)((nblocks + a.blocks_per_wg - 1) / a.blocks_per_wg);
    const dim3 sgrid((unsigned)wgs, gy), sblock(64 * LN_WAVES);
    if (dtype == SHFLBW_BF16) {
        if (a.normalize) hipLaunchKernelGGL((layernorm_transpose_kernel<true, true>), sgrid, sblock, 0, st, a);
        else hipLaunchKernelGGL((layernorm_transpose_kernel<true, false>), sgrid, sblock, 0, st, a);
    } else {
        if (a.normalize) hipLaunchKernelGGL((layernorm_transpose_kernel<false, true>), sgrid, sblock, 0, st, a);
        else hipLaunchKernelGGL((layernorm_transpose_kernel<false, false>), sgrid, sblock, 0, st, a);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(SHFLBW_ERR_HIP, std::string("kernel launch: ") + hipGetErrorString(e));
    return SHFLBW_OK;
}
