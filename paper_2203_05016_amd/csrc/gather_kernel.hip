// Per-wavefront gather kernel for the Shfl-BW product on gfx950 (CDNA4).
//
// One wavefront owns one row group (V stored rows) x WN output columns and
// runs Algorithm 1's loop on its own, with no workgroup barrier:
//   BulkLoadMeta  - the column indices of a k-step are fetched 2*PD steps
//                   ahead of their use, one 16-byte load per lane;
//   StitchTile    - the TK activation rows named by those indices are loaded
//                   (16 bytes per lane, coalesced along N) PD steps ahead into
//                   registers, then written to the wavefront's private LDS
//                   tile; the weight tile is one 16-byte load per lane from
//                   the packed array, already in operand order;
//   WarpMMA       - the activation tile is read back transposed
//                   (ds_read_b64_tr_b16) as the first matrix-core operand and
//                   multiplied with the weight operand, fp32 accumulation;
//   ReorderedWriteBack - accumulators go through LDS so that every stored
//                   row leaves as full 16-byte-per-lane row segments, to the
//                   row named by row_indices.
//
// The product is computed as (X^T tile) x (W^T tile), i.e. the instruction's
// row dimension runs over output columns n and its column dimension over the
// group's rows: each lane then holds 4 consecutive n of one row, which packs
// into one 8-byte LDS write in the epilogue.
//
// Operand and accumulator lane maps (checked on hardware):
//   v_mfma_f32_32x32x16_f16  A: lane l = row l%32, k = 8*(l/32)+e
//                            B: lane l = col l%32, k = 8*(l/32)+e
//                            D: lane l, reg r = row 8*(r/4)+4*(l/32)+r%4, col l%32
//   v_mfma_f32_16x16x32_f16  A: lane l = row l%16, k = 8*(l/16)+e; B alike;
//                            D: lane l, reg r = row 4*(l/16)+r, col l%16
//   ds_read_b64_tr_b16: inside each block of 16 lanes, result element e of
//     lane i is element i%4 of the 8 bytes addressed by lane 4*e + i/4; with
//     lanes 4q..4q+3 pointing at 16 consecutive n of row k_q, lane i ends up
//     with column n_i of rows k_0..k_3.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>
#include <type_traits>

#include "shflbw_internal.h"

namespace shflbw {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef short short4v __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef int intx4 __attribute__((ext_vector_type(4)));
typedef int intx2 __attribute__((ext_vector_type(2)));
typedef __attribute__((address_space(3))) short4v* lds_short4_ptr;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

// The matrix-core products.  Operands travel as 16-bit patterns in half8
// registers whatever their format; BF selects the bfloat16 instruction, whose
// operand and accumulator lane maps are those of the binary16 one.
template <bool BF>
__device__ __forceinline__ floatx16 mma32(half8 a, half8 b, floatx16 c)
{
    if constexpr (BF)
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a),
                                                       __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
}
template <bool BF>
__device__ __forceinline__ floatx4 mma16(half8 a, half8 b, floatx4 c)
{
    if constexpr (BF)
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a),
                                                       __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0);
}

// Orders LDS traffic between the lanes of one wavefront.  The hardware runs a
// wavefront's LDS instructions in order; this only stops the compiler from
// moving accesses across the point.
#define SHFLBW_WAVE_LDS_SYNC()                                   \
    do {                                                         \
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");   \
        __builtin_amdgcn_wave_barrier();                         \
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");   \
    } while (0)

struct PackedView {
    const int32_t* row_indices;
    const int32_t* step_ptr;
    const int32_t* col_idx;
    const half8* values;  // 16-byte units
    int G;
};

// ---------------------------------------------------------------- geometry
// A geometry answers two questions: which 8 activation values sit at
// (reduction index k, output columns n..n+7), and where do output values
// (original row, columns n..n+cnt-1) go.

// Linear layer: X[K][N] and Y[M][N] row-major.  ALIGNED: N, ldx, ldy are
// multiples of 8 and both bases are 16-byte aligned.
template <bool ALIGNED>
struct GeomLinear {
    const _Float16* X;
    void* Y;
    long ldx, ldy, N;

    __device__ __forceinline__ void init(long) {}

    __device__ __forceinline__ half8 load8(int col, long n) const
    {
        half8 v = {0, 0, 0, 0, 0, 0, 0, 0};
        if (col < 0) return v;
        const _Float16* p = X + (long)col * ldx + n;
        if (ALIGNED) {
            if (n < N) v = *reinterpret_cast<const half8*>(p);
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e)
                if (n + e < N) v[e] = p[e];
        }
        return v;
    }

    template <typename OutT, int CNT>
    __device__ __forceinline__ void store(int row, long n, const OutT* vals) const
    {
        OutT* p = static_cast<OutT*>(Y) + (long)row * ldy + n;
        if (ALIGNED) {
            if (n < N) {
                typedef OutT vec_t __attribute__((ext_vector_type(CNT)));
                vec_t v;
#pragma unroll
                for (int e = 0; e < CNT; ++e) v[e] = vals[e];
                // the output is not read again by this kernel: keep it from displacing X and W in the L2
                __builtin_nontemporal_store(v, reinterpret_cast<vec_t*>(p));
            }
        } else {
#pragma unroll
            for (int e = 0; e < CNT; ++e)
                if (n + e < N) p[e] = vals[e];
        }
    }
};

// The aligned linear layer again, with X behind a buffer descriptor: a load's
// address is one 24-bit multiply-add in a vector register (byte offset of the
// row plus the lane's column offset) instead of 64-bit arithmetic, and the
// descriptor's range check stands in for the two conditions - a padded slot
// (column -1) and a lane beyond N get an offset past the end and read as zero.
// The host uses it when K and 2*ldx are below 2^24 and X spans less than 4 GiB.
constexpr int GATHER_BUFFER_FLAGS = 0x00020000;   // last word of a raw buffer descriptor: untyped 32-bit data
struct GeomLinearBuf {
    const _Float16* X;
    void* Y;
    long ldx, ldy, N;
    unsigned xbytes;          // (K-1)*ldx*2 + N*2: what the descriptor covers
    __amdgpu_buffer_rsrc_t xd;
    unsigned ldx2, ln2;
    // beyond every descriptor the host admits, and 16 bytes from there do not wrap
    static constexpr unsigned PAST_END = 0xffffffe0u;

    __device__ __forceinline__ void init(long n)
    {
        xd = __builtin_amdgcn_make_buffer_rsrc(const_cast<_Float16*>(X), 0, (int)xbytes, GATHER_BUFFER_FLAGS);
        ldx2 = (unsigned)ldx * 2u;
        ln2 = n < N ? (unsigned)n * 2u : PAST_END;
    }

    // zero (the same for the whole wavefront): read zeros whatever the column, at the price of
    // scalar instructions only
    __device__ __forceinline__ half8 load8(int col, long, bool zero = false) const
    {
        typedef unsigned uint4v __attribute__((ext_vector_type(4)));
        // a lane beyond N keeps its offset past the end whatever the column
        unsigned off = __umul24((unsigned)col, ldx2) + ln2;
        off = (col < 0 || ln2 == PAST_END || zero) ? PAST_END : off;
        return __builtin_bit_cast(half8, __builtin_amdgcn_raw_buffer_load_b128(xd, (int)off, 0, 0));
    }

    template <typename OutT, int CNT>
    __device__ __forceinline__ void store(int row, long n, const OutT* vals) const
    {
        OutT* p = static_cast<OutT*>(Y) + (long)row * ldy + n;
        if (n < N) {
            typedef OutT vec_t __attribute__((ext_vector_type(CNT)));
            vec_t v;
#pragma unroll
            for (int e = 0; e < CNT; ++e) v[e] = vals[e];
            // the output is not read again by this kernel: keep it from displacing X and W in the L2
            __builtin_nontemporal_store(v, reinterpret_cast<vec_t*>(p));
        }
    }
};

// 1x1 convolution with unit stride and no padding on NCHW tensors (Section 4.1's
// implicit GEMM with R = S = 1): image b is a row-major [K][HW] matrix, so column
// n = b*HW + hw of the product lives at X + (b*K + k)*HW + hw, and its output at
// Y + (b*M + row)*HW + hw.  The loads are GeomLinearBuf's with a per-lane image base;
// HW is a multiple of 8, so the 8 columns of a lane stay inside one image.
struct GeomBatchedBuf : GeomLinearBuf {
    int HW, K, M;

    __device__ __forceinline__ void init(long n)
    {
        xd = __builtin_amdgcn_make_buffer_rsrc(const_cast<_Float16*>(X), 0, (int)xbytes, GATHER_BUFFER_FLAGS);
        ldx2 = (unsigned)HW * 2u;
        ln2 = PAST_END;
        if (n < N) {
            const unsigned b = (unsigned)n / (unsigned)HW, hw = (unsigned)n - b * (unsigned)HW;
            ln2 = (b * (unsigned)K * (unsigned)HW + hw) * 2u;
        }
    }

    template <typename OutT, int CNT>
    __device__ __forceinline__ void store(int row, long n, const OutT* vals) const
    {
        if (n < N) {
            const unsigned b = (unsigned)n / (unsigned)HW, hw = (unsigned)n - b * (unsigned)HW;
            OutT* p = static_cast<OutT*>(Y) + ((long)b * M + row) * HW + hw;
            typedef OutT vec_t __attribute__((ext_vector_type(CNT)));
            vec_t v;
#pragma unroll
            for (int e = 0; e < CNT; ++e) v[e] = vals[e];
            __builtin_nontemporal_store(v, reinterpret_cast<vec_t*>(p));
        }
    }
};

// The same for H*W a multiple of 4 only (14 x 14 images): a lane's 8 columns may cross
// from one image into the next, but each half of 4 stays inside one, so every load and
// every 8-wide store is done as two halves with an image base of their own.
struct GeomBatchedBuf4 : GeomLinearBuf {
    int HW, K, M;
    unsigned ln2b;   // offset of the lane's columns 4..7

    __device__ __forceinline__ unsigned image_offset(long n) const
    {
        if (n >= N) return PAST_END;
        const unsigned b = (unsigned)n / (unsigned)HW, hw = (unsigned)n - b * (unsigned)HW;
        return (b * (unsigned)K * (unsigned)HW + hw) * 2u;
    }
    __device__ __forceinline__ void init(long n)
    {
        xd = __builtin_amdgcn_make_buffer_rsrc(const_cast<_Float16*>(X), 0, (int)xbytes, GATHER_BUFFER_FLAGS);
        ldx2 = (unsigned)HW * 2u;
        ln2 = image_offset(n);
        ln2b = image_offset(n + 4);
    }
    __device__ __forceinline__ half8 load8(int col, long, bool zero = false) const
    {
        typedef unsigned uint2v __attribute__((ext_vector_type(2)));
        typedef unsigned uint4v __attribute__((ext_vector_type(4)));
        const unsigned o = __umul24((unsigned)col, ldx2);
        const bool none = col < 0 || zero;
        const unsigned oa = (none || ln2 == PAST_END) ? PAST_END : o + ln2;
        const unsigned ob = (none || ln2b == PAST_END) ? PAST_END : o + ln2b;
        const uint2v lo = __builtin_amdgcn_raw_buffer_load_b64(xd, (int)oa, 0, 0);
        const uint2v hi = __builtin_amdgcn_raw_buffer_load_b64(xd, (int)ob, 0, 0);
        return __builtin_bit_cast(half8, uint4v{lo[0], lo[1], hi[0], hi[1]});
    }
    template <typename OutT, int CNT>
    __device__ __forceinline__ void store(int row, long n, const OutT* vals) const
    {
        typedef OutT vec_t __attribute__((ext_vector_type(4)));
#pragma unroll
        for (int h = 0; h < CNT / 4; ++h) {
            const long nh = n + 4 * h;
            if (nh < N) {
                const unsigned b = (unsigned)nh / (unsigned)HW, hw = (unsigned)nh - b * (unsigned)HW;
                OutT* p = static_cast<OutT*>(Y) + ((long)b * M + row) * HW + hw;
                vec_t v = {vals[4 * h], vals[4 * h + 1], vals[4 * h + 2], vals[4 * h + 3]};
                __builtin_nontemporal_store(v, reinterpret_cast<vec_t*>(p));
            }
        }
    }
};

// Convolution as implicit GEMM (Section 4.1): k = (c*R + r)*S + s, and
// n = (b*Ho + y)*Wo + x for NCHW or n = (y*Wo + x)*B + b for CHWN.  This is
// the general element-wise form; the unfolded matrix never exists in memory.
struct GeomConv {
    const _Float16* in;
    void* out;
    int B, Cin, H, W, Cout, R, S, sh, sw, ph, pw, Ho, Wo;
    int chwn;
    long N;
    // per-lane decode of the 8 output positions this lane gathers for:
    // base[e] = offset of the window origin (may be negative), yx[e] = packed
    // (iy0, ix0) window origin; valid bit e of `live` = position exists
    int base[8];
    int yx[8];
    int live;

    __device__ __forceinline__ void split_n(long n, int& b, int& y, int& x) const
    {
        int q;
        if (chwn) {
            b = (int)(n % B);
            q = (int)(n / B);
        } else {
            q = (int)(n % ((long)Ho * Wo));
            b = (int)(n / ((long)Ho * Wo));
        }
        y = q / Wo;
        x = q % Wo;
    }

    __device__ __forceinline__ void init(long n)
    {
        live = 0;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            base[e] = 0;
            yx[e] = 0;
            if (n + e >= N) continue;
            int b, y, x;
            split_n(n + e, b, y, x);
            const int iy0 = y * sh - ph, ix0 = x * sw - pw;
            yx[e] = (iy0 << 16) | (ix0 & 0xffff);
            base[e] = chwn ? (iy0 * W + ix0) * B + b : (b * Cin * H + iy0) * W + ix0;
            live |= 1 << e;
        }
    }

    __device__ __forceinline__ half8 load8(int col, long) const
    {
        half8 v = {0, 0, 0, 0, 0, 0, 0, 0};
        if (col < 0) return v;
        const int c = col / (R * S);
        const int rs = col - c * (R * S);
        const int r = rs / S, s = rs - r * S;
        const int koff = ((c * H + r) * W + s) * (chwn ? B : 1);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int iy = (yx[e] >> 16) + r, ix = (int)(short)(yx[e] & 0xffff) + s;
            const bool ok = ((live >> e) & 1) && iy >= 0 && iy < H && ix >= 0 && ix < W;
            if (ok) v[e] = in[(long)base[e] + koff];
        }
        return v;
    }

    template <typename OutT, int CNT>
    __device__ __forceinline__ void store(int row, long n, const OutT* vals) const
    {
        OutT* o = static_cast<OutT*>(out);
#pragma unroll
        for (int e = 0; e < CNT; ++e) {
            if (n + e >= N) break;
            int b, y, x;
            split_n(n + e, b, y, x);
            const long idx = chwn ? (((long)row * Ho + y) * Wo + x) * B + b
                                  : (((long)b * Cout + row) * Ho + y) * Wo + x;
            o[idx] = vals[e];
        }
    }
};

// ---------------------------------------------------------------- kernel
template <int V, int WN>
struct GatherShape {
    static constexpr bool SMALL = (V == 16);          // 16x16x32 instruction
    static constexpr int TK = SMALL ? 32 : 16;        // columns per k-step
    static constexpr int RB = SMALL ? 1 : V / 32;     // row blocks per group
    static constexpr int TILE_N = SMALL ? 16 : 32;    // output columns per instruction
    static constexpr int NT = WN / TILE_N;
    static constexpr int LPR = WN / 8;                // lanes per activation row (16 B each)
    static constexpr int RPI = 64 / LPR;              // rows per load instruction
    static constexpr int NLD = TK / RPI;              // loads per lane per k-step
    static constexpr int PITCH = WN + 8;              // LDS row pitch in binary16
    static constexpr int STAGE = TK * PITCH;          // binary16 per staged tile
    static constexpr int ROWS_E = SMALL ? 16 : 32;    // rows per epilogue pass
    static constexpr int EPI = ROWS_E * PITCH;        // binary16 needed by one epilogue pass
    static constexpr int REGION = (2 * STAGE > EPI) ? 2 * STAGE : EPI;
};

// SPLIT = false: the wavefronts of a workgroup own different column tiles of one
// group.  SPLIT = true (few column tiles, the matrix-vector-like regime of
// recurrent layers): they share one tile, each takes a contiguous share of
// the group's k-steps, and the partial accumulators are summed through LDS
// before the first wavefront writes the tile back.
template <int V, int WN, int WAVES, int PD, typename OutT, class Geom, bool BF, bool SPLIT>
__global__ __launch_bounds__(64 * WAVES) void shflbw_gather_kernel(PackedView A, Geom geom,
                                                                  int n_tiles)
{
    using S = GatherShape<V, WN>;
    constexpr int TK = S::TK, RB = S::RB, NT = S::NT, LPR = S::LPR, NLD = S::NLD;
    constexpr int PITCH = S::PITCH;
    constexpr int ACC_REGS = S::SMALL ? NT * 4 : RB * NT * 16;       // fp32 accumulators per lane
    constexpr int SPLIT_HALVES = SPLIT ? ACC_REGS * 64 * 2 : 0;      // LDS for one wavefront's partials
    constexpr int SMEM_HALVES = WAVES * S::REGION > SPLIT_HALVES ? WAVES * S::REGION : SPLIT_HALVES;
    __shared__ __attribute__((aligned(16))) _Float16 smem[SMEM_HALVES];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int tile = SPLIT ? (int)blockIdx.x : (int)blockIdx.x * WAVES + wave;
    // without SPLIT a whole wavefront leaves and no workgroup barrier is used; with
    // SPLIT the condition is the same for every wavefront of the workgroup
    if (tile >= n_tiles) return;
    const int g = blockIdx.y;
    const long n0 = (long)tile * WN;
    _Float16* my = smem + wave * S::REGION;

    int sbeg = A.step_ptr[g];
    int nsteps = A.step_ptr[g + 1] - sbeg;
    if (SPLIT) {
        const int first = (int)((long)nsteps * wave / WAVES);
        const int end = (int)((long)nsteps * (wave + 1) / WAVES);
        sbeg += first;
        nsteps = end - first;
    }

    // this lane's share of a staged tile: rows lrow..lrow+NLD-1, 8 columns at lcol
    const int lrow = (lane / LPR) * NLD;
    const int lcol = (lane % LPR) * 8;
    const long ln = n0 + lcol;
    geom.init(ln);

    floatx16 acc32[S::SMALL ? 1 : RB][S::SMALL ? 1 : NT];
    floatx4 acc16[S::SMALL ? NT : 1];
    if (S::SMALL) {
#pragma unroll
        for (int t = 0; t < NT; ++t) acc16[t] = floatx4{0, 0, 0, 0};
    } else {
#pragma unroll
        for (int rb = 0; rb < RB; ++rb)
#pragma unroll
            for (int t = 0; t < NT; ++t)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc32[rb][t][r] = 0.f;
    }

    // ---- pipeline registers
    int cols[PD][NLD];
    half8 xr[PD][NLD];
    half8 wr[PD][RB];

    // Column indices and weights of the wavefront's steps through buffer descriptors: the
    // step's offset is a scalar register, the lane's a constant vector register.
    typedef unsigned uint2v __attribute__((ext_vector_type(2)));
    typedef unsigned uint4v __attribute__((ext_vector_type(4)));
    const __amdgpu_buffer_rsrc_t col_rsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<int32_t*>(A.col_idx + (long)sbeg * TK), 0, nsteps * TK * 4, GATHER_BUFFER_FLAGS);
    const __amdgpu_buffer_rsrc_t val_rsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<half8*>(A.values + (long)sbeg * RB * 64), 0, nsteps * RB * 1024, GATHER_BUFFER_FLAGS);
    // A buffer load checks lane offset + immediate against the descriptor's size, NOT the
    // scalar offset.  CHECKED puts the step into the lane offset, so that a step beyond the
    // wavefront's range reads zeros instead of memory past it; the steady-state batches,
    // whose steps all exist, keep the step in the scalar offset (no vector arithmetic).
    auto load_cols = [&](int step, int (&c)[NLD], auto checked_tag) {
        constexpr bool CHECKED = decltype(checked_tag)::value;
        const int vo = CHECKED ? lrow * 4 + step * TK * 4 : lrow * 4;
        const int so = CHECKED ? 0 : step * TK * 4;
        if (NLD == 4) {
            uint4v v = __builtin_amdgcn_raw_buffer_load_b128(col_rsrc, vo, so, 0);
            c[0] = (int)v[0]; c[1] = (int)v[1]; c[2] = (int)v[2]; c[3] = (int)v[3];
        } else if (NLD == 2) {
            uint2v v = __builtin_amdgcn_raw_buffer_load_b64(col_rsrc, vo, so, 0);
            c[0] = (int)v[0]; c[1] = (int)v[1];
        } else {
#pragma unroll
            for (int i = 0; i < NLD; ++i)
                c[i] = (int)__builtin_amdgcn_raw_buffer_load_b32(col_rsrc, vo + i * 4, so, 0);
        }
    };
    // in_range false: the step lies beyond the wavefront's range and gets zeros, like a padded slot
    auto load_x = [&](const int (&c)[NLD], half8 (&x)[NLD], bool in_range) {
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
            if constexpr (std::is_base_of<GeomLinearBuf, Geom>::value) x[i] = geom.load8(c[i], ln, !in_range);
            else x[i] = geom.load8(in_range ? c[i] : -1, ln);
        }
    };
    auto load_w = [&](int step, half8 (&w)[RB], auto checked_tag) {
        constexpr bool CHECKED = decltype(checked_tag)::value;
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) {
            const int off = (step * RB + rb) * 1024;
            w[rb] = __builtin_bit_cast(half8, __builtin_amdgcn_raw_buffer_load_b128(
                val_rsrc, CHECKED ? lane * 16 + off : lane * 16, CHECKED ? 0 : off, 0));
        }
    };

    // The loop below is straight-line code over whole batches of PD steps, so that the
    // register sets stay static and the compiler's wait counts exact (a conditional refill
    // turns into a copy behind a full wait).  A step beyond the wavefront's range multiplies
    // zero weights (range-checked loads) with gathered zeros.
    const int nsteps_r = (nsteps + PD - 1) / PD * PD;
#pragma unroll
    for (int u = 0; u < PD; ++u) {
        int c0[NLD];
        load_cols(u, c0, std::true_type{});
        load_x(c0, xr[u], u < nsteps);
        load_cols(u + PD, cols[u], std::true_type{});
        load_w(u, wr[u], std::true_type{});
        // sets in the order the loop issues them: its wait counts assume set 0 is the oldest
        __builtin_amdgcn_sched_barrier(0);
    }

    // transposed-read addresses (in binary16 units inside a staged tile)
    // 32-wide: block b = lane/16 covers n = 16*(b%2)+0..15, k = 8*(b/2)+4h+0..3
    // 16-wide: block b covers n = 0..15,                k = 8*b+4h+0..3
    const int bl = lane >> 4, il = lane & 15;
    const int tr_row = S::SMALL ? (8 * bl + (il >> 2)) : (8 * (bl >> 1) + (il >> 2));
    const int tr_col = S::SMALL ? (4 * (il & 3)) : (16 * (bl & 1) + 4 * (il & 3));
    const int tr_off = tr_row * PITCH + tr_col;

    // One batch.  NEXT: the batch after this one exists, its X rows and weights are
    // requested; AFTER: so does the one after that, whose column indices are requested.
    // The last two batches therefore issue no loads that nobody waits for.
    auto batch = [&](int s0, auto next_tag, auto after_tag) __attribute__((always_inline)) {
        constexpr bool NEXT = decltype(next_tag)::value, AFTER = decltype(after_tag)::value;
#pragma unroll
        for (int u = 0; u < PD; ++u) {
            const int s = s0 + u;
            _Float16* buf = my + (s & 1) * S::STAGE;
#pragma unroll
            for (int i = 0; i < NLD; ++i)
                *reinterpret_cast<half8*>(buf + (lrow + i) * PITCH + lcol) = xr[u][i];
            SHFLBW_WAVE_LDS_SYNC();

            if (NEXT) load_x(cols[u], xr[u], AFTER || s + PD < nsteps);
            // may name up to PD - 1 steps past the range: those indices (whatever follows in the
            // packed matrix) are never turned into addresses
            if (AFTER) load_cols(s + 2 * PD, cols[u], std::false_type{});

#pragma unroll
            for (int t = 0; t < NT; ++t) {
                const _Float16* base = buf + tr_off + t * S::TILE_N;
                short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_ptr)(base));
                short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_ptr)(base + 4 * PITCH));
                half4 l4 = __builtin_bit_cast(half4, lo), h4 = __builtin_bit_cast(half4, hi);
                half8 a = {l4[0], l4[1], l4[2], l4[3], h4[0], h4[1], h4[2], h4[3]};
                if (S::SMALL) {
                    acc16[t] = mma16<BF>(a, wr[u][0], acc16[t]);
                } else {
#pragma unroll
                    for (int rb = 0; rb < RB; ++rb)
                        acc32[rb][t] = mma32<BF>(a, wr[u][rb], acc32[rb][t]);
                }
            }
            // refilled after its last use, so the load lands in the set's own registers
            // the last loading batch may reach past the range: checked there
            if (NEXT) load_w(s + PD, wr[u], std::integral_constant<bool, !AFTER>{});
            // steps stay in program order: hoisting the next step's LDS writes above this
            // step's products would make them wait for the loads issued just above
            __builtin_amdgcn_sched_barrier(0);
            // no second sync: the next step writes the other buffer, and its own
            // sync separates these reads from the writes of the step after it
        }
    };
    int s0 = 0;
    for (; s0 + 2 * PD < nsteps_r; s0 += PD) batch(s0, std::true_type{}, std::true_type{});
    if (s0 + PD < nsteps_r) {
        batch(s0, std::true_type{}, std::false_type{});
        s0 += PD;
    }
    if (s0 < nsteps_r) batch(s0, std::false_type{}, std::false_type{});
    SHFLBW_WAVE_LDS_SYNC();

    if (SPLIT) {
        // sum the partial accumulators into wavefront 0, one wavefront at a time;
        // register r of lane l sits at float4 index (r/4)*64 + l, free of bank conflicts
        floatx4* red = reinterpret_cast<floatx4*>(smem);
        for (int w = WAVES - 1; w >= 1; --w) {
            __syncthreads();   // the buffer (and, first time, every private region) is free
            if (wave == w) {
                if (S::SMALL) {
#pragma unroll
                    for (int t = 0; t < NT; ++t) red[t * 64 + lane] = acc16[t];
                } else {
#pragma unroll
                    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
                        for (int t = 0; t < NT; ++t)
#pragma unroll
                            for (int q = 0; q < 4; ++q)
                                red[((rb * NT + t) * 4 + q) * 64 + lane] =
                                    floatx4{acc32[rb][t][4 * q], acc32[rb][t][4 * q + 1],
                                            acc32[rb][t][4 * q + 2], acc32[rb][t][4 * q + 3]};
                }
            }
            __syncthreads();
            if (wave == 0) {
                if (S::SMALL) {
#pragma unroll
                    for (int t = 0; t < NT; ++t) acc16[t] += red[t * 64 + lane];
                } else {
#pragma unroll
                    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
                        for (int t = 0; t < NT; ++t)
#pragma unroll
                            for (int q = 0; q < 4; ++q) {
                                const floatx4 v = red[((rb * NT + t) * 4 + q) * 64 + lane];
                                acc32[rb][t][4 * q] += v[0]; acc32[rb][t][4 * q + 1] += v[1];
                                acc32[rb][t][4 * q + 2] += v[2]; acc32[rb][t][4 * q + 3] += v[3];
                            }
                }
            }
        }
        __syncthreads();       // wavefront 0 has read the last partials; its region is reused below
        if (wave != 0) return;
    }

    // ---- reordered write-back
    // Each pass moves ROWS_E stored rows x CW columns through LDS.  A lane
    // holds 4 consecutive n of one row per accumulator quad.
    constexpr int OUT_PER_16B = 16 / (int)sizeof(OutT);             // 8 (fp16) or 4 (fp32)
    constexpr int PASSES = (int)sizeof(OutT) / 2;                   // column halves per row block
    constexpr int CW = WN / PASSES;                                  // columns per pass
    constexpr int EP = CW + 16 / (int)sizeof(OutT);                 // pitch in OutT units
    static_assert(S::ROWS_E * EP * (int)sizeof(OutT) <= S::REGION * 2, "epilogue tile must fit");
    OutT* ep = reinterpret_cast<OutT*>(my);
    constexpr int LPR_E = CW / OUT_PER_16B;                          // lanes per row at readback
    constexpr int RPI_E = 64 / LPR_E;
    const int erow = lane / LPR_E, echunk = lane % LPR_E;
    const int32_t* rows_g = A.row_indices + (long)g * V;

#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
#pragma unroll
        for (int pass = 0; pass < PASSES; ++pass) {
            constexpr int TPP = NT / PASSES;  // instruction tiles per pass
#pragma unroll
            for (int tt = 0; tt < TPP; ++tt) {
                const int t = pass * TPP + tt;
                if (S::SMALL) {
                    // lane: row l%16, n = 16*tt + 4*(l/16) + 0..3
                    OutT* d = ep + (lane & 15) * EP + 16 * tt + 4 * (lane >> 4);
                    typedef OutT vec4 __attribute__((ext_vector_type(4)));
                    vec4 v = {(OutT)acc16[t][0], (OutT)acc16[t][1], (OutT)acc16[t][2], (OutT)acc16[t][3]};
                    *reinterpret_cast<vec4*>(d) = v;
                } else {
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        OutT* d = ep + (lane & 31) * EP + 32 * tt + 8 * q + 4 * (lane >> 5);
                        typedef OutT vec4 __attribute__((ext_vector_type(4)));
                        vec4 v = {(OutT)acc32[rb][t][4 * q + 0], (OutT)acc32[rb][t][4 * q + 1],
                                  (OutT)acc32[rb][t][4 * q + 2], (OutT)acc32[rb][t][4 * q + 3]};
                        *reinterpret_cast<vec4*>(d) = v;
                    }
                }
            }
            SHFLBW_WAVE_LDS_SYNC();
#pragma unroll
            for (int i = 0; i < S::ROWS_E / RPI_E; ++i) {
                const int row = i * RPI_E + erow;
                typedef OutT vecw __attribute__((ext_vector_type(OUT_PER_16B)));
                vecw v = *reinterpret_cast<const vecw*>(ep + row * EP + echunk * OUT_PER_16B);
                OutT tmp[OUT_PER_16B];
#pragma unroll
                for (int e = 0; e < OUT_PER_16B; ++e) tmp[e] = v[e];
                const int orig = rows_g[rb * 32 + row];
                geom.template store<OutT, OUT_PER_16B>(orig, n0 + pass * CW + echunk * OUT_PER_16B, tmp);
            }
            SHFLBW_WAVE_LDS_SYNC();
        }
    }
}

}  // namespace shflbw
