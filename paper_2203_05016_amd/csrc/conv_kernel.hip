// Staged implicit-GEMM convolution for the Shfl-BW product on gfx950 (CDNA4).
//
// Section 4.1 runs a pruned convolution as the same sparse-times-dense
// product, with the unfolded activation matrix (row k = (c, r, s), column
// n = (b, y, x)) existing only on chip.  Here a workgroup owns a box of
// output positions (tb images x th output rows x tw output columns, at most
// 128 positions) and up to eight row groups.  It first copies the input box
// that those positions can touch, all channels, zero padding included, into
// LDS once; after that every element of the unfolded tile is an LDS read at
//     koff[k] + noff[n]
// where koff depends only on the reduction index (channel plane, kernel row
// and column) and noff only on the output position (its top-left input
// element inside the box).  Each wavefront turns the column indices of its
// group into koff values 64 k-steps at a time and keeps them in a private LDS
// list of byte offsets (two 16-byte reads per lane and step in the loop, no
// unpacking); noff lives in registers.  A padded slot of a k-step (column
// index -1) points at an extra all-zero channel plane.  The box is staged with
// 2-byte loads, or with 4-byte loads of two elements that are neighbours in
// memory where the host has laid the box out for it.
//
// Algorithm 1's parts: BulkLoadMeta = column indices in bulks of 64 k-steps,
// the weight operand four (V = 128: two) k-steps ahead in as many register sets;
// V = 16 runs on the 16x16x32 instruction: tiles of 16 positions, k-steps of 32 indices;
// StitchTile = the LDS gather above (each lane reads the 8 reduction indices
// x up to 4 positions it feeds to the matrix cores); WarpMMA =
// v_mfma_f32_32x32x16_f16 with the activation tile as first operand;
// ReorderedWriteBack = accumulators through LDS, then element stores that run
// along the output's innermost dimension, to the channel named by
// row_indices.
//
// Both activation layouts go through the same code: only the element strides
// and the order in which a tile's local index n' walks (image, row, column)
// differ.  NCHW: n' = (bb*th + yy)*tw + xx; CHWN (batch innermost, the
// layout of Section 4.3): n' = (yy*tw + xx)*tb + bb.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

#include "gather_kernel.hip"

namespace shflbw {

constexpr int CONV_GW = 8;             // compute wavefronts (row groups) per workgroup
constexpr int CONV_TN = 128;           // most output positions per workgroup
constexpr int CONV_SCRATCH = 32 * 33 * 4;  // write-back scratch of one wavefront (fp32, pitch 33)
constexpr int CONV_BULK = 64;          // k-steps of koff values a wavefront holds at a time
constexpr int CONV_LIST_BYTES = CONV_GW * CONV_BULK * 16 * 4;   // byte offsets as 32-bit words: no unpacking in the loop

struct ConvArgs {
    PackedView A;
    const _Float16* in;
    void* out;
    int B, C, H, W, R, S, sh, sw, ph, pw, Ho, Wo, K;
    long isB, isC, isH, isW;  // input element strides
    long osB, osM, osH, osW;  // output element strides
    int th, tw, tb;           // box of output positions per workgroup
    int ny, nx, nb;           // boxes along y, x, batch
    int rows_in, cols_in;     // input rows / columns one box can touch
    int b_fast;               // 1: batch runs fastest in the local index (CHWN)
    int gblocks;              // blocks of gpb groups
    int gpb, tsplit;          // groups per workgroup; wavefronts that share a group's instruction tiles
    int uniform_steps;        // k-steps of every group when they all have the same number, else -1
    int stage_pairs;          // the box is laid out for staging with 4-byte loads (1), but the input is not 4-byte aligned (2)
    int dx;                   // columns by which the staged box starts left of the first one needed (0 or 1)
    int in_bytes;             // LDS bytes reserved for the staged input (and the scratch)
    unsigned in_bytes_total;  // bytes of the whole input tensor (below 2^32 - 64: the host checks)
    // ceil(2^40 / d) for the divisors the kernel needs: x / d == (x * m) >> 40 for x, d < 2^20
    unsigned long long m_RS, m_S, m_tb, m_cols_in, m_tw, m_th;
    unsigned long long m_cols2, m_tb2;   // the same for cols_in / 2 and tb / 2 (4-byte staging)
};

// Exact quotient by a divisor known on the host (both below 2^20).
__device__ __forceinline__ int conv_div(int x, unsigned long long m)
{
    return (int)(((unsigned long long)(unsigned)x * m) >> 40);
}

// NT: 32-position instruction tiles per wavefront (1, 2 or 4; a box holds at most 32*NT*tsplit positions).
// SP: the input box is staged with 4-byte loads, two elements that are neighbours in memory each
// (the host lays the box out for it and asks for it when that takes fewer load instructions).
template <int V, int NT, typename OutT, bool BF, bool SP = false>
__global__ __launch_bounds__(64 * CONV_GW) void shflbw_conv_kernel(ConvArgs a)
{
    constexpr bool SMALL = (V == 16);                 // 16x16x32 instruction: 16 positions x 16 rows, 32 reduction indices
    constexpr int RB = SMALL ? 1 : V / 32;
    constexpr int TK = SMALL ? 32 : 16;               // reduction indices per k-step
    constexpr int POS = SMALL ? 16 : 32;              // output positions per instruction tile
    constexpr int NTI = NT * (32 / POS);              // instruction tiles per wavefront
    constexpr int KBLOCKS = TK / 8;                   // a lane feeds 8 reduction indices of block lane / POS
    constexpr int BULK = CONV_BULK * 16 / TK;         // k-steps of koff values held at a time (the list's size is fixed)
    constexpr int CONV_PD = RB <= 2 ? 4 : 2;   // k-steps the weight operand is fetched ahead
    static_assert(BULK % CONV_PD == 0, "bulk boundaries fall on batch boundaries");
    extern __shared__ __attribute__((aligned(16))) char conv_smem[];
    _Float16* xin = reinterpret_cast<_Float16*>(conv_smem);
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // this wavefront's list of koff values: CONV_BULK steps x 16 slots
    uint32_t* klist = reinterpret_cast<uint32_t*>(conv_smem + a.in_bytes) + wave * (CONV_BULK * 16);

    // which box, which block of groups
    int box = blockIdx.x / a.gblocks;
    const int gb = blockIdx.x - box * a.gblocks;
    const int bx = box % a.nx; box /= a.nx;
    const int by = box % a.ny; box /= a.ny;
    const int b0 = box * a.tb, y0 = by * a.th, x0 = bx * a.tw;
    const int plane = a.rows_in * a.cols_in * a.tb;   // staged elements per channel
    const int dx = a.dx;   // not zero only in a box laid out for 4-byte staging
    const int iy0 = y0 * a.sh - a.ph, ix0 = x0 * a.sw - a.pw - dx;
    const int zero_off = a.C * plane;
    const int RS = a.R * a.S;

    // wavefront -> (group of the block, share of the box's instruction tiles): with few row
    // groups the wavefronts left over split the positions of the box instead of idling
    const int gi = wave % a.gpb, ts = wave / a.gpb;
    const int g = gb * a.gpb + gi;
    const bool have_group = g < a.A.G && ts < a.tsplit;
    // the group's steps: without a memory access when every group has the same number (the
    // column indices and first weights can then be requested at once)
    int sbeg = 0, nsteps = 0;
    if (have_group) {
        sbeg = a.uniform_steps >= 0 ? g * a.uniform_steps : a.A.step_ptr[g];
        nsteps = a.uniform_steps >= 0 ? a.uniform_steps : a.A.step_ptr[g + 1] - sbeg;
    }

    // koff values of steps [s0, s0 + BULK) of this group into the list
    constexpr int BULK_LOADS = BULK * TK / 64;
    auto load_cols = [&](int s0, int (&cols)[BULK_LOADS]) __attribute__((always_inline)) {
        const int32_t* cp = a.A.col_idx + ((long)sbeg + s0) * TK;
        const int avail = (nsteps - s0) * TK;
#pragma unroll
        for (int i = 0; i < BULK_LOADS; ++i) {
            const int j = i * 64 + lane;
            cols[i] = j < avail ? cp[j] : -1;
        }
    };
    // `steps`: k-steps of the bulk that the group has; the loop reads up to CONV_PD + 1 entries past
    // them (whole batches, one entry ahead), which must name the zero plane; later ones are not read
    auto store_koff = [&](const int (&cols)[BULK_LOADS], int steps) __attribute__((always_inline)) {
        const int wanted = (steps + CONV_PD + 2) * TK;
#pragma unroll
        for (int i = 0; i < BULK_LOADS; ++i) {
            if (i * 64 >= wanted) break;   // uniform
            const int k = cols[i];
            int off = zero_off;
            if (k >= 0) {
                const int c = conv_div(k, a.m_RS), rs = k - c * RS;
                const int r = conv_div(rs, a.m_S), sx = rs - r * a.S;
                off = c * plane + (r * a.cols_in + sx) * a.tb;
            }
            klist[i * 64 + lane] = (uint32_t)off * 2u;
        }
    };
    int cols0[BULK_LOADS];
    load_cols(0, cols0);   // in flight while the input box is staged
    // so are the weight operands of the first CONV_PD steps.  Buffer loads with the step in
    // the lane offset, which the hardware checks against the descriptor's size (the scalar
    // offset is not checked): a step beyond the group's reads as zero, so no load is conditional
    const __amdgpu_buffer_rsrc_t val_rsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<half8*>(a.A.values + (long)sbeg * RB * 64), 0, nsteps * RB * 1024, GATHER_BUFFER_FLAGS);
    auto load_w = [&](int s, int rb) __attribute__((always_inline)) {
        return __builtin_bit_cast(half8, __builtin_amdgcn_raw_buffer_load_b128(
            val_rsrc, lane * 16 + (s * RB + rb) * 1024, 0, 0));
    };
    half8 w[CONV_PD][RB];
#pragma unroll
    for (int u = 0; u < CONV_PD; ++u) {
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) w[u][rb] = load_w(u, rb);
        __builtin_amdgcn_sched_barrier(0);   // sets in issue order: the loop's wait counts assume set 0 is the oldest
    }

    // ---- stage the input box: element (c, iy, ix, bb) at xin[c*plane + (iy*cols_in + ix)*tb + bb]
    // Branch-free: the input sits behind a buffer descriptor, an element outside the image
    // (padding, ragged boxes) or a channel beyond C gets an offset past its end and reads as
    // zero; a channel beyond C is written onto the all-zero plane, which is channel C.
    const __amdgpu_buffer_rsrc_t in_rsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<_Float16*>(a.in), 0, (int)a.in_bytes_total, GATHER_BUFFER_FLAGS);
    constexpr unsigned IN_PAST_END = 0xfffffff0u;
    const unsigned isC2 = (unsigned)a.isC * 2u;
    if constexpr (SP) {
        // Two elements that are neighbours in memory per load - along x (NCHW) or along the batch
        // (CHWN).  The host has made sure that a pair is 4-byte aligned and lies inside or outside
        // the image as a whole (even image width / batch, even box origin).  When a channel's
        // pairs fill half a wavefront or less, the lanes left over take further channels.
        const int plane2 = plane >> 1;
        const int lpp = plane2 <= 8 ? 8 : plane2 <= 16 ? 16 : plane2 <= 32 ? 32 : 64;   // lanes per plane
        const int subs = 64 / lpp, sub = lane / lpp;
        const int vwave = wave * subs + sub, vwaves = CONV_GW * subs;
        const int half_step = a.b_fast ? 1 : a.tb;          // LDS distance of a pair's elements
        for (int p2 = lane & (lpp - 1); p2 < plane2; p2 += lpp) {
            int iy, ix, bb;
            if (a.b_fast) {
                const int q = conv_div(p2, a.m_tb2);
                bb = 2 * (p2 - q * (a.tb >> 1));
                iy = conv_div(q, a.m_cols_in); ix = q - iy * a.cols_in;
            } else {
                const int q = conv_div(p2, a.m_tb);
                bb = p2 - q * a.tb;
                iy = conv_div(q, a.m_cols2); ix = 2 * (q - iy * (a.cols_in >> 1));
            }
            const int p = (iy * a.cols_in + ix) * a.tb + bb;   // the pair's first element
            const int yy = iy0 + iy, xx = ix0 + ix, b = b0 + bb;
            const bool inside = yy >= 0 && yy < a.H && xx >= 0 && xx < a.W && b < a.B;
            const unsigned base = (unsigned)(b * a.isB + yy * a.isH + xx * a.isW) * 2u;
            constexpr int MLP = 16;   // loads in flight per lane
            for (int c0 = vwave; c0 < a.C; c0 += vwaves * MLP) {
                unsigned v[MLP];
#pragma unroll
                for (int j = 0; j < MLP; ++j) {
                    const int c = c0 + j * vwaves;
                    const unsigned off = (inside && c < a.C) ? base + (unsigned)c * isC2 : IN_PAST_END;
                    v[j] = __builtin_amdgcn_raw_buffer_load_b32(in_rsrc, (int)off, 0, 0);
                }
#pragma unroll
                for (int j = 0; j < MLP; ++j) {
                    const int c = c0 + j * vwaves;
                    unsigned short* dst = reinterpret_cast<unsigned short*>(xin) + (c < a.C ? c : a.C) * plane + p;
                    dst[0] = (unsigned short)(v[j] & 0xffffu);
                    dst[half_step] = (unsigned short)(v[j] >> 16);
                }
            }
            if (vwave == 0) {   // the all-zero plane
                xin[zero_off + p] = (_Float16)0.f;
                xin[zero_off + p + half_step] = (_Float16)0.f;
            }
        }
    } else
    for (int p = lane; p < plane; p += 64) {
        const int q = conv_div(p, a.m_tb), bb = p - q * a.tb;
        const int iy = conv_div(q, a.m_cols_in), ix = q - iy * a.cols_in;
        const int yy = iy0 + iy, xx = ix0 + ix, b = b0 + bb;
        const bool inside = yy >= 0 && yy < a.H && xx >= 0 && xx < a.W && b < a.B;
        const unsigned base = (unsigned)(b * a.isB + yy * a.isH + xx * a.isW) * 2u;
        constexpr int MLP = 16;   // loads in flight per lane
        for (int c0 = wave; c0 < a.C; c0 += CONV_GW * MLP) {
            unsigned short v[MLP];
#pragma unroll
            for (int j = 0; j < MLP; ++j) {
                const int c = c0 + j * CONV_GW;
                const unsigned off = (inside && c < a.C) ? base + (unsigned)c * isC2 : IN_PAST_END;
                v[j] = __builtin_amdgcn_raw_buffer_load_b16(in_rsrc, (int)off, 0, 0);
            }
#pragma unroll
            for (int j = 0; j < MLP; ++j) {
                const int c = c0 + j * CONV_GW;
                reinterpret_cast<unsigned short*>(xin)[(c < a.C ? c : a.C) * plane + p] = v[j];
            }
        }
        if (wave == 0) xin[zero_off + p] = (_Float16)0.f;   // the all-zero plane
    }
    store_koff(cols0, nsteps);
    __syncthreads();

    // ---- this lane's output positions: n' = POS*(ts*NTI + t) + lane%POS
    const int npos = a.tb * a.th * a.tw;
    int noff[NTI], ooff[NTI];
    bool live[NTI];
#pragma unroll
    for (int t = 0; t < NTI; ++t) {
        const int n = POS * (ts * NTI + t) + (lane & (POS - 1));
        int bb, yy, xx;
        if (a.b_fast) {
            const int q = conv_div(n, a.m_tb);
            bb = n - q * a.tb; yy = conv_div(q, a.m_tw); xx = q - yy * a.tw;
        } else {
            const int q = conv_div(n, a.m_tw);
            xx = n - q * a.tw; bb = conv_div(q, a.m_th); yy = q - bb * a.th;
        }
        const int b = b0 + bb, y = y0 + yy, x = x0 + xx;
        live[t] = n < npos && b < a.B && y < a.Ho && x < a.Wo;
        noff[t] = live[t] ? 2 * ((yy * a.sh * a.cols_in + xx * a.sw + dx) * a.tb + bb) : 0;   // in bytes
        ooff[t] = live[t] ? (int)(b * a.osB + y * a.osH + x * a.osW) : 0;
    }

    floatx16 acc[SMALL ? 1 : RB][SMALL ? 1 : NTI];
    floatx4 acc16[SMALL ? NTI : 1];
    if (SMALL) {
#pragma unroll
        for (int t = 0; t < NTI; ++t) acc16[t] = floatx4{0, 0, 0, 0};
    } else {
#pragma unroll
        for (int rb = 0; rb < RB; ++rb)
#pragma unroll
            for (int t = 0; t < NTI; ++t)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[rb][t][r] = 0.f;
    }

    if (nsteps > 0) {
        const int kblock = lane / POS;
        typedef unsigned uint8v __attribute__((ext_vector_type(8)));
        const uint8v* kl = reinterpret_cast<const uint8v*>(klist) + kblock;   // 8 slots of this lane's block

        // StitchTile of one step: 8 reduction indices x up to NT positions per lane.  The
        // list entry of a step is read one step before its gathers go out, the gathers one
        // step before their product, so a step waits for one LDS round trip at most.  The
        // loop is straight-line code over whole batches of CONV_PD steps: a step past the
        // group's last one multiplies zero weights (the descriptor's range) with the zero
        // plane (the list's filler), and every load is unconditional, which keeps the
        // register sets static and the wait counts exact.
        auto read_list = [&](int s) __attribute__((always_inline)) { return kl[(s & (BULK - 1)) * KBLOCKS]; };
        static_assert(CONV_PD % 2 == 0, "entries and tiles alternate between two register sets");
        // Order inside a step (pinned, or the scheduler moves a step's gathers next to their use and
        // every step waits for two LDS round trips): the halves gathered a step ago become this
        // step's operand; the products go out; the next step's gathers go out, then the list entry of
        // the step after that, then the refill of this step's weight registers.  LDS results come
        // back in order, so the only wait a step has is for gathers that had a whole step to land.
        uint8v ko[2];                       // list entry of step j in ko[j & 1]
        unsigned short raw[2][NTI][8];       // gathered halves of step j in raw[j & 1]
        auto gather_raw = [&](const uint8v& e8, unsigned short (&r)[NTI][8]) __attribute__((always_inline)) {
#pragma unroll
            for (int t = 0; t < NTI; ++t)
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    r[t][e] = *reinterpret_cast<const unsigned short*>(reinterpret_cast<const char*>(xin) + (e8[e] + (unsigned)noff[t]));
        };
        ko[0] = read_list(0);
        gather_raw(ko[0], raw[0]);
        ko[1] = read_list(1);
        const int nsteps_r = (nsteps + CONV_PD - 1) / CONV_PD * CONV_PD;
        for (int s0 = 0; s0 < nsteps_r; s0 += CONV_PD) {
#pragma unroll
            for (int u = 0; u < CONV_PD; ++u) {
                const int s = s0 + u;
                if ((u + 2) % CONV_PD == 0) {
                    // the entry read below may open the next bulk of column indices; every entry
                    // of the old bulk is in registers by now
                    if (((s + 2) & (BULK - 1)) == 0 && s + 2 < nsteps) {   // uniform
                        // Rare (every BULK steps): what it needs of the arguments is read again from
                        // the kernel-argument segment here, so that none of it occupies scalar
                        // registers across the loop (they are short: the loop had spills to lanes).
                        typedef const __attribute__((address_space(4))) ConvArgs* karg_ptr;
                        karg_ptr ka = (karg_ptr)__builtin_amdgcn_kernarg_segment_ptr();
                        asm volatile("" : "+s"(ka));
                        const int k_tb = ka->tb, k_cols = ka->cols_in, k_S = ka->S;
                        const int k_plane = ka->rows_in * k_cols * k_tb, k_RS = ka->R * k_S;
                        const int k_zero = ka->C * k_plane;
                        const unsigned long long k_mRS = ka->m_RS, k_mS = ka->m_S;
                        const int32_t* cp = ka->A.col_idx + ((long)sbeg + (s + 2)) * TK;
                        const int avail = (nsteps - (s + 2)) * TK;
                        const int wanted = (nsteps - (s + 2) + CONV_PD + 2) * TK;
                        int cols[BULK_LOADS];
#pragma unroll
                        for (int i = 0; i < BULK_LOADS; ++i) {
                            const int j = i * 64 + lane;
                            cols[i] = j < avail ? cp[j] : -1;
                        }
                        SHFLBW_WAVE_LDS_SYNC();   // reads of the old list are over
#pragma unroll
                        for (int i = 0; i < BULK_LOADS; ++i) {
                            if (i * 64 >= wanted) break;   // uniform
                            const int k = cols[i];
                            int off = k_zero;
                            if (k >= 0) {
                                const int c = conv_div(k, k_mRS), rs = k - c * k_RS;
                                const int r = conv_div(rs, k_mS), sx = rs - r * k_S;
                                off = c * k_plane + (r * k_cols + sx) * k_tb;
                            }
                            klist[i * 64 + lane] = (uint32_t)off * 2u;
                        }
                        SHFLBW_WAVE_LDS_SYNC();
                    }
                }
                half8 x[NTI];
#pragma unroll
                for (int t = 0; t < NTI; ++t) {
                    typedef unsigned short us8 __attribute__((ext_vector_type(8)));
                    const us8 v = {raw[u & 1][t][0], raw[u & 1][t][1], raw[u & 1][t][2], raw[u & 1][t][3],
                                   raw[u & 1][t][4], raw[u & 1][t][5], raw[u & 1][t][6], raw[u & 1][t][7]};
                    x[t] = __builtin_bit_cast(half8, v);
                }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int t = 0; t < NTI; ++t) {
                    if (SMALL) {
                        acc16[t] = mma16<BF>(x[t], w[u][0], acc16[t]);
                    } else {
#pragma unroll
                        for (int rb = 0; rb < RB; ++rb)
                            acc[rb][t] = mma32<BF>(x[t], w[u][rb], acc[rb][t]);
                    }
                }
                gather_raw(ko[(u + 1) & 1], raw[(u + 1) & 1]);   // step s + 1
                __builtin_amdgcn_sched_barrier(0);
                ko[u & 1] = read_list(s + 2);
#pragma unroll
                for (int rb = 0; rb < RB; ++rb) w[u][rb] = load_w(s + CONV_PD, rb);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    }
    __syncthreads();   // every wavefront is done reading the staged input; its LDS becomes scratch
    if (!have_group) return;

    // ---- reordered write-back
    float* ep = reinterpret_cast<float*>(conv_smem + wave * CONV_SCRATCH);
    OutT* out = static_cast<OutT*>(a.out);
    const int32_t* rows_g = a.A.row_indices + (long)g * V;
    if (SMALL) {
        const long my_row = (long)rows_g[lane & 15] * a.osM;
#pragma unroll
        for (int t = 0; t < NTI; ++t) {
            // accumulator register j of lane l: position 4*(l/16) + j, stored row l%16
#pragma unroll
            for (int j = 0; j < 4; ++j) ep[(lane & 15) * 17 + 4 * (lane >> 4) + j] = acc16[t][j];
            SHFLBW_WAVE_LDS_SYNC();
            // the four 16-lane blocks take four stored rows per pass, one position each
#pragma unroll
            for (int i = 0; i < 16; i += 4) {
                const int row = i + (lane >> 4);
                const float v = ep[row * 17 + (lane & 15)];
                const long ro = __shfl(my_row, row, 64);
                if (live[t]) out[ro + ooff[t]] = (OutT)v;
            }
            SHFLBW_WAVE_LDS_SYNC();
        }
        return;
    }
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        const long my_row = (long)rows_g[rb * 32 + (lane & 31)] * a.osM;
#pragma unroll
        for (int t = 0; t < NTI; ++t) {
            {
                // accumulator register r of lane l: position 8*(r/4) + 4*(l/32) + r%4, stored row l%32
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    ep[(lane & 31) * 33 + 8 * (r / 4) + 4 * (lane >> 5) + (r % 4)] = acc[rb][t][r];
                SHFLBW_WAVE_LDS_SYNC();
                // lanes 0..31 and 32..63 take two stored rows per pass, one position each
#pragma unroll 4
                for (int i = 0; i < 32; i += 2) {
                    const int row = i + (lane >> 5);
                    const float v = ep[row * 33 + (lane & 31)];
                    // the two rows' offsets through scalar registers (my_row fits 32 bits: the host checks the tensor's size)
                    const int r0 = __builtin_amdgcn_readlane((int)my_row, i), r1 = __builtin_amdgcn_readlane((int)my_row, i + 1);
                    const long ro = lane < 32 ? r0 : r1;
                    if (live[t]) out[ro + ooff[t]] = (OutT)v;
                }
                SHFLBW_WAVE_LDS_SYNC();
            }
        }
    }
}

}  // namespace shflbw
