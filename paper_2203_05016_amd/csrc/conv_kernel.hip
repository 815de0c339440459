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
// element inside the box).  koff for all K reduction indices is tabulated in
// LDS by the workgroup, noff lives in registers.  A padded slot of a k-step
// (column index -1) points at an extra all-zero channel plane.
//
// Algorithm 1's parts: BulkLoadMeta = the 16 column indices and the weight
// operand of the next k-step are fetched while the current one is multiplied;
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
    int gblocks;              // blocks of CONV_GW groups
    int in_bytes;             // LDS bytes reserved for the staged input (and the scratch)
};

template <int V, typename OutT>
__global__ __launch_bounds__(64 * CONV_GW) void shflbw_conv_kernel(ConvArgs a)
{
    constexpr int RB = V / 32;
    constexpr int NT = CONV_TN / 32;
    extern __shared__ __attribute__((aligned(16))) char conv_smem[];
    _Float16* xin = reinterpret_cast<_Float16*>(conv_smem);
    uint16_t* koff = reinterpret_cast<uint16_t*>(conv_smem + a.in_bytes);

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

    // which box, which block of groups
    int box = blockIdx.x / a.gblocks;
    const int gb = blockIdx.x - box * a.gblocks;
    const int bx = box % a.nx; box /= a.nx;
    const int by = box % a.ny; box /= a.ny;
    const int b0 = box * a.tb, y0 = by * a.th, x0 = bx * a.tw;
    const int plane = a.rows_in * a.cols_in * a.tb;   // staged elements per channel
    const int iy0 = y0 * a.sh - a.ph, ix0 = x0 * a.sw - a.pw;

    // ---- stage the input box: element (c, iy, ix, bb) at xin[c*plane + (iy*cols_in + ix)*tb + bb]
    for (int p = lane; p < plane; p += 64) {
        const int bb = p % a.tb;
        const int q = p / a.tb;
        const int ix = q % a.cols_in, iy = q / a.cols_in;
        const int yy = iy0 + iy, xx = ix0 + ix, b = b0 + bb;
        const bool inside = yy >= 0 && yy < a.H && xx >= 0 && xx < a.W && b < a.B;
        const _Float16* src = a.in + (inside ? b * a.isB + yy * a.isH + xx * a.isW : 0);
#pragma unroll 4
        for (int c = wave; c < a.C; c += CONV_GW) {
            _Float16 v = (_Float16)0.f;
            if (inside) v = src[c * a.isC];
            xin[c * plane + p] = v;
        }
        if (wave == 0) xin[a.C * plane + p] = (_Float16)0.f;   // the all-zero plane
    }
    // ---- tabulate koff[k] for k = (c*R + r)*S + s
    {
        const int RS = a.R * a.S;
        for (int k = tid; k < a.K; k += 64 * CONV_GW) {
            const int c = k / RS, rs = k - c * RS;
            const int r = rs / a.S, s = rs - r * a.S;
            koff[k] = (uint16_t)(c * plane + (r * a.cols_in + s) * a.tb);
        }
    }
    __syncthreads();

    // ---- this lane's output positions: n' = 32*t + lane%32
    const int npos = a.tb * a.th * a.tw;
    int noff[NT], ooff[NT];
    bool live[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        const int n = 32 * t + (lane & 31);
        int bb, yy, xx;
        if (a.b_fast) { bb = n % a.tb; const int q = n / a.tb; xx = q % a.tw; yy = q / a.tw; }
        else { xx = n % a.tw; const int q = n / a.tw; yy = q % a.th; bb = q / a.th; }
        const int b = b0 + bb, y = y0 + yy, x = x0 + xx;
        live[t] = n < npos && b < a.B && y < a.Ho && x < a.Wo;
        noff[t] = live[t] ? (yy * a.sh * a.cols_in + xx * a.sw) * a.tb + bb : 0;
        ooff[t] = live[t] ? (int)(b * a.osB + y * a.osH + x * a.osW) : 0;
    }
    const int nt_live = (npos + 31) / 32;   // uniform: instruction tiles that hold any position

    const int g = gb * CONV_GW + wave;
    const bool have_group = g < a.A.G;
    floatx16 acc[RB][NT];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[rb][t][r] = 0.f;

    if (have_group) {
        const int sbeg = a.A.step_ptr[g];
        const int nsteps = a.A.step_ptr[g + 1] - sbeg;
        const int khalf = lane >> 5;
        const intx4* colp = reinterpret_cast<const intx4*>(a.A.col_idx + (long)sbeg * 16 + 8 * khalf);
        const half8* valp = a.A.values + (long)sbeg * RB * 64 + lane;
        const int zero_off = a.C * plane;

        intx4 c_lo = {-1, -1, -1, -1}, c_hi = {-1, -1, -1, -1};
        half8 w[RB];
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) w[rb] = half8{0, 0, 0, 0, 0, 0, 0, 0};
        if (nsteps > 0) {
            c_lo = colp[0]; c_hi = colp[1];
#pragma unroll
            for (int rb = 0; rb < RB; ++rb) w[rb] = valp[rb * 64];
        }
        for (int s = 0; s < nsteps; ++s) {
            // BulkLoadMeta for the next step (clamped, so the loads are unconditional)
            const int sn = s + 1 < nsteps ? s + 1 : s;
            const intx4 n_lo = colp[(long)sn * 4], n_hi = colp[(long)sn * 4 + 1];
            half8 wn[RB];
#pragma unroll
            for (int rb = 0; rb < RB; ++rb) wn[rb] = valp[((long)sn * RB + rb) * 64];

            int ko[8];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                ko[e] = c_lo[e] < 0 ? zero_off : (int)koff[c_lo[e]];
                ko[4 + e] = c_hi[e] < 0 ? zero_off : (int)koff[c_hi[e]];
            }
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                if (t < nt_live) {
                    half8 x;
#pragma unroll
                    for (int e = 0; e < 8; ++e) x[e] = xin[ko[e] + noff[t]];
#pragma unroll
                    for (int rb = 0; rb < RB; ++rb)
                        acc[rb][t] = __builtin_amdgcn_mfma_f32_32x32x16_f16(x, w[rb], acc[rb][t], 0, 0, 0);
                }
            }
            c_lo = n_lo; c_hi = n_hi;
#pragma unroll
            for (int rb = 0; rb < RB; ++rb) w[rb] = wn[rb];
        }
    }
    __syncthreads();   // every wavefront is done reading the staged input; its LDS becomes scratch
    if (!have_group) return;

    // ---- reordered write-back
    float* ep = reinterpret_cast<float*>(conv_smem + wave * CONV_SCRATCH);
    OutT* out = static_cast<OutT*>(a.out);
    const int32_t* rows_g = a.A.row_indices + (long)g * V;
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        const long my_row = (long)rows_g[rb * 32 + (lane & 31)] * a.osM;
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            if (t < nt_live) {
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
                    const long ro = __shfl(my_row, row, 64);
                    if (live[t]) out[ro + ooff[t]] = (OutT)v;
                }
                SHFLBW_WAVE_LDS_SYNC();
            }
        }
    }
}

}  // namespace shflbw
