// Shared-slab kernel for the Shfl-BW product on gfx950 (CDNA4).
//
// A workgroup owns GW row groups (one wavefront each) x 128 output columns.
// All of its wavefronts need rows of the same 128-column slab of X, each a
// different subset, so the slab is streamed through LDS once, DENSE, in
// chunks of KC = 128 rows, and the stitching of Section 4.3 happens at
// LDS-read time: the transposing LDS read takes one address per lane, so a
// wavefront simply points its lanes at the rows its column indices name.
// HBM/L2 -> LDS traffic is then K*128*2 bytes per GW groups instead of
// k_g*128*2 bytes per group, loads are fully coalesced, and nothing is
// written to LDS per wavefront.
//
// Residency.  Three LDS stages hold chunks c-1 and c (readable) while chunk
// c+1 is being written from registers and chunk c+2, c+3 are in flight from
// memory.  The packed matrix is cut into k-steps that never span more than
// two adjacent chunks, and iter_ptr lists, per group, which steps have their
// last column in chunk c: those run in iteration c.  One workgroup barrier
// per iteration.
//
// Algorithm 1's parts: BulkLoadMeta = column indices and weight tiles of
// the next steps prefetched into registers independent of the chunk loop;
// StitchTile = chunk streaming + gathered transposed reads; WarpMMA =
// v_mfma_f32_32x32x16_f16 (16x16x32 for V = 16) with X^T as first operand;
// ReorderedWriteBack = accumulators through LDS, 128-byte row segments stored
// to the rows named by row_indices.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

#include "gather_kernel.hip"

namespace shflbw {

constexpr int SLAB_TN = 128;                       // output columns per workgroup
constexpr int SLAB_STAGES = 3;
constexpr int SLAB_ROW_BYTES = SLAB_TN * 2;        // 256 B per staged row
constexpr int SLAB_STAGE_BYTES = SLAB_KC * SLAB_ROW_BYTES;
constexpr int SLAB_ZERO_ROW = SLAB_STAGES * SLAB_KC;  // index of the all-zero row
constexpr int SLAB_LDS_BYTES = (SLAB_ZERO_ROW + 1) * SLAB_ROW_BYTES;

// Position of 16-byte chunk q of staged row r inside the row: rows that land
// on the same banks get their chunks rotated against each other.
__device__ __forceinline__ int slab_swizzle(int row, int q) { return q ^ ((row & 7) << 1); }

struct SlabArgs {
    PackedView A;
    const int32_t* iter_ptr;  // G*(C+1)
    const _Float16* X;
    void* Y;
    long ldx, ldy, N;
    int K, C;
    int n_tiles, gblocks;     // 128-column tiles, blocks of GW groups
};

template <int V, int GW, typename OutT>
__global__ __launch_bounds__(64 * GW) void shflbw_slab_kernel(SlabArgs a)
{
    constexpr bool SMALL = (V == 16);
    constexpr int TK = SMALL ? 32 : 16;
    constexpr int RB = SMALL ? 1 : V / 32;
    constexpr int TILE_N = SMALL ? 16 : 32;
    constexpr int NT = SLAB_TN / TILE_N;
    constexpr int THREADS = 64 * GW;
    constexpr int ITEMS = SLAB_KC * 16 / THREADS;  // 16-byte pieces per thread per chunk
    static_assert(ITEMS * THREADS == SLAB_KC * 16, "chunk must divide evenly");
    __shared__ __attribute__((aligned(256))) char smem[SLAB_LDS_BYTES];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

    // Workgroups are dealt round-robin to the 8 XCDs; the blocks that share a
    // slab of X (same column tile, different group blocks) are given ids that
    // land on the same XCD one after the other, so its L2 serves the re-reads.
    const int wg = blockIdx.x;
    const int xcd = wg & 7, slot = wg >> 3;
    const int gb = slot % a.gblocks;
    const int nt = (slot / a.gblocks) * 8 + xcd;
    if (nt >= a.n_tiles) return;  // uniform for the whole workgroup
    const long n0 = (long)nt * SLAB_TN;
    const int g = gb * GW + wave;
    const bool have_group = g < a.A.G;

    int sbeg = 0, nsteps = 0;
    const int32_t* my_iter = a.iter_ptr;
    if (have_group) {
        sbeg = a.A.step_ptr[g];
        nsteps = a.A.step_ptr[g + 1] - sbeg;
        my_iter = a.iter_ptr + (long)g * (a.C + 1);
    }

    // ---- chunk loader: thread t moves pieces t, t+THREADS, ... of a chunk;
    // piece p is row p/16, 16-byte column chunk p%16.
    half8 xs[2][ITEMS];
    auto issue_chunk = [&](int c, half8 (&dst)[ITEMS]) {
#pragma unroll
        for (int i = 0; i < ITEMS; ++i) {
            const int p = tid + i * THREADS;
            const int row = c * SLAB_KC + (p >> 4);
            const long n = n0 + (p & 15) * 8;
            half8 v = {0, 0, 0, 0, 0, 0, 0, 0};
            if (row < a.K && n < a.N) v = *reinterpret_cast<const half8*>(a.X + (long)row * a.ldx + n);
            dst[i] = v;
        }
    };
    auto write_chunk = [&](int c, const half8 (&src)[ITEMS]) {
        char* stage = smem + (c % SLAB_STAGES) * SLAB_STAGE_BYTES;
#pragma unroll
        for (int i = 0; i < ITEMS; ++i) {
            const int p = tid + i * THREADS;
            const int r = p >> 4;
            *reinterpret_cast<half8*>(stage + r * SLAB_ROW_BYTES + (slab_swizzle(r, p & 15) << 4)) = src[i];
        }
    };

    // ---- per-step prefetch state (two register sets, picked by step parity)
    constexpr int NC = SMALL ? 2 : 2;  // column indices a lane needs per step (one per transposed read)
    int cols[2][NC];
    half8 wr[2][RB];
    const int bl = lane >> 4, il = lane & 15;
    // k index of this lane's first transposed read inside a step
    const int kq = SMALL ? (8 * bl + (il >> 2)) : (8 * (bl >> 1) + (il >> 2));
    // 16-byte chunk (before the tile offset) and byte inside it that this lane reads
    const int qc = SMALL ? ((il & 3) >> 1) : (2 * (bl & 1) + ((il & 3) >> 1));
    const int qbyte = (il & 1) << 3;

    auto load_meta = [&](int s, int (&c)[NC], half8 (&w)[RB]) {
        const int32_t* p = a.A.col_idx + (long)(sbeg + s) * TK + kq;
        c[0] = p[0];
        c[1] = p[4];
        const half8* q = a.A.values + ((long)(sbeg + s) * RB) * 64 + lane;
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) w[rb] = q[rb * 64];
    };

    floatx16 acc32[SMALL ? 1 : RB][SMALL ? 1 : NT];
    floatx4 acc16[SMALL ? NT : 1];
    if (SMALL) {
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

    auto do_step = [&](const int (&c)[NC], const half8 (&w)[RB]) {
        int base[2], swz[2];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int row = (c[h] < 0) ? SLAB_ZERO_ROW : (c[h] % (SLAB_STAGES * SLAB_KC));
            base[h] = row * SLAB_ROW_BYTES + qbyte;
            swz[h] = (row & 7) << 1;
        }
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            const int q = (SMALL ? 2 * t : 4 * t) + qc;
            short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                (lds_short4_ptr)(smem + base[0] + ((q ^ swz[0]) << 4)));
            short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                (lds_short4_ptr)(smem + base[1] + ((q ^ swz[1]) << 4)));
            half4 l4 = __builtin_bit_cast(half4, lo), h4 = __builtin_bit_cast(half4, hi);
            half8 x = {l4[0], l4[1], l4[2], l4[3], h4[0], h4[1], h4[2], h4[3]};
            if (SMALL) {
                acc16[t] = __builtin_amdgcn_mfma_f32_16x16x32_f16(x, w[0], acc16[t], 0, 0, 0);
            } else {
#pragma unroll
                for (int rb = 0; rb < RB; ++rb)
                    acc32[rb][t] = __builtin_amdgcn_mfma_f32_32x32x16_f16(x, w[rb], acc32[rb][t], 0, 0, 0);
            }
        }
    };

    // ---- prologue
    if (tid < 16) *reinterpret_cast<half8*>(smem + SLAB_ZERO_ROW * SLAB_ROW_BYTES + tid * 16) =
        half8{0, 0, 0, 0, 0, 0, 0, 0};
    const int C = a.C;
    {
        half8 first[ITEMS];
        issue_chunk(0, first);
        if (1 < C) issue_chunk(1, xs[1]);
        if (2 < C) issue_chunk(2, xs[0]);
        if (0 < nsteps) load_meta(0, cols[0], wr[0]);
        if (1 < nsteps) load_meta(1, cols[1], wr[1]);
        write_chunk(0, first);
    }
    int s = 0;
    int it_end = have_group ? my_iter[1] : 0;

    auto iteration = [&](int c, half8 (&write_set)[ITEMS], bool) {
        __syncthreads();  // chunk c is complete; nobody still reads chunk c-2
        if (c + 1 < C) write_chunk(c + 1, write_set);
        if (c + 3 < C) issue_chunk(c + 3, write_set);
        const int s_end = it_end;
        if (have_group && c + 2 <= C) it_end = my_iter[(c + 2 <= C) ? c + 2 : C];
        for (; s < s_end; ++s) {
            if (s & 1) {
                do_step(cols[1], wr[1]);
                if (s + 2 < nsteps) load_meta(s + 2, cols[1], wr[1]);
            } else {
                do_step(cols[0], wr[0]);
                if (s + 2 < nsteps) load_meta(s + 2, cols[0], wr[0]);
            }
        }
    };
    // chunk x travels in register set x%2... chunk 1 -> xs[1], chunk 2 -> xs[0]
    for (int c = 0; c < C; c += 2) {
        iteration(c, xs[1], true);
        if (c + 1 < C) iteration(c + 1, xs[0], true);
    }
    __syncthreads();  // all transposed reads done: the stages become epilogue scratch

    // ---- reordered write-back: per wavefront, 32 (16) stored rows x 128 bytes per pass
    if (!have_group) return;
    constexpr int OUT16 = 16 / (int)sizeof(OutT);        // values per 16 bytes
    constexpr int CW = 128 / (int)sizeof(OutT);           // columns per pass: 64 (fp16) or 32 (fp32)
    constexpr int PASSES = SLAB_TN / CW;
    constexpr int TPP = CW / TILE_N;                      // instruction tiles per pass
    constexpr int EP = CW + OUT16;                        // pitch in OutT units (144 bytes)
    constexpr int ROWS_E = SMALL ? 16 : 32;
    constexpr int WAVE_BYTES = 32 * 144;
    static_assert(GW * WAVE_BYTES <= SLAB_STAGES * SLAB_STAGE_BYTES, "epilogue scratch must fit");
    OutT* ep = reinterpret_cast<OutT*>(smem + wave * WAVE_BYTES);
    const int erow = lane >> 3, echunk = lane & 7;        // 8 lanes x 16 B per row
    const int32_t* rows_g = a.A.row_indices + (long)g * V;
    typedef OutT vec4 __attribute__((ext_vector_type(4)));
    typedef OutT vecw __attribute__((ext_vector_type(OUT16)));

#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
#pragma unroll
        for (int pass = 0; pass < PASSES; ++pass) {
#pragma unroll
            for (int tt = 0; tt < TPP; ++tt) {
                const int t = pass * TPP + tt;
                if (SMALL) {
                    vec4 v = {(OutT)acc16[t][0], (OutT)acc16[t][1], (OutT)acc16[t][2], (OutT)acc16[t][3]};
                    *reinterpret_cast<vec4*>(ep + (lane & 15) * EP + 16 * tt + 4 * (lane >> 4)) = v;
                } else {
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        vec4 v = {(OutT)acc32[rb][t][4 * q + 0], (OutT)acc32[rb][t][4 * q + 1],
                                  (OutT)acc32[rb][t][4 * q + 2], (OutT)acc32[rb][t][4 * q + 3]};
                        *reinterpret_cast<vec4*>(ep + (lane & 31) * EP + 32 * tt + 8 * q + 4 * (lane >> 5)) = v;
                    }
                }
            }
            SHFLBW_WAVE_LDS_SYNC();
#pragma unroll
            for (int i = 0; i < ROWS_E / 8; ++i) {
                const int row = i * 8 + erow;
                vecw v = *reinterpret_cast<const vecw*>(ep + row * EP + echunk * OUT16);
                const int orig = rows_g[rb * 32 + row];
                const long n = n0 + pass * CW + echunk * OUT16;
                if (n < a.N)
                    *reinterpret_cast<vecw*>(static_cast<OutT*>(a.Y) + (long)orig * a.ldy + n) = v;
            }
            SHFLBW_WAVE_LDS_SYNC();
        }
    }
}

}  // namespace shflbw
