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
// Residency.  A ring of four LDS stages: chunks c-1 and c are readable in
// iteration c while chunks c+1 and c+2 arrive through direct global-to-LDS
// loads (no register round trip).  The ring position of column k is
// k mod 512, so a wavefront turns a column index into an LDS row with one
// AND.  The packed matrix is cut into k-steps that never span more than two
// adjacent chunks, and iter_ptr lists, per group, which steps have their last
// column in chunk c: those run in iteration c.  One workgroup barrier per
// iteration.
//
// Algorithm 1's parts: BulkLoadMeta = column indices and weight tile of the
// next step prefetched into registers, independent of the chunk loop;
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
constexpr int SLAB_STAGES = 4;                     // power of two: ring row = column & (STAGES*KC-1)
constexpr int SLAB_ROW_BYTES = SLAB_TN * 2;        // 256 B per staged row
constexpr int SLAB_STAGE_BYTES = SLAB_KC * SLAB_ROW_BYTES;
constexpr int SLAB_ZERO_ROW = SLAB_STAGES * SLAB_KC;  // index of the all-zero row
constexpr int SLAB_LDS_BYTES = (SLAB_ZERO_ROW + 1) * SLAB_ROW_BYTES;
static_assert((SLAB_STAGES & (SLAB_STAGES - 1)) == 0 && (SLAB_KC & (SLAB_KC - 1)) == 0, "ring must be a power of two");

typedef __attribute__((address_space(3))) void* lds_void_ptr;
typedef __attribute__((address_space(1))) const void* global_void_ptr;

// s_waitcnt immediates for gfx9-family encodings: vmcnt in bits [3:0] and
// [15:14], expcnt [6:4] and lgkmcnt [11:8] left at "do not wait".
#define SHFLBW_WAIT_VMCNT0() __builtin_amdgcn_s_waitcnt(0x0F70)

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
    constexpr int IPW = SLAB_KC / 4 / GW;  // direct-to-LDS loads (4 rows each) per wavefront per chunk
    static_assert(IPW * GW * 4 == SLAB_KC, "chunk must divide evenly");
    __shared__ __attribute__((aligned(1024))) char smem[SLAB_LDS_BYTES];

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

    // ---- chunk loader.  One direct-to-LDS load moves 64 x 16 bytes = 4 staged
    // rows; lane L lands in LDS slot L of that kilobyte, so it fetches the
    // 16-byte column chunk that the swizzle assigns to its slot.  Rows beyond K
    // and columns beyond N are skipped: their LDS bytes are never used for a
    // stored result.
    const int lrow = lane >> 4;                       // row inside the 4-row piece
    const int lpos = lane & 15;                       // slot inside the row
    auto issue_chunk = [&](int c) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < IPW; ++i) {
            const int r = 4 * (wave * IPW + i) + lrow;            // row inside the chunk
            const int q = lpos ^ ((r & 7) << 1);                  // column chunk for this slot
            const int row = c * SLAB_KC + r;
            const long n = n0 + q * 8;
            char* dst = smem + (c & (SLAB_STAGES - 1)) * SLAB_STAGE_BYTES + 4 * (wave * IPW + i) * SLAB_ROW_BYTES;
            if (row < a.K && n < a.N)
                __builtin_amdgcn_global_load_lds((global_void_ptr)(a.X + (long)row * a.ldx + n),
                                                 (lds_void_ptr)dst, 16, 0, 0);
        }
    };

    const int bl = lane >> 4, il = lane & 15;
    // k index of this lane's first transposed read inside a step
    const int kq = SMALL ? (8 * bl + (il >> 2)) : (8 * (bl >> 1) + (il >> 2));
    // 16-byte chunk (before the tile offset) and byte inside it that this lane reads
    const int qc = SMALL ? ((il & 3) >> 1) : (2 * (bl & 1) + ((il & 3) >> 1));
    const int qbyte = (il & 1) << 3;

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

    // ---- prologue
    if (tid < 16) *reinterpret_cast<half8*>(smem + SLAB_ZERO_ROW * SLAB_ROW_BYTES + tid * 16) =
        half8{0, 0, 0, 0, 0, 0, 0, 0};
    const int C = a.C;
    issue_chunk(0);
    if (1 < C) issue_chunk(1);

    // metadata of the next step (column indices of this lane's two transposed
    // reads, weight operand), fetched one step ahead; the index is clamped so
    // the loads are unconditional
    const int last = nsteps > 0 ? nsteps - 1 : 0;
    const int32_t* colp = a.A.col_idx + (long)sbeg * TK + kq;
    const half8* valp = a.A.values + (long)sbeg * RB * 64 + lane;
    int c0n = -1, c1n = -1;
    half8 wn[RB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) wn[rb] = half8{0, 0, 0, 0, 0, 0, 0, 0};
    if (nsteps > 0) {
        c0n = colp[0];
        c1n = colp[4];
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) wn[rb] = valp[rb * 64];
    }

    int s = 0;
    int it_end = have_group ? my_iter[1] : 0;

    for (int c = 0; c < C; ++c) {
        // my pieces of chunk c (issued two iterations ago) and of chunk c+1 have
        // landed; after the barrier everybody's have, and nobody still reads
        // chunk c-2, whose stage chunk c+2 now takes
        SHFLBW_WAIT_VMCNT0();
        __syncthreads();
        if (c + 2 < C) issue_chunk(c + 2);
        const int s_end = it_end;
        if (have_group) it_end = my_iter[(c + 2 <= C) ? c + 2 : C];
        for (; s < s_end; ++s) {
            const int c0 = c0n, c1 = c1n;
            half8 w[RB];
#pragma unroll
            for (int rb = 0; rb < RB; ++rb) w[rb] = wn[rb];
            {
                const int sn = (s + 1 < nsteps) ? s + 1 : last;
                c0n = colp[(long)sn * TK];
                c1n = colp[(long)sn * TK + 4];
#pragma unroll
                for (int rb = 0; rb < RB; ++rb) wn[rb] = valp[((long)sn * RB + rb) * 64];
            }
            const int row0 = (c0 < 0) ? SLAB_ZERO_ROW : (c0 & (SLAB_ZERO_ROW - 1));
            const int row1 = (c1 < 0) ? SLAB_ZERO_ROW : (c1 & (SLAB_ZERO_ROW - 1));
            const int base0 = row0 * SLAB_ROW_BYTES + qbyte, swz0 = (row0 & 7) << 1;
            const int base1 = row1 * SLAB_ROW_BYTES + qbyte, swz1 = (row1 & 7) << 1;
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                const int q = (SMALL ? 2 * t : 4 * t) + qc;
                short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                    (lds_short4_ptr)(smem + base0 + ((q ^ swz0) << 4)));
                short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                    (lds_short4_ptr)(smem + base1 + ((q ^ swz1) << 4)));
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
        }
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
