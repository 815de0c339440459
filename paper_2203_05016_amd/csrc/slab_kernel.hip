// Shared-slab kernel for the Shfl-BW product on gfx950 (CDNA4).
//
// A workgroup owns GW row groups (one compute wavefront each) x 128 output
// columns.  All of its wavefronts need rows of the same 128-column slab of X,
// each a different subset, so the slab is streamed through LDS once, DENSE,
// in chunks of KC = 64 rows, and the stitching of Section 4.3 happens at
// LDS-read time: the transposing LDS read takes one address per lane, so a
// wavefront simply points its lanes at the rows its column indices name.
// HBM/L2 -> LDS traffic is then K*128*2 bytes per GW groups instead of
// k_g*128*2 bytes per group, loads are fully coalesced, and nothing is
// written to LDS per compute wavefront.
//
// Roles.  Four extra wavefronts per workgroup (one per SIMD) do nothing but
// stream chunks with direct global-to-LDS loads.  Their vector-memory queues
// hold only those loads, a fixed number per chunk, so "chunk c has landed" is
// an exact s_waitcnt vmcnt(n); the compute wavefronts never wait on X traffic
// and the loaders never wait on weights.
//
// Residency.  A ring of six 16 KB stages: in iteration c the chunks
// c-3 .. c are readable and c+1, c+2 are in flight.  The ring row of column
// k is k mod 384; the compressor stores it, per lane, in a table next to
// the weights.  The packed matrix is cut into k-steps whose columns span at
// most four adjacent chunks, and iter_ptr lists, per group, which steps have
// their last column in chunk c: those run in iteration c.  One workgroup
// barrier per iteration.
//
// Algorithm 1's parts: BulkLoadMeta = each step's weight tile and lane table
// brought into a per-wavefront LDS ring by direct loads three steps ahead,
// independent of the chunk loop;
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
constexpr int SLAB_STAGES = SLAB_WINDOW + SLAB_LEAD;
constexpr int SLAB_ROW_BYTES = SLAB_TN * 2;        // 256 B per staged row
constexpr int SLAB_STAGE_BYTES = SLAB_KC * SLAB_ROW_BYTES;
constexpr int SLAB_X_BYTES = (SLAB_ZERO_ROW + 1) * SLAB_ROW_BYTES;  // ring + the all-zero row
constexpr int SLAB_LOADERS = 4;                    // loader wavefronts per workgroup
constexpr int SLAB_IPL = SLAB_KC / 4 / SLAB_LOADERS;  // direct loads (4 rows each) per loader per chunk
static_assert(SLAB_IPL * SLAB_LOADERS * 4 == SLAB_KC, "chunk must divide evenly");
static_assert(SLAB_IPL * (SLAB_LEAD - 1) < 16, "vmcnt immediates below use the low four bits only");

typedef __attribute__((address_space(3))) void* lds_void_ptr;
typedef __attribute__((address_space(3))) char* lds_char_ptr;
typedef __attribute__((address_space(1))) const void* global_void_ptr;

// s_waitcnt immediate for gfx9-family encodings: vmcnt (< 16) in bits [3:0],
// expcnt [6:4] and lgkmcnt [11:8] left at "do not wait".
#define SHFLBW_WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt(0x0F70 | (n))

// Direct global-to-LDS loads issued from inline assembly, for the compute
// wavefronts' metadata ring: lane L's 16 (4) bytes land at lds_off + 16*L
// (4*L).  The compiler does not know these are loads, so it neither counts
// them in its own s_waitcnt bookkeeping nor drains them in front of unrelated
// LDS reads; the code that issues them waits with an explicit vmcnt.
__device__ __forceinline__ void meta_dma16(const void* g, unsigned lds_off)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"
                 :: "s"(lds_off), "v"(g) : "memory");
}
__device__ __forceinline__ void meta_dma4(const void* g, unsigned lds_off)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, off"
                 :: "s"(lds_off), "v"(g) : "memory");
}

struct SlabArgs {
    PackedView A;
    const int32_t* iter_ptr;  // G*(C+1)
    const uint32_t* table;    // steps*64 lane table of LDS ring rows
    const _Float16* X;
    void* Y;
    long ldx, ldy, N;
    int K, C;
    int n_tiles, gblocks;     // 128-column tiles, blocks of GW groups
};

template <int V, int GW, typename OutT>
__global__ __launch_bounds__(64 * (GW + SLAB_LOADERS)) void shflbw_slab_kernel(SlabArgs a)
{
    constexpr bool SMALL = (V == 16);
    constexpr int TK = SMALL ? 32 : 16;
    constexpr int RB = SMALL ? 1 : V / 32;
    constexpr int TILE_N = SMALL ? 16 : 32;
    constexpr int NT = SLAB_TN / TILE_N;
    // metadata ring of a compute wavefront: RING slots of (weight tile, lane table)
    constexpr int RING = (RB == 1) ? 4 : 3;
    constexpr int SLOT_BYTES = RB * 1024 + 256;
    constexpr int LPS = RB + 1;                      // direct loads per step
    constexpr int META_WAIT = LPS * (RING - 1);      // loads younger than the current step's
    static_assert(META_WAIT < 16, "vmcnt immediate");
    constexpr int LDS_BYTES = SLAB_X_BYTES + GW * RING * SLOT_BYTES;
    static_assert(LDS_BYTES <= 160 * 1024, "LDS budget of one CU");
    __shared__ __attribute__((aligned(1024))) char smem[LDS_BYTES];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

    // Workgroups are dealt round-robin to the 8 XCDs; the blocks that share a
    // slab of X (same column tile, different group blocks) are given ids that
    // land on the same XCD one after the other, so its L2 serves the re-reads.
    const int wg = blockIdx.x;
    const int xcd = wg & 7, wslot = wg >> 3;
    const int gb = wslot % a.gblocks;
    const int nt = (wslot / a.gblocks) * 8 + xcd;
    if (nt >= a.n_tiles) return;  // uniform for the whole workgroup
    const long n0 = (long)nt * SLAB_TN;
    const int C = a.C;

    if (wave >= GW) {
        // ------------------------------------------------------------ loader
        // One direct-to-LDS load moves 64 x 16 bytes = 4 staged rows; lane L
        // lands in LDS slot L of that kilobyte, so it fetches the 16-byte column
        // chunk that the swizzle assigns to its slot.  Rows beyond K and columns
        // beyond N are redirected to valid addresses (their LDS bytes never
        // reach a stored result), so every load is issued and the count of
        // loads per chunk is exact.
        const int lw = wave - GW;
        const int lrow = lane >> 4, lpos = lane & 15;
        auto issue_chunk = [&](int c) __attribute__((always_inline)) {
#pragma unroll
            for (int i = 0; i < SLAB_IPL; ++i) {
                const int piece = lw * SLAB_IPL + i;
                const int r = 4 * piece + lrow;                       // row inside the chunk
                const int q = lpos ^ ((r & 7) << 1);                  // column chunk for this slot
                int row = c * SLAB_KC + r;
                row = row < a.K ? row : a.K - 1;
                long n = n0 + q * 8;
                n = n < a.N ? n : n0;
                char* dst = smem + (c % SLAB_STAGES) * SLAB_STAGE_BYTES + piece * 4 * SLAB_ROW_BYTES;
                __builtin_amdgcn_global_load_lds((global_void_ptr)(a.X + (long)row * a.ldx + n),
                                                 (lds_void_ptr)dst, 16, 0, 0);
            }
        };
        // lanes 0..15 of the first loader clear the zero row
        if (lw == 0 && lane < 16)
            *reinterpret_cast<half8*>(smem + SLAB_ZERO_ROW * SLAB_ROW_BYTES + lane * 16) =
                half8{0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
        for (int c = 0; c < SLAB_LEAD; ++c)
            if (c < C) issue_chunk(c);
        for (int c = 0; c < C; ++c) {
            // chunk c must have landed; chunks c+1 .. c+LEAD-1 (those that exist)
            // are younger and may stay in flight
            int younger = C - 1 - c;
            younger = younger < SLAB_LEAD - 1 ? younger : SLAB_LEAD - 1;
            switch (younger) {
                case 0: SHFLBW_WAIT_VMCNT(0); break;
                case 1: SHFLBW_WAIT_VMCNT(SLAB_IPL); break;
                case 2: SHFLBW_WAIT_VMCNT(2 * SLAB_IPL); break;
                default: SHFLBW_WAIT_VMCNT(3 * SLAB_IPL); break;
            }
            static_assert(SLAB_LEAD <= 4, "extend the switch above");
            __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0): the zero-row write
            __builtin_amdgcn_s_barrier();
            // after the barrier nobody reads chunk c-WINDOW any more: its stage
            // takes chunk c+LEAD
            if (c + SLAB_LEAD < C) issue_chunk(c + SLAB_LEAD);
        }
        __builtin_amdgcn_s_barrier();  // pairs with the compute wavefronts' last barrier
        return;
    }

    // ---------------------------------------------------------------- compute
    const int g = gb * GW + wave;
    const bool have_group = g < a.A.G;
    int sbeg = 0, nsteps = 0;
    const int32_t* my_iter = a.iter_ptr;
    if (have_group) {
        sbeg = a.A.step_ptr[g];
        nsteps = a.A.step_ptr[g + 1] - sbeg;
        my_iter = a.iter_ptr + (long)g * (C + 1);
    }

    const int bl = lane >> 4, il = lane & 15;
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

    // row indices for the write-back, fetched now so that the epilogue's loads
    // do not queue behind its stores
    constexpr int ROWS_E = SMALL ? 16 : 32;
    int out_row[RB][ROWS_E / 8];
    {
        const int32_t* rows_g = a.A.row_indices + (long)(have_group ? g : 0) * V;
#pragma unroll
        for (int rb = 0; rb < RB; ++rb)
#pragma unroll
            for (int i = 0; i < ROWS_E / 8; ++i) out_row[rb][i] = rows_g[rb * 32 + i * 8 + (lane >> 3)];
    }

    // BulkLoadMeta: each step's weight tile (RB KB, already in operand order)
    // and lane table (256 B) are brought into this wavefront's LDS ring by
    // direct loads issued RING-1 steps ahead.  Nothing else sits in this
    // wavefront's vector-memory queue inside the loop, and every step issues
    // exactly LPS loads (the step index is clamped at the end), so "the
    // current step's metadata has landed" is vmcnt(META_WAIT).
    const int last = nsteps > 0 ? nsteps - 1 : 0;
    const char* val_g = reinterpret_cast<const char*>(a.A.values) + ((long)sbeg * RB * 64 + lane) * 16;
    const char* tab_g = reinterpret_cast<const char*>(a.table) + ((long)sbeg * 64 + lane) * 4;
    char* my_ring = smem + SLAB_X_BYTES + wave * (RING * SLOT_BYTES);
    const unsigned ring_off = (unsigned)(size_t)(lds_char_ptr)my_ring;
    auto issue_meta = [&](int step, int slot) __attribute__((always_inline)) {
        const int sn = step < nsteps ? step : last;
        const unsigned dst = ring_off + slot * SLOT_BYTES;
#pragma unroll
        for (int rb = 0; rb < RB; ++rb)
            meta_dma16(val_g + ((long)sn * RB + rb) * 1024, dst + rb * 1024);
        meta_dma4(tab_g + (long)sn * 256, dst + RB * 1024);
    };
#pragma unroll
    for (int u = 0; u < RING - 1; ++u) issue_meta(u, u);

    // iter_ptr[c+1] for 64 iterations at a time, one entry per lane
    int itv = 0;
    int s = 0;
    int slot = 0;  // s % RING

    for (int c = 0; c < C; ++c) {
        if ((c & 63) == 0) {
            const int idx = c + 1 + lane;
            itv = have_group ? my_iter[idx < C ? idx : C] : 0;
            // consume the value here, so that the wait for this load sits inside
            // this rarely taken block and not in front of every iteration
            asm volatile("" : "+v"(itv));
        }
        const int s_end = __builtin_amdgcn_readlane(itv, c & 63);
        // chunks up to c are in LDS for everybody; c-WINDOW+1 .. c are readable
        __syncthreads();
        for (; s < s_end; ++s) {
            // refill the slot the previous step has just released
            {
                int free_slot = slot - 1;
                free_slot = free_slot < 0 ? RING - 1 : free_slot;
                issue_meta(s + RING - 1, free_slot);
            }
            asm volatile("s_waitcnt vmcnt(%0)" :: "n"(META_WAIT) : "memory");
            const char* sl = my_ring + slot * SLOT_BYTES;
            const unsigned tab = *reinterpret_cast<const unsigned*>(sl + RB * 1024 + lane * 4);
            half8 w[RB];
#pragma unroll
            for (int rb = 0; rb < RB; ++rb) w[rb] = *reinterpret_cast<const half8*>(sl + rb * 1024 + lane * 16);
            const int row0 = tab & 0xffff, row1 = tab >> 16;
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
            slot = (slot + 1 == RING) ? 0 : slot + 1;
        }
    }
    // drain the metadata loads still in flight before LDS is reused
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();  // all transposed reads done: the stages become epilogue scratch

    // ---- reordered write-back: per wavefront, 32 (16) stored rows x 128 bytes per pass
    if (!have_group) return;
    constexpr int OUT16 = 16 / (int)sizeof(OutT);        // values per 16 bytes
    constexpr int CW = 128 / (int)sizeof(OutT);           // columns per pass: 64 (fp16) or 32 (fp32)
    constexpr int PASSES = SLAB_TN / CW;
    constexpr int TPP = CW / TILE_N;                      // instruction tiles per pass
    constexpr int EP = CW + OUT16;                        // pitch in OutT units (144 bytes)
    constexpr int WAVE_BYTES = 32 * 144;
    static_assert(GW * WAVE_BYTES <= SLAB_STAGES * SLAB_STAGE_BYTES, "epilogue scratch must fit");
    OutT* ep = reinterpret_cast<OutT*>(smem + wave * WAVE_BYTES);
    const int erow = lane >> 3, echunk = lane & 7;        // 8 lanes x 16 B per row
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
                const int orig = out_row[rb][i];
                const long n = n0 + pass * CW + echunk * OUT16;
                if (n < a.N)
                    *reinterpret_cast<vecw*>(static_cast<OutT*>(a.Y) + (long)orig * a.ldy + n) = v;
            }
            SHFLBW_WAVE_LDS_SYNC();
        }
    }
}

}  // namespace shflbw
