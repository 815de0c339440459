// Shared-slab kernel for the Shfl-BW product on gfx950 (CDNA4).
//
// A workgroup owns GW row groups (one compute wavefront each; for V = 128 two
// wavefronts share a group, 64 of its rows each) x 128 output columns.  All of its wavefronts need rows of the same 128-column slab of X,
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
// Residency and hand-over.  A ring of six 16 KB stages.  The packed matrix is
// cut into k-steps whose columns span at most WINDOW = 3 adjacent chunks; a step
// may run once the chunk c of its last column has landed, when chunks
// c-2 .. c are resident; the other three stages are chunks in flight.  There
// is no workgroup barrier in the loop.  Each loader publishes in LDS how many
// chunks it has landed, each compute wavefront the chunk of the step it is
// working on (it has finished every step of an earlier chunk); a compute
// wavefront polls the former before a step, a loader looks at the latter
// before it reuses a stage and never lets that hold back the announcement of
// a chunk that has landed.  Wavefronts therefore drift apart by up to three
// chunks, which is what overlaps one wavefront's LDS latency with another's
// matrix-core time.  The polls are
// bounded: a wavefront that does not see its condition within spin_limit
// tries (about a million by default) goes on regardless - wrong numbers
// instead of a hang - and sets a status word that the host can read back.
//
// Per step the compressor stores 8 table words (16 for V = 16), one per pair
// of rows that a lane's two transposed reads take: the rows' LDS offsets with
// the swizzle folded in, and by how many chunks the step lies past the one
// before it.  A lane loads the word of its pair (the 64 lanes of a wavefront
// read 32 or 64 bytes in all) and gets its read addresses by an exclusive-or
// with a per-lane constant that holds its position in the operand and the
// instruction tile: two shifts and eight fused mask-and-xor per step.  The
// loop is bound by instruction issue (address arithmetic and matrix
// instructions share the vector issue port) and by bytes from the L2, which is
// why the table is small and pre-digested.
//
// Algorithm 1's parts: BulkLoadMeta = each step's weight tile and table word
// fetched into registers four steps ahead (two for V = 64, whose two row
// blocks of accumulators leave no room for more; the steps of a group come
// in batches of four, so the register sets are compile-time choices and the
// compiler's own wait counts are exact);
// StitchTile = chunk streaming + gathered transposed reads; WarpMMA =
// v_mfma_f32_32x32x16_f16 (16x16x32 for V = 16; the bf16 forms with BF) with
// X^T as first operand;
// ReorderedWriteBack = accumulators through LDS, 128-byte row segments stored
// to the rows named by row_indices.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

#include "gather_kernel.hip"

namespace shflbw {

constexpr int SLAB_STAGES = SLAB_WINDOW + SLAB_LEAD;
constexpr int SLAB_STAGE_BYTES = SLAB_KC * SLAB_ROW_BYTES;
constexpr int SLAB_X_BYTES = (SLAB_ZERO_ROW + 1) * SLAB_ROW_BYTES;  // ring + the all-zero row
constexpr int SLAB_LOADERS = 4;                    // loader wavefronts per workgroup
constexpr int SLAB_IPL = SLAB_KC / 4 / SLAB_LOADERS;  // direct loads (4 rows each) per loader per chunk
static_assert(SLAB_IPL * SLAB_LOADERS * 4 == SLAB_KC, "chunk must divide evenly");
static_assert(SLAB_IPL * (SLAB_LEAD - 1) < 64, "vmcnt is a six-bit count");

constexpr int SLAB_BUFFER_FLAGS = 0x00020000;     // last word of a raw buffer descriptor: untyped 32-bit data

typedef __attribute__((address_space(3))) char* lds_char_ptr;

// Direct global-to-LDS load issued from inline assembly: lane L's 16 bytes
// land at lds_off + 16*L.  The compiler does not know this is a load, so it
// neither counts it in its own s_waitcnt bookkeeping nor drains it in front
// of unrelated LDS reads; the loader that issues it waits with an explicit
// vmcnt.
__device__ __forceinline__ void meta_dma16(const void* g, unsigned lds_off)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"
                 :: "s"(lds_off), "v"(g) : "memory");
}
struct SlabArgs {
    PackedView A;
    const uint32_t* table;    // steps*TK/2 table words (LDS offsets of row pairs, chunk difference)
    const int32_t* first_chunk;  // chunk of each group's first step
    const _Float16* X;
    void* Y;
    long ldx, ldy, N;
    int K, C;
    int n_tiles, gblocks;     // 128-column tiles, blocks of GW groups
    int gb_side;              // 0, or the group-block side of the blocks an XCD works on at a time (divides gblocks, and 32)
    int spin_limit;           // polls per bounded wait
    int uniform_steps;        // k-steps of every group when they all have the same number, else -1
    int* status;              // set to non-zero by a wavefront whose wait ran out
};

template <int V, int GW, typename OutT, bool BF>
__global__ __launch_bounds__(64 * (GW + SLAB_LOADERS)) void shflbw_slab_kernel(SlabArgs a)
{
    constexpr bool SMALL = (V == 16);
    constexpr int TK = SMALL ? 32 : 16;
    constexpr int RBG = SMALL ? 1 : V / 32;           // 32-row blocks of a group
    constexpr int SPLITW = V == 128 ? 2 : 1;          // compute wavefronts per group: V = 128 is shared by two,
                                                      // same steps and X rows, two row blocks of the weights each
    constexpr int RB = RBG / SPLITW;                  // row blocks (accumulator sets) of one wavefront
    static_assert(GW % SPLITW == 0, "whole groups per workgroup");
    constexpr int TILE_N = SMALL ? 16 : 32;
    constexpr int NT = SLAB_TN / TILE_N;
    constexpr int PD = RB >= 2 ? 2 : SLAB_UNROLL;     // register sets of prefetched metadata (divides SLAB_UNROLL)
    constexpr int WAVE_BYTES = 32 * 144;              // write-back scratch of one compute wavefront
    constexpr int SCRATCH_OFF = SLAB_X_BYTES;
    constexpr int FLAGS_OFF = SCRATCH_OFF + GW * WAVE_BYTES;  // landed[4], progress[GW]
    constexpr int LDS_BYTES = FLAGS_OFF + 128;
    static_assert(SLAB_LOADERS + GW <= 31, "flag block: landed, progress, and the last word for a wait that ran out");
    static_assert((SLAB_LOADERS & (SLAB_LOADERS - 1)) == 0, "the landed counts are read with lane & (SLAB_LOADERS - 1)");
    static_assert(LDS_BYTES <= 160 * 1024, "LDS budget of one CU");
    __shared__ __attribute__((aligned(1024))) char smem[LDS_BYTES];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

    // Workgroups are dealt round-robin to the 8 XCDs; the blocks that share a
    // slab of X (same column tile, different group blocks) are given ids that
    // land on the same XCD one after the other, so its L2 serves the re-reads.
    //
    // When the packed weights are far larger than an L2 (4 MB per XCD), running all group
    // blocks of two column tiles side by side makes every workgroup fetch its weights over the
    // fabric.  The 32 workgroups an XCD runs at a time then form a block of gb_side group blocks
    // x 32/gb_side column tiles instead: weights are fetched once per 32/gb_side column tiles,
    // activations once per gb_side group blocks.
    const int wg = blockIdx.x;
    const int xcd = wg & 7, wslot = wg >> 3;
    int gb, nt;
    if (a.gb_side == 0) {
        // an XCD takes a run of neighbouring column tiles: the tiles it works on at a time are
        // adjacent in X and in Y (1 % faster than tiles 8 apart)
        gb = wslot % a.gblocks;
        nt = xcd * ((a.n_tiles + 7) / 8) + wslot / a.gblocks;
    } else {
        const int side_n = 32 / a.gb_side, blocks_g = a.gblocks / a.gb_side;
        const int block = wslot >> 5, inside = wslot & 31;
        gb = (block % blocks_g) * a.gb_side + inside % a.gb_side;
        nt = ((block / blocks_g) * side_n + inside / a.gb_side) * 8 + xcd;
    }
    if (nt >= a.n_tiles) return;  // uniform for the whole workgroup
    const long n0 = (long)nt * SLAB_TN;
    const int C = a.C;

    typedef __attribute__((address_space(3))) volatile int* lds_flag_ptr;
    lds_flag_ptr landed = (lds_flag_ptr)(smem + FLAGS_OFF);  // per loader: chunks landed
    lds_flag_ptr progress = landed + SLAB_LOADERS;           // per compute wavefront: iterations done
    if (tid < 32) landed[tid] = 0;
    if (tid >= 64 && tid < 80)  // the all-zero row
        *reinterpret_cast<half8*>(smem + SLAB_ZERO_ROW * SLAB_ROW_BYTES + (tid - 64) * 16) =
            half8{0, 0, 0, 0, 0, 0, 0, 0};
    __syncthreads();
    // true once flags[0..count) are all >= need
    auto reached = [&](lds_flag_ptr flags, int count, int need) __attribute__((always_inline)) {
        const int v = flags[lane & 15];
        return __builtin_amdgcn_ballot_w64(lane < count && v < need) == 0;
    };
    static_assert(GW <= 16 && SLAB_LOADERS + 16 + 16 <= 32 + 4, "flag reads stay inside the flag block");
    // a wait that ran out is recorded for the host (the wavefront goes on: wrong numbers, no hang)
    // ... and for the workgroup: every compute wavefront that finishes after this stores NaN
    // instead of a tile it cannot vouch for (a loader gives up only on behalf of a compute
    // wavefront that still lags behind, a compute wavefront for itself)
    lds_flag_ptr poisoned = landed + 31;
    auto give_up = [&](int who) __attribute__((always_inline)) {
        if (lane == 0) {
            *poisoned = 1;
            atomicOr(a.status, who);
        }
    };

    if (wave >= GW) {
        // ------------------------------------------------------------ loader
        // One direct-to-LDS load moves 64 x 16 bytes = 4 staged rows; lane L
        // lands in LDS slot L of that kilobyte, so it fetches the 16-byte column
        // chunk that the swizzle assigns to its slot.  Rows beyond K and columns
        // beyond N are redirected to valid addresses (their LDS bytes never
        // reach a stored result), so every load is issued and the count of
        // loads per chunk is exact.
        __builtin_amdgcn_s_setprio(3);   // loaders issue ahead of the compute wavefronts of their SIMD
        const int lw = wave - GW;
        const int lrow = lane >> 4, lpos = lane & 15;
        const unsigned x_off = (unsigned)(size_t)(lds_char_ptr)smem;
        auto issue_chunk = [&](int c) __attribute__((always_inline)) {
#pragma unroll
            for (int i = 0; i < SLAB_IPL; ++i) {
                const int piece = lw * SLAB_IPL + i;
                const int r = 4 * piece + lrow;                       // row inside the chunk
                const int q = lpos ^ slab_swizzle(r);                 // column chunk for this slot
                int row = c * SLAB_KC + r;
                row = row < a.K ? row : a.K - 1;
                long n = n0 + q * 8;
                n = n < a.N ? n : n0;
                meta_dma16(a.X + (long)row * a.ldx + n,
                           x_off + (c % SLAB_STAGES) * SLAB_STAGE_BYTES + piece * 4 * SLAB_ROW_BYTES);
            }
        };
        // `published` chunks have been announced to the compute wavefronts, `issued`
        // requested.  A wavefront's loads complete in order, so "chunk `published` has
        // landed" is a wait until only the loads of the younger chunks in flight remain.
        // A landed chunk is announced at once, whether or not the ring has room for the
        // next request: a fast compute wavefront may then run up to LEAD chunks ahead of
        // the slowest one, whose progress is what frees a stage.  (Announcing chunk c+1
        // only after the request for chunk c+LEAD had found its stage free kept every
        // compute wavefront within one chunk of the slowest.)
        int issued = 0, published = 0;
#pragma unroll
        for (int c = 0; c < SLAB_LEAD; ++c)
            if (c < C) { issue_chunk(c); issued = c + 1; }
        while (published < C) {
            switch (issued - published - 1) {   // chunks younger than the one awaited
                case 0: asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); break;
                case 1: asm volatile("s_waitcnt vmcnt(%0)" :: "n"(SLAB_IPL) : "memory"); break;
                case 2: asm volatile("s_waitcnt vmcnt(%0)" :: "n"(2 * SLAB_IPL) : "memory"); break;
                default: asm volatile("s_waitcnt vmcnt(%0)" :: "n"(3 * SLAB_IPL) : "memory"); break;
            }
            static_assert(SLAB_LEAD <= 4, "extend the switch above");
            ++published;
            landed[lw] = published;
            // chunk j takes the stage of chunk j-STAGES, whose last readers are the steps that end
            // in chunk j-LEAD-1: it may go out once every compute wavefront works on chunk j-LEAD or
            // a later one
            while (issued < C && issued - published < SLAB_LEAD) {
                if (issued >= SLAB_STAGES && !reached(progress, GW, issued - SLAB_LEAD)) {
                    if (issued > published) break;   // announce what is in flight first, then look again
                    int tries = 0;
                    for (; !reached(progress, GW, issued - SLAB_LEAD) && tries < a.spin_limit; ++tries)
                        __builtin_amdgcn_s_sleep(1);
                    if (tries >= a.spin_limit && !reached(progress, GW, issued - SLAB_LEAD)) give_up(2);
                }
                asm volatile("" ::: "memory");
                issue_chunk(issued);
                ++issued;
            }
        }
        return;
    }

    // ---------------------------------------------------------------- compute
    const int g = gb * (GW / SPLITW) + wave / SPLITW;
    const int half = wave % SPLITW;                   // which of the group's row-block halves (V = 128)
    const bool have_group = g < a.A.G;
    if (!have_group) {
        progress[wave] = C;  // nothing to read: never hold a stage back
        return;
    }
    // the group's steps: without a memory access when every group has the same number (the
    // first weights can then be requested at once instead of after a dependent scalar load)
    const int sbeg = a.uniform_steps >= 0 ? g * a.uniform_steps : a.A.step_ptr[g];
    const int nsteps = a.uniform_steps >= 0 ? a.uniform_steps : a.A.step_ptr[g + 1] - sbeg;  // a multiple of PD
    const int first_chunk_g = a.first_chunk[g];   // wanted only when the first step is decoded

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
    constexpr bool EARLY_ROWS = RB < 2;   // with two row blocks the registers are needed in the loop
    auto load_rows = [&]() __attribute__((always_inline)) {
        const int32_t* rows_g = a.A.row_indices + (long)g * V + half * RB * 32;
#pragma unroll
        for (int rb = 0; rb < RB; ++rb)
#pragma unroll
            for (int i = 0; i < ROWS_E / 8; ++i) out_row[rb][i] = rows_g[rb * 32 + i * 8 + (lane >> 3)];
    };
    if (EARLY_ROWS) load_rows();

    // BulkLoadMeta: table word and weight operand of the next PD steps sit in PD
    // register sets; step s uses set s % PD and refills it for step s + PD (the
    // index is clamped at the end, so the loads are unconditional).
    const int last = nsteps - 1;
    // Buffer loads: the descriptor holds the group's base address, the step's offset goes in a
    // scalar register and the lane's in one vector register, so a load costs no vector
    // arithmetic.  The hardware checks only the lane offset against the descriptor's size, so
    // the step index is kept in range by the code (the refills clamp it to the last step).
    typedef unsigned uint4v __attribute__((ext_vector_type(4)));
    constexpr int WPS = TK / 2;                       // table words per step
    const __amdgpu_buffer_rsrc_t tab_rsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint32_t*>(a.table + (long)sbeg * WPS), 0, nsteps * WPS * 4, SLAB_BUFFER_FLAGS);
    // this lane's pair of rows and its position inside them (see the transposed read's lane map)
    const int bl = lane >> 4, il = lane & 15;
    const int pair = SMALL ? 4 * bl + (il >> 2) : 4 * (bl >> 1) + (il >> 2);
    const int qc = SMALL ? ((il & 3) >> 1) : (2 * (bl & 1) + ((il & 3) >> 1));
    const unsigned lane_bits = (unsigned)(qc << 4) | (unsigned)((il & 1) << 3);
    const __amdgpu_buffer_rsrc_t val_rsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<half8*>(a.A.values + (long)sbeg * RBG * 64), 0, nsteps * RBG * 1024, SLAB_BUFFER_FLAGS);
    auto load_table = [&](int s) __attribute__((always_inline)) {
        return __builtin_amdgcn_raw_buffer_load_b32(tab_rsrc, pair * 4, s * (WPS * 4), 0);
    };
    auto load_weights = [&](int s, int rb) __attribute__((always_inline)) {
        return __builtin_bit_cast(half8, __builtin_amdgcn_raw_buffer_load_b128(val_rsrc, lane * 16,
                                                                                (s * RBG + half * RB + rb) * 1024, 0));
    };
    unsigned mt[PD];
    half8 mw[PD][RB];
#pragma unroll
    for (int u = 0; u < PD; ++u) {
        // a group without steps has an empty descriptor: these read as zero
        mt[u] = load_table(u);
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) mw[u][rb] = load_weights(u, rb);
        // keep the sets in issue order: the loop's wait counts assume set 0 is the oldest
        __builtin_amdgcn_sched_barrier(0);
    }

    int chunk = first_chunk_g;   // of the step in hand, from the table's differences
    int cur = 0;   // chunk last published; every step of an earlier chunk is done
    int seen = 0;  // chunks known to have landed (the least of the loaders' counts when last read)
    for (int s0 = 0; s0 < nsteps; s0 += PD) {
#pragma unroll
        for (int u = 0; u < PD; ++u) {
            const unsigned tab = mt[u];
            const unsigned head = __builtin_amdgcn_readfirstlane(tab);
            chunk += (head >> 26) & 15;
            const int e = chunk;
            if (e != cur) {
                // this wavefront's reads of chunks below e - WINDOW + 1 are over
                asm volatile("" ::: "memory");
                progress[wave] = e;
                cur = e;
            }
            if (seen < e + 1) {
                // the flags are read only when the chunk is not already known to be in
                int tries = 0;
#pragma nounroll
                for (;; ++tries) {
                    const int v = landed[lane & (SLAB_LOADERS - 1)];
                    int m = __builtin_amdgcn_readlane(v, 0);
#pragma unroll
                    for (int l = 1; l < SLAB_LOADERS; ++l) {
                        const int o = __builtin_amdgcn_readlane(v, l);
                        m = o < m ? o : m;
                    }
                    seen = m;
                    if (m >= e + 1) break;
                    if (tries >= a.spin_limit) {
                        give_up(1);
                        break;
                    }
                    __builtin_amdgcn_s_sleep(1);
                }
            }
            asm volatile("" ::: "memory");

            const unsigned row0 = tab << 4, row1 = tab >> 9;   // the offsets sit in bits 4-16 of these
            // all transposed reads of the step go out before the first product
            half8 x[NT];
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                // tile t: 16-byte slot (SMALL ? 2t : 4t) further on, before the swizzle
                constexpr int TILE_BITS = SMALL ? 32 : 64;
                const unsigned pos = lane_bits ^ (unsigned)(t * TILE_BITS);
                short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_ptr)(smem + ((row0 & 0x1fff0u) ^ pos)));
                short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_ptr)(smem + ((row1 & 0x1fff0u) ^ pos)));
                half4 l4 = __builtin_bit_cast(half4, lo), h4 = __builtin_bit_cast(half4, hi);
                x[t] = half8{l4[0], l4[1], l4[2], l4[3], h4[0], h4[1], h4[2], h4[3]};
            }
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                if (SMALL) {
                    acc16[t] = mma16<BF>(x[t], mw[u][0], acc16[t]);
                } else {
#pragma unroll
                    for (int rb = 0; rb < RB; ++rb)
                        acc32[rb][t] = mma32<BF>(x[t], mw[u][rb], acc32[rb][t]);
                }
            }
            {
                const int sn = (s0 + u + PD < nsteps) ? s0 + u + PD : last;
                mt[u] = load_table(sn);
#pragma unroll
                for (int rb = 0; rb < RB; ++rb) mw[u][rb] = load_weights(sn, rb);
            }
        }
    }
    asm volatile("" ::: "memory");
    progress[wave] = C;  // all of this wavefront's reads of X are over
    if (!EARLY_ROWS) load_rows();

    // ---- reordered write-back: per wavefront, 32 (16) stored rows x 128 bytes per pass
    constexpr int OUT16 = 16 / (int)sizeof(OutT);        // values per 16 bytes
    constexpr int CW = 128 / (int)sizeof(OutT);           // columns per pass: 64 (fp16) or 32 (fp32)
    constexpr int PASSES = SLAB_TN / CW;
    constexpr int TPP = CW / TILE_N;                      // instruction tiles per pass
    constexpr int EP = CW + OUT16;                        // pitch in OutT units (144 bytes)
    OutT* ep = reinterpret_cast<OutT*>(smem + SCRATCH_OFF + wave * WAVE_BYTES);
    const int erow = lane >> 3, echunk = lane & 7;        // 8 lanes x 16 B per row
    typedef OutT vec4 __attribute__((ext_vector_type(4)));
    typedef OutT vecw __attribute__((ext_vector_type(OUT16)));
    const bool spoiled = *poisoned != 0;                  // a hand-over wait ran out: the tile is stored as NaN

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
                if (spoiled) {
#pragma unroll
                    for (int j = 0; j < OUT16; ++j) v[j] = (OutT)__builtin_nanf("");
                }
                const int orig = out_row[rb][i];
                const long n = n0 + pass * CW + echunk * OUT16;
                if (n < a.N)
                    // streaming store: Y must not displace the slab and the weights in the L2
                    __builtin_nontemporal_store(v, reinterpret_cast<vecw*>(static_cast<OutT*>(a.Y) + (long)orig * a.ldy + n));
            }
            SHFLBW_WAVE_LDS_SYNC();
        }
    }
}

}  // namespace shflbw
