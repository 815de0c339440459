// Internal definitions shared by the host-side compressor and the kernel
// launchers.  Not part of the public ABI.
#ifndef SHFLBW_INTERNAL_H
#define SHFLBW_INTERNAL_H

#include <cstdint>
#include <string>
#include <vector>

#include "shflbw.h"

// Packed Shfl-BW matrix (offline step (a), Sections 4.1-4.3).
//
// Stored rows are the permuted rows; group g owns stored rows gV..gV+V-1.
// The kept columns of a group are cut into "k-steps" of TK columns, the
// reduction depth one matrix-core pass consumes (TK = 16 for V >= 32 on the
// 32x32x16 instruction, TK = 32 for V = 16 on the 16x16x32 instruction).  The
// steps are padded where needed: padded column slots hold -1 and their weights
// are zero.
//
// Two step layouts exist.  Plain: consecutive runs of TK kept columns; only a
// group's last step is padded.  Windowed (slab_ok): the columns are seen as
// chunks of SLAB_KC consecutive indices and a step never spans more than
// SLAB_WINDOW adjacent chunks, so that a kernel which streams X through LDS chunk by
// chunk finds all rows of a step resident at once; a step whose columns
// would reach one chunk more is cut short and padded, and every group's step
// count is rounded up to a multiple of SLAB_UNROLL with empty steps.
// slab_table holds what the slab kernel needs to run a step: T_K/2 words per
// step, word w for the slot pair (j, j+4), j = 8*(w/4) + w%4, that one lane's
// two transposed reads cover.  Bits 0-12 and 13-25: the LDS offsets, in
// 16-byte units, of the two slots' rows (row of the ring = column mod
// SLAB_RING_ROWS, or SLAB_ZERO_ROW for padding) with the row's swizzle in the
// low four bits - a lane gets its read address by an exclusive-or with its own
// position in the operand; bits 26-29: how many chunks the step's last column
// lies past that of the group's previous step (the step may run once that
// chunk is resident).  first_chunk holds the chunk of each group's first step.
// Steps more than SLAB_MAX_CHUNK_STEP chunks apart are bridged by empty steps.
//
// values: for each k-step, for each 32-row block rb of the group (one block
// when V = 16), 64 lanes x 8 binary16 in the operand order of the
// instruction:
//   V >= 32: lane l, element e  ->  stored row 32*rb + l%32, step column 8*(l/32) + e
//   V == 16: lane l, element e  ->  stored row l%16,         step column 8*(l/16) + e
// so one wavefront fetches its operand with one 16-byte load per lane.
struct shflbw_matrix {
    int M = 0, K = 0, V = 0, G = 0, TK = 0;
    int64_t nnz = 0;
    std::vector<int32_t> row_indices;  // M: original row of each stored row
    std::vector<int32_t> step_ptr;     // G+1: first k-step of each group
    std::vector<int32_t> kcount;       // G: kept columns per group (no padding)
    int uniform_steps = -1;            // k-steps per group when all groups have the same number, else -1
    std::vector<int32_t> col_idx;      // steps*TK: ascending columns, -1 = padding
    bool slab_ok = false;              // windowed layout in use
    int slab_chunks = 0;               // C = ceil(K / SLAB_KC)
    std::vector<int32_t> step_iter;    // steps, only when slab_ok: chunk of each step's last column
    std::vector<uint32_t> slab_table;  // steps*TK/2, only when slab_ok (see above)
    std::vector<int32_t> first_chunk;  // G, only when slab_ok: chunk of each group's first step
    std::vector<uint16_t> values;      // steps*V*TK binary16 bit patterns

    // device image (caller-owned buffer), byte offsets of the sections
    size_t off_rows = 0, off_steps = 0, off_iter = 0, off_cols = 0, off_table = 0, off_vals = 0, off_status = 0, dev_bytes = 0;
    void* dev_base = nullptr;
    int dev_id = -1;

    int tune_kernel = 0, tune_tile_n = 0;
    int wait_limit = 1 << 20;          // polls per bounded wait of the slab kernel
    int dtype = 0;                     // SHFLBW_F16 or SHFLBW_BF16: format of the values and of the activations

    int total_steps() const { return step_ptr.empty() ? 0 : step_ptr.back(); }
};

namespace shflbw {
#ifndef SHFLBW_SLAB_KC
#define SHFLBW_SLAB_KC 64
#define SHFLBW_SLAB_WINDOW 3
#define SHFLBW_SLAB_LEAD 3
#endif
constexpr int SLAB_KC = SHFLBW_SLAB_KC;          // rows of X per LDS chunk in the slab kernel
constexpr int SLAB_WINDOW = SHFLBW_SLAB_WINDOW;  // adjacent chunks a k-step may span (readable at once)
constexpr int SLAB_LEAD = SHFLBW_SLAB_LEAD;      // chunks in flight ahead of the readable window
constexpr int SLAB_RING_ROWS = SLAB_KC * (SLAB_WINDOW + SLAB_LEAD);  // rows of X resident in LDS; row of column k = k % RING_ROWS
constexpr int SLAB_ZERO_ROW = SLAB_RING_ROWS;                       // one extra all-zero row for padded slots
constexpr int SLAB_UNROLL = 4;                                      // steps per unrolled batch of the slab kernel
constexpr int SLAB_TN = 128;                                        // output columns per workgroup of the slab kernel
constexpr int SLAB_ROW_BYTES = SLAB_TN * 2;                         // one staged row of X in LDS
constexpr int SLAB_MAX_CHUNK_STEP = 15;                             // largest chunk difference a table word can hold
static_assert((SLAB_ZERO_ROW + 1) * SLAB_ROW_BYTES / 16 <= (1 << 13), "LDS offsets are stored in 13 bits, in units of 16 bytes");
// Swizzle of the 16-byte slots inside a staged row of X (the loader stores logical slot q of
// ring row r at slot q ^ slab_swizzle(r); the table's read addresses include it).  One
// transposed read covers, per 32 lanes, four rows of a step and a 64-byte window (four slots,
// 16 banks) of each: bits 2-3 of the value move the window, and they come from the row's low
// two bits so that four consecutive rows - every quad of a dense matrix - land in four
// different bank groups; bit 1 varies with the next row bit.
constexpr int slab_swizzle(int r) { return ((r & 3) << 2) | (((r >> 2) & 1) << 1); }
int fail(int status, const std::string& detail);  // records the thread-local text, returns status
void note_kernel(const std::string& name);        // records what the calling thread launched last (shflbw_last_kernel)
// Where the packed arrays of A live on the device for launches of the calling thread: the buffer given
// to shflbw_bind_device, unless an entry point that brings its own device image has set an override.
const void* device_base(const shflbw_matrix* A);
void set_device_base_override(const void* base);  // nullptr = none; thread-local
inline size_t align256(size_t x) { return (x + 255) & ~size_t(255); }
}  // namespace shflbw

#endif
