// Host-side offline step (a) (Sections 4.1-4.3): pattern check, row
// reordering into vector-wise form, original-row index array, and kept
// vectors stitched into V x TK tiles in matrix-core operand order.
// No HIP calls here: everything in this file works without a GPU.
#include <algorithm>
#include <cstdio>
#include <cstring>
#include <new>
#include <string>

#include "shflbw_internal.h"

namespace {
thread_local std::string g_last_error;
thread_local std::string g_last_kernel;
thread_local const void* g_base_override = nullptr;

// Position of (stored row i of the group, step column j) inside one k-step's
// V*TK values; see the layout comment in shflbw_internal.h.
inline size_t value_slot(int V, int i, int j)
{
    if (V == 16) {
        int lane = (j / 8) * 16 + i;
        return (size_t)lane * 8 + (j % 8);
    }
    int rb = i / 32, r = i % 32;
    int lane = (j / 8) * 32 + r;
    return ((size_t)rb * 64 + lane) * 8 + (j % 8);
}

// Order of a k-step's columns over its slots.  Any order is a valid packing (the weights follow
// their columns); this one serves the slab kernel's transposed LDS reads: one read covers, per
// 32 lanes, the rows of one slot group - 4 slots (V >= 32), or 8 (V = 16: slots 0-3 with 8-11,
// 4-7 with 12-15, and so on) - and is free of bank conflicts when the group's columns differ in
// their low two (three) bits, which pick the bank group through the row swizzle.  Columns are
// therefore dealt to the groups one residue class at a time, largest class first.
// c: the step's columns, ascending; slot_of[j]: slot of c[j].
void arrange_step(const int32_t* c, int len, int V, int* slot_of)
{
    const bool small = (V == 16);
    const int GS = small ? 8 : 4, TK = small ? 32 : 16;
    int slots[32];   // slots in group order
    for (int grp = 0, n = 0; grp < TK / GS; ++grp)
        for (int i = 0; i < GS; ++i)
            slots[n++] = small ? 16 * (grp >> 1) + 4 * (grp & 1) + (i < 4 ? i : 4 + i) : 4 * grp + i;
    int bucket[8][32], count[8] = {0};
    for (int j = 0; j < len; ++j) {
        const int cls = c[j] & (GS - 1);
        bucket[cls][count[cls]++] = j;
    }
    int taken[8] = {0};
    for (int n = 0; n < len;) {
        // one group: at most one column of each class while classes last, then whatever is left
        bool used[8] = {false};
        for (int i = 0; i < GS && n < len; ++i) {
            int best = -1;
            for (int pass = 0; pass < 2 && best < 0; ++pass)
                for (int cls = 0; cls < GS; ++cls) {
                    const int left = count[cls] - taken[cls];
                    if (left <= 0 || (pass == 0 && used[cls])) continue;
                    if (best < 0 || left > count[best] - taken[best]) best = cls;
                }
            used[best] = true;
            slot_of[bucket[best][taken[best]++]] = slots[n++];
        }
    }
}
}  // namespace

namespace shflbw {
int fail(int status, const std::string& detail)
{
    g_last_error = detail;
    return status;
}
void note_kernel(const std::string& name) { g_last_kernel = name; }
const void* device_base(const shflbw_matrix* A) { return g_base_override ? g_base_override : A->dev_base; }
void set_device_base_override(const void* base) { g_base_override = base; }
}  // namespace shflbw

extern "C" {

const char* shflbw_last_error(void) { return g_last_error.c_str(); }
const char* shflbw_last_kernel(void) { return g_last_kernel.c_str(); }

const char* shflbw_status_string(int status)
{
    switch (status) {
        case SHFLBW_OK: return "ok";
        case SHFLBW_ERR_NULL_ARG: return "null argument";
        case SHFLBW_ERR_BAD_SHAPE: return "bad shape";
        case SHFLBW_ERR_BAD_PERM: return "perm is not a permutation";
        case SHFLBW_ERR_BAD_PATTERN: return "mask is not a Shfl-BW pattern under perm";
        case SHFLBW_ERR_BAD_DTYPE: return "unsupported dtype";
        case SHFLBW_ERR_NOT_ON_DEVICE: return "matrix not bound to a device buffer";
        case SHFLBW_ERR_HIP: return "HIP runtime error";
        case SHFLBW_ERR_NO_MEMORY: return "out of host memory";
        case SHFLBW_ERR_BAD_OPTION: return "bad tuning option";
        case SHFLBW_ERR_HANDOVER: return "a bounded wait of a kernel ran out";
        default: return "unknown status";
    }
}

int shflbw_compress(const void* W, int ldw, const uint8_t* mask, const int32_t* perm,
                    int M, int K, int V, shflbw_dtype wdtype, shflbw_matrix** out)
{
    using shflbw::fail;
    if (!W || !out) return fail(SHFLBW_ERR_NULL_ARG, "W and out must not be NULL");
    *out = nullptr;
    if (wdtype != SHFLBW_F16 && wdtype != SHFLBW_BF16)
        return fail(SHFLBW_ERR_BAD_DTYPE, "weights must be SHFLBW_F16 or SHFLBW_BF16");
    if (V != 16 && V != 32 && V != 64 && V != 128)
        return fail(SHFLBW_ERR_BAD_SHAPE, "V must be 16, 32, 64 or 128");
    if (M <= 0 || K <= 0) return fail(SHFLBW_ERR_BAD_SHAPE, "M and K must be positive");
    if (M % V) return fail(SHFLBW_ERR_BAD_SHAPE, "M must be a multiple of V");
    if (ldw < K) return fail(SHFLBW_ERR_BAD_SHAPE, "ldw < K");
    const uint16_t* Wb = static_cast<const uint16_t*>(W);

    try {
        shflbw_matrix* A = new shflbw_matrix();
        struct Guard { shflbw_matrix* p; ~Guard() { delete p; } } guard{A};
        A->M = M; A->K = K; A->V = V; A->G = M / V;
        A->dtype = (int)wdtype;
        A->TK = (V == 16) ? 32 : 16;
        const int TK = A->TK, G = A->G;

        A->row_indices.resize(M);
        std::vector<uint8_t> seen(M, 0);
        for (int i = 0; i < M; ++i) {
            int r = perm ? perm[i] : i;
            if (r < 0 || r >= M || seen[r]) {
                char buf[96];
                snprintf(buf, sizeof buf, "perm[%d] = %d is out of range or repeated", i, r);
                return fail(SHFLBW_ERR_BAD_PERM, buf);
            }
            seen[r] = 1;
            A->row_indices[i] = r;
        }

        // Column set of each group; every row of the group must agree with it.
        std::vector<std::vector<int32_t>> cols(G);
        for (int g = 0; g < G; ++g) {
            const int32_t* rows = &A->row_indices[(size_t)g * V];
            if (mask) {
                const uint8_t* m0 = mask + (size_t)rows[0] * K;
                for (int i = 1; i < V; ++i) {
                    const uint8_t* mi = mask + (size_t)rows[i] * K;
                    for (int k = 0; k < K; ++k)
                        if ((m0[k] != 0) != (mi[k] != 0)) {
                            char buf[160];
                            snprintf(buf, sizeof buf,
                                     "group %d: stored row %d (original row %d) differs from the "
                                     "group's first row at column %d",
                                     g, g * V + i, rows[i], k);
                            return fail(SHFLBW_ERR_BAD_PATTERN, buf);
                        }
                }
                for (int k = 0; k < K; ++k)
                    if (m0[k]) cols[g].push_back(k);
            } else {
                for (int k = 0; k < K; ++k) {
                    bool any = false;
                    for (int i = 0; i < V && !any; ++i)
                        any = (Wb[(size_t)rows[i] * ldw + k] & 0x7fffu) != 0;
                    if (any) cols[g].push_back(k);
                }
            }
        }

        // Cut each group's ascending column list into k-steps.  The windowed
        // cut is used when it costs at most 15 % more steps than the plain one.
        auto cut = [&](const std::vector<int32_t>& c, bool windowed, std::vector<int>& lens) {
            lens.clear();
            size_t i = 0;
            while (i < c.size()) {
                size_t j = i;
                const int first_chunk = c[i] / shflbw::SLAB_KC;
                while (j < c.size() && j < i + (size_t)TK &&
                       (!windowed || c[j] / shflbw::SLAB_KC < first_chunk + shflbw::SLAB_WINDOW))
                    ++j;
                lens.push_back((int)(j - i));
                i = j;
            }
        };
        // Pairs of full steps trade columns so that each gets its share of every residue class
        // of the column index (mod 4; mod 8 for V = 16): arrange_step can then give every
        // transposed read rows that fall into different bank groups, which a run of 16 random
        // columns often cannot (seven columns of one class leave a read with two of them).  The
        // lower columns of a class go to the first step of the pair; the pair is left alone where
        // a new step would span more than the window.  c: the group's columns in step order
        // (ascending on entry; afterwards ascending inside each step only).
        auto balance_pairs = [&](std::vector<int32_t>& c, const std::vector<int>& lens) {
            const int GS = (V == 16) ? 8 : 4;
            size_t off = 0;
            for (size_t st = 0; st + 1 < lens.size(); st += 2) {
                const size_t n0 = (size_t)lens[st], n1 = (size_t)lens[st + 1];
                if ((int)n0 == TK && (int)n1 == TK) {
                    std::vector<int32_t> cls[8], a, b;
                    for (size_t j = 0; j < n0 + n1; ++j) cls[c[off + j] & (GS - 1)].push_back(c[off + j]);
                    int take[8], total = 0;
                    for (int k = 0; k < GS; ++k) { take[k] = (int)cls[k].size() / 2; total += take[k]; }
                    for (int k = 0; k < GS && total < TK; ++k)
                        if (cls[k].size() & 1) { ++take[k]; ++total; }
                    for (int k = 0; k < GS; ++k)
                        for (size_t j = 0; j < cls[k].size(); ++j) ((int)j < take[k] ? a : b).push_back(cls[k][j]);
                    std::sort(a.begin(), a.end());
                    std::sort(b.begin(), b.end());
                    if (a.back() / shflbw::SLAB_KC > b.back() / shflbw::SLAB_KC) a.swap(b);   // chunks must not decrease
                    auto fits = [&](const std::vector<int32_t>& v) {
                        return v.back() / shflbw::SLAB_KC - v.front() / shflbw::SLAB_KC < shflbw::SLAB_WINDOW;
                    };
                    if ((int)a.size() == TK && (int)b.size() == TK && fits(a) && fits(b)) {
                        std::copy(a.begin(), a.end(), c.begin() + off);
                        std::copy(b.begin(), b.end(), c.begin() + off + n0);
                    }
                }
                off += n0 + n1;
            }
        };
        // The slab kernel learns a step's chunk from a 4-bit difference to the step
        // before it (the group's first chunk is stored per group), so where two
        // consecutive steps of the windowed layout lie more than 15 chunks apart,
        // empty steps (length 0) are put between them, each carrying 15 chunks.
        auto bridge_gaps = [&](const std::vector<int32_t>& c, std::vector<int>& lens, std::vector<int>& chunk) {
            std::vector<int> out_len, out_chunk;
            size_t t = 0;
            int prev = -1;
            for (int len : lens) {
                t += (size_t)len;
                const int e = *std::max_element(c.begin() + (t - len), c.begin() + t) / shflbw::SLAB_KC;
                if (prev >= 0)
                    while (e - prev > shflbw::SLAB_MAX_CHUNK_STEP) {
                        prev += shflbw::SLAB_MAX_CHUNK_STEP;
                        out_len.push_back(0);
                        out_chunk.push_back(prev);
                    }
                out_len.push_back(len);
                out_chunk.push_back(e);
                prev = e;
            }
            lens.swap(out_len);
            chunk.swap(out_chunk);
        };
        std::vector<std::vector<int>> plain(G), win(G), win_chunk(G);
        std::vector<std::vector<int32_t>> wcols(cols);   // the columns in the step order of the windowed layout
        size_t n_plain = 0, n_win = 0;
        for (int g = 0; g < G; ++g) {
            cut(cols[g], false, plain[g]);
            cut(cols[g], true, win[g]);
            balance_pairs(wcols[g], win[g]);
            bridge_gaps(wcols[g], win[g], win_chunk[g]);
            n_plain += plain[g].size();
            n_win += win[g].size();
        }
        A->slab_chunks = (K + shflbw::SLAB_KC - 1) / shflbw::SLAB_KC;
        A->slab_ok = n_plain > 0 && (double)n_win <= 1.15 * (double)n_plain;
        const std::vector<std::vector<int>>& lens = A->slab_ok ? win : plain;
        const std::vector<std::vector<int32_t>>& scols = A->slab_ok ? wcols : cols;   // columns in step order

        // In the windowed layout every group gets a multiple of SLAB_UNROLL steps
        // (the slab kernel runs its steps in unrolled batches); the extra steps are
        // empty: no columns, zero weights.
        auto padded = [&](size_t n) {
            return A->slab_ok ? (n + shflbw::SLAB_UNROLL - 1) / shflbw::SLAB_UNROLL * shflbw::SLAB_UNROLL : n;
        };
        A->step_ptr.assign(G + 1, 0);
        A->kcount.resize(G);
        for (int g = 0; g < G; ++g) {
            A->kcount[g] = (int)cols[g].size();
            A->nnz += (int64_t)cols[g].size() * V;
            A->step_ptr[g + 1] = A->step_ptr[g] + (int)padded(lens[g].size());
        }
        A->uniform_steps = A->step_ptr[1] - A->step_ptr[0];
        for (int g = 1; g < G; ++g)
            if (A->step_ptr[g + 1] - A->step_ptr[g] != A->uniform_steps) A->uniform_steps = -1;
        const size_t steps = (size_t)A->step_ptr[G];
        A->col_idx.assign(steps * TK, -1);
        A->values.assign(steps * (size_t)V * TK, 0);
        if (A->slab_ok) A->step_iter.assign(steps, 0);
        for (int g = 0; g < G; ++g) {
            const int32_t* rows = &A->row_indices[(size_t)g * V];
            size_t step = (size_t)A->step_ptr[g];
            size_t t = 0;
            size_t nth = 0;   // position in the group's step list
            for (int len : lens[g]) {
                uint16_t* dst = &A->values[step * (size_t)V * TK];
                int slot_of[32];
                arrange_step(&scols[g][t], len, V, slot_of);
                for (int j = 0; j < len; ++j, ++t) {
                    const int k = scols[g][t];
                    A->col_idx[step * TK + slot_of[j]] = k;
                    for (int i = 0; i < V; ++i)
                        dst[value_slot(V, i, slot_of[j])] = Wb[(size_t)rows[i] * ldw + k];
                }
                if (A->slab_ok) {
                    // this step runs once the chunk of its last column is resident
                    A->step_iter[step] = win_chunk[g][nth];
                }
                ++step;
                ++nth;
            }
            // empty padding steps inherit the iteration of the step before them
            for (; step < (size_t)A->step_ptr[g + 1]; ++step)
                if (A->slab_ok)
                    A->step_iter[step] = step > (size_t)A->step_ptr[g] ? A->step_iter[step - 1] : 0;
        }

        if (A->slab_ok) {
            // What the slab kernel needs to run a step (see slab_kernel.hip): per pair of
            // slots (j, j+4) that one lane reads, the LDS offsets (in 16-byte units, row
            // swizzle included) of the two rows, and how many chunks the step lies past
            // the one before.  Word w of a step serves slots j = 8*(w/4) + w%4 and j+4.
            const int WPS = TK / 2;
            A->slab_table.resize(steps * WPS);
            A->first_chunk.assign(G, 0);
            for (int g = 0; g < G; ++g) {
                int prev = 0;
                for (size_t st = (size_t)A->step_ptr[g]; st < (size_t)A->step_ptr[g + 1]; ++st) {
                    if (st == (size_t)A->step_ptr[g]) prev = A->first_chunk[g] = A->step_iter[st];
                    const uint32_t d = (uint32_t)(A->step_iter[st] - prev);   // 0 .. SLAB_MAX_CHUNK_STEP
                    prev = A->step_iter[st];
                    for (int w = 0; w < WPS; ++w) {
                        const int j = 8 * (w >> 2) + (w & 3);
                        uint32_t word = d << 26;
                        for (int h = 0; h < 2; ++h) {
                            const int k = A->col_idx[st * TK + j + 4 * h];
                            const int row = k < 0 ? shflbw::SLAB_ZERO_ROW : k % shflbw::SLAB_RING_ROWS;
                            const uint32_t field = (uint32_t)(row * (shflbw::SLAB_ROW_BYTES / 16) + shflbw::slab_swizzle(row));
                            word |= field << (13 * h);
                        }
                        A->slab_table[st * WPS + w] = word;
                    }
                }
            }
        }

        A->off_rows = 0;
        A->off_steps = shflbw::align256(A->off_rows + sizeof(int32_t) * (size_t)M);
        A->off_iter = shflbw::align256(A->off_steps + sizeof(int32_t) * (size_t)(G + 1));
        A->off_cols = shflbw::align256(A->off_iter + sizeof(int32_t) * A->first_chunk.size());
        A->off_table = shflbw::align256(A->off_cols + sizeof(int32_t) * A->col_idx.size());
        A->off_vals = shflbw::align256(A->off_table + sizeof(uint32_t) * A->slab_table.size());
        A->off_status = shflbw::align256(A->off_vals + sizeof(uint16_t) * A->values.size());
        A->dev_bytes = A->off_status + 256;   // one word set by kernels whose bounded wait ran out

        guard.p = nullptr;
        *out = A;
        return SHFLBW_OK;
    } catch (const std::bad_alloc&) {
        return fail(SHFLBW_ERR_NO_MEMORY, "allocation failed while packing");
    }
}

void shflbw_destroy(shflbw_matrix* A) { delete A; }

int shflbw_info(const shflbw_matrix* A, int* M, int* K, int* V, int* groups, int64_t* nnz,
                double* sparsity)
{
    if (!A) return shflbw::fail(SHFLBW_ERR_NULL_ARG, "A is NULL");
    if (M) *M = A->M;
    if (K) *K = A->K;
    if (V) *V = A->V;
    if (groups) *groups = A->G;
    if (nnz) *nnz = A->nnz;
    if (sparsity) *sparsity = 1.0 - (double)A->nnz / ((double)A->M * (double)A->K);
    return SHFLBW_OK;
}

int shflbw_row_indices(const shflbw_matrix* A, int32_t* rows_out)
{
    if (!A || !rows_out) return shflbw::fail(SHFLBW_ERR_NULL_ARG, "NULL argument");
    std::memcpy(rows_out, A->row_indices.data(), sizeof(int32_t) * (size_t)A->M);
    return SHFLBW_OK;
}

int shflbw_group_columns(const shflbw_matrix* A, int g, int32_t* cols, int cap)
{
    if (!A) return shflbw::fail(SHFLBW_ERR_NULL_ARG, "A is NULL");
    if (g < 0 || g >= A->G) return shflbw::fail(SHFLBW_ERR_BAD_SHAPE, "group index out of range");
    const int kg = A->kcount[g];
    if (!cols) return kg;
    if (cap < kg) return shflbw::fail(SHFLBW_ERR_BAD_SHAPE, "cols buffer too small");
    const int32_t* src = A->col_idx.data() + (size_t)A->step_ptr[g] * A->TK;   // may be empty: no operator[]
    const size_t slots = (size_t)(A->step_ptr[g + 1] - A->step_ptr[g]) * A->TK;
    int n = 0;
    for (size_t t = 0; t < slots; ++t)
        if (src[t] >= 0) cols[n++] = src[t];
    std::sort(cols, cols + n);   // inside a step the columns are not stored in ascending order
    return n;
}

int shflbw_decompress(const shflbw_matrix* A, void* W_out, int ldw)
{
    if (!A || !W_out) return shflbw::fail(SHFLBW_ERR_NULL_ARG, "NULL argument");
    if (ldw < A->K) return shflbw::fail(SHFLBW_ERR_BAD_SHAPE, "ldw < K");
    uint16_t* Wb = static_cast<uint16_t*>(W_out);
    const int V = A->V, TK = A->TK;
    for (int r = 0; r < A->M; ++r) std::memset(Wb + (size_t)r * ldw, 0, sizeof(uint16_t) * A->K);
    for (int g = 0; g < A->G; ++g) {
        const int32_t* rows = &A->row_indices[(size_t)g * V];
        for (size_t step = (size_t)A->step_ptr[g]; step < (size_t)A->step_ptr[g + 1]; ++step) {
            const uint16_t* src = &A->values[step * (size_t)V * TK];
            for (int j = 0; j < TK; ++j) {
                const int k = A->col_idx[step * TK + j];
                if (k < 0) continue;
                for (int i = 0; i < V; ++i)
                    Wb[(size_t)rows[i] * ldw + k] = src[value_slot(V, i, j)];
            }
        }
    }
    return SHFLBW_OK;
}

size_t shflbw_device_bytes(const shflbw_matrix* A) { return A ? A->dev_bytes : 0; }

int shflbw_set_tuning(shflbw_matrix* A, int kernel, int tile_n)
{
    if (!A) return shflbw::fail(SHFLBW_ERR_NULL_ARG, "A is NULL");
    if (kernel < 0 || kernel > 3) return shflbw::fail(SHFLBW_ERR_BAD_OPTION, "kernel must be 0, 1, 2 or 3");
    if (tile_n != 0 && tile_n != 64 && tile_n != 128)
        return shflbw::fail(SHFLBW_ERR_BAD_OPTION, "tile_n must be 0, 64 or 128");
    A->tune_kernel = kernel;
    A->tune_tile_n = tile_n;
    return SHFLBW_OK;
}


int shflbw_set_wait_limit(shflbw_matrix* A, int tries)
{
    if (!A) return shflbw::fail(SHFLBW_ERR_NULL_ARG, "A is NULL");
    if (tries < 0) return shflbw::fail(SHFLBW_ERR_BAD_OPTION, "tries must be >= 0");
    A->wait_limit = tries;
    return SHFLBW_OK;
}

}  // extern "C"
