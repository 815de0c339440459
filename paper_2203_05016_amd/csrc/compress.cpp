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
}  // namespace

namespace shflbw {
int fail(int status, const std::string& detail)
{
    g_last_error = detail;
    return status;
}
}  // namespace shflbw

extern "C" {

const char* shflbw_last_error(void) { return g_last_error.c_str(); }

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
        default: return "unknown status";
    }
}

int shflbw_compress(const void* W, int ldw, const uint8_t* mask, const int32_t* perm,
                    int M, int K, int V, shflbw_dtype wdtype, shflbw_matrix** out)
{
    using shflbw::fail;
    if (!W || !out) return fail(SHFLBW_ERR_NULL_ARG, "W and out must not be NULL");
    *out = nullptr;
    if (wdtype != SHFLBW_F16) return fail(SHFLBW_ERR_BAD_DTYPE, "weights must be SHFLBW_F16");
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

        A->step_ptr.assign(G + 1, 0);
        A->kcount.resize(G);
        for (int g = 0; g < G; ++g) {
            int kg = (int)cols[g].size();
            A->kcount[g] = kg;
            A->nnz += (int64_t)kg * V;
            A->step_ptr[g + 1] = A->step_ptr[g] + (kg + TK - 1) / TK;
        }
        const size_t steps = (size_t)A->step_ptr[G];
        A->col_idx.assign(steps * TK, -1);
        A->values.assign(steps * (size_t)V * TK, 0);
        for (int g = 0; g < G; ++g) {
            const int32_t* rows = &A->row_indices[(size_t)g * V];
            const size_t s0 = (size_t)A->step_ptr[g];
            for (int t = 0; t < (int)cols[g].size(); ++t) {
                const int k = cols[g][t];
                const size_t step = s0 + t / TK;
                const int j = t % TK;
                A->col_idx[step * TK + j] = k;
                uint16_t* dst = &A->values[step * (size_t)V * TK];
                for (int i = 0; i < V; ++i)
                    dst[value_slot(V, i, j)] = Wb[(size_t)rows[i] * ldw + k];
            }
        }

        A->off_rows = 0;
        A->off_steps = shflbw::align256(A->off_rows + sizeof(int32_t) * (size_t)M);
        A->off_cols = shflbw::align256(A->off_steps + sizeof(int32_t) * (size_t)(G + 1));
        A->off_vals = shflbw::align256(A->off_cols + sizeof(int32_t) * A->col_idx.size());
        A->dev_bytes = shflbw::align256(A->off_vals + sizeof(uint16_t) * A->values.size());
        if (A->dev_bytes == 0) A->dev_bytes = 256;

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
    const int32_t* src = &A->col_idx[(size_t)A->step_ptr[g] * A->TK];
    std::memcpy(cols, src, sizeof(int32_t) * (size_t)kg);
    return kg;
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
        const size_t s0 = (size_t)A->step_ptr[g];
        for (int t = 0; t < A->kcount[g]; ++t) {
            const size_t step = s0 + t / TK;
            const int j = t % TK;
            const int k = A->col_idx[step * TK + j];
            const uint16_t* src = &A->values[step * (size_t)V * TK];
            for (int i = 0; i < V; ++i) Wb[(size_t)rows[i] * ldw + k] = src[value_slot(V, i, j)];
        }
    }
    return SHFLBW_OK;
}

size_t shflbw_device_bytes(const shflbw_matrix* A) { return A ? A->dev_bytes : 0; }

int shflbw_set_tuning(shflbw_matrix* A, int kernel, int tile_n)
{
    if (!A) return shflbw::fail(SHFLBW_ERR_NULL_ARG, "A is NULL");
    if (kernel < 0 || kernel > 1) return shflbw::fail(SHFLBW_ERR_BAD_OPTION, "kernel must be 0 or 1");
    if (tile_n != 0 && tile_n != 64 && tile_n != 128)
        return shflbw::fail(SHFLBW_ERR_BAD_OPTION, "tile_n must be 0, 64 or 128");
    A->tune_kernel = kernel;
    A->tune_tile_n = tile_n;
    return SHFLBW_OK;
}

}  // extern "C"
