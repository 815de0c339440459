// Device-facing entry points of the C ABI: binding the packed matrix to a
// caller-owned device buffer, and the launchers of the SpMM / conv2d kernels.
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstring>
#include <mutex>
#include <string>

#include "gather_kernel.hip"
#include "slab_kernel.hip"
#include "conv_kernel.hip"
#include "shflbw_internal.h"
#include "launch_gather.h"

namespace shflbw {
namespace {

// Device image of one packed matrix for shflbw_spmm_unbound: the library's own memory,
// one copy per GPU, held until the process ends.
constexpr size_t STATIC_IMAGE_BYTES = SHFLBW_UNBOUND_MAX_BYTES;
static __device__ __align__(256) unsigned char scratch[STATIC_IMAGE_BYTES];
constexpr int MAX_DEVICES = 64;
void* g_scratch_ptr[MAX_DEVICES];          // address of `scratch` on each device, resolved on first use
std::mutex g_scratch_mutex;

__global__ void clear_status_kernel(int* word)
{
    if (threadIdx.x < 64) word[threadIdx.x] = 0;
}

int hip_fail(hipError_t e, const char* what)
{
    return fail(SHFLBW_ERR_HIP, std::string(what) + ": " + hipGetErrorString(e));
}

// "name<V,second,operand format,output format>" for shflbw_last_kernel
std::string kernel_name(const char* base, int V, int second, bool f32_out, bool bf)
{
    char buf[128];
    snprintf(buf, sizeof buf, "%s<%d,%d,%s,%s>", base, V, second, bf ? "bf16" : "f16",
             f32_out ? "f32 out" : (bf ? "bf16 out" : "f16 out"));
    return buf;
}

PackedView view_of(const shflbw_matrix* A)
{
    const char* b = static_cast<const char*>(device_base(A));
    PackedView v;
    v.row_indices = reinterpret_cast<const int32_t*>(b + A->off_rows);
    v.step_ptr = reinterpret_cast<const int32_t*>(b + A->off_steps);
    v.col_idx = reinterpret_cast<const int32_t*>(b + A->off_cols);
    v.values = reinterpret_cast<const half8*>(b + A->off_vals);
    v.G = A->G;
    return v;
}

template <int V, int GW, typename OutT, bool BF>
int launch_slab(const shflbw_matrix* A, const void* X, long ldx, void* Y, long ldy, long N,
                hipStream_t stream)
{
    SlabArgs a;
    a.A = view_of(A);
    char* base = static_cast<char*>(const_cast<void*>(device_base(A)));
    a.table = reinterpret_cast<const uint32_t*>(base + A->off_table);
    a.first_chunk = reinterpret_cast<const int32_t*>(base + A->off_iter);
    a.status = reinterpret_cast<int*>(base + A->off_status);
    a.spin_limit = A->wait_limit;
    a.X = static_cast<const _Float16*>(X);
    a.Y = Y;
    a.ldx = ldx; a.ldy = ldy; a.N = N;
    a.K = A->K; a.C = A->slab_chunks;
    const long n_tiles = (N + SLAB_TN - 1) / SLAB_TN;
    a.n_tiles = (int)n_tiles;
    constexpr int GROUPS = V == 128 ? GW / 2 : GW;   // row groups per workgroup
    a.gblocks = (A->G + GROUPS - 1) / GROUPS;
    long wgs = ((n_tiles + 7) / 8) * 8 * a.gblocks;
    // packed weights well beyond an L2: blocks of 8 group blocks x 4 column tiles per XCD
    // (fabric traffic of 8192 x 8192 x 16384 at 75 %: 2.7 -> 1.6 GB); the column tiles of an
    // XCD are rounded up to whole blocks
    a.uniform_steps = A->uniform_steps;
    a.gb_side = 0;
    if (a.gblocks % 8 == 0 && A->values.size() * sizeof(uint16_t) > (size_t)(16 << 20)) {
        a.gb_side = 8;
        const long per_xcd = (n_tiles + 7) / 8;                 // column tiles of one XCD
        wgs = (per_xcd + 3) / 4 * 4 * 8 * a.gblocks;
    }
    if (wgs > 0x7fffffffL) return fail(SHFLBW_ERR_BAD_SHAPE, "grid too large");
    hipLaunchKernelGGL((shflbw_slab_kernel<V, GW, OutT, BF>), dim3((unsigned)wgs), dim3(64 * (GW + SLAB_LOADERS)), 0,
                       stream, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(e, "kernel launch");
    note_kernel(kernel_name("shflbw_slab_kernel", V, GW, sizeof(OutT) == 4, BF));
    return SHFLBW_OK;
}

template <typename OutT, bool BF>
int dispatch_slab(const shflbw_matrix* A, const void* X, long ldx, void* Y, long ldy, long N,
                  hipStream_t stream)
{
    switch (A->V) {
        case 16: return launch_slab<16, 12, OutT, BF>(A, X, ldx, Y, ldy, N, stream);
        case 32: return launch_slab<32, 12, OutT, BF>(A, X, ldx, Y, ldy, N, stream);
        case 64: return launch_slab<64, 8, OutT, BF>(A, X, ldx, Y, ldy, N, stream);
        case 128: return launch_slab<128, 8, OutT, BF>(A, X, ldx, Y, ldy, N, stream);
    }
    return fail(SHFLBW_ERR_BAD_OPTION, "the slab kernel supports V = 16, 32, 64, 128");
}

// The gather kernel's instantiations live in their own translation units, one per
// operand format (launch_gather_f16.hip, launch_gather_bf16.hip).
template <class Geom>
int dispatch_out(const shflbw_matrix* A, const Geom& geom, long N, shflbw_dtype ydtype,
                 hipStream_t stream)
{
    if (A->dtype == SHFLBW_BF16) return run_gather_bf16(A, geom, N, ydtype, stream);
    return run_gather_f16(A, geom, N, ydtype, stream);
}

// ydtype must be the operand format of the matrix or fp32
int check_ydtype(const shflbw_matrix* A, shflbw_dtype ydtype)
{
    if (ydtype == SHFLBW_F32 || (int)ydtype == A->dtype) return SHFLBW_OK;
    return fail(SHFLBW_ERR_BAD_DTYPE, A->dtype == SHFLBW_BF16
                    ? "ydtype must be SHFLBW_BF16 or SHFLBW_F32 for a bfloat16 matrix"
                    : "ydtype must be SHFLBW_F16 or SHFLBW_F32 for a binary16 matrix");
}

// Picks the box of output positions one workgroup of the staged convolution
// kernel owns, and fills the geometry part of its arguments.  Returns false
// when no box fits (too many channels for the LDS, or a V the kernel does not
// cover); the caller then takes the gather kernel.
bool plan_conv(const shflbw_matrix* A, int B, int C, int H, int W, int R, int S, int sh, int sw,
               int ph, int pw, int Ho, int Wo, bool chwn, ConvArgs& a, size_t& lds_bytes)
{
    if (A->V != 16 && A->V != 32 && A->V != 64 && A->V != 128) return false;
    if (A->K >= (1 << 20) || (long)R * S >= (1 << 20)) return false;   // exact division by multiplication
    // the kernel addresses the input through a buffer descriptor with 32-bit byte offsets
    const unsigned long long in_total = 2ULL * (unsigned long long)B * C * H * W;
    if (in_total >= 0xffffff00ULL) return false;
    // up to four groups: the wavefronts left over share a group's instruction tiles
    const int gpb = A->G <= 4 ? (A->G > 0 ? A->G : 1) : CONV_GW;
    const int gblocks = (A->G + gpb - 1) / gpb;
    const size_t list_bytes = CONV_LIST_BYTES;   // per-wavefront lists of LDS offsets
    const size_t lds_cap = 160 * 1024 - 512;
    const double kg_avg = A->G > 0 ? (double)A->nnz / ((double)A->V * A->G) : 0.0;
    const double groups_per_box = A->G < CONV_GW ? A->G : CONV_GW;
    // Staging with 4-byte loads wants pairs of elements that are neighbours in memory, 4-byte
    // aligned, and inside or outside the image together.  NCHW: pairs along x - an even image
    // width, boxes that start at even x (tw * sw even), the staged box widened by one column on the
    // left when the padding is odd, and an even staged row pitch.  CHWN: pairs along the batch - an
    // even batch and an even number of images per box.
    // It is asked for when it needs at most 0.7 of the load instructions of 2-byte staging (a
    // wavefront covers 64 elements of a channel per instruction there; with pairs it covers 64
    // pairs, or several channels when a channel has 32 pairs or fewer).
    auto pair_cols = [&](int tw) {
        size_t cols = (size_t)(tw - 1) * sw + S;
        if (!chwn) cols = (cols + (pw & 1) + 1) / 2 * 2;
        return cols;
    };
    auto pairs_ok = [&](int th, int tw, int tb) {
        if (!(chwn ? (B % 2 == 0 && tb % 2 == 0) : (W % 2 == 0 && (tw * sw) % 2 == 0))) return false;
        const size_t rows = (size_t)(th - 1) * sh + R;
        const size_t plane1 = rows * ((size_t)(tw - 1) * sw + S) * tb, plane2 = rows * pair_cols(tw) * tb / 2;
        const size_t lpp = plane2 <= 8 ? 8 : plane2 <= 16 ? 16 : plane2 <= 32 ? 32 : 64;
        const double n1 = (double)((plane1 + 63) / 64), n2 = (double)((plane2 + lpp - 1) / lpp) * (double)lpp / 64.0;
        return n2 <= 0.7 * n1;
    };
    auto staged_cols = [&](int th, int tw, int tb) {
        return pairs_ok(th, tw, tb) ? pair_cols(tw) : (size_t)(tw - 1) * sw + S;
    };
    auto staged_elems = [&](int th, int tw, int tb) {
        return ((size_t)C + 1) * ((size_t)(th - 1) * sh + R) * staged_cols(th, tw, tb) * tb;
    };
    auto fits = [&](int th, int tw, int tb) {
        const size_t e = staged_elems(th, tw, tb);
        return e * 2 + 16 + list_bytes <= lds_cap;   // the staged box and the wavefronts' lists share the LDS
    };
    // Candidate boxes: every split of at most `target` positions into images x rows x
    // columns whose innermost-running dimension keeps runs of 8 where the tensor allows
    // it.  The cost of a split is what all its boxes together read: the staged input
    // (global loads, weighted 4x; the halo of a small box is read again by its
    // neighbours) plus the LDS gathers of every 32-position instruction tile, ragged
    // edge tiles included.
    int th = 1, tw = 1, tb = 1;
    long boxes = 0;
    bool found = false;
    const int targets[3] = {CONV_TN, 64, 32};
    for (int target : targets) {
        if (A->V == 128 && target > 64) continue;   // four row blocks: accumulators for two instruction tiles at most
        double best_cost = 0;
        int bh = 0, bw = 0, bb = 0;
        for (int b = 1; b <= B && b <= target; b = (b < B && 2 * b > B) ? B : 2 * b) {
            if (chwn && b < 8 && b < B) continue;
            for (int w = 1; w <= Wo && b * w <= target; ++w) {
                if (!chwn && w < 8 && w < Wo) continue;
                int h = target / (b * w);
                if (h > Ho) h = Ho;
                if (h < 1) continue;
                while (h > 1 && !fits(h, w, b)) --h;
                if (!fits(h, w, b)) continue;
                const int npos = b * w * h;
                const double nboxes = (double)((B + b - 1) / b) * ((Ho + h - 1) / h) * ((Wo + w - 1) / w);
                const double cost = nboxes * (4.0 * staged_elems(h, w, b) +
                                              (double)((npos + 31) / 32) * 32.0 * kg_avg * groups_per_box);
                if (bh == 0 || cost < best_cost * (1 - 1e-9) ||
                    (cost < best_cost * (1 + 1e-9) && npos > bb * bw * bh)) {
                    best_cost = cost; bh = h; bw = w; bb = b;
                }
            }
            if (b == B) break;
        }
        if (bh == 0) continue;
        th = bh; tw = bw; tb = bb; found = true;
        boxes = (long)((B + tb - 1) / tb) * ((Ho + th - 1) / th) * ((Wo + tw - 1) / tw);
        if (boxes * gblocks >= 256) break;   // enough workgroups to fill the chip
    }
    if (!found || boxes * gblocks > 0x7fffffffL) return false;
    a.B = B; a.C = C; a.H = H; a.W = W; a.R = R; a.S = S; a.sh = sh; a.sw = sw; a.ph = ph; a.pw = pw;
    a.Ho = Ho; a.Wo = Wo; a.K = A->K;
    if (chwn) {
        a.isB = 1; a.isW = B; a.isH = (long)W * B; a.isC = (long)H * W * B;
        a.osB = 1; a.osW = B; a.osH = (long)Wo * B; a.osM = (long)Ho * Wo * B;
    } else {
        a.isW = 1; a.isH = W; a.isC = (long)H * W; a.isB = (long)C * H * W;
        a.osW = 1; a.osH = Wo; a.osM = (long)Ho * Wo; a.osB = (long)A->M * Ho * Wo;
    }
    a.th = th; a.tw = tw; a.tb = tb;
    a.ny = (Ho + th - 1) / th; a.nx = (Wo + tw - 1) / tw; a.nb = (B + tb - 1) / tb;
    a.rows_in = (th - 1) * sh + R; a.cols_in = (int)staged_cols(th, tw, tb);
    a.stage_pairs = pairs_ok(th, tw, tb) ? 1 : 0;
    a.dx = (!chwn && a.stage_pairs) ? (pw & 1) : 0;
    a.b_fast = chwn ? 1 : 0;
    a.gblocks = gblocks;
    a.in_bytes_total = (unsigned)in_total;
    a.gpb = gpb;
    a.uniform_steps = A->uniform_steps;
    {
        const int tiles = (th * tw * tb + 31) / 32;
        const int spare = CONV_GW / gpb;   // wavefronts per group
        a.tsplit = spare < tiles ? spare : tiles;
        if (a.tsplit == 3) a.tsplit = 2;   // tiles per wavefront come as 1, 2 or 4
    }
    auto magic = [](int d) { return (((unsigned long long)1 << 40) + d - 1) / (unsigned long long)d; };
    a.m_RS = magic(R * S); a.m_S = magic(S); a.m_tb = magic(tb); a.m_cols_in = magic(a.cols_in);
    a.m_tw = magic(tw); a.m_th = magic(th);
    a.m_cols2 = magic(a.cols_in / 2 > 0 ? a.cols_in / 2 : 1); a.m_tb2 = magic(tb / 2 > 0 ? tb / 2 : 1);
    size_t in_bytes = (staged_elems(th, tw, tb) * 2 + 15) / 16 * 16;
    const size_t scratch = (size_t)CONV_GW * CONV_SCRATCH;
    if (in_bytes < scratch) in_bytes = scratch;
    a.in_bytes = (int)in_bytes;
    lds_bytes = in_bytes + list_bytes;
    return true;
}

template <int V, int NT, typename OutT, bool BF, bool SP = false>
int launch_conv_nt(const shflbw_matrix* A, ConvArgs& a, size_t lds_bytes, hipStream_t stream)
{
    if constexpr (!SP)
        if (a.stage_pairs == 1) return launch_conv_nt<V, NT, OutT, BF, true>(A, a, lds_bytes, stream);
    a.A = view_of(A);
    // the attribute is raised once per kernel and device, to the most any box can ask for
    static thread_local int raised_on = -1;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e, "hipGetDevice");
    if (raised_on != dev) {
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(&shflbw_conv_kernel<V, NT, OutT, BF, SP>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) return hip_fail(e, "hipFuncSetAttribute");
        raised_on = dev;
    }
    const long wgs = (long)a.nb * a.ny * a.nx * a.gblocks;
    hipLaunchKernelGGL((shflbw_conv_kernel<V, NT, OutT, BF, SP>), dim3((unsigned)wgs), dim3(64 * CONV_GW), lds_bytes,
                       stream, a);
    e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(e, "kernel launch");
    {
        std::string name = kernel_name("shflbw_conv_kernel", V, NT, sizeof(OutT) == 4, BF);
        if (SP) name.insert(name.size() - 1, ",4-byte staging");
        note_kernel(name);
    }
    return SHFLBW_OK;
}

template <int V, typename OutT, bool BF>
int launch_conv(const shflbw_matrix* A, ConvArgs& a, size_t lds_bytes, hipStream_t stream)
{
    const int tiles = (a.tb * a.th * a.tw + 31) / 32;
    const int npos = (tiles + a.tsplit - 1) / a.tsplit * 32;   // positions one wavefront covers
    if (npos <= 32) return launch_conv_nt<V, 1, OutT, BF>(A, a, lds_bytes, stream);
    if (npos <= 64) return launch_conv_nt<V, 2, OutT, BF>(A, a, lds_bytes, stream);
    if constexpr (V <= 64) return launch_conv_nt<V, 4, OutT, BF>(A, a, lds_bytes, stream);
    else return fail(SHFLBW_ERR_BAD_SHAPE, "box too large for V = 128");   // plan_conv never asks for it
}

template <int V>
int dispatch_conv_v(const shflbw_matrix* A, ConvArgs& a, size_t lds_bytes, shflbw_dtype ydtype,
                    hipStream_t stream)
{
    if (A->dtype == SHFLBW_BF16) {
        if (ydtype == SHFLBW_BF16) return launch_conv<V, __bf16, true>(A, a, lds_bytes, stream);
        return launch_conv<V, float, true>(A, a, lds_bytes, stream);
    }
    if (ydtype == SHFLBW_F16) return launch_conv<V, _Float16, false>(A, a, lds_bytes, stream);
    return launch_conv<V, float, false>(A, a, lds_bytes, stream);
}

int dispatch_conv(const shflbw_matrix* A, ConvArgs& a, size_t lds_bytes, shflbw_dtype ydtype,
                  hipStream_t stream)
{
    if (A->V == 16) return dispatch_conv_v<16>(A, a, lds_bytes, ydtype, stream);
    if (A->V == 32) return dispatch_conv_v<32>(A, a, lds_bytes, ydtype, stream);
    if (A->V == 64) return dispatch_conv_v<64>(A, a, lds_bytes, ydtype, stream);
    return dispatch_conv_v<128>(A, a, lds_bytes, ydtype, stream);
}

int check_bound(const shflbw_matrix* A)
{
    if (!device_base(A)) return fail(SHFLBW_ERR_NOT_ON_DEVICE, "call shflbw_bind_device first");
    return SHFLBW_OK;
}

}  // namespace
}  // namespace shflbw

extern "C" {

int shflbw_bind_device(shflbw_matrix* A, void* dev_buf, void* stream)
{
    using namespace shflbw;
    if (!A || !dev_buf) return fail(SHFLBW_ERR_NULL_ARG, "NULL argument");
    if (reinterpret_cast<uintptr_t>(dev_buf) % 256)
        return fail(SHFLBW_ERR_BAD_SHAPE, "dev_buf must be 256-byte aligned");
    hipStream_t st = static_cast<hipStream_t>(stream);
    char* b = static_cast<char*>(dev_buf);
    struct Part { size_t off; const void* src; size_t bytes; };
    const Part parts[] = {
        {A->off_rows, A->row_indices.data(), A->row_indices.size() * sizeof(int32_t)},
        {A->off_steps, A->step_ptr.data(), A->step_ptr.size() * sizeof(int32_t)},
        {A->off_iter, A->first_chunk.data(), A->first_chunk.size() * sizeof(int32_t)},
        {A->off_cols, A->col_idx.data(), A->col_idx.size() * sizeof(int32_t)},
        {A->off_table, A->slab_table.data(), A->slab_table.size() * sizeof(uint32_t)},
        {A->off_vals, A->values.data(), A->values.size() * sizeof(uint16_t)},
    };
    for (const Part& p : parts) {
        if (!p.bytes) continue;
        hipError_t e = hipMemcpyAsync(b + p.off, p.src, p.bytes, hipMemcpyHostToDevice, st);
        if (e != hipSuccess) return hip_fail(e, "hipMemcpyAsync");
    }
    hipError_t e = hipMemsetAsync(b + A->off_status, 0, 256, st);
    if (e != hipSuccess) return hip_fail(e, "hipMemsetAsync");
    e = hipStreamSynchronize(st);
    if (e != hipSuccess) return hip_fail(e, "hipStreamSynchronize");
    A->dev_base = dev_buf;
    return SHFLBW_OK;
}

int shflbw_device_status(shflbw_matrix* A, void* stream)
{
    using namespace shflbw;
    if (!A) return fail(SHFLBW_ERR_NULL_ARG, "A is NULL");
    int rc = check_bound(A);
    if (rc) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    char* word = static_cast<char*>(A->dev_base) + A->off_status;
    int seen = 0;
    hipError_t e = hipMemcpyAsync(&seen, word, sizeof seen, hipMemcpyDeviceToHost, st);
    if (e != hipSuccess) return hip_fail(e, "hipMemcpyAsync");
    e = hipStreamSynchronize(st);
    if (e != hipSuccess) return hip_fail(e, "hipStreamSynchronize");
    if (seen == 0) return SHFLBW_OK;
    e = hipMemsetAsync(word, 0, sizeof seen, st);
    if (e != hipSuccess) return hip_fail(e, "hipMemsetAsync");
    e = hipStreamSynchronize(st);
    if (e != hipSuccess) return hip_fail(e, "hipStreamSynchronize");
    return fail(SHFLBW_ERR_HANDOVER,
                seen == 1 ? "a compute wavefront of the slab kernel gave up waiting for a chunk of X"
                : seen == 2 ? "a loader wavefront of the slab kernel gave up waiting for a free stage"
                            : "compute and loader wavefronts of the slab kernel gave up waiting");
}

int shflbw_spmm(const shflbw_matrix* A, const void* X, int64_t ldx, void* Y, int64_t ldy,
                int64_t N, shflbw_dtype ydtype, void* stream)
{
    using namespace shflbw;
    if (!A) return fail(SHFLBW_ERR_NULL_ARG, "A is NULL");
    if (int rcd = check_ydtype(A, ydtype)) return rcd;
    if (N < 0) return fail(SHFLBW_ERR_BAD_SHAPE, "N < 0");
    if (N == 0) return SHFLBW_OK;
    if (!X || !Y) return fail(SHFLBW_ERR_NULL_ARG, "X and Y must not be NULL");
    if (ldx < N || ldy < N) return fail(SHFLBW_ERR_BAD_SHAPE, "leading dimension smaller than N");
    if (N > (int64_t)1 << 40) return fail(SHFLBW_ERR_BAD_SHAPE, "N too large");
    int rc = check_bound(A);
    if (rc) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const bool aligned = (N % 8 == 0) && (ldx % 8 == 0) && (ldy % 8 == 0) &&
                         (reinterpret_cast<uintptr_t>(X) % 16 == 0) &&
                         (reinterpret_cast<uintptr_t>(Y) % 16 == 0);
    const bool slab_possible = aligned && A->slab_ok;
    if (A->tune_kernel == 2 && !slab_possible)
        return fail(SHFLBW_ERR_BAD_OPTION, "slab kernel needs the windowed layout and aligned operands");
    bool use_slab = A->tune_kernel == 2;
    if (A->tune_kernel == 0 && slab_possible) {
        // automatic choice, from timings of both kernels over the benchmark shapes: the
        // slab kernel streams all of X whatever the sparsity, so it pays when enough of
        // each chunk is used (density), sooner on problems with many tiles; it also
        // needs enough groups to fill its compute wavefronts
        const int gw = A->V == 128 ? 4 : A->V == 64 ? 8 : 12;   // groups per workgroup
        const long tiles = ((N + SLAB_TN - 1) / SLAB_TN) * ((A->G + gw - 1) / gw);
        const double density = (double)A->nnz / ((double)A->M * A->K);
        // Crossovers measured with at least one workgroup per CU: 85 % sparsity for V = 16 and
        // 32, 80-83 % for V = 64 and 128, whose gathered bytes serve more rows.  With fewer
        // workgroups the slab kernel leaves part of the chip idle: from half a round it still pays
        // on the denser half of the range, below that only for V = 16 (whose gather kernel has
        // the least reuse), and on nearly dense matrices.
        double need;
        if (A->V == 16) need = tiles >= 128 ? 0.17 : 0.6;
        else need = tiles >= 256 ? (A->V >= 64 ? 0.19 : 0.17) : tiles >= 128 ? 0.5 : 2.0;
        // very few column tiles: the gather kernel with split k-steps fills the chip better
        const bool skinny = ((N + 63) / 64) * A->G <= 512;
        use_slab = A->G >= gw && density >= need && !skinny;
    }
    if (use_slab) {
        if (A->dtype == SHFLBW_BF16) {
            if (ydtype == SHFLBW_BF16)
                return dispatch_slab<__bf16, true>(A, X, (long)ldx, Y, (long)ldy, (long)N, st);
            return dispatch_slab<float, true>(A, X, (long)ldx, Y, (long)ldy, (long)N, st);
        }
        if (ydtype == SHFLBW_F16)
            return dispatch_slab<_Float16, false>(A, X, (long)ldx, Y, (long)ldy, (long)N, st);
        return dispatch_slab<float, false>(A, X, (long)ldx, Y, (long)ldy, (long)N, st);
    }
    if (aligned) {
        // X behind a buffer descriptor where 24-bit offset arithmetic and a 32-bit range cover it
        const int64_t xbytes = ((int64_t)A->K - 1) * ldx * 2 + N * 2;
        if (A->K < (1 << 24) && ldx * 2 < (1 << 24) && xbytes + 2 * ldx * 2 < ((int64_t)1 << 32) - 64) {
            GeomLinearBuf g;
            g.X = static_cast<const _Float16*>(X);
            g.Y = Y;
            g.ldx = (long)ldx; g.ldy = (long)ldy; g.N = (long)N;
            g.xbytes = (unsigned)xbytes;
            return dispatch_out(A, g, (long)N, ydtype, st);
        }
        GeomLinear<true> g{static_cast<const _Float16*>(X), Y, (long)ldx, (long)ldy, (long)N};
        return dispatch_out(A, g, (long)N, ydtype, st);
    }
    GeomLinear<false> g{static_cast<const _Float16*>(X), Y, (long)ldx, (long)ldy, (long)N};
    return dispatch_out(A, g, (long)N, ydtype, st);
}

int shflbw_spmm_unbound(const shflbw_matrix* A, const void* X, int64_t ldx, void* Y, int64_t ldy,
                        int64_t N, shflbw_dtype ydtype, void* stream)
{
    using namespace shflbw;
    if (!A) return fail(SHFLBW_ERR_NULL_ARG, "A is NULL");
    if (A->dev_bytes > STATIC_IMAGE_BYTES)
        return fail(SHFLBW_ERR_BAD_SHAPE, "packed matrix of " + std::to_string(A->dev_bytes) +
                    " bytes exceeds the library's static device image of " + std::to_string(STATIC_IMAGE_BYTES) +
                    " bytes (SHFLBW_UNBOUND_MAX_BYTES): bind it to a buffer of your own and call shflbw_spmm");
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e, "hipGetDevice");
    if (dev < 0 || dev >= MAX_DEVICES) return fail(SHFLBW_ERR_HIP, "device ordinal out of range");
    char* base;
    {
        // the array's name is a host-side stand-in: its device address comes from the runtime, per device
        std::lock_guard<std::mutex> lock(g_scratch_mutex);
        if (!g_scratch_ptr[dev]) {
            void* p = nullptr;
            e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
            if (e != hipSuccess || !p) return hip_fail(e, "hipGetSymbolAddress(scratch)");
            g_scratch_ptr[dev] = p;
        }
        base = static_cast<char*>(g_scratch_ptr[dev]);
    }
    hipStream_t st = static_cast<hipStream_t>(stream);
    struct Part { size_t off; const void* src; size_t bytes; };
    const Part parts[] = {
        {A->off_rows, A->row_indices.data(), A->row_indices.size() * sizeof(int32_t)},
        {A->off_steps, A->step_ptr.data(), A->step_ptr.size() * sizeof(int32_t)},
        {A->off_iter, A->first_chunk.data(), A->first_chunk.size() * sizeof(int32_t)},
        {A->off_cols, A->col_idx.data(), A->col_idx.size() * sizeof(int32_t)},
        {A->off_table, A->slab_table.data(), A->slab_table.size() * sizeof(uint32_t)},
        {A->off_vals, A->values.data(), A->values.size() * sizeof(uint16_t)},
    };
    for (const Part& p : parts) {
        if (!p.bytes) continue;
        e = hipMemcpyAsync(base + p.off, p.src, p.bytes, hipMemcpyHostToDevice, st);
        if (e != hipSuccess) return hip_fail(e, "hipMemcpyAsync");
    }
    // the status block keeps the last call's contents: it must start at zero (a kernel, not a
    // memset node, so that the call can also be recorded into a graph)
    hipLaunchKernelGGL(clear_status_kernel, dim3(1), dim3(64), 0, st, reinterpret_cast<int*>(base + A->off_status));
    e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(e, "kernel launch");
    set_device_base_override(base);
    const int rc = shflbw_spmm(A, X, ldx, Y, ldy, N, ydtype, stream);
    set_device_base_override(nullptr);
    return rc;
}

int shflbw_conv2d(const shflbw_matrix* A, const void* in, void* out, int batch, int C_in, int H,
                  int W, int R, int S, int stride_h, int stride_w, int pad_h, int pad_w,
                  shflbw_layout layout, shflbw_dtype ydtype, void* stream)
{
    using namespace shflbw;
    if (!A) return fail(SHFLBW_ERR_NULL_ARG, "A is NULL");
    if (int rcd = check_ydtype(A, ydtype)) return rcd;
    if (layout != SHFLBW_NCHW && layout != SHFLBW_CHWN)
        return fail(SHFLBW_ERR_BAD_SHAPE, "unknown layout");
    if (batch < 0 || C_in <= 0 || H <= 0 || W <= 0 || R <= 0 || S <= 0 || stride_h <= 0 ||
        stride_w <= 0 || pad_h < 0 || pad_w < 0)
        return fail(SHFLBW_ERR_BAD_SHAPE, "non-positive convolution dimension");
    if ((int64_t)C_in * R * S != A->K)
        return fail(SHFLBW_ERR_BAD_SHAPE, "C_in*R*S does not match the packed matrix's K");
    if (H + 2 * pad_h < R || W + 2 * pad_w < S)
        return fail(SHFLBW_ERR_BAD_SHAPE, "kernel larger than the padded input");
    if (H + 2 * pad_h > 32767 || W + 2 * pad_w > 32767)
        return fail(SHFLBW_ERR_BAD_SHAPE, "padded image side above 32767");
    const int Ho = (H + 2 * pad_h - R) / stride_h + 1;
    const int Wo = (W + 2 * pad_w - S) / stride_w + 1;
    const int64_t N = (int64_t)batch * Ho * Wo;
    if (N == 0) return SHFLBW_OK;
    if (!in || !out) return fail(SHFLBW_ERR_NULL_ARG, "in and out must not be NULL");
    const int64_t lim = (int64_t)1 << 31;
    // 32-bit element offsets inside the kernel, including the padded halo
    if ((int64_t)batch * C_in * (H + 2 * pad_h) * (W + 2 * pad_w) >= lim ||
        (int64_t)A->M * N >= lim)
        return fail(SHFLBW_ERR_BAD_SHAPE, "tensor above 2^31 elements");
    int rc = check_bound(A);
    if (rc) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    // A 1x1 convolution with unit stride and no padding on a batch-innermost tensor IS the
    // linear-layer product: [C_in][H*W*batch] in, [C_out][H*W*batch] out, both row-major.
    if (A->tune_kernel == 0 && layout == SHFLBW_CHWN && R == 1 && S == 1 && stride_h == 1 &&
        stride_w == 1 && pad_h == 0 && pad_w == 0)
        return shflbw_spmm(A, in, N, out, N, N, ydtype, stream);
    // The same on NCHW tensors is one such product per image; with H*W a multiple of 4 the
    // gather kernel takes all images in one launch (a lane's columns stay inside an image in
    // runs of 8, or of 4),
    // reading only the channels a group keeps instead of staging every channel of a box.
    {
        const int64_t HW = (int64_t)H * W;
        const int64_t in_total = 2 * (int64_t)batch * C_in * HW;
        if (A->tune_kernel == 0 && layout == SHFLBW_NCHW && R == 1 && S == 1 && stride_h == 1 &&
            stride_w == 1 && pad_h == 0 && pad_w == 0 && HW % 4 == 0 && HW * 2 < (1 << 24) &&
            C_in < (1 << 24) && in_total < ((int64_t)1 << 32) - 64 &&
            reinterpret_cast<uintptr_t>(in) % 16 == 0 && reinterpret_cast<uintptr_t>(out) % 16 == 0) {
            auto fill = [&](auto& g) {
                g.X = static_cast<const _Float16*>(in);
                g.Y = out;
                g.ldx = (long)HW; g.ldy = (long)HW; g.N = (long)N;
                g.xbytes = (unsigned)in_total;
                g.HW = (int)HW; g.K = C_in; g.M = A->M;
            };
            if (HW % 8 == 0) {
                GeomBatchedBuf g;
                fill(g);
                return dispatch_out(A, g, (long)N, ydtype, st);
            }
            // H*W a multiple of 4 only: every load and 8-wide store in two halves
            GeomBatchedBuf4 g;
            fill(g);
            return dispatch_out(A, g, (long)N, ydtype, st);
        }
    }
    if (A->tune_kernel != 1 && A->tune_kernel != 3) {
        // the plan depends on the matrix and the geometry only: keep the last one
        struct PlanKey { const shflbw_matrix* A; int64_t nnz; int v[14]; };
        static thread_local PlanKey last_key = {nullptr, 0, {0}};
        static thread_local bool last_ok = false;
        static thread_local ConvArgs last_args;
        static thread_local size_t last_lds = 0;
        const PlanKey key = {A, A->nnz, {A->K, A->V, A->G, batch, C_in, H, W, R * 65536 + S,
                                         stride_h * 65536 + stride_w, pad_h, pad_w, (int)layout, A->M, 0}};
        if (memcmp(&key, &last_key, sizeof key) != 0) {
            last_ok = plan_conv(A, batch, C_in, H, W, R, S, stride_h, stride_w, pad_h, pad_w, Ho, Wo,
                                layout == SHFLBW_CHWN, last_args, last_lds);
            last_key = key;
        }
        if (last_ok) {
            ConvArgs ca = last_args;
            const size_t lds_bytes = last_lds;
            ca.in = static_cast<const _Float16*>(in);
            ca.out = out;
            if (reinterpret_cast<uintptr_t>(in) % 4) ca.stage_pairs = 2;   // laid out for pairs, staged with 2-byte loads
            return dispatch_conv(A, ca, lds_bytes, ydtype, st);
        }
        if (A->tune_kernel == 2)
            return fail(SHFLBW_ERR_BAD_OPTION,
                        "staged convolution kernel needs an input box that fits the LDS");
    }
    GeomConv g;
    g.in = static_cast<const _Float16*>(in);
    g.out = out;
    g.B = batch; g.Cin = C_in; g.H = H; g.W = W; g.Cout = A->M; g.R = R; g.S = S;
    g.sh = stride_h; g.sw = stride_w; g.ph = pad_h; g.pw = pad_w; g.Ho = Ho; g.Wo = Wo;
    g.chwn = (layout == SHFLBW_CHWN);
    g.N = N;
    return dispatch_out(A, g, (long)N, ydtype, st);
}

}  // extern "C"
