// L2-to-LDS streaming probe (measurement aid for the benchmark, not part of
// the product path).  It moves data the way the slab kernel's loader
// wavefronts do - direct global-to-LDS loads of 16 bytes per lane, 64-row x
// 256-byte chunks of a row-major matrix, a fixed number of chunks in flight -
// and nothing else, so its rate is the ceiling for that kernel's activation
// stream:
//   mode 0  256 workgroups re-read 64 slabs `passes` times, four sharers per
//           slab, the 8 slabs of an XCD (2 MB at K = 1024) staying in its L2
//           (what the L2s can deliver into the CUs at best);
//   mode 1  the slab kernel's grid and sharing pattern (workgroups that share
//           a slab run side by side on one XCD), one pass, operands cold.
// Built as its own small library (bench_l2_probe.so, next to bench.py, by
// bench.build_probe()); only bench.py loads it.
#include <hip/hip_runtime.h>

#include <cstdint>

namespace {

constexpr int PROBE_KC = 64;        // rows per chunk
constexpr int PROBE_STAGES = 8;     // LDS ring
constexpr int PROBE_LEAD = 4;       // chunks in flight
constexpr int PROBE_LOADERS = 4;    // wavefronts per workgroup

__device__ __forceinline__ void dma16(const void* g, unsigned lds_off)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"
                 :: "s"(lds_off), "v"(g) : "memory");
}

__global__ __launch_bounds__(64 * PROBE_LOADERS) void l2_stream_kernel(
    const uint16_t* X, long ldx, int K, int n_tiles, int gblocks, int passes, float* sink)
{
    __shared__ __attribute__((aligned(1024))) char smem[PROBE_STAGES * PROBE_KC * 256];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const unsigned base = (unsigned)(size_t)(__attribute__((address_space(3))) char*)smem;
    const int lrow = lane >> 4, lpos = lane & 15;
    const int C = K / PROBE_KC;                      // K is a multiple of 64 (checked on the host)
    const int wg = blockIdx.x, xcd = wg & 7, wslot = wg >> 3;
    const int nt = xcd * ((n_tiles + 7) / 8) + wslot / gblocks;   // the slab kernel's mapping
    if (nt >= n_tiles) return;
    const uint16_t* Xt = X + (long)nt * 128;
    const int total = C * passes;
    auto issue = [&](int cg) __attribute__((always_inline)) {
        const int c = cg % C;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int piece = wave * 4 + i;
            const int row = c * PROBE_KC + 4 * piece + lrow;
            dma16(Xt + (long)row * ldx + lpos * 8,
                  base + (cg % PROBE_STAGES) * (PROBE_KC * 256) + piece * 1024);
        }
    };
#pragma unroll
    for (int cg = 0; cg < PROBE_LEAD; ++cg)
        if (cg < total) issue(cg);
    for (int cg = 0; cg < total; ++cg) {
        int younger = total - 1 - cg;
        younger = younger < PROBE_LEAD - 1 ? younger : PROBE_LEAD - 1;
        switch (younger) {
            case 0: asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); break;
            case 1: asm volatile("s_waitcnt vmcnt(4)" ::: "memory"); break;
            case 2: asm volatile("s_waitcnt vmcnt(8)" ::: "memory"); break;
            default: asm volatile("s_waitcnt vmcnt(12)" ::: "memory"); break;
        }
        static_assert(PROBE_LEAD <= 4, "extend the switch above");
        if (cg + PROBE_LEAD < total) issue(cg + PROBE_LEAD);
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (threadIdx.x == 0 && *(volatile float*)(smem + 4 * (wg & 63)) == 12345.678f) sink[0] = 1.f;
}

// LDS read rate: every wavefront issues batches of eight independent 8-byte-per-lane reads at
// conflict-free addresses, transposing (ds_read_b64_tr_b16, what the slab kernel feeds its
// matrix instructions with) or plain (ds_read_b64).
typedef short probe_short4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) probe_short4* probe_lds_short4_ptr;
template <bool TRANSPOSING>
__global__ __launch_bounds__(1024) void lds_read_kernel(int iters, float* sink)
{
    __shared__ __attribute__((aligned(1024))) char smem[64 * 1024];
    for (int i = threadIdx.x; i < 64 * 1024 / 4; i += blockDim.x) reinterpret_cast<int*>(smem)[i] = i;
    __syncthreads();
    const unsigned base = (unsigned)(size_t)(__attribute__((address_space(3))) char*)smem + (threadIdx.x & 63) * 8;
    typedef unsigned probe_uint2 __attribute__((ext_vector_type(2)));
    unsigned acc = 0;
    // The reads are volatile assembly so that the compiler neither merges reads of equal addresses
    // across iterations nor moves them; the wait names the results so that their uses stay behind it.
    for (int it = 0; it < iters; ++it) {
        const unsigned a = base + (it & 3) * 16384;
        probe_uint2 v0, v1, v2, v3, v4, v5, v6, v7;
#define PROBE_READ(V, OFF)                                                                              \
        if (TRANSPOSING) asm volatile("ds_read_b64_tr_b16 %0, %1 offset:" #OFF : "=v"(V) : "v"(a));       \
        else asm volatile("ds_read_b64 %0, %1 offset:" #OFF : "=v"(V) : "v"(a));
        PROBE_READ(v0, 0) PROBE_READ(v1, 2048) PROBE_READ(v2, 4096) PROBE_READ(v3, 6144)
        PROBE_READ(v4, 8192) PROBE_READ(v5, 10240) PROBE_READ(v6, 12288) PROBE_READ(v7, 14336)
#undef PROBE_READ
        asm volatile("s_waitcnt lgkmcnt(0)"
                     : "+v"(v0), "+v"(v1), "+v"(v2), "+v"(v3), "+v"(v4), "+v"(v5), "+v"(v6), "+v"(v7));
        acc ^= v0[0] ^ v1[1] ^ v2[0] ^ v3[1] ^ v4[0] ^ v5[1] ^ v6[0] ^ v7[1];
    }
    if (acc == 0x12345678u) sink[0] = 1.f;
}


// Loads and stores of one CU together: wavefronts 0-3 stream 128-column slabs of X into LDS as above
// (`passes` times 16 chunks of 64 rows), wavefronts 4-15 write `tiles` tiles of 32 rows x 256 bytes of
// Y each with non-temporal 16-byte stores, 8 rows x 128 bytes per instruction - the slab kernel's
// write-back pattern.  Either half can be switched off.
typedef unsigned probe_uint4 __attribute__((ext_vector_type(4)));
__global__ __launch_bounds__(1024) void stream_store_kernel(const uint16_t* X, long ldx, uint16_t* Y, long ldy,
                                                             int do_stream, int do_store, int passes, int tiles,
                                                             float* sink)
{
    __shared__ __attribute__((aligned(1024))) char smem[PROBE_STAGES * PROBE_KC * 256];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wg = blockIdx.x, xcd = wg & 7, wslot = wg >> 3;
    if (wave < PROBE_LOADERS) {
        if (!do_stream) return;
        const unsigned base = (unsigned)(size_t)(__attribute__((address_space(3))) char*)smem;
        const int lrow = lane >> 4, lpos = lane & 15;
        const uint16_t* Xt = X + (long)(xcd * 8 + wslot / 4) * 128;      // 64 slabs, 4 sharers each
        const int total = 16 * passes;
        auto issue = [&](int cg) __attribute__((always_inline)) {
            const int c = cg % 16;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int piece = wave * 4 + i;
                const int row = c * PROBE_KC + 4 * piece + lrow;
                dma16(Xt + (long)row * ldx + lpos * 8,
                      base + (cg % PROBE_STAGES) * (PROBE_KC * 256) + piece * 1024);
            }
        };
#pragma unroll
        for (int cg = 0; cg < PROBE_LEAD; ++cg)
            if (cg < total) issue(cg);
        for (int cg = 0; cg < total; ++cg) {
            int younger = total - 1 - cg;
            younger = younger < PROBE_LEAD - 1 ? younger : PROBE_LEAD - 1;
            switch (younger) {
                case 0: asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); break;
                case 1: asm volatile("s_waitcnt vmcnt(4)" ::: "memory"); break;
                case 2: asm volatile("s_waitcnt vmcnt(8)" ::: "memory"); break;
                default: asm volatile("s_waitcnt vmcnt(12)" ::: "memory"); break;
            }
            if (cg + PROBE_LEAD < total) issue(cg + PROBE_LEAD);
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        if (lane == 0 && *(volatile float*)(smem + 4 * (wg & 63)) == 12345.678f) sink[0] = 1.f;
        return;
    }
    if (!do_store) return;
    const long row0 = ((long)(wg % 10) * 12 + (wave - PROBE_LOADERS)) * 32;   // below 3840
    const probe_uint4 v = {0x3c003c00u, 0x3c003c00u, 0x3c003c00u, 0x3c003c00u};
    for (int i = 0; i < tiles; ++i) {
        const int ct = (wg / 10 + 26 * i) % 64;
#pragma unroll
        for (int p = 0; p < 2; ++p)
#pragma unroll
            for (int r = 0; r < 4; ++r)
                __builtin_nontemporal_store(
                    v, reinterpret_cast<probe_uint4*>(Y + (row0 + r * 8 + (lane >> 3)) * ldy + ct * 128 + p * 64 + (lane & 7) * 8));
    }
}

}  // namespace

extern "C" {

/* 256 workgroups of `waves` wavefronts each read `iters` x 8 x 512 bytes of LDS per wavefront, with
 * the transposing 16-bit read (transposing != 0) or the plain 8-byte read.  Enqueues on `stream`;
 * returns the bytes read over the chip, or a negative value on bad arguments. */
long long shflbw_probe_lds_read(int transposing, int waves, int iters, void* sink, void* stream)
{
    if (!sink || waves < 1 || waves > 16 || iters < 1) return -1;
    if (transposing)
        hipLaunchKernelGGL(lds_read_kernel<true>, dim3(256), dim3(64 * waves), 0, static_cast<hipStream_t>(stream), iters, static_cast<float*>(sink));
    else
        hipLaunchKernelGGL(lds_read_kernel<false>, dim3(256), dim3(64 * waves), 0, static_cast<hipStream_t>(stream), iters, static_cast<float*>(sink));
    if (hipGetLastError() != hipSuccess) return -2;
    return 256LL * waves * iters * 8 * 512;
}


/* 256 workgroups of 16 wavefronts: four stream slabs of the row-major 16-bit matrix X (at least 1024
 * rows and 8192 columns) into LDS, `passes` x 256 KB per workgroup, twelve write `tiles` tiles of 32
 * rows x 256 bytes each to the row-major 16-bit matrix Y (at least 3840 rows and 8192 columns).
 * Enqueues on `stream`; *load_bytes and *store_bytes receive what was moved; returns 0, or a negative
 * value on bad arguments. */
int shflbw_probe_stream_store(const void* X, long long ldx, void* Y, long long ldy, int do_stream, int do_store,
                              int passes, int tiles, long long* load_bytes, long long* store_bytes, void* sink,
                              void* stream)
{
    if (!X || !Y || !sink || !load_bytes || !store_bytes || ldx < 8192 || ldy < 8192 || passes < 1 || tiles < 1)
        return -1;
    hipLaunchKernelGGL(stream_store_kernel, dim3(256), dim3(1024), 0, static_cast<hipStream_t>(stream),
                       static_cast<const uint16_t*>(X), (long)ldx, static_cast<uint16_t*>(Y), (long)ldy, do_stream,
                       do_store, passes, tiles, static_cast<float*>(sink));
    if (hipGetLastError() != hipSuccess) return -2;
    *load_bytes = do_stream ? 256LL * passes * 16 * PROBE_KC * 256 : 0;
    *store_bytes = do_store ? 256LL * 12 * tiles * 32 * 256 : 0;
    return 0;
}

/* Streams K x 128-column slabs of the row-major 16-bit matrix X (K x N, leading dimension
 * ldx, device memory) into LDS.  mode 0: 256 workgroups over the first 64 slabs, `passes` times.
 * mode 1: the slab kernel's grid for `gblocks` sharers per slab, one pass.  Enqueues on
 * `stream`; returns the bytes moved into LDS, or a negative value on bad arguments.
 * K must be a multiple of 64, N a multiple of 128 and at least 8192. */
long long shflbw_probe_l2_stream(const void* X, long long ldx, int K, long long N, int mode,
                                 int gblocks, int passes, void* sink, void* stream)
{
    if (!X || !sink || K <= 0 || K % PROBE_KC || N < 8192 || N % 128 || ldx < N || passes < 1 ||
        gblocks < 1)
        return -1;
    const int n_tiles = (int)(N / 128);
    int wgs, gb;
    int tiles = n_tiles;
    if (mode == 0) { gb = 4; tiles = 64; wgs = 256; }
    else { gb = gblocks; passes = 1; wgs = (n_tiles + 7) / 8 * 8 * gb; }
    if (tiles > n_tiles) return -1;
    hipLaunchKernelGGL(l2_stream_kernel, dim3((unsigned)wgs), dim3(64 * PROBE_LOADERS), 0,
                       static_cast<hipStream_t>(stream), static_cast<const uint16_t*>(X), (long)ldx, K,
                       tiles, gb, passes, static_cast<float*>(sink));
    if (hipGetLastError() != hipSuccess) return -2;
    long long active = 0;   // workgroups whose column tile exists
    for (int wg = 0; wg < wgs; ++wg)
        if ((wg & 7) * ((tiles + 7) / 8) + (wg >> 3) / gb < tiles) ++active;
    return active * (long long)K * 256 * passes;
}

}  // extern "C"
