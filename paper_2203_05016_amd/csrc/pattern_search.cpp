// Host-side pattern search for the Shfl-BW pattern (Section 5): given the
// weights, decide the row shuffle and which V x 1 vectors to keep.
//
// Steps, in the paper's order: importance = |w|; unstructured pruning to the
// ratio beta gives a binary mask; K-Means with clusters of fixed size V on
// the rows of that mask decides which rows share a group; vector-wise
// pruning to the ratio alpha on the shuffled matrix; the mask is returned in
// the original row order, together with the permutation.
//
// Where the paper leaves choices open this file takes: magnitudes compared by
// the 15 low bits of the binary16 pattern, ties to the lower flat index;
// clusters start as consecutive blocks of V rows; a round assigns greedily
// over all (row, cluster) pairs by increasing squared distance to the
// cluster centre (ties: lower row, then lower cluster) while the row is free
// and the cluster has room; distances and vector scores are exact integers
// (V^2 |b - c|^2, and sums of |w| in units of 2^-24), so the result does not
// depend on floating-point summation order; every group keeps round(alpha K)
// vectors, ties to the lower column.  bfloat16 weights take the same steps:
// their magnitude bits order them like binary16's do, and a vector's score is
// summed exactly in a 320-bit integer (units of 2^-133), since 64 bits cannot
// hold bfloat16's exponent range.
//
// Cost: one K-Means round is O(M * G * K) byte operations (every row against
// every cluster centre) and holds M*G 8-byte distances plus M*G 4-byte pair
// indices; the unstructured step holds M*K 4-byte indices.  Flat indices are
// 32-bit: M*K and M*G above 2^32 - 1 are refused.
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <numeric>
#include <string>
#include <vector>

#include "shflbw.h"
#include "shflbw_internal.h"

namespace {

// |w| * 2^24 of a finite binary16 value, exactly
inline int64_t half_magnitude_fixed(uint16_t h)
{
    const int e = (h >> 10) & 31, f = h & 1023;
    if (e == 0) return f;                        // f * 2^-24
    return (int64_t)(1024 + f) << (e - 1);       // (1024 + f) * 2^(e - 25) * 2^24
}

// |w| of a finite bfloat16 value in units of 2^-133, added into a 320-bit sum
struct Wide {
    uint64_t limb[5] = {0, 0, 0, 0, 0};
    void add_bfloat16_magnitude(uint16_t h)
    {
        const int e = (h >> 7) & 255, f = h & 127;
        const uint64_t mant = e == 0 ? (uint64_t)f : (uint64_t)(128 + f);
        const int shift = e == 0 ? 0 : e - 1;          // at most 253
        const int word = shift / 64, bit = shift % 64;
        uint64_t lo = mant << bit, hi = bit ? mant >> (64 - bit) : 0;
        unsigned __int128 c = (unsigned __int128)limb[word] + lo;
        limb[word] = (uint64_t)c;
        c = (c >> 64) + hi;
        for (int w = word + 1; w < 5 && c; ++w) {
            c += limb[w];
            limb[w] = (uint64_t)c;
            c >>= 64;
        }
    }
    bool operator==(const Wide& o) const
    {
        for (int w = 0; w < 5; ++w) if (limb[w] != o.limb[w]) return false;
        return true;
    }
    bool operator>(const Wide& o) const
    {
        for (int w = 4; w >= 0; --w) if (limb[w] != o.limb[w]) return limb[w] > o.limb[w];
        return false;
    }
};

}  // namespace

extern "C" int shflbw_pattern_search(const void* W, int ldw, int M, int K, int V, double alpha,
                                     double beta, int iterations, shflbw_dtype wdtype,
                                     int32_t* perm_out, uint8_t* mask_out)
{
    using shflbw::fail;
    if (!W || !perm_out || !mask_out) return fail(SHFLBW_ERR_NULL_ARG, "NULL argument");
    if (wdtype != SHFLBW_F16 && wdtype != SHFLBW_BF16)
        return fail(SHFLBW_ERR_BAD_DTYPE, "pattern search takes SHFLBW_F16 or SHFLBW_BF16 weights");
    const bool bf = wdtype == SHFLBW_BF16;
    if (V != 16 && V != 32 && V != 64 && V != 128)
        return fail(SHFLBW_ERR_BAD_SHAPE, "V must be 16, 32, 64 or 128");
    if (M <= 0 || K <= 0 || M % V || ldw < K) return fail(SHFLBW_ERR_BAD_SHAPE, "bad M, K or ldw");
    if ((uint64_t)M * (uint64_t)K > 0xffffffffULL || (uint64_t)M * (uint64_t)(M / V) > 0xffffffffULL)
        return fail(SHFLBW_ERR_BAD_SHAPE, "pattern search indexes weights and (row, cluster) pairs with 32 bits: "
                                          "M*K and M*(M/V) must stay below 2^32");
    if (!(alpha >= 0.0 && alpha <= 1.0) || !(beta <= 1.0) || iterations < 0)
        return fail(SHFLBW_ERR_BAD_OPTION, "alpha in [0,1], beta <= 1 (negative: 2*alpha), iterations >= 0");
    if (beta < 0.0) beta = std::min(1.0, 2.0 * alpha);
    try {
        const uint16_t* Wb = static_cast<const uint16_t*>(W);
        const size_t MK = (size_t)M * K;
        const int G = M / V;
        for (int i = 0; i < M; ++i)
            for (int k = 0; k < K; ++k)
                if (bf ? ((Wb[(size_t)i * ldw + k] >> 7) & 255) == 255 : ((Wb[(size_t)i * ldw + k] >> 10) & 31) == 31)
                    return fail(SHFLBW_ERR_BAD_PATTERN, "pattern search needs finite weights");

        // ---- unstructured pruning to the ratio beta: a binary mask B
        size_t keep = (size_t)std::llround(beta * (double)MK);
        keep = std::min(keep, MK);
        std::vector<uint32_t> order(MK);
        std::iota(order.begin(), order.end(), 0u);
        auto key = [&](uint32_t idx) { return (int)(Wb[(size_t)(idx / K) * ldw + idx % K] & 0x7fff); };
        auto by_score = [&](uint32_t a, uint32_t b) {
            const int ka = key(a), kb = key(b);
            return ka != kb ? ka > kb : a < b;
        };
        if (keep > 0 && keep < MK) std::nth_element(order.begin(), order.begin() + (keep - 1), order.end(), by_score);
        std::vector<uint8_t> B(MK, 0);
        for (size_t t = 0; t < keep; ++t) B[order[t]] = 1;
        order.clear(); order.shrink_to_fit();

        // ---- K-Means with clusters of fixed size V on the rows of B
        std::vector<int32_t> assign(M), next(M);
        for (int i = 0; i < M; ++i) assign[i] = i / V;
        std::vector<int64_t> ones(M, 0);
        for (int i = 0; i < M; ++i)
            for (int k = 0; k < K; ++k) ones[i] += B[(size_t)i * K + k];
        std::vector<int32_t> counts((size_t)G * K);
        std::vector<int64_t> csq(G), dist((size_t)M * G);
        std::vector<uint32_t> pairs((size_t)M * G);
        std::vector<int32_t> room(G);
        for (int it = 0; it < iterations; ++it) {
            std::fill(counts.begin(), counts.end(), 0);
            for (int i = 0; i < M; ++i) {
                int32_t* c = &counts[(size_t)assign[i] * K];
                const uint8_t* b = &B[(size_t)i * K];
                for (int k = 0; k < K; ++k) c[k] += b[k];
            }
            for (int g = 0; g < G; ++g) {
                int64_t s = 0;
                for (int k = 0; k < K; ++k) s += (int64_t)counts[(size_t)g * K + k] * counts[(size_t)g * K + k];
                csq[g] = s;
            }
            for (int i = 0; i < M; ++i) {
                const uint8_t* b = &B[(size_t)i * K];
                for (int g = 0; g < G; ++g) {
                    const int32_t* c = &counts[(size_t)g * K];
                    int64_t dot = 0;
                    for (int k = 0; k < K; ++k) dot += b[k] ? c[k] : 0;
                    dist[(size_t)i * G + g] = (int64_t)V * V * ones[i] - 2 * (int64_t)V * dot + csq[g];
                }
            }
            std::iota(pairs.begin(), pairs.end(), 0u);   // pair index = row * G + cluster: ties resolve by it
            std::sort(pairs.begin(), pairs.end(), [&](uint32_t a, uint32_t b) {
                return dist[a] != dist[b] ? dist[a] < dist[b] : a < b;
            });
            std::fill(next.begin(), next.end(), -1);
            std::fill(room.begin(), room.end(), V);
            int left = M;
            for (uint32_t pr : pairs) {
                const int r = (int)(pr / G), c = (int)(pr % G);
                if (next[r] < 0 && room[c] > 0) {
                    next[r] = c;
                    --room[c];
                    if (--left == 0) break;
                }
            }
            if (next == assign) break;
            assign.swap(next);
        }

        // ---- the row shuffle: by cluster, rows of a cluster in their original order
        std::vector<int32_t> perm(M);
        std::iota(perm.begin(), perm.end(), 0);
        std::stable_sort(perm.begin(), perm.end(), [&](int32_t a, int32_t b) { return assign[a] < assign[b]; });

        // ---- vector-wise pruning to the ratio alpha on the shuffled matrix
        int kg = (int)std::llround(alpha * (double)K);
        kg = std::max(0, std::min(K, kg));
        std::fill(mask_out, mask_out + MK, (uint8_t)0);
        std::vector<int64_t> vscore(bf ? 0 : K);
        std::vector<Wide> wscore(bf ? K : 0);
        std::vector<int32_t> cols(K);
        for (int g = 0; g < G; ++g) {
            if (bf) std::fill(wscore.begin(), wscore.end(), Wide());
            else std::fill(vscore.begin(), vscore.end(), 0);
            for (int i = 0; i < V; ++i) {
                const uint16_t* w = Wb + (size_t)perm[(size_t)g * V + i] * ldw;
                if (bf) for (int k = 0; k < K; ++k) wscore[k].add_bfloat16_magnitude(w[k] & 0x7fff);
                else for (int k = 0; k < K; ++k) vscore[k] += half_magnitude_fixed(w[k] & 0x7fff);
            }
            std::iota(cols.begin(), cols.end(), 0);
            auto by_vs = [&](int32_t a, int32_t b) {
                if (bf) return wscore[a] == wscore[b] ? a < b : wscore[a] > wscore[b];
                return vscore[a] != vscore[b] ? vscore[a] > vscore[b] : a < b;
            };
            if (kg > 0 && kg < K) std::nth_element(cols.begin(), cols.begin() + (kg - 1), cols.end(), by_vs);
            for (int i = 0; i < V; ++i) {
                uint8_t* m = mask_out + (size_t)perm[(size_t)g * V + i] * K;
                for (int t = 0; t < kg; ++t) m[cols[t]] = 1;
            }
        }
        std::copy(perm.begin(), perm.end(), perm_out);
        return SHFLBW_OK;
    } catch (const std::bad_alloc&) {
        return fail(SHFLBW_ERR_NO_MEMORY, "out of host memory in pattern search");
    }
}
