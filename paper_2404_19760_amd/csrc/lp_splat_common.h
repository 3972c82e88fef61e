// Pieces shared by the Splatter's wavefront-per-ray kernels (Section 3.3 "Splatter").
#pragma once
#include "lp_mfma.h"
#include "lp_mfma_bwd_common.h"

namespace lp {

// Weight sums: lane `corner` (< 8 voxel and hash table, < 12 triplane) of each lane group walks the
// group's 16 points and adds the summed weight of every run into theta_w (hash table: a run = the
// points whose corner `corner` falls into the same entry).
template <int KIND, int C>
__device__ __forceinline__ void scatter_weights(const GridDev& g, float* const theta_w[3], int scene,
                                                const float* info, int corner, int grp)
{
    constexpr int NC = KIND == LP_GRID_TRIPLANE ? 12 : 8;
    const bool live = corner < NC;
    const int cid = live ? corner : 0;
    float* dst;
    int widx, bidx;
    if constexpr (KIND == LP_GRID_HASH) {
        // the record holds the entry offset (entry x channels) of every corner beside its weight
        dst = theta_w[0] + (size_t)scene * g.hash_size;
        widx = cid;
        bidx = 8 + cid;
    } else if constexpr (KIND == LP_GRID_VOXEL) {
        // record order of the 8 weights: 4dx + 2dy + dz (32 channels), 4dz + 2dx + dy (16 channels)
        const int dx = C == 16 ? (cid >> 1) & 1 : cid >> 2;
        const int dy = C == 16 ? cid & 1 : (cid >> 1) & 1;
        const int dz = C == 16 ? cid >> 2 : cid & 1;
        dst = theta_w[0] + (size_t)scene * g.N[0] * g.N[1] * g.N[2] + ((size_t)dx * g.N[1] + dy) * g.N[2] + dz;
        widx = cid;
        bidx = 8;
    } else {
        const int p = cid >> 2, a = p, b = (p + 1) % 3, da = (cid >> 1) & 1, db = cid & 1;
        dst = theta_w[p] + (size_t)scene * g.N[a] * g.N[b] + (size_t)da * g.N[b] + db;
        widx = cid;
        bidx = 12 + p;
    }
    float acc = 0.0f;
    unsigned prev = 0;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const float* rec = info + d_row(r, grp) * 16;
        const float w = rec[widx];
        const unsigned base = reinterpret_cast<const unsigned*>(rec)[bidx];
        if (r > 0 && base != prev) {
            if (live) atomicAdd(dst + prev / C, acc);
            acc = 0.0f;
        }
        prev = base;
        acc += w;
    }
    if (live) atomicAdd(dst + prev / C, acc);
}

// multiplier of the scrambled order of the ray groups: a prime that does not divide their number
inline long long splat_group_multiplier(long long n_groups)
{
    for (long long p : {7919LL, 7907LL, 7901LL, 7883LL})
        if (n_groups > p && n_groups % p != 0) return p;
    return 1;
}

}  // namespace lp
