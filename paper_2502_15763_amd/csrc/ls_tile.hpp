// Swap-tile arithmetic shared by the LDS-resident and the multi-workgroup local-search kernels
// (gfx950, wave64).  See ls_lds.hip for the derivation: inside a tile (rows of client a x columns
// of client b) the candidate with the smallest makespan is the one with the smallest |y - x|,
// y = cu of the column, x = cu of the row - (l_a - l_b), cu = 2*T_i + 2^30.
#pragma once
#include "mmbp_dev.hpp"

namespace mmbp {
namespace {

constexpr uint32_t kBias = 1u << 30;
constexpr uint32_t kNarrowLimit = 1u << 29;   // narrowing needs T0 + 2 * max cost below this
constexpr uint32_t kPad = 0xC0000000u;        // cu of an empty position
constexpr uint32_t kKeyLimit = 1u << 29;      // |y - x| of a real candidate is below this; keys that come
                                              // from empty columns or from the absent side are >= 3 * 2^29
constexpr uint32_t kInf = 0xFFFFFFFFu;
constexpr uint16_t kNoJob = 0xFFFFu;
#ifndef MMBP_RMAX
#define MMBP_RMAX 4
#endif
constexpr int kRMax = MMBP_RMAX;                       // row segments (of 64 positions) per tile

__device__ __forceinline__ uint32_t absdiff_u32(uint32_t a, uint32_t b) { return max(a, b) - min(a, b); }

// Running nearest-above / nearest-below search of one row against four columns.
struct RowAcc {
    uint32_t up;   // min over columns of (y - x) mod 2^32
    uint32_t mx;   // max over columns of (y - x) mod 2^32
};
__device__ __forceinline__ void nearest_x4(RowAcc &a, uint32_t x, const uint4 &c)
{
    const uint32_t d0 = c.x - x, d1 = c.y - x, d2 = c.z - x, d3 = c.w - x;
    a.up = min(min(a.up, d0), d1);
    a.mx = max(max(a.mx, d0), d1);
    a.up = min(min(a.up, d2), d3);
    a.mx = max(max(a.mx, d2), d3);
}
__device__ __forceinline__ uint32_t nearest_key(const RowAcc &a) { return min(a.up, 0u - a.mx); }

__device__ __forceinline__ unsigned long long sat_add62(unsigned long long a, unsigned long long b)
{
    unsigned long long r = a + b;
    return r >= (unsigned long long)kCostSumLimit ? (unsigned long long)kCostSumLimit : r;
}

__device__ __forceinline__ int uni(int x) { return __builtin_amdgcn_readfirstlane(x); }
__device__ __forceinline__ uint32_t uniu(uint32_t x) { return (uint32_t)__builtin_amdgcn_readfirstlane((int)x); }

// three largest loads with their clients (lowest client index first among equal loads)
// (scalar members, not arrays: the selection below must stay in registers)
struct Top3 {
    uint32_t v0, v1, v2;
    int j0, j1, j2;
};

__device__ __forceinline__ Top3 wave_top3(const long long *load, int M, int lane)
{
    // largest load among the clients other than ex0 and ex1; client -1 when there is none
    auto next = [&](int ex0, int ex1, uint32_t &v, int &jout) {
        uint32_t bv = 0, bj = kInf;
        for (int j = lane; j < M; j += kWave) {
            if (j == ex0 || j == ex1) continue;
            uint32_t l = (uint32_t)load[j];
            if (bj == kInf || l > bv) { bv = l; bj = (uint32_t)j; }
        }
        uint32_t mv = wave_max_u32(bv);
        uint32_t mj = wave_min_u32((bv == mv) ? bj : kInf);
        v = (mj == kInf) ? 0u : mv;
        jout = (int)mj;
    };
    Top3 t;
    next(-1, -1, t.v0, t.j0);
    next(t.j0, -1, t.v1, t.j1);
    next(t.j0, t.j1, t.v2, t.j2);
    return t;
}

__device__ __forceinline__ uint32_t others_max(const Top3 &t, int a, int b)
{
    const bool f0 = t.j0 != a && t.j0 != b;
    const bool f1 = t.j1 != a && t.j1 != b;
    return f0 ? t.v0 : (f1 ? t.v1 : t.v2);
}

// makespan of a swap candidate from its key |y - x|: twice the larger changed load is
// l_a + l_b + key; the other loads contribute the largest untouched one
__device__ __forceinline__ uint32_t swap_value(uint32_t key, uint32_t lsum, uint32_t others)
{
    return key < kKeyLimit ? max(others, (lsum + key) >> 1) : kInf;
}

// Tile: R rows per lane (x[r], already shifted by l_a - l_b) against the columns [c0, c1)
// ((c1 - c0) % 8 == 0, > 0).  key[r] = min over the columns of |cu[col] - x[r]|.  Two register
// sets in ping-pong: the LDS loads of one are in flight while the other is evaluated.
template <int R>
__device__ __forceinline__ void tile_columns(const uint32_t *cu, const uint32_t (&x)[R], int c0, int c1,
                                             uint32_t (&key)[R])
{
    RowAcc acc[R];
#pragma unroll
    for (int r = 0; r < R; r++) { acc[r].up = kInf; acc[r].mx = 0u; }
    const uint4 *col = reinterpret_cast<const uint4 *>(cu + c0);
    const int n8 = (c1 - c0) >> 3;
    uint4 a0 = col[0], a1 = col[1], b0, b1;
    int k = 1;
    for (; k + 1 < n8; k += 2) {
        b0 = col[2 * k]; b1 = col[2 * k + 1];
#pragma unroll
        for (int r = 0; r < R; r++) { nearest_x4(acc[r], x[r], a0); nearest_x4(acc[r], x[r], a1); }
        a0 = col[2 * k + 2]; a1 = col[2 * k + 3];
#pragma unroll
        for (int r = 0; r < R; r++) { nearest_x4(acc[r], x[r], b0); nearest_x4(acc[r], x[r], b1); }
    }
    if (k < n8) {
        b0 = col[2 * k]; b1 = col[2 * k + 1];
#pragma unroll
        for (int r = 0; r < R; r++) { nearest_x4(acc[r], x[r], a0); nearest_x4(acc[r], x[r], a1); }
#pragma unroll
        for (int r = 0; r < R; r++) { nearest_x4(acc[r], x[r], b0); nearest_x4(acc[r], x[r], b1); }
    } else {
#pragma unroll
        for (int r = 0; r < R; r++) { nearest_x4(acc[r], x[r], a0); nearest_x4(acc[r], x[r], a1); }
    }
#pragma unroll
    for (int r = 0; r < R; r++) key[r] = nearest_key(acc[r]);
}


}  // namespace
}  // namespace mmbp
