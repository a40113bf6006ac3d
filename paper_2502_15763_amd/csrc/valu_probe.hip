// Calibration probe for the vector-ALU roofline of the local search: the instruction mix of the swap
// tile's inner loop (one v_sub_u32 per candidate, one v_min3_u32 and one v_max3_u32 per two
// candidates) on registers only, no memory traffic, every SIMD filled with resident waves.  The
// benchmark times it with HIP events and reports lane-ops per second beside the nominal peak
// (256 CUs x 64 lanes x clock); it plays no part in any result.
#include "mmbp_dev.hpp"

namespace mmbp {
namespace {

constexpr int kProbeBlock = 256;
constexpr int kProbeRows = 4;          // independent accumulator pairs per lane, as in a 4-segment tile
constexpr int kProbeCols = 8;          // columns per trip

__global__ __launch_bounds__(kProbeBlock) void valu_probe_kernel(uint32_t *out, int trips, uint32_t seed)
{
    const uint32_t gid = blockIdx.x * kProbeBlock + threadIdx.x;
    uint32_t x[kProbeRows], up[kProbeRows], mx[kProbeRows], c[kProbeCols];
#pragma unroll
    for (int r = 0; r < kProbeRows; r++) { x[r] = (gid + 1u) * 2654435761u + seed * (uint32_t)(r + 1); up[r] = 0xFFFFFFFFu; mx[r] = 0u; }
#pragma unroll
    for (int k = 0; k < kProbeCols; k++) c[k] = seed * 40503u + (uint32_t)k * 0x9E3779B9u + gid;
    for (int t = 0; t < trips; t++) {
#pragma unroll
        for (int r = 0; r < kProbeRows; r++) {
#pragma unroll
            for (int k = 0; k < kProbeCols; k += 2) {
                const uint32_t d0 = c[k] - x[r], d1 = c[k + 1] - x[r];
                up[r] = min(min(up[r], d0), d1);
                mx[r] = max(max(mx[r], d0), d1);
            }
        }
#pragma unroll
        for (int k = 0; k < kProbeCols; k++) c[k] += 0x61C88647u;   // new columns every trip (counted below)
    }
    uint32_t acc = 0;
#pragma unroll
    for (int r = 0; r < kProbeRows; r++) acc ^= up[r] ^ mx[r];
    out[gid] = acc;
}

}  // namespace

// lane-ops one thread issues per trip: rows x columns x 2 (sub + half min3 + half max3) + the column updates
int valu_probe_ops_per_trip() { return kProbeRows * kProbeCols * 2 + kProbeCols; }

hipError_t launch_valu_probe(uint32_t *out, int blocks, int trips, hipStream_t st)
{
    valu_probe_kernel<<<dim3(blocks), dim3(kProbeBlock), 0, st>>>(out, trips, 12345u);
    return hipGetLastError();
}

}  // namespace mmbp
