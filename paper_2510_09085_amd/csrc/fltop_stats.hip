// "Index of the chosen token" statistic (paper Sec. 4.1): where in the descending order
// of a frame's emissions the tokens of the decoded prefixes sit.  One wavefront per
// output token: it reads that token's frame (V values), counts the emissions that a
// descending sort (equal values in ascending token order) puts ahead of the token, and
// adds the token to the per-position count and log-probability sum.
#include "fltop_internal.h"

namespace fltop {
namespace {

constexpr int kThreads = 256;
constexpr int kWave = 64;
constexpr int kWaves = kThreads / kWave;

__global__ __launch_bounds__(kThreads) void token_ranks_kernel(
    const float* __restrict__ logprobs, int32_t B, int32_t T, int32_t V,
    const int32_t* __restrict__ tokens, const int32_t* __restrict__ token_frames,
    const int32_t* __restrict__ token_counts, int32_t* __restrict__ out_ranks,
    unsigned long long* __restrict__ rank_count, double* __restrict__ rank_lp_sum) {
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = blockIdx.x * kWaves + threadIdx.x / kWave;
    const int n_waves = gridDim.x * kWaves;
    for (int32_t b = blockIdx.y; b < B; b += gridDim.y) {
        int32_t n = token_counts[b];
        n = n < 0 ? 0 : (n > T ? T : n);
        for (int32_t i = wave; i < n; i += n_waves) {
            const int64_t at = (int64_t)b * T + i;
            const int32_t tok = tokens[at];
            const int32_t f = token_frames[at];
            if (tok < 0 || tok >= V || f < 0 || f >= T) {  // not a decoder output: no statistic
                if (out_ranks && lane == 0) out_ranks[at] = -1;
                continue;
            }
            const float* row = logprobs + ((int64_t)b * T + f) * V;
            const float x = row[tok];
            int ahead = 0;
            for (int32_t v = lane; v < V; v += kWave) {
                const float y = row[v];
                ahead += (y > x || (y == x && v < tok)) ? 1 : 0;
            }
#pragma unroll
            for (int o = kWave / 2; o > 0; o >>= 1) ahead += __shfl_xor(ahead, o, kWave);
            if (lane == 0) {
                if (out_ranks) out_ranks[at] = ahead;
                if (rank_count) atomicAdd(&rank_count[ahead], 1ull);
                if (rank_lp_sum) atomicAdd(&rank_lp_sum[ahead], (double)x);
            }
        }
    }
}

}  // namespace

hipError_t launch_token_ranks(const float* logprobs, int32_t B, int32_t T, int32_t V,
                              const int32_t* tokens, const int32_t* token_frames,
                              const int32_t* token_counts, int32_t* out_ranks,
                              uint64_t* rank_count, double* rank_lp_sum, hipStream_t stream) {
    int bx = (T + kWaves - 1) / kWaves;
    if (bx > 16) bx = 16;
    const dim3 grid((unsigned)bx, (unsigned)(B < 65535 ? B : 65535));
    hipLaunchKernelGGL(token_ranks_kernel, grid, dim3(kThreads), 0, stream, logprobs, B, T, V,
                       tokens, token_frames, token_counts, out_ranks,
                       reinterpret_cast<unsigned long long*>(rank_count), rank_lp_sum);
    return hipGetLastError();
}

}  // namespace fltop
