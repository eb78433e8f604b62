// Frame-level token pruning (paper Sec. 3, Algorithm 1: the top-emission lookup
// and the relative-threshold test).  The test does not depend on the hypotheses
// (Sec. 2, last paragraph but one), so it runs for every valid frame of the
// batch at once, ahead of the beam search, and is bound by the HBM read of the
// emissions.
//
// Output per frame: a header (count, record offset, top emission) and the
// surviving (token, log-prob) records in ascending token order.  Records of one
// workgroup's frames are packed back to back so the beam kernel streams them.
#include "fltop_internal.h"

namespace fltop {
namespace {

constexpr int kThreads = 256;
constexpr int kWave = 64;
constexpr int kWaves = kThreads / kWave;

__device__ inline float wave_max(float x) {
#pragma unroll
    for (int o = kWave / 2; o > 0; o >>= 1) x = fmaxf(x, __shfl_xor(x, o, kWave));
    return x;
}

__device__ inline int wave_sum(int x) {
#pragma unroll
    for (int o = kWave / 2; o > 0; o >>= 1) x += __shfl_xor(x, o, kWave);
    return x;
}

__device__ inline int lanes_below(uint64_t mask, int lane) {
    return __popcll(mask & ((1ull << lane) - 1ull));
}

// Any V >= 1: one wavefront per frame, lanes strided over the vocabulary.
__global__ __launch_bounds__(kThreads) void prune_generic_kernel(
    const float* __restrict__ logprobs, const int32_t* __restrict__ lengths, int32_t B, int32_t T,
    int32_t V, float ln_r, int32_t fpb, FrameHdr* __restrict__ hdr, Survivor* __restrict__ rec) {
    __shared__ int s_cnt[256];
    __shared__ int s_off[256];
    __shared__ float s_thr[256];
    __shared__ float s_top[256];
    __shared__ int s_wave_tot[kWaves];

    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = tid / kWave;
    const int64_t total_frames = (int64_t)B * T;
    const int64_t g0 = (int64_t)blockIdx.x * fpb;
    const int nF = (int)min((int64_t)fpb, total_frames - g0);

    // pass 1: top emission, threshold, survivor count
    for (int f = wave; f < nF; f += kWaves) {
        const int64_t g = g0 + f;
        const int32_t b = (int32_t)(g / T);
        const int32_t t = (int32_t)(g - (int64_t)b * T);
        int32_t len = lengths[b];
        len = len < 0 ? 0 : (len > T ? T : len);
        int c = 0;
        float m = 0.0f, thr = 0.0f;
        if (t < len) {
            const float* row = logprobs + g * V;
            m = -INFINITY;
            for (int v = lane; v < V; v += kWave) m = fmaxf(m, row[v]);
            m = wave_max(m);
            thr = m + ln_r;  // one fp32 add
            for (int v = lane; v < V; v += kWave) c += (row[v] >= thr) ? 1 : 0;
            c = wave_sum(c);
        }
        if (lane == 0) {
            s_cnt[f] = c;
            s_thr[f] = thr;
            s_top[f] = m;
        }
    }
    __syncthreads();

    // exclusive scan of the counts over the block's frames
    {
        int v = (tid < nF) ? s_cnt[tid] : 0;
        int incl = v;
#pragma unroll
        for (int o = 1; o < kWave; o <<= 1) {
            int up = __shfl_up(incl, o, kWave);
            if (lane >= o) incl += up;
        }
        if (lane == kWave - 1) s_wave_tot[wave] = incl;
        __syncthreads();
        int base = 0;
        for (int w = 0; w < wave; ++w) base += s_wave_tot[w];
        if (tid < nF) {
            s_off[tid] = base + incl - v;
            FrameHdr h;
            h.count = v;
            h.offset = (uint32_t)(base + incl - v);
            h.top = s_top[tid];
            h.pad = 0;
            hdr[g0 + tid] = h;
        }
    }
    __syncthreads();

    // pass 2: write the survivors in ascending token order
    Survivor* region = rec + g0 * V;
    for (int f = wave; f < nF; f += kWaves) {
        if (s_cnt[f] == 0) continue;
        const int64_t g = g0 + f;
        const float* row = logprobs + g * V;
        const float thr = s_thr[f];
        Survivor* dst = region + s_off[f];
        int running = 0;
        for (int v0 = 0; v0 < V; v0 += kWave) {
            const int v = v0 + lane;
            const float x = (v < V) ? row[v] : 0.0f;
            const bool keep = (v < V) && (x >= thr);
            const uint64_t mask = __ballot(keep);
            if (keep) {
                Survivor s;
                s.tok = v;
                s.lp = x;
                dst[running + lanes_below(mask, lane)] = s;
            }
            running += __popcll(mask);
        }
    }
}

__global__ __launch_bounds__(kThreads) void unpack_kernel(
    const FrameHdr* __restrict__ hdr, const Survivor* __restrict__ rec, int64_t total_frames,
    int32_t V, int32_t fpb, int32_t* __restrict__ counts, int32_t* __restrict__ tokens,
    float* __restrict__ values, float* __restrict__ frame_max) {
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t g = (int64_t)blockIdx.x * kWaves + threadIdx.x / kWave;
    if (g >= total_frames) return;
    const FrameHdr h = hdr[g];
    if (lane == 0) {
        counts[g] = h.count;
        if (frame_max) frame_max[g] = h.top;
    }
    const Survivor* src = rec + (g / fpb) * (int64_t)fpb * V + h.offset;
    for (int k = lane; k < h.count; k += kWave) {
        const Survivor s = src[k];
        tokens[g * V + k] = s.tok;
        values[g * V + k] = s.lp;
    }
}

// max over the table of lm_weight * table + bonus: bounds every LM term from above.
__global__ __launch_bounds__(kThreads) void lm_bound_kernel(const float* __restrict__ table,
                                                            int64_t n, float w, float bonus,
                                                            float* __restrict__ out) {
    __shared__ float s_part[kWaves];
    float m = -INFINITY;
    for (int64_t i = threadIdx.x; i < n; i += kThreads) m = fmaxf(m, fmaf(w, table[i], bonus));
    m = wave_max(m);
    if ((threadIdx.x & (kWave - 1)) == 0) s_part[threadIdx.x / kWave] = m;
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int i = 1; i < kWaves; ++i) m = fmaxf(m, s_part[i]);
        out[0] = m;
    }
}

}  // namespace

hipError_t launch_prune(const float* logprobs, const int32_t* lengths, int32_t B, int32_t T,
                        int32_t V, float ln_r, const Workspace& ws, hipStream_t stream) {
    const int32_t fpb = frames_per_block(V);
    const int64_t frames = (int64_t)B * T;
    const int64_t blocks = (frames + fpb - 1) / fpb;
    hipLaunchKernelGGL(prune_generic_kernel, dim3((unsigned)blocks), dim3(kThreads), 0, stream,
                       logprobs, lengths, B, T, V, ln_r, fpb, ws.hdr, ws.rec);
    return hipGetLastError();
}

hipError_t launch_unpack(const Workspace& ws, int32_t B, int32_t T, int32_t V, int32_t* counts,
                         int32_t* tokens, float* values, float* frame_max, hipStream_t stream) {
    const int64_t frames = (int64_t)B * T;
    const int64_t blocks = (frames + kWaves - 1) / kWaves;
    hipLaunchKernelGGL(unpack_kernel, dim3((unsigned)blocks), dim3(kThreads), 0, stream, ws.hdr,
                       ws.rec, frames, V, frames_per_block(V), counts, tokens, values, frame_max);
    return hipGetLastError();
}

hipError_t launch_lm_bound(const float* lm_table, int32_t V, float lm_weight, float bonus,
                           float* out, hipStream_t stream) {
    hipLaunchKernelGGL(lm_bound_kernel, dim3(1), dim3(kThreads), 0, stream, lm_table,
                       (int64_t)V * V, lm_weight, bonus, out);
    return hipGetLastError();
}

}  // namespace fltop
