// Frame-level token pruning (paper Sec. 3, Algorithm 1: the top-emission lookup
// and the relative-threshold test).  The test does not depend on the hypotheses
// (Sec. 2, last paragraph but one), so it runs for every valid frame of the
// batch at once, ahead of the beam search, and is bound by the HBM read of the
// emissions.
//
// Output per frame: a header (count, record offset, top emission) and the
// surviving (token, log-prob) records in ascending token order.
//
// Mapping: a frame is owned by LPF lanes of one wavefront (LPF = 1..64, a power
// of two >= V/4), each lane holding 4*ITERS consecutive-in-chunks values in
// registers, so a wavefront handles 64/LPF frames per round with one coalesced
// 16-byte load per lane.  Max, threshold, ballot and prefix sums are wave-local:
// no LDS, no barrier.  The records of one round's frames (a "pack group") are
// written back to back, so the beam kernel reads a contiguous stream.
#include "fltop_internal.h"

namespace fltop {
namespace {

constexpr int kThreads = 256;
constexpr int kWave = 64;
constexpr int kWaves = kThreads / kWave;
constexpr int kRoundsPerWave = 4;  // consecutive pack groups handled by one wavefront

__device__ inline float wave_max_f(float x) {
#pragma unroll
    for (int o = kWave / 2; o > 0; o >>= 1) x = fmaxf(x, __shfl_xor(x, o, kWave));
    return x;
}

__device__ inline int below(uint64_t mask, int lane) {
    return __popcll(mask & ((1ull << lane) - 1ull));
}

// max over the LPF lanes of a frame's lane group (groups are LPF-aligned)
template <int LPF>
__device__ inline float group_max(float x) {
#pragma unroll
    for (int o = LPF / 2; o > 0; o >>= 1) x = fmaxf(x, __shfl_xor(x, o, kWave));
    return x;
}

template <int LPF, int ITERS, bool VEC4>
__global__ __launch_bounds__(kThreads) void prune_kernel(
    const float* __restrict__ logprobs, const int32_t* __restrict__ lengths, int32_t B, int32_t T,
    int32_t V, float ln_r, FrameHdr* __restrict__ hdr, Survivor* __restrict__ rec) {
    constexpr int FPR = kWave / LPF;  // frames per wave round = pack group size
    static_assert(LPF == kWave || ITERS == 1, "several chunks per lane only for whole-wave frames");
    const int lane = threadIdx.x & (kWave - 1);
    const int lg = lane & (LPF - 1);  // lane within the frame's group
    const int gw = lane / LPF;        // group within the wave
    const int64_t total_frames = (int64_t)B * T;
    const int64_t wave_id = (int64_t)blockIdx.x * kWaves + threadIdx.x / kWave;
    const uint64_t group_mask =
        (LPF == kWave) ? ~0ull : (((1ull << LPF) - 1ull) << (gw * LPF));

#pragma unroll 1
    for (int rd = 0; rd < kRoundsPerWave; ++rd) {
        const int64_t pack = wave_id * kRoundsPerWave + rd;  // pack group index
        const int64_t g_first = pack * FPR;
        if (g_first >= total_frames) break;
        const int64_t g = g_first + gw;
        bool valid = g < total_frames;
        if (valid) {
            const int32_t b = (int32_t)(g / T);
            const int32_t t = (int32_t)(g - (int64_t)b * T);
            int32_t len = lengths[b];
            len = len < 0 ? 0 : (len > T ? T : len);
            valid = t < len;
        }
        // ---- load this lane's values ------------------------------------------------
        float x[ITERS][4];
        const float* row = logprobs + g * V;
#pragma unroll
        for (int it = 0; it < ITERS; ++it) {
            const int v0 = 4 * (lg + LPF * it);
            if (VEC4) {
                float4 q = make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
                if (valid && v0 < V) q = *reinterpret_cast<const float4*>(row + v0);
                x[it][0] = q.x;
                x[it][1] = q.y;
                x[it][2] = q.z;
                x[it][3] = q.w;
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    x[it][e] = (valid && v0 + e < V) ? row[v0 + e] : -INFINITY;
            }
        }
        // ---- top emission and threshold ------------------------------------------------
        float m = -INFINITY;
#pragma unroll
        for (int it = 0; it < ITERS; ++it)
#pragma unroll
            for (int e = 0; e < 4; ++e) m = fmaxf(m, x[it][e]);
        m = (LPF == kWave) ? wave_max_f(m) : group_max<LPF>(m);
        const float thr = m + ln_r;  // one fp32 add
        // ---- survivors, packed over the whole round in (frame, token) order -----------
        Survivor* region = rec + g_first * V;
        int running = 0;       // records written by earlier chunks of this round
        int frame_count = 0;   // survivors of this lane's frame
        int frame_offset = 0;  // first record of this lane's frame
#pragma unroll
        for (int it = 0; it < ITERS; ++it) {
            const int v0 = 4 * (lg + LPF * it);
            bool keep[4];
            uint64_t mk[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                keep[e] = valid && (v0 + e < V) && (x[it][e] >= thr);
                mk[e] = __ballot(keep[e]);
            }
            int pos = running;  // records of lower lanes (all four slots) + my lower slots
#pragma unroll
            for (int e = 0; e < 4; ++e) pos += below(mk[e], lane);
            int in_group = 0, before_group = 0, all = 0;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                in_group += __popcll(mk[e] & group_mask);
                before_group += below(mk[e], gw * LPF);
                all += __popcll(mk[e]);
            }
            if (it == 0) frame_offset = running + before_group;
            int mine = 0;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                if (keep[e]) {
                    Survivor s;
                    s.tok = v0 + e;
                    s.lp = x[it][e];
                    region[pos + mine] = s;
                    const int in_frame = pos + mine - frame_offset;  // rank within the frame
                    if (in_frame < kInlineSurvivors) hdr[g].first[in_frame] = s;
                    ++mine;
                }
            }
            frame_count += in_group;
            running += all;
        }
        if (lg == 0 && g < total_frames) {
            int4 h;
            h.x = frame_count;
            h.y = frame_offset;
            h.z = __float_as_int(valid ? m : 0.0f);
            h.w = 0;
            *reinterpret_cast<int4*>(&hdr[g]) = h;  // count, offset, top, pad
        }
    }
}

__global__ __launch_bounds__(kThreads) void unpack_kernel(
    const FrameHdr* __restrict__ hdr, const Survivor* __restrict__ rec, int64_t total_frames,
    int32_t V, int32_t pg, int32_t* __restrict__ counts, int32_t* __restrict__ tokens,
    float* __restrict__ values, float* __restrict__ frame_max) {
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t g = (int64_t)blockIdx.x * kWaves + threadIdx.x / kWave;
    if (g >= total_frames) return;
    struct Head { int32_t count; uint32_t offset; float top; int32_t pad; };
    const Head h = *reinterpret_cast<const Head*>(&hdr[g]);
    if (lane == 0) {
        counts[g] = h.count;
        if (frame_max) frame_max[g] = h.top;
    }
    const Survivor* src = rec + (g / pg) * (int64_t)pg * V + h.offset;
    for (int k = lane; k < h.count; k += kWave) {
        Survivor s = src[k];
        if (k < kInlineSurvivors) {
            const Survivor in = hdr[g].first[k];
            // the two copies must agree bit for bit; a mismatch is made visible
            if (in.tok != s.tok || __float_as_int(in.lp) != __float_as_int(s.lp)) s.tok = -2;
        }
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
    m = wave_max_f(m);
    if ((threadIdx.x & (kWave - 1)) == 0) s_part[threadIdx.x / kWave] = m;
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int i = 1; i < kWaves; ++i) m = fmaxf(m, s_part[i]);
        out[0] = m;
    }
}

template <int LPF, int ITERS>
hipError_t launch_prune_t(const float* logprobs, const int32_t* lengths, int32_t B, int32_t T,
                          int32_t V, float ln_r, const Workspace& ws, hipStream_t stream) {
    constexpr int FPR = kWave / LPF;
    const int64_t frames = (int64_t)B * T;
    const int64_t packs = (frames + FPR - 1) / FPR;
    const int64_t waves = (packs + kRoundsPerWave - 1) / kRoundsPerWave;
    const int64_t blocks = (waves + kWaves - 1) / kWaves;
    const bool vec4 = (V % 4 == 0) && ((reinterpret_cast<uintptr_t>(logprobs) & 15u) == 0);
    if (vec4)
        hipLaunchKernelGGL((prune_kernel<LPF, ITERS, true>), dim3((unsigned)blocks),
                           dim3(kThreads), 0, stream, logprobs, lengths, B, T, V, ln_r, ws.hdr,
                           ws.rec);
    else
        hipLaunchKernelGGL((prune_kernel<LPF, ITERS, false>), dim3((unsigned)blocks),
                           dim3(kThreads), 0, stream, logprobs, lengths, B, T, V, ln_r, ws.hdr,
                           ws.rec);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_prune(const float* logprobs, const int32_t* lengths, int32_t B, int32_t T,
                        int32_t V, float ln_r, const Workspace& ws, hipStream_t stream) {
    const int lpf = lanes_per_frame(V);
    const int chunks = (V + 4 * lpf - 1) / (4 * lpf);  // 16-byte chunks per lane
#define FLTOP_PRUNE_CASE(L, I) \
    return launch_prune_t<L, I>(logprobs, lengths, B, T, V, ln_r, ws, stream)
    switch (lpf) {
        case 1: FLTOP_PRUNE_CASE(1, 1);
        case 2: FLTOP_PRUNE_CASE(2, 1);
        case 4: FLTOP_PRUNE_CASE(4, 1);
        case 8: FLTOP_PRUNE_CASE(8, 1);
        case 16: FLTOP_PRUNE_CASE(16, 1);
        case 32: FLTOP_PRUNE_CASE(32, 1);
        default: break;
    }
    if (chunks <= 1) FLTOP_PRUNE_CASE(64, 1);
    if (chunks <= 2) FLTOP_PRUNE_CASE(64, 2);
    if (chunks <= 4) FLTOP_PRUNE_CASE(64, 4);
    if (chunks <= 8) FLTOP_PRUNE_CASE(64, 8);
    FLTOP_PRUNE_CASE(64, 16);  // V <= 4096
#undef FLTOP_PRUNE_CASE
}

hipError_t launch_unpack(const Workspace& ws, int32_t B, int32_t T, int32_t V, int32_t* counts,
                         int32_t* tokens, float* values, float* frame_max, hipStream_t stream) {
    const int64_t frames = (int64_t)B * T;
    const int64_t blocks = (frames + kWaves - 1) / kWaves;
    hipLaunchKernelGGL(unpack_kernel, dim3((unsigned)blocks), dim3(kThreads), 0, stream, ws.hdr,
                       ws.rec, frames, V, pack_group(V), counts, tokens, values, frame_max);
    return hipGetLastError();
}

hipError_t launch_lm_bound(const float* lm_table, int32_t V, float lm_weight, float bonus,
                           float* out, hipStream_t stream) {
    hipLaunchKernelGGL(lm_bound_kernel, dim3(1), dim3(kThreads), 0, stream, lm_table,
                       (int64_t)V * V, lm_weight, bonus, out);
    return hipGetLastError();
}

}  // namespace fltop
