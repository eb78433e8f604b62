// Frame-level token pruning (paper Sec. 3, Algorithm 1: the top-emission lookup
// and the relative-threshold test).  The test does not depend on the hypotheses
// (Sec. 2, last paragraph but one), so it runs for every valid frame of the
// batch at once, ahead of the beam search, and is bound by the HBM read of the
// emissions.
//
// The optional static stage of Algorithm 1 (only the N best tokens of a frame take the
// threshold test at all) is applied to the threshold's survivors: both tests keep an
// upper part of the frame's descending order, so "N best, then threshold" equals
// "threshold, then the N best of what is left".  The N-th best survivor is found with a
// bitwise search over an order-preserving integer image of the fp32 values (32 counting
// steps inside the frame's lane group); equal values are taken in ascending token order.
//
// Output per frame: a 64-byte header (count, top emission, survivors 0..5 in
// ascending token order) and, for frames with more than six survivors, survivors
// 6.. as (token, log-prob) records in a stretch of the record array that the frame
// takes from one counter (one atomic per wavefront round that needs any), so the array
// holds what the threshold lets through and no more; a frame that finds it full is
// marked, and the search stage reports the utterance instead of decoding it.
//
// Mapping: a frame is owned by LPF lanes of one wavefront (LPF = 1..64, a power
// of two >= V/4), each lane holding 4*ITERS values in registers, so a wavefront
// handles 64/LPF frames per round with one coalesced 16-byte load per lane and
// chunk.  Max, threshold and the prefix sums that place the survivors are
// wave-local DPP operations; LDS is used only as a wave-private staging area for
// the headers (no barrier).  Wavefronts walk the frames of an utterance with a
// grid stride and load the next rounds before working on the current ones.
#include "fltop_internal.h"

namespace fltop {
namespace {

constexpr int kThreads = 256;
constexpr int kWave = 64;
constexpr int kWaves = kThreads / kWave;

// Value of `v` in the lane selected by a DPP control word; `old` where that lane
// does not exist or the row is masked off.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ int dpp_int(int old, int v) {
    return __builtin_amdgcn_update_dpp(old, v, CTRL, ROW_MASK, 0xf, false);
}
template <int CTRL>
__device__ __forceinline__ float dpp_float(float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(v), __float_as_int(v), CTRL,
                                                      0xf, 0xf, false));
}

// Max over the LPF lanes of a frame's lane group (groups are LPF-aligned); every lane of
// the group ends up with the result.  Steps 1, 2 use quad permutes, 4 the half-row
// mirror, 8 the row mirror (a mirror pairs each lane with one of the other half, which
// is all a max needs); 16 and 32 go through the cross-lane network.
template <int LPF>
__device__ __forceinline__ float group_max(float x) {
    if (LPF >= 2) x = fmaxf(x, dpp_float<0xB1>(x));   // quad_perm [1,0,3,2]
    if (LPF >= 4) x = fmaxf(x, dpp_float<0x4E>(x));   // quad_perm [2,3,0,1]
    if (LPF >= 8) x = fmaxf(x, dpp_float<0x141>(x));  // row_half_mirror
    if (LPF >= 16) x = fmaxf(x, dpp_float<0x140>(x)); // row_mirror
    if (LPF >= 32) x = fmaxf(x, __shfl_xor(x, 16, kWave));
    if (LPF >= 64) x = fmaxf(x, __shfl_xor(x, 32, kWave));
    return x;
}

// Inclusive prefix sum of `c` over the lanes of each LPF-lane group.  Every DPP read is
// executed by all lanes (never inside a lane-dependent branch: a lane that is switched
// off cannot be read), and masked afterwards.
template <int LPF>
__device__ __forceinline__ int group_inclusive_scan(int c, int lg) {
    int v = c;
    if (LPF >= 2) {
        const int up = dpp_int<0x111, 0xf>(0, v);  // row_shr:1
        v += (lg >= 1) ? up : 0;
    }
    if (LPF >= 4) {
        const int up = dpp_int<0x112, 0xf>(0, v);  // row_shr:2
        v += (lg >= 2) ? up : 0;
    }
    if (LPF >= 8) {
        const int up = dpp_int<0x114, 0xf>(0, v);  // row_shr:4
        v += (lg >= 4) ? up : 0;
    }
    if (LPF >= 16) {
        const int up = dpp_int<0x118, 0xf>(0, v);  // row_shr:8
        v += (lg >= 8) ? up : 0;
    }
    if (LPF >= 32) v += dpp_int<0x142, 0xa>(0, v);  // lane 15 of rows 0,2 into rows 1,3
    if (LPF >= 64) v += dpp_int<0x143, 0xc>(0, v);  // lane 31 into rows 2,3
    return v;
}

// Sum over the LPF lanes of a frame's lane group, result in every lane (same exchange
// pattern as group_max).
template <int LPF>
__device__ __forceinline__ int group_sum(int x) {
    if (LPF >= 2) x += dpp_int<0xB1, 0xf>(0, x);
    if (LPF >= 4) x += dpp_int<0x4E, 0xf>(0, x);
    if (LPF >= 8) x += dpp_int<0x141, 0xf>(0, x);
    if (LPF >= 16) x += dpp_int<0x140, 0xf>(0, x);
    if (LPF >= 32) x += __shfl_xor(x, 16, kWave);
    if (LPF >= 64) x += __shfl_xor(x, 32, kWave);
    return x;
}

// Order-preserving image of an fp32 value (larger value, larger integer); -0.0 counts
// as +0.0, as it does for a floating-point comparison.
__device__ __forceinline__ uint32_t order_bits(float x) {
    const uint32_t b = (uint32_t)__float_as_int(x + 0.0f);
    return (b >> 31) ? ~b : (b | 0x80000000u);
}

template <int LPF, int ITERS, bool VEC4>
struct FrameRegs {
    float x[ITERS][4];
    bool valid;
};

// Load the values of frame `t` of one utterance (row = first emission of that frame).
template <int LPF, int ITERS, bool VEC4>
__device__ __forceinline__ void load_frame(FrameRegs<LPF, ITERS, VEC4>& r,
                                           const float* __restrict__ row, bool valid, int32_t V,
                                           int lg) {
    r.valid = valid;
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
        const int v0 = 4 * (lg + LPF * it);
        if (VEC4) {
            float4 q = make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
            if (valid && v0 < V) q = *reinterpret_cast<const float4*>(row + v0);
            r.x[it][0] = q.x;
            r.x[it][1] = q.y;
            r.x[it][2] = q.z;
            r.x[it][3] = q.w;
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
                r.x[it][e] = (valid && v0 + e < V) ? row[v0 + e] : -INFINITY;
        }
    }
}

// DENSE: the record array holds the worst case (every token of every frame), so frame g simply
// owns the stretch [g * (V - 6), (g + 1) * (V - 6)) and nothing has to be counted; otherwise the
// array is smaller and stretches are handed out as frames ask for them.
template <int LPF, int ITERS, bool VEC4, bool DENSE>
__global__ __launch_bounds__(kThreads) void prune_kernel(
    const float* __restrict__ logprobs, const int32_t* __restrict__ lengths, int32_t B, int32_t T,
    int32_t V, float ln_r, int32_t top_n, FrameHdr* __restrict__ hdr,
    Survivor* __restrict__ rec, unsigned long long* __restrict__ rec_used,
    uint32_t rec_capacity) {
    constexpr int FPR = kWave / LPF;  // frames per wave round
    static_assert(LPF == kWave || ITERS == 1, "several chunks per lane only for whole-wave frames");
    static_assert(ITERS <= 8 || ITERS == 16, "flag word holds 4*ITERS <= 64 bits");
    __shared__ FrameHdr stage[kWaves][FPR];  // header images of one round, per wavefront
    const int lane = threadIdx.x & (kWave - 1);
    const int lg = lane & (LPF - 1);  // lane within the frame's group
    const int gw = lane / LPF;        // group within the wave
    // blockIdx.y walks the utterances: no division, and rounds beyond a length are not run
    for (int32_t b = blockIdx.y; b < B; b += gridDim.y) {
    int32_t len = lengths[b];
    len = len < 0 ? 0 : (len > T ? T : len);
    const int n_rounds = (len + FPR - 1) / FPR;
    const int wave_id = blockIdx.x * kWaves + threadIdx.x / kWave;
    const int n_waves = gridDim.x * kWaves;
    const int64_t g_base = (int64_t)b * T;
    const float* utt = logprobs + g_base * V;

    // U rounds are loaded together (more bytes in flight per wavefront), one batch ahead; two
    // measured best for one-chunk frames (4 and 8 lengthen the wavefront that finishes last)
    constexpr int U = ITERS >= 4 ? 1 : 2;
    FrameRegs<LPF, ITERS, VEC4> cur[U], nxt[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int t = (wave_id * U + u) * FPR + gw;
        load_frame(cur[u], utt + (int64_t)t * V, t < len, V, lg);
    }

    for (int base = wave_id * U; base < n_rounds; base += n_waves * U) {
        // next batch's loads go out before this batch's work
        const int base_next = base + n_waves * U;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int t = (base_next + u) * FPR + gw;
            load_frame(nxt[u], utt + (int64_t)t * V, t < len, V, lg);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
        const int rd = base + u;
        if (rd >= n_rounds) break;
        const FrameRegs<LPF, ITERS, VEC4>& fr = cur[u];
        // ---- top emission and threshold ------------------------------------------------
        float m = -INFINITY;
#pragma unroll
        for (int it = 0; it < ITERS; ++it)
#pragma unroll
            for (int e = 0; e < 4; ++e) m = fmaxf(m, fr.x[it][e]);
        m = group_max<LPF>(m);
        const float thr = m + ln_r;  // one fp32 add

        // ---- survivors in ascending token order: rank = survivors before it in the frame.
        // Ranks 0..5 go into the header, ranks >= 6 into the frame's record list (slot =
        // rank), so every store is decided by the lane's own rank.  The headers of the
        // round's frames are assembled in LDS (wave-local, no barrier) and leave as
        // whole 64-byte lines, 16 bytes per lane: a partly written line would cost the
        // memory system a read-modify-write.
        FrameHdr* img = &stage[threadIdx.x / kWave][gw];
        unsigned keep[ITERS];  // bit e of keep[it]: value x[it][e] survives
        int kept_here = 0;
#pragma unroll
        for (int it = 0; it < ITERS; ++it) {
            const int v0 = 4 * (lg + LPF * it);
            keep[it] = 0;
#pragma unroll
            for (int e = 0; e < 4; ++e)
                keep[it] |= (fr.valid && (v0 + e < V) && (fr.x[it][e] >= thr)) ? (1u << e) : 0u;
            kept_here += __popc(keep[it]);
        }
        // ---- static stage: at most top_n survivors, the best by (value desc, token asc) ----
        if (top_n > 0) {  // uniform
            const int kept_frame = group_sum<LPF>(kept_here);
            if (__any(kept_frame > top_n)) {  // wave-uniform: every lane joins the exchanges
                // largest `cut` with at least top_n kept values >= cut: the top_n-th best value
                uint32_t cut = 0;
                for (int bit = 31; bit >= 0; --bit) {
                    const uint32_t trial = cut | (1u << bit);
                    int c = 0;
#pragma unroll
                    for (int it = 0; it < ITERS; ++it)
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            c += (((keep[it] >> e) & 1u) && order_bits(fr.x[it][e]) >= trial) ? 1 : 0;
                    if (group_sum<LPF>(c) >= top_n) cut = trial;
                }
                // everything above the cut stays; of the values equal to it, the first few
                // in token order fill the remaining places
                int above = 0;
#pragma unroll
                for (int it = 0; it < ITERS; ++it)
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        above += (((keep[it] >> e) & 1u) && order_bits(fr.x[it][e]) > cut) ? 1 : 0;
                const int places = top_n - group_sum<LPF>(above);
                int equal_before = 0;  // values equal to the cut at lower token ids
#pragma unroll
                for (int it = 0; it < ITERS; ++it) {
                    unsigned eq = 0;
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        eq |= (((keep[it] >> e) & 1u) && order_bits(fr.x[it][e]) == cut) ? (1u << e)
                                                                                         : 0u;
                    const int n_eq = __popc(eq);
                    const int incl = group_inclusive_scan<LPF>(n_eq, lg);
                    int r = equal_before + incl - n_eq;
                    unsigned stay = 0;  // above the cut, or equal to it and early enough
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        if ((eq >> e) & 1u) {
                            if (r < places) stay |= 1u << e;
                            ++r;
                        } else if (order_bits(fr.x[it][e]) > cut) {
                            stay |= 1u << e;
                        }
                    }
                    if (kept_frame > top_n) keep[it] &= stay;
                    if (LPF == kWave)
                        equal_before += __builtin_amdgcn_readlane(incl, kWave - 1);
                    // LPF < 64 has ITERS == 1: no further chunk
                }
            }
        }
        // ---- a place in the record array for the survivors beyond the header's six ---------
        uint32_t rec_base = kNoRecords;
        if (DENSE) {
            rec_base = (uint32_t)((g_base + rd * FPR + gw) * (int64_t)max(0, V - kInlineSurvivors));
        } else {
        int kept_now = 0;
#pragma unroll
        for (int it = 0; it < ITERS; ++it) kept_now += __popc(keep[it]);
        const int need = max(0, group_sum<LPF>(kept_now) - kInlineSurvivors);  // same in the group
        if (__any(need > 0)) {  // wave-uniform: one request for the round's frames together
            const int incl = group_inclusive_scan<kWave>(lg == 0 ? need : 0, lane);
            const int wave_total = __builtin_amdgcn_readlane(incl, kWave - 1);
            // the array is handed out in kRecArenas slices with a counter each; a request that
            // does not fit the wavefront's own slice goes on to the next ones
            const uint32_t per_arena = rec_capacity / kRecArenas;
            for (int attempt = 0; attempt < kRecArenas; ++attempt) {
                const int arena = (wave_id + (int)b + attempt) & (kRecArenas - 1);
                unsigned long long base = 0;
                if (lane == 0)
                    base = atomicAdd(rec_used + arena, (unsigned long long)wave_total);
                base = ((unsigned long long)(uint32_t)__builtin_amdgcn_readfirstlane(
                            (int)(base >> 32)) << 32) |
                       (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)base);
                if (base + (unsigned long long)wave_total <= (unsigned long long)per_arena) {
                    // every lane of a group sees the needs of the groups up to its own
                    if (need > 0)
                        rec_base = (uint32_t)arena * per_arena + (uint32_t)base +
                                   (uint32_t)(incl - need);
                    break;
                }
            }
        }
        }  // !DENSE
        Survivor* list = rec + ((int64_t)rec_base - kInlineSurvivors);  // used only if it fits
        const bool fits = rec_base != kNoRecords;
        // whether the blank (token 0, held by the group's first lane) survived: the search
        // stage wants the number of other survivors ready-made
        const int has_blank = group_sum<LPF>(lg == 0 ? (int)(keep[0] & 1u) : 0);
        // unused places of the header's inline list read as (token -1, log-prob -inf)
        for (int p = lg; p < 3; p += LPF)
            reinterpret_cast<int4*>(img)[1 + p] =
                make_int4(-1, __float_as_int(-INFINITY), -1, __float_as_int(-INFINITY));
        int total = 0;
#pragma unroll
        for (int it = 0; it < ITERS; ++it) {
            const int v0 = 4 * (lg + LPF * it);
            unsigned bits = keep[it];
            const int cnt = __popc(bits);
            const int incl = group_inclusive_scan<LPF>(cnt, lg);
            int rank = total + incl - cnt;
            while (bits != 0) {  // usually zero or one survivor per lane
                const int e = __ffs(bits) - 1;
                bits &= bits - 1;
                Survivor s;
                s.tok = v0 + e;
                s.lp = e == 0 ? fr.x[it][0] : e == 1 ? fr.x[it][1] : e == 2 ? fr.x[it][2] : fr.x[it][3];
                if (rank < kInlineSurvivors)
                    img->first[rank] = s;
                else if (fits)
                    list[rank] = s;
                ++rank;
            }
            if (LPF == kWave) {
                total += __builtin_amdgcn_readlane(incl, kWave - 1);
            } else {
                total = incl;  // exact in the group's last lane, which writes the header
            }
        }
        if (lg == LPF - 1) {
            const uint32_t others = (uint32_t)(total - has_blank);
            int4 h;
            h.x = total;
            h.y = (int)rec_base;
            h.z = __float_as_int(m);
            h.w = others > 1u ? (int)(0xFFFFFFFFu / others + 1u) : 0;
            *reinterpret_cast<int4*>(img) = h;  // count, rec_base, top, div_magic
        }
        // LDS operations of one wavefront execute in order, so the images are complete
        // for the reads below.  Frames beyond the length get no header: never read, and
        // the slots past T belong to the next utterance.
        {
            const int4* src = reinterpret_cast<const int4*>(&stage[threadIdx.x / kWave][0]);
            int4* dst = reinterpret_cast<int4*>(hdr + g_base + (int64_t)rd * FPR);
#pragma unroll
            for (int p0 = 0; p0 < 4 * FPR; p0 += kWave) {
                const int p = p0 + lane;
                if (p < 4 * FPR && rd * FPR + (p >> 2) < len) dst[p] = src[p];
            }
        }
        }  // rounds of the batch
#pragma unroll
        for (int u = 0; u < U; ++u) cur[u] = nxt[u];
    }
    }  // utterances
}

__global__ __launch_bounds__(kThreads) void unpack_kernel(
    const FrameHdr* __restrict__ hdr, const Survivor* __restrict__ rec,
    const int32_t* __restrict__ lengths, int64_t total_frames, int32_t T, int32_t V,
    int32_t* __restrict__ counts, int32_t* __restrict__ tokens, float* __restrict__ values,
    float* __restrict__ frame_max) {
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t g = (int64_t)blockIdx.x * kWaves + threadIdx.x / kWave;
    if (g >= total_frames) return;
    const int32_t b = (int32_t)(g / T);
    const int32_t t = (int32_t)(g - (int64_t)b * T);
    int32_t len = lengths[b];
    len = len < 0 ? 0 : (len > T ? T : len);
    if (t >= len) {  // no header was written for this frame
        if (lane == 0) {
            counts[g] = 0;
            if (frame_max) frame_max[g] = 0.0f;
        }
        return;
    }
    struct Head {
        int32_t count;
        uint32_t rec_base;
        float top;
        int32_t pad;
    };
    const Head h = *reinterpret_cast<const Head*>(&hdr[g]);
    if (lane == 0) {
        counts[g] = h.count;
        if (frame_max) frame_max[g] = h.top;
    }
    // survivors beyond the sixth sit in the frame's stretch of the record array (if they fitted)
    const Survivor* src = rec + ((int64_t)h.rec_base - kInlineSurvivors);
    const int have = h.rec_base == kNoRecords ? min(h.count, kInlineSurvivors) : h.count;
    for (int k = lane; k < have; k += kWave) {
        const Survivor s = (k < kInlineSurvivors) ? hdr[g].first[k] : src[k];
        tokens[g * V + k] = s.tok;
        values[g * V + k] = s.lp;
    }
}

// max over the table of lm_weight * table + bonus: bounds every LM term from above.  One
// partial maximum per workgroup (kLmBoundParts of them; the search stage takes the max of
// those), so that a 4 MB table is read by 64 workgroups and not by one.
__global__ __launch_bounds__(kThreads) void lm_bound_kernel(const float* __restrict__ table,
                                                            int64_t n, float w, float bonus,
                                                            float* __restrict__ out) {
    __shared__ float s_part[kWaves];
    float m = -INFINITY;
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < n;
         i += (int64_t)gridDim.x * kThreads)
        m = fmaxf(m, fmaf(w, table[i], bonus));
    m = group_max<kWave>(m);
    if ((threadIdx.x & (kWave - 1)) == 0) s_part[threadIdx.x / kWave] = m;
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int i = 1; i < kWaves; ++i) m = fmaxf(m, s_part[i]);
        out[blockIdx.x] = m;
    }
}

__global__ void clear_record_counters_kernel(unsigned long long* rec_used) {
    rec_used[threadIdx.x] = 0ull;
}

template <int LPF, int ITERS>
hipError_t launch_prune_t(const float* logprobs, const int32_t* lengths, int32_t B, int32_t T,
                          int32_t V, float ln_r, int32_t top_n, const Workspace& ws,
                          hipStream_t stream) {
    constexpr int FPR = kWave / LPF;
    constexpr int U = ITERS >= 4 ? 1 : 2;
    // grid = (blocks per utterance, B), never more wavefronts per utterance than it has batches
    // of rounds.  Large frames (4 or more chunks per lane): about 2048 workgroups in all (8 per
    // CU).  Small frames: about 8192 -- a launch over a few tens of MB is bound by the latency of
    // its first loads, not by bandwidth, and short utterances leave many wavefronts without
    // work, so more and lighter wavefronts finish sooner (measured on 256 utterances of 250 to
    // 1500 frames, V = 32: 13.0 us against 19.6 us).
    const int rounds = (T + FPR - 1) / FPR;
    int bx = (rounds + kWaves * U - 1) / (kWaves * U);
    const int cap = ((ITERS >= 4 ? 2048 : 8192) + B - 1) / B;
    if (bx > cap) bx = cap;
    if (bx < 1) bx = 1;
    const dim3 grid((unsigned)bx, (unsigned)(B < 65535 ? B : 65535));
    const bool vec4 = (V % 4 == 0) && ((reinterpret_cast<uintptr_t>(logprobs) & 15u) == 0);
    unsigned long long* const used = ws.rec_used;
    // With room for the worst case every frame has its fixed stretch of the record array: no
    // counters, no atomics.  A smaller array is handed out on demand (costs the prune stage a
    // few microseconds: a global atomic with a result sits on every wavefront's path).
    const bool dense = worst_case_records(B, T, V) <= (uint64_t)ws.rec_capacity;
#define FLTOP_LAUNCH_PRUNE(VEC4_, DENSE_)                                                        \
    hipLaunchKernelGGL((prune_kernel<LPF, ITERS, VEC4_, DENSE_>), grid, dim3(kThreads), 0, stream, \
                       logprobs, lengths, B, T, V, ln_r, top_n, ws.hdr, ws.rec, used,            \
                       ws.rec_capacity)
    if (dense) {
        if (vec4) FLTOP_LAUNCH_PRUNE(true, true);
        else FLTOP_LAUNCH_PRUNE(false, true);
    } else {
        // a kernel, not a memset: a call may be captured into a HIP graph
        hipLaunchKernelGGL(clear_record_counters_kernel, dim3(1), dim3(kRecArenas), 0, stream, used);
        if (vec4) FLTOP_LAUNCH_PRUNE(true, false);
        else FLTOP_LAUNCH_PRUNE(false, false);
    }
#undef FLTOP_LAUNCH_PRUNE
    return hipGetLastError();
}

}  // namespace

hipError_t launch_prune(const float* logprobs, const int32_t* lengths, int32_t B, int32_t T,
                        int32_t V, float ln_r, int32_t top_n, const Workspace& ws,
                        hipStream_t stream) {
    if (top_n >= V) top_n = 0;  // the static stage keeps everything
    const int lpf = lanes_per_frame(V);
    const int chunks = (V + 4 * lpf - 1) / (4 * lpf);  // 16-byte chunks per lane
#define FLTOP_PRUNE_CASE(L, I) \
    return launch_prune_t<L, I>(logprobs, lengths, B, T, V, ln_r, top_n, ws, stream)
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

hipError_t launch_unpack(const Workspace& ws, const int32_t* lengths, int32_t B, int32_t T,
                         int32_t V, int32_t* counts, int32_t* tokens, float* values,
                         float* frame_max, hipStream_t stream) {
    const int64_t frames = (int64_t)B * T;
    const int64_t blocks = (frames + kWaves - 1) / kWaves;
    hipLaunchKernelGGL(unpack_kernel, dim3((unsigned)blocks), dim3(kThreads), 0, stream, ws.hdr,
                       ws.rec, lengths, frames, T, V, counts, tokens, values, frame_max);
    return hipGetLastError();
}

hipError_t launch_lm_bound(const float* lm_table, int32_t V, float lm_weight, float bonus,
                           float* out, hipStream_t stream) {
    hipLaunchKernelGGL(lm_bound_kernel, dim3(kLmBoundParts), dim3(kThreads), 0, stream, lm_table,
                       (int64_t)V * V, lm_weight, bonus, out);
    return hipGetLastError();
}

}  // namespace fltop
