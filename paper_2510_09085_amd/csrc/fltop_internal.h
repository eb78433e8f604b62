// Internal definitions shared by the HIP translation units of the FLToP CTC decoder.
#ifndef FLTOP_INTERNAL_H_
#define FLTOP_INTERNAL_H_

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "fltop_ctc.h"

namespace fltop {

// One survivor of a frame: token id and its fp32 log-probability.
struct alignas(8) Survivor {
    int32_t tok;
    float lp;
};

// Survivors kept inside the frame header itself (ranks 0..5 in ascending token
// order).  Further survivors of a frame live in the record array: a frame with K > 6
// survivors owns K - 6 consecutive records from `rec_base` on (rank k >= 6 at
// rec_base + k - 6), handed out by the prune stage from one counter, so the array only has
// to hold what the threshold lets through.
constexpr int kInlineSurvivors = 6;
constexpr uint32_t kNoRecords = 0xFFFFFFFFu;  // rec_base of a frame whose records did not fit
// The record array is handed out from kRecArenas counters, one per equal slice of the array
// (thousands of wavefronts adding to ONE counter cost the prune stage several times its
// run time); a request that does not fit its slice tries the next one.
constexpr int kRecArenas = 64;

// Per-frame header written by the prune stage (one 64-byte line).
constexpr int kLmBoundParts = 64;  // workgroups of the LM bound kernel = lanes that read them

struct alignas(64) FrameHdr {
    int32_t count;       // |S_t| (0 for frames at or beyond the utterance length)
    uint32_t rec_base;   // count > 6: first record of this frame (survivor 6), or kNoRecords
                         // when the record array was full; unused otherwise
    float top;           // max_v lp[t][v]
    uint32_t div_magic;  // floor((2^32 - 1) / n) + 1 for n = non-blank survivors > 1, else 0:
                         // umulhi(e, div_magic) == e / n for every e < 2^19, and at most one
                         // more than that for any larger e below 2^32
    Survivor first[kInlineSurvivors];  // survivors 0..min(count,6)-1, ascending token; unused
                                       // places hold (token -1, log-prob -inf).  The blank
                                       // (token 0), if it survived, is first[0].
};
static_assert(sizeof(FrameHdr) == 64, "FrameHdr must be one 64-byte line");

// One node of the prefix trie (global memory): a prefix is a chain of nodes.
// `xup` is the nearest ancestor whose depth is a multiple of 8 (strictly above
// this node), so the final back-walk takes depth/8 dependent loads and the
// 8-token segments in between are walked in parallel.
struct alignas(16) TrieNode {
    int32_t parent;
    int32_t xup;
    int32_t tok;
    int32_t depth;
};

// Lanes of a wavefront that own one frame in the prune stage: the smallest power
// of two >= ceil(V/4), at most 64.
__host__ __device__ inline int32_t lanes_per_frame(int32_t V) {
    const int32_t q = (V + 3) / 4;
    int32_t l = 1;
    while (l < q && l < 64) l <<= 1;
    return l;
}

// Beams beyond 512 entries keep four fields of every beam entry (parent hash, trie node,
// length, skip ancestor: 20 bytes) in global memory, two generations per utterance.
constexpr int32_t kBeamInLds = 512;
constexpr size_t kColdBytesPerGeneration = (size_t)FLTOP_MAX_BEAM * 20;

struct Workspace {
    FrameHdr* hdr;      // [B*T]
    TrieNode* trie;     // [B][trie_stride]
    float* lm_bound;    // [kLmBoundParts] partial maxima of lm_weight*table+bonus
    unsigned long long* rec_used;  // [kRecArenas] records handed out per slice of the record array
                                   // (cleared before the prune stage runs)
    void* cold;         // [B][2][kColdBytesPerGeneration] when beam > kBeamInLds, else unused
    Survivor* rec;      // [rec_capacity]: survivors of rank >= 6, last region of the workspace
    uint32_t rec_capacity;  // a multiple of kRecArenas: every slice holds rec_capacity / kRecArenas
    int64_t trie_stride;
    size_t fixed_bytes;  // everything but the records
    size_t bytes;        // fixed_bytes + 8 * rec_capacity
};

// Records a batch can need at most: every frame keeps every token.
inline uint64_t worst_case_records(int32_t B, int32_t T, int32_t V) {
    return V > kInlineSurvivors ? (uint64_t)B * (uint64_t)T * (uint64_t)(V - kInlineSurvivors) : 0;
}

// Places added to a record budget so that it is usable in full: the frames of one wavefront
// round ask for their records together, and each slice of the array may end on a stretch that
// is shorter than such a request.
inline uint64_t record_slack(int32_t V) {
    if (V <= kInlineSurvivors) return 0;
    const uint64_t frames_per_round = 64 / (uint64_t)lanes_per_frame(V);
    return (uint64_t)kRecArenas * frames_per_round * (uint64_t)(V - kInlineSurvivors);
}
constexpr uint64_t kMaxRecords = 0xFFFFFFF0ull;  // record indices are 32 bits

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Lays the regions out in `base`; the record array takes `max_records` places (the caller
// derives that from the bytes it was given, see records_that_fit).
inline Workspace carve_workspace(void* base, int32_t B, int32_t T, int32_t V, int32_t beam,
                                 uint64_t max_records) {
    Workspace w;
    (void)V;
    const size_t frames = (size_t)B * (size_t)T;
    const size_t off_hdr = 0;
    const size_t off_trie = align_up(off_hdr + frames * sizeof(FrameHdr), 256);
    w.trie_stride = (int64_t)T * beam + 1;
    const size_t off_lmb =
        align_up(off_trie + (size_t)B * (size_t)w.trie_stride * sizeof(TrieNode), 256);
    const size_t off_used = off_lmb + 256;
    const size_t off_cold = off_used + align_up(kRecArenas * sizeof(unsigned long long), 256);
    const size_t off_rec =
        off_cold + (beam > kBeamInLds ? align_up((size_t)B * 2 * kColdBytesPerGeneration, 256) : 0);
    if (max_records > kMaxRecords) max_records = kMaxRecords;
    max_records -= max_records % kRecArenas;
    w.rec_capacity = (uint32_t)max_records;
    w.fixed_bytes = off_rec;
    w.bytes = align_up(off_rec + (size_t)max_records * sizeof(Survivor), 256);
    char* p = static_cast<char*>(base);
    w.hdr = p ? reinterpret_cast<FrameHdr*>(p + off_hdr) : nullptr;
    w.trie = p ? reinterpret_cast<TrieNode*>(p + off_trie) : nullptr;
    w.lm_bound = p ? reinterpret_cast<float*>(p + off_lmb) : nullptr;
    w.rec_used = p ? reinterpret_cast<unsigned long long*>(p + off_used) : nullptr;
    w.cold = p ? p + off_cold : nullptr;
    w.rec = p ? reinterpret_cast<Survivor*>(p + off_rec) : nullptr;
    return w;
}

// How many records a workspace of `bytes` holds behind the fixed regions (never more than the
// batch can need), or -1 if not even the fixed regions fit.
inline int64_t records_that_fit(size_t bytes, int32_t B, int32_t T, int32_t V, int32_t beam) {
    const size_t fixed = carve_workspace(nullptr, B, T, V, beam, 0).fixed_bytes;
    if (bytes < fixed) return -1;
    uint64_t n = (bytes - fixed) / sizeof(Survivor);
    const uint64_t most = worst_case_records(B, T, V) + record_slack(V);
    if (n > most) n = most;
    if (n > kMaxRecords) n = kMaxRecords;
    return (int64_t)n;
}

// Device memory of a streaming decode: one fixed-size record per utterance (the carried
// beam), then the prefix trie for up to t_total frames.
struct StreamSpace {
    void* records;
    TrieNode* trie;
    int64_t trie_stride;  // nodes per utterance: t_total * beam + 1
    int32_t* out_nodes;   // [B, t_total]: trie node behind each token of the transcript as it was
                          // last written (-1 beyond its length)
    int32_t t_total;
    size_t bytes;
};

size_t stream_record_bytes(int32_t beam);

inline StreamSpace carve_stream(void* base, int32_t B, int32_t t_total, int32_t beam) {
    StreamSpace s;
    s.t_total = t_total;
    s.trie_stride = (int64_t)t_total * beam + 1;
    const size_t off_trie = align_up((size_t)B * stream_record_bytes(beam), 256);
    const size_t off_nodes =
        align_up(off_trie + (size_t)B * (size_t)s.trie_stride * sizeof(TrieNode), 256);
    s.bytes = align_up(off_nodes + (size_t)B * (size_t)t_total * sizeof(int32_t), 256);
    char* p = static_cast<char*>(base);
    s.records = p;
    s.trie = p ? reinterpret_cast<TrieNode*>(p + off_trie) : nullptr;
    s.out_nodes = p ? reinterpret_cast<int32_t*>(p + off_nodes) : nullptr;
    return s;
}

hipError_t launch_stream_begin(const StreamSpace& sp, int32_t B, int32_t beam, hipStream_t stream);
hipError_t launch_log_add(const double* a, const double* b, double* out, int64_t n,
                          hipStream_t stream);

// Launchers (defined next to their kernels); each returns a hipError_t.
// (clears the record counter, then runs the prune kernel)
hipError_t launch_prune(const float* logprobs, const int32_t* lengths, int32_t B, int32_t T,
                        int32_t V, float ln_r, int32_t top_n, const Workspace& ws,
                        hipStream_t stream);
hipError_t launch_token_ranks(const float* logprobs, int32_t B, int32_t T, int32_t V,
                              const int32_t* tokens, const int32_t* token_frames,
                              const int32_t* token_counts, int32_t* out_ranks,
                              uint64_t* rank_count, double* rank_lp_sum, hipStream_t stream);
hipError_t launch_unpack(const Workspace& ws, const int32_t* lengths, int32_t B, int32_t T,
                         int32_t V, int32_t* counts, int32_t* tokens, float* values,
                         float* frame_max, hipStream_t stream);
hipError_t launch_lm_bound(const float* lm_table, int32_t V, float lm_weight, float bonus,
                           float* out, hipStream_t stream);
hipError_t launch_beam(const int32_t* lengths, int32_t B, int32_t T, int32_t V,
                       const fltop_params& p, const Workspace& ws, const StreamSpace* carried,
                       int32_t* out_tokens, int32_t* out_lengths, float* out_scores,
                       fltop_stats* stats, hipStream_t stream);

}  // namespace fltop
#endif  // FLTOP_INTERNAL_H_
