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
// order).  Further survivors of a frame live in the record array at a fixed
// place: frame g owns records [g*V, g*V + V), survivor of rank k >= 6 in slot k.
constexpr int kInlineSurvivors = 6;

// Per-frame header written by the prune stage (one 64-byte line).
constexpr int kLmBoundParts = 64;  // workgroups of the LM bound kernel = lanes that read them

struct alignas(64) FrameHdr {
    int32_t count;       // |S_t| (0 for frames at or beyond the utterance length)
    int32_t has_blank;   // 1 if token 0 survived (it is survivor 0 then), else 0
    float top;           // max_v lp[t][v]
    uint32_t div_magic;  // floor((2^32 - 1) / n) + 1 for n = count - has_blank > 1, else 0:
                         // umulhi(e, div_magic) == e / n for every e < 2^19, and at most one
                         // more than that for any larger e below 2^32
    Survivor first[kInlineSurvivors];  // survivors 0..min(count,6)-1, ascending token; unused
                                       // places hold (token -1, log-prob -inf)
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
    Survivor* rec;      // [B*T][V]: survivors of rank >= 6 (slot = rank)
    TrieNode* trie;     // [B][trie_stride]
    float* lm_bound;    // [kLmBoundParts] partial maxima of lm_weight*table+bonus
    void* cold;         // [B][2][kColdBytesPerGeneration] when beam > kBeamInLds, else unused
    int64_t trie_stride;
    size_t bytes;
};

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

inline Workspace carve_workspace(void* base, int32_t B, int32_t T, int32_t V, int32_t beam) {
    Workspace w;
    const size_t frames = (size_t)B * (size_t)T;
    const size_t off_hdr = 0;
    const size_t off_rec = align_up(off_hdr + frames * sizeof(FrameHdr), 256);
    const size_t off_trie = align_up(off_rec + frames * (size_t)V * sizeof(Survivor), 256);
    w.trie_stride = (int64_t)T * beam + 1;
    const size_t off_lmb =
        align_up(off_trie + (size_t)B * (size_t)w.trie_stride * sizeof(TrieNode), 256);
    const size_t off_cold = off_lmb + 256;
    w.bytes = off_cold + (beam > kBeamInLds ? align_up((size_t)B * 2 * kColdBytesPerGeneration, 256)
                                            : 0);
    char* p = static_cast<char*>(base);
    w.hdr = p ? reinterpret_cast<FrameHdr*>(p + off_hdr) : nullptr;
    w.rec = p ? reinterpret_cast<Survivor*>(p + off_rec) : nullptr;
    w.trie = p ? reinterpret_cast<TrieNode*>(p + off_trie) : nullptr;
    w.lm_bound = p ? reinterpret_cast<float*>(p + off_lmb) : nullptr;
    w.cold = p ? p + off_cold : nullptr;
    return w;
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
