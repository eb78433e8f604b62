// CTC prefix beam search over the survivor lists (paper Sec. 3, Algorithm 1: the
// loop over beam entries and kept tokens, the set-insert that merges equal
// prefixes, SelectTopK and GetHighestScorePrefix).
//
// One workgroup decodes one utterance and stays resident for all its frames.
// The beam (prefix hash, parent hash, last token, p_b, p_nb, trie node) lives in
// LDS.  A candidate is either "entry j stays" or "entry i extended by survivor
// k"; candidates are held in registers (or recomputed when there are more than
// the registers hold), never written to memory.  An extension i+s can only
// coincide with a prefix that is already in the beam (a prefix has one parent),
// so merging is done from the side of that beam entry: it knows its parent's
// place in the beam and adds the parent's extension mass to its own p_nb; the
// extension itself is then skipped.  Every log-sum-exp has two operands.  The
// parent links are carried from frame to frame through a map "old place -> new
// place" of the entries that stay; only a prefix whose parent was absent looks
// it up in a small LDS hash table of the prefixes that entered in this frame.
//
// Top-`beam` selection works on an order-preserving 64-bit image of the fp64
// score: a two-level histogram over the distance to an upper bound locates the
// bucket holding the beam-th best candidate, buckets are refined until the
// boundary bucket is small, and its members are ranked exactly by (score, hash).
//
// Latency is what matters here (frames of one utterance are strictly serial):
//  - frame headers (which carry the first six survivors) are staged through LDS
//    32 frames at a time, one chunk ahead, and barriers wait for LDS traffic only,
//    so global loads and trie stores stay in flight across them;
//  - frames whose only survivor is blank change no prefix and no order: every entry's
//    total takes the frame's log-prob (the thread that owns the entry adds it in a
//    register, in the order a plain implementation adds them) and a flag says that
//    p_b = total, p_nb = -inf holds for every entry; a run of such frames is consumed at
//    once (the frames of a chunk are classified together) and costs one LDS round trip
//    and one barrier for the whole run;
//  - frames with at most six survivors keep them in registers; what the prune
//    stage can say about a frame by itself (blank kept?, the division constant
//    that maps a candidate index to its beam entry) comes with the header;
//  - "stay" candidates (which need the log-sum-exps) and extension candidates are
//    mapped to different wavefronts so that they are evaluated side by side, and
//    the end-of-frame clean-up is done by the wavefronts that have no links to set.
//
// The kernel is built several times over (workgroup size, beam capacity, register budget):
// four wavefronts for the frames of a pruned small vocabulary, eight with an entry-major
// candidate mapping where frames hold hundreds to thousands of candidates, and two with a
// tighter register budget for batches that fill the chip, where instruction issue and
// residency count instead of one frame's latency (see launch_beam).
#include <type_traits>

#include "fltop_internal.h"

namespace fltop {
namespace {

constexpr int kThreadsSmall = 256;  // workgroup size for small vocabularies
constexpr int kThreadsLarge = 512;  // and for large ones (see launch_beam)
constexpr int kThreadsHuge = 1024;  // beams beyond 512 entries: still one thread per entry
constexpr int kThreadsDense = 128;  // small frames, batches larger than the chip holds at once
constexpr int kWave = 64;
// The beam lives in LDS, so its capacity is a compile-time size: kernels are built for a
// small one (which keeps several workgroups per CU for large batches) and for the largest.
constexpr int kBeamSmall = 128;
constexpr int kBeamTiny = 64;  // one-shot decodes of dense batches (17 KB of LDS)
constexpr int kBeamLarge = 512;
constexpr int kBeamHuge = FLTOP_MAX_BEAM;  // 1000-entry beams (paper Sec. 4: beam-size 1000)
static_assert(kBeamHuge == 1024, "the LDS budget below is worked out for 1024 entries");
constexpr int kFine = 1024;  // histogram bins
constexpr int kCoarse = 64;  // one per lane; a coarse bin covers 16 fine bins
constexpr int kExactCap = 64;
constexpr int kMaxShift = 54;  // kFine << kMaxShift covers all 64-bit distances
constexpr int kRegK = kInlineSurvivors;  // survivors kept in registers
constexpr int kRegCand = 1;              // extension candidates kept in registers per thread
constexpr int kChunk = 32;               // frame headers staged per chunk
constexpr int kWaypoints = 256;
constexpr uint64_t kGolden = 0x9E3779B97F4A7C15ull;
constexpr uint64_t kAllOnes = ~0ull;

// Two generations of a 1024-entry beam with everything in LDS would take 219 KB of the 160 KB
// a workgroup can have.  For that capacity the fields that only the trie bookkeeping needs
// (parent hash, trie node, length, skip ancestor: read once per emitted entry, never by the
// candidate evaluation) live in global memory instead (ColdSlab, in the workspace; L2-resident),
// the children lists are left out (builds with 512 threads and more use the pair table) and the
// two open-addressing tables are half as large per entry.
template <int MB>
struct SlabTraits {
    static constexpr bool kColdGlobal = MB > 512;
    static constexpr int kColdInLds = kColdGlobal ? 1 : MB;   // places of the cold fields in LDS
    static constexpr int kKidLists = kColdGlobal ? 4 : MB;    // places of the children lists
    static constexpr int kHashSlots = kColdGlobal ? 2 * MB : 4 * MB;
};

template <int MB>
struct BeamSlab {
    uint64_t h[MB];   // prefix hash
    uint64_t hp[SlabTraits<MB>::kColdInLds];  // parent prefix hash (unused when plen == 0)
    double pb[MB];
    double pnb[MB];
    double ptot[MB];
    int32_t last[MB];  // last token, -1 for the empty prefix
    int32_t node[SlabTraits<MB>::kColdInLds];  // trie node of the prefix
    int32_t plen[SlabTraits<MB>::kColdInLds];  // prefix length
    int32_t xanc[SlabTraits<MB>::kColdInLds];  // trie node of the ancestor at depth 8*floor(plen/8)
};

// The same four fields of one beam generation in global memory (kColdGlobal builds).
template <int MB>
struct ColdSlab {
    uint64_t hp[MB];
    int32_t node[MB];
    int32_t plen[MB];
    int32_t xanc[MB];
};
static_assert(sizeof(ColdSlab<FLTOP_MAX_BEAM>) == kColdBytesPerGeneration,
              "the workspace reserves two of these per utterance");

// One generation's trie bookkeeping fields, wherever they live.
template <int MB>
struct ColdRef {
    BeamSlab<MB>* lds;
    ColdSlab<MB>* glb;
    __device__ __forceinline__ uint64_t hp(int i) const {
        if constexpr (SlabTraits<MB>::kColdGlobal) return glb->hp[i];
        else return lds->hp[i];
    }
    __device__ __forceinline__ int32_t node(int i) const {
        if constexpr (SlabTraits<MB>::kColdGlobal) return glb->node[i];
        else return lds->node[i];
    }
    __device__ __forceinline__ int32_t plen(int i) const {
        if constexpr (SlabTraits<MB>::kColdGlobal) return glb->plen[i];
        else return lds->plen[i];
    }
    __device__ __forceinline__ int32_t xanc(int i) const {
        if constexpr (SlabTraits<MB>::kColdGlobal) return glb->xanc[i];
        else return lds->xanc[i];
    }
    __device__ __forceinline__ void set(int i, uint64_t hp_, int32_t node_, int32_t plen_,
                                        int32_t xanc_) const {
        if constexpr (SlabTraits<MB>::kColdGlobal) {
            glb->hp[i] = hp_;
            glb->node[i] = node_;
            glb->plen[i] = plen_;
            glb->xanc[i] = xanc_;
        } else {
            lds->hp[i] = hp_;
            lds->node[i] = node_;
            lds->plen[i] = plen_;
            lds->xanc[i] = xanc_;
        }
    }
};

// parent / children links of one beam generation
template <int MB>
struct alignas(16) Links {
    int32_t par[MB];
    int32_t first_kid[SlabTraits<MB>::kKidLists];
    int32_t next_kid[SlabTraits<MB>::kKidLists];
    uint32_t kidmask[MB];  // bit (token & 31) set for every child in the beam
    int32_t ht[SlabTraits<MB>::kHashSlots];  // open addressing: slot -> beam index of a prefix that
                                             // entered in this generation's frame, keyed by prefix hash
};

// What a streaming (chunked) decode carries from one call to the next, per utterance: the
// beam and its links as they stand after the last frame seen, plus the scalars the frame
// loop keeps in registers.  The prefix trie lives behind the array of these records.
template <int MB>
struct StreamState {
    int32_t frames_done;  // frames decoded so far (= trie frame index of the next one)
    int32_t n_live;
    int32_t collapsed;
    int32_t out_len;      // length of the transcript as last written
    double kmax, kmin;
    // where the transcript and its entry frames were last written: the record of trie nodes
    // behind the written tokens holds for those rows only
    uint64_t out_tokens_at, out_frames_at;
    BeamSlab<MB> slab;
    int32_t par[MB];
    int32_t first_kid[MB];
    int32_t next_kid[MB];
    uint32_t kidmask[MB];
};
static_assert(sizeof(StreamState<kBeamSmall>) % 8 == 0 && sizeof(StreamState<kBeamLarge>) % 8 == 0,
              "records sit in an array: doubles stay aligned");
static_assert(offsetof(Links<kBeamSmall>, ht) == 4 * kBeamSmall * sizeof(int32_t) &&
                  offsetof(Links<kBeamLarge>, ht) == 4 * kBeamLarge * sizeof(int32_t),
              "the four link arrays are the head of Links (streaming copies them as one block)");

struct BeamArgs {
    const int32_t* lengths;
    const FrameHdr* hdr;
    const Survivor* rec;
    TrieNode* trie;
    int64_t trie_stride;
    void* cold;             // kColdGlobal builds: [B][2] ColdSlab, else unused
    const float* lm_table;  // global copy (always valid when LM is on)
    const float* lm_bound;
    double lm_alpha, lm_beta;
    int32_t B, T, V, beam;
    int32_t lm_in_lds;  // 1: table staged into LDS
    int32_t dcache_off;   // dynamic LDS: byte offset of the distance cache ...
    int32_t dcache_rows;  // ... and its size in rows of one distance per thread (0: none)
    void* stream;          // streaming decode: array of StreamState<MB> (NULL for a one-shot decode)
    int32_t* out_nodes;    // streaming: [B, t_total] trie node behind each written token
    int32_t t_total;       // streaming: frames the trie and the output rows are sized for
    int32_t out_stride;    // row length of out_tokens and of the traces
    double beam_window;  // SelectTopK's score window below the frame's best candidate; <= 0: off
    int32_t* frame_beam;        // optional trace: entries kept after each frame
    int32_t* out_token_frames;  // optional trace: frame at which each output token was appended
    int32_t* out_tokens;
    int32_t* out_lengths;
    float* out_scores;
    fltop_stats* stats;
    int32_t* nbest_count;
    int32_t* nbest_tokens;
    int32_t* nbest_lengths;
    double* nbest_pb;
    double* nbest_pnb;
};

__device__ inline uint64_t mix64(uint64_t z) {
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

__device__ inline uint64_t child_hash(uint64_t h, int32_t tok) {
    return mix64(h + kGolden * (uint64_t)((int64_t)tok + 1));
}

// Order-preserving map fp64 -> u64 (larger score, larger key); -0.0 is folded into +0.0.
__device__ inline uint64_t order_key(double x) {
    if (x == 0.0) x = 0.0;
    const uint64_t b = (uint64_t)__double_as_longlong(x);
    return (b >> 63) ? ~b : (b | 0x8000000000000000ull);
}

__device__ inline double key_value(uint64_t k) {
    const uint64_t b = (k >> 63) ? (k & 0x7FFFFFFFFFFFFFFFull) : ~k;
    return __longlong_as_double((long long)b);
}

// ---- log-sum-exp of two log-masses ------------------------------------------------------
// hi + log1p(exp(lo - hi)).  The general-purpose exp and log1p of the device math library
// take about 250 instructions for this, and two of these sit on every frame's critical path;
// the argument ranges here are narrow (exp of a non-positive number, log1p of a number in
// [0,1]), so both are written out for just that: exp by n ln2 + r reduction and the Taylor
// series to r^13, log1p(u) as log(w) + c/w with w = fl(1+u), c its rounding error, log(w)
// = k ln2 + 2 atanh(s), s = f/(2+f), series to s^25, the quotient's rounding error carried
// along.  The term is within 2.4 ulp of the exact one (measured against 80-bit arithmetic
// on the host), i.e. far below half an ulp of the sum it is added to.
__device__ __forceinline__ double exp_nonpositive(double x) {
    const double n = rint(x * 1.4426950408889634);  // log2(e)
    // ln2 in two pieces; the upper one has 21 trailing zero bits, so n * upper is exact
    double r = fma(-n, 0.6931471803691238, x);
    r = fma(-n, 1.9082149292705877e-10, r);
    double p = 1.6059043836821613e-10;  // 1/13!, then 1/12! ... 1/2!, 1, 1
    p = fma(p, r, 2.08767569878681e-09);
    p = fma(p, r, 2.505210838544172e-08);
    p = fma(p, r, 2.755731922398589e-07);
    p = fma(p, r, 2.7557319223985893e-06);
    p = fma(p, r, 2.48015873015873e-05);
    p = fma(p, r, 0.0001984126984126984);
    p = fma(p, r, 0.001388888888888889);
    p = fma(p, r, 0.008333333333333333);
    p = fma(p, r, 0.041666666666666664);
    p = fma(p, r, 0.16666666666666666);
    p = fma(p, r, 0.5);
    p = fma(p, r, 1.0);
    p = fma(p, r, 1.0);
    return ldexp(p, (int)n);  // underflows to 0 for very negative x, which is what is wanted
}

__device__ __forceinline__ double log1p_unit(double u) {  // 0 <= u <= 1
    const double w = 1.0 + u;
    const double c = u - (w - 1.0);  // what the addition lost
    const bool upper = w > 1.4142135623730951;
    const double f = upper ? fma(w, 0.5, -1.0) : w - 1.0;  // exact; w / 2^k = 1 + f
    const double den = 2.0 + f;
    const double s = f / den;
    const double s_lo = fma(-s, den, f) * __builtin_amdgcn_rcp(den);
    const double z = s * s;
    double q = 0.08;  // 2/25, then 2/23 ... 2/3
    q = fma(q, z, 0.08695652173913043);
    q = fma(q, z, 0.09523809523809523);
    q = fma(q, z, 0.10526315789473684);
    q = fma(q, z, 0.11764705882352941);
    q = fma(q, z, 0.13333333333333333);
    q = fma(q, z, 0.15384615384615385);
    q = fma(q, z, 0.18181818181818182);
    q = fma(q, z, 0.2222222222222222);
    q = fma(q, z, 0.2857142857142857);
    q = fma(q, z, 0.4);
    q = fma(q, z, 0.6666666666666666);
    const double cw = (upper ? 0.5 * c : c) * __builtin_amdgcn_rcp(1.0 + f);  // c / w
    double tail = fma(s * z, q, 2.0 * s_lo + cw);
    if (upper) tail += 1.9082149292705877e-10;
    const double body = 2.0 * s + tail;
    return upper ? 0.6931471803691238 + body : body;
}

__device__ __forceinline__ double lse2(double a, double b) {
    if (a == -INFINITY) return b;
    if (b == -INFINITY) return a;
    const double hi = a > b ? a : b;
    const double lo = a > b ? b : a;
    return hi + log1p_unit(exp_nonpositive(lo - hi));
}

// number of set bits of `mask` below this lane's own position
__device__ inline int lanes_below(uint64_t mask, int lane) {
    (void)lane;
    return (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32),
                                          __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
}

__device__ inline uint64_t sat_add(uint64_t a, uint64_t b) {
    const uint64_t s = a + b;
    return s < a ? kAllOnes : s;
}

// top of bucket `b` of a window starting at lo with bucket width 2^sh (inclusive, saturating)
__device__ inline uint64_t bucket_top(uint64_t lo, int b, int sh) {
    const uint64_t nb = (uint64_t)(b + 1);
    if (sh > 0 && (nb >> (64 - sh)) != 0) return kAllOnes;  // nb << sh overflows
    return sat_add(lo, (nb << sh) - 1ull);
}

// Workgroup barrier that orders LDS traffic only: global loads and stores issued
// earlier (header chunks, survivor records, trie nodes) stay in flight across it.
__device__ __forceinline__ void lds_barrier() {
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// Value of `v` in the lane selected by a DPP control word, 0 where that lane does
// not exist or the row is masked off.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ int dpp_or_zero(int v) {
    return __builtin_amdgcn_update_dpp(0, v, CTRL, ROW_MASK, 0xf, false);
}

// Inclusive prefix sum inside each row of 16 lanes (row_shr 1,2,3 then 4 and 8).
__device__ __forceinline__ int row_inclusive_scan(int v0) {
    int v1 = v0 + dpp_or_zero<0x111, 0xf>(v0);
    v1 += dpp_or_zero<0x112, 0xf>(v0);
    v1 += dpp_or_zero<0x113, 0xf>(v0);
    v1 += dpp_or_zero<0x114, 0xf>(v1);
    v1 += dpp_or_zero<0x118, 0xf>(v1);
    return v1;
}

// Inclusive prefix sum over the 64 lanes: row scans, then lane 15 of a row is
// broadcast into the next row (rows 1 and 3), then lane 31 into rows 2 and 3.
__device__ __forceinline__ int wave_inclusive_scan(int v0) {
    int v1 = row_inclusive_scan(v0);
    v1 += dpp_or_zero<0x142, 0xa>(v1);
    v1 += dpp_or_zero<0x143, 0xc>(v1);
    return v1;
}

// Minimum of an unsigned value over the wavefront, returned in every lane: pairwise
// exchanges inside a row of 16 lanes, then lane 15 / lane 31 carried into the next rows
// (the last lane then holds the result).
__device__ __forceinline__ uint32_t wave_min_u32(uint32_t v) {
    v = min(v, (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, 0xB1, 0xf, 0xf, false));
    v = min(v, (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, 0x4E, 0xf, 0xf, false));
    v = min(v, (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, 0x141, 0xf, 0xf, false));
    v = min(v, (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, 0x140, 0xf, 0xf, false));
    v = min(v, (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, 0x142, 0xa, 0xf, false));
    v = min(v, (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, 0x143, 0xc, 0xf, false));
    return (uint32_t)__builtin_amdgcn_readlane((int)v, kWave - 1);
}

// The same for a 64-bit value: high words first, then the low words of the lanes that
// hold the smallest high word.
__device__ __forceinline__ uint64_t wave_min_u64(uint64_t v) {
    const uint32_t hi = wave_min_u32((uint32_t)(v >> 32));
    const uint32_t lo = wave_min_u32((uint32_t)(v >> 32) == hi ? (uint32_t)v : 0xFFFFFFFFu);
    return ((uint64_t)hi << 32) | lo;
}

// dynamic LDS: dense_lp[V] fp32, s_tok[V] u16, in the 512-thread builds s_lp[V] fp32, then
// (optionally) the LM table
__host__ __device__ inline size_t s_lp_lds_offset(int V) {
    return (((size_t)V * (sizeof(float) + sizeof(uint16_t))) + 15) / 16 * 16;
}
__host__ __device__ inline size_t lm_lds_offset(int V, bool with_s_lp) {
    return s_lp_lds_offset(V) + (with_s_lp ? ((size_t)V * sizeof(float) + 15) / 16 * 16 : 0);
}

// Optional per-phase cycle accounting, compiled in only with -DFLTOP_PHASE_CLOCKS; the default
// build carries none of it.  The wavefronts of a workgroup form four groups (group 0 holds the
// stay candidates, group 2 the first extension candidates); lane 0 of each group's first
// wavefront keeps the clocks, so the table shows which group a barrier waits for.
#ifdef FLTOP_PHASE_CLOCKS
#define PHASE_MARK(idx)                      \
    do {                                     \
        if (ph_rec) {                        \
            const uint64_t now_ = clock64(); \
            ph_clk[idx] += now_ - ph_last;   \
            ph_last = now_;                  \
        }                                    \
    } while (0)
#else
#define PHASE_MARK(idx) \
    do {                \
    } while (0)
#endif

// What a frame header holds besides survivors 2..5 (one 32-byte LDS read).
struct HdrHead {
    int32_t count;
    uint32_t rec_base;
    float top;
    uint32_t div_magic;
    Survivor s0, s1;
};

// An LDS-typed pointer: reads through it are LDS reads, not generic (flat) ones, which
// would wait on the global-memory counter as well.
typedef const __attribute__((address_space(3))) float* LdsFloatPtr;

// Uniform per-frame values the candidate evaluation needs.  Only ever read through
// constant field names, so it dissolves into registers after inlining.
template <int MB>
struct FrameCtx {
    const BeamSlab<MB>* cur;
    const Links<MB>* lk;
    const float* dense_lp;   // LDS, K > 6 only: log-prob by token, -inf if pruned
    const uint16_t* s_tok;   // LDS, K > 6 only: surviving tokens, ascending
    const float* s_lp;       // LDS, K > 6 only, 512-thread builds: their log-probs, same order
    LdsFloatPtr lm_lds;      // LM table staged in LDS (kernel variant kLmLds)
    const float* lm_glb;     // LM table in global memory (kernel variant kLmGlobal)
    double lm_alpha, lm_beta;
    int V;
    bool big;                // survivors staged through LDS
    bool collapsed;          // blank-only frames came last: read p_b as total, p_nb as -inf
    int nb0;                 // 1 if blank survived (it is record 0 then)
    int Knb;                 // non-blank survivors
    uint32_t div_magic;      // from the frame header: umulhi(e, div_magic) is e / Knb, or one
                             // more when e is large (Knb > 1)
    uint64_t Rk;             // key of an upper bound of every candidate score
    // survivors 0..5 as plain scalars (an indexed private array would live in scratch)
    int32_t t0, t1, t2, t3, t4, t5;
    float l0, l1, l2, l3, l4, l5;
};

// Selection window: bucket(x) = (x - lo) >> sh over score distances (mode 0) or over
// prefix hashes of the candidates whose distance is exactly Dfix (mode 1).
struct Window {
    uint64_t lo, Dfix;
    int sh, mode;
};

// The register-resident survivors travel by value (twelve scalars): selecting among
// fields read through a pointer would be turned into an indexed load, i.e. scratch.
__device__ __forceinline__ float pick_lp(int32_t tok, int32_t t0, int32_t t1, int32_t t2,
                                         int32_t t3, int32_t t4, int32_t t5, float l0, float l1,
                                         float l2, float l3, float l4, float l5) {
    float r = -INFINITY;
    r = (t0 == tok) ? l0 : r;
    r = (t1 == tok) ? l1 : r;
    r = (t2 == tok) ? l2 : r;
    r = (t3 == tok) ? l3 : r;
    r = (t4 == tok) ? l4 : r;
    r = (t5 == tok) ? l5 : r;
    return r;
}

// (token, log-prob) of survivor k in one pass: the index compares serve both selections
template <int MB>
__device__ __forceinline__ int32_t surv_tok_lp(const FrameCtx<MB>& f, int k, double& lp) {
    if (f.big) {
        const int32_t s = (int32_t)f.s_tok[k];
        lp = (double)f.dense_lp[s];
        return s;
    }
    const int32_t t0 = f.t0, t1 = f.t1, t2 = f.t2, t3 = f.t3, t4 = f.t4, t5 = f.t5;
    const float l0 = f.l0, l1 = f.l1, l2 = f.l2, l3 = f.l3, l4 = f.l4, l5 = f.l5;
    int32_t r = t0;
    float l = l0;
    r = (k == 1) ? t1 : r;
    l = (k == 1) ? l1 : l;
    r = (k == 2) ? t2 : r;
    l = (k == 2) ? l2 : l;
    r = (k == 3) ? t3 : r;
    l = (k == 3) ? l3 : l;
    r = (k == 4) ? t4 : r;
    l = (k == 4) ? l4 : l;
    r = (k == 5) ? t5 : r;
    l = (k == 5) ? l5 : l;
    lp = (double)l;
    return r;
}

// log-prob of a token in this frame, -inf when it did not survive (or tok < 0)
template <int MB>
__device__ __forceinline__ double lp_of(const FrameCtx<MB>& f, int32_t tok) {
    if (tok < 0) return -INFINITY;
    if (f.big) return (double)f.dense_lp[tok];
    const int32_t t0 = f.t0, t1 = f.t1, t2 = f.t2, t3 = f.t3, t4 = f.t4, t5 = f.t5;
    const float l0 = f.l0, l1 = f.l1, l2 = f.l2, l3 = f.l3, l4 = f.l4, l5 = f.l5;
    return (double)pick_lp(tok, t0, t1, t2, t3, t4, t5, l0, l1, l2, l3, l4, l5);
}

// The LM flavour is a kernel template parameter: with one kernel serving all three, the
// LDS read and the global read would meet at a joint wait on both memory counters.
enum : int { kLmNone = 0, kLmLds = 1, kLmGlobal = 2 };

template <int LM, int MB>
__device__ __forceinline__ double lm_term(const FrameCtx<MB>& f, int32_t prev, int32_t tok) {
    if (LM == kLmNone) return 0.0;
    const int32_t row = prev < 0 ? 0 : prev;
    const int64_t at = (int64_t)row * f.V + tok;
    const float v = (LM == kLmLds) ? f.lm_lds[at] : f.lm_glb[at];
    return f.lm_alpha * (double)v + f.lm_beta;
}

// Extension candidate e = i * Knb + k (entry i, non-blank survivor k): distance of its
// score below the reference, or ~0 when it has no mass or coincides with a beam entry
// (that entry's own update absorbs it).
// Extension candidate number e names entry i = e / Knb and non-blank survivor k = e % Knb.
template <int MB>
__device__ __forceinline__ void cand_of(const FrameCtx<MB>& f, int e, int& entry, int32_t& tok,
                                        double& lp) {
    // the reciprocal is rounded up, so for large e the quotient can come out one too large
    // (never more): a negative remainder says so
    int i = f.Knb > 1 ? (int)__umulhi((uint32_t)e, f.div_magic) : e;
    int k = e - i * f.Knb;
    if (k < 0) {
        --i;
        k += f.Knb;
    }
    entry = i;
    tok = surv_tok_lp(f, f.nb0 + k, lp);
}

// What a new prefix takes over from the entry it extends.  Builds with four wavefronts read it
// together with that entry's masses when the thread's first extension is evaluated, so that
// entering the beam does not begin with a round trip to LDS.
struct ExtSource {
    uint64_t h;  // the entry's prefix hash
    int32_t node, plen, xanc;
};

template <int LM, int MB, bool WITH_SOURCE = false>
__device__ __forceinline__ uint64_t eval_ext(const FrameCtx<MB>& f, int e, int& src_entry,
                                             int32_t& tok, const ColdRef<MB>* cold = nullptr,
                                             ExtSource* source = nullptr) {
    int i;
    int32_t s;
    double lps;
    cand_of(f, e, i, s, lps);
    src_entry = i;
    tok = s;
    // the four reads go out together; the children list is walked only on a mask hit
    const int32_t li = f.cur->last[i];
    const uint32_t km = f.lk->kidmask[i];
    const double pti = f.cur->ptot[i];
    const double pbi = f.collapsed ? pti : f.cur->pb[i];
    if constexpr (WITH_SOURCE) {
        source->h = f.cur->h[i];
        source->node = cold->node(i);
        source->plen = cold->plen(i);
        source->xanc = cold->xanc(i);
    }
    if ((km >> (s & 31)) & 1u) {  // maybe a child i+s is in the beam
        int guard = 0;
        for (int kid = f.lk->first_kid[i]; kid >= 0 && guard < MB;
             kid = f.lk->next_kid[kid], ++guard)
            if (f.cur->last[kid] == s) return kAllOnes;
    }
    const double src = (s == li) ? pbi : pti;
    const double sc = src + lps + lm_term<LM>(f, li, s);
    if (!(sc > -INFINITY)) return kAllOnes;
    return f.Rk - order_key(sc);
}

// ---- 512-thread builds: entry-major candidates --------------------------------------------
// Frames of a large vocabulary (or a large beam) have thousands of candidates, dozens per
// thread.  There a thread takes all its candidates from ONE beam entry, which it reads once
// per frame, and "is entry i extended by token s already in the beam?" is one probe of a
// table of (parent place, token) pairs, whatever the number of children (with lanes on
// different entries, walking the children lists would cost every lane the longest list).

// What an extension candidate needs of its beam entry.
struct EntryView {
    int32_t last;      // the entry's last token
    uint32_t kidmask;  // bit (token & 31) of every child in the beam
    double ptot, pb;   // total mass, and the mass of alignments ending in blank
};

template <int MB>
__device__ __forceinline__ EntryView view_entry(const FrameCtx<MB>& f, int i) {
    EntryView v;
    v.last = f.cur->last[i];
    v.kidmask = f.lk->kidmask[i];
    v.ptot = f.cur->ptot[i];
    v.pb = f.collapsed ? v.ptot : f.cur->pb[i];
    return v;
}

__device__ __forceinline__ uint32_t kid_key(int parent, int32_t tok) {
    return ((uint32_t)parent << 16) | ((uint32_t)tok & 0xffffu);
}
static_assert(FLTOP_MAX_VOCAB <= 65536 && FLTOP_MAX_BEAM <= 32768, "a (place, token) pair is 32 bits");
constexpr uint32_t kNoKid = 0xffffffffu;

// kidset: open addressing over `slots` (a power of two) words, kNoKid = empty
__device__ __forceinline__ void kidset_insert(uint32_t* kidset, int slots, int parent, int32_t tok) {
    const uint32_t key = kid_key(parent, tok);
    uint32_t hs = (key * 2654435761u >> 12) & (slots - 1);
    for (int probe = 0; probe < slots; ++probe) {
        if (atomicCAS(&kidset[hs], kNoKid, key) == kNoKid) break;
        hs = (hs + 1) & (slots - 1);
    }
}

__device__ __forceinline__ bool kidset_has(const uint32_t* kidset, int slots, int parent, int32_t tok) {
    const uint32_t key = kid_key(parent, tok);
    uint32_t hs = (key * 2654435761u >> 12) & (slots - 1);
    bool found = false, done = false;  // (one way out of the loop)
    for (int probe = 0; probe < slots && !done; ++probe) {
        const uint32_t v = kidset[hs];
        found = v == key;
        done = found || v == kNoKid;
        hs = (hs + 1) & (slots - 1);
    }
    return found;
}

// (token, log-prob) of survivor k, the staged ones by rank
template <int MB>
__device__ __forceinline__ int32_t surv_by_rank(const FrameCtx<MB>& f, int k, double& lp) {
    if (f.big) {
        lp = (double)f.s_lp[k];
        return (int32_t)f.s_tok[k];
    }
    return surv_tok_lp(f, k, lp);
}

// Extension of entry i (seen as `v`) by non-blank survivor k: distance of its score below
// the reference, or ~0 when it has no mass or coincides with a beam entry.
template <int LM, int MB>
__device__ __forceinline__ uint64_t eval_ext_of(const FrameCtx<MB>& f, const EntryView& v, int i,
                                                int k, const uint32_t* kidset, int kid_slots,
                                                int32_t& tok) {
    double lps;
    const int32_t s = surv_by_rank(f, f.nb0 + k, lps);
    tok = s;
    if ((v.kidmask >> (s & 31)) & 1u) {  // maybe a child i+s is in the beam
        if (kidset_has(kidset, kid_slots, i, s)) return kAllOnes;
    }
    const double src = (s == v.last) ? v.pb : v.ptot;
    const double sc = src + lps + lm_term<LM>(f, v.last, s);
    if (!(sc > -INFINITY)) return kAllOnes;
    return f.Rk - order_key(sc);
}

// Token of non-blank survivor k alone (for a candidate whose distance is already known).
template <int MB>
__device__ __forceinline__ int32_t ext_token(const FrameCtx<MB>& f, int k) {
    double lp_unused;
    return surv_by_rank(f, f.nb0 + k, lp_unused);
}

template <int MB>
__device__ __forceinline__ uint64_t cand_hash(const FrameCtx<MB>& f, int src_entry, int32_t tok) {
    const uint64_t h = f.cur->h[src_entry];
    return tok < 0 ? h : child_hash(h, tok);
}

__device__ __forceinline__ int window_bin(const Window& w, uint64_t x) {
    const uint64_t q = (x - w.lo) >> w.sh;
    return q > (uint64_t)(kFine - 1) ? (kFine - 1) : (int)q;
}

// One candidate into the two-level histogram of the current window.
template <int MB>
__device__ __forceinline__ void hist_add(const FrameCtx<MB>& f, const Window& w, uint64_t D, int se,
                                         int32_t tk, uint32_t* hfine, uint32_t* hcoarse) {
    uint64_t x = D;
    if (w.mode != 0) {
        if (D != w.Dfix) return;
        x = cand_hash(f, se, tk);
    }
    if (x < w.lo) return;
    const int bin = window_bin(w, x);
    atomicAdd(&hfine[bin], 1u);
    atomicAdd(&hcoarse[bin >> 4], 1u);
}

// The same for the candidates beyond the register cache, of which a frame may have
// thousands.  All that lie beyond the window share the last bin, and one LDS word cannot
// take that many atomics quickly: those are counted in a register (`n_clamp`) instead.
template <int MB>
__device__ __forceinline__ void hist_add_many(const FrameCtx<MB>& f, const Window& w, uint64_t D,
                                              int se, int32_t tk, uint32_t* hfine,
                                              uint32_t* hcoarse, int& n_clamp) {
    uint64_t x = D;
    if (w.mode != 0) {
        if (D != w.Dfix) return;
        x = cand_hash(f, se, tk);
    }
    if (x < w.lo) return;
    const int bin = window_bin(w, x);
    if (bin == kFine - 1) {
        ++n_clamp;
        return;
    }
    atomicAdd(&hfine[bin], 1u);
    atomicAdd(&hcoarse[bin >> 4], 1u);
}

// One candidate into the boundary list if it falls into bucket `bstar`.
template <int MB>
__device__ __forceinline__ void boundary_add(const FrameCtx<MB>& f, const Window& w, int bstar,
                                             uint64_t D, int se, int32_t tk, int32_t* count,
                                             uint64_t* bl_D, uint64_t* bl_h) {
    uint64_t x = D;
    uint64_t hh = 0;
    bool have_h = false;
    if (w.mode != 0) {
        if (D != w.Dfix) return;
        hh = cand_hash(f, se, tk);
        have_h = true;
        x = hh;
    }
    if (x < w.lo) return;
    if (window_bin(w, x) != bstar) return;
    if (!have_h) hh = cand_hash(f, se, tk);
    const int pos = atomicAdd(count, 1);
    if (pos < kExactCap) {
        bl_D[pos] = D;
        bl_h[pos] = hh;
    }
}

// Kept iff (D, hash) <= (selD, selH) lexicographically; the hash is computed only on
// a distance tie.
template <int MB>
__device__ __forceinline__ bool is_selected(const FrameCtx<MB>& f, uint64_t selD, uint64_t selH,
                                            uint64_t D, int se, int32_t tk, uint64_t& hh,
                                            bool& have_h) {
    if (D < selD) return true;
    if (D != selD) return false;
    hh = cand_hash(f, se, tk);
    have_h = true;
    return hh <= selH;
}

template <int MB>
__device__ __forceinline__ void publish_hash(Links<MB>* lkn, uint64_t hh, int slot) {
    constexpr int kHashSlots = SlabTraits<MB>::kHashSlots;
    uint32_t hs = (uint32_t)hh & (kHashSlots - 1);
    if (atomicCAS(&lkn->ht[hs], -1, slot) == -1) return;  // the usual case: the first place is free
    for (int probe = 1; probe < kHashSlots; ++probe) {
        hs = (hs + 1) & (kHashSlots - 1);
        if (atomicCAS(&lkn->ht[hs], -1, slot) == -1) break;
    }
}

// What an entry that stays in the beam carries over unchanged.  It is read together with the
// entry's masses when the stay candidate is evaluated, so that the copy into the next beam
// does not begin with a round trip to wherever these fields live.
struct StayFields {
    uint64_t h, hp;
    int32_t par, last, node, plen, xanc;
};

// Entry `se` keeps its prefix: copy it into `slot` of the next beam with its new masses.
template <int MB, bool PREFETCHED>
__device__ __forceinline__ void emit_stay(const FrameCtx<MB>& f, BeamSlab<MB>* nxt, Links<MB>* lkn,
                                          const ColdRef<MB>& ccur, const ColdRef<MB>& cnxt,
                                          int32_t* newslot, int slot, int beam, int se, double pb,
                                          double pnb, double tot, const StayFields& sf) {
    if (slot >= beam) return;  // only after a hash collision
    // where this entry went, and where its parent was (or -2: the parent was not in the
    // beam, so it can only be in the new one as a fresh extension)
    if constexpr (PREFETCHED) {
        newslot[se] = slot;
        lkn->par[slot] = sf.par >= 0 ? sf.par : -2;
        nxt->h[slot] = sf.h;
        nxt->pb[slot] = pb;
        nxt->pnb[slot] = pnb;
        nxt->ptot[slot] = tot;
        nxt->last[slot] = sf.last;
        cnxt.set(slot, sf.hp, sf.node, sf.plen, sf.xanc);
    } else {
        const BeamSlab<MB>* cur = f.cur;
        const uint64_t hh = cur->h[se];
        const int32_t par_old = f.lk->par[se];
        newslot[se] = slot;
        lkn->par[slot] = par_old >= 0 ? par_old : -2;
        nxt->h[slot] = hh;
        nxt->pb[slot] = pb;
        nxt->pnb[slot] = pnb;
        nxt->ptot[slot] = tot;
        nxt->last[slot] = cur->last[se];
        cnxt.set(slot, ccur.hp(se), ccur.node(se), ccur.plen(se), ccur.xanc(se));
    }
}

// Entry `se` extended by token `tk` becomes a new prefix in `slot`; its trie node id is
// fixed by (frame, slot), so no counter is needed.
template <int MB>
__device__ __forceinline__ void emit_ext(const FrameCtx<MB>& f, BeamSlab<MB>* nxt, Links<MB>* lkn,
                                         const ColdRef<MB>& ccur, const ColdRef<MB>& cnxt, int slot,
                                         int beam, int t, uint64_t D, int se, int32_t tk,
                                         uint64_t hh, bool have_h, TrieNode* trie,
                                         int64_t trie_stride) {
    if (slot >= beam) return;
    const BeamSlab<MB>* cur = f.cur;
    if (!have_h) hh = cand_hash(f, se, tk);
    const double sc = key_value(f.Rk - D);
    const int node = 1 + t * beam + slot;
    const int depth = ccur.plen(se) + 1;
    const int32_t xa = ccur.xanc(se);
    nxt->h[slot] = hh;
    nxt->pb[slot] = -INFINITY;
    nxt->pnb[slot] = sc;
    nxt->ptot[slot] = sc;
    nxt->last[slot] = tk;
    cnxt.set(slot, cur->h[se], node, depth, (depth & 7) == 0 ? node : xa);
    TrieNode tn;
    tn.parent = ccur.node(se);
    tn.xup = xa;
    tn.tok = tk;
    tn.depth = depth;
    if ((int64_t)node < trie_stride) trie[node] = tn;
    lkn->par[slot] = se;  // the parent's place in the old beam
    publish_hash(lkn, hh, slot);
}

// The same with what the new prefix takes over from entry `se` already in registers.
template <int MB>
__device__ __forceinline__ void emit_ext_prefetched(const FrameCtx<MB>& f, BeamSlab<MB>* nxt, Links<MB>* lkn,
                                         const ColdRef<MB>& ccur, const ColdRef<MB>& cnxt, int slot,
                                         int beam, int t, uint64_t D, int se, int32_t tk,
                                         uint64_t hh, bool have_h, TrieNode* trie,
                                         int64_t trie_stride, const ExtSource* source) {
    constexpr bool WITH_SOURCE = true;
    if (slot >= beam) return;
    const BeamSlab<MB>* cur = f.cur;
    if (!have_h) {
        if constexpr (WITH_SOURCE) hh = child_hash(source->h, tk);
        else hh = cand_hash(f, se, tk);
    }
    const double sc = key_value(f.Rk - D);
    const int node = 1 + t * beam + slot;
    const int depth = (WITH_SOURCE ? source->plen : ccur.plen(se)) + 1;
    const int32_t xa = WITH_SOURCE ? source->xanc : ccur.xanc(se);
    nxt->h[slot] = hh;
    nxt->pb[slot] = -INFINITY;
    nxt->pnb[slot] = sc;
    nxt->ptot[slot] = sc;
    nxt->last[slot] = tk;
    cnxt.set(slot, WITH_SOURCE ? source->h : cur->h[se], node, depth, (depth & 7) == 0 ? node : xa);
    TrieNode tn;
    tn.parent = WITH_SOURCE ? source->node : ccur.node(se);
    tn.xup = xa;
    tn.tok = tk;
    tn.depth = depth;
    if ((int64_t)node < trie_stride) trie[node] = tn;
    lkn->par[slot] = se;  // the parent's place in the old beam
    publish_hash(lkn, hh, slot);
}

// WAVES = wavefronts per SIMD the register budget is cut for: 2 leaves the allocator all it
// asks for (no spills: the fastest single workgroup); 3 and 4 spill a few registers (each
// frame some per cent slower) so that more utterances are resident when the batch has more
// workgroups than the chip can hold at 2.
template <int LM, int THREADS, int MB, int WAVES>
__global__ __launch_bounds__(THREADS) __attribute__((amdgpu_waves_per_eu(WAVES, WAVES)))
void beam_kernel(BeamArgs a) {
    constexpr int kThreads = THREADS;
    constexpr int kWalkers = kThreads < kWaypoints ? kThreads : kWaypoints;  // back-walk batch
    static_assert(THREADS >= 4 * kChunk, "a chunk of headers is staged 16 bytes per thread");
    constexpr int kMaxBeam = MB;
    constexpr int kHashSlots = SlabTraits<MB>::kHashSlots;
    constexpr bool kColdGlobal = SlabTraits<MB>::kColdGlobal;
    static_assert(THREADS >= MB, "one thread per beam entry");
    // builds with 512 threads or more take a thread's candidates from one entry (see EntryView)
    constexpr bool kEntryMajor = THREADS >= kThreadsLarge;
    static_assert(kEntryMajor || !kColdGlobal, "the largest capacity has no children lists");
    // Builds with four wavefronts read what a staying entry carries over together with its
    // masses (measured: cfg 3 -1.7%); the larger builds, shorter of registers, read it when the
    // entry is copied (measured there: +0.4% to +1.4% otherwise).
    constexpr bool kPrefetchStay = !kEntryMajor;
    // Which way a uniform branch of the frame loop usually goes, for the block layout of the
    // four-wavefront builds: a lone wavefront per SIMD pays for every taken branch, and with the
    // usual path laid out straight a frame is 2-4% shorter (the set below was chosen by timing
    // builds with each hint on and off; the builds with 512 and 1024 threads gained nothing from
    // any of them and are left to the compiler's own guesses).
#define FLTOP_RARE(c) (kEntryMajor ? !!(c) : __builtin_expect(!!(c), 0))
#define FLTOP_USUAL(c) (kEntryMajor ? !!(c) : __builtin_expect(!!(c), 1))
    constexpr int kKidSlots = kEntryMajor ? (kColdGlobal ? 2 * MB : 4 * MB) : 4;
    __shared__ uint32_t kidset2[2][kKidSlots];  // (parent place, token) pairs, per generation
    __shared__ BeamSlab<MB> slab[2];
    __shared__ Links<MB> links[2];
    __shared__ __align__(16) uint32_t hfine[kFine];
    __shared__ __align__(16) uint32_t hcoarse[kCoarse];
    __shared__ uint64_t bl_D[kExactCap], bl_h[kExactCap];
    __shared__ FrameHdr ring[kChunk];
    __shared__ uint64_t sh_selD, sh_selH, sh_kbest;
    __shared__ uint64_t sh_minD;  // smallest distance (= best score) among a frame's candidates
    __shared__ int32_t sh_nnew, sh_blcount, sh_best;
    __shared__ unsigned long long sh_stat[8];
    __shared__ __align__(16) int32_t newslot[kMaxBeam];  // old beam index -> new beam index of an entry that stays
    extern __shared__ __align__(16) unsigned char dyn_lds[];

    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int b = blockIdx.x;
    const int V = a.V;
    const int beam = a.beam;
    const int64_t trie_stride = a.trie_stride;

    float* dense_lp = reinterpret_cast<float*>(dyn_lds);
    uint16_t* s_tok = reinterpret_cast<uint16_t*>(dyn_lds + (size_t)V * sizeof(float));
    float* s_lp = reinterpret_cast<float*>(dyn_lds + s_lp_lds_offset(V));  // kEntryMajor only
    float* lm_s = reinterpret_cast<float*>(dyn_lds + lm_lds_offset(V, kEntryMajor));
    constexpr bool has_lm = LM != kLmNone;
    // Distances of the candidates beyond the register cache, as the first histogram pass
    // worked them out: the later passes and the selection read them back instead of
    // evaluating the candidate again (row j, this thread's place = its candidate number
    // kRegCand + j).  A thread only ever reads what it wrote itself.
    uint64_t* const dcache = reinterpret_cast<uint64_t*>(dyn_lds + a.dcache_off) + tid;
    const int drows = a.dcache_rows;

    StreamState<MB>* const carried =
        a.stream ? static_cast<StreamState<MB>*>(a.stream) + b : nullptr;  // uniform
    // kColdGlobal: this utterance's two generations of trie bookkeeping fields
    ColdSlab<MB>* const cold_gen =
        kColdGlobal ? static_cast<ColdSlab<MB>*>(a.cold) + 2 * (int64_t)b : nullptr;
    const int32_t t_base = carried ? carried->frames_done : 0;
    int32_t len = a.lengths[b];
    len = len < 0 ? 0 : (len > a.T ? a.T : len);
    if (carried && len > a.t_total - t_base) len = max(0, a.t_total - t_base);
    const int64_t g_base = (int64_t)b * a.T;
    const int64_t trace_base = (int64_t)b * a.out_stride + t_base;
    const Survivor* rec_all = a.rec;

    // ---- header chunks: 32 frames x 64 B = 128 threads x 16 B ------------------------
    // Chunk c+1 is loaded into registers while chunk c is decoded and moved into LDS at
    // the chunk boundary, so the only wait for it sits in the outer (per-chunk) loop.
    const uint4* hdr_words = reinterpret_cast<const uint4*>(a.hdr + g_base);
#define FLTOP_LOAD_CHUNK(dst, c)                                                         \
    do {                                                                                 \
        (dst) = make_uint4(0u, 0u, 0u, 0u);                                              \
        if (tid < 4 * kChunk && (c) * kChunk + (tid >> 2) < len)                         \
            (dst) = hdr_words[(int64_t)(c) * (4 * kChunk) + tid];                        \
    } while (0)
#define FLTOP_RING_HEAD(t) (*reinterpret_cast<const HdrHead*>(&ring[(t) % kChunk]))

    uint4 staged;
    FLTOP_LOAD_CHUNK(staged, 0);

    // ---- one-time initialisation ------------------------------------------------
    for (int v = tid; v < V; v += kThreads) dense_lp[v] = -INFINITY;
    for (int i = tid; i < kFine; i += kThreads) hfine[i] = 0u;
    if (tid < kCoarse) hcoarse[tid] = 0u;
    if (LM == kLmLds)
        for (int i = tid; i < V * V; i += kThreads) lm_s[i] = a.lm_table[i];
    for (int g2 = 0; g2 < 2; ++g2) {
        if (tid < kMaxBeam) {
            links[g2].par[tid] = -1;
            if (!kColdGlobal) {
                links[g2].first_kid[tid] = -1;
                links[g2].next_kid[tid] = -1;
            }
            links[g2].kidmask[tid] = 0u;
        }
        for (int i = tid; i < kHashSlots; i += kThreads) links[g2].ht[i] = -1;
    }
    if (kEntryMajor)
        for (int i = tid; i < 2 * kKidSlots; i += kThreads) (&kidset2[0][0])[i] = kNoKid;
    if (tid == 0) {
        sh_nnew = 0;
        sh_blcount = 0;
        sh_minD = kAllOnes;
    }
    if (tid < 8) sh_stat[tid] = 0ull;
    if (carried) {  // the beam as the previous chunk left it
        __syncthreads();  // the link arrays were just preset by other threads
        const uint32_t* src = reinterpret_cast<const uint32_t*>(&carried->slab);
        uint32_t* dst = reinterpret_cast<uint32_t*>(&slab[0]);
        for (int i = tid; i < (int)(sizeof(BeamSlab<MB>) / 4); i += kThreads) dst[i] = src[i];
        const uint32_t* lsrc = reinterpret_cast<const uint32_t*>(carried->par);
        uint32_t* ldst = reinterpret_cast<uint32_t*>(&links[0]);
        for (int i = tid; i < 4 * kMaxBeam; i += kThreads) ldst[i] = lsrc[i];
    } else if (tid == 0) {
        BeamSlab<MB>& s0 = slab[0];
        s0.h[0] = kGolden;
        s0.pb[0] = 0.0;
        s0.pnb[0] = -INFINITY;
        s0.ptot[0] = 0.0;
        s0.last[0] = -1;
        ColdRef<MB>{&slab[0], cold_gen}.set(0, 0, 0, 0, 0);
    }
    TrieNode* trie = a.trie + (int64_t)b * trie_stride;
    double lm_ub = 0.0;  // upper bound of any LM term (never below 0)
    if (has_lm) {
        static_assert(kLmBoundParts == kWave, "one partial maximum per lane");
        float part = a.lm_bound[lane];
#pragma unroll
        for (int o = kWave / 2; o > 0; o >>= 1) part = fmaxf(part, __shfl_xor(part, o, kWave));
        lm_ub = fmax(0.0, (double)part);
    }
    __syncthreads();
    if (kEntryMajor && carried) {  // the pair table is not carried: rebuild it from the links
        if (tid < carried->n_live && links[0].par[tid] >= 0)
            kidset_insert(kidset2[0], kKidSlots, links[0].par[tid], slab[0].last[tid]);
        __syncthreads();
    }

    FrameCtx<MB> fc;
    fc.dense_lp = dense_lp;
    fc.s_tok = s_tok;
    fc.s_lp = s_lp;
    fc.lm_lds = (LdsFloatPtr)lm_s;
    fc.lm_glb = a.lm_table;
    fc.lm_alpha = a.lm_alpha;
    fc.lm_beta = a.lm_beta;
    fc.V = V;

    int mapped_for = -1;  // kEntryMajor: the beam size the thread -> entry mapping was made for
    int ext_i = 0, ext_g = 0, ext_G = 1;
    int gen = 0;         // beam generation: slab[gen], links[gen]
    int n_live = 1;
    bool collapsed = false;  // blank-only frames since the beam was last written
    double kmax_v = 0.0, kmin_v = 0.0;  // bounds of the best / worst score
    bool failed = false;     // a frame's survivor records did not fit the workspace
    int prev_out_len = 0;       // streaming: length of the transcript the last call wrote ...
    uint64_t prev_tokens_at = 0, prev_frames_at = 0;  // ... and the rows it wrote it to
    if (carried) {
        prev_out_len = carried->out_len;
        prev_tokens_at = carried->out_tokens_at;
        prev_frames_at = carried->out_frames_at;
        n_live = carried->n_live;
        collapsed = carried->collapsed != 0;
        kmax_v = carried->kmax;
        kmin_v = carried->kmin;
    }

    // Statistics of this utterance live in LDS, not in 64-bit registers that every thread would
    // carry through the whole kernel.  What the frames of one chunk add up to is wave-uniform
    // and collects in 32-bit counters (scalar registers); once per chunk the last thread of the
    // workgroup (its wavefront has the least to do) moves them into LDS.
    enum : int { kStSurv, kStCand, kStPeak, kStBeam, kStPass, kStExact, kStDrop, kStRecords };
    const bool stat_thread = tid == kThreads - 1;
    uint32_t pd_cand = 0, pd_peak = 0, pd_beam = 0, pd_pass = 0, pd_exact = 0, pd_drop = 0;
    auto flush_stats = [&]() {
        if (stat_thread) {
            atomicAdd(&sh_stat[kStCand], (unsigned long long)pd_cand);
            atomicMax(&sh_stat[kStPeak], (unsigned long long)pd_peak);
            atomicAdd(&sh_stat[kStBeam], (unsigned long long)pd_beam);
            atomicAdd(&sh_stat[kStPass], (unsigned long long)pd_pass);
            if (pd_exact) atomicAdd(&sh_stat[kStExact], (unsigned long long)pd_exact);
            if (pd_drop) atomicAdd(&sh_stat[kStDrop], (unsigned long long)pd_drop);
        }
        pd_cand = pd_peak = pd_beam = pd_pass = pd_exact = pd_drop = 0;
    };
#ifdef FLTOP_PHASE_CLOCKS
    constexpr int kWavesPerGroup = kThreads / kWave >= 4 ? kThreads / kWave / 4 : 1;
    const int ph_grp = (tid / kWave) / kWavesPerGroup;
    const bool ph_rec = lane == 0 && (tid / kWave) % kWavesPerGroup == 0;
    uint64_t ph_clk[16] = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
    uint64_t ph_last = clock64();
#endif

    const int n_chunks = (len + kChunk - 1) / kChunk;
    for (int c = 0; c < n_chunks; ++c) {
    // ---- chunk boundary: headers of frames [32c, 32c+32) into LDS, next chunk requested --
    lds_barrier();  // nobody still reads the previous chunk's headers
    if (tid < 4 * kChunk) reinterpret_cast<uint4*>(&ring[0])[tid] = staged;
    lds_barrier();
    FLTOP_LOAD_CHUNK(staged, c + 1);
    const int t_end = min(len, (c + 1) * kChunk);

    // ---- classify the chunk's frames (lane l looks at frame 32c + l): blank-only frames
    //      change no prefix and no order, and a run of them costs a few additions ----------
    uint32_t blank_only;  // bit l: blank is the only survivor of frame 32c + l
    int lp_bits;          // lane l: that frame's blank log-prob (fp32 bits)
    {
        const int fl = c * kChunk + (lane & (kChunk - 1));
        const HdrHead hh = FLTOP_RING_HEAD(fl);
        const bool inside = lane < kChunk && fl < len;
        const bool lone_blank =
            inside && hh.count == 1 && hh.s0.tok == 0 && hh.s0.lp > -INFINITY;
        blank_only = (uint32_t)__ballot(lone_blank);
        lp_bits = __float_as_int(hh.s0.lp);
        const int chunk_survivors = __builtin_amdgcn_readlane(
            wave_inclusive_scan(inside ? hh.count : 0), kWave - 1);
        // records the chunk's frames take beyond the survivors in their headers
        const int chunk_records = __builtin_amdgcn_readlane(
            wave_inclusive_scan(inside ? max(0, hh.count - kRegK) : 0), kWave - 1);
        flush_stats();  // of the previous chunk (at most 32 frames: the counters cannot wrap)
        if (stat_thread) {
            atomicAdd(&sh_stat[kStSurv], (unsigned long long)chunk_survivors);
            if (chunk_records) atomicAdd(&sh_stat[kStRecords], (unsigned long long)chunk_records);
        }
        // after a frame whose records did not fit the workspace the utterance is not decoded
        // any further, but its survivors are still counted: the caller learns what to ask for
        if (failed) continue;
    }

    for (int t = c * kChunk; t < t_end; ++t) {
        const int l = t & (kChunk - 1);
        if (FLTOP_RARE(n_live == 0)) {  // the beam died: nothing left to decode
            if (a.frame_beam && tid < t_end - t) a.frame_beam[trace_base + t + tid] = 0;
            t = t_end;  // (the loop keeps its single exit: leaving it from several places costs
            continue;   // every frame a dispatch on the way round)
        }
        // ---- run of blank-only frames --------------------------------------------------
        const int run = __builtin_ctz(~(blank_only >> l) | 0x80000000u);
        if (FLTOP_RARE(run > 0)) {
            // every entry's total takes the run's log-probs one by one, in frame order, as a
            // plain implementation adds them (the owner thread keeps the sum in a register)
            BeamSlab<MB>* const cur_run = &slab[gen];
            double own = tid < n_live ? cur_run->ptot[tid] : 0.0;
            for (int k = 0; k < run; ++k) {
                const double x = (double)__int_as_float(__builtin_amdgcn_readlane(lp_bits, l + k));
                own += x;
                kmax_v += x;
                kmin_v += x;
            }
            if (tid < n_live) cur_run->ptot[tid] = own;
            collapsed = true;
            lds_barrier();  // the new totals are read by other threads in the next full frame
            pd_cand += (uint32_t)(n_live * run);
            pd_peak = max(pd_peak, (uint32_t)n_live);
            pd_beam += (uint32_t)(n_live * run);
            if (a.frame_beam && tid < run) a.frame_beam[trace_base + t + tid] = n_live;
            t += run - 1;
            PHASE_MARK(7);
            continue;
        }
        const FrameHdr hd = ring[t % kChunk];  // all 64 bytes in one round trip
        const int K = hd.count;

        BeamSlab<MB>* const cur = &slab[gen];
        BeamSlab<MB>* const nxt = &slab[gen ^ 1];
        Links<MB>* const lk = &links[gen];
        Links<MB>* const lkn = &links[gen ^ 1];
        const ColdRef<MB> ccur{cur, kColdGlobal ? cold_gen + gen : nullptr};
        const ColdRef<MB> cnxt{nxt, kColdGlobal ? cold_gen + (gen ^ 1) : nullptr};

        // ---- survivors: registers for K <= 6, LDS staging beyond ------------------------
        const bool big = K > kRegK;
        fc.cur = cur;
        fc.lk = lk;
        fc.big = big;
        fc.collapsed = collapsed;
        // unused places of the inline list hold (-1, -inf), so they can be taken as they are
        fc.t0 = hd.first[0].tok;
        fc.l0 = hd.first[0].lp;
        fc.t1 = hd.first[1].tok;
        fc.l1 = hd.first[1].lp;
        fc.t2 = hd.first[2].tok;
        fc.l2 = hd.first[2].lp;
        fc.t3 = hd.first[3].tok;
        fc.l3 = hd.first[3].lp;
        fc.t4 = hd.first[4].tok;
        fc.l4 = hd.first[4].lp;
        fc.t5 = hd.first[5].tok;
        fc.l5 = hd.first[5].lp;
        if (tid == 0) {
            sh_nnew = 0;
            sh_blcount = 0;
        }
        if (tid >= kThreads / 2 && tid - kThreads / 2 < kMaxBeam / 4)
            reinterpret_cast<int4*>(newslot)[tid - kThreads / 2] = make_int4(-1, -1, -1, -1);
        if (big && hd.rec_base == kNoRecords) {  // uniform: the record array was too small
            failed = true;
            t = t_end;
            continue;
        }
        if (big) {
            const Survivor* recs = rec_all + ((int64_t)hd.rec_base - kRegK);
            const FrameHdr* full = &ring[t % kChunk];
            for (int k = tid; k < K; k += kThreads) {
                const Survivor s = (k < kRegK) ? full->first[k] : recs[k];
                s_tok[k] = (uint16_t)s.tok;
                if (kEntryMajor) s_lp[k] = s.lp;
                dense_lp[s.tok] = s.lp;
            }
        }
        if (big) lds_barrier();

        PHASE_MARK(0);
        fc.nb0 = hd.first[0].tok == 0 ? 1 : 0;  // survivors ascend by token: the blank, if kept, is the first
        fc.Knb = K - fc.nb0;
        fc.div_magic = hd.div_magic;
        const double lp_blank = fc.nb0 ? (double)hd.first[0].lp : -INFINITY;
        // Extension candidate e = i * Knb + k is entry i extended by non-blank survivor k.
        // Thread numbers are taken from the upper half of the wavefronts first (the lower
        // half has the stays).  Plain builds: a thread takes e = e_first, e_first + kThreads, ...
        // Entry-major builds: entry i is shared by G = kThreads / n_live threads, of which
        // number g takes k = g, g + G, g + 2G, ...
        const int n_ext = n_live * fc.Knb;
        const int e_first = (tid + kThreads / 2) & (kThreads - 1);
        if (kEntryMajor && n_live != mapped_for) {  // uniform; the beam is full most of the time
            ext_g = e_first / n_live;
            ext_i = e_first - ext_g * n_live;
            ext_G = kThreads / n_live;
            mapped_for = n_live;
        }
        const int G = ext_G;
        const bool ext_thread = ext_g < G && ext_g < fc.Knb;  // kEntryMajor only
        const int M = kEntryMajor ? (fc.Knb + G - 1) / G  // most candidates any thread has
                                  : (n_ext + kThreads - 1) / kThreads;
        const uint32_t* const kids = kidset2[gen];
        EntryView ev;
        ev.last = -1;
        ev.kidmask = 0u;
        ev.ptot = ev.pb = -INFINITY;
        // candidate number m of this thread: does it exist, and what names it
        auto cand_at = [&](int m, int& e, int& k) -> bool {
            if (kEntryMajor) {
                k = ext_g + G * m;
                e = 0;
                return ext_thread && k < fc.Knb;
            }
            e = e_first + m * kThreads;
            k = 0;
            return e < n_ext;
        };
        auto cand_eval = [&](int e, int k, int& se, int32_t& tk) -> uint64_t {
            if (kEntryMajor) {
                se = ext_i;
                return eval_ext_of<LM>(fc, ev, ext_i, k, kids, kKidSlots, tk);
            }
            return eval_ext<LM>(fc, e, se, tk);
        };
        auto cand_name = [&](int e, int k, int& se, int32_t& tk) {  // without evaluating it
            if (kEntryMajor) {
                se = ext_i;
                tk = ext_token(fc, k);
            } else {
                double lp_unused;
                cand_of(fc, e, se, tk, lp_unused);
            }
        };

        // upper bound of every candidate score -> reference key
        const double ref = kmax_v + (double)hd.top + lm_ub + 1.0986122886681098 + 1e-3;
        fc.Rk = order_key(ref);
        const uint64_t Rk = fc.Rk;

        // ---- candidates owned by this thread ----------------------------------------
        // the first extension candidate stays in registers (the others, if any, are worked
        // on one after the other and leave their distances in LDS) ...
        ExtSource xs0{};
        uint64_t cD0 = kAllOnes;  // ~0 marks "no live candidate"
        int cI0 = 0;
        int32_t cT0 = 0;
        if constexpr (kEntryMajor) {
            if (ext_thread) {
                ev = view_entry(fc, ext_i);
                cD0 = cand_eval(0, ext_g, cI0, cT0);
            }
        } else {
            if (e_first < n_ext)
                cD0 = eval_ext<LM, MB, kPrefetchStay>(fc, e_first, cI0, cT0, &ccur, &xs0);
        }
        PHASE_MARK(8);
        // ... and the stay candidate of entry `tid`
        double my_pb = -INFINITY, my_pnb = -INFINITY, my_tot = -INFINITY;
        uint64_t D_stay = kAllOnes;
        StayFields sf;
        sf.h = sf.hp = 0;
        sf.par = sf.last = sf.node = sf.plen = sf.xanc = -1;
        if (tid < n_live) {
            const int j = tid;
            const int32_t lj = cur->last[j];
            if constexpr (kPrefetchStay) {
                sf.h = cur->h[j];
                sf.hp = ccur.hp(j);
                sf.node = ccur.node(j);
                sf.plen = ccur.plen(j);
                sf.xanc = ccur.xanc(j);
                sf.last = lj;
            }
            const double lpl = lp_of(fc, lj);
            my_pb = cur->ptot[j] + lp_blank;
            const double a1 = (collapsed ? -INFINITY : cur->pnb[j]) + lpl;
            double a2 = -INFINITY;
            const int p = lk->par[j];
            if constexpr (kPrefetchStay) sf.par = p;
            if (p >= 0 && lpl > -INFINITY) {
                const int32_t lpar = cur->last[p];
                const double ptp = cur->ptot[p];
                const double src = (lpar == lj && !collapsed) ? cur->pb[p] : ptp;
                a2 = src + lpl + lm_term<LM>(fc, lpar, lj);
            }
            my_pnb = lse2(a1, a2);
            my_tot = lse2(my_pb, my_pnb);
            if (my_tot > -INFINITY) D_stay = Rk - order_key(my_tot);
        }
        PHASE_MARK(1);

        // ---- selection: find (selD, selH); keep D < selD or (D == selD and hash <= selH)
        uint64_t selD = kAllOnes, selH = kAllOnes;
        uint64_t kbest_key = 0;  // upper bound of the best candidate's key
        uint64_t Dcut = kAllOnes;  // candidates farther than this from the reference lie
                                   // outside the score window
        {
            // initial bucket width from the spread of the current beam
            const double est_low = kmin_v + (double)hd.top - 2.0;
            uint64_t Dest = Rk - order_key(est_low);
            if (Dest < 1024) Dest = 1024;
            Window w;
            w.sh = 64 - __clzll((long long)Dest) - 10;
            if (w.sh < 0) w.sh = 0;
            if (w.sh > kMaxShift) w.sh = kMaxShift;
            w.lo = 0;
            w.mode = 0;
            w.Dfix = 0;
            int need = beam;
            const bool windowed = a.beam_window > 0.0;  // uniform
            // One pass over the candidates: histogram, scan, and either the threshold (true) or a
            // narrower window for the next pass (false).  The first pass, the only one in all but
            // a few frames, is compiled with its window constants folded in.
            auto pass = [&](auto first_tag) -> bool {
                constexpr bool kFirst = decltype(first_tag)::value;
                if (kFirst) {
                    w.lo = 0;
                    w.mode = 0;
                    w.Dfix = 0;
                    need = beam;
                }
                if (!kFirst) {  // rare: the single histogram is reused for a refined window
                    lds_barrier();
                    for (int i = tid; i < kFine; i += kThreads) hfine[i] = 0u;
                    if (tid < kCoarse) hcoarse[tid] = 0u;
                    lds_barrier();
                }
                if (D_stay != kAllOnes) hist_add(fc, w, D_stay, tid, -1, hfine, hcoarse);
                if (cD0 != kAllOnes) hist_add(fc, w, cD0, cI0, cT0, hfine, hcoarse);
                uint64_t nearest = kAllOnes;  // this thread's best candidate (score window only)
                if (FLTOP_RARE(windowed)) {
                    nearest = D_stay < cD0 ? D_stay : cD0;
                }
                if (FLTOP_RARE(M > kRegCand)) {
                    int n_clamp = 0;
                    for (int m = kRegCand; m < M; ++m) {
                        int e, k;
                        if (!cand_at(m, e, k)) continue;  // (and none at any later m)
                        int se = 0;
                        int32_t tk = 0;
                        uint64_t D;
                        const int row = m - kRegCand;
                        if (!kFirst && row < drows) {
                            D = dcache[row * kThreads];
                            if (w.mode != 0 && D == w.Dfix) cand_name(e, k, se, tk);  // for its hash
                        } else {
                            D = cand_eval(e, k, se, tk);
                            if (row < drows) dcache[row * kThreads] = D;
                        }
                        if (windowed) nearest = D < nearest ? D : nearest;
                        if (D != kAllOnes)
                            hist_add_many(fc, w, D, se, tk, hfine, hcoarse, n_clamp);
                    }
                    const int wave_clamp = wave_inclusive_scan(n_clamp);  // lane 63: the sum
                    if (lane == kWave - 1 && wave_clamp > 0) {
                        atomicAdd(&hfine[kFine - 1], (uint32_t)wave_clamp);
                        atomicAdd(&hcoarse[kCoarse - 1], (uint32_t)wave_clamp);
                    }
                }
                if (kFirst && windowed) {  // one LDS atomic per wavefront
                    const uint64_t wave_nearest = wave_min_u64(nearest);
                    if (lane == 0 && wave_nearest != kAllOnes)
                        atomicMin((unsigned long long*)&sh_minD,
                                  (unsigned long long)wave_nearest);
                }
                lds_barrier();
                PHASE_MARK(2);
                if (kFirst && windowed) {
                    // the frame's best score, exactly; the window's floor in the same fp64
                    // subtraction a plain implementation does, mapped back to a distance
                    const uint64_t minD = sh_minD;
                    if (minD != kAllOnes && minD <= Rk) {
                        const double floor_score = key_value(Rk - minD) - a.beam_window;
                        const uint64_t floor_key = order_key(floor_score);
                        Dcut = floor_key <= Rk ? Rk - floor_key : 0;
                    }
                }
                // every wave scans the histogram redundantly (results are uniform)
                const int cs = (int)hcoarse[lane];
                const int incl = wave_inclusive_scan(cs);
                const int total = __builtin_amdgcn_readlane(incl, kWave - 1);
                // The two rows of fine bins looked at below -- the one with the first occupied
                // bin (lanes 0..15) and the one in which the need-th candidate lies (lanes
                // 16..31) -- are asked for together: one LDS round trip instead of two.
                const uint64_t occ = __ballot(cs > 0);
                const uint64_t cross = __ballot(incl >= need);
                const int lmin = occ != 0 ? __ffsll((long long)occ) - 1 : 0;
                const int lstar = cross != 0 ? __ffsll((long long)cross) - 1 : 0;
                const int fine_row = (lane & 16) ? lstar : lmin;
                const int fine_val = (int)hfine[fine_row * 16 + (lane & 15)];
                if (kFirst) {
                    pd_cand += (uint32_t)total;
                    pd_peak = max(pd_peak, (uint32_t)total);
                    // first occupied bin -> bound of the best candidate (window starts at 0)
                    if (FLTOP_USUAL(occ != 0)) {
                        const uint32_t f = (uint32_t)fine_val;
                        const uint64_t occf = __ballot(f > 0 && lane < 16);
                        const int bmin = lmin * 16 + (__ffsll((long long)occf) - 1);
                        const uint64_t dmin = (w.sh > 0 && ((uint64_t)bmin >> (64 - w.sh)) != 0)
                                                  ? kAllOnes
                                                  : ((uint64_t)bmin << w.sh);
                        kbest_key = dmin > Rk ? 0 : Rk - dmin;
                    }
                }
                ++pd_pass;
                if (FLTOP_RARE(total <= need)) {  // everything left in the window is kept
                    selD = (w.mode == 0) ? kAllOnes : w.Dfix;
                    selH = kAllOnes;
                    return true;
                }
                // coarse bin holding the need-th candidate (lstar), then the fine bin inside it
                // (its row sits in lanes 16..31; the row scan works within each 16 lanes)
                const int above_c =
                    __builtin_amdgcn_readlane(incl, lstar) - __builtin_amdgcn_readlane(cs, lstar);
                const int fs = fine_val;
                const int fincl = row_inclusive_scan(fs);
                const uint64_t fcross =
                    __ballot((lane & 48) == 16 && above_c + fincl >= need) >> 16;
                const int fl = __ffsll((long long)fcross) - 1;
                const int bstar = lstar * 16 + fl;
                const int n_b = __builtin_amdgcn_readlane(fs, 16 + fl);
                const int n_above = above_c + __builtin_amdgcn_readlane(fincl, 16 + fl) - n_b;
                const int r = need - n_above;  // 1 <= r <= n_b
                const bool clamp_bin = (bstar == kFine - 1) && (w.sh < kMaxShift);

                if (FLTOP_USUAL(n_b == r)) {  // the boundary bucket is taken whole
                    const uint64_t top = clamp_bin ? kAllOnes : bucket_top(w.lo, bstar, w.sh);
                    if (w.mode == 0) {
                        selD = top;
                        selH = kAllOnes;
                    } else {
                        selD = w.Dfix;
                        selH = top;
                    }
                    return true;
                }
                if (FLTOP_USUAL(n_b <= kExactCap)) {
                    // ---- exact ranking of the boundary bucket by (distance, hash)
                    ++pd_exact;
                    if (D_stay != kAllOnes)
                        boundary_add(fc, w, bstar, D_stay, tid, -1, &sh_blcount, bl_D, bl_h);
                    if (cD0 != kAllOnes)
                        boundary_add(fc, w, bstar, cD0, cI0, cT0, &sh_blcount, bl_D, bl_h);
                    for (int m = kRegCand; m < M; ++m) {
                        int e, k;
                        if (!cand_at(m, e, k)) continue;  // (and none at any later m)
                        int se = 0;
                        int32_t tk = 0;
                        uint64_t D;
                        const int row = m - kRegCand;
                        if (row < drows) {
                            D = dcache[row * kThreads];
                            // only a member of the boundary bucket is looked at further
                            const bool maybe = w.mode != 0 ? D == w.Dfix
                                                           : (D >= w.lo && window_bin(w, D) == bstar);
                            if (!maybe) continue;
                            cand_name(e, k, se, tk);
                        } else {
                            D = cand_eval(e, k, se, tk);
                        }
                        if (D != kAllOnes)
                            boundary_add(fc, w, bstar, D, se, tk, &sh_blcount, bl_D, bl_h);
                    }
                    lds_barrier();
                    if (tid < kWave) {
                        const int n = min(sh_blcount, kExactCap);
                        const bool mine = lane < n;
                        const uint64_t myD = mine ? bl_D[lane] : 0;
                        const uint64_t myH = mine ? bl_h[lane] : 0;
                        int rank = 0, same = 0;
                        for (int e = 0; e < n; ++e) {
                            const uint64_t oD = bl_D[e], oH = bl_h[e];
                            rank += (oD < myD || (oD == myD && oH < myH)) ? 1 : 0;
                            same += (oD == myD && oH == myH) ? 1 : 0;
                        }
                        // the r-th best member (members that collide in both fields tie)
                        if (mine && rank <= r - 1 && r - 1 < rank + same) {
                            sh_selD = myD;
                            sh_selH = myH;
                        }
                    }
                    lds_barrier();
                    selD = sh_selD;
                    selH = sh_selH;
                    PHASE_MARK(4);
                    return true;
                }
                // ---- boundary bucket too large: narrow (or widen) the window
                need = r;
                if (clamp_bin) {
                    w.lo = sat_add(w.lo, (uint64_t)(kFine - 1) << w.sh);
                    w.sh = min(kMaxShift, w.sh + 8);
                } else if (w.sh > 0) {
                    w.lo = sat_add(w.lo, (uint64_t)bstar << w.sh);
                    w.sh = max(0, w.sh - 10);
                } else if (w.mode == 0) {
                    // more than kExactCap candidates share one score: order them by hash
                    w.Dfix = w.lo + (uint64_t)bstar;
                    w.mode = 1;
                    w.lo = 0;
                    w.sh = kMaxShift;
                } else {
                    // identical score and identical hash (collision): keep them all
                    selD = w.Dfix;
                    selH = w.lo + (uint64_t)bstar;
                    return true;
                }
                return false;
            };
            bool found = pass(std::true_type{});
            // (hinted in every build: the 1024-thread build is 6% faster per frame with it)
            for (int iter = 1; __builtin_expect(!found && iter < 40, 0); ++iter)
                found = pass(std::false_type{});
        }
        if (FLTOP_RARE(Dcut < selD)) {  // the score window is narrower than the top-`beam` cut
            selD = Dcut;
            selH = kAllOnes;
        }
        PHASE_MARK(3);

        // ---- compaction: selected candidates become the next beam ------------------
        {
            // the stay candidate and the first extension share one slot allocation per wave
            uint64_t hh0 = 0, hhs = 0;
            bool hv0 = false, hvs = false;
            const bool sel_s =
                D_stay != kAllOnes && is_selected(fc, selD, selH, D_stay, tid, -1, hhs, hvs);
            const bool sel_0 =
                cD0 != kAllOnes && is_selected(fc, selD, selH, cD0, cI0, cT0, hh0, hv0);
            // places inside the wavefront from two ballots (the selected stays first, then the
            // selected extensions): a handful of scalar and count instructions
            const uint64_t m_s = __ballot(sel_s), m_0 = __ballot(sel_0);
            const int n_s = __popcll(m_s);
            const int wave_total = n_s + __popcll(m_0);
            int base = 0;
            if (wave_total > 0) {
                if (lane == 0) base = atomicAdd(&sh_nnew, wave_total);
                base = __builtin_amdgcn_readfirstlane(base);
            }
            const int slot_s = base + lanes_below(m_s, lane);
            const int slot_0 = base + n_s + lanes_below(m_0, lane);
            PHASE_MARK(9);
            if (sel_s)
                emit_stay<MB, kPrefetchStay>(fc, nxt, lkn, ccur, cnxt, newslot, slot_s, beam, tid, my_pb,
                                             my_pnb, my_tot, sf);
            if (sel_0)
            {
                if constexpr (kPrefetchStay)
                    emit_ext_prefetched(fc, nxt, lkn, ccur, cnxt, slot_0, beam, t_base + t, cD0, cI0,
                                        cT0, hh0, hv0, trie, trie_stride, &xs0);
                else
                    emit_ext(fc, nxt, lkn, ccur, cnxt, slot_0, beam, t_base + t, cD0, cI0, cT0, hh0,
                             hv0, trie, trie_stride);
            }
        }
        for (int m = kRegCand; m < M; ++m) {  // candidates beyond the register cache
            int e, k;
            const bool there = cand_at(m, e, k);
            bool sel = false;
            int se = 0;
            int32_t tk = 0;
            uint64_t D = kAllOnes, hh = 0;
            bool have_h = false;
            if (there) {
                const int row = m - kRegCand;
                if (row < drows) {
                    D = dcache[row * kThreads];
                    if (D != kAllOnes && D <= selD) cand_name(e, k, se, tk);  // a contender
                } else {
                    D = cand_eval(e, k, se, tk);
                }
                if (D != kAllOnes && D <= selD)
                    sel = is_selected(fc, selD, selH, D, se, tk, hh, have_h);
            }
            const uint64_t m_sel = __ballot(sel);
            if (m_sel == 0) continue;
            int base = 0;
            if (lane == 0) base = atomicAdd(&sh_nnew, __popcll(m_sel));
            base = __builtin_amdgcn_readfirstlane(base);
            if (sel)
                emit_ext(fc, nxt, lkn, ccur, cnxt, base + lanes_below(m_sel, lane), beam, t_base + t,
                         D, se, tk, hh, have_h, trie, trie_stride);
        }
        // the links phase reads what other threads have just emitted: LDS always, and in
        // kColdGlobal builds their stores to global memory too
        if (kColdGlobal) __syncthreads();
        else lds_barrier();
        PHASE_MARK(5);

        // ---- adopt the new beam; rebuild parent / children links ---------------------
        int n_new = __builtin_amdgcn_readfirstlane(sh_nnew);  // the same in every lane
        if (FLTOP_RARE(n_new > beam)) {
            pd_drop += (uint32_t)(n_new - beam);
            n_new = beam;
        }
        pd_beam += (uint32_t)n_new;
        // A run of blank-only frames that follows inside this chunk is taken here: the thread
        // that owns a place of the new beam adds the run's log-probs to its total, one by one in
        // frame order, behind the barrier this frame ends on anyway.  (A run at the start of a
        // chunk or of the utterance takes the path at the top of the loop.)
        int run_after = 0;
        if (l + 1 < kChunk && n_new > 0)
            run_after = __builtin_ctz(~(blank_only >> (l + 1)) | 0x80000000u);
        double own_total = 0.0;  // of the entry this thread owns in the new beam (for the run)
        if (tid < n_new) {
            int p = -1;
            if constexpr (!kColdGlobal) {
                // Two LDS round trips: everything the entry's own fields can say, asked for
                // together; then ONE lookup, in the table of moves if the parent was in the old
                // beam (did it stay, and where), else in the hash table of the new prefixes
                // (a parent that was not in the beam can only have entered it just now).
                const int32_t code = lkn->par[tid];
                const int32_t depth = cnxt.plen(tid);
                const uint64_t want = cnxt.hp(tid);
                const int32_t tok_me = nxt->last[tid];
                own_total = nxt->ptot[tid];
                uint32_t hs = (uint32_t)want & (kHashSlots - 1);
                const int32_t* where = code >= 0 ? &newslot[code] : &lkn->ht[hs];
                int v = *where;
                if (code >= 0) {
                    p = v;
                } else if (depth > 0 && v >= 0) {  // rare: walk on until found or free
                    for (int probe = 0; probe < kHashSlots; ++probe) {
                        if (nxt->h[v] == want) {
                            p = v;
                            break;
                        }
                        hs = (hs + 1) & (kHashSlots - 1);
                        v = lkn->ht[hs];
                        if (v < 0) break;
                    }
                }
                lkn->par[tid] = p;
                if (p >= 0) {
                    if (kEntryMajor)
                        kidset_insert(kidset2[gen ^ 1], kKidSlots, p, tok_me);
                    else
                        lkn->next_kid[tid] = atomicExch(&lkn->first_kid[p], tid);
                    atomicOr(&lkn->kidmask[p], 1u << (tok_me & 31));
                }
            } else {
                const int32_t code = lkn->par[tid];
                if (code >= 0) {
                    p = newslot[code];  // the parent was in the old beam: did it stay, and where
                } else if (cnxt.plen(tid) > 0) {
                    const uint64_t want = cnxt.hp(tid);
                    uint32_t hs = (uint32_t)want & (kHashSlots - 1);
                    int v = lkn->ht[hs];
                    if (v >= 0) {  // rare: something hashes to this place; walk on until found or free
                        for (int probe = 0; probe < kHashSlots; ++probe) {
                            if (nxt->h[v] == want) {
                                p = v;
                                break;
                            }
                            hs = (hs + 1) & (kHashSlots - 1);
                            v = lkn->ht[hs];
                            if (v < 0) break;
                        }
                    }
                }
                lkn->par[tid] = p;
                if (p >= 0) {
                    if (kEntryMajor)
                        kidset_insert(kidset2[gen ^ 1], kKidSlots, p, nxt->last[tid]);
                    else
                        lkn->next_kid[tid] = atomicExch(&lkn->first_kid[p], tid);
                    atomicOr(&lkn->kidmask[p], 1u << (nxt->last[tid] & 31));
                }
            }
        }
        PHASE_MARK(10);
        // housekeeping behind this frame's last readers: the old generation's links
        // (next used as the new generation of the following frame) and the histogram.
        // The upper half of the threads does it: the lower half has just done the links.
        if (tid >= kThreads / 2) {
            // 16 bytes per store
            const int u = tid - kThreads / 2;
            const int4 ones = make_int4(-1, -1, -1, -1), zeros = make_int4(0, 0, 0, 0);
            // (trip counts known at compile time: straight-line stores, no loops)
            constexpr int kHalf = kThreads / 2;
            auto fill = [&](int4* dst, auto n_tag, const int4& v) {
                constexpr int n = decltype(n_tag)::value;  // 16-byte words to fill
#pragma unroll
                for (int j = 0; j < n / kHalf; ++j) dst[u + j * kHalf] = v;
                if (n % kHalf != 0 && u < n % kHalf) dst[u + (n / kHalf) * kHalf] = v;
            };
            fill(reinterpret_cast<int4*>(lk->ht), std::integral_constant<int, kHashSlots / 4>{}, ones);
            if (kEntryMajor)
                fill(reinterpret_cast<int4*>(kidset2[gen]), std::integral_constant<int, kKidSlots / 4>{},
                     ones);
            if (!kColdGlobal)
                fill(reinterpret_cast<int4*>(lk->first_kid), std::integral_constant<int, kMaxBeam / 4>{},
                     ones);
            fill(reinterpret_cast<int4*>(lk->kidmask), std::integral_constant<int, kMaxBeam / 4>{}, zeros);
            fill(reinterpret_cast<int4*>(hfine), std::integral_constant<int, kFine / 4>{}, zeros);
            if (u < kCoarse / 4) reinterpret_cast<int4*>(hcoarse)[u] = zeros;
        }
        if (tid == 0) {
            sh_minD = kAllOnes;
            if (a.frame_beam) a.frame_beam[trace_base + t] = n_new;
        }
        if (big)
            for (int k = tid; k < K; k += kThreads) dense_lp[s_tok[k]] = -INFINITY;
        if (n_new > 0) {
            kmax_v = key_value(kbest_key);
            // worst kept score: the selection threshold when there was one
            kmin_v = (selD != kAllOnes && selD <= Rk) ? key_value(Rk - selD)
                                                      : kmin_v + (double)hd.top - 4.0;
            if (!(kmin_v <= kmax_v)) kmin_v = kmax_v;
        }
        n_live = n_new;
        gen ^= 1;
        collapsed = run_after > 0;  // otherwise every entry carries its own p_b / p_nb
        if (run_after > 0) {
            double own = own_total;
            if (kColdGlobal && tid < n_new) own = nxt->ptot[tid];
            for (int k = 0; k < run_after; ++k) {
                const double x = (double)__int_as_float(__builtin_amdgcn_readlane(lp_bits, l + 1 + k));
                own += x;
                kmax_v += x;
                kmin_v += x;
            }
            if (tid < n_new) nxt->ptot[tid] = own;
            pd_cand += (uint32_t)(n_new * run_after);
            pd_peak = max(pd_peak, (uint32_t)n_new);
            pd_beam += (uint32_t)(n_new * run_after);
            if (a.frame_beam && tid < run_after) a.frame_beam[trace_base + t + 1 + tid] = n_new;
            t += run_after;
        }
        lds_barrier();
        PHASE_MARK(6);
    }  // frames of the chunk
    }  // chunks
#undef FLTOP_RARE
#undef FLTOP_USUAL
#undef FLTOP_LOAD_CHUNK
#undef FLTOP_RING_HEAD

    flush_stats();
    if (failed) n_live = 0;  // nothing to report, and a stream that carries on finds no beam
    // every trie store must have landed before the back-walk reads the nodes
    __threadfence_block();
    __syncthreads();

    // ---- best prefix (paper: GetHighestScorePrefix) ----------------------------------
    BeamSlab<MB>& fin = slab[gen];
    const ColdRef<MB> cfin{&slab[gen], kColdGlobal ? cold_gen + gen : nullptr};
    int32_t* wp_node = reinterpret_cast<int32_t*>(hfine);  // the histogram is idle now
    int32_t* wp_depth = wp_node + kWaypoints;
    static_assert(2 * kWaypoints <= kFine, "way-points alias the histogram");
    if (tid == 0) {
        sh_kbest = 0;
        sh_selH = kAllOnes;
        sh_best = -1;
    }
    __syncthreads();
    if (tid < n_live)
        atomicMax((unsigned long long*)&sh_kbest, (unsigned long long)order_key(fin.ptot[tid]));
    __syncthreads();
    if (tid < n_live && order_key(fin.ptot[tid]) == sh_kbest)
        atomicMin((unsigned long long*)&sh_selH, (unsigned long long)fin.h[tid]);
    __syncthreads();
    if (tid < n_live && order_key(fin.ptot[tid]) == sh_kbest && fin.h[tid] == sh_selH)
        sh_best = tid;
    __syncthreads();

    const int best = sh_best;
    if (tid == 0) {
        if (failed) {  // said loudly: no transcript, not an empty one
            a.out_lengths[b] = -1;
            a.out_scores[b] = __int_as_float(0x7fc00000);  // NaN
        } else if (best < 0) {
            a.out_lengths[b] = 0;
            a.out_scores[b] = -INFINITY;
        } else {
            a.out_lengths[b] = cfin.plen(best);
            a.out_scores[b] = (float)fin.ptot[best];
        }
        if (a.stats) {
            atomicAdd((unsigned long long*)&a.stats->frames, (unsigned long long)len);
            atomicAdd((unsigned long long*)&a.stats->sum_survivors, sh_stat[kStSurv]);
            atomicAdd((unsigned long long*)&a.stats->sum_candidates, sh_stat[kStCand]);
            atomicMax((unsigned long long*)&a.stats->peak_candidates, sh_stat[kStPeak]);
            atomicAdd((unsigned long long*)&a.stats->sum_beam, sh_stat[kStBeam]);
            atomicAdd((unsigned long long*)&a.stats->select_passes, sh_stat[kStPass]);
            atomicAdd((unsigned long long*)&a.stats->exact_rankings, sh_stat[kStExact]);
            atomicAdd((unsigned long long*)&a.stats->overflow_drops, sh_stat[kStDrop]);
            if (failed) atomicAdd((unsigned long long*)&a.stats->record_overflows, 1ull);
            atomicAdd((unsigned long long*)&a.stats->survivor_records, sh_stat[kStRecords]);
        }
    }
#ifdef FLTOP_PHASE_CLOCKS
    if (ph_rec && a.stats)
        for (int i = 0; i < 16; ++i)
            atomicAdd((unsigned long long*)&a.stats->phase_clocks[ph_grp * 16 + i],
                      (unsigned long long)ph_clk[i]);
#endif
    // Back-walk: thread 0 follows the every-8th-level links and records way-points; then
    // one thread per way-point walks the (at most 8) parents down to the next way-point.
    // A streaming decode remembers the trie node behind every token it wrote: where the walk
    // meets the node that is already written at that position, everything before it is in
    // place (a node's ancestors never change), so a call rewrites only what has changed.
    int32_t* const out_row = a.out_tokens + (int64_t)b * a.out_stride;
    int32_t* const born_row =
        a.out_token_frames ? a.out_token_frames + (int64_t)b * a.out_stride : nullptr;
    int32_t* const wrote = a.out_nodes ? a.out_nodes + (int64_t)b * a.out_stride : nullptr;
    const bool same_rows = wrote && prev_tokens_at == (uint64_t)(uintptr_t)out_row &&
                           prev_frames_at == (uint64_t)(uintptr_t)born_row;
    const int new_out_len = best >= 0 ? cfin.plen(best) : 0;
    if (best >= 0) {
        int node = cfin.node(best);
        int depth = new_out_len;
        while (depth > 0) {  // uniform: node/depth are re-read from LDS after each batch
            if (tid == 0) {
                int n = 0;
                int nd = node, dp = depth;
                bool met = false;
                while (dp > 0 && n < kWalkers - 1 && nd > 0 && (int64_t)nd < a.trie_stride) {
                    if (same_rows && wrote[dp - 1] == nd) {
                        met = true;
                        break;
                    }
                    wp_node[n] = nd;
                    wp_depth[n] = dp;
                    ++n;
                    const TrieNode tn = trie[nd];
                    nd = tn.xup;
                    dp = (dp - 1) & ~7;
                }
                const bool ok = !met && nd > 0 && (int64_t)nd < a.trie_stride;
                wp_node[n] = nd;             // where the next batch starts ...
                wp_depth[n] = met ? dp : (ok ? dp : 0);  // ... and the last walker stops
                sh_blcount = ok ? dp : 0;    // depth left for the next batch
                sh_nnew = n;
            }
            __syncthreads();
            const int n = sh_nnew;
            if (tid < n) {
                int nd = wp_node[tid];
                int dp = wp_depth[tid];
                const int stop = wp_depth[tid + 1];
                while (dp > stop && nd > 0 && (int64_t)nd < a.trie_stride) {
                    if (same_rows && wrote[dp - 1] == nd) break;
                    const TrieNode tn = trie[nd];
                    out_row[dp - 1] = tn.tok;
                    if (born_row) born_row[dp - 1] = (nd - 1) / beam;  // node id = 1 + frame * beam + slot
                    if (wrote) wrote[dp - 1] = nd;
                    nd = tn.parent;
                    --dp;
                }
            }
            node = wp_node[n];
            depth = sh_blcount;
            __syncthreads();
        }
    }
    if (wrote)  // positions the shorter transcript no longer covers
        for (int q = new_out_len + tid; q < prev_out_len; q += kThreads) wrote[q] = -1;

    // ---- optional: the whole final beam in rank order ---------------------------------
    if (a.nbest_count) {
        if (tid == 0) a.nbest_count[b] = n_live;
        if (tid < n_live) {
            const uint64_t myK = order_key(fin.ptot[tid]);
            const uint64_t myH = fin.h[tid];
            int rank = 0;
            for (int e = 0; e < n_live; ++e) {
                const uint64_t oK = order_key(fin.ptot[e]);
                const uint64_t oH = fin.h[e];
                rank += (oK > myK || (oK == myK && oH < myH)) ? 1 : 0;
            }
            const int64_t row = (int64_t)b * beam + rank;
            const int n = cfin.plen(tid);
            a.nbest_lengths[row] = n;
            a.nbest_pb[row] = collapsed ? fin.ptot[tid] : fin.pb[tid];
            a.nbest_pnb[row] = collapsed ? -INFINITY : fin.pnb[tid];
            int node = cfin.node(tid);
            int32_t* dst = a.nbest_tokens + row * a.out_stride;
            for (int p = n - 1; p >= 0 && node > 0 && (int64_t)node < a.trie_stride; --p) {
                const TrieNode tn = trie[node];
                dst[p] = tn.tok;
                node = tn.parent;
            }
        }
    }

    // ---- streaming: leave the beam for the next chunk -----------------------------------
    if (carried) {
        const uint32_t* src = reinterpret_cast<const uint32_t*>(&slab[gen]);
        uint32_t* dst = reinterpret_cast<uint32_t*>(&carried->slab);
        for (int i = tid; i < (int)(sizeof(BeamSlab<MB>) / 4); i += kThreads) dst[i] = src[i];
        const uint32_t* lsrc = reinterpret_cast<const uint32_t*>(&links[gen]);
        uint32_t* ldst = reinterpret_cast<uint32_t*>(carried->par);
        for (int i = tid; i < 4 * kMaxBeam; i += kThreads) ldst[i] = lsrc[i];
        if (tid == 0) {
            carried->frames_done = t_base + len;
            carried->out_len = new_out_len;
            carried->out_tokens_at = (uint64_t)(uintptr_t)out_row;
            carried->out_frames_at = (uint64_t)(uintptr_t)born_row;
            carried->n_live = n_live;
            carried->collapsed = collapsed ? 1 : 0;
            carried->kmax = kmax_v;
            carried->kmin = kmin_v;
        }
    }
}

// A fresh stream: the empty prefix with score 0, no links, no frames seen.
template <int MB>
__global__ __launch_bounds__(kThreadsSmall) void stream_begin_kernel(StreamState<MB>* st, int32_t B,
                                                                     int32_t* out_nodes,
                                                                     int64_t n_out_nodes) {
    constexpr int kThreads = kThreadsSmall;
    constexpr int kMaxBeam = MB;
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < n_out_nodes;
         i += (int64_t)gridDim.x * kThreads)
        out_nodes[i] = -1;
    for (int32_t b = blockIdx.x; b < B; b += gridDim.x) {
        StreamState<MB>* s = st + b;
        uint32_t* words = reinterpret_cast<uint32_t*>(s);
        for (int i = threadIdx.x; i < (int)(sizeof(StreamState<MB>) / 4); i += kThreads) words[i] = 0u;
        __syncthreads();
        for (int i = threadIdx.x; i < kMaxBeam; i += kThreads) {
            s->par[i] = -1;
            s->first_kid[i] = -1;
            s->next_kid[i] = -1;
        }
        if (threadIdx.x == 0) {
            s->n_live = 1;
            s->slab.h[0] = kGolden;
            s->slab.pb[0] = 0.0;
            s->slab.pnb[0] = -INFINITY;
            s->slab.ptot[0] = 0.0;
            s->slab.last[0] = -1;
        }
        __syncthreads();
    }
}

// The search stage's log-sum-exp, element-wise over two arrays (for checking its rounding).
__global__ __launch_bounds__(256) void log_add_kernel(const double* __restrict__ a,
                                                      const double* __restrict__ b,
                                                      double* __restrict__ out, int64_t n) {
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256)
        out[i] = lse2(a[i], b[i]);
}

}  // namespace

hipError_t launch_log_add(const double* a, const double* b, double* out, int64_t n,
                          hipStream_t stream) {
    if (n <= 0) return hipSuccess;
    const int64_t blocks = (n + 255) / 256;
    hipLaunchKernelGGL(log_add_kernel, dim3((unsigned)(blocks < 4096 ? blocks : 4096)), dim3(256),
                       0, stream, a, b, out, n);
    return hipGetLastError();
}

size_t stream_record_bytes(int32_t beam) {
    return beam <= kBeamSmall ? sizeof(StreamState<kBeamSmall>) : sizeof(StreamState<kBeamLarge>);
}

hipError_t launch_stream_begin(const StreamSpace& sp, int32_t B, int32_t beam, hipStream_t stream) {
    const dim3 grid((unsigned)(B < 1024 ? B : 1024));
    const int64_t n_out_nodes = (int64_t)B * sp.t_total;
    if (beam <= kBeamSmall)
        hipLaunchKernelGGL(stream_begin_kernel<kBeamSmall>, grid, dim3(kThreadsSmall), 0, stream,
                           static_cast<StreamState<kBeamSmall>*>(sp.records), B, sp.out_nodes,
                           n_out_nodes);
    else
        hipLaunchKernelGGL(stream_begin_kernel<kBeamLarge>, grid, dim3(kThreadsSmall), 0, stream,
                           static_cast<StreamState<kBeamLarge>*>(sp.records), B, sp.out_nodes,
                           n_out_nodes);
    return hipGetLastError();
}

// Compute units of the current device (asked once per device).
static hipError_t compute_units(int* n_cu) {
    constexpr int kMaxDevices = 64;
    static int cached[kMaxDevices] = {0};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev >= 0 && dev < kMaxDevices && cached[dev] > 0) {
        *n_cu = cached[dev];
        return hipSuccess;
    }
    int n = 0;
    e = hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev);
    if (e != hipSuccess) return e;
    if (n <= 0) n = 1;
    if (dev >= 0 && dev < kMaxDevices) cached[dev] = n;  // racing callers write the same value
    *n_cu = n;
    return hipSuccess;
}

hipError_t launch_beam(const int32_t* lengths, int32_t B, int32_t T, int32_t V,
                       const fltop_params& p, const Workspace& ws, const StreamSpace* carried,
                       int32_t* out_tokens, int32_t* out_lengths, float* out_scores,
                       fltop_stats* stats, hipStream_t stream) {
    BeamArgs a;
    a.lengths = lengths;
    a.hdr = ws.hdr;
    a.rec = ws.rec;
    a.trie = carried ? carried->trie : ws.trie;
    a.trie_stride = carried ? carried->trie_stride : ws.trie_stride;
    a.cold = ws.cold;
    a.stream = carried ? carried->records : nullptr;
    a.out_nodes = carried ? carried->out_nodes : nullptr;
    a.t_total = carried ? carried->t_total : T;
    a.out_stride = carried ? carried->t_total : T;
    a.lm_table = p.lm_table;
    a.lm_bound = ws.lm_bound;
    a.lm_alpha = (double)p.lm_weight;
    a.lm_beta = (double)p.insertion_bonus;
    a.beam_window = p.beam_threshold;
    a.frame_beam = p.frame_beam;
    a.out_token_frames = p.out_token_frames;
    a.B = B;
    a.T = T;
    a.V = V;
    a.beam = p.beam;
    a.lm_in_lds = (p.lm_table != nullptr && (size_t)V * V * sizeof(float) <= 16384) ? 1 : 0;
    a.out_tokens = out_tokens;
    a.out_lengths = out_lengths;
    a.out_scores = out_scores;
    a.stats = stats;
    a.nbest_count = p.nbest_count;
    a.nbest_tokens = p.nbest_tokens;
    a.nbest_lengths = p.nbest_lengths;
    a.nbest_pb = p.nbest_pb;
    a.nbest_pnb = p.nbest_pnb;
    // "wide" = frames are expected to hold hundreds of candidates or more: a large vocabulary,
    // or a search that is known to keep every token (R = 0) of a small one with a beam to
    // match (measured on V = 32: from 512 candidates per frame on, the 512-thread build is
    // 9-41% faster; how many tokens a threshold R > 0 keeps is not known here)
    const int kept_at_most = p.top_n > 0 && p.top_n < V ? p.top_n : V;
    const bool wide =
        V > 64 || (p.rel_threshold == 0.0f && (int64_t)p.beam * kept_at_most >= 512);
    const bool large_beam = p.beam > kBeamSmall;
    const bool huge_beam = p.beam > kBeamLarge;  // 1024-entry build, 1024 threads, one per CU
    if (huge_beam && (carried != nullptr || V > FLTOP_MAX_VOCAB_WIDE_BEAM))
        return hipErrorInvalidValue;  // the entry points refuse these before they get here
    int n_cu = 0;
    hipError_t qe = compute_units(&n_cu);
    if (qe != hipSuccess) return qe;
    const bool dense = (int64_t)B > (int64_t)n_cu * (wide ? 1 : 2);
    const bool very_dense = (int64_t)B > (int64_t)n_cu * 2;
    const bool threads_512 = large_beam || (wide && !very_dense);  // as dispatched below
    size_t dyn = lm_lds_offset(V, threads_512);
    if (a.lm_in_lds) dyn += (size_t)V * V * sizeof(float);
    dyn = (dyn + 15) / 16 * 16;
    a.dcache_off = (int32_t)dyn;
    a.dcache_rows = 0;
    // Workgroup size: frames of a small vocabulary have a few dozen candidates, and the cost of
    // a frame is its barriers and its longest wavefront, so four wavefronts are best; a large
    // vocabulary leaves hundreds to thousands of candidates per frame, which eight wavefronts
    // (two per SIMD) evaluate twice as fast (measured: V = 1024 27% faster per decode with 512
    // threads, V = 32 at r = 0.01 6% slower).
    // Beam capacity: up to 128 entries the beam state takes 30 KB of LDS; beyond, the
    // 512-entry build (116 KB, one thread per entry, one workgroup per CU) is used, and beyond
    // that the 1024-entry build (1024 threads, 134 KB, part of the state in global memory).
    // Residency: at two wavefronts per SIMD a CU holds two 256-thread workgroups (one of 512
    // threads).  A batch with more utterances than that over the whole chip is bound by
    // instruction issue, not by one frame's latency, and small frames then run best as two
    // wavefronts per utterance (one for the stays, one for the extensions: the other two of
    // the four mostly repeat wave-uniform bookkeeping), with registers cut for three
    // wavefronts per SIMD and, where a one-shot decode's beam allows, the 64-entry state
    // (17 KB of LDS) so that more workgroups fit a CU.  Measured on B = 4096, V = 32,
    // beam 32: 287 M frames/s with the four-wavefront build alone, 470 M with its registers
    // cut for four wavefronts per SIMD, 564 M with two wavefronts per utterance, 679 M with
    // the small state as well.  A streaming decode keeps the 128-entry state throughout (its
    // carried records are laid out for it).
    // (large vocabulary: eight wavefronts per utterance while the whole batch is resident that
    // way, two workgroups per CU, four beyond: B = 1024, V = 1024: 143 M frames/s against
    // 120 M; B = 512: 93 M against 111 M)
    const bool tiny_state = p.beam <= kBeamTiny && carried == nullptr;
    // Distance cache: rows for the candidates beyond the one a thread keeps in registers.  A
    // batch that leaves LDS to spare (at most two workgroups per CU) gets 48 KB with 512
    // threads (frames of up to 6656 candidates are evaluated once) or 16 KB with 256; the
    // builds for large batches get one row (1-4 KB: up to two candidates per thread).
    if (!large_beam) {
        const int threads = threads_512 ? kThreadsLarge
                                        : (wide || !dense ? kThreadsSmall : kThreadsDense);
        a.dcache_rows = dense ? 1 : (wide ? 12 : 8);
        dyn += (size_t)a.dcache_rows * threads * sizeof(uint64_t);
    }
#define FLTOP_LAUNCH_BEAM(LM_)                                                               \
    do {                                                                                     \
        if (huge_beam)                                                                       \
            hipLaunchKernelGGL((beam_kernel<LM_, kThreadsHuge, kBeamHuge, 4>),               \
                               dim3((unsigned)B), dim3(kThreadsHuge), dyn, stream, a);       \
        else if (large_beam)                                                                 \
            hipLaunchKernelGGL((beam_kernel<LM_, kThreadsLarge, kBeamLarge, 2>),             \
                               dim3((unsigned)B), dim3(kThreadsLarge), dyn, stream, a);      \
        else if (wide && very_dense)                                                         \
            hipLaunchKernelGGL((beam_kernel<LM_, kThreadsSmall, kBeamSmall, 4>),             \
                               dim3((unsigned)B), dim3(kThreadsSmall), dyn, stream, a);      \
        else if (wide && dense)                                                              \
            hipLaunchKernelGGL((beam_kernel<LM_, kThreadsLarge, kBeamSmall, 4>),             \
                               dim3((unsigned)B), dim3(kThreadsLarge), dyn, stream, a);      \
        else if (wide)                                                                       \
            hipLaunchKernelGGL((beam_kernel<LM_, kThreadsLarge, kBeamSmall, 2>),             \
                               dim3((unsigned)B), dim3(kThreadsLarge), dyn, stream, a);      \
        else if (dense && tiny_state)                                                        \
            hipLaunchKernelGGL((beam_kernel<LM_, kThreadsDense, kBeamTiny, 3>),              \
                               dim3((unsigned)B), dim3(kThreadsDense), dyn, stream, a);      \
        else if (dense)                                                                      \
            hipLaunchKernelGGL((beam_kernel<LM_, kThreadsDense, kBeamSmall, 3>),             \
                               dim3((unsigned)B), dim3(kThreadsDense), dyn, stream, a);      \
        else                                                                                 \
            hipLaunchKernelGGL((beam_kernel<LM_, kThreadsSmall, kBeamSmall, 2>),             \
                               dim3((unsigned)B), dim3(kThreadsSmall), dyn, stream, a);      \
    } while (0)
    if (p.lm_table == nullptr)
        FLTOP_LAUNCH_BEAM(kLmNone);
    else if (a.lm_in_lds)
        FLTOP_LAUNCH_BEAM(kLmLds);
    else
        FLTOP_LAUNCH_BEAM(kLmGlobal);
#undef FLTOP_LAUNCH_BEAM
    return hipGetLastError();
}

}  // namespace fltop
