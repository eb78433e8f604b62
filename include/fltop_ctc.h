/*
 * fltop_ctc.h -- C ABI of the FLToP CTC decoder for AMD MI355X (gfx950).
 *
 * What is computed (paper: "FLToP CTC", Sec. 3, Algorithm 1): CTC prefix beam
 * search in which, at every frame, only the tokens whose probability is at
 * least R times the frame's top probability are expanded.  Per utterance:
 *
 *   beam <- { (empty prefix, score 0) }
 *   for each frame t < length:
 *       S_t  <- { v : lp[t][v] >= max_v lp[t][v] + ln R }      (relative threshold)
 *               restricted, if N is given, to the N best tokens of the frame
 *               (PartialSortDesc; equal emissions in ascending token order)
 *       expand every beam entry by every token of S_t           (blank / repeat / extend)
 *       merge equal prefixes (log-sum-exp),
 *       drop what scores more than beam_threshold below the frame's best candidate
 *       (if that window is given), keep the best `beam`         (SelectTopK)
 *   return the best prefix                                      (GetHighestScorePrefix)
 *
 * Algorithm 1 leaves the CTC collapse abstract ("prefix + token", "score +
 * logit"); this library uses the standard two-mass form: a prefix carries
 * p_b (log-mass of its alignments ending in blank) and p_nb (ending in its last
 * token); blank feeds p_b of the same prefix, a repeat of the last token feeds
 * p_nb of the same prefix and -- from p_b only -- the prefix extended by that
 * token, any other token extends from p_b (+) p_nb.  A prefix's score is
 * LSE(p_b, p_nb).  The optional LM term of Algorithm 1 (score' += LM(prefix'))
 * is a dense bigram table applied once per emitted token.
 *
 * All decoding arithmetic on scores is fp64; the threshold test is one fp32
 * addition and fp32 comparisons.  Score ties are ordered by a 64-bit prefix
 * hash: h(empty) = 0x9E3779B97F4A7C15, h(p + c) = mix(h(p) + 0x9E3779B97F4A7C15
 * * (c + 1)), mix = the splitmix64 output function; smaller hash wins.  Equal
 * prefixes are recognised by this hash.
 *
 * Conventions: "dev" = device (HBM) pointer, "host" = host pointer.  Arrays are
 * row-major and densely packed.  The caller owns every buffer; the library
 * allocates nothing, keeps no decoding state between calls (it only remembers, per
 * device, constants such as the number of compute units) and may be called
 * concurrently on different streams with different workspaces.  All work is
 * enqueued on `stream` as kernel launches only (so a call may be captured in a HIP
 * graph); no entry point synchronises with the host, so outputs are valid once the
 * stream has reached that point.  Every function that
 * returns int returns FLTOP_OK (0) or a negative FLTOP_ERR_* value; on an
 * error nothing has been enqueued.  There is no CPU fallback.
 */
#ifndef FLTOP_CTC_H_
#define FLTOP_CTC_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define FLTOP_OK                  0
#define FLTOP_ERR_NULL_POINTER   -1  /* a required pointer is NULL                          */
#define FLTOP_ERR_BAD_SHAPE      -2  /* B < 1, T < 1, V < 2, or T * beam >= 2^31            */
#define FLTOP_ERR_BAD_BEAM       -3  /* beam < 1 or > FLTOP_MAX_BEAM; or beam > 512 together
                                        with V > FLTOP_MAX_VOCAB_WIDE_BEAM or with streaming */
#define FLTOP_ERR_BAD_THRESHOLD  -4  /* rel_threshold outside [0, 1] or NaN                 */
#define FLTOP_ERR_WORKSPACE      -5  /* workspace smaller than fltop_ctc_workspace_bytes_for(
                                        ..., 0)                                             */
#define FLTOP_ERR_VOCAB_TOO_BIG  -6  /* V > FLTOP_MAX_VOCAB                                 */
#define FLTOP_ERR_HIP            -7  /* a HIP call or kernel launch failed                  */
#define FLTOP_ERR_ALIGNMENT      -8  /* workspace not 256-byte aligned                      */
#define FLTOP_ERR_BAD_OPTION     -9  /* top_n < 0, or beam_threshold NaN                    */
#define FLTOP_ERR_STATIC_SCRATCH -10 /* fltop_ctc_decode_static: the shapes need more than
                                        FLTOP_STATIC_SCRATCH_BYTES of workspace             */

#define FLTOP_MAX_BEAM   1024  /* the paper's decoder runs beam-size 1000 (Sec. 4)            */
#define FLTOP_MAX_VOCAB  4096
/* A beam of more than 512 entries fills the compute unit's local memory: such a decode takes
 * vocabularies up to FLTOP_MAX_VOCAB_WIDE_BEAM only, and the streaming entry points take beams
 * up to 512. */
#define FLTOP_MAX_VOCAB_WIDE_BEAM 2048

/* Decoder settings (host POD, read during the call only; zero-initialise it, then set
 * what is needed).  Algorithm 1's arguments: beam_size -> beam, R -> rel_threshold,
 * N -> top_n, beam_threshold -> beam_threshold, LM -> the three lm fields. */
typedef struct fltop_params {
    int32_t      beam;             /* 1 .. FLTOP_MAX_BEAM                                       */
    float        rel_threshold;    /* R in [0,1]; 0 keeps every token (unpruned search)         */
    int32_t      top_n;            /* N: only the N best tokens of a frame take the threshold
                                      test; 0 (or >= V) = all tokens                            */
    int32_t      reserved;         /* set to 0                                                  */
    double       beam_threshold;   /* SelectTopK's score window: candidates scoring more than
                                      this below the frame's best candidate are dropped before
                                      the top-`beam` cut; <= 0 = no window                      */
    const float* lm_table;         /* dev [V,V] fp32 log-probs, row = previous token (row 0 for
                                      the first token of a prefix), or NULL for no LM           */
    float        lm_weight;        /* extension adds lm_weight * lm_table[prev][tok]            */
    float        insertion_bonus;  /*                + insertion_bonus   (only if lm_table)     */
    /* Optional export of the whole final beam in rank order (all NULL to skip).               */
    int32_t*     nbest_count;      /* dev [B]          entries written for utterance b          */
    int32_t*     nbest_tokens;     /* dev [B,beam,T]   entry e of b: first nbest_lengths tokens */
    int32_t*     nbest_lengths;    /* dev [B,beam]                                              */
    double*      nbest_pb;         /* dev [B,beam]     log-mass ending in blank                 */
    double*      nbest_pnb;        /* dev [B,beam]     log-mass ending in the last token        */
    /* Optional statistics traces (paper Sec. 4.1 and 4.4; each NULL to skip).                 */
    int32_t*     frame_beam;       /* dev [B,T]  beam entries kept after frame t (valid frames
                                      only, rest untouched): hypotheses per time step           */
    int32_t*     out_token_frames; /* dev [B,T]  for token i of the returned prefix, the frame at
                                      which the prefix of length i+1 entered the beam           */
} fltop_params;

/* Counters accumulated (added to) by fltop_ctc_decode; zero them beforehand. */
typedef struct fltop_stats {
    uint64_t frames;            /* valid frames decoded                                        */
    uint64_t sum_survivors;     /* sum over frames of |S_t|                                    */
    uint64_t sum_candidates;    /* sum over frames of distinct live candidate prefixes         */
    uint64_t peak_candidates;   /* max over frames (and utterances) of the same                */
    uint64_t sum_beam;          /* sum over frames of entries kept by SelectTopK               */
    uint64_t select_passes;     /* diagnostic: histogram passes of the top-`beam` selection    */
    uint64_t exact_rankings;    /* diagnostic: selections that needed the exact (score, hash)
                                   ranking                                                     */
    uint64_t overflow_drops;    /* entries dropped because a hash collision overfilled a beam
                                   (0 unless two different prefixes share a 64-bit hash)       */
    uint64_t survivor_records;  /* records the survivor lists asked for: the max_records this
                                   input needs (fltop_ctc_workspace_bytes_for)                 */
    uint64_t record_overflows;  /* utterances not decoded because a frame's survivor records
                                   did not fit the workspace (their out_lengths are -1)        */
#ifdef FLTOP_PHASE_CLOCKS
    uint64_t phase_clocks[64];  /* profiling builds only (library AND caller compiled with
                                   -DFLTOP_PHASE_CLOCKS): shader-clock cycles per phase of the
                                   search stage, [wavefront group 0..3][phase 0..15], summed
                                   over workgroups                                             */
#endif
} fltop_stats;

/* Bytes of device workspace that are enough for these shapes whatever the emissions and the
 * threshold are (0 if the shapes are invalid).  Holds the per-frame survivor lists and the
 * prefix trie. */
size_t fltop_ctc_workspace_bytes(int32_t B, int32_t T, int32_t V, int32_t beam);

/* The same for a caller who knows how little the pruning leaves (the method's memory saving,
 * paper Sec. 4.4): a frame keeps its first six survivors in a fixed 64-byte header and every
 * further one in an 8-byte record, and this workspace has room for `max_records` records in
 * all.  Every entry point accepts any workspace of at least
 * fltop_ctc_workspace_bytes_for(B, T, V, beam, 0) bytes and uses what lies beyond the fixed
 * regions for records (never more than the shapes can need: B * T * (V - 6)).  If the
 * survivor lists of a call ask for more, nothing is written out of bounds: the utterances
 * that meet a frame whose records did not fit are not decoded -- out_lengths[b] = -1,
 * out_scores[b] = NaN, stats->record_overflows counts them -- and the caller retries with
 * a larger workspace (stats->survivor_records says how many records the call asked for).
 * fltop_ctc_workspace_bytes(...) is this function at max_records = B * T * (V - 6). */
size_t fltop_ctc_workspace_bytes_for(int32_t B, int32_t T, int32_t V, int32_t beam,
                                     uint64_t max_records);

/* The whole path: survivor lists for all valid frames, then the beam search,
 * then the best prefix of every utterance.
 *   logprobs     dev [B,T,V] fp32 log-probabilities, token 0 = blank.  -inf is
 *                allowed; NaN is undefined.  Rows need not be normalised.
 *   lengths      dev [B] int32; values are clamped to [0,T]; frames at or
 *                beyond lengths[b] are never read.
 *   workspace    dev, 256-byte aligned, >= fltop_ctc_workspace_bytes_for(B,T,V,beam,0); with
 *                fltop_ctc_workspace_bytes(B,T,V,beam) bytes no input can overflow it.
 *   out_tokens   dev [B,T] int32; row b holds out_lengths[b] tokens (rest untouched).
 *   out_lengths  dev [B] int32 (-1: not decoded, the workspace was too small for the
 *                utterance's survivor lists).
 *   out_scores   dev [B] fp32: LSE(p_b,p_nb) of the returned prefix, rounded
 *                from fp64.  A zero-length utterance returns the empty prefix
 *                with score 0; an utterance whose every route has zero mass
 *                returns the empty prefix with score -inf.
 *   stats        dev or NULL.
 */
int fltop_ctc_decode(const float* logprobs, const int32_t* lengths,
                     int32_t B, int32_t T, int32_t V, const fltop_params* params,
                     void* workspace, size_t workspace_bytes,
                     int32_t* out_tokens, int32_t* out_lengths, float* out_scores,
                     fltop_stats* stats, void* hip_stream);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving
 * loops, harnesses that forbid it): fltop_ctc_decode without the workspace arguments.  The
 * survivor lists and the prefix trie go into an array of FLTOP_STATIC_SCRATCH_BYTES that is
 * part of the library's device image (every GPU the library runs on holds its own copy until
 * the process ends); the call allocates and frees nothing.  Inputs, outputs, argument rules
 * and results are those of fltop_ctc_decode with a workspace of that size: shapes whose fixed
 * regions alone (fltop_ctc_workspace_bytes_for(B, T, V, beam, 0)) exceed it are refused with
 * FLTOP_ERR_STATIC_SCRATCH before anything is enqueued; survivor records take the rest of the
 * array, and a call whose survivor lists ask for more reports the utterances concerned as
 * fltop_ctc_workspace_bytes_for describes.  All calls on one GPU share the one array,
 * whatever their stream: calls that overlap in time on one GPU race, so order them (one
 * stream, or events).  Nothing in the array has to be cleared between calls: each call writes
 * what it later reads. */
#define FLTOP_STATIC_SCRATCH_BYTES (64u << 20)
int fltop_ctc_decode_static(const float* logprobs, const int32_t* lengths,
                            int32_t B, int32_t T, int32_t V, const fltop_params* params,
                            int32_t* out_tokens, int32_t* out_lengths, float* out_scores,
                            fltop_stats* stats, void* hip_stream);

/* The first stage alone (Algorithm 1's top-emission lookup and relative-
 * threshold test, which do not depend on the hypotheses, for every valid frame
 * at once, preceded by the static top-N stage when top_n > 0): writes the
 * survivor lists into `workspace` in the library's internal layout.  Same
 * argument rules as fltop_ctc_decode (`beam` only sizes the workspace check). */
int fltop_ctc_prune(const float* logprobs, const int32_t* lengths,
                    int32_t B, int32_t T, int32_t V, int32_t beam, float rel_threshold,
                    int32_t top_n, void* workspace, size_t workspace_bytes, void* hip_stream);

/* The second stage alone (Algorithm 1's loop over beam entries and kept tokens,
 * SelectTopK and GetHighestScorePrefix) over survivor lists that fltop_ctc_prune
 * left in `workspace` for the same logprobs, lengths, shapes and beam.
 * fltop_ctc_decode is exactly fltop_ctc_prune followed by this call; the split
 * exists so that each stage can be timed and tested by itself.  Argument rules as
 * for fltop_ctc_decode; params->rel_threshold and params->top_n are not used here. */
int fltop_ctc_search(const int32_t* lengths, int32_t B, int32_t T, int32_t V,
                     const fltop_params* params, void* workspace, size_t workspace_bytes,
                     int32_t* out_tokens, int32_t* out_lengths, float* out_scores,
                     fltop_stats* stats, void* hip_stream);

/* Copy the survivor lists fltop_ctc_prune left in `workspace` into plain
 * arrays (for inspection and tests): counts dev [B*T] int32 (0 for frames at or
 * beyond lengths[b]), tokens dev [B*T,V] int32 and values dev [B*T,V] fp32
 * (first counts[f] entries of row f, ascending token id, rest untouched),
 * frame_max dev [B*T] fp32 (NULL to skip).  `lengths` as given to
 * fltop_ctc_prune. */
int fltop_ctc_unpack_survivors(const void* workspace, size_t workspace_bytes,
                               const int32_t* lengths, int32_t B, int32_t T, int32_t V,
                               int32_t beam, int32_t* counts, int32_t* tokens, float* values,
                               float* frame_max, void* hip_stream);

/* Streaming (chunked) decoding: the emissions of an utterance arrive in pieces and the beam
 * is carried from call to call, so that partial transcripts are available while audio is
 * still coming in (the real-time use the paper's Sec. 1 aims at).  Decoding T_total frames
 * in chunks gives exactly what fltop_ctc_decode gives on the whole utterance.
 *
 *   state    dev, 256-byte aligned, >= fltop_ctc_stream_state_bytes(B, T_total, beam): per
 *            utterance the carried beam, then the prefix trie for up to T_total frames,
 *            then a note of which prefix stands behind every transcript token written so
 *            far.  Caller-owned; one state per batch of streams; the same B and beam in
 *            every call.
 *   fltop_ctc_stream_begin   resets every stream of the batch to the empty prefix.
 *   fltop_ctc_stream_decode  consumes the next chunk: logprobs dev [B,T_chunk,V], lengths
 *            dev [B] = valid frames of this chunk per stream (0 for a stream that has
 *            ended; frames beyond T_total in all are ignored); workspace sized by
 *            fltop_ctc_workspace_bytes(B, T_chunk, V, beam).  Outputs as for
 *            fltop_ctc_decode but for everything decoded so far: out_tokens dev
 *            [B,T_total]; the traces and the n-best token rows of params, if given, are
 *            [B,T_total] / [B,beam,T_total] and indexed by the frame number since the
 *            stream began.  stats count this chunk only.
 *            While out_tokens (and params->out_token_frames) stay the same buffers from
 *            call to call, with their contents left alone, a call rewrites only the part of
 *            a transcript that has changed, so its cost does not grow with the transcript;
 *            other buffers are noticed and written in full.
 * Calls on one state must be ordered (same stream, or synchronised by the caller). */
size_t fltop_ctc_stream_state_bytes(int32_t B, int32_t T_total, int32_t beam);
int fltop_ctc_stream_begin(void* state, size_t state_bytes, int32_t B, int32_t T_total,
                           int32_t beam, void* hip_stream);
int fltop_ctc_stream_decode(const float* logprobs, const int32_t* lengths,
                            int32_t B, int32_t T_chunk, int32_t V, const fltop_params* params,
                            void* workspace, size_t workspace_bytes,
                            void* state, size_t state_bytes, int32_t T_total,
                            int32_t* out_tokens, int32_t* out_lengths, float* out_scores,
                            fltop_stats* stats, void* hip_stream);

/* "Index of the chosen token" statistic (paper Sec. 4.1): for every token i of the
 * returned prefixes, its position in the descending sort of the emissions of the frame
 * out_token_frames[b][i] (0 = top emission; equal emissions in ascending token order).
 *   tokens, token_frames  dev [B,T] as written by fltop_ctc_decode (out_tokens and
 *                         params->out_token_frames), token_counts dev [B] (out_lengths)
 *   out_ranks   dev [B,T] int32, first token_counts[b] entries of row b, or NULL
 *   rank_count  dev [V] uint64, rank_count[k] += tokens chosen at position k, or NULL
 *   rank_lp_sum dev [V] fp64,   rank_lp_sum[k] += their log-probabilities (the order of
 *               the additions is not fixed), or NULL; zero both beforehand. */
int fltop_ctc_token_ranks(const float* logprobs, int32_t B, int32_t T, int32_t V,
                          const int32_t* tokens, const int32_t* token_frames,
                          const int32_t* token_counts, int32_t* out_ranks,
                          uint64_t* rank_count, double* rank_lp_sum, void* hip_stream);

/* The two-operand log-sum-exp with which the search stage merges the masses of equal
 * prefixes (Algorithm 1's set insert B'.add) and forms a prefix's score, LSE(a,b) = max + log1p(
 * exp(min - max)) in fp64 with -inf as the neutral element, applied element-wise to dev
 * arrays of n values: exposed so that its rounding can be checked against a reference
 * (it is written out for the narrow argument ranges that occur, not taken from the math
 * library: the log1p(exp(.)) term is within 2.5 ulp of its exact value, to which the final
 * addition adds its half ulp). */
int fltop_ctc_log_add(const double* a, const double* b, double* out, int64_t n,
                      void* hip_stream);

/* Human-readable name of a status code (static storage). */
const char* fltop_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* FLTOP_CTC_H_ */
