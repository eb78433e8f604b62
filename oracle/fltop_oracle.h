/*
 * CPU oracle for FLToP CTC decoding -- TEST INFRASTRUCTURE, not a product path.
 *
 * A plain, slow, fp64 prefix beam search that follows the paper's Algorithm 1
 * (Sec. 3) step by step: per frame take the top emission, keep the tokens whose
 * probability is at least R times the top one, expand every beam entry by every
 * kept token, merge equal prefixes, keep the best `beam`, and return the best
 * prefix after the last frame.  Algorithm 1 writes "prefix + token" and
 * "score + logit" abstractly; the CTC collapse is made concrete here in the
 * usual way: each prefix carries two log-masses (alignments ending in blank,
 * p_b, and ending in its last token, p_nb), equal prefixes are merged by
 * log-sum-exp, and a prefix's score is LSE(p_b, p_nb).
 *
 * Only tests, the smoke check and the benchmark's CPU-baseline leg may call
 * this library.  It shares no source with the HIP decoder.
 *
 * Parity pins (tests marked "not gpu"): exhaustive alignment enumeration on
 * tiny inputs (pruned and unpruned, with and without LM), torch's ctc_loss as a
 * closed form for the per-prefix mass, r = 0 against the separately written
 * unpruned routine below, greedy collapse on one-hot rows, beam = 1 / r = 1
 * against the arg-max path, and the subset / arg-max invariants of the
 * survivor sets.  Unpinned: that this search reproduces the paper's WER and
 * timing figures on real speech (dataset, encoder and LM are not available).
 *
 * All pointers are host pointers.  Layouts are row-major.
 */
#ifndef FLTOP_ORACLE_H_
#define FLTOP_ORACLE_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct fltop_oracle_stats {
    int64_t frames;           /* valid frames decoded                                      */
    int64_t sum_survivors;    /* sum over frames of |S_t|                                  */
    int64_t sum_candidates;   /* sum over frames of distinct live candidate prefixes       */
    int64_t peak_candidates;  /* max over frames of the same                               */
    int64_t sum_beam;         /* sum over frames of entries kept after the top-`beam` cut  */
    int64_t max_addends;      /* most terms ever log-summed into one p_b or p_nb           */
    int64_t hash_collisions;  /* distinct candidate prefixes of one frame sharing a hash   */
    double  min_cut_margin;   /* min over frames of score[beam-1] - score[beam]            */
    double  min_decision_margin; /* smallest score gap that decided anything: a beam cut, the
                                    window floor (nearest candidate on either side), the final
                                    choice of the best prefix; 0 = an exact tie that the hash
                                    order resolved; +inf = nothing was ever cut              */
} fltop_oracle_stats;

/* Variant selector for the decode entry points. */
#define FLTOP_ORACLE_FLTOP     0  /* Algorithm 1 with the relative-threshold test        */
#define FLTOP_ORACLE_TEXTBOOK  1  /* separately written classic search, every token kept */

/* 64-bit prefix hash used only to order exactly tied scores:
 * h(empty) = 0x9E3779B97F4A7C15, h(p + c) = mix(h(p) + 0x9E3779B97F4A7C15 * (c + 1)),
 * mix = the splitmix64 output function. */
uint64_t fltop_oracle_prefix_hash(const int32_t* tokens, int32_t n);

/* Per-frame survivor sets (Alg. 1, the relative-threshold test, read in the
 * probability domain): token v survives iff lp[v] >= max_v lp[v] + ln(r), the
 * sum taken as one fp32 addition of fp32 operands, ln(r) rounded to fp32 once
 * (r = 0 gives -inf).  With top_n > 0 only the N best tokens of the frame (Alg. 1's
 * partial sort; equal emissions ordered by ascending token id) take the test at all.
 * counts[f] = |S_f|; tokens[f*V .. f*V+counts[f]) ascending; frame_max[f] = the top
 * emission.  Returns 0, or -1 on bad arguments. */
int fltop_oracle_survivors(const float* logprobs, int64_t n_frames, int32_t V,
                           float rel_threshold, int32_t top_n, int32_t* counts,
                           int32_t* tokens, float* frame_max);

/* Batch decode, best prefix per utterance.
 *  logprobs [B,T,V] fp32, lengths [B] (frames >= lengths[b] are never read),
 *  top_n: Alg. 1's N (0 = all tokens), beam_threshold: SelectTopK's score window --
 *  candidates scoring more than this below the frame's best one are dropped before the
 *  top-`beam` cut (<= 0 = no window),
 *  lm_table NULL or [V,V] fp32 log-probs (row = previous token, row 0 for the
 *  first token; applied as lm_weight*table + insertion_bonus on every extension),
 *  out_tokens [B,T], out_lengths [B], out_scores [B] (fp64),
 *  out_token_frames NULL or [B,T]: for token i of the best prefix, the frame at which
 *  the prefix of length i+1 entered the beam (on the lineage of the final entry),
 *  frame_beam NULL or [B,T]: number of beam entries kept after each frame,
 *  out_margins NULL or [B]: min_decision_margin (see the stats) of each utterance by itself,
 *  stats NULL or one struct accumulated over the batch, n_threads >= 1.
 * The TEXTBOOK variant takes neither top_n, beam_threshold nor the two traces.
 * Returns 0, or -1 on bad arguments. */
int fltop_oracle_decode(const float* logprobs, const int32_t* lengths,
                        int32_t B, int32_t T, int32_t V, int32_t beam,
                        float rel_threshold, int32_t top_n, double beam_threshold,
                        const float* lm_table, float lm_weight, float insertion_bonus,
                        int32_t variant, int32_t* out_tokens, int32_t* out_lengths,
                        double* out_scores, int32_t* out_token_frames, int32_t* frame_beam,
                        double* out_margins, fltop_oracle_stats* stats, int32_t n_threads);

/* Single utterance, whole final beam in rank order (score desc, hash asc).
 *  logprobs [T,V]; beam_tokens [max_entries, T]; beam_lengths, beam_pb, beam_pnb
 *  [max_entries].  Returns the number of entries written (<= max_entries), or
 *  -1 on bad arguments. */
int fltop_oracle_decode_beam(const float* logprobs, int32_t T, int32_t V, int32_t beam,
                             float rel_threshold, int32_t top_n, double beam_threshold,
                             const float* lm_table,
                             float lm_weight, float insertion_bonus, int32_t variant,
                             int32_t max_entries, int32_t* beam_tokens,
                             int32_t* beam_lengths, double* beam_pb, double* beam_pnb);

/* Position of tokens[i] in the descending sort of frame frames[i] of one [T,V] utterance
 * (0 = the top emission; equal emissions by ascending token id): the "index of the chosen
 * token" statistic of the paper's Sec. 4.1.  Returns 0, or -1 on bad arguments. */
int fltop_oracle_token_ranks(const float* logprobs, int32_t T, int32_t V,
                             const int32_t* tokens, const int32_t* frames, int32_t n,
                             int32_t* ranks);

#ifdef __cplusplus
}
#endif
#endif /* FLTOP_ORACLE_H_ */
