/*
 * CPU oracle for FLToP CTC decoding -- TEST INFRASTRUCTURE (see fltop_oracle.h).
 *
 * Two independent routines live here:
 *   - decode_fltop():    Algorithm 1 of the paper (Sec. 3), frame by frame, with
 *                        the relative-threshold token test, generic map-based
 *                        merging and fp64 log-masses.
 *   - decode_textbook(): a classic CTC prefix beam search that looks at every
 *                        token of every frame, written on different data
 *                        structures and with a different log-add, so that
 *                        "r = 0 reproduces the unpruned search" is a real check.
 * Nothing here is tuned; clarity over speed.
 */
#include "fltop_oracle.h"

#include <algorithm>
#include <atomic>
#include <cmath>
#include <limits>
#include <map>
#include <mutex>
#include <thread>
#include <utility>
#include <vector>

namespace {

typedef std::vector<int32_t> Prefix;
const double NEG_INF = -std::numeric_limits<double>::infinity();

/* ---- prefix hash: tie-break only ------------------------------------------------ */
const uint64_t GOLDEN = 0x9E3779B97F4A7C15ULL;

uint64_t splitmix_out(uint64_t z) {
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
    return z ^ (z >> 31);
}

uint64_t hash_of(const Prefix& p) {
    uint64_t h = GOLDEN;
    for (size_t i = 0; i < p.size(); ++i)
        h = splitmix_out(h + GOLDEN * (uint64_t)((int64_t)p[i] + 1));
    return h;
}

/* ---- log-sum-exp of two log-masses, -inf safe ----------------------------------- */
double log_add(double a, double b) {
    if (a == NEG_INF) return b;
    if (b == NEG_INF) return a;
    double hi = a > b ? a : b;
    double lo = a > b ? b : a;
    return hi + std::log1p(std::exp(lo - hi));
}

/* ---- LM term on extension: alpha * table[prev][cur] + beta ---------------------- */
struct LmSpec {
    const float* table;  /* NULL = no LM */
    int32_t V;
    double alpha, beta;
    double term(int32_t last, int32_t cur) const {
        if (!table) return 0.0;
        int32_t row = last < 0 ? 0 : last; /* first token: row 0 stands for sentence start */
        return alpha * (double)table[(int64_t)row * V + cur] + beta;
    }
};

/* ---- survivor set of one frame (Alg. 1: top emission, relative threshold) -------- */
float ln_r_fp32(float r) {
    if (r <= 0.0f) return -std::numeric_limits<float>::infinity();
    return (float)std::log((double)r);
}

struct EmissionBefore { /* descending emission, equal emissions by ascending token id */
    const float* row;
    bool operator()(int32_t a, int32_t b) const {
        if (row[a] != row[b]) return row[a] > row[b];
        return a < b;
    }
};

/* Alg. 1 in its printed order: partial sort of the frame to its N best tokens, the top
 * emission is the first of them, then walk down the sorted list and stop at the first
 * token that fails the relative-threshold test.  top_n <= 0 or >= V: all V tokens enter
 * the walk.  S is returned in ascending token order (the expansion is a set union, so
 * the order in which survivors are visited does not matter). */
void frame_survivors(const float* row, int32_t V, int32_t top_n, float ln_r,
                     std::vector<int32_t>& S, float* top) {
    const int32_t n = (top_n <= 0 || top_n > V) ? V : top_n;
    std::vector<int32_t> sorted_idx(V);
    for (int32_t v = 0; v < V; ++v) sorted_idx[v] = v;
    EmissionBefore before;
    before.row = row;
    std::partial_sort(sorted_idx.begin(), sorted_idx.begin() + n, sorted_idx.end(), before);
    const float m = row[sorted_idx[0]];
    volatile float thr = m + ln_r; /* one fp32 add; volatile keeps it in fp32 */
    S.clear();
    for (int32_t i = 0; i < n; ++i) {
        const int32_t v = sorted_idx[i];
        if (!(row[v] >= thr)) break;
        S.push_back(v);
    }
    std::sort(S.begin(), S.end());
    if (top) *top = m;
}

/* ---- beam bookkeeping ----------------------------------------------------------- */
struct Mass {
    double pb, pnb;
    int32_t terms_b, terms_nb;
    /* born[i] = frame at which the prefix of length i+1 entered the beam on the way to this
     * entry (statistics only; plays no part in the search) */
    std::vector<int32_t> born;
    Mass() : pb(NEG_INF), pnb(NEG_INF), terms_b(0), terms_nb(0) {}
    double total() const { return log_add(pb, pnb); }
};

typedef std::map<Prefix, Mass> Beam;

struct Ranked {
    double total;
    uint64_t hash;
    Beam::const_iterator it;
};

bool rank_before(const Ranked& x, const Ranked& y) {
    if (x.total != y.total) return x.total > y.total;
    return x.hash < y.hash;
}

struct LocalStats {
    int64_t frames, sum_survivors, sum_candidates, peak_candidates, sum_beam, max_addends,
        hash_collisions;
    double min_cut_margin;
    /* smallest score gap that decided anything: the beam cut, the window floor (distance of
     * the nearest candidate on either side), the choice of the final best prefix.  0 means
     * an exact tie, which the hash order resolved.  Reporting only. */
    double min_decision_margin;
    LocalStats()
        : frames(0), sum_survivors(0), sum_candidates(0), peak_candidates(0), sum_beam(0),
          max_addends(0), hash_collisions(0),
          min_cut_margin(std::numeric_limits<double>::infinity()),
          min_decision_margin(std::numeric_limits<double>::infinity()) {}
};

/* SelectTopK of Alg. 1: rank the live candidates of `next` (score desc, hash asc), drop
 * those whose score lies more than `beam_threshold` below the best one (when that
 * window is switched on, i.e. > 0), and return the best `beam` of the rest. */
Beam keep_best(const Beam& next, int32_t beam, double beam_threshold, LocalStats& st) {
    std::vector<Ranked> order;
    for (Beam::const_iterator it = next.begin(); it != next.end(); ++it) {
        double tot = it->second.total();
        if (tot == NEG_INF) continue; /* dead: every route into it was pruned */
        Ranked r;
        r.total = tot;
        r.hash = hash_of(it->first);
        r.it = it;
        order.push_back(r);
        int64_t terms = std::max(it->second.terms_b, it->second.terms_nb);
        if (terms > st.max_addends) st.max_addends = terms;
    }
    std::sort(order.begin(), order.end(), rank_before);
    for (size_t i = 1; i < order.size(); ++i)
        if (order[i].hash == order[i - 1].hash) st.hash_collisions++;
    int64_t n = (int64_t)order.size();
    st.sum_candidates += n;
    if (n > st.peak_candidates) st.peak_candidates = n;
    if (beam_threshold > 0.0 && n > 0) {
        const double floor_score = order[0].total - beam_threshold;
        size_t inside = 0;
        while (inside < order.size() && order[inside].total >= floor_score) ++inside;
        for (size_t i = 1; i < order.size(); ++i) /* order[0] is the window's own anchor */
            st.min_decision_margin =
                std::min(st.min_decision_margin, std::fabs(order[i].total - floor_score));
        order.resize(inside); /* the list is sorted, so the window is a leading run */
        n = (int64_t)order.size();
    }
    if (n > beam) {
        double margin = order[beam - 1].total - order[beam].total;
        if (margin < st.min_cut_margin) st.min_cut_margin = margin;
        if (margin < st.min_decision_margin) st.min_decision_margin = margin;
        order.resize(beam);
    }
    st.sum_beam += (int64_t)order.size();
    Beam kept;
    for (size_t i = 0; i < order.size(); ++i) kept.insert(*order[i].it);
    return kept;
}

/* Final beam in rank order. */
std::vector<Ranked> rank_all(const Beam& b) {
    std::vector<Ranked> order;
    for (Beam::const_iterator it = b.begin(); it != b.end(); ++it) {
        Ranked r;
        r.total = it->second.total();
        r.hash = hash_of(it->first);
        r.it = it;
        order.push_back(r);
    }
    std::sort(order.begin(), order.end(), rank_before);
    return order;
}

/* What Alg. 1 takes besides the emissions and the LM. */
struct SearchSpec {
    int32_t beam;          /* beam_size */
    float rel_threshold;   /* R */
    int32_t top_n;         /* N; <= 0: all tokens */
    double beam_threshold; /* score window of SelectTopK; <= 0: off */
    int32_t* frame_beam;   /* NULL or [len]: entries kept after each frame (statistics) */
};

/* A candidate that is not in the current beam is a prefix that enters now. */
void note_birth(Mass& fresh, const Beam& cur, const Prefix& ext, const Mass& parent, int32_t t) {
    if (!fresh.born.empty() || ext.empty()) return;
    Beam::const_iterator old = cur.find(ext);
    if (old != cur.end()) {
        fresh.born = old->second.born;
    } else {
        fresh.born = parent.born;
        fresh.born.push_back(t);
    }
}

/* ---- Algorithm 1 (FLToP) --------------------------------------------------------- */
Beam decode_fltop(const float* lp, int32_t len, int32_t V, const SearchSpec& spec,
                  const LmSpec& lm, LocalStats& st) {
    const float ln_r = ln_r_fp32(spec.rel_threshold);
    Beam cur;
    Mass start;
    start.pb = 0.0; /* the empty prefix with score 0 */
    cur[Prefix()] = start;
    std::vector<int32_t> S;
    for (int32_t t = 0; t < len; ++t) {
        const float* row = lp + (int64_t)t * V;
        frame_survivors(row, V, spec.top_n, ln_r, S, 0);
        st.frames++;
        st.sum_survivors += (int64_t)S.size();
        Beam next;
        for (Beam::const_iterator it = cur.begin(); it != cur.end(); ++it) {
            const Prefix& prefix = it->first;
            const Mass& m = it->second;
            const double p_tot = m.total();
            const int32_t last = prefix.empty() ? -1 : prefix.back();
            for (size_t k = 0; k < S.size(); ++k) {
                const int32_t s = S[k];
                const double x = (double)row[s];
                if (s == 0) {
                    /* blank: prefix unchanged, mass moves to "ends in blank" */
                    Mass& d = next[prefix];
                    d.pb = log_add(d.pb, p_tot + x);
                    d.terms_b++;
                    d.born = m.born;
                } else if (s == last) {
                    /* repeat of the last token: collapses onto the same prefix ... */
                    Mass& d = next[prefix];
                    d.pnb = log_add(d.pnb, m.pnb + x);
                    d.terms_nb++;
                    d.born = m.born;
                    /* ... unless a blank separated them: then it is a new token */
                    Prefix ext(prefix);
                    ext.push_back(s);
                    Mass& e = next[ext];
                    e.pnb = log_add(e.pnb, m.pb + x + lm.term(last, s));
                    e.terms_nb++;
                    note_birth(e, cur, ext, m, t);
                } else {
                    Prefix ext(prefix);
                    ext.push_back(s);
                    Mass& e = next[ext];
                    e.pnb = log_add(e.pnb, p_tot + x + lm.term(last, s));
                    e.terms_nb++;
                    note_birth(e, cur, ext, m, t);
                }
            }
        }
        cur = keep_best(next, spec.beam, spec.beam_threshold, st);
        if (spec.frame_beam) spec.frame_beam[t] = (int32_t)cur.size();
    }
    return cur;
}

/* ---- textbook prefix beam search, every token, written separately ---------------- */
struct Hyp {
    Prefix toks;
    double blank_mass, label_mass;
};

double log_add_plain(double a, double b) {
    if (a == NEG_INF && b == NEG_INF) return NEG_INF;
    double m = std::max(a, b);
    return m + std::log(std::exp(a - m) + std::exp(b - m));
}

Hyp& find_or_add(std::vector<Hyp>& pool, const Prefix& toks) {
    for (size_t i = 0; i < pool.size(); ++i)
        if (pool[i].toks == toks) return pool[i];
    Hyp h;
    h.toks = toks;
    h.blank_mass = NEG_INF;
    h.label_mass = NEG_INF;
    pool.push_back(h);
    return pool.back();
}

Beam decode_textbook(const float* lp, int32_t len, int32_t V, int32_t beam, const LmSpec& lm,
                     LocalStats& st) {
    std::vector<Hyp> hyps(1);
    hyps[0].blank_mass = 0.0;
    hyps[0].label_mass = NEG_INF;
    for (int32_t t = 0; t < len; ++t) {
        const float* row = lp + (int64_t)t * V;
        st.frames++;
        st.sum_survivors += V;
        std::vector<Hyp> pool;
        for (int32_t v = 0; v < V; ++v) {
            const double e = (double)row[v];
            for (size_t i = 0; i < hyps.size(); ++i) {
                const Hyp src = hyps[i]; /* copy: pool growth must not alias */
                const double whole = log_add_plain(src.blank_mass, src.label_mass);
                const int32_t tail = src.toks.empty() ? -1 : src.toks.back();
                if (v == 0) {
                    Hyp& same = find_or_add(pool, src.toks);
                    same.blank_mass = log_add_plain(same.blank_mass, whole + e);
                    continue;
                }
                Prefix longer(src.toks);
                longer.push_back(v);
                const double from = (v == tail) ? src.blank_mass : whole;
                {
                    Hyp& grown = find_or_add(pool, longer);
                    grown.label_mass = log_add_plain(grown.label_mass, from + e + lm.term(tail, v));
                }
                if (v == tail) {
                    Hyp& same = find_or_add(pool, src.toks);
                    same.label_mass = log_add_plain(same.label_mass, src.label_mass + e);
                }
            }
        }
        /* order by score then hash, cut to `beam` */
        std::vector<std::pair<std::pair<double, uint64_t>, size_t> > keyed;
        for (size_t i = 0; i < pool.size(); ++i) {
            double sc = log_add_plain(pool[i].blank_mass, pool[i].label_mass);
            if (sc == NEG_INF) continue;
            keyed.push_back(std::make_pair(std::make_pair(-sc, hash_of(pool[i].toks)), i));
        }
        std::sort(keyed.begin(), keyed.end());
        int64_t n = (int64_t)keyed.size();
        st.sum_candidates += n;
        if (n > st.peak_candidates) st.peak_candidates = n;
        if (n > beam) {
            double margin = keyed[beam].first.first - keyed[beam - 1].first.first;
            if (margin < st.min_cut_margin) st.min_cut_margin = margin;
            keyed.resize(beam);
        }
        st.sum_beam += (int64_t)keyed.size();
        std::vector<Hyp> kept;
        for (size_t i = 0; i < keyed.size(); ++i) kept.push_back(pool[keyed[i].second]);
        hyps.swap(kept);
    }
    Beam out;
    for (size_t i = 0; i < hyps.size(); ++i) {
        Mass m;
        m.pb = hyps[i].blank_mass;
        m.pnb = hyps[i].label_mass;
        out[hyps[i].toks] = m;
    }
    return out;
}

Beam decode_one(const float* lp, int32_t len, int32_t V, const SearchSpec& spec, const LmSpec& lm,
                int32_t variant, LocalStats& st) {
    if (variant == FLTOP_ORACLE_TEXTBOOK) return decode_textbook(lp, len, V, spec.beam, lm, st);
    return decode_fltop(lp, len, V, spec, lm, st);
}

bool bad_common(const void* lp, int32_t T, int32_t V, int32_t beam, float r, int32_t top_n,
                double beam_threshold, int32_t variant) {
    if (!lp || T < 0 || V < 1 || beam < 1) return true;
    if (!(r >= 0.0f && r <= 1.0f)) return true; /* also rejects NaN */
    if (top_n < 0 || beam_threshold != beam_threshold) return true;
    if (variant != FLTOP_ORACLE_FLTOP && variant != FLTOP_ORACLE_TEXTBOOK) return true;
    /* the classic search has neither a token stage nor a score window */
    if (variant == FLTOP_ORACLE_TEXTBOOK && (top_n > 0 || beam_threshold > 0.0)) return true;
    return false;
}

} /* namespace */

extern "C" uint64_t fltop_oracle_prefix_hash(const int32_t* tokens, int32_t n) {
    Prefix p;
    for (int32_t i = 0; i < n; ++i) p.push_back(tokens[i]);
    return hash_of(p);
}

extern "C" int fltop_oracle_survivors(const float* logprobs, int64_t n_frames, int32_t V,
                                      float rel_threshold, int32_t top_n, int32_t* counts,
                                      int32_t* tokens, float* frame_max) {
    if (!logprobs || !counts || !tokens || n_frames < 0 || V < 1 || top_n < 0) return -1;
    if (!(rel_threshold >= 0.0f && rel_threshold <= 1.0f)) return -1;
    const float ln_r = ln_r_fp32(rel_threshold);
    std::vector<int32_t> S;
    for (int64_t f = 0; f < n_frames; ++f) {
        float top;
        frame_survivors(logprobs + f * V, V, top_n, ln_r, S, &top);
        counts[f] = (int32_t)S.size();
        for (size_t k = 0; k < S.size(); ++k) tokens[f * V + (int64_t)k] = S[k];
        if (frame_max) frame_max[f] = top;
    }
    return 0;
}

extern "C" int fltop_oracle_decode(const float* logprobs, const int32_t* lengths, int32_t B,
                                   int32_t T, int32_t V, int32_t beam, float rel_threshold,
                                   int32_t top_n, double beam_threshold, const float* lm_table,
                                   float lm_weight, float insertion_bonus, int32_t variant,
                                   int32_t* out_tokens, int32_t* out_lengths, double* out_scores,
                                   int32_t* out_token_frames, int32_t* frame_beam,
                                   double* out_margins, fltop_oracle_stats* stats,
                                   int32_t n_threads) {
    if (bad_common(logprobs, T, V, beam, rel_threshold, top_n, beam_threshold, variant))
        return -1;
    if (variant == FLTOP_ORACLE_TEXTBOOK && (out_token_frames || frame_beam)) return -1;
    if (!lengths || B < 0 || !out_tokens || !out_lengths || !out_scores || n_threads < 1)
        return -1;
    for (int32_t b = 0; b < B; ++b)
        if (lengths[b] < 0 || lengths[b] > T) return -1;
    LmSpec lm;
    lm.table = lm_table;
    lm.V = V;
    lm.alpha = (double)lm_weight;
    lm.beta = (double)insertion_bonus;

    std::atomic<int32_t> next_utt(0);
    std::mutex merge_lock;
    LocalStats all;
    auto worker = [&]() {
        LocalStats mine;
        for (;;) {
            int32_t b = next_utt.fetch_add(1);
            if (b >= B) break;
            SearchSpec spec;
            spec.beam = beam;
            spec.rel_threshold = rel_threshold;
            spec.top_n = top_n;
            spec.beam_threshold = beam_threshold;
            spec.frame_beam = frame_beam ? frame_beam + (int64_t)b * T : 0;
            LocalStats one;
            Beam fin = decode_one(logprobs + (int64_t)b * T * V, lengths[b], V, spec, lm, variant,
                                  one);
            std::vector<Ranked> order = rank_all(fin);
            if (order.size() > 1)
                one.min_decision_margin =
                    std::min(one.min_decision_margin, order[0].total - order[1].total);
            if (out_margins) out_margins[b] = one.min_decision_margin;
            mine.frames += one.frames;
            mine.sum_survivors += one.sum_survivors;
            mine.sum_candidates += one.sum_candidates;
            mine.sum_beam += one.sum_beam;
            mine.hash_collisions += one.hash_collisions;
            mine.peak_candidates = std::max(mine.peak_candidates, one.peak_candidates);
            mine.max_addends = std::max(mine.max_addends, one.max_addends);
            mine.min_cut_margin = std::min(mine.min_cut_margin, one.min_cut_margin);
            mine.min_decision_margin = std::min(mine.min_decision_margin, one.min_decision_margin);
            int32_t* dst = out_tokens + (int64_t)b * T;
            if (order.empty()) { /* every route died (a frame of all -inf) */
                out_lengths[b] = 0;
                out_scores[b] = NEG_INF;
                continue;
            }
            const Prefix& best = order[0].it->first;
            out_lengths[b] = (int32_t)best.size();
            for (size_t i = 0; i < best.size(); ++i) dst[i] = best[i];
            out_scores[b] = order[0].total;
            if (out_token_frames) {
                const std::vector<int32_t>& born = order[0].it->second.born;
                for (size_t i = 0; i < born.size(); ++i)
                    out_token_frames[(int64_t)b * T + (int64_t)i] = born[i];
            }
        }
        std::lock_guard<std::mutex> g(merge_lock);
        all.frames += mine.frames;
        all.sum_survivors += mine.sum_survivors;
        all.sum_candidates += mine.sum_candidates;
        all.sum_beam += mine.sum_beam;
        all.hash_collisions += mine.hash_collisions;
        all.peak_candidates = std::max(all.peak_candidates, mine.peak_candidates);
        all.max_addends = std::max(all.max_addends, mine.max_addends);
        all.min_cut_margin = std::min(all.min_cut_margin, mine.min_cut_margin);
        all.min_decision_margin = std::min(all.min_decision_margin, mine.min_decision_margin);
    };
    std::vector<std::thread> pool;
    for (int32_t i = 1; i < n_threads; ++i) pool.emplace_back(worker);
    worker();
    for (size_t i = 0; i < pool.size(); ++i) pool[i].join();

    if (stats) {
        stats->frames = all.frames;
        stats->sum_survivors = all.sum_survivors;
        stats->sum_candidates = all.sum_candidates;
        stats->peak_candidates = all.peak_candidates;
        stats->sum_beam = all.sum_beam;
        stats->max_addends = all.max_addends;
        stats->hash_collisions = all.hash_collisions;
        stats->min_cut_margin = all.min_cut_margin;
        stats->min_decision_margin = all.min_decision_margin;
    }
    return 0;
}

extern "C" int fltop_oracle_decode_beam(const float* logprobs, int32_t T, int32_t V, int32_t beam,
                                        float rel_threshold, int32_t top_n,
                                        double beam_threshold, const float* lm_table,
                                        float lm_weight, float insertion_bonus, int32_t variant,
                                        int32_t max_entries, int32_t* beam_tokens,
                                        int32_t* beam_lengths, double* beam_pb,
                                        double* beam_pnb) {
    if (bad_common(logprobs, T, V, beam, rel_threshold, top_n, beam_threshold, variant))
        return -1;
    if (max_entries < 0 || !beam_tokens || !beam_lengths || !beam_pb || !beam_pnb) return -1;
    LmSpec lm;
    lm.table = lm_table;
    lm.V = V;
    lm.alpha = (double)lm_weight;
    lm.beta = (double)insertion_bonus;
    LocalStats st;
    SearchSpec spec;
    spec.beam = beam;
    spec.rel_threshold = rel_threshold;
    spec.top_n = top_n;
    spec.beam_threshold = beam_threshold;
    spec.frame_beam = 0;
    Beam fin = decode_one(logprobs, T, V, spec, lm, variant, st);
    std::vector<Ranked> order = rank_all(fin);
    int32_t n = (int32_t)std::min<size_t>(order.size(), (size_t)max_entries);
    for (int32_t i = 0; i < n; ++i) {
        const Prefix& p = order[i].it->first;
        beam_lengths[i] = (int32_t)p.size();
        for (size_t k = 0; k < p.size(); ++k) beam_tokens[(int64_t)i * T + (int64_t)k] = p[k];
        beam_pb[i] = order[i].it->second.pb;
        beam_pnb[i] = order[i].it->second.pnb;
    }
    return n;
}

extern "C" int fltop_oracle_token_ranks(const float* logprobs, int32_t T, int32_t V,
                                        const int32_t* tokens, const int32_t* frames, int32_t n,
                                        int32_t* ranks) {
    if (!logprobs || T < 0 || V < 1 || n < 0 || (n > 0 && (!tokens || !frames || !ranks)))
        return -1;
    for (int32_t i = 0; i < n; ++i) {
        if (frames[i] < 0 || frames[i] >= T || tokens[i] < 0 || tokens[i] >= V) return -1;
        const float* row = logprobs + (int64_t)frames[i] * V;
        EmissionBefore before;
        before.row = row;
        int32_t ahead = 0; /* tokens that the descending sort of the frame puts first */
        for (int32_t v = 0; v < V; ++v)
            if (v != tokens[i] && before(v, tokens[i])) ++ahead;
        ranks[i] = ahead;
    }
    return 0;
}
