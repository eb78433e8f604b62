/*
 * Exercises every entry point of the CPU oracle on small random inputs so that a build with
 * -fsanitize=address,undefined can report out-of-bounds accesses, overflows and the like.
 * TEST INFRASTRUCTURE, like the oracle itself.  Checks only what a sanitizer cannot: status
 * codes and that outputs stay inside their documented ranges.  Prints "ok" and exits 0.
 */
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <limits>
#include <vector>

#include "fltop_oracle.h"

namespace {

// xorshift64*: the inputs only have to be varied, not of any particular distribution
struct Rng {
    uint64_t s;
    explicit Rng(uint64_t seed) : s(seed * 0x9E3779B97F4A7C15ull + 1) {}
    uint64_t next() {
        s ^= s >> 12;
        s ^= s << 25;
        s ^= s >> 27;
        return s * 0x2545F4914F6CDD1Dull;
    }
    double uniform() { return (double)(next() >> 11) * (1.0 / 9007199254740992.0); }
};

std::vector<float> random_rows(Rng& rng, int64_t rows, int V, double spread) {
    std::vector<float> lp((size_t)rows * V);
    for (int64_t f = 0; f < rows; ++f) {
        std::vector<double> z(V);
        double mx = -1e300;
        for (int v = 0; v < V; ++v) {
            z[v] = spread * (rng.uniform() * 2.0 - 1.0) * 3.0;
            mx = std::fmax(mx, z[v]);
        }
        double sum = 0.0;
        for (int v = 0; v < V; ++v) sum += std::exp(z[v] - mx);
        for (int v = 0; v < V; ++v) lp[(size_t)f * V + v] = (float)(z[v] - mx - std::log(sum));
    }
    return lp;
}

int fail(const char* what) {
    std::fprintf(stderr, "sanitize_driver: %s\n", what);
    return 1;
}

}  // namespace

int main() {
    Rng rng(20251009);
    const float kInf = std::numeric_limits<float>::infinity();
    struct Case {
        int B, T, V, beam, top_n;
        float r;
        double window;
        bool lm;
    };
    const Case cases[] = {
        {1, 1, 2, 1, 0, 0.0f, 0.0, false},    {3, 17, 5, 4, 0, 0.01f, 0.0, false},
        {2, 40, 32, 32, 4, 0.007f, 25.0, true}, {4, 25, 33, 7, 0, 0.0f, 3.0, true},
        {2, 30, 100, 64, 10, 0.05f, 0.0, false}, {3, 12, 8, 200, 0, 0.0f, 0.0, false},
        {2, 9, 3, 2, 1, 1.0f, 0.5, false},
    };
    for (const Case& c : cases) {
        std::vector<float> lp = random_rows(rng, (int64_t)c.B * c.T, c.V, 1.5);
        // a few -inf entries and a dead row exercise the zero-mass paths
        lp[(size_t)(c.T / 2) * c.V + (c.V - 1)] = -kInf;
        std::vector<int32_t> len(c.B);
        for (int b = 0; b < c.B; ++b) len[b] = (b == 1) ? c.T / 2 : c.T;
        if (c.B > 2) len[2] = 0;
        std::vector<float> lm;
        if (c.lm) lm = random_rows(rng, c.V, c.V, 1.0);

        // survivors
        std::vector<int32_t> counts((size_t)c.B * c.T), toks((size_t)c.B * c.T * c.V);
        std::vector<float> fmax((size_t)c.B * c.T);
        if (fltop_oracle_survivors(lp.data(), (int64_t)c.B * c.T, c.V, c.r, c.top_n, counts.data(),
                                   toks.data(), fmax.data()) != 0)
            return fail("survivors status");
        for (size_t f = 0; f < counts.size(); ++f)
            if (counts[f] < 1 || counts[f] > c.V) return fail("survivor count out of range");

        // decode, both variants where the variant takes the options
        for (int variant = 0; variant < 2; ++variant) {
            const bool textbook = variant == FLTOP_ORACLE_TEXTBOOK;
            if (textbook && (c.top_n > 0 || c.window > 0.0)) continue;
            std::vector<int32_t> out_tok((size_t)c.B * c.T), out_len(c.B);
            std::vector<int32_t> tf((size_t)c.B * c.T), fb((size_t)c.B * c.T);
            std::vector<double> score(c.B), margins(c.B);
            fltop_oracle_stats st = {};
            const int rc = fltop_oracle_decode(
                lp.data(), len.data(), c.B, c.T, c.V, c.beam, textbook ? 0.0f : c.r, c.top_n,
                c.window, c.lm ? lm.data() : nullptr, 0.5f, 1.0f, variant, out_tok.data(),
                out_len.data(), score.data(), textbook ? nullptr : tf.data(),
                textbook ? nullptr : fb.data(), margins.data(), &st, 1 + variant * 2);
            if (rc != 0) return fail("decode status");
            for (int b = 0; b < c.B; ++b) {
                if (out_len[b] < 0 || out_len[b] > len[b]) return fail("output length out of range");
                for (int i = 0; i < out_len[b]; ++i) {
                    const int32_t t = out_tok[(size_t)b * c.T + i];
                    if (t < 1 || t >= c.V) return fail("output token out of range");
                    if (!textbook) {
                        const int32_t fr = tf[(size_t)b * c.T + i];
                        if (fr < 0 || fr >= len[b]) return fail("token frame out of range");
                    }
                }
            }
            if (st.frames < 0 || st.sum_beam > st.sum_candidates) return fail("stats");

            // token ranks of the first utterance's best prefix
            if (!textbook && out_len[0] > 0) {
                std::vector<int32_t> ranks(out_len[0]);
                if (fltop_oracle_token_ranks(lp.data(), c.T, c.V, out_tok.data(), tf.data(),
                                             out_len[0], ranks.data()) != 0)
                    return fail("token_ranks status");
                for (int32_t rk : ranks)
                    if (rk < 0 || rk >= c.V) return fail("rank out of range");
            }
        }

        // whole final beam of the first utterance, with fewer places than entries as well
        for (int cap : {c.beam, 1}) {
            std::vector<int32_t> bt((size_t)cap * c.T), bl(cap);
            std::vector<double> pb(cap), pnb(cap);
            const int n = fltop_oracle_decode_beam(lp.data(), c.T, c.V, c.beam, c.r, c.top_n, c.window,
                                                   c.lm ? lm.data() : nullptr, 0.5f, 1.0f,
                                                   FLTOP_ORACLE_FLTOP, cap, bt.data(), bl.data(),
                                                   pb.data(), pnb.data());
            if (n < 0 || n > cap) return fail("decode_beam count");
        }
    }

    // bad arguments come back as -1 and touch nothing
    std::vector<float> lp = random_rows(rng, 4, 4, 1.0);
    int32_t one_len = 4, tok[4], ol;
    double sc;
    if (fltop_oracle_decode(lp.data(), &one_len, 1, 4, 4, 0, 0.01f, 0, 0.0, nullptr, 0.f, 0.f, 0, tok,
                            &ol, &sc, nullptr, nullptr, nullptr, nullptr, 1) != -1)
        return fail("beam 0 accepted");
    if (fltop_oracle_decode(lp.data(), &one_len, 1, 4, 4, 2, 2.0f, 0, 0.0, nullptr, 0.f, 0.f, 0, tok,
                            &ol, &sc, nullptr, nullptr, nullptr, nullptr, 1) != -1)
        return fail("r > 1 accepted");
    const int32_t empty[1] = {0};
    if (fltop_oracle_prefix_hash(empty, 0) != 0x9E3779B97F4A7C15ull) return fail("hash of empty");

    std::puts("ok");
    return 0;
}
