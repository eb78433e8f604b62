// CTC prefix beam search over the survivor lists (paper Sec. 3, Algorithm 1: the
// loop over beam entries and kept tokens, the set-insert that merges equal
// prefixes, SelectTopK and GetHighestScorePrefix).
//
// One workgroup decodes one utterance and stays resident for all its frames.
// The beam (prefix hash, parent hash, last token, p_b, p_nb, trie node) lives in
// LDS.  Candidates are never materialised: a candidate is either "entry j stays"
// or "entry i extended by survivor k", and its score is recomputed from the
// LDS-resident beam whenever a pass needs it.  An extension i+s can only
// coincide with a prefix that is already in the beam (a prefix has one parent),
// so merging is done from the side of that beam entry: it looks its parent up
// in an LDS hash table and adds the parent's extension mass to its own p_nb;
// the extension itself is then skipped.  Every log-sum-exp has two operands.
//
// Top-`beam` selection works on an order-preserving 64-bit image of the fp64
// score: a histogram over the distance to an upper bound locates the bucket
// holding the beam-th best candidate, buckets are refined until the boundary
// bucket is small, and its members are ranked exactly by (score, prefix hash).
#include "fltop_internal.h"

namespace fltop {
namespace {

constexpr int kThreads = 256;
constexpr int kWave = 64;
constexpr int kMaxBeam = FLTOP_MAX_BEAM;
constexpr int kHashSlots = 4 * kMaxBeam;
constexpr int kBins = 1024;
constexpr int kBinsPerLane = kBins / kWave;  // 16
constexpr int kExactCap = 64;
constexpr int kMaxShift = 54;  // kBins << kMaxShift covers all 64-bit distances
constexpr uint64_t kGolden = 0x9E3779B97F4A7C15ull;
constexpr uint64_t kAllOnes = ~0ull;

struct BeamSlab {
    uint64_t h[kMaxBeam];   // prefix hash
    uint64_t hp[kMaxBeam];  // parent prefix hash (unused when plen == 0)
    double pb[kMaxBeam];
    double pnb[kMaxBeam];
    double ptot[kMaxBeam];
    int32_t last[kMaxBeam];  // last token, -1 for the empty prefix
    int32_t node[kMaxBeam];  // trie node of the prefix
    int32_t plen[kMaxBeam];  // prefix length
};

struct BeamArgs {
    const int32_t* lengths;
    const FrameHdr* hdr;
    const Survivor* rec;
    TrieNode* trie;
    int64_t trie_stride;
    const float* lm_table;  // global copy (always valid when LM is on)
    const float* lm_bound;
    double lm_alpha, lm_beta;
    int32_t B, T, V, fpb, beam;
    int32_t lm_in_lds;  // 1: table staged into LDS
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

__device__ inline double lse2(double a, double b) {
    if (a == -INFINITY) return b;
    if (b == -INFINITY) return a;
    const double hi = a > b ? a : b;
    const double lo = a > b ? b : a;
    return hi + log1p(exp(lo - hi));
}

__device__ inline int lanes_below(uint64_t mask, int lane) {
    return __popcll(mask & ((1ull << lane) - 1ull));
}

// bin b is stored transposed so that lane l of a wave owns bins [16l, 16l+16)
// at conflict-free addresses (q*64 + l).
__device__ inline int bin_slot(int b) { return (b & (kBinsPerLane - 1)) * kWave + (b >> 4); }

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

// dynamic LDS: dense_lp[V] fp32, s_tok[V] u16, then (optionally) the LM table
__host__ __device__ inline size_t lm_lds_offset(int V) {
    return (((size_t)V * (sizeof(float) + sizeof(uint16_t))) + 15) / 16 * 16;
}

__global__ __launch_bounds__(kThreads) void beam_kernel(BeamArgs a) {
    __shared__ BeamSlab slab[2];
    __shared__ double st_pb[kMaxBeam], st_pnb[kMaxBeam], st_tot[kMaxBeam];
    __shared__ int32_t par[kMaxBeam], first_kid[kMaxBeam], next_kid[kMaxBeam];
    __shared__ int32_t ht[kHashSlots];
    __shared__ uint32_t hist[3][kBins];
    __shared__ uint64_t bl_D[kExactCap], bl_h[kExactCap];
    __shared__ uint64_t sh_kmax, sh_kmin, sh_selD, sh_selH;
    __shared__ int32_t sh_nnew, sh_nodes, sh_blcount, sh_best;
    extern __shared__ __align__(16) unsigned char dyn_lds[];

    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int b = blockIdx.x;
    const int V = a.V;
    const int beam = a.beam;

    float* dense_lp = reinterpret_cast<float*>(dyn_lds);
    uint16_t* s_tok = reinterpret_cast<uint16_t*>(dyn_lds + (size_t)V * sizeof(float));
    float* lm_s = reinterpret_cast<float*>(dyn_lds + lm_lds_offset(V));
    const bool has_lm = a.lm_table != nullptr;
    const float* lm = a.lm_in_lds ? lm_s : a.lm_table;

    int32_t len = a.lengths[b];
    len = len < 0 ? 0 : (len > a.T ? a.T : len);

    // ---- one-time initialisation ------------------------------------------------
    for (int v = tid; v < V; v += kThreads) dense_lp[v] = -INFINITY;
    for (int i = tid; i < 3 * kBins; i += kThreads) (&hist[0][0])[i] = 0u;
    if (a.lm_in_lds)
        for (int i = tid; i < V * V; i += kThreads) lm_s[i] = a.lm_table[i];
    if (tid < kMaxBeam) {
        par[tid] = -1;
        first_kid[tid] = -1;
        next_kid[tid] = -1;
    }
    if (tid == 0) {
        BeamSlab& s0 = slab[0];
        s0.h[0] = kGolden;
        s0.hp[0] = 0;
        s0.pb[0] = 0.0;
        s0.pnb[0] = -INFINITY;
        s0.ptot[0] = 0.0;
        s0.last[0] = -1;
        s0.node[0] = 0;
        s0.plen[0] = 0;
        sh_kmax = order_key(0.0);
        sh_kmin = order_key(0.0);
        sh_nodes = 1;
        sh_nnew = 0;
        sh_blcount = 0;
    }
    TrieNode* trie = a.trie + (int64_t)b * a.trie_stride;
    const double lm_ub = has_lm ? fmax(0.0, (double)a.lm_bound[0]) : 0.0;
    __syncthreads();

    int cur_i = 0;
    int n_live = 1;
    int hist_pass = 0;  // running index of histogram passes: pass p uses hist[p % 3]

    // statistics kept by thread 0
    uint64_t st_surv = 0, st_cand = 0, st_peak = 0, st_beam = 0, st_pass = 0, st_exact = 0,
             st_drop = 0;

    const int64_t g_base = (int64_t)b * a.T;
    FrameHdr hd_next;
    hd_next.count = 0;
    hd_next.offset = 0;
    hd_next.top = 0.0f;
    if (len > 0) hd_next = a.hdr[g_base];

    for (int t = 0; t < len; ++t) {
        const int64_t g = g_base + t;
        const FrameHdr hd = hd_next;
        if (t + 1 < len) hd_next = a.hdr[g + 1];
        const int K = hd.count;
        const Survivor* recs = a.rec + (g / a.fpb) * (int64_t)a.fpb * V + hd.offset;

        // ---- stage the frame's survivors -------------------------------------
        for (int k = tid; k < K; k += kThreads) {
            const Survivor s = recs[k];
            s_tok[k] = (uint16_t)s.tok;
            dense_lp[s.tok] = s.lp;
        }
        __syncthreads();

        if (n_live > 0) {
            BeamSlab& cur = slab[cur_i];
            BeamSlab& nxt = slab[cur_i ^ 1];
            const int nb0 = (K > 0 && s_tok[0] == 0) ? 1 : 0;  // records ascend: blank first
            const int Knb = K - nb0;
            const double lp_blank = (double)dense_lp[0];

            auto lm_term = [&](int32_t prev, int32_t tok) -> double {
                if (!has_lm) return 0.0;
                const int32_t row = prev < 0 ? 0 : prev;
                return a.lm_alpha * (double)lm[(int64_t)row * V + tok] + a.lm_beta;
            };

            // ---- stay candidates: entry j keeps its prefix ---------------------
            if (tid < n_live) {
                const int j = tid;
                const int32_t lj = cur.last[j];
                const double lpl = (lj >= 0) ? (double)dense_lp[lj] : -INFINITY;
                const double pb2 = cur.ptot[j] + lp_blank;
                const double a1 = cur.pnb[j] + lpl;
                double a2 = -INFINITY;
                const int p = par[j];
                if (p >= 0 && lpl > -INFINITY) {
                    const int32_t lpar = cur.last[p];
                    const double src = (lpar == lj) ? cur.pb[p] : cur.ptot[p];
                    a2 = src + lpl + lm_term(lpar, lj);
                }
                const double pnb2 = lse2(a1, a2);
                st_pb[j] = pb2;
                st_pnb[j] = pnb2;
                st_tot[j] = lse2(pb2, pnb2);
            }
            __syncthreads();

            // virtual candidate c: [0, n_live) stay, then n_live*Knb extensions
            const int n_virtual = n_live + n_live * Knb;
            auto cand_score = [&](int c, int& src_entry, int32_t& tok) -> double {
                if (c < n_live) {
                    src_entry = c;
                    tok = -1;
                    return st_tot[c];
                }
                const int e = c - n_live;
                const int i = e / Knb;
                const int k = e - i * Knb;
                const int32_t s = s_tok[nb0 + k];
                src_entry = i;
                tok = s;
                const int32_t li = cur.last[i];
                int guard = 0;
                for (int kid = first_kid[i]; kid >= 0 && guard < kMaxBeam; kid = next_kid[kid], ++guard)
                    if (cur.last[kid] == s) return -INFINITY;  // merged into that beam entry
                const double src = (s == li) ? cur.pb[i] : cur.ptot[i];
                return src + (double)dense_lp[s] + lm_term(li, s);
            };
            auto cand_hash = [&](int src_entry, int32_t tok) -> uint64_t {
                return tok < 0 ? cur.h[src_entry] : child_hash(cur.h[src_entry], tok);
            };

            // upper bound of every candidate score -> reference key
            const double ref = key_value(sh_kmax) + (double)hd.top + lm_ub + 1.0986122886681098 + 1e-3;
            const uint64_t Rk = order_key(ref);

            // ---- selection: find (selD, selH); keep D < selD or (D == selD and hash <= selH)
            uint64_t selD = kAllOnes, selH = kAllOnes;
            {
                // initial bucket width from the spread of the current beam
                const double est_low = key_value(sh_kmin) + (double)hd.top - 2.0;
                uint64_t Dest = Rk - order_key(est_low);
                if (Dest < 1024) Dest = 1024;
                int sh = 64 - __clzll((long long)Dest) - 10;
                if (sh < 0) sh = 0;
                if (sh > kMaxShift) sh = kMaxShift;
                uint64_t lo = 0;
                int need = beam;
                int mode = 0;  // 0: window over score distance, 1: window over hash at D == Dfix
                uint64_t Dfix = 0;
                bool first = true;
                for (int iter = 0; iter < 40; ++iter) {
                    uint32_t* H = hist[hist_pass % 3];
                    uint32_t* Hz = hist[(hist_pass + 1) % 3];
                    ++hist_pass;
                    for (int i = tid; i < kBins; i += kThreads) Hz[i] = 0u;
                    for (int c = tid; c < n_virtual; c += kThreads) {
                        int se;
                        int32_t tk;
                        const double sc = cand_score(c, se, tk);
                        if (!(sc > -INFINITY)) continue;
                        const uint64_t D = Rk - order_key(sc);
                        uint64_t x;
                        if (mode == 0) {
                            x = D;
                        } else {
                            if (D != Dfix) continue;
                            x = cand_hash(se, tk);
                        }
                        if (x < lo) continue;
                        uint64_t q = (x - lo) >> sh;
                        const int bin = q > (uint64_t)(kBins - 1) ? (kBins - 1) : (int)q;
                        atomicAdd(&H[bin_slot(bin)], 1u);
                    }
                    __syncthreads();
                    // every wave scans the histogram redundantly (results are uniform)
                    uint32_t v[kBinsPerLane];
                    uint32_t s = 0;
#pragma unroll
                    for (int q = 0; q < kBinsPerLane; ++q) {
                        v[q] = H[q * kWave + lane];
                        s += v[q];
                    }
                    uint32_t incl = s;
#pragma unroll
                    for (int o = 1; o < kWave; o <<= 1) {
                        const uint32_t up = __shfl_up(incl, o, kWave);
                        if (lane >= o) incl += up;
                    }
                    const uint32_t excl = incl - s;
                    const int total = (int)__shfl(incl, kWave - 1, kWave);
                    if (first) {
                        first = false;
                        if (tid == 0) {
                            st_cand += (uint64_t)total;
                            if ((uint64_t)total > st_peak) st_peak = (uint64_t)total;
                        }
                    }
                    if (tid == 0) st_pass++;
                    if (total <= need) {  // everything left in the window is kept
                        if (mode == 0) {
                            selD = kAllOnes;
                            selH = kAllOnes;
                        } else {
                            selD = Dfix;
                            selH = kAllOnes;
                        }
                        break;
                    }
                    const bool here = (excl < (uint32_t)need) && ((uint32_t)need <= incl);
                    const uint64_t hm = __ballot(here);
                    const int src_lane = __ffsll((long long)hm) - 1;
                    int bstar = 0, n_above = 0, n_b = 0;
                    if (here) {
                        uint32_t cum = excl;
#pragma unroll
                        for (int q = 0; q < kBinsPerLane; ++q) {
                            if (n_b == 0 && cum + v[q] >= (uint32_t)need) {
                                bstar = lane * kBinsPerLane + q;
                                n_above = (int)cum;
                                n_b = (int)v[q];
                            }
                            cum += v[q];
                        }
                    }
                    bstar = __shfl(bstar, src_lane, kWave);
                    n_above = __shfl(n_above, src_lane, kWave);
                    n_b = __shfl(n_b, src_lane, kWave);
                    const int r = need - n_above;  // 1 <= r <= n_b
                    const bool clamp_bin = (bstar == kBins - 1) && (sh < kMaxShift);

                    if (n_b == r) {  // the boundary bucket is taken whole
                        const uint64_t top = clamp_bin ? kAllOnes : bucket_top(lo, bstar, sh);
                        if (mode == 0) {
                            selD = top;
                            selH = kAllOnes;
                        } else {
                            selD = Dfix;
                            selH = top;
                        }
                        break;
                    }
                    if (n_b <= kExactCap) {
                        // ---- exact ranking of the boundary bucket by (distance, hash)
                        if (tid == 0) st_exact++;
                        for (int c = tid; c < n_virtual; c += kThreads) {
                            int se;
                            int32_t tk;
                            const double sc = cand_score(c, se, tk);
                            if (!(sc > -INFINITY)) continue;
                            const uint64_t D = Rk - order_key(sc);
                            uint64_t x;
                            uint64_t hh = 0;
                            bool have_h = false;
                            if (mode == 0) {
                                x = D;
                            } else {
                                if (D != Dfix) continue;
                                hh = cand_hash(se, tk);
                                have_h = true;
                                x = hh;
                            }
                            if (x < lo) continue;
                            uint64_t q = (x - lo) >> sh;
                            const int bin = q > (uint64_t)(kBins - 1) ? (kBins - 1) : (int)q;
                            if (bin != bstar) continue;
                            if (!have_h) hh = cand_hash(se, tk);
                            const int pos = atomicAdd(&sh_blcount, 1);
                            if (pos < kExactCap) {
                                bl_D[pos] = D;
                                bl_h[pos] = hh;
                            }
                        }
                        __syncthreads();
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
                        __syncthreads();
                        selD = sh_selD;
                        selH = sh_selH;
                        if (tid == 0) sh_blcount = 0;
                        break;
                    }
                    // ---- boundary bucket too large: narrow (or widen) the window
                    need = r;
                    if (clamp_bin) {
                        lo = sat_add(lo, (uint64_t)(kBins - 1) << sh);
                        sh = min(kMaxShift, sh + 8);
                    } else if (sh > 0) {
                        lo = sat_add(lo, (uint64_t)bstar << sh);
                        sh = max(0, sh - 10);
                    } else if (mode == 0) {
                        // more than kExactCap candidates share one score: order them by hash
                        Dfix = lo + (uint64_t)bstar;
                        mode = 1;
                        lo = 0;
                        sh = kMaxShift;
                    } else {
                        // identical score and identical hash (collision): keep them all
                        selD = Dfix;
                        selH = lo + (uint64_t)bstar;
                        break;
                    }
                }
            }

            // ---- compaction: selected candidates become the next beam ------------
            for (int c0 = 0; c0 < n_virtual; c0 += kThreads) {
                const int c = c0 + tid;
                bool sel = false;
                int se = 0;
                int32_t tk = -1;
                double sc = -INFINITY;
                uint64_t hh = 0;
                bool have_h = false;
                if (c < n_virtual) {
                    sc = cand_score(c, se, tk);
                    if (sc > -INFINITY) {
                        const uint64_t D = Rk - order_key(sc);
                        if (D < selD) {
                            sel = true;
                        } else if (D == selD) {
                            hh = cand_hash(se, tk);
                            have_h = true;
                            sel = hh <= selH;
                        }
                    }
                }
                const uint64_t m_sel = __ballot(sel);
                const uint64_t m_ext = __ballot(sel && tk >= 0);
                if (m_sel == 0) continue;
                int slot_base = 0, node_base = 0;
                const int leader = __ffsll((long long)m_sel) - 1;
                if (lane == leader) {
                    slot_base = atomicAdd(&sh_nnew, __popcll(m_sel));
                    if (m_ext) node_base = atomicAdd(&sh_nodes, __popcll(m_ext));
                }
                slot_base = __shfl(slot_base, leader, kWave);
                node_base = __shfl(node_base, leader, kWave);
                if (!sel) continue;
                const int slot = slot_base + lanes_below(m_sel, lane);
                if (slot >= beam) continue;  // only after a hash collision; counted below
                if (tk < 0) {
                    nxt.h[slot] = cur.h[se];
                    nxt.hp[slot] = cur.hp[se];
                    nxt.pb[slot] = st_pb[se];
                    nxt.pnb[slot] = st_pnb[se];
                    nxt.ptot[slot] = sc;
                    nxt.last[slot] = cur.last[se];
                    nxt.node[slot] = cur.node[se];
                    nxt.plen[slot] = cur.plen[se];
                } else {
                    if (!have_h) hh = cand_hash(se, tk);
                    const int node = node_base + lanes_below(m_ext, lane);
                    nxt.h[slot] = hh;
                    nxt.hp[slot] = cur.h[se];
                    nxt.pb[slot] = -INFINITY;
                    nxt.pnb[slot] = sc;
                    nxt.ptot[slot] = sc;
                    nxt.last[slot] = tk;
                    nxt.node[slot] = node;
                    nxt.plen[slot] = cur.plen[se] + 1;
                    TrieNode tn;
                    tn.parent = cur.node[se];
                    tn.tok = tk;
                    if ((int64_t)node < a.trie_stride) trie[node] = tn;
                }
            }
            __syncthreads();

            // ---- adopt the new beam; rebuild parent links ------------------------
            int n_new = sh_nnew;
            if (n_new > beam) {
                if (tid == 0) st_drop += (uint64_t)(n_new - beam);
                n_new = beam;
            }
            if (tid == 0) st_beam += (uint64_t)n_new;
            for (int i = tid; i < kHashSlots; i += kThreads) ht[i] = -1;
            if (tid < kMaxBeam) first_kid[tid] = -1;
            __syncthreads();
            if (tid == 0) {
                sh_nnew = 0;
                sh_kmax = 0;
                sh_kmin = kAllOnes;
            }
            if (tid < n_new) {
                uint32_t slot = (uint32_t)nxt.h[tid] & (kHashSlots - 1);
                for (int probe = 0; probe < kHashSlots; ++probe) {
                    if (atomicCAS(&ht[slot], -1, tid) == -1) break;
                    slot = (slot + 1) & (kHashSlots - 1);
                }
            }
            __syncthreads();
            if (tid < n_new) {
                int p = -1;
                if (nxt.plen[tid] > 0) {
                    const uint64_t want = nxt.hp[tid];
                    uint32_t slot = (uint32_t)want & (kHashSlots - 1);
                    for (int probe = 0; probe < kHashSlots; ++probe) {
                        const int v = ht[slot];
                        if (v < 0) break;
                        if (nxt.h[v] == want) {
                            p = v;
                            break;
                        }
                        slot = (slot + 1) & (kHashSlots - 1);
                    }
                }
                par[tid] = p;
                if (p >= 0) next_kid[tid] = atomicExch(&first_kid[p], tid);
                const uint64_t k = order_key(nxt.ptot[tid]);
                atomicMax((unsigned long long*)&sh_kmax, (unsigned long long)k);
                atomicMin((unsigned long long*)&sh_kmin, (unsigned long long)k);
            }
            n_live = n_new;
            cur_i ^= 1;
        }

        // un-stage the frame's survivors (every read of dense_lp is behind a barrier above
        // or, when the beam is dead, there were none)
        for (int k = tid; k < K; k += kThreads) dense_lp[s_tok[k]] = -INFINITY;
        if (tid == 0) st_surv += (uint64_t)K;
        __syncthreads();
    }

    // ---- best prefix (paper: GetHighestScorePrefix) ----------------------------------
    BeamSlab& fin = slab[cur_i];
    if (tid == 0) {
        sh_kmax = 0;
        sh_selH = kAllOnes;
        sh_best = -1;
    }
    __syncthreads();
    if (tid < n_live) atomicMax((unsigned long long*)&sh_kmax, (unsigned long long)order_key(fin.ptot[tid]));
    __syncthreads();
    if (tid < n_live && order_key(fin.ptot[tid]) == sh_kmax)
        atomicMin((unsigned long long*)&sh_selH, (unsigned long long)fin.h[tid]);
    __syncthreads();
    if (tid < n_live && order_key(fin.ptot[tid]) == sh_kmax && fin.h[tid] == sh_selH) sh_best = tid;
    __syncthreads();

    if (tid == 0) {
        const int best = sh_best;
        if (best < 0) {
            a.out_lengths[b] = 0;
            a.out_scores[b] = -INFINITY;
        } else {
            const int n = fin.plen[best];
            a.out_lengths[b] = n;
            a.out_scores[b] = (float)fin.ptot[best];
            int node = fin.node[best];
            int32_t* dst = a.out_tokens + (int64_t)b * a.T;
            for (int p = n - 1; p >= 0 && node > 0 && (int64_t)node < a.trie_stride; --p) {
                const TrieNode tn = trie[node];
                dst[p] = tn.tok;
                node = tn.parent;
            }
        }
        if (a.stats) {
            atomicAdd((unsigned long long*)&a.stats->frames, (unsigned long long)len);
            atomicAdd((unsigned long long*)&a.stats->sum_survivors, (unsigned long long)st_surv);
            atomicAdd((unsigned long long*)&a.stats->sum_candidates, (unsigned long long)st_cand);
            atomicMax((unsigned long long*)&a.stats->peak_candidates, (unsigned long long)st_peak);
            atomicAdd((unsigned long long*)&a.stats->sum_beam, (unsigned long long)st_beam);
            atomicAdd((unsigned long long*)&a.stats->select_passes, (unsigned long long)st_pass);
            atomicAdd((unsigned long long*)&a.stats->exact_rankings, (unsigned long long)st_exact);
            atomicAdd((unsigned long long*)&a.stats->overflow_drops, (unsigned long long)st_drop);
        }
    }

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
            const int n = fin.plen[tid];
            a.nbest_lengths[row] = n;
            a.nbest_pb[row] = fin.pb[tid];
            a.nbest_pnb[row] = fin.pnb[tid];
            int node = fin.node[tid];
            int32_t* dst = a.nbest_tokens + row * a.T;
            for (int p = n - 1; p >= 0 && node > 0 && (int64_t)node < a.trie_stride; --p) {
                const TrieNode tn = trie[node];
                dst[p] = tn.tok;
                node = tn.parent;
            }
        }
    }
}

}  // namespace

hipError_t launch_beam(const int32_t* lengths, int32_t B, int32_t T, int32_t V,
                       const fltop_params& p, const Workspace& ws, int32_t* out_tokens,
                       int32_t* out_lengths, float* out_scores, fltop_stats* stats,
                       hipStream_t stream) {
    BeamArgs a;
    a.lengths = lengths;
    a.hdr = ws.hdr;
    a.rec = ws.rec;
    a.trie = ws.trie;
    a.trie_stride = ws.trie_stride;
    a.lm_table = p.lm_table;
    a.lm_bound = ws.lm_bound;
    a.lm_alpha = (double)p.lm_weight;
    a.lm_beta = (double)p.insertion_bonus;
    a.B = B;
    a.T = T;
    a.V = V;
    a.fpb = frames_per_block(V);
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
    size_t dyn = lm_lds_offset(V);
    if (a.lm_in_lds) dyn += (size_t)V * V * sizeof(float);
    hipLaunchKernelGGL(beam_kernel, dim3((unsigned)B), dim3(kThreads), dyn, stream, a);
    return hipGetLastError();
}

}  // namespace fltop
