// C ABI of the FLToP CTC decoder: argument checks, workspace carve-up, launches.
// See include/fltop_ctc.h for the contract of every entry point.
#include <cmath>
#include <mutex>

#include "fltop_internal.h"

namespace {

int check_shapes(int32_t B, int32_t T, int32_t V, int32_t beam) {
    if (B < 1 || T < 1 || V < 2) return FLTOP_ERR_BAD_SHAPE;
    if (V > FLTOP_MAX_VOCAB) return FLTOP_ERR_VOCAB_TOO_BIG;
    if (beam < 1 || beam > FLTOP_MAX_BEAM) return FLTOP_ERR_BAD_BEAM;
    if (beam > fltop::kBeamInLds && V > FLTOP_MAX_VOCAB_WIDE_BEAM) return FLTOP_ERR_BAD_BEAM;
    // trie node ids (1 + frame * beam + slot) are 32-bit
    if ((int64_t)T * beam + 1 > (int64_t)INT32_MAX) return FLTOP_ERR_BAD_SHAPE;
    return FLTOP_OK;
}

int check_threshold(float r) {
    if (!(r >= 0.0f && r <= 1.0f)) return FLTOP_ERR_BAD_THRESHOLD;  // NaN fails both
    return FLTOP_OK;
}

int check_options(int32_t top_n, double beam_threshold) {
    if (top_n < 0 || beam_threshold != beam_threshold) return FLTOP_ERR_BAD_OPTION;
    return FLTOP_OK;
}

int check_workspace(const void* ws, size_t bytes, size_t need) {
    if (!ws) return FLTOP_ERR_NULL_POINTER;
    if ((reinterpret_cast<uintptr_t>(ws) & 255u) != 0) return FLTOP_ERR_ALIGNMENT;
    if (bytes < need) return FLTOP_ERR_WORKSPACE;
    return FLTOP_OK;
}

// The caller's workspace laid out for these shapes: the fixed regions, and behind them as many
// survivor records as the remaining bytes hold.
int lay_out(void* workspace, size_t bytes, int32_t B, int32_t T, int32_t V, int32_t beam,
            fltop::Workspace* ws) {
    if (!workspace) return FLTOP_ERR_NULL_POINTER;
    if ((reinterpret_cast<uintptr_t>(workspace) & 255u) != 0) return FLTOP_ERR_ALIGNMENT;
    const int64_t records = fltop::records_that_fit(bytes, B, T, V, beam);
    if (records < 0) return FLTOP_ERR_WORKSPACE;
    *ws = fltop::carve_workspace(workspace, B, T, V, beam, (uint64_t)records);
    return FLTOP_OK;
}

// ln(R) rounded to fp32 once; R = 0 keeps everything.
float ln_threshold(float r) {
    if (r <= 0.0f) return -INFINITY;
    return (float)std::log((double)r);
}

}  // namespace

extern "C" size_t fltop_ctc_workspace_bytes_for(int32_t B, int32_t T, int32_t V, int32_t beam,
                                                uint64_t max_records) {
    if (check_shapes(B, T, V, beam) != FLTOP_OK) return 0;
    // the budget asked for (never more than the shapes can need), plus the slack that makes
    // all of it usable, rounded up to whole slices
    const uint64_t most = fltop::worst_case_records(B, T, V);
    uint64_t n = (max_records < most ? max_records : most);
    if (n > 0) n += fltop::record_slack(V);
    n = (n + fltop::kRecArenas - 1) / fltop::kRecArenas * fltop::kRecArenas;
    return fltop::carve_workspace(nullptr, B, T, V, beam, n).bytes;
}

extern "C" size_t fltop_ctc_workspace_bytes(int32_t B, int32_t T, int32_t V, int32_t beam) {
    return fltop_ctc_workspace_bytes_for(B, T, V, beam, ~0ull);
}

extern "C" int fltop_ctc_prune(const float* logprobs, const int32_t* lengths, int32_t B, int32_t T,
                               int32_t V, int32_t beam, float rel_threshold, int32_t top_n,
                               void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (!logprobs || !lengths) return FLTOP_ERR_NULL_POINTER;
    int rc = check_shapes(B, T, V, beam);
    if (rc != FLTOP_OK) return rc;
    rc = check_threshold(rel_threshold);
    if (rc != FLTOP_OK) return rc;
    rc = check_options(top_n, 0.0);
    if (rc != FLTOP_OK) return rc;
    fltop::Workspace ws;
    rc = lay_out(workspace, workspace_bytes, B, T, V, beam, &ws);
    if (rc != FLTOP_OK) return rc;
    hipError_t e = fltop::launch_prune(logprobs, lengths, B, T, V, ln_threshold(rel_threshold),
                                       top_n, ws, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? FLTOP_OK : FLTOP_ERR_HIP;
}

extern "C" int fltop_ctc_unpack_survivors(const void* workspace, size_t workspace_bytes,
                                          const int32_t* lengths, int32_t B, int32_t T,
                                          int32_t V, int32_t beam, int32_t* counts,
                                          int32_t* tokens, float* values, float* frame_max,
                                          void* hip_stream) {
    if (!lengths || !counts || !tokens || !values) return FLTOP_ERR_NULL_POINTER;
    int rc = check_shapes(B, T, V, beam);
    if (rc != FLTOP_OK) return rc;
    fltop::Workspace ws;
    rc = lay_out(const_cast<void*>(workspace), workspace_bytes, B, T, V, beam, &ws);
    if (rc != FLTOP_OK) return rc;
    hipError_t e = fltop::launch_unpack(ws, lengths, B, T, V, counts, tokens, values, frame_max,
                                        static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? FLTOP_OK : FLTOP_ERR_HIP;
}

namespace {

int check_nbest(const fltop_params* p) {
    const bool any = p->nbest_count || p->nbest_tokens || p->nbest_lengths || p->nbest_pb ||
                     p->nbest_pnb;
    const bool all = p->nbest_count && p->nbest_tokens && p->nbest_lengths && p->nbest_pb &&
                     p->nbest_pnb;
    return (any && !all) ? FLTOP_ERR_NULL_POINTER : FLTOP_OK;
}

int enqueue_search(const int32_t* lengths, int32_t B, int32_t T, int32_t V,
                   const fltop_params* params, const fltop::Workspace& ws,
                   const fltop::StreamSpace* carried, int32_t* out_tokens, int32_t* out_lengths,
                   float* out_scores, fltop_stats* stats, hipStream_t stream) {
    hipError_t e = hipSuccess;
    if (params->lm_table) {
        e = fltop::launch_lm_bound(params->lm_table, V, params->lm_weight, params->insertion_bonus,
                                   ws.lm_bound, stream);
        if (e != hipSuccess) return FLTOP_ERR_HIP;
    }
    e = fltop::launch_beam(lengths, B, T, V, *params, ws, carried, out_tokens, out_lengths,
                           out_scores, stats, stream);
    return e == hipSuccess ? FLTOP_OK : FLTOP_ERR_HIP;
}

}  // namespace

extern "C" int fltop_ctc_search(const int32_t* lengths, int32_t B, int32_t T, int32_t V,
                                const fltop_params* params, void* workspace,
                                size_t workspace_bytes, int32_t* out_tokens, int32_t* out_lengths,
                                float* out_scores, fltop_stats* stats, void* hip_stream) {
    if (!lengths || !params || !out_tokens || !out_lengths || !out_scores)
        return FLTOP_ERR_NULL_POINTER;
    int rc = check_shapes(B, T, V, params->beam);
    if (rc != FLTOP_OK) return rc;
    rc = check_options(0, params->beam_threshold);
    if (rc != FLTOP_OK) return rc;
    rc = check_nbest(params);
    if (rc != FLTOP_OK) return rc;
    fltop::Workspace ws;
    rc = lay_out(workspace, workspace_bytes, B, T, V, params->beam, &ws);
    if (rc != FLTOP_OK) return rc;
    return enqueue_search(lengths, B, T, V, params, ws, nullptr, out_tokens, out_lengths,
                          out_scores, stats, static_cast<hipStream_t>(hip_stream));
}

extern "C" int fltop_ctc_decode(const float* logprobs, const int32_t* lengths, int32_t B, int32_t T,
                                int32_t V, const fltop_params* params, void* workspace,
                                size_t workspace_bytes, int32_t* out_tokens, int32_t* out_lengths,
                                float* out_scores, fltop_stats* stats, void* hip_stream) {
    if (!logprobs || !lengths || !params || !out_tokens || !out_lengths || !out_scores)
        return FLTOP_ERR_NULL_POINTER;
    int rc = check_shapes(B, T, V, params->beam);
    if (rc != FLTOP_OK) return rc;
    rc = check_threshold(params->rel_threshold);
    if (rc != FLTOP_OK) return rc;
    rc = check_options(params->top_n, params->beam_threshold);
    if (rc != FLTOP_OK) return rc;
    rc = check_nbest(params);
    if (rc != FLTOP_OK) return rc;
    fltop::Workspace ws;
    rc = lay_out(workspace, workspace_bytes, B, T, V, params->beam, &ws);
    if (rc != FLTOP_OK) return rc;

    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    hipError_t e = fltop::launch_prune(logprobs, lengths, B, T, V,
                                       ln_threshold(params->rel_threshold), params->top_n, ws,
                                       stream);
    if (e != hipSuccess) return FLTOP_ERR_HIP;
    return enqueue_search(lengths, B, T, V, params, ws, nullptr, out_tokens, out_lengths,
                          out_scores, stats, stream);
}

// ---- decode for callers that cannot allocate -------------------------------------------
// The workspace of fltop_ctc_decode_static: one array in the library's own device image,
// which every GPU the library runs on holds at its own address until the process ends.
// `scratch` itself is only the host-side handle of that array; the device address is asked
// for once per device (fetch_scratch) and only that address is ever handed to a kernel.
static __device__ __align__(256) unsigned char scratch[FLTOP_STATIC_SCRATCH_BYTES];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_lock;
void* g_scratch_at[kMaxDevices] = {};  // device address of `scratch`, per device

// Device address of `scratch` on the current device, or nullptr with *err set.
void* fetch_scratch(hipError_t* err) {
    int dev = 0;
    *err = hipGetDevice(&dev);
    if (*err != hipSuccess) return nullptr;
    if (dev < 0 || dev >= kMaxDevices) {
        *err = hipErrorInvalidDevice;
        return nullptr;
    }
    std::lock_guard<std::mutex> hold(g_scratch_lock);
    if (!g_scratch_at[dev]) {
        void* at = nullptr;
        *err = hipGetSymbolAddress(&at, HIP_SYMBOL(scratch));
        if (*err != hipSuccess || !at) {
            if (*err == hipSuccess) *err = hipErrorInvalidSymbol;
            return nullptr;
        }
        g_scratch_at[dev] = at;
    }
    return g_scratch_at[dev];
}

}  // namespace

extern "C" int fltop_ctc_decode_static(const float* logprobs, const int32_t* lengths, int32_t B,
                                       int32_t T, int32_t V, const fltop_params* params,
                                       int32_t* out_tokens, int32_t* out_lengths,
                                       float* out_scores, fltop_stats* stats, void* hip_stream) {
    if (!params) return FLTOP_ERR_NULL_POINTER;
    // what the shapes need whatever the survivor lists hold; records take the rest of the array
    const size_t need = fltop_ctc_workspace_bytes_for(B, T, V, params->beam, 0);
    if (need > (size_t)FLTOP_STATIC_SCRATCH_BYTES) return FLTOP_ERR_STATIC_SCRATCH;
    hipError_t e = hipSuccess;
    void* at = fetch_scratch(&e);
    if (!at) return FLTOP_ERR_HIP;
    // need == 0 (bad shapes) falls through to the checks of the plain entry point
    return fltop_ctc_decode(logprobs, lengths, B, T, V, params, at,
                            (size_t)FLTOP_STATIC_SCRATCH_BYTES, out_tokens, out_lengths,
                            out_scores, stats, hip_stream);
}

extern "C" size_t fltop_ctc_stream_state_bytes(int32_t B, int32_t T_total, int32_t beam) {
    if (check_shapes(B, T_total, 2, beam) != FLTOP_OK || beam > fltop::kBeamInLds) return 0;
    return fltop::carve_stream(nullptr, B, T_total, beam).bytes;
}

extern "C" int fltop_ctc_stream_begin(void* state, size_t state_bytes, int32_t B, int32_t T_total,
                                      int32_t beam, void* hip_stream) {
    int rc = check_shapes(B, T_total, 2, beam);
    if (rc != FLTOP_OK) return rc;
    if (beam > fltop::kBeamInLds) return FLTOP_ERR_BAD_BEAM;  // the carried record is laid out for 512
    rc = check_workspace(state, state_bytes, fltop_ctc_stream_state_bytes(B, T_total, beam));
    if (rc != FLTOP_OK) return rc;
    const fltop::StreamSpace sp = fltop::carve_stream(state, B, T_total, beam);
    hipError_t e =
        fltop::launch_stream_begin(sp, B, beam, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? FLTOP_OK : FLTOP_ERR_HIP;
}

extern "C" int fltop_ctc_stream_decode(const float* logprobs, const int32_t* lengths, int32_t B,
                                       int32_t T_chunk, int32_t V, const fltop_params* params,
                                       void* workspace, size_t workspace_bytes, void* state,
                                       size_t state_bytes, int32_t T_total, int32_t* out_tokens,
                                       int32_t* out_lengths, float* out_scores,
                                       fltop_stats* stats, void* hip_stream) {
    if (!logprobs || !lengths || !params || !out_tokens || !out_lengths || !out_scores)
        return FLTOP_ERR_NULL_POINTER;
    int rc = check_shapes(B, T_chunk, V, params->beam);
    if (rc != FLTOP_OK) return rc;
    if (params->beam > fltop::kBeamInLds) return FLTOP_ERR_BAD_BEAM;
    if (T_total < T_chunk) return FLTOP_ERR_BAD_SHAPE;
    rc = check_threshold(params->rel_threshold);
    if (rc != FLTOP_OK) return rc;
    rc = check_options(params->top_n, params->beam_threshold);
    if (rc != FLTOP_OK) return rc;
    rc = check_nbest(params);
    if (rc != FLTOP_OK) return rc;
    fltop::Workspace ws;
    rc = lay_out(workspace, workspace_bytes, B, T_chunk, V, params->beam, &ws);
    if (rc != FLTOP_OK) return rc;
    rc = check_workspace(state, state_bytes,
                         fltop_ctc_stream_state_bytes(B, T_total, params->beam));
    if (rc != FLTOP_OK) return rc;

    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const fltop::StreamSpace sp = fltop::carve_stream(state, B, T_total, params->beam);
    hipError_t e = fltop::launch_prune(logprobs, lengths, B, T_chunk, V,
                                       ln_threshold(params->rel_threshold), params->top_n, ws,
                                       stream);
    if (e != hipSuccess) return FLTOP_ERR_HIP;
    return enqueue_search(lengths, B, T_chunk, V, params, ws, &sp, out_tokens, out_lengths,
                          out_scores, stats, stream);
}

extern "C" int fltop_ctc_token_ranks(const float* logprobs, int32_t B, int32_t T, int32_t V,
                                     const int32_t* tokens, const int32_t* token_frames,
                                     const int32_t* token_counts, int32_t* out_ranks,
                                     uint64_t* rank_count, double* rank_lp_sum,
                                     void* hip_stream) {
    if (!logprobs || !tokens || !token_frames || !token_counts) return FLTOP_ERR_NULL_POINTER;
    if (B < 1 || T < 1 || V < 2) return FLTOP_ERR_BAD_SHAPE;
    if (V > FLTOP_MAX_VOCAB) return FLTOP_ERR_VOCAB_TOO_BIG;
    hipError_t e = fltop::launch_token_ranks(logprobs, B, T, V, tokens, token_frames,
                                             token_counts, out_ranks, rank_count, rank_lp_sum,
                                             static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? FLTOP_OK : FLTOP_ERR_HIP;
}

extern "C" int fltop_ctc_log_add(const double* a, const double* b, double* out, int64_t n,
                                 void* hip_stream) {
    if (n < 0) return FLTOP_ERR_BAD_SHAPE;
    if (n > 0 && (!a || !b || !out)) return FLTOP_ERR_NULL_POINTER;
    hipError_t e = fltop::launch_log_add(a, b, out, n, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? FLTOP_OK : FLTOP_ERR_HIP;
}

extern "C" const char* fltop_status_string(int status) {
    switch (status) {
        case FLTOP_OK: return "ok";
        case FLTOP_ERR_NULL_POINTER: return "a required pointer is NULL";
        case FLTOP_ERR_BAD_SHAPE: return "bad shape: need B >= 1, T >= 1, V >= 2, T * beam < 2^31";
        case FLTOP_ERR_BAD_BEAM:
            return "beam outside 1..FLTOP_MAX_BEAM (or above 512 with V > 2048 or with streaming)";
        case FLTOP_ERR_BAD_THRESHOLD: return "rel_threshold outside [0,1]";
        case FLTOP_ERR_WORKSPACE: return "workspace too small";
        case FLTOP_ERR_VOCAB_TOO_BIG: return "V exceeds FLTOP_MAX_VOCAB";
        case FLTOP_ERR_HIP: return "HIP launch failed";
        case FLTOP_ERR_ALIGNMENT: return "workspace not 256-byte aligned";
        case FLTOP_ERR_BAD_OPTION: return "top_n negative or beam_threshold NaN";
        case FLTOP_ERR_STATIC_SCRATCH:
            return "shapes need more workspace than FLTOP_STATIC_SCRATCH_BYTES";  // fixed regions
        default: return "unknown status";
    }
}
