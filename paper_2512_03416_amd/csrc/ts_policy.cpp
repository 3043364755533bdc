// Token-Velocity policy functions (host only): the autoscaler's instance counts (Sec. 4.3), the
// Convertible Decoder's prefill velocity and memory reservation (Sec. 4.4) and the router's two
// policies (Sec. 4.5).  Pure functions over caller-owned arrays.
#include "tokenscale_policy.h"

#include <cmath>
#include <limits>

namespace {
constexpr double kNaN = std::numeric_limits<double>::quiet_NaN();

// seconds a new prefill task would wait behind `tokens` in-flight tokens
inline double waiting_time(double tokens, double velocity)
{
    if (tokens == 0.0) return 0.0;
    return velocity > 0.0 ? tokens / velocity : std::numeric_limits<double>::infinity();
}

inline int first_within_slo(const double* inflight, const double* velocity, int n, double slo_s)
{
    for (int i = 0; i < n; ++i)
        if (waiting_time(inflight[i], velocity[i]) <= slo_s) return i;
    return TS_POLICY_NONE;
}
}  // namespace

extern "C" double ts_tv_decode_velocity(const int64_t* request_tokens, int n, double tpot_s)
{
    if (!(tpot_s > 0.0) || n < 0 || (n > 0 && !request_tokens)) return kNaN;
    int64_t released = 0;
    for (int r = 0; r < n; ++r) {
        if (request_tokens[r] < 0) return kNaN;
        released += request_tokens[r];
    }
    return (double)released / tpot_s;
}

extern "C" double ts_tv_prefillers(double lambda, double v_p, double v_bw)
{
    if (!(lambda >= 0.0) || !(v_p > 0.0) || !(v_bw > 0.0)) return kNaN;
    return lambda / std::fmin(v_p, v_bw);
}

extern "C" double ts_tv_decoders(const double* lambda_b, const double* v_d_b, int n, double* per_bucket)
{
    if (n < 0 || (n > 0 && (!lambda_b || !v_d_b))) return kNaN;
    for (int b = 0; b < n; ++b)
        if (!(lambda_b[b] >= 0.0) || !(v_d_b[b] > 0.0)) return kNaN;   // before any output is written
    double i_d = 0.0;
    for (int b = 0; b < n; ++b) {
        const double i_b = lambda_b[b] / v_d_b[b];
        if (per_bucket) per_bucket[b] = i_b;
        i_d += i_b;
    }
    return i_d;
}

extern "C" double ts_tv_regular_decoders(double i_d, double i_d_c)
{
    if (!(i_d >= 0.0) || !(i_d_c >= 0.0)) return kNaN;
    return std::fmax(i_d - i_d_c, 0.0);
}

extern "C" double ts_tv_decode_batch(double available_bytes, double mean_request_bytes)
{
    if (!(available_bytes >= 0.0) || !(mean_request_bytes > 0.0)) return kNaN;
    return available_bytes / mean_request_bytes;
}

extern "C" double ts_tv_convertible_prefill_velocity(double chunk_size, double batch_size, double tpot_slo_s)
{
    if (!(chunk_size >= 0.0) || !(batch_size >= 0.0) || !(tpot_slo_s > 0.0)) return kNaN;
    const double room = chunk_size - batch_size;
    return (room > 0.0 ? room : 0.0) / tpot_slo_s;
}

extern "C" double ts_tv_reserved_memory(double v_d_p, double mem_t_bytes, double ttft_slo_s)
{
    if (!(v_d_p >= 0.0) || !(mem_t_bytes >= 0.0) || !(ttft_slo_s >= 0.0)) return kNaN;
    return v_d_p * mem_t_bytes * ttft_slo_s;
}

extern "C" int ts_tv_largest_chunk(const double* iteration_time_s, int n, double tpot_slo_s)
{
    if (n < 0 || (n > 0 && !iteration_time_s)) return TS_POLICY_INVALID;
    int chosen = TS_POLICY_NONE;
    for (int i = 0; i < n && iteration_time_s[i] <= tpot_slo_s; ++i) chosen = i;   // stops at the first violation (or NaN)
    return chosen;
}

extern "C" int64_t ts_tv_token_bytes(const ts_attn_desc* desc, int num_layers)
{
    if (num_layers < 1 || ts_check_desc(desc) != TS_OK) return 0;
    const int64_t elem = desc->kv_dtype == TS_F32 ? 4 : desc->kv_dtype == TS_BF16 ? 2 : 1;
    return 2 * (int64_t)desc->num_kv_heads * desc->head_dim * elem * num_layers;
}

extern "C" int64_t ts_tv_instances(double requirement)
{
    if (!(requirement >= 0.0) || !std::isfinite(requirement) || requirement > 9.0e18) return TS_POLICY_INVALID;
    return (int64_t)std::ceil(requirement);
}

extern "C" int ts_route_prefill(const double* prefiller_inflight, const double* prefiller_velocity,
                                int n_prefillers, const double* conv_inflight, const double* conv_velocity,
                                int n_conv, double slo_s, int* kind)
{
    if (!kind || n_prefillers < 0 || n_conv < 0 || (n_prefillers > 0 && (!prefiller_inflight || !prefiller_velocity)) ||
        (n_conv > 0 && (!conv_inflight || !conv_velocity)) || !(slo_s >= 0.0))
        return TS_POLICY_INVALID;
    int idx = first_within_slo(prefiller_inflight, prefiller_velocity, n_prefillers, slo_s);
    if (idx >= 0) { *kind = TS_ROUTE_PREFILLER; return idx; }
    idx = first_within_slo(conv_inflight, conv_velocity, n_conv, slo_s);
    if (idx >= 0) { *kind = TS_ROUTE_CONVERTIBLE; return idx; }
    *kind = TS_ROUTE_QUEUE;
    return TS_POLICY_NONE;
}

extern "C" int ts_route_decode(const int32_t* inflight, int n_decoders, int n_types, int type,
                               const uint8_t* convertible, const double* mem_util, double mem_threshold)
{
    if (n_decoders < 0 || n_types < 1 || type < 0 || type >= n_types ||
        (n_decoders > 0 && (!inflight || !convertible || !mem_util)))
        return TS_POLICY_INVALID;
    int best = TS_POLICY_NONE;
    int32_t best_load = 0;
    for (int d = 0; d < n_decoders; ++d) {
        if (convertible[d] && mem_util[d] > mem_threshold) continue;
        const int32_t load = inflight[(int64_t)d * n_types + type];
        if (best < 0 || load < best_load) { best = d; best_load = load; }
    }
    return best;
}
