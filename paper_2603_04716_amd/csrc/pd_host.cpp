// Host-only entry points: the allocation model (Eqs. (5)-(7), (12), (13)), the single-server FIFO
// replay used by the queue check, status strings and the thread-local error text.
// Compiled with floating-point contraction off so that every product and quotient below is one
// IEEE binary64 operation, in the order the header documents.
#include <math.h>
#include <stdarg.h>
#include <stdio.h>

#include <algorithm>
#include <vector>

#include "pd.h"

namespace pd {
static thread_local char g_err[512] = "";
void set_error(const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}
}  // namespace pd

extern "C" const char *pd_last_error(void) { return pd::g_err; }

extern "C" const char *pd_status_string(pd_status s)
{
    switch (s) {
    case PD_OK: return "ok";
    case PD_ERR_INVALID_ARG: return "invalid argument";
    case PD_ERR_SHAPE: return "unsupported or inconsistent shape";
    case PD_ERR_DTYPE: return "unsupported dtype";
    case PD_ERR_OOM: return "out of device memory";
    case PD_ERR_DEVICE: return "device error";
    case PD_ERR_KV_CAPACITY: return "KV cache capacity exceeded";
    case PD_ERR_TTFT_INFEASIBLE: return "TTFT target infeasible";
    case PD_ERR_TPOT_INFEASIBLE: return "TPOT target infeasible";
    }
    return "unknown status";
}

static bool pos_finite(double v) { return std::isfinite(v) && v > 0.0; }

static int32_t to_count(double n_real, int32_t rounding)
{
    double n = rounding == 0 ? floor(n_real + 0.5) : ceil(n_real);
    if (!(n >= 1.0)) return 1;
    if (n > 2147483647.0) return 2147483647;
    return (int32_t)n;
}

extern "C" pd_status pd_allocate(double tp_total_tps, double l_in, double l_out, double ttft_slo_s,
                                 double tpot_slo_s, const pd_measured_curves *cv, pd_allocation *out)
{
    if (!cv || !out) {
        pd::set_error("pd_allocate: NULL curves or output");
        return PD_ERR_INVALID_ARG;
    }
    if (!pos_finite(tp_total_tps) || !pos_finite(l_in) || !pos_finite(l_out) ||
        !pos_finite(ttft_slo_s) || !pos_finite(tpot_slo_s) || !pos_finite(cv->prefill_max_tps)) {
        pd::set_error("pd_allocate: throughput, lengths and SLOs must be finite and positive");
        return PD_ERR_INVALID_ARG;
    }
    if (!std::isfinite(cv->t_overhead_s) || cv->t_overhead_s < 0.0 ||
        (cv->rounding != 0 && cv->rounding != 1)) {
        pd::set_error("pd_allocate: bad t_overhead_s or rounding mode");
        return PD_ERR_INVALID_ARG;
    }
    if (cv->n_decode <= 0 || !cv->decode_batch || !cv->decode_tpot_s) {
        pd::set_error("pd_allocate: empty decode curve");
        return PD_ERR_INVALID_ARG;
    }
    std::vector<std::pair<int32_t, double>> pts;
    pts.reserve((size_t)cv->n_decode);
    for (int32_t i = 0; i < cv->n_decode; ++i) {
        if (cv->decode_batch[i] <= 0 || !pos_finite(cv->decode_tpot_s[i])) {
            pd::set_error("pd_allocate: curve point %d is not positive and finite", i);
            return PD_ERR_INVALID_ARG;
        }
        pts.emplace_back(cv->decode_batch[i], cv->decode_tpot_s[i]);
    }
    // sort by batch, then TPOT: the first entry of each batch is its smallest TPOT
    std::sort(pts.begin(), pts.end());

    // Eq. (12) and Eq. (13)
    const double t_s = ttft_slo_s - cv->t_overhead_s;
    if (!(t_s > 0.0)) {
        pd::set_error("pd_allocate: TTFT - T_overhead = %g s leaves no time for prefill", t_s);
        return PD_ERR_TTFT_INFEASIBLE;
    }
    const double tp_prefill = cv->prefill_max_tps - l_in / t_s;
    if (!(tp_prefill > 0.0)) {
        pd::set_error("pd_allocate: Eq. (13) gives %g tokens/s; the bare compute time already exceeds the TTFT budget",
                      tp_prefill);
        return PD_ERR_TTFT_INFEASIBLE;
    }

    // largest measured batch meeting the TPOT target
    int32_t b_star = -1;
    double tpot_star = 0.0;
    int32_t non_monotone = 0;
    double prev_tpot = -1.0;
    int32_t prev_b = -1;
    for (const auto &p : pts) {
        if (p.first == prev_b) continue;  // duplicate batch: keep the smaller TPOT seen first
        if (prev_tpot >= 0.0 && p.second < prev_tpot) non_monotone = 1;
        prev_b = p.first;
        prev_tpot = p.second;
        if (p.second <= tpot_slo_s) {
            b_star = p.first;
            tpot_star = p.second;
        }
    }
    if (b_star < 0) {
        pd::set_error("pd_allocate: no measured batch meets TPOT <= %g s", tpot_slo_s);
        return PD_ERR_TPOT_INFEASIBLE;
    }
    const double tp_decode = (double)b_star / tpot_star;

    // Eqs. (5), (6), (7)
    const double n_p = (tp_total_tps * l_in) / ((l_in + l_out) * tp_prefill);
    const double n_d = (tp_total_tps * l_out) / ((l_in + l_out) * tp_decode);
    const double r = (l_in * tp_decode) / (l_out * tp_prefill);

    out->tp_prefill_eff = tp_prefill;
    out->tp_decode_eff = tp_decode;
    out->decode_batch = b_star;
    out->decode_tpot_s = tpot_star;
    out->n_prefill_real = n_p;
    out->n_decode_real = n_d;
    out->ratio_pd = r;
    out->n_prefill = to_count(n_p, cv->rounding);
    out->n_decode = to_count(n_d, cv->rounding);
    out->curve_non_monotone = non_monotone;
    return PD_OK;
}

extern "C" pd_status pd_fifo_replay(int32_t n, const double *arrival_s, const double *service_s,
                                    double *sojourn_s)
{
    if (n < 0 || (n > 0 && (!arrival_s || !service_s || !sojourn_s))) {
        pd::set_error("pd_fifo_replay: bad arguments");
        return PD_ERR_INVALID_ARG;
    }
    double done = -INFINITY, prev_a = -INFINITY;
    for (int32_t i = 0; i < n; ++i) {
        if (!std::isfinite(arrival_s[i]) || !std::isfinite(service_s[i]) || service_s[i] < 0.0 ||
            arrival_s[i] < prev_a) {
            pd::set_error("pd_fifo_replay: request %d has a bad arrival or service time", i);
            return PD_ERR_INVALID_ARG;
        }
        prev_a = arrival_s[i];
    }
    for (int32_t i = 0; i < n; ++i) {
        const double start = arrival_s[i] > done ? arrival_s[i] : done;
        done = start + service_s[i];
        sojourn_s[i] = done - arrival_s[i];
    }
    return PD_OK;
}

extern "C" pd_status pd_allocate_stages(int32_t n_stages, double tp_total_tps, double l_in, double l_out,
                                        const double *work_per_request, const double *stage_tps,
                                        int32_t rounding, double *n_real, int32_t *n_instances)
{
    if (n_stages < 1 || !work_per_request || !stage_tps || !n_real || !n_instances ||
        (rounding != 0 && rounding != 1) || !pos_finite(tp_total_tps) || !pos_finite(l_in) || !pos_finite(l_out)) {
        pd::set_error("pd_allocate_stages: bad arguments");
        return PD_ERR_INVALID_ARG;
    }
    for (int32_t k = 0; k < n_stages; ++k)
        if (!pos_finite(work_per_request[k]) || !pos_finite(stage_tps[k])) {
            pd::set_error("pd_allocate_stages: stage %d has a non-positive work or throughput", k);
            return PD_ERR_INVALID_ARG;
        }
    for (int32_t k = 0; k < n_stages; ++k) {
        const double n = (tp_total_tps * work_per_request[k]) / ((l_in + l_out) * stage_tps[k]);   // Eqs. (5), (6)
        n_real[k] = n;
        n_instances[k] = to_count(n, rounding);
    }
    return PD_OK;
}

extern "C" pd_status pd_fifo_replay_batched(int32_t n, const double *arrival_s, int32_t max_batch,
                                            const double *batch_service_s, double *sojourn_s)
{
    if (n < 0 || max_batch < 1 || !batch_service_s || (n > 0 && (!arrival_s || !sojourn_s))) {
        pd::set_error("pd_fifo_replay_batched: bad arguments");
        return PD_ERR_INVALID_ARG;
    }
    for (int32_t b = 0; b < max_batch; ++b)
        if (!std::isfinite(batch_service_s[b]) || batch_service_s[b] < 0.0) {
            pd::set_error("pd_fifo_replay_batched: bad service time for a batch of %d", b + 1);
            return PD_ERR_INVALID_ARG;
        }
    double prev_a = -INFINITY;
    for (int32_t i = 0; i < n; ++i) {
        if (!std::isfinite(arrival_s[i]) || arrival_s[i] < prev_a) {
            pd::set_error("pd_fifo_replay_batched: request %d has a bad arrival time", i);
            return PD_ERR_INVALID_ARG;
        }
        prev_a = arrival_s[i];
    }
    double free_at = -INFINITY;
    int32_t i = 0;
    while (i < n) {
        const double start = arrival_s[i] > free_at ? arrival_s[i] : free_at;
        int32_t b = 1;
        while (b < max_batch && i + b < n && arrival_s[i + b] <= start) ++b;
        const double done = start + batch_service_s[b - 1];
        for (int32_t j = i; j < i + b; ++j) sojourn_s[j] = done - arrival_s[j];
        free_at = done;
        i += b;
    }
    return PD_OK;
}

extern "C" pd_status pd_prefill_throughput_dp(double prefill_max_tps, double l_in, double ttft_slo_s,
                                              double t_overhead_s, int32_t dp_groups, double *tp_prefill)
{
    if (!tp_prefill || !pos_finite(prefill_max_tps) || !pos_finite(l_in) || !pos_finite(ttft_slo_s) ||
        !std::isfinite(t_overhead_s) || t_overhead_s < 0.0 || dp_groups < 1) {
        pd::set_error("pd_prefill_throughput_dp: bad arguments");
        return PD_ERR_INVALID_ARG;
    }
    const double t_s = ttft_slo_s - t_overhead_s;                       // Eq. (12)
    if (!(t_s > 0.0)) {
        pd::set_error("pd_prefill_throughput_dp: TTFT - T_overhead = %g <= 0", t_s);
        return PD_ERR_TTFT_INFEASIBLE;
    }
    const double per_group = (prefill_max_tps / dp_groups) - (l_in / t_s);   // Eq. (13) of one group
    if (!(per_group > 0.0)) {
        pd::set_error("pd_prefill_throughput_dp: a group's bare compute time exceeds TTFT - T_overhead");
        return PD_ERR_TTFT_INFEASIBLE;
    }
    *tp_prefill = dp_groups * per_group;
    return PD_OK;
}

extern "C" pd_status pd_mg1_sojourn(double lambda_rps, double mean_service_s, double mean_service_sq_s2,
                                    double *t_s)
{
    if (!t_s || !std::isfinite(lambda_rps) || lambda_rps < 0.0 || !pos_finite(mean_service_s) ||
        !pos_finite(mean_service_sq_s2)) {
        pd::set_error("pd_mg1_sojourn: bad arguments");
        return PD_ERR_INVALID_ARG;
    }
    const double rho = lambda_rps * mean_service_s;
    if (!(rho < 1.0)) {
        pd::set_error("pd_mg1_sojourn: utilisation %g >= 1", rho);
        return PD_ERR_TTFT_INFEASIBLE;
    }
    *t_s = mean_service_s + lambda_rps * mean_service_sq_s2 / (2.0 * (1.0 - rho));
    return PD_OK;
}

extern "C" pd_status pd_kv_transfer_overhead(double l_in, int32_t n_layers, int32_t n_kv_heads,
                                             int32_t head_dim, double bytes_per_elem,
                                             double link_bytes_per_s, double fixed_s, double *t_overhead_s)
{
    if (!t_overhead_s || !std::isfinite(l_in) || l_in < 0.0 || n_layers <= 0 || n_kv_heads <= 0 ||
        head_dim <= 0 || !pos_finite(bytes_per_elem) || !pos_finite(link_bytes_per_s) ||
        !std::isfinite(fixed_s) || fixed_s < 0.0) {
        pd::set_error("pd_kv_transfer_overhead: bad arguments");
        return PD_ERR_INVALID_ARG;
    }
    // bytes of keys and values per prompt token over all layers, then the whole prompt over the link
    const double per_token = (double)n_layers * 2.0 * (double)n_kv_heads * (double)head_dim * bytes_per_elem;
    *t_overhead_s = fixed_s + l_in * per_token / link_bytes_per_s;
    return PD_OK;
}

extern "C" pd_status pd_mm1_sojourn(double prefill_max_tps, double l_in, double lambda_rps,
                                    double *t_s)
{
    if (!t_s || !pos_finite(prefill_max_tps) || !pos_finite(l_in) || !std::isfinite(lambda_rps) ||
        lambda_rps < 0.0) {
        pd::set_error("pd_mm1_sojourn: bad arguments");
        return PD_ERR_INVALID_ARG;
    }
    const double mu = prefill_max_tps / l_in;  // Eq. (9)
    if (!(lambda_rps < mu)) {
        pd::set_error("pd_mm1_sojourn: arrival rate %g >= service rate %g", lambda_rps, mu);
        return PD_ERR_TTFT_INFEASIBLE;
    }
    *t_s = 1.0 / (mu - lambda_rps);  // Eq. (12)
    return PD_OK;
}
