// Host-only part of libooco: the roofline latency model of the attention operator
// (paper Section 3.3: operator model of Table 2, operator latency of Equation 1, iteration latency
// = sum of operator latencies + static overhead).  No device code, no device state.
#include "ooco.h"

#include <algorithm>
#include <cstdio>
#include <numeric>
#include <vector>

extern "C" ooco_status ooco_predict_latency(const ooco_model_params *params, int num_q_heads, int num_kv_heads,
                                            int head_dim, int bytes_per_value, int causal_flops, int num_seqs,
                                            const int32_t *h_query_start_loc, const int32_t *h_ctx_lens, double *out,
                                            char *msg, size_t msg_cap)
{
    auto bad = [&](ooco_status code, const char *text) {
        if (msg && msg_cap) snprintf(msg, msg_cap, "ooco_predict_latency: %s", text);
        return code;
    };
    if (msg && msg_cap) msg[0] = 0;
    if (!params || !out) return bad(OOCO_EINVAL, "NULL params or out");
    if (!(params->F_ap > 0) || !(params->F_ad > 0) || !(params->M_a > 0) || !(params->O_p >= 0) || !(params->O_d >= 0))
        return bad(OOCO_EINVAL, "F_ap, F_ad, M_a must be positive and O_p, O_d non-negative");
    if (num_q_heads <= 0 || num_kv_heads <= 0 || num_q_heads % num_kv_heads || head_dim <= 0 || bytes_per_value <= 0)
        return bad(OOCO_ESHAPE, "bad head geometry");
    if (num_seqs < 0 || (num_seqs > 0 && (!h_query_start_loc || !h_ctx_lens))) return bad(OOCO_EINVAL, "bad length arrays");
    const double D_h = (double)num_q_heads * head_dim, d = bytes_per_value;
    const double kv_ratio = (double)num_kv_heads / num_q_heads;
    double t_p = 0, t_d = 0, flops = 0, bytes = 0, t_c = 0, t_m = 0;
    bool any_p = false, any_d = false;
    for (int i = 0; i < num_seqs; ++i) {
        const int64_t ql = (int64_t)h_query_start_loc[i + 1] - h_query_start_loc[i];
        if (ql < 0 || h_ctx_lens[i] < 0) return bad(OOCO_ESHAPE, "negative length");
        if (ql == 0) continue;
        const double S_q = (double)ql, S_kv = (double)h_ctx_lens[i] + (double)ql;
        // Table 2, attention row; optionally only the (row, key) pairs a causal kernel visits
        const double f = causal_flops ? 4.0 * D_h * (S_q * (double)h_ctx_lens[i] + S_q * (S_q + 1.0) / 2.0) : 4.0 * D_h * S_q * S_kv;
        const double b = 2.0 * d * (S_q * D_h + S_kv * D_h * kv_ratio);
        const double tf = f / (ql > 1 ? params->F_ap : params->F_ad), tb = b / params->M_a;
        const double t = tf >= tb ? tf : tb;                                  // Equation 1
        (tf >= tb ? t_c : t_m) += t;
        if (ql > 1) {
            t_p += t;
            any_p = true;
        } else {
            t_d += t;
            any_d = true;
        }
        flops += f;
        bytes += b;
    }
    const double overhead = (any_p ? params->O_p : 0.0) + (any_d ? params->O_d : 0.0);
    out[0] = t_p + t_d + overhead;
    out[1] = t_p;
    out[2] = t_d;
    out[3] = overhead;
    out[4] = flops;
    out[5] = bytes;
    out[6] = t_c;
    out[7] = t_m;
    return OOCO_OK;
}

namespace {
// Latency of one decode operator over n keys (Table 2 with S_q = 1, Equation 1).
double decode_op_time(const ooco_model_params &p, double D_h, double kv_ratio, double d, double n)
{
    const double f = 4.0 * D_h * n, b = 2.0 * d * (D_h + n * D_h * kv_ratio);
    const double tf = f / p.F_ad, tb = b / p.M_a;
    return tf >= tb ? tf : tb;
}
}  // namespace

// Mix Decoding Selection (paper Algorithm 2).  L(B) of a decode-only batch is the sum of its operators' times
// plus O_d, so the batch latency is kept as a running sum: one look costs O(1), the sorted phase one sort, one
// prefix sum and a bisection.  The sums are accumulated in the same order as a from-scratch evaluation of the
// batch (online requests, accepted looks in order, then the sorted prefix).
extern "C" ooco_status ooco_mix_decoding_select(const ooco_model_params *params, int num_q_heads, int num_kv_heads,
                                                int head_dim, int bytes_per_value, double slo_s, int num_online,
                                                const int32_t *h_online_lens, int num_offline,
                                                const int32_t *h_offline_lens, int num_looks, const int32_t *h_random_order,
                                                uint8_t *h_selected, double *latency_out, char *msg, size_t msg_cap)
{
    auto bad = [&](ooco_status code, const char *text) {
        if (msg && msg_cap) snprintf(msg, msg_cap, "ooco_mix_decoding_select: %s", text);
        return code;
    };
    if (msg && msg_cap) msg[0] = 0;
    if (!params) return bad(OOCO_EINVAL, "NULL params");
    if (!(params->F_ad > 0) || !(params->M_a > 0) || !(params->O_d >= 0)) return bad(OOCO_EINVAL, "F_ad, M_a must be positive, O_d non-negative");
    if (num_q_heads <= 0 || num_kv_heads <= 0 || num_q_heads % num_kv_heads || head_dim <= 0 || bytes_per_value <= 0)
        return bad(OOCO_ESHAPE, "bad head geometry");
    if (num_online < 0 || num_offline < 0 || num_looks < 0 || (num_online > 0 && !h_online_lens) ||
        (num_offline > 0 && (!h_offline_lens || !h_selected)) || (num_looks > 0 && !h_random_order))
        return bad(OOCO_EINVAL, "bad array arguments");
    const double D_h = (double)num_q_heads * head_dim, d = bytes_per_value, kv_ratio = (double)num_kv_heads / num_q_heads;
    auto op = [&](int32_t n) { return decode_op_time(*params, D_h, kv_ratio, d, (double)n); };
    for (int i = 0; i < num_online; ++i)
        if (h_online_lens[i] < 1) return bad(OOCO_ESHAPE, "request length below 1");
    for (int i = 0; i < num_offline; ++i)
        if (h_offline_lens[i] < 1) return bad(OOCO_ESHAPE, "request length below 1");
    double sum = 0.0;          // operator times of the batch so far
    int members = num_online;
    for (int i = 0; i < num_online; ++i) sum += op(h_online_lens[i]);
    auto L = [&](double s, int n) { return n > 0 ? s + params->O_d : 0.0; };
    std::vector<uint8_t> looked((size_t)num_offline, 0);
    for (int i = 0; i < num_offline; ++i) h_selected[i] = 0;
    for (int k = 0; k < num_looks; ++k) {                      // the random looks
        const int32_t r = h_random_order[k];
        if (r < 0 || r >= num_offline || looked[(size_t)r]) continue;
        looked[(size_t)r] = 1;
        const double with = sum + op(h_offline_lens[r]);
        if (L(with, members + 1) <= slo_s) {
            sum = with;
            ++members;
            h_selected[r] = 1;
        }
    }
    std::vector<int32_t> rest;
    for (int i = 0; i < num_offline; ++i)
        if (!looked[(size_t)i]) rest.push_back(i);
    if (!rest.empty() && L(sum, members) < slo_s) {            // shortest first, longest admissible prefix
        std::sort(rest.begin(), rest.end(), [&](int32_t a, int32_t b) {
            return h_offline_lens[a] != h_offline_lens[b] ? h_offline_lens[a] < h_offline_lens[b] : a < b;
        });
        std::vector<double> pre(rest.size() + 1);
        pre[0] = sum;
        for (size_t m = 0; m < rest.size(); ++m) pre[m + 1] = pre[m] + op(h_offline_lens[rest[m]]);
        size_t lo = 0, hi = rest.size();
        while (lo < hi) {
            const size_t mid = (lo + hi + 1) / 2;
            if (L(pre[mid], members + (int)mid) <= slo_s)
                lo = mid;
            else
                hi = mid - 1;
        }
        for (size_t m = 0; m < lo; ++m) h_selected[rest[m]] = 1;
        sum = pre[lo];
        members += (int)lo;
    }
    if (latency_out) *latency_out = L(sum, members);
    return OOCO_OK;
}
