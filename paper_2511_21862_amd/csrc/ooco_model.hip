// Host-only part of libooco: the roofline latency model of the attention operator
// (paper Section 3.3: operator model of Table 2, operator latency of Equation 1, iteration latency
// = sum of operator latencies + static overhead).  No device code, no device state.
#include "ooco.h"

#include <cstdio>

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
