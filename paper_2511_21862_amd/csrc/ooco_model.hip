// Host-only part of libooco: the roofline latency model of the attention operator
// (paper Section 3.3: operator model of Table 2, operator latency of Equation 1, iteration latency
// = sum of operator latencies + static overhead) and the scheduling rules that consume it (Algorithm 2,
// Algorithm 1, the eviction rule of Section 3.4.1).  No device code, no device state.
#include "ooco.h"

#include <algorithm>
#include <cstdio>
#include <cstdlib>
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
        // Table 2, attention row; optionally only the (row, key) pairs a causal kernel visits.  The table prints
        // the head ratio of the KV term as H_q/H_kv; H_kv/H_q is used, since the KV tensors have H_kv heads.
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

namespace {
bool model_args_ok(const ooco_model_params *p, int Hq, int Hkv, int hd, int bpv)
{
    return p && p->F_ad > 0 && p->M_a > 0 && p->O_d >= 0 && Hq > 0 && Hkv > 0 && Hq % Hkv == 0 && hd > 0 && bpv > 0;
}
int64_t blocks_of(int64_t len, int block_size) { return (len + block_size - 1) / block_size; }
}  // namespace

// Offline Request Migration Decision (paper Algorithm 1).  The batch's operator times are summed once; a
// hypothetical group of n requests of length l adds n times the same operator time, accumulated one by one as a
// from-scratch evaluation of the enlarged batch would; both L and the block count grow with l, so the largest
// admissible length is found by bisection over [len_min, len_max].
extern "C" ooco_status ooco_migration_preference(const ooco_model_params *params, int num_q_heads, int num_kv_heads,
                                                 int head_dim, int bytes_per_value, double slo_s, int batch_size,
                                                 const int32_t *h_batch_lens, int all_included, int bs_sat, int block_size,
                                                 int64_t capacity_blocks, int32_t len_min, int32_t len_max,
                                                 int32_t *pref_out, int32_t *branch_out, char *msg, size_t msg_cap)
{
    auto bad = [&](ooco_status code, const char *text) {
        if (msg && msg_cap) snprintf(msg, msg_cap, "ooco_migration_preference: %s", text);
        return code;
    };
    if (msg && msg_cap) msg[0] = 0;
    if (!pref_out) return bad(OOCO_EINVAL, "NULL pref_out");
    if (!model_args_ok(params, num_q_heads, num_kv_heads, head_dim, bytes_per_value))
        return bad(OOCO_EINVAL, "bad model parameters or head geometry");
    if (batch_size < 0 || (batch_size > 0 && !h_batch_lens) || bs_sat < 1 || block_size < 1 || capacity_blocks < 0 ||
        len_min < 1 || len_max < len_min)
        return bad(OOCO_EINVAL, "bad sizes (batch_size >= 0, bs_sat >= 1, block_size >= 1, 1 <= len_min <= len_max)");
    const double D_h = (double)num_q_heads * head_dim, d = bytes_per_value, kv_ratio = (double)num_kv_heads / num_q_heads;
    double base = 0.0;
    int64_t used = 0;
    for (int i = 0; i < batch_size; ++i) {
        if (h_batch_lens[i] < 1) return bad(OOCO_ESHAPE, "request length below 1");
        base += decode_op_time(*params, D_h, kv_ratio, d, (double)h_batch_lens[i]);
        used += blocks_of(h_batch_lens[i], block_size);
    }
    auto L_with = [&](int32_t len, int n) {        // L(B + n requests of length len)
        double s = base;
        const double t = decode_op_time(*params, D_h, kv_ratio, d, (double)len);
        for (int k = 0; k < n; ++k) s += t;
        return batch_size + n > 0 ? s + params->O_d : 0.0;
    };
    auto largest = [&](int n, bool memory) -> int32_t {     // largest admissible length, or -1
        auto fits = [&](int32_t len) {
            return L_with(len, n) <= slo_s && (!memory || used + (int64_t)n * blocks_of(len, block_size) <= capacity_blocks);
        };
        if (!fits(len_min)) return -1;
        int32_t lo = len_min, hi = len_max;
        while (lo < hi) {
            const int32_t mid = (int32_t)(((int64_t)lo + hi + 1) / 2);
            if (fits(mid))
                lo = mid;
            else
                hi = mid - 1;
        }
        return lo;
    };
    int32_t pref = -1, branch = 0;
    if (L_with(len_min, 0) < slo_s && all_included) {
        if (batch_size >= bs_sat) {
            pref = largest(1, true);
            branch = pref >= 0 ? 1 : 0;
        } else {
            const int n = bs_sat - batch_size;
            pref = largest(n, false);
            branch = 2;
            if (pref < 0) {
                pref = len_min;
                branch = 3;
            }
        }
    }
    *pref_out = pref;
    if (branch_out) *branch_out = branch;
    return OOCO_OK;
}

// The latency-relaxed node's side of Algorithm 1: its ongoing offline requests nearest to the preferred length
// first; a request goes if the strict node's batch with it keeps L <= S and fits the cache.
extern "C" ooco_status ooco_migration_select(const ooco_model_params *params, int num_q_heads, int num_kv_heads,
                                             int head_dim, int bytes_per_value, double slo_s, int batch_size,
                                             const int32_t *h_batch_lens, int num_relaxed, const int32_t *h_relaxed_lens,
                                             int32_t pref, int block_size, int64_t capacity_blocks, int max_migrate,
                                             int32_t *h_chosen, int32_t *num_chosen, char *msg, size_t msg_cap)
{
    auto bad = [&](ooco_status code, const char *text) {
        if (msg && msg_cap) snprintf(msg, msg_cap, "ooco_migration_select: %s", text);
        return code;
    };
    if (msg && msg_cap) msg[0] = 0;
    if (!num_chosen) return bad(OOCO_EINVAL, "NULL num_chosen");
    *num_chosen = 0;
    if (!model_args_ok(params, num_q_heads, num_kv_heads, head_dim, bytes_per_value))
        return bad(OOCO_EINVAL, "bad model parameters or head geometry");
    if (batch_size < 0 || (batch_size > 0 && !h_batch_lens) || num_relaxed < 0 || (num_relaxed > 0 && !h_relaxed_lens) ||
        block_size < 1 || capacity_blocks < 0 || max_migrate < 0 || pref < 1 || (max_migrate > 0 && num_relaxed > 0 && !h_chosen))
        return bad(OOCO_EINVAL, "bad sizes or NULL arrays (pref >= 1, block_size >= 1)");
    const double D_h = (double)num_q_heads * head_dim, d = bytes_per_value, kv_ratio = (double)num_kv_heads / num_q_heads;
    double sum = 0.0;
    int64_t used = 0;
    for (int i = 0; i < batch_size; ++i) {
        if (h_batch_lens[i] < 1) return bad(OOCO_ESHAPE, "request length below 1");
        sum += decode_op_time(*params, D_h, kv_ratio, d, (double)h_batch_lens[i]);
        used += blocks_of(h_batch_lens[i], block_size);
    }
    for (int i = 0; i < num_relaxed; ++i)
        if (h_relaxed_lens[i] < 1) return bad(OOCO_ESHAPE, "request length below 1");
    std::vector<int32_t> order((size_t)num_relaxed);
    std::iota(order.begin(), order.end(), 0);
    auto dist = [&](int32_t i) { return std::abs((int64_t)h_relaxed_lens[i] - (int64_t)pref); };
    std::sort(order.begin(), order.end(), [&](int32_t a, int32_t b) {
        if (dist(a) != dist(b)) return dist(a) < dist(b);
        if (h_relaxed_lens[a] != h_relaxed_lens[b]) return h_relaxed_lens[a] < h_relaxed_lens[b];
        return a < b;
    });
    int taken = 0;
    for (int32_t i : order) {
        if (taken >= max_migrate) break;
        const double with = sum + decode_op_time(*params, D_h, kv_ratio, d, (double)h_relaxed_lens[i]);
        const int64_t blk = blocks_of(h_relaxed_lens[i], block_size);
        if (with + params->O_d <= slo_s && used + blk <= capacity_blocks) {
            sum = with;
            used += blk;
            h_chosen[taken++] = i;
        }
    }
    *num_chosen = taken;
    return OOCO_OK;
}

// Which offline requests leave a latency-strict node to free need_blocks KV blocks (paper Section 3.4.1):
// long ones first when the node is compute-bound (batch_size >= bs_sat), short ones first otherwise; then, in
// the order taken, whoever is not needed for the total any more stays.
extern "C" ooco_status ooco_eviction_victims(int num_offline, const int32_t *h_offline_lens, int64_t need_blocks,
                                             int block_size, int batch_size, int bs_sat, int32_t *h_victims,
                                             int32_t *num_victims, int32_t *enough, char *msg, size_t msg_cap)
{
    auto bad = [&](ooco_status code, const char *text) {
        if (msg && msg_cap) snprintf(msg, msg_cap, "ooco_eviction_victims: %s", text);
        return code;
    };
    if (msg && msg_cap) msg[0] = 0;
    if (!num_victims) return bad(OOCO_EINVAL, "NULL num_victims");
    *num_victims = 0;
    if (num_offline < 0 || (num_offline > 0 && (!h_offline_lens || !h_victims)) || need_blocks < 0 || block_size < 1 ||
        batch_size < 0 || bs_sat < 1)
        return bad(OOCO_EINVAL, "bad sizes or NULL arrays");
    for (int i = 0; i < num_offline; ++i)
        if (h_offline_lens[i] < 1) return bad(OOCO_ESHAPE, "request length below 1");
    const bool compute_bound = batch_size >= bs_sat;
    std::vector<int32_t> order((size_t)num_offline);
    std::iota(order.begin(), order.end(), 0);
    std::sort(order.begin(), order.end(), [&](int32_t a, int32_t b) {
        if (h_offline_lens[a] != h_offline_lens[b])
            return compute_bound ? h_offline_lens[a] > h_offline_lens[b] : h_offline_lens[a] < h_offline_lens[b];
        return a < b;
    });
    int64_t freed = 0;
    size_t k = 0;
    while (k < order.size() && freed < need_blocks) freed += blocks_of(h_offline_lens[order[k++]], block_size);
    const bool ok = freed >= need_blocks;
    int n = 0;
    for (size_t j = 0; j < k; ++j) {
        const int64_t b = blocks_of(h_offline_lens[order[j]], block_size);
        if (ok && freed - b >= need_blocks)
            freed -= b;                      // not needed after all
        else
            h_victims[n++] = order[j];
    }
    *num_victims = n;
    if (enough) *enough = ok ? 1 : 0;
    return OOCO_OK;
}
