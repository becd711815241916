// hc_taxonomy.hip -- offline head taxonomy and budget allocation (Sec. 4.1-4.2, Eq. 4-8; App. C.2;
// Algorithm 1 stages 1-2).  Host code only: a layer has tens of heads, and this runs once per model.
// Its results are the roles, pivots and resident lengths that the head table of hc_layer_create takes.
#include <math.h>

#include <algorithm>
#include <vector>

#include "hc_internal.h"

#pragma clang fp contract(off)      // budgets are decided in plain IEEE double arithmetic, operation by operation

// Greedy star clustering on the similarity graph (App. C.2): the unassigned head with the most unassigned
// neighbours (lowest index on a tie) becomes a pivot and takes all of them as satellites; when no
// unassigned head has an unassigned neighbour left, the rest are anchors (stability >= tau_stable, Eq. 5)
// or volatile heads, which like pivots keep their full cache (HC_ROLE_FULL).
extern "C" hc_status hc_taxonomy(int32_t n_heads, const uint8_t* adjacency, const double* s_stable, double tau_stable,
                                 int32_t* role_out, int32_t* rep_out, int32_t* is_pivot_out)
{
    if (n_heads < 1 || n_heads > 4096 || !adjacency || !s_stable || !role_out || !rep_out) return HC_EINVAL;
    const int n = n_heads;
    for (int i = 0; i < n; ++i) {
        if (!(s_stable[i] == s_stable[i])) return HC_EINVAL;                               // NaN
        for (int j = 0; j < i; ++j)
            if ((adjacency[(size_t)i * n + j] != 0) != (adjacency[(size_t)j * n + i] != 0)) return HC_EINVAL;   // not symmetric
    }
    std::vector<char> unassigned(n, 1);
    for (int i = 0; i < n; ++i) {
        role_out[i] = -1;
        rep_out[i] = -1;
        if (is_pivot_out) is_pivot_out[i] = 0;
    }
    for (;;) {
        int best = -1, best_deg = 0;
        for (int h = 0; h < n; ++h) {
            if (!unassigned[h]) continue;
            int deg = 0;
            for (int j = 0; j < n; ++j) deg += j != h && unassigned[j] && adjacency[(size_t)h * n + j];
            if (deg > best_deg) {
                best = h;
                best_deg = deg;
            }
        }
        if (best < 0) break;
        role_out[best] = HC_ROLE_FULL;
        if (is_pivot_out) is_pivot_out[best] = 1;
        unassigned[best] = 0;
        for (int j = 0; j < n; ++j)
            if (unassigned[j] && adjacency[(size_t)best * n + j]) {
                role_out[j] = HC_ROLE_SATELLITE;
                rep_out[j] = best;
                unassigned[j] = 0;
            }
    }
    for (int h = 0; h < n; ++h)
        if (unassigned[h]) role_out[h] = s_stable[h] >= tau_stable ? HC_ROLE_ANCHOR : HC_ROLE_FULL;
    return HC_OK;
}

// Eq. 7-8.  total = (rho N - N_full) L in integers; share_i = (total * w_i) / sum(w), w_i = 1.0 / S_i, sums in
// head order, in double precision; rounded down, the slots left over to the largest fractional parts (lowest
// index first); a share above L is cut to L and the others share the rest in the same proportion.
extern "C" hc_status hc_budgets(int32_t n_heads, const int32_t* role, const double* s_stable, int32_t rho_num, int32_t rho_den,
                                int32_t L, int32_t* len_out)
{
    if (n_heads < 1 || n_heads > 4096 || !role || !s_stable || !len_out || rho_num < 1 || rho_den < 1 || L < 1) return HC_EINVAL;
    const int n = n_heads;
    std::vector<int> free_heads;
    for (int i = 0; i < n; ++i) {
        if (role[i] != HC_ROLE_FULL && role[i] != HC_ROLE_SATELLITE && role[i] != HC_ROLE_ANCHOR) return HC_EINVAL;
        if (role[i] != HC_ROLE_FULL) {
            if (!(s_stable[i] > 0.0)) return HC_EINVAL;
            free_heads.push_back(i);
        }
    }
    const int64_t n_comp = (int64_t)free_heads.size(), n_full = n - n_comp;
    if (n_comp == 0 || (int64_t)rho_num * n <= n_full * rho_den) return HC_EINVAL;          // nothing left for compressed heads
    int64_t left = ((int64_t)rho_num * n - n_full * rho_den) * L / rho_den;
    if (left <= 0) return HC_EINVAL;
    left = std::min<int64_t>(left, n_comp * L);
    for (int i = 0; i < n; ++i) len_out[i] = L;
    std::vector<double> w(n, 0.0);
    for (int i : free_heads) w[i] = 1.0 / s_stable[i];
    double sw = 0.0;
    for (;;) {
        sw = 0.0;
        for (int i : free_heads) sw += w[i];
        std::vector<int> keep;
        int64_t cut = 0;
        for (int i : free_heads) {
            if (((double)left * w[i]) / sw > (double)L) ++cut;
            else keep.push_back(i);
        }
        if (cut == 0) break;
        left -= cut * L;
        free_heads.swap(keep);
        if (free_heads.empty()) return HC_OK;
    }
    std::vector<double> share(n, 0.0);
    int64_t given = 0;
    for (int i : free_heads) {
        share[i] = ((double)left * w[i]) / sw;
        len_out[i] = (int32_t)floor(share[i]);
        given += len_out[i];
    }
    std::vector<int> order(free_heads);
    std::stable_sort(order.begin(), order.end(), [&](int a, int b) {
        const double fa = share[a] - (double)len_out[a], fb = share[b] - (double)len_out[b];
        return fa > fb;        // stable: equal fractions stay in index order
    });
    const int64_t rest = std::max<int64_t>(0, left - given);
    for (int64_t k = 0; k < rest; ++k) len_out[order[k % order.size()]] += 1;
    return HC_OK;
}
