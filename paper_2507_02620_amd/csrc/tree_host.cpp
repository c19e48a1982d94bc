// Draft-stage tree bookkeeping on the host: score-based segmentation, pruning, expansion by merging.
#include <stdint.h>

#include <algorithm>
#include <numeric>
#include <unordered_map>
#include <vector>

#include "../../include/flowspec.h"

namespace {
bool topo_ok(const int32_t* parent, int n) {
    if (n > 0 && parent[0] != -1) return false;
    for (int i = 1; i < n; ++i)
        if (parent[i] < 0 || parent[i] >= i) return false;
    return true;
}
inline uint64_t edge_key(int parent_node, int32_t token) { return ((uint64_t)(uint32_t)parent_node << 32) | (uint32_t)token; }
}  // namespace

extern "C" {

int fs_tree_segment(const int32_t* parent_base, const int32_t* token_base, const float* conf, int n_base, int L0, int32_t* parent,
                    int32_t* token, double* score, int32_t* base_index) {
    if (!parent_base || !token_base || !conf || !parent || !token || !score || !base_index || n_base < 1 || L0 < 1) return FS_EINVAL;
    if (!topo_ok(parent_base, n_base)) return FS_ETOPO;
    std::vector<double> cu(n_base);
    cu[0] = 1.0;
    for (int i = 1; i < n_base; ++i) cu[i] = (double)conf[i] * cu[parent_base[i]];
    std::vector<int> order(n_base);
    std::iota(order.begin(), order.end(), 0);
    std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return cu[a] > cu[b]; });
    const int keep = std::min(L0, n_base);
    std::vector<int> rank(n_base, -1);
    for (int j = 0; j < keep; ++j) rank[order[j]] = j;
    for (int j = 0; j < keep; ++j) {
        const int b = order[j];
        const int p = parent_base[b];
        if (p >= 0 && rank[p] < 0) return FS_EINVAL;  // a confidence above 1 put a child ahead of its parent
        parent[j] = p < 0 ? -1 : rank[p];
        if (p >= 0 && parent[j] >= j) return FS_EINVAL;
        token[j] = token_base[b];
        score[j] = cu[b];
        base_index[j] = b;
    }
    return keep;
}

int fs_tree_prune(const int32_t* parent, const int32_t* token, int T, const int32_t* retain, int n_acc, int n_retain, int32_t* new_parent,
                  int32_t* new_token) {
    if (!parent || !token || !retain || T < 1 || n_acc < 0 || n_retain < n_acc || n_retain > T) return FS_EINVAL;
    if (n_retain > n_acc && (!new_parent || !new_token)) return FS_EINVAL;
    std::vector<int> rank(T, -1);
    for (int j = 0; j < n_retain; ++j) {
        if (retain[j] < 0 || retain[j] >= T || (j > 0 && retain[j] <= retain[j - 1])) return FS_EINVAL;
        if (j >= n_acc) rank[retain[j]] = j - n_acc;
    }
    for (int j = n_acc; j < n_retain; ++j) {
        const int i = retain[j], p = parent[i];
        new_parent[j - n_acc] = (j == n_acc || p < 0) ? -1 : rank[p];
        new_token[j - n_acc] = token[i];
    }
    return n_retain - n_acc;
}

int fs_tree_merge(const int32_t* parent_pr, const int32_t* token_pr, int n_pr, const int32_t* parent_new, const int32_t* token_new, int n_new,
                  int limit, int max_out, int32_t* parent, int32_t* token, int32_t* app_src, int32_t* map_new) {
    if (n_pr < 0 || n_new < 0 || max_out < 0 || !parent || !token) return FS_EINVAL;
    if ((n_pr > 0 && (!parent_pr || !token_pr)) || (n_new > 0 && (!parent_new || !token_new || !map_new || !app_src))) return FS_EINVAL;
    if (!topo_ok(parent_pr, n_pr) || !topo_ok(parent_new, n_new)) return FS_ETOPO;
    if (n_pr > 0 && n_new > 0 && token_pr[0] != token_new[0]) return FS_EINVAL;
    if (n_pr > max_out) return FS_ECAP;
    // P_pr: every path of T_pr, represented by (node of the parent path, last token); first occurrence wins
    std::unordered_map<uint64_t, int> paths;
    paths.reserve((size_t)(n_pr + n_new) * 2);
    for (int i = 0; i < n_pr; ++i) {
        parent[i] = parent_pr[i];
        token[i] = token_pr[i];
        if (i > 0) paths.emplace(edge_key(parent_pr[i], token_pr[i]), i);
    }
    int n = n_pr, n_app = 0;
    for (int j = 0; j < n_new; ++j) {
        if (j == 0 && n_pr > 0) {
            map_new[0] = 0;  // the shared root
            continue;
        }
        const int pm = (j == 0) ? -1 : map_new[parent_new[j]];
        if (j > 0 && pm < 0) {  // its parent fell beyond the limit
            map_new[j] = -1;
            continue;
        }
        if (j > 0) {
            auto it = paths.find(edge_key(pm, token_new[j]));
            if (it != paths.end()) {
                map_new[j] = it->second;
                continue;
            }
        }
        if (limit >= 0 && n_app >= limit) {
            map_new[j] = -1;
            continue;
        }
        if (n >= max_out) return FS_ECAP;
        parent[n] = pm;
        token[n] = token_new[j];
        if (j > 0) paths.emplace(edge_key(pm, token_new[j]), n);
        map_new[j] = n;
        app_src[n_app++] = j;
        ++n;
    }
    return n;
}

}  // extern "C"
