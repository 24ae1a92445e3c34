// Shared candidate cache of CARD (Cache Construction, eqs. (1)-(9); Cache Correction):
// the tree the draft side writes level by level and the target side queries before and
// corrects after every verification step.  Host-side integer work on at most K * depth nodes.
#include "card.h"

#include <algorithm>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

namespace {

struct Level {
    std::vector<int32_t> tok;
    std::vector<int32_t> par;
    std::vector<float> score;
    int32_t size() const { return static_cast<int32_t>(tok.size()); }
};

}  // namespace

struct card_cache {
    int32_t K = 0;
    int32_t max_depth = 0;
    int64_t epoch = 0;
    std::vector<Level> levels;
    mutable std::mutex mu;
};

namespace {

// Node of `lv` carrying `token` (and, if parent >= 0, hanging below that parent) with the
// largest score; the lowest index wins among equal scores.  -1 if none.
int32_t find_node(const Level& lv, int32_t token, int32_t parent) {
    int32_t best = -1;
    for (int32_t i = 0; i < lv.size(); ++i) {
        if (lv.tok[i] != token) continue;
        if (parent >= 0 && lv.par[i] != parent) continue;
        if (best < 0 || lv.score[i] > lv.score[best]) best = i;
    }
    return best;
}

}  // namespace

extern "C" {

int card_cache_create(int32_t K, int32_t max_depth, card_cache** out) {
    if (!out || K <= 0 || max_depth <= 0) return CARD_EINVAL;
    card_cache* c = new (std::nothrow) card_cache();
    if (!c) return CARD_EINVAL;
    c->K = K;
    c->max_depth = max_depth;
    c->levels.reserve(max_depth);
    *out = c;
    return CARD_OK;
}

void card_cache_destroy(card_cache* c) { delete c; }

int card_cache_write(card_cache* c, int64_t epoch, int32_t level, int32_t n, const int32_t* tokens,
                     const int32_t* parent_idx, const float* path_score) {
    if (!c || !tokens || !parent_idx || !path_score) return CARD_EINVAL;
    std::lock_guard<std::mutex> lock(c->mu);
    if (epoch != c->epoch) return CARD_ESTALE;
    if (n <= 0 || n > c->K) return CARD_ERANGE;
    if (level < 0 || level >= c->max_depth || level > static_cast<int32_t>(c->levels.size()))
        return CARD_ERANGE;
    const int32_t n_parents = level == 0 ? 0 : c->levels[level - 1].size();
    for (int32_t i = 0; i < n; ++i) {
        if (level == 0 ? parent_idx[i] != -1 : (parent_idx[i] < 0 || parent_idx[i] >= n_parents))
            return CARD_ERANGE;
    }
    c->levels.resize(level);
    Level lv;
    lv.tok.assign(tokens, tokens + n);
    lv.par.assign(parent_idx, parent_idx + n);
    lv.score.assign(path_score, path_score + n);
    c->levels.push_back(std::move(lv));
    return CARD_OK;
}

int card_cache_query(const card_cache* c, int32_t verified_token, int32_t max_len,
                     int32_t* out_tokens, int32_t* out_len, float* out_score) {
    if (!c || !out_tokens || !out_len) return CARD_EINVAL;
    if (max_len < 1) return CARD_ERANGE;
    std::lock_guard<std::mutex> lock(c->mu);
    *out_len = 0;
    if (out_score) *out_score = 0.0f;
    if (c->levels.empty()) return 0;
    const int32_t root = find_node(c->levels[0], verified_token, -1);
    if (root < 0) return 0;
    // alive[l][i] != 0 iff node i of level l descends from root
    const int32_t depth_cap = std::min<int32_t>(max_len, static_cast<int32_t>(c->levels.size()));
    std::vector<std::vector<uint8_t>> alive;
    alive.emplace_back(c->levels[0].size(), 0);
    alive[0][root] = 1;
    for (int32_t l = 1; l < depth_cap; ++l) {
        const Level& lv = c->levels[l];
        std::vector<uint8_t> cur(lv.size(), 0);
        bool any = false;
        for (int32_t i = 0; i < lv.size(); ++i) {
            if (alive[l - 1][lv.par[i]]) {
                cur[i] = 1;
                any = true;
            }
        }
        if (!any) break;
        alive.push_back(std::move(cur));
    }
    const int32_t deepest = static_cast<int32_t>(alive.size()) - 1;
    const Level& last = c->levels[deepest];
    int32_t leaf = -1;
    for (int32_t i = 0; i < last.size(); ++i) {
        if (alive[deepest][i] && (leaf < 0 || last.score[i] > last.score[leaf])) leaf = i;
    }
    int32_t node = leaf;
    for (int32_t l = deepest; l >= 0; --l) {
        out_tokens[l] = c->levels[l].tok[node];
        node = c->levels[l].par[node];
    }
    *out_len = deepest + 1;
    if (out_score) *out_score = last.score[leaf];
    return 1;
}

int card_cache_correct(card_cache* c, const int32_t* verified_tokens, int32_t n) {
    if (!c || (n > 0 && !verified_tokens) || n < 0) return CARD_EINVAL;
    std::lock_guard<std::mutex> lock(c->mu);
    c->epoch += 1;
    if (n == 0) return 1;
    int32_t node = -1;
    for (int32_t d = 0; d < n; ++d) {
        if (d >= static_cast<int32_t>(c->levels.size())) {
            c->levels.clear();
            return 0;
        }
        node = find_node(c->levels[d], verified_tokens[d], d == 0 ? -1 : node);
        if (node < 0) {
            c->levels.clear();
            return 0;
        }
    }
    // keep the subtree strictly below `node`; re-index parents level by level
    std::vector<Level> kept;
    std::vector<int32_t> remap(c->levels[n - 1].size(), -1);  // old index in previous level -> new
    remap[node] = 0;
    for (int32_t l = n; l < static_cast<int32_t>(c->levels.size()); ++l) {
        const Level& lv = c->levels[l];
        Level nl;
        std::vector<int32_t> next_remap(lv.size(), -1);
        for (int32_t i = 0; i < lv.size(); ++i) {
            const int32_t np = remap[lv.par[i]];
            if (np < 0) continue;
            next_remap[i] = nl.size();
            nl.tok.push_back(lv.tok[i]);
            nl.par.push_back(l == n ? -1 : np);
            nl.score.push_back(lv.score[i]);
        }
        if (nl.size() == 0) break;
        kept.push_back(std::move(nl));
        remap.swap(next_remap);
    }
    c->levels.swap(kept);
    return 1;
}

int64_t card_cache_epoch(const card_cache* c) {
    if (!c) return CARD_EINVAL;
    std::lock_guard<std::mutex> lock(c->mu);
    return c->epoch;
}

int32_t card_cache_depth(const card_cache* c) {
    if (!c) return CARD_EINVAL;
    std::lock_guard<std::mutex> lock(c->mu);
    return static_cast<int32_t>(c->levels.size());
}

int card_cache_read_level(const card_cache* c, int32_t level, int32_t* tokens, int32_t* parent_idx,
                          float* path_score) {
    if (!c) return CARD_EINVAL;
    std::lock_guard<std::mutex> lock(c->mu);
    if (level < 0 || level >= static_cast<int32_t>(c->levels.size())) return CARD_ERANGE;
    const Level& lv = c->levels[level];
    if (tokens) std::memcpy(tokens, lv.tok.data(), lv.tok.size() * sizeof(int32_t));
    if (parent_idx) std::memcpy(parent_idx, lv.par.data(), lv.par.size() * sizeof(int32_t));
    if (path_score) std::memcpy(path_score, lv.score.data(), lv.score.size() * sizeof(float));
    return lv.size();
}

}  // extern "C"
