// Host routine of the frontend's scheduling round (App. A, Alg. 1; Sec. 7.2 - 7.4; App. B.2).
// No GPU call: the round works on block hashes, token counts and the per-worker FLOPs counters.
#include <cmath>
#include <new>
#include <unordered_map>
#include <vector>

#include "../../include/moe_prefill.h"
#include "../../include/moe_sched.h"

#pragma clang fp contract(off)

namespace {

enum : uint8_t { COMMITTED = 1, PENDING = 2 };

// The keys are already well-mixed 64-bit hashes.
struct KeyIsHash {
    size_t operator()(uint64_t k) const noexcept { return static_cast<size_t>(k); }
};
using BlockTable = std::unordered_map<uint64_t, uint8_t, KeyIsHash>;

inline uint64_t mix64(uint64_t z) {
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

// Tokens covered by the leading blocks of the request that the table holds without a gap.
inline int64_t block_match(const BlockTable& tab, const uint64_t* h, int64_t n_blocks, int32_t B) {
    int64_t j = 0;
    while (j < n_blocks && tab.find(h[j]) != tab.end()) ++j;
    return j * B;
}

inline bool valid_worker(const moe_sched* s, int32_t w);

}  // namespace

struct moe_sched {
    int32_t n_workers;
    int32_t block_tokens;
    std::vector<BlockTable> tables;
};

namespace {
inline bool valid_worker(const moe_sched* s, int32_t w) { return s && w >= 0 && w < s->n_workers; }
}  // namespace

extern "C" {

int32_t moe_sched_create(int32_t n_workers, int32_t block_tokens, moe_sched_t** out) {
    if (!out) return MOE_ERR_NULL_PTR;
    if (n_workers < 1 || n_workers > 4096 || block_tokens < 1 || block_tokens > 65536) return MOE_ERR_BAD_SHAPE;
    moe_sched* s = new (std::nothrow) moe_sched;
    if (!s) return MOE_ERR_UNSUPPORTED;
    s->n_workers = n_workers;
    s->block_tokens = block_tokens;
    s->tables.resize(n_workers);
    *out = s;
    return MOE_OK;
}

void moe_sched_destroy(moe_sched_t* s) { delete s; }

int32_t moe_sched_hash_blocks(const int32_t* tokens, int64_t n_tokens, int32_t block_tokens, uint64_t* hashes) {
    if (n_tokens < 0 || block_tokens < 1) return MOE_ERR_BAD_SHAPE;
    const int64_t nb = n_tokens / block_tokens;
    if (nb > 0 && (!tokens || !hashes)) return MOE_ERR_NULL_PTR;
    uint64_t h = 0x6A09E667F3BCC908ull ^ static_cast<uint64_t>(block_tokens);
    for (int64_t j = 0; j < nb; ++j) {
        const int32_t* t = tokens + j * block_tokens;
        for (int32_t k = 0; k < block_tokens; ++k) h = mix64(h + 0x9E3779B97F4A7C15ull + static_cast<uint32_t>(t[k]));
        hashes[j] = h;
    }
    return MOE_OK;
}

int32_t moe_sched_round(moe_sched_t* s, const moe_cost_model_t* cost, double threshold, int64_t n_requests,
                        const uint64_t* block_hashes, const int64_t* hash_offsets, const int64_t* prefix_tokens,
                        const int64_t* suffix_tokens, double* loads, int32_t* assigned, int64_t* matched_tokens,
                        double* delta, int64_t* n_assigned) {
    if (!s || !cost || !loads || !n_assigned) return MOE_ERR_NULL_PTR;
    if (n_requests < 0) return MOE_ERR_BAD_SHAPE;
    if (n_requests > 0 && (!hash_offsets || !prefix_tokens || !suffix_tokens || !assigned)) return MOE_ERR_NULL_PTR;
    if (!(cost->f_tok >= 0.0) || !(cost->f_attn >= 0.0) || !std::isfinite(cost->f_tok) || !std::isfinite(cost->f_attn) ||
        std::isnan(threshold))
        return MOE_ERR_BAD_SHAPE;
    const int32_t B = s->block_tokens, N = s->n_workers;
    for (int32_t i = 0; i < N; ++i)
        if (!std::isfinite(loads[i])) return MOE_ERR_BAD_SHAPE;
    for (int64_t r = 0; r < n_requests; ++r) {
        const int64_t nb = hash_offsets[r + 1] - hash_offsets[r];
        if (hash_offsets[r] < 0 || nb < 0 || prefix_tokens[r] < 0 || suffix_tokens[r] < 0 || nb != prefix_tokens[r] / B ||
            prefix_tokens[r] > (int64_t)1 << 30 || suffix_tokens[r] > (int64_t)1 << 30)
            return MOE_ERR_BAD_SHAPE;
        if (nb > 0 && !block_hashes) return MOE_ERR_NULL_PTR;
    }

    std::vector<int32_t> active;   // A of Alg. 1, ascending worker index
    active.reserve(N);
    for (int32_t i = 0; i < N; ++i)
        if (loads[i] < threshold) active.push_back(i);

    int64_t r = 0;
    for (; r < n_requests && !active.empty(); ++r) {
        const uint64_t* h = block_hashes + hash_offsets[r];
        const int64_t nb = hash_offsets[r + 1] - hash_offsets[r];
        const int64_t P = prefix_tokens[r], S = suffix_tokens[r];
        // F3 -> F1 -> F2: longest match over the active set, then smaller load, then lower index.
        size_t best_pos = 0;
        int64_t best_m = -1;
        for (size_t a = 0; a < active.size(); ++a) {
            const int32_t i = active[a];
            const int64_t m = block_match(s->tables[i], h, nb, B);
            if (m > best_m || (m == best_m && loads[i] < loads[active[best_pos]])) {
                best_m = m;
                best_pos = a;
            }
        }
        const int32_t w = active[best_pos];
        const int64_t u = P - best_m;                                   // uncached prefix tokens
        const int64_t pairs = u * (u + 1) / 2 + S * (S + 1) / 2 + S * P;  // C_pfx, C_self, C_cross pair counts
        const double lin = cost->f_tok * static_cast<double>(u + S);
        const double att = cost->f_attn * static_cast<double>(pairs);
        const double d = lin + att;
        loads[w] += d;
        BlockTable& tab = s->tables[w];
        for (int64_t j = best_m / B; j < nb; ++j) tab.emplace(h[j], PENDING);   // keeps a committed entry as it is
        assigned[r] = w;
        if (matched_tokens) matched_tokens[r] = best_m;
        if (delta) delta[r] = d;
        if (loads[w] >= threshold) active.erase(active.begin() + static_cast<std::ptrdiff_t>(best_pos));
    }
    *n_assigned = r;
    for (; r < n_requests; ++r) {
        assigned[r] = -1;
        if (matched_tokens) matched_tokens[r] = 0;
        if (delta) delta[r] = 0.0;
    }
    return MOE_OK;
}

int32_t moe_sched_blocks_stored(moe_sched_t* s, int32_t worker, const uint64_t* hashes, int64_t n) {
    if (!s || (n > 0 && !hashes)) return MOE_ERR_NULL_PTR;
    if (!valid_worker(s, worker) || n < 0) return MOE_ERR_BAD_SHAPE;
    BlockTable& tab = s->tables[worker];
    for (int64_t j = 0; j < n; ++j) tab[hashes[j]] = COMMITTED;
    return MOE_OK;
}

int32_t moe_sched_blocks_evicted(moe_sched_t* s, int32_t worker, const uint64_t* hashes, int64_t n) {
    if (!s || (n > 0 && !hashes)) return MOE_ERR_NULL_PTR;
    if (!valid_worker(s, worker) || n < 0) return MOE_ERR_BAD_SHAPE;
    BlockTable& tab = s->tables[worker];
    for (int64_t j = 0; j < n; ++j) {
        auto it = tab.find(hashes[j]);
        if (it != tab.end() && it->second == COMMITTED) tab.erase(it);
    }
    return MOE_OK;
}

int32_t moe_sched_tokens_executed(const moe_sched_t* s, double* loads, int32_t worker, int64_t tokens,
                                  double f_tok) {
    if (!s || !loads) return MOE_ERR_NULL_PTR;
    if (!valid_worker(s, worker) || tokens < 0 || !(f_tok >= 0.0) || !std::isfinite(f_tok)) return MOE_ERR_BAD_SHAPE;
    const double done = f_tok * static_cast<double>(tokens);
    const double left = loads[worker] - done;
    loads[worker] = left > 0.0 ? left : 0.0;
    return MOE_OK;
}

int32_t moe_sched_table_size(const moe_sched_t* s, int32_t worker, int64_t* committed, int64_t* pending) {
    if (!s || !committed || !pending) return MOE_ERR_NULL_PTR;
    if (!valid_worker(s, worker)) return MOE_ERR_BAD_SHAPE;
    int64_t c = 0, p = 0;
    for (const auto& kv : s->tables[worker]) (kv.second == COMMITTED ? c : p) += 1;
    *committed = c;
    *pending = p;
    return MOE_OK;
}

}  // extern "C"
