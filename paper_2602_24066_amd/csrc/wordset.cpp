// Word-set construction and work-unit planning (host, integer only).
//
// Canonical order (Appendix A): words sorted by length, then lexicographically; for a full
// truncation that is "cumulative level offset + base-d encoding", so parent = floor(phi/d) and
// last letter = phi mod d (prefix / suffix extraction corollaries).
#include "wordset.hpp"

#include <algorithm>
#include <cmath>
#include <cstring>
#include <functional>
#include <limits>
#include <new>
#include <unordered_map>

#include "../../include/sig.h"

namespace sig {

static const int64_t kMaxWords = (int64_t)SIG_MAX_WORDS;

// Suffix structure of sets that are not full truncations (those have kernels and product rules of their own): the
// word without its first letter, found through the word without first letter of the parent; if every such word is
// in the set, the tables for products of signatures restricted to the set are appended to the device image (sets of
// up to 65,535 words).
static void suffix_tables(WordSet* ws)
{
    ws->suffix_closed = false;
    ws->pair_tables = false;
    const int64_t n = ws->size();
    if (ws->kind == 0 || !ws->kernels_supported || n == 0 || n > 0x3fffffff) return;
    for (int64_t k = 0; k < n; ++k)
        if (ws->child_list[(size_t)k] != (int32_t)k) return;          // children of every word contiguous and in order
    // child of word q (q = -1: the empty word) with last letter i, or -1
    auto child = [&](int32_t q, int32_t i) -> int32_t {
        for (int32_t k = ws->child_off[(size_t)(q + 1)]; k < ws->child_off[(size_t)(q + 2)]; ++k)
            if (ws->letter[(size_t)k] == i) return k;
        return -1;
    };
    std::vector<int32_t> tail((size_t)n, -1);                         // -1: the empty word (words of length 1)
    for (int64_t w = 0; w < n; ++w) {
        const int32_t p = ws->parent[(size_t)w];
        if (p < 0) continue;
        const int32_t t = child(tail[(size_t)p], ws->letter[(size_t)w]);   // parents precede their children
        if (t < 0) return;                                             // a suffix is missing: not closed
        tail[(size_t)w] = t;
    }
    ws->tail_off.assign((size_t)ws->max_len + 2, 0);
    size_t total = 0;
    for (int len = 2; len <= ws->max_len; ++len) {
        ws->tail_off[(size_t)len] = (int32_t)total;
        total += (size_t)(len - 1) * (size_t)(ws->level_start[(size_t)len + 1] - ws->level_start[(size_t)len]);
    }
    if (total > 0x7fffffff) return;
    ws->tail_tab.assign(std::max<size_t>(total, 1), 0);
    for (int len = 2; len <= ws->max_len; ++len) {
        const int64_t lo = ws->level_start[(size_t)len], cnt = ws->level_start[(size_t)len + 1] - lo;
        for (int64_t i = 0; i < cnt; ++i) {
            int32_t t = (int32_t)(lo + i);
            for (int m = 1; m < len; ++m) {
                t = tail[(size_t)t];
                ws->tail_tab[(size_t)ws->tail_off[(size_t)len] + (size_t)(m - 1) * (size_t)cnt + (size_t)i] = t;
            }
        }
    }
    ws->suffix_closed = true;
    if (n > 0xffff) return;                                            // two word indices share an entry of the tables below
    // Terms of the product (a (x) b)(w) = a(w) + b(w) + sum_m a(w_1..w_m) b(w_{m+1}..w_n), in two orders:
    // prod_pairs, laid out like tail_tab (word-major per length: entry (m, w) = prefix | suffix << 16), for the product
    // itself, and adj_pairs, grouped by the prefix u (entries adj_off[u] .. adj_off[u + 1]: w | suffix << 16, by length
    // of w, then w; adj_key holds u for every entry), for sums over all words that extend u.
    ws->prod_pairs.assign(ws->tail_tab.size(), 0);
    ws->adj_off.assign((size_t)n + 1, 0);
    for (int len = 2; len <= ws->max_len; ++len) {
        const int64_t lo = ws->level_start[(size_t)len], cnt = ws->level_start[(size_t)len + 1] - lo;
        for (int64_t i = 0; i < cnt; ++i) {
            int32_t p = (int32_t)(lo + i);
            for (int m = len - 1; m >= 1; --m) {
                p = ws->parent[(size_t)p];                             // the prefix of m letters
                const size_t at = (size_t)ws->tail_off[(size_t)len] + (size_t)(m - 1) * (size_t)cnt + (size_t)i;
                ws->prod_pairs[at] = (uint32_t)p | ((uint32_t)ws->tail_tab[at] << 16);
                ws->adj_off[(size_t)p + 1]++;
            }
        }
    }
    for (int64_t u = 0; u < n; ++u) ws->adj_off[(size_t)u + 1] += ws->adj_off[(size_t)u];
    // padded to whole groups of 256 terms with terms of the dummy prefix n, so that the kernel needs no bounds checks
    const size_t n_terms = ((size_t)ws->adj_off[(size_t)n] + 255) / 256 * 256;
    ws->adj_pairs.assign(std::max<size_t>(n_terms, 256), 0);
    ws->adj_key.assign(ws->adj_pairs.size(), (uint32_t)n);
    {
        std::vector<int32_t> fill(ws->adj_off.begin(), ws->adj_off.end() - 1);
        for (int len = 2; len <= ws->max_len; ++len) {
            const int64_t lo = ws->level_start[(size_t)len], cnt = ws->level_start[(size_t)len + 1] - lo;
            for (int64_t i = 0; i < cnt; ++i) {
                int32_t p = (int32_t)(lo + i);
                for (int m = len - 1; m >= 1; --m) {
                    p = ws->parent[(size_t)p];
                    const size_t at = (size_t)ws->tail_off[(size_t)len] + (size_t)(m - 1) * (size_t)cnt + (size_t)i;
                    ws->adj_key[(size_t)fill[(size_t)p]] = (uint32_t)p;
                    ws->adj_pairs[(size_t)fill[(size_t)p]++] = (uint32_t)(lo + i) | ((uint32_t)ws->tail_tab[at] << 16);
                }
            }
        }
    }
    auto append = [&](const void* src, size_t bytes) {
        const size_t off = (ws->image.size() + 255) & ~(size_t)255;
        ws->image.resize(off + ((bytes + 255) & ~(size_t)255), 0);
        std::memcpy(&ws->image[off], src, bytes);
        return off;
    };
    ws->dev_prod_off = append(ws->prod_pairs.data(), ws->prod_pairs.size() * sizeof(uint32_t));
    ws->dev_adj_key_off = append(ws->adj_key.data(), ws->adj_key.size() * sizeof(uint32_t));
    ws->dev_adj_pairs_off = append(ws->adj_pairs.data(), ws->adj_pairs.size() * sizeof(uint32_t));
    ws->pair_tables = true;
}

// Fills everything that follows from (parent, letter, level_start).
static int finish(WordSet* ws)
{
    const int64_t n = ws->size();
    ws->max_len = (int)ws->level_start.size() - 2;
    ws->length.assign((size_t)n, 0);
    for (int len = 1; len <= ws->max_len; ++len)
        for (int64_t w = ws->level_start[(size_t)len]; w < ws->level_start[(size_t)len + 1]; ++w)
            ws->length[(size_t)w] = (uint8_t)len;
    // children are contiguous in canonical order: count, then prefix-sum
    ws->child_off.assign((size_t)n + 2, 0);
    for (int64_t w = 0; w < n; ++w) ws->child_off[(size_t)(ws->parent[(size_t)w] + 1) + 1]++;
    for (int64_t k = 1; k <= n + 1; ++k) ws->child_off[(size_t)k] += ws->child_off[(size_t)k - 1];
    ws->child_list.resize((size_t)n);
    {
        std::vector<int32_t> fill(ws->child_off.begin(), ws->child_off.end() - 1);
        for (int64_t w = 0; w < n; ++w) ws->child_list[(size_t)fill[(size_t)(ws->parent[(size_t)w] + 1)]++] = (int32_t)w;
    }
    ws->height.assign((size_t)n, 0);
    for (int64_t w = n - 1; w >= 0; --w) {
        const int32_t p = ws->parent[(size_t)w];
        if (p >= 0) ws->height[(size_t)p] = std::max<uint8_t>(ws->height[(size_t)p], (uint8_t)(ws->height[(size_t)w] + 1));
    }
    ws->min_fma = 0;
    for (int64_t w = 0; w < n; ++w) ws->min_fma += 1 + ws->height[(size_t)w];

    ws->kernels_supported = ws->max_len <= SIG_MAX_KERNEL_LEN && ws->d <= 4096;
    if (ws->kernels_supported) {
        // forward: one fp32 per word per lane in LDS; backward: two.
        const int64_t fwd_targets[] = {160, 80, 40, 20};
        const int64_t bwd_targets[] = {96, 48, 24, 12};
        for (int64_t t : fwd_targets) {
            ws->plans[0].emplace_back();
            build_plan(*ws, 112, t, false, ws->plans[0].back());
        }
        for (int64_t t : bwd_targets) {
            ws->plans[1].emplace_back();
            build_plan(*ws, 56, t, true, ws->plans[1].back());
        }
    }
    // device image
    size_t off = 0;
    auto reserve = [&](size_t bytes) { size_t o = off; off = (off + bytes + 255) & ~(size_t)255; return o; };
    for (int dir = 0; dir < 2; ++dir) {
        ws->offsets[dir].clear();
        for (const Plan& p : ws->plans[dir]) {
            WordSet::PlanOffsets po;
            po.units = reserve(p.units.size() * sizeof(UnitDesc));
            po.ops = reserve(p.ops.size() * sizeof(uint32_t));
            po.slots = reserve(p.slot_word.size() * sizeof(int32_t));
            ws->offsets[dir].push_back(po);
        }
    }
    ws->image.assign(std::max<size_t>(off, 256), 0);
    for (int dir = 0; dir < 2; ++dir)
        for (size_t v = 0; v < ws->plans[dir].size(); ++v) {
            const Plan& p = ws->plans[dir][v];
            const WordSet::PlanOffsets& po = ws->offsets[dir][v];
            if (!p.units.empty()) std::memcpy(&ws->image[po.units], p.units.data(), p.units.size() * sizeof(UnitDesc));
            if (!p.ops.empty()) std::memcpy(&ws->image[po.ops], p.ops.data(), p.ops.size() * sizeof(uint32_t));
            if (!p.slot_word.empty()) std::memcpy(&ws->image[po.slots], p.slot_word.data(), p.slot_word.size() * sizeof(int32_t));
        }
    suffix_tables(ws);
    return SIG_OK;
}

void build_plan(const WordSet& ws, int max_slots, int64_t target_cost, bool with_leave, Plan& plan)
{
    const int64_t n = ws.size();
    std::vector<int64_t> sub_size((size_t)n, 1), sub_cost((size_t)n, 0);
    for (int64_t w = n - 1; w >= 0; --w) {
        sub_cost[(size_t)w] += 1 + ws.height[(size_t)w];
        const int32_t p = ws.parent[(size_t)w];
        if (p >= 0) {
            sub_size[(size_t)p] += sub_size[(size_t)w];
            sub_cost[(size_t)p] += sub_cost[(size_t)w];
        }
    }
    std::vector<char> owned((size_t)n, 0);
    std::vector<int32_t> chain;

    auto children = [&](int32_t u, const int32_t*& first, int32_t& count) {
        first = ws.child_list.data() + ws.child_off[(size_t)(u + 1)];
        count = ws.child_off[(size_t)(u + 1) + 1] - ws.child_off[(size_t)(u + 1)];
    };

    auto emit_unit = [&](const std::vector<int32_t>& group) {
        UnitDesc ud;
        ud.op_off = (int32_t)plan.ops.size();
        ud.slot_off = (int32_t)plan.slot_word.size();
        int hmax = 0;
        for (int32_t g : group) hmax = std::max<int>(hmax, ws.height[(size_t)g]);
        const int K = (int)chain.size();
        int64_t fma = 0;
        for (int k = 0; k < K; ++k) {
            const int32_t w = chain[(size_t)k];
            const int h = hmax + 1 + (K - 1 - k);
            plan.ops.push_back(op_pack((uint32_t)ws.letter[(size_t)w], (uint32_t)(k + 1), (uint32_t)h, OP_ENTER));
            plan.slot_word.push_back(owned[(size_t)w] ? ~w : w);
            owned[(size_t)w] = 1;
            fma += h + 1;
            plan.pairs_nonleaf += h;
        }
        std::function<void(int32_t)> dfs = [&](int32_t v) {
            const int h = ws.height[(size_t)v];
            const uint32_t lev = ws.length[(size_t)v];
            plan.slot_word.push_back(v);
            owned[(size_t)v] = 1;
            fma += h + 1;
            if (h == 0) {
                plan.ops.push_back(op_pack((uint32_t)ws.letter[(size_t)v], lev, 0, OP_LEAF));
                plan.leaves++;
                return;
            }
            plan.pairs_nonleaf += h;
            plan.ops.push_back(op_pack((uint32_t)ws.letter[(size_t)v], lev, (uint32_t)h, OP_ENTER));
            const int32_t* first; int32_t count;
            children(v, first, count);
            for (int32_t c = 0; c < count; ++c) dfs(first[c]);
            if (with_leave) plan.ops.push_back(op_pack((uint32_t)ws.letter[(size_t)v], lev, (uint32_t)h, OP_LEAVE));
        };
        for (int32_t g : group) dfs(g);
        if (with_leave)
            for (int k = K - 1; k >= 0; --k) {
                const int32_t w = chain[(size_t)k];
                const int h = hmax + 1 + (K - 1 - k);
                plan.ops.push_back(op_pack((uint32_t)ws.letter[(size_t)w], (uint32_t)(k + 1), (uint32_t)h, OP_LEAVE));
            }
        ud.n_ops = (int32_t)plan.ops.size() - ud.op_off;
        ud.n_slots = (int32_t)plan.slot_word.size() - ud.slot_off;
        plan.max_slots = std::max(plan.max_slots, ud.n_slots);
        plan.fma_per_step += fma;
        plan.units.push_back(ud);
    };

    std::function<void(int32_t)> split = [&](int32_t u) {
        std::vector<int32_t> group;
        int64_t gsize = 0, gcost = 0;
        auto flush = [&]() {
            if (group.empty()) return;
            emit_unit(group);
            group.clear();
            gsize = gcost = 0;
        };
        const int32_t* first; int32_t count;
        children(u, first, count);
        const int64_t room = (int64_t)max_slots - (int64_t)chain.size();
        for (int32_t ci = 0; ci < count; ++ci) {
            const int32_t c = first[ci];
            const bool too_big = sub_size[(size_t)c] > room || sub_cost[(size_t)c] > 2 * target_cost;
            if (too_big && ws.height[(size_t)c] > 0) {
                flush();
                chain.push_back(c);
                split(c);
                chain.pop_back();
                continue;
            }
            if (!group.empty() && (gsize + sub_size[(size_t)c] > room || gcost + sub_cost[(size_t)c] > target_cost)) flush();
            group.push_back(c);
            gsize += sub_size[(size_t)c];
            gcost += sub_cost[(size_t)c];
        }
        flush();
    };
    if (n > 0) split(-1);
}

void build_plan_balanced(const WordSet& ws, int64_t n_units, int max_slots, bool with_leave, int cost_word, int cost_pair,
                         Plan& plan)
{
    const int64_t n = ws.size();
    plan = Plan();
    if (n == 0) return;
    n_units = std::max<int64_t>(1, std::min(n_units, n));
    max_slots = std::max(max_slots, ws.max_len + 1);

    // depth-first order, children by letter
    std::vector<int32_t> order;
    order.reserve((size_t)n);
    {
        std::vector<int32_t> stack;
        const int32_t r0 = ws.child_off[0], r1 = ws.child_off[1];
        for (int32_t c = r1 - 1; c >= r0; --c) stack.push_back(ws.child_list[(size_t)c]);
        while (!stack.empty()) {
            const int32_t w = stack.back();
            stack.pop_back();
            order.push_back(w);
            const int32_t c0 = ws.child_off[(size_t)(w + 1)], c1 = ws.child_off[(size_t)(w + 1) + 1];
            for (int32_t c = c1 - 1; c >= c0; --c) stack.push_back(ws.child_list[(size_t)c]);
        }
    }

    // One sweep: closes a unit before the word that would push its cost above `limit` (or its size above
    // max_slots).  path_h[m] = height, inside the current unit, of the word at level m on the current root path.
    // Returns the number of units; fills `cuts` (first position of every unit) when asked.
    std::vector<int> path_h((size_t)ws.max_len + 2, 0);
    auto sweep = [&](int64_t limit, std::vector<int64_t>* cuts) -> int64_t {
        int64_t units = 0, i = 0;
        while (i < n) {
            ++units;
            if (cuts) cuts->push_back(i);
            const int k0 = ws.length[(size_t)order[(size_t)i]];
            int64_t cost = 0, slots = k0 - 1;
            for (int m = 1; m < k0; ++m) {
                path_h[(size_t)m] = k0 - m;
                cost += cost_word + (int64_t)cost_pair * (k0 - m);
            }
            const int64_t start = i;
            for (int64_t j = start; j < n; ++j) {
                const int k = ws.length[(size_t)order[(size_t)j]];
                int64_t delta = cost_word;
                for (int m = 1; m < k; ++m)
                    if (k - m > path_h[(size_t)m]) delta += (int64_t)cost_pair * (k - m - path_h[(size_t)m]);
                if (j > start && (cost + delta > limit || slots + 1 > max_slots)) break;
                for (int m = 1; m < k; ++m) path_h[(size_t)m] = std::max(path_h[(size_t)m], k - m);
                path_h[(size_t)k] = 0;
                cost += delta;
                ++slots;
                i = j + 1;
            }
        }
        return units;
    };
    int64_t total = 0;
    for (int64_t w = 0; w < n; ++w) total += cost_word + (int64_t)cost_pair * ws.height[(size_t)w];
    int64_t lo = std::max<int64_t>(1, total / n_units), hi = total + (int64_t)ws.max_len * ws.max_len * (cost_word + cost_pair);
    while (lo < hi) {                               // smallest limit that needs no more than n_units units
        const int64_t mid = lo + (hi - lo) / 2;
        if (sweep(mid, nullptr) <= n_units) hi = mid; else lo = mid + 1;
    }
    std::vector<int64_t> cuts;
    sweep(lo, &cuts);
    cuts.push_back(n);

    struct Elem { int32_t word; int level; int h; bool own; };
    std::vector<Elem> el;
    std::vector<int> path_el((size_t)ws.max_len + 2, -1);
    std::vector<int> open;                          // indices into el of the ENTER ops not yet closed
    for (size_t u = 0; u + 1 < cuts.size(); ++u) {
        el.clear();
        const int32_t first = order[(size_t)cuts[u]];
        const int k0 = ws.length[(size_t)first];
        el.resize((size_t)k0 - 1);
        for (int32_t a = ws.parent[(size_t)first], m = k0 - 1; m >= 1; a = ws.parent[(size_t)a], --m) {
            el[(size_t)m - 1] = Elem{a, m, 0, false};
            path_el[(size_t)m] = m - 1;
        }
        for (int64_t j = cuts[u]; j < cuts[u + 1]; ++j) {
            const int32_t w = order[(size_t)j];
            const int k = ws.length[(size_t)w];
            for (int m = 1; m < k; ++m) {
                Elem& a = el[(size_t)path_el[(size_t)m]];
                a.h = std::max(a.h, k - m);
            }
            path_el[(size_t)k] = (int)el.size();
            el.push_back(Elem{w, k, 0, true});
        }
        UnitDesc ud;
        ud.op_off = (int32_t)plan.ops.size();
        ud.slot_off = (int32_t)plan.slot_word.size();
        open.clear();
        auto close_to = [&](int level) {            // closes every open ENTER at `level` or deeper
            while (!open.empty() && el[(size_t)open.back()].level >= level) {
                const Elem& e = el[(size_t)open.back()];
                if (with_leave)
                    plan.ops.push_back(op_pack((uint32_t)ws.letter[(size_t)e.word], (uint32_t)e.level, (uint32_t)e.h, OP_LEAVE));
                open.pop_back();
            }
        };
        for (size_t x = 0; x < el.size(); ++x) {
            const Elem& e = el[x];
            close_to(e.level);
            plan.slot_word.push_back(e.own ? e.word : ~e.word);
            plan.fma_per_step += 1 + e.h;
            plan.pairs_nonleaf += e.h;
            if (e.h == 0) {
                plan.ops.push_back(op_pack((uint32_t)ws.letter[(size_t)e.word], (uint32_t)e.level, 0, OP_LEAF));
                plan.leaves++;
            } else {
                plan.ops.push_back(op_pack((uint32_t)ws.letter[(size_t)e.word], (uint32_t)e.level, (uint32_t)e.h, OP_ENTER));
                open.push_back((int)x);
            }
        }
        close_to(0);
        ud.n_ops = (int32_t)plan.ops.size() - ud.op_off;
        ud.n_slots = (int32_t)plan.slot_word.size() - ud.slot_off;
        plan.max_slots = std::max(plan.max_slots, ud.n_slots);
        plan.units.push_back(ud);
    }
}

// ---------------------------------------------------------------------------------------------------------

static int check_d(int d) { return (d >= 1 && d <= 4096) ? SIG_OK : SIG_EINVAL; }

int build_truncated(int d, int depth, WordSet** out)
{
    if (!out) return SIG_EINVAL;
    if (check_d(d) != SIG_OK || depth < 1) return SIG_EINVAL;
    if (depth > SIG_MAX_WORD_LEN) return SIG_ETOOLARGE;
    // |W| = sum_{n=1..depth} d^n must stay below 2^31
    int64_t total = 0, pw = 1;
    std::vector<int64_t> start(1, 0);
    for (int n = 1; n <= depth; ++n) {
        if (pw > kMaxWords / d) return SIG_ETOOLARGE;
        pw *= d;
        start.push_back(total);
        total += pw;
        if (total > kMaxWords) return SIG_ETOOLARGE;
    }
    start.push_back(total);
    WordSet* ws = new (std::nothrow) WordSet;
    if (!ws) return SIG_ENOMEM;
    try {
        ws->d = d; ws->kind = 0; ws->depth = depth;
        ws->parent.resize((size_t)total);
        ws->letter.resize((size_t)total);
        ws->level_start.assign(start.begin(), start.end());   // [0, start(1)=0, start(2), ..., total]
        pw = 1;
        for (int n = 1; n <= depth; ++n) {
            pw *= d;
            const int64_t s = start[(size_t)n], sp = n >= 2 ? start[(size_t)n - 1] : 0;
            for (int64_t phi = 0; phi < pw; ++phi) {
                ws->letter[(size_t)(s + phi)] = (int32_t)(phi % d);
                ws->parent[(size_t)(s + phi)] = n == 1 ? -1 : (int32_t)(sp + phi / d);
            }
        }
        int rc = finish(ws);
        if (rc != SIG_OK) { delete ws; return rc; }
    } catch (const std::bad_alloc&) { delete ws; return SIG_ENOMEM; }
    *out = ws;
    return SIG_OK;
}

int build_anisotropic(int d, const double* weights, double cutoff, WordSet** out)
{
    if (!out || !weights) return SIG_EINVAL;
    if (check_d(d) != SIG_OK) return SIG_EINVAL;
    if (!(cutoff >= 0.0) || !std::isfinite(cutoff)) return SIG_EINVAL;
    double wmin = std::numeric_limits<double>::infinity();
    for (int i = 0; i < d; ++i) {
        if (!(weights[i] > 0.0) || !std::isfinite(weights[i])) return SIG_EINVAL;
        wmin = std::min(wmin, weights[i]);
    }
    if (cutoff / wmin > (double)SIG_MAX_WORD_LEN + 0.5) return SIG_ETOOLARGE;
    WordSet* ws = new (std::nothrow) WordSet;
    if (!ws) return SIG_ENOMEM;
    try {
        ws->d = d; ws->kind = 1;
        // breadth first: each level is generated from the previous one in (parent order, letter)
        // order, which is lexicographic order inside the level.
        std::vector<double> deg_prev(1, 0.0), deg_cur;
        std::vector<int32_t> idx_prev(1, -1);
        ws->level_start.assign(1, 0);
        ws->level_start.push_back(0);
        while (!deg_prev.empty()) {
            deg_cur.clear();
            std::vector<int32_t> idx_cur;
            for (size_t q = 0; q < deg_prev.size(); ++q)
                for (int i = 0; i < d; ++i) {
                    const double s = deg_prev[q] + weights[i];
                    if (s <= cutoff) {
                        if ((int64_t)ws->parent.size() >= kMaxWords) { delete ws; return SIG_ETOOLARGE; }
                        idx_cur.push_back((int32_t)ws->parent.size());
                        ws->parent.push_back(idx_prev[q]);
                        ws->letter.push_back(i);
                        deg_cur.push_back(s);
                    }
                }
            if (deg_cur.empty()) break;
            ws->level_start.push_back((int32_t)ws->parent.size());
            if ((int)ws->level_start.size() - 2 > SIG_MAX_WORD_LEN) { delete ws; return SIG_ETOOLARGE; }
            deg_prev.swap(deg_cur);
            idx_prev.swap(idx_cur);
        }
        if (ws->parent.empty()) { delete ws; return SIG_EEMPTYWORD; }   // no non-empty word is admissible
        int rc = finish(ws);
        if (rc != SIG_OK) { delete ws; return rc; }
    } catch (const std::bad_alloc&) { delete ws; return SIG_ENOMEM; }
    *out = ws;
    return SIG_OK;
}

int build_list(int d, const int32_t* letters, const int64_t* offsets, int64_t n_words, WordSet** out)
{
    if (!out || !offsets) return SIG_EINVAL;
    if (check_d(d) != SIG_OK || n_words < 0) return SIG_EINVAL;
    if (n_words == 0) return SIG_EEMPTYWORD;
    if (offsets[0] != 0) return SIG_EINVAL;
    for (int64_t k = 0; k < n_words; ++k) {
        const int64_t len = offsets[k + 1] - offsets[k];
        if (len < 0) return SIG_EINVAL;
        if (len == 0) return SIG_EEMPTYWORD;
        if (len > SIG_MAX_WORD_LEN) return SIG_ETOOLARGE;
    }
    if (!letters) return SIG_EINVAL;
    for (int64_t q = 0; q < offsets[n_words]; ++q)
        if (letters[q] < 0 || letters[q] >= d) return SIG_ELETTER;
    WordSet* ws = new (std::nothrow) WordSet;
    if (!ws) return SIG_ENOMEM;
    try {
        ws->d = d; ws->kind = 2;
        // trie of all prefixes; node 0 is the empty word
        struct Node { int32_t parent, letter, len; };
        std::vector<Node> nodes(1, Node{-1, -1, 0});
        std::unordered_map<uint64_t, int32_t> edge;
        edge.reserve((size_t)offsets[n_words] * 2 + 16);
        std::vector<int32_t> user_node((size_t)n_words);
        int max_len = 0;
        for (int64_t k = 0; k < n_words; ++k) {
            int32_t cur = 0;
            for (int64_t q = offsets[k]; q < offsets[k + 1]; ++q) {
                const uint64_t key = ((uint64_t)(uint32_t)cur << 32) | (uint32_t)letters[q];
                auto it = edge.find(key);
                if (it == edge.end()) {
                    if ((int64_t)nodes.size() > kMaxWords) { delete ws; return SIG_ETOOLARGE; }
                    const int32_t id = (int32_t)nodes.size();
                    nodes.push_back(Node{cur, letters[q], nodes[(size_t)cur].len + 1});
                    edge.emplace(key, id);
                    cur = id;
                } else cur = it->second;
            }
            user_node[(size_t)k] = cur;
            max_len = std::max(max_len, nodes[(size_t)cur].len);
        }
        // children lists sorted by letter, then breadth-first numbering = canonical order
        const size_t nn = nodes.size();
        std::vector<int32_t> coff(nn + 1, 0), clist(nn - 1);
        for (size_t v = 1; v < nn; ++v) coff[(size_t)nodes[v].parent + 1]++;
        for (size_t v = 1; v <= nn; ++v) coff[v] += coff[v - 1];
        {
            std::vector<int32_t> fill(coff.begin(), coff.end() - 1);
            for (size_t v = 1; v < nn; ++v) clist[(size_t)fill[(size_t)nodes[v].parent]++] = (int32_t)v;
        }
        for (size_t v = 0; v < nn; ++v)
            std::sort(clist.begin() + coff[v], clist.begin() + coff[v + 1],
                      [&](int32_t a, int32_t b) { return nodes[(size_t)a].letter < nodes[(size_t)b].letter; });
        std::vector<int32_t> canon(nn, -1);      // trie node -> canonical index
        std::vector<int32_t> level(1, 0), next;
        ws->level_start.assign(1, 0);
        ws->level_start.push_back(0);
        while (true) {
            next.clear();
            for (int32_t v : level)
                for (int32_t q = coff[(size_t)v]; q < coff[(size_t)v + 1]; ++q) {
                    const int32_t c = clist[(size_t)q];
                    canon[(size_t)c] = (int32_t)ws->parent.size();
                    ws->parent.push_back(v == 0 ? -1 : canon[(size_t)v]);
                    ws->letter.push_back(nodes[(size_t)c].letter);
                    next.push_back(c);
                }
            if (next.empty()) break;
            ws->level_start.push_back((int32_t)ws->parent.size());
            level.swap(next);
        }
        ws->user_index.resize((size_t)n_words);
        for (int64_t k = 0; k < n_words; ++k) ws->user_index[(size_t)k] = canon[(size_t)user_node[(size_t)k]];
        int rc = finish(ws);
        if (rc != SIG_OK) { delete ws; return rc; }
    } catch (const std::bad_alloc&) { delete ws; return SIG_ENOMEM; }
    *out = ws;
    return SIG_OK;
}

// Words of length <= depth whose consecutive letters are joined by an edge (Section 7.1, graph-induced word set).
// Generated level by level from the canonically ordered previous level with the successors of the last letter in
// increasing order, which is the canonical order already; build_list then makes the tables.
int build_graph(int d, const int32_t* edges, int64_t n_edges, int depth, WordSet** out)
{
    if (!out || check_d(d) != SIG_OK || n_edges < 0 || depth < 1 || (n_edges > 0 && !edges)) return SIG_EINVAL;
    if (depth > SIG_MAX_WORD_LEN) return SIG_ETOOLARGE;
    try {
        std::vector<std::vector<int32_t>> succ((size_t)d);
        for (int64_t e = 0; e < n_edges; ++e) {
            const int32_t a = edges[2 * e], b = edges[2 * e + 1];
            if (a < 0 || a >= d || b < 0 || b >= d) return SIG_ELETTER;
            succ[(size_t)a].push_back(b);
        }
        for (auto& v : succ) {
            std::sort(v.begin(), v.end());
            v.erase(std::unique(v.begin(), v.end()), v.end());
        }
        std::vector<int32_t> letters;
        std::vector<int64_t> offsets(1, 0);
        size_t lev_begin = 0;                        // first word of the previous level in `offsets`
        for (int i = 0; i < d; ++i) { letters.push_back(i); offsets.push_back((int64_t)letters.size()); }
        for (int n = 2; n <= depth; ++n) {
            const size_t lev_end = offsets.size() - 1;
            for (size_t w = lev_begin; w < lev_end; ++w) {
                const int64_t a = offsets[w], b = offsets[w + 1];
                const int32_t last = letters[(size_t)b - 1];
                for (int32_t nx : succ[(size_t)last]) {
                    if ((int64_t)offsets.size() > kMaxWords) return SIG_ETOOLARGE;
                    // the range is copied by index: letters may reallocate while it grows
                    for (int64_t q = a; q < b; ++q) letters.push_back(letters[(size_t)q]);
                    letters.push_back(nx);
                    offsets.push_back((int64_t)letters.size());
                }
            }
            if (offsets.size() - 1 == lev_end) break;      // no word of this length
            lev_begin = lev_end;
        }
        return build_list(d, letters.data(), offsets.data(), (int64_t)offsets.size() - 1, out);
    } catch (const std::bad_alloc&) { return SIG_ENOMEM; }
}

// Sparse lead-lag word set (Section 8): alphabet of 2 d letters, lag channel of coordinate i = letter i, lead channel
// = letter d + i; all concatenations of the generators (L_i), (l_i L_i), (L_i l_i) of length <= depth.  The set is
// not prefix-closed (l_i alone is not in it); build_list closes it and user_index locates the generated words.
int build_leadlag_sparse(int d, int depth, WordSet** out)
{
    if (!out || d < 1 || d > 2048 || depth < 1) return SIG_EINVAL;
    if (depth > SIG_MAX_WORD_LEN) return SIG_ETOOLARGE;
    try {
        std::vector<int32_t> letters;
        std::vector<int64_t> offsets(1, 0);
        // breadth-first over the number of generators; words can be reached in several ways (never, in fact: the
        // factorisation is unique, but duplicates would be harmless)
        size_t begin = 0, end = 0;                   // frontier = words [begin, end) of `offsets`; starts with the empty word
        bool first = true;
        while (first || begin < end) {
            const size_t nb = offsets.size() - 1;
            const size_t count = first ? 1 : end - begin;
            for (size_t f = 0; f < count; ++f) {
                const int64_t a = first ? 0 : offsets[begin + f], b = first ? 0 : offsets[begin + f + 1];
                const int64_t len = b - a;
                for (int g = 0; g < 3 * d; ++g) {
                    const int i = g % d, kind = g / d;            // 0: (L_i), 1: (l_i, L_i), 2: (L_i, l_i)
                    const int glen = kind == 0 ? 1 : 2;
                    if (len + glen > depth) continue;
                    if ((int64_t)offsets.size() > kMaxWords) return SIG_ETOOLARGE;
                    for (int64_t q = a; q < b; ++q) letters.push_back(letters[(size_t)q]);
                    if (kind == 0) letters.push_back(d + i);
                    else if (kind == 1) { letters.push_back(i); letters.push_back(d + i); }
                    else { letters.push_back(d + i); letters.push_back(i); }
                    offsets.push_back((int64_t)letters.size());
                }
            }
            first = false;
            begin = nb;
            end = offsets.size() - 1;
        }
        return build_list(2 * d, letters.data(), offsets.data(), (int64_t)offsets.size() - 1, out);
    } catch (const std::bad_alloc&) { return SIG_ENOMEM; }
}

// Lyndon words of length exactly n over {0..d-1} in lexicographic order (Duval's generation algorithm).
static void lyndon_words_of_length(int d, int n, std::vector<int32_t>& letters, std::vector<int64_t>& offsets)
{
    std::vector<int32_t> w(1, -1);
    while (!w.empty()) {
        w.back() += 1;
        if ((int)w.size() == n) {
            letters.insert(letters.end(), w.begin(), w.end());
            offsets.push_back((int64_t)letters.size());
        }
        const size_t m = w.size();
        while ((int)w.size() < n) w.push_back(w[w.size() - m]);
        while (!w.empty() && w.back() == d - 1) w.pop_back();
    }
}

bool trunc_forward_available(int d, int depth);      // kernels_trunc.hip
bool trunc_backward_available(int d, int depth);

int build_logsig(int d, int depth, WordSet** out)
{
    if (!out || check_d(d) != SIG_OK || depth < 1) return SIG_EINVAL;
    if (depth > SIG_MAX_KERNEL_LEN) return SIG_ETOOLARGE;
    try {
        // user list: the Lyndon words of length 1..depth, then every word of length depth - 1 (whose prefixes
        // complete the lower levels)
        std::vector<int32_t> letters;
        std::vector<int64_t> offsets(1, 0);
        for (int n = 1; n <= depth; ++n) lyndon_words_of_length(d, n, letters, offsets);
        const int64_t n_lyn = (int64_t)offsets.size() - 1;
        if (depth >= 2) {
            double cnt = 1.0;
            for (int k = 0; k < depth - 1; ++k) cnt *= d;
            if (cnt > (double)kMaxWords) return SIG_ETOOLARGE;
            std::vector<int32_t> w((size_t)depth - 1, 0);
            while (true) {
                letters.insert(letters.end(), w.begin(), w.end());
                offsets.push_back((int64_t)letters.size());
                int k = depth - 2;
                while (k >= 0 && w[(size_t)k] == d - 1) { w[(size_t)k] = 0; --k; }
                if (k < 0) break;
                w[(size_t)k] += 1;
            }
        }
        // Shapes with a kernel for the full truncation take that set instead (it holds every factor too, and its
        // kernels are several times faster than the specialised ones on the reduced set).
        WordSet* ws = nullptr;
        const bool full = trunc_forward_available(d, depth) && trunc_backward_available(d, depth);
        int rc = full ? build_truncated(d, depth, &ws)
                      : build_list(d, letters.data(), offsets.data(), (int64_t)offsets.size() - 1, &ws);
        if (rc != SIG_OK) return rc;
        ws->user_index.assign((size_t)n_lyn, 0);         // only the Lyndon words are "requested"; filled below
        // sub-word table: walk the trie by the parent/letter tables through a (parent, letter) -> child map
        std::unordered_map<uint64_t, int32_t> child;
        child.reserve((size_t)ws->size() * 2);
        for (int64_t v = 0; v < ws->size(); ++v)
            child.emplace(((uint64_t)(uint32_t)(ws->parent[(size_t)v] + 1) << 32) | (uint32_t)ws->letter[(size_t)v], (int32_t)v);
        ws->n_lyndon = n_lyn;
        ws->lyn_stride = (depth + 1) * (depth + 1);
        ws->lyn_len.assign((size_t)n_lyn, 0);
        ws->lyn_sub.assign((size_t)n_lyn * (size_t)ws->lyn_stride, -1);
        for (int64_t k = 0; k < n_lyn; ++k) {
            const int n = (int)(offsets[(size_t)k + 1] - offsets[(size_t)k]);
            const int32_t* w = letters.data() + offsets[(size_t)k];
            ws->lyn_len[(size_t)k] = n;
            for (int i = 0; i < n; ++i) {
                int32_t cur = -1;
                for (int j = i + 1; j <= n; ++j) {
                    auto it = child.find(((uint64_t)(uint32_t)(cur + 1) << 32) | (uint32_t)w[j - 1]);
                    if (it == child.end()) { delete ws; return SIG_EINVAL; }       // cannot happen: the set holds all factors
                    cur = it->second;
                    ws->lyn_sub[(size_t)k * (size_t)ws->lyn_stride + (size_t)i * (size_t)(depth + 1) + (size_t)j] = cur;
                }
            }
            ws->user_index[(size_t)k] = ws->lyn_sub[(size_t)k * (size_t)ws->lyn_stride + (size_t)n];   // the word itself
        }
        // inverse table (counting sort by sub-word)
        ws->lyn_pairs = depth * (depth + 1) / 2;
        ws->lyn_inv_off.assign((size_t)ws->size() + 1, 0);
        for (int64_t k = 0; k < n_lyn; ++k)
            for (int i = 0; i < ws->lyn_len[(size_t)k]; ++i)
                for (int j = i + 1; j <= ws->lyn_len[(size_t)k]; ++j)
                    ws->lyn_inv_off[(size_t)ws->lyn_sub[(size_t)k * (size_t)ws->lyn_stride + (size_t)i * (size_t)(depth + 1) + (size_t)j] + 1]++;
        for (int64_t u = 0; u < ws->size(); ++u) ws->lyn_inv_off[(size_t)u + 1] += ws->lyn_inv_off[(size_t)u];
        ws->lyn_inv.assign((size_t)ws->lyn_inv_off[(size_t)ws->size()], 0);
        {
            std::vector<int32_t> fill(ws->lyn_inv_off.begin(), ws->lyn_inv_off.end() - 1);
            for (int64_t k = 0; k < n_lyn; ++k) {
                int pair = 0;
                for (int i = 0; i < depth; ++i)
                    for (int j = i + 1; j <= depth; ++j, ++pair) {
                        if (j > ws->lyn_len[(size_t)k]) continue;
                        const int32_t u = ws->lyn_sub[(size_t)k * (size_t)ws->lyn_stride + (size_t)i * (size_t)(depth + 1) + (size_t)j];
                        ws->lyn_inv[(size_t)fill[(size_t)u]++] = (int32_t)(k * ws->lyn_pairs + pair);
                    }
            }
        }
        if ((int64_t)n_lyn * ws->lyn_pairs > 0x7fffffff) { delete ws; return SIG_ETOOLARGE; }
        // append the tables to the device image
        auto append = [&](const void* src, size_t bytes) {
            const size_t off = (ws->image.size() + 255) & ~(size_t)255;
            ws->image.resize(off + ((bytes + 255) & ~(size_t)255), 0);
            std::memcpy(&ws->image[off], src, bytes);
            return off;
        };
        ws->lyn_len_off = append(ws->lyn_len.data(), ws->lyn_len.size() * sizeof(int32_t));
        ws->lyn_sub_off = append(ws->lyn_sub.data(), ws->lyn_sub.size() * sizeof(int32_t));
        ws->lyn_inv_off_off = append(ws->lyn_inv_off.data(), ws->lyn_inv_off.size() * sizeof(int32_t));
        ws->lyn_inv_ent_off = append(ws->lyn_inv.data(), std::max<size_t>(ws->lyn_inv.size(), 1) * sizeof(int32_t));
        ws->depth = depth;
        *out = ws;
        return SIG_OK;
    } catch (const std::bad_alloc&) { return SIG_ENOMEM; }
}

}  // namespace sig
