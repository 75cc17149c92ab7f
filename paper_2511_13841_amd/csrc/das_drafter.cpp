// Adaptive nonparametric drafter (Sec. 4.1.2 of the paper): online suffix trees over a window of recent rollouts.
// Host code behind include/das_drafter.h.
//
// One SuffixTree per epoch, built with Ukkonen's online construction over the concatenation of the epoch's rollouts, each
// followed by a unique negative terminator, so that (a) every suffix ends in a leaf once a rollout has been added and (b) no
// match runs across two rollouts.  Every node keeps the number of leaves below it (= occurrences of its path label), updated
// on the way up when a leaf is created, so that a draft can follow the most frequent continuation.
#include "../../include/das_drafter.h"

#include <cstdint>
#include <deque>
#include <new>
#include <unordered_map>
#include <vector>

namespace {

struct Node {
    int32_t start = 0, end = 0;           // edge label text[start, end); leaves: end = OPEN
    int32_t link = 0, parent = -1;
    int32_t first_kid = -1, next_sib = -1, prev_sib = -1;
    int32_t count = 0;                     // leaves below (a leaf counts itself)
};

constexpr int32_t OPEN = INT32_MAX;

class SuffixTree {
public:
    SuffixTree() { nodes_.emplace_back(); }     // node 0 = root

    void add_rollout(const int32_t *tok, int32_t n) {
        for (int32_t i = 0; i < n; ++i) extend(tok[i]);
        extend(next_terminator_--);              // unique, negative: makes every suffix explicit, matches nothing
    }
    int64_t tokens() const { return (int64_t)text_.size(); }
    int64_t node_count() const { return (int64_t)nodes_.size(); }

    // Longest suffix of ctx[0..m) that is a substring of the text (matching statistics with suffix links): leaves the
    // locus in (node, kid, off): the match ends `off` tokens down the edge to `kid` (off == 0: exactly at `node`).
    int32_t longest_suffix_match(const int32_t *ctx, int32_t m, int32_t &node, int32_t &kid, int32_t &off) const {
        int32_t v = 0, c = -1, o = 0, depth = 0;
        int32_t lo = 0;                           // the current match is ctx[lo, i)
        for (int32_t i = 0; i < m; ++i) {
            const int32_t x = ctx[i];
            for (;;) {
                if (o == 0) {                     // at node v
                    const int32_t ch = child(v, x);
                    if (ch >= 0) { c = ch; o = 1; ++depth; if (edge_len(c) == 1) { v = c; c = -1; o = 0; } break; }
                } else if (text_[nodes_[c].start + o] == x) {
                    ++o; ++depth;
                    if (o == edge_len(c)) { v = c; c = -1; o = 0; }
                    break;
                }
                if (depth == 0) break;            // x does not occur at all: empty match, move on
                // drop the first token of the match: suffix link of v, then walk down again over the remembered edge part
                ++lo; --depth;
                int32_t from, len;                // tokens still to be re-read below the link target: ctx[from, from+len)
                if (o == 0) { from = 0; len = 0; } else { from = i - o; len = o; }
                if (v == 0) {                     // at the root there is no link: the dropped token was on this edge
                    if (o == 0) { /* depth was >0 but at root with o==0 cannot happen */ }
                    else { from += 1; len -= 1; }
                } else {
                    v = nodes_[v].link;
                }
                c = -1; o = 0;
                while (len > 0) {                 // skip/count: the path exists, only edge lengths matter
                    const int32_t ch = child(v, ctx[from]);
                    const int32_t el = edge_len(ch);
                    if (len >= el) { v = ch; from += el; len -= el; }
                    else { c = ch; o = len; len = 0; }
                }
            }
        }
        (void)lo;
        node = v; kid = c; off = o;
        return depth;
    }

    // up to k tokens along the matched path: forced inside an edge, most frequent continuation at a node
    int32_t draft(int32_t v, int32_t c, int32_t o, int32_t k, int32_t *out) const {
        int32_t n = 0;
        while (n < k) {
            if (o == 0) {
                int32_t best = -1;
                for (int32_t ch = nodes_[v].first_kid; ch >= 0; ch = nodes_[ch].next_sib) {
                    const int32_t t = text_[nodes_[ch].start];
                    if (t < 0) continue;          // a rollout ended here: not a continuation
                    if (best < 0 || nodes_[ch].count > nodes_[best].count ||
                        (nodes_[ch].count == nodes_[best].count && t < text_[nodes_[best].start]))
                        best = ch;
                }
                if (best < 0) break;
                c = best; o = 0;
            }
            const int32_t t = text_[nodes_[c].start + o];
            if (t < 0) break;
            out[n++] = t;
            if (++o == edge_len(c)) { v = c; c = -1; o = 0; }
        }
        return n;
    }

private:
    std::vector<int32_t> text_;
    std::vector<Node> nodes_;
    std::unordered_map<uint64_t, int32_t> kids_;      // (node, first token of the edge) -> child
    int32_t active_node_ = 0, active_edge_ = 0, active_len_ = 0, remainder_ = 0;
    int32_t next_terminator_ = -1;

    static uint64_t key(int32_t node, int32_t tok) { return ((uint64_t)(uint32_t)node << 32) | (uint32_t)tok; }
    int32_t child(int32_t node, int32_t tok) const {
        auto it = kids_.find(key(node, tok));
        return it == kids_.end() ? -1 : it->second;
    }
    int32_t edge_len(int32_t n) const {
        const int32_t e = nodes_[n].end == OPEN ? (int32_t)text_.size() : nodes_[n].end;
        return e - nodes_[n].start;
    }
    int32_t new_node(int32_t start, int32_t end) {
        Node nd;
        nd.start = start; nd.end = end;
        nodes_.push_back(nd);
        return (int32_t)nodes_.size() - 1;
    }
    void attach(int32_t parent, int32_t kid) {        // kid becomes the first child of parent
        Node &k = nodes_[kid];
        k.parent = parent; k.prev_sib = -1; k.next_sib = nodes_[parent].first_kid;
        if (k.next_sib >= 0) nodes_[k.next_sib].prev_sib = kid;
        nodes_[parent].first_kid = kid;
        kids_[key(parent, text_[k.start])] = kid;
    }
    void replace(int32_t parent, int32_t old_kid, int32_t new_kid) {   // new_kid takes old_kid's place in the sibling list
        Node &o = nodes_[old_kid], &n = nodes_[new_kid];
        n.parent = parent; n.prev_sib = o.prev_sib; n.next_sib = o.next_sib;
        if (n.prev_sib >= 0) nodes_[n.prev_sib].next_sib = new_kid; else nodes_[parent].first_kid = new_kid;
        if (n.next_sib >= 0) nodes_[n.next_sib].prev_sib = new_kid;
        kids_[key(parent, text_[n.start])] = new_kid;
        o.prev_sib = o.next_sib = -1;
    }
    void new_leaf(int32_t parent, int32_t start) {
        const int32_t leaf = new_node(start, OPEN);
        nodes_[leaf].count = 1;
        attach(parent, leaf);
        for (int32_t v = parent; v >= 0; v = nodes_[v].parent) ++nodes_[v].count;
    }

    // Ukkonen: extend the implicit suffix tree of text_ by one token
    void extend(int32_t x) {
        text_.push_back(x);
        const int32_t pos = (int32_t)text_.size() - 1;
        ++remainder_;
        int32_t last_internal = -1;
        while (remainder_ > 0) {
            if (active_len_ == 0) active_edge_ = pos;
            const int32_t ch = child(active_node_, text_[active_edge_]);
            if (ch < 0) {
                new_leaf(active_node_, pos);
                if (last_internal >= 0) { nodes_[last_internal].link = active_node_; last_internal = -1; }
            } else {
                const int32_t el = edge_len(ch);
                if (active_len_ >= el) {              // walk down
                    active_edge_ += el; active_len_ -= el; active_node_ = ch;
                    continue;
                }
                if (text_[nodes_[ch].start + active_len_] == x) {      // already there: the suffix stays implicit
                    ++active_len_;
                    if (last_internal >= 0) { nodes_[last_internal].link = active_node_; last_internal = -1; }
                    break;
                }
                // split the edge: active_node -> mid -> {ch, new leaf}
                const int32_t mid = new_node(nodes_[ch].start, nodes_[ch].start + active_len_);
                nodes_[mid].count = nodes_[ch].count;
                replace(active_node_, ch, mid);
                nodes_[ch].start += active_len_;
                attach(mid, ch);
                new_leaf(mid, pos);
                if (last_internal >= 0) nodes_[last_internal].link = mid;
                last_internal = mid;
            }
            --remainder_;
            if (active_node_ == 0 && active_len_ > 0) { --active_len_; active_edge_ = pos - remainder_ + 1; }
            else if (active_node_ != 0) active_node_ = nodes_[active_node_].link;
        }
    }
};

}  // namespace

struct das_drafter {
    int32_t max_epochs = 1;
    std::deque<SuffixTree> epochs;
};

extern "C" int das_drafter_create(int32_t max_epochs, das_drafter **out) {
    if (!out || max_epochs < 1) return DAS_DRAFTER_ERR_INVALID;
    das_drafter *d = new (std::nothrow) das_drafter;
    if (!d) return DAS_DRAFTER_ERR_NOMEM;
    d->max_epochs = max_epochs;
    d->epochs.emplace_back();
    *out = d;
    return DAS_DRAFTER_OK;
}

extern "C" int das_drafter_free(das_drafter *d) {
    if (!d) return DAS_DRAFTER_ERR_INVALID;
    delete d;
    return DAS_DRAFTER_OK;
}

extern "C" int das_drafter_new_epoch(das_drafter *d) {
    if (!d) return DAS_DRAFTER_ERR_INVALID;
    try {
        d->epochs.emplace_back();
    } catch (const std::bad_alloc &) { return DAS_DRAFTER_ERR_NOMEM; }
    while ((int32_t)d->epochs.size() > d->max_epochs) d->epochs.pop_front();
    return DAS_DRAFTER_OK;
}

extern "C" int das_drafter_add(das_drafter *d, const int32_t *tokens, int32_t n) {
    if (!d || !tokens || n < 1) return DAS_DRAFTER_ERR_INVALID;
    for (int32_t i = 0; i < n; ++i)
        if (tokens[i] < 0) return DAS_DRAFTER_ERR_INVALID;
    try {
        d->epochs.back().add_rollout(tokens, n);
    } catch (const std::bad_alloc &) { return DAS_DRAFTER_ERR_NOMEM; }
    return DAS_DRAFTER_OK;
}

extern "C" int das_drafter_propose(das_drafter *d, const int32_t *ctx, int32_t m, int32_t max_match, int32_t min_match, int32_t k,
                                   int32_t *match_len, int32_t *draft, int32_t *n_draft) {
    if (!d || !match_len || !n_draft || m < 0 || (m > 0 && !ctx) || max_match < 0 || min_match < 0 || k < 0 || (k > 0 && !draft))
        return DAS_DRAFTER_ERR_INVALID;
    const int32_t use = m < max_match ? m : max_match;
    const int32_t *tail = ctx + (m - use);
    for (int32_t i = 0; i < use; ++i)
        if (tail[i] < 0) return DAS_DRAFTER_ERR_INVALID;
    int32_t best_len = 0, bn = 0, bc = -1, bo = 0;
    const SuffixTree *best = nullptr;
    for (auto it = d->epochs.rbegin(); it != d->epochs.rend(); ++it) {       // newest first: ties stay with the newest
        int32_t v, c, o;
        const int32_t len = it->longest_suffix_match(tail, use, v, c, o);
        if (len > best_len) { best_len = len; best = &*it; bn = v; bc = c; bo = o; }
    }
    *match_len = best_len;
    *n_draft = (best && best_len >= min_match && best_len > 0 && k > 0) ? best->draft(bn, bc, bo, k, draft) : 0;
    return DAS_DRAFTER_OK;
}

extern "C" int das_drafter_size(das_drafter *d, int64_t *tokens, int64_t *nodes, int32_t *epochs) {
    if (!d || !tokens || !nodes || !epochs) return DAS_DRAFTER_ERR_INVALID;
    int64_t t = 0, n = 0;
    for (const auto &e : d->epochs) { t += e.tokens(); n += e.node_count(); }
    *tokens = t; *nodes = n; *epochs = (int32_t)d->epochs.size();
    return DAS_DRAFTER_OK;
}
