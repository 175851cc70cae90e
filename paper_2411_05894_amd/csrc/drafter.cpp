// Host-side drafter of SSSD: input trie (App. A, Alg. 1), suffix-array datastore (Alg. 2) and the
// priority-queue merge of both into one draft tree (Alg. 3), plus the roofline rule for the
// speculation length (Sec. 3.2).  Plain C++17, no device code: the paper places drafting on the
// host so that the accelerator only runs the verification pass.
//
// Readings where the pseudocode leaves a choice (the paper presents it as a logical equivalent of
// its implementation, not the implementation itself):
//  * a node's probability is count(node) / count(parent); along a path the factors telescope to
//    count(v) / count(u), the definition the text gives for a prefix node u and a descendant v;
//  * children are visited in ascending token id; the queue pops the largest probability, the
//    element pushed first among equals;
//  * Alg. 2 shortens the ORIGINAL prefix by one token per round (lengths P, P-1, ..., 2) while
//    the tree has fewer than max_tree_nodes nodes; each sub-index is sampled with step
//    max(1, floor(matches / (max_samples / sub-indices)));
//  * no draft node lies deeper than branch_len below the root, whatever its source;
//  * dec_len counts the root, so it is the speculation length s_q.
#include "../../include/sssd_draft.h"

#include <algorithm>
#include <cstring>
#include <deque>
#include <map>
#include <new>
#include <queue>
#include <vector>

namespace {

struct TrieNode {
    int32_t token;
    int32_t parent;
    int32_t depth;
    int64_t count;
    std::map<int32_t, int32_t> children;   // token -> node, ascending token order
};

// Counted trie.  Node 0 is the root.
struct Trie {
    std::vector<TrieNode> nodes;
    Trie() { clear(0); }
    void clear(int32_t root_token)
    {
        nodes.clear();
        nodes.push_back(TrieNode{root_token, -1, 0, 0, {}});
    }
    int32_t child(int32_t node, int32_t token) const
    {
        auto it = nodes[node].children.find(token);
        return it == nodes[node].children.end() ? -1 : it->second;
    }
    int32_t child_or_add(int32_t node, int32_t token)
    {
        const int32_t c = child(node, token);
        if (c >= 0) return c;
        const int32_t id = (int32_t)nodes.size();
        nodes.push_back(TrieNode{token, node, nodes[node].depth + 1, 0, {}});
        nodes[node].children[token] = id;
        return id;
    }
    // Alg. 2's Insert: add the missing nodes of the path with count 1, increment the existing ones.
    void insert_path(const int32_t *tok, int n)
    {
        int32_t node = 0;
        nodes[0].count += 1;
        for (int i = 0; i < n; ++i) {
            node = child_or_add(node, tok[i]);
            nodes[node].count += 1;
        }
    }
};

struct Input {
    std::vector<int32_t> tokens;
    Trie trie;
    std::vector<int32_t> tails;   // tails[m-1] = node of the last m tokens, m = 1 .. min(len, depth)
};

struct SubIndex {
    std::vector<int32_t> text;
    std::vector<int64_t> sa;
};

}  // namespace

struct sssd_drafter {
    sssd_draft_params p;
    int depth;   // trie depth = prefix_len + branch_len
    std::vector<Input> inputs;
    std::deque<SubIndex> subs;
};

namespace {

// Compare the suffix at `pos` with key[0..n): -1, 0 (key is a prefix of the suffix), +1.  A suffix
// that ends inside the key is smaller than the key.
int cmp_suffix_key(const SubIndex &s, int64_t pos, const int32_t *key, int n)
{
    const int64_t N = (int64_t)s.text.size();
    for (int i = 0; i < n; ++i) {
        if (pos + i >= N) return -1;
        const int32_t a = s.text[pos + i];
        if (a != key[i]) return a < key[i] ? -1 : 1;
    }
    return 0;
}

// [lo, hi) of the suffix array whose suffixes start with key: two binary searches (App. A.2).
void sa_range(const SubIndex &s, const int32_t *key, int n, int64_t &lo, int64_t &hi)
{
    int64_t a = 0, b = (int64_t)s.sa.size();
    while (a < b) {
        const int64_t m = a + (b - a) / 2;
        if (cmp_suffix_key(s, s.sa[m], key, n) < 0) a = m + 1;
        else b = m;
    }
    lo = a;
    b = (int64_t)s.sa.size();
    while (a < b) {
        const int64_t m = a + (b - a) / 2;
        if (cmp_suffix_key(s, s.sa[m], key, n) <= 0) a = m + 1;
        else b = m;
    }
    hi = a;
}

// Alg. 2: tree of sampled continuations of the tail, rooted at the last token.
void datastore_tree(const sssd_drafter &d, const Input &in, Trie &tree)
{
    const int len = (int)in.tokens.size();
    const int P = std::min(d.p.prefix_len, len);
    tree.clear(in.tokens[len - 1]);
    if (d.subs.empty()) return;
    const int n_sub = (int)d.subs.size();
    const int64_t quota = std::max<int64_t>(1, d.p.max_samples / n_sub);
    for (int iter = 0; iter < P - 1 && (int)tree.nodes.size() < d.p.max_tree_nodes; ++iter) {
        const int n = P - iter;
        const int32_t *key = in.tokens.data() + (len - n);
        for (const SubIndex &s : d.subs) {
            int64_t lo, hi;
            sa_range(s, key, n, lo, hi);
            const int64_t step = std::max<int64_t>(1, (hi - lo) / quota);
            for (int64_t i = lo; i < hi; i += step) {
                const int64_t at = s.sa[i] + n, N = (int64_t)s.text.size();
                const int m = (int)std::min<int64_t>(d.p.branch_len, N - at);
                tree.insert_path(s.text.data() + at, m > 0 ? m : 0);
            }
        }
    }
}

struct QueueItem {
    double prob;
    int64_t seq;
    const Trie *tree;
    int32_t node;        // node of the source tree
    int32_t parent;      // node of the draft tree it hangs under
    int32_t depth;       // depth of the draft node it would become
    double child_disc;
};
struct QueueOrder {
    bool operator()(const QueueItem &a, const QueueItem &b) const
    {
        if (a.prob != b.prob) return a.prob < b.prob;   // max-heap on probability
        return a.seq > b.seq;                           // earlier push first among equals
    }
};

bool seq_ok(const sssd_drafter *d, int32_t seq) { return d && seq >= 0 && seq < (int32_t)d->inputs.size(); }

}  // namespace

extern "C" {

void sssd_draft_default_params(sssd_draft_params *p)
{
    if (!p) return;
    p->prefix_len = 4;
    p->branch_len = 4;
    p->max_tree_nodes = 50;
    p->max_samples = 100;
    p->max_sub_indices = 8;
    p->input_discount = 0.6;
    p->datastore_match = 4.0;
    p->child_disc_base = 0.6;
    p->child_disc_per_match = 0.1;
}

int sssd_draft_create(const sssd_draft_params *p, int32_t n_sequences, sssd_drafter **out)
{
    if (!p || !out || n_sequences <= 0) return SSSD_EINVAL;
    if (p->prefix_len < 1 || p->branch_len < 1 || p->prefix_len + p->branch_len > 64 || p->max_tree_nodes < 1 ||
        p->max_samples < 1 || p->max_sub_indices < 1)
        return SSSD_EINVAL;
    sssd_drafter *d = new (std::nothrow) sssd_drafter();
    if (!d) return SSSD_EINVAL;
    d->p = *p;
    d->depth = p->prefix_len + p->branch_len;
    d->inputs.resize(n_sequences);
    *out = d;
    return SSSD_OK;
}

int sssd_draft_destroy(sssd_drafter *d)
{
    if (!d) return SSSD_EINVAL;
    delete d;
    return SSSD_OK;
}

int sssd_draft_input_reset(sssd_drafter *d, int32_t seq)
{
    if (!seq_ok(d, seq)) return SSSD_EINVAL;
    Input &in = d->inputs[seq];
    in.tokens.clear();
    in.trie.clear(0);
    in.tails.clear();
    return SSSD_OK;
}

int sssd_draft_input_append(sssd_drafter *d, int32_t seq, const int32_t *tokens, int32_t n)
{
    if (!seq_ok(d, seq) || n < 0 || (n > 0 && !tokens)) return SSSD_EINVAL;
    Input &in = d->inputs[seq];
    for (int32_t i = 0; i < n; ++i) {
        const int32_t t = tokens[i];
        // n-grams ending at this token: the 1-gram, and every n-gram that ended at the previous
        // token extended by it (up to the trie depth)
        std::vector<int32_t> next;
        next.reserve(in.tails.size() + 1);
        next.push_back(in.trie.child_or_add(0, t));
        for (int32_t node : in.tails)
            if (in.trie.nodes[node].depth < d->depth) next.push_back(in.trie.child_or_add(node, t));
        for (int32_t node : next) in.trie.nodes[node].count += 1;
        in.trie.nodes[0].count += 1;
        in.tails.swap(next);
        in.tokens.push_back(t);
    }
    return SSSD_OK;
}

int sssd_draft_datastore_add(sssd_drafter *d, const int32_t *tokens, int64_t n)
{
    if (!d || n < 0 || (n > 0 && !tokens)) return SSSD_EINVAL;
    SubIndex s;
    s.text.assign(tokens, tokens + n);
    s.sa.resize(n);
    for (int64_t i = 0; i < n; ++i) s.sa[i] = i;
    const int L = d->depth;
    const std::vector<int32_t> &tx = s.text;
    std::sort(s.sa.begin(), s.sa.end(), [&](int64_t a, int64_t b) {
        for (int i = 0; i < L; ++i) {
            const bool ea = a + i >= n, eb = b + i >= n;
            if (ea || eb) {
                if (ea != eb) return ea;   // the suffix that ends first is the smaller one
                break;
            }
            if (tx[a + i] != tx[b + i]) return tx[a + i] < tx[b + i];
        }
        return a < b;
    });
    d->subs.push_back(std::move(s));
    while ((int)d->subs.size() > d->p.max_sub_indices) d->subs.pop_front();   // the oldest goes (Sec. 3.1.3)
    return SSSD_OK;
}

int sssd_draft_propose(sssd_drafter *d, int32_t seq, int32_t dec_len, int32_t *tokens, int32_t *parents,
                       int32_t *n_nodes)
{
    if (!seq_ok(d, seq) || dec_len < 1 || !tokens || !parents || !n_nodes) return SSSD_EINVAL;
    const Input &in = d->inputs[seq];
    if (in.tokens.empty()) return SSSD_EINVAL;

    Trie ds_tree;
    datastore_tree(*d, in, ds_tree);

    // draft tree: token, parent, children by token
    struct DraftNode {
        int32_t token, parent;
        std::map<int32_t, int32_t> children;
    };
    std::vector<DraftNode> draft;
    draft.push_back(DraftNode{in.tokens.back(), 0, {}});

    std::priority_queue<QueueItem, std::vector<QueueItem>, QueueOrder> pq;
    int64_t pushed = 0;
    auto push_children = [&](const Trie &tree, int32_t node, double prob, double factor, double child_disc, int32_t parent,
                             int32_t depth) {
        if (depth > d->p.branch_len) return;
        const TrieNode &n = tree.nodes[node];
        for (const auto &kv : n.children) {
            const TrieNode &c = tree.nodes[kv.second];
            const double cp = (double)c.count / (double)n.count;
            pq.push(QueueItem{cp * prob * factor, pushed++, &tree, kv.second, parent, depth, child_disc});
        }
    };
    // all_trees = [<datastore tree, datastore_match>] followed by the input matches, longest first
    if (ds_tree.nodes.size() > 1)
        push_children(ds_tree, 0, 1.0, 1.0, d->p.child_disc_base + d->p.child_disc_per_match * d->p.datastore_match, 0, 1);
    const int n_match = (int)in.tails.size() < d->p.prefix_len ? (int)in.tails.size() : d->p.prefix_len;
    for (int m = n_match; m >= 1; --m)
        push_children(in.trie, in.tails[m - 1], 1.0, d->p.input_discount,
                      d->p.child_disc_base + d->p.child_disc_per_match * (double)m, 0, 1);

    while (!pq.empty() && (int32_t)draft.size() < dec_len) {
        const QueueItem el = pq.top();
        pq.pop();
        const int32_t tok = el.tree->nodes[el.node].token;
        int32_t id;
        auto it = draft[el.parent].children.find(tok);
        if (it != draft[el.parent].children.end()) {
            id = it->second;
        } else {
            id = (int32_t)draft.size();
            draft.push_back(DraftNode{tok, el.parent, {}});
            draft[el.parent].children[tok] = id;
        }
        push_children(*el.tree, el.node, el.prob, el.child_disc, el.child_disc, id, el.depth + 1);
    }
    for (size_t i = 0; i < draft.size(); ++i) {
        tokens[i] = draft[i].token;
        parents[i] = draft[i].parent;
    }
    *n_nodes = (int32_t)draft.size();
    return SSSD_OK;
}

int32_t sssd_draft_speculation_length(double peak_flops, double peak_bytes_per_s, int32_t b, int32_t cap)
{
    if (!(peak_flops > 0.0) || !(peak_bytes_per_s > 0.0) || b < 1 || cap < 1) return 1;
    const double knee = peak_flops / peak_bytes_per_s;
    double sq = knee / (double)b + 0.5;   // to the nearest integer (the paper's example: 173.7 / 8 -> 22)
    if (sq < 1.0) sq = 1.0;
    if (sq > (double)cap) sq = (double)cap;
    return (int32_t)sq;
}

int64_t sssd_draft_input_count(const sssd_drafter *d, int32_t seq, const int32_t *gram, int32_t n)
{
    if (!seq_ok(d, seq) || n < 0 || (n > 0 && !gram)) return 0;
    const Trie &t = d->inputs[seq].trie;
    int32_t node = 0;
    for (int32_t i = 0; i < n; ++i) {
        node = t.child(node, gram[i]);
        if (node < 0) return 0;
    }
    return t.nodes[node].count;
}

int32_t sssd_draft_match_input(const sssd_drafter *d, int32_t seq, int32_t *match_len)
{
    if (!seq_ok(d, seq) || !match_len) return SSSD_EINVAL;
    const Input &in = d->inputs[seq];
    // Nothing is searched here: appending a token extends the node of every suffix that ended at the
    // previous token, so tails[m-1] already IS the trie node of the last m tokens (the matches Alg. 1
    // looks for).  Reported: the suffix lengths sssd_draft_propose seeds its queue from, longest first.
    const int32_t n_match = std::min<int32_t>((int32_t)in.tails.size(), d->p.prefix_len);
    int32_t found = 0;
    for (int32_t m = n_match; m >= 1; --m) {
        const TrieNode &nd = in.trie.nodes[in.tails[m - 1]];
        if (nd.depth == m && nd.count > 0) match_len[found++] = m;
    }
    return found;
}

int sssd_draft_datastore_lookup(const sssd_drafter *d, int32_t sub, const int32_t *prefix, int32_t n, int64_t *positions,
                                int64_t max_out, int64_t *total)
{
    if (!d || sub < 0 || sub >= (int32_t)d->subs.size() || n < 0 || (n > 0 && !prefix) || !total || max_out < 0 ||
        (max_out > 0 && !positions))
        return SSSD_EINVAL;
    const SubIndex &s = d->subs[sub];
    int64_t lo, hi;
    sa_range(s, prefix, n, lo, hi);
    *total = hi - lo;
    for (int64_t i = lo; i < hi && i - lo < max_out; ++i) positions[i - lo] = s.sa[i];
    return SSSD_OK;
}

int sssd_draft_datastore_tree(const sssd_drafter *d, int32_t seq, int32_t *tokens, int32_t *parents, int64_t *counts,
                              int32_t *n_nodes)
{
    if (!seq_ok(d, seq) || !tokens || !parents || !counts || !n_nodes) return SSSD_EINVAL;
    const Input &in = d->inputs[seq];
    if (in.tokens.empty()) return SSSD_EINVAL;
    Trie tree;
    datastore_tree(*d, in, tree);
    for (size_t i = 0; i < tree.nodes.size(); ++i) {
        tokens[i] = tree.nodes[i].token;
        parents[i] = i == 0 ? 0 : tree.nodes[i].parent;
        counts[i] = tree.nodes[i].count;
    }
    *n_nodes = (int32_t)tree.nodes.size();
    return SSSD_OK;
}

}  // extern "C"
