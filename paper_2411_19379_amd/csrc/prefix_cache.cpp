// Radix tree with judicious admission of SSM states and FLOP-aware eviction (Sections 4.1 to 4.3, Eq. 1 and 2,
// Table 1).  Host code only; built into its own shared library, apart from the GPU library.
//
// Tree invariants, kept by every operation:
//   * an edge is a non-empty run of tokens; a node sits at the end of its edge and knows its depth in tokens;
//   * every node other than the root holds a state, or has at least two children (a branch point): a node with
//     one child and no state is merged into that child at once, and a leaf without a state does not arise because
//     the state after a sequence's last token is always cached;
//   * KVs are accounted per token of every edge, SSM states per state-holding node.
#include "prefix_cache.h"

#include <algorithm>
#include <map>
#include <memory>
#include <new>
#include <string>
#include <vector>

namespace {

thread_local std::string g_error;

int fail(int code, const char *msg)
{
    g_error = msg;
    return code;
}

struct Node {
    Node *parent = nullptr;
    std::vector<int32_t> edge;          // tokens from the parent's depth to this node's depth
    int32_t depth = 0;                  // tokens from the root to the end of the edge
    std::map<int32_t, Node *> children; // by first token of the child's edge
    bool has_state = false;
    int64_t handle = -1;
    int64_t last_access = 0;
    int32_t pins = 0;
    int32_t holder_index = -1;          // position in the cache's list of state-holding nodes, -1 if none
};

double prefill_flops(const pc_config_t &c, int64_t L)
{
    // Table 1, first row, summed over the layers
    const double D = (double)c.d_model, N = (double)c.d_state, Lf = (double)L;
    const double attn = 8.0 * Lf * D * D + 4.0 * Lf * Lf * D;
    const double mlp = 16.0 * Lf * D * D;
    const double ssm = 12.0 * Lf * D * D + 16.0 * Lf * D * N + 10.0 * Lf;
    return c.n_attn_layers * attn + c.n_mlp_layers * mlp + c.n_ssm_layers * ssm;
}

}  // namespace

struct pc_cache {
    pc_config_t cfg;
    Node root;
    int64_t kv_tokens = 0;
    int64_t n_states = 0;
    int64_t n_nodes = 0;
    std::vector<Node *> holders;    // every node that holds a state, in no particular order
    std::vector<double> scratch_ts, scratch_fe, scratch_s;
    std::vector<int64_t> released;  // of the last pc_finish: evicted, then rejected
    int32_t n_evicted_last = 0;

    int64_t kv_bytes_per_token() const { return (int64_t)cfg.n_attn_layers * 4 * cfg.d_model; }
    int64_t ssm_bytes_per_state() const
    {
        return (int64_t)cfg.n_ssm_layers * (2 * (int64_t)cfg.d_model * cfg.d_state + cfg.conv_state_bytes);
    }
    int64_t used_bytes() const { return kv_tokens * kv_bytes_per_token() + n_states * ssm_bytes_per_state(); }

    ~pc_cache() { free_subtree(&root); }

    void free_subtree(Node *n)
    {
        for (auto &kv : n->children) {
            free_subtree(kv.second);
            delete kv.second;
        }
        n->children.clear();
    }

    // Follow tokens[0..n) from the root.  Returns the last node whose whole edge was matched; *matched is the
    // number of matched tokens, *child / *in_edge describe a partial match into the next edge (in_edge > 0).
    Node *walk(const int32_t *tokens, int32_t n, int32_t *matched, Node **child, int32_t *in_edge)
    {
        Node *cur = &root;
        int32_t pos = 0;
        *child = nullptr;
        *in_edge = 0;
        while (pos < n) {
            auto it = cur->children.find(tokens[pos]);
            if (it == cur->children.end())
                break;
            Node *c = it->second;
            const int32_t elen = (int32_t)c->edge.size();
            int32_t k = 0;
            while (k < elen && pos + k < n && c->edge[k] == tokens[pos + k])
                ++k;
            if (k < elen) {
                *child = c;
                *in_edge = k;
                pos += k;
                break;
            }
            pos += elen;
            cur = c;
        }
        *matched = pos;
        return cur;
    }

    // Cut the edge of `c` after its first k tokens (0 < k < edge length); returns the new node in between.
    Node *split(Node *c, int32_t k)
    {
        Node *mid = new Node();
        mid->parent = c->parent;
        mid->edge.assign(c->edge.begin(), c->edge.begin() + k);
        mid->depth = c->depth - ((int32_t)c->edge.size() - k);
        mid->last_access = c->last_access;
        c->parent->children[mid->edge[0]] = mid;
        c->edge.erase(c->edge.begin(), c->edge.begin() + k);
        c->parent = mid;
        mid->children[c->edge[0]] = c;
        ++n_nodes;
        return mid;
    }

    // Make tokens[0..m) a path of the tree with node boundaries at every depth listed in `cuts` (ascending,
    // each in 1..m).  Returns the nodes at those depths.
    void insert(const int32_t *tokens, int32_t m, const std::vector<int32_t> &cuts, std::vector<Node *> *at_cut)
    {
        at_cut->assign(cuts.size(), nullptr);
        // the path first
        int32_t matched, in_edge;
        Node *child;
        Node *cur = walk(tokens, m, &matched, &child, &in_edge);
        if (in_edge > 0) {
            cur = split(child, in_edge);  // the sequence leaves, or ends in, the middle of an edge
        }
        if (matched < m) {
            Node *leaf = new Node();
            leaf->parent = cur;
            leaf->edge.assign(tokens + matched, tokens + m);
            leaf->depth = m;
            cur->children[leaf->edge[0]] = leaf;
            kv_tokens += m - matched;
            ++n_nodes;
        }
        // then the boundaries
        for (size_t i = 0; i < cuts.size(); ++i) {
            Node *n = walk(tokens, cuts[i], &matched, &child, &in_edge);
            if (in_edge > 0)
                n = split(child, in_edge);
            (*at_cut)[i] = n;
        }
    }

    void give_state(Node *n, int64_t handle)
    {
        n->has_state = true;
        n->handle = handle;
        n->holder_index = (int32_t)holders.size();
        holders.push_back(n);
        ++n_states;
    }

    void take_state(Node *n)
    {
        Node *last = holders.back();
        holders[n->holder_index] = last;
        last->holder_index = n->holder_index;
        holders.pop_back();
        n->holder_index = -1;
        n->has_state = false;
        --n_states;
    }

    // A node without state and with exactly one child is not a node: join its edge to the child's.
    void merge_into_child(Node *n)
    {
        Node *c = n->children.begin()->second;
        c->edge.insert(c->edge.begin(), n->edge.begin(), n->edge.end());
        c->parent = n->parent;
        n->parent->children[c->edge[0]] = c;
        n->children.clear();
        delete n;
        --n_nodes;
    }

    void normalise(Node *n)
    {
        if (n != &root && !n->has_state && n->children.size() == 1)
            merge_into_child(n);
    }

    void evict(Node *n)
    {
        take_state(n);
        if (n->children.empty()) {
            // leaf: its KVs go with it
            Node *p = n->parent;
            p->children.erase(n->edge[0]);
            kv_tokens -= (int64_t)n->edge.size();
            delete n;
            --n_nodes;
            normalise(p);
        } else {
            // intermediate node with one child: the state is released, the child absorbs the KVs
            merge_into_child(n);
        }
    }

    double flop_efficiency(const Node *n) const
    {
        // FLOPs saved relative to the parent over the bytes of this node's own KVs and state (Eq. 1)
        const int32_t pd = n->parent->depth;
        const double saved = prefill_flops(cfg, n->depth) - prefill_flops(cfg, pd);
        const int64_t mem = (int64_t)(n->depth - pd) * kv_bytes_per_token() + ssm_bytes_per_state();
        return saved / (double)mem;
    }

    // S(n) of Eq. 2 for every state-holding node (same order as `holders`), both terms min-max normalised over
    // those nodes
    void scores(std::vector<double> *s)
    {
        const size_t k = holders.size();
        s->resize(k);
        if (k == 0)
            return;
        scratch_ts.resize(k);
        scratch_fe.resize(k);
        double tlo = 0, thi = 0, flo = 0, fhi = 0;
        for (size_t i = 0; i < k; ++i) {
            const double t = (double)holders[i]->last_access, f = flop_efficiency(holders[i]);
            scratch_ts[i] = t;
            scratch_fe[i] = f;
            if (i == 0) {
                tlo = thi = t;
                flo = fhi = f;
            } else {
                tlo = t < tlo ? t : tlo;
                thi = t > thi ? t : thi;
                flo = f < flo ? f : flo;
                fhi = f > fhi ? f : fhi;
            }
        }
        for (size_t i = 0; i < k; ++i) {
            const double r = thi > tlo ? (scratch_ts[i] - tlo) / (thi - tlo) : 0.0;
            const double f = fhi > flo ? (scratch_fe[i] - flo) / (fhi - flo) : 0.0;
            (*s)[i] = r + cfg.alpha * f;
        }
    }

    static void path_of(const Node *n, std::vector<int32_t> *out)
    {
        std::vector<const Node *> chain;
        for (const Node *p = n; p->parent; p = p->parent)
            chain.push_back(p);
        out->clear();
        for (auto it = chain.rbegin(); it != chain.rend(); ++it)
            out->insert(out->end(), (*it)->edge.begin(), (*it)->edge.end());
    }

    // lowest score first; ties: older access, then smaller depth, then smaller token sequence
    static bool goes_first(double sa, const Node *a, double sb, const Node *b)
    {
        if (sa != sb)
            return sa < sb;
        if (a->last_access != b->last_access)
            return a->last_access < b->last_access;
        if (a->depth != b->depth)
            return a->depth < b->depth;
        std::vector<int32_t> pa, pb;
        path_of(a, &pa);
        path_of(b, &pb);
        return pa < pb;
    }

    Node *pick_victim(Node *own0, Node *own1)
    {
        scores(&scratch_s);
        Node *best = nullptr;
        double best_s = 0.0;
        for (size_t i = 0; i < holders.size(); ++i) {
            Node *n = holders[i];
            if (n == own0 || n == own1 || n->pins > 0 || n->children.size() > 1)
                continue;
            if (!best || goes_first(scratch_s[i], n, best_s, best)) {
                best = n;
                best_s = scratch_s[i];
            }
        }
        return best;
    }

    Node *clone_subtree(const Node *src, Node *parent)
    {
        Node *n = new Node();
        n->parent = parent;
        n->edge = src->edge;
        n->depth = src->depth;
        n->has_state = src->has_state;
        n->handle = src->handle;
        n->last_access = src->last_access;
        n->pins = 0;  // pins belong to requests in flight on the original, not to the copy
        if (n->has_state) {
            n->holder_index = (int32_t)holders.size();
            holders.push_back(n);
        }
        for (auto &kv : src->children)
            n->children[kv.first] = clone_subtree(kv.second, n);
        return n;
    }
};

extern "C" const char *pc_last_error(void) { return g_error.c_str(); }

extern "C" double pc_prefill_flops(const pc_config_t *config, int64_t L)
{
    return config ? prefill_flops(*config, L) : 0.0;
}

static int check_config(const pc_config_t *c)
{
    if (!c)
        return fail(PC_ERR_INVALID_ARG, "config is NULL");
    if (c->n_attn_layers < 0 || c->n_ssm_layers < 0 || c->n_mlp_layers < 0 || c->d_model <= 0 || c->d_state <= 0 ||
        c->conv_state_bytes < 0 || c->capacity_bytes < 0)
        return fail(PC_ERR_INVALID_ARG, "negative layer count, size or capacity");
    if (!(c->alpha >= 0.0))
        return fail(PC_ERR_INVALID_ARG, "alpha must be a non-negative number");
    return PC_OK;
}

extern "C" int pc_create(const pc_config_t *config, pc_cache_t **out)
{
    if (!out)
        return fail(PC_ERR_INVALID_ARG, "out is NULL");
    *out = nullptr;
    const int rc = check_config(config);
    if (rc != PC_OK)
        return rc;
    pc_cache *c = new (std::nothrow) pc_cache();
    if (!c)
        return fail(PC_ERR_INVALID_ARG, "out of host memory");
    c->cfg = *config;
    *out = c;
    return PC_OK;
}

extern "C" void pc_destroy(pc_cache_t *cache) { delete cache; }

extern "C" int pc_clone(const pc_cache_t *cache, pc_cache_t **out)
{
    if (!cache || !out)
        return fail(PC_ERR_INVALID_ARG, "cache or out is NULL");
    pc_cache *c = new (std::nothrow) pc_cache();
    if (!c)
        return fail(PC_ERR_INVALID_ARG, "out of host memory");
    c->cfg = cache->cfg;
    c->kv_tokens = cache->kv_tokens;
    c->n_states = cache->n_states;
    c->n_nodes = cache->n_nodes;
    try {
        for (auto &kv : cache->root.children)
            c->root.children[kv.first] = c->clone_subtree(kv.second, &c->root);
    } catch (const std::bad_alloc &) {
        delete c;
        return fail(PC_ERR_INVALID_ARG, "out of host memory");
    }
    *out = c;
    return PC_OK;
}

extern "C" int pc_begin(pc_cache_t *cache, const int32_t *tokens, int32_t n, int64_t now, pc_lookup_t *out)
{
    if (!cache || !out || n < 0 || (n > 0 && !tokens))
        return fail(PC_ERR_INVALID_ARG, "cache, out or tokens is NULL, or n is negative");
    out->hit_len = 0;
    out->checkpoint_pos = 0;
    out->hit_handle = -1;
    // deepest state-holding node on the matched path that leaves at least the last input token to compute
    Node *cur = &cache->root, *hit = nullptr;
    int32_t pos = 0;
    bool mid_edge = false;
    while (pos < n) {
        auto it = cur->children.find(tokens[pos]);
        if (it == cur->children.end())
            break;
        Node *c = it->second;
        const int32_t elen = (int32_t)c->edge.size();
        int32_t k = 0;
        while (k < elen && pos + k < n && c->edge[k] == tokens[pos + k])
            ++k;
        pos += k;
        if (k < elen) {
            mid_edge = true;  // the input leaves the cached paths, or ends, inside this edge
            break;
        }
        cur = c;
        if (c->has_state && c->depth <= n - 1)
            hit = c;
    }
    if (hit) {
        hit->last_access = now;  // only the accessed node (Section 4.3, item 2)
        ++hit->pins;
        out->hit_len = hit->depth;
        out->hit_handle = hit->handle;
    }
    // speculative insertion: a new intermediate node appears exactly if the walk stopped inside an edge
    if (mid_edge && pos >= 1 && pos > out->hit_len)
        out->checkpoint_pos = pos;
    return PC_OK;
}

static int finish_impl(pc_cache_t *cache, const int32_t *tokens, int32_t m, int32_t hit_len, int32_t checkpoint_pos,
                       int64_t branch_handle, int64_t final_handle, int64_t now, int32_t *n_evicted,
                       int32_t *n_rejected);

// No exception crosses the C boundary: running out of host memory is reported as an error code.
extern "C" int pc_finish(pc_cache_t *cache, const int32_t *tokens, int32_t m, int32_t hit_len, int32_t checkpoint_pos,
                         int64_t branch_handle, int64_t final_handle, int64_t now, int32_t *n_evicted,
                         int32_t *n_rejected)
{
    try {
        return finish_impl(cache, tokens, m, hit_len, checkpoint_pos, branch_handle, final_handle, now, n_evicted,
                           n_rejected);
    } catch (const std::bad_alloc &) {
        return fail(PC_ERR_INVALID_ARG, "out of host memory");
    }
}

static int finish_impl(pc_cache_t *cache, const int32_t *tokens, int32_t m, int32_t hit_len, int32_t checkpoint_pos,
                       int64_t branch_handle, int64_t final_handle, int64_t now, int32_t *n_evicted,
                       int32_t *n_rejected)
{
    if (!cache || !tokens || m <= 0 || !n_evicted || !n_rejected)
        return fail(PC_ERR_INVALID_ARG, "cache, tokens or a count pointer is NULL, or the sequence is empty");
    if (final_handle < 0 || branch_handle < -1)
        return fail(PC_ERR_INVALID_ARG, "handles are non-negative (branch_handle may be -1)");
    if (hit_len < 0 || hit_len >= m || checkpoint_pos < 0 || checkpoint_pos > m)
        return fail(PC_ERR_BAD_REQUEST, "hit_len or checkpoint_pos outside the sequence");
    *n_evicted = *n_rejected = 0;
    cache->released.clear();
    cache->n_evicted_last = 0;

    Node *pinned = nullptr;
    if (hit_len > 0) {
        int32_t matched, in_edge;
        Node *child;
        pinned = cache->walk(tokens, hit_len, &matched, &child, &in_edge);
        if (matched != hit_len || in_edge != 0 || !pinned->has_state || pinned->pins <= 0)
            return fail(PC_ERR_BAD_REQUEST, "hit_len does not name the pinned state of this sequence");
    }

    // the states of this sequence, in the order they were taken: the checkpoint found by speculative insertion (if
    // the caller took it), then the state after the last token
    std::vector<int32_t> cuts;
    std::vector<int64_t> handles;
    if (branch_handle >= 0 && checkpoint_pos > 0) {
        cuts.push_back(checkpoint_pos);
        handles.push_back(branch_handle);
    }
    cuts.push_back(m);
    handles.push_back(final_handle);
    std::vector<Node *> at;
    cache->insert(tokens, m, cuts, &at);
    // The pin goes only now: if the insertion ran out of memory the request still holds its hit state and can
    // call pc_finish again or give up with pc_abort.  The sequence runs through the hit node, whose path matched
    // in full, so the insertion never splits an edge above it and the pointer is still that node.
    if (pinned)
        --pinned->pins;

    std::vector<int64_t> rejected;
    Node *own[2] = {nullptr, nullptr};
    for (size_t i = 0; i < cuts.size(); ++i) {
        Node *n = at[i];
        if (n->has_state) {
            rejected.push_back(handles[i]);  // a state is already cached for this prefix: keep it
        } else {
            cache->give_state(n, handles[i]);
        }
        n->last_access = now;
        own[i] = n;
    }

    while (cache->used_bytes() > cache->cfg.capacity_bytes) {
        Node *victim = cache->pick_victim(own[0], own[1]);
        if (!victim)
            break;  // nothing evictable is left: the request's own states alone exceed the capacity
        cache->released.push_back(victim->handle);
        cache->evict(victim);
    }
    cache->n_evicted_last = (int32_t)cache->released.size();
    cache->released.insert(cache->released.end(), rejected.begin(), rejected.end());
    *n_evicted = cache->n_evicted_last;
    *n_rejected = (int32_t)rejected.size();
    return PC_OK;
}

extern "C" int pc_abort(pc_cache_t *cache, const int32_t *tokens, int32_t hit_len)
{
    if (!cache || hit_len < 0 || (hit_len > 0 && !tokens))
        return fail(PC_ERR_INVALID_ARG, "cache or tokens is NULL, or hit_len is negative");
    if (hit_len == 0)
        return PC_OK;  // the request started from nothing: there is no pin to give back
    int32_t matched, in_edge;
    Node *child;
    Node *h = cache->walk(tokens, hit_len, &matched, &child, &in_edge);
    if (matched != hit_len || in_edge != 0 || !h->has_state || h->pins <= 0)
        return fail(PC_ERR_BAD_REQUEST, "hit_len does not name the pinned state of this sequence");
    --h->pins;
    return PC_OK;
}

extern "C" int pc_released(const pc_cache_t *cache, int64_t *out, int32_t cap)
{
    if (!cache || cap < 0 || (cap > 0 && !out))
        return fail(PC_ERR_INVALID_ARG, "cache or out is NULL");
    const int32_t k = (int32_t)cache->released.size();
    if (cap < k)
        return fail(PC_ERR_BUFFER_TOO_SMALL, "out is smaller than the list of released handles");
    std::copy(cache->released.begin(), cache->released.end(), out);
    return k;
}

extern "C" int pc_stats(const pc_cache_t *cache, pc_stats_t *out)
{
    if (!cache || !out)
        return fail(PC_ERR_INVALID_ARG, "cache or out is NULL");
    out->used_bytes = cache->used_bytes();
    out->kv_tokens = cache->kv_tokens;
    out->n_states = cache->n_states;
    out->n_nodes = cache->n_nodes;
    return PC_OK;
}

extern "C" int pc_set_alpha(pc_cache_t *cache, double alpha)
{
    if (!cache || !(alpha >= 0.0))
        return fail(PC_ERR_INVALID_ARG, "cache is NULL or alpha is not a non-negative number");
    cache->cfg.alpha = alpha;
    return PC_OK;
}

extern "C" int pc_set_capacity(pc_cache_t *cache, int64_t capacity_bytes)
{
    if (!cache || capacity_bytes < 0)
        return fail(PC_ERR_INVALID_ARG, "cache is NULL or the capacity is negative");
    cache->cfg.capacity_bytes = capacity_bytes;
    return PC_OK;
}

extern "C" int pc_node_score(const pc_cache_t *cache, const int32_t *tokens, int32_t depth, double *score)
{
    if (!cache || !tokens || depth <= 0 || !score)
        return fail(PC_ERR_INVALID_ARG, "cache, tokens or score is NULL, or depth is not positive");
    pc_cache *c = const_cast<pc_cache *>(cache);  // walk does not modify the tree
    int32_t matched, in_edge;
    Node *child;
    Node *n = c->walk(tokens, depth, &matched, &child, &in_edge);
    if (matched != depth || in_edge != 0 || !n->has_state)
        return fail(PC_ERR_BAD_REQUEST, "no state is cached for this prefix");
    std::vector<double> s;
    c->scores(&s);
    *score = s[n->holder_index];
    return PC_OK;
}

