// Host-side session prefix tree: the bookkeeping that makes trajectories of
// one session share the physical KV pages of a common prefix.
//
// The paper's Trajectory Manager keeps every trajectory of a session in a
// prefix tree built by longest-prefix matching, so that shared prefixes are
// stored once, and annotates every token with the model version that produced
// it (Data Plane, Trajectory Manager paragraph).  This tree does the same at
// KV-page granularity: a node is one full page (16 tokens with their version
// tags); two trajectories share a node, and therefore the physical page, only
// if all tokens AND versions up to the end of that page are equal -- KV
// written under other weights is not the same KV.  The last, partly filled
// page of a trajectory is private (it will still grow).  The tree hands out
// page ids from a free list, reference-counts shared pages, and emits the
// block-table rows and the (group_start, shared_len) arrays that
// paged_decode_attention_prefix consumes.  Pure host code: no HIP calls.
#include "../../include/seamdecode.h"

#include <algorithm>
#include <cstring>
#include <map>
#include <new>
#include <vector>

namespace {

constexpr int kPage = 16;

struct PageKey {
    int32_t tok[kPage];
    uint32_t ver[kPage];
    bool operator<(const PageKey &o) const
    {
        const int c = std::memcmp(tok, o.tok, sizeof tok);
        if (c) return c < 0;
        return std::memcmp(ver, o.ver, sizeof ver) < 0;
    }
};

struct Node {
    int32_t page = -1;
    int32_t parent = -1;  // node index, -1 for children of the root
    int32_t refs = 0;     // trajectories whose path contains this node
    bool listed = true;   // reachable through its parent's child map (a page that filled up during
                          // decoding next to an equal, already listed page stays unlisted)
    PageKey key;
    std::map<PageKey, int32_t> children;
};

struct Traj {
    bool live = false;
    int32_t length = 0;               // tokens
    std::vector<int32_t> path;        // node indices of the full pages, root first
    int32_t tail_page = -1;           // private page of the partly filled last page, -1 if none
    std::vector<int32_t> tail_tok;    // its tokens (< 16)
    std::vector<uint32_t> tail_ver;
};

}  // namespace

struct sd_tree {
    std::vector<Node> nodes;
    std::vector<int32_t> free_nodes;
    std::map<PageKey, int32_t> roots;
    std::vector<Traj> trajs;
    std::vector<int32_t> free_pages;  // stack; lowest ids on top
    int32_t num_pages = 0;
    int32_t in_use = 0;

    int32_t take_page()
    {
        if (free_pages.empty()) return -1;
        const int32_t p = free_pages.back();
        free_pages.pop_back();
        ++in_use;
        return p;
    }
    void give_page(int32_t p)
    {
        free_pages.push_back(p);
        --in_use;
    }
    std::map<PageKey, int32_t> &kids(int32_t node) { return node < 0 ? roots : nodes[node].children; }
};

extern "C" {

sd_tree *sd_tree_create(int32_t num_pages)
{
    if (num_pages <= 0) return nullptr;
    sd_tree *t = new (std::nothrow) sd_tree;
    if (!t) return nullptr;
    t->num_pages = num_pages;
    t->free_pages.resize(num_pages);
    for (int32_t i = 0; i < num_pages; ++i) t->free_pages[i] = num_pages - 1 - i;
    return t;
}

void sd_tree_destroy(sd_tree *t) { delete t; }

int32_t sd_tree_pages_in_use(const sd_tree *t) { return t ? t->in_use : SD_EINVAL; }

// Tokens of the longest stored prefix of (tokens, versions) that lie in shared
// (full) pages: a multiple of 16.  versions == NULL means version 0 everywhere.
int32_t sd_tree_match(const sd_tree *t, const int32_t *tokens, const uint32_t *versions, int32_t n)
{
    if (!t || n < 0 || (n > 0 && !tokens)) return SD_EINVAL;
    const std::map<PageKey, int32_t> *level = &t->roots;
    int32_t matched = 0;
    for (int32_t p = 0; (p + 1) * kPage <= n; ++p) {
        PageKey k;
        for (int i = 0; i < kPage; ++i) {
            k.tok[i] = tokens[p * kPage + i];
            k.ver[i] = versions ? versions[p * kPage + i] : 0u;
        }
        auto it = level->find(k);
        if (it == level->end()) break;
        matched += kPage;
        level = &t->nodes[it->second].children;
    }
    return matched;
}

// Stores a trajectory.  Full pages that already exist are shared (no new page);
// the others get fresh pages.  *matched_tokens (optional) receives the number
// of leading tokens whose KV is already in the cache: the caller appends K/V
// from that position on.  Returns the trajectory id, SD_EINVAL, or
// SD_EWORKSPACE when the pool has no free page left (nothing is changed then).
int32_t sd_tree_insert(sd_tree *t, const int32_t *tokens, const uint32_t *versions, int32_t n, int32_t *matched_tokens)
{
    if (!t || n < 0 || (n > 0 && !tokens)) return SD_EINVAL;
    const int32_t matched = sd_tree_match(t, tokens, versions, n);
    const int32_t full = n / kPage, tail = n % kPage;
    const int32_t need = (full - matched / kPage) + (tail ? 1 : 0);
    if (need > (int32_t)t->free_pages.size()) return SD_EWORKSPACE;

    Traj tr;
    tr.live = true;
    tr.length = n;
    int32_t parent = -1;
    for (int32_t p = 0; p < full; ++p) {
        PageKey k;
        for (int i = 0; i < kPage; ++i) {
            k.tok[i] = tokens[p * kPage + i];
            k.ver[i] = versions ? versions[p * kPage + i] : 0u;
        }
        auto &level = t->kids(parent);
        auto it = level.find(k);
        int32_t node;
        if (it != level.end()) {
            node = it->second;
        } else {
            if (!t->free_nodes.empty()) {
                node = t->free_nodes.back();
                t->free_nodes.pop_back();
                t->nodes[node] = Node();
            } else {
                node = (int32_t)t->nodes.size();
                t->nodes.emplace_back();
            }
            t->nodes[node].page = t->take_page();
            t->nodes[node].parent = parent;
            t->nodes[node].key = k;
            t->kids(parent)[k] = node;  // kids() again: nodes may have been reallocated
        }
        t->nodes[node].refs++;
        tr.path.push_back(node);
        parent = node;
    }
    if (tail) {
        tr.tail_page = t->take_page();
        tr.tail_tok.assign(tokens + full * kPage, tokens + n);
        tr.tail_ver.resize(tail);
        for (int i = 0; i < tail; ++i) tr.tail_ver[i] = versions ? versions[full * kPage + i] : 0u;
    }
    if (matched_tokens) *matched_tokens = matched;
    for (size_t i = 0; i < t->trajs.size(); ++i)
        if (!t->trajs[i].live) {
            t->trajs[i] = std::move(tr);
            return (int32_t)i;
        }
    t->trajs.push_back(std::move(tr));
    return (int32_t)t->trajs.size() - 1;
}

// Drops a trajectory: pages nobody else references go back to the free list.
int sd_tree_release(sd_tree *t, int32_t traj)
{
    if (!t || traj < 0 || traj >= (int32_t)t->trajs.size() || !t->trajs[traj].live) return SD_EINVAL;
    Traj &tr = t->trajs[traj];
    for (int32_t i = (int32_t)tr.path.size() - 1; i >= 0; --i) {
        const int32_t node = tr.path[i];
        if (--t->nodes[node].refs == 0) {
            if (t->nodes[node].listed) t->kids(t->nodes[node].parent).erase(t->nodes[node].key);
            t->give_page(t->nodes[node].page);
            t->free_nodes.push_back(node);
        }
    }
    if (tr.tail_page >= 0) t->give_page(tr.tail_page);
    tr = Traj();
    return SD_OK;
}

// A second trajectory with the same tokens: it shares every full page of `traj`;
// a partly filled last page is private, so the copy gets a fresh page and the
// caller must copy the old one into it (kv_copy_pages) before either side appends.
// *copy_src / *copy_dst receive that page pair, or -1 / -1 when there is nothing
// to copy.  Returns the new trajectory id, SD_EINVAL, or SD_EWORKSPACE (no free
// page; nothing is changed then).
int32_t sd_tree_fork(sd_tree *t, int32_t traj, int32_t *copy_src, int32_t *copy_dst)
{
    if (!t || traj < 0 || traj >= (int32_t)t->trajs.size() || !t->trajs[traj].live) return SD_EINVAL;
    Traj copy = t->trajs[traj];
    int32_t src = -1, dst = -1;
    if (copy.tail_page >= 0) {
        dst = t->take_page();
        if (dst < 0) return SD_EWORKSPACE;
        src = copy.tail_page;
        copy.tail_page = dst;
    }
    for (int32_t node : copy.path) t->nodes[node].refs++;
    if (copy_src) *copy_src = src;
    if (copy_dst) *copy_dst = dst;
    for (size_t i = 0; i < t->trajs.size(); ++i)
        if (!t->trajs[i].live) {
            t->trajs[i] = std::move(copy);
            return (int32_t)i;
        }
    t->trajs.push_back(std::move(copy));
    return (int32_t)t->trajs.size() - 1;
}

// One more token at the end of a trajectory (a decode step).  *page / *slot
// (optional) receive where its K/V rows go: the trajectory's last page, which is
// taken from the pool when the previous one was full.  A page that fills up
// becomes a tree node: listed under its parent (later inserts can share it)
// unless an equal page is already listed there, in which case it stays private.
// Returns SD_OK, SD_EINVAL, or SD_EWORKSPACE (no free page; nothing is changed).
int sd_tree_append(sd_tree *t, int32_t traj, int32_t token, uint32_t version, int32_t *page, int32_t *slot)
{
    if (!t || traj < 0 || traj >= (int32_t)t->trajs.size() || !t->trajs[traj].live) return SD_EINVAL;
    if (t->trajs[traj].tail_page < 0) {
        const int32_t fresh = t->take_page();
        if (fresh < 0) return SD_EWORKSPACE;
        t->trajs[traj].tail_page = fresh;
    }
    Traj &tr = t->trajs[traj];
    if (page) *page = tr.tail_page;
    if (slot) *slot = (int32_t)tr.tail_tok.size();
    tr.tail_tok.push_back(token);
    tr.tail_ver.push_back(version);
    tr.length++;
    if ((int32_t)tr.tail_tok.size() < kPage) return SD_OK;

    PageKey k;
    for (int i = 0; i < kPage; ++i) {
        k.tok[i] = tr.tail_tok[i];
        k.ver[i] = tr.tail_ver[i];
    }
    const int32_t parent = tr.path.empty() ? -1 : tr.path.back();
    int32_t node;
    if (!t->free_nodes.empty()) {
        node = t->free_nodes.back();
        t->free_nodes.pop_back();
        t->nodes[node] = Node();
    } else {
        node = (int32_t)t->nodes.size();
        t->nodes.emplace_back();
    }
    Node &nd = t->nodes[node];
    nd.page = tr.tail_page;
    nd.parent = parent;
    nd.key = k;
    nd.refs = 1;
    auto &level = t->kids(parent);  // after emplace_back: nodes may have moved
    nd.listed = level.find(k) == level.end();
    if (nd.listed) level[k] = node;
    tr.path.push_back(node);
    tr.tail_page = -1;
    tr.tail_tok.clear();
    tr.tail_ver.clear();
    return SD_OK;
}

int32_t sd_tree_length(const sd_tree *t, int32_t traj)
{
    if (!t || traj < 0 || traj >= (int32_t)t->trajs.size() || !t->trajs[traj].live) return SD_EINVAL;
    return t->trajs[traj].length;
}

// Block-table row of a trajectory: physical page of every logical page.
// Writes min(pages, cap) entries and returns the number of pages.
int32_t sd_tree_block_table(const sd_tree *t, int32_t traj, int32_t *pages_out, int32_t cap)
{
    if (!t || traj < 0 || traj >= (int32_t)t->trajs.size() || !t->trajs[traj].live || cap < 0 || (cap > 0 && !pages_out))
        return SD_EINVAL;
    const Traj &tr = t->trajs[traj];
    int32_t n = 0;
    for (int32_t node : tr.path) {
        if (n < cap) pages_out[n] = t->nodes[node].page;
        ++n;
    }
    if (tr.tail_page >= 0) {
        if (n < cap) pages_out[n] = tr.tail_page;
        ++n;
    }
    return n;
}

// Token id and model version at a position of a trajectory (both optional outputs).
int sd_tree_token_at(const sd_tree *t, int32_t traj, int32_t pos, int32_t *token, uint32_t *version)
{
    if (!t || traj < 0 || traj >= (int32_t)t->trajs.size() || !t->trajs[traj].live) return SD_EINVAL;
    const Traj &tr = t->trajs[traj];
    if (pos < 0 || pos >= tr.length) return SD_EINVAL;
    const int32_t p = pos / kPage, i = pos % kPage;
    if (p < (int32_t)tr.path.size()) {
        if (token) *token = t->nodes[tr.path[p]].key.tok[i];
        if (version) *version = t->nodes[tr.path[p]].key.ver[i];
    } else {
        if (token) *token = tr.tail_tok[i];
        if (version) *version = tr.tail_ver[i];
    }
    return SD_OK;
}

// Groups for paged_decode_attention_prefix over a batch of trajectories (in
// batch order): consecutive trajectories whose first page is the same node
// form a group; shared_len of its members = 16 * (leading pages common to all
// of them).  Trajectories without a full page, and groups of one, get
// shared_len 0.  group_start_out needs B + 1 entries, shared_len_out B.
// Returns the number of groups.
int32_t sd_tree_batch_groups(const sd_tree *t, const int32_t *trajs, int32_t B, int32_t *group_start_out,
                             int32_t *shared_len_out)
{
    if (!t || B < 0 || (B > 0 && (!trajs || !group_start_out || !shared_len_out))) return SD_EINVAL;
    for (int32_t b = 0; b < B; ++b)
        if (trajs[b] < 0 || trajs[b] >= (int32_t)t->trajs.size() || !t->trajs[trajs[b]].live) return SD_EINVAL;
    int32_t ng = 0, b = 0;
    while (b < B) {
        const std::vector<int32_t> &first = t->trajs[trajs[b]].path;
        int32_t e = b + 1;
        size_t common = first.size();
        while (e < B && !first.empty()) {
            const std::vector<int32_t> &p = t->trajs[trajs[e]].path;
            if (p.empty() || p[0] != first[0]) break;
            size_t c = 0;
            while (c < common && c < p.size() && p[c] == first[c]) ++c;
            common = c;
            ++e;
        }
        const int32_t shared = (e - b > 1) ? (int32_t)common * kPage : 0;
        group_start_out[ng++] = b;
        for (int32_t i = b; i < e; ++i) shared_len_out[i] = shared;
        b = e;
    }
    group_start_out[ng] = B;
    return ng;
}

}  // extern "C"
