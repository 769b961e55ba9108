// Global prefix identification on the host (BatchLLM Sec. 3.2): a compact prefix tree
// (radix tree) over the prompts of a batch, the fork-and-merge pass of Alg. 1 that enlarges
// the first-level prefixes, and the prefix-sharing groups read off the children of the root.
// The result feeds bllm_prefix_group_create (group prefix lengths, request -> group).
//
// Nodes live in one vector and refer to each other by index; a node's tokens are a span of
// one of the prompts below it, never a copy.  Children are kept in visiting order: first the
// children of the plain tree by first token, then the nodes forked into this level, in the
// order of the forks.
#include "bllm_internal.h"

#include <algorithm>
#include <cstdint>
#include <vector>

namespace bllm {
namespace {

struct Node {
    int32_t prompt = -1;            // tokens = tokens[start[prompt] + first .. + n_tokens)
    int64_t first = 0;
    int64_t n_tokens = 0;
    int64_t leaves = 0;             // prompts that end at or below this node
    bool forked = false;            // created by fork-and-merge (sorts after the plain children)
    std::vector<int32_t> children;  // node indices
    std::vector<int32_t> ends;      // prompts that end exactly here
};

class PrefixTree {
public:
    PrefixTree(int32_t n_prompts, const int64_t* start, const int32_t* tokens)
        : start_(start), tokens_(tokens) {
        nodes_.reserve(2 * static_cast<size_t>(n_prompts) + 1);
        nodes_.emplace_back();      // root
        for (int32_t r = 0; r < n_prompts; ++r) insert(r);
        count_leaves(0);
    }

    size_t depth() const { return depth_; }
    void maximize_reuse() { maximize(0); }

    // first-level nodes (children of the root) and the prompts ending at the root itself
    const Node& root() const { return nodes_[0]; }
    const Node& node(int32_t i) const { return nodes_[i]; }

    void members(int32_t i, std::vector<int32_t>* out) const {
        // explicit stack: the tree can be as deep as there are prompts
        std::vector<int32_t> todo{i};
        while (!todo.empty()) {
            const Node& n = nodes_[todo.back()];
            todo.pop_back();
            out->insert(out->end(), n.ends.begin(), n.ends.end());
            todo.insert(todo.end(), n.children.begin(), n.children.end());
        }
    }

private:
    int32_t token_at(const Node& n, int64_t k) const { return tokens_[start_[n.prompt] + n.first + k]; }
    int64_t length(int32_t r) const { return start_[r + 1] - start_[r]; }

    // While the tree is built, children are kept sorted by their first token.
    // Position of the first child whose first token is not below `tok`.
    size_t child_slot(const Node& parent, int32_t tok) const {
        size_t lo = 0, hi = parent.children.size();
        while (lo < hi) {
            const size_t mid = (lo + hi) / 2;
            if (token_at(nodes_[parent.children[mid]], 0) < tok) lo = mid + 1; else hi = mid;
        }
        return lo;
    }

    void insert(int32_t r) {
        const int32_t* p = tokens_ + start_[r];
        const int64_t len = length(r);
        int32_t at = 0;
        int64_t pos = 0;
        for (;;) {
            if (pos == len) {
                nodes_[at].ends.push_back(r);
                return;
            }
            const size_t slot = child_slot(nodes_[at], p[pos]);
            const bool found = slot < nodes_[at].children.size() && token_at(nodes_[nodes_[at].children[slot]], 0) == p[pos];
            if (!found) {
                Node leaf;
                leaf.prompt = r;
                leaf.first = pos;
                leaf.n_tokens = len - pos;
                leaf.ends.push_back(r);
                nodes_.push_back(std::move(leaf));
                std::vector<int32_t>& ch = nodes_[at].children;
                ch.insert(ch.begin() + static_cast<std::ptrdiff_t>(slot), static_cast<int32_t>(nodes_.size()) - 1);
                return;
            }
            const int32_t c = nodes_[at].children[slot];
            int64_t k = 0;
            {
                const Node& cn = nodes_[c];
                while (k < cn.n_tokens && pos + k < len && token_at(cn, k) == p[pos + k]) ++k;
            }
            if (k < nodes_[c].n_tokens) {
                // split after k tokens: a new upper node takes the child's place, the child keeps the rest
                Node upper;
                upper.prompt = nodes_[c].prompt;
                upper.first = nodes_[c].first;
                upper.n_tokens = k;
                upper.children.push_back(c);
                nodes_[c].first += k;
                nodes_[c].n_tokens -= k;
                nodes_.push_back(std::move(upper));
                const int32_t u = static_cast<int32_t>(nodes_.size()) - 1;
                nodes_[at].children[slot] = u;       // same first token: the order is unchanged
                at = u;
            } else {
                at = c;
            }
            pos += k;
        }
    }

    int64_t count_leaves(int32_t root_index) {
        // post-order without recursion
        std::vector<std::pair<int32_t, size_t>> stack{{root_index, 0}};
        while (!stack.empty()) {
            depth_ = std::max(depth_, stack.size());
            auto& [i, next] = stack.back();
            if (next < nodes_[i].children.size()) {
                const int32_t c = nodes_[i].children[next++];
                stack.emplace_back(c, 0);
            } else {
                int64_t total = static_cast<int64_t>(nodes_[i].ends.size());
                for (int32_t c : nodes_[i].children) total += nodes_[c].leaves;
                nodes_[i].leaves = total;
                stack.pop_back();
            }
        }
        return nodes_[root_index].leaves;
    }

    // visiting order of a node's children: plain children by first token, then forked ones as created
    void order_children(int32_t i) {
        std::vector<int32_t>& ch = nodes_[i].children;
        std::stable_sort(ch.begin(), ch.end(), [&](int32_t a, int32_t b) {
            const Node& na = nodes_[a];
            const Node& nb = nodes_[b];
            if (na.forked != nb.forked) return !na.forked;
            if (na.forked) return false;                     // keep creation order
            return token_at(na, 0) < token_at(nb, 0);
        });
    }

    // Alg. 1 for node d (the first-level prefixes of a node are its children).  Recursive like the
    // paper's statement; the depth is bounded by the number of branching levels of the tree.
    void maximize(int32_t d) {
        if (nodes_[d].children.empty()) return;
        order_children(d);
        const std::vector<int32_t> visit = nodes_[d].children;      // forks append to the live list
        std::vector<int32_t> kept;
        std::vector<int32_t> forked;
        for (int32_t c : visit) {
            maximize(c);                                            // solve sub-problems
            order_children(c);
            const std::vector<int32_t> grand = nodes_[c].children;
            std::vector<int32_t> stay;
            for (int32_t g : grand) {
                const int64_t gain = (nodes_[g].leaves - 1) * nodes_[g].n_tokens;
                const int64_t penalty = nodes_[c].n_tokens;
                if (gain > penalty) {
                    // fork c and merge with g: g's span grows backwards over c's tokens
                    nodes_[g].first -= nodes_[c].n_tokens;
                    nodes_[g].n_tokens += nodes_[c].n_tokens;
                    nodes_[g].forked = true;
                    nodes_[c].leaves -= nodes_[g].leaves;
                    forked.push_back(g);
                } else {
                    stay.push_back(g);
                }
            }
            nodes_[c].children = stay;
            if (stay.empty() && nodes_[c].ends.empty()) continue;   // nothing left below c
            if (stay.size() == 1 && nodes_[c].ends.empty()) {
                // keep the tree compact: the only child absorbs c's tokens and takes its place
                const int32_t only = stay[0];
                nodes_[only].first -= nodes_[c].n_tokens;
                nodes_[only].n_tokens += nodes_[c].n_tokens;
                nodes_[only].forked = nodes_[c].forked;
                kept.push_back(only);
            } else {
                kept.push_back(c);
            }
        }
        kept.insert(kept.end(), forked.begin(), forked.end());
        nodes_[d].children = kept;
    }

    const int64_t* start_;
    const int32_t* tokens_;
    std::vector<Node> nodes_;
    size_t depth_ = 0;
};

}  // namespace
}  // namespace bllm

using namespace bllm;

extern "C" int bllm_identify_prefix_groups(int32_t n_prompts, const int64_t* prompt_start, const int32_t* tokens,
                                           int32_t* req_group, int32_t* group_prefix_len, int32_t* n_groups,
                                           int64_t* n_logical_tokens, int64_t* n_processed_tokens) {
    if (n_prompts < 0 || !prompt_start || !n_groups || (n_prompts > 0 && (!req_group || !group_prefix_len))) {
        set_error("null pointer argument or negative prompt count");
        return BLLM_INVALID_ARG;
    }
    if (prompt_start[0] != 0) {
        set_error("prompt_start[0] must be 0");
        return BLLM_INVALID_ARG;
    }
    for (int32_t r = 0; r < n_prompts; ++r) {
        const int64_t len = prompt_start[r + 1] - prompt_start[r];
        if (len < 0 || len > INT32_MAX) {
            set_error("prompt " + std::to_string(r) + " has a negative or too large length");
            return BLLM_INVALID_ARG;
        }
    }
    if (n_prompts > 0 && prompt_start[n_prompts] > 0 && !tokens) {
        set_error("null token array");
        return BLLM_INVALID_ARG;
    }
    try {
        PrefixTree tree(n_prompts, prompt_start, tokens);
        if (tree.depth() > 20000) {
            set_error("prefix tree deeper than 20000 levels (prompts that extend one another in a long chain)");
            return BLLM_UNSUPPORTED;
        }
        tree.maximize_reuse();
        struct Group {
            int32_t first_member;
            int32_t prefix_len;
            std::vector<int32_t> members;
        };
        std::vector<Group> groups;
        std::vector<int32_t> loners(tree.root().ends);
        for (int32_t c : tree.root().children) {
            std::vector<int32_t> m;
            tree.members(c, &m);
            if (m.size() >= 2) {
                Group g;
                g.first_member = *std::min_element(m.begin(), m.end());
                g.prefix_len = static_cast<int32_t>(tree.node(c).n_tokens);
                g.members = std::move(m);
                groups.push_back(std::move(g));
            } else {
                loners.insert(loners.end(), m.begin(), m.end());
            }
        }
        if (!loners.empty()) {
            Group g;
            g.first_member = *std::min_element(loners.begin(), loners.end());
            g.prefix_len = 0;
            g.members = std::move(loners);
            groups.push_back(std::move(g));
        }
        std::sort(groups.begin(), groups.end(), [](const Group& a, const Group& b) { return a.first_member < b.first_member; });
        int64_t logical = 0, processed = 0;
        for (size_t g = 0; g < groups.size(); ++g) {
            group_prefix_len[g] = groups[g].prefix_len;
            processed += groups[g].prefix_len;
            for (int32_t r : groups[g].members) {
                req_group[r] = static_cast<int32_t>(g);
                const int64_t len = prompt_start[r + 1] - prompt_start[r];
                logical += len;
                processed += len - groups[g].prefix_len;
            }
        }
        *n_groups = static_cast<int32_t>(groups.size());
        if (n_logical_tokens) *n_logical_tokens = logical;
        if (n_processed_tokens) *n_processed_tokens = processed;
    } catch (const std::bad_alloc&) {
        set_error("out of host memory while building the prefix tree");
        return BLLM_OUT_OF_MEMORY;
    }
    return BLLM_OK;
}
