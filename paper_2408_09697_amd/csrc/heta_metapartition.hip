// Meta-partitioning of a heterogeneous graph by its weighted metagraph (Section 5, Algorithm 2 of
// the paper).  Host code only: the metagraph has a handful of vertices and links, so the whole
// procedure is a few small loops; it lives in the library so that the relation set a GPU holds
// comes from the same place as the kernels that process it.
#include <algorithm>
#include <cstring>
#include <numeric>

#include <new>

#include "heta_internal.h"

namespace {

struct Walk {        // one vertex of the metatree = one walk from the root
    int32_t type;    // node type the walk stands on
    int32_t parent;  // vertex it extends (-1: the root)
    int32_t via;     // relation followed last (-1: the root)
    int32_t depth;
    int32_t sub;     // sub-metatree it belongs to (-1: the root)
};

constexpr size_t kMaxWalks = size_t(1) << 22;

}  // namespace

static heta_status heta_meta_partition_impl(int32_t n_types, const int64_t *type_weight, int32_t n_rels,
                                           const int32_t *rel_src, const int32_t *rel_dst, const int64_t *rel_weight,
                                           int32_t root, int32_t k, int32_t p, int32_t n_metapaths,
                                           const int32_t *metapath_ptr, const int32_t *metapath_rels, int32_t *n_sub,
                                           int32_t *sub_rel, int64_t *sub_weight, int64_t *sub_links, int32_t *sub_part,
                                           int64_t *part_weight, int32_t *replica_of, uint8_t *rel_mask,
                                           uint8_t *type_mask)
{
    using heta::fail;
    if (n_types < 1 || n_rels < 0 || k < 1 || p < 1 || n_metapaths < 0)
        return fail(HETA_ERR_INVALID_ARG, "heta_meta_partition: n_types %d, n_rels %d, k %d, p %d, n_metapaths %d",
                    n_types, n_rels, k, p, n_metapaths);
    if (!type_weight || !n_sub || !part_weight || !replica_of || !type_mask ||
        (n_rels > 0 && (!rel_src || !rel_dst || !rel_weight || !sub_rel || !sub_weight || !sub_links || !sub_part || !rel_mask)) ||
        (n_metapaths > 0 && (!metapath_ptr || !metapath_rels)))
        return fail(HETA_ERR_INVALID_ARG, "heta_meta_partition: null argument");
    if (root < 0 || root >= n_types) return fail(HETA_ERR_INVALID_ARG, "heta_meta_partition: root %d of %d types", root, n_types);
    for (int32_t t = 0; t < n_types; ++t)
        if (type_weight[t] < 0) return fail(HETA_ERR_INVALID_ARG, "heta_meta_partition: negative weight of type %d", t);
    for (int32_t i = 0; i < n_rels; ++i) {
        if (rel_src[i] < 0 || rel_src[i] >= n_types || rel_dst[i] < 0 || rel_dst[i] >= n_types)
            return fail(HETA_ERR_INVALID_ARG, "heta_meta_partition: relation %d joins types %d -> %d of %d", i, rel_src[i],
                        rel_dst[i], n_types);
        if (rel_weight[i] < 0) return fail(HETA_ERR_INVALID_ARG, "heta_meta_partition: negative weight of relation %d", i);
    }

    // relations grouped by the type they end in: the links a walk standing on that type can follow
    std::vector<std::vector<int32_t>> into(n_types);
    for (int32_t i = 0; i < n_rels; ++i) into[rel_dst[i]].push_back(i);

    // ---- step 1: the metatree, breadth first -------------------------------------------------------
    std::vector<Walk> tree;
    tree.push_back({root, -1, -1, 0, -1});
    if (n_metapaths == 0) {
        for (size_t head = 0; head < tree.size(); ++head) {
            const Walk w = tree[head];
            if (w.depth == k) continue;
            for (int32_t i : into[w.type]) {
                if (tree.size() >= kMaxWalks)
                    return fail(HETA_ERR_UNSUPPORTED, "heta_meta_partition: more than %zu walks of %d relations from type %d",
                                kMaxWalks, k, root);
                tree.push_back({rel_src[i], int32_t(head), i, w.depth + 1, -1});
            }
        }
    } else {
        if (metapath_ptr[0] != 0) return fail(HETA_ERR_INVALID_ARG, "heta_meta_partition: metapath_ptr[0] = %d", metapath_ptr[0]);
        // children of each vertex, to merge metapaths on their common prefixes
        std::vector<std::vector<int32_t>> kids(1);
        for (int32_t m = 0; m < n_metapaths; ++m) {
            if (metapath_ptr[m + 1] < metapath_ptr[m])
                return fail(HETA_ERR_INVALID_ARG, "heta_meta_partition: metapath_ptr decreases at %d", m);
            int32_t at = 0;
            for (int32_t j = metapath_ptr[m]; j < metapath_ptr[m + 1]; ++j) {
                const int32_t i = metapath_rels[j];
                if (i < 0 || i >= n_rels || rel_dst[i] != tree[at].type)
                    return fail(HETA_ERR_INVALID_ARG, "heta_meta_partition: metapath %d leaves the metagraph at its relation %d",
                                m, j - metapath_ptr[m]);
                int32_t next = -1;
                for (int32_t c : kids[at])
                    if (tree[c].via == i) next = c;
                if (next < 0) {
                    if (tree.size() >= kMaxWalks)
                        return fail(HETA_ERR_UNSUPPORTED, "heta_meta_partition: more than %zu metatree vertices", kMaxWalks);
                    next = int32_t(tree.size());
                    tree.push_back({rel_src[i], at, i, tree[at].depth + 1, -1});
                    kids.emplace_back();
                    kids[at].push_back(next);
                }
                at = next;
            }
        }
    }

    // ---- step 2: one sub-metatree per child of the root, and its weight ---------------------------
    // A vertex's parent always precedes it, so one forward sweep hands every vertex its sub-metatree.
    int32_t subs = 0;
    for (size_t j = 1; j < tree.size(); ++j) {
        Walk &w = tree[j];
        if (w.parent == 0) {
            w.sub = subs;
            sub_rel[subs++] = w.via;
        } else {
            w.sub = tree[w.parent].sub;
        }
    }
    *n_sub = subs;
    std::vector<uint8_t> sub_types(size_t(subs) * n_types, 0), sub_rels(size_t(subs) * std::max(n_rels, 1), 0);
    for (int32_t c = 0; c < subs; ++c) {
        sub_links[c] = 0;
        sub_types[size_t(c) * n_types + root] = 1;
    }
    for (size_t j = 1; j < tree.size(); ++j) {
        const Walk &w = tree[j];
        sub_links[w.sub] += rel_weight[w.via];                   // a link counts once per occurrence
        sub_types[size_t(w.sub) * n_types + w.type] = 1;         // a node type counts once
        sub_rels[size_t(w.sub) * n_rels + w.via] = 1;
    }
    for (int32_t c = 0; c < subs; ++c) {
        int64_t nodes = 0;
        for (int32_t t = 0; t < n_types; ++t)
            if (sub_types[size_t(c) * n_types + t]) nodes += type_weight[t];
        sub_weight[c] = nodes + sub_links[c];
    }

    // ---- step 3: longest-processing-time-first assignment ------------------------------------------
    const int32_t n_real = std::min(p, subs);
    std::vector<int32_t> order(subs);
    std::iota(order.begin(), order.end(), 0);
    std::stable_sort(order.begin(), order.end(), [&](int32_t a, int32_t b) { return sub_weight[a] > sub_weight[b]; });
    for (int32_t q = 0; q < p; ++q) {
        part_weight[q] = 0;
        replica_of[q] = -1;
    }
    for (int32_t c : order) {
        int32_t best = 0;
        for (int32_t q = 1; q < n_real; ++q)
            if (part_weight[q] < part_weight[best]) best = q;
        sub_part[c] = best;
        part_weight[best] += sub_weight[c];
    }

    // ---- step 4: a partition holds each relation and type of its sub-metatrees once -----------------
    std::memset(type_mask, 0, size_t(p) * n_types);
    if (n_rels > 0) std::memset(rel_mask, 0, size_t(p) * n_rels);
    for (int32_t c = 0; c < subs; ++c) {
        const int32_t q = sub_part[c];
        for (int32_t t = 0; t < n_types; ++t) type_mask[size_t(q) * n_types + t] |= sub_types[size_t(c) * n_types + t];
        for (int32_t i = 0; i < n_rels; ++i) rel_mask[size_t(q) * n_rels + i] |= sub_rels[size_t(c) * n_rels + i];
    }

    // ---- more partitions than sub-metatrees: replicate the heaviest per replica --------------------
    if (n_real > 0) {
        std::vector<int64_t> copies(n_real, 1);
        for (int32_t q = n_real; q < p; ++q) {
            int32_t best = 0;
            for (int32_t j = 1; j < n_real; ++j)   // a / ca > b / cb  <=>  a * cb > b * ca, in 128 bits
                if ((__int128)part_weight[j] * copies[best] > (__int128)part_weight[best] * copies[j]) best = j;
            ++copies[best];
            replica_of[q] = best;
            std::memcpy(type_mask + size_t(q) * n_types, type_mask + size_t(best) * n_types, n_types);
            if (n_rels > 0) std::memcpy(rel_mask + size_t(q) * n_rels, rel_mask + size_t(best) * n_rels, n_rels);
        }
    }
    return HETA_OK;
}

// No exception crosses the boundary: host containers may throw std::bad_alloc.
extern "C" heta_status heta_meta_partition(int32_t n_types, const int64_t *type_weight, int32_t n_rels,
                                           const int32_t *rel_src, const int32_t *rel_dst, const int64_t *rel_weight,
                                           int32_t root, int32_t k, int32_t p, int32_t n_metapaths,
                                           const int32_t *metapath_ptr, const int32_t *metapath_rels, int32_t *n_sub,
                                           int32_t *sub_rel, int64_t *sub_weight, int64_t *sub_links, int32_t *sub_part,
                                           int64_t *part_weight, int32_t *replica_of, uint8_t *rel_mask,
                                           uint8_t *type_mask)
{
    try {
        return heta_meta_partition_impl(n_types, type_weight, n_rels, rel_src, rel_dst, rel_weight, root, k, p, n_metapaths, metapath_ptr, metapath_rels, n_sub, sub_rel, sub_weight, sub_links, sub_part, part_weight, replica_of, rel_mask, type_mask);
    } catch (const std::bad_alloc &) {
        return heta::fail(HETA_ERR_OOM, "heta_meta_partition: host allocation failed");
    } catch (...) {
        return heta::fail(HETA_ERR_DEVICE, "heta_meta_partition: unexpected exception");
    }
}
