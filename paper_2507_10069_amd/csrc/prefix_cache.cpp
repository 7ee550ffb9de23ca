// Host-side unified multimodal prefix cache (Section 3.3 "Unified Multimodal Prefix Cache", Appendix A):
// a content hash for multimodal inputs and a page-granular prefix tree over the unified token sequence
// with per-node user counts and least-recently-used eviction.  It produces the page-table rows and
// prefix lengths the device kernels consume.  Host code only; the contract, including the order of
// evictions and of page reuse, is stated in emm_prefix_cache.h.
//
// Data structures, chosen for a scheduler that calls this once per request per iteration:
//   nodes      flat arrays indexed by node id (0 = root), at most one node per pool page, ids recycled;
//   children   ONE open-addressing hash table for the whole tree, keyed by (parent id, the page's
//              tokens); a hit is confirmed by comparing the tokens, so hash collisions cannot alias two
//              prefixes; never rehashed (capacity fixed at creation), deletion by backward shift;
//   evictable  an ordered set of the nodes with no users and no children, keyed by (stamp, creation
//              number): eviction pops its minimum, and a parent enters it when its last child goes;
//   free pages a ring buffer used as a FIFO queue.
// A request remembers only the deepest node of its path; the path is that node's chain of parents.
#include "emm_prefix_cache.h"

#include <cstring>
#include <new>
#include <set>
#include <unordered_map>
#include <vector>

namespace {

// ---------------------------------------------------------------------------------------------
// SHA-256 (FIPS 180-4).  The round constants are the first 32 bits of the fractional parts of the
// cube roots of the first 64 primes and the initial state those of the square roots of the first 8;
// they are derived here with exact integer roots instead of being typed in.
struct Sha256Tables {
    uint32_t k[64], h0[8];
    Sha256Tables()
    {
        int primes[64], n = 0;
        for (int c = 2; n < 64; ++c) {
            bool is_prime = true;
            for (int d = 2; d * d <= c; ++d)
                if (c % d == 0) is_prime = false;
            if (is_prime) primes[n++] = c;
        }
        typedef unsigned __int128 u128;
        for (int i = 0; i < 64; ++i) {                       // x = floor(cbrt(p) * 2^32): x^3 <= p * 2^96
            const u128 target = (u128)primes[i] << 96;
            uint64_t lo = 0, hi = (uint64_t)8 << 32;         // cbrt(311) < 7
            while (hi - lo > 1) {
                const uint64_t mid = lo + (hi - lo) / 2;
                if ((u128)mid * mid * mid <= target) lo = mid; else hi = mid;
            }
            k[i] = (uint32_t)lo;
        }
        for (int i = 0; i < 8; ++i) {                        // x = floor(sqrt(p) * 2^32): x^2 <= p * 2^64
            const u128 target = (u128)primes[i] << 64;
            uint64_t lo = 0, hi = (uint64_t)8 << 32;
            while (hi - lo > 1) {
                const uint64_t mid = lo + (hi - lo) / 2;
                if ((u128)mid * mid <= target) lo = mid; else hi = mid;
            }
            h0[i] = (uint32_t)lo;
        }
    }
};

inline uint32_t rotr(uint32_t x, int n) { return (x >> n) | (x << (32 - n)); }

void sha256_block(const Sha256Tables& t, uint32_t state[8], const uint8_t* block)
{
    uint32_t w[64];
    for (int i = 0; i < 16; ++i)
        w[i] = (uint32_t)block[4 * i] << 24 | (uint32_t)block[4 * i + 1] << 16 | (uint32_t)block[4 * i + 2] << 8 |
               (uint32_t)block[4 * i + 3];
    for (int i = 16; i < 64; ++i) {
        const uint32_t s0 = rotr(w[i - 15], 7) ^ rotr(w[i - 15], 18) ^ (w[i - 15] >> 3);
        const uint32_t s1 = rotr(w[i - 2], 17) ^ rotr(w[i - 2], 19) ^ (w[i - 2] >> 10);
        w[i] = w[i - 16] + s0 + w[i - 7] + s1;
    }
    uint32_t a = state[0], b = state[1], c = state[2], d = state[3], e = state[4], f = state[5], g = state[6],
             h = state[7];
    for (int i = 0; i < 64; ++i) {
        const uint32_t S1 = rotr(e, 6) ^ rotr(e, 11) ^ rotr(e, 25);
        const uint32_t ch = (e & f) ^ (~e & g);
        const uint32_t t1 = h + S1 + ch + t.k[i] + w[i];
        const uint32_t S0 = rotr(a, 2) ^ rotr(a, 13) ^ rotr(a, 22);
        const uint32_t maj = (a & b) ^ (a & c) ^ (b & c);
        const uint32_t t2 = S0 + maj;
        h = g; g = f; f = e; e = d + t1; d = c; c = b; b = a; a = t1 + t2;
    }
    state[0] += a; state[1] += b; state[2] += c; state[3] += d;
    state[4] += e; state[5] += f; state[6] += g; state[7] += h;
}

void sha256(const uint8_t* data, size_t n, uint8_t digest[32])
{
    static const Sha256Tables tables;
    uint32_t state[8];
    std::memcpy(state, tables.h0, sizeof(state));
    size_t off = 0;
    for (; off + 64 <= n; off += 64) sha256_block(tables, state, data + off);
    uint8_t tail[128] = {0};                                 // the rest, 0x80, zeros, 64-bit bit count
    const size_t rem = n - off;
    if (rem) std::memcpy(tail, data + off, rem);
    tail[rem] = 0x80;
    const size_t tail_len = rem + 9 <= 64 ? 64 : 128;
    const uint64_t bits = (uint64_t)n * 8;
    for (int i = 0; i < 8; ++i) tail[tail_len - 1 - i] = (uint8_t)(bits >> (8 * i));
    for (size_t o = 0; o < tail_len; o += 64) sha256_block(tables, state, tail + o);
    for (int i = 0; i < 8; ++i)
        for (int j = 0; j < 4; ++j) digest[4 * i + j] = (uint8_t)(state[i] >> (24 - 8 * j));
}

// ---------------------------------------------------------------------------------------------
struct Node {
    int32_t parent, page, users, n_children;
    uint64_t stamp, number, hash;
};

struct EvictKey {
    uint64_t stamp, number;
    int32_t node;
    bool operator<(const EvictKey& o) const { return stamp != o.stamp ? stamp < o.stamp : number < o.number; }
};

struct Request {
    std::vector<int64_t> tokens;
    std::vector<int32_t> pages;
    std::vector<uint8_t> is_private;     // per page: owned by this request alone
    int32_t deepest = 0;                 // last node of the path (0: none)
    int32_t resolved_pages = 0;          // leading pages that have a node on the path
    int32_t n_computed = 0;
    int32_t n_private = 0;
};

}  // namespace

struct emm_prefix_cache {
    int32_t num_pages = 0, page_size = 0;
    std::vector<Node> nodes;             // [num_pages + 1]
    std::vector<int64_t> node_tokens;    // [num_pages + 1][page_size]
    std::vector<int32_t> free_nodes;     // recycled ids, used as a stack
    std::vector<int32_t> table;          // open addressing, -1 = empty
    uint32_t mask = 0;
    std::vector<int32_t> fifo;           // free pages
    int64_t fifo_head = 0;
    int32_t fifo_count = 0;
    std::set<EvictKey> evictable;
    int32_t n_nodes = 0, unused_nodes = 0, private_pages = 0;
    uint64_t clock = 0, created = 0;
    std::unordered_map<int64_t, Request> requests;
    int64_t next_request = 1;
    int64_t lookups = 0, lookup_tokens = 0, hit_tokens = 0, evictions = 0;

    // ---- children table
    uint64_t hash_of(int32_t parent, const int64_t* tok) const
    {
        uint64_t h = 0x9E3779B97F4A7C15ull ^ (uint64_t)(uint32_t)parent;
        for (int i = 0; i < page_size; ++i) {
            h ^= (uint64_t)tok[i];
            h *= 0xFF51AFD7ED558CCDull;
            h ^= h >> 32;
        }
        h *= 0xC4CEB9FE1A85EC53ull;
        return h ^ (h >> 29);
    }
    int32_t find_child(int32_t parent, const int64_t* tok, uint64_t h) const
    {
        for (uint32_t i = (uint32_t)h & mask;; i = (i + 1) & mask) {
            const int32_t n = table[i];
            if (n < 0) return -1;
            if (nodes[n].hash == h && nodes[n].parent == parent &&
                std::memcmp(&node_tokens[(size_t)n * page_size], tok, sizeof(int64_t) * page_size) == 0)
                return n;
        }
    }
    void table_insert(int32_t n)
    {
        uint32_t i = (uint32_t)nodes[n].hash & mask;
        while (table[i] >= 0) i = (i + 1) & mask;
        table[i] = n;
    }
    void table_erase(int32_t n)
    {
        uint32_t i = (uint32_t)nodes[n].hash & mask;
        while (table[i] != n) i = (i + 1) & mask;
        for (uint32_t j = i;;) {                             // backward shift: close the gap at i
            j = (j + 1) & mask;
            if (table[j] < 0) break;
            const uint32_t home = (uint32_t)nodes[table[j]].hash & mask;
            const bool stays = (i <= j) ? (i < home && home <= j) : (i < home || home <= j);
            if (stays) continue;
            table[i] = table[j];
            i = j;
        }
        table[i] = -1;
    }

    // ---- free pages
    void push_page(int32_t page)
    {
        fifo[(size_t)((fifo_head + fifo_count) % num_pages)] = page;
        ++fifo_count;
    }
    int32_t pop_page()
    {
        const int32_t page = fifo[(size_t)fifo_head];
        fifo_head = (fifo_head + 1) % num_pages;
        --fifo_count;
        return page;
    }

    // ---- users and eviction
    void add_user(int32_t n)
    {
        Node& nd = nodes[n];
        if (nd.users++ == 0) {
            --unused_nodes;
            if (nd.n_children == 0) evictable.erase(EvictKey{nd.stamp, nd.number, n});
        }
    }
    void drop_user(int32_t n, bool stamp_it)
    {
        Node& nd = nodes[n];
        if (stamp_it) nd.stamp = clock;                      // only ever changes while the node has a user
        if (--nd.users == 0) {
            ++unused_nodes;
            // a release stamps with the newest clock value, so the key usually belongs at the end
            if (nd.n_children == 0) evictable.insert(evictable.end(), EvictKey{nd.stamp, nd.number, n});
        }
    }
    void evict_one()
    {
        const EvictKey key = *evictable.begin();
        evictable.erase(evictable.begin());
        const int32_t n = key.node;
        table_erase(n);
        const int32_t parent = nodes[n].parent;
        if (--nodes[parent].n_children == 0 && parent != 0 && nodes[parent].users == 0)
            // released together with the child it just lost, as a rule: same stamp, older number, new minimum
            evictable.insert(evictable.begin(), EvictKey{nodes[parent].stamp, nodes[parent].number, parent});
        push_page(nodes[n].page);
        free_nodes.push_back(n);
        --n_nodes;
        --unused_nodes;
        ++evictions;
    }
    int32_t take_page()
    {
        if (fifo_count == 0) evict_one();
        return pop_page();
    }
    int32_t pages_for(int64_t n_tokens) const { return (int32_t)((n_tokens + page_size - 1) / page_size); }
    static void write_row(const Request& rq, int32_t max_pages, int32_t* row)
    {
        const int32_t n = (int32_t)rq.pages.size();
        std::memcpy(row, rq.pages.data(), sizeof(int32_t) * n);
        for (int32_t i = n; i < max_pages; ++i) row[i] = -1;
    }
};

extern "C" {

emm_status emm_mm_content_hash(const void* data, size_t n_bytes, uint8_t digest[32])
{
    if (digest == nullptr || (data == nullptr && n_bytes != 0)) return EMM_ERR_NULL;
    sha256((const uint8_t*)data, n_bytes, digest);
    return EMM_OK;
}

emm_status emm_mm_token_ids(const uint8_t digest[32], int32_t n_tokens, int64_t* ids)
{
    if (digest == nullptr || (ids == nullptr && n_tokens != 0)) return EMM_ERR_NULL;
    if (n_tokens < 0) return EMM_ERR_INVALID_ARG;
    uint64_t w0 = 0, w1 = 0;
    for (int i = 0; i < 8; ++i) {
        w0 = w0 << 8 | digest[i];
        w1 = w1 << 8 | digest[8 + i];
    }
    for (int32_t j = 0; j < n_tokens; ++j)
        ids[j] = -1 - (int64_t)(((w0 + (uint64_t)j * 0x9E3779B97F4A7C15ull) ^ w1) >> 1);
    return EMM_OK;
}

emm_status emm_prefix_cache_create(int32_t num_pages, int32_t page_size, emm_prefix_cache** cache)
{
    if (cache == nullptr) return EMM_ERR_NULL;
    *cache = nullptr;
    if (num_pages < 1 || page_size < 1 || num_pages > (1 << 29)) return EMM_ERR_INVALID_ARG;
    emm_prefix_cache* c = nullptr;
    try {
        c = new emm_prefix_cache();
        c->num_pages = num_pages;
        c->page_size = page_size;
        c->nodes.resize((size_t)num_pages + 1);
        c->nodes[0] = Node{-1, -1, 0, 0, 0, 0, 0};
        c->node_tokens.resize(((size_t)num_pages + 1) * page_size);
        c->free_nodes.reserve(num_pages);
        for (int32_t n = num_pages; n >= 1; --n) c->free_nodes.push_back(n);     // ids 1, 2, ... come out first
        uint32_t cap = 16;
        while (cap < 2u * (uint32_t)num_pages + 2u) cap <<= 1;
        c->table.assign(cap, -1);
        c->mask = cap - 1;
        c->fifo.resize(num_pages);
        for (int32_t p = 0; p < num_pages; ++p) c->fifo[p] = p;
        c->fifo_count = num_pages;
    } catch (const std::bad_alloc&) {
        delete c;
        return EMM_ERR_NO_SPACE;
    }
    *cache = c;
    return EMM_OK;
}

void emm_prefix_cache_destroy(emm_prefix_cache* cache) { delete cache; }

emm_status emm_prefix_cache_begin(emm_prefix_cache* c, const int64_t* tokens, int32_t n_tokens, int32_t max_pages,
                                  int32_t* page_table_row, int32_t* prefix_len, int64_t* request)
{
    if (c == nullptr || tokens == nullptr || page_table_row == nullptr || prefix_len == nullptr || request == nullptr)
        return EMM_ERR_NULL;
    if (n_tokens < 1 || max_pages < c->pages_for(n_tokens)) return EMM_ERR_INVALID_ARG;
    const int32_t ps = c->page_size, total = c->pages_for(n_tokens);
    // longest cached run of leading full pages, never the page that holds the last token
    int32_t node = 0, matched = 0;
    for (const int32_t limit = (n_tokens - 1) / ps; matched < limit; ++matched) {
        const int64_t* tok = tokens + (size_t)matched * ps;
        const int32_t child = c->find_child(node, tok, c->hash_of(node, tok));
        if (child < 0) break;
        node = child;
    }
    for (int32_t x = node; x != 0; x = c->nodes[x].parent) c->add_user(x);      // in use: cannot be evicted below
    const int32_t need = total - matched;
    Request rq;
    bool ok = (int64_t)need <= (int64_t)c->fifo_count + c->unused_nodes;
    if (ok) {
        try {
            rq.tokens.assign(tokens, tokens + n_tokens);
            rq.pages.resize(total);
            rq.is_private.assign(total, 1);
            c->requests.reserve(c->requests.size() + 1);
        } catch (const std::bad_alloc&) {
            ok = false;
        }
    }
    if (!ok) {
        for (int32_t x = node; x != 0; x = c->nodes[x].parent) c->drop_user(x, false);
        return EMM_ERR_NO_SPACE;
    }
    ++c->clock;
    int32_t i = matched;
    for (int32_t x = node; x != 0; x = c->nodes[x].parent) {
        --i;
        rq.pages[i] = c->nodes[x].page;
        rq.is_private[i] = 0;
    }
    for (int32_t p = matched; p < total; ++p) rq.pages[p] = c->take_page();
    rq.deepest = node;
    rq.resolved_pages = matched;
    rq.n_computed = matched * ps;
    rq.n_private = need;
    c->private_pages += need;
    emm_prefix_cache::write_row(rq, max_pages, page_table_row);
    *prefix_len = rq.n_computed;
    *request = c->next_request++;
    c->lookups += 1;
    c->lookup_tokens += n_tokens;
    c->hit_tokens += rq.n_computed;
    c->requests.emplace(*request, std::move(rq));
    return EMM_OK;
}

emm_status emm_prefix_cache_append(emm_prefix_cache* c, int64_t request, const int64_t* tokens, int32_t n_tokens,
                                   int32_t max_pages, int32_t* page_table_row)
{
    if (c == nullptr || page_table_row == nullptr || (tokens == nullptr && n_tokens != 0)) return EMM_ERR_NULL;
    if (n_tokens < 0) return EMM_ERR_INVALID_ARG;
    auto it = c->requests.find(request);
    if (it == c->requests.end()) return EMM_ERR_NOT_FOUND;
    Request& rq = it->second;
    const int64_t new_len = (int64_t)rq.tokens.size() + n_tokens;
    if (new_len > INT32_MAX) return EMM_ERR_INVALID_ARG;
    const int32_t total = c->pages_for(new_len);
    if (max_pages < total) return EMM_ERR_INVALID_ARG;
    const int32_t need = total - (int32_t)rq.pages.size();
    if ((int64_t)need > (int64_t)c->fifo_count + c->unused_nodes) return EMM_ERR_NO_SPACE;
    try {
        rq.tokens.reserve((size_t)new_len);
        rq.pages.reserve(total);
        rq.is_private.reserve(total);
    } catch (const std::bad_alloc&) {
        return EMM_ERR_NO_SPACE;
    }
    rq.tokens.insert(rq.tokens.end(), tokens, tokens + n_tokens);
    for (int32_t p = 0; p < need; ++p) {
        rq.pages.push_back(c->take_page());
        rq.is_private.push_back(1);
    }
    rq.n_private += need;
    c->private_pages += need;
    emm_prefix_cache::write_row(rq, max_pages, page_table_row);
    return EMM_OK;
}

emm_status emm_prefix_cache_commit(emm_prefix_cache* c, int64_t request, int32_t n_computed)
{
    if (c == nullptr) return EMM_ERR_NULL;
    auto it = c->requests.find(request);
    if (it == c->requests.end()) return EMM_ERR_NOT_FOUND;
    Request& rq = it->second;
    if (n_computed > (int64_t)rq.tokens.size() || n_computed < rq.n_computed) return EMM_ERR_INVALID_ARG;
    const int32_t ps = c->page_size;
    ++c->clock;
    rq.n_computed = n_computed;
    for (int32_t p = rq.resolved_pages; p < n_computed / ps; ++p) {
        const int64_t* tok = rq.tokens.data() + (size_t)p * ps;
        const int32_t parent = rq.deepest;
        const uint64_t h = c->hash_of(parent, tok);
        int32_t child = c->find_child(parent, tok, h);
        if (child < 0) {                                     // publish this request's page as a new node
            child = c->free_nodes.back();                    // never empty: fewer nodes than pages exist
            c->free_nodes.pop_back();
            c->nodes[child] = Node{parent, rq.pages[p], 0, 0, c->clock, ++c->created, h};
            std::memcpy(&c->node_tokens[(size_t)child * ps], tok, sizeof(int64_t) * ps);
            c->table_insert(child);
            ++c->nodes[parent].n_children;                   // the parent has a user (this request) or is the root
            ++c->n_nodes;
            ++c->unused_nodes;                               // add_user below takes it out again
            rq.is_private[p] = 0;
            --rq.n_private;
            --c->private_pages;
        }
        // else: another request published the same content first; this one keeps its page as a
        // private duplicate and its path goes on through the existing node
        c->add_user(child);
        rq.deepest = child;
    }
    if (n_computed / ps > rq.resolved_pages) rq.resolved_pages = n_computed / ps;
    return EMM_OK;
}

emm_status emm_prefix_cache_release(emm_prefix_cache* c, int64_t request)
{
    if (c == nullptr) return EMM_ERR_NULL;
    auto it = c->requests.find(request);
    if (it == c->requests.end()) return EMM_ERR_NOT_FOUND;
    Request& rq = it->second;
    ++c->clock;
    for (int32_t x = rq.deepest; x != 0; x = c->nodes[x].parent) c->drop_user(x, true);
    for (size_t p = 0; p < rq.pages.size(); ++p)
        if (rq.is_private[p]) c->push_page(rq.pages[p]);
    c->private_pages -= rq.n_private;
    c->requests.erase(it);
    return EMM_OK;
}

emm_status emm_prefix_cache_get_stats(const emm_prefix_cache* c, emm_prefix_cache_stats* s)
{
    if (c == nullptr || s == nullptr) return EMM_ERR_NULL;
    s->lookups = c->lookups;
    s->lookup_tokens = c->lookup_tokens;
    s->hit_tokens = c->hit_tokens;
    s->evictions = c->evictions;
    s->num_pages = c->num_pages;
    s->free_pages = c->fifo_count;
    s->cached_pages = c->n_nodes;
    s->evictable_pages = c->unused_nodes;
    s->private_pages = c->private_pages;
    s->live_requests = (int32_t)c->requests.size();
    return EMM_OK;
}

}  // extern "C"
