/*
 * CPU oracle for the Global Neighbor Sampling (GNS) hot path.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, single-threaded
 * definition the HIP library is checked against.  It shares no code with the
 * HIP path and is never called by it.  Only the tests, the smoke check and the
 * benchmark's cpu_baseline leg may load it.
 *
 * What is computed (paper: arxiv 2106.06150, KDD'21):
 *   - cache draw ............ Section 3.2, Eq. (1) (degree-proportional probability) or
 *                             the random-walk probability P^L = (DA + I)^L P^0,
 *                             Theorem 1 (drawn without replacement, |C| nodes)
 *   - layer sampling ........ Algorithm 1 top-down loop, Section 3.3 (neighbors
 *                             from the cache first, a shortfall filled uniformly from
 *                             the rest of the neighborhood), Section 4.1 (input layer
 *                             sampled only from the cache), Section 2.1 (uniform
 *                             node-wise sampling with fan-out k)
 *   - importance weights .... Section 3.4 (p^C_u = 1-(1-p_u)^|C|, coefficient
 *                             p^C_u * k / min(k, N_C(v)), aggregation uses 1/coef)
 *   - frontier union ........ Algorithm 1, B^{l-1} <- B^{l-1} U N_l(u)
 *   - gather ................ Section 2.2 steps 2-3 (slice the input-node features)
 *   - aggregation ........... Algorithm 1 bottom-up loop, mean aggregator (Section 2.1)
 *   - update ................ Algorithm 1, h_u = g(W . (h_u, h_N(u))) (forward only)
 *
 * Conventions of this build that the paper leaves open (random source, order
 * inside a frontier, how a without-replacement draw is realised) are stated at
 * each function.  Pins: see tests/test_oracle_*.py.  Parity unpinned: the choice
 * of Floyd's subset algorithm, the Philox counter layout and the ascending order
 * of the frontier tail are conventions; only invariants constrain them.  The same
 * holds for two choices of the cache-first policy the paper does not fix: that the
 * fill is drawn from N(v) \ C (so no neighbor is taken twice) and the fill
 * neighbors' weights (1, or |N(v) \ C| / r in the unbiased mode).
 *
 * All floating point is fp64 with one final rounding to fp32.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define GNS_ORACLE_UNIFORM 0
#define GNS_ORACLE_CACHE_ONLY 1
#define GNS_ORACLE_CACHE_FIRST 2
#define GNS_ORACLE_W_PRINTED 0
#define GNS_ORACLE_W_UNBIASED 1

/* ------------------------------------------------------------------------ */
/* Philox4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11): a 4-word counter and a
 * 2-word key; ten rounds; each round multiplies words 0 and 2 by fixed odd
 * constants, swaps the products' halves into the other lanes xor-ed with the
 * key, and the key is advanced by the two Weyl constants between rounds.      */
void gns_oracle_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        uint64_t prod0 = (uint64_t)0xD2511F53u * (uint64_t)c0;
        uint64_t prod1 = (uint64_t)0xCD9E8D57u * (uint64_t)c2;
        uint32_t hi0 = (uint32_t)(prod0 >> 32), lo0 = (uint32_t)prod0;
        uint32_t hi1 = (uint32_t)(prod1 >> 32), lo1 = (uint32_t)prod1;
        uint32_t n0 = hi1 ^ c1 ^ k0;
        uint32_t n1 = lo1;
        uint32_t n2 = hi0 ^ c3 ^ k1;
        uint32_t n3 = lo0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* Counter layouts of this build (a convention, the paper names no generator).
 * The key is always the 64-bit seed split into (low, high) words.
 *   cache stream, draw j:       (lo32(j), hi32(j), lo32(epoch), 'CACH')
 *   neighbor draw (l, v, slot): (v, slot >> 2, l, 'NBHS'), word slot & 3     */
#define TAG_CACHE 0x43414348u
#define TAG_NEIGHBOR 0x4E424853u

static uint64_t cache_stream_r64(uint64_t seed, uint64_t epoch, uint64_t j)
{
    uint32_t ctr[4] = { (uint32_t)j, (uint32_t)(j >> 32), (uint32_t)epoch, TAG_CACHE };
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    uint32_t w[4];
    gns_oracle_philox4x32_10(ctr, key, w);
    return ((uint64_t)w[1] << 32) | (uint64_t)w[0];
}

static uint32_t neighbor_word(uint64_t seed, uint32_t layer, uint32_t node, uint32_t slot)
{
    uint32_t ctr[4] = { node, slot >> 2, layer, TAG_NEIGHBOR };
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    uint32_t w[4];
    gns_oracle_philox4x32_10(ctr, key, w);
    return w[slot & 3u];
}

/* floor(r * range / 2^64) for range < 2^63 */
static uint64_t mulhi64(uint64_t r, uint64_t range)
{
    return (uint64_t)(((unsigned __int128)r * (unsigned __int128)range) >> 64);
}

/* ------------------------------------------------------------------------ */
/* One draw of the cache stream -> a node.
 * Eq. (1): P(node = i) = deg(i) / sum_k deg(k).  A CSR entry is chosen
 * uniformly from [0, nnz) and the node is the row that owns it, which has
 * exactly that probability (up to the < nnz/2^64 bias of the range map).
 * deg(i) is the row length indptr[i+1]-indptr[i].                            */
static int64_t row_owning_entry(int64_t n, const int64_t* indptr, int64_t e)
{
    /* the unique i with indptr[i] <= e < indptr[i+1] */
    int64_t lo = 0, hi = n; /* answer in [lo, hi) */
    while (hi - lo > 1) {
        int64_t mid = lo + (hi - lo) / 2;
        if (indptr[mid] <= e) lo = mid; else hi = mid;
    }
    return lo;
}

int64_t gns_oracle_cache_draw_node(int64_t n, const int64_t* indptr, uint64_t seed, uint64_t epoch, uint64_t j)
{
    uint64_t nnz = (uint64_t)indptr[n];
    uint64_t e = mulhi64(cache_stream_r64(seed, epoch, j), nnz);
    return row_owning_entry(n, indptr, (int64_t)e);
}

/* The cache C (Section 3.2; Theorem 1: "without replacement", exactly
 * cache_size nodes): the first cache_size DISTINCT nodes of the i.i.d. stream
 * node_0, node_1, ... -- skipping repeats of an i.i.d. weighted stream is
 * successive weighted sampling without replacement.
 * Outputs: cache_nodes ascending; bitmap bit i set iff i in C (may be NULL).
 * Returns the number of stream draws consumed (index of the last used draw
 * + 1), or -1 if max_draws was reached first, -2 on bad arguments.           */
int64_t gns_oracle_sample_cache(int64_t n, const int64_t* indptr, uint64_t seed, uint64_t epoch,
                                int64_t cache_size, int64_t max_draws,
                                int32_t* cache_nodes, uint64_t* bitmap)
{
    if (n <= 0 || cache_size <= 0 || indptr[n] <= 0) return -2;
    unsigned char* in_cache = (unsigned char*)calloc((size_t)n, 1);
    if (!in_cache) return -2;
    int64_t distinct = 0, j = 0;
    while (distinct < cache_size && j < max_draws) {
        int64_t node = gns_oracle_cache_draw_node(n, indptr, seed, epoch, (uint64_t)j);
        ++j;
        if (!in_cache[node]) { in_cache[node] = 1; ++distinct; }
    }
    if (distinct < cache_size) { free(in_cache); return -1; }
    int64_t words = (n + 63) / 64;
    if (bitmap) memset(bitmap, 0, (size_t)words * sizeof(uint64_t));
    int64_t slot = 0;
    for (int64_t i = 0; i < n; ++i) {
        if (in_cache[i]) {
            cache_nodes[slot++] = (int32_t)i;
            if (bitmap) bitmap[i >> 6] |= (uint64_t)1 << (i & 63);
        }
    }
    free(in_cache);
    return j;
}

/* ------------------------------------------------------------------------ */
/* Section 3.2, second approach: the cache probability from short random walks,
 *   P^0_i = 1/|V_S| on the training nodes, 0 elsewhere,
 *   P^l   = (D_l A + I) P^(l-1),   D_l = diag(N_l(v)/deg(v)),   l = 1..L,
 * and the cache is drawn with probability proportional to P^L.
 * Readings: N_l(v), "the number of sampled neighbors of v in layer l", is
 * min(k_l, deg(v)); step l of the walk uses the fan-out of the l-th layer counted
 * from the seeds (fanouts[l-1], the same indexing as everywhere else here); the
 * product is taken as printed, (D A P)_i = d_i * sum over j in N(i) of P_j.
 * So that two implementations can agree bit for bit the vector is kept in integer
 * units of 2^-scale_log2 of one training node's initial mass (the common factor
 * 1/|V_S| does not change a proportional draw) and every step rounds down:
 *   W^l_i = W^(l-1)_i + floor(min(k_l, deg_i) * S_i / deg_i),  S_i = sum_j W^(l-1)_j
 * (computed as k'*(S div deg) + (k'*(S mod deg)) div deg, which is that floor exactly).
 * weights[i] = W^L_i, prefix = its exclusive prefix sum (prefix[n] = total).
 * Returns 0; -1 on bad arguments; -2 if a row sum, a product or the total would
 * not fit in 62 bits (lower scale_log2).                                        */
int gns_oracle_walk_weights(int64_t n, const int64_t* indptr, const int32_t* indices,
                            int64_t num_train, const int32_t* train_nodes,
                            int32_t num_layers, const int32_t* fanouts, int32_t scale_log2,
                            uint64_t* weights, int64_t* prefix)
{
    if (n <= 0 || num_train <= 0 || num_layers < 1 || scale_log2 < 0 || scale_log2 > 40) return -1;
    const uint64_t limit = (uint64_t)1 << 62;
    uint64_t* cur = (uint64_t*)calloc((size_t)n, sizeof(uint64_t));
    uint64_t* nxt = (uint64_t*)calloc((size_t)n, sizeof(uint64_t));
    if (!cur || !nxt) { free(cur); free(nxt); return -1; }
    int rc = 0;
    for (int64_t t = 0; t < num_train; ++t) {
        int64_t v = train_nodes[t];
        if (v < 0 || v >= n) { rc = -1; goto done; }
        cur[v] = (uint64_t)1 << scale_log2;
    }
    for (int32_t l = 0; l < num_layers && rc == 0; ++l) {
        int64_t k = fanouts[l];
        if (k < 1) { rc = -1; break; }
        for (int64_t i = 0; i < n; ++i) {
            int64_t deg = indptr[i + 1] - indptr[i];
            uint64_t sum = 0;
            for (int64_t e = indptr[i]; e < indptr[i + 1]; ++e) {
                sum += cur[indices[e]];
                if (sum >= limit) { rc = -2; break; }
            }
            if (rc) break;
            uint64_t add = 0;
            if (deg > 0) {
                uint64_t kk = (uint64_t)(k < deg ? k : deg);
                uint64_t q = sum / (uint64_t)deg, rem = sum % (uint64_t)deg;
                if (q >= limit / 64) { rc = -2; break; }
                add = kk * q + (kk * rem) / (uint64_t)deg;
            }
            nxt[i] = cur[i] + add;
            if (nxt[i] >= limit) { rc = -2; break; }
        }
        uint64_t* tmp = cur; cur = nxt; nxt = tmp;
    }
    if (rc == 0) {
        uint64_t total = 0;
        for (int64_t i = 0; i < n; ++i) {
            prefix[i] = (int64_t)total;
            weights[i] = cur[i];
            total += cur[i];
            if (total >= limit) { rc = -2; break; }
        }
        prefix[n] = (int64_t)total;
    }
done:
    free(cur);
    free(nxt);
    return rc;
}

/* ------------------------------------------------------------------------ */
/* Robert Floyd's subset algorithm: a uniformly random k-subset of {0..m-1}
 * from k random words.  For s = 0..k-1: j = m-k+s; t = floor(word_s*(j+1)/2^32);
 * take t unless already taken, else take j.  Requires 0 < k < m.  The ranks
 * are returned ascending.                                                    */
void gns_oracle_floyd(int64_t m, int32_t k, const uint32_t* words, int64_t* ranks)
{
    int32_t have = 0;
    for (int32_t s = 0; s < k; ++s) {
        int64_t j = m - k + s;
        int64_t t = (int64_t)(((uint64_t)words[s] * (uint64_t)(j + 1)) >> 32);
        int taken = 0;
        for (int32_t q = 0; q < have; ++q) if (ranks[q] == t) { taken = 1; break; }
        ranks[have++] = taken ? j : t;
    }
    for (int32_t a = 1; a < k; ++a) {          /* insertion sort, ascending */
        int64_t x = ranks[a];
        int32_t b = a - 1;
        while (b >= 0 && ranks[b] > x) { ranks[b + 1] = ranks[b]; --b; }
        ranks[b + 1] = x;
    }
}

/* Section 3.4.  p_u = deg(u)/nnz (Eq. (1)); p^C_u = 1-(1-p_u)^|C| written as
 * -expm1(|C| * log1p(-p_u)) so that tiny p_u keeps its digits.
 *   printed:   coefficient = p^C_u * k / min(k, N_C(v)),  weight = 1/coefficient
 *   unbiased:  weight = N_C(v) / (min(k, N_C(v)) * p^C_u)   (Horvitz-Thompson
 *              form: 1 / (P(u in C) * P(u picked | N_C(v) eligible)); it is the
 *              printed weight times N_C(v)*k / min(k, N_C(v))^2)               */
double gns_oracle_p_cache(double p_u, int64_t cache_size)
{
    if (p_u >= 1.0) return 1.0;
    return -expm1((double)cache_size * log1p(-p_u));
}

float gns_oracle_edge_weight(int64_t deg_u, int64_t nnz, int64_t cache_size, int32_t k, int64_t n_c, int32_t wmode)
{
    double p_u = (double)deg_u / (double)nnz;
    double pc = gns_oracle_p_cache(p_u, cache_size);
    double taken = (double)(n_c < k ? n_c : (int64_t)k);
    double w;
    if (wmode == GNS_ORACLE_W_UNBIASED) {
        w = (double)n_c / (taken * pc);
    } else {
        double coef = pc * (double)k / taken;
        w = 1.0 / coef;
    }
    return (float)w;
}

/* Picks min(k, m) of the m entries of a list: all of them if m <= k, otherwise
 * Floyd's subset with the Philox words of slots slot0 .. slot0+k-1 of (layer, v).
 * Ranks come back ascending (= CSR order).  Returns how many were taken.       */
static int32_t pick_ranks(int64_t m, int32_t k, uint64_t seed, int32_t layer, int64_t v, int32_t slot0, int64_t* ranks)
{
    if (m <= k) {
        for (int32_t s = 0; s < (int32_t)m; ++s) ranks[s] = s;
        return (int32_t)m;
    }
    uint32_t words[64];
    for (int32_t s = 0; s < k; ++s)
        words[s] = neighbor_word(seed, (uint32_t)layer, (uint32_t)v, (uint32_t)(slot0 + s));
    gns_oracle_floyd(m, k, words, ranks);
    return k;
}

/* One layer of Algorithm 1's top-down loop: for every dst row v independently,
 * N_l(v) <- sample(N(v), C).
 *   UNIFORM:     eligible list E(v) = N(v) in CSR order                      (Section 2.1)
 *   CACHE_ONLY:  E(v) = entries of N(v) whose node is in C                   (Sections 3.3, 4.1)
 *   CACHE_FIRST: first from E_C(v) = N(v) & C as CACHE_ONLY does; if that gave
 *                fewer than k (N_C(v) < k), the remaining k - N_C(v) are drawn
 *                uniformly without replacement from E_N(v) = N(v) \ C           (Section 3.3)
 * m = |E(v)|.  If m <= k all of E(v) is taken; otherwise Floyd picks k ranks
 * with the Philox words of slots 0..k-1.  CACHE_FIRST's fill draw takes
 * r = min(k - N_C, |E_N|) ranks of E_N with the words of slots N_C .. N_C+r-1, so a
 * row's slots are never used twice.  Chosen neighbors are emitted in ascending rank
 * (= CSR position), cached ones before fill ones.  Row v writes
 * out_nbr[r*k .. r*k+cnt), out_w likewise, out_cnt[r] = number taken,
 * out_elig[r] = |E(v)| (N_C(v) for both cache policies).
 * Weights: UNIFORM 1; cached neighbors Section 3.4 (gns_oracle_edge_weight with
 * N_C(v)); fill neighbors 1 in the printed mode (they are a node-wise sample,
 * Section 2.1), |E_N|/r in the unbiased mode (inverse inclusion probability of a
 * uniform r-subset, given the cache).
 * Returns 0, or -1 on bad arguments.                                          */
int gns_oracle_sample_layer_p(int64_t n, const int64_t* indptr, const int32_t* indices,
                              const uint64_t* cache_bitmap, int64_t cache_size, const int64_t* prob_prefix,
                              uint64_t seed, int32_t layer, int32_t policy, int32_t wmode, int32_t k,
                              int64_t num_dst, const int32_t* dst_nodes,
                              int32_t* out_nbr, float* out_w, int32_t* out_cnt, int32_t* out_elig);

int gns_oracle_sample_layer(int64_t n, const int64_t* indptr, const int32_t* indices,
                            const uint64_t* cache_bitmap, int64_t cache_size,
                            uint64_t seed, int32_t layer, int32_t policy, int32_t wmode, int32_t k,
                            int64_t num_dst, const int32_t* dst_nodes,
                            int32_t* out_nbr, float* out_w, int32_t* out_cnt, int32_t* out_elig)
{
    /* Eq. (1): the cache probability of node u is deg(u) / nnz, i.e. the prefix is indptr itself */
    return gns_oracle_sample_layer_p(n, indptr, indices, cache_bitmap, cache_size, indptr, seed, layer, policy,
                                     wmode, k, num_dst, dst_nodes, out_nbr, out_w, out_cnt, out_elig);
}

/* The same with the cache probability given as an integer prefix array over the nodes:
 * p_u = (prob_prefix[u+1] - prob_prefix[u]) / prob_prefix[n]  (Section 3.2: either Eq. (1)
 * or the random-walk probability; Section 3.4 only needs p_u).                          */
int gns_oracle_sample_layer_p(int64_t n, const int64_t* indptr, const int32_t* indices,
                              const uint64_t* cache_bitmap, int64_t cache_size, const int64_t* prob_prefix,
                              uint64_t seed, int32_t layer, int32_t policy, int32_t wmode, int32_t k,
                              int64_t num_dst, const int32_t* dst_nodes,
                              int32_t* out_nbr, float* out_w, int32_t* out_cnt, int32_t* out_elig)
{
    if (k <= 0 || k > 64) return -1;
    if (policy != GNS_ORACLE_UNIFORM && (!cache_bitmap || !prob_prefix)) return -1;
    int64_t nnz = prob_prefix ? prob_prefix[n] : indptr[n];
    for (int64_t r = 0; r < num_dst; ++r) {
        int64_t v = dst_nodes[r];
        if (v < 0 || v >= n) return -1;
        int64_t start = indptr[v], deg = indptr[v + 1] - start;
        int32_t* elig = (int32_t*)malloc((size_t)(deg > 0 ? deg : 1) * sizeof(int32_t));
        int32_t* rest = (int32_t*)malloc((size_t)(deg > 0 ? deg : 1) * sizeof(int32_t));
        if (!elig || !rest) { free(elig); free(rest); return -1; }
        int64_t m = 0, m_rest = 0;
        for (int64_t e = 0; e < deg; ++e) {
            int32_t u = indices[start + e];
            int ok = 1;
            if (policy != GNS_ORACLE_UNIFORM)
                ok = (int)((cache_bitmap[u >> 6] >> (u & 63)) & 1u);
            if (ok) elig[m++] = u; else rest[m_rest++] = u;
        }
        int64_t ranks[64];
        int32_t cnt = pick_ranks(m, k, seed, layer, v, 0, ranks);
        for (int32_t s = 0; s < cnt; ++s) {
            int32_t u = elig[ranks[s]];
            out_nbr[r * k + s] = u;
            if (policy == GNS_ORACLE_UNIFORM) {
                out_w[r * k + s] = 1.0f;
            } else {
                int64_t mass_u = prob_prefix[(int64_t)u + 1] - prob_prefix[u];
                out_w[r * k + s] = gns_oracle_edge_weight(mass_u, nnz, cache_size, k, m, wmode);
            }
        }
        if (policy == GNS_ORACLE_CACHE_FIRST && cnt < k && m_rest > 0) {
            int32_t fill = pick_ranks(m_rest, k - cnt, seed, layer, v, cnt, ranks);
            for (int32_t s = 0; s < fill; ++s) {
                out_nbr[r * k + cnt + s] = rest[ranks[s]];
                out_w[r * k + cnt + s] = (wmode == GNS_ORACLE_W_UNBIASED) ? (float)((double)m_rest / (double)fill) : 1.0f;
            }
            cnt += fill;
        }
        out_cnt[r] = cnt;
        out_elig[r] = (int32_t)m;
        free(elig);
        free(rest);
    }
    return 0;
}

/* ------------------------------------------------------------------------ */
/* Frontier union and relabelling (Algorithm 1: B^{l-1} <- B^{l-1} U N_l(u); the
 * update step needs h_u^{l-1} of the dst node too, so dst nodes are kept).
 * Canonical order of this build: src_nodes = dst_nodes in their given order,
 * followed by the ascending list of sampled ids that are not dst nodes.
 * indptr = exclusive prefix sum of the row counts; indices[e] = position of the
 * neighbor in src_nodes; edges stay in (row, ascending rank) order.
 * Returns num_src (>= num_dst), or -1 on allocation failure.                  */
static int cmp_i32(const void* a, const void* b)
{
    int32_t x = *(const int32_t*)a, y = *(const int32_t*)b;
    return (x > y) - (x < y);
}

typedef struct { int32_t node; int32_t pos; } node_pos;
static int cmp_node_pos(const void* a, const void* b)
{
    int32_t x = ((const node_pos*)a)->node, y = ((const node_pos*)b)->node;
    return (x > y) - (x < y);
}

int64_t gns_oracle_build_block(int64_t num_dst, const int32_t* dst_nodes, int32_t k,
                               const int32_t* nbr, const float* w, const int32_t* cnt,
                               int32_t* indptr, int32_t* indices, float* weights, int32_t* src_nodes)
{
    int64_t edges = 0;
    for (int64_t r = 0; r < num_dst; ++r) { indptr[r] = (int32_t)edges; edges += cnt[r]; }
    indptr[num_dst] = (int32_t)edges;

    node_pos* dst_sorted = (node_pos*)malloc((size_t)(num_dst > 0 ? num_dst : 1) * sizeof(node_pos));
    int32_t* tail = (int32_t*)malloc((size_t)(edges > 0 ? edges : 1) * sizeof(int32_t));
    if (!dst_sorted || !tail) { free(dst_sorted); free(tail); return -1; }
    for (int64_t r = 0; r < num_dst; ++r) { dst_sorted[r].node = dst_nodes[r]; dst_sorted[r].pos = (int32_t)r; }
    qsort(dst_sorted, (size_t)num_dst, sizeof(node_pos), cmp_node_pos);

    /* every sampled id that is not a dst node, sorted, duplicates removed */
    int64_t nt = 0;
    for (int64_t r = 0; r < num_dst; ++r)
        for (int32_t s = 0; s < cnt[r]; ++s) {
            node_pos key = { nbr[r * k + s], 0 };
            if (!bsearch(&key, dst_sorted, (size_t)num_dst, sizeof(node_pos), cmp_node_pos))
                tail[nt++] = key.node;
        }
    qsort(tail, (size_t)nt, sizeof(int32_t), cmp_i32);
    int64_t nu = 0;
    for (int64_t i = 0; i < nt; ++i)
        if (i == 0 || tail[i] != tail[i - 1]) tail[nu++] = tail[i];

    for (int64_t r = 0; r < num_dst; ++r) src_nodes[r] = dst_nodes[r];
    for (int64_t i = 0; i < nu; ++i) src_nodes[num_dst + i] = tail[i];

    for (int64_t r = 0; r < num_dst; ++r)
        for (int32_t s = 0; s < cnt[r]; ++s) {
            int32_t u = nbr[r * k + s];
            node_pos key = { u, 0 };
            node_pos* hit = (node_pos*)bsearch(&key, dst_sorted, (size_t)num_dst, sizeof(node_pos), cmp_node_pos);
            int32_t local;
            if (hit) {
                local = hit->pos;
            } else {
                int32_t* t = (int32_t*)bsearch(&u, tail, (size_t)nu, sizeof(int32_t), cmp_i32);
                local = (int32_t)(num_dst + (t - tail));
            }
            indices[indptr[r] + s] = local;
            weights[indptr[r] + s] = w[r * k + s];
        }
    free(dst_sorted);
    free(tail);
    return num_dst + nu;
}

/* ------------------------------------------------------------------------ */
/* Section 2.2 steps 2-3: the feature rows of the input nodes, copied bit for
 * bit.  Where a row physically lives (device cache table, device store, host)
 * cannot change its bits, so the oracle indexes the one full matrix.          */
void gns_oracle_gather(int64_t feat_dim, const float* x, int64_t num_nodes, const int32_t* nodes, float* out)
{
    for (int64_t j = 0; j < num_nodes; ++j)
        memcpy(out + j * feat_dim, x + (int64_t)nodes[j] * feat_dim, (size_t)feat_dim * sizeof(float));
}

/* Algorithm 1 bottom-up loop with the mean aggregator and Section 3.4's
 * rescaling: out[v,:] = (1/n_v) * sum_{e in row v} w_e * x_src[indices[e],:],
 * n_v = number of sampled neighbors of v; an empty row gives zeros.
 * Accumulated in fp64 in row order, rounded once to fp32.                     */
void gns_oracle_aggregate(int64_t num_dst, const int32_t* indptr, const int32_t* indices, const float* weights,
                          int64_t feat_dim, const float* x_src, float* out)
{
    double* acc = (double*)malloc((size_t)(feat_dim > 0 ? feat_dim : 1) * sizeof(double));
    for (int64_t r = 0; r < num_dst; ++r) {
        int32_t b = indptr[r], e = indptr[r + 1];
        for (int64_t f = 0; f < feat_dim; ++f) acc[f] = 0.0;
        for (int32_t q = b; q < e; ++q) {
            const float* row = x_src + (int64_t)indices[q] * feat_dim;
            double wq = (double)weights[q];
            for (int64_t f = 0; f < feat_dim; ++f) acc[f] += wq * (double)row[f];
        }
        double inv = (e > b) ? 1.0 / (double)(e - b) : 0.0;
        for (int64_t f = 0; f < feat_dim; ++f) out[r * feat_dim + f] = (float)(acc[f] * inv);
    }
    free(acc);
}

/* ------------------------------------------------------------------------ */
/* The update step of Algorithm 1 for one layer (GraphSAGE form, Section 2.1):
 *   h_u^l = g( W^l . (h_u^(l-1), h_N(u)^l) )
 * with the concatenation written out: out[r, :] = g( h_self[r, :] . W[0:F1, :] +
 * h_neigh[r, :] . W[F1:F1+F2, :] + bias ),  g = max(0, .) if relu else identity.
 * W is (F1+F2) x H row-major (the paper's W^l transposed, so that rows of W match
 * the entries of the concatenated vector), bias may be NULL.  fp64 accumulation in
 * index order, one rounding to fp32.                                           */
void gns_oracle_sage_dense(int64_t rows, int64_t f1, const float* h_self, int64_t f2, const float* h_neigh,
                           int64_t hdim, const float* w, const float* bias, int32_t relu, float* out)
{
    for (int64_t r = 0; r < rows; ++r) {
        for (int64_t j = 0; j < hdim; ++j) {
            double acc = bias ? (double)bias[j] : 0.0;
            for (int64_t k = 0; k < f1; ++k) acc += (double)h_self[r * f1 + k] * (double)w[k * hdim + j];
            for (int64_t k = 0; k < f2; ++k) acc += (double)h_neigh[r * f2 + k] * (double)w[(f1 + k) * hdim + j];
            if (relu && acc < 0.0) acc = 0.0;
            out[r * hdim + j] = (float)acc;
        }
    }
}
