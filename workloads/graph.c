/*
 * Seeded synthetic power-law graphs and minibatch neighbour sampling: the source
 * of the node-ID lists for the GraphSAGE-style gather workloads.
 *
 * Input generation only (no part of the gather).  Stands in for the DGL
 * sampler and the datasets of PyTorch-Direct's GNN experiments (arXiv
 * 2101.07956, Section 5.1 and its dataset table), of which only the shapes are
 * used: node counts, feature widths, fanouts.
 *
 * Graph model
 *   - every node has a popularity rank rho in [1, N]; node_of_rank(k) =
 *     (A*k + B) mod N with gcd(A, N) = 1 is a seeded permutation, so ranks are
 *     scattered over the ID space (neighbouring IDs are unrelated);
 *   - degree(rank) = clip(round(c / rank), dmin, N-1): a Zipf(1.0) law with a
 *     floor, c solved so that the mean degree is the requested one.  The floor
 *     is set to the largest fanout so that every sampled node yields its full
 *     fanout;
 *   - each neighbour slot holds a node drawn with probability ~ rank^-alpha
 *     (inverse CDF of the continuous density x^-alpha on [1, N+1)); alpha = 1 is
 *     the log-uniform (Zipf 1.0) law.  alpha is the knob that sets how many
 *     distinct IDs a minibatch contains.  Multi-edges may occur.
 *
 * Sampling (one minibatch): seeds are uniform nodes; hop h draws fanout[h]
 * neighbours (uniformly, with replacement, from the node's list; the whole
 * list if it is not longer than the fanout) for every distinct node gathered
 * so far; the result is the list of distinct IDs in first-occurrence order,
 * seeds first.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

uint64_t wl_mix64(uint64_t seed, uint64_t counter); /* gen.c */

static uint64_t gcd_u64(uint64_t a, uint64_t b)
{
    while (b) {
        const uint64_t t = a % b;
        a = b;
        b = t;
    }
    return a;
}

/* multiplier and offset of the rank -> node permutation */
static void perm_params(uint64_t N, uint64_t seed, uint64_t *A, uint64_t *B)
{
    uint64_t a = (wl_mix64(seed, 0x9e37) % N) | 1u;
    while (gcd_u64(a, N) != 1)
        a += 2;
    *A = a % N ? a % N : 1;
    *B = wl_mix64(seed, 0x79b9) % N;
}

static inline int64_t node_of_rank0(uint64_t k, uint64_t N, uint64_t A, uint64_t B)
{
    return (int64_t)(((__uint128_t)A * k + B) % N);
}

int64_t wl_node_of_rank(uint64_t rank, uint64_t N, uint64_t seed)
{
    uint64_t A, B;
    perm_params(N, seed, &A, &B);
    return node_of_rank0(rank - 1, N, A, B);
}

/* out[k] = node whose popularity rank is first_rank + k (ranks start at 1) */
void wl_nodes_of_ranks(int64_t *out, uint64_t first_rank, uint64_t n, uint64_t N, uint64_t seed)
{
    uint64_t A, B;
    perm_params(N, seed, &A, &B);
    for (uint64_t k = 0; k < n; ++k)
        out[k] = node_of_rank0(first_rank - 1 + k, N, A, B);
}

/* rank in [1, N] with P(rank = k) ~ k^-alpha, from one 64-bit hash */
static inline uint64_t rank_from_hash(uint64_t h, uint64_t N, double alpha)
{
    const double u = (double)(h >> 11) * (1.0 / 9007199254740992.0); /* [0, 1) */
    double x;
    if (fabs(alpha - 1.0) < 1e-12)
        x = exp(u * log((double)N + 1.0));
    else
        x = pow(1.0 + u * (pow((double)N + 1.0, 1.0 - alpha) - 1.0), 1.0 / (1.0 - alpha));
    uint64_t k = (uint64_t)x;
    if (k < 1)
        k = 1;
    if (k > N)
        k = N;
    return k;
}

uint64_t wl_zipf_rank(uint64_t seed, uint64_t counter, uint64_t N, double alpha)
{
    return rank_from_hash(wl_mix64(seed, counter), N, alpha);
}

static double mean_degree_for(double c, uint64_t N, int64_t dmin)
{
    /* ranks beyond c/dmin all sit on the floor: sum the head exactly, the tail in closed form */
    double sum = 0.0;
    uint64_t head = (uint64_t)(c / (double)(dmin > 0 ? dmin : 1)) + 2;
    if (head > N)
        head = N;
    for (uint64_t r = 1; r <= head; ++r) {
        double d = nearbyint(c / (double)r);
        if (d < (double)dmin)
            d = (double)dmin;
        if (d > (double)(N - 1))
            d = (double)(N - 1);
        sum += d;
    }
    sum += (double)(N - head) * (double)dmin;
    return sum / (double)N;
}

/* deg[node] for all N nodes; returns the total number of neighbour slots */
int64_t wl_graph_degrees(int64_t *deg, uint64_t N, double mean_degree, int64_t dmin, uint64_t seed)
{
    uint64_t A, B;
    perm_params(N, seed, &A, &B);
    double lo = 1.0, hi = (double)N * mean_degree;
    for (int it = 0; it < 64; ++it) {
        const double c = 0.5 * (lo + hi);
        if (mean_degree_for(c, N, dmin) > mean_degree)
            hi = c;
        else
            lo = c;
    }
    const double c = lo;
    int64_t total = 0;
    for (uint64_t r = 1; r <= N; ++r) {
        double d = nearbyint(c / (double)r);
        if (d < (double)dmin)
            d = (double)dmin;
        if (d > (double)(N - 1))
            d = (double)(N - 1);
        deg[node_of_rank0(r - 1, N, A, B)] = (int64_t)d;
        total += (int64_t)d;
    }
    return total;
}

/* CSR neighbour IDs: offsets[N+1] must already hold the exclusive prefix sum of
 * the degrees; slot e of the whole array is filled from hash(seed, e). */
void wl_graph_fill_ids(const int64_t *offsets, int64_t *ids, uint64_t N, double alpha, uint64_t seed)
{
    uint64_t A, B;
    perm_params(N, seed, &A, &B);
    const int64_t E = offsets[N];
#pragma omp parallel for schedule(static)
    for (int64_t e = 0; e < E; ++e)
        ids[e] = node_of_rank0(rank_from_hash(wl_mix64(seed ^ 0xabcdef12345ull, (uint64_t)e), N, alpha) - 1, N, A, B);
}

/* ---- distinct-ID set, first-occurrence order ---- */
typedef struct {
    int64_t *slots; /* -1 = empty */
    uint64_t mask;
    int64_t *list;
    int64_t n, cap;
} idset;

static int idset_init(idset *s, int64_t *list, int64_t cap)
{
    uint64_t size = 16;
    while (size < (uint64_t)cap * 2)
        size <<= 1;
    s->slots = (int64_t *)malloc(size * sizeof(int64_t));
    if (!s->slots)
        return 1;
    memset(s->slots, 0xff, size * sizeof(int64_t));
    s->mask = size - 1;
    s->list = list;
    s->n = 0;
    s->cap = cap;
    return 0;
}

/* returns 0 if added or present, 1 if the list is full */
static int idset_add(idset *s, int64_t v)
{
    uint64_t p = wl_mix64(0x5eed, (uint64_t)v) & s->mask;
    while (s->slots[p] != -1) {
        if (s->slots[p] == v)
            return 0;
        p = (p + 1) & s->mask;
    }
    if (s->n >= s->cap)
        return 1;
    s->slots[p] = v;
    s->list[s->n++] = v;
    return 0;
}

static void draw_seeds(idset *s, uint64_t N, int64_t nseeds, uint64_t seed, uint64_t batch)
{
    for (int64_t k = 0; k < nseeds; ++k) {
        const uint64_t h = wl_mix64(seed, batch * 0x100000ull + (uint64_t)k);
        idset_add(s, (int64_t)(((__uint128_t)h * N) >> 64));
    }
}

/*
 * One minibatch from a CSR graph.  out must hold cap IDs; cap >= the slot upper
 * bound nseeds * prod(1 + fanout[h]) is always enough.  Returns the number of
 * distinct IDs, or -1 on allocation failure / overflow of cap.
 */
int64_t wl_sample_csr(const int64_t *offsets, const int64_t *ids, uint64_t N, int64_t nseeds,
                      const int64_t *fanout, int nhops, uint64_t seed, uint64_t batch,
                      int64_t *out, int64_t cap)
{
    idset s;
    if (idset_init(&s, out, cap))
        return -1;
    draw_seeds(&s, N, nseeds, seed, batch);
    uint64_t ctr = 0;
    for (int h = 0; h < nhops; ++h) {
        const int64_t frontier = s.n; /* every distinct node gathered so far */
        for (int64_t f = 0; f < frontier; ++f) {
            const int64_t v = out[f];
            const int64_t lo = offsets[v], d = offsets[v + 1] - lo;
            if (d <= fanout[h]) {
                for (int64_t j = 0; j < d; ++j)
                    if (idset_add(&s, ids[lo + j]))
                        goto full;
            } else {
                for (int64_t j = 0; j < fanout[h]; ++j) {
                    const uint64_t hsh = wl_mix64(seed ^ 0x51ed270b5ull, (batch << 40) + ctr++);
                    const int64_t pick = (int64_t)(((__uint128_t)hsh * (uint64_t)d) >> 64);
                    if (idset_add(&s, ids[lo + pick]))
                        goto full;
                }
            }
        }
    }
    free(s.slots);
    return s.n;
full:
    free(s.slots);
    return -1;
}

/*
 * Same for a procedural graph that is never materialised: every node has
 * `degree` neighbour slots and slot j of node v holds
 * node_of_rank(rank_from_hash(hash(graph_seed, v*degree + j))).
 */
int64_t wl_sample_procedural(uint64_t N, int64_t degree, double alpha, uint64_t graph_seed, int64_t nseeds,
                             const int64_t *fanout, int nhops, uint64_t seed, uint64_t batch,
                             int64_t *out, int64_t cap)
{
    uint64_t A, B;
    perm_params(N, graph_seed, &A, &B);
    idset s;
    if (idset_init(&s, out, cap))
        return -1;
    draw_seeds(&s, N, nseeds, seed, batch);
    uint64_t ctr = 0;
    for (int h = 0; h < nhops; ++h) {
        const int64_t frontier = s.n;
        for (int64_t f = 0; f < frontier; ++f) {
            const uint64_t v = (uint64_t)out[f];
            const int64_t k = degree <= fanout[h] ? degree : fanout[h];
            for (int64_t j = 0; j < k; ++j) {
                uint64_t slot = (uint64_t)j;
                if (degree > fanout[h]) {
                    const uint64_t hsh = wl_mix64(seed ^ 0x51ed270b5ull, (batch << 40) + ctr++);
                    slot = (uint64_t)(((__uint128_t)hsh * (uint64_t)degree) >> 64);
                }
                const uint64_t r = rank_from_hash(wl_mix64(graph_seed ^ 0xabcdef12345ull, v * (uint64_t)degree + slot), N, alpha);
                if (idset_add(&s, node_of_rank0(r - 1, N, A, B))) {
                    free(s.slots);
                    return -1;
                }
            }
        }
    }
    free(s.slots);
    return s.n;
}
