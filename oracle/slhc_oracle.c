/*
 * CPU oracle for exact single-linkage clustering of N points in d dimensions.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the GPU library is
 * checked against.  It shares no code with the GPU library and nothing in the product path may
 * call it.  All arithmetic is in double precision on the float32 input values.
 *
 * What it computes, and the passage of the cuSLINK paper (Nolet et al., ECML PKDD 2023) each
 * part follows:
 *
 *   oracle_knn_rows     brute-force k nearest neighbours under squared L2: all distances of a
 *                       query row are evaluated and the k smallest kept (Sec. 3.1.1 "k-NN Graph
 *                       Construction": the method is a brute-force k-NN, it only fuses selection
 *                       into the distance computation; Sec. 3 complexity paragraph: N^2 distance
 *                       evaluations).  The selection is the definition, not the fused algorithm.
 *   oracle_cross_1nn    nearest point that carries a different colour (Sec. 3.1.2 "k-NN Graph
 *                       Connection": a 1-NN that joins points only across different
 *                       supervertices; Alg. "connect_graph").
 *   oracle_mst_prim     exact minimum spanning tree of the complete squared-L2 graph by dense
 *                       Prim (Sec. 1: the result is an exact solution of single-linkage
 *                       clustering; Sec. 2 notes SLINK is Prim's iteration).  This is the plain
 *                       definition of what the paper's Boruvka + connection loop must reach.
 *   oracle_csr_msf      minimum spanning forest of an undirected weighted graph given in CSR form, by
 *                       Kruskal over its edges in the strict order (weight, min endpoint, max
 *                       endpoint) (Sec. 3.2 "Spanning Trees": the MST primitive takes a CSR graph and
 *                       returns a forest when the graph is not connected).  Under a strict total
 *                       order the forest is unique, so it can be compared edge by edge.
 *   oracle_dendrogram   edges sorted by weight, then a union-find pass that gives merge i the
 *                       node id N+i, in the scipy linkage layout (Sec. 3.3.1 "Relabel into
 *                       Dendrogram"; Sec. 2 last paragraph adopts scipy.hierarchy.linkage).
 *
 * Readings where the paper is silent: a point is never its own neighbour (excluded by index, so
 * an exact duplicate at distance 0 is a neighbour); equal distances are ordered by the smaller
 * index; equal-weight edges are ordered by (weight, min endpoint, max endpoint); the two children
 * of a merge are stored smaller id first.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#include <math.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* D(a,b) = sum_t (a_t - b_t)^2, direct form, double precision. */
static double sqdist(const float* a, const float* b, int32_t d)
{
    double s = 0.0;
    for (int32_t t = 0; t < d; ++t) {
        double diff = (double)a[t] - (double)b[t];
        s += diff * diff;
    }
    return s;
}

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* (dist, index) strict order: smaller distance first, then smaller index. */
static int pair_less(double da, int64_t ia, double db, int64_t ib)
{
    return (da < db) || (da == db && ia < ib);
}

/*
 * For every query row rows[q] (q < m): the k points j != rows[q] with the smallest
 * (D(rows[q], j), j), ascending.  out_idx [m*k] int32, out_dist [m*k] double.
 * Requires 1 <= k <= N-1.  Returns 0, or -1 on bad arguments.
 */
int oracle_knn_rows(const float* X, int64_t N, int32_t d, int32_t k,
                    const int64_t* rows, int64_t m, int32_t* out_idx, double* out_dist)
{
    if (!X || !rows || !out_idx || !out_dist || N < 2 || d < 1 || k < 1 || k > N - 1) return -1;
#pragma omp parallel for schedule(dynamic, 4)
    for (int64_t q = 0; q < m; ++q) {
        const int64_t i = rows[q];
        int32_t* bi = out_idx + q * k;
        double* bd = out_dist + q * k;
        int32_t filled = 0;
        for (int64_t j = 0; j < N; ++j) {
            if (j == i) continue;
            const double D = sqdist(X + i * d, X + j * d, d);
            if (filled == k && !pair_less(D, j, bd[k - 1], bi[k - 1])) continue;
            /* insert (D, j) into the ascending list, dropping the last entry when full */
            int32_t p = (filled < k) ? filled : k - 1;
            while (p > 0 && pair_less(D, j, bd[p - 1], bi[p - 1])) {
                bd[p] = bd[p - 1];
                bi[p] = bi[p - 1];
                --p;
            }
            bd[p] = D;
            bi[p] = (int32_t)j;
            if (filled < k) ++filled;
        }
    }
    return 0;
}

/*
 * For every query row rows[q]: the point j with colour[j] != colour[rows[q]] that minimises
 * (D(rows[q], j), j); out_idx[q] = -1 and out_dist[q] = +inf when every point shares the colour.
 */
int oracle_cross_1nn(const float* X, int64_t N, int32_t d, const int32_t* colour,
                     const int64_t* rows, int64_t m, int32_t* out_idx, double* out_dist)
{
    if (!X || !colour || !rows || !out_idx || !out_dist || N < 1 || d < 1) return -1;
#pragma omp parallel for schedule(dynamic, 4)
    for (int64_t q = 0; q < m; ++q) {
        const int64_t i = rows[q];
        double best = INFINITY;
        int64_t arg = -1;
        for (int64_t j = 0; j < N; ++j) {
            if (colour[j] == colour[i]) continue;
            const double D = sqdist(X + i * d, X + j * d, d);
            if (arg < 0 || pair_less(D, j, best, arg)) {
                best = D;
                arg = j;
            }
        }
        out_idx[q] = (int32_t)arg;
        out_dist[q] = best;
    }
    return 0;
}

/*
 * Dense Prim from vertex 0 on the complete graph with weights D(i,j).  Emits N-1 edges in the
 * order they are attached: src = the tree vertex, dst = the attached vertex, w = D(src,dst).
 * Among equal keys the smaller vertex index is attached first; a key is replaced only by a
 * strictly smaller one.
 */
int oracle_mst_prim(const float* X, int64_t N, int32_t d,
                    int32_t* out_src, int32_t* out_dst, double* out_w)
{
    if (!X || !out_src || !out_dst || !out_w || N < 2 || d < 1) return -1;
    double* key = (double*)malloc((size_t)N * sizeof(double));
    int32_t* parent = (int32_t*)malloc((size_t)N * sizeof(int32_t));
    unsigned char* in_tree = (unsigned char*)calloc((size_t)N, 1);
    if (!key || !parent || !in_tree) { free(key); free(parent); free(in_tree); return -2; }
    for (int64_t j = 0; j < N; ++j) { key[j] = INFINITY; parent[j] = -1; }
    int64_t v = 0;
    in_tree[0] = 1;
    for (int64_t step = 0; step < N - 1; ++step) {
        /* relax every outside vertex against the vertex attached last */
#pragma omp parallel for schedule(static)
        for (int64_t j = 0; j < N; ++j) {
            if (in_tree[j]) continue;
            const double D = sqdist(X + v * d, X + j * d, d);
            if (D < key[j]) { key[j] = D; parent[j] = (int32_t)v; }
        }
        /* pick the outside vertex with the smallest (key, index) */
        int64_t arg = -1;
        double best = INFINITY;
        for (int64_t j = 0; j < N; ++j) {
            if (in_tree[j]) continue;
            if (arg < 0 || key[j] < best) { best = key[j]; arg = j; }
        }
        out_src[step] = parent[arg];
        out_dst[step] = (int32_t)arg;
        out_w[step] = best;
        in_tree[arg] = 1;
        v = arg;
    }
    free(key); free(parent); free(in_tree);
    return 0;
}

typedef struct { double w; int32_t lo, hi; } edge_t;

static int edge_cmp(const void* pa, const void* pb)
{
    const edge_t* a = (const edge_t*)pa;
    const edge_t* b = (const edge_t*)pb;
    if (a->w < b->w) return -1;
    if (a->w > b->w) return 1;
    if (a->lo != b->lo) return a->lo < b->lo ? -1 : 1;
    if (a->hi != b->hi) return a->hi < b->hi ? -1 : 1;
    return 0;
}

static int32_t uf_find(int32_t* up, int32_t a)
{
    int32_t r = a;
    while (up[r] != r) r = up[r];
    while (up[a] != r) { int32_t nx = up[a]; up[a] = r; a = nx; }   /* path compression */
    return r;
}

/*
 * n_edges = N-1 tree edges (any order, any orientation) -> linkage arrays.
 * Edges are sorted ascending by (w, min(u,v), max(u,v)).  Merge i joins the clusters that hold
 * the endpoints of sorted edge i into node N+i: children[2i] < children[2i+1] are the node ids
 * of those two clusters, heights[i] = w, sizes[i] = points in the new cluster.
 * sorted_src/dst/w (optional, may be NULL) receive the sorted edges with src < dst.
 * Returns 0; -3 if the edges contain a cycle (the endpoints of an edge are already joined).
 */
int oracle_dendrogram(const int32_t* src, const int32_t* dst, const double* w, int64_t N,
                      int32_t* children, double* heights, int32_t* sizes,
                      int32_t* sorted_src, int32_t* sorted_dst, double* sorted_w)
{
    if (!src || !dst || !w || !children || !heights || !sizes || N < 2) return -1;
    const int64_t E = N - 1;
    edge_t* e = (edge_t*)malloc((size_t)E * sizeof(edge_t));
    int32_t* up = (int32_t*)malloc((size_t)N * sizeof(int32_t));     /* union-find parent */
    int32_t* rnk = (int32_t*)calloc((size_t)N, sizeof(int32_t));      /* union by rank */
    int32_t* node = (int32_t*)malloc((size_t)N * sizeof(int32_t));   /* dendrogram id of a set */
    int32_t* cnt = (int32_t*)malloc((size_t)N * sizeof(int32_t));    /* points in a set */
    if (!e || !up || !rnk || !node || !cnt) { free(e); free(up); free(rnk); free(node); free(cnt); return -2; }
    for (int64_t i = 0; i < E; ++i) {
        e[i].w = w[i];
        e[i].lo = src[i] < dst[i] ? src[i] : dst[i];
        e[i].hi = src[i] < dst[i] ? dst[i] : src[i];
    }
    qsort(e, (size_t)E, sizeof(edge_t), edge_cmp);
    for (int64_t v = 0; v < N; ++v) { up[v] = (int32_t)v; node[v] = (int32_t)v; cnt[v] = 1; }
    int rc = 0;
    for (int64_t i = 0; i < E; ++i) {
        int32_t ra = uf_find(up, e[i].lo), rb = uf_find(up, e[i].hi);
        if (ra == rb) { rc = -3; break; }
        int32_t a = node[ra], b = node[rb];
        children[2 * i] = a < b ? a : b;
        children[2 * i + 1] = a < b ? b : a;
        heights[i] = e[i].w;
        sizes[i] = cnt[ra] + cnt[rb];
        if (rnk[ra] < rnk[rb]) { int32_t t = ra; ra = rb; rb = t; }
        up[rb] = ra;
        if (rnk[ra] == rnk[rb]) ++rnk[ra];
        node[ra] = (int32_t)(N + i);
        cnt[ra] = sizes[i];
        if (sorted_src) sorted_src[i] = e[i].lo;
        if (sorted_dst) sorted_dst[i] = e[i].hi;
        if (sorted_w) sorted_w[i] = e[i].w;
    }
    free(e); free(up); free(rnk); free(node); free(cnt);
    return rc;
}

/*
 * Kruskal on the CSR graph (offsets[V+1], indices[E], weights[E]; every undirected edge may be stored
 * in one or both rows).  Self loops are ignored.  Emits the forest edges ascending by
 * (w, lo, hi) into out_lo/out_hi/out_w (capacity V-1), their number into *n_out, and comp[v] = the
 * smallest vertex id of v's connected component.  Returns 0, or -1 on bad arguments.
 */
typedef struct { float w; int32_t lo, hi; } csr_edge;

static int csr_edge_cmp(const void* pa, const void* pb)
{
    const csr_edge* a = (const csr_edge*)pa;
    const csr_edge* b = (const csr_edge*)pb;
    if (a->w != b->w) return a->w < b->w ? -1 : 1;
    if (a->lo != b->lo) return a->lo < b->lo ? -1 : 1;
    if (a->hi != b->hi) return a->hi < b->hi ? -1 : 1;
    return 0;
}

int oracle_csr_msf(const int32_t* offsets, const int32_t* indices, const float* weights, int64_t V,
                   int32_t* out_lo, int32_t* out_hi, float* out_w, int64_t* n_out, int32_t* comp)
{
    if (!offsets || !n_out || !comp || V < 1) return -1;
    const int64_t E = offsets[V];
    if (E < 0 || offsets[0] != 0) return -1;
    csr_edge* edges = (csr_edge*)malloc(sizeof(csr_edge) * (size_t)(E > 0 ? E : 1));
    int32_t* up = (int32_t*)malloc(sizeof(int32_t) * (size_t)V);
    if (!edges || !up) { free(edges); free(up); return -1; }
    int64_t m = 0;
    for (int64_t v = 0; v < V; ++v) {
        if (offsets[v + 1] < offsets[v]) { free(edges); free(up); return -1; }
        for (int64_t e = offsets[v]; e < offsets[v + 1]; ++e) {
            const int32_t u = indices[e];
            if (u < 0 || u >= V) { free(edges); free(up); return -1; }
            if (u == v) continue;
            edges[m].w = weights[e];
            edges[m].lo = (int32_t)(v < u ? v : u);
            edges[m].hi = (int32_t)(v < u ? u : v);
            ++m;
        }
    }
    qsort(edges, (size_t)m, sizeof(csr_edge), csr_edge_cmp);
    for (int64_t v = 0; v < V; ++v) up[v] = (int32_t)v;
    int64_t n = 0;
    for (int64_t i = 0; i < m; ++i) {
        const int32_t a = uf_find(up, edges[i].lo), b = uf_find(up, edges[i].hi);
        if (a == b) continue;
        up[a > b ? a : b] = a > b ? b : a;          /* the smaller id stays the representative */
        out_lo[n] = edges[i].lo;
        out_hi[n] = edges[i].hi;
        out_w[n] = edges[i].w;
        ++n;
    }
    for (int64_t v = 0; v < V; ++v) comp[v] = uf_find(up, (int32_t)v);
    *n_out = n;
    free(edges);
    free(up);
    return 0;
}

