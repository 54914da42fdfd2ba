/*
 * CPU ORACLE for N:M transposable sparsity masks  --  TEST INFRASTRUCTURE, NOT THE PRODUCT.
 *
 * A plain, slow, obviously-correct implementation of what the GPU library computes, written from
 * the paper (arXiv 2102.08124, Sec. 4 "Computing transposable sparsity masks", Eq. 3, Fig. 3,
 * Algorithm 1, App. A.2-A.3).  Only tests, the smoke check and the benchmark's cpu_baseline leg
 * may call it.  It shares no code with the HIP path and does no blocking, fusion or reordering
 * beyond what the definitions state.
 *
 * Conventions (block = M x M tile of a row-major matrix, grid origin (0,0), stride M both ways):
 *   N = entries KEPT per row/column of a block (Eq. 3: row and column sums of the mask S equal N)
 *   K = M - N = entries PRUNED per row/column
 *   mask byte 1 = kept (S_ij = 1), 0 = pruned
 *   dtype 0 = IEEE fp32, dtype 1 = bfloat16 given as raw 16-bit patterns
 *
 * Functions and the passage each follows:
 *   oracle_approx      Algorithm 1 (greedy 2-approximation), literal sort + sweep
 *   oracle_exact       Eq. 3 optimum through the Fig. 3 min-cost-flow network, textbook
 *                      successive shortest paths in fp64
 *   oracle_score       Eq. 3's objective and constraint counts for a given mask
 *   oracle_apply_pack  W (.) S and compression of W and W^T into N values + N indices per group
 *                      of M (format is this project's; the paper only motivates it in Sec. 4)
 *   oracle_unpack      inverse of the packing, used by round-trip checks
 *   oracle_prune_1d    structured N:M magnitude pruning along rows (Sec. 3, constraint 2), the
 *                      non-transposable baseline
 *
 * Pins (tests/test_oracle_*.py): brute force over all valid patterns for tiny (N,M), an LP
 * solved by an independent library, the assignment-problem special case, the appendix's 7/4
 * worked example, the per-node "K lightest" characterisation, the Lemma W(P) <= 2 W*, and
 * symmetry invariants.  No function here is unpinned.
 */
#include <math.h>
#include <pthread.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORACLE_MAX_M 32
#define ORACLE_OK 0
#define ORACLE_ERR_ARG (-1)

/* ------------------------------------------------------------------ element access ---------- */

/* Magnitude ordering key: the bit pattern with the sign cleared, compared as an unsigned integer.
 * -0 == +0, denormals are kept, +Inf is above every finite value and NaNs are above Inf. */
static uint32_t abs_key(const void *w, int dtype, int64_t idx)
{
    if (dtype == 0)
        return ((const uint32_t *)w)[idx] & 0x7FFFFFFFu;
    return (uint32_t)(((const uint16_t *)w)[idx] & 0x7FFFu);
}

/* |W_ij| as a double (exact widening). */
static double abs_val(const void *w, int dtype, int64_t idx)
{
    uint32_t bits = (dtype == 0) ? (((const uint32_t *)w)[idx] & 0x7FFFFFFFu)
                                 : ((uint32_t)(((const uint16_t *)w)[idx] & 0x7FFFu) << 16);
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

static int check_shape(const void *w, int dtype, int64_t rows, int64_t cols, int64_t ld, int N, int M)
{
    if (!w || (dtype != 0 && dtype != 1))
        return ORACLE_ERR_ARG;
    if (M < 2 || M > ORACLE_MAX_M || N <= 0 || N >= M)
        return ORACLE_ERR_ARG;
    if (rows <= 0 || cols <= 0 || rows % M || cols % M || ld < cols)
        return ORACLE_ERR_ARG;
    return ORACLE_OK;
}

/* ------------------------------------------------------------------ Algorithm 1 ------------- */

typedef struct {
    uint32_t key; /* |W_ij| as ordering key */
    int pos;      /* i*M + j */
} edge_t;

/* Stable bottom-up merge sort by key: equal keys keep their row-major order, which realises the
 * (magnitude, then linear index) total order. */
static void sort_edges(edge_t *e, edge_t *tmp, int n)
{
    for (int width = 1; width < n; width *= 2) {
        for (int lo = 0; lo < n; lo += 2 * width) {
            int mid = lo + width < n ? lo + width : n;
            int hi = lo + 2 * width < n ? lo + 2 * width : n;
            int a = lo, b = mid, o = lo;
            while (a < mid && b < hi)
                tmp[o++] = (e[b].key < e[a].key) ? e[b++] : e[a++];
            while (a < mid)
                tmp[o++] = e[a++];
            while (b < hi)
                tmp[o++] = e[b++];
        }
        memcpy(e, tmp, (size_t)n * sizeof *e);
    }
}

/* Algorithm 1 on one block.  pruned[i*M+j] = 1 iff coefficient edge (row i, column j) ends in P.
 * The bipartite graph of Fig. 3 has one node per row and per column; degree(.) counts a node's
 * edges already in P.  An edge joins P while either endpoint still has fewer than K edges in P
 * (strict test: the appendix's worked example stops as soon as every node is covered). */
static void approx_block(const void *w, int dtype, int64_t base, int64_t ld, int M, int K, uint8_t *pruned)
{
    edge_t e[ORACLE_MAX_M * ORACLE_MAX_M], tmp[ORACLE_MAX_M * ORACLE_MAX_M];
    int deg_row[ORACLE_MAX_M] = {0}, deg_col[ORACLE_MAX_M] = {0};
    int n = M * M;
    for (int i = 0; i < M; i++)
        for (int j = 0; j < M; j++) {
            e[i * M + j].key = abs_key(w, dtype, base + i * ld + j);
            e[i * M + j].pos = i * M + j;
        }
    sort_edges(e, tmp, n); /* step 1: light to heavy */
    memset(pruned, 0, (size_t)n);
    for (int k = 0; k < n; k++) { /* step 2: sweep */
        int u = e[k].pos / M, v = e[k].pos % M;
        if (deg_row[u] < K || deg_col[v] < K) {
            pruned[e[k].pos] = 1;
            deg_row[u]++;
            deg_col[v]++;
        }
    }
}

/* ------------------------------------------------------------------ Fig. 3 min-cost flow ---- */

#define MCF_MAX_NODES (2 * ORACLE_MAX_M + 2)
#define MCF_MAX_ARCS (2 * (ORACLE_MAX_M * ORACLE_MAX_M + 2 * ORACLE_MAX_M))

typedef struct {
    int n_nodes, n_arcs;
    int head[MCF_MAX_NODES];  /* first arc out of a node, -1 if none */
    int next[MCF_MAX_ARCS];   /* next arc out of the same node */
    int to[MCF_MAX_ARCS];
    int cap[MCF_MAX_ARCS];    /* residual capacity */
    double cost[MCF_MAX_ARCS];
} mcf_t;

static void mcf_init(mcf_t *g, int n_nodes)
{
    g->n_nodes = n_nodes;
    g->n_arcs = 0;
    for (int v = 0; v < n_nodes; v++)
        g->head[v] = -1;
}

/* Adds arc u->v and its residual twin v->u; arcs 2k and 2k+1 are twins. Returns the forward id. */
static int mcf_add(mcf_t *g, int u, int v, int cap, double cost)
{
    int a = g->n_arcs;
    g->to[a] = v; g->cap[a] = cap; g->cost[a] = cost; g->next[a] = g->head[u]; g->head[u] = a;
    g->to[a + 1] = u; g->cap[a + 1] = 0; g->cost[a + 1] = -cost; g->next[a + 1] = g->head[v]; g->head[v] = a + 1;
    g->n_arcs += 2;
    return a;
}

/* Successive shortest paths: repeatedly send flow along a cheapest s->t path of the residual
 * network until `demand` units are sent.  Node potentials keep reduced costs non-negative so each
 * search is a dense Dijkstra (all original costs are >= 0, so zero potentials are valid at the
 * start).  Returns the flow sent. */
static int mcf_solve(mcf_t *g, int s, int t, int demand)
{
    double pot[MCF_MAX_NODES] = {0.0};
    int sent = 0;
    while (sent < demand) {
        double dist[MCF_MAX_NODES];
        int done[MCF_MAX_NODES], pred_arc[MCF_MAX_NODES];
        for (int v = 0; v < g->n_nodes; v++) {
            dist[v] = INFINITY; done[v] = 0; pred_arc[v] = -1;
        }
        dist[s] = 0.0;
        for (;;) {
            int u = -1;
            for (int v = 0; v < g->n_nodes; v++)
                if (!done[v] && dist[v] < INFINITY && (u < 0 || dist[v] < dist[u]))
                    u = v;
            if (u < 0)
                break;
            done[u] = 1;
            for (int a = g->head[u]; a >= 0; a = g->next[a]) {
                int v = g->to[a];
                if (g->cap[a] <= 0 || done[v])
                    continue;
                double nd = dist[u] + (g->cost[a] + pot[u] - pot[v]);
                if (nd < dist[v]) {
                    dist[v] = nd; pred_arc[v] = a;
                }
            }
        }
        if (!done[t])
            break; /* no augmenting path: demand infeasible */
        /* Reached nodes move by their distance; unreached ones by the largest distance found,
         * which keeps every residual arc's reduced cost non-negative for the next search. */
        double far = 0.0;
        for (int v = 0; v < g->n_nodes; v++)
            if (done[v] && dist[v] > far)
                far = dist[v];
        for (int v = 0; v < g->n_nodes; v++)
            pot[v] += done[v] ? dist[v] : far;
        int push = demand - sent;
        for (int v = t; v != s; v = g->to[pred_arc[v] ^ 1])
            if (g->cap[pred_arc[v]] < push)
                push = g->cap[pred_arc[v]];
        for (int v = t; v != s; v = g->to[pred_arc[v] ^ 1]) {
            g->cap[pred_arc[v]] -= push;
            g->cap[pred_arc[v] ^ 1] += push;
        }
        sent += push;
    }
    return sent;
}

/* Exact optimum of Eq. 3 on one block via the network of Fig. 3:
 *   source -> row i   capacity K, cost 0      (K entries of row i are selected for pruning)
 *   row i  -> col j   capacity 1, cost |W_ij| (unit flow <=> W_ij is pruned)
 *   col j  -> sink    capacity K, cost 0
 * A min-cost flow of value M*K selects the pruned set of least total magnitude; S = 1 - flow.
 * (The figure prints capacity M/2 because it draws the N = M/2 case.)
 * Returns 0 on success, non-zero if the flow could not be routed (cannot happen for 0 < K < M). */
static int exact_block(const void *w, int dtype, int64_t base, int64_t ld, int M, int K, uint8_t *pruned)
{
    mcf_t g;
    int coef_arc[ORACLE_MAX_M * ORACLE_MAX_M];
    int s = 0, t = 2 * M + 1;
    mcf_init(&g, 2 * M + 2);
    for (int i = 0; i < M; i++)
        mcf_add(&g, s, 1 + i, K, 0.0);
    for (int i = 0; i < M; i++)
        for (int j = 0; j < M; j++)
            coef_arc[i * M + j] = mcf_add(&g, 1 + i, 1 + M + j, 1, abs_val(w, dtype, base + i * ld + j));
    for (int j = 0; j < M; j++)
        mcf_add(&g, 1 + M + j, t, K, 0.0);
    int sent = mcf_solve(&g, s, t, M * K);
    for (int k = 0; k < M * M; k++)
        pruned[k] = (uint8_t)(g.cap[coef_arc[k]] == 0);
    return sent == M * K ? 0 : 1;
}

/* Sizes of the Fig. 3 network, exported so a test can check them against the paper's counts
 * (2M+2 nodes, M^2+2M edges, demand M*K). out[0]=nodes, out[1]=edges, out[2]=demand. */
void oracle_network_sizes(int N, int M, int64_t *out)
{
    mcf_t g;
    mcf_init(&g, 2 * M + 2);
    for (int i = 0; i < M; i++) mcf_add(&g, 0, 1 + i, M - N, 0.0);
    for (int i = 0; i < M; i++)
        for (int j = 0; j < M; j++) mcf_add(&g, 1 + i, 1 + M + j, 1, 0.0);
    for (int j = 0; j < M; j++) mcf_add(&g, 1 + M + j, 2 * M + 1, M - N, 0.0);
    out[0] = g.n_nodes;
    out[1] = g.n_arcs / 2;
    out[2] = (int64_t)M * (M - N);
}

/* ------------------------------------------------------------------ matrix drivers ---------- */

typedef struct {
    int kind; /* 0 approx, 1 exact */
    const void *w; int dtype; int64_t rows, cols, ld; int N, M;
    uint8_t *mask; int64_t mask_ld;
    double *per_block; /* nullable: retained L1 of each block, block-row-major */
    int64_t br0, br1;  /* block-row range of this worker */
    double partial;    /* retained L1 over the range */
    int failed;
} job_t;

static void *mask_worker(void *arg)
{
    job_t *jb = (job_t *)arg;
    int M = jb->M, K = jb->M - jb->N;
    int64_t bpr = jb->cols / M;
    uint8_t pruned[ORACLE_MAX_M * ORACLE_MAX_M];
    double total = 0.0;
    for (int64_t br = jb->br0; br < jb->br1; br++)
        for (int64_t bc = 0; bc < bpr; bc++) {
            int64_t base = br * M * jb->ld + bc * M;
            if (jb->kind == 0)
                approx_block(jb->w, jb->dtype, base, jb->ld, M, K, pruned);
            else
                jb->failed |= exact_block(jb->w, jb->dtype, base, jb->ld, M, K, pruned);
            double blk = 0.0;
            for (int i = 0; i < M; i++)
                for (int j = 0; j < M; j++) {
                    uint8_t keep = (uint8_t)!pruned[i * M + j];
                    jb->mask[(br * M + i) * jb->mask_ld + bc * M + j] = keep;
                    if (keep)
                        blk += abs_val(jb->w, jb->dtype, base + i * jb->ld + j);
                }
            if (jb->per_block)
                jb->per_block[br * bpr + bc] = blk;
            total += blk;
        }
    jb->partial = total;
    return NULL;
}

static int run_mask(int kind, const void *w, int dtype, int64_t rows, int64_t cols, int64_t ld, int N, int M,
                    uint8_t *mask, int64_t mask_ld, double *objective, double *per_block, int n_threads)
{
    int rc = check_shape(w, dtype, rows, cols, ld, N, M);
    if (rc)
        return rc;
    if (!mask || mask_ld < cols)
        return ORACLE_ERR_ARG;
    int64_t n_br = rows / M;
    if (n_threads < 1) n_threads = 1;
    if (n_threads > 256) n_threads = 256;
    if ((int64_t)n_threads > n_br) n_threads = (int)n_br;
    job_t jobs[256];
    pthread_t th[256];
    for (int t = 0; t < n_threads; t++) {
        job_t *jb = &jobs[t];
        jb->kind = kind; jb->w = w; jb->dtype = dtype; jb->rows = rows; jb->cols = cols; jb->ld = ld;
        jb->N = N; jb->M = M; jb->mask = mask; jb->mask_ld = mask_ld; jb->per_block = per_block;
        jb->br0 = n_br * t / n_threads; jb->br1 = n_br * (t + 1) / n_threads;
        jb->partial = 0.0; jb->failed = 0;
    }
    if (n_threads == 1)
        mask_worker(&jobs[0]);
    else {
        for (int t = 0; t < n_threads; t++) pthread_create(&th[t], NULL, mask_worker, &jobs[t]);
        for (int t = 0; t < n_threads; t++) pthread_join(th[t], NULL);
    }
    double total = 0.0;
    int failed = 0;
    for (int t = 0; t < n_threads; t++) { total += jobs[t].partial; failed |= jobs[t].failed; }
    if (objective)
        *objective = total;
    return failed ? -2 : ORACLE_OK;
}

/* Algorithm 1 over every block. mask: rows x cols bytes (1 = kept). objective: sum S|W|. */
int oracle_approx(const void *w, int dtype, int64_t rows, int64_t cols, int64_t ld, int N, int M,
                  uint8_t *mask, int64_t mask_ld, double *objective, double *per_block, int n_threads)
{
    return run_mask(0, w, dtype, rows, cols, ld, N, M, mask, mask_ld, objective, per_block, n_threads);
}

/* Eq. 3 optimum over every block (Fig. 3 network). */
int oracle_exact(const void *w, int dtype, int64_t rows, int64_t cols, int64_t ld, int N, int M,
                 uint8_t *mask, int64_t mask_ld, double *objective, double *per_block, int n_threads)
{
    return run_mask(1, w, dtype, rows, cols, ld, N, M, mask, mask_ld, objective, per_block, n_threads);
}

/* ------------------------------------------------------------------ 1-D N:M pruning --------- */

/* Structured (non-transposable) N:M magnitude pruning, the baseline of Sec. 3 (constraint 2 of the
 * mask-diversity list): in every group of M consecutive elements of a row the M - N lightest are pruned,
 * lightest = smallest (magnitude key, position).  Written as the definition: order the group with a stable
 * insertion sort, prune the first M - N.  objective = sum S|W|. */
int oracle_prune_1d(const void *w, int dtype, int64_t rows, int64_t cols, int64_t ld, int N, int M,
                    uint8_t *mask, int64_t mask_ld, double *objective)
{
    if (!w || !mask || rows <= 0 || cols <= 0 || M < 2 || M > ORACLE_MAX_M || N <= 0 || N >= M || cols % M ||
        ld < cols || mask_ld < cols)
        return ORACLE_ERR_ARG;
    double obj = 0.0;
    for (int64_t r = 0; r < rows; r++)
        for (int64_t g = 0; g < cols / M; g++) {
            int order[ORACLE_MAX_M];
            for (int j = 0; j < M; j++) {          /* stable insertion sort by magnitude key */
                uint32_t kj = abs_key(w, dtype, r * ld + g * M + j);
                int pos = j;
                while (pos > 0 && abs_key(w, dtype, r * ld + g * M + order[pos - 1]) > kj) {
                    order[pos] = order[pos - 1];
                    pos--;
                }
                order[pos] = j;
            }
            for (int q = 0; q < M; q++) {
                int j = order[q];
                uint8_t keep = q >= M - N;
                mask[r * mask_ld + g * M + j] = keep;
                if (keep)
                    obj += abs_val(w, dtype, r * ld + g * M + j);
            }
        }
    if (objective)
        *objective = obj;
    return ORACLE_OK;
}

/* ------------------------------------------------------------------ score ------------------- */

/* out[0] = retained L1 = sum S|W| (Eq. 3's objective), out[1] = total L1.
 * cnt[0] = kept entries, cnt[1] = (block,row) pairs with more than N kept,
 * cnt[2] = (block,column) pairs with more than N kept,
 * cnt[3] = (block,row) pairs with kept != N, cnt[4] = same for columns.
 * per_block (nullable) receives each block's retained L1. Any non-zero mask byte counts as kept. */
int oracle_score(const void *w, int dtype, int64_t rows, int64_t cols, int64_t ld, int N, int M,
                 const uint8_t *mask, int64_t mask_ld, double *out, uint64_t *cnt, double *per_block)
{
    int rc = check_shape(w, dtype, rows, cols, ld, N, M);
    if (rc)
        return rc;
    if (!mask || mask_ld < cols || !out || !cnt)
        return ORACLE_ERR_ARG;
    double retained = 0.0, total = 0.0;
    uint64_t kept = 0, rowv = 0, colv = 0, rowne = 0, colne = 0;
    int64_t bpr = cols / M;
    for (int64_t br = 0; br < rows / M; br++)
        for (int64_t bc = 0; bc < bpr; bc++) {
            int rs[ORACLE_MAX_M] = {0}, cs[ORACLE_MAX_M] = {0};
            double blk = 0.0;
            for (int i = 0; i < M; i++)
                for (int j = 0; j < M; j++) {
                    double a = abs_val(w, dtype, (br * M + i) * ld + bc * M + j);
                    total += a;
                    if (mask[(br * M + i) * mask_ld + bc * M + j]) {
                        blk += a; rs[i]++; cs[j]++; kept++;
                    }
                }
            for (int i = 0; i < M; i++) {
                rowv += rs[i] > N; colv += cs[i] > N; rowne += rs[i] != N; colne += cs[i] != N;
            }
            if (per_block)
                per_block[br * bpr + bc] = blk;
            retained += blk;
        }
    out[0] = retained; out[1] = total;
    cnt[0] = kept; cnt[1] = rowv; cnt[2] = colv; cnt[3] = rowne; cnt[4] = colne;
    return ORACLE_OK;
}

/* ------------------------------------------------------------------ apply + pack ------------ */

static int index_bits(int M)
{
    int b = 0;
    while ((1 << b) < M) b++;
    return b;
}

static void put_bits(uint8_t *row, int64_t bit_off, int n_bits, uint32_t v)
{
    for (int b = 0; b < n_bits; b++)
        if ((v >> b) & 1u)
            row[(bit_off + b) >> 3] |= (uint8_t)(1u << ((bit_off + b) & 7));
}

static uint32_t get_bits(const uint8_t *row, int64_t bit_off, int n_bits)
{
    uint32_t v = 0;
    for (int b = 0; b < n_bits; b++)
        v |= (uint32_t)((row[(bit_off + b) >> 3] >> ((bit_off + b) & 7)) & 1u) << b;
    return v;
}

/* Compress one operand. Element (r, c) of the operand is W[r*sr + c*sc] with mask byte
 * S[r*mr + c*mc]; groups are M consecutive c of one r. Each group yields exactly N slots:
 * the kept positions, then (if fewer than N are kept) the lowest-numbered unused positions as
 * zero-valued fillers, all ordered by position. vals: R x (C*N/M) elements, bit copies of W
 * (+0 for fillers); idx: per row, slots of ceil(log2 M) bits packed LSB-first, rows padded to
 * whole bytes. A group with more than N kept entries keeps only its first N (caller error). */
static void pack_operand(const void *w, int dtype, const uint8_t *mask, int64_t R, int64_t C,
                         int64_t sr, int64_t sc, int64_t mr, int64_t mc, int N, int M,
                         void *vals, uint8_t *idx)
{
    int ib = index_bits(M);
    int64_t slots_per_row = C / M * N;
    int64_t idx_row_bytes = (slots_per_row * ib + 7) / 8;
    memset(idx, 0, (size_t)(R * idx_row_bytes));
    for (int64_t r = 0; r < R; r++)
        for (int64_t g = 0; g < C / M; g++) {
            int chosen[ORACLE_MAX_M] = {0};
            int n_kept = 0;
            for (int p = 0; p < M && n_kept < N; p++)
                if (mask[r * mr + (g * M + p) * mc]) { chosen[p] = 1; n_kept++; }
            for (int p = 0, fill = N - n_kept; p < M && fill > 0; p++)
                if (!chosen[p]) { chosen[p] = 2; fill--; }
            int slot = 0;
            for (int p = 0; p < M; p++) {
                if (!chosen[p])
                    continue;
                int64_t o = r * slots_per_row + g * N + slot;
                int64_t src = r * sr + (g * M + p) * sc;
                if (dtype == 0)
                    ((uint32_t *)vals)[o] = chosen[p] == 1 ? ((const uint32_t *)w)[src] : 0u;
                else
                    ((uint16_t *)vals)[o] = chosen[p] == 1 ? ((const uint16_t *)w)[src] : (uint16_t)0;
                put_bits(idx + r * idx_row_bytes, (g * N + slot) * ib, ib, (uint32_t)p);
                slot++;
            }
        }
}

/* W (.) S (a select: pruned entries become +0), then pack W (groups along columns) into
 * vals/idx and W^T (groups along rows of W) into valsT/idxT. */
int oracle_apply_pack(const void *w, int dtype, int64_t rows, int64_t cols, int64_t ld, int N, int M,
                      const uint8_t *mask, int64_t mask_ld, void *vals, uint8_t *idx, void *valsT, uint8_t *idxT)
{
    int rc = check_shape(w, dtype, rows, cols, ld, N, M);
    if (rc)
        return rc;
    if (!mask || mask_ld < cols || !vals || !idx || !valsT || !idxT)
        return ORACLE_ERR_ARG;
    pack_operand(w, dtype, mask, rows, cols, ld, 1, mask_ld, 1, N, M, vals, idx);
    pack_operand(w, dtype, mask, cols, rows, 1, ld, 1, mask_ld, N, M, valsT, idxT);
    return ORACLE_OK;
}

/* Expand a packed operand (R x C logical) back to dense, zeros elsewhere. dense has leading dim C. */
int oracle_unpack(const void *vals, const uint8_t *idx, int dtype, int64_t R, int64_t C, int N, int M, void *dense)
{
    if (!vals || !idx || !dense || M < 2 || M > ORACLE_MAX_M || N <= 0 || N >= M || C % M)
        return ORACLE_ERR_ARG;
    int ib = index_bits(M);
    int64_t slots_per_row = C / M * N;
    int64_t idx_row_bytes = (slots_per_row * ib + 7) / 8;
    memset(dense, 0, (size_t)(R * C) * (dtype == 0 ? 4 : 2));
    for (int64_t r = 0; r < R; r++)
        for (int64_t g = 0; g < C / M; g++)
            for (int slot = 0; slot < N; slot++) {
                uint32_t p = get_bits(idx + r * idx_row_bytes, (g * N + slot) * ib, ib);
                int64_t o = r * slots_per_row + g * N + slot;
                if (dtype == 0)
                    ((uint32_t *)dense)[r * C + g * M + p] = ((const uint32_t *)vals)[o];
                else
                    ((uint16_t *)dense)[r * C + g * M + p] = ((const uint16_t *)vals)[o];
            }
    return ORACLE_OK;
}
