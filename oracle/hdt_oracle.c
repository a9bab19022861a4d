/*
 * CPU oracle for hierarchical document attention (HDT, arXiv 2407.08330).
 *
 * TEST INFRASTRUCTURE ONLY.  This is a plain, slow, fp64 statement of what the
 * method computes; it exists so that the HIP library can be checked against
 * something written independently of it.  Only the tests, the smoke check and
 * the benchmark's cpu_baseline leg may call it.  It shares no code, header or
 * table with the HIP library.
 *
 * What is implemented, and the passage each part follows:
 *   - the attention mask, pair by pair from explicit parent pointers: a position
 *     sees its parent, its siblings (itself included) and its children
 *     (Sec. 3.2 "Hierarchical Attention", Eqs. for M^DOC / M^SEC / M^SENT and
 *     their OR; Fig. 2 caption); and the thinned, directed variants of it that
 *     Sec. 4.1 uses on ListOps (no edge to the parent; no edges between siblings);
 *   - masked softmax attention by its definition, two-pass softmax, no tiling
 *     and no online rescaling (Sec. 3.2, the equation S = softmax(A (.) 1_M),
 *     A = Q K^T / sqrt(d_k), O = S V; -inf where M = 0);
 *   - its gradient, by differentiating that definition (the paper does not
 *     describe a backward pass);
 *   - the key order "sorted by hierarchy level" and the block partition with
 *     the skip-empty-blocks rule (Sec. 3.2 last paragraphs; App. A.1, Alg. 1
 *     steps "Sort K, V", "Partition", "If non-zero values in M"), by brute force
 *     over all pairs of every block;
 *   - per-query-block key lists (the keys any row of the block may attend to, in
 *     that key order, cut into entries of a fixed number of keys), again by brute
 *     force: the library's default schedule, a refinement of the fixed windows
 *     that the paper's closing remark of Sec. 3.2 on better permutations invites;
 *   - the hierarchical positional encoding: index vectors from the tree and the
 *     sum of sinusoidal encodings over the levels (Sec. 3.2, Eq. pos_enc).
 *
 * Readings where the paper is silent (each also listed in the design notes):
 *   - a position attends to itself (M^SENT_ii = 1);
 *   - the root has no siblings: two positions with parent -1 are not siblings;
 *   - pad positions (level < 0) see nothing and are seen by nothing; their
 *     output row is 0, their log-sum-exp is -inf, their gradients are 0;
 *   - ties inside a level keep document order (stable sort); pads go last;
 *   - the log-sum-exp returned is natural-log: lse_i = ln sum_j exp(s_ij).
 *
 * Every function has pins in tests/ that do not come from this file: masks
 * enumerated by hand, the paper's three mask equations on index vectors, dense
 * softmax attention for a one-group document, closed-form row counts, closed
 * forms for Q = 0, central finite differences for the gradients, key lists written
 * out by hand for a 16-position document.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ---- mask: parent / siblings / children, pair by pair ------------------- */

/* Which kinds of edges of the hierarchy carry attention (Sec. 4.1 "Mathematical Reasoning": the
 * full pattern of Sec. 3.2 is red + green + blue; the sparser ListOps variants drop the edge from a
 * position to its parent ("operands do not attend to their operators": green + blue) and then
 * also the edges between siblings ("operands do not attend to each other": blue only)).
 * A position always attends to itself. */
#define ORACLE_EDGE_UP 1      /* a position attends to its parent             */
#define ORACLE_EDGE_SIBLING 2 /* a position attends to its siblings           */
#define ORACLE_EDGE_DOWN 4    /* a position attends to its children           */
#define ORACLE_EDGE_ALL 7

/* 1 iff position i may attend to position j under the edge kinds `edges`. */
int oracle_allowed_edges(const int32_t *level, const int32_t *parent, int64_t i, int64_t j, int edges)
{
    if (level[i] < 0 || level[j] < 0) return 0;        /* pads */
    if (i == j) return 1;                               /* itself */
    if ((edges & ORACLE_EDGE_SIBLING) && parent[i] >= 0 && parent[i] == parent[j]) return 1; /* same parent */
    if ((edges & ORACLE_EDGE_UP) && parent[i] == j) return 1;   /* j is i's parent */
    if ((edges & ORACLE_EDGE_DOWN) && parent[j] == i) return 1; /* j is i's child */
    return 0;
}

/* The edge kinds every function below uses; ORACLE_EDGE_ALL (the paper's full pattern) unless a test
 * selects a variant.  (A process-wide setting: the oracle is test infrastructure, called from one
 * thread at a time; the OpenMP workers only read it.) */
static int g_edges = ORACLE_EDGE_ALL;
void oracle_set_edges(int edges) { g_edges = edges & ORACLE_EDGE_ALL; }
int oracle_get_edges(void) { return g_edges; }

/* 1 iff position i may attend to position j. */
int oracle_allowed(const int32_t *level, const int32_t *parent, int64_t i, int64_t j)
{
    return oracle_allowed_edges(level, parent, i, j, g_edges);
}

/* Dense mask M[n][n] (row i, column j in document order). */
void oracle_mask(const int32_t *level, const int32_t *parent, int64_t n, uint8_t *M)
{
    for (int64_t i = 0; i < n; i++)
        for (int64_t j = 0; j < n; j++)
            M[i * n + j] = (uint8_t)oracle_allowed(level, parent, i, j);
}

/* Number of allowed keys of every row (rowcount[n]); returns their total. */
int64_t oracle_row_counts(const int32_t *level, const int32_t *parent, int64_t n, int64_t *rowcount)
{
    int64_t total = 0;
#pragma omp parallel for schedule(dynamic, 64) reduction(+ : total)
    for (int64_t i = 0; i < n; i++) {
        int64_t c = 0;
        for (int64_t j = 0; j < n; j++) c += oracle_allowed(level, parent, i, j);
        rowcount[i] = c;
        total += c;
    }
    return total;
}

/* The mask as per-row lists of allowed columns, ascending: rowptr[n+1] must hold the
 * exclusive prefix sum of oracle_row_counts; cols[rowptr[n]] is filled.  (A cache of
 * the pairwise test, so that it is not repeated for every head.) */
void oracle_row_lists(const int32_t *level, const int32_t *parent, int64_t n,
                      const int64_t *rowptr, int32_t *cols)
{
#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t i = 0; i < n; i++) {
        int64_t w = rowptr[i];
        for (int64_t j = 0; j < n; j++)
            if (oracle_allowed(level, parent, i, j)) cols[w++] = (int32_t)j;
    }
}

/* ---- forward: masked softmax attention by definition -------------------- */

/* One sample, `heads` heads.  q,k,v,o: [heads][n][d] fp64; lse: [heads][n].
 * rowptr/cols: the mask lists of this sample. */
void oracle_attn_fwd(const double *q, const double *k, const double *v, int64_t heads, int64_t n,
                     int64_t d, double scale, const int64_t *rowptr, const int32_t *cols,
                     double *o, double *lse)
{
#pragma omp parallel for collapse(2) schedule(dynamic, 16)
    for (int64_t h = 0; h < heads; h++) {
        for (int64_t i = 0; i < n; i++) {
            const double *qi = q + (h * n + i) * d;
            double *oi = o + (h * n + i) * d;
            int64_t cnt = rowptr[i + 1] - rowptr[i];
            for (int64_t c = 0; c < d; c++) oi[c] = 0.0;
            if (cnt == 0) { lse[h * n + i] = -INFINITY; continue; }
            double *s = (double *)malloc((size_t)cnt * sizeof(double));
            double m = -INFINITY;
            for (int64_t t = 0; t < cnt; t++) {
                const double *kj = k + (h * n + cols[rowptr[i] + t]) * d;
                double acc = 0.0;
                for (int64_t c = 0; c < d; c++) acc += qi[c] * kj[c];
                s[t] = scale * acc;
                if (s[t] > m) m = s[t];
            }
            double z = 0.0;
            for (int64_t t = 0; t < cnt; t++) z += exp(s[t] - m);
            double l = m + log(z);
            lse[h * n + i] = l;
            for (int64_t t = 0; t < cnt; t++) {
                double p = exp(s[t] - l);
                const double *vj = v + (h * n + cols[rowptr[i] + t]) * d;
                for (int64_t c = 0; c < d; c++) oi[c] += p * vj[c];
            }
            free(s);
        }
    }
}

/* ---- backward: gradient of the definition ------------------------------- */

/* Given dO, with p_ij = exp(s_ij - lse_i), o_i = sum_j p_ij v_j:
 *   D_i   = sum_c dO_ic o_ic
 *   dV_j  = sum_i p_ij dO_i
 *   dp_ij = sum_c dO_ic v_jc
 *   ds_ij = p_ij (dp_ij - D_i)
 *   dQ_i  = scale sum_j ds_ij k_j,   dK_j = scale sum_i ds_ij q_i
 * Recomputes the forward quantities itself; uses neither O nor LSE from outside. */
void oracle_attn_bwd(const double *q, const double *k, const double *v, const double *d_o,
                     int64_t heads, int64_t n, int64_t d, double scale, const int64_t *rowptr,
                     const int32_t *cols, double *dq, double *dk, double *dv)
{
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t h = 0; h < heads; h++) {
        const double *qh = q + h * n * d, *kh = k + h * n * d, *vh = v + h * n * d;
        const double *doh = d_o + h * n * d;
        double *dqh = dq + h * n * d, *dkh = dk + h * n * d, *dvh = dv + h * n * d;
        memset(dqh, 0, (size_t)(n * d) * sizeof(double));
        memset(dkh, 0, (size_t)(n * d) * sizeof(double));
        memset(dvh, 0, (size_t)(n * d) * sizeof(double));
        double *oi = (double *)malloc((size_t)d * sizeof(double));
        for (int64_t i = 0; i < n; i++) {
            int64_t cnt = rowptr[i + 1] - rowptr[i];
            if (cnt == 0) continue;
            const int32_t *ci = cols + rowptr[i];
            double *p = (double *)malloc((size_t)cnt * sizeof(double));
            double m = -INFINITY;
            for (int64_t t = 0; t < cnt; t++) {
                double acc = 0.0;
                for (int64_t c = 0; c < d; c++) acc += qh[i * d + c] * kh[(int64_t)ci[t] * d + c];
                p[t] = scale * acc;
                if (p[t] > m) m = p[t];
            }
            double z = 0.0;
            for (int64_t t = 0; t < cnt; t++) z += exp(p[t] - m);
            double l = m + log(z);
            for (int64_t c = 0; c < d; c++) oi[c] = 0.0;
            for (int64_t t = 0; t < cnt; t++) {
                p[t] = exp(p[t] - l);
                for (int64_t c = 0; c < d; c++) oi[c] += p[t] * vh[(int64_t)ci[t] * d + c];
            }
            double D = 0.0;
            for (int64_t c = 0; c < d; c++) D += doh[i * d + c] * oi[c];
            for (int64_t t = 0; t < cnt; t++) {
                int64_t j = ci[t];
                double dp = 0.0;
                for (int64_t c = 0; c < d; c++) dp += doh[i * d + c] * vh[j * d + c];
                double ds = p[t] * (dp - D);
                for (int64_t c = 0; c < d; c++) {
                    dvh[j * d + c] += p[t] * doh[i * d + c];
                    dqh[i * d + c] += scale * ds * kh[j * d + c];
                    dkh[j * d + c] += scale * ds * qh[i * d + c];
                }
            }
            free(p);
        }
        free(oi);
    }
}

/* ---- key order and block schedule --------------------------------------- */

/* kperm[s] = document position held by sorted slot s: positions ordered by level
 * (0, 1, 2, ... ; pads last), ties in document order. */
void oracle_kperm(const int32_t *level, int64_t n, int32_t *kperm)
{
    int32_t maxl = -1;
    for (int64_t i = 0; i < n; i++) if (level[i] > maxl) maxl = level[i];
    int64_t s = 0;
    for (int32_t l = 0; l <= maxl; l++)
        for (int64_t i = 0; i < n; i++) if (level[i] == l) kperm[s++] = (int32_t)i;
    for (int64_t i = 0; i < n; i++) if (level[i] < 0) kperm[s++] = (int32_t)i;
}

/* Block (I, J) covers query rows [I*bm, (I+1)*bm) in document order and key slots
 * [J*bn, (J+1)*bn) in sorted order (both cut off at n).  For every block this writes
 *   count[I*tc + J] = number of allowed (row, slot) pairs in it,
 * and, if bits != NULL, the block's bitmap at bits + (I*tc + J) * bm * (bn/32) words:
 * word r*(bn/32) + c/32, bit c%32  <=>  row I*bm + r may attend to slot J*bn + c.
 * tr = ceil(n/bm), tc = ceil(n/bn); bn must be a multiple of 32. */
void oracle_block_scan(const int32_t *level, const int32_t *parent, const int32_t *kperm,
                       int64_t n, int64_t bm, int64_t bn, int32_t *count, uint32_t *bits)
{
    int64_t tr = (n + bm - 1) / bm, tc = (n + bn - 1) / bn, wpr = bn / 32;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t I = 0; I < tr; I++) {
        for (int64_t J = 0; J < tc; J++) {
            int32_t cnt = 0;
            uint32_t *bw = bits ? bits + (I * tc + J) * bm * wpr : NULL;
            if (bw) memset(bw, 0, (size_t)(bm * wpr) * sizeof(uint32_t));
            for (int64_t r = 0; r < bm; r++) {
                int64_t i = I * bm + r;
                if (i >= n) break;
                for (int64_t c = 0; c < bn; c++) {
                    int64_t s = J * bn + c;
                    if (s >= n) break;
                    if (oracle_allowed(level, parent, i, kperm[s])) {
                        cnt++;
                        if (bw) bw[r * wpr + c / 32] |= (uint32_t)1 << (c % 32);
                    }
                }
            }
            count[I * tc + J] = cnt;
        }
    }
}

/* Bitmaps of the listed blocks only: block b = (bi[b], bj[b]); layout of each bitmap as in
 * oracle_block_scan, written at bits + b * bm * (bn/32). */
void oracle_block_bitmaps(const int32_t *level, const int32_t *parent, const int32_t *kperm,
                          int64_t n, int64_t bm, int64_t bn, int64_t n_blocks, const int32_t *bi,
                          const int32_t *bj, uint32_t *bits)
{
    int64_t wpr = bn / 32;
#pragma omp parallel for schedule(dynamic, 8)
    for (int64_t b = 0; b < n_blocks; b++) {
        uint32_t *bw = bits + b * bm * wpr;
        memset(bw, 0, (size_t)(bm * wpr) * sizeof(uint32_t));
        for (int64_t r = 0; r < bm; r++) {
            int64_t i = (int64_t)bi[b] * bm + r;
            if (i >= n) break;
            for (int64_t c = 0; c < bn; c++) {
                int64_t s = (int64_t)bj[b] * bn + c;
                if (s >= n) break;
                if (oracle_allowed(level, parent, i, kperm[s]))
                    bw[r * wpr + c / 32] |= (uint32_t)1 << (c % 32);
            }
        }
    }
}

/* ---- key lists per query block (the library's default schedule) ----------
 *
 * A refinement of the block schedule above that the paper leaves open ("more advanced
 * permutation algorithms", Sec. 3.2 last paragraph): instead of cutting the level-sorted key
 * order into fixed windows shared by all query blocks, every query block I gets its OWN list
 *     U_I = { j : some row i of block I may attend to j },
 * written in key order (the order of kperm: level by level, ties in document order), and that
 * list is cut into entries of bn keys; the last entry of a block is filled up with -1.
 * The result of attention does not depend on this choice (softmax over a set of keys). */

/* ucount[I] = |U_I| for every query block of bm rows; tr = ceil(n/bm) values. */
void oracle_keylist_counts(const int32_t *level, const int32_t *parent, int64_t n, int64_t bm,
                           int32_t *ucount)
{
    int64_t tr = (n + bm - 1) / bm;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t I = 0; I < tr; I++) {
        int32_t u = 0;
        for (int64_t j = 0; j < n; j++) {
            int any = 0;
            for (int64_t i = I * bm; i < (I + 1) * bm && i < n && !any; i++)
                any = oracle_allowed(level, parent, i, j);
            u += any;
        }
        ucount[I] = u;
    }
}

/* entry_ptr[tr+1]: entries of block I are [entry_ptr[I], entry_ptr[I+1]), with
 * entry_ptr[I+1] - entry_ptr[I] = ceil(ucount[I] / bn).  Writes, for every entry e,
 *   keys[e*bn + c]  = c-th key of the entry (document position), -1 past the end of U_I,
 *   bits[(e*bm + r)*wpr + c/32] bit c%32  <=>  row I*bm + r may attend to keys[e*bn + c]
 *                                              (wpr = ceil(bn/32) words per row),
 *   pairs[e]        = number of set bits of the entry. */
void oracle_keylist_fill(const int32_t *level, const int32_t *parent, const int32_t *kperm,
                         int64_t n, int64_t bm, int64_t bn, const int64_t *entry_ptr,
                         int32_t *keys, uint32_t *bits, int32_t *pairs)
{
    int64_t tr = (n + bm - 1) / bm, wpr = (bn + 31) / 32;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t I = 0; I < tr; I++) {
        int64_t e0 = entry_ptr[I], e1 = entry_ptr[I + 1];
        for (int64_t t = e0 * bn; t < e1 * bn; t++) keys[t] = -1;
        memset(bits + e0 * bm * wpr, 0, (size_t)((e1 - e0) * bm * wpr) * sizeof(uint32_t));
        for (int64_t e = e0; e < e1; e++) pairs[e] = 0;
        int64_t u = 0; /* keys of U_I found so far */
        for (int64_t s = 0; s < n; s++) { /* key order */
            int64_t j = kperm[s];
            int any = 0;
            for (int64_t i = I * bm; i < (I + 1) * bm && i < n; i++) {
                if (!oracle_allowed(level, parent, i, j)) continue;
                int64_t e = e0 + u / bn, c = u % bn, r = i - I * bm;
                bits[(e * bm + r) * wpr + c / 32] |= (uint32_t)1 << (c % 32);
                pairs[e]++;
                any = 1;
            }
            if (any) {
                keys[(e0 + u / bn) * bn + u % bn] = (int32_t)j;
                u++;
            }
        }
    }
}

/* ---- hierarchical positional encoding -------------------------------------
 *
 * Sec. 3.2 "Hierarchical Positional Encoding", Eq. (pos_enc) and the caption of Fig. 3: every
 * position carries one linear index p^l per hierarchy level l = 1..L (level 0, the document,
 * needs none); each index goes through the standard sinusoidal functions and the L encodings
 * are summed:
 *     HPE(p, i) = sum_l sin(w_k p^l)  if i = 2k,   sum_l cos(w_k p^l)  if i = 2k + 1,
 *     w_k = 10000^(-2k / d_model).
 * Reading of the (missing) figure: indices are 1-based ordinals among the siblings, and an
 * anchor carries 0 at every level below its own: [DOC] = (0,0,0), the k-th [SEC] = (k,0,0), its
 * m-th [SENT] = (k,m,0), that sentence's t-th token = (k,m,t).  For a general tree: the entry
 * for level l of position i is the ordinal (among the children of its parent, in document order)
 * of i's ancestor-or-self whose level is l, and 0 if there is none.  Pads carry all zeros. */

/* p[i*L + (l-1)], l = 1..L */
void oracle_index_vectors(const int32_t *level, const int32_t *parent, int64_t n, int64_t L, int32_t *p)
{
#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t i = 0; i < n; i++) {
        for (int64_t l = 0; l < L; l++) p[i * L + l] = 0;
        if (level[i] < 0) continue;
        int64_t a = i;
        for (int steps = 0; a >= 0 && steps < 64; steps++) {
            int64_t l = level[a];
            if (l >= 1 && l <= L) {
                int32_t ord = 1; /* earlier positions with the same parent */
                for (int64_t j = 0; j < a; j++)
                    if (level[j] >= 0 && parent[j] == parent[a]) ord++;
                p[i * L + (l - 1)] = ord;
            }
            a = parent[a];
        }
    }
}

/* out[i*d_model + c] = HPE(p_i, c) */
void oracle_hpe(const int32_t *p, int64_t n, int64_t L, int64_t d_model, double *out)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; i++)
        for (int64_t c = 0; c < d_model; c++) {
            int64_t k = c / 2;
            double w = pow(10000.0, -2.0 * (double)k / (double)d_model);
            double acc = 0.0;
            for (int64_t l = 0; l < L; l++) {
                double x = w * (double)p[i * L + l];
                acc += (c % 2 == 0) ? sin(x) : cos(x);
            }
            out[i * d_model + c] = acc;
        }
}

int oracle_num_threads(void)
{
    int n = 1;
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    n = omp_get_max_threads();
#endif
    return n;
}
