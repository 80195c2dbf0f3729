/*
 * CPU oracle for DeepPoly bound propagation -- TEST INFRASTRUCTURE ONLY.
 *
 * Plain float64, neuron-at-a-time loops.  Nothing here is shared with the GPU
 * library: no headers, helpers, tables or pre/post-processing.  Only tests,
 * the smoke check and the benchmark's cpu_baseline leg may call it.
 *
 * What it computes, following the paper:
 *   - abstract shape per neuron (l, u, L, U): concrete interval plus polyhedral
 *     lower/upper expressions (Section 2.1; DeepPoly specification, Appendix C);
 *   - a polyhedral expression is c0 + sum_i c_i * eta_i (Section 2.1); in a chain
 *     network all non-zero coefficients of an expression sit in one layer at a
 *     time (Section 3.1, "Generality"), so an expression is held as a constant
 *     and one coefficient per neuron of that layer;
 *   - Affine transformer: L = U = prev.dot(w) + b, l = backsubs_lower(L),
 *     u = backsubs_upper(U) (Appendix C, DeepPoly, "Affine ->");
 *   - ReLU transformer: l = relu(prev.l), u = relu(prev.u), L = relu_n(prev),
 *     U = compute_upper(prev) (Appendix C, DeepPoly, "Relu ->");
 *   - backsubs_* = traverse(backward, priority2 = -layer, stop_traverse = false,
 *     replace_*) followed by map(simplify_*): every iteration replaces each term
 *     c*eta of the deepest layer present by c*L_eta or c*U_eta chosen by the sign
 *     of c ("coeff >= 0.0"), sums the results and adds the old constant back
 *     (map semantics, Section 3.2 and Algorithm 2's final merge); the loop ends
 *     when only input neurons remain, which have no L/U to substitute; then
 *     simplify_* replaces c*eta by c*l or c*u by sign and sums to a real;
 *   - a convolution layer is an affine layer whose weight matrix is the
 *     expanded kernel (Section 3.3: "for a convolutional layer, it represents
 *     an expanded convolution kernel"), zero padding, neurons flattened
 *     (channel, row, column);
 *   - property check: output constraints compared against psi (Section 2).  For
 *     robustness psi is "logit[label] > every other logit"; each difference
 *     logit[label] - logit[o] is itself an affine expression over the last
 *     hidden layer and is lower-bounded with backsubs_lower; verified iff every
 *     such bound is > 0.
 *   - max_depth >= 0 gives the DeepPoly_p variant of Section 6.2: at most p
 *     traverse iterations, then simplify_* against the stored l, u of the layer
 *     reached.  max_depth < 0: full traversal.  max_depth_last (-2: same as
 *     max_depth) is the limit used for the last layer and the property rows:
 *     max_depth = 0 with max_depth_last = -1 is CROWN-IBP (Appendix C: every
 *     affine layer maps simplify_* over its own expression -- interval bounds --
 *     except the last one, which back-substitutes fully).
 *   - Add layer (residual / skip networks; Section 5.2 on expressions that span several blocks; the
 *     specification language names two predecessors prev0, prev1 but the paper prints no Add
 *     transformer -- reading): neuron i of an Add layer is eta_i of the layer directly below plus eta_i of
 *     an earlier layer `skip`; its transformer is the Affine one with unit weights over the two
 *     predecessors: L = U = prev0 + prev1, l = backsubs_lower(L), u = backsubs_upper(U).  An expression
 *     may then hold terms of several layers at once; traverse with priority = layer index replaces, in
 *     every iteration, all terms of the deepest layer that holds any (Section 4.2), and simplify_* maps
 *     over whatever terms are left, each against its own layer's l, u.
 *
 * Build: gcc -O2 -fopenmp -shared -fPIC (see oracle/__init__.py).
 */
#include <stdlib.h>
#include <string.h>
#include <math.h>

enum { DPO_AFFINE = 0, DPO_CONV = 1, DPO_RELU = 2, DPO_ADD = 3 };
enum { DPO_LOWER = 0, DPO_UPPER = 1 };

typedef struct {
    int kind;
    int n_in, n_out;
    const float* W;          /* affine: [n_out, n_in]; conv: [Co, Ci, kh, kw] */
    const float* b;          /* [n_out] or [Co] */
    int Ci, H, Wd, Co, kh, kw, stride, pad, Ho, Wo;   /* conv only */
    int skip;                /* Add only: layer index (0 = input) of the second operand */
} dpo_layer;

/* Per-network, per-batch state: l,u of every layer, relaxation of ReLU layers.
 * Layer index 0 is the input; index i (1-based) is the i-th network layer. */
typedef struct {
    int nlayers;
    const dpo_layer* layers;     /* layers[i-1] describes layer index i */
    int B;
    double** l;                  /* [nlayers+1] -> [B, n_i] */
    double** u;
    double** lam;                /* ReLU layers only: L = lam * eta_prev            */
    double** mu;                 /*                   U = mu * eta_prev + nu        */
    double** nu;
} dpo_state;

static int layer_size(const dpo_state* st, int idx)
{
    if (idx == 0) return st->layers[0].n_in;
    return st->layers[idx - 1].n_out;
}

/* One traverse iteration (replace_lower / replace_upper, Appendix C): every term
 * c * eta_i with eta_i in layer `at` becomes c * L_i when (c >= 0) on the lower
 * side, c * U_i otherwise (mirrored on the upper side); results are summed and
 * the running constant is kept.  Output coefficients are over layer at-1. */
static void replace_layer(const dpo_state* st, int bi, int at, int side,
                          const double* cin, double* c0, double* cout)
{
    const dpo_layer* L = &st->layers[at - 1];
    const int n_out = L->n_out, n_in = L->n_in;
    for (int p = 0; p < n_in; ++p) cout[p] = 0.0;

    if (L->kind == DPO_AFFINE) {
        /* L_i = U_i = b_i + sum_p W[i,p] eta_p : the sign choice picks the same expression */
        for (int i = 0; i < n_out; ++i) {
            const double c = cin[i];
            if (c == 0.0) continue;
            *c0 += c * (double)L->b[i];
            const float* w = L->W + (size_t)i * n_in;
            for (int p = 0; p < n_in; ++p) cout[p] += c * (double)w[p];
        }
    } else if (L->kind == DPO_CONV) {
        /* expanded kernel: W[(co,ho,wo),(ci,hi,wi)] = K[co,ci,hi-ho*s+pad,wi-wo*s+pad] */
        for (int co = 0; co < L->Co; ++co)
            for (int ho = 0; ho < L->Ho; ++ho)
                for (int wo = 0; wo < L->Wo; ++wo) {
                    const double c = cin[((size_t)co * L->Ho + ho) * L->Wo + wo];
                    if (c == 0.0) continue;
                    *c0 += c * (double)L->b[co];
                    for (int ci = 0; ci < L->Ci; ++ci)
                        for (int ky = 0; ky < L->kh; ++ky) {
                            const int hi = ho * L->stride - L->pad + ky;
                            if (hi < 0 || hi >= L->H) continue;
                            for (int kx = 0; kx < L->kw; ++kx) {
                                const int wi = wo * L->stride - L->pad + kx;
                                if (wi < 0 || wi >= L->Wd) continue;
                                const double k = (double)L->W[(((size_t)co * L->Ci + ci) * L->kh + ky) * L->kw + kx];
                                cout[((size_t)ci * L->H + hi) * L->Wd + wi] += c * k;
                            }
                        }
                }
    } else {
        /* ReLU neuron i over predecessor i: L_i = lam_i * eta_i, U_i = mu_i * eta_i + nu_i */
        const double* lam = st->lam[at] + (size_t)bi * n_out;
        const double* mu = st->mu[at] + (size_t)bi * n_out;
        const double* nu = st->nu[at] + (size_t)bi * n_out;
        for (int i = 0; i < n_out; ++i) {
            const double c = cin[i];
            const int use_L = (side == DPO_LOWER) ? (c >= 0.0) : !(c >= 0.0);
            if (use_L) {
                cout[i] += c * lam[i];
            } else {
                cout[i] += c * mu[i];
                *c0 += c * nu[i];
            }
        }
    }
}

/* simplify_lower / simplify_upper (Appendix C): c >= 0 ? c*l : c*u (mirrored). */
static double simplify(const dpo_state* st, int bi, int at, int side, double c0, const double* c)
{
    const int n = layer_size(st, at);
    const double* l = st->l[at] + (size_t)bi * n;
    const double* u = st->u[at] + (size_t)bi * n;
    double acc = c0;
    for (int i = 0; i < n; ++i) {
        const double ci = c[i];
        if (side == DPO_LOWER) acc += (ci >= 0.0) ? ci * l[i] : ci * u[i];
        else                   acc += (ci >= 0.0) ? ci * u[i] : ci * l[i];
    }
    return acc;
}

/* backsubs_lower / backsubs_upper.  `e` (constant *c0, coefficients in buf_a over
 * layer `at`) is traversed backwards; returns the concrete bound.  If sym_c is
 * not NULL and the traversal reached the input, the final input-level
 * expression is copied out. */
static double backsubs(const dpo_state* st, int bi, int at, int side, double c0,
                       double* buf_a, double* buf_b, int max_depth,
                       double* sym_c, double* sym_c0)
{
    int depth = 0;
    double* cur = buf_a;
    double* nxt = buf_b;
    while (at > 0 && (max_depth < 0 || depth < max_depth)) {
        replace_layer(st, bi, at, side, cur, &c0, nxt);
        double* t = cur; cur = nxt; nxt = t;
        --at;
        ++depth;
    }
    if (sym_c && at == 0) {
        memcpy(sym_c, cur, sizeof(double) * (size_t)layer_size(st, 0));
        *sym_c0 = c0;
    }
    return simplify(st, bi, at, side, c0, cur);
}

/* The polyhedral expression prev.dot(w_r) + b_r of neuron r of an affine/conv
 * layer, written over the previous layer. */
static double neuron_expr(const dpo_layer* L, int r, double* coeff)
{
    for (int p = 0; p < L->n_in; ++p) coeff[p] = 0.0;
    if (L->kind == DPO_AFFINE) {
        const float* w = L->W + (size_t)r * L->n_in;
        for (int p = 0; p < L->n_in; ++p) coeff[p] = (double)w[p];
        return (double)L->b[r];
    }
    const int wo = r % L->Wo, ho = (r / L->Wo) % L->Ho, co = r / (L->Wo * L->Ho);
    for (int ci = 0; ci < L->Ci; ++ci)
        for (int ky = 0; ky < L->kh; ++ky) {
            const int hi = ho * L->stride - L->pad + ky;
            if (hi < 0 || hi >= L->H) continue;
            for (int kx = 0; kx < L->kw; ++kx) {
                const int wi = wo * L->stride - L->pad + kx;
                if (wi < 0 || wi >= L->Wd) continue;
                coeff[((size_t)ci * L->H + hi) * L->Wd + wi] =
                    (double)L->W[(((size_t)co * L->Ci + ci) * L->kh + ky) * L->kw + kx];
            }
        }
    return (double)L->b[co];
}

/* ---- networks with Add layers: an expression may hold terms of several layers at once ---- */
typedef struct {
    double** c;        /* [nlayers+1]: coefficient vector per layer index */
    int* present;      /* [nlayers+1]: the layer holds terms of the expression */
    double* tmp;       /* one replacement step's result */
} dpo_multi;

static void multi_free(const dpo_state* st, dpo_multi* e)
{
    if (!e) return;
    if (e->c) for (int i = 0; i <= st->nlayers; ++i) free(e->c[i]);
    free(e->c); free(e->present); free(e->tmp); free(e);
}

static dpo_multi* multi_new(const dpo_state* st, int nmax)
{
    dpo_multi* e = (dpo_multi*)calloc(1, sizeof(dpo_multi));
    if (!e) return NULL;
    e->c = (double**)calloc((size_t)st->nlayers + 1, sizeof(double*));
    e->present = (int*)calloc((size_t)st->nlayers + 1, sizeof(int));
    e->tmp = (double*)malloc(sizeof(double) * (size_t)nmax);
    int ok = e->c && e->present && e->tmp;
    for (int i = 0; ok && i <= st->nlayers; ++i) {
        e->c[i] = (double*)calloc((size_t)layer_size(st, i), sizeof(double));
        if (!e->c[i]) ok = 0;
    }
    if (!ok) { multi_free(st, e); return NULL; }
    return e;
}

static void multi_clear(const dpo_state* st, dpo_multi* e)
{
    for (int i = 0; i <= st->nlayers; ++i) {
        if (e->present[i]) memset(e->c[i], 0, sizeof(double) * (size_t)layer_size(st, i));
        e->present[i] = 0;
    }
}

/* e += the expression of neuron r of layer k written over its predecessor(s); returns its constant */
static double multi_neuron_expr(const dpo_state* st, dpo_multi* e, int k, int r)
{
    const dpo_layer* L = &st->layers[k - 1];
    if (L->kind == DPO_ADD) {
        e->c[k - 1][r] += 1.0; e->present[k - 1] = 1;
        e->c[L->skip][r] += 1.0; e->present[L->skip] = 1;
        return 0.0;
    }
    const double c0 = neuron_expr(L, r, e->tmp);
    for (int p = 0; p < L->n_in; ++p) e->c[k - 1][p] += e->tmp[p];
    e->present[k - 1] = 1;
    return c0;
}

/* backsubs_lower / backsubs_upper for an expression with terms on several layers. */
static double backsubs_multi(const dpo_state* st, int bi, int side, double c0, dpo_multi* e, int max_depth,
                             double* sym_c, double* sym_c0)
{
    int depth = 0;
    for (;;) {
        int at = st->nlayers;
        while (at > 0 && !e->present[at]) --at;              /* deepest layer that holds terms */
        if (at == 0 || (max_depth >= 0 && depth >= max_depth)) break;
        const dpo_layer* L = &st->layers[at - 1];
        if (L->kind == DPO_ADD) {
            /* L_i = U_i = eta_i(layer at-1) + eta_i(layer skip) */
            for (int i = 0; i < L->n_out; ++i) {
                e->c[at - 1][i] += e->c[at][i];
                e->c[L->skip][i] += e->c[at][i];
            }
            e->present[at - 1] = 1;
            e->present[L->skip] = 1;
        } else {
            replace_layer(st, bi, at, side, e->c[at], &c0, e->tmp);
            for (int p = 0; p < L->n_in; ++p) e->c[at - 1][p] += e->tmp[p];
            e->present[at - 1] = 1;
        }
        memset(e->c[at], 0, sizeof(double) * (size_t)L->n_out);
        e->present[at] = 0;
        ++depth;
    }
    int only_input = 1;
    for (int i = 1; i <= st->nlayers; ++i) if (e->present[i]) only_input = 0;
    if (sym_c && only_input) {
        memcpy(sym_c, e->c[0], sizeof(double) * (size_t)layer_size(st, 0));
        *sym_c0 = c0;
    }
    double acc = c0;
    for (int i = 0; i <= st->nlayers; ++i)
        if (e->present[i]) acc = simplify(st, bi, i, side, acc, e->c[i]);
    return acc;
}

/*
 * Run DeepPoly over the whole network.
 *   l,u,lam,mu,nu : arrays of nlayers+1 pointers (index 0 = input layer); l[i],u[i]
 *                   are [B, n_i] and written for every i; lam/mu/nu are written
 *                   for ReLU layers only (other entries may be NULL).
 *   label         : [B] or NULL.  With a label, margin [B, nK-1] and verdict [B]
 *                   are written (last layer must be affine).
 *   sym_layer     : layer index (>=1, affine/conv) whose input-level expressions
 *                   are exported (needs full traversal), or -1.
 *                   sym_cl/sym_cu: [B, n_sym, n0]; sym_kl/sym_ku: [B, n_sym].
 *                   nlayers + 1 names the property's rows (with a label): their lower
 *                   expressions go to sym_cl [B, nK-1, n0], sym_kl [B, nK-1].
 * Returns 0 on success, non-zero on malformed input.
 */
int dpo_run(int nlayers, const dpo_layer* layers, int B,
            const float* lo, const float* hi, const int* label,
            double** l, double** u, double** lam, double** mu, double** nu,
            double* margin, int* verdict,
            int sym_layer, double* sym_cl, double* sym_kl, double* sym_cu, double* sym_ku,
            int max_depth, int max_depth_last)
{
    if (nlayers < 1 || B < 0) return 1;
    if (layers[0].kind == DPO_RELU) return 2;
    if (max_depth_last == -2) max_depth_last = max_depth;
    int nmax = layers[0].n_in;
    int has_add = 0;
    for (int i = 0; i < nlayers; ++i) {
        if (i > 0 && layers[i].n_in != layers[i - 1].n_out) return 3;
        if (layers[i].kind == DPO_RELU && layers[i].n_in != layers[i].n_out) return 3;
        if (layers[i].kind == DPO_ADD) {
            /* second operand: an earlier layer (index < i in 0-based layer numbering = layer index <= i) of equal size */
            if (i == 0 || layers[i].n_in != layers[i].n_out || layers[i].skip < 0 || layers[i].skip > i) return 3;
            const int ns = layers[i].skip == 0 ? layers[0].n_in : layers[layers[i].skip - 1].n_out;
            if (ns != layers[i].n_out) return 3;
            has_add = 1;
        }
        if (layers[i].n_out > nmax) nmax = layers[i].n_out;
    }
    if (label && layers[nlayers - 1].kind != DPO_AFFINE) return 4;

    dpo_state st = { nlayers, layers, B, l, u, lam, mu, nu };
    const int n0 = layers[0].n_in;

    /* input layer: the box is the abstract shape of the input neurons */
    for (size_t i = 0; i < (size_t)B * n0; ++i) {
        if (!(lo[i] <= hi[i])) return 5;
        l[0][i] = (double)lo[i];
        u[0][i] = (double)hi[i];
    }

    for (int k = 1; k <= nlayers; ++k) {
        const dpo_layer* L = &layers[k - 1];
        const int n = L->n_out;
        if (L->kind == DPO_RELU) {
            for (int bi = 0; bi < B; ++bi)
                for (int i = 0; i < n; ++i) {
                    const size_t o = (size_t)bi * n + i;
                    const double pl = l[k - 1][o], pu = u[k - 1][o];
                    l[k][o] = pl >= 0.0 ? pl : 0.0;                 /* relu(prev[l]) */
                    u[k][o] = pu >= 0.0 ? pu : 0.0;                 /* relu(prev[u]) */
                    lam[k][o] = (pl + pu >= 0.0) ? 1.0 : 0.0;       /* relu_n        */
                    if (pl >= 0.0)      { mu[k][o] = 1.0; nu[k][o] = 0.0; }   /* compute_upper */
                    else if (pu <= 0.0) { mu[k][o] = 0.0; nu[k][o] = 0.0; }
                    else { mu[k][o] = pu / (pu - pl); nu[k][o] = -(pu * pl) / (pu - pl); }
                }
            continue;
        }
        const int want_sym = (sym_layer == k);
        const int depth_k = (k == nlayers) ? max_depth_last : max_depth;
        int fail = 0;
        #pragma omp parallel
        {
            double* buf_a = (double*)malloc(sizeof(double) * (size_t)nmax);
            double* buf_b = (double*)malloc(sizeof(double) * (size_t)nmax);
            dpo_multi* e = has_add ? multi_new(&st, nmax) : NULL;
            if (!buf_a || !buf_b || (has_add && !e)) {
                #pragma omp atomic write
                fail = 1;
            }
            #pragma omp for collapse(2) schedule(dynamic, 8)
            for (int bi = 0; bi < B; ++bi)
                for (int r = 0; r < n; ++r) {
                    if (!buf_a || !buf_b || (has_add && !e)) continue;
                    const size_t o = (size_t)bi * n + r;
                    if (has_add) {
                        for (int side = DPO_LOWER; side <= DPO_UPPER; ++side) {
                            multi_clear(&st, e);
                            const double k0 = multi_neuron_expr(&st, e, k, r);
                            const double v = backsubs_multi(&st, bi, side, k0, e, depth_k,
                                                            want_sym ? (side == DPO_LOWER ? sym_cl : sym_cu) + o * n0 : NULL,
                                                            want_sym ? (side == DPO_LOWER ? sym_kl : sym_ku) + o : NULL);
                            if (side == DPO_LOWER) l[k][o] = v; else u[k][o] = v;
                        }
                        continue;
                    }
                    double c0 = neuron_expr(L, r, buf_a);
                    l[k][o] = backsubs(&st, bi, k - 1, DPO_LOWER, c0, buf_a, buf_b, depth_k,
                                       want_sym ? sym_cl + o * n0 : NULL, want_sym ? sym_kl + o : NULL);
                    c0 = neuron_expr(L, r, buf_a);
                    u[k][o] = backsubs(&st, bi, k - 1, DPO_UPPER, c0, buf_a, buf_b, depth_k,
                                       want_sym ? sym_cu + o * n0 : NULL, want_sym ? sym_ku + o : NULL);
                }
            free(buf_a);
            free(buf_b);
            multi_free(&st, e);
        }
        if (fail) return 6;
    }

    if (label) {
        const dpo_layer* L = &layers[nlayers - 1];
        const int nK = L->n_out, nP = L->n_in;
        for (int bi = 0; bi < B; ++bi)
            if (label[bi] < 0 || label[bi] >= nK) return 7;
        int fail = 0;
        #pragma omp parallel
        {
            double* buf_a = (double*)malloc(sizeof(double) * (size_t)nmax);
            double* buf_b = (double*)malloc(sizeof(double) * (size_t)nmax);
            if (!buf_a || !buf_b) {
                #pragma omp atomic write
                fail = 1;
            }
            dpo_multi* e = has_add ? multi_new(&st, nmax) : NULL;
            if (has_add && !e) {
                #pragma omp atomic write
                fail = 1;
            }
            #pragma omp for collapse(2) schedule(dynamic, 1)
            for (int bi = 0; bi < B; ++bi)
                for (int q = 0; q < nK - 1; ++q) {
                    if (!buf_a || !buf_b || (has_add && !e)) continue;
                    const int t = label[bi];
                    const int o = q < t ? q : q + 1;
                    const int want_msym = (sym_layer == nlayers + 1);
                    const size_t mo = (size_t)bi * (nK - 1) + q;
                    /* logit[t] - logit[o] as a polyhedral expression over the last hidden layer */
                    for (int p = 0; p < nP; ++p)
                        buf_a[p] = (double)L->W[(size_t)t * nP + p] - (double)L->W[(size_t)o * nP + p];
                    const double c0 = (double)L->b[t] - (double)L->b[o];
                    if (has_add) {
                        multi_clear(&st, e);
                        memcpy(e->c[nlayers - 1], buf_a, sizeof(double) * (size_t)nP);
                        e->present[nlayers - 1] = 1;
                        margin[(size_t)bi * (nK - 1) + q] = backsubs_multi(&st, bi, DPO_LOWER, c0, e, max_depth_last,
                                                                           want_msym ? sym_cl + mo * n0 : NULL, want_msym ? sym_kl + mo : NULL);
                        continue;
                    }
                    margin[(size_t)bi * (nK - 1) + q] =
                        backsubs(&st, bi, nlayers - 1, DPO_LOWER, c0, buf_a, buf_b, max_depth_last,
                                 want_msym ? sym_cl + mo * n0 : NULL, want_msym ? sym_kl + mo : NULL);
                }
            free(buf_a);
            free(buf_b);
            multi_free(&st, e);
        }
        if (fail) return 6;
        for (int bi = 0; bi < B; ++bi) {
            int ok = 1;
            for (int q = 0; q < nK - 1; ++q)
                if (!(margin[(size_t)bi * (nK - 1) + q] > 0.0)) ok = 0;
            verdict[bi] = ok;
        }
    }
    return 0;
}

/*
 * ReuseCert (Appendix C, "ReuseCert"; Section 6.1): DeepPoly that keeps, for every affine layer, the
 * polyhedral bounds already back-substituted to the input layer and reuses them, so that every later
 * traversal is a single replacement step.
 *   - first affine layer (curr[layer] == 1): L = U = prev.dot(w) + b, which is over the input layer; l, u by
 *     simplify_* against the box;
 *   - ReLU layer over an affine neuron p: (l, u) = (p[L].map(simplify_lower), p[U].map(simplify_upper)), the
 *     concretisation of p's stored input-level bounds; L = relu_n(l, u, p) = (l + u >= 0) ? p[L] : 0 and
 *     U = compute_upper(l, u, p) = l >= 0 ? p[U] : u <= 0 ? 0 : u/(u-l) * p[U] - u*l/(u-l): both are again
 *     input-level expressions.  The transformer leaves the ReLU neuron's own l, u at 0;
 *   - any later affine layer: backsubs_*_L/U = traverse with stop_traverse(n) = (n[layer] <= 1): the terms on
 *     the ReLU layer below are replaced by c >= 0 ? c*L : c*U (mirrored for the upper side), which lands on
 *     the input layer at once, where the traversal stops.  Middle layers store the result as L, U (their l, u
 *     stay 0 in the specification); the last layer also maps simplify_* over it to get l, u;
 *   - property check as for DeepPoly: logit[label] - logit[o] is lower-bounded with backsubs_lower.
 * Outputs: l[k], u[k] of an affine layer k are the concretisations of its stored L, U (the values the next
 * ReLU transformer uses; for the first and last layer these are the specification's l, u); entries of ReLU
 * layers are left at 0 as in the specification.  sym_layer exports the stored L, U of one affine layer.
 * Supported topology: affine (or convolution) and ReLU layers strictly alternating, affine first and last.
 * Returns 0 on success, 8 when the topology is not covered.
 */
int dpo_run_reuse(int nlayers, const dpo_layer* layers, int B,
                  const float* lo, const float* hi, const int* label,
                  double** l, double** u, double** lam, double** mu, double** nu,
                  double* margin, int* verdict,
                  int sym_layer, double* sym_cl, double* sym_kl, double* sym_cu, double* sym_ku)
{
    if (nlayers < 1 || B < 0) return 1;
    int nmax = 1;
    for (int i = 0; i < nlayers; ++i) {
        const int want_relu = (i % 2 == 1);
        if ((layers[i].kind == DPO_RELU) != want_relu) return 8;
        if (i > 0 && layers[i].n_in != layers[i - 1].n_out) return 3;
        if (layers[i].kind == DPO_RELU && layers[i].n_in != layers[i].n_out) return 3;
        if (layers[i].n_out > nmax) nmax = layers[i].n_out;
    }
    if (layers[nlayers - 1].kind == DPO_RELU) return 8;
    if (label && layers[nlayers - 1].kind != DPO_AFFINE) return 4;
    const int n0 = layers[0].n_in;
    const size_t w = (size_t)n0 + 1;                   /* coefficients over the inputs, then the constant */
    for (size_t i = 0; i < (size_t)B * n0; ++i) {
        if (!(lo[i] <= hi[i])) return 5;
        l[0][i] = (double)lo[i];
        u[0][i] = (double)hi[i];
    }
    if (label)
        for (int bi = 0; bi < B; ++bi)
            if (label[bi] < 0 || label[bi] >= layers[nlayers - 1].n_out) return 7;

    /* stored input-level bounds of the current affine layer (EL, EU), and the ReLU layer's L, U built
     * from them (RL, RU): [n, n0 + 1] each */
    double* EL = (double*)malloc(sizeof(double) * nmax * w);
    double* EU = (double*)malloc(sizeof(double) * nmax * w);
    double* RL = (double*)malloc(sizeof(double) * nmax * w);
    double* RU = (double*)malloc(sizeof(double) * nmax * w);
    if (!EL || !EU || !RL || !RU) { free(EL); free(EU); free(RL); free(RU); return 6; }

    int rc = 0;
    for (int bi = 0; bi < B && rc == 0; ++bi) {
        const double* bl = l[0] + (size_t)bi * n0;
        const double* bu = u[0] + (size_t)bi * n0;
        for (int k = 1; k <= nlayers; ++k) {
            const dpo_layer* L = &layers[k - 1];
            const int n = L->n_out;
            if (L->kind == DPO_RELU) {
                /* (l, u) of the predecessor were written when its stored bounds were concretised */
                for (int i = 0; i < n; ++i) {
                    const size_t o = (size_t)bi * n + i;
                    const double pl = l[k - 1][o], pu = u[k - 1][o];
                    l[k][o] = 0.0;
                    u[k][o] = 0.0;
                    lam[k][o] = (pl + pu >= 0.0) ? 1.0 : 0.0;
                    if (pl >= 0.0)      { mu[k][o] = 1.0; nu[k][o] = 0.0; }
                    else if (pu <= 0.0) { mu[k][o] = 0.0; nu[k][o] = 0.0; }
                    else { mu[k][o] = pu / (pu - pl); nu[k][o] = -(pu * pl) / (pu - pl); }
                    for (size_t c = 0; c < w; ++c) {
                        RL[i * w + c] = lam[k][o] * EL[i * w + c];
                        RU[i * w + c] = mu[k][o] * EU[i * w + c];
                    }
                    RU[i * w + n0] += nu[k][o];
                }
                continue;
            }
            /* affine / convolution layer: new stored bounds, one row per neuron */
            double* NL = (k == 1) ? EL : (double*)malloc(sizeof(double) * (size_t)n * w);
            double* NU = (k == 1) ? EU : (double*)malloc(sizeof(double) * (size_t)n * w);
            if (!NL || !NU) { rc = 6; if (k != 1) { free(NL); free(NU); } break; }
            const int nrows = n + ((k == nlayers && label) ? L->n_out - 1 : 0);   /* margin rows ride along */
            #pragma omp parallel
            {
                double* coef = (double*)malloc(sizeof(double) * (size_t)L->n_in);
                double* el = (double*)malloc(sizeof(double) * w);
                #pragma omp for schedule(dynamic, 4)
                for (int r = 0; r < nrows; ++r) {
                    if (!coef || !el) continue;
                    double c0;
                    if (r < n) {
                        c0 = neuron_expr(L, r, coef);
                    } else {
                        const int q = r - n, t = label[bi], o = q < t ? q : q + 1;
                        for (int p = 0; p < L->n_in; ++p)
                            coef[p] = (double)L->W[(size_t)t * L->n_in + p] - (double)L->W[(size_t)o * L->n_in + p];
                        c0 = (double)L->b[t] - (double)L->b[o];
                    }
                    for (int side = 0; side < 2; ++side) {
                        if (r >= n && side == DPO_UPPER) break;
                        double* dst = r < n ? (side == DPO_LOWER ? NL : NU) + (size_t)r * w : el;
                        if (k == 1) {
                            for (int p = 0; p < n0; ++p) dst[p] = coef[p];
                            dst[n0] = c0;
                        } else {
                            for (size_t c = 0; c < w; ++c) dst[c] = 0.0;
                            dst[n0] = c0;
                            for (int j = 0; j < L->n_in; ++j) {
                                const double cj = coef[j];
                                if (cj == 0.0) continue;
                                const int use_L = (side == DPO_LOWER) ? (cj >= 0.0) : !(cj >= 0.0);
                                const double* src = (use_L ? RL : RU) + (size_t)j * w;
                                for (size_t c = 0; c < w; ++c) dst[c] += cj * src[c];
                            }
                        }
                        /* map(simplify_*) over the input-level expression */
                        double acc = dst[n0];
                        for (int p = 0; p < n0; ++p) {
                            const double cp = dst[p];
                            if (side == DPO_LOWER) acc += (cp >= 0.0) ? cp * bl[p] : cp * bu[p];
                            else                   acc += (cp >= 0.0) ? cp * bu[p] : cp * bl[p];
                        }
                        if (r < n) (side == DPO_LOWER ? l[k] : u[k])[(size_t)bi * n + r] = acc;
                        else margin[(size_t)bi * (L->n_out - 1) + (r - n)] = acc;
                    }
                }
                free(coef);
                free(el);
            }
            if (sym_layer == k) {
                for (int r = 0; r < n; ++r) {
                    const size_t o = (size_t)bi * n + r;
                    memcpy(sym_cl + o * n0, NL + (size_t)r * w, sizeof(double) * n0);
                    memcpy(sym_cu + o * n0, NU + (size_t)r * w, sizeof(double) * n0);
                    sym_kl[o] = NL[(size_t)r * w + n0];
                    sym_ku[o] = NU[(size_t)r * w + n0];
                }
            }
            if (k != 1) {
                memcpy(EL, NL, sizeof(double) * (size_t)n * w);
                memcpy(EU, NU, sizeof(double) * (size_t)n * w);
                free(NL);
                free(NU);
            }
        }
        if (rc == 0 && label) {
            const int nq = layers[nlayers - 1].n_out - 1;
            int ok = 1;
            for (int q = 0; q < nq; ++q)
                if (!(margin[(size_t)bi * nq + q] > 0.0)) ok = 0;
            verdict[bi] = ok;
        }
    }
    free(EL); free(EU); free(RL); free(RU);
    return rc;
}

int dpo_layer_struct_size(void) { return (int)sizeof(dpo_layer); }
