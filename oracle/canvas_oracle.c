/*
 * canvas_oracle.c -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A plain, slow, fp64 CPU interpreter of micro-DAG kernels built from the
 * fine-grained primitives of "Canvas: End-to-End Kernel Architecture Search"
 * (Section 5, Table "Three classes of fine-grained primitives").  It exists
 * only so that tests, the smoke check and the benchmark's CPU-baseline leg can
 * compare the GPU library against the primitive definitions written out
 * directly.  It shares no code, header, table or helper with the GPU library
 * and must never be called from the product path.
 *
 * Every tensor is fully materialised per image as [C, T, H, W] (T = number of
 * unfolded taps, 1 when none), every primitive is its definition as a loop
 * nest, every backward rule is the exact vector-Jacobian product of that
 * definition.  Images of a batch are independent (the paper's shapes are
 * per-image, Section 4); only the FC weight gradients sum over the batch.
 * The only parallelism is an OpenMP loop over the batch index.
 *
 * Tie margin (a device of the comparison rule, not of the method): the backward
 * rules decide at kinks (relu, abs, the clip bounds, min / max, the arg-max of a
 * max fold) and fp32 kernels resolve near-ties differently from fp64.  With
 * canvas_oracle_set_tie_margin(m), m != 0, those decisions move by |m| times the
 * largest magnitude of the deciding tensor (per image): m < 0 and m > 0 bracket
 * the default m = 0, which is the definition itself (first maximum, relu'(0) = 0,
 * sign(0) = 0, ties of min / max to the LHS) and the only setting the pins use.
 * A rule selects which decisions move: 0 all, 1 / 2 those at even / odd flat
 * element index (so that of two near-ties that feed one output element the
 * bracketing runs also cover "one moved, the other not"), 3 all, and a max fold
 * takes the runner-up inside the margin instead of the first / last one.
 * The forward pass never depends on it.
 *
 * Decisions of the backward pass (which operand of a max was the larger, the
 * sign at a relu) are taken on the operands rounded to fp32, the precision in
 * which the kernels decide: fp64 rounding noise then cannot order what is an
 * exact tie mathematically and in fp32 (e.g. the zero-padded taps of a max fold
 * downstream of a softmax), and the first-maximum rule applies to it instead.
 * Values are never rounded.
 *
 * Parity pins (see tests/test_oracle_*.py): brute-force direct (grouped)
 * convolution and its gradients, adjoint dot-product identities, central
 * finite differences, closed forms and invariants.  No function here is
 * "parity unpinned".
 *
 * Serialized DAG ("blob"), UTF-8 text, one node per line, topological order:
 *     canvas-dag 1
 *     %1 = unfold %0 kh=3 kw=3
 *     %2 = fc %1 groups=8 out=64
 *     %3 = unary %2 op=gelu            (relu | abs | gelu | sin | expclip lo=.. hi=..)
 *     %4 = shift %3 dh=0 dw=1 c0=32 c1=64
 *     %5 = binary %0 %4 op=mul         (first operand LHS, second RHS; add | sub | mul | min | max;
 *                                       sub is tile(LHS) - RHS; a tie of min / max sends the gradient to the LHS)
 *     %6 = fold %5 op=avg              (sum | avg | max; axis=T (default) folds the taps; axis=HW folds the
 *                                       pixels, axis=H / axis=W one spatial dim: the result is a [C, T, 1, 1],
 *                                       [C, T, 1, W] or [C, T, H, 1] tensor, which FC, unary, softmax, the
 *                                       other folds and binary accept; as the LHS of a binary it is
 *                                       replicated along its folded dims onto an RHS that has them; axis=C groups=G folds the
 *                                       C/G channels of each of G groups: the result has G channels)
 *     %7 = softmax %6 axis=C           (C | T | CT: over channels, over taps, or over both jointly; H | W | HW: over one
 *                                       spatial dim or over both jointly, of every (channel, tap) plane: the table of
 *                                       primitives allows Softmax at any continuous dims)
 *     %9 = binary %a %b op=mul lhs=pixels   (a pooled LHS [H*W, 1, 1, 1] whose channels are laid over the
 *                                       pixels of a full-size RHS: out(c,t,h,w) = op(LHS(h*W+w), RHS(c,t,h,w));
 *                                       Section 8's kernel that pools to [C], maps to H x W with an FC and
 *                                       multiplies the input with the result)
 *     %8 = group %7 groups=4           (the Group primitive as a node of its own: the same data seen as
 *                                       [G, C/G, T, H, W]; groups=C makes every channel a group.  The view
 *                                       travels through unfold, shift, unary, softmax, fold over T / HW and
 *                                       through an fc, whose `groups=` may then be left out (it contracts per
 *                                       group and its output is [G, out/G]); a binary result has the view of
 *                                       its RHS; when both operands of a binary have the same view, G is a
 *                                       common leading dim and the LHS is replicated inside each group)
 *     output %8
 * %0 is the input [N, C, H, W].
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define MAX_NODES 64

enum { OP_INPUT = 0, OP_UNFOLD, OP_SHIFT, OP_FC, OP_UNARY, OP_BINARY, OP_SOFTMAX, OP_FOLD, OP_GROUP };
enum { UN_RELU = 0, UN_ABS, UN_GELU, UN_EXPCLIP, UN_SIN };
enum { BIN_ADD = 0, BIN_MUL, BIN_SUB, BIN_MIN, BIN_MAX };
enum { AXIS_C = 0, AXIS_T, AXIS_CT, AXIS_H, AXIS_W, AXIS_HW };
enum { FOLD_SUM = 0, FOLD_AVG, FOLD_MAX };

typedef struct {
    int op;
    int a, b;           /* operand node ids (binary: a = LHS, b = RHS) */
    int kh, kw;         /* unfold */
    int dh, dw, c0, c1; /* shift */
    int groups, out;    /* fc */
    int kind;           /* unary / binary / fold kind, softmax axis */
    double lo, hi;      /* expclip */
    int C, T;           /* inferred shape [C, T, H, W] */
    int pooled;         /* mask of folded spatial dims: 1 = H (shape [C, T, 1, W]), 2 = W ([C, T, H, 1]), 3 = both */
    int axis_hw;        /* fold: mask of the spatial dims folded by this node (1 = H, 2 = W, 3 = both), 0 = over the taps */
    int axis_c;         /* fold: 1 = over the C / groups channels of each of `groups` channel groups */
    int widx;           /* fc: index into the weight list */
    int grp;            /* Group view of the channel dim: [grp, C/grp]; 1 = not grouped */
    int lhs_pixels;     /* binary: the pooled LHS's H*W channels are laid over the pixels of the RHS */
} Node;

typedef struct {
    int n_nodes;        /* including node 0 (the input) */
    int out;            /* output node id */
    int n_weights;
    int H, W;
    Node node[MAX_NODES];
} Dag;

/* 0 = the definitions; see "Tie margin" above.  Set before a run, read-only during it. */
static double g_tie_margin = 0.0;
static int g_tie_rule = 0;
void canvas_oracle_set_tie_margin(double m) { g_tie_margin = m; }
void canvas_oracle_set_tie_rule(int r) { g_tie_rule = r; }
/* does the margin apply to the decision at flat element index j? */
static int tie_applies(size_t j) { return g_tie_rule == 1 ? (j & 1) == 0 : (g_tie_rule == 2 ? (j & 1) == 1 : 1); }

static double max_abs(const double *v, size_t n) {
    double s = 0.0;
    size_t j;
    for (j = 0; j < n; j++)
        if (fabs(v[j]) > s) s = fabs(v[j]);
    return s;
}

static void set_err(char *err, size_t errlen, const char *msg, int line) {
    if (err && errlen) snprintf(err, errlen, "line %d: %s", line, msg);
}

/* ---------------------------------------------------------------- parsing */

static int parse_ref(const char *tok, int *id) {
    char *end;
    long v;
    if (tok[0] != '%') return 0;
    v = strtol(tok + 1, &end, 10);
    if (end == tok + 1 || *end) return 0;
    *id = (int)v;
    return 1;
}

static const char *find_attr(char **tok, int ntok, const char *key) {
    size_t kl = strlen(key);
    int i;
    for (i = 0; i < ntok; i++)
        if (!strncmp(tok[i], key, kl) && tok[i][kl] == '=') return tok[i] + kl + 1;
    return NULL;
}

static int attr_int(char **tok, int ntok, const char *key, int *out) {
    const char *v = find_attr(tok, ntok, key);
    char *end;
    long x;
    if (!v) return 0;
    x = strtol(v, &end, 10);
    if (end == v || *end) return -1;
    *out = (int)x;
    return 1;
}

static int attr_dbl(char **tok, int ntok, const char *key, double *out) {
    const char *v = find_attr(tok, ntok, key);
    char *end;
    double x;
    if (!v) return 0;
    x = strtod(v, &end);
    if (end == v || *end) return -1;
    *out = x;
    return 1;
}

/* Shape rule of the Broadcast primitive (Section 5, "Blending primitives"):
 * the dim lists [C, (T)] of both sides (H, W always common, batch outside) are
 * stripped of a common prefix, then of a common suffix; the product of what is
 * left of the LHS must divide the product of what is left of the RHS.  A tap
 * dim of size 1 is the same as no tap dim.  Returns 1 when legal. */
static int broadcast_legal(int CL, int TL, int CR, int TR) {
    if (CL == CR) return TR % TL == 0;
    return ((long)CR * TR) % ((long)CL * TL) == 0;
}

/* Index map of the Broadcast primitive: which LHS element (cl, tl) is applied
 * to RHS element (c, t).  The LHS is replicated ("tiled") along the flattened
 * non-common dims with its innermost dims aligned to those of the RHS, which is
 * what the Involution example of Section 5 requires ([K*K] onto [C/G, K, K]). */
static void broadcast_index(int CL, int TL, int CR, int TR, int c, int t, int *cl, int *tl) {
    if (CL == CR) {
        *cl = c;
        *tl = t % TL;
    } else {
        long j = ((long)c * TR + t) % ((long)CL * TL);
        *cl = (int)(j / TL);
        *tl = (int)(j % TL);
    }
    (void)CR;
}

/* With the same Group view [G, ./G] on both sides, G is a common prefix of the two dim lists: the rule
 * above applies inside each group, to [CL/G, TL] and [CR/G, TR] (Section 5: [G, x/G, H, W] onto
 * [G, C/G, K_H, H, W] needs x/G | C/G * K_H). */
static int broadcast_legal_g(int G, int CL, int TL, int CR, int TR) { return broadcast_legal(CL / G, TL, CR / G, TR); }

static void broadcast_index_g(int G, int CL, int TL, int CR, int TR, int c, int t, int *cl, int *tl) {
    int g = c / (CR / G);
    broadcast_index(CL / G, TL, CR / G, TR, c % (CR / G), t, cl, tl);
    *cl += g * (CL / G);
}

static int parse_dag(const char *blob, size_t len, int C0, int H, int W, Dag *d, char *err, size_t errlen) {
    char *buf = (char *)malloc(len + 1), *save1 = NULL, *line;
    int lineno = 0, seen_header = 0, seen_output = 0, rc = -1;
    if (!buf) return -1;
    memcpy(buf, blob, len);
    buf[len] = 0;
    memset(d, 0, sizeof *d);
    d->H = H;
    d->W = W;
    d->n_nodes = 1;
    d->node[0].op = OP_INPUT;
    d->node[0].C = C0;
    d->node[0].T = 1;
    d->node[0].grp = 1;
    d->out = -1;
    for (line = strtok_r(buf, "\n", &save1); line; line = strtok_r(NULL, "\n", &save1)) {
        char *tok[32], *save2 = NULL, *t;
        int ntok = 0, id;
        Node *nd;
        lineno++;
        for (t = strtok_r(line, " \t\r", &save2); t && ntok < 32; t = strtok_r(NULL, " \t\r", &save2)) tok[ntok++] = t;
        if (ntok == 0 || tok[0][0] == '#') continue;
        if (!seen_header) {
            if (ntok != 2 || strcmp(tok[0], "canvas-dag") || strcmp(tok[1], "1")) {
                set_err(err, errlen, "missing header 'canvas-dag 1'", lineno);
                goto done;
            }
            seen_header = 1;
            continue;
        }
        if (seen_output) { set_err(err, errlen, "text after output", lineno); goto done; }
        if (!strcmp(tok[0], "output")) {
            if (ntok != 2 || !parse_ref(tok[1], &id) || id < 0 || id >= d->n_nodes) {
                set_err(err, errlen, "bad output", lineno);
                goto done;
            }
            d->out = id;
            seen_output = 1;
            continue;
        }
        if (ntok < 4 || !parse_ref(tok[0], &id) || strcmp(tok[1], "=")) {
            set_err(err, errlen, "expected '%k = op ...'", lineno);
            goto done;
        }
        if (id != d->n_nodes || id >= MAX_NODES) { set_err(err, errlen, "node ids must be 1,2,3,...", lineno); goto done; }
        nd = &d->node[id];
        memset(nd, 0, sizeof *nd);
        nd->widx = -1;
        if (!parse_ref(tok[3], &nd->a) || nd->a < 0 || nd->a >= id) { set_err(err, errlen, "bad operand", lineno); goto done; }
        {
            const Node *A = &d->node[nd->a];
            const char *opn = tok[2];
            nd->pooled = A->pooled;  /* (binary takes the RHS's below) */
            nd->grp = A->grp;        /* (likewise) */
            if ((!strcmp(opn, "unfold") || !strcmp(opn, "shift")) && A->pooled) {
                set_err(err, errlen, "unfold / shift need the spatial dims", lineno);
                goto done;
            }
            if (!strcmp(opn, "unfold")) {
                nd->op = OP_UNFOLD;
                if (attr_int(tok, ntok, "kh", &nd->kh) != 1 || attr_int(tok, ntok, "kw", &nd->kw) != 1 ||
                    nd->kh < 1 || nd->kw < 1 || nd->kh % 2 == 0 || nd->kw % 2 == 0) {
                    set_err(err, errlen, "unfold needs odd kh, kw >= 1", lineno);
                    goto done;
                }
                nd->C = A->C;
                nd->T = A->T * nd->kh * nd->kw;
            } else if (!strcmp(opn, "shift")) {
                nd->op = OP_SHIFT;
                nd->c0 = 0;
                nd->c1 = A->C;
                if (attr_int(tok, ntok, "dh", &nd->dh) != 1 || attr_int(tok, ntok, "dw", &nd->dw) != 1 ||
                    attr_int(tok, ntok, "c0", &nd->c0) < 0 || attr_int(tok, ntok, "c1", &nd->c1) < 0 ||
                    nd->c0 < 0 || nd->c1 > A->C || nd->c0 > nd->c1) {
                    set_err(err, errlen, "bad shift attributes", lineno);
                    goto done;
                }
                nd->C = A->C;
                nd->T = A->T;
            } else if (!strcmp(opn, "group")) {
                nd->op = OP_GROUP;
                if (attr_int(tok, ntok, "groups", &nd->grp) != 1 || nd->grp < 1 || A->C % nd->grp) {
                    set_err(err, errlen, "group needs groups | C", lineno);
                    goto done;
                }
                nd->C = A->C;
                nd->T = A->T;
            } else if (!strcmp(opn, "fc")) {
                int has;
                nd->op = OP_FC;
                nd->groups = A->grp;  /* a grouped operand: per-group FC unless stated otherwise ... */
                has = attr_int(tok, ntok, "groups", &nd->groups);
                if (has < 0 || (has == 1 && A->grp > 1 && nd->groups != A->grp)) {  /* ... and stating otherwise is an error */
                    set_err(err, errlen, "fc groups= contradicts the Group view of its operand", lineno);
                    goto done;
                }
                if (attr_int(tok, ntok, "out", &nd->out) != 1 ||
                    nd->groups < 1 || nd->out < 1 || A->C % nd->groups || nd->out % nd->groups) {
                    set_err(err, errlen, "fc needs groups | C and groups | out", lineno);
                    goto done;
                }
                nd->C = nd->out;
                nd->T = 1;
                nd->widx = d->n_weights++;
            } else if (!strcmp(opn, "unary")) {
                const char *k2 = find_attr(tok, ntok, "op");
                nd->op = OP_UNARY;
                if (!k2) { set_err(err, errlen, "unary needs op=", lineno); goto done; }
                if (!strcmp(k2, "relu")) nd->kind = UN_RELU;
                else if (!strcmp(k2, "abs")) nd->kind = UN_ABS;
                else if (!strcmp(k2, "gelu")) nd->kind = UN_GELU;
                else if (!strcmp(k2, "sin")) nd->kind = UN_SIN;
                else if (!strcmp(k2, "expclip")) {
                    nd->kind = UN_EXPCLIP;
                    if (attr_dbl(tok, ntok, "lo", &nd->lo) != 1 || attr_dbl(tok, ntok, "hi", &nd->hi) != 1 || !(nd->lo < nd->hi)) {
                        set_err(err, errlen, "expclip needs lo < hi", lineno);
                        goto done;
                    }
                } else { set_err(err, errlen, "unknown unary op", lineno); goto done; }
                nd->C = A->C;
                nd->T = A->T;
            } else if (!strcmp(opn, "binary")) {
                const char *k2 = find_attr(tok, ntok, "op");
                const Node *B;
                nd->op = OP_BINARY;
                if (ntok < 5 || !parse_ref(tok[4], &nd->b) || nd->b < 0 || nd->b >= id || !k2) {
                    set_err(err, errlen, "binary needs two operands and op=", lineno);
                    goto done;
                }
                if (!strcmp(k2, "add")) nd->kind = BIN_ADD;
                else if (!strcmp(k2, "mul")) nd->kind = BIN_MUL;
                else if (!strcmp(k2, "sub")) nd->kind = BIN_SUB;
                else if (!strcmp(k2, "min")) nd->kind = BIN_MIN;
                else if (!strcmp(k2, "max")) nd->kind = BIN_MAX;
                else { set_err(err, errlen, "unknown binary op", lineno); goto done; }
                B = &d->node[nd->b];
                {
                    const char *al = find_attr(tok, ntok, "lhs");
                    if (al && strcmp(al, "pixels")) { set_err(err, errlen, "binary lhs= must be pixels", lineno); goto done; }
                    nd->lhs_pixels = al != NULL;
                }
                if (nd->lhs_pixels) {
                    /* the dim lists [X] and [C, T, H, W] share the suffix once X is read as [H, W] */
                    if (A->pooled != 3 || B->pooled || (long)A->C * A->T != (long)H * W) {
                        set_err(err, errlen, "binary lhs=pixels needs a pooled LHS with H*W elements and a full-size RHS", lineno);
                        goto done;
                    }
                } else
                if (!(A->grp == B->grp && A->grp > 1 ? broadcast_legal_g(A->grp, A->C, A->T, B->C, B->T)
                                                     : broadcast_legal(A->C, A->T, B->C, B->T)) ||
                    (A->pooled & B->pooled) != B->pooled) {  /* a dim folded on the RHS must be folded on the LHS */
                    set_err(err, errlen, "broadcast: LHS size does not divide RHS size", lineno);
                    goto done;
                }
                nd->pooled = B->pooled;
                nd->grp = B->grp;
                nd->C = B->C;
                nd->T = B->T;
            } else if (!strcmp(opn, "softmax")) {
                const char *k2 = find_attr(tok, ntok, "axis");
                nd->op = OP_SOFTMAX;
                if (k2 && !strcmp(k2, "C")) nd->kind = AXIS_C;
                else if (k2 && !strcmp(k2, "T")) nd->kind = AXIS_T;
                else if (k2 && !strcmp(k2, "CT")) nd->kind = AXIS_CT;
                else if (k2 && !strcmp(k2, "H")) nd->kind = AXIS_H;
                else if (k2 && !strcmp(k2, "W")) nd->kind = AXIS_W;
                else if (k2 && !strcmp(k2, "HW")) nd->kind = AXIS_HW;
                else { set_err(err, errlen, "softmax needs axis=C|T|CT|H|W|HW", lineno); goto done; }
                nd->C = A->C;
                nd->T = A->T;
            } else if (!strcmp(opn, "fold")) {
                const char *k2 = find_attr(tok, ntok, "op");
                nd->op = OP_FOLD;
                if (k2 && !strcmp(k2, "sum")) nd->kind = FOLD_SUM;
                else if (k2 && !strcmp(k2, "avg")) nd->kind = FOLD_AVG;
                else if (k2 && !strcmp(k2, "max")) nd->kind = FOLD_MAX;
                else { set_err(err, errlen, "fold needs op=sum|avg|max", lineno); goto done; }
                {
                    const char *ax = find_attr(tok, ntok, "axis");
                    if (ax && !strcmp(ax, "HW")) nd->axis_hw = 3;
                    else if (ax && !strcmp(ax, "H")) nd->axis_hw = 1;
                    else if (ax && !strcmp(ax, "W")) nd->axis_hw = 2;
                    else if (ax && !strcmp(ax, "C")) nd->axis_c = 1;
                    else if (ax && strcmp(ax, "T")) { set_err(err, errlen, "fold axis must be T, H, W, HW or C", lineno); goto done; }
                }
                nd->C = A->C;
                if (nd->axis_c) {
                    nd->groups = 1;
                    if (attr_int(tok, ntok, "groups", &nd->groups) < 0 || nd->groups < 1 || A->C % nd->groups) {
                        set_err(err, errlen, "fold axis=C: groups must divide the channels", lineno);
                        goto done;
                    }
                    nd->C = nd->groups;
                    nd->T = A->T;
                    nd->grp = 1;
                } else if (nd->axis_hw) {
                    if (A->pooled & nd->axis_hw) { set_err(err, errlen, "fold: that spatial dim is already folded", lineno); goto done; }
                    nd->T = A->T;
                    nd->pooled = A->pooled | nd->axis_hw;
                } else {
                    nd->T = 1;
                }
            } else {
                set_err(err, errlen, "unknown op", lineno);
                goto done;
            }
        }
        d->n_nodes++;
    }
    if (!seen_header) { set_err(err, errlen, "empty blob", lineno); goto done; }
    if (d->out < 0) { set_err(err, errlen, "missing output", lineno); goto done; }
    rc = 0;
done:
    free(buf);
    return rc;
}

/* ------------------------------------------------------- forward, one image */

/* pooled is a mask of the spatial dims that have been folded away: 1 = H, 2 = W, 3 = both */
static int node_H(const Dag *d, const Node *nd) { return (nd->pooled & 1) ? 1 : d->H; }
static int node_W(const Dag *d, const Node *nd) { return (nd->pooled & 2) ? 1 : d->W; }
static int node_P(const Dag *d, const Node *nd) { return node_H(d, nd) * node_W(d, nd); }
static size_t node_numel(const Dag *d, int k) { return (size_t)d->node[k].C * d->node[k].T * node_P(d, &d->node[k]); }

/* Unfold (Section 5): U(c, kh, kw, h, w) = I(c, h + kh, w + kw) with the window
 * centred on the pixel (kh, kw run over [-K/2, K/2]) and zeros outside the
 * image, the reading under which Unfold followed by FC is a same-size
 * convolution.  New taps are the innermost channel dim: t = t_in*KH*KW + kh*KW + kw. */
static void fwd_unfold(const Dag *d, const Node *nd, const double *in, double *out) {
    const Node *A = &d->node[nd->a];
    int H = d->H, W = d->W, K = nd->kh * nd->kw;
    int c, ti, kh, kw, h, w;
    for (c = 0; c < A->C; c++)
        for (ti = 0; ti < A->T; ti++)
            for (kh = 0; kh < nd->kh; kh++)
                for (kw = 0; kw < nd->kw; kw++) {
                    int t = ti * K + kh * nd->kw + kw;
                    for (h = 0; h < H; h++)
                        for (w = 0; w < W; w++) {
                            int hs = h + kh - nd->kh / 2, ws = w + kw - nd->kw / 2;
                            double v = 0.0;
                            if (hs >= 0 && hs < H && ws >= 0 && ws < W) v = in[(((size_t)c * A->T + ti) * H + hs) * W + ws];
                            out[(((size_t)c * nd->T + t) * H + h) * W + w] = v;
                        }
                }
}

/* Shift (Section 5): S(c, h, w) = I(c, h + dh, w + dw) on channels [c0, c1),
 * zeros where the source pixel is outside; other channels pass through. */
static void fwd_shift(const Dag *d, const Node *nd, const double *in, double *out) {
    int H = d->H, W = d->W, c, t, h, w;
    for (c = 0; c < nd->C; c++)
        for (t = 0; t < nd->T; t++)
            for (h = 0; h < H; h++)
                for (w = 0; w < W; w++) {
                    size_t base = ((size_t)c * nd->T + t) * H;
                    double v;
                    if (c >= nd->c0 && c < nd->c1) {
                        int hs = h + nd->dh, ws = w + nd->dw;
                        v = (hs >= 0 && hs < H && ws >= 0 && ws < W) ? in[(base + hs) * W + ws] : 0.0;
                    } else {
                        v = in[(base + h) * W + w];
                    }
                    out[(base + h) * W + w] = v;
                }
}

/* Fully-connected (Section 5): every channel dim (channels of the group and all
 * taps) is contracted into a new channel dim; groups are kept apart; no bias.
 * y[g*Og + o, p] = sum_{c', t} Wt[g, o, c'*T + t] * x[g*Cg + c', t, p]. */
static void fwd_fc(const Dag *d, const Node *nd, const double *in, const double *wt, double *out) {
    const Node *A = &d->node[nd->a];
    int P = node_P(d, nd), G = nd->groups, Cg = A->C / G, Og = nd->out / G, K = Cg * A->T;
    int g, o, i, p;
    for (g = 0; g < G; g++)
        for (o = 0; o < Og; o++) {
            double *yrow = out + ((size_t)g * Og + o) * P;
            for (p = 0; p < P; p++) yrow[p] = 0.0;
            for (i = 0; i < K; i++) {
                double wv = wt[((size_t)g * Og + o) * K + i];
                const double *xrow = in + ((size_t)g * K + i) * P; /* (g*Cg + c')*T + t == g*K + i */
                for (p = 0; p < P; p++) yrow[p] += wv * xrow[p];
            }
        }
}

static double gelu_cdf(double x) { return 0.5 * (1.0 + erf(x * 0.70710678118654752440)); }
static double gelu_pdf(double x) { return 0.39894228040143267794 * exp(-0.5 * x * x); }

static void fwd_unary(const Dag *d, const Node *nd, int k, const double *in, double *out) {
    size_t n = node_numel(d, k), j;
    for (j = 0; j < n; j++) {
        double x = in[j], y = 0.0;
        switch (nd->kind) {
        case UN_RELU: y = x > 0.0 ? x : 0.0; break;
        case UN_ABS: y = fabs(x); break;
        case UN_GELU: y = x * gelu_cdf(x); break;
        case UN_EXPCLIP: y = exp(x < nd->lo ? nd->lo : (x > nd->hi ? nd->hi : x)); break;
        case UN_SIN: y = sin(x); break;
        }
        out[j] = y;
    }
}

/* Pixel of the LHS that meets pixel p of the result: a spatial dim that the LHS has folded away is
 * replicated (index 0), the others are common dims. */
static int lhs_pixel(const Dag *d, const Node *L, const Node *R, int p) {
    int Wr = node_W(d, R), h = p / Wr, w = p % Wr;
    return ((L->pooled & 1) ? 0 : h) * node_W(d, L) + ((L->pooled & 2) ? 0 : w);
}

static double blend(int kind, double a, double b) {
    switch (kind) {
    case BIN_ADD: return a + b;
    case BIN_MUL: return a * b;
    case BIN_SUB: return a - b;
    case BIN_MIN: return a <= b ? a : b;
    default: return a >= b ? a : b;
    }
}

static void fwd_binary(const Dag *d, const Node *nd, const double *lhs, const double *rhs, double *out) {
    const Node *L = &d->node[nd->a];
    int P = node_P(d, nd), PL = node_P(d, L), c, t, p, cl, tl;  /* PL < P: the LHS is replicated along its folded spatial dims */
    for (c = 0; c < nd->C; c++)
        for (t = 0; t < nd->T; t++) {
            const double *lrow, *rrow = rhs + ((size_t)c * nd->T + t) * P;
            double *orow = out + ((size_t)c * nd->T + t) * P;
            if (nd->lhs_pixels) {  /* LHS element p meets pixel p of every channel and tap */
                for (p = 0; p < P; p++) orow[p] = blend(nd->kind, lhs[p], rrow[p]);
                continue;
            }
            if (L->grp == nd->grp && nd->grp > 1) broadcast_index_g(nd->grp, L->C, L->T, nd->C, nd->T, c, t, &cl, &tl);
            else broadcast_index(L->C, L->T, nd->C, nd->T, c, t, &cl, &tl);
            lrow = lhs + ((size_t)cl * L->T + tl) * PL;
            for (p = 0; p < P; p++) {
                orow[p] = blend(nd->kind, lrow[lhs_pixel(d, L, nd, p)], rrow[p]);
            }
        }
}

/* Softmax along channels, along taps, or along both jointly (the [C, T] block is contiguous), every other index fixed. */
static void fwd_softmax(const Dag *d, const Node *nd, const double *in, double *out) {
    int P = node_P(d, nd), C = nd->C, T = nd->T;
    if (nd->kind >= AXIS_H) {  /* along H, along W or along both, of every (channel, tap) plane */
        int Hn = node_H(d, nd), Wn = node_W(d, nd), overH = nd->kind != AXIS_W, overW = nd->kind != AXIS_H, c, ho, wo, h, w;
        for (c = 0; c < C * T; c++)
            for (ho = 0; ho < (overH ? 1 : Hn); ho++)
                for (wo = 0; wo < (overW ? 1 : Wn); wo++) {
                    int h0 = overH ? 0 : ho, h1 = overH ? Hn : ho + 1, w0 = overW ? 0 : wo, w1 = overW ? Wn : wo + 1;
                    double m = -INFINITY, sum = 0.0;
                    for (h = h0; h < h1; h++)
                        for (w = w0; w < w1; w++)
                            if (in[((size_t)c * Hn + h) * Wn + w] > m) m = in[((size_t)c * Hn + h) * Wn + w];
                    for (h = h0; h < h1; h++)
                        for (w = w0; w < w1; w++) {
                            size_t idx = ((size_t)c * Hn + h) * Wn + w;
                            out[idx] = exp(in[idx] - m);
                            sum += out[idx];
                        }
                    for (h = h0; h < h1; h++)
                        for (w = w0; w < w1; w++) out[((size_t)c * Hn + h) * Wn + w] /= sum;
                }
        return;
    }
    int len = nd->kind == AXIS_C ? C : (nd->kind == AXIS_T ? T : C * T), outer = nd->kind == AXIS_C ? T : (nd->kind == AXIS_T ? C : 1);
    int o, p, k;
    for (o = 0; o < outer; o++)
        for (p = 0; p < P; p++) {
            double m = -INFINITY, s = 0.0;
            for (k = 0; k < len; k++) {
                size_t idx = nd->kind == AXIS_C ? ((size_t)k * T + o) * P + p : (nd->kind == AXIS_T ? ((size_t)o * T + k) * P + p : (size_t)k * P + p);
                if (in[idx] > m) m = in[idx];
            }
            for (k = 0; k < len; k++) {
                size_t idx = nd->kind == AXIS_C ? ((size_t)k * T + o) * P + p : (nd->kind == AXIS_T ? ((size_t)o * T + k) * P + p : (size_t)k * P + p);
                out[idx] = exp(in[idx] - m);
                s += out[idx];
            }
            for (k = 0; k < len; k++) {
                size_t idx = nd->kind == AXIS_C ? ((size_t)k * T + o) * P + p : (nd->kind == AXIS_T ? ((size_t)o * T + k) * P + p : (size_t)k * P + p);
                out[idx] /= s;
            }
        }
}

/* Folding: sum, average or max over the tap dim (it disappears) or over the spatial dims (they become 1 x 1). */
static void fwd_fold(const Dag *d, const Node *nd, const double *in, double *out) {
    const Node *A = &d->node[nd->a];
    int P = node_P(d, A), T = A->T, c, t, p;
    if (nd->axis_c) {  /* over the channels of each group: out[g, t, p] from in[g*Cg + c', t, p] */
        int Cg = A->C / nd->groups, g;
        for (g = 0; g < nd->groups; g++)
            for (t = 0; t < T; t++)
                for (p = 0; p < P; p++) {
                    double acc = in[(((size_t)g * Cg) * T + t) * P + p];
                    for (c = 1; c < Cg; c++) {
                        double v = in[(((size_t)g * Cg + c) * T + t) * P + p];
                        if (nd->kind == FOLD_MAX) { if (v > acc) acc = v; }
                        else acc += v;
                    }
                    if (nd->kind == FOLD_AVG) acc /= Cg;
                    out[((size_t)g * T + t) * P + p] = acc;
                }
        return;
    }
    if (nd->axis_hw) {  /* over H, over W or over both, of every (channel, tap) plane; scan order h, then w */
        int Hi = node_H(d, A), Wi = node_W(d, A), Ho = node_H(d, nd), Wo = node_W(d, nd), ho, wo, h, w;
        for (c = 0; c < nd->C * T; c++)
            for (ho = 0; ho < Ho; ho++)
                for (wo = 0; wo < Wo; wo++) {
                    int h0 = (nd->axis_hw & 1) ? 0 : ho, h1 = (nd->axis_hw & 1) ? Hi : ho + 1;
                    int w0 = (nd->axis_hw & 2) ? 0 : wo, w1 = (nd->axis_hw & 2) ? Wi : wo + 1, first = 1;
                    double acc = 0.0;
                    for (h = h0; h < h1; h++)
                        for (w = w0; w < w1; w++) {
                            double v = in[((size_t)c * Hi + h) * Wi + w];
                            if (first) { acc = v; first = 0; }
                            else if (nd->kind == FOLD_MAX) { if (v > acc) acc = v; }
                            else acc += v;
                        }
                    if (nd->kind == FOLD_AVG) acc /= (double)((h1 - h0) * (w1 - w0));
                    out[((size_t)c * Ho + ho) * Wo + wo] = acc;
                }
        return;
    }
    for (c = 0; c < nd->C; c++)
        for (p = 0; p < P; p++) {
            double acc = in[((size_t)c * T) * P + p];
            for (t = 1; t < T; t++) {
                double v = in[((size_t)c * T + t) * P + p];
                if (nd->kind == FOLD_MAX) { if (v > acc) acc = v; }
                else acc += v;
            }
            if (nd->kind == FOLD_AVG) acc /= T;
            out[(size_t)c * P + p] = acc;
        }
}

/* ------------------------------------------------------ backward, one image */
/* Each routine ADDS the contribution of node nd to the gradient(s) of its
 * operand(s); a tensor consumed several times thus receives the sum. */

static void bwd_unfold(const Dag *d, const Node *nd, const double *gout, double *gin) {
    const Node *A = &d->node[nd->a];
    int H = d->H, W = d->W, K = nd->kh * nd->kw;
    int c, ti, kh, kw, h, w;
    for (c = 0; c < A->C; c++)
        for (ti = 0; ti < A->T; ti++)
            for (kh = 0; kh < nd->kh; kh++)
                for (kw = 0; kw < nd->kw; kw++) {
                    int t = ti * K + kh * nd->kw + kw;
                    for (h = 0; h < H; h++)
                        for (w = 0; w < W; w++) {
                            int hs = h + kh - nd->kh / 2, ws = w + kw - nd->kw / 2;
                            if (hs >= 0 && hs < H && ws >= 0 && ws < W)
                                gin[(((size_t)c * A->T + ti) * H + hs) * W + ws] += gout[(((size_t)c * nd->T + t) * H + h) * W + w];
                        }
                }
}

static void bwd_shift(const Dag *d, const Node *nd, const double *gout, double *gin) {
    int H = d->H, W = d->W, c, t, h, w;
    for (c = 0; c < nd->C; c++)
        for (t = 0; t < nd->T; t++)
            for (h = 0; h < H; h++)
                for (w = 0; w < W; w++) {
                    size_t base = ((size_t)c * nd->T + t) * H;
                    if (c >= nd->c0 && c < nd->c1) {
                        int hs = h + nd->dh, ws = w + nd->dw;
                        if (hs >= 0 && hs < H && ws >= 0 && ws < W) gin[(base + hs) * W + ws] += gout[(base + h) * W + w];
                    } else {
                        gin[(base + h) * W + w] += gout[(base + h) * W + w];
                    }
                }
}

static void bwd_fc(const Dag *d, const Node *nd, const double *in, const double *wt, const double *gout, double *gin, double *gw) {
    const Node *A = &d->node[nd->a];
    int P = node_P(d, nd), G = nd->groups, Cg = A->C / G, Og = nd->out / G, K = Cg * A->T;
    int g, o, i, p;
    for (g = 0; g < G; g++)
        for (o = 0; o < Og; o++) {
            const double *grow = gout + ((size_t)g * Og + o) * P;
            for (i = 0; i < K; i++) {
                size_t wi = ((size_t)g * Og + o) * K + i;
                const double *xrow = in + ((size_t)g * K + i) * P;
                double *girow = gin + ((size_t)g * K + i) * P;
                double wv = wt[wi], acc = 0.0;
                for (p = 0; p < P; p++) {
                    girow[p] += wv * grow[p];
                    acc += grow[p] * xrow[p];
                }
                gw[wi] += acc;
            }
        }
}

static void bwd_unary(const Dag *d, const Node *nd, int k, const double *in, const double *out, const double *gout, double *gin) {
    size_t n = node_numel(d, k), j;
    /* e = 0 unless a tie margin is set: then the kink moves by e */
    double e = g_tie_margin != 0.0 ? g_tie_margin * max_abs(in, n) : 0.0;
    for (j = 0; j < n; j++) {
        double x = in[j], dv = 0.0, xd = (double)(float)x;  /* xd: what the decisions look at */
        double ej = (e != 0.0 && tie_applies(j)) ? e : 0.0;
        switch (nd->kind) {
        case UN_RELU: dv = xd > ej ? 1.0 : 0.0; break;
        case UN_ABS: dv = xd > ej ? 1.0 : (xd < ej ? -1.0 : 0.0); break;
        case UN_GELU: dv = gelu_cdf(x) + x * gelu_pdf(x); break;
        case UN_EXPCLIP: dv = (xd > (double)(float)nd->lo + ej && xd < (double)(float)nd->hi - ej) ? out[j] : 0.0; break;
        case UN_SIN: dv = cos(x); break;
        }
        gin[j] += gout[j] * dv;
    }
}

static void bwd_binary(const Dag *d, const Node *nd, const double *lhs, const double *rhs, const double *gout, double *glhs, double *grhs) {
    const Node *L = &d->node[nd->a];
    int P = node_P(d, nd), PL = node_P(d, L), c, t, p, cl, tl;
    double e = 0.0;  /* tie margin of min / max: 0 = the definition (ties to the LHS) */
    if (g_tie_margin != 0.0 && (nd->kind == BIN_MIN || nd->kind == BIN_MAX)) {
        double sl = max_abs(lhs, (size_t)L->C * L->T * PL), sr = max_abs(rhs, (size_t)nd->C * nd->T * P);
        e = g_tie_margin * (sl > sr ? sl : sr);
    }
    for (c = 0; c < nd->C; c++)
        for (t = 0; t < nd->T; t++) {
            size_t ro = ((size_t)c * nd->T + t) * P, lo;
            if (nd->lhs_pixels) { cl = 0; tl = 0; }
            else if (L->grp == nd->grp && nd->grp > 1) broadcast_index_g(nd->grp, L->C, L->T, nd->C, nd->T, c, t, &cl, &tl);
            else broadcast_index(L->C, L->T, nd->C, nd->T, c, t, &cl, &tl);
            lo = ((size_t)cl * L->T + tl) * PL;
            for (p = 0; p < P; p++) {
                size_t lp = nd->lhs_pixels ? (size_t)p : lo + (size_t)lhs_pixel(d, L, nd, p);
                double g = gout[ro + p], a = lhs[lp], b = rhs[ro + p];
                switch (nd->kind) {
                case BIN_ADD: glhs[lp] += g; grhs[ro + p] += g; break;
                case BIN_MUL: glhs[lp] += g * b; grhs[ro + p] += g * a; break;
                case BIN_SUB: glhs[lp] += g; grhs[ro + p] -= g; break;
                case BIN_MIN: if ((double)(float)a <= (double)(float)b + (tie_applies(ro + p) ? e : 0.0)) glhs[lp] += g; else grhs[ro + p] += g; break;
                case BIN_MAX: if ((double)(float)a >= (double)(float)b - (tie_applies(ro + p) ? e : 0.0)) glhs[lp] += g; else grhs[ro + p] += g; break;
                }
            }
        }
}

static void bwd_softmax(const Dag *d, const Node *nd, const double *out, const double *gout, double *gin) {
    int P = node_P(d, nd), C = nd->C, T = nd->T;
    if (nd->kind >= AXIS_H) {
        int Hn = node_H(d, nd), Wn = node_W(d, nd), overH = nd->kind != AXIS_W, overW = nd->kind != AXIS_H, c, ho, wo, h, w;
        for (c = 0; c < C * T; c++)
            for (ho = 0; ho < (overH ? 1 : Hn); ho++)
                for (wo = 0; wo < (overW ? 1 : Wn); wo++) {
                    int h0 = overH ? 0 : ho, h1 = overH ? Hn : ho + 1, w0 = overW ? 0 : wo, w1 = overW ? Wn : wo + 1;
                    double dot = 0.0;
                    for (h = h0; h < h1; h++)
                        for (w = w0; w < w1; w++) dot += gout[((size_t)c * Hn + h) * Wn + w] * out[((size_t)c * Hn + h) * Wn + w];
                    for (h = h0; h < h1; h++)
                        for (w = w0; w < w1; w++) {
                            size_t idx = ((size_t)c * Hn + h) * Wn + w;
                            gin[idx] += out[idx] * (gout[idx] - dot);
                        }
                }
        return;
    }
    int len = nd->kind == AXIS_C ? C : (nd->kind == AXIS_T ? T : C * T), outer = nd->kind == AXIS_C ? T : (nd->kind == AXIS_T ? C : 1);
    int o, p, k;
    for (o = 0; o < outer; o++)
        for (p = 0; p < P; p++) {
            double dot = 0.0;
            for (k = 0; k < len; k++) {
                size_t idx = nd->kind == AXIS_C ? ((size_t)k * T + o) * P + p : (nd->kind == AXIS_T ? ((size_t)o * T + k) * P + p : (size_t)k * P + p);
                dot += gout[idx] * out[idx];
            }
            for (k = 0; k < len; k++) {
                size_t idx = nd->kind == AXIS_C ? ((size_t)k * T + o) * P + p : (nd->kind == AXIS_T ? ((size_t)o * T + k) * P + p : (size_t)k * P + p);
                gin[idx] += out[idx] * (gout[idx] - dot);
            }
        }
}

/* Max takes the gradient to the first maximal tap (lowest t) only.  With a tie margin e != 0 every element
 * within |e| of the maximum counts as maximal, and e < 0 takes the first, e > 0 the last of them. */
#define DEC(v) ((double)(float)(v)) /* the operand as a decision sees it */
static void bwd_fold(const Dag *d, const Node *nd, const double *in, const double *gout, double *gin) {
    const Node *A = &d->node[nd->a];
    int P = node_P(d, A), T = A->T, c, t, p;
    double e = (g_tie_margin != 0.0 && nd->kind == FOLD_MAX) ? g_tie_margin * max_abs(in, (size_t)A->C * T * P) : 0.0;
    if (nd->axis_c) {  /* max: to the first maximal channel of the group only */
        int Cg = A->C / nd->groups, g;
        for (g = 0; g < nd->groups; g++)
            for (t = 0; t < T; t++)
                for (p = 0; p < P; p++) {
                    double gg = gout[((size_t)g * T + t) * P + p];
                    if (nd->kind == FOLD_MAX) {
                        int best = 0;
                        for (c = 1; c < Cg; c++)
                            if (DEC(in[(((size_t)g * Cg + c) * T + t) * P + p]) > DEC(in[(((size_t)g * Cg + best) * T + t) * P + p])) best = c;
                        if (e != 0.0) {
                            double m = DEC(in[(((size_t)g * Cg + best) * T + t) * P + p]) - fabs(e);
                            if (e < 0.0) { for (c = 0; c < Cg; c++) if (DEC(in[(((size_t)g * Cg + c) * T + t) * P + p]) >= m) { best = c; break; } }
                            else { for (c = Cg - 1; c >= 0; c--) if (DEC(in[(((size_t)g * Cg + c) * T + t) * P + p]) >= m) { best = c; break; } }
                        }
                        gin[(((size_t)g * Cg + best) * T + t) * P + p] += gg;
                    } else {
                        if (nd->kind == FOLD_AVG) gg /= Cg;
                        for (c = 0; c < Cg; c++) gin[(((size_t)g * Cg + c) * T + t) * P + p] += gg;
                    }
                }
        return;
    }
    if (nd->axis_hw) {  /* max: to the first maximal pixel in scan order (h, then w) only */
        int Hi = node_H(d, A), Wi = node_W(d, A), Ho = node_H(d, nd), Wo = node_W(d, nd), ho, wo, h, w;
        for (c = 0; c < nd->C * T; c++)
            for (ho = 0; ho < Ho; ho++)
                for (wo = 0; wo < Wo; wo++) {
                    int h0 = (nd->axis_hw & 1) ? 0 : ho, h1 = (nd->axis_hw & 1) ? Hi : ho + 1;
                    int w0 = (nd->axis_hw & 2) ? 0 : wo, w1 = (nd->axis_hw & 2) ? Wi : wo + 1;
                    double g = gout[((size_t)c * Ho + ho) * Wo + wo];
                    if (nd->kind == FOLD_MAX) {
                        size_t best = ((size_t)c * Hi + h0) * Wi + w0;
                        for (h = h0; h < h1; h++)
                            for (w = w0; w < w1; w++)
                                if (DEC(in[((size_t)c * Hi + h) * Wi + w]) > DEC(in[best])) best = ((size_t)c * Hi + h) * Wi + w;
                        if (e != 0.0) {
                            double m = DEC(in[best]) - fabs(e);
                            int found = 0;
                            if (e < 0.0) {
                                for (h = h0; h < h1 && !found; h++)
                                    for (w = w0; w < w1 && !found; w++)
                                        if (DEC(in[((size_t)c * Hi + h) * Wi + w]) >= m) { best = ((size_t)c * Hi + h) * Wi + w; found = 1; }
                            } else {
                                for (h = h1 - 1; h >= h0 && !found; h--)
                                    for (w = w1 - 1; w >= w0 && !found; w--)
                                        if (DEC(in[((size_t)c * Hi + h) * Wi + w]) >= m) { best = ((size_t)c * Hi + h) * Wi + w; found = 1; }
                            }
                        }
                        gin[best] += g;
                    } else {
                        if (nd->kind == FOLD_AVG) g /= (double)((h1 - h0) * (w1 - w0));
                        for (h = h0; h < h1; h++)
                            for (w = w0; w < w1; w++) gin[((size_t)c * Hi + h) * Wi + w] += g;
                    }
                }
        return;
    }
    for (c = 0; c < nd->C; c++)
        for (p = 0; p < P; p++) {
            double g = gout[(size_t)c * P + p];
            if (nd->kind == FOLD_MAX) {
                int best = 0;
                for (t = 1; t < T; t++)
                    if (DEC(in[((size_t)c * T + t) * P + p]) > DEC(in[((size_t)c * T + best) * P + p])) best = t;
                if (e != 0.0 && tie_applies((size_t)c * P + p)) {
                    double m = DEC(in[((size_t)c * T + best) * P + p]) - fabs(e);
                    if (g_tie_rule == 3) {  /* the runner-up, if it is inside the margin */
                        int second = -1;
                        for (t = 0; t < T; t++)
                            if (t != best && (second < 0 || DEC(in[((size_t)c * T + t) * P + p]) > DEC(in[((size_t)c * T + second) * P + p]))) second = t;
                        if (second >= 0 && DEC(in[((size_t)c * T + second) * P + p]) >= m) best = second;
                    }
                    else if (e < 0.0) { for (t = 0; t < T; t++) if (DEC(in[((size_t)c * T + t) * P + p]) >= m) { best = t; break; } }
                    else { for (t = T - 1; t >= 0; t--) if (DEC(in[((size_t)c * T + t) * P + p]) >= m) { best = t; break; } }
                }
                gin[((size_t)c * T + best) * P + p] += g;
            } else {
                if (nd->kind == FOLD_AVG) g /= T;
                for (t = 0; t < T; t++) gin[((size_t)c * T + t) * P + p] += g;
            }
        }
}

/* ------------------------------------------------------------- entry points */

/* Shape inference only.  shapes: n_nodes rows of [C, T, H, W]; wshapes:
 * n_weights rows of [G, C_out/G, (C_in/G)*T].  Returns 0, or -1 with err set. */
int canvas_oracle_infer(const char *blob, size_t len, const int64_t in_shape[4], int max_nodes, int64_t *shapes,
                        int *n_nodes, int *out_node, int max_weights, int64_t *wshapes, int *n_weights, char *err,
                        size_t errlen) {
    Dag d;
    int k;
    if (parse_dag(blob, len, (int)in_shape[1], (int)in_shape[2], (int)in_shape[3], &d, err, errlen)) return -1;
    if (d.n_nodes > max_nodes || d.n_weights > max_weights) { set_err(err, errlen, "too many nodes for caller", 0); return -1; }
    for (k = 0; k < d.n_nodes; k++) {
        shapes[4 * k + 0] = d.node[k].C;
        shapes[4 * k + 1] = d.node[k].T;
        shapes[4 * k + 2] = node_H(&d, &d.node[k]);
        shapes[4 * k + 3] = node_W(&d, &d.node[k]);
        if (d.node[k].op == OP_FC) {
            const Node *A = &d.node[d.node[k].a];
            int wi = d.node[k].widx;
            wshapes[3 * wi + 0] = d.node[k].groups;
            wshapes[3 * wi + 1] = d.node[k].out / d.node[k].groups;
            wshapes[3 * wi + 2] = (int64_t)(A->C / d.node[k].groups) * A->T;
        }
    }
    *n_nodes = d.n_nodes;
    *out_node = d.out;
    *n_weights = d.n_weights;
    return 0;
}

/* Forward (and, when dy != NULL, backward) of the whole batch.
 *   x        [N, C, H, W] fp64, weights[k] [G, Og, K] fp64 in FC-node order
 *   y        [N, C_out, T_out, H, W]; dy same shape; dx like x; dw[k] like weights[k]
 * Returns the number of OpenMP threads used (>= 1), or -1 with err set. */
int canvas_oracle_run(const char *blob, size_t len, const int64_t in_shape[4], const double *x,
                      const double *const *weights, int n_weights, const double *dy, double *y, double *dx,
                      double *const *dw, int n_threads, char *err, size_t errlen) {
    Dag d;
    int N = (int)in_shape[0], k, nthr = 1, n, failed = 0;
    size_t wn[MAX_NODES], xn, yn;
    double **dwacc = NULL;
    if (parse_dag(blob, len, (int)in_shape[1], (int)in_shape[2], (int)in_shape[3], &d, err, errlen)) return -1;
    if (n_weights != d.n_weights) { set_err(err, errlen, "wrong number of weight tensors", 0); return -1; }
    for (k = 0; k < d.n_nodes; k++)
        if (d.node[k].op == OP_FC) {
            const Node *A = &d.node[d.node[k].a];
            wn[d.node[k].widx] = (size_t)d.node[k].out * (A->C / d.node[k].groups) * A->T;
        }
    xn = node_numel(&d, 0);
    yn = node_numel(&d, d.out);
#ifdef _OPENMP
    if (n_threads > 0) omp_set_num_threads(n_threads);
    nthr = omp_get_max_threads();
    if (nthr > N && N > 0) nthr = N;
    if (nthr < 1) nthr = 1;
#endif
    if (dy) {
        int t;
        dwacc = (double **)calloc((size_t)nthr * (d.n_weights + 1), sizeof(double *));
        for (t = 0; t < nthr; t++)
            for (k = 0; k < d.n_weights; k++) dwacc[(size_t)t * d.n_weights + k] = (double *)calloc(wn[k], sizeof(double));
    }
#ifdef _OPENMP
#pragma omp parallel for schedule(static) num_threads(nthr)
#endif
    for (n = 0; n < N; n++) {
        double *val[MAX_NODES], *grad[MAX_NODES];
        int tid = 0, j;
#ifdef _OPENMP
        tid = omp_get_thread_num();
#endif
        memset(val, 0, sizeof val);
        memset(grad, 0, sizeof grad);
        val[0] = (double *)(x + (size_t)n * xn);
        for (j = 1; j < d.n_nodes; j++) {
            const Node *nd = &d.node[j];
            val[j] = (double *)malloc(node_numel(&d, j) * sizeof(double));
            if (!val[j]) { failed = 1; break; }
            switch (nd->op) {
            case OP_UNFOLD: fwd_unfold(&d, nd, val[nd->a], val[j]); break;
            case OP_SHIFT: fwd_shift(&d, nd, val[nd->a], val[j]); break;
            case OP_FC: fwd_fc(&d, nd, val[nd->a], weights[nd->widx], val[j]); break;
            case OP_UNARY: fwd_unary(&d, nd, j, val[nd->a], val[j]); break;
            case OP_BINARY: fwd_binary(&d, nd, val[nd->a], val[nd->b], val[j]); break;
            case OP_SOFTMAX: fwd_softmax(&d, nd, val[nd->a], val[j]); break;
            case OP_FOLD: fwd_fold(&d, nd, val[nd->a], val[j]); break;
            case OP_GROUP: memcpy(val[j], val[nd->a], node_numel(&d, j) * sizeof(double)); break;  /* a view: same data */
            }
        }
        if (!failed) memcpy(y + (size_t)n * yn, val[d.out], yn * sizeof(double));
        if (dy && !failed) {
            for (j = 0; j < d.n_nodes; j++) {
                grad[j] = (double *)calloc(node_numel(&d, j), sizeof(double));
                if (!grad[j]) failed = 1;
            }
            if (!failed) {
                memcpy(grad[d.out], dy + (size_t)n * yn, yn * sizeof(double));
                for (j = d.n_nodes - 1; j >= 1; j--) {
                    const Node *nd = &d.node[j];
                    switch (nd->op) {
                    case OP_UNFOLD: bwd_unfold(&d, nd, grad[j], grad[nd->a]); break;
                    case OP_SHIFT: bwd_shift(&d, nd, grad[j], grad[nd->a]); break;
                    case OP_FC: bwd_fc(&d, nd, val[nd->a], weights[nd->widx], grad[j], grad[nd->a], dwacc[(size_t)tid * d.n_weights + nd->widx]); break;
                    case OP_UNARY: bwd_unary(&d, nd, j, val[nd->a], val[j], grad[j], grad[nd->a]); break;
                    case OP_BINARY: bwd_binary(&d, nd, val[nd->a], val[nd->b], grad[j], grad[nd->a], grad[nd->b]); break;
                    case OP_SOFTMAX: bwd_softmax(&d, nd, val[j], grad[j], grad[nd->a]); break;
                    case OP_FOLD: bwd_fold(&d, nd, val[nd->a], grad[j], grad[nd->a]); break;
                    case OP_GROUP: {
                        size_t i, cnt = node_numel(&d, j);
                        for (i = 0; i < cnt; i++) grad[nd->a][i] += grad[j][i];
                        break;
                    }
                    }
                }
                memcpy(dx + (size_t)n * xn, grad[0], xn * sizeof(double));
            }
            for (j = 0; j < d.n_nodes; j++) free(grad[j]);
        }
        for (j = 1; j < d.n_nodes; j++) free(val[j]);
    }
    if (dy) {
        int t;
        for (k = 0; k < d.n_weights; k++) {
            size_t i;
            for (i = 0; i < wn[k]; i++) dw[k][i] = 0.0;
            for (t = 0; t < nthr; t++) {
                const double *src = dwacc[(size_t)t * d.n_weights + k];
                for (i = 0; i < wn[k]; i++) dw[k][i] += src[i];
                free(dwacc[(size_t)t * d.n_weights + k]);
            }
        }
        free(dwacc);
    }
    if (failed) { set_err(err, errlen, "out of memory", 0); return -1; }
    return nthr;
}
