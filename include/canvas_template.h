/*
 * canvas_template.h -- C ABI for kernel TEMPLATES: micro-DAGs whose sizes are symbols.
 *
 * In "Canvas: End-to-End Kernel Architecture Search" a sampled kernel is a
 * template [C, H, W] => [C, H, W]: every FC output width is a dynamic variable
 * x_j, window sizes and the group number are symbols, and one template
 * replaces many convolutions of a network, each with its own C, K_H, K_W, H,
 * W (Section 6).  This part of the library is host-only (no GPU):
 *
 *   - symbolic shape inference of a template;
 *   - the shape-matching solver (Section 6.2): for a Broadcast whose LHS
 *     carries a dynamic variable, the set of its valid substitutions;
 *   - the candidates of the global group number G (Section 6.3);
 *   - the constraint solver (Section 6.3): base values x_ij = k_ij * lcm_ij
 *     proportional to C_i, then greedy doubling under FLOPs / parameter budgets;
 *   - instantiation: the concrete blob of canvas_dag.h for one target, to be
 *     handed to canvas_dag_compile.
 *
 * Template text: the grammar of canvas_dag.h with the header line
 * "canvas-template 1", where every integer attribute may be a product /
 * quotient of integers and the symbols
 *     C  G  KH  KW  H  W  x1 .. x8          e.g.  out=x1  out=G*KH  groups=G  kh=KH  c0=C/2  out=H*W
 * (no parentheses; `/` divides by the one factor that follows it).
 * C is treated as G * (C/G): the group number divides the channels (Section 6.2).
 *
 * All functions return CANVAS_OK or a negative canvas_status (canvas_dag.h);
 * canvas_last_error() has the message.  Handles are used by one thread at a time.
 * Text results are written to caller-owned host buffers, NUL-terminated; when the
 * buffer is too small the call returns CANVAS_BAD_ARG and *needed (if given)
 * holds the size required.
 */
#ifndef CANVAS_TEMPLATE_H
#define CANVAS_TEMPLATE_H

#include <stddef.h>
#include <stdint.h>

#include "canvas_dag.h"

#ifdef __cplusplus
extern "C" {
#endif

#define CANVAS_MAX_VARS 8

typedef struct canvas_template canvas_template; /* opaque, owned by the library */

/* One replacement target (Section 6.3: "each individual convolution has a specific
 * assignment of C, K_H, K_W, H, W"). */
typedef struct canvas_target {
    int64_t C, KH, KW, H, W;
} canvas_target;

typedef struct canvas_template_info {
    int32_t n_nodes;                 /* including node 0, the input [C, H, W] */
    int32_t out_node;
    int32_t n_fc;
    int32_t n_free;                  /* dynamic variables still free (not substituted) */
    int32_t free_var[CANVAS_MAX_VARS]; /* their numbers j of x_j, ascending */
    int32_t uses_G;                  /* 1 when the symbol G occurs (also through C = G * C/G in a Group view) */
    int32_t reserved[5];
} canvas_template_info;

/* Parse a template and infer its symbolic shapes.  blob: host pointer, not
 * retained.  Errors: INVALID_BLOB, UNKNOWN_OP, SHAPE_MISMATCH (a size that can
 * be no integer for any assignment, a dynamic variable where Theorem 1 of
 * Section 6.2 forbids one), UNSUPPORTED (too many nodes / variables). */
int canvas_template_parse(const void* blob, size_t blob_len, canvas_template** out);

int canvas_template_query(const canvas_template* t, canvas_template_info* info);

/* Symbolic shape of node `node` as text "[C-dims | tap dims | H, W]", e.g.
 * "[G, x2/G | KH, KW | H, W]", "[x1 | H, W]" without taps; a folded spatial dim reads 1 ("| 1, W]", "| 1, 1]"). */
int canvas_template_node_shape(const canvas_template* t, int node, char* buf, size_t buf_len, size_t* needed);

/* Shape-matching solver (Section 6.2).  node: a binary node whose LHS carries a
 * free dynamic variable x_L.  With M = #RHS / #LHS = (x_R^k * R_RHS) / (x_L * R_LHS)
 * fully simplified, the valid substitutions of x_L are the factors of the
 * numerator x_R^k * R_RHS (divided by R_LHS when that divides it; none
 * otherwise).  Writes them as one line of text each ("1", "x2", "KW", "KW*x2",
 * ...; sorted as text) and stores their number in
 * *count; *var receives the number of x_L.  Errors: BAD_ARG (not a binary
 * node, no free variable on its LHS). */
int canvas_template_substitutions(const canvas_template* t, int node, int* var, int* count, char* buf, size_t buf_len,
                                  size_t* needed);

/* Replace x_var by the expression `expr` (same syntax as attributes) in the
 * whole template and infer the shapes again.  Errors: INVALID_BLOB (syntax),
 * BAD_ARG (x_var not free, expr mentions x_var), SHAPE_MISMATCH (as parse;
 * the template is left unchanged then). */
int canvas_template_substitute(canvas_template* t, int var, const char* expr);

/* Candidates of the global group number (Section 6.3): the factors of
 * gcd(C_1 .. C_n) other than 1, ascending.  out: host array of `cap` entries. */
int canvas_group_candidates(const int64_t* C, int n_targets, int64_t* out, int cap, int* count);

typedef struct canvas_solve_result {
    double flops, params;            /* of the whole net (sum over targets), multiply-accumulates and weights of all fc nodes */
    int32_t rounds;                  /* doubling iterations that changed something */
    int32_t reserved[7];
} canvas_solve_result;

/* Constraint solver (Section 6.3).  targets: n_targets assignments, G the global
 * group number (1 when the template does not use G).  x: host array
 * [n_targets][CANVAS_MAX_VARS], entry [i][j-1] receives x_ij for every free
 * variable (0 for the others).  Step 1: every size that holds x_j is p*x_j/q;
 * lcm_ij = lcm of the reduced q; with target 1 the one of least C (ties: first),
 * k_1j = 1 and k_ij = ceil(C_i*lcm_1j / (C_1*lcm_ij)), x_ij = k_ij*lcm_ij.
 * Step 2: while something changes: compute every Delta_ij (increase of the
 * constrained cost when x_ij alone is doubled), and in ascending order of
 * Delta_ij (ties: by i, then j) double each x_ij that keeps all budgets.
 * flops_budget / params_budget <= 0: no such budget; Delta is measured in FLOPs
 * when there is a FLOPs budget, else in parameters; with no budget step 2 is
 * skipped.  Errors: BAD_ARG; SHAPE_MISMATCH (a size of some target is no
 * integer, a free variable is left in a denominator: substitute it first);
 * UNSUPPORTED (the base values already exceed a budget: the sampler would discard
 * the kernel). */
int canvas_template_solve(const canvas_template* t, const canvas_target* targets, int n_targets, int64_t G,
                          double flops_budget, double params_budget, int64_t* x, canvas_solve_result* result);

/* Concrete blob ("canvas-dag 1" text of canvas_dag.h) of one target.  x: host
 * array of CANVAS_MAX_VARS values (entry j-1 for x_j).  Errors: BAD_ARG,
 * SHAPE_MISMATCH (an attribute is no integer for these values). */
int canvas_template_instantiate(const canvas_template* t, const canvas_target* target, int64_t G, const int64_t* x,
                                char* buf, size_t buf_len, size_t* needed);

void canvas_template_destroy(canvas_template* t);

#ifdef __cplusplus
}
#endif
#endif /* CANVAS_TEMPLATE_H */
