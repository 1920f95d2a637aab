/*
 * CPU oracle (test infrastructure, not a product path) of the instantiation enumeration of
 * Section 4.2.1, Eq. 5 of the Oobleck paper: all count vectors (x_0 .. x_{p-1}) with
 * sum x_j n_j = N in the order in which the equation's concatenation lists them, then the
 * paper's second requirement (at least f+1 pipelines) as a filter that keeps that order.
 *
 * Eq. 5, with p' read as the number of template sizes in play (sizes n_0 .. n_{p'-1}):
 *     X(p', N') = X(p'-1, N')  ++  theta( X(p', N' - n_{p'-1}), p'-1 )
 *     X(0, 0) = [ the all-zero vector ],  X(0, N' > 0) = [],  the second term is [] if N' < n_{p'-1}
 * theta adds one to x_{p'-1} of every vector of its list.  This file evaluates the equation
 * top-down without a memo: the increments theta will apply on the way back are carried in x[],
 * so vectors come out one by one, in list order, without any list being stored.
 * oracle/instantiation.py holds the same equation as the table of lists the paper draws;
 * tests pin the two against each other, against exhaustive enumeration and partition numbers.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
    const int32_t *sizes;
    int p, need;  /* need = f + 1 pipelines */
    int64_t *x;   /* increments pending from enclosing theta()s */
    uint16_t *out;
    int64_t cap, count, all;
} Ctx;

static void expand(Ctx *c, int pp, int64_t N, int64_t pipes) {
    if (pp == 0) {
        if (N != 0) return;            /* X(0, N' > 0) is empty */
        c->all++;
        if (pipes < c->need) return;   /* requirement 2, applied to the finished list */
        if (c->out && c->count < c->cap)
            for (int j = 0; j < c->p; ++j) c->out[c->count * c->p + j] = (uint16_t)c->x[j];
        c->count++;
        return;
    }
    expand(c, pp - 1, N, pipes);                      /* X(p'-1, N') */
    if (N >= c->sizes[pp - 1]) {                      /* theta(X(p', N' - n), p'-1) */
        c->x[pp - 1]++;
        expand(c, pp, N - c->sizes[pp - 1], pipes + 1);
        c->x[pp - 1]--;
    }
}

/* Vectors of X(p, N) with at least f+1 pipelines, row-major [vector][p] into out (may be NULL;
 * at most cap rows are written).  Returns their number; *all_out gets |X(p, N)|. */
int64_t oob_oracle_instantiate(const int32_t *sizes, int p, int N, int f, uint16_t *out, int64_t cap,
                               int64_t *all_out) {
    Ctx c;
    c.sizes = sizes; c.p = p; c.need = f + 1; c.out = out; c.cap = cap; c.count = 0; c.all = 0;
    c.x = (int64_t *)calloc((size_t)(p > 0 ? p : 1), sizeof(int64_t));
    expand(&c, p, N, 0);
    free(c.x);
    if (all_out) *all_out = c.all;
    return c.count;
}
