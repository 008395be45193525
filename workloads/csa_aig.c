/*
 * Seedless carry-save-array (CSA) multiplier And-Inverter-Graph generator.
 *
 * This file is an INPUT generator: it produces the synthetic stand-in for the
 * paper's ABC-generated CSA multiplier AIGs (Section "Converting Netlists into
 * Transitional Graph": a DAG of two-input AND nodes whose edges may be
 * inverted, with primary inputs and primary outputs).  It holds none of the
 * aggregation / planning / partition arithmetic; both the HIP library and the
 * CPU oracle take its output as their input.
 *
 * Node order (0-based ids): a_0..a_{n-1}, b_0..b_{n-1}, AND nodes in emission
 * order, then the 2n primary outputs m_0..m_{2n-1}.  For n = 2 the emission
 * order reproduces the paper's two-bit worked example (1-based: node 5 is
 * a0*b0; nodes 6..10 form m1 = a0b1 xor a1b0 with node 10 having both inputs
 * inverted; POs are 15..18).
 *
 * A literal is 2*id + inv.  A PI has fanins -1,-1.  A PO stores its driver
 * literal in BOTH fanin slots, so that every non-PI node contributes two
 * edge records: that is the edge count the paper prints for the 1024-bit,
 * batch-16 graph (268,140,544 = 16 * (16 n^2 - 18 n) at n = 1024).
 */
#include <stdint.h>
#include <stdlib.h>

enum { WL_PI = 0, WL_AND = 1, WL_PO = 2 };

/* node classes of the paper's ground truth (Section "Node Features and Node Label creation") */
enum { WL_LABEL_PO = 0, WL_LABEL_MAJ = 1, WL_LABEL_XOR = 2, WL_LABEL_AND = 3, WL_LABEL_PI = 4 };

typedef struct {
    int n;
    int64_t next;          /* next free node id */
    uint8_t *type;
    int32_t *f0, *f1;
    int32_t *pp;           /* n*n memo of partial-product literals, -1 = not emitted */
    uint8_t *label;        /* optional: class of every node */
} gen_t;

static int32_t lit_not(int32_t l) { return l ^ 1; }

static int32_t emit_and(gen_t *g, int32_t x, int32_t y)
{
    int64_t id = g->next++;
    g->type[id] = WL_AND;
    g->f0[id] = x;
    g->f1[id] = y;
    if (g->label) g->label[id] = WL_LABEL_AND;
    return (int32_t)(2 * id);
}

static void set_label(gen_t *g, int32_t lit, uint8_t label)
{
    if (g->label) g->label[lit >> 1] = label;
}

/* partial product a_j & b_i, emitted the first time it is used */
static int32_t pp(gen_t *g, int i, int j)
{
    int32_t *slot = &g->pp[(size_t)i * g->n + j];
    if (*slot < 0)
        *slot = emit_and(g, 2 * j, 2 * (g->n + i));
    return *slot;
}

/* xor as three ANDs; *carry receives x&y, which doubles as the half-adder carry */
static int32_t emit_xor(gen_t *g, int32_t x, int32_t y, int32_t *carry)
{
    int32_t both = emit_and(g, x, y);
    int32_t none = emit_and(g, lit_not(x), lit_not(y));
    *carry = both;
    int32_t top = emit_and(g, lit_not(both), lit_not(none));
    set_label(g, top, WL_LABEL_XOR);          /* the node with both inputs inverted is the xor root */
    return top;
}

static int32_t half_adder(gen_t *g, int32_t x, int32_t y, int32_t *carry)
{
    int32_t sum = emit_xor(g, x, y, carry);
    set_label(g, *carry, WL_LABEL_MAJ);       /* x&y is the majority of (x, y, 0): the carry root */
    return sum;
}

/* full adder: two xors (6 ANDs) plus one AND whose inverted output is the carry */
static int32_t full_adder(gen_t *g, int32_t x, int32_t y, int32_t z, int32_t *carry)
{
    int32_t g1, g2;
    int32_t t1 = emit_xor(g, x, y, &g1);
    int32_t s = emit_xor(g, t1, z, &g2);
    int32_t k = emit_and(g, lit_not(g1), lit_not(g2));
    set_label(g, k, WL_LABEL_MAJ);            /* !k = g1 | g2 = maj(x, y, z): the carry root */
    *carry = lit_not(k);
    return s;
}

int64_t wl_csa_num_nodes(int32_t n) { return 8LL * n * n - 7LL * n; }

/*
 * Fill type[N1], fanin0[N1], fanin1[N1] (N1 = wl_csa_num_nodes(n)) and
 * po_driver[2n] (the literal that drives each m_k).  Returns the number of
 * nodes written, or -1 on bad arguments / allocation failure.
 */
int64_t wl_csa_generate_labeled(int32_t n, uint8_t *type, int32_t *fanin0, int32_t *fanin1,
                                int32_t *po_driver, uint8_t *label);

int64_t wl_csa_generate(int32_t n, uint8_t *type, int32_t *fanin0, int32_t *fanin1,
                        int32_t *po_driver)
{
    return wl_csa_generate_labeled(n, type, fanin0, fanin1, po_driver, NULL);
}

/* Same, and label[N1] (may be NULL) receives the class of every node:
   4 = PI, 3 = plain AND, 2 = XOR root, 1 = MAJ (carry) root, 0 = PO. */
int64_t wl_csa_generate_labeled(int32_t n, uint8_t *type, int32_t *fanin0, int32_t *fanin1,
                                int32_t *po_driver, uint8_t *label)
{
    if (n < 2 || n > 4096 || !type || !fanin0 || !fanin1) return -1;
    gen_t g;
    g.n = n;
    g.type = type; g.f0 = fanin0; g.f1 = fanin1; g.label = label;
    g.pp = (int32_t *)malloc(sizeof(int32_t) * (size_t)n * n);
    int32_t *s = (int32_t *)malloc(sizeof(int32_t) * (size_t)n);
    int32_t *c = (int32_t *)malloc(sizeof(int32_t) * (size_t)n);
    int32_t *m = (int32_t *)malloc(sizeof(int32_t) * 2 * (size_t)n);
    if (!g.pp || !s || !c || !m) { free(g.pp); free(s); free(c); free(m); return -1; }
    for (size_t t = 0; t < (size_t)n * n; ++t) g.pp[t] = -1;

    for (int v = 0; v < 2 * n; ++v) {
        type[v] = WL_PI; fanin0[v] = -1; fanin1[v] = -1;
        if (label) label[v] = WL_LABEL_PI;
    }
    g.next = 2 * n;

    m[0] = pp(&g, 0, 0);
    /* array row 1: half adders over pp(0,j+1) and pp(1,j) */
    for (int j = 0; j <= n - 2; ++j) {
        int32_t x = pp(&g, 0, j + 1);
        int32_t y = pp(&g, 1, j);
        s[j] = half_adder(&g, x, y, &c[j]);
    }
    m[1] = s[0];
    /* array rows 2..n-1: full adders; sums shift one column, carries stay (carry-save) */
    for (int i = 2; i <= n - 1; ++i) {
        for (int j = 0; j <= n - 2; ++j) {
            int32_t x = pp(&g, i, j);
            int32_t y = (j < n - 2) ? s[j + 1] : pp(&g, i - 1, n - 1);
            /* s[j+1] is still the previous row's value: s[j] is overwritten only after use */
            int32_t cy;
            int32_t sum = full_adder(&g, x, y, c[j], &cy);
            s[j] = sum;
            c[j] = cy;
        }
        m[i] = s[0];
    }
    /* final ripple-carry adder over the remaining sums and carries */
    {
        int32_t cy;
        int32_t top0 = (0 < n - 2) ? s[1] : pp(&g, n - 1, n - 1);
        m[n] = half_adder(&g, top0, c[0], &cy);
        for (int k = 1; k <= n - 2; ++k) {
            int32_t top = (k < n - 2) ? s[k + 1] : pp(&g, n - 1, n - 1);
            m[n + k] = full_adder(&g, top, c[k], cy, &cy);
        }
        m[2 * n - 1] = cy;
    }
    for (int k = 0; k < 2 * n; ++k) {
        int64_t id = g.next++;
        type[id] = WL_PO;
        fanin0[id] = m[k];
        fanin1[id] = m[k];
        if (label) label[id] = WL_LABEL_PO;
        if (po_driver) po_driver[k] = m[k];
    }
    int64_t written = g.next;
    free(g.pp); free(s); free(c); free(m);
    return written;
}
