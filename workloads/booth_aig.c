/*
 * Radix-4 Booth multiplier And-Inverter-Graph generator (unsigned n x n bits, n even).
 *
 * An INPUT generator like csa_aig.c: the synthetic stand-in for the paper's Booth multiplier
 * dataset (Section "Experiment", kernel evaluation on Booth / mapped netlists of 64 to 512 bits with
 * embedding dimension 32).  It holds none of the aggregation / planning / partition arithmetic.
 * What matters for the kernels is the degree profile, which differs from the carry-save array's:
 * besides the 2n primary inputs, the three recoding signals of each of the n/2 + 1 digit rows
 * ("one", "two", "neg") fan out to a whole row of partial-product cells, so there are about 3.5 n
 * high-degree rows of n to 2n entries instead of 2n rows of n.
 *
 * Construction (checked by simulation against integer multiplication in the tests):
 *   digit i of b (i = 0 .. n/2):  d_i = -2 b_{2i+1} + b_{2i} + b_{2i-1}   (b_{-1} = b_n = b_{n+1} = 0)
 *   one_i = b_{2i} xor b_{2i-1},  two_i = |d_i| == 2,  neg_i = d_i < 0
 *   magnitude bit k (k = 0..n) of row i:  (one_i & a_k) | (two_i & a_{k-1})
 *   row i = magnitude xor neg_i, sign-extended with neg_i up to bit 2n-1, weight 4^i, plus neg_i at its
 *   least significant column (two's complement), all arithmetic modulo 2^(2n).
 *   The rows are accumulated in carry-save form (one full adder per column and row), the final sum
 *   and carry vectors go through a ripple-carry adder.  Constants are folded, no constant node exists.
 *
 * Node order: a_0..a_{n-1}, b_0..b_{n-1}, AND nodes in emission order, then the 2n primary outputs.
 * Literals and the PO convention are those of csa_aig.c (a PO stores its driver in both fanin slots).
 */
#include <stdint.h>
#include <stdlib.h>

enum { BW_PI = 0, BW_AND = 1, BW_PO = 2 };
#define LIT0 ((int32_t)(-2147483647 - 1))      /* constant false; LIT0 ^ 1 is constant true */
#define LIT1 (LIT0 ^ 1)

typedef struct {
    int64_t next;
    uint8_t *type;        /* NULL: count only */
    int32_t *f0, *f1;
} bgen_t;

static int32_t b_and(bgen_t *g, int32_t x, int32_t y)
{
    if (x == LIT0 || y == LIT0) return LIT0;
    if (x == LIT1) return y;
    if (y == LIT1) return x;
    if (x == y) return x;
    if (x == (y ^ 1)) return LIT0;
    int64_t id = g->next++;
    if (g->type) { g->type[id] = BW_AND; g->f0[id] = x; g->f1[id] = y; }
    return (int32_t)(2 * id);
}

static int32_t b_or(bgen_t *g, int32_t x, int32_t y) { return b_and(g, x ^ 1, y ^ 1) ^ 1; }

/* x xor y; *both receives x & y */
static int32_t b_xor(bgen_t *g, int32_t x, int32_t y, int32_t *both)
{
    int32_t bo = b_and(g, x, y);
    if (both) *both = bo;
    if (x == LIT0) return y;
    if (y == LIT0) return x;
    if (x == LIT1) return y ^ 1;
    if (y == LIT1) return x ^ 1;
    if (x == y) return LIT0;
    if (x == (y ^ 1)) return LIT1;
    int32_t none = b_and(g, x ^ 1, y ^ 1);
    return b_and(g, bo ^ 1, none ^ 1);
}

static int32_t b_full_adder(bgen_t *g, int32_t x, int32_t y, int32_t z, int32_t *carry)
{
    int32_t g1, g2;
    int32_t t = b_xor(g, x, y, &g1);
    int32_t s = b_xor(g, t, z, &g2);
    *carry = b_or(g, g1, g2);
    return s;
}

/*
 * type == NULL: returns the number of nodes the generator would write (2n PIs + ANDs + 2n POs).
 * Otherwise fills type/fanin0/fanin1 (that many entries) and po_driver[2n]; returns the node count,
 * or -1 on bad arguments / allocation failure / a constant product bit.
 */
int64_t wl_booth_generate(int32_t n, uint8_t *type, int32_t *fanin0, int32_t *fanin1, int32_t *po_driver)
{
    if (n < 2 || n > 2048 || (n & 1)) return -1;
    if (type && (!fanin0 || !fanin1)) return -1;
    const int w = 2 * n;
    bgen_t g;
    g.type = type; g.f0 = fanin0; g.f1 = fanin1;
    int32_t *S = (int32_t *)malloc(sizeof(int32_t) * (size_t)w);
    int32_t *C = (int32_t *)malloc(sizeof(int32_t) * (size_t)w);
    if (!S || !C) { free(S); free(C); return -1; }
    if (type)
        for (int v = 0; v < 2 * n; ++v) { type[v] = BW_PI; fanin0[v] = -1; fanin1[v] = -1; }
    g.next = 2 * n;
    for (int k = 0; k < w; ++k) { S[k] = LIT0; C[k] = LIT0; }
#define A_BIT(k) ((k) >= 0 && (k) < n ? (int32_t)(2 * (k)) : LIT0)
#define B_BIT(k) ((k) >= 0 && (k) < n ? (int32_t)(2 * (n + (k))) : LIT0)
    for (int i = 0; i <= n / 2; ++i) {
        const int32_t x0 = B_BIT(2 * i - 1), x1 = B_BIT(2 * i), x2 = B_BIT(2 * i + 1);
        const int32_t x10 = b_and(&g, x1, x0), n10 = b_and(&g, x1 ^ 1, x0 ^ 1);
        const int32_t one = b_xor(&g, x1, x0, NULL);
        const int32_t two = b_or(&g, b_and(&g, x2, n10), b_and(&g, x2 ^ 1, x10));
        const int32_t neg = b_and(&g, x2, x10 ^ 1);
        int32_t carry_in = neg;                            /* the +1 of the two's complement, at column 2i */
        for (int col = 2 * i; col < w; ++col) {
            const int k = col - 2 * i;
            int32_t r;
            if (k <= n) {
                const int32_t m = b_or(&g, b_and(&g, one, A_BIT(k)), b_and(&g, two, A_BIT(k - 1)));
                r = b_xor(&g, m, neg, NULL);
            } else {
                r = neg;
            }
            int32_t c_out;
            const int32_t s = b_full_adder(&g, S[col], C[col], r, &c_out);
            S[col] = s;
            C[col] = carry_in;                             /* slot freed by the adder of this column */
            carry_in = c_out;
        }
    }
    int32_t carry = LIT0;
    int64_t result = -1;
    int ok = 1;
    for (int col = 0; col < w; ++col) {
        int32_t c_out;
        const int32_t m = b_full_adder(&g, S[col], C[col], carry, &c_out);
        carry = c_out;
        if (m == LIT0 || m == LIT1) ok = 0;
        if (po_driver) po_driver[col] = m;
        S[col] = m;
    }
    if (ok) {
        if (type)
            for (int col = 0; col < w; ++col) {
                const int64_t id = g.next + col;
                type[id] = BW_PO; fanin0[id] = S[col]; fanin1[id] = S[col];
            }
        result = g.next + w;
    }
    free(S); free(C);
    return result;
}
