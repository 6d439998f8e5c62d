/*
 * gtree_oracle.c — TEST INFRASTRUCTURE ONLY (see gtree_oracle.h).
 *
 * Plain CPU simulation of GTree's three-party protocols over Z_2^64.
 * Components are indexed j = 0,1,2 for the paper's x_1,x_2,x_3; party P_{j+1}
 * holds components (j, j+1 mod 3) and keys (k_j, k_{j+1}).  Each protocol is
 * written per element, on the three components at once; a step of party j only
 * touches components j and j+1 and the word it received, as Section II-B says.
 *
 * All arithmetic is uint64_t, i.e. mod 2^64 with no reduction code (Sec. II-B).
 */
#include "gtree_oracle.h"
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef uint64_t u64;
typedef uint32_t u32;

#define NX(j) (((j) + 1) % 3)
#define KEY_DEALER 3
#define KEY_OWNER 4

struct orc_ctx {
    u32 key[5][8];
    u32 tau, K;
    u32 op;          /* operation counter, one per protocol invocation */
    u64 rounds;
    u64 wire[3][3];  /* bytes sent from party a to party b */
    u64 bits[3][3];  /* the same messages in payload bits, n*bits per message with no rounding */
    u64 scorer[2];   /* heuristic by reconstruction: bytes the three parties send to the scorer, and get back */
};

/* ------------------------------------------------------------------------- */
/* Randomness.  The paper's parties expand pairwise seeds with a PRNG (Sec. III);
 * here the PRNG is the ChaCha block function with 8 rounds, used as a
 * counter-based PRF.  State words 12..15 are (block lo, block hi, op, stream);
 * word j of stream (op, stream) under a key is the 64-bit little-endian pair
 * (out[2(j&7)], out[2(j&7)+1]) of block j>>3.                                 */

static u32 rotl32(u32 x, int r) { return (x << r) | (x >> (32 - r)); }

void orc_chacha_quarter(u32 v[4])
{
    u32 a = v[0], b = v[1], c = v[2], d = v[3];
    a += b; d ^= a; d = rotl32(d, 16);
    c += d; b ^= c; b = rotl32(b, 12);
    a += b; d ^= a; d = rotl32(d, 8);
    c += d; b ^= c; b = rotl32(b, 7);
    v[0] = a; v[1] = b; v[2] = c; v[3] = d;
}

static void quarter_at(u32 s[16], int a, int b, int c, int d)
{
    u32 v[4] = { s[a], s[b], s[c], s[d] };
    orc_chacha_quarter(v);
    s[a] = v[0]; s[b] = v[1]; s[c] = v[2]; s[d] = v[3];
}

void orc_chacha_block(const u32 key[8], u32 c12, u32 c13, u32 c14, u32 c15, int rounds,
                      u32 out[16])
{
    u32 in[16], s[16];
    in[0] = 0x61707865u; in[1] = 0x3320646eu; in[2] = 0x79622d32u; in[3] = 0x6b206574u;
    for (int i = 0; i < 8; i++) in[4 + i] = key[i];
    in[12] = c12; in[13] = c13; in[14] = c14; in[15] = c15;
    memcpy(s, in, sizeof s);
    for (int r = 0; r < rounds; r += 2) {
        quarter_at(s, 0, 4, 8, 12);  /* column round */
        quarter_at(s, 1, 5, 9, 13);
        quarter_at(s, 2, 6, 10, 14);
        quarter_at(s, 3, 7, 11, 15);
        quarter_at(s, 0, 5, 10, 15); /* diagonal round */
        quarter_at(s, 1, 6, 11, 12);
        quarter_at(s, 2, 7, 8, 13);
        quarter_at(s, 3, 4, 9, 14);
    }
    for (int i = 0; i < 16; i++) out[i] = s[i] + in[i];
}

#define PRF_ROUNDS 8

static u64 prf(const orc_ctx *c, int key_index, u32 op, u32 stream, u64 j)
{
    u32 out[16];
    u64 blk = j >> 3;
    orc_chacha_block(c->key[key_index], (u32)blk, (u32)(blk >> 32), op, stream, PRF_ROUNDS, out);
    int w = (int)(j & 7);
    return (u64)out[2 * w] | ((u64)out[2 * w + 1] << 32);
}

uint64_t orc_prf_word(const orc_ctx *c, int key_index, uint32_t op, uint32_t stream, uint64_t j)
{
    return prf(c, key_index, op, stream, j);
}

/* Zero sharing from pairwise seeds (Sec. II-B, multiplication): alpha_j is the
 * difference of the word under k_j and the word under k_{j+1}; party j+1 holds
 * both keys.  The three values sum (xor) to zero. */
static void zero_a(const orc_ctx *c, u32 op, u32 stream, u64 e, u64 alpha[3])
{
    u64 w[3];
    for (int j = 0; j < 3; j++) w[j] = prf(c, j, op, stream, e);
    for (int j = 0; j < 3; j++) alpha[j] = w[j] - w[NX(j)];
}

static void zero_b(const orc_ctx *c, u32 op, u32 stream, u64 e, u64 alpha[3])
{
    u64 w[3];
    for (int j = 0; j < 3; j++) w[j] = prf(c, j, op, stream, e);
    for (int j = 0; j < 3; j++) alpha[j] = w[j] ^ w[NX(j)];
}

void orc_zero_sharing(const orc_ctx *c, uint32_t op, uint32_t stream, uint64_t e, int boolean,
                      uint64_t alpha[3])
{
    if (boolean) zero_b(c, op, stream, e, alpha); else zero_a(c, op, stream, e, alpha);
}

/* Offline material of one element (the paper excludes its generation from the
 * timed online phase, Sec. VI): an edaBit, i.e. a random r shared arithmetically
 * and bitwise, and a daBit, a random bit beta shared both ways.  A dealer holding
 * key k_D derives them from stream 0, words 8e..8e+7. */
typedef struct {
    u64 rA[3];   /* arithmetic components of r */
    u64 rho[3];  /* Boolean components of the 64 bits of r */
    u64 bB[3];   /* Boolean components of beta (one bit) */
    u64 bA[3];   /* arithmetic components of beta */
    u64 r, beta;
} dealer_t;

static void dealer(const orc_ctx *c, u32 op, u64 e, dealer_t *D)
{
    /* words 8e..8e+7 of stream 0 are exactly block e */
    u32 out[16];
    u64 w[8];
    orc_chacha_block(c->key[KEY_DEALER], (u32)e, (u32)(e >> 32), op, 0, PRF_ROUNDS, out);
    for (int i = 0; i < 8; i++) w[i] = (u64)out[2 * i] | ((u64)out[2 * i + 1] << 32);
    D->r = w[0];
    D->rA[0] = w[1]; D->rA[1] = w[2]; D->rA[2] = D->r - w[1] - w[2];
    D->rho[0] = w[3]; D->rho[1] = w[4]; D->rho[2] = D->r ^ w[3] ^ w[4];
    D->beta = w[5] & 1;
    D->bB[0] = (w[5] >> 1) & 1; D->bB[1] = (w[5] >> 2) & 1;
    D->bB[2] = D->beta ^ D->bB[0] ^ D->bB[1];
    D->bA[0] = w[6]; D->bA[1] = w[7]; D->bA[2] = D->beta - w[6] - w[7];
}

/* daBit of test e of an equality grid.  In a grid the masked index of a row is opened
 * once and serves the comparisons with all columns (see eq_grid_rs), so a test needs no
 * edaBit of its own, only the daBit of its conversion: 131 bits.  The eight tests
 * 8g..8g+7 share the three blocks 3g, 3g+1, 3g+2 of stream 4: test j takes slot j%3 of
 * block 3g + j/3; slot q holds the arithmetic components in words 2q and 2q+1 and the
 * bit and its first two Boolean components in bits 3q, 3q+1, 3q+2 of word 6. */
static void dabit_grid(const orc_ctx *c, u32 op, u64 e, dealer_t *D)
{
    u64 g = e >> 3, j = e & 7, blk = 3 * g + j / 3, q = j % 3;
    u32 out[16];
    u64 w[8];
    orc_chacha_block(c->key[KEY_DEALER], (u32)blk, (u32)(blk >> 32), op, 4, PRF_ROUNDS, out);
    for (int i = 0; i < 8; i++) w[i] = (u64)out[2 * i] | ((u64)out[2 * i + 1] << 32);
    D->beta = (w[6] >> (3 * q)) & 1;
    D->bB[0] = (w[6] >> (3 * q + 1)) & 1; D->bB[1] = (w[6] >> (3 * q + 2)) & 1;
    D->bB[2] = D->beta ^ D->bB[0] ^ D->bB[1];
    D->bA[0] = w[2 * q]; D->bA[1] = w[2 * q + 1]; D->bA[2] = D->beta - w[2 * q] - w[2 * q + 1];
}

void orc_dabit_grid(const orc_ctx *c, uint32_t op, uint64_t e, uint64_t out[7])
{
    dealer_t D;
    dabit_grid(c, op, e, &D);
    for (int j = 0; j < 3; j++) { out[j] = D.bB[j]; out[3 + j] = D.bA[j]; }
    out[6] = D.beta;
}

void orc_dealer(const orc_ctx *c, uint32_t op, uint64_t e, uint64_t out[14])
{
    dealer_t D;
    dealer(c, op, e, &D);
    for (int j = 0; j < 3; j++) {
        out[j] = D.rA[j]; out[3 + j] = D.rho[j]; out[6 + j] = D.bB[j]; out[9 + j] = D.bA[j];
    }
    out[12] = D.r; out[13] = D.beta;
}

/* ------------------------------------------------------------------------- */
/* Message accounting.  dir = +1: every party sends to its successor (opening:
 * P_i gives its first component to P_{i+1}, Sec. II-B Rec); dir = -1: to its
 * predecessor (resharing after a product, so that P_{i-1} then holds
 * (z_{i-1}, z_i)).  One message of n elements of `bits` bits is ceil(n*bits/8) bytes. */
static void wire(orc_ctx *c, int dir, u64 n, u64 bits)
{
    u64 bytes = (n * bits + 7) / 8;
    for (int p = 0; p < 3; p++) {
        c->wire[p][(p + dir + 3) % 3] += bytes;
        c->bits[p][(p + dir + 3) % 3] += n * bits;
    }
}

/* ------------------------------------------------------------------------- */
/* Per-element protocol steps on the three components.                       */

/* Three-term product of Sec. II-B: z_j = x_j y_j + x_{j+1} y_j + x_j y_{j+1}. */
static void prod3(const u64 x[3], const u64 y[3], u64 z[3])
{
    for (int j = 0; j < 3; j++) z[j] = x[j] * y[j] + x[NX(j)] * y[j] + x[j] * y[NX(j)];
}

static void mult_el(const u64 x[3], const u64 y[3], const u64 alpha[3], u64 z[3])
{
    u64 t[3];
    prod3(x, y, t);
    for (int j = 0; j < 3; j++) z[j] = t[j] + alpha[j];
}

/* Same with xor / and on words restricted to `mask`. */
static void and_el(const u64 x[3], const u64 y[3], const u64 alpha[3], u64 mask, u64 z[3])
{
    u64 t[3];
    for (int j = 0; j < 3; j++)
        t[j] = ((x[j] & y[j]) ^ (x[NX(j)] & y[j]) ^ (x[j] & y[NX(j)]) ^ alpha[j]) & mask;
    for (int j = 0; j < 3; j++) z[j] = t[j];
}

/* Equality test (Sec. V-A): bit [v == 0] for a shared v.  Mask v with the edaBit,
 * open c = v + r; v == 0 iff c == r, i.e. every bit of not(c xor r) is one; the 64
 * bits are ANDed pairwise in six rounds on words of width 32,16,...,1 (round k
 * ands bit i with bit i+w, mask bit off_k+i of the stream-1 word, off = 0,32,48,
 * 56,60,62).  64 + 63 bits per party, 7 rounds = 2l-1 bits, log l + 1 rounds. */
static void eq_el(const orc_ctx *c, u32 op, u64 e, const u64 v[3], const dealer_t *D,
                  u64 A[3] /* out: Boolean zero-sharing word of stream 1 */, u64 t[3])
{
    u64 m[3], cpub;
    for (int j = 0; j < 3; j++) m[j] = v[j] + D->rA[j];
    cpub = m[0] + m[1] + m[2];                         /* opened */
    for (int j = 0; j < 3; j++) t[j] = D->rho[j];
    t[0] ^= ~cpub;                                     /* public term goes to component 1 */
    zero_b(c, op, 1, e, A);
    unsigned off = 0;
    for (int k = 0; k < 6; k++) {
        unsigned w = 32u >> k;
        u64 mask = (w == 32) ? 0xffffffffull : ((1ull << w) - 1);
        u64 a[3], b[3], al[3];
        for (int j = 0; j < 3; j++) {
            a[j] = t[j] & mask; b[j] = (t[j] >> w) & mask; al[j] = (A[j] >> off) & mask;
        }
        and_el(a, b, al, mask, t);
        off += w;
    }
}

/* Comparison: bit [v >= 0] for a shared v read as a signed number, |v| < 2^63.
 * Open c = v + r.  Then v = c - r and msb(v) = c_63 xor r_63 xor borrow, where
 * borrow = [c' < r'] on the low 63 bits.  [c' < r'] comes from the prefix pairs
 * (g_i, e_i) = (not c_i and r_i, not (c_i xor r_i)), combined over adjacent blocks
 * hi,lo as (G_hi xor (E_hi and G_lo), E_hi and E_lo) in six levels; bit 63 is
 * padded with (0,1).  The gate of level k whose low block starts at bit i uses
 * mask bit i + 2^k - 1 of stream 1 (G) and stream 2 (E).  The last level needs G
 * only: 64 + 2(32+16+8+4+2) + 1 = 189 bits, 7 rounds. */
static void ge_el(const orc_ctx *c, u32 op, u64 e, const u64 v[3], const dealer_t *D, u64 ge[3])
{
    u64 m[3], cpub, AG[3], AE[3];
    u64 G[64][3], E[64][3];
    for (int j = 0; j < 3; j++) m[j] = v[j] + D->rA[j];
    cpub = m[0] + m[1] + m[2];                         /* opened */
    for (int i = 0; i < 63; i++) {
        u64 nc = (~cpub >> i) & 1;
        for (int j = 0; j < 3; j++) {
            u64 rb = (D->rho[j] >> i) & 1;
            G[i][j] = nc & rb;                         /* and with a public bit is local */
            E[i][j] = rb;
        }
        E[i][0] ^= nc;                                 /* not(c_i xor r_i) = not c_i xor r_i */
    }
    for (int j = 0; j < 3; j++) { G[63][j] = 0; E[63][j] = 0; }
    E[63][0] = 1;
    zero_b(c, op, 1, e, AG);
    zero_b(c, op, 2, e, AE);
    for (int k = 0; k < 6; k++) {
        int s = 1 << k;
        for (int i = 0; i < 64; i += 2 * s) {
            int hi = i + s, lo = i, bit = i + s - 1;
            u64 al[3], p[3];
            for (int j = 0; j < 3; j++) al[j] = (AG[j] >> bit) & 1;
            and_el(E[hi], G[lo], al, 1, p);
            for (int j = 0; j < 3; j++) G[lo][j] = G[hi][j] ^ p[j];
            if (k < 5) {
                for (int j = 0; j < 3; j++) al[j] = (AE[j] >> bit) & 1;
                and_el(E[hi], E[lo], al, 1, E[lo]);
            }
        }
    }
    for (int j = 0; j < 3; j++) ge[j] = ((D->rho[j] >> 63) & 1) ^ G[0][j];   /* msb(v) */
    ge[0] ^= (cpub >> 63) & 1;
    ge[0] ^= 1;                                        /* v >= 0 iff msb is 0 */
}

/* Bit to arithmetic: open f = s xor beta (one bit); s = beta if f = 0, else 1 - beta. */
static void b2a_el(const u64 s[3], const dealer_t *D, u64 out[3])
{
    u64 f = 0;
    for (int j = 0; j < 3; j++) f ^= (s[j] ^ D->bB[j]) & 1;   /* opened */
    for (int j = 0; j < 3; j++) out[j] = f ? (u64)(j == 0) - D->bA[j] : D->bA[j];
}

#define EQ_ROUNDS 7
#define GE_ROUNDS 7
static void wire_eq(orc_ctx *c, u64 n)
{
    wire(c, +1, n, 64);
    for (int k = 0; k < 6; k++) wire(c, -1, n, 32u >> k);
    c->rounds += EQ_ROUNDS;
}
static void wire_ge(orc_ctx *c, u64 n)
{
    wire(c, +1, n, 64);
    for (int k = 0; k < 5; k++) wire(c, -1, n, 2 * (32u >> k));
    wire(c, -1, n, 1);
    c->rounds += GE_ROUNDS;
}
static void wire_b2a(orc_ctx *c, u64 n) { wire(c, +1, n, 1); c->rounds += 1; }
static void wire_and1(orc_ctx *c, u64 n) { wire(c, -1, n, 1); c->rounds += 1; }
static void wire_reshare(orc_ctx *c, u64 n, u64 words) { wire(c, -1, n, 64 * words); c->rounds += 1; }

/* ------------------------------------------------------------------------- */
/* Shared vectors.                                                           */
typedef struct { u64 *c[3]; size_t n; } sh;

static sh sh_alloc(size_t n)
{
    sh v; v.n = n;
    for (int j = 0; j < 3; j++) v.c[j] = (u64 *)calloc(n ? n : 1, sizeof(u64));
    return v;
}
static void sh_free(sh *v) { for (int j = 0; j < 3; j++) { free(v->c[j]); v->c[j] = NULL; } v->n = 0; }
static void sh_get(const sh *v, size_t e, u64 x[3]) { for (int j = 0; j < 3; j++) x[j] = v->c[j][e]; }
static void sh_set(sh *v, size_t e, const u64 x[3]) { for (int j = 0; j < 3; j++) v->c[j][e] = x[j]; }
static void sh_from_flat(sh *v, const u64 *flat) { for (int j = 0; j < 3; j++) memcpy(v->c[j], flat + (size_t)j * v->n, v->n * 8); }
static void sh_to_flat(const sh *v, u64 *flat) { for (int j = 0; j < 3; j++) memcpy(flat + (size_t)j * v->n, v->c[j], v->n * 8); }
static void sh_zero(sh *v) { for (int j = 0; j < 3; j++) memset(v->c[j], 0, v->n * 8); }
/* public constant as a sharing: (c, 0, 0) (Sec. II-B, linear operation) */
static void sh_set_const(sh *v, size_t e, u64 cst) { v->c[0][e] = cst; v->c[1][e] = 0; v->c[2][e] = 0; }

static size_t pad8(size_t n) { return (n + 7) & ~(size_t)7; }

/* ------------------------------------------------------------------------- */
orc_ctx *orc_ctx_create(const uint64_t seed[5][4], uint32_t tau, uint32_t K)
{
    orc_ctx *c = (orc_ctx *)calloc(1, sizeof *c);
    for (int k = 0; k < 5; k++)
        for (int i = 0; i < 4; i++) {
            c->key[k][2 * i] = (u32)seed[k][i];
            c->key[k][2 * i + 1] = (u32)(seed[k][i] >> 32);
        }
    c->tau = tau; c->K = K;
    return c;
}
void orc_ctx_destroy(orc_ctx *c) { free(c); }
void orc_stats(const orc_ctx *c, uint64_t *rounds, uint64_t wire_bytes[9])
{
    *rounds = c->rounds;
    for (int a = 0; a < 3; a++) for (int b = 0; b < 3; b++) wire_bytes[3 * a + b] = c->wire[a][b];
}
void orc_stats_bits(const orc_ctx *c, uint64_t wire_bits[9])
{
    for (int a = 0; a < 3; a++) for (int b = 0; b < 3; b++) wire_bits[3 * a + b] = c->bits[a][b];
}
void orc_stats_scorer(const orc_ctx *c, uint64_t bytes[2]) { bytes[0] = c->scorer[0]; bytes[1] = c->scorer[1]; }
void orc_stats_reset(orc_ctx *c)
{
    c->rounds = 0; memset(c->wire, 0, sizeof c->wire); memset(c->bits, 0, sizeof c->bits);
    memset(c->scorer, 0, sizeof c->scorer);
}
uint32_t orc_op_counter(const orc_ctx *c) { return c->op; }
void orc_set_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}
int orc_get_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ------------------------------------------------------------------------- */
/* Share^A (Sec. II-B): x1, x2 random, x3 = x - x1 - x2; the owner's key plays
 * the data owner / query user.  Words e of streams 0 and 1. */
void orc_share_a(orc_ctx *c, const uint64_t *plain, size_t n, uint64_t *comp)
{
    u32 op = c->op++;
#pragma omp parallel for schedule(static)
    for (size_t e = 0; e < n; e++) {
        u64 x1 = prf(c, KEY_OWNER, op, 0, e), x2 = prf(c, KEY_OWNER, op, 1, e);
        comp[e] = x1; comp[n + e] = x2; comp[2 * n + e] = plain[e] - x1 - x2;
    }
}
void orc_reconstruct_a(const uint64_t *comp, size_t n, uint64_t *plain)
{
    for (size_t e = 0; e < n; e++) plain[e] = comp[e] + comp[n + e] + comp[2 * n + e];
}
void orc_reconstruct_b(const uint64_t *comp, size_t n, uint64_t *plain)
{
    for (size_t e = 0; e < n; e++) plain[e] = comp[e] ^ comp[n + e] ^ comp[2 * n + e];
}

/* ------------------------------------------------------------------------- */
void orc_mult(orc_ctx *c, const uint64_t *x, const uint64_t *y, size_t n, uint64_t *z)
{
    u32 op = c->op++;
#pragma omp parallel for schedule(static)
    for (size_t e = 0; e < n; e++) {
        u64 a[3], b[3], al[3], r[3];
        for (int j = 0; j < 3; j++) { a[j] = x[j * n + e]; b[j] = y[j * n + e]; }
        zero_a(c, op, 0, e, al);
        mult_el(a, b, al, r);
        for (int j = 0; j < 3; j++) z[j * n + e] = r[j];
    }
    wire_reshare(c, n, 1);
}

void orc_eq_b(orc_ctx *c, const uint64_t *x, const uint64_t *y_pub, size_t n, uint64_t *out)
{
    u32 op = c->op++;
#pragma omp parallel for schedule(static)
    for (size_t e = 0; e < n; e++) {
        u64 v[3], A[3], t[3]; dealer_t D;
        for (int j = 0; j < 3; j++) v[j] = x[j * n + e];
        if (y_pub) v[0] -= y_pub[e];
        dealer(c, op, e, &D);
        eq_el(c, op, e, v, &D, A, t);
        for (int j = 0; j < 3; j++) out[j * n + e] = t[j];
    }
    wire_eq(c, n);
}

void orc_eq_a(orc_ctx *c, const uint64_t *x, const uint64_t *y_pub, size_t n, uint64_t *out)
{
    u32 op = c->op++;
#pragma omp parallel for schedule(static)
    for (size_t e = 0; e < n; e++) {
        u64 v[3], A[3], t[3], a[3]; dealer_t D;
        for (int j = 0; j < 3; j++) v[j] = x[j * n + e];
        if (y_pub) v[0] -= y_pub[e];
        dealer(c, op, e, &D);
        eq_el(c, op, e, v, &D, A, t);
        b2a_el(t, &D, a);
        for (int j = 0; j < 3; j++) out[j * n + e] = a[j];
    }
    wire_eq(c, n); wire_b2a(c, n);
}

void orc_ge_a(orc_ctx *c, const uint64_t *x, const uint64_t *y, size_t n, uint64_t *out)
{
    u32 op = c->op++;
#pragma omp parallel for schedule(static)
    for (size_t e = 0; e < n; e++) {
        u64 v[3], g[3], a[3]; dealer_t D;
        for (int j = 0; j < 3; j++) v[j] = x[j * n + e] - y[j * n + e];
        dealer(c, op, e, &D);
        ge_el(c, op, e, v, &D, g);
        b2a_el(g, &D, a);
        for (int j = 0; j < 3; j++) out[j * n + e] = a[j];
    }
    wire_ge(c, n); wire_b2a(c, n);
}

/* ------------------------------------------------------------------------- */
/* Equality grid: the first two lines of the array-access protocol (Sec. V-A: the index u
 * is compared with every position 0..|W|-1), also used for the per-sample leaf flags of
 * the learning protocol (Sec. V-B).  Rows are samples i < n, columns k < w;
 * E[k][i] = [u[i] - base == k], optionally ANDed with a shared bit g[k] common to all
 * rows, then converted to arithmetic.  Element index (and position in EA) is k*n8 + i with
 * n8 = n padded to 8.
 * All comparisons of a row are with PUBLIC constants, so one masked opening serves them
 * all: the row has one edaBit r_i (dealer block i of stream 0), c_i = u_i + r_i is opened
 * once, and u_i - base - k = 0 iff r_i = c_i - base - k, which is tested bit by bit on the
 * shared bits of r_i with fresh masks per test (stream 1, word of the element).  Per row
 * l bits for the opening, per test l-1 bits for the AND rounds [+1 for the AND with g]
 * and 1 for the conversion, whose daBit is the test's own (dabit_grid). */
/* A row subset (rows != NULL) computes only the listed samples, with the element
 * indices of the full problem; results are stored compactly, row r of the list at
 * position k*pad8(nrows) + r.  This lets a test check sampled outputs of a problem
 * that is too large to simulate in full. */
typedef struct { const size_t *rows; size_t nrows; } rowsel;
static size_t rs_count(const rowsel *rs, size_t n) { return rs && rs->rows ? rs->nrows : n; }
static size_t rs_row(const rowsel *rs, size_t r) { return rs && rs->rows ? rs->rows[r] : r; }

static void eq_grid_rs(orc_ctx *c, u32 op, const sh *u, u64 base, size_t w, size_t n,
                       const sh *g, sh *EA, const rowsel *rs)
{
    size_t n8 = pad8(n), nr = rs_count(rs, n), s8 = pad8(nr);
#pragma omp parallel for schedule(static) collapse(2)
    for (size_t k = 0; k < w; k++)
        for (size_t r = 0; r < nr; r++) {
            size_t i = rs_row(rs, r);
            size_t e = k * n8 + i;
            u64 v[3], A[3], t[3], a[3]; dealer_t D;
            sh_get(u, r, v);                           /* u is stored per listed row */
            v[0] -= base + k;                          /* public operand: component 1 only */
            dealer(c, op, i, &D);                      /* the edaBit of the ROW: c_i - base - k = u_i - base - k + r_i */
            dabit_grid(c, op, e, &D);                  /* the daBit of the test */
            eq_el(c, op, e, v, &D, A, t);
            if (g) {
                u64 gb[3], al[3];
                sh_get(g, k, gb);
                for (int j = 0; j < 3; j++) al[j] = (A[j] >> 63) & 1;
                and_el(t, gb, al, 1, t);
            }
            b2a_el(t, &D, a);
            sh_set(EA, k * s8 + r, a);
        }
    wire(c, +1, nr, 64);                               /* one opening per row */
    for (int k = 0; k < 6; k++) wire(c, -1, (u64)w * nr, 32u >> k);
    c->rounds += EQ_ROUNDS;
    if (g) wire_and1(c, (u64)w * nr);
    wire_b2a(c, (u64)w * nr);
}

static void eq_grid(orc_ctx *c, u32 op, const sh *u, u64 base, size_t w, size_t n,
                    const sh *g, sh *EA)
{
    eq_grid_rs(c, op, u, base, w, n, g, EA, NULL);
}

/* z[i] = sum_k EA[k][i] * W[k] + alpha (stream `stream`, word i): the select and
 * sum of the array-access protocol done as one inner product, one reshare per row. */
static void dot_common_rs(const orc_ctx *c, u32 op, u32 stream, const sh *EA, const sh *W,
                          size_t woff, size_t w, size_t n, sh *z, const rowsel *rs)
{
    size_t nr = rs_count(rs, n), s8 = pad8(nr);
#pragma omp parallel for schedule(static)
    for (size_t r = 0; r < nr; r++) {
        u64 acc[3] = { 0, 0, 0 }, al[3];
        for (size_t k = 0; k < w; k++) {
            u64 a[3], b[3], p[3];
            sh_get(EA, k * s8 + r, a); sh_get(W, woff + k, b);
            prod3(a, b, p);
            for (int j = 0; j < 3; j++) acc[j] += p[j];
        }
        zero_a(c, op, stream, rs_row(rs, r), al);
        for (int j = 0; j < 3; j++) acc[j] += al[j];
        sh_set(z, r, acc);
    }
}
static void dot_common(const orc_ctx *c, u32 op, u32 stream, const sh *EA, const sh *W,
                       size_t woff, size_t w, size_t n, sh *z)
{
    dot_common_rs(c, op, stream, EA, W, woff, w, n, z, NULL);
}

/* same with a per-row array: z[i] = sum_k EA[k][i] * XT[k][i]; XT is stored like EA */
static void dot_rows_rs(const orc_ctx *c, u32 op, u32 stream, const sh *EA, const sh *XT,
                        size_t w, size_t n, sh *z, const rowsel *rs)
{
    size_t nr = rs_count(rs, n), s8 = pad8(nr);
#pragma omp parallel for schedule(static)
    for (size_t r = 0; r < nr; r++) {
        u64 acc[3] = { 0, 0, 0 }, al[3];
        for (size_t k = 0; k < w; k++) {
            u64 a[3], b[3], p[3];
            sh_get(EA, k * s8 + r, a); sh_get(XT, k * s8 + r, b);
            prod3(a, b, p);
            for (int j = 0; j < 3; j++) acc[j] += p[j];
        }
        zero_a(c, op, stream, rs_row(rs, r), al);
        for (int j = 0; j < 3; j++) acc[j] += al[j];
        sh_set(z, r, acc);
    }
}
static void dot_rows(const orc_ctx *c, u32 op, u32 stream, const sh *EA, const sh *XT,
                     size_t w, size_t n, sh *z)
{
    dot_rows_rs(c, op, stream, EA, XT, w, n, z, NULL);
}

/* Oblivious array access (Sec. V-A): 7 + 1 + 1 rounds = log l + 3. */
void orc_oaa(orc_ctx *c, const uint64_t *Wf, size_t w, const uint64_t *uf, size_t n, uint64_t *zf)
{
    u32 op = c->op++;
    sh W = sh_alloc(w), u = sh_alloc(n), z = sh_alloc(n), EA = sh_alloc(w * pad8(n));
    sh_from_flat(&W, Wf); sh_from_flat(&u, uf);
    eq_grid(c, op, &u, 0, w, n, NULL, &EA);
    dot_common(c, op, 2, &EA, &W, 0, w, n, &z);
    wire_reshare(c, n, 1);
    sh_to_flat(&z, zf);
    sh_free(&W); sh_free(&u); sh_free(&z); sh_free(&EA);
}

/* ------------------------------------------------------------------------- */
/* The protocols as the paper prints them (Sec. V-A, Alg. "Oblivious Array Access";
 * Sec. V-B, Alg. "Oblivious Learning"), without the fusion into inner products used
 * above: every array element goes through its own SelectShare - the comparison bit is
 * converted with a daBit of the element's own, the opened value travelling as a ring
 * element of l bits as the paper's cost formula counts it, then multiplied with the array
 * element with a zero-sharing word and a reshare of the element's own - and the selected
 * elements are added up locally.  Per element: equality test 2l-1 bits, conversion l,
 * product l = 4l-1 bits, in log l + 3 rounds.  Reconstructed results equal those of the
 * fused protocols.  Streams: 0 dealer, 1 masks, 2 product; all indexed by the element. */
static void wire_b2a_wide(orc_ctx *c, u64 n) { wire(c, +1, n, 64); c->rounds += 1; }

/* z[i] = sum_k Select(E[k][i], W) with E[k][i] = [u[i] - base == k]; W is common to all
 * rows (Wcommon, offset woff) or the row's own (Wrows[k*n8 + i]) */
static void oaa_literal(orc_ctx *c, const sh *u, u64 base, size_t w, size_t n, const sh *Wcommon,
                        size_t woff, const sh *Wrows, sh *z)
{
    u32 op = c->op++;
    size_t n8 = pad8(n);
    sh_zero(z);
#pragma omp parallel for schedule(static)
    for (size_t i = 0; i < n; i++) {
        u64 acc[3] = { 0, 0, 0 };
        for (size_t k = 0; k < w; k++) {
            size_t e = k * n8 + i;
            u64 v[3], A[3], t[3], a[3], b[3], al[3], p[3]; dealer_t D;
            sh_get(u, i, v);
            v[0] -= base + k;
            dealer(c, op, e, &D);
            eq_el(c, op, e, v, &D, A, t);
            b2a_el(t, &D, a);
            if (Wcommon) sh_get(Wcommon, woff + k, b); else sh_get(Wrows, e, b);
            zero_a(c, op, 2, e, al);
            mult_el(a, b, al, p);
            for (int j = 0; j < 3; j++) acc[j] += p[j];
        }
        sh_set(z, i, acc);
    }
    wire_eq(c, (u64)w * n); wire_b2a_wide(c, (u64)w * n); wire_reshare(c, (u64)w * n, 1);
}

void orc_oaa_literal(orc_ctx *c, const uint64_t *Wf, size_t w, const uint64_t *uf, size_t n, uint64_t *zf)
{
    sh W = sh_alloc(w), u = sh_alloc(n), z = sh_alloc(n);
    sh_from_flat(&W, Wf); sh_from_flat(&u, uf);
    oaa_literal(c, &u, 0, w, n, &W, 0, NULL, &z);
    sh_to_flat(&z, zf);
    sh_free(&W); sh_free(&u); sh_free(&z);
}

/* ------------------------------------------------------------------------- */
/* One step of restoring division on n elements (one op): b = [r >= Q],
 * r <- r - b*Q, quo <- 2*quo + b.  Streams: 0 dealer, 1/2 comparison, 3 product. */
static void div_step(orc_ctx *c, sh *r, const sh *Q, sh *quo, size_t n)
{
    u32 op = c->op++;
#pragma omp parallel for schedule(static)
    for (size_t e = 0; e < n; e++) {
        u64 rv[3], qv[3], v[3], g[3], b[3], al[3], p[3], q[3]; dealer_t D;
        sh_get(r, e, rv); sh_get(Q, e, qv); sh_get(quo, e, q);
        for (int j = 0; j < 3; j++) v[j] = rv[j] - qv[j];
        dealer(c, op, e, &D);
        ge_el(c, op, e, v, &D, g);
        b2a_el(g, &D, b);
        zero_a(c, op, 3, e, al);
        mult_el(b, qv, al, p);
        for (int j = 0; j < 3; j++) { rv[j] -= p[j]; q[j] = 2 * q[j] + b[j]; }
        sh_set(r, e, rv); sh_set(quo, e, q);
    }
    wire_ge(c, n); wire_b2a(c, n); wire_reshare(c, n, 1);
}

/* quo = floor(S * 2^tau / Q) for 0 <= S <= Q, Q > 0: tau+1 steps, the remainder is
 * doubled between steps. */
static void divide(orc_ctx *c, const sh *S, const sh *Q, sh *quo, size_t n)
{
    sh r = sh_alloc(n);
    for (int j = 0; j < 3; j++) memcpy(r.c[j], S->c[j], n * 8);
    sh_zero(quo);
    for (u32 t = 0; t <= c->tau; t++) {
        if (t) for (int j = 0; j < 3; j++) for (size_t e = 0; e < n; e++) r.c[j][e] *= 2;
        div_step(c, &r, Q, quo, n);
    }
    sh_free(&r);
}

void orc_div(orc_ctx *c, const uint64_t *Sf, const uint64_t *Qf, size_t n, uint64_t *qf)
{
    sh S = sh_alloc(n), Q = sh_alloc(n), q = sh_alloc(n);
    sh_from_flat(&S, Sf); sh_from_flat(&Q, Qf);
    divide(c, &S, &Q, &q, n);
    sh_to_flat(&q, qf);
    sh_free(&S); sh_free(&Q); sh_free(&q);
}

/* One compare-and-select op on n pairs: b = [right > left] (left wins ties);
 * val <- left + b*(right-left), idx <- idxL + b*(idxR-idxL).
 * Streams: 0 dealer, 1/2 comparison, 3 value product, 4 index product. */
static void select_max(orc_ctx *c, size_t n, const sh *vl, const sh *vr, const sh *il,
                       const sh *ir, sh *vout, sh *iout)
{
    u32 op = c->op++;
#pragma omp parallel for schedule(static)
    for (size_t e = 0; e < n; e++) {
        u64 L[3], R[3], IL[3], IR[3], v[3], g[3], b[3], al[3], d[3], p[3]; dealer_t D;
        sh_get(vl, e, L); sh_get(vr, e, R); sh_get(il, e, IL); sh_get(ir, e, IR);
        for (int j = 0; j < 3; j++) v[j] = L[j] - R[j];
        dealer(c, op, e, &D);
        ge_el(c, op, e, v, &D, g);      /* [left >= right] */
        g[0] ^= 1;                      /* [right > left] */
        b2a_el(g, &D, b);
        zero_a(c, op, 3, e, al);
        for (int j = 0; j < 3; j++) d[j] = R[j] - L[j];
        mult_el(b, d, al, p);
        for (int j = 0; j < 3; j++) L[j] += p[j];
        zero_a(c, op, 4, e, al);
        for (int j = 0; j < 3; j++) d[j] = IR[j] - IL[j];
        mult_el(b, d, al, p);
        for (int j = 0; j < 3; j++) IL[j] += p[j];
        sh_set(vout, e, L); sh_set(iout, e, IL);
    }
    wire_ge(c, n); wire_b2a(c, n); wire_reshare(c, n, 2);
}

/* ------------------------------------------------------------------------- */
/* Training state (Sec. IV: arrays T, F, M, C, gamma).                       */
struct orc_train {
    size_t N, N8;
    u32 d, K, H, CW;       /* CW = d*K + K words of statistics per node */
    u32 level;             /* next level to process */
    sh XT, YT, XYT;        /* [k][i], [c][i], [k*K+c][i], rows padded to N8 */
    sh M;                  /* N */
    sh T, F;               /* 2^(H+1)-1 */
    sh C, gamma;           /* current level: n_h x CW, n_h x d (inherited, then counted) */
    sh isLeaf;             /* Boolean, n_h */
    sh LT;                 /* n_h x N8 */
    sh SD, split;          /* n_h */
    sh Clast, Glast, Slast;/* copies kept for export */
    u32 last;              /* level the copies belong to */
    int fresh_import;      /* state was imported and no level has run since: the copies are not valid */
    int hc_open;           /* heuristic computation by reconstruction instead of the MPC protocol */
    int literal;           /* learning protocol as printed: whole-T scans, per-element SelectShare */
    int part_matmul;       /* data partition by products with the previous level's leaf one-hot */
    u32 lt_level;          /* level whose per-sample one-hot LT holds, or (u32)-1 */
    sh LB;                 /* literal mode: per-sample leaf flags as Boolean bits, n_h x N8 */
};

static size_t nodes_upto(u32 H) { return ((size_t)2 << H) - 1; }

orc_train *orc_train_create(orc_ctx *c, const uint64_t *Xf, const uint64_t *Yf, size_t N,
                            uint32_t d, uint32_t H)
{
    orc_train *t = (orc_train *)calloc(1, sizeof *t);
    u32 K = c->K;
    size_t N8 = pad8(N), nmax = (size_t)1 << H;
    t->N = N; t->N8 = N8; t->d = d; t->K = K; t->H = H; t->CW = d * K + K; t->level = 0;
    t->XT = sh_alloc(d * N8); t->YT = sh_alloc(K * N8); t->XYT = sh_alloc((size_t)d * K * N8);
    t->M = sh_alloc(N);
    t->T = sh_alloc(nodes_upto(H)); t->F = sh_alloc(nodes_upto(H));
    t->C = sh_alloc(nmax * t->CW); t->gamma = sh_alloc(nmax * d);
    t->isLeaf = sh_alloc(nmax); t->LT = sh_alloc(nmax * N8);
    t->SD = sh_alloc(nmax); t->split = sh_alloc(nmax);
    t->Clast = sh_alloc(nmax * t->CW); t->Glast = sh_alloc(nmax * d); t->Slast = sh_alloc(nmax * d);
    t->LB = sh_alloc(0);
    t->lt_level = (u32)-1;
    for (int j = 0; j < 3; j++) {
        for (size_t i = 0; i < N; i++) {
            for (u32 k = 0; k < d; k++) t->XT.c[j][k * N8 + i] = Xf[(size_t)j * N * d + i * d + k];
            for (u32 q = 0; q < K; q++) t->YT.c[j][q * N8 + i] = Yf[(size_t)j * N * K + i * K + q];
        }
    }
    /* one-time products feature value x class indicator (Sec. V-B, statistics
     * counting: the per-sample products are computed once and reused) */
    u32 op = c->op++;
#pragma omp parallel for schedule(static) collapse(2)
    for (size_t col = 0; col < (size_t)d * K; col++)
        for (size_t i = 0; i < N; i++) {
            size_t k = col / K, q = col % K, e = col * N8 + i;
            u64 a[3], b[3], al[3], z[3];
            sh_get(&t->XT, k * N8 + i, a); sh_get(&t->YT, q * N8 + i, b);
            zero_a(c, op, 0, e, al);
            mult_el(a, b, al, z);
            sh_set(&t->XYT, e, z);
        }
    wire_reshare(c, (u64)N * d * K, 1);
    /* M = 0; root is a leaf; no feature used yet (Sec. V-B) */
    sh_set_const(&t->F, 0, 1);
    for (u32 k = 0; k < d; k++) sh_set_const(&t->gamma, k, 1);
    return t;
}

void orc_train_destroy(orc_train *t)
{
    if (!t) return;
    sh *all[] = { &t->XT, &t->YT, &t->XYT, &t->M, &t->T, &t->F, &t->C, &t->gamma, &t->isLeaf,
                  &t->LT, &t->SD, &t->split, &t->Clast, &t->Glast, &t->Slast, &t->LB };
    for (size_t i = 0; i < sizeof all / sizeof all[0]; i++) sh_free(all[i]);
    free(t);
}

/* Data partition of the learning protocol: fetch the feature assigned to each
 * sample's node at level h-1, fetch that feature's value, M <- 2M + value + 1. */
static void partition(orc_ctx *c, orc_train *t, u32 h)
{
    size_t N = t->N, N8 = t->N8, wprev = (size_t)1 << (h - 1), base = wprev - 1;
    sh EA = sh_alloc((wprev > t->d ? wprev : t->d) * N8), Tval = sh_alloc(N), Dval = sh_alloc(N);
    u32 op = c->op++;
    eq_grid(c, op, &t->M, base, wprev, N, NULL, &EA);
    dot_common(c, op, 2, &EA, &t->T, base, wprev, N, &Tval);
    wire_reshare(c, N, 1);
    op = c->op++;
    eq_grid(c, op, &Tval, 0, t->d, N, NULL, &EA);
    dot_rows(c, op, 2, &EA, &t->XT, t->d, N, &Dval);
    wire_reshare(c, N, 1);
    for (int j = 0; j < 3; j++)
        for (size_t i = 0; i < N; i++)
            t->M.c[j][i] = 2 * t->M.c[j][i] + Dval.c[j][i] + (j == 0 ? 1 : 0);
    sh_free(&EA); sh_free(&Tval); sh_free(&Dval);
}

/* Data partition without per-sample equality tests (a variant beyond the paper's listing,
 * which fetches T[M] and then D[i][T[M]] by two array accesses per sample).  The previous
 * level has left the per-sample leaf one-hot L (of the statistics counting) and the split
 * decisions T_{h-1}[r]; then
 *   OH[r][k]  = [T_{h-1}[r] = k]                 n_{h-1} * d equality tests, sample-independent
 *   sel[k][i] = sum_r L[r][i] * OH[r][k]          one reshare per (k, i)
 *   Dval[i]   = sum_k sel[k][i] * X[k][i]          one reshare per sample
 * and M <- 2M + Dval + 1 as before.  A sample whose node at level h-1 is not a real leaf has
 * an all-zero one-hot, so its Dval is 0: it goes to the left child of a node that has no
 * real leaves below it any more, which no later step can tell from the right one; for every
 * sample in a real leaf Dval = X[i][T[M]] as in the paper.  Streams: op 1: 0 dealer, 1 masks;
 * op 2 and 3: zero sharing of stream 0, word k*N8+i resp. i. */
static int partition_matmul(orc_ctx *c, orc_train *t, u32 h)
{
    size_t N = t->N, N8 = t->N8, d = t->d, np = (size_t)1 << (h - 1), base = np - 1;
    if (t->lt_level != h - 1) return -1;               /* needs the one-hot of the level just processed */
    sh OH = sh_alloc(np * d), sel = sh_alloc(d * N8);
    u32 op = c->op++;
#pragma omp parallel for schedule(static)
    for (size_t e = 0; e < np * d; e++) {
        size_t r = e / d, k = e % d;
        u64 v[3], A[3], b[3], a[3]; dealer_t D;
        sh_get(&t->T, base + r, v);
        v[0] -= k;
        dealer(c, op, e, &D);
        eq_el(c, op, e, v, &D, A, b);
        b2a_el(b, &D, a);
        sh_set(&OH, e, a);
    }
    wire_eq(c, np * d); wire_b2a(c, np * d);
    op = c->op++;
#pragma omp parallel for schedule(static) collapse(2)
    for (size_t k = 0; k < d; k++)
        for (size_t i = 0; i < N; i++) {
            u64 acc[3] = { 0, 0, 0 }, al[3];
            for (size_t r = 0; r < np; r++) {
                u64 a[3], b[3], p[3];
                sh_get(&t->LT, r * N8 + i, a); sh_get(&OH, r * d + k, b);
                prod3(a, b, p);
                for (int j = 0; j < 3; j++) acc[j] += p[j];
            }
            zero_a(c, op, 0, k * N8 + i, al);
            for (int j = 0; j < 3; j++) acc[j] += al[j];
            sh_set(&sel, k * N8 + i, acc);
        }
    wire_reshare(c, (u64)N * d, 1);
    op = c->op++;
#pragma omp parallel for schedule(static)
    for (size_t i = 0; i < N; i++) {
        u64 acc[3] = { 0, 0, 0 }, al[3];
        for (size_t k = 0; k < d; k++) {
            u64 a[3], b[3], p[3];
            sh_get(&sel, k * N8 + i, a); sh_get(&t->XT, k * N8 + i, b);
            prod3(a, b, p);
            for (int j = 0; j < 3; j++) acc[j] += p[j];
        }
        zero_a(c, op, 0, i, al);
        for (int j = 0; j < 3; j++) t->M.c[j][i] = 2 * t->M.c[j][i] + acc[j] + al[j] + (j == 0 ? 1 : 0);
    }
    wire_reshare(c, N, 1);
    sh_free(&OH); sh_free(&sel);
    return 0;
}

void orc_train_set_partition(orc_train *t, int by_products) { t->part_matmul = by_products ? 1 : 0; }

/* Leaf flags and per-sample one-hot of the statistics-counting step. */
static void leaf_onehot(orc_ctx *c, orc_train *t, u32 h)
{
    size_t nh = (size_t)1 << h, base = nh - 1;
    u32 op = c->op++;
    for (size_t r = 0; r < nh; r++) {
        u64 v[3], A[3], b[3]; dealer_t D;
        sh_get(&t->F, base + r, v);
        v[0] -= 1;
        dealer(c, op, r, &D);
        eq_el(c, op, r, v, &D, A, b);
        sh_set(&t->isLeaf, r, b);
    }
    wire_eq(c, nh);
    op = c->op++;
    eq_grid(c, op, &t->M, base, nh, t->N, &t->isLeaf, &t->LT);
    t->lt_level = h;
}

/* counts[r][col] += sum_i L[r][i] * B[col][i] for columns [col0, col1) of the
 * statistics block (XY columns, then the K class columns); one zero-sharing word
 * and one reshare per output; the word index is the position in the output. */
static void count(orc_ctx *c, orc_train *t, u32 h, int totals_only)
{
    size_t nh = (size_t)1 << h, N = t->N, N8 = t->N8, dK = (size_t)t->d * t->K;
    size_t ncol = totals_only ? t->K : t->CW;
    u32 op = c->op++;
#pragma omp parallel for schedule(dynamic) collapse(2)
    for (size_t r = 0; r < nh; r++)
        for (size_t oc = 0; oc < ncol; oc++) {
            size_t col = totals_only ? dK + oc : oc;
            const sh *B = col < dK ? &t->XYT : &t->YT;
            size_t boff = (col < dK ? col : col - dK) * N8;
            u64 acc[3] = { 0, 0, 0 }, al[3];
            for (size_t i = 0; i < N; i++) {
                u64 a[3], b[3], p[3];
                sh_get(&t->LT, r * N8 + i, a); sh_get(B, boff + i, b);
                prod3(a, b, p);
                for (int j = 0; j < 3; j++) acc[j] += p[j];
            }
            zero_a(c, op, 0, r * ncol + oc, al);
            for (int j = 0; j < 3; j++) t->C.c[j][r * t->CW + col] += acc[j] + al[j];
        }
    wire_reshare(c, (u64)nh * ncol, 1);
}

/* The learning protocol as printed (Alg. "Oblivious Learning").  Data partition: array
 * access over the WHOLE tree array (all 2^(H+1)-1 entries, index M itself), then over the
 * sample's features. */
static void partition_literal(orc_ctx *c, orc_train *t, u32 h)
{
    (void)h;
    size_t N = t->N;
    sh Tval = sh_alloc(N), Dval = sh_alloc(N);
    oaa_literal(c, &t->M, 0, nodes_upto(t->H), N, &t->T, 0, NULL, &Tval);
    oaa_literal(c, &Tval, 0, t->d, N, NULL, 0, &t->XT, &Dval);
    for (int j = 0; j < 3; j++)
        for (size_t i = 0; i < N; i++)
            t->M.c[j][i] = 2 * t->M.c[j][i] + Dval.c[j][i] + (j == 0 ? 1 : 0);
    sh_free(&Tval); sh_free(&Dval);
}

/* Leaf flags as Boolean bits: LCF[r][i] = [M[i] - (2^h - 1) == r] and isLeaf[r], no
 * conversion (the per-element SelectShare of the counting step converts). */
static void leaf_bits_literal(orc_ctx *c, orc_train *t, u32 h)
{
    size_t nh = (size_t)1 << h, base = nh - 1, N = t->N, N8 = t->N8;
    u32 op = c->op++;
    for (size_t r = 0; r < nh; r++) {
        u64 v[3], A[3], b[3]; dealer_t D;
        sh_get(&t->F, base + r, v);
        v[0] -= 1;
        dealer(c, op, r, &D);
        eq_el(c, op, r, v, &D, A, b);
        sh_set(&t->isLeaf, r, b);
    }
    wire_eq(c, nh);
    op = c->op++;
    sh_free(&t->LB);
    t->LB = sh_alloc(nh * N8);
#pragma omp parallel for schedule(static) collapse(2)
    for (size_t r = 0; r < nh; r++)
        for (size_t i = 0; i < N; i++) {
            size_t e = r * N8 + i;
            u64 v[3], A[3], b[3], g[3], al[3]; dealer_t D;
            sh_get(&t->M, i, v);
            v[0] -= base + r;
            dealer(c, op, e, &D);
            eq_el(c, op, e, v, &D, A, b);
            sh_get(&t->isLeaf, r, g);
            for (int j = 0; j < 3; j++) al[j] = (A[j] >> 63) & 1;
            and_el(b, g, al, 1, b);
            sh_set(&t->LB, e, b);
        }
    wire_eq(c, (u64)nh * N); wire_and1(c, (u64)nh * N);
}

/* Statistics counting as printed: the per-sample counter array C'[i] of (1+K) x 2d
 * entries (row 0: [X_k = v]; row c+1: [X_k = v and class c]; column 2k+v) is selected by
 * LCF[r][i] element by element and accumulated into the counter array of leaf r.  With
 * totals_only (label level) only the entries of candidate 0 are needed.  The compact
 * statistics (count of X_k = 1 and class c; class totals) are read off the counter array
 * by local linear operations and added to the inherited ones.  Element index of the
 * conversion and the product: (r*PW + q)*N8 + i, q the position in the counter array. */
static void count_literal(orc_ctx *c, orc_train *t, u32 h, int totals_only)
{
    size_t nh = (size_t)1 << h, N = t->N, N8 = t->N8, d = t->d, K = t->K, dK = d * K, CW = t->CW;
    size_t dd = totals_only ? 1 : d, PW = (1 + K) * 2 * dd;
    u32 op = c->op++;
    sh Cp = sh_alloc(nh * PW);
#pragma omp parallel for schedule(dynamic) collapse(2)
    for (size_t r = 0; r < nh; r++)
        for (size_t q = 0; q < PW; q++) {
            size_t row = q / (2 * dd), k = (q % (2 * dd)) / 2, v = q & 1;
            u64 acc[3] = { 0, 0, 0 };
            for (size_t i = 0; i < N; i++) {
                size_t e = (r * PW + q) * N8 + i;
                u64 s[3], a[3], cv[3], al[3], p[3]; dealer_t D;
                /* C'[i][row][2k+v] by local linear operations on X, Y and the one-time products */
                for (int j = 0; j < 3; j++) {
                    u64 x = t->XT.c[j][k * N8 + i];
                    if (row == 0) cv[j] = v ? x : (u64)(j == 0) - x;
                    else {
                        u64 xy = t->XYT.c[j][(k * K + (row - 1)) * N8 + i], y = t->YT.c[j][(row - 1) * N8 + i];
                        cv[j] = v ? xy : y - xy;
                    }
                }
                sh_get(&t->LB, r * N8 + i, s);
                dealer(c, op, e, &D);
                b2a_el(s, &D, a);
                zero_a(c, op, 2, e, al);
                mult_el(a, cv, al, p);
                for (int j = 0; j < 3; j++) acc[j] += p[j];
            }
            sh_set(&Cp, r * PW + q, acc);
        }
    wire_b2a_wide(c, (u64)nh * PW * N); wire_reshare(c, (u64)nh * PW * N, 1);
    for (int j = 0; j < 3; j++)
        for (size_t r = 0; r < nh; r++) {
            const u64 *o = Cp.c[j] + r * PW;
            for (size_t cl = 0; cl < K; cl++) {
                t->C.c[j][r * CW + dK + cl] += o[(cl + 1) * 2 * dd] + o[(cl + 1) * 2 * dd + 1];
                if (!totals_only)
                    for (size_t k = 0; k < d; k++) t->C.c[j][r * CW + k * K + cl] += o[(cl + 1) * 2 * dd + 2 * k + 1];
            }
        }
    sh_free(&Cp);
}

void orc_train_set_literal(orc_train *t, int literal) { t->literal = literal ? 1 : 0; }

/* Heuristic computation (Sec. V-B, MPC-based): for every node r, candidate k and
 * branch j the class counts n_jc, S = sum_c n_jc^2 and Q = n_j * n; the score
 * sum_j S/Q is one minus the Gini index of Eq. (1) (P = n_j^2 - S), so the largest
 * score is the smallest Gini index; used candidates are zeroed by gamma. */
static void heuristic(orc_ctx *c, orc_train *t, u32 h)
{
    size_t nh = (size_t)1 << h, d = t->d, K = t->K, dK = d * K, CW = t->CW;
    size_t nq = nh * d * 2;
    sh S = sh_alloc(nq), Q = sh_alloc(nq), quo = sh_alloc(nq);
    u32 op = c->op++;
#pragma omp parallel for schedule(static)
    for (size_t q = 0; q < nq; q++) {
        size_t r = q / (2 * d), k = (q / 2) % d, br = q & 1;
        u64 nj[3] = { 0, 0, 0 }, n[3] = { 0, 0, 0 }, s[3] = { 0, 0, 0 }, al[3], p[3];
        for (size_t cl = 0; cl < K; cl++) {
            u64 n1[3], tot[3], njc[3];
            sh_get(&t->C, r * CW + k * K + cl, n1); sh_get(&t->C, r * CW + dK + cl, tot);
            for (int j = 0; j < 3; j++) {
                njc[j] = br ? n1[j] : tot[j] - n1[j];
                nj[j] += njc[j]; n[j] += tot[j];
            }
            prod3(njc, njc, p);
            for (int j = 0; j < 3; j++) s[j] += p[j];
        }
        zero_a(c, op, 0, q, al);
        for (int j = 0; j < 3; j++) s[j] += al[j];
        sh_set(&S, q, s);
        zero_a(c, op, 1, q, al);
        mult_el(nj, n, al, p);
        sh_set(&Q, q, p);
    }
    wire_reshare(c, nq, 2);
    /* empty branch: Q = 0 and S = 0; make the divisor 1 so that the term is 0 */
    op = c->op++;
#pragma omp parallel for schedule(static)
    for (size_t q = 0; q < nq; q++) {
        u64 v[3], A[3], b[3], a[3]; dealer_t D;
        sh_get(&Q, q, v);
        dealer(c, op, q, &D);
        eq_el(c, op, q, v, &D, A, b);
        b2a_el(b, &D, a);
        for (int j = 0; j < 3; j++) v[j] += a[j];
        sh_set(&Q, q, v);
    }
    wire_eq(c, nq); wire_b2a(c, nq);
    divide(c, &S, &Q, &quo, nq);
    /* score = quotient of branch 0 + quotient of branch 1, masked by gamma */
    size_t ns = nh * d;
    sh score = sh_alloc(ns);
    op = c->op++;
#pragma omp parallel for schedule(static)
    for (size_t e = 0; e < ns; e++) {
        u64 s[3], g[3], al[3], z[3];
        for (int j = 0; j < 3; j++) s[j] = quo.c[j][2 * e] + quo.c[j][2 * e + 1];
        sh_get(&t->gamma, e, g);
        zero_a(c, op, 0, e, al);
        mult_el(s, g, al, z);
        sh_set(&score, e, z);
    }
    wire_reshare(c, ns, 1);
    for (int j = 0; j < 3; j++) memcpy(t->Slast.c[j], score.c[j], ns * 8);
    /* argmax by a knockout tournament over the candidates padded with zeros to a
     * power of two; the lower index wins ties */
    size_t P2 = 1; while (P2 < d) P2 *= 2;
    sh val = sh_alloc(nh * P2), idx = sh_alloc(nh * P2);
    for (size_t r = 0; r < nh; r++)
        for (size_t k = 0; k < P2; k++) {
            if (k < d) { u64 s[3]; sh_get(&score, r * d + k, s); sh_set(&val, r * P2 + k, s); }
            sh_set_const(&idx, r * P2 + k, k);
        }
    for (size_t len = P2; len > 1; len /= 2) {
        size_t half = len / 2, n = nh * half;
        sh vl = sh_alloc(n), vr = sh_alloc(n), il = sh_alloc(n), ir = sh_alloc(n);
        for (size_t r = 0; r < nh; r++)
            for (size_t m = 0; m < half; m++) {
                u64 x[3];
                sh_get(&val, r * len + 2 * m, x); sh_set(&vl, r * half + m, x);
                sh_get(&val, r * len + 2 * m + 1, x); sh_set(&vr, r * half + m, x);
                sh_get(&idx, r * len + 2 * m, x); sh_set(&il, r * half + m, x);
                sh_get(&idx, r * len + 2 * m + 1, x); sh_set(&ir, r * half + m, x);
            }
        select_max(c, n, &vl, &vr, &il, &ir, &val, &idx);   /* results packed as [r][half] */
        sh_free(&vl); sh_free(&vr); sh_free(&il); sh_free(&ir);
    }
    for (size_t r = 0; r < nh; r++) { u64 x[3]; sh_get(&idx, r, x); sh_set(&t->SD, r, x); }
    sh_free(&S); sh_free(&Q); sh_free(&quo); sh_free(&score); sh_free(&val); sh_free(&idx);
}

/* Updates of gamma, F, C and T (end of the heuristic protocol and node split,
 * Sec. V-B): the chosen candidate is marked used; a real leaf that is not pure
 * becomes internal and its children start as leaves with empty statistics; in
 * every other case the children are dummies that inherit the statistics; gamma is
 * always inherited; T at this level takes the split decisions. */
static void update_flags(orc_ctx *c, orc_train *t, u32 h)
{
    size_t nh = (size_t)1 << h, base = nh - 1, d = t->d, K = t->K, dK = d * K, CW = t->CW;
    u32 op = c->op++;
#pragma omp parallel for schedule(static)
    for (size_t e = 0; e < nh * d; e++) {
        size_t r = e / d, k = e % d;
        u64 v[3], A[3], b[3], oh[3], g[3], al[3], z[3]; dealer_t D;
        sh_get(&t->SD, r, v);
        v[0] -= k;
        dealer(c, op, e, &D);
        eq_el(c, op, e, v, &D, A, b);
        b2a_el(b, &D, oh);
        for (int j = 0; j < 3; j++) oh[j] = (u64)(j == 0) - oh[j];      /* 1 - onehot */
        sh_get(&t->gamma, e, g);
        zero_a(c, op, 2, e, al);
        mult_el(g, oh, al, z);
        sh_set(&t->gamma, e, z);
    }
    wire_eq(c, nh * d); wire_b2a(c, nh * d); wire_reshare(c, nh * d, 1);
    /* pure node: n^2 - sum_c tot_c^2 = 0, i.e. at most one class present (the
     * node's own Gini numerator vanishes); split = isLeaf and not pure */
    op = c->op++;
    for (size_t r = 0; r < nh; r++) {
        u64 n[3] = { 0, 0, 0 }, dv[3], p[3], al[3], A[3], b[3], leaf[3], sA[3], f[3], z[3];
        dealer_t D;
        for (size_t cl = 0; cl < K; cl++)
            for (int j = 0; j < 3; j++) n[j] += t->C.c[j][r * CW + dK + cl];
        prod3(n, n, dv);
        for (size_t cl = 0; cl < K; cl++) {
            u64 tc[3];
            sh_get(&t->C, r * CW + dK + cl, tc);
            prod3(tc, tc, p);
            for (int j = 0; j < 3; j++) dv[j] -= p[j];
        }
        zero_a(c, op, 2, r, al);
        for (int j = 0; j < 3; j++) dv[j] += al[j];
        dealer(c, op, r, &D);
        eq_el(c, op, r, dv, &D, A, b);           /* pure */
        b[0] ^= 1;                               /* not pure */
        sh_get(&t->isLeaf, r, leaf);
        for (int j = 0; j < 3; j++) al[j] = (A[j] >> 63) & 1;
        and_el(leaf, b, al, 1, b);
        b2a_el(b, &D, sA);
        sh_set(&t->split, r, sA);
        for (int j = 0; j < 3; j++) sA[j] = (u64)(j == 0) - sA[j];       /* 1 - split */
        sh_get(&t->F, base + r, f);
        zero_a(c, op, 3, r, al);
        mult_el(f, sA, al, z);
        sh_set(&t->F, base + r, z);              /* leaf 1 -> internal 0 when split */
        for (int j = 0; j < 3; j++) z[j] = sA[j] + (u64)(j == 0);        /* 2 - split */
        sh_set(&t->F, 2 * (base + r) + 1, z);
        sh_set(&t->F, 2 * (base + r) + 2, z);
    }
    wire_reshare(c, nh, 1); wire_eq(c, nh); wire_and1(c, nh); wire_b2a(c, nh); wire_reshare(c, nh, 1);
}

/* Node split (Sec. V-B): T takes the split decisions; the children of a node that was split
 * start with empty statistics, all others inherit them; gamma is always inherited. */
static void node_split(orc_ctx *c, orc_train *t, u32 h)
{
    size_t nh = (size_t)1 << h, base = nh - 1, d = t->d, CW = t->CW;
    u32 op;
    /* keep this level's statistics and flags for export, then build level h+1 */
    for (int j = 0; j < 3; j++) {
        memcpy(t->Clast.c[j], t->C.c[j], nh * CW * 8);
        memcpy(t->Glast.c[j], t->gamma.c[j], nh * d * 8);
    }
    t->last = h;
    for (size_t r = 0; r < nh; r++) { u64 x[3]; sh_get(&t->SD, r, x); sh_set(&t->T, base + r, x); }
    sh Cn = sh_alloc(nh * CW);
    op = c->op++;
#pragma omp parallel for schedule(static)
    for (size_t e = 0; e < nh * CW; e++) {
        size_t r = e / CW;
        u64 x[3], s[3], al[3], z[3];
        sh_get(&t->C, e, x); sh_get(&t->split, r, s);
        for (int j = 0; j < 3; j++) s[j] = (u64)(j == 0) - s[j];
        zero_a(c, op, 0, e, al);
        mult_el(x, s, al, z);
        sh_set(&Cn, e, z);
    }
    wire_reshare(c, nh * CW, 1);
    if (h < t->H) {
        sh Gn = sh_alloc(nh * d);
        for (int j = 0; j < 3; j++) memcpy(Gn.c[j], t->gamma.c[j], nh * d * 8);
        for (size_t r = 0; r < nh; r++)
            for (int ch = 0; ch < 2; ch++)
                for (int j = 0; j < 3; j++) {
                    memcpy(t->C.c[j] + (2 * r + ch) * CW, Cn.c[j] + r * CW, CW * 8);
                    memcpy(t->gamma.c[j] + (2 * r + ch) * d, Gn.c[j] + r * d, d * 8);
                }
        sh_free(&Gn);
    }
    sh_free(&Cn);
}

/* Heuristic computation by reconstruction: the host analogue of the TEE-based protocol of
 * Sec. V-B.  The parties hand the shares of the level's C, gamma and F to a scorer (the
 * enclave of the paper; here a fourth role with the dealer's key), which reconstructs them,
 * computes in the clear what the MPC protocol computes - the fixed-point scores
 * sum_j floor(S_j 2^tau / Q_j) with an empty branch counting 0, masked by gamma, the first
 * maximum, the updated gamma, the purity test n^2 = sum_c tot_c^2 and the node types - and
 * hands back fresh sharings of SD, gamma, F (node and children), the split flags and the
 * masked scores, one operation id each in this order: x1, x2 = words e of streams 0 and 1
 * under the dealer's key, x3 = x - x1 - x2.  Two rounds; the bytes to and from the scorer
 * are counted apart from the messages between the parties. */
static void share_from_scorer(orc_ctx *c, const u64 *plain, size_t n, sh *out, size_t off)
{
    u32 op = c->op++;
    for (size_t e = 0; e < n; e++) {
        u64 x1 = prf(c, KEY_DEALER, op, 0, e), x2 = prf(c, KEY_DEALER, op, 1, e);
        out->c[0][off + e] = x1; out->c[1][off + e] = x2; out->c[2][off + e] = plain[e] - x1 - x2;
    }
    c->scorer[1] += 3 * 2 * 8 * (u64)n;            /* every party receives its two components */
}

static void heuristic_open(orc_ctx *c, orc_train *t, u32 h)
{
    size_t nh = (size_t)1 << h, base = nh - 1, d = t->d, K = t->K, dK = d * K, CW = t->CW;
    u64 *SDp = (u64 *)calloc(nh, 8), *Gp = (u64 *)calloc(nh * d, 8), *Fn = (u64 *)calloc(nh, 8),
        *Fc = (u64 *)calloc(nh, 8), *Sp = (u64 *)calloc(nh, 8), *SCp = (u64 *)calloc(nh * d, 8);
    c->scorer[0] += 3 * 8 * (u64)(nh * (CW + d + 1)); /* every party sends its first component of C, gamma, F */
    c->rounds += 1;
    for (size_t r = 0; r < nh; r++) {
        u64 tot[64], n = 0, sq = 0, best = 0, bi = 0;
        for (size_t cl = 0; cl < K; cl++) {
            tot[cl] = t->C.c[0][r * CW + dK + cl] + t->C.c[1][r * CW + dK + cl] + t->C.c[2][r * CW + dK + cl];
            n += tot[cl]; sq += tot[cl] * tot[cl];
        }
        for (size_t k = 0; k < d; k++) {
            u64 score = 0;
            for (int br = 0; br < 2; br++) {
                u64 nj = 0, S = 0;
                for (size_t cl = 0; cl < K; cl++) {
                    size_t e = r * CW + k * K + cl;
                    u64 n1 = t->C.c[0][e] + t->C.c[1][e] + t->C.c[2][e];
                    u64 njc = br ? n1 : tot[cl] - n1;
                    nj += njc; S += njc * njc;
                }
                u64 Q = nj * n;
                if (Q == 0) Q = 1;                 /* empty branch: the term is 0 */
                score += (S << c->tau) / Q;        /* S <= Q < 2^40, tau <= 20: no overflow */
            }
            u64 g = t->gamma.c[0][r * d + k] + t->gamma.c[1][r * d + k] + t->gamma.c[2][r * d + k];
            score *= g;
            SCp[r * d + k] = score; Gp[r * d + k] = g;
            if (score > best) { best = score; bi = k; }     /* first maximum: the lowest index wins ties */
        }
        SDp[r] = bi;
        Gp[r * d + bi] = 0;
        u64 F = t->F.c[0][base + r] + t->F.c[1][base + r] + t->F.c[2][base + r];
        u64 split = (F == 1 && n * n - sq != 0) ? 1 : 0;
        Sp[r] = split; Fn[r] = F * (1 - split); Fc[r] = 2 - split;
    }
    share_from_scorer(c, SDp, nh, &t->SD, 0);
    share_from_scorer(c, Gp, nh * d, &t->gamma, 0);
    share_from_scorer(c, Fn, nh, &t->F, base);
    {   /* both children of node r get the same sharing */
        sh tmp = sh_alloc(nh);
        share_from_scorer(c, Fc, nh, &tmp, 0);
        for (size_t r = 0; r < nh; r++) { u64 x[3]; sh_get(&tmp, r, x); sh_set(&t->F, 2 * (base + r) + 1, x); sh_set(&t->F, 2 * (base + r) + 2, x); }
        sh_free(&tmp);
    }
    share_from_scorer(c, Sp, nh, &t->split, 0);
    share_from_scorer(c, SCp, nh * d, &t->Slast, 0);
    c->rounds += 1;
    free(SDp); free(Gp); free(Fn); free(Fc); free(Sp); free(SCp);
}

void orc_train_set_heuristic(orc_train *t, int by_reconstruction) { t->hc_open = by_reconstruction ? 1 : 0; }

int orc_train_level(orc_ctx *c, orc_train *t, uint32_t h)
{
    if (h != t->level || h >= t->H) return -1;
    if (t->literal) {
        if (h > 0) partition_literal(c, t, h);
        leaf_bits_literal(c, t, h);
        count_literal(c, t, h, 0);
    } else {
        if (h > 0 && t->part_matmul) { if (partition_matmul(c, t, h)) return -1; }
        else if (h > 0) partition(c, t, h);
        leaf_onehot(c, t, h);
        count(c, t, h, 0);
    }
    if (t->hc_open) heuristic_open(c, t, h);
    else { heuristic(c, t, h); update_flags(c, t, h); }
    node_split(c, t, h);
    t->level = h + 1;
    t->fresh_import = 0;
    return 0;
}

/* Level H holds labels (Sec. IV, model representation).  The paper does not say
 * how they are produced; here: class totals of the node (counted if it is a real
 * leaf, inherited otherwise), first maximum by a compare-and-select chain. */
int orc_train_finish(orc_ctx *c, orc_train *t, uint64_t *feat, uint64_t *leaf)
{
    u32 H = t->H, K = t->K;
    if (t->level != H) return -1;
    size_t nh = (size_t)1 << H, base = nh - 1, dK = (size_t)t->d * K, CW = t->CW;
    if (t->literal) {
        if (H > 0) partition_literal(c, t, H);
        leaf_bits_literal(c, t, H);
        count_literal(c, t, H, 1);
    } else {
        if (H > 0 && t->part_matmul) { if (partition_matmul(c, t, H)) return -1; }
        else if (H > 0) partition(c, t, H);
        leaf_onehot(c, t, H);
        count(c, t, H, 1);
    }
    sh best = sh_alloc(nh), lab = sh_alloc(nh), cand = sh_alloc(nh), ci = sh_alloc(nh);
    for (size_t r = 0; r < nh; r++) { u64 x[3]; sh_get(&t->C, r * CW + dK, x); sh_set(&best, r, x); }
    for (u32 cl = 1; cl < K; cl++) {
        for (size_t r = 0; r < nh; r++) {
            u64 x[3]; sh_get(&t->C, r * CW + dK + cl, x); sh_set(&cand, r, x);
            sh_set_const(&ci, r, cl);
        }
        select_max(c, nh, &best, &cand, &lab, &ci, &best, &lab);
    }
    for (size_t r = 0; r < nh; r++) { u64 x[3]; sh_get(&lab, r, x); sh_set(&t->T, base + r, x); }
    for (int j = 0; j < 3; j++) memcpy(t->Clast.c[j], t->C.c[j], nh * CW * 8);
    t->last = H;
    t->level = H + 1;
    t->fresh_import = 0;
    for (int j = 0; j < 3; j++) {
        if (feat) memcpy(feat + (size_t)j * base, t->T.c[j], base * 8);
        if (leaf) memcpy(leaf + (size_t)j * nh, t->T.c[j] + base, nh * 8);
    }
    sh_free(&best); sh_free(&lab); sh_free(&cand); sh_free(&ci);
    return 0;
}

static int of_last_level(int what)
{
    return what == ORC_X_C || what == ORC_X_GAMMA || what == ORC_X_SD || what == ORC_X_L ||
           what == ORC_X_SCORE || what == ORC_X_C_PAPER;
}

size_t orc_train_export_size(const orc_train *t, int what)
{
    if (t->fresh_import && of_last_level(what)) return 0;
    size_t nh = (size_t)1 << t->last;
    switch (what) {
    case ORC_X_T: case ORC_X_F: return nodes_upto(t->H);
    case ORC_X_M: return t->N;
    case ORC_X_C: return nh * t->CW;
    case ORC_X_GAMMA: case ORC_X_SCORE: return nh * t->d;
    case ORC_X_SD: return nh;
    case ORC_X_L: return nh * t->N8;
    case ORC_X_C_PAPER: return nh * (1 + t->K) * 2 * t->d;
    default: return 0;
    }
}

int orc_train_export(const orc_train *t, int what, uint64_t *comp)
{
    if (t->fresh_import && of_last_level(what)) return -1;
    size_t n = orc_train_export_size(t, what);
    const sh *src = NULL;
    switch (what) {
    case ORC_X_T: src = &t->T; break;
    case ORC_X_F: src = &t->F; break;
    case ORC_X_M: src = &t->M; break;
    case ORC_X_C: src = &t->Clast; break;
    case ORC_X_GAMMA: src = &t->Glast; break;
    case ORC_X_SCORE: src = &t->Slast; break;
    case ORC_X_SD: src = &t->SD; break;
    case ORC_X_L: if (t->literal) return -1; src = &t->LT; break;
    case ORC_X_C_PAPER: {
        /* counter array of Sec. V-B: per node, rows 1..K hold the (value, class)
         * counts, column 2k+v for value v of candidate k; row 0 is their sum */
        size_t nh = (size_t)1 << t->last, d = t->d, K = t->K, dK = d * K, CW = t->CW;
        size_t per = (1 + K) * 2 * d;
        for (int j = 0; j < 3; j++)
            for (size_t r = 0; r < nh; r++) {
                u64 *o = comp + (size_t)j * n + r * per;
                for (size_t col = 0; col < 2 * d; col++) o[col] = 0;
                for (size_t cl = 0; cl < K; cl++)
                    for (size_t k = 0; k < d; k++) {
                        u64 n1 = t->Clast.c[j][r * CW + k * K + cl];
                        u64 tot = t->Clast.c[j][r * CW + dK + cl];
                        o[(cl + 1) * 2 * d + 2 * k + 1] = n1;
                        o[(cl + 1) * 2 * d + 2 * k] = tot - n1;
                        o[2 * k + 1] += n1; o[2 * k] += tot - n1;
                    }
            }
        return 0;
    }
    default: return -1;
    }
    for (int j = 0; j < 3; j++) memcpy(comp + (size_t)j * n, src->c[j], n * 8);
    return 0;
}

int orc_train_import(orc_train *t, uint32_t h, const uint64_t *M, const uint64_t *Tprev,
                     const uint64_t *Flevel, const uint64_t *C, const uint64_t *gamma)
{
    if (h > t->H) return -1;
    size_t nh = (size_t)1 << h, base = nh - 1;
    for (int j = 0; j < 3; j++) {
        memcpy(t->M.c[j], M + (size_t)j * t->N, t->N * 8);
        if (h > 0) memcpy(t->T.c[j] + (base - nh / 2), Tprev + (size_t)j * (nh / 2), (nh / 2) * 8);
        memcpy(t->F.c[j] + base, Flevel + (size_t)j * nh, nh * 8);
        memcpy(t->C.c[j], C + (size_t)j * nh * t->CW, nh * t->CW * 8);
        memcpy(t->gamma.c[j], gamma + (size_t)j * nh * t->d, nh * t->d * 8);
    }
    t->level = h;
    t->fresh_import = 1;
    t->lt_level = (u32)-1;
    return 0;
}

/* ------------------------------------------------------------------------- */
/* Inference (Sec. V-C): H times fetch the node's feature id (and threshold) by
 * array access over the level's slice of the tree, fetch that feature of the
 * instance, step to a child; the label is the value fetched at level H.
 * Binary mode: the fetched feature value is the branch bit.  Threshold mode (an
 * extension for non-binary inputs): the bit is [value > threshold]. */
static int infer_rs(orc_ctx *c, const uint64_t *featf, const uint64_t *thrf, const uint64_t *leaff,
                    uint32_t H, const uint64_t *If, size_t NI, uint32_t d, uint64_t *Rf, const rowsel *rs)
{
    /* If holds the listed rows only (nr x d, row-major); NI is the size of the full batch */
    size_t nr = rs_count(rs, NI), S8 = pad8(nr), nint = ((size_t)1 << H) - 1, nleaf = (size_t)1 << H;
    size_t wmax = nleaf > d ? nleaf : d;
    sh feat = sh_alloc(nint), thr = sh_alloc(nint), leaf = sh_alloc(nleaf);
    sh IT = sh_alloc(d * S8), Tidx = sh_alloc(nr), f = sh_alloc(nr), th = sh_alloc(nr),
       x = sh_alloc(nr), R = sh_alloc(nr), EA = sh_alloc(wmax * S8);
    sh_from_flat(&feat, featf); if (thrf) sh_from_flat(&thr, thrf); sh_from_flat(&leaf, leaff);
    for (int j = 0; j < 3; j++)
        for (size_t r = 0; r < nr; r++)
            for (u32 k = 0; k < d; k++) IT.c[j][k * S8 + r] = If[(size_t)j * nr * d + r * d + k];
    for (u32 n = 0; n < H; n++) {
        size_t w = (size_t)1 << n, base = w - 1;
        u32 op = c->op++;
        eq_grid_rs(c, op, &Tidx, base, w, NI, NULL, &EA, rs);
        dot_common_rs(c, op, 2, &EA, &feat, base, w, NI, &f, rs);
        if (thrf) dot_common_rs(c, op, 3, &EA, &thr, base, w, NI, &th, rs);
        wire_reshare(c, nr, thrf ? 2 : 1);
        op = c->op++;
        eq_grid_rs(c, op, &f, 0, d, NI, NULL, &EA, rs);
        dot_rows_rs(c, op, 2, &EA, &IT, d, NI, &x, rs);
        wire_reshare(c, nr, 1);
        if (thrf) {
            op = c->op++;
#pragma omp parallel for schedule(static)
            for (size_t r = 0; r < nr; r++) {
                size_t i = rs_row(rs, r);
                u64 v[3], g[3], b[3]; dealer_t D;
                for (int j = 0; j < 3; j++) v[j] = th.c[j][r] - x.c[j][r];
                dealer(c, op, i, &D);
                ge_el(c, op, i, v, &D, g);     /* [threshold >= value] */
                g[0] ^= 1;                     /* [value > threshold] */
                b2a_el(g, &D, b);
                sh_set(&x, r, b);
            }
            wire_ge(c, nr); wire_b2a(c, nr);
        }
        for (int j = 0; j < 3; j++)
            for (size_t r = 0; r < nr; r++)
                Tidx.c[j][r] = 2 * Tidx.c[j][r] + x.c[j][r] + (j == 0 ? 1 : 0);
    }
    u32 op = c->op++;
    eq_grid_rs(c, op, &Tidx, nleaf - 1, nleaf, NI, NULL, &EA, rs);
    dot_common_rs(c, op, 2, &EA, &leaf, 0, nleaf, NI, &R, rs);
    wire_reshare(c, nr, 1);
    sh_to_flat(&R, Rf);
    sh_free(&feat); sh_free(&thr); sh_free(&leaf); sh_free(&IT); sh_free(&Tidx); sh_free(&f);
    sh_free(&th); sh_free(&x); sh_free(&R); sh_free(&EA);
    return 0;
}

int orc_infer_batch(orc_ctx *c, const uint64_t *featf, const uint64_t *thrf, const uint64_t *leaff,
                    uint32_t H, const uint64_t *If, size_t NI, uint32_t d, uint64_t *Rf)
{
    return infer_rs(c, featf, thrf, leaff, H, If, NI, d, Rf, NULL);
}

/* The same protocol for the listed rows of a batch of NI instances: I holds those rows
 * only (nrows x d), R receives nrows results.  Shares equal those of the full run. */
int orc_infer_rows(orc_ctx *c, const uint64_t *featf, const uint64_t *thrf, const uint64_t *leaff,
                   uint32_t H, const uint64_t *If, size_t NI, uint32_t d, const size_t *rows,
                   size_t nrows, uint64_t *Rf)
{
    rowsel rs = { rows, nrows };
    return infer_rs(c, featf, thrf, leaff, H, If, NI, d, Rf, &rs);
}
