/*
 * gtree_oracle.h — TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow CPU simulation of the three-party protocols of GTree
 * (secret-shared decision-tree training and inference over Z_2^64).
 * It exists to check the GPU library bit for bit; the product never calls it.
 * It shares no code with the GPU path.
 *
 * Representation: a shared vector of n elements is three component arrays laid
 * out component-major, comp[j*n + e] = component j+1 of element e
 * (Section II-B: x = x1 + x2 + x3, party P_i holds (x_i, x_{i+1})).
 * Boolean sharings use the same layout with XOR.
 *
 * Every protocol invocation takes the next value of the context's operation
 * counter; randomness is a pure function of (key, op, stream, word index), so
 * the order of calls is part of the definition.
 *
 * Parity pins (tests/, marked "not gpu"): ChaCha block function against the
 * RFC 8439 vectors; sharing/zero-sharing identities; Mult, EQ, GE, B2A, OAA by
 * brute force against plain integer arithmetic; Division against exact integer
 * division; training against a plaintext fixed-point Gini CART and against the
 * real-valued Gini definition; inference against plaintext traversal; the
 * paper's round and bit counts for EQ and OAA.
 * Parity unpinned (design choices that no external source fixes): the PRF and
 * its stream/word assignment, the dealer's derivation of edaBits/daBits, the
 * direction of messages, tie-breaks (lowest index), the node-type state
 * machine details, threshold-mode inference.
 */
#ifndef GTREE_ORACLE_H
#define GTREE_ORACLE_H
#include <stddef.h>
#include <stdint.h>
#ifdef __cplusplus
extern "C" {
#endif

typedef struct orc_ctx orc_ctx;
typedef struct orc_train orc_train;

/* selectors for orc_train_export */
enum {
    ORC_X_T = 0,      /* tree array, 2^(H+1)-1 nodes */
    ORC_X_F = 1,      /* node types, same size */
    ORC_X_M = 2,      /* leaf id per sample, N */
    ORC_X_C = 3,      /* counted statistics of the level last processed: n_h x (d*K+K) */
    ORC_X_GAMMA = 4,  /* feature-unused flags of the level last processed (after update): n_h x d */
    ORC_X_SD = 5,     /* split decisions of the level last processed: n_h */
    ORC_X_L = 6,      /* per-sample leaf one-hot (arithmetic), n_h x N8, node-major */
    ORC_X_SCORE = 7,  /* masked scores of the level last processed: n_h x d */
    ORC_X_C_PAPER = 8 /* the same statistics in the paper's (1+K) x 2d layout per node */
};

/* ---- context ------------------------------------------------------------ */
/* seed[0..2] = pairwise keys k1..k3, seed[3] = dealer key, seed[4] = owner key */
orc_ctx *orc_ctx_create(const uint64_t seed[5][4], uint32_t tau, uint32_t K);
void orc_ctx_destroy(orc_ctx *);
void orc_stats(const orc_ctx *, uint64_t *rounds, uint64_t wire_bytes[9]);
/* payload bits of the same messages, n*bits per message without rounding up to bytes */
void orc_stats_bits(const orc_ctx *c, uint64_t wire_bits[9]);
/* heuristic by reconstruction: bytes the parties sent to the scorer [0] and got back [1] */
void orc_stats_scorer(const orc_ctx *c, uint64_t bytes[2]);
void orc_stats_reset(orc_ctx *);
uint32_t orc_op_counter(const orc_ctx *);
void orc_set_threads(int n); /* OpenMP threads for the element loops; 0 = default */
int orc_get_threads(void);

/* ---- randomness (exported so that tests can pin it) ---------------------- */
void orc_chacha_block(const uint32_t key[8], uint32_t c12, uint32_t c13, uint32_t c14,
                      uint32_t c15, int rounds, uint32_t out[16]);
void orc_chacha_quarter(uint32_t v[4]);
uint64_t orc_prf_word(const orc_ctx *, int key_index, uint32_t op, uint32_t stream, uint64_t j);
/* zero sharing of element e: arithmetic (sum 0) or Boolean (xor 0) */
void orc_zero_sharing(const orc_ctx *, uint32_t op, uint32_t stream, uint64_t e, int boolean,
                      uint64_t alpha[3]);
/* dealer material of element e: out[0..2]=r comps, [3..5]=rho comps (Boolean),
 * [6..8]=beta Boolean comps, [9..11]=beta arithmetic comps, [12]=r, [13]=beta */
/* daBit of test e of an equality grid: out = Boolean components [0..2], arithmetic components [3..5], the bit [6] */
void orc_dabit_grid(const orc_ctx *c, uint32_t op, uint64_t e, uint64_t out[7]);
void orc_dealer(const orc_ctx *, uint32_t op, uint64_t e, uint64_t out[14]);

/* ---- sharing ------------------------------------------------------------- */
void orc_share_a(orc_ctx *, const uint64_t *plain, size_t n, uint64_t *comp);
void orc_reconstruct_a(const uint64_t *comp, size_t n, uint64_t *plain);
void orc_reconstruct_b(const uint64_t *comp, size_t n, uint64_t *plain);

/* ---- building blocks (each consumes one op) ------------------------------ */
void orc_mult(orc_ctx *, const uint64_t *x, const uint64_t *y, size_t n, uint64_t *z);
/* Boolean result bit of [x == y] (y public, may be NULL = 0) */
void orc_eq_b(orc_ctx *, const uint64_t *x, const uint64_t *y_pub, size_t n, uint64_t *e_bool);
/* arithmetic 0/1 sharing of [x == y] */
void orc_eq_a(orc_ctx *, const uint64_t *x, const uint64_t *y_pub, size_t n, uint64_t *e_arith);
/* arithmetic 0/1 sharing of [x >= y] for shared x, y with |x-y| < 2^63 */
void orc_ge_a(orc_ctx *, const uint64_t *x, const uint64_t *y, size_t n, uint64_t *g_arith);
/* z[i] = W[u[i]] (0 if u[i] outside [0,w)), W shared of length w, u shared of length n */
void orc_oaa(orc_ctx *, const uint64_t *W, size_t w, const uint64_t *u, size_t n, uint64_t *z);
/* exact fixed-point quotient floor(S*2^tau / Q) for 0 <= S <= Q, Q > 0 */
void orc_div(orc_ctx *, const uint64_t *S, const uint64_t *Q, size_t n, uint64_t *q);

/* ---- training ------------------------------------------------------------ */
orc_train *orc_train_create(orc_ctx *, const uint64_t *X /*N x d comps*/,
                            const uint64_t *Y /*N x K comps*/, size_t N, uint32_t d,
                            uint32_t H);
void orc_train_destroy(orc_train *);
/* The array access as the paper prints it (Sec. V-A): a SelectShare of its own for every
 * array element (conversion with the opened value sent as a ring element, product with a
 * reshare), local sum.  N(4l-1) bits for N = w*n, log l + 3 rounds.  Same reconstructed z. */
void orc_oaa_literal(orc_ctx *c, const uint64_t *W, size_t w, const uint64_t *u, size_t n, uint64_t *z);
/* Learning protocol of the following levels as printed (Sec. V-B, Alg. "Oblivious
 * Learning"): array access over the whole tree array, per-element SelectShare of the
 * per-sample counter arrays and local accumulation.  Same reconstructed state; X_L is not
 * exported in this mode.  For small inputs only. */
void orc_train_set_literal(orc_train *t, int literal);
/* Data partition of the following levels by products with the previous level's per-sample
 * leaf one-hot instead of two array accesses per sample (see partition_matmul in the source):
 * same M for every sample that sits in a real leaf, same tree, N*d*64 + N*64 bits per party
 * instead of N*(n_{h-1} + d)*128.  Needs the previous level to have run in this object. */
void orc_train_set_partition(orc_train *t, int by_products);
/* Heuristic computation of the following levels by reconstruction (host analogue of the
 * TEE-based protocol of Sec. V-B: a scorer reconstructs C, gamma, F, scores in the clear with
 * the same fixed-point rule and hands back fresh sharings) instead of the MPC protocol. */
void orc_train_set_heuristic(orc_train *t, int by_reconstruction);
int orc_train_level(orc_ctx *, orc_train *, uint32_t h);
/* level H: partition, class totals, labels. feat: 2^H-1 comps, leaf: 2^H comps */
int orc_train_finish(orc_ctx *, orc_train *, uint64_t *feat, uint64_t *leaf);
size_t orc_train_export_size(const orc_train *, int what);
int orc_train_export(const orc_train *, int what, uint64_t *comp);
/* overwrite M and the node arrays of level h (T level h-1, F level h, C, gamma) so that a
 * single level can be run from a synthetic state */
int orc_train_import(orc_train *, uint32_t h, const uint64_t *M, const uint64_t *Tprev,
                     const uint64_t *Flevel, const uint64_t *C, const uint64_t *gamma);

/* ---- inference ----------------------------------------------------------- */
/* feat: 2^H-1 comps, thr: 2^H-1 comps or NULL (binary mode), leaf: 2^H comps,
 * I: N_I x d comps (row-major), R: N_I comps */
int orc_infer_batch(orc_ctx *, const uint64_t *feat, const uint64_t *thr, const uint64_t *leaf,
                    uint32_t H, const uint64_t *I, size_t NI, uint32_t d, uint64_t *R);

/* Sampled rows of a large batch: I holds the listed rows only (nrows x d comps, row-major),
 * rows[] their indices in the batch of NI instances, R receives nrows comps. */
int orc_infer_rows(orc_ctx *, const uint64_t *feat, const uint64_t *thr, const uint64_t *leaf,
                   uint32_t H, const uint64_t *I, size_t NI, uint32_t d, const size_t *rows,
                   size_t nrows, uint64_t *R);

#ifdef __cplusplus
}
#endif
#endif
