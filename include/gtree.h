/*
 * gtree.h — C ABI of the MI355X (gfx950) library for the hot path of GTree
 * (arXiv 2305.00645): three-party semi-honest decision-tree training and
 * inference on 2-out-of-3 replicated secret shares over Z_2^64.
 *
 * All three computing parties are simulated on ONE GPU.  Each party has its own
 * share buffers and keys; a message between parties is a store into a message
 * region on the device (the workgroup's LDS) that the receiving party's wavefront
 * loads after a barrier; rounds and wire bytes are counted.  Offline material (edaBits, daBits) is derived from a
 * dealer key inside the kernels, because the paper times only the online phase
 * (Sec. VI).  This is a performance simulation, not a deployable secure system.
 *
 * Conventions
 *  - Every pointer in a gt_shares is DEVICE memory, 8-byte aligned, owned by the
 *    caller, of `n` 64-bit words.  party[p].own holds component p, party[p].next
 *    component p+1 mod 3 (Sec. II-B: P_i holds (x_i, x_{i+1})).
 *  - `plain` buffers are device memory too.
 *  - Calls only enqueue work on the context's HIP stream and return; gt_stats_get,
 *    gt_prof_get, gt_stats_reset and the destroy calls wait for it.  Calls on one
 *    context must not overlap.  Device memory is allocated by the create/import calls;
 *    gt_train_level, gt_train_finish and gt_train_reset allocate nothing (the tree that
 *    gt_train_finish returns uses buffers made by gt_train_create, unless the tree of an
 *    earlier finish of the same object is still alive); gt_infer_batch, gt_oaa and
 *    gt_div keep a workspace in the context that grows on first use or for a larger
 *    batch (then they wait for the stream and allocate).
 *  - Return value 0 = success, negative = error; nothing is thrown or aborted.
 *    After an error the output buffers are unspecified; the context stays usable
 *    unless the error is GT_EHIP.
 *  - Every protocol invocation consumes operation ids from the context's
 *    counter; shares are a pure function of (keys, operation id, element index),
 *    so results do not depend on launch shapes.  Two contexts created with the
 *    same parameters and driven with the same calls produce identical shares.
 *  - Public values (leaked by design, Sec. I): all sizes, depths, tau, K.
 */
#ifndef GTREE_H
#define GTREE_H
#include <stddef.h>
#include <stdint.h>
#ifdef __cplusplus
extern "C" {
#endif

#define GT_OK 0
#define GT_EINVAL (-1) /* null pointer, zero/oversized dimension, bad selector */
#define GT_ENOMEM (-2) /* device allocation failed */
#define GT_ESTATE (-3) /* level called out of order, object used after finish */
#define GT_EHIP (-4)   /* a HIP runtime call or kernel launch failed */

#define GT_MAX_DEPTH 16u       /* decision levels of a tree */
#define GT_MAX_N (1u << 20)    /* training samples: keeps Gini terms below 2^40 */
#define GT_MAX_K 16u           /* classes */
#define GT_MAX_TAU 20u         /* fractional bits of the Gini quotients */
#define GT_STATIC_MAX_N (1u << 18) /* rows of gt_oaa_static */

typedef struct gt_ctx gt_ctx;     /* keys, operation counter, stream, scratch for partial sums */
typedef struct gt_train gt_train; /* per-party shares of T, F, M, C, gamma and the data */
typedef struct gt_tree gt_tree;   /* per-party shares of feature ids [, thresholds], labels */

typedef struct { uint64_t *own, *next; } gt_plane2;
typedef struct { gt_plane2 party[3]; size_t n; } gt_shares;

/* rounds: protocol rounds; wire_bytes[a][b]: bytes party a sent to party b, each
 * message of n elements of w bits counted as ceil(n*w/8) from the public sizes on the
 * host; wire_bits_dev[a][b]: payload bits of the same messages counted by the kernels
 * where they store them (per element that exists, so padding lanes count nothing);
 * kernel_ms: GPU time of the launches, from HIP events on the context's stream
 * (only with GT_FLAG_PROFILE, otherwise 0). */
typedef struct {
    uint64_t rounds; uint64_t wire_bytes[3][3]; uint64_t wire_bits_dev[3][3];
    uint64_t scorer_bytes[2]; /* heuristic by reconstruction: bytes the parties sent to the scorer, and got back */
    double kernel_ms;
} gt_stats;

/* tau: fractional bits of the fixed-point Gini quotients (Sec. V-B); K: classes;
 * seed[0..2]: pairwise keys k1..k3 (party p uses seed[p], seed[p+1 mod 3], Sec. III),
 * seed[3]: dealer key for offline material, seed[4]: data owner / query user key;
 * hip_stream: a hipStream_t or NULL for the default stream. */
typedef struct {
    uint32_t tau, K;
    uint64_t seed[5][4];
    uint32_t flags; /* 0 or GT_FLAG_PROFILE */
    void *hip_stream;
} gt_params;

/* GT_FLAG_PROFILE: bracket every kernel launch with a pair of HIP events on the
 * context's stream and accumulate time and launch count per kernel class; the pairs
 * are read when the times are asked for (gt_prof_get, gt_stats_get). */
#define GT_FLAG_PROFILE 1u
/* GT_FLAG_LEVELWISE_INFER: gt_infer_batch runs level by level (two equality-grid launches
 * per level with the node index in device memory) instead of one launch that carries every
 * instance through all levels; same shares, kept for comparison. */
#define GT_FLAG_LEVELWISE_INFER 2u
/* tuning knob of the one-launch inference: instances per workgroup 16 / 32 / 64 instead of
 * the choice made from the batch size (flags |= GT_FLAG_INFER_TILE(16)) */
#define GT_FLAG_INFER_TILE_MASK 0x300u
#define GT_FLAG_INFER_TILE(n) ((n) == 16 ? 0x100u : (n) == 32 ? 0x200u : (n) == 64 ? 0x300u : 0u)
enum {
    GT_KC_SHARE = 0, /* share / reconstruct */
    GT_KC_MULT = 1,  /* elementwise products with reshare */
    GT_KC_EQGRID = 2,/* equality grid with inner product against a shared array (array access over a
                        tree level or the leaf labels) */
    GT_KC_COUNT = 3, /* statistics contraction */
    GT_KC_SMALL = 4, /* per-node protocols: division, arg-max, updates */
    GT_KC_LOCAL = 5, /* copies, transposes, fills (no messages) */
    GT_KC_EQGRID_ROWS = 6,  /* equality grid with inner product against the sample's own row */
    GT_KC_EQGRID_STORE = 7, /* equality grid that stores the per-sample leaf one-hot */
    GT_KC_INFER = 8,        /* one-launch inference */
    GT_KC_PARTMM = 9,       /* data partition by products on the matrix cores */
    GT_KC_N = 10
};
typedef struct { double ms[GT_KC_N]; uint64_t launches[GT_KC_N]; } gt_prof;

int gt_ctx_create(gt_ctx **out, const gt_params *params);
/* per-class kernel times since creation or the last gt_stats_reset (zeros without
 * GT_FLAG_PROFILE); synchronises the stream */
int gt_prof_get(gt_ctx *ctx, gt_prof *out);
int gt_ctx_destroy(gt_ctx *ctx);
/* accumulated counters since creation or the last reset; synchronises the stream */
int gt_stats_get(gt_ctx *ctx, gt_stats *out);
int gt_stats_reset(gt_ctx *ctx);
uint32_t gt_op_counter(const gt_ctx *ctx);
const char *gt_strerror(int code);

/* ---- sharing (Sec. II-B, Share^A / Rec^A; the data owner's and query user's role) */
/* out.party[p] receive components (p, p+1) of a fresh sharing of plain[0..n). */
int gt_share_a(gt_ctx *ctx, const uint64_t *plain_dev, size_t n, const gt_shares *out);
/* plain[e] = x1 + x2 + x3, read as party 0's two components plus party 2's first. */
int gt_reconstruct_a(gt_ctx *ctx, const gt_shares *in, uint64_t *plain_dev, size_t n);

/* ---- building blocks (Sec. II-B multiplication; Sec. V-A equality test and
 *      oblivious array access); each consumes one operation id (gt_div: tau+1) */
int gt_mult(gt_ctx *ctx, const gt_shares *x, const gt_shares *y, size_t n, const gt_shares *z);
/* z = arithmetic 0/1 sharing of [x == y]; y_pub_dev: public operand or NULL for 0 */
int gt_eq_a(gt_ctx *ctx, const gt_shares *x, const uint64_t *y_pub_dev, size_t n, const gt_shares *z);
/* z = arithmetic 0/1 sharing of [x >= y]; requires |x - y| < 2^63 as signed numbers */
int gt_ge_a(gt_ctx *ctx, const gt_shares *x, const gt_shares *y, size_t n, const gt_shares *z);
/* z[i] = W[u[i]], 0 when u[i] is outside [0, w); linear scan over all w entries.  The w
 * equality tests of a row compare one shared index with public constants: the index is
 * masked and opened once per row (64 bits), every entry then costs its AND rounds and its
 * conversion (63 + 1 bits), the selected entry one reshare (64 bits); 9 rounds. */
int gt_oaa(gt_ctx *ctx, const gt_shares *W, size_t w, const gt_shares *u, size_t n, const gt_shares *z);
/* gt_oaa for callers that cannot allocate device memory (code under HIP graph capture,
 * serving loops, harnesses that forbid it): same arguments, same shares, same operation
 * id, but the partial inner products live in a static device array of the library
 * (6 * GT_STATIC_MAX_N words = 12 MiB per GPU, held until the process ends) instead of
 * the context's workspace, the array is cleared by a fill kernel, and no allocating call
 * of any kind is made.  n > GT_STATIC_MAX_N returns GT_EINVAL.  All contexts on one GPU
 * share the array: calls that overlap on one GPU race. */
int gt_oaa_static(gt_ctx *ctx, const gt_shares *W, size_t w, const gt_shares *u, size_t n, const gt_shares *z);
/* gt_oaa run as the paper prints it (Sec. V-A, Alg. "Oblivious Array Access"): every one of
 * the N = w*n array elements goes through a SelectShare of its own (conversion with the
 * opened value counted as a ring element, product with a reshare), the selected elements are
 * added up locally: N(4l-1) bits per party, log l + 3 rounds, same reconstructed z.  For
 * setting the counted bytes beside the paper's formula; one element per lane, small inputs. */
int gt_oaa_literal(gt_ctx *ctx, const gt_shares *W, size_t w, const gt_shares *u, size_t n, const gt_shares *z);
/* q = floor(S * 2^tau / Q) for 0 <= S <= Q < 2^40, Q > 0 (restoring division) */
int gt_div(gt_ctx *ctx, const gt_shares *S, const gt_shares *Q, size_t n, const gt_shares *q);

/* ---- training (Sec. V-B: learning, heuristic computation, node split) ---- */
/* X: N x dcols row-major 0/1 candidate columns, Y: N x K one-hot class indicators.
 * Copies the data into the library's sample-contiguous layout and computes the
 * one-time products X[i][k]*Y[i][c].  max_depth = H decision levels; level H holds
 * labels.  N <= GT_MAX_N, 1 <= dcols, H <= GT_MAX_DEPTH. */
int gt_train_create(gt_ctx *ctx, const gt_shares *X, const gt_shares *Y, size_t N,
                    uint32_t dcols, uint32_t max_depth, gt_train **out);
/* Start a new job in an existing gt_train of the same N, dcols, depth: copy X, Y in,
 * recompute the one-time products, reset M, T, F, C, gamma.  Allocates nothing. */
int gt_train_reset(gt_ctx *ctx, gt_train *tr, const gt_shares *X, const gt_shares *Y);
/* one level h (0 <= h < H, in order): data partition (h > 0), per-sample leaf
 * flags, class counts for every (node, candidate), Gini scores by exact
 * fixed-point division, first arg-max, updates of gamma, F, C, T. */
int gt_train_level(gt_ctx *ctx, gt_train *tr, uint32_t h);
/* level H: partition, class totals, majority label per node.  The tree's shares
 * are copied into a new gt_tree (binary mode). */
int gt_train_finish(gt_ctx *ctx, gt_train *tr, gt_tree **out);
/* Heuristic computation of the following levels by reconstruction instead of the MPC
 * protocol: the host analogue of the TEE-based protocol (Sec. V-B, Alg. "Oblivious
 * Heuristic Computation via TEE"), as a debugging aid and an upper bound for the MPC
 * heuristic.  A scorer (a fourth role, played by a kernel that reads all three components)
 * reconstructs the level's C, gamma and F, computes scores, first maximum, gamma and node
 * types in the clear with the same fixed-point rule, and hands back fresh sharings under
 * the dealer's key.  Same reconstructed SD, gamma, F, T as the MPC heuristic; two rounds.
 * There is no enclave here: the scorer sees the statistics in the clear. */
int gt_train_set_heuristic(gt_train *tr, int by_reconstruction);
/* Data partition of the following levels by products with the previous level's per-sample
 * leaf one-hot (a variant beyond the paper's listing, which makes two array accesses per
 * sample): OH[r][k] = [T_{h-1}[r] = k] (n_{h-1}*d equality tests, sample-independent),
 * sel[k][i] = sum_r L[r][i] OH[r][k], Dval[i] = sum_k sel[k][i] X[i][k], M <- 2M + Dval + 1.
 * Per party N*d*64 + N*64 bits instead of N*(n_{h-1} + d)*64 + 4*N*64, 10 rounds instead
 * of 18.  Same tree and statistics; M equals the paper's for every sample in a real leaf (a
 * sample below a node that stopped being one keeps going left).  The level before must have
 * run in this object (GT_ESTATE after gt_train_import).  Depth at most 13.  The first call
 * allocates the operand buffers (48 * d * 2^(H-1) bytes). */
int gt_train_set_partition(gt_ctx *ctx, gt_train *tr, int by_products);
/* Learning protocol of the following levels as printed (Sec. V-B, Alg. "Oblivious
 * Learning"): array access over the whole tree array, a SelectShare per element of the
 * per-sample (1+K) x 2d counter arrays, local accumulation - instead of the level slice and
 * the fused inner products.  Same reconstructed state, the paper's message volume; meant
 * for small inputs (first call allocates 2^H * N8 shares; GT_X_L is not exported). */
int gt_train_set_literal(gt_ctx *ctx, gt_train *tr, int literal);
int gt_train_destroy(gt_train *tr);

enum {
    GT_X_T = 0,      /* 2^(H+1)-1 words */
    GT_X_F = 1,      /* 2^(H+1)-1 */
    GT_X_M = 2,      /* N */
    GT_X_C = 3,      /* statistics of the level last processed: n_h x (d*K+K),
                        [k*K+c] = count(column k = 1, class c), [d*K+c] = count(class c) */
    GT_X_GAMMA = 4,  /* n_h x d, after the update */
    GT_X_SD = 5,     /* n_h */
    GT_X_L = 6,      /* n_h x N8 (N padded to a multiple of 8), node-major */
    GT_X_SCORE = 7,  /* n_h x d masked scores */
    GT_X_C_PAPER = 8 /* the statistics in the (1+K) x 2d counter-array layout of Sec. V-B */
};
size_t gt_train_export_size(const gt_train *tr, int what);
int gt_train_export(gt_ctx *ctx, const gt_train *tr, int what, const gt_shares *out);
/* Overwrite the state so that level h can be run next: M (N words), the tree entries
 * of level h-1 (2^(h-1) words, ignored for h = 0), F, C and gamma of level h
 * (2^h, 2^h*(d*K+K), 2^h*d words). */
int gt_train_import(gt_ctx *ctx, gt_train *tr, uint32_t h, const gt_shares *M,
                    const gt_shares *Tprev, const gt_shares *Flevel, const gt_shares *C,
                    const gt_shares *gamma);

/* ---- inference (Sec. V-C) ------------------------------------------------ */
/* feat: 2^H-1 feature ids, thr: 2^H-1 thresholds or NULL (binary features),
 * leaf: 2^H labels.  The shares are copied. */
int gt_tree_import(gt_ctx *ctx, const gt_shares *feat, const gt_shares *thr,
                   const gt_shares *leaf, uint32_t depth, gt_tree **out);
int gt_tree_export(gt_ctx *ctx, const gt_tree *tree, const gt_shares *feat, const gt_shares *leaf);
int gt_tree_destroy(gt_tree *tree);
/* I: N_I x d row-major.  Binary mode: the fetched feature value is the branch bit.
 * Threshold mode: branch bit = [value > threshold], values and thresholds in
 * [0, 2^62).  R: N_I labels. */
int gt_infer_batch(gt_ctx *ctx, const gt_tree *tree, const gt_shares *I, size_t N_I,
                   uint32_t d, const gt_shares *R_out);

/* ---- forests (Sec. VI, inference results: for deep trees a random forest of shallow
 * trees may serve better).  ntrees trees of the same depth and mode are evaluated on the
 * same batch in ONE launch: R[t*N_I + i] = label of instance i by tree t.  Shares, operation
 * ids, rounds and bytes are those of gt_infer_batch called for tree 0, 1, ... in this
 * order.  gt_forest_create copies the trees' shares (the trees may be destroyed afterwards);
 * how the per-tree labels are combined (vote) is left to the caller. */
typedef struct gt_forest gt_forest;
int gt_forest_create(gt_ctx *ctx, const gt_tree *const *trees, size_t ntrees, gt_forest **out);
int gt_forest_destroy(gt_forest *forest);
int gt_infer_forest(gt_ctx *ctx, const gt_forest *forest, const gt_shares *I, size_t N_I,
                    uint32_t d, const gt_shares *R_out);

#ifdef __cplusplus
}
#endif
#endif
