// Host side of the C ABI declared in include/gtree.h: argument checks, device
// state, the operation schedule of each protocol, message accounting, launches.
#include "gtree.h"
#include "gt_kernels.hpp"
#include "gt_infer.hpp"
#include "gt_partmm.hpp"
#include <algorithm>
#include <cstdio>
#include <cstring>
#include <new>
#include <vector>

#define GT_MAX_BLOCKS 4096u

// Scratch of the entry point that allocates nothing (gt_oaa_static): the partial inner
// products of an array access whose columns are split over workgroups, six planes of
// GT_STATIC_MAX_N words.  One copy per GPU, held until the process ends.  In host code the
// array's name is not a device address: its address on a device is taken once per device
// with hipGetSymbolAddress (gt_ctx_create, with that device current) and kept below.
static __device__ __align__(256) u64 scratch[6 * (size_t)GT_STATIC_MAX_N];
#define GT_MAX_DEVICES 64
static u64 *g_scratch_ptr[GT_MAX_DEVICES];

#define HIPCHK(x)                                                                             \
    do { hipError_t e_ = (x); if (e_ != hipSuccess) {                                         \
        fprintf(stderr, "gtree: %s failed: %s (%s:%d)\n", #x, hipGetErrorString(e_), __FILE__, __LINE__); \
        return GT_EHIP; } } while (0)
#define GTCHK(x) do { int r_ = (x); if (r_ != GT_OK) return r_; } while (0)

// ---------------------------------------------------------------------------------
struct DSh {                 // a shared vector in device memory: six planes in one allocation
    u64 *base = nullptr;
    size_t n = 0;
    P6 v{};
};

struct gt_ctx {
    u32 tau, K;
    u32 op;
    hipStream_t stream;
    u32 *keys_d;
    u64 *wire_d;              // GT_WIRE_SLOTS x six counters filled by the kernels: payload bits party p sent to p+1 [2p], to p-1 [2p+1]
    unsigned resident;        // workgroups of 192 lanes that fit on the device at once
    gt_stats acc;
    bool profile;
    bool levelwise_infer;     // GT_FLAG_LEVELWISE_INFER
    int infer_lgi;            // forced log2 of the instances per workgroup of k_infer (0: chosen from the batch size)
    std::vector<hipEvent_t> ev_pool;   // GT_FLAG_PROFILE: a pair of events per launch, resolved when the times are read
    size_t ev_used;
    std::vector<int> ev_cls;
    gt_prof prof;
    DSh ws[5];                // inference workspace, grown on demand, kept between calls
    DSh divrem;               // remainders of gt_div, grown on demand, kept between calls
    u64 *dacc;                // partial inner products of split equality grids
    size_t dacc_words;
    u64 *scratch_d;           // this device's copy of the static scratch array
    bool noalloc;             // inside gt_oaa_static: nothing may be allocated
};

// Buffers of the tree that gt_train_finish hands out, allocated with the training
// object so that finishing a job allocates nothing.  The slot is shared by the training
// object and the tree made from it; whoever is destroyed last frees it.
struct TreeSlot { DSh feat, leaf; bool in_use = false, orphan = false; };

struct gt_tree {
    u32 H;
    bool has_thr;
    DSh feat, thr, leaf;
    TreeSlot *slot;           // non-null: feat and leaf are the slot's buffers
};

struct gt_forest {             // trees of one depth and mode, their shares tree after tree
    u32 H, ntrees;
    bool has_thr;
    DSh feat, thr, leaf;
};

struct gt_train {
    size_t N, N8;
    u32 d, K, H, CW, level, last, P2;
    bool finished;
    bool part_matmul;                // data partition by products with the previous level's leaf one-hot
    u32 lt_level;                    // level whose leaf one-hot the limb tiles LQ hold, or ~0u
    DSh OH;                          // partition by products: one-hot of the split decisions
    unsigned char *OHL;              // ... and its limb bytes, the matrix cores' operand
    bool literal;                    // learning protocol as printed (whole-tree scans, per-element SelectShare)
    DSh LB;                          // literal mode: per-sample leaf flags as Boolean bits, n_h x N8
    u64 *lit_acc;                    // literal mode: local sums, max(6*N8, 6*nmax*(1+K)*2d) words
    bool hc_open;                    // heuristic computation by reconstruction instead of the MPC protocol
    u64 *hcp;                        // the scorer's plain results: SD, gamma, F node, F children, split, scores
    bool fresh_import;               // state was imported and no level has run since: nothing to export for "last"
    TreeSlot *slot;
    DSh XT, YT;                      // [k][i], [c][i]: sample-contiguous copies of the inputs
    unsigned char *LQ, *BQ;          // limb tiles: leaf one-hot (one matrix per component), columns (own+next, own) per party
    size_t nblk, Lrows, Brows;       // sample blocks of 32, row strides of the limb planes
    DSh M, T, F, C, Cn, gamma, Gn, isLeaf, SD, split;
    DSh S, Q, quo, rem, val[2], idx[2], tval, best, lab;
    DSh Clast, Glast, Slast;
    u64 *Zacc;
};

static size_t pad8(size_t n) { return (n + 7) & ~(size_t)7; }

static int dsh_alloc(DSh &s, size_t n, hipStream_t st)
{
    s.n = n;
    const size_t stride = pad8(n ? n : 1);           // planes start 64-byte aligned
    const size_t words = 6 * stride;
    if (hipMalloc(&s.base, words * 8) != hipSuccess) { s.base = nullptr; return GT_ENOMEM; }
    HIPCHK(hipMemsetAsync(s.base, 0, words * 8, st));
    for (int p = 0; p < 3; p++) { s.v.o[p] = s.base + (size_t)(2 * p) * stride; s.v.n[p] = s.base + (size_t)(2 * p + 1) * stride; }
    return GT_OK;
}
static void dsh_free(DSh &s) { if (s.base) (void)hipFree(s.base); s.base = nullptr; s.n = 0; }

static P6 off6(P6 a, size_t off) { for (int j = 0; j < 3; j++) { a.o[j] += off; a.n[j] += off; } return a; }

static bool shares_ok(const gt_shares *s, size_t n)
{
    if (!s) return false;
    if (n == 0) return true;
    if (s->n < n) return false;
    for (int p = 0; p < 3; p++) if (!s->party[p].own || !s->party[p].next) return false;
    return true;
}
static P6 to_p6(const gt_shares *s)
{
    P6 a;
    for (int p = 0; p < 3; p++) { a.o[p] = s->party[p].own; a.n[p] = s->party[p].next; }
    return a;
}

static unsigned blocks_for(u64 n, unsigned per)
{
    u64 b = (n + per - 1) / per;
    if (b < 1) b = 1;
    return (unsigned)std::min<u64>(b, GT_MAX_BLOCKS);
}
static unsigned tiles(u64 n) { return blocks_for(n, GT_LANES); }          // one element per lane
// eight elements per lane
static unsigned tiles8(u64 n) { return blocks_for((n + 7) / 8, GT_LANES); }

// ---- message accounting: one message of n elements of `bits` bits is ceil(n*bits/8)
// bytes; dir = +1 to the successor (opening), -1 to the predecessor (resharing).
static void wire_add(gt_ctx *c, int dir, u64 n, u64 bits)
{
    u64 bytes = (n * bits + 7) / 8;
    for (int p = 0; p < 3; p++) c->acc.wire_bytes[p][(p + dir + 3) % 3] += bytes;
}
static void acct_eq(gt_ctx *c, u64 n)
{
    wire_add(c, +1, n, 64);
    for (int k = 0; k < 6; k++) wire_add(c, -1, n, 32u >> k);
    c->acc.rounds += 7;
}
// equality grid: the masked index is opened once per row, the AND rounds run per test
static void acct_eq_grid(gt_ctx *c, u64 rows, u64 n)
{
    wire_add(c, +1, rows, 64);
    for (int k = 0; k < 6; k++) wire_add(c, -1, n, 32u >> k);
    c->acc.rounds += 7;
}
static void acct_ge(gt_ctx *c, u64 n)
{
    wire_add(c, +1, n, 64);
    for (int k = 0; k < 5; k++) wire_add(c, -1, n, 2 * (32u >> k));
    wire_add(c, -1, n, 1);
    c->acc.rounds += 7;
}
static void acct_b2a(gt_ctx *c, u64 n) { wire_add(c, +1, n, 1); c->acc.rounds += 1; }
static void acct_b2a_wide(gt_ctx *c, u64 n) { wire_add(c, +1, n, 64); c->acc.rounds += 1; }   // opened value sent as a ring element
static void acct_and1(gt_ctx *c, u64 n) { wire_add(c, -1, n, 1); c->acc.rounds += 1; }
static void acct_reshare(gt_ctx *c, u64 n, u64 words) { wire_add(c, -1, n, 64 * words); c->acc.rounds += 1; }

// Sum up the event pairs recorded so far (GT_FLAG_PROFILE).  Waits for the stream.
static int resolve_events(gt_ctx *c)
{
    if (c->ev_cls.empty()) return GT_OK;
    HIPCHK(hipStreamSynchronize(c->stream));
    for (size_t i = 0; i < c->ev_cls.size(); i++) {
        float t = 0.f;
        if (hipEventElapsedTime(&t, c->ev_pool[2 * i], c->ev_pool[2 * i + 1]) == hipSuccess) {
            c->prof.ms[c->ev_cls[i]] += t; c->prof.launches[c->ev_cls[i]] += 1; c->acc.kernel_ms += t;
        }
    }
    c->ev_cls.clear(); c->ev_used = 0;
    return GT_OK;
}

// End of an API call: the work is enqueued, nothing waits for it.  Launch errors that the
// runtime has already noticed are reported.
struct Timed {
    gt_ctx *c;
    explicit Timed(gt_ctx *ctx) : c(ctx) {}
    int finish(int rc)
    {
        if (rc == GT_OK && hipPeekAtLastError() != hipSuccess) { (void)hipGetLastError(); return GT_EHIP; }
        return rc;
    }
};

static KCommon kc(gt_ctx *c, u32 op) { KCommon k; k.keys = c->keys_d; k.op = op; k.wire = c->wire_d; return k; }

// Every kernel goes through here.  With GT_FLAG_PROFILE the launch is bracketed by a
// pair of events of its kernel class; the pairs are resolved when the API call ends.
template <typename Kern, typename... Args>
static int launch(gt_ctx *c, int cls, Kern kern, dim3 grid, dim3 block, Args... args)
{
    hipEvent_t e1 = nullptr;
    if (c->profile) {
        if (c->ev_used >= 16384) GTCHK(resolve_events(c));    // bound the pool
        if (c->ev_used + 2 > c->ev_pool.size() && c->noalloc) goto plain;   // no new events: this launch goes untimed
        if (c->ev_used + 2 > c->ev_pool.size())
            for (int i = 0; i < 64; i++) { hipEvent_t e; if (hipEventCreate(&e) != hipSuccess) return GT_EHIP; c->ev_pool.push_back(e); }
        hipEvent_t e0 = c->ev_pool[c->ev_used++];
        e1 = c->ev_pool[c->ev_used++];
        c->ev_cls.push_back(cls);
        (void)hipEventRecord(e0, c->stream);
    }
plain:
    hipLaunchKernelGGL(kern, grid, block, 0, c->stream, args...);
    if (e1) (void)hipEventRecord(e1, c->stream);
    return hipGetLastError() == hipSuccess ? GT_OK : GT_EHIP;
}
static dim3 g1(u64 n) { return dim3(blocks_for(n, 256)); }   // plain elementwise kernels
static const dim3 B256(256);
static dim3 gT(u64 N, u64 w) { return dim3((unsigned)std::min<u64>(((N + 31) / 32) * ((w + 31) / 32), 65535), 1, 6); }  // k_transpose

// ---------------------------------------------------------------------------------
extern "C" const char *gt_strerror(int code)
{
    switch (code) {
    case GT_OK: return "ok";
    case GT_EINVAL: return "invalid argument";
    case GT_ENOMEM: return "device allocation failed";
    case GT_ESTATE: return "call out of order";
    case GT_EHIP: return "HIP runtime error";
    default: return "unknown error";
    }
}

extern "C" int gt_ctx_create(gt_ctx **out, const gt_params *prm)
{
    if (!out || !prm) return GT_EINVAL;
    if (prm->K < 1 || prm->K > GT_MAX_K || prm->tau < 1 || prm->tau > GT_MAX_TAU) return GT_EINVAL;
    gt_ctx *c = new (std::nothrow) gt_ctx();
    if (!c) return GT_ENOMEM;
    c->noalloc = false; c->scratch_d = nullptr;
    c->op = 0; c->ev_used = 0; c->keys_d = nullptr; c->wire_d = nullptr; c->dacc = nullptr; c->dacc_words = 0; c->resident = 1024;
    memset(&c->acc, 0, sizeof c->acc); memset(&c->prof, 0, sizeof c->prof);
    c->profile = (prm->flags & GT_FLAG_PROFILE) != 0;
    c->levelwise_infer = (prm->flags & GT_FLAG_LEVELWISE_INFER) != 0;
    c->infer_lgi = 0;
    if (prm->flags & GT_FLAG_INFER_TILE_MASK) c->infer_lgi = 3 + (int)((prm->flags & GT_FLAG_INFER_TILE_MASK) >> 8);
    c->tau = prm->tau; c->K = prm->K; c->stream = (hipStream_t)prm->hip_stream;
    u32 keys[5][8];
    for (int k = 0; k < 5; k++)
        for (int i = 0; i < 4; i++) { keys[k][2 * i] = (u32)prm->seed[k][i]; keys[k][2 * i + 1] = (u32)(prm->seed[k][i] >> 32); }
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= GT_MAX_DEVICES) { delete c; return GT_EHIP; }
    if (!g_scratch_ptr[dev]) {                 // once per device, with that device current
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) { delete c; return GT_EHIP; }
        g_scratch_ptr[dev] = (u64 *)ptr;
    }
    c->scratch_d = g_scratch_ptr[dev];
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && cus > 0)
        c->resident = std::min<unsigned>(GT_MAX_BLOCKS, 4u * (unsigned)cus);
    if (hipMalloc(&c->keys_d, sizeof keys) != hipSuccess) { delete c; return GT_ENOMEM; }
    if (hipMalloc(&c->wire_d, 6 * GT_WIRE_SLOTS * sizeof(u64)) != hipSuccess) { (void)hipFree(c->keys_d); delete c; return GT_ENOMEM; }
    if (hipMemcpy(c->keys_d, keys, sizeof keys, hipMemcpyHostToDevice) != hipSuccess ||
        hipMemset(c->wire_d, 0, 6 * GT_WIRE_SLOTS * sizeof(u64)) != hipSuccess) {
        (void)hipFree(c->keys_d); (void)hipFree(c->wire_d); delete c; return GT_EHIP;
    }
    *out = c;
    return GT_OK;
}

extern "C" int gt_ctx_destroy(gt_ctx *c)
{
    if (!c) return GT_EINVAL;
    (void)hipStreamSynchronize(c->stream);
    for (hipEvent_t e : c->ev_pool) (void)hipEventDestroy(e);
    for (DSh &w : c->ws) dsh_free(w);
    dsh_free(c->divrem);
    if (c->dacc) (void)hipFree(c->dacc);
    (void)hipFree(c->wire_d);
    (void)hipFree(c->keys_d);
    delete c;
    return GT_OK;
}

extern "C" int gt_stats_get(gt_ctx *c, gt_stats *out)
{
    if (!c || !out) return GT_EINVAL;
    HIPCHK(hipStreamSynchronize(c->stream));
    GTCHK(resolve_events(c));
    u64 bits[6 * GT_WIRE_SLOTS];
    HIPCHK(hipMemcpy(bits, c->wire_d, sizeof bits, hipMemcpyDeviceToHost));
    memset(c->acc.wire_bits_dev, 0, sizeof c->acc.wire_bits_dev);
    for (int sl = 0; sl < GT_WIRE_SLOTS; sl++)
        for (int p = 0; p < 3; p++) {
            c->acc.wire_bits_dev[p][(p + 1) % 3] += bits[6 * sl + 2 * p];
            c->acc.wire_bits_dev[p][(p + 2) % 3] += bits[6 * sl + 2 * p + 1];
        }
    *out = c->acc;
    return GT_OK;
}
extern "C" int gt_stats_reset(gt_ctx *c)
{
    if (!c) return GT_EINVAL;
    GTCHK(resolve_events(c));
    HIPCHK(hipMemsetAsync(c->wire_d, 0, 6 * GT_WIRE_SLOTS * sizeof(u64), c->stream));
    memset(&c->acc, 0, sizeof c->acc); memset(&c->prof, 0, sizeof c->prof);
    return GT_OK;
}
extern "C" int gt_prof_get(gt_ctx *c, gt_prof *out)
{
    if (!c || !out) return GT_EINVAL;
    HIPCHK(hipStreamSynchronize(c->stream));
    GTCHK(resolve_events(c));
    *out = c->prof;
    return GT_OK;
}
extern "C" uint32_t gt_op_counter(const gt_ctx *c) { return c ? c->op : 0; }

// ---------------------------------------------------------------------------------
extern "C" int gt_share_a(gt_ctx *c, const uint64_t *plain, size_t n, const gt_shares *out)
{
    if (!c || !shares_ok(out, n) || (n && !plain)) return GT_EINVAL;
    Timed T(c);
    u32 op = c->op++;
    int rc = GT_OK;
    if (n) rc = launch(c, GT_KC_SHARE, k_share, g1((n + 7) / 8), B256, (const u32 *)c->keys_d, (int)GT_KEY_OWNER, op, plain, (u64)n, to_p6(out), (u64)0);
    return T.finish(rc);
}

extern "C" int gt_reconstruct_a(gt_ctx *c, const gt_shares *in, uint64_t *plain, size_t n)
{
    if (!c || !shares_ok(in, n) || (n && !plain)) return GT_EINVAL;
    Timed T(c);
    int rc = GT_OK;
    if (n) rc = launch(c, GT_KC_SHARE, k_reconstruct, g1(n), B256, to_p6(in), (u64)n, plain);
    return T.finish(rc);
}

static int copy6(gt_ctx *c, P6 dst, u64 doff, P6 src, u64 soff, u64 sstride, u64 n)
{
    if (!n) return GT_OK;
    return launch(c, GT_KC_LOCAL, k_copy, g1(n), B256, dst, doff, src, soff, sstride, n);
}

// ---- building blocks ---------------------------------------------------------------
static int do_mult(gt_ctx *c, int mode, MultArgs a)
{
    a.c = kc(c, c->op++);
    if (a.n) {
        dim3 g(tiles8(a.n));
        if (mode == 0) return launch(c, GT_KC_MULT, k_mult<0>, g, GT_BLOCK, a);
        return launch(c, GT_KC_MULT, k_mult<2>, g, GT_BLOCK, a);
    }
    return GT_OK;
}

extern "C" int gt_mult(gt_ctx *c, const gt_shares *x, const gt_shares *y, size_t n, const gt_shares *z)
{
    if (!c || !shares_ok(x, n) || !shares_ok(y, n) || !shares_ok(z, n)) return GT_EINVAL;
    Timed T(c);
    MultArgs a{}; a.x = to_p6(x); a.y = to_p6(y); a.z = to_p6(z); a.n = n;
    int rc = do_mult(c, 0, a);
    acct_reshare(c, n, 1);
    return T.finish(rc);
}

static int do_eq(gt_ctx *c, bool bool_out, P6 x, u64 xoff, const u64 *ypub, u64 ysub, P6 z, u64 n)
{
    EqArgs a{}; a.c = kc(c, c->op++); a.x = x; a.xoff = xoff; a.ypub = ypub; a.ysub = ysub; a.z = z; a.n = n;
    if (n) GTCHK(bool_out ? launch(c, GT_KC_SMALL, k_eq<true>, dim3(tiles(n)), GT_BLOCK, a)
                          : launch(c, GT_KC_SMALL, k_eq<false>, dim3(tiles(n)), GT_BLOCK, a));
    acct_eq(c, n);
    if (!bool_out) acct_b2a(c, n);
    return GT_OK;
}

extern "C" int gt_eq_a(gt_ctx *c, const gt_shares *x, const uint64_t *ypub, size_t n, const gt_shares *z)
{
    if (!c || !shares_ok(x, n) || !shares_ok(z, n)) return GT_EINVAL;
    Timed T(c);
    return T.finish(do_eq(c, false, to_p6(x), 0, ypub, 0, to_p6(z), n));
}

extern "C" int gt_ge_a(gt_ctx *c, const gt_shares *x, const gt_shares *y, size_t n, const gt_shares *z)
{
    if (!c || !shares_ok(x, n) || !shares_ok(y, n) || !shares_ok(z, n)) return GT_EINVAL;
    Timed T(c);
    GeArgs a{}; a.c = kc(c, c->op++); a.x = to_p6(x); a.y = to_p6(y); a.z = to_p6(z); a.n = n;
    int rc = GT_OK;
    if (n) rc = launch(c, GT_KC_SMALL, k_ge, dim3(tiles(n)), GT_BLOCK, a);
    acct_ge(c, n); acct_b2a(c, n);
    return T.finish(rc);
}

// work items (tile, column range) per resident workgroup slot that the column split aims at: every range
// replays the row's edaBits and opening, so few long ranges beat many short ones (measured: 2 is best
// for the census-shaped and the 10^6-sample workloads alike; 4 costs 6 % of the former's training time)
#define GT_GRID_WANT 2
// the equality grid with its accounting
static int do_grid(gt_ctx *c, int mode, bool has_g, int ndot, GridArgs a, u64 *ext = nullptr, size_t ext_words = 0)
{
    a.c = kc(c, c->op++);
    a.ndot = ndot;
    const u64 nel = (u64)a.w * a.N;
    if (a.N && a.w) {
        // the leaf one-hot grid takes four adjacent columns per step when it can (whole
        // lines of the limb tiles per store); all other grids one column per step
        a.lgs = (mode == GM_STORE && a.w % 4 == 0) ? 4 : 6;
        const u64 kstep = GT_LANES >> a.lgs, nsteps = (a.w + kstep - 1) / kstep;
        // enough work items (tile, column range) to keep every resident workgroup slot busy for several rounds
        const u64 ntile = (a.N8 / 8 + (GT_LANES >> (6 - a.lgs)) - 1) >> a.lgs, want = (u64)GT_GRID_WANT * c->resident;
        u64 nkc = std::min<u64>(nsteps, std::max<u64>(1, (want + ntile - 1) / ntile));
        a.kchunk = (u32)(((nsteps + nkc - 1) / nkc) * kstep);
        a.nkc = (a.w + a.kchunk - 1) / a.kchunk;
        a.dacc = nullptr;
        if (mode != GM_STORE && a.nkc > 1) {
            const size_t need = (size_t)6 * a.N8;
            if (ext) {                         // caller-provided scratch: cleared by a fill kernel, never grown
                if (need > ext_words) return GT_EINVAL;
                GTCHK(launch(c, GT_KC_LOCAL, k_fill_words, g1(need), B256, ext, (u64)need, (u64)0));
                a.dacc = ext;
            } else if (c->dacc_words < need) {
                (void)hipStreamSynchronize(c->stream);
                if (c->dacc) (void)hipFree(c->dacc);
                c->dacc = nullptr; c->dacc_words = 0;
                if (hipMalloc(&c->dacc, need * 8) != hipSuccess) return GT_ENOMEM;
                c->dacc_words = need;
                // zero once: k_dot_fin leaves every word it has read at zero again
                HIPCHK(hipMemsetAsync(c->dacc, 0, need * 8, c->stream));
            }
            if (!ext) a.dacc = c->dacc;
        }
        // more workgroups than fit at once: the hardware balances them over the compute units
        dim3 g((unsigned)std::min<u64>(ntile * a.nkc, GT_MAX_BLOCKS));
        int rc;
        if (mode == GM_STORE && has_g) rc = launch(c, GT_KC_EQGRID_STORE, k_eqgrid<GM_STORE, true, 1>, g, GT_BLOCK, a);
        else if (mode == GM_STORE) rc = launch(c, GT_KC_EQGRID_STORE, k_eqgrid<GM_STORE, false, 1>, g, GT_BLOCK, a);
        else if (mode == GM_COMMON && ndot == 2) rc = launch(c, GT_KC_EQGRID, k_eqgrid<GM_COMMON, false, 2>, g, GT_BLOCK, a);
        else if (mode == GM_COMMON) rc = launch(c, GT_KC_EQGRID, k_eqgrid<GM_COMMON, false, 1>, g, GT_BLOCK, a);
        else rc = launch(c, GT_KC_EQGRID_ROWS, k_eqgrid<GM_ROWS, false, 1>, g, GT_BLOCK, a);
        GTCHK(rc);
        if (a.dacc) GTCHK(launch(c, GT_KC_SMALL, k_dot_fin, dim3(tiles8(a.N8)), GT_BLOCK, a));
    }
    acct_eq_grid(c, a.N, nel);
    if (has_g) acct_and1(c, nel);
    acct_b2a(c, nel);
    if (mode != GM_STORE) acct_reshare(c, a.N, ndot);
    return GT_OK;
}

extern "C" int gt_oaa(gt_ctx *c, const gt_shares *W, size_t w, const gt_shares *u, size_t n, const gt_shares *z)
{
    if (!c || !shares_ok(W, w) || !shares_ok(u, n) || !shares_ok(z, n) || w == 0 || w > 0xffffffffu) return GT_EINVAL;
    Timed T(c);
    GridArgs a{}; a.u = to_p6(u); a.base = 0; a.w = (u32)w; a.N = n; a.N8 = pad8(n);
    a.W1 = to_p6(W); a.w1off = 0; a.out = to_p6(z); a.epi = 0;
    return T.finish(do_grid(c, GM_COMMON, false, 1, a));
}

// The same array access with the partial inner products in the static scratch array:
// no allocation of any kind, for callers that cannot allocate (HIP graph capture, serving
// loops).  n is limited by the array's size.
extern "C" int gt_oaa_static(gt_ctx *c, const gt_shares *W, size_t w, const gt_shares *u, size_t n, const gt_shares *z)
{
    if (!c || !shares_ok(W, w) || !shares_ok(u, n) || !shares_ok(z, n) || w == 0 || w > 0xffffffffu) return GT_EINVAL;
    if (n > GT_STATIC_MAX_N) return GT_EINVAL;
    Timed T(c);
    GridArgs a{}; a.u = to_p6(u); a.base = 0; a.w = (u32)w; a.N = n; a.N8 = pad8(n);
    a.W1 = to_p6(W); a.w1off = 0; a.out = to_p6(z); a.epi = 0;
    c->noalloc = true;
    const int rc = do_grid(c, GM_COMMON, false, 1, a, c->scratch_d, (size_t)6 * GT_STATIC_MAX_N);
    c->noalloc = false;
    return T.finish(rc);
}

static int div_steps(gt_ctx *c, P6 S, P6 Q, P6 rem, P6 quo, u64 n)
{
    // tau+1 protocol steps, one operation id each, in one launch
    DivArgs a{}; a.c = kc(c, c->op); a.S = S; a.Q = Q; a.r = rem; a.quo = quo; a.n = n; a.nsteps = c->tau + 1;
    c->op += c->tau + 1;
    if (n) GTCHK(launch(c, GT_KC_SMALL, k_div, dim3(tiles(n)), GT_BLOCK, a));
    for (u32 t = 0; t <= c->tau; t++) { acct_ge(c, n); acct_b2a(c, n); acct_reshare(c, n, 1); }
    return GT_OK;
}

extern "C" int gt_div(gt_ctx *c, const gt_shares *S, const gt_shares *Q, size_t n, const gt_shares *q)
{
    if (!c || !shares_ok(S, n) || !shares_ok(Q, n) || !shares_ok(q, n)) return GT_EINVAL;
    Timed T(c);
    int rc = GT_OK;
    if (c->divrem.n < n) {                      // first use or a larger batch: grow the kept scratch
        (void)hipStreamSynchronize(c->stream);
        dsh_free(c->divrem);
        rc = dsh_alloc(c->divrem, n, c->stream);
    }
    if (rc == GT_OK) rc = div_steps(c, to_p6(S), to_p6(Q), c->divrem.v, to_p6(q), n);
    return T.finish(rc);
}

// ---- training -------------------------------------------------------------------------
static void train_free(gt_train *t)
{
    if (t->LQ) (void)hipFree(t->LQ);
    if (t->BQ) (void)hipFree(t->BQ);
    DSh *all[] = { &t->XT, &t->YT, &t->M, &t->T, &t->F, &t->C, &t->Cn, &t->gamma, &t->Gn, &t->isLeaf, &t->SD,
                   &t->split, &t->S, &t->Q, &t->quo, &t->rem, &t->val[0], &t->val[1], &t->idx[0], &t->idx[1],
                   &t->tval, &t->best, &t->lab, &t->Clast, &t->Glast, &t->Slast };
    for (DSh *s : all) dsh_free(*s);
    if (t->Zacc) (void)hipFree(t->Zacc);
    if (t->hcp) (void)hipFree(t->hcp);
    if (t->lit_acc) (void)hipFree(t->lit_acc);
    dsh_free(t->LB); dsh_free(t->OH);
    if (t->OHL) (void)hipFree(t->OHL);
    if (t->slot) {
        if (t->slot->in_use) t->slot->orphan = true;     // the tree made from it frees it
        else { dsh_free(t->slot->feat); dsh_free(t->slot->leaf); delete t->slot; }
    }
    delete t;
}

static LimbSet limbs_of(unsigned char *base, size_t nblk, size_t rows)
{
    LimbSet L;
    const size_t per = nblk * 8 * rows * 32;
    for (int p = 0; p < 3; p++) for (int m = 0; m < 2; m++) { L.m[p][m].base = base + (size_t)(2 * p + m) * per; L.m[p][m].rows = rows; }
    return L;
}
static LimbTri limbs_L(const gt_train *t)
{
    LimbTri L;
    const size_t per = t->nblk * 8 * t->Lrows * 32;
    for (int j = 0; j < 3; j++) { L.m[j].base = t->LQ + (size_t)j * per; L.m[j].rows = t->Lrows; }
    return L;
}
static LimbSet limbs_B(const gt_train *t) { return limbs_of(t->BQ, t->nblk, t->Brows); }

extern "C" int gt_train_destroy(gt_train *t) { if (!t) return GT_EINVAL; (void)hipDeviceSynchronize(); train_free(t); return GT_OK; }

// copy the data in, compute the one-time products, set the initial state (no allocation)
static int train_start(gt_ctx *c, gt_train *t, const gt_shares *X, const gt_shares *Y)
{
    const u32 d = t->d, K = t->K;
    const size_t N = t->N, N8 = t->N8, nmax = (size_t)1 << t->H, nodes = ((size_t)2 << t->H) - 1;
    // sample-contiguous copies of X and Y (Y goes behind the d*K product columns)
    GTCHK(launch(c, GT_KC_LOCAL, k_transpose, gT(N, d), B256, t->XT.v, to_p6(X), (u64)N, (u64)N8, d));
    GTCHK(launch(c, GT_KC_LOCAL, k_transpose, gT(N, K), B256, t->YT.v, to_p6(Y), (u64)N, (u64)N8, K));
    // one-time products X[i][k] * Y[i][c] and the class columns, as limb tiles
    XyArgs a{}; a.c = kc(c, c->op++); a.XT = t->XT.v; a.YT = t->YT.v; a.B = limbs_B(t); a.N = N; a.N8 = N8; a.K = K;
    a.ncol = d * K;
    const unsigned gy = std::min((a.ncol + 3) / 4, 4u);
    const unsigned gx = (unsigned)std::max<u64>(1, std::min<u64>((N8 / 8 + 15) / 16, GT_MAX_BLOCKS / gy));
    GTCHK(launch(c, GT_KC_MULT, k_xy, dim3(gx, gy), GT_BLOCK, a));
    acct_reshare(c, (u64)N * d * K, 1);
    GTCHK(launch(c, GT_KC_LOCAL, k_y_limbs, g1((N8 / 8) * K), B256, t->YT.v, limbs_B(t), (u64)N, (u64)N8, K, (u64)d * K));
    // M = 0, T = 0, the root is a leaf with empty statistics, no candidate used yet
    GTCHK(launch(c, GT_KC_LOCAL, k_fill_const, g1(N), B256, t->M.v, (u64)0, (u64)N, (u64)0));
    GTCHK(launch(c, GT_KC_LOCAL, k_fill_const, g1(nodes), B256, t->T.v, (u64)0, (u64)nodes, (u64)0));
    GTCHK(launch(c, GT_KC_LOCAL, k_fill_const, g1(nodes), B256, t->F.v, (u64)0, (u64)nodes, (u64)0));
    GTCHK(launch(c, GT_KC_LOCAL, k_fill_const, g1(nmax * t->CW), B256, t->C.v, (u64)0, (u64)(nmax * t->CW), (u64)0));
    GTCHK(launch(c, GT_KC_LOCAL, k_fill_const, dim3(1), B256, t->F.v, (u64)0, (u64)1, (u64)1));
    GTCHK(launch(c, GT_KC_LOCAL, k_fill_const, g1(d), B256, t->gamma.v, (u64)0, (u64)d, (u64)1));
    t->level = 0; t->last = 0; t->finished = false; t->fresh_import = false; t->lt_level = ~0u;
    return GT_OK;
}

extern "C" int gt_train_create(gt_ctx *c, const gt_shares *X, const gt_shares *Y, size_t N, uint32_t d,
                               uint32_t H, gt_train **out)
{
    if (!c || !out || N == 0 || N > GT_MAX_N || d == 0 || d > 65536 || H > GT_MAX_DEPTH) return GT_EINVAL;
    if (!shares_ok(X, N * d) || !shares_ok(Y, N * c->K)) return GT_EINVAL;
    Timed T(c);
    gt_train *t = new (std::nothrow) gt_train();
    if (!t) return T.finish(GT_ENOMEM);
    const u32 K = c->K;
    const size_t N8 = pad8(N), nmax = (size_t)1 << H, nodes = ((size_t)2 << H) - 1, CW = (size_t)d * K + K;
    size_t P2 = 1; while (P2 < d) P2 *= 2;
    t->N = N; t->N8 = N8; t->d = d; t->K = K; t->H = H; t->CW = (u32)CW; t->level = 0; t->last = 0; t->P2 = (u32)P2;
    t->finished = false; t->fresh_import = false; t->Zacc = nullptr; t->LQ = nullptr; t->BQ = nullptr; t->slot = nullptr;
    t->hc_open = false; t->hcp = nullptr; t->literal = false; t->lit_acc = nullptr; t->part_matmul = false; t->lt_level = ~0u; t->OHL = nullptr;
    hipStream_t s = c->stream;
    int rc = GT_OK;
    struct { DSh *v; size_t n; } plan[] = {
        { &t->XT, d * N8 }, { &t->YT, K * N8 }, { &t->M, N }, { &t->T, nodes }, { &t->F, nodes },
        { &t->C, nmax * CW }, { &t->Cn, nmax * CW }, { &t->gamma, nmax * d }, { &t->Gn, nmax * d }, { &t->isLeaf, nmax },
        { &t->SD, nmax }, { &t->split, nmax }, { &t->S, nmax * d * 2 }, { &t->Q, nmax * d * 2 },
        { &t->quo, nmax * d * 2 }, { &t->rem, nmax * d * 2 }, { &t->val[0], nmax * P2 }, { &t->val[1], nmax * P2 },
        { &t->idx[0], nmax * P2 }, { &t->idx[1], nmax * P2 }, { &t->tval, N }, { &t->best, nmax }, { &t->lab, nmax },
        { &t->Clast, nmax * CW }, { &t->Glast, nmax * d }, { &t->Slast, nmax * d },
    };
    for (auto &pl : plan) { rc = dsh_alloc(*pl.v, pl.n, s); if (rc != GT_OK) break; }
    if (rc == GT_OK) {
        t->slot = new (std::nothrow) TreeSlot();
        if (!t->slot) rc = GT_ENOMEM;
        if (rc == GT_OK) rc = dsh_alloc(t->slot->feat, nmax - 1, s);
        if (rc == GT_OK) rc = dsh_alloc(t->slot->leaf, nmax, s);
    }
    if (rc == GT_OK && hipMalloc(&t->Zacc, 3 * nmax * CW * 8) != hipSuccess) rc = GT_ENOMEM;
    if (rc == GT_OK && hipMalloc(&t->hcp, nmax * (2 * (size_t)d + 4) * 8) != hipSuccess) rc = GT_ENOMEM;
    // zero once: k_count_fin leaves every word it has read at zero again
    if (rc == GT_OK && hipMemsetAsync(t->Zacc, 0, 3 * nmax * CW * 8, s) != hipSuccess) rc = GT_EHIP;
    t->nblk = (N + 31) / 32;
    t->Lrows = std::max<size_t>(32, (nmax + 31) / 32 * 32);
    t->Brows = (CW + 63) / 64 * 64 + 64;
    const size_t lq = 3 * t->nblk * 8 * t->Lrows * 32, bq = 6 * t->nblk * 8 * t->Brows * 32;
    if (rc == GT_OK && hipMalloc(&t->LQ, lq) != hipSuccess) rc = GT_ENOMEM;
    if (rc == GT_OK && hipMalloc(&t->BQ, bq) != hipSuccess) rc = GT_ENOMEM;
    if (rc == GT_OK && (hipMemsetAsync(t->LQ, 0, lq, s) != hipSuccess || hipMemsetAsync(t->BQ, 0, bq, s) != hipSuccess)) rc = GT_EHIP;
    if (rc != GT_OK) { (void)hipStreamSynchronize(s); train_free(t); return T.finish(rc); }
    rc = train_start(c, t, X, Y);
    rc = T.finish(rc);
    if (rc != GT_OK) { train_free(t); return rc; }
    *out = t;
    return GT_OK;
}

extern "C" int gt_train_set_heuristic(gt_train *t, int by_reconstruction)
{
    if (!t) return GT_EINVAL;
    t->hc_open = by_reconstruction != 0;
    return GT_OK;
}

extern "C" int gt_train_reset(gt_ctx *c, gt_train *t, const gt_shares *X, const gt_shares *Y)
{
    if (!c || !t || !shares_ok(X, t->N * t->d) || !shares_ok(Y, t->N * t->K) || t->K != c->K) return GT_EINVAL;
    Timed T(c);
    return T.finish(train_start(c, t, X, Y));
}

// data partition: Tval = T_level(h-1)[M - base], Dval = X[i][Tval], M <- 2M + Dval + 1
static int partition(gt_ctx *c, gt_train *t, u32 h)
{
    const u64 wprev = (u64)1 << (h - 1), base = wprev - 1;
    GridArgs a{}; a.u = t->M.v; a.base = base; a.w = (u32)wprev; a.N = t->N; a.N8 = t->N8;
    a.W1 = t->T.v; a.w1off = base; a.out = t->tval.v; a.epi = 0;
    GTCHK(do_grid(c, GM_COMMON, false, 1, a));
    GridArgs b{}; b.u = t->tval.v; b.base = 0; b.w = t->d; b.N = t->N; b.N8 = t->N8;
    b.XT = t->XT.v; b.out = t->M.v; b.prev = t->M.v; b.epi = 1;
    return do_grid(c, GM_ROWS, false, 1, b);
}

static int leaf_onehot(gt_ctx *c, gt_train *t, u32 h)
{
    const u64 nh = (u64)1 << h, base = nh - 1;
    GTCHK(do_eq(c, true, t->F.v, base, nullptr, 1, t->isLeaf.v, nh));
    GridArgs a{}; a.u = t->M.v; a.base = base; a.w = (u32)nh; a.N = t->N; a.N8 = t->N8;
    a.g = t->isLeaf.v; a.L = limbs_L(t);
    GTCHK(do_grid(c, GM_STORE, true, 1, a));
    t->lt_level = h;
    return GT_OK;
}

// data partition by products: OH = onehot(T level h-1), sel = L^T OH, M <- 2M + <sel, X> + 1
static int partition_matmul(gt_ctx *c, gt_train *t, u32 h)
{
    if (t->lt_level != h - 1) return GT_ESTATE;         // needs the one-hot of the level just processed
    const u64 np = (u64)1 << (h - 1), base = np - 1, d = t->d, N = t->N;
    OnehotArgs oa{}; oa.c = kc(c, c->op++); oa.T = t->T.v; oa.OH = t->OH.v; oa.base = base; oa.n = np * d; oa.d = t->d;
    GTCHK(launch(c, GT_KC_SMALL, k_onehot, dim3(tiles(np * d)), GT_BLOCK, oa));
    acct_eq(c, np * d); acct_b2a(c, np * d);
    const u32 rpad = (u32)((np + 31) / 32 * 32), dpad = (t->d + 63) / 64 * 64;
    GTCHK(launch(c, GT_KC_LOCAL, k_oh_limbs, g1(6ull * dpad * rpad), B256, t->OH.v, t->OHL, (u32)np, t->d, rpad, dpad));
    PartMmArgs pa{}; pa.c = kc(c, c->op); c->op += 2;
    pa.L = limbs_L(t); pa.OHL = t->OHL; pa.XT = t->XT.v; pa.M = t->M.v; pa.N = N; pa.N8 = t->N8; pa.nblk = t->nblk;
    pa.d = t->d; pa.dpad = dpad; pa.rpad = rpad;
    GTCHK(launch(c, GT_KC_PARTMM, k_part_mm, dim3((unsigned)std::min<u64>(t->nblk, 16 * (u64)c->resident)), GT_BLOCK, pa));
    acct_reshare(c, N * d, 1);
    acct_reshare(c, N, 1);
    return GT_OK;
}

static int count(gt_ctx *c, gt_train *t, u32 h, bool totals_only)
{
    const u64 nh = (u64)1 << h, dK = (u64)t->d * t->K;
    const u32 ncol = totals_only ? t->K : t->CW;
    const u64 colbase = totals_only ? dK : 0;
    const u32 op = c->op++;
    CountArgs a{}; a.L = limbs_L(t); a.B = limbs_B(t); a.nblk = t->nblk; a.nh = (u32)nh; a.ncol = ncol;
    a.Zacc = t->Zacc;
    // wavefront arrangement: 4, 2 or 1 row tiles of 32 per workgroup, the rest over columns
    a.rt = nh > 64 ? 4 : (nh > 32 ? 2 : 1);
    a.nrowgrp = (u32)((nh + 32 * a.rt - 1) / (32 * a.rt));
    const u32 cper = 4 / a.rt;
    // groups of 64 columns; a remainder of at most 16 columns joins their launch as a
    // narrow group, one of 17 to 32 columns runs in a launch of its own with a 32-wide tile
    const u32 rem = ncol % 64, nfull = ncol / 64 + (rem > 32 ? 1 : 0);
    // (a remainder of at most 16 columns with no full group beside it - the class totals of the
    // label level - runs on the 16-wide tiles alone)
    const u32 narrow = (rem && rem <= 16) ? 1 : 0;
    const u32 ncg2 = (nfull + cper - 1) / cper, ncg1 = (rem && rem <= 32 && !narrow) ? 1 : 0;
    // narrow slots per chunk: a workgroup of the narrow group covers 64 rows (4 tiles of 16, all parties)
    const u32 nns = narrow ? (u32)((nh + 64ull * a.nrowgrp - 1) / (64ull * a.nrowgrp)) : 0;
    // sample chunk per workgroup: at most CT_CHUNK_BLOCKS blocks, shorter when that is needed to
    // give every compute unit several workgroups
    const u64 wgs_per_chunk = (u64)(3 * (ncg2 + ncg1) + nns) * a.nrowgrp;
    u64 want_chunks = ((u64)c->resident + wgs_per_chunk - 1) / wgs_per_chunk;
    u64 cb = (t->nblk + want_chunks - 1) / want_chunks;
    cb = std::max<u64>(8, std::min<u64>(CT_CHUNK_BLOCKS, cb));
    a.chunkblk = (u32)cb;
    a.nchunk = (u32)((t->nblk + cb - 1) / cb);
    if (nfull || narrow) {
        a.ncg = ncg2; a.ncoltiles = nfull; a.bcol0 = colbase; a.zcol0 = 0;
        a.nns = nns; a.nbcol0 = colbase + (u64)nfull * 64; a.nzcol0 = nfull * 64;
        GTCHK(launch(c, GT_KC_COUNT, k_count<2>, dim3(((a.nchunk + 7) / 8) * (3 * a.ncg + nns) * 8, 1, a.nrowgrp), B256, a));
    }
    if (ncg1) {
        a.nns = 0;
        a.ncg = 1; a.ncoltiles = 1; a.bcol0 = colbase + (u64)nfull * 64; a.zcol0 = nfull * 64;
        GTCHK(launch(c, GT_KC_COUNT, k_count<1>, dim3(((a.nchunk + 7) / 8) * 3 * 8, 1, a.nrowgrp), B256, a));
    }
    CountFinArgs f{}; f.c = kc(c, op); f.Zacc = t->Zacc; f.C = t->C.v; f.n = nh * ncol; f.ncol = ncol; f.CW = t->CW; f.colbase = colbase;
    GTCHK(launch(c, GT_KC_SMALL, k_count_fin, dim3(tiles(f.n)), GT_BLOCK, f));
    acct_reshare(c, nh * ncol, 1);
    return GT_OK;
}

static int select_max(gt_ctx *c, SelArgs a)
{
    a.c = kc(c, c->op++);
    if (a.n) GTCHK(launch(c, GT_KC_SMALL, k_select_max, dim3(tiles(a.n)), GT_BLOCK, a));
    acct_ge(c, a.n); acct_b2a(c, a.n); acct_reshare(c, a.n, 2);
    return GT_OK;
}

static int heuristic(gt_ctx *c, gt_train *t, u32 h)
{
    const u64 nh = (u64)1 << h, d = t->d, nq = nh * d * 2, ns = nh * d;
    PrepArgs pa{}; pa.c = kc(c, c->op++); pa.C = t->C.v; pa.S = t->S.v; pa.Q = t->Q.v; pa.n = nq; pa.d = t->d; pa.K = t->K; pa.CW = t->CW;
    GTCHK(launch(c, GT_KC_SMALL, k_score_prep, dim3(tiles(nq)), GT_BLOCK, pa));
    acct_reshare(c, nq, 2);
    // empty branch: make the divisor 1
    DSh &z = t->rem;    // scratch for the 0/1 sharing of [Q == 0]
    GTCHK(do_eq(c, false, t->Q.v, 0, nullptr, 0, z.v, nq));
    GTCHK(launch(c, GT_KC_LOCAL, k_add_inplace, g1(nq), B256, t->Q.v, z.v, nq));
    GTCHK(div_steps(c, t->S.v, t->Q.v, t->rem.v, t->quo.v, nq));
    GTCHK(launch(c, GT_KC_LOCAL, k_iota, g1(nh * t->P2), B256, t->idx[0].v, t->val[0].v, (u32)nh, t->P2, t->d));
    MaskArgs ma{}; ma.c = kc(c, c->op++); ma.quo = t->quo.v; ma.gamma = t->gamma.v; ma.score = t->Slast.v; ma.val = t->val[0].v; ma.n = ns; ma.d = t->d; ma.P2 = t->P2;
    GTCHK(launch(c, GT_KC_SMALL, k_mask_score, dim3(tiles(ns)), GT_BLOCK, ma));
    acct_reshare(c, ns, 1);
    int cur = 0;
    for (u64 len = t->P2; len > 1; len /= 2) {
        SelArgs sa{}; sa.vin = t->val[cur].v; sa.iin = t->idx[cur].v; sa.vout = t->val[cur ^ 1].v; sa.iout = t->idx[cur ^ 1].v;
        sa.n = nh * (len / 2); sa.len = (u32)len; sa.mode = 0;
        GTCHK(select_max(c, sa));
        cur ^= 1;
    }
    return copy6(c, t->SD.v, 0, t->idx[cur].v, 0, 1, nh);
}

static int update_flags(gt_ctx *c, gt_train *t, u32 h)
{
    const u64 nh = (u64)1 << h, base = nh - 1, d = t->d;
    GammaArgs ga{}; ga.c = kc(c, c->op++); ga.SD = t->SD.v; ga.gamma = t->gamma.v; ga.n = nh * d; ga.d = t->d;
    GTCHK(launch(c, GT_KC_SMALL, k_gamma, dim3(tiles(ga.n)), GT_BLOCK, ga));
    acct_eq(c, nh * d); acct_b2a(c, nh * d); acct_reshare(c, nh * d, 1);
    SplitArgs sa{}; sa.c = kc(c, c->op++); sa.C = t->C.v; sa.isLeaf = t->isLeaf.v; sa.F = t->F.v; sa.split = t->split.v;
    sa.n = nh; sa.base = base; sa.K = t->K; sa.CW = t->CW; sa.dK = (u64)t->d * t->K;
    GTCHK(launch(c, GT_KC_SMALL, k_split, dim3(tiles(nh)), GT_BLOCK, sa));
    acct_reshare(c, nh, 1); acct_eq(c, nh); acct_and1(c, nh); acct_b2a(c, nh); acct_reshare(c, nh, 1);
    return GT_OK;
}

// Heuristic by reconstruction: the scorer's kernel, then six sharings under the dealer's key
// (SD, gamma, F of the nodes, F of the children, split flags, masked scores), one operation
// id each.  Two rounds; bytes to and from the scorer are counted apart.
static int heuristic_open(gt_ctx *c, gt_train *t, u32 h)
{
    const u64 nh = (u64)1 << h, base = nh - 1, d = t->d, nmax = (u64)1 << t->H;
    u64 *SDp = t->hcp, *Gp = SDp + nmax, *Fn = Gp + nmax * d, *Fc = Fn + nmax, *Sp = Fc + nmax, *SCp = Sp + nmax;
    HcOpenArgs a{}; a.C = t->C.v; a.gamma = t->gamma.v; a.F = t->F.v; a.base = base; a.nh = (u32)nh; a.d = t->d; a.K = t->K; a.CW = t->CW;
    a.tau = c->tau; a.SD = SDp; a.G = Gp; a.Fn = Fn; a.Fc = Fc; a.Sp = Sp; a.SC = SCp;
    GTCHK(launch(c, GT_KC_SMALL, k_hc_open, dim3((unsigned)std::min<u64>(nh, 4096)), B256, a));
    c->acc.scorer_bytes[0] += 3 * 8 * nh * (t->CW + d + 1);
    c->acc.rounds += 1;
    struct { const u64 *plain; u64 n; P6 out; u64 off; } sh[6] = {
        { SDp, nh, t->SD.v, 0 }, { Gp, nh * d, t->gamma.v, 0 }, { Fn, nh, t->F.v, base }, { Fc, nh, t->best.v, 0 },
        { Sp, nh, t->split.v, 0 }, { SCp, nh * d, t->Slast.v, 0 } };
    for (int i = 0; i < 6; i++) {
        GTCHK(launch(c, GT_KC_SHARE, k_share, g1((sh[i].n + 7) / 8), B256, (const u32 *)c->keys_d, (int)GT_KEY_DEALER, c->op++,
                     sh[i].plain, sh[i].n, sh[i].out, sh[i].off));
        c->acc.scorer_bytes[1] += 3 * 2 * 8 * sh[i].n;
        if (i == 3) GTCHK(launch(c, GT_KC_LOCAL, k_children, g1(nh), B256, t->F.v, t->best.v, base, nh));
    }
    c->acc.rounds += 1;
    return GT_OK;
}

// Node split: T takes the split decisions, children inherit or clear the statistics.
static int node_split(gt_ctx *c, gt_train *t, u32 h)
{
    const u64 nh = (u64)1 << h, base = nh - 1, d = t->d, CW = t->CW;
    // keep this level's statistics and flags for export; T takes the split decisions
    GTCHK(copy6(c, t->Clast.v, 0, t->C.v, 0, 1, nh * CW));
    GTCHK(copy6(c, t->Glast.v, 0, t->gamma.v, 0, 1, nh * d));
    GTCHK(copy6(c, t->T.v, base, t->SD.v, 0, 1, nh));
    t->last = h;
    // children: statistics inherited unless the node was split; gamma always inherited
    MultArgs m{}; m.x = t->C.v; m.y = t->split.v; m.z = t->Cn.v; m.n = nh * CW; m.CW = t->CW;
    GTCHK(do_mult(c, 2, m));
    acct_reshare(c, nh * CW, 1);
    std::swap(t->C, t->Cn);
    if (h + 1 <= t->H && 2 * nh <= ((u64)1 << t->H)) {
        GTCHK(launch(c, GT_KC_LOCAL, k_dup_rows, g1(nh * d), B256, t->Gn.v, t->gamma.v, nh, d));
        std::swap(t->gamma, t->Gn);
    }
    return GT_OK;
}

// ---- the learning protocol as printed (small inputs) --------------------------------------
static int oaa_literal(gt_ctx *c, bool rows, P6 u, u64 base, u64 w, u64 N, u64 N8, P6 W1, u64 w1off, P6 XT,
                       u64 *acc, P6 out, P6 prev, int epi)
{
    LitOaaArgs a{}; a.c = kc(c, c->op++); a.u = u; a.base = base; a.w = (u32)w; a.N = N; a.N8 = N8; a.W1 = W1; a.w1off = w1off;
    a.XT = XT; a.acc = acc;
    const dim3 g(tiles(w * N8));
    GTCHK(launch(c, GT_KC_LOCAL, k_fill_words, g1(6 * N8), B256, acc, (u64)(6 * N8), (u64)0));   // the counting step shares this buffer
    GTCHK(rows ? launch(c, GT_KC_SMALL, k_oaa_literal<true>, g, GT_BLOCK, a) : launch(c, GT_KC_SMALL, k_oaa_literal<false>, g, GT_BLOCK, a));
    GTCHK(launch(c, GT_KC_LOCAL, k_lit_fin, g1(N), B256, acc, N, N8, out, prev, epi));
    acct_eq(c, w * N); acct_b2a_wide(c, w * N); acct_reshare(c, w * N, 1);
    return GT_OK;
}

static int partition_literal(gt_ctx *c, gt_train *t)
{
    const u64 nodes = ((u64)2 << t->H) - 1;
    GTCHK(oaa_literal(c, false, t->M.v, 0, nodes, t->N, t->N8, t->T.v, 0, t->XT.v, t->lit_acc, t->tval.v, t->M.v, 0));
    return oaa_literal(c, true, t->tval.v, 0, t->d, t->N, t->N8, t->T.v, 0, t->XT.v, t->lit_acc, t->M.v, t->M.v, 1);
}

static int leaf_bits_literal(gt_ctx *c, gt_train *t, u32 h)
{
    const u64 nh = (u64)1 << h, base = nh - 1;
    GTCHK(do_eq(c, true, t->F.v, base, nullptr, 1, t->isLeaf.v, nh));
    LcfArgs a{}; a.c = kc(c, c->op++); a.M = t->M.v; a.isLeaf = t->isLeaf.v; a.LB = t->LB.v; a.base = base; a.nh = (u32)nh; a.N = t->N; a.N8 = t->N8;
    GTCHK(launch(c, GT_KC_SMALL, k_lcf_bits, dim3(tiles(nh * t->N8)), GT_BLOCK, a));
    acct_eq(c, nh * t->N); acct_and1(c, nh * t->N);
    return GT_OK;
}

static int count_literal(gt_ctx *c, gt_train *t, u32 h, bool totals_only)
{
    const u64 nh = (u64)1 << h;
    const u32 dd = totals_only ? 1 : t->d;
    const u64 PW = (u64)(1 + t->K) * 2 * dd;
    GTCHK(launch(c, GT_KC_LOCAL, k_fill_words, g1(6 * nh * PW), B256, t->lit_acc, 6 * nh * PW, (u64)0));
    LitCountArgs a{}; a.c = kc(c, c->op++); a.LB = t->LB.v; a.XT = t->XT.v; a.YT = t->YT.v; a.B = limbs_B(t); a.N = t->N; a.N8 = t->N8;
    a.nh = (u32)nh; a.d = t->d; a.dd = dd; a.K = t->K; a.acc = t->lit_acc;
    GTCHK(launch(c, GT_KC_SMALL, k_count_literal, dim3(tiles(nh * PW * t->N8)), GT_BLOCK, a));
    GTCHK(launch(c, GT_KC_LOCAL, k_from_paper, g1(nh * t->K), B256, t->lit_acc, t->C.v, (u32)nh, t->d, dd, t->K, t->CW));
    acct_b2a_wide(c, nh * PW * t->N); acct_reshare(c, nh * PW * t->N, 1);
    return GT_OK;
}

extern "C" int gt_train_set_partition(gt_ctx *c, gt_train *t, int by_products)
{
    if (!c || !t) return GT_EINVAL;
    if (by_products && !t->OHL) {
        if (t->H > 13) return GT_EINVAL;               // int32 accumulators of the limb products: at most 4096 nodes in the level before
        const size_t nprev = std::max<size_t>(32, (size_t)1 << (t->H ? t->H - 1 : 0)), dpad = ((size_t)t->d + 63) / 64 * 64;
        GTCHK(dsh_alloc(t->OH, nprev * t->d, c->stream));
        if (hipMalloc(&t->OHL, 48 * dpad * nprev) != hipSuccess) { t->OHL = nullptr; return GT_ENOMEM; }
    }
    t->part_matmul = by_products != 0;
    return GT_OK;
}

extern "C" int gt_train_set_literal(gt_ctx *c, gt_train *t, int literal)
{
    if (!c || !t) return GT_EINVAL;
    if (literal && !t->lit_acc) {
        const size_t nmax = (size_t)1 << t->H;
        const size_t words = std::max<size_t>(6 * t->N8, 6 * nmax * (size_t)(1 + t->K) * 2 * t->d);
        if (nmax * t->N8 > ((size_t)1 << 31)) return GT_EINVAL;          // this mode is for small inputs
        if (hipMalloc(&t->lit_acc, words * 8) != hipSuccess) { t->lit_acc = nullptr; return GT_ENOMEM; }
        HIPCHK(hipMemsetAsync(t->lit_acc, 0, words * 8, c->stream));
        GTCHK(dsh_alloc(t->LB, nmax * t->N8, c->stream));
    }
    t->literal = literal != 0;
    return GT_OK;
}

extern "C" int gt_oaa_literal(gt_ctx *c, const gt_shares *W, size_t w, const gt_shares *u, size_t n, const gt_shares *z)
{
    if (!c || !shares_ok(W, w) || !shares_ok(u, n) || !shares_ok(z, n) || w == 0 || w > 0xffffffffu) return GT_EINVAL;
    Timed T(c);
    const size_t N8 = pad8(n), need = 6 * N8;
    if (c->dacc_words < need) {
        (void)hipStreamSynchronize(c->stream);
        if (c->dacc) (void)hipFree(c->dacc);
        c->dacc = nullptr; c->dacc_words = 0;
        if (hipMalloc(&c->dacc, need * 8) != hipSuccess) return T.finish(GT_ENOMEM);
        c->dacc_words = need;
        HIPCHK(hipMemsetAsync(c->dacc, 0, need * 8, c->stream));     // both users leave it at zero
    }
    return T.finish(oaa_literal(c, false, to_p6(u), 0, w, n, N8, to_p6(W), 0, to_p6(W), c->dacc, to_p6(z), to_p6(z), 0));
}

extern "C" int gt_train_level(gt_ctx *c, gt_train *t, uint32_t h)
{
    if (!c || !t) return GT_EINVAL;
    if (t->finished || h != t->level || h >= t->H) return GT_ESTATE;
    Timed T(c);
    int rc = GT_OK;
    if (t->literal) {
        if (h > 0) rc = partition_literal(c, t);
        if (rc == GT_OK) rc = leaf_bits_literal(c, t, h);
        if (rc == GT_OK) rc = count_literal(c, t, h, false);
    } else {
        if (h > 0) rc = t->part_matmul ? partition_matmul(c, t, h) : partition(c, t, h);
        if (rc == GT_OK) rc = leaf_onehot(c, t, h);
        if (rc == GT_OK) rc = count(c, t, h, false);
    }
    if (rc == GT_OK && t->hc_open) rc = heuristic_open(c, t, h);
    if (rc == GT_OK && !t->hc_open) rc = heuristic(c, t, h);
    if (rc == GT_OK && !t->hc_open) rc = update_flags(c, t, h);
    if (rc == GT_OK) rc = node_split(c, t, h);
    if (rc == GT_OK) { t->level = h + 1; t->fresh_import = false; }
    return T.finish(rc);
}

static int tree_alloc(gt_ctx *c, u32 H, bool thr, gt_tree **out)
{
    gt_tree *tr = new (std::nothrow) gt_tree();
    if (!tr) return GT_ENOMEM;
    tr->H = H; tr->has_thr = thr; tr->slot = nullptr;
    const size_t nint = ((size_t)1 << H) - 1, nleaf = (size_t)1 << H;
    int rc = dsh_alloc(tr->feat, nint, c->stream);
    if (rc == GT_OK) rc = dsh_alloc(tr->leaf, nleaf, c->stream);
    if (rc == GT_OK && thr) rc = dsh_alloc(tr->thr, nint, c->stream);
    if (rc != GT_OK) { (void)hipStreamSynchronize(c->stream); dsh_free(tr->feat); dsh_free(tr->leaf); dsh_free(tr->thr); delete tr; return rc; }
    *out = tr;
    return GT_OK;
}

extern "C" int gt_train_finish(gt_ctx *c, gt_train *t, gt_tree **out)
{
    if (!c || !t || !out) return GT_EINVAL;
    if (t->finished || t->level != t->H) return GT_ESTATE;
    Timed T(c);
    const u32 H = t->H;
    const u64 nh = (u64)1 << H, base = nh - 1, dK = (u64)t->d * t->K;
    int rc = GT_OK;
    if (t->literal) {
        if (H > 0) rc = partition_literal(c, t);
        if (rc == GT_OK) rc = leaf_bits_literal(c, t, H);
        if (rc == GT_OK) rc = count_literal(c, t, H, true);
    } else {
        if (H > 0) rc = t->part_matmul ? partition_matmul(c, t, H) : partition(c, t, H);
        if (rc == GT_OK) rc = leaf_onehot(c, t, H);
        if (rc == GT_OK) rc = count(c, t, H, true);
    }
    // label = first maximum of the class totals
    if (rc == GT_OK) rc = copy6(c, t->best.v, 0, t->C.v, dK, t->CW, nh);
    if (rc == GT_OK) rc = launch(c, GT_KC_LOCAL, k_fill_const, g1(nh), B256, t->lab.v, (u64)0, nh, (u64)0);
    for (u32 cl = 1; cl < t->K && rc == GT_OK; cl++) {
        SelArgs sa{}; sa.vin = t->best.v; sa.iin = t->lab.v; sa.vout = t->best.v; sa.iout = t->lab.v; sa.C = t->C.v;
        sa.n = nh; sa.CW = t->CW; sa.coff = dK + cl; sa.cidx = cl; sa.mode = 1;
        rc = select_max(c, sa);
    }
    if (rc == GT_OK) rc = copy6(c, t->T.v, base, t->lab.v, 0, 1, nh);
    if (rc == GT_OK) rc = copy6(c, t->Clast.v, 0, t->C.v, 0, 1, nh * t->CW);
    gt_tree *tr = nullptr;
    if (rc == GT_OK) {
        if (t->slot && !t->slot->in_use) {       // the buffers allocated with the training object
            tr = new (std::nothrow) gt_tree();
            if (!tr) rc = GT_ENOMEM;
            else { tr->H = H; tr->has_thr = false; tr->feat = t->slot->feat; tr->leaf = t->slot->leaf; tr->slot = t->slot; t->slot->in_use = true; }
        } else rc = tree_alloc(c, H, false, &tr);  // the previous tree of this object is still alive
    }
    if (rc == GT_OK) rc = copy6(c, tr->feat.v, 0, t->T.v, 0, 1, base);
    if (rc == GT_OK) rc = copy6(c, tr->leaf.v, 0, t->T.v, base, 1, nh);
    if (rc == GT_OK) { t->last = H; t->level = H + 1; t->finished = true; t->fresh_import = false; }
    rc = T.finish(rc);
    if (rc != GT_OK) { if (tr) gt_tree_destroy(tr); return rc; }
    *out = tr;
    return GT_OK;
}

static bool of_last_level(int what) { return what == GT_X_C || what == GT_X_GAMMA || what == GT_X_SD || what == GT_X_L || what == GT_X_SCORE || what == GT_X_C_PAPER; }

extern "C" size_t gt_train_export_size(const gt_train *t, int what)
{
    if (!t) return 0;
    if (t->fresh_import && of_last_level(what)) return 0;     // no level has run on the imported state yet
    const size_t nh = (size_t)1 << t->last;
    switch (what) {
    case GT_X_T: case GT_X_F: return ((size_t)2 << t->H) - 1;
    case GT_X_M: return t->N;
    case GT_X_C: return nh * t->CW;
    case GT_X_GAMMA: case GT_X_SCORE: return nh * t->d;
    case GT_X_SD: return nh;
    case GT_X_L: return nh * t->N8;
    case GT_X_C_PAPER: return nh * (1 + t->K) * 2 * t->d;
    default: return 0;
    }
}

extern "C" int gt_train_export(gt_ctx *c, const gt_train *t, int what, const gt_shares *out)
{
    if (!c || !t) return GT_EINVAL;
    if (what < GT_X_T || what > GT_X_C_PAPER) return GT_EINVAL;
    if (t->fresh_import && of_last_level(what)) return GT_ESTATE;
    if (t->literal && what == GT_X_L) return GT_ESTATE;               // no arithmetic one-hot exists in that mode
    const size_t n = gt_train_export_size(t, what);
    if (!shares_ok(out, n)) return GT_EINVAL;
    Timed T(c);
    const DSh *src = nullptr;
    switch (what) {
    case GT_X_T: src = &t->T; break;
    case GT_X_F: src = &t->F; break;
    case GT_X_M: src = &t->M; break;
    case GT_X_C: src = &t->Clast; break;
    case GT_X_GAMMA: src = &t->Glast; break;
    case GT_X_SD: src = &t->SD; break;
    case GT_X_L: break;
    case GT_X_SCORE: src = &t->Slast; break;
    default: break;
    }
    int rc = GT_OK;
    if (src) rc = copy6(c, to_p6(out), 0, src->v, 0, 1, n);
    else if (what == GT_X_L) rc = launch(c, GT_KC_LOCAL, k_l_export, g1(n), B256, limbs_L(t), to_p6(out), (u64)1 << t->last, (u64)t->N, (u64)t->N8);
    else {
        const u32 nh = 1u << t->last;
        rc = launch(c, GT_KC_LOCAL, k_c_paper, g1(n), B256, t->Clast.v, to_p6(out), nh, t->d, t->K, t->CW);
    }
    return T.finish(rc);
}

extern "C" int gt_train_import(gt_ctx *c, gt_train *t, uint32_t h, const gt_shares *M, const gt_shares *Tprev,
                               const gt_shares *Fl, const gt_shares *Cc, const gt_shares *gm)
{
    if (!c || !t || h > t->H) return GT_EINVAL;
    const size_t nh = (size_t)1 << h, base = nh - 1;
    if (!shares_ok(M, t->N) || !shares_ok(Fl, nh) || !shares_ok(Cc, nh * t->CW) || !shares_ok(gm, nh * t->d)) return GT_EINVAL;
    if (h > 0 && !shares_ok(Tprev, nh / 2)) return GT_EINVAL;
    Timed T(c);
    int rc = copy6(c, t->M.v, 0, to_p6(M), 0, 1, t->N);
    if (rc == GT_OK && h > 0) rc = copy6(c, t->T.v, base - nh / 2, to_p6(Tprev), 0, 1, nh / 2);
    if (rc == GT_OK) rc = copy6(c, t->F.v, base, to_p6(Fl), 0, 1, nh);
    if (rc == GT_OK) rc = copy6(c, t->C.v, 0, to_p6(Cc), 0, 1, nh * t->CW);
    if (rc == GT_OK) rc = copy6(c, t->gamma.v, 0, to_p6(gm), 0, 1, nh * t->d);
    if (rc == GT_OK) { t->level = h; t->finished = false; t->fresh_import = true; t->lt_level = ~0u; }
    return T.finish(rc);
}

// ---- inference ------------------------------------------------------------------------
extern "C" int gt_tree_import(gt_ctx *c, const gt_shares *feat, const gt_shares *thr, const gt_shares *leaf,
                              uint32_t H, gt_tree **out)
{
    if (!c || !out || H > GT_MAX_DEPTH) return GT_EINVAL;
    const size_t nint = ((size_t)1 << H) - 1, nleaf = (size_t)1 << H;
    if (!shares_ok(feat, nint) || !shares_ok(leaf, nleaf) || (thr && !shares_ok(thr, nint))) return GT_EINVAL;
    Timed T(c);
    gt_tree *tr = nullptr;
    int rc = tree_alloc(c, H, thr != nullptr, &tr);
    if (rc == GT_OK) rc = copy6(c, tr->feat.v, 0, to_p6(feat), 0, 1, nint);
    if (rc == GT_OK) rc = copy6(c, tr->leaf.v, 0, to_p6(leaf), 0, 1, nleaf);
    if (rc == GT_OK && thr) rc = copy6(c, tr->thr.v, 0, to_p6(thr), 0, 1, nint);
    rc = T.finish(rc);
    if (rc != GT_OK) { if (tr) gt_tree_destroy(tr); return rc; }
    *out = tr;
    return GT_OK;
}

extern "C" int gt_tree_export(gt_ctx *c, const gt_tree *tr, const gt_shares *feat, const gt_shares *leaf)
{
    if (!c || !tr) return GT_EINVAL;
    const size_t nint = ((size_t)1 << tr->H) - 1, nleaf = (size_t)1 << tr->H;
    if (!shares_ok(feat, nint) || !shares_ok(leaf, nleaf)) return GT_EINVAL;
    Timed T(c);
    int rc = copy6(c, to_p6(feat), 0, tr->feat.v, 0, 1, nint);
    if (rc == GT_OK) rc = copy6(c, to_p6(leaf), 0, tr->leaf.v, 0, 1, nleaf);
    return T.finish(rc);
}

extern "C" int gt_tree_destroy(gt_tree *tr)
{
    if (!tr) return GT_EINVAL;
    if (tr->slot && !tr->slot->orphan) {         // buffers go back to the training object: nothing is freed
        tr->slot->in_use = false;
        delete tr;
        return GT_OK;
    }
    (void)hipDeviceSynchronize();
    dsh_free(tr->feat); dsh_free(tr->thr); dsh_free(tr->leaf);
    if (tr->slot) delete tr->slot;
    delete tr;
    return GT_OK;
}

// One launch for the whole batch (and for every tree of a forest): a workgroup carries a
// tile of instances through all levels of one tree.  Smaller tiles (more lanes per instance,
// more columns per step) for batches that would otherwise leave compute units without a
// workgroup.
static int infer_one_launch(gt_ctx *c, P6 feat, P6 thr, P6 leaf, bool has_thr, u32 H, u32 ntrees,
                            const gt_shares *I, size_t NI, uint32_t d, const gt_shares *R)
{
    const size_t N8 = pad8(NI);
    InferArgs a{}; a.c = kc(c, c->op); a.feat = feat; a.thr = thr; a.leaf = leaf;
    a.I = to_p6(I); a.out = to_p6(R); a.NI = NI; a.N8 = N8; a.d = d; a.H = H; a.ntrees = ntrees; a.has_thr = has_thr ? 1 : 0;
    const u32 S = has_thr ? 3 : 2;
    c->op += ntrees * (H * S + 1);
    int lgi = c->infer_lgi;
    const u64 per64 = (NI + 63) / 64 * ntrees, per32 = (NI + 31) / 32 * ntrees;
    if (!lgi) lgi = per64 >= 2ull * c->resident ? 6 : (per32 >= c->resident / 4 ? 5 : 4);
    const u64 nitem = ((NI + ((u64)1 << lgi) - 1) >> lgi) * ntrees;
    const dim3 g((unsigned)std::min<u64>(nitem, 1u << 20));
    const bool small = nitem <= 2ull * (c->resident / 4);      // at most two workgroups per compute unit
    int rc;
    if (small) rc = lgi == 6 ? launch(c, GT_KC_INFER, k_infer<6, 2>, g, GT_BLOCK, a)
                  : lgi == 5 ? launch(c, GT_KC_INFER, k_infer<5, 2>, g, GT_BLOCK, a)
                             : launch(c, GT_KC_INFER, k_infer<4, 2>, g, GT_BLOCK, a);
    else rc = lgi == 6 ? launch(c, GT_KC_INFER, k_infer<6, 3>, g, GT_BLOCK, a)
            : lgi == 5 ? launch(c, GT_KC_INFER, k_infer<5, 3>, g, GT_BLOCK, a)
                       : launch(c, GT_KC_INFER, k_infer<4, 3>, g, GT_BLOCK, a);
    for (u32 t = 0; t < ntrees; t++) {
        for (u32 n = 0; n < H; n++) {
            const u64 nel = ((u64)1 << n) * NI;
            acct_eq_grid(c, NI, nel); acct_b2a(c, nel); acct_reshare(c, NI, has_thr ? 2 : 1);
            acct_eq_grid(c, NI, (u64)d * NI); acct_b2a(c, (u64)d * NI); acct_reshare(c, NI, 1);
            if (has_thr) { acct_ge(c, NI); acct_b2a(c, NI); }
        }
        acct_eq_grid(c, NI, ((u64)1 << H) * NI); acct_b2a(c, ((u64)1 << H) * NI); acct_reshare(c, NI, 1);
    }
    return rc;
}

extern "C" int gt_infer_batch(gt_ctx *c, const gt_tree *tr, const gt_shares *I, size_t NI, uint32_t d, const gt_shares *R)
{
    if (!c || !tr || NI == 0 || d == 0 || d > 65536) return GT_EINVAL;
    if (!shares_ok(I, NI * d) || !shares_ok(R, NI)) return GT_EINVAL;
    Timed T(c);
    const size_t N8 = pad8(NI);
    const u32 H = tr->H;
    if (!c->levelwise_infer)
        return T.finish(infer_one_launch(c, tr->feat.v, tr->has_thr ? tr->thr.v : tr->feat.v, tr->leaf.v, tr->has_thr, H, 1, I, NI, d, R));
    // workspace: transposed instances, node index, fetched id / threshold / value
    const size_t need[5] = { (size_t)d * N8, NI, NI, tr->has_thr ? NI : 0, tr->has_thr ? NI : 0 };
    int rc = GT_OK;
    for (int i = 0; i < 5 && rc == GT_OK; i++)
        if (c->ws[i].n < need[i]) { (void)hipStreamSynchronize(c->stream); dsh_free(c->ws[i]); rc = dsh_alloc(c->ws[i], need[i], c->stream); }
    DSh &IT = c->ws[0], &tidx = c->ws[1], &f = c->ws[2], &th = c->ws[3], &x = c->ws[4];
    if (rc == GT_OK) rc = launch(c, GT_KC_LOCAL, k_fill_const, g1(NI), B256, tidx.v, (u64)0, (u64)NI, (u64)0);
    if (rc == GT_OK) rc = launch(c, GT_KC_LOCAL, k_transpose, gT(NI, d), B256, IT.v, to_p6(I), (u64)NI, (u64)N8, d);
    for (u32 n = 0; n < H && rc == GT_OK; n++) {
        const u64 w = (u64)1 << n, base = w - 1;
        GridArgs a{}; a.u = tidx.v; a.base = base; a.w = (u32)w; a.N = NI; a.N8 = N8;
        a.W1 = tr->feat.v; a.w1off = base; a.out = f.v; a.epi = 0;
        if (tr->has_thr) { a.W2 = tr->thr.v; a.w2off = base; a.out2 = th.v; }
        rc = do_grid(c, GM_COMMON, false, tr->has_thr ? 2 : 1, a);
        if (rc != GT_OK) break;
        GridArgs b{}; b.u = f.v; b.base = 0; b.w = d; b.N = NI; b.N8 = N8; b.XT = IT.v;
        if (tr->has_thr) { b.out = x.v; b.epi = 0; } else { b.out = tidx.v; b.prev = tidx.v; b.epi = 1; }
        rc = do_grid(c, GM_ROWS, false, 1, b);
        if (rc != GT_OK) break;
        if (tr->has_thr) {
            CmpArgs ca{}; ca.c = kc(c, c->op++); ca.th = th.v; ca.x = x.v; ca.tidx = tidx.v; ca.n = NI;
            rc = launch(c, GT_KC_SMALL, k_cmp_step, dim3(tiles(NI)), GT_BLOCK, ca);
            acct_ge(c, NI); acct_b2a(c, NI);
        }
    }
    if (rc == GT_OK) {
        const u64 nleaf = (u64)1 << H;
        GridArgs a{}; a.u = tidx.v; a.base = nleaf - 1; a.w = (u32)nleaf; a.N = NI; a.N8 = N8;
        a.W1 = tr->leaf.v; a.w1off = 0; a.out = to_p6(R); a.epi = 0;
        rc = do_grid(c, GM_COMMON, false, 1, a);
    }
    return T.finish(rc);
}

// ---- forests: many trees of one depth on the same batch, one launch -----------------------
extern "C" int gt_forest_create(gt_ctx *c, const gt_tree *const *trees, size_t ntrees, gt_forest **out)
{
    if (!c || !trees || !out || ntrees == 0 || ntrees > 65536) return GT_EINVAL;
    for (size_t t = 0; t < ntrees; t++)
        if (!trees[t] || trees[t]->H != trees[0]->H || trees[t]->has_thr != trees[0]->has_thr) return GT_EINVAL;
    Timed T(c);
    gt_forest *f = new (std::nothrow) gt_forest();
    if (!f) return GT_ENOMEM;
    f->H = trees[0]->H; f->ntrees = (u32)ntrees; f->has_thr = trees[0]->has_thr;
    const size_t nint = ((size_t)1 << f->H) - 1, nleaf = (size_t)1 << f->H;
    int rc = dsh_alloc(f->feat, ntrees * nint, c->stream);
    if (rc == GT_OK) rc = dsh_alloc(f->leaf, ntrees * nleaf, c->stream);
    if (rc == GT_OK && f->has_thr) rc = dsh_alloc(f->thr, ntrees * nint, c->stream);
    for (size_t t = 0; t < ntrees && rc == GT_OK; t++) {
        rc = copy6(c, f->feat.v, t * nint, trees[t]->feat.v, 0, 1, nint);
        if (rc == GT_OK) rc = copy6(c, f->leaf.v, t * nleaf, trees[t]->leaf.v, 0, 1, nleaf);
        if (rc == GT_OK && f->has_thr) rc = copy6(c, f->thr.v, t * nint, trees[t]->thr.v, 0, 1, nint);
    }
    rc = T.finish(rc);
    if (rc != GT_OK) { (void)hipStreamSynchronize(c->stream); dsh_free(f->feat); dsh_free(f->leaf); dsh_free(f->thr); delete f; return rc; }
    *out = f;
    return GT_OK;
}

extern "C" int gt_forest_destroy(gt_forest *f)
{
    if (!f) return GT_EINVAL;
    (void)hipDeviceSynchronize();
    dsh_free(f->feat); dsh_free(f->thr); dsh_free(f->leaf);
    delete f;
    return GT_OK;
}

extern "C" int gt_infer_forest(gt_ctx *c, const gt_forest *f, const gt_shares *I, size_t NI, uint32_t d, const gt_shares *R)
{
    if (!c || !f || NI == 0 || d == 0 || d > 65536) return GT_EINVAL;
    if (!shares_ok(I, NI * d) || !shares_ok(R, NI * f->ntrees)) return GT_EINVAL;
    Timed T(c);
    return T.finish(infer_one_launch(c, f->feat.v, f->has_thr ? f->thr.v : f->feat.v, f->leaf.v, f->has_thr, f->H, f->ntrees, I, NI, d, R));
}
