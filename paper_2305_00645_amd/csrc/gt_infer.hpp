// Oblivious inference in one launch (Sec. V-C of the GTree paper).  The H iterations of an
// instance - array access over the level's slice of the tree, array access into the
// instance's own features, optional threshold comparison, index update - and the final
// access over the leaf labels do not interact with any other instance, so a workgroup
// carries a tile of instances through all of them with the node index and the fetched
// id / threshold / value in registers: no per-level launches, no partial sums in device
// memory, no workspace.  Operation ids, element indices (k*N8 + i) and streams are those
// of the level-by-level path, so every share is the same.
#pragma once
#include "gt_kernels.hpp"

struct InferArgs {
    KCommon c;                 // c.op: first operation id of the batch
    P6 feat, thr, leaf;        // per tree 2^H-1 ids, 2^H-1 thresholds (has_thr), 2^H labels, tree after tree
    P6 I, out;                 // NI x d row-major instances; results out[t*NI + i]
    u64 NI, N8;
    u32 d, H, ntrees;          // ntrees > 1: a forest; tree t takes the operation ids that the t-th of
    int has_thr;               // ntrees single-tree batches in a row would take
};

// Words of NS streams under the own and the next key for the tile's IT consecutive
// elements e0 .. e0+IT-1 (e0 a multiple of 8), element e0 + (lane mod IT) in every lane
// that works on it.  A PRF block holds the words of 8 consecutive elements: IT/8 blocks
// per key and stream, one lane each, handed round through the wavefront's scratch in LDS.
template <int NS, int LGI>
__device__ __forceinline__ void prf_tile_it(const PartyKeys &K, u32 op, const u32 (&st)[NS], u64 e0, u64 (&wo)[NS], u64 (&wn)[NS])
{
    constexpr u32 IT = 1u << LGI, NB = IT / 8;
    static_assert(2 * NS * NB <= GT_LANES, "more blocks than lanes");
    const u32 lane = threadIdx.x, inst = lane & (IT - 1);
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
    if (lane < 2 * NS * NB) {
        const u32 q = lane / (2 * NB), r = lane % (2 * NB), ks = r / NB, g = r % NB;
        const u32 mk = 0u - ks;
        Key kv;
#pragma unroll
        for (int i = 0; i < 8; i++) kv.k[i] = K.own.k[i] ^ ((K.own.k[i] ^ K.nxt.k[i]) & mk);
        u32 stream = 0;
#pragma unroll
        for (int j = 0; j < NS; j++) stream |= st[j] & (0u - (u32)(q == (u32)j));
        u64 blk[8];
        chacha8(kv, (e0 >> 3) + g, op, stream, blk);
#pragma unroll
        for (int i = 0; i < 8; i++) K.scr[(q * 2 + ks) * IT + g * 8 + i] = blk[i];
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int j = 0; j < NS; j++) { wo[j] = K.scr[(2 * j) * IT + inst]; wn[j] = K.scr[(2 * j + 1) * IT + inst]; }
}

// sum over the 64/IT lanes that hold the same instance (lane = cg*IT + inst)
template <int LGI>
__device__ __forceinline__ u64 sum_over_column_groups(u64 v)
{
#pragma unroll
    for (int m = 1 << LGI; m < GT_LANES; m <<= 1) v += (u64)__shfl_xor((unsigned long long)v, m, GT_LANES);
    return v;
}

// State of one workgroup: LDS rows as in k_eqgrid (rows 0-2: the mask words; rows 3-5: the
// messages of the openings, AND rounds, conversions and reshares; rows 6-8: beta
// arithmetic components, between two steps party p's PRF scratch in row 6+p).
template <int LGI>
struct InferWg {
    static constexpr u32 IT = 1u << LGI, LPI = GT_LANES >> LGI, CS = 8 * LPI;   // instances per tile, lanes per instance, columns per step
    u64 (*s_mat)[GT_TILE_EL];
    u32 (*s_bitw)[GT_LANES];
    LWire LW;
    PartyKeys K;
    int p, pn, pp, lane, tid;
    u32 inst, cg, par;
    u64 N8, tile0;            // first instance of the tile
    u64 i;                    // this lane's instance
    bool valid;

    // One array access: E[k] = [u - base == k] for k < w, converted to arithmetic, and
    // z = sum_k E[k] * W1[w1off + k] (ROWS: * the instance's own feature k), z2 likewise
    // with W2 (NDOT = 2); zero sharing of stream 2 (3), word i; one reshare round.
    template <bool ROWS, int NDOT>
    __device__ __forceinline__ void access(u32 op, Sh u, u64 base, u32 w, const P6 &W1, u64 w1off, const P6 &W2, u64 w2off,
                                           const P6 &I, u32 d, Sh &z, Sh &z2)
    {
        const Sh one = pub(p, 1);
        u64 acc = 0, acc2 = 0;
        // the instance's edaBit and the one opening of the access: c = u + r - base is public
        // afterwards; the lanes of one instance replay the same message, one of them counts
        u64 cpub; Sh rho;
        {
            const Dealer D = dealer_of(K, p, op, i);
            rho = D.rho;
            const u64 snd = u.o + D.rA.o;
            cpub = snd + (u.n + D.rA.n) + LW.open1(snd, (valid && cg == 0) ? 64u : 0u) - base;
        }
        for (u32 k0 = 0; k0 < w; k0 += CS) {
            // This lane evaluates, for column k0 + lane / (IT/8) and instances
            // 8 * (lane mod IT/8) .. +7 of the tile, the block of mask words under the own
            // key and the party-th of the group's three daBit blocks
            u64 A[8];
            {
                const u32 cc = (u32)lane >> (LGI - 3), gg = (u32)lane & (IT / 8 - 1);
                const u64 g = (((u64)(k0 + cc) * N8 + tile0) >> 3) + gg;
                u64 D[8];
                chacha8(K.dlr, 3 * g + p, op, 4, D);
                // the 8 tests of a block go to 8 neighbouring lanes: positions in a row of LDS
                // are swizzled (low three bits of the lane xor the next three) so that neither
                // the producers' stores nor the consumers' loads pile up on a few banks
                const u32 sl = cc & 7, ln0 = (cc >> 3) * IT + gg * 8;
#pragma unroll
                for (int q = 0; q < 3; q++) {
                    const u32 j = 3 * p + q;
                    if (j < 8) {
                        const u32 ln = ln0 + j, el = sl * GT_LANES + (ln ^ ((ln >> 3) & 7));
                        const u64 beta = (D[6] >> (3 * q)) & 1;
                        s_mat[6][el] = D[2 * q]; s_mat[7][el] = D[2 * q + 1]; s_mat[8][el] = beta - D[2 * q] - D[2 * q + 1];
                        const u32 b0 = (u32)(D[6] >> (3 * q + 1)) & 1, b1 = (u32)(D[6] >> (3 * q + 2)) & 1, b2 = ((u32)beta ^ b0 ^ b1) & 1;
                        atomicOr(&s_bitw[par][ln], (b0 << sl) | (b1 << (8 + sl)) | (b2 << (16 + sl)));
                    }
                }
                chacha8(K.own, g, op, 1, A);
            }
#pragma unroll
            for (int s = 0; s < 8; s++) s_mat[p][8 * lane + (s ^ (lane & 7))] = A[s];   // block (cc, gg): words of 8 instances
            __syncthreads();
            if (p == 0) s_bitw[par ^ 1][lane] = 0;
            u32 nl = 0;
            Sh t[8];
#pragma unroll
            for (int s = 0; s < 8; s++) {
                const u32 col = k0 + cg * 8 + s;
                nl += (valid && col < w) ? 1u : 0u;
                const u32 li = (cg * 8 + s) * IT + inst, idx = li ^ ((li >> 3) & 7);
                A[s] = s_mat[p][idx] ^ s_mat[pn][idx];
                // t = rho with the complement of (c - base - col) xored into component 0
                const u64 nx = ~(cpub - col);                // columns beyond w, instances beyond NI: any value serves
                t[s].o = p == 0 ? rho.o ^ nx : rho.o;
                t[s].n = p == 2 ? rho.n ^ nx : rho.n;
            }
            u32 To8, Tn8;
            eq_rounds8_packed(LW, t, A, nl, To8, Tn8);
            u32 f;
            {
                const u32 bw = s_bitw[par][lane];
                const u32 fo = To8 ^ ((bw >> (8 * p)) & 0xffu), fn = Tn8 ^ ((bw >> (8 * pn)) & 0xffu);
                f = fo ^ fn ^ (u32)LW.open1((u64)fo, nl);
            }
#pragma unroll
            for (int s = 0; s < 8; s++) {
                const u32 col = k0 + cg * 8 + s;
                const int el = s * GT_LANES + (lane ^ ((lane >> 3) & 7));
                const Sh bA = { s_mat[6 + p][el], s_mat[6 + pn][el] };
                Sh E;
                E.o = ((f >> s) & 1) ? one.o - bA.o : bA.o;
                E.n = ((f >> s) & 1) ? one.n - bA.n : bA.n;
                if (col < w) {
                    if (ROWS) {
                        Sh x = { 0, 0 };
                        if (valid) x = ld(I, p, i * d + col);
                        acc += prod3(E, x);
                    } else {
                        acc += prod3(E, ld(W1, p, w1off + col));
                        if (NDOT == 2) acc2 += prod3(E, ld(W2, p, w2off + col));
                    }
                }
            }
            par ^= 1;
            __syncthreads();                           // the material in LDS is overwritten next
        }
        acc = sum_over_column_groups<LGI>(acc);
        if (NDOT == 2) acc2 = sum_over_column_groups<LGI>(acc2);
        const u32 bits = (valid && cg == 0) ? 64u : 0u;   // the lanes of one instance hold the same result: one of them counts
        if (NDOT == 2) {
            const u32 st[2] = { 2, 3 }; u64 wo[2], wn[2];
            prf_tile_it<2, LGI>(K, op, st, tile0, wo, wn);
            u64 s2[2] = { acc + (wo[0] - wn[0]), acc2 + (wo[1] - wn[1]) }, r2[2];
            LW.reshare<2>(s2, r2, 2 * bits);
            z.o = s2[0]; z.n = r2[0]; z2.o = s2[1]; z2.n = r2[1];
        } else {
            const u32 st[1] = { 2 }; u64 wo[1], wn[1];
            prf_tile_it<1, LGI>(K, op, st, tile0, wo, wn);
            z.o = acc + (wo[0] - wn[0]);
            z.n = LW.reshare1(z.o, bits);
        }
        __syncthreads();                               // message slots and scratch are free again
    }

    // bit = [x > theta] as an arithmetic sharing (threshold mode)
    __device__ __forceinline__ Sh greater(u32 op, Sh th, Sh x)
    {
        const bool act = valid && cg == 0;
        const Dealer D = dealer_of(K, p, op, i);
        const u32 st[2] = { 1, 2 }; u64 wo[2], wn[2];
        prf_tile_it<2, LGI>(K, op, st, tile0, wo, wn);
        const Sh b = b2a(LW, p, not_bit(p, ge_bit_masks(LW, p, th - x, D, wo[0] ^ wn[0], wo[1] ^ wn[1], act)), D, act);
        __syncthreads();
        return b;
    }
};

// OCC: wavefronts per SIMD the register budget is cut for (3: four workgroups per compute
// unit, for batches that fill the device; 2: no register spills, for small batches whose
// few workgroups gain nothing from a higher occupancy)
template <int LGI, int OCC>
__global__ __launch_bounds__(192, OCC) void k_infer(InferArgs a)
{
    __shared__ u64 s_mat[9][GT_TILE_EL];
    __shared__ u32 s_bitw[2][GT_LANES];
    __shared__ u64 s_cnt[6];
    InferWg<LGI> X;
    constexpr u32 IT = InferWg<LGI>::IT;
    X.s_mat = s_mat; X.s_bitw = s_bitw;
    X.p = party_of_wave(); X.lane = threadIdx.x; X.tid = X.p * GT_LANES + X.lane;
    X.pn = X.p == 2 ? 0 : X.p + 1; X.pp = X.p == 0 ? 2 : X.p - 1;
    X.LW.init(&s_mat[3][0], s_cnt);
    X.K = load_party_keys(a.c.keys, X.p, &s_mat[6 + X.p][0]);
    X.inst = (u32)X.lane & (IT - 1); X.cg = (u32)X.lane >> LGI; X.par = 0; X.N8 = a.N8;
    if (X.tid < 2 * GT_LANES) (&s_bitw[0][0])[X.tid] = 0;
    __syncthreads();
    const u32 S = a.has_thr ? 3 : 2;
    const u64 ntile = (a.NI + IT - 1) / IT, nleaf = (u64)1 << a.H, nint = nleaf - 1;
    for (u64 item = blockIdx.x; item < ntile * a.ntrees; item += gridDim.x) {
        const u64 tree = item / ntile, tile = item % ntile;
        const u32 op0 = a.c.op + (u32)tree * (a.H * S + 1);
        X.tile0 = tile * IT; X.i = X.tile0 + X.inst; X.valid = X.i < a.NI;
        Sh tidx = { 0, 0 }, zz = { 0, 0 };
        for (u32 n = 0; n < a.H; n++) {
            const u64 wn = (u64)1 << n, base = wn - 1, off = tree * nint + base;
            const u32 op = op0 + n * S;
            Sh f, th = { 0, 0 }, x;
            if (a.has_thr) X.template access<false, 2>(op, tidx, base, (u32)wn, a.feat, off, a.thr, off, a.I, a.d, f, th);
            else X.template access<false, 1>(op, tidx, base, (u32)wn, a.feat, off, a.feat, off, a.I, a.d, f, zz);
            X.template access<true, 1>(op + 1, f, 0, a.d, a.feat, 0, a.feat, 0, a.I, a.d, x, zz);
            if (a.has_thr) x = X.greater(op + 2, th, x);
            tidx = scale(tidx, 2) + x + pub(X.p, 1);
        }
        Sh R;
        X.template access<false, 1>(op0 + a.H * S, tidx, nint, (u32)nleaf, a.leaf, tree * nleaf, a.leaf, 0, a.I, a.d, R, zz);
        if (X.valid && X.cg == 0) st(a.out, X.p, tree * a.NI + X.i, R);
        X.LW.drain();
    }
    X.LW.flush(a.c.wire);
}
