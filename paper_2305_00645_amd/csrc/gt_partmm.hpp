// Data partition by products on the matrix cores (a variant beyond the paper's listing,
// see k_onehot in gt_kernels.hpp for the protocol):
//   sel[k][i] = sum_r L[r][i] * OH[r][k]     (op, zero sharing of stream 0, word k*N8+i, reshare)
//   M[i]     <- 2 M[i] + sum_k sel[k][i] * X[k][i] + 1   (op+1, zero sharing of stream 0, word i, reshare)
// fused in one launch: a workgroup = the three parties' wavefronts works on a block of 32
// samples; each wavefront computes its party's three-term product
//   L_p (OH_p + OH_{p+1}) + L_{p+1} OH_p
// as an int8-limb GEMM (64 columns x 32 samples per pass, contraction over the nodes r of
// both terms), adds the zero sharing, sends its component to the predecessor through LDS
// and accumulates the row inner product with X; sel never reaches device memory.
//
// Operands.  OH comes as limb bytes with the node index contiguous (k_oh_limbs): that is the
// A operand as it is.  L lives in the limb tiles of the statistics contraction, where the
// SAMPLES are contiguous ([block][limb][row r][32 samples]); the matrix core wants the
// contraction index contiguous per lane, so every 32 x 32 byte tile is transposed through a
// small wavefront-private LDS area: dword columns are written with a padded stride, lanes
// read 16 dwords of their sample's dword column and pick their byte with byte permutes.
#pragma once
#include "gt_kernels.hpp"

// OH as limb bytes: OHL[((p*2 + w)*8 + s)*dpad + k)*rpad + r] = limb s of (w ? own : own + next)
// of party p's OH[r][k]; zero for r >= np or k >= d.
__global__ __launch_bounds__(256) void k_oh_limbs(P6 OH, unsigned char *OHL, u32 np, u32 d, u32 rpad, u32 dpad)
{
    const u64 per = (u64)dpad * rpad, total = 6 * per;
    for (u64 t = (u64)blockIdx.x * blockDim.x + threadIdx.x; t < total; t += (u64)gridDim.x * blockDim.x) {
        const u32 pw = (u32)(t / per), k = (u32)((t % per) / rpad), r = (u32)(t % rpad), p = pw >> 1, w = pw & 1;
        u64 x = 0;
        if (r < np && k < d) x = OH.o[p][(u64)r * d + k] + (w ? 0 : OH.n[p][(u64)r * d + k]);
        const u64 y = (x + GT_BIAS) ^ GT_BIAS;
#pragma unroll
        for (int s = 0; s < 8; s++) OHL[(((u64)pw * 8 + s) * dpad + k) * rpad + r] = (unsigned char)(y >> (8 * s));
    }
}

#define PM_TP_STRIDE 36                      // dwords between the dword columns of the transpose area
#define PM_TP_WORDS (8 * PM_TP_STRIDE)       // dwords per area

struct PartMmArgs {
    KCommon c;                 // c.op: the column-selection op; c.op + 1: the row inner product
    LimbTri L;                 // leaf one-hot of the previous level, one matrix per component
    const unsigned char *OHL;
    P6 XT, M;
    u64 N, N8, nblk;
    u32 d, dpad, rpad;         // columns, padded to 64; node rows padded to 32
};

// Zero-sharing words of one pass of the epilogue: the pass (t, vq) covers the 8 rows
// m = t*32 + 8*vq + ri, ri < 8, of the 64 x 32 tile; lane l < 32 evaluates the own-key block
// of row ri = l/4, sample group l%4, lanes 32.. the next-key blocks; words to
// scr[((pass*2 + key)*8 + ri)*32 + sample].
__device__ __forceinline__ void pm_prf_pass(const PartMmArgs &a, const PartyKeys &K, u64 *scr, u32 pass, u32 kg, u64 ib, u32 n, u32 hi)
{
    const u32 ri = n >> 2, g = n & 3;
    const u64 kcol = (u64)kg * 64 + (pass >> 2) * 32 + 8 * (pass & 3) + ri;
    const u32 mk = 0u - hi;
    Key kv;
#pragma unroll
    for (int q = 0; q < 8; q++) kv.k[q] = K.own.k[q] ^ ((K.own.k[q] ^ K.nxt.k[q]) & mk);
    u64 blk[8];
    chacha8(kv, ((kcol * a.N8 + ib * 32) >> 3) + g, a.c.op, 0, blk);
#pragma unroll
    for (int q = 0; q < 8; q++) scr[((pass * 2 + hi) * 8 + ri) * 32 + g * 8 + q] = blk[q];
}

__global__ __launch_bounds__(192, 1) void k_part_mm(PartMmArgs a)
{
    __shared__ u64 s_wire[GT_LWIRE_WORDS];
    __shared__ u64 s_cnt[6];
    __shared__ u64 s_prf[3][8 * 2 * 8 * 32];     // per party: the zero-sharing words of a 64 x 32 tile under two keys
    __shared__ u64 s_x[3][16 * GT_LANES];        // the reshared components, 16 per lane and exchange
    __shared__ u32 s_tp[3][2 * PM_TP_WORDS];     // two transpose areas per wavefront, used alternately
    const int p = party_of_wave(), lane = threadIdx.x, pn = p == 2 ? 0 : p + 1;
    LWire W; W.init(s_wire, s_cnt);
    const PartyKeys K = load_party_keys(a.c.keys, p);
    u64 *scr = s_prf[p];
    u32 *tp = s_tp[p];
    const u32 n = lane & 31, hi = (u32)lane >> 5;
    const Sh one = pub(p, 1);
    const u32 bsel = (n & 3) | ((4 + (n & 3)) << 8) | 0x0c0c0000u;   // byte n%4 of two dwords into bytes 0 and 1
    const u32 nrc = a.rpad / 32, nkg = a.dpad / 64, nch = 2 * nrc;
    for (u64 ib = blockIdx.x; ib < a.nblk; ib += gridDim.x) {
        const u64 i = ib * 32 + n;
        const bool ilive = i < a.N;
        u64 dacc = 0;
        for (u32 kg = 0; kg < nkg; kg++) {
            v16i acc[8][2];
#pragma unroll
            for (int u = 0; u < 8; u++)
#pragma unroll
                for (int t = 0; t < 2; t++)
#pragma unroll
                    for (int v = 0; v < 16; v++) acc[u][t][v] = 0;
            // chunks of 32 node rows: first those of L_p x (OH own+next), then those of L_{p+1} x OH own.
            // The eight limb tiles of the next chunk are in flight while this one is transposed and
            // multiplied (the last iteration loads its own chunk again, unused, so that the number of
            // loads in flight at every wait is the same).  Two passes of the epilogue's zero-sharing
            // words are evaluated per chunk, in the shadow of the matrix-core instructions.
            v4i xn[8];
#define PM_LOAD(X, CH)                                                                               \
            {                                                                                        \
                const u32 w_ = (CH) / nrc, rc_ = (CH) % nrc;                                         \
                const u32 j_ = (u32)p + w_ >= 3 ? 0 : (u32)p + w_;                                   \
                const LimbMat LM_ = j_ == 0 ? a.L.m[0] : (j_ == 1 ? a.L.m[1] : a.L.m[2]);            \
                _Pragma("unroll") for (int s = 0; s < 8; s++)                                        \
                    X[s] = *(const v4i *)(LM_.base + limb_addr(LM_, ib, s, (u64)rc_ * 32) + (lane >> 1) * 32 + (lane & 1) * 16); \
            }
            PM_LOAD(xn, 0)
            for (u32 ch = 0; ch < nch; ch++) {
                const u32 w = ch / nrc, rc = ch % nrc;
                v4i x[8], A[2][8];
#pragma unroll
                for (int s = 0; s < 8; s++) x[s] = xn[s];
                PM_LOAD(xn, (ch + 1 < nch ? ch + 1 : ch))
#pragma unroll
                for (int t = 0; t < 2; t++) {
                    const u64 col = (u64)kg * 64 + t * 32 + n;
#pragma unroll
                    for (int s = 0; s < 8; s++)
                        A[t][s] = *(const v4i *)(a.OHL + ((((u64)(p * 2 + w) * 8 + s) * a.dpad + col) * a.rpad + rc * 32 + hi * 16));
                }
                // B operand: the eight limb tiles [32 rows r][32 samples] of this chunk, transposed
                v4i Bt[8];
#pragma unroll
                for (int s = 0; s < 8; s++) {
                    __builtin_amdgcn_wave_barrier();
#pragma unroll
                    for (int q = 0; q < 4; q++) tp[(s & 1) * PM_TP_WORDS + ((lane & 1) * 4 + q) * PM_TP_STRIDE + (lane >> 1)] = (u32)x[s][q];
                    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
                    __builtin_amdgcn_wave_barrier();
                    u32 dw[16];
#pragma unroll
                    for (int jj = 0; jj < 4; jj++) {
                        const v4i y = *(const v4i *)&tp[(s & 1) * PM_TP_WORDS + (n >> 2) * PM_TP_STRIDE + hi * 16 + jj * 4];
                        dw[jj * 4 + 0] = (u32)y[0]; dw[jj * 4 + 1] = (u32)y[1]; dw[jj * 4 + 2] = (u32)y[2]; dw[jj * 4 + 3] = (u32)y[3];
                    }
                    v4i o;
#pragma unroll
                    for (int q = 0; q < 4; q++) {
                        const u32 lo2 = __builtin_amdgcn_perm(dw[4 * q + 1], dw[4 * q + 0], bsel);
                        const u32 hi2 = __builtin_amdgcn_perm(dw[4 * q + 3], dw[4 * q + 2], bsel);
                        o[q] = (int)__builtin_amdgcn_perm(hi2, lo2, 0x05040100u);
                    }
                    Bt[s] = o;
                }
                pm_prf_pass(a, K, scr, (2 * ch) & 7, kg, ib, n, hi);
                pm_prf_pass(a, K, scr, (2 * ch + 1) & 7, kg, ib, n, hi);
#pragma unroll
                for (int t = 0; t < 2; t++)
#pragma unroll
                    for (int s = 0; s < 8; s++)
#pragma unroll
                        for (int u = 0; u < 8 - s; u++)
                            acc[s + u][t] = __builtin_amdgcn_mfma_i32_32x32x32_i8(A[t][s], Bt[u], acc[s + u][t], 0, 0, 0);
                // one matrix-core instruction, then a dozen vector instructions of the PRF, and so on
#pragma unroll
                for (int q = 0; q < 72; q++) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                    __builtin_amdgcn_sched_group_barrier(0x002, 12, 0);
                }
            }
#undef PM_LOAD
            for (u32 pass = 2 * nch; pass < 8; pass++) pm_prf_pass(a, K, scr, pass, kg, ib, n, hi);   // fewer than four chunks
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            __builtin_amdgcn_wave_barrier();
            // epilogue, one half of the tile (32 columns, 16 per lane) at a time: recombine the limb
            // levels, add the zero sharing, send the component to the predecessor, inner product with X
#pragma unroll
            for (int t = 0; t < 2; t++) {
                Sh xv[16];
                u32 nl = 0;
#pragma unroll
                for (int v = 0; v < 16; v++) {
                    const u64 kcol = (u64)kg * 64 + t * 32 + 8 * (v >> 2) + hi * 4 + (v & 3);
                    const bool live = ilive && kcol < a.d;
                    nl += live ? 1u : 0u;
                    xv[v] = live ? ld(a.XT, p, kcol * a.N8 + i) : Sh{ 0, 0 };
                }
                u64 snd[16];
#pragma unroll
                for (int v = 0; v < 16; v++) {
                    u64 z = 0;
#pragma unroll
                    for (int u = 0; u < 8; u++) z += (u64)(long long)acc[u][t][v] << (8 * u);
                    const u32 pass = t * 4 + (v >> 2), ri = hi * 4 + (v & 3);
                    snd[v] = z + (scr[((pass * 2) * 8 + ri) * 32 + n] - scr[((pass * 2 + 1) * 8 + ri) * 32 + n]);
                    s_x[p][v * GT_LANES + lane] = snd[v];
                }
                W.nresh += 64u * nl;
                __syncthreads();
#pragma unroll
                for (int v = 0; v < 16; v++) {
                    const Sh sel = { snd[v], s_x[pn][v * GT_LANES + lane] };
                    dacc += prod3(sel, xv[v]);                       // X is zero where the element does not exist
                }
                __syncthreads();
            }
        }
        // the two halves of the wavefront hold the sums over different rows of the same sample
        dacc += (u64)__shfl_xor((unsigned long long)dacc, 32, GT_LANES);
        {
            // zero sharing of the inner product: words ib*32 .. +31 of stream 0 under op+1, four blocks per key
            if (lane < 8) {
                const u32 mk = 0u - ((u32)lane >> 2);
                Key kv;
#pragma unroll
                for (int q = 0; q < 8; q++) kv.k[q] = K.own.k[q] ^ ((K.own.k[q] ^ K.nxt.k[q]) & mk);
                u64 blk[8];
                chacha8(kv, ib * 4 + (lane & 3), a.c.op + 1, 0, blk);
#pragma unroll
                for (int q = 0; q < 8; q++) scr[(lane >> 2) * 32 + (lane & 3) * 8 + q] = blk[q];
            }
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            __builtin_amdgcn_wave_barrier();
        }
        Sh z;
        z.o = dacc + (scr[n] - scr[32 + n]);
        z.n = W.reshare1(z.o, (ilive && hi == 0) ? 64u : 0u);
        if (ilive && hi == 0) st(a.M, p, i, scale(ld(a.M, p, i), 2) + z + one);
        __syncthreads();                         // the message slots and the scratch are rewritten by the next block
        W.drain();
    }
    W.flush(a.c.wire);
}
