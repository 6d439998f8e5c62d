// Kernels of the GTree hot path for gfx950.  See gt_device.hpp for the execution
// model (workgroup = 3 wavefronts = 3 parties; messages through LDS).
#pragma once
#include "gt_device.hpp"

#define GT_BLOCK dim3(GT_LANES, 3, 1)

// grid-stride loop over tiles of 64 elements; every lane of the workgroup runs the
// same number of iterations, so the barriers inside the protocols stay uniform
#define GT_FOR_TILES(n)                                                                    \
    for (u64 tile_ = blockIdx.x, ntiles_ = ((u64)(n) + GT_LANES - 1) / GT_LANES; tile_ < ntiles_; tile_ += gridDim.x)
#define GT_ELEM() (tile_ * GT_LANES + threadIdx.x)

// keys: the five keys; op: operation id; wire: the context's six message counters
// (payload bits sent by party p to its successor [2p] and to its predecessor [2p+1])
struct KCommon { const u32 *keys; u32 op; u64 *wire; };

// number of the lane's 8 consecutive elements (first one i0) that exist below n
__device__ __forceinline__ u32 live8(u64 i0, u64 n) { return i0 >= n ? 0u : (n - i0 >= 8 ? 8u : (u32)(n - i0)); }

__device__ __forceinline__ P6 p6_off(P6 a, size_t off)
{
    for (int j = 0; j < 3; j++) { a.o[j] += off; a.n[j] += off; }
    return a;
}

// ---------------------------------------------------------------------------------
// Share^A (Sec. II-B): x1, x2 from the owner's key (streams 0 and 1), x3 = x - x1 - x2.
// One lane produces 8 consecutive elements (one PRF block per stream).
// key: whose randomness shares the values (the data owner / query user, or the scorer of the
// heuristic by reconstruction, who uses the dealer's key); off: first element of `out`.
__global__ __launch_bounds__(256) void k_share(const u32 *keys, int key, u32 op, const u64 *plain, u64 n, P6 out, u64 off)
{
    const Key ko = load_key(keys, key);
    const u64 ngrp = (n + 7) / 8;
    for (u64 g = (u64)blockIdx.x * blockDim.x + threadIdx.x; g < ngrp; g += (u64)gridDim.x * blockDim.x) {
        u64 a[8], b[8];
        chacha8(ko, g, op, 0, a);
        chacha8(ko, g, op, 1, b);
#pragma unroll
        for (int s = 0; s < 8; s++) {
            const u64 e = g * 8 + s;
            if (e < n) {
                const u64 x3 = plain[e] - a[s] - b[s];
                out.o[0][off + e] = a[s]; out.n[0][off + e] = b[s];
                out.o[1][off + e] = b[s]; out.n[1][off + e] = x3;
                out.o[2][off + e] = x3;   out.n[2][off + e] = a[s];
            }
        }
    }
}

// Rec^A: party 0 adds its two components and the one it receives from party 2.
__global__ __launch_bounds__(256) void k_reconstruct(P6 in, u64 n, u64 *plain)
{
    for (u64 e = (u64)blockIdx.x * blockDim.x + threadIdx.x; e < n; e += (u64)gridDim.x * blockDim.x)
        plain[e] = in.o[0][e] + in.n[0][e] + in.o[2][e];
}

// local copy / strided gather of shares: dst[doff + e] = src[soff + e*sstride]
__global__ __launch_bounds__(256) void k_copy(P6 dst, u64 doff, P6 src, u64 soff, u64 sstride, u64 n)
{
    for (u64 e = (u64)blockIdx.x * blockDim.x + threadIdx.x; e < n; e += (u64)gridDim.x * blockDim.x)
        for (int j = 0; j < 3; j++) {
            dst.o[j][doff + e] = src.o[j][soff + e * sstride];
            dst.n[j][doff + e] = src.n[j][soff + e * sstride];
        }
}

// dst[k][i] (row stride N8) = src[i][k] (row stride w): sample-contiguous layout.
// 32 x 32 tiles through LDS so that both the reads and the writes are contiguous;
// blockIdx.z selects one of the six planes.
__global__ __launch_bounds__(256) void k_transpose(P6 dst, P6 src, u64 N, u64 N8, u32 w)
{
    __shared__ u64 tile[32][33];
    const int pl = blockIdx.z, tx = threadIdx.x & 31, ty = threadIdx.x >> 5;   // 32 x 8 threads
    const u64 *in = pl < 3 ? src.o[pl] : src.n[pl - 3];
    u64 *out = pl < 3 ? dst.o[pl] : dst.n[pl - 3];
    const u64 ntx = (w + 31) / 32, nty = (N + 31) / 32;
    for (u64 t = blockIdx.x; t < ntx * nty; t += gridDim.x) {
        const u64 k0 = (t % ntx) * 32, i0 = (t / ntx) * 32;
#pragma unroll
        for (int r = 0; r < 4; r++) {
            const u64 i = i0 + ty + 8 * r, k = k0 + tx;
            tile[ty + 8 * r][tx] = (i < N && k < w) ? in[i * w + k] : 0;
        }
        __syncthreads();
#pragma unroll
        for (int r = 0; r < 4; r++) {
            const u64 k = k0 + ty + 8 * r, i = i0 + tx;
            if (i < N && k < w) out[k * N8 + i] = tile[tx][ty + 8 * r];
        }
        __syncthreads();
    }
}

// eight consecutive words starting at a multiple of 8: vector loads when all eight lie
// inside the array and the address is 16-byte aligned, guarded loads (zero beyond n) otherwise
__device__ __forceinline__ void ld8(const u64 *ptr, u64 i0, u64 n, u64 (&x)[8])
{
    if (i0 + 8 <= n && ((size_t)(ptr + i0) & 15) == 0) {
        const ulonglong2 *q = (const ulonglong2 *)(ptr + i0);
#pragma unroll
        for (int j = 0; j < 4; j++) { const ulonglong2 v = q[j]; x[2 * j] = v.x; x[2 * j + 1] = v.y; }
    } else {
#pragma unroll
        for (int j = 0; j < 8; j++) x[j] = i0 + j < n ? ptr[i0 + j] : 0;
    }
}

// every element := public constant c
__global__ __launch_bounds__(256) void k_fill_const(P6 dst, u64 off, u64 n, u64 c)
{
    for (u64 e = (u64)blockIdx.x * blockDim.x + threadIdx.x; e < n; e += (u64)gridDim.x * blockDim.x)
        for (int j = 0; j < 3; j++) {
            dst.o[j][off + e] = j == 0 ? c : 0;
            dst.n[j][off + e] = j == 2 ? c : 0;
        }
}

// plain words := c
__global__ __launch_bounds__(256) void k_fill_words(u64 *dst, u64 n, u64 c)
{
    for (u64 e = (u64)blockIdx.x * blockDim.x + threadIdx.x; e < n; e += (u64)gridDim.x * blockDim.x) dst[e] = c;
}

// dst += src (local)
__global__ __launch_bounds__(256) void k_add_inplace(P6 dst, P6 src, u64 n)
{
    for (u64 e = (u64)blockIdx.x * blockDim.x + threadIdx.x; e < n; e += (u64)gridDim.x * blockDim.x)
        for (int j = 0; j < 3; j++) { dst.o[j][e] += src.o[j][e]; dst.n[j][e] += src.n[j][e]; }
}

// rows of width d: dst[2r] = dst[2r+1] = src[r] (children inherit gamma, Sec. V-B)
__global__ __launch_bounds__(256) void k_dup_rows(P6 dst, P6 src, u64 nh, u64 d)
{
    const u64 n = nh * d;
    for (u64 e = (u64)blockIdx.x * blockDim.x + threadIdx.x; e < n; e += (u64)gridDim.x * blockDim.x) {
        const u64 r = e / d, k = e % d;
        for (int j = 0; j < 3; j++) {
            dst.o[j][(2 * r) * d + k] = dst.o[j][(2 * r + 1) * d + k] = src.o[j][e];
            dst.n[j][(2 * r) * d + k] = dst.n[j][(2 * r + 1) * d + k] = src.n[j][e];
        }
    }
}

// idx[r*P2 + k] := k (public), val padding := 0
__global__ __launch_bounds__(256) void k_iota(P6 idx, P6 val, u32 nh, u32 P2, u32 d)
{
    const u64 n = (u64)nh * P2;
    for (u64 e = (u64)blockIdx.x * blockDim.x + threadIdx.x; e < n; e += (u64)gridDim.x * blockDim.x) {
        const u64 k = e % P2;
        for (int j = 0; j < 3; j++) {
            idx.o[j][e] = j == 0 ? k : 0;
            idx.n[j][e] = j == 2 ? k : 0;
            if (k >= d) { val.o[j][e] = 0; val.n[j][e] = 0; }
        }
    }
}

// ---------------------------------------------------------------------------------
// Limb-tiled layout of the two operands of the statistics contraction.  A 64-bit
// ring element is written as eight signed bytes d_s in [-128,127] with
// x = sum_s d_s 256^s (mod 2^64): add 0x80 to every byte position with carries, then
// flip the top bit of every byte.  A matrix M[row][sample] is stored as
// [sample block of 32][limb s][row][32 bytes], so that one lane of a matrix-core
// operand (one row, 16 consecutive samples, one limb) is one 16-byte load and a
// wavefront reads 1 KB contiguous per limb.  Samples beyond N hold zero bytes.
struct LimbMat { unsigned char *base; u64 rows; };      // rows = row stride of a limb plane
#define GT_BIAS 0x8080808080808080ull

__device__ __forceinline__ u64 limb_addr(const LimbMat &m, u64 ib, u32 s, u64 row) { return ((ib * 8 + s) * m.rows + row) * 32; }

// x[0..8) are 8 consecutive samples (first sample i0, a multiple of 8) of one row
// 8 x 8 byte transpose: afterwards byte j of y[s] is what byte s of y[j] was.  Three
// butterfly stages on byte, 16-bit and 32-bit units; the first two are byte permutes of
// register pairs, the last is a renaming of 32-bit halves.  Its own inverse.
__device__ __forceinline__ void transpose8x8(u64 (&y)[8])
{
    u32 lo[8], hi[8];
#pragma unroll
    for (int j = 0; j < 8; j++) { lo[j] = (u32)y[j]; hi[j] = (u32)(y[j] >> 32); }
#pragma unroll
    for (int j = 0; j < 8; j += 2) {
        const u32 al = lo[j], bl = lo[j + 1], ah = hi[j], bh = hi[j + 1];
        lo[j] = __builtin_amdgcn_perm(bl, al, 0x06020400u); lo[j + 1] = __builtin_amdgcn_perm(bl, al, 0x07030501u);
        hi[j] = __builtin_amdgcn_perm(bh, ah, 0x06020400u); hi[j + 1] = __builtin_amdgcn_perm(bh, ah, 0x07030501u);
    }
#pragma unroll
    for (int j = 0; j < 8; j += 4)
#pragma unroll
        for (int q = 0; q < 2; q++) {
            const u32 al = lo[j + q], bl = lo[j + q + 2], ah = hi[j + q], bh = hi[j + q + 2];
            lo[j + q] = __builtin_amdgcn_perm(bl, al, 0x05040100u); lo[j + q + 2] = __builtin_amdgcn_perm(bl, al, 0x07060302u);
            hi[j + q] = __builtin_amdgcn_perm(bh, ah, 0x05040100u); hi[j + q + 2] = __builtin_amdgcn_perm(bh, ah, 0x07060302u);
        }
#pragma unroll
    for (int q = 0; q < 4; q++) {
        y[q] = (u64)lo[q] | ((u64)lo[q + 4] << 32);
        y[q + 4] = (u64)hi[q] | ((u64)hi[q + 4] << 32);
    }
}

__device__ __forceinline__ void store_limbs8(const LimbMat &m, u64 row, u64 i0, const u64 (&x)[8])
{
    u64 y[8];
#pragma unroll
    for (int j = 0; j < 8; j++) y[j] = (x[j] + GT_BIAS) ^ GT_BIAS;
    transpose8x8(y);                                  // byte j of y[s] is limb s of sample j
    const u64 ib = i0 >> 5;
    const u32 off = (u32)i0 & 31;
#pragma unroll
    for (int sl = 0; sl < 8; sl++) *(u64 *)(m.base + limb_addr(m, ib, sl, row) + off) = y[sl];
}

// value of sample i of a row
__device__ __forceinline__ u64 load_limbs1(const LimbMat &m, u64 row, u64 i)
{
    u64 y = 0;
#pragma unroll
    for (int sl = 0; sl < 8; sl++) y |= (u64)m.base[limb_addr(m, i >> 5, sl, row) + (i & 31)] << (8 * sl);
    return (y ^ GT_BIAS) - GT_BIAS;
}

// The operands of the contraction z_p = x_p (y_p + y_{p+1}) + x_{p+1} y_p (the three-term
// product of Sec. II-B with the sum moved to the factor that is written once):
// B, the columns made at set-up, per party as (own+next, own); L, the leaf one-hot made anew at
// every level, one matrix per COMPONENT: component j is what party j holds as its own and
// party j-1 as its next part - the two copies are equal by construction, party j's
// wavefront writes the one that both holders read.
struct LimbSet { LimbMat m[3][2]; };
struct LimbTri { LimbMat m[3]; };

// ---------------------------------------------------------------------------------
// Elementwise product (Sec. II-B), 8 consecutive elements per lane.
// MODE 0: z[e] = x[e]*y[e].
// MODE 2 (node split): e = r*CW + col, z = C[e] * (1 - split[r]), written to both
//         children (2r, 2r+1) of the next level.
struct MultArgs { KCommon c; P6 x, y, z; u64 n, N, N8; u32 K, CW; };

template <int MODE>
__global__ __launch_bounds__(192) void k_mult(MultArgs a)
{
    const int p = party_of_wave(), lane = threadIdx.x;
    __shared__ u64 s_wire[GT_LWIRE_WORDS];
    __shared__ u64 s_cnt[6];
    Wire W; W.init(s_wire, s_cnt);
    const PartyKeys K = load_party_keys(a.c.keys, p);
    const u64 ngrp = (a.n + 7) / 8;
    for (u64 tile = blockIdx.x, nt = (ngrp + GT_LANES - 1) / GT_LANES; tile < nt; tile += gridDim.x) {
        const u64 g = tile * GT_LANES + lane, e0 = g * 8;
        u64 ao[8], an[8], snd[8], rcv[8];
        chacha8(K.own, g, a.c.op, 0, ao);
        chacha8(K.nxt, g, a.c.op, 0, an);
#pragma unroll
        for (int s = 0; s < 8; s++) {
            const u64 e = e0 + s;
            Sh x = { 0, 0 }, y = { 0, 0 };
            if (e < a.n) {
                if (MODE == 0) { x = ld(a.x, p, e); y = ld(a.y, p, e); }
                if (MODE == 2) { x = ld(a.x, p, e); y = pub(p, 1) - ld(a.y, p, e / a.CW); }
            }
            snd[s] = prod3(x, y) + (ao[s] - an[s]);
        }
        W.reshare<8>(snd, rcv, 64u * live8(e0, a.n));
#pragma unroll
        for (int s = 0; s < 8; s++) {
            const u64 e = e0 + s;
            if (e < a.n) {
                Sh z = { snd[s], rcv[s] };
                if (MODE == 0) st(a.z, p, e, z);
                if (MODE == 2) {
                    const u64 r = e / a.CW, col = e % a.CW;
                    st(a.z, p, (2 * r) * a.CW + col, z);
                    st(a.z, p, (2 * r + 1) * a.CW + col, z);
                }
            }
        }
    }
    W.flush(a.c.wire);
}

// One-time products of the learning protocol (Sec. V-B): column col = k*K + c,
// element e = col*N8 + i, z = XT[k][i] * YT[c][i] for i < N, written as limb tiles
// (own + next component into B.m[p][0], own into B.m[p][1]).  A step covers 16 groups of 8
// samples of four adjacent columns (blockIdx.y = column quad): the four 32-byte pieces
// that one wavefront writes per sample block and limb make up a whole 128-byte line
// of the tile layout.
struct XyArgs { KCommon c; P6 XT, YT; LimbSet B; u64 N, N8; u32 K, ncol; };
__global__ __launch_bounds__(192, 2) void k_xy(XyArgs a)
{
    __shared__ u64 s_wire[GT_LWIRE_WORDS];
    // the zero-sharing words under key k_j are evaluated by party j's wavefront and read
    // through LDS by party j-1, the other holder of k_j
    __shared__ u64 s_prf[3][8 * GT_LANES];
    __shared__ u64 s_cnt[6];
    const int p = party_of_wave(), lane = threadIdx.x, pn = p == 2 ? 0 : p + 1;
    LWire W; W.init(s_wire, s_cnt);
    const PartyKeys K = load_party_keys(a.c.keys, p);
    const u64 ngrp = a.N8 / 8, nq = (a.ncol + 3) / 4, nt = (ngrp + 15) / 16;
    // tiles outside, column quads inside: a workgroup meets the same class columns of Y
    // again and again for one tile of samples (cache hits) and each value of X once
    for (u64 tile = blockIdx.x; tile < nt; tile += gridDim.x) {
        const u64 g = tile * 16 + (lane & 15), i0 = g * 8;
        // the lane's class column of Y stays in registers while the class does not change from one
        // column quad to the next (never, when K divides 4 or 4 divides K)
        u64 yo[8] = { 0, 0, 0, 0, 0, 0, 0, 0 }, yn[8] = { 0, 0, 0, 0, 0, 0, 0, 0 }, cyc = ~(u64)0;
        for (u64 q = blockIdx.y; q < nq; q += gridDim.y) {
            const u64 colq = q * 4 + (lane >> 4);
            const bool act = colq < a.ncol && g < ngrp;
            const u64 col = act ? colq : 0, kx = col / a.K, cy = col % a.K;
            const u64 nv = act ? a.N : 0;               // rows start at multiples of 8
            u64 ao[8], snd[8], rcv[8];
            const u64 blk = (col * a.N8 + i0) >> 3;
            chacha8(K.own, blk, a.c.op, 0, ao);
#pragma unroll
            for (int s = 0; s < 8; s++) s_prf[p][s * GT_LANES + lane] = ao[s];
            u64 xo[8], xn[8];
            ld8(own_of(a.XT, p) + kx * a.N8, i0, nv, xo); ld8(nxt_of(a.XT, p) + kx * a.N8, i0, nv, xn);
            if (act && cy != cyc) {
                ld8(own_of(a.YT, p) + cy * a.N8, i0, nv, yo); ld8(nxt_of(a.YT, p) + cy * a.N8, i0, nv, yn);
                cyc = cy;
            }
#pragma unroll
            for (int s = 0; s < 8; s++) {
                const Sh x = { xo[s], xn[s] }, y = { yo[s], yn[s] };
                snd[s] = prod3(x, y) + ao[s];
            }
            __syncthreads();
#pragma unroll
            for (int s = 0; s < 8; s++) snd[s] -= s_prf[pn][s * GT_LANES + lane];
            W.reshare<8>(snd, rcv, 64u * live8(i0, nv));
            if (act) {
#pragma unroll
                for (int s = 0; s < 8; s++) { if (i0 + s >= a.N) { snd[s] = 0; rcv[s] = 0; } rcv[s] += snd[s]; }
                store_limbs8(a.B.m[p][0], col, i0, rcv);
                store_limbs8(a.B.m[p][1], col, i0, snd);
            }
        }
    }
    W.flush(a.c.wire);
}

// class indicator columns into limb tiles: row = rowbase + c
__global__ __launch_bounds__(256) void k_y_limbs(P6 YT, LimbSet B, u64 N, u64 N8, u32 K, u64 rowbase)
{
    const u64 ngrp = N8 / 8, total = ngrp * K;
    for (u64 t = (u64)blockIdx.x * blockDim.x + threadIdx.x; t < total; t += (u64)gridDim.x * blockDim.x) {
        const u64 c = t / ngrp, i0 = (t % ngrp) * 8;
        for (int p = 0; p < 3; p++) {
            u64 xo[8], xn[8];
#pragma unroll
            for (int s = 0; s < 8; s++) {
                const bool live = i0 + s < N;
                xo[s] = live ? YT.o[p][c * N8 + i0 + s] : 0; xn[s] = live ? xo[s] + YT.n[p][c * N8 + i0 + s] : 0;
            }
            store_limbs8(B.m[p][0], rowbase + c, i0, xn);
            store_limbs8(B.m[p][1], rowbase + c, i0, xo);
        }
    }
}

// per-sample leaf one-hot back to 64-bit words for export: out[r*N8 + i]
__global__ __launch_bounds__(256) void k_l_export(LimbTri L, P6 out, u64 nh, u64 N, u64 N8)
{
    const u64 total = nh * N8;
    for (u64 t = (u64)blockIdx.x * blockDim.x + threadIdx.x; t < total; t += (u64)gridDim.x * blockDim.x) {
        const u64 r = t / N8, i = t % N8;
        for (int p = 0; p < 3; p++) {
            u64 own = 0, nxt = 0;
            if (i < N) { own = load_limbs1(L.m[p], r, i); nxt = load_limbs1(L.m[p == 2 ? 0 : p + 1], r, i); }
            out.o[p][t] = own; out.n[p][t] = nxt;
        }
    }
}

// ---------------------------------------------------------------------------------
// Equality grid (first lines of the array-access protocol, Sec. V-A; per-sample leaf
// flags of the learning protocol, Sec. V-B).  Rows are samples i < N, columns k < w;
// element (k, i) has index k*N8 + i.  A lane owns 8 consecutive samples and walks
// over the columns, so that one PRF block yields the mask words of its 8 elements
// and the inner products of the array access accumulate in registers.
//   E[k][i] = [u[i] - base == k]  (and g[k] if HAS_G)  -> arithmetic sharing, then
//   GM_STORE : E written as limb tiles, the left operand of the statistics contraction
//   GM_COMMON: z[i] = sum_k E[k][i] * W1[w1off+k]   (NDOT = 2: also W2 -> out2)
//   GM_ROWS  : z[i] = sum_k E[k][i] * XT[k*N8+i]
//   epilogue 0: out[i] = z;  1: out[i] = 2*prev[i] + z + 1  (index update of the
//   partition and inference protocols).
enum { GM_STORE = 0, GM_COMMON = 1, GM_ROWS = 2 };
struct GridArgs {
    KCommon c;
    P6 u; u64 base; u32 w; u64 N, N8;
    P6 g, out, out2, W1, W2, XT, prev;
    u64 w1off, w2off;
    int epi;
    LimbTri L;      // GM_STORE: limb tiles of the components, row = column k
    u32 nkc, kchunk;// column ranges per tile and their length
    int lgs;        // GM_STORE: log2 of the lanes that share a column in one step (6 or 4)
    u64 *dacc;      // [2][3][N8] partial inner products when nkc > 1
    int ndot;
};

// The six AND rounds of eight equality tests held by one lane.  From the second round
// on the eight values stay packed in the format of the messages (fields of 16, 8, 4, 2
// bits and finally single bits, test s in field s), so that one word operation serves
// several tests: a round shifts the packed words by the field's half width, forms the
// three-term AND in every field at once (the upper half of each field then holds
// garbage that the compaction drops) and compacts the lower halves into the fields of
// the next message.  t: the lane's two Boolean components of the 64-bit inputs; A: the
// lane's mask words (own xor next key): bits 0-31 round 0, 32-47 round 1, 48-55 round 2,
// 56-59 round 3, 60-61 round 4, 62 round 5.  nl: how many of the eight tests exist (their
// bits are what the messages carry).  To8/Tn8: result bits, test s in bit s.
__device__ __forceinline__ u32 and3w(u32 ao, u32 an, u32 bo, u32 bn) { return (ao & (bo ^ bn)) ^ (an & bo); }

template <class WireT>
__device__ __forceinline__ void eq_rounds8_packed(WireT &W, const Sh (&t)[8], const u64 (&A)[8], u32 nl, u32 &To8, u32 &Tn8)
{
    u32 xo[8], xn[8], Ah[8];
    {   // round 0, width 32: the high word onto the low word; message 8 x 32 bits
        u64 snd[4], rcv[4];
#pragma unroll
        for (int s = 0; s < 8; s++)
            xo[s] = and3w((u32)t[s].o, (u32)t[s].n, (u32)(t[s].o >> 32), (u32)(t[s].n >> 32)) ^ (u32)A[s];
#pragma unroll
        for (int j = 0; j < 4; j++) snd[j] = (u64)xo[2 * j] | ((u64)xo[2 * j + 1] << 32);
        W.template reshare<4>(snd, rcv, 32u * nl);
#pragma unroll
        for (int j = 0; j < 4; j++) { xn[2 * j] = (u32)rcv[j]; xn[2 * j + 1] = (u32)(rcv[j] >> 32); }
    }
#pragma unroll
    for (int s = 0; s < 8; s++) Ah[s] = (u32)(A[s] >> 32);
    u32 Po[4], Pn[4];
    {   // round 1, width 16: message 8 x 16 bits, two tests per 32-bit word
        u64 snd[2], rcv[2];
        u32 z[8];
#pragma unroll
        for (int s = 0; s < 8; s++) z[s] = and3w(xo[s], xn[s], xo[s] >> 16, xn[s] >> 16) ^ Ah[s];
#pragma unroll
        for (int j = 0; j < 4; j++) Po[j] = __builtin_amdgcn_perm(z[2 * j + 1], z[2 * j], 0x05040100u);
#pragma unroll
        for (int j = 0; j < 2; j++) snd[j] = (u64)Po[2 * j] | ((u64)Po[2 * j + 1] << 32);
        W.template reshare<2>(snd, rcv, 16u * nl);
#pragma unroll
        for (int j = 0; j < 2; j++) { Pn[2 * j] = (u32)rcv[j]; Pn[2 * j + 1] = (u32)(rcv[j] >> 32); }
    }
    u32 Qo[2], Qn[2];
    {   // round 2, width 8: fields of 16 bits in, 8 bits out; masks = byte 2 of Ah
        u32 z[4];
#pragma unroll
        for (int j = 0; j < 4; j++)
            z[j] = and3w(Po[j], Pn[j], Po[j] >> 8, Pn[j] >> 8) ^ __builtin_amdgcn_perm(Ah[2 * j + 1], Ah[2 * j], 0x0c060c02u);
#pragma unroll
        for (int j = 0; j < 2; j++) Qo[j] = __builtin_amdgcn_perm(z[2 * j + 1], z[2 * j], 0x06040200u);
        u64 snd[1] = { (u64)Qo[0] | ((u64)Qo[1] << 32) }, rcv[1];
        W.template reshare<1>(snd, rcv, 8u * nl);
        Qn[0] = (u32)rcv[0]; Qn[1] = (u32)(rcv[0] >> 32);
    }
    // byte 3 of every Ah, test s in byte s: low nibble = masks of round 3, bits 4-5 of
    // round 4, bit 6 of round 5, bit 7 = mask of a following AND (bit 63 of A)
    u32 B3[2];
#pragma unroll
    for (int j = 0; j < 2; j++)
        B3[j] = __builtin_amdgcn_perm(Ah[4 * j + 1], Ah[4 * j], 0x0c0c0703u) | __builtin_amdgcn_perm(Ah[4 * j + 3], Ah[4 * j + 2], 0x07030c0cu);
    u32 Ro, Rn;
    {   // round 3, width 4: fields of 8 bits in, 4 bits out
        u32 y[2];
#pragma unroll
        for (int j = 0; j < 2; j++) {
            const u32 z = (and3w(Qo[j], Qn[j], Qo[j] >> 4, Qn[j] >> 4) ^ B3[j]) & 0x0f0f0f0fu;
            y[j] = z | (z >> 4);
        }
        Ro = __builtin_amdgcn_perm(y[1], y[0], 0x06040200u);
        u64 snd[1] = { (u64)Ro }, rcv[1];
        W.template reshare<1>(snd, rcv, 4u * nl);
        Rn = (u32)rcv[0];
    }
    u32 H;      // bits 28-31 of every Ah, test s in nibble s
    {
        u32 h[2];
#pragma unroll
        for (int j = 0; j < 2; j++) { const u32 x = (B3[j] >> 4) & 0x0f0f0f0fu; h[j] = x | (x >> 4); }
        H = __builtin_amdgcn_perm(h[1], h[0], 0x06040200u);
    }
    u32 So, Sn;
    {   // round 4, width 2: fields of 4 bits in, 2 bits out
        u32 z = (and3w(Ro, Rn, Ro >> 2, Rn >> 2) ^ H) & 0x33333333u;
        z = (z | (z >> 2)) & 0x0f0f0f0fu; z = (z | (z >> 4)) & 0x00ff00ffu; So = (z | (z >> 8)) & 0xffffu;
        u64 snd[1] = { (u64)So }, rcv[1];
        W.template reshare<1>(snd, rcv, 2u * nl);
        Sn = (u32)rcv[0];
    }
    {   // round 5, width 1: fields of 2 bits in, single bits out
        u32 m = (H >> 2) & 0x11111111u;
        m = (m | (m >> 2)) & 0x0f0f0f0fu; m = (m | (m >> 4)) & 0x00ff00ffu; m = (m | (m >> 8)) & 0xffffu;
        u32 z = (and3w(So, Sn, So >> 1, Sn >> 1) ^ m) & 0x5555u;
        z = (z | (z >> 1)) & 0x3333u; z = (z | (z >> 2)) & 0x0f0fu; To8 = (z | (z >> 4)) & 0xffu;
        u64 snd[1] = { (u64)To8 }, rcv[1];
        W.template reshare<1>(snd, rcv, nl);
        Tn8 = (u32)rcv[0];
    }
}

// bit 63 of the eight mask words, test s in bit s (mask of an AND that follows the rounds)
__device__ __forceinline__ u32 mask63_packed(const u64 (&A)[8])
{
    u32 g[2];
#pragma unroll
    for (int j = 0; j < 2; j++) {
        u32 x = 0;
#pragma unroll
        for (int i = 0; i < 4; i++) x |= (u32)(A[4 * j + i] >> 63) << (8 * i);
        g[j] = x;
    }
#pragma unroll
    for (int j = 0; j < 2; j++) { g[j] = (g[j] | (g[j] >> 7)) & 0x00030003u; g[j] = (g[j] | (g[j] >> 14)) & 0xfu; }
    return g[0] | (g[1] << 4);
}

// Offline and pairwise-key material is produced once per workgroup and handed out
// through LDS; a dealer block yields the components of all three parties (the dealer is a
// role of its own, not one of the parties), each party's wavefront then reads only its
// two components.
//  - Per work item: the edaBits of the lane's 8 samples (one per ROW of the grid: all
//    comparisons of a row are with public constants, so its masked index is opened once);
//    the three wavefronts split the 8 blocks, the opening goes through LDS, afterwards
//    every lane keeps the public c and its two Boolean components of r in registers.
//  - Per step (one column for the lane's 8 samples): the daBits of the 8 tests come from
//    three dealer blocks (stream 4, blocks 3g..3g+2 of the group g = e/8; test j in slot
//    j%3 of block 3g + j/3): party p's wavefront evaluates block 3g+p, one block per
//    lane; the mask word under key k_j is evaluated by party j's wavefront and also read
//    by party j-1, the other holder of k_j.
#define GT_TILE_EL (8 * GT_LANES)

// the three daBits of one dealer block into the rows of the arithmetic components (rows
// 6-8) and the packed bit words of lane ln: slot q serves test j = 3b + q of the group
__device__ __forceinline__ void deal_dabits(u64 (*s_mat)[GT_TILE_EL], u32 *bitw, const u64 (&D)[8], u32 b, u32 ln)
{
    u32 bits = 0;
#pragma unroll
    for (int q = 0; q < 3; q++) {
        const u32 j = 3 * b + q;
        if (j < 8) {
            const u32 el = j * GT_LANES + ln;
            const u64 beta = (D[6] >> (3 * q)) & 1;
            s_mat[6][el] = D[2 * q]; s_mat[7][el] = D[2 * q + 1]; s_mat[8][el] = beta - D[2 * q] - D[2 * q + 1];
            const u32 b0 = (u32)(D[6] >> (3 * q + 1)) & 1, b1 = (u32)(D[6] >> (3 * q + 2)) & 1, b2 = ((u32)beta ^ b0 ^ b1) & 1;
            bits |= (b0 << j) | (b1 << (8 + j)) | (b2 << (16 + j));
        }
    }
    atomicOr(&bitw[ln], bits);
}

template <int MODE, bool HAS_G, int NDOT>
__global__ __launch_bounds__(192, 3) void k_eqgrid(GridArgs a)
{
    // rows 0-2: the mask words under k_0..k_2; rows 3-5: the messages of the AND rounds, of
    // the bit conversion and of the reshared inner products; rows 6-8: beta arithmetic
    // components.  At the start of a work item rows 0-5 carry the edaBit components of the
    // lane's samples and the opening.
    __shared__ u64 s_mat[9][GT_TILE_EL];
    // beta Boolean components, packed per lane: bit 8j+s = component j of the lane's test s.
    // The dealer's lanes OR their bits in; two copies alternate between steps so that
    // one can be cleared while the other is in use.
    __shared__ u32 s_bitw[2][GT_LANES];
    __shared__ u64 s_cnt[6];
    const int p = party_of_wave(), lane = threadIdx.x, tid = p * GT_LANES + lane, pn = p == 2 ? 0 : p + 1, pp = p == 0 ? 2 : p - 1;
    LWire LW; LW.init(&s_mat[3][0], s_cnt);
    static_assert(GT_LWIRE_WORDS <= 3 * GT_TILE_EL, "LDS wire does not fit the rows it uses");
    const PartyKeys K = load_party_keys(a.c.keys, p);
    const u32 op = a.c.op;
    const u64 ngrp = a.N8 / 8;
    const Sh one = pub(p, 1);
    // work item = (tile of samples, range of columns); with more than one column
    // range per tile the inner products are completed by atomic adds (exact in the
    // ring) and the reshare runs in k_dot_fin.  A step covers 64 groups of 8 samples
    // of one column, or (leaf one-hot with a column count that is a multiple of four)
    // 16 groups of four adjacent columns each: the four 32-byte pieces that one
    // wavefront then writes per sample block and limb make up whole 128-byte lines of
    // the tile layout.
    const int lgs = MODE == GM_STORE ? a.lgs : 6;      // log2 of the lanes per column
    const u32 lgm = (1u << lgs) - 1, kstep = GT_LANES >> lgs, ro = lane >> lgs;
    const u64 nt = (ngrp + lgm) >> lgs;
    if (tid < 2 * GT_LANES) (&s_bitw[0][0])[tid] = 0;
    __syncthreads();
    u32 par = 0;
    for (u64 item = blockIdx.x; item < nt * a.nkc; item += gridDim.x) {
        const u64 tile = item / a.nkc;
        const u32 kbeg = (u32)(item % a.nkc) * a.kchunk, kend = kbeg + a.kchunk < a.w ? kbeg + a.kchunk : a.w;
        const u64 grp = (tile << lgs) + (lane & lgm), i0 = grp * 8;
        const bool actg = grp < ngrp;
        const u64 nvg = actg ? a.N : 0;
        // ---- the row's part: edaBits of the 8 samples, masked indices, one opening
        u64 cpub[8], rho_o[8], rho_n[8];
        {
#pragma unroll 1
            for (int s = p; s < 8; s += 3) {            // this party's share of the 8 dealer blocks of the lane
                u64 D[8];
                chacha8(K.dlr, i0 + s, op, 0, D);
                const int el = s * GT_LANES + lane;
                s_mat[0][el] = D[1]; s_mat[1][el] = D[2]; s_mat[2][el] = D[0] - D[1] - D[2];
                s_mat[3][el] = D[3]; s_mat[4][el] = D[4]; s_mat[5][el] = D[0] ^ D[3] ^ D[4];
            }
            u64 snd[8], mn[8];
            ld8(own_of(a.u, p), i0, nvg, snd); ld8(nxt_of(a.u, p), i0, nvg, mn);
            __syncthreads();
#pragma unroll
            for (int s = 0; s < 8; s++) {
                const int el = s * GT_LANES + lane;
                snd[s] += s_mat[p][el];                 // samples beyond N: any value serves
                mn[s] += s_mat[pn][el];
                rho_o[s] = s_mat[3 + p][el]; rho_n[s] = s_mat[3 + pn][el];
            }
            __syncthreads();
            // the opening, 64 bits per sample: party p's message takes the place of row p.  The column
            // ranges of one tile (and the four column lanes of the leaf grid) replay the same opening;
            // it is counted once.
#pragma unroll
            for (int s = 0; s < 8; s++) s_mat[p][s * GT_LANES + lane] = snd[s];
            if (kbeg == 0 && ro == 0) LW.nopen += 64u * live8(i0, nvg);
            __syncthreads();
#pragma unroll
            for (int s = 0; s < 8; s++) cpub[s] = snd[s] + mn[s] + s_mat[pp][s * GT_LANES + lane] - a.base;
            __syncthreads();
        }
        u64 acc[8], acc2[8];
#pragma unroll
        for (int s = 0; s < 8; s++) { acc[s] = 0; acc2[s] = 0; }
        for (u32 k0 = kbeg; k0 < kend; k0 += kstep) {
            const bool act = MODE == GM_STORE ? actg && k0 + ro < kend : actg;
            const u32 k = MODE == GM_STORE ? (act ? k0 + ro : kbeg) : k0;   // this lane's column (an existing one when idle)
            const u64 nv = act ? a.N : 0;              // samples of this lane that exist
            const u32 nl = live8(i0, nv);              // how many of the lane's eight tests exist
            const u64 e0 = (u64)k * a.N8 + i0;
            u64 A[8];
            {
                u64 D[8];
                chacha8(K.dlr, 3 * (e0 >> 3) + p, op, 4, D);       // daBits of the tests 3p, 3p+1, 3p+2 of the lane
                deal_dabits(s_mat, s_bitw[par], D, (u32)p, (u32)lane);
            }
            chacha8(K.own, e0 >> 3, op, 1, A);         // mask words under this party's own key
#pragma unroll
            for (int s = 0; s < 8; s++) s_mat[p][s * GT_LANES + lane] = A[s];
            __syncthreads();
            if (p == 0) s_bitw[par ^ 1][lane] = 0;     // the next step's bit words
#pragma unroll
            for (int s = 0; s < 8; s++) A[s] ^= s_mat[pn][s * GT_LANES + lane];
            // t = rho with the complement of (c - base - k) xored into component 0, which
            // party 0 holds as its own and party 2 as its next component
            Sh t[8];
#pragma unroll
            for (int s = 0; s < 8; s++) {
                const u64 nx = ~(cpub[s] - k);
                t[s].o = p == 0 ? rho_o[s] ^ nx : rho_o[s];
                t[s].n = p == 2 ? rho_n[s] ^ nx : rho_n[s];
            }
            u32 To8, Tn8;
            eq_rounds8_packed(LW, t, A, nl, To8, Tn8); // six AND rounds, 63 bits
            if (HAS_G) {                               // and with the column's shared bit
                const Sh gk = ld(a.g, p, k);
                const u32 go = 0u - ((u32)gk.o & 1), gn = 0u - ((u32)gk.n & 1);
                To8 = (and3w(To8, Tn8, go, gn) ^ mask63_packed(A)) & 0xffu;
                u64 s1[1] = { (u64)To8 }, r1[1];
                LW.reshare<1>(s1, r1, nl);
                Tn8 = (u32)r1[0];
            }
            u32 f;
            {                                          // bit -> arithmetic: open s xor beta
                const u32 bw = s_bitw[par][lane];
                const u32 fo = To8 ^ ((bw >> (8 * p)) & 0xffu), fn = Tn8 ^ ((bw >> (8 * pn)) & 0xffu);
                f = fo ^ fn ^ (u32)LW.open1((u64)fo, nl);
            }
            Sh Wk = { 0, 0 }, Wk2 = { 0, 0 };
            if (MODE == GM_COMMON) {
                Wk = ld(a.W1, p, a.w1off + k);
                if (NDOT == 2) Wk2 = ld(a.W2, p, a.w2off + k);
            }
            u64 Eo[8], xo[8], xn[8];
            if (MODE == GM_ROWS) { ld8(own_of(a.XT, p) + (u64)k * a.N8, i0, nv, xo); ld8(nxt_of(a.XT, p) + (u64)k * a.N8, i0, nv, xn); }
#pragma unroll
            for (int s = 0; s < 8; s++) {
                const int el = s * GT_LANES + lane;
                const Sh bA = { s_mat[6 + p][el], s_mat[6 + pn][el] };
                Sh E;
                E.o = ((f >> s) & 1) ? one.o - bA.o : bA.o;
                E.n = ((f >> s) & 1) ? one.n - bA.n : bA.n;
                const bool live = i0 + s < nv;
                if (MODE == GM_STORE) Eo[s] = live ? E.o : 0;
                if (MODE == GM_COMMON) { acc[s] += prod3(E, Wk); if (NDOT == 2) acc2[s] += prod3(E, Wk2); }
                if (MODE == GM_ROWS) { const Sh x = { xo[s], xn[s] }; acc[s] += prod3(E, x); }
            }
            if (MODE == GM_STORE && act) {
                store_limbs8(a.L.m[p], k, i0, Eo);
            }
            par ^= 1;
            __syncthreads();                           // the material in LDS is overwritten next
        }
        if (MODE != GM_STORE && a.nkc > 1) {
#pragma unroll
            for (int s = 0; s < 8; s++)
                if (i0 + s < nvg) {
                    atomicAdd((unsigned long long *)&a.dacc[(u64)p * a.N8 + i0 + s], (unsigned long long)acc[s]);
                    if (NDOT == 2) atomicAdd((unsigned long long *)&a.dacc[(u64)(3 + p) * a.N8 + i0 + s], (unsigned long long)acc2[s]);
                }
        }
        if (MODE != GM_STORE && a.nkc == 1) {
            u64 ao[8], an[8], snd[8], rcv[8];
            chacha8(K.own, grp, op, 2, ao);
            chacha8(K.nxt, grp, op, 2, an);
#pragma unroll
            for (int s = 0; s < 8; s++) snd[s] = acc[s] + (ao[s] - an[s]);
            LW.reshare<8>(snd, rcv, 64u * live8(i0, nvg));
#pragma unroll
            for (int s = 0; s < 8; s++) {
                if (actg && i0 + s < a.N) {
                    Sh z = { snd[s], rcv[s] };
                    if (a.epi == 1) z = scale(ld(a.prev, p, i0 + s), 2) + z + one;
                    st(a.out, p, i0 + s, z);
                }
            }
            if (NDOT == 2) {
                chacha8(K.own, grp, op, 3, ao);
                chacha8(K.nxt, grp, op, 3, an);
#pragma unroll
                for (int s = 0; s < 8; s++) snd[s] = acc2[s] + (ao[s] - an[s]);
                LW.reshare<8>(snd, rcv, 64u * live8(i0, nvg));
#pragma unroll
                for (int s = 0; s < 8; s++)
                    if (actg && i0 + s < a.N) { Sh z = { snd[s], rcv[s] }; st(a.out2, p, i0 + s, z); }
            }
        }
        LW.drain();
    }
    LW.flush(a.c.wire);
}

// Completion of split inner products: z_p = partial sum + alpha (stream 2, second
// output stream 3), reshare, epilogue as in k_eqgrid.  Eight rows per lane.
__global__ __launch_bounds__(192) void k_dot_fin(GridArgs a)
{
    const int p = party_of_wave(), lane = threadIdx.x;
    __shared__ u64 s_wire[GT_LWIRE_WORDS];
    __shared__ u64 s_cnt[6];
    Wire W; W.init(s_wire, s_cnt);
    const PartyKeys K = load_party_keys(a.c.keys, p);
    const u64 ngrp = a.N8 / 8;
    const Sh one = pub(p, 1);
    for (u64 tile = blockIdx.x, nt = (ngrp + GT_LANES - 1) / GT_LANES; tile < nt; tile += gridDim.x) {
        const u64 grp = tile * GT_LANES + lane, i0 = grp * 8;
        const u64 nv = grp < ngrp ? a.N : 0;
        for (int q = 0; q < a.ndot; q++) {
            u64 ao[8], an[8], snd[8], rcv[8];
            chacha8(K.own, grp, a.c.op, 2 + q, ao);
            chacha8(K.nxt, grp, a.c.op, 2 + q, an);
#pragma unroll
            for (int s = 0; s < 8; s++) {
                u64 part = 0;
                if (i0 + s < nv) {                     // take the partial sum and leave zero for the next grid
                    u64 *d = &a.dacc[(u64)(3 * q + p) * a.N8 + i0 + s];
                    part = *d; *d = 0;
                }
                snd[s] = part + (ao[s] - an[s]);
            }
            W.reshare<8>(snd, rcv, 64u * live8(i0, nv));
#pragma unroll
            for (int s = 0; s < 8; s++)
                if (i0 + s < nv) {
                    Sh z = { snd[s], rcv[s] };
                    if (q == 0 && a.epi == 1) z = scale(ld(a.prev, p, i0 + s), 2) + z + one;
                    st(q == 0 ? a.out : a.out2, p, i0 + s, z);
                }
        }
    }
    W.flush(a.c.wire);
}

// ---------------------------------------------------------------------------------
// Small per-element protocols, one element per lane.

// z = B2A([x - y_pub == 0]) or the Boolean bit (BOOL_OUT)
struct EqArgs { KCommon c; P6 x; const u64 *ypub; u64 ysub; P6 z; u64 n, xoff; };
template <bool BOOL_OUT>
__global__ __launch_bounds__(192) void k_eq(EqArgs a)
{
    const int p = party_of_wave();
    __shared__ u64 s_wire[GT_LWIRE_WORDS];
    __shared__ u64 s_cnt[6];
    Wire W; W.init(s_wire, s_cnt);
    __shared__ u64 s_prf[3][GT_PRF_SCRATCH_WORDS];
    const PartyKeys K = load_party_keys(a.c.keys, p, s_prf[p]);
    GT_FOR_TILES(a.n) {
        const u64 e = GT_ELEM();
        const bool act = e < a.n;
        Sh v = { 0, 0 };
        if (act) v = ld(a.x, p, a.xoff + e) - pub(p, a.ysub + (a.ypub ? a.ypub[e] : 0));
        const Dealer D = dealer_of(K, p, a.c.op, e);
        u64 A;
        Sh b = eq_bit(W, K, p, a.c.op, e, v, D, A, act);
        if (!BOOL_OUT) b = b2a(W, p, b, D, act);
        if (act) st(a.z, p, e, b);
    }
    W.flush(a.c.wire);
}

// z = B2A([x >= y])
struct GeArgs { KCommon c; P6 x, y, z; u64 n; };
__global__ __launch_bounds__(192) void k_ge(GeArgs a)
{
    const int p = party_of_wave();
    __shared__ u64 s_wire[GT_LWIRE_WORDS];
    __shared__ u64 s_cnt[6];
    Wire W; W.init(s_wire, s_cnt);
    __shared__ u64 s_prf[3][GT_PRF_SCRATCH_WORDS];
    const PartyKeys K = load_party_keys(a.c.keys, p, s_prf[p]);
    GT_FOR_TILES(a.n) {
        const u64 e = GT_ELEM();
        const bool act = e < a.n;
        Sh v = { 0, 0 };
        if (act) v = ld(a.x, p, e) - ld(a.y, p, e);
        const Dealer D = dealer_of(K, p, a.c.op, e);
        Sh b = b2a(W, p, ge_bit(W, K, p, a.c.op, e, v, D, act), D, act);
        if (act) st(a.z, p, e, b);
    }
    W.flush(a.c.wire);
}

// Inference, threshold mode: bit = [x > theta]; Tidx <- 2 Tidx + bit + 1.
struct CmpArgs { KCommon c; P6 th, x, tidx; u64 n; };
__global__ __launch_bounds__(192) void k_cmp_step(CmpArgs a)
{
    const int p = party_of_wave();
    __shared__ u64 s_wire[GT_LWIRE_WORDS];
    __shared__ u64 s_cnt[6];
    Wire W; W.init(s_wire, s_cnt);
    __shared__ u64 s_prf[3][GT_PRF_SCRATCH_WORDS];
    const PartyKeys K = load_party_keys(a.c.keys, p, s_prf[p]);
    GT_FOR_TILES(a.n) {
        const u64 e = GT_ELEM();
        const bool act = e < a.n;
        Sh v = { 0, 0 };
        if (act) v = ld(a.th, p, e) - ld(a.x, p, e);
        const Dealer D = dealer_of(K, p, a.c.op, e);
        Sh b = b2a(W, p, not_bit(p, ge_bit(W, K, p, a.c.op, e, v, D, act)), D, act);
        if (act) st(a.tidx, p, e, scale(ld(a.tidx, p, e), 2) + b + pub(p, 1));
    }
    W.flush(a.c.wire);
}

// Restoring division, all steps of an element in one launch (the steps of different
// elements do not interact): step t uses operation id op + t; b = [r >= Q]; r <- r - b Q;
// quo <- 2 quo + b; r starts as S and is doubled between steps.
struct DivArgs { KCommon c; P6 S, Q, r, quo; u64 n; u32 nsteps; };
__global__ __launch_bounds__(192) void k_div(DivArgs a)
{
    const int p = party_of_wave();
    __shared__ u64 s_wire[GT_LWIRE_WORDS];
    __shared__ u64 s_cnt[6];
    Wire W; W.init(s_wire, s_cnt);
    __shared__ u64 s_prf[3][GT_PRF_SCRATCH_WORDS];
    const PartyKeys K = load_party_keys(a.c.keys, p, s_prf[p]);
    GT_FOR_TILES(a.n) {
        const u64 e = GT_ELEM();
        const bool act = e < a.n;
        Sh r = { 0, 0 }, Q = { 0, 0 }, quo = { 0, 0 };
        if (act) { Q = ld(a.Q, p, e); r = ld(a.S, p, e); }
        for (u32 t = 0; t < a.nsteps; t++) {
            const u32 op = a.c.op + t;
            if (t) r = scale(r, 2);
            const Dealer D = dealer_of(K, p, op, e);
            const Sh b = b2a(W, p, ge_bit(W, K, p, op, e, r - Q, D, act), D, act);
            const Sh bq = mult_sh(W, b, Q, zero_a(K, op, 3, e), act);
            r = r - bq;
            quo = scale(quo, 2) + b;
        }
        if (act) { st(a.r, p, e, r); st(a.quo, p, e, quo); }
    }
    W.flush(a.c.wire);
}

// Gini numerator/denominator terms (Sec. V-B, Eq. (1)): element q = (r*d+k)*2 + j,
// S = sum_c n_jc^2, Q = n_j * n with n_1c = C[r][k*K+c], n_0c = tot_c - n_1c.
struct PrepArgs { KCommon c; P6 C, S, Q; u64 n; u32 d, K, CW; };
__global__ __launch_bounds__(192) void k_score_prep(PrepArgs a)
{
    const int p = party_of_wave();
    __shared__ u64 s_wire[GT_LWIRE_WORDS];
    __shared__ u64 s_cnt[6];
    Wire W; W.init(s_wire, s_cnt);
    __shared__ u64 s_prf[3][GT_PRF_SCRATCH_WORDS];
    const PartyKeys K = load_party_keys(a.c.keys, p, s_prf[p]);
    const u64 dK = (u64)a.d * a.K;
    GT_FOR_TILES(a.n) {
        const u64 q = GT_ELEM();
        const bool act = q < a.n;
        Sh nj = { 0, 0 }, n = { 0, 0 };
        u64 s = 0;
        if (act) {
            const u64 r = q / (2 * a.d), k = (q / 2) % a.d, br = q & 1;
            for (u32 cl = 0; cl < a.K; cl++) {
                const Sh n1 = ld(a.C, p, r * a.CW + k * a.K + cl), tot = ld(a.C, p, r * a.CW + dK + cl);
                const Sh njc = br ? n1 : tot - n1;
                nj = nj + njc; n = n + tot;
                s += prod3(njc, njc);
            }
        }
        u64 z0, z1;
        zero_a2(K, a.c.op, 0, 1, q, z0, z1);
        u64 snd[2] = { s + z0, prod3(nj, n) + z1 }, rcv[2];
        W.reshare<2>(snd, rcv, act ? 128u : 0u);
        if (act) { Sh S = { snd[0], rcv[0] }, Q = { snd[1], rcv[1] }; st(a.S, p, q, S); st(a.Q, p, q, Q); }
    }
    W.flush(a.c.wire);
}

// score = quo[2e] + quo[2e+1]; masked = score * gamma[e]; written to the export copy
// and into the tournament array val[r*P2 + k].
struct MaskArgs { KCommon c; P6 quo, gamma, score, val; u64 n; u32 d, P2; };
__global__ __launch_bounds__(192) void k_mask_score(MaskArgs a)
{
    const int p = party_of_wave();
    __shared__ u64 s_wire[GT_LWIRE_WORDS];
    __shared__ u64 s_cnt[6];
    Wire W; W.init(s_wire, s_cnt);
    __shared__ u64 s_prf[3][GT_PRF_SCRATCH_WORDS];
    const PartyKeys K = load_party_keys(a.c.keys, p, s_prf[p]);
    GT_FOR_TILES(a.n) {
        const u64 e = GT_ELEM();
        const bool act = e < a.n;
        Sh s = { 0, 0 }, g = { 0, 0 };
        if (act) { s = ld(a.quo, p, 2 * e) + ld(a.quo, p, 2 * e + 1); g = ld(a.gamma, p, e); }
        const Sh z = mult_sh(W, s, g, zero_a(K, a.c.op, 0, e), act);
        if (act) { st(a.score, p, e, z); st(a.val, p, (e / a.d) * a.P2 + e % a.d, z); }
    }
    W.flush(a.c.wire);
}

// Compare-and-select: b = [right > left]; val = left + b (right-left); idx likewise.
// mode 0 (tournament level over arrays of length len per node): e = r*half + m,
//        left = in[r*len+2m], right = in[r*len+2m+1], out[e].
// mode 1 (label chain): left = val_in[e] / idx_in[e], right = C[e*CW + coff], index
//        constant cidx; in place.
struct SelArgs { KCommon c; P6 vin, iin, vout, iout, C; u64 n; u32 len, CW; u64 coff, cidx; int mode; };
__global__ __launch_bounds__(192) void k_select_max(SelArgs a)
{
    const int p = party_of_wave();
    __shared__ u64 s_wire[GT_LWIRE_WORDS];
    __shared__ u64 s_cnt[6];
    Wire W; W.init(s_wire, s_cnt);
    __shared__ u64 s_prf[3][GT_PRF_SCRATCH_WORDS];
    const PartyKeys K = load_party_keys(a.c.keys, p, s_prf[p]);
    GT_FOR_TILES(a.n) {
        const u64 e = GT_ELEM();
        const bool act = e < a.n;
        Sh L = { 0, 0 }, R = { 0, 0 }, IL = { 0, 0 }, IR = { 0, 0 };
        if (act) {
            if (a.mode == 0) {
                const u64 half = a.len / 2, r = e / half, m = e % half, l = r * a.len + 2 * m;
                L = ld(a.vin, p, l); R = ld(a.vin, p, l + 1); IL = ld(a.iin, p, l); IR = ld(a.iin, p, l + 1);
            } else {
                L = ld(a.vin, p, e); IL = ld(a.iin, p, e);
                R = ld(a.C, p, e * a.CW + a.coff); IR = pub(p, a.cidx);
            }
        }
        const Dealer D = dealer_of(K, p, a.c.op, e);
        const Sh b = b2a(W, p, not_bit(p, ge_bit(W, K, p, a.c.op, e, L - R, D, act)), D, act);
        u64 z3, z4;
        zero_a2(K, a.c.op, 3, 4, e, z3, z4);
        u64 snd[2] = { prod3(b, R - L) + z3, prod3(b, IR - IL) + z4 }, rcv[2];
        W.reshare<2>(snd, rcv, act ? 128u : 0u);
        if (act) {
            Sh dv = { snd[0], rcv[0] }, di = { snd[1], rcv[1] };
            st(a.vout, p, e, L + dv); st(a.iout, p, e, IL + di);
        }
    }
    W.flush(a.c.wire);
}

// gamma[r][k] <- gamma[r][k] * (1 - [SD[r] == k])
struct GammaArgs { KCommon c; P6 SD, gamma; u64 n; u32 d; };
__global__ __launch_bounds__(192) void k_gamma(GammaArgs a)
{
    const int p = party_of_wave();
    __shared__ u64 s_wire[GT_LWIRE_WORDS];
    __shared__ u64 s_cnt[6];
    Wire W; W.init(s_wire, s_cnt);
    __shared__ u64 s_prf[3][GT_PRF_SCRATCH_WORDS];
    const PartyKeys K = load_party_keys(a.c.keys, p, s_prf[p]);
    GT_FOR_TILES(a.n) {
        const u64 e = GT_ELEM();
        const bool act = e < a.n;
        Sh v = { 0, 0 }, g = { 0, 0 };
        if (act) { v = ld(a.SD, p, e / a.d) - pub(p, e % a.d); g = ld(a.gamma, p, e); }
        const Dealer D = dealer_of(K, p, a.c.op, e);
        u64 A;
        const Sh oh = b2a(W, p, eq_bit(W, K, p, a.c.op, e, v, D, A, act), D, act);
        const Sh z = mult_sh(W, g, pub(p, 1) - oh, zero_a(K, a.c.op, 2, e), act);
        if (act) st(a.gamma, p, e, z);
    }
    W.flush(a.c.wire);
}

// Node r: pure = [n^2 - sum_c tot_c^2 == 0]; split = isLeaf and not pure;
// F[base+r] <- F (1 - split); children F <- 2 - split.
struct SplitArgs { KCommon c; P6 C, isLeaf, F, split; u64 n, base; u32 K, CW; u64 dK; };
__global__ __launch_bounds__(192) void k_split(SplitArgs a)
{
    const int p = party_of_wave();
    __shared__ u64 s_wire[GT_LWIRE_WORDS];
    __shared__ u64 s_cnt[6];
    Wire W; W.init(s_wire, s_cnt);
    __shared__ u64 s_prf[3][GT_PRF_SCRATCH_WORDS];
    const PartyKeys K = load_party_keys(a.c.keys, p, s_prf[p]);
    GT_FOR_TILES(a.n) {
        const u64 r = GT_ELEM();
        const bool act = r < a.n;
        Sh n = { 0, 0 }, leaf = { 0, 0 }, f = { 0, 0 };
        u64 dv = 0;
        if (act) {
            for (u32 cl = 0; cl < a.K; cl++) {
                const Sh tc = ld(a.C, p, r * a.CW + a.dK + cl);
                n = n + tc;
                dv -= prod3(tc, tc);
            }
            dv += prod3(n, n);
            leaf = ld(a.isLeaf, p, r);
            f = ld(a.F, p, a.base + r);
        }
        Sh d;
        d.o = dv + zero_a(K, a.c.op, 2, r);
        d.n = W.reshare1(d.o, act ? 64u : 0u);
        const Dealer D = dealer_of(K, p, a.c.op, r);
        u64 A;
        const Sh npure = not_bit(p, eq_bit(W, K, p, a.c.op, r, d, D, A, act));
        const Sh sA = b2a(W, p, and_bit(W, leaf, npure, A >> 63, act), D, act);
        const Sh keep = pub(p, 1) - sA;
        const Sh fz = mult_sh(W, f, keep, zero_a(K, a.c.op, 3, r), act);
        if (act) {
            st(a.split, p, r, sA);
            st(a.F, p, a.base + r, fz);
            const Sh ch = keep + pub(p, 1);
            st(a.F, p, 2 * (a.base + r) + 1, ch);
            st(a.F, p, 2 * (a.base + r) + 2, ch);
        }
    }
    W.flush(a.c.wire);
}

// ---------------------------------------------------------------------------------
// Data partition by products with the previous level's per-sample leaf one-hot (a variant
// beyond the paper's listing: no per-sample equality tests).
//   k_onehot  : OH[r*d + k] = [T[base + r] == k] as an arithmetic sharing
//   k_part_mm : sel[k][i] = sum_r L[r][i] * OH[r][k], zero sharing of stream 0, word k*N8+i, and
//               M[i] <- 2 M[i] + sum_k sel[k][i] * X[k][i] + 1, zero sharing of stream 0, word i
//               (gt_partmm.hpp, on the matrix cores)
struct OnehotArgs { KCommon c; P6 T, OH; u64 base, n; u32 d; };
__global__ __launch_bounds__(192) void k_onehot(OnehotArgs a)
{
    const int p = party_of_wave();
    __shared__ u64 s_wire[GT_LWIRE_WORDS];
    __shared__ u64 s_cnt[6];
    Wire W; W.init(s_wire, s_cnt);
    __shared__ u64 s_prf[3][GT_PRF_SCRATCH_WORDS];
    const PartyKeys K = load_party_keys(a.c.keys, p, s_prf[p]);
    GT_FOR_TILES(a.n) {
        const u64 e = GT_ELEM();
        const bool act = e < a.n;
        Sh v = { 0, 0 };
        if (act) v = ld(a.T, p, a.base + e / a.d) - pub(p, e % a.d);
        const Dealer D = dealer_of(K, p, a.c.op, e);
        u64 A;
        const Sh oh = b2a(W, p, eq_bit(W, K, p, a.c.op, e, v, D, A, act), D, act);
        if (act) st(a.OH, p, e, oh);
    }
    W.flush(a.c.wire);
}

// ---------------------------------------------------------------------------------
// The protocols as the paper prints them (Sec. V-A, Alg. "Oblivious Array Access"; Sec. V-B,
// Alg. "Oblivious Learning"), for small inputs: every array element goes through a
// SelectShare of its own - conversion of the comparison bit with the element's own daBit,
// the opened value counted as a ring element, then a product with a zero-sharing word and
// a reshare of its own - and the selected elements are added up locally (atomic adds of
// both components: exact and order-free in the ring).  One element per lane; streams 0
// dealer, 1 masks, 2 product, all indexed by the element.
struct LitOaaArgs { KCommon c; P6 u; u64 base; u32 w; u64 N, N8; P6 W1; u64 w1off; P6 XT; u64 *acc; };
template <bool ROWS>
__global__ __launch_bounds__(192) void k_oaa_literal(LitOaaArgs a)
{
    const int p = party_of_wave();
    __shared__ u64 s_wire[GT_LWIRE_WORDS];
    __shared__ u64 s_cnt[6];
    Wire W; W.init(s_wire, s_cnt);
    __shared__ u64 s_prf[3][GT_PRF_SCRATCH_WORDS];
    const PartyKeys K = load_party_keys(a.c.keys, p, s_prf[p]);
    GT_FOR_TILES((u64)a.w * a.N8) {
        const u64 e = GT_ELEM(), k = e / a.N8, i = e % a.N8;
        const bool act = k < a.w && i < a.N;
        Sh v = { 0, 0 }, wv = { 0, 0 };
        if (act) {
            v = ld(a.u, p, i) - pub(p, a.base + k);
            wv = ROWS ? ld(a.XT, p, k * a.N8 + i) : ld(a.W1, p, a.w1off + k);
        }
        const Dealer D = dealer_of(K, p, a.c.op, e);
        u64 A;
        const Sh E = b2a(W, p, eq_bit(W, K, p, a.c.op, e, v, D, A, act), D, act, 64);
        const Sh z = mult_sh(W, E, wv, zero_a(K, a.c.op, 2, e), act);
        if (act) {
            atomicAdd((unsigned long long *)&a.acc[(u64)(2 * p) * a.N8 + i], (unsigned long long)z.o);
            atomicAdd((unsigned long long *)&a.acc[(u64)(2 * p + 1) * a.N8 + i], (unsigned long long)z.n);
        }
    }
    W.flush(a.c.wire);
}

// out[i] = the sums (own, next) [epi 1: 2*prev[i] + sum + 1]; the sums are left at zero
__global__ __launch_bounds__(256) void k_lit_fin(u64 *acc, u64 N, u64 N8, P6 out, P6 prev, int epi)
{
    for (u64 i = (u64)blockIdx.x * blockDim.x + threadIdx.x; i < N; i += (u64)gridDim.x * blockDim.x)
        for (int p = 0; p < 3; p++) {
            u64 *ao = &acc[(u64)(2 * p) * N8 + i], *an = &acc[(u64)(2 * p + 1) * N8 + i];
            Sh z = { *ao, *an };
            *ao = 0; *an = 0;
            if (epi == 1) z = scale(ld(prev, p, i), 2) + z + pub(p, 1);
            st(out, p, i, z);
        }
}

// per-sample leaf flags as Boolean bits: LB[r*N8 + i] = [M[i] - base == r] and isLeaf[r]
struct LcfArgs { KCommon c; P6 M, isLeaf, LB; u64 base; u32 nh; u64 N, N8; };
__global__ __launch_bounds__(192) void k_lcf_bits(LcfArgs a)
{
    const int p = party_of_wave();
    __shared__ u64 s_wire[GT_LWIRE_WORDS];
    __shared__ u64 s_cnt[6];
    Wire W; W.init(s_wire, s_cnt);
    __shared__ u64 s_prf[3][GT_PRF_SCRATCH_WORDS];
    const PartyKeys K = load_party_keys(a.c.keys, p, s_prf[p]);
    GT_FOR_TILES((u64)a.nh * a.N8) {
        const u64 e = GT_ELEM(), r = e / a.N8, i = e % a.N8;
        const bool act = r < a.nh && i < a.N;
        Sh v = { 0, 0 }, g = { 0, 0 };
        if (act) { v = ld(a.M, p, i) - pub(p, a.base + r); g = ld(a.isLeaf, p, r); }
        const Dealer D = dealer_of(K, p, a.c.op, e);
        u64 A;
        Sh b = eq_bit(W, K, p, a.c.op, e, v, D, A, act);
        b = and_bit(W, b, g, A >> 63, act);
        if (act) st(a.LB, p, e, b);
    }
    W.flush(a.c.wire);
}

// Statistics counting element by element: e = (r*PW + q)*N8 + i, q = row*2dd + 2k + v the
// position in the (1+K) x 2dd counter array (dd = d, or 1 at the label level).
struct LitCountArgs { KCommon c; P6 LB, XT, YT; LimbSet B; u64 N, N8; u32 nh, d, dd, K; u64 *acc; };
__global__ __launch_bounds__(192) void k_count_literal(LitCountArgs a)
{
    const int p = party_of_wave();
    __shared__ u64 s_wire[GT_LWIRE_WORDS];
    __shared__ u64 s_cnt[6];
    Wire W; W.init(s_wire, s_cnt);
    __shared__ u64 s_prf[3][GT_PRF_SCRATCH_WORDS];
    const PartyKeys K = load_party_keys(a.c.keys, p, s_prf[p]);
    const u64 PW = (u64)(1 + a.K) * 2 * a.dd, total = (u64)a.nh * PW * a.N8;
    GT_FOR_TILES(total) {
        const u64 e = GT_ELEM(), i = e % a.N8, rq = e / a.N8, r = rq / PW, q = rq % PW;
        const bool act = e < total && i < a.N;
        Sh s = { 0, 0 }, cv = { 0, 0 };
        if (act) {
            const u64 row = q / (2 * a.dd), k = (q % (2 * a.dd)) / 2, v = q & 1;
            const Sh x = ld(a.XT, p, k * a.N8 + i);
            if (row == 0) cv = v ? x : pub(p, 1) - x;
            else {
                const u64 col = k * a.K + (row - 1);
                const u64 xyo = load_limbs1(a.B.m[p][1], col, i);
                const Sh xy = { xyo, load_limbs1(a.B.m[p][0], col, i) - xyo };
                cv = v ? xy : ld(a.YT, p, (row - 1) * a.N8 + i) - xy;
            }
            s = ld(a.LB, p, r * a.N8 + i);
        }
        const Dealer D = dealer_of(K, p, a.c.op, e);
        const Sh E = b2a(W, p, s, D, act, 64);
        const Sh z = mult_sh(W, E, cv, zero_a(K, a.c.op, 2, e), act);
        if (act) {
            atomicAdd((unsigned long long *)&a.acc[(u64)(2 * p) * a.nh * PW + rq], (unsigned long long)z.o);
            atomicAdd((unsigned long long *)&a.acc[(u64)(2 * p + 1) * a.nh * PW + rq], (unsigned long long)z.n);
        }
    }
    W.flush(a.c.wire);
}

// compact statistics from the accumulated counter arrays (local linear operations), added
// to the inherited ones
__global__ __launch_bounds__(256) void k_from_paper(u64 *acc, P6 C, u32 nh, u32 d, u32 dd, u32 K, u32 CW)
{
    const u64 PW = (u64)(1 + K) * 2 * dd, n = (u64)nh * K;
    for (u64 t = (u64)blockIdx.x * blockDim.x + threadIdx.x; t < n; t += (u64)gridDim.x * blockDim.x) {
        const u64 r = t / K, cl = t % K;
        for (int p = 0; p < 3; p++)
            for (int pl = 0; pl < 2; pl++) {
                u64 *o = acc + (u64)(2 * p + pl) * nh * PW + r * PW + (cl + 1) * 2 * dd;
                u64 *dst = pl ? C.n[p] : C.o[p];
                dst[r * CW + (u64)d * K + cl] += o[0] + o[1];
                if (dd == d) for (u32 k = 0; k < d; k++) dst[r * CW + (u64)k * K + cl] += o[2 * k + 1];
            }
    }
}

// ---------------------------------------------------------------------------------
// Heuristic computation by reconstruction, the host analogue of the TEE-based protocol of
// Sec. V-B: the scorer (a fourth role, not one of the parties) reconstructs the level's C,
// gamma and F from the three components and computes in the clear what the MPC protocol
// computes: fixed-point scores sum_j floor(S_j 2^tau / Q_j) (empty branch: 0) masked by
// gamma, the first maximum, the updated gamma, purity n^2 = sum_c tot_c^2, node types.
// One workgroup per node; plain results for the sharing kernel.
struct HcOpenArgs { P6 C, gamma, F; u64 base; u32 nh, d, K, CW, tau; u64 *SD, *G, *Fn, *Fc, *Sp, *SC; };
__device__ __forceinline__ u64 rec3(const P6 &a, u64 e) { return a.o[0][e] + a.n[0][e] + a.o[2][e]; }

__global__ __launch_bounds__(256) void k_hc_open(HcOpenArgs a)
{
    __shared__ u64 s_tot[16], s_best[256];
    __shared__ u32 s_idx[256];
    const u32 tid = threadIdx.x;
    const u64 dK = (u64)a.d * a.K;
    for (u32 r = blockIdx.x; r < a.nh; r += gridDim.x) {
        if (tid < a.K) s_tot[tid] = rec3(a.C, (u64)r * a.CW + dK + tid);
        __syncthreads();
        u64 n = 0;
        for (u32 cl = 0; cl < a.K; cl++) n += s_tot[cl];
        u64 best = 0; u32 bi = 0xffffffffu;
        for (u32 k = tid; k < a.d; k += blockDim.x) {
            u64 score = 0;
            for (int br = 0; br < 2; br++) {
                u64 nj = 0, S = 0;
                for (u32 cl = 0; cl < a.K; cl++) {
                    const u64 n1 = rec3(a.C, (u64)r * a.CW + (u64)k * a.K + cl);
                    const u64 njc = br ? n1 : s_tot[cl] - n1;
                    nj += njc; S += njc * njc;
                }
                u64 Q = nj * n;
                if (Q == 0) Q = 1;
                score += (S << a.tau) / Q;
            }
            const u64 g = rec3(a.gamma, (u64)r * a.d + k);
            score *= g;
            a.SC[(u64)r * a.d + k] = score; a.G[(u64)r * a.d + k] = g;
            if (bi == 0xffffffffu || score > best) { best = score; bi = k; }   // ascending k: the first maximum of this thread
        }
        s_best[tid] = best; s_idx[tid] = bi;
        __syncthreads();
        for (u32 st = 128; st > 0; st >>= 1) {         // larger score wins, then the lower index
            if (tid < st) {
                const u64 ob = s_best[tid + st]; const u32 oi = s_idx[tid + st];
                if (oi != 0xffffffffu && (s_idx[tid] == 0xffffffffu || ob > s_best[tid] || (ob == s_best[tid] && oi < s_idx[tid]))) {
                    s_best[tid] = ob; s_idx[tid] = oi;
                }
            }
            __syncthreads();
        }
        if (tid == 0) {
            const u32 sd = s_idx[0];
            u64 sq = 0;
            for (u32 cl = 0; cl < a.K; cl++) sq += s_tot[cl] * s_tot[cl];
            const u64 F = rec3(a.F, a.base + r);
            const u64 split = (F == 1 && n * n - sq != 0) ? 1 : 0;
            a.SD[r] = sd; a.G[(u64)r * a.d + sd] = 0;
            a.Sp[r] = split; a.Fn[r] = F * (1 - split); a.Fc[r] = 2 - split;
        }
        __syncthreads();
    }
}

// F of both children of node r := the sharing of node r in src
__global__ __launch_bounds__(256) void k_children(P6 F, P6 src, u64 base, u64 nh)
{
    for (u64 r = (u64)blockIdx.x * blockDim.x + threadIdx.x; r < nh; r += (u64)gridDim.x * blockDim.x)
        for (int j = 0; j < 3; j++) {
            F.o[j][2 * (base + r) + 1] = F.o[j][2 * (base + r) + 2] = src.o[j][r];
            F.n[j][2 * (base + r) + 1] = F.n[j][2 * (base + r) + 2] = src.n[j][r];
        }
}

// ---------------------------------------------------------------------------------
// Statistics counting as a contraction in Z_2^64 (Sec. V-B):
//   Z_p[r][col] = sum_i L_p[r][i] * (B_p + B_{p+1})[col][i] + L_{p+1}[r][i] * B_p[col][i]
// with L the per-sample leaf one-hot and B the sample-contiguous columns (XY products,
// then the K class indicators).  Both operands are uniformly random 64-bit shares, so
// this is a dense integer GEMM; it runs on the matrix cores in signed 8-bit limbs:
//   x*y mod 2^64 = sum_{s+t<=7} d_s(x) d_t(y) 256^(s+t),
// 36 limb pairs, one v_mfma_i32_32x32x32_i8 each, accumulated per u = s+t in int32.
// |d_s d_t| <= 2^14 and at most 8 pairs x 2 products x 4096 samples meet in one
// accumulator, which stays below 2^31.  A wavefront owns a 32 x 64 output tile
// (8 x 2 accumulators of 16 registers); the sample range is split over workgroups
// and the recombined 64-bit partial sums meet by atomic adds (exact, order-free).
typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
// sample blocks of 32 per workgroup: the int32 accumulators would allow 128; with 64 the launch
// has twice the workgroups to balance over the compute units and takes 3 % less time
#define CT_CHUNK_BLOCKS 64
// bcol0: first column (row of B) of this launch, zcol0: its column in the output
// rt: row tiles of 32 per workgroup (4, 2 or 1); the other 4/rt wavefronts take further column tiles
// chunkblk: sample blocks of 32 per workgroup (at most CT_CHUNK_BLOCKS; the int32 accumulators bound it by 128)
// nns: slots per chunk (0 = none) for one more column group of at most 16 columns (first column
// nbcol0 of B, column nzcol0 of the output), handled by the same launch with 16-wide tiles
struct CountArgs { LimbTri L; LimbSet B; u64 nblk; u32 nh, ncol; u64 bcol0; u32 zcol0; u64 *Zacc; u32 nchunk, nrowgrp, ncg, rt, chunkblk, ncoltiles;   // ncoltiles: column tiles of 32*NB in this launch
                   u32 nns; u64 nbcol0; u32 nzcol0; };

// A remainder of at most 16 columns (the class totals): 16 rows per wavefront with
// v_mfma_i32_16x16x64_i8 (lane l holds row or column l%16 and the 16 samples
// 16*(l/16).. of a pair of sample blocks; result C[4*(l/16)+v][l%16]), for ALL THREE
// parties at once.  With so few columns the products are limited by the rate at which L
// arrives, so every component L_j of L is fetched once and multiplied by one tile that
// holds both operands it meets in the three-term products,
//   columns 0-7:  up to 8 columns of (B_j + B_{j+1})   ->  Z_j     (L_j is party j's own part)
//   columns 8-15: the same columns of B_{j-1}          ->  Z_{j-1} (and party j-1's next part)
// (each party's sums still come from the two components that party holds); more than 8
// columns take a second pass.  It runs inside the launch of the wide groups, as one more
// column group of each sample chunk.
__device__ __forceinline__ void count_narrow(const CountArgs &a, u64 r0, u64 ib0, u64 ib1, int lane)
{
    const u32 lr = lane & 15, kq = lane >> 4, half = (kq & 1) * 16, nreal = a.ncol - a.nzcol0;
    for (u32 c0 = 0; c0 < nreal; c0 += 8) {
        const u32 nc = nreal - c0 < 8 ? nreal - c0 : 8;
        const bool bcol = (lr & 7) < nc;                 // this lane's column of the tile exists
        const u64 brow = a.nbcol0 + c0 + (lr & 7);
        v4i acc[3][8];
#pragma unroll
        for (int j = 0; j < 3; j++)
#pragma unroll
            for (int u = 0; u < 8; u++) acc[j][u] = v4i{ 0, 0, 0, 0 };
        v4i A[3][8], B[3][8];
        // the lane's sample block of a pair; the second block of an odd tail does not belong
        // to this chunk: its lanes load the first block again and multiply zeros
#define CN_LOAD_A(J, IB)                                                                      \
        {                                                                                     \
            const u64 ibl = (IB) + (kq >> 1) >= ib1 ? (IB) : (IB) + (kq >> 1);                \
            _Pragma("unroll") for (int sl = 0; sl < 8; sl++)                                  \
                A[J][sl] = *(const v4i *)(a.L.m[J].base + limb_addr(a.L.m[J], ibl, sl, r0 + lr) + half); \
        }
#define CN_LOAD_B(J, IB)                                                                      \
        {                                                                                     \
            const bool tail = (IB) + (kq >> 1) >= ib1;                                        \
            const u64 ibl = tail ? (IB) : (IB) + (kq >> 1);                                   \
            const LimbMat &Bs_ = a.B.m[J][0], &Bo_ = a.B.m[((J) + 2) % 3][1];                 \
            const unsigned char *bb_ = lr < 8 ? Bs_.base : Bo_.base;                          \
            _Pragma("unroll") for (int sl = 0; sl < 8; sl++) {                                \
                B[J][sl] = v4i{ 0, 0, 0, 0 };                                                 \
                if (!tail && bcol) B[J][sl] = *(const v4i *)(bb_ + limb_addr(Bs_, ibl, sl, brow) + half); \
            }                                                                                 \
        }
#define CN_MMA(J)                                                                             \
        _Pragma("unroll") for (int sl = 0; sl < 8; sl++)                                      \
            _Pragma("unroll") for (int t = 0; t < 8 - sl; t++)                                \
                acc[J][sl + t] = __builtin_amdgcn_mfma_i32_16x16x64_i8(A[J][sl], B[J][t], acc[J][sl + t], 0, 0, 0);
        // 16 loads between the first MFMAs of the stage, one by one (see k_count)
#define CN_SPREAD()                                                                           \
        _Pragma("unroll") for (int q_ = 0; q_ < 16; q_++) {                                   \
            __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);                                \
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                                \
        }                                                                                     \
        __builtin_amdgcn_sched_group_barrier(0x008, 20, 0);                                   \
        __builtin_amdgcn_sched_barrier(0);
        // One pair of sample blocks = three stages of 36 MFMAs, one per component.  While a stage
        // multiplies, L for the stage after the next and the columns for the next are fetched.
        CN_LOAD_A(0, ib0)
        CN_LOAD_A(1, ib0)
        CN_LOAD_B(0, ib0)
        for (u64 ib = ib0; ib < ib1; ib += 2) {
            // the loads for the pair after the last are issued all the same (they read the chunk's
            // last pair again and are not used): the number of loads in flight stays fixed
            const u64 ibn = ib + 2 < ib1 ? ib + 2 : ib;
            __builtin_amdgcn_sched_barrier(0);
            CN_LOAD_A(2, ib)  CN_LOAD_B(1, ib)  CN_MMA(0) CN_SPREAD()
            CN_LOAD_A(0, ibn) CN_LOAD_B(2, ib)  CN_MMA(1) CN_SPREAD()
            CN_LOAD_A(1, ibn) CN_LOAD_B(0, ibn) CN_MMA(2) CN_SPREAD()
        }
#undef CN_LOAD_A
#undef CN_LOAD_B
#undef CN_MMA
#undef CN_SPREAD
#pragma unroll
        for (int j = 0; j < 3; j++) {
            const int pz = lr < 8 ? j : (j + 2) % 3;     // the party whose sum this column of the tile belongs to
            u64 *Z = a.Zacc + (u64)pz * a.nh * a.ncol;
#pragma unroll
            for (int v = 0; v < 4; v++) {
                const u64 r = r0 + 4 * kq + v;
                const u64 c = a.nzcol0 + c0 + (lr & 7);
                u64 z = 0;
#pragma unroll
                for (int u = 0; u < 8; u++) z += (u64)(long long)acc[j][u][v] << (8 * u);
                if (r < a.nh && bcol) atomicAdd((unsigned long long *)&Z[r * a.ncol + c], (unsigned long long)z);
            }
        }
    }
}

// Workgroup = 4 wavefronts = 128 rows x (32*NB) columns; NB = 2 for full groups of 64
// columns, NB = 1 for a remainder of at most 32.  The kernel is limited by the rate at
// which the L1 cache can fetch the two operands (about 24 KB per wavefront and
// product), not by the matrix cores; the operands of the next product are in flight
// while the current one is multiplied.
template <int NB>
__global__ __launch_bounds__(256) void k_count(CountArgs a)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    // Workgroups go round-robin to the 8 XCDs, each with its own L2.  The column groups of
    // one sample chunk, of all three parties, read the same rows of the three components of
    // L, so they are given consecutive slots of the same XCD: id = slot*8 + xcd; per chunk
    // 3*ncg wide slots (party-major) and nns narrow ones.
    const u32 per = 3 * a.ncg + a.nns, id = blockIdx.x, xcd = id & 7, slot = id >> 3;
    const u32 sl = slot % per, chunk = (slot / per) * 8 + xcd;
    if (chunk >= a.nchunk) return;                            // whole workgroup, no barrier in this kernel
    const u64 ib0 = (u64)chunk * a.chunkblk;
    const u64 ib1 = ib0 + a.chunkblk < a.nblk ? ib0 + a.chunkblk : a.nblk;
    const u32 rg = blockIdx.z;
    if (sl >= 3 * a.ncg) {
        // a narrow slot of this chunk: its workgroups of 4 wavefronts share out the row tiles
        // of 16 (each tile for all three parties)
        const u64 rn = ((u64)((sl - 3 * a.ncg) * a.nrowgrp + rg) * 4 + wave) * 16;
        if (rn < a.nh) count_narrow(a, rn, ib0, ib1, lane);
        return;
    }
    const int p = sl / a.ncg;
    const u32 cg = sl % a.ncg;
    const u32 wr = wave % a.rt, wc = wave / a.rt, cper = 4 / a.rt;   // this wavefront's row / column tile
    const u64 r0 = ((u64)rg * a.rt + wr) * 32;
    if (r0 >= a.nh) return;                                   // whole wavefront
    // product 0: L_p x (B_p + B_{p+1}), product 1: L_{p+1} x B_p
    const LimbMat LA0 = p == 0 ? a.L.m[0] : (p == 1 ? a.L.m[1] : a.L.m[2]);
    const LimbMat LA1 = p == 0 ? a.L.m[1] : (p == 1 ? a.L.m[2] : a.L.m[0]);
    const LimbMat LB0 = p == 0 ? a.B.m[0][0] : (p == 1 ? a.B.m[1][0] : a.B.m[2][0]);
    const LimbMat LB1 = p == 0 ? a.B.m[0][1] : (p == 1 ? a.B.m[1][1] : a.B.m[2][1]);
    const u64 ctile = (u64)cg * cper + wc;                   // column tile of 32*NB
    if (ctile >= a.ncoltiles) return;                         // whole wavefront
    const u64 c0 = a.bcol0 + ctile * (32 * NB);
    const u32 lr = lane & 31;
    v16i acc[8][NB];
#pragma unroll
    for (int u = 0; u < 8; u++)
#pragma unroll
        for (int nb = 0; nb < NB; nb++)
#pragma unroll
            for (int v = 0; v < 16; v++) acc[u][nb][v] = 0;
    // addresses = wave-uniform base (scalar registers) + a 32-bit lane offset
    const u32 offA = (u32)((r0 + lr) * 32 + (lane >> 5) * 16), offB = (u32)(lr * 32 + (lane >> 5) * 16);
    v4i av0[8], bv0[NB][8], av1[8], bv1[NB][8];
#define CT_LOAD(AV, BV, LA, LB, IB)                                                           \
    _Pragma("unroll") for (int s = 0; s < 8; s++) {                                           \
        AV[s] = *(const v4i *)(LA.base + limb_addr(LA, IB, s, 0) + offA);                     \
        _Pragma("unroll") for (int nb = 0; nb < NB; nb++)                                     \
            BV[nb][s] = *(const v4i *)(LB.base + limb_addr(LB, IB, s, c0 + nb * 32) + offB);  \
    }
    // limb s of the left operand against limbs 0..7-s of the right one: successive MFMAs
    // go to different accumulators (level s+t), none waits for the one before it
#define CT_MMA(AV, BV)                                                                        \
    _Pragma("unroll") for (int s = 0; s < 8; s++)                                             \
        _Pragma("unroll") for (int t = 0; t < 8 - s; t++)                                     \
            _Pragma("unroll") for (int nb = 0; nb < NB; nb++)                                 \
                acc[s + t][nb] = __builtin_amdgcn_mfma_i32_32x32x32_i8(AV[s], BV[nb][t], acc[s + t][nb], 0, 0, 0);
    // The loads of the next product are issued one by one between the first MFMAs of this
    // product (a burst of 8*(1+NB) loads at once fills the L1 cache's queue of outstanding
    // misses and the matrix cores wait for it to drain); without the scheduling groups
    // the compiler would sink the loads to their uses to save registers.
#define CT_SPREAD()                                                                           \
    _Pragma("unroll") for (int q = 0; q < 8 * (1 + NB); q++) {                                \
        __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);                                    \
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                                    \
    }                                                                                         \
    __builtin_amdgcn_sched_group_barrier(0x008, 36 * NB - 8 * (1 + NB), 0);
    CT_LOAD(av0, bv0, LA0, LB0, ib0)
    for (u64 ib = ib0; ib < ib1; ib++) {
        __builtin_amdgcn_sched_barrier(0);
        CT_LOAD(av1, bv1, LA1, LB1, ib)
        CT_MMA(av0, bv0)
        CT_SPREAD()
        __builtin_amdgcn_sched_barrier(0);
        // always issued (the last one re-reads the chunk's last block and is not used): with a
        // fixed number of loads in flight the wait before the next product leaves them pending
        CT_LOAD(av0, bv0, LA0, LB0, (ib + 1 < ib1 ? ib + 1 : ib))
        CT_MMA(av1, bv1)
        CT_SPREAD()
        __builtin_amdgcn_sched_barrier(0);
    }
#undef CT_SPREAD
#undef CT_LOAD
#undef CT_MMA
    u64 *Z = a.Zacc + (u64)p * a.nh * a.ncol;
#pragma unroll
    for (int nb = 0; nb < NB; nb++)
#pragma unroll
        for (int v = 0; v < 16; v++) {
            const u64 r = r0 + 8 * (v / 4) + 4 * (lane >> 5) + (v & 3);
            const u64 c = a.zcol0 + ctile * (32 * NB) + nb * 32 + lr;
            u64 z = 0;
#pragma unroll
            for (int u = 0; u < 8; u++) z += (u64)(long long)acc[u][nb][v] << (8 * u);
            if (r < a.nh && c < a.ncol) atomicAdd((unsigned long long *)&Z[r * a.ncol + c], (unsigned long long)z);
        }
}

// add the zero sharing, reshare, accumulate into the node statistics
struct CountFinArgs { KCommon c; u64 *Zacc; P6 C; u64 n; u32 ncol, CW; u64 colbase; };
__global__ __launch_bounds__(192) void k_count_fin(CountFinArgs a)
{
    const int p = party_of_wave();
    __shared__ u64 s_wire[GT_LWIRE_WORDS];
    __shared__ u64 s_cnt[6];
    Wire W; W.init(s_wire, s_cnt);
    __shared__ u64 s_prf[3][GT_PRF_SCRATCH_WORDS];
    const PartyKeys K = load_party_keys(a.c.keys, p, s_prf[p]);
    GT_FOR_TILES(a.n) {
        const u64 o = GT_ELEM();
        const bool act = o < a.n;
        Sh z;
        u64 part = 0;
        if (act) { part = a.Zacc[(u64)p * a.n + o]; a.Zacc[(u64)p * a.n + o] = 0; }   // zero again for the next contraction
        z.o = part + zero_a(K, a.c.op, 0, o);
        z.n = W.reshare1(z.o, act ? 64u : 0u);
        if (act) {
            const u64 idx = (o / a.ncol) * a.CW + a.colbase + o % a.ncol;
            st(a.C, p, idx, ld(a.C, p, idx) + z);
        }
    }
    W.flush(a.c.wire);
}

// counter-array layout of Sec. V-B for export: per node (1+K) x 2d, local linear ops
__global__ __launch_bounds__(256) void k_c_paper(P6 C, P6 out, u32 nh, u32 d, u32 K, u32 CW)
{
    const u64 per = (u64)(1 + K) * 2 * d, n = (u64)nh * per;
    for (u64 t = (u64)blockIdx.x * blockDim.x + threadIdx.x; t < n; t += (u64)gridDim.x * blockDim.x) {
        const u64 r = t / per, q = t % per, row = q / (2 * d), col = q % (2 * d), k = col / 2, v = col & 1;
        for (int j = 0; j < 3; j++)
            for (int pl = 0; pl < 2; pl++) {
                const u64 *src = pl ? C.n[j] : C.o[j];
                u64 val = 0;
                for (u32 cl = (row ? row - 1 : 0); cl < (row ? row : K); cl++) {
                    const u64 n1 = src[r * CW + k * K + cl], tot = src[r * CW + (u64)d * K + cl];
                    val += v ? n1 : tot - n1;
                }
                (pl ? out.n[j] : out.o[j])[t] = val;
            }
    }
}
