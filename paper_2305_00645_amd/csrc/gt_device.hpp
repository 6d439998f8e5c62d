// Device-side toolkit: PRF, per-party share arithmetic, message exchange and the
// per-element protocol steps (Sec. II-B and Sec. V-A of the GTree paper), for gfx950.
//
// Execution model.  A workgroup is 3 wavefronts of 64 lanes: wavefront p IS party p
// (threadIdx.y = p).  Lane l of each of the three wavefronts works on the same
// element(s), each on its own party's two components.  A protocol message is a
// store into the workgroup's message region in LDS; the receiving wavefront loads it
// after a workgroup barrier.  A party's lanes never
// read another party's shares or keys, only the words sent to it.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef uint64_t u64;
typedef uint32_t u32;

#define GT_LANES 64
#define GT_KEY_DEALER 3
#define GT_KEY_OWNER 4

// ---------------------------------------------------------------------------------
// ChaCha block function, 8 rounds, as a counter-based PRF.  State words 12..15 are
// (block lo, block hi, op, stream); output word w (64 bit) is the little-endian pair
// (2w, 2w+1).  The key is wave-uniform and lives in scalar registers.
struct Key { u32 k[8]; };

__device__ __forceinline__ u32 rotl32(u32 x, int r) { return __builtin_rotateleft32(x, r); }

#define GT_QR(a, b, c, d)                                                                     \
    a += b; d ^= a; d = rotl32(d, 16); c += d; b ^= c; b = rotl32(b, 12);                     \
    a += b; d ^= a; d = rotl32(d, 8);  c += d; b ^= c; b = rotl32(b, 7);

#ifndef GT_PRF_ROUNDS
#define GT_PRF_ROUNDS 8          // ChaCha rounds of the PRF (the CPU check uses the same number)
#endif
__device__ __forceinline__ void chacha8(const Key &key, u64 blk, u32 op, u32 stream, u64 (&out)[8])
{
    const u32 i0 = 0x61707865u, i1 = 0x3320646eu, i2 = 0x79622d32u, i3 = 0x6b206574u;
    const u32 c12 = (u32)blk, c13 = (u32)(blk >> 32);
    u32 x0 = i0, x1 = i1, x2 = i2, x3 = i3;
    u32 x4 = key.k[0], x5 = key.k[1], x6 = key.k[2], x7 = key.k[3];
    u32 x8 = key.k[4], x9 = key.k[5], x10 = key.k[6], x11 = key.k[7];
    u32 x12 = c12, x13 = c13, x14 = op, x15 = stream;
#pragma unroll
    for (int r = 0; r < GT_PRF_ROUNDS / 2; r++) {
        GT_QR(x0, x4, x8, x12) GT_QR(x1, x5, x9, x13) GT_QR(x2, x6, x10, x14) GT_QR(x3, x7, x11, x15)
        GT_QR(x0, x5, x10, x15) GT_QR(x1, x6, x11, x12) GT_QR(x2, x7, x8, x13) GT_QR(x3, x4, x9, x14)
    }
    x0 += i0; x1 += i1; x2 += i2; x3 += i3;
    x4 += key.k[0]; x5 += key.k[1]; x6 += key.k[2]; x7 += key.k[3];
    x8 += key.k[4]; x9 += key.k[5]; x10 += key.k[6]; x11 += key.k[7];
    x12 += c12; x13 += c13; x14 += op; x15 += stream;
    out[0] = (u64)x0 | ((u64)x1 << 32);   out[1] = (u64)x2 | ((u64)x3 << 32);
    out[2] = (u64)x4 | ((u64)x5 << 32);   out[3] = (u64)x6 | ((u64)x7 << 32);
    out[4] = (u64)x8 | ((u64)x9 << 32);   out[5] = (u64)x10 | ((u64)x11 << 32);
    out[6] = (u64)x12 | ((u64)x13 << 32); out[7] = (u64)x14 | ((u64)x15 << 32);
}

__device__ __forceinline__ u64 sel8(const u64 (&w)[8], u32 i)
{
    u64 a = (i & 1) ? w[1] : w[0], b = (i & 1) ? w[3] : w[2];
    u64 c = (i & 1) ? w[5] : w[4], d = (i & 1) ? w[7] : w[6];
    u64 ab = (i & 2) ? b : a, cd = (i & 2) ? d : c;
    return (i & 4) ? cd : ab;
}

__device__ __forceinline__ Key load_key(const u32 *keys, int idx)
{
    Key k;
#pragma unroll
    for (int i = 0; i < 8; i++) k.k[i] = __builtin_amdgcn_readfirstlane(keys[idx * 8 + i]);
    return k;
}

// The keys one party may use: its two pairwise keys (Sec. III) and, in this
// simulation, the dealer key from which the offline material is derived.
// scr: this wavefront's 8 x 64 words of LDS for handing PRF words round its lanes
// (kernels with one element per lane, see prf_tile), else null.
struct PartyKeys { Key own, nxt, dlr; u64 *scr; };
#define GT_PRF_SCRATCH_WORDS (8 * GT_LANES)

__device__ __forceinline__ PartyKeys load_party_keys(const u32 *keys, int p, u64 *scr = nullptr)
{
    PartyKeys K;
    K.own = load_key(keys, p);
    K.nxt = load_key(keys, p == 2 ? 0 : p + 1);
    K.dlr = load_key(keys, GT_KEY_DEALER);
    K.scr = scr;
    return K;
}

// word j of stream (op, stream) under one key
__device__ __forceinline__ u64 prf_word(const Key &k, u32 op, u32 stream, u64 j)
{
    u64 w[8];
    chacha8(k, j >> 3, op, stream, w);
    return sel8(w, (u32)j & 7);
}

// Words of NS streams under the own and the next key for a tile of 64 consecutive
// elements, element 64*tile + lane in lane `lane` (every kernel with one element per
// lane indexes that way, and all 64 lanes call together).  A block of the PRF holds
// the words of 8 consecutive elements, so the tile needs 8 blocks per key and stream:
// lane l < 16*NS evaluates block l%8 of stream (l/16), own key if (l/8) is even, next key
// otherwise, and leaves its 8 words in the wavefront's scratch; then every lane picks
// its own.  One pass of the block function instead of 2*NS.  LDS operations of one
// wavefront complete in order, so no hardware barrier is needed; the wavefront-scope
// fences keep the compiler from moving the loads of other lanes' words across the stores.
template <int NS>
__device__ __forceinline__ void prf_tile(const PartyKeys &K, u32 op, const u32 (&st)[NS], u64 e, u64 (&wo)[NS], u64 (&wn)[NS])
{
    static_assert(NS >= 1 && NS <= 4, "at most 8 key/stream pairs per pass");
    const u32 lane = threadIdx.x, c = lane >> 3;
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");      // the previous call's loads come first
    __builtin_amdgcn_wave_barrier();
    if (c < 2 * NS) {
        // selections by masks: plain ALU work on the scalar key words
        const u32 mk = 0u - (c & 1);
        Key kv;
#pragma unroll
        for (int i = 0; i < 8; i++) kv.k[i] = K.own.k[i] ^ ((K.own.k[i] ^ K.nxt.k[i]) & mk);
        u32 stream = 0;
#pragma unroll
        for (int q = 0; q < NS; q++) stream |= st[q] & (0u - (u32)((c >> 1) == (u32)q));
        u64 blk[8];
        chacha8(kv, (e >> 6) * 8 + (lane & 7), op, stream, blk);
#pragma unroll
        for (int i = 0; i < 8; i++) K.scr[c * GT_LANES + (lane & 7) * 8 + i] = blk[i];
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int q = 0; q < NS; q++) { wo[q] = K.scr[(2 * q) * GT_LANES + lane]; wn[q] = K.scr[(2 * q + 1) * GT_LANES + lane]; }
}

// party p's component of the zero sharing of element e: arithmetic / Boolean
__device__ __forceinline__ u64 zero_a(const PartyKeys &K, u32 op, u32 stream, u64 e)
{
    const u32 st[1] = { stream }; u64 wo[1], wn[1];
    prf_tile<1>(K, op, st, e, wo, wn);
    return wo[0] - wn[0];
}
__device__ __forceinline__ u64 zero_b(const PartyKeys &K, u32 op, u32 stream, u64 e)
{
    const u32 st[1] = { stream }; u64 wo[1], wn[1];
    prf_tile<1>(K, op, st, e, wo, wn);
    return wo[0] ^ wn[0];
}
// two streams in one pass
__device__ __forceinline__ void zero_a2(const PartyKeys &K, u32 op, u32 s0, u32 s1, u64 e, u64 &z0, u64 &z1)
{
    const u32 st[2] = { s0, s1 }; u64 wo[2], wn[2];
    prf_tile<2>(K, op, st, e, wo, wn);
    z0 = wo[0] - wn[0]; z1 = wo[1] - wn[1];
}
__device__ __forceinline__ void zero_b2(const PartyKeys &K, u32 op, u32 s0, u32 s1, u64 e, u64 &z0, u64 &z1)
{
    const u32 st[2] = { s0, s1 }; u64 wo[2], wn[2];
    prf_tile<2>(K, op, st, e, wo, wn);
    z0 = wo[0] ^ wn[0]; z1 = wo[1] ^ wn[1];
}

// ---------------------------------------------------------------------------------
// A party's view of one shared element: components p (own) and p+1 (next).
struct Sh { u64 o, n; };

// kernel-argument view of a shared vector: six planes
struct P6 { u64 *o[3]; u64 *n[3]; };

__device__ __forceinline__ u64 *own_of(const P6 &a, int p) { return p == 0 ? a.o[0] : (p == 1 ? a.o[1] : a.o[2]); }
__device__ __forceinline__ u64 *nxt_of(const P6 &a, int p) { return p == 0 ? a.n[0] : (p == 1 ? a.n[1] : a.n[2]); }
__device__ __forceinline__ Sh ld(const P6 &a, int p, size_t e) { Sh v; v.o = own_of(a, p)[e]; v.n = nxt_of(a, p)[e]; return v; }
__device__ __forceinline__ void st(const P6 &a, int p, size_t e, Sh v) { own_of(a, p)[e] = v.o; nxt_of(a, p)[e] = v.n; }

// public constant c as the sharing (c, 0, 0): component 1 is party 0's own and party 2's next
__device__ __forceinline__ Sh pub(int p, u64 c) { Sh v; v.o = p == 0 ? c : 0; v.n = p == 2 ? c : 0; return v; }
__device__ __forceinline__ Sh operator+(Sh a, Sh b) { Sh v; v.o = a.o + b.o; v.n = a.n + b.n; return v; }
__device__ __forceinline__ Sh operator-(Sh a, Sh b) { Sh v; v.o = a.o - b.o; v.n = a.n - b.n; return v; }
__device__ __forceinline__ Sh operator^(Sh a, Sh b) { Sh v; v.o = a.o ^ b.o; v.n = a.n ^ b.n; return v; }
__device__ __forceinline__ Sh scale(Sh a, u64 c) { Sh v; v.o = a.o * c; v.n = a.n * c; return v; }

// party-local part of a product: z_p = x_p y_p + x_{p+1} y_p + x_p y_{p+1}
__device__ __forceinline__ u64 prod3(Sh x, Sh y) { return x.o * (y.o + y.n) + x.n * y.o; }
__device__ __forceinline__ u64 and3(Sh x, Sh y) { return (x.o & (y.o ^ y.n)) ^ (x.n & y.o); }

// The party of this wavefront.  All 64 lanes of a wavefront share threadIdx.y (the
// workgroup is 64 x 3), so the value is read into a scalar register: selections and
// branches on the party then cost no vector instructions.
__device__ __forceinline__ int party_of_wave() { return __builtin_amdgcn_readfirstlane((int)threadIdx.y); }

// ---------------------------------------------------------------------------------
// Message exchange inside the workgroup.  `reshare`: every party sends to its
// predecessor (after a product, so that the receiver then holds (z_p, z_{p+1}));
// `open`: every party sends to its successor (it hands over its first component).
// The message region is GT_LWIRE_WORDS words of LDS that the workgroup owns: two
// alternating slots for messages of up to four words per lane, so that one barrier per
// message suffices (a slot is rewritten only after the barrier of the message that
// followed it); a message of more than four words takes the whole region and is
// followed by a second barrier, after which the region may be written again.
#define GT_WIRE_SLOTS 64
#define GT_LWIRE_SLOT (3 * 4 * GT_LANES)
#define GT_LWIRE_WORDS (2 * GT_LWIRE_SLOT)
// Every send states how many payload bits the lane's message carries (0 for a lane whose
// element does not exist); the lane adds them up per direction, the sums are collected
// per party in six words of LDS (drain) and handed to the context's counters when the
// kernel ends (flush), so that the bytes reported for a call are counted where the
// messages are stored, not derived from the sizes on the host.  Party p's wavefront is the
// only one that touches words 2p and 2p+1 of the LDS counters, and the LDS operations of
// one wavefront complete in order, so the counting needs no barrier.
struct LWire {
    u64 *base, *cnt;
    int slot, p, lane;
    u32 nopen, nresh;            // payload bits this lane has sent to its successor / predecessor since the last drain
    __device__ __forceinline__ void init(u64 *lds, u64 *s_cnt)
    {
        base = lds; cnt = s_cnt; slot = 0; p = party_of_wave(); lane = threadIdx.x; nopen = 0; nresh = 0;
        if (lane < 2) cnt[2 * p + lane] = 0;
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
    }
    template <int NW>
    __device__ __forceinline__ void exchange(const u64 (&snd)[NW], u64 (&rcv)[NW], int from)
    {
        static_assert(NW <= 8, "message too wide");
        constexpr int XW = NW <= 4 ? 4 : 8;
        u64 *buf = NW <= 4 ? base + slot * GT_LWIRE_SLOT : base;
        if (NW <= 4) slot ^= 1;
        else __syncthreads();    // a wide message overwrites both slots: the last slot message must have been read
#pragma unroll
        for (int j = 0; j < NW; j++) buf[(p * XW + j) * GT_LANES + lane] = snd[j];
        __syncthreads();
#pragma unroll
        for (int j = 0; j < NW; j++) rcv[j] = buf[(from * XW + j) * GT_LANES + lane];
        if (NW > 4) __syncthreads();
    }
    template <int NW>
    __device__ __forceinline__ void reshare(const u64 (&snd)[NW], u64 (&rcv)[NW], u32 bits) { nresh += bits; exchange<NW>(snd, rcv, p == 2 ? 0 : p + 1); }
    template <int NW>
    __device__ __forceinline__ void open(const u64 (&snd)[NW], u64 (&rcv)[NW], u32 bits) { nopen += bits; exchange<NW>(snd, rcv, p == 0 ? 2 : p - 1); }
    __device__ __forceinline__ u64 reshare1(u64 v, u32 bits) { u64 s[1] = { v }, r[1]; reshare<1>(s, r, bits); return r[0]; }
    __device__ __forceinline__ u64 open1(u64 v, u32 bits) { u64 s[1] = { v }, r[1]; open<1>(s, r, bits); return r[0]; }
    // move the lane's sums into the party's LDS counters (long loops call it once per work
    // item, before the 32-bit sums could overflow)
    __device__ __forceinline__ void drain()
    {
        if (nopen) atomicAdd((unsigned long long *)&cnt[2 * p], (unsigned long long)nopen);
        if (nresh) atomicAdd((unsigned long long *)&cnt[2 * p + 1], (unsigned long long)nresh);
        nopen = 0; nresh = 0;
    }
    // end of the kernel: add the party's sums to the context's counters, g[6*slot + 2p] (bits
    // sent to the successor) and g[6*slot + 2p+1] (to the predecessor); the workgroups of a
    // launch spread over GT_WIRE_SLOTS slots so that their atomic adds do not queue up on one
    // address (the host adds the slots up).  Every lane calls it once.
    __device__ __forceinline__ void flush(u64 *g)
    {
        drain();
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
        if (lane < 2) {
            const u64 v = cnt[2 * p + lane];
            const u32 slot = (blockIdx.x + blockIdx.y) & (GT_WIRE_SLOTS - 1);
            if (v) atomicAdd((unsigned long long *)&g[6 * slot + 2 * p + lane], (unsigned long long)v);
        }
    }
};
typedef LWire Wire;

// ---------------------------------------------------------------------------------
// Offline material of one element, party p's components (dealer stream 0, block e).
struct Dealer { Sh rA, rho, bA; u32 bBo, bBn; };

__device__ __forceinline__ Dealer dealer_from_block(const u64 (&D)[8], int p)
{
    const u64 r = D[0], beta = D[5] & 1;
    const u64 rA2 = r - D[1] - D[2], rho2 = r ^ D[3] ^ D[4], bA2 = beta - D[6] - D[7];
    const u32 b0 = (u32)(D[5] >> 1) & 1, b1 = (u32)(D[5] >> 2) & 1, b2 = ((u32)beta ^ b0 ^ b1) & 1;
    Dealer d;
    d.rA.o = p == 0 ? D[1] : (p == 1 ? D[2] : rA2);   d.rA.n = p == 0 ? D[2] : (p == 1 ? rA2 : D[1]);
    d.rho.o = p == 0 ? D[3] : (p == 1 ? D[4] : rho2); d.rho.n = p == 0 ? D[4] : (p == 1 ? rho2 : D[3]);
    d.bA.o = p == 0 ? D[6] : (p == 1 ? D[7] : bA2);   d.bA.n = p == 0 ? D[7] : (p == 1 ? bA2 : D[6]);
    d.bBo = p == 0 ? b0 : (p == 1 ? b1 : b2);         d.bBn = p == 0 ? b1 : (p == 1 ? b2 : b0);
    return d;
}

__device__ __forceinline__ Dealer dealer_of(const PartyKeys &K, int p, u32 op, u64 e)
{
    u64 D[8];
    chacha8(K.dlr, e, op, 0, D);
    return dealer_from_block(D, p);
}

// ---------------------------------------------------------------------------------
// Per-element protocols, one element per lane.  Every lane of the workgroup must
// call them together (they contain barriers); inactive lanes pass zeros.

// product with reshare: returns (z_p, z_{p+1})
__device__ __forceinline__ Sh mult_sh(Wire &W, Sh x, Sh y, u64 alpha, bool act)
{
    Sh z;
    z.o = prod3(x, y) + alpha;
    z.n = W.reshare1(z.o, act ? 64u : 0u);
    return z;
}

// Equality test [v == 0] -> Boolean bit sharing.  A receives the Boolean
// zero-sharing word of stream 1 (bits 0..62 used here, bit 63 free for a following AND).
__device__ __forceinline__ Sh eq_bit(Wire &W, const PartyKeys &K, int p, u32 op, u64 e, Sh v, const Dealer &D, u64 &A, bool act)
{
    Sh m = v + D.rA;
    const u64 c = m.o + m.n + W.open1(m.o, act ? 64u : 0u);
    Sh t = D.rho;
    if (p == 0) t.o ^= ~c;
    if (p == 2) t.n ^= ~c;
    A = zero_b(K, op, 1, e);
    u32 off = 0;
#pragma unroll
    for (int k = 0; k < 6; k++) {
        const u32 w = 32u >> k;
        const u64 mask = (w == 32) ? 0xffffffffull : ((1ull << w) - 1);
        Sh a, b;
        a.o = t.o & mask; a.n = t.n & mask;
        b.o = (t.o >> w) & mask; b.n = (t.n >> w) & mask;
        t.o = (and3(a, b) ^ (A >> off)) & mask;
        t.n = W.reshare1(t.o, act ? w : 0u);
        off += w;
    }
    return t;
}

// one-bit AND with reshare; alpha is the mask bit
__device__ __forceinline__ Sh and_bit(Wire &W, Sh x, Sh y, u64 alpha, bool act)
{
    Sh z;
    z.o = (and3(x, y) ^ alpha) & 1;
    z.n = W.reshare1(z.o, act ? 1u : 0u);
    return z;
}

// Comparison [v >= 0] (v signed, |v| < 2^63) -> Boolean bit sharing.
// AG, AE: the lane's Boolean zero-sharing words of streams 1 and 2 (own xor next key).
__device__ __forceinline__ Sh ge_bit_masks(Wire &W, int p, Sh v, const Dealer &D, u64 AG, u64 AE, bool act)
{
    const u64 LOW63 = 0x7fffffffffffffffull, TOP = 0x8000000000000000ull;
    Sh m = v + D.rA;
    const u64 c = m.o + m.n + W.open1(m.o, act ? 64u : 0u);
    const u64 nc = ~c;
    Sh G, E;
    G.o = nc & D.rho.o & LOW63; G.n = nc & D.rho.n & LOW63;
    E.o = D.rho.o & LOW63;      E.n = D.rho.n & LOW63;
    if (p == 0) E.o = ((D.rho.o ^ nc) & LOW63) | TOP;
    if (p == 2) E.n = ((D.rho.n ^ nc) & LOW63) | TOP;
#pragma unroll
    for (int k = 0; k < 6; k++) {
        const int s = 1 << k;
        // positions that start a block of 2s bits
        const u64 sm = k == 0 ? 0x5555555555555555ull : k == 1 ? 0x1111111111111111ull
                     : k == 2 ? 0x0101010101010101ull : k == 3 ? 0x0001000100010001ull
                     : k == 4 ? 0x0000000100000001ull : 0x1ull;
        Sh Eh, Gh;
        Eh.o = E.o >> s; Eh.n = E.n >> s; Gh.o = G.o >> s; Gh.n = G.n >> s;
        const u64 zg = (and3(Eh, G) ^ (AG >> (s - 1))) & sm;
        if (k < 5) {
            const u64 ze = (and3(Eh, E) ^ (AE >> (s - 1))) & sm;
            u64 snd[2] = { zg, ze }, rcv[2];
            W.reshare<2>(snd, rcv, act ? 2u * (32u >> k) : 0u);   // one bit per block start, G and E
            G.o = (Gh.o & sm) ^ zg; G.n = (Gh.n & sm) ^ rcv[0];
            E.o = ze; E.n = rcv[1];
        } else {
            const u64 r = W.reshare1(zg, act ? 1u : 0u);
            G.o = (Gh.o & sm) ^ zg; G.n = (Gh.n & sm) ^ r;
        }
    }
    Sh ge;
    ge.o = ((D.rho.o >> 63) ^ G.o) & 1;
    ge.n = ((D.rho.n >> 63) ^ G.n) & 1;
    if (p == 0) ge.o ^= (c >> 63) ^ 1;
    if (p == 2) ge.n ^= (c >> 63) ^ 1;
    return ge;
}

// the same with the mask words of element e taken from the wavefront's PRF tile
// (element 64*tile + lane in every lane)
__device__ __forceinline__ Sh ge_bit(Wire &W, const PartyKeys &K, int p, u32 op, u64 e, Sh v, const Dealer &D, bool act)
{
    u64 AG, AE;
    zero_b2(K, op, 1, 2, e, AG, AE);
    return ge_bit_masks(W, p, v, D, AG, AE, act);
}

// bit -> arithmetic: open f = s xor beta; s = beta if f = 0 else 1 - beta
// (bits: what the opened value is counted as - one bit, or a ring element of 64 bits where
// the protocol is run as the paper's cost formula prices it)
__device__ __forceinline__ Sh b2a(Wire &W, int p, Sh s, const Dealer &D, bool act, u32 bits = 1)
{
    const u64 fo = (s.o ^ D.bBo) & 1, fn = (s.n ^ D.bBn) & 1;
    const u64 f = (fo ^ fn ^ W.open1(fo, act ? bits : 0u)) & 1;
    Sh one = pub(p, 1), out;
    out.o = f ? one.o - D.bA.o : D.bA.o;
    out.n = f ? one.n - D.bA.n : D.bA.n;
    return out;
}

__device__ __forceinline__ Sh not_bit(int p, Sh b) { if (p == 0) b.o ^= 1; if (p == 2) b.n ^= 1; return b; }
