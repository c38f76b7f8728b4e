// Secure ReLU (Alg. 2 + Sec. 4.2) and 2x2 max-pool by composition.
//
// Per party the protocol is a chain of streaming kernels separated by the
// exchange of masked words over the wire stream:
//
//   wire: A2B masks r_i                                   (1 word / element)
//   K_first   U, V from x_i, r_i, received r; mask for G = U & V        -> wire (2)
//   K_level l (l = 0..5): finish the AND(s) of the previous round, then mask
//             the operands of prefix level l: (P, G << 2^l), (P, P << 2^l) -> wire (4; 2 at l = 5)
//   K_sign    finish level 5, sign share = bit63(U^V) ^ bit62(G),
//             mask it with the shared random bit                          -> wire (1 byte)
//   K_b2a     additive share of the sign, m = 1 - s, mask x and m          -> wire (2)
//   K_select  y = x * m (element-wise Alg. 1)
//
// Every kernel is HBM-bound: it reads the triple words of its round once,
// carries (G, P) as state, and writes what it sends.  Chunks (Alg. 4's tiles)
// are disjoint element ranges; all chunks of a round are launched back to
// back and chunk m of the next round waits only for chunk m's copy.
//
// mpc_relu_msb is the same protocol with the carry network pruned to what the
// sign needs (the circuit of Sec. 4.2 evaluated only where bit 63 depends on
// it): prefix level l keeps the bit positions p = 2^(l+1)-2 (mod 2^(l+1)), so
// 2^(l+1) consecutive elements share one word, element k rotated left by k.
// The triples of the levels arrive packed the same way, and every exchange
// after G = U & V shrinks by the same factor.  Bit for bit the same shares.
#include "common.h"

#include <atomic>
#include "msb_pack.h"

namespace {

constexpr int kThreads = 256;
constexpr int kMaxChunks = 64;
// chunk size picked when the caller passes n_chunks = 0 and the lane sets none (mpc_ctx_set_relu_chunk)
constexpr size_t kAutoChunkElems = (size_t)1 << 20;
constexpr size_t kAutoChunkElemsPacked = (size_t)1 << 22;   // the packed path: a third of the bytes per element

struct alignas(16) u64x2 { u64 a, b; };

// Everything one party's kernels may touch.
struct ReluParty {
    const u64* x; const u64* r;
    const u64* ta; const u64* tb; const u64* tc;       // [12][n]
    const u8* rb; const u64* ra;
    const u64* ma; const u64* mb; const u64* mc;
    u64* send;      // [4][n] words this party sends in the current round
    const u64* recv;   // [4][n] words received from the other party
    u8* sendb; const u8* recvb;    // byte exchange (B2A)
    u64* G; u64* P; u8* p63;       // carried state
    u64* put; u8* putb; u64* putL; // exchange by remote store: the peer's receive buffers (null: copy kernels)
    u64* recv_alt;                 // second receive buffer, alternating with recv from stage to stage in that mode
    u64* sendL; const u64* recvL;  // packed levels (mpc_relu_msb): per level a [4][pw] block
    u64* gsel;                     // packed levels: the G bits a level keeps
    u64* y; u8* s_bit; u64* s_arith;
    size_t n;       // total elements (stride of the [12][n] / [4][n] arrays)
};

template <int V> struct Pack;
template <> struct Pack<1> {
    u64 v[1];
    __device__ static Pack ld(const u64* p, size_t i) { Pack r; r.v[0] = p[i]; return r; }
    __device__ void st(u64* p, size_t i) const { p[i] = v[0]; }
};
template <> struct Pack<2> {
    u64 v[2];
    __device__ static Pack ld(const u64* p, size_t i)
    {
        const u64x2 t = *reinterpret_cast<const u64x2*>(p + i);
        Pack r; r.v[0] = t.a; r.v[1] = t.b; return r;
    }
    __device__ void st(u64* p, size_t i) const
    {
        u64x2 t; t.a = v[0]; t.b = v[1];
        *reinterpret_cast<u64x2*>(p + i) = t;
    }
};

template <> struct Pack<4> {
    u64 v[4];
    __device__ static Pack ld(const u64* p, size_t i)
    {
        const u64x2 t = *reinterpret_cast<const u64x2*>(p + i), u = *reinterpret_cast<const u64x2*>(p + i + 2);
        Pack r; r.v[0] = t.a; r.v[1] = t.b; r.v[2] = u.a; r.v[3] = u.b; return r;
    }
    __device__ void st(u64* p, size_t i) const
    {
        u64x2 t, u; t.a = v[0]; t.b = v[1]; u.a = v[2]; u.b = v[3];
        *reinterpret_cast<u64x2*>(p + i) = t; *reinterpret_cast<u64x2*>(p + i + 2) = u;
    }
};

// V consecutive bytes (one per element): a single 16- or 32-bit access when V is 2 or 4
template <int V> __device__ __forceinline__ void ld_bytes(const u8* p, size_t i, u8 (&out)[V])
{
    if constexpr (V == 4) { const uint32_t w = *reinterpret_cast<const uint32_t*>(p + i);
                            out[0] = (u8)w; out[1] = (u8)(w >> 8); out[2] = (u8)(w >> 16); out[3] = (u8)(w >> 24); }
    else if constexpr (V == 2) { const uint16_t w = *reinterpret_cast<const uint16_t*>(p + i);
                                 out[0] = (u8)w; out[1] = (u8)(w >> 8); }
    else out[0] = p[i];
}
template <int V> __device__ __forceinline__ void st_bytes(u8* p, size_t i, const u8 (&in)[V])
{
    if constexpr (V == 4) *reinterpret_cast<uint32_t*>(p + i) = (uint32_t)in[0] | ((uint32_t)in[1] << 8) | ((uint32_t)in[2] << 16) | ((uint32_t)in[3] << 24);
    else if constexpr (V == 2) *reinterpret_cast<uint16_t*>(p + i) = (uint16_t)((uint16_t)in[0] | ((uint16_t)in[1] << 8));
    else p[i] = in[0];
}

// Beaver AND, one party's side (Eq. 4; Alg. 4 for the party that adds d & g):
// d, g are the opened masked operands, (a, b, c) this party's triple words.
template <int PARTY>
__device__ __forceinline__ u64 and_finish(u64 d, u64 g, u64 a, u64 b, u64 c)
{
    u64 t = c ^ (d & b) ^ (g & a);
    if (PARTY == 0) t ^= d & g;
    return t;
}

#define FOR_ELEMS(V)                                                                         \
    const size_t stride_ = (size_t)gridDim.x * blockDim.x * V;                               \
    for (size_t i = lo + ((size_t)blockIdx.x * blockDim.x + threadIdx.x) * V; i < hi; i += stride_)

// ---- K_first ------------------------------------------------------------------
template <int PARTY, int V, bool PUT>
__device__ __forceinline__ void b_first(const ReluParty& p, size_t lo, size_t hi)
{
    const size_t n = p.n;
    FOR_ELEMS(V) {
        const Pack<V> x = Pack<V>::ld(p.x, i), r = Pack<V>::ld(p.r, i), rr = Pack<V>::ld(p.recv, i);
        const Pack<V> a0 = Pack<V>::ld(p.ta, i), b0 = Pack<V>::ld(p.tb, i);
        Pack<V> d, g, P;
        u8 top[V];
#pragma unroll
        for (int k = 0; k < V; ++k) {
            // Alg. 2: U is the sharing of the word x_0, V of the word x_1
            const u64 U = PARTY == 0 ? (x.v[k] ^ r.v[k]) : rr.v[k];
            const u64 Vv = PARTY == 0 ? rr.v[k] : (x.v[k] ^ r.v[k]);
            d.v[k] = U ^ a0.v[k];
            g.v[k] = Vv ^ b0.v[k];
            P.v[k] = U ^ Vv;
            top[k] = (u8)(P.v[k] >> 63);
        }
        // with the exchange by remote store the next stage re-forms this party's own masked words from x, r and P
        // (U or V is the own x ^ r, the other one P ^ that), so they go to the peer only
        if constexpr (PUT) { d.st(p.put, i); g.st(p.put + n, i); }
        else               { d.st(p.send, i); g.st(p.send + n, i); }
        P.st(p.P, i);
        st_bytes<V>(p.p63, i, top);
    }
}

// ---- adder topologies -----------------------------------------------------------
// TOPO 0: Kogge-Stone, level l combines every position p with p - 2^l.
// TOPO 1: the prefix tree of the listing in Sec. 4.2, level l joins blocks of
// 2^l bits: the upper half of each 2^(l+1)-bit block (om) combines with the top
// bit of its lower half (im), copied over the upper half by a multiply (mu).
constexpr u64 tree_im(int l) { u64 m = 0; for (int b = 0; b < 64; b += 2 << l) m |= (u64)1 << (b + (1 << l) - 1); return m; }
constexpr u64 tree_om(int l)
{
    const int half = 1 << l; u64 m = 0;
    for (int b = 0; b < 64; b += 2 * half) m |= (half == 64 ? ~(u64)0 : (((u64)1 << half) - 1)) << (b + half);
    return m;
}
constexpr u64 tree_mu(int l) { u64 m = 0; for (int k = 1; k <= (1 << l); ++k) m |= (u64)1 << k; return m; }
// left operand of a level's ANDs, from P
template <int TOPO, int L> __device__ __forceinline__ u64 op_x(u64 P) { if constexpr (TOPO) return P & tree_om(L); else return P; }
// right operand, from G (first AND) or P (second AND)
template <int TOPO, int L> __device__ __forceinline__ u64 op_y(u64 w)
{
    if constexpr (TOPO) return (w & tree_im(L)) * tree_mu(L); else return w << (1 << L);
}
// the part of P a level leaves untouched
template <int TOPO, int L> __device__ __forceinline__ u64 keep_p(u64 P) { if constexpr (TOPO) return P & ~tree_om(L); else return 0; }

// ---- K_level ------------------------------------------------------------------
// LEVEL 0 finishes G = U & V (triple 0, own masked words re-read from the send
// buffer); LEVEL l > 0 finishes the two ANDs of level l-1 from the carried
// (G, P).  Then masks the operands of level LEVEL.
template <int PARTY, int LEVEL, int V, int TOPO, bool PUT>
__device__ __forceinline__ void b_level(const ReluParty& p, size_t lo, size_t hi)
{
    const size_t n = p.n;
    FOR_ELEMS(V) {
        Pack<V> G, P;
        if constexpr (LEVEL == 0) {
            const Pack<V> rd = Pack<V>::ld(p.recv, i), rg = Pack<V>::ld(p.recv + n, i);
            const Pack<V> a = Pack<V>::ld(p.ta, i), b = Pack<V>::ld(p.tb, i), c = Pack<V>::ld(p.tc, i);
            P = Pack<V>::ld(p.P, i);
            Pack<V> sd, sg;
            if constexpr (PUT) {
                // own masked words of G = U & V, re-formed: the own word of the pair (U, V) is x ^ r, the other P ^ it
                const Pack<V> x = Pack<V>::ld(p.x, i), r = Pack<V>::ld(p.r, i);
#pragma unroll
                for (int k = 0; k < V; ++k) {
                    const u64 own = x.v[k] ^ r.v[k], other = P.v[k] ^ own;
                    sd.v[k] = (PARTY == 0 ? own : other) ^ a.v[k];
                    sg.v[k] = (PARTY == 0 ? other : own) ^ b.v[k];
                }
            } else {
                sd = Pack<V>::ld(p.send, i); sg = Pack<V>::ld(p.send + n, i);
            }
#pragma unroll
            for (int k = 0; k < V; ++k)
                G.v[k] = and_finish<PARTY>(sd.v[k] ^ rd.v[k], sg.v[k] ^ rg.v[k], a.v[k], b.v[k], c.v[k]);
        } else {
            constexpr int q = LEVEL - 1;
            constexpr int t1 = 1 + 2 * q, t2 = 2 + 2 * q;
            const Pack<V> Go = Pack<V>::ld(p.G, i), Po = Pack<V>::ld(p.P, i);
            const Pack<V> rd1 = Pack<V>::ld(p.recv, i), rg1 = Pack<V>::ld(p.recv + n, i);
            const Pack<V> rd2 = Pack<V>::ld(p.recv + 2 * n, i), rg2 = Pack<V>::ld(p.recv + 3 * n, i);
            const Pack<V> a1 = Pack<V>::ld(p.ta + t1 * n, i), b1 = Pack<V>::ld(p.tb + t1 * n, i),
                          c1 = Pack<V>::ld(p.tc + t1 * n, i);
            const Pack<V> a2 = Pack<V>::ld(p.ta + t2 * n, i), b2 = Pack<V>::ld(p.tb + t2 * n, i),
                          c2 = Pack<V>::ld(p.tc + t2 * n, i);
#pragma unroll
            for (int k = 0; k < V; ++k) {
                // own masked words are recomputed from the carried state
                const u64 X = op_x<TOPO, q>(Po.v[k]);
                const u64 d1 = (X ^ a1.v[k]) ^ rd1.v[k];
                const u64 g1 = (op_y<TOPO, q>(Go.v[k]) ^ b1.v[k]) ^ rg1.v[k];
                const u64 d2 = (X ^ a2.v[k]) ^ rd2.v[k];
                const u64 g2 = (op_y<TOPO, q>(Po.v[k]) ^ b2.v[k]) ^ rg2.v[k];
                G.v[k] = Go.v[k] ^ and_finish<PARTY>(d1, g1, a1.v[k], b1.v[k], c1.v[k]);
                P.v[k] = keep_p<TOPO, q>(Po.v[k]) ^ and_finish<PARTY>(d2, g2, a2.v[k], b2.v[k], c2.v[k]);
            }
        }
        constexpr int u1 = 1 + 2 * LEVEL, u2 = 2 + 2 * LEVEL;
        const Pack<V> na1 = Pack<V>::ld(p.ta + u1 * n, i), nb1 = Pack<V>::ld(p.tb + u1 * n, i);
        Pack<V> d1, g1;
#pragma unroll
        for (int k = 0; k < V; ++k) { d1.v[k] = op_x<TOPO, LEVEL>(P.v[k]) ^ na1.v[k]; g1.v[k] = op_y<TOPO, LEVEL>(G.v[k]) ^ nb1.v[k]; }
        // The next stage recomputes this party's own masked words from the carried (G, P), so with the
        // exchange by remote store they go to the peer only; the copy exchange needs them in the send buffer.
        if constexpr (PUT) { d1.st(p.put, i); g1.st(p.put + n, i); }
        else               { d1.st(p.send, i); g1.st(p.send + n, i); }
        if constexpr (LEVEL < 5) {
            const Pack<V> na2 = Pack<V>::ld(p.ta + u2 * n, i), nb2 = Pack<V>::ld(p.tb + u2 * n, i);
            Pack<V> d2, g2;
#pragma unroll
            for (int k = 0; k < V; ++k) { d2.v[k] = op_x<TOPO, LEVEL>(P.v[k]) ^ na2.v[k]; g2.v[k] = op_y<TOPO, LEVEL>(P.v[k]) ^ nb2.v[k]; }
            if constexpr (PUT) { d2.st(p.put + 2 * n, i); g2.st(p.put + 3 * n, i); }
            else               { d2.st(p.send + 2 * n, i); g2.st(p.send + 3 * n, i); }
        }
        G.st(p.G, i); P.st(p.P, i);
    }
}

// ---- K_sign -------------------------------------------------------------------
template <int PARTY, int V, int TOPO, bool PUT>
__device__ __forceinline__ void b_sign(const ReluParty& p, size_t lo, size_t hi)
{
    const size_t n = p.n;
    constexpr int t1 = 11;
    FOR_ELEMS(V) {
        const Pack<V> Go = Pack<V>::ld(p.G, i), Po = Pack<V>::ld(p.P, i);
        const Pack<V> rd1 = Pack<V>::ld(p.recv, i), rg1 = Pack<V>::ld(p.recv + n, i);
        const Pack<V> a1 = Pack<V>::ld(p.ta + t1 * n, i), b1 = Pack<V>::ld(p.tb + t1 * n, i),
                      c1 = Pack<V>::ld(p.tc + t1 * n, i);
        u8 top[V], rb[V], sb[V], mb[V];
        ld_bytes<V>(p.p63, i, top); ld_bytes<V>(p.rb, i, rb);
#pragma unroll
        for (int k = 0; k < V; ++k) {
            const u64 d1 = (op_x<TOPO, 5>(Po.v[k]) ^ a1.v[k]) ^ rd1.v[k];
            const u64 g1 = (op_y<TOPO, 5>(Go.v[k]) ^ b1.v[k]) ^ rg1.v[k];
            const u64 G = Go.v[k] ^ and_finish<PARTY>(d1, g1, a1.v[k], b1.v[k], c1.v[k]);
            // bit 63 of the sum = bit 63 of U^V xor the carry out of bits [0..62]
            sb[k] = (u8)(top[k] ^ (u8)((G >> 62) & 1));
            mb[k] = (u8)(sb[k] ^ rb[k]);
        }
        if (p.s_bit) st_bytes<V>(p.s_bit, i, sb);
        st_bytes<V>(p.sendb, i, mb);
        if constexpr (PUT) st_bytes<V>(p.putb, i, mb);
    }
}

// ---- K_b2a --------------------------------------------------------------------
template <int PARTY, int V, bool PUT>
__device__ __forceinline__ void b_b2a(const ReluParty& p, size_t lo, size_t hi)
{
    const size_t n = p.n;
    FOR_ELEMS(V) {
        const Pack<V> x = Pack<V>::ld(p.x, i), ra = Pack<V>::ld(p.ra, i);
        const Pack<V> ma = Pack<V>::ld(p.ma, i), mb = Pack<V>::ld(p.mb, i);
        Pack<V> e, f, sa;
        u8 own[V], got[V];
        ld_bytes<V>(p.sendb, i, own); ld_bytes<V>(p.recvb, i, got);
#pragma unroll
        for (int k = 0; k < V; ++k) {
            const u64 v = (u64)(own[k] ^ got[k]);                      // opened s ^ rb
            // s = v xor rb = v + rb - 2 v rb on additive shares of rb
            sa.v[k] = ra.v[k] - 2 * v * ra.v[k] + (PARTY == 0 ? v : 0);
            const u64 m = (PARTY == 0 ? (u64)1 : (u64)0) - sa.v[k];    // shares of 1 - s
            e.v[k] = x.v[k] - ma.v[k];
            f.v[k] = m - mb.v[k];
        }
        // with the exchange by remote store the select stage re-forms this party's own masked words: peer only
        if constexpr (PUT) { e.st(p.put, i); f.st(p.put + n, i); }
        else               { e.st(p.send, i); f.st(p.send + n, i); }
        if (p.s_arith) sa.st(p.s_arith, i);
    }
}

// ---- K_select -----------------------------------------------------------------
template <int PARTY, int V, bool PUT>
__device__ __forceinline__ void b_select(const ReluParty& p, size_t lo, size_t hi)
{
    const size_t n = p.n;
    FOR_ELEMS(V) {
        const Pack<V> re = Pack<V>::ld(p.recv, i), rf = Pack<V>::ld(p.recv + n, i);
        const Pack<V> ma = Pack<V>::ld(p.ma, i), mb = Pack<V>::ld(p.mb, i), mc = Pack<V>::ld(p.mc, i);
        Pack<V> se, sf;
        if constexpr (PUT) {
            // own masked words of the select product, re-formed as the B2A stage formed them
            const Pack<V> x = Pack<V>::ld(p.x, i), ra = Pack<V>::ld(p.ra, i);
            u8 own[V], got[V];
            ld_bytes<V>(p.sendb, i, own); ld_bytes<V>(p.recvb, i, got);
#pragma unroll
            for (int k = 0; k < V; ++k) {
                const u64 v = (u64)(own[k] ^ got[k]);
                const u64 sa = ra.v[k] - 2 * v * ra.v[k] + (PARTY == 0 ? v : 0);
                se.v[k] = x.v[k] - ma.v[k];
                sf.v[k] = ((PARTY == 0 ? (u64)1 : (u64)0) - sa) - mb.v[k];
            }
        } else {
            se = Pack<V>::ld(p.send, i); sf = Pack<V>::ld(p.send + n, i);
        }
        Pack<V> y;
#pragma unroll
        for (int k = 0; k < V; ++k) {
            const u64 e = se.v[k] + re.v[k], f = sf.v[k] + rf.v[k];
            u64 t = mc.v[k] + e * mb.v[k] + ma.v[k] * f;
            if (PARTY == 0) t += e * f;
            y.v[k] = t;
        }
        y.st(p.y, i);
    }
}

// ---- MSB-only carry chain on packed words (bit geometry: msb_pack.h) -----------
// Word counts and offsets of the packed arrays for n elements.
struct MsbGeom {
    size_t n;
    size_t pw[6];      // words of level l's packed arrays: ceil64(n) / 2^(l+1), rounded up to 4
    size_t toff[12];   // offset of triple t inside a packed and_a / and_b / and_c buffer
    size_t loff[6];    // offset of level l's [4][pw] block inside sendL / recvL
    size_t goff[6];    // offset of level l's words inside gsel
    size_t words_triples, words_level_blocks, words_gsel;
};

MsbGeom msb_geom(size_t n)
{
    MsbGeom g{};
    g.n = n;
    size_t lo = 0, go = 0;
    for (int l = 0; l < 6; ++l) {
        g.pw[l] = msb_level_words(n, l);
        g.loff[l] = lo; lo += 4 * g.pw[l];
        g.goff[l] = go; go += g.pw[l];
    }
    g.toff[0] = 0;
    size_t to = (n + 3) / 4 * 4;
    for (int t = 1; t < 12; ++t) { g.toff[t] = to; to += g.pw[(t - 1) / 2]; }
    g.words_triples = to; g.words_level_blocks = lo; g.words_gsel = go;
    return g;
}

template <int V> __device__ __forceinline__ Pack<V> ld_upto(const u64* p, size_t i, size_t n)
{
    if constexpr (V == 4) return Pack<4>::ld(p, i);      // the caller guarantees i + 3 < n
    else { Pack<V> r;
#pragma unroll
           for (int k = 0; k < V; ++k) r.v[k] = i + k < n ? p[i + k] : 0;
           return r; }
}

// Stage 1 + LEVEL of the packed chain: finish the previous round's ANDs for the
// 2 W input words behind W output words, regroup, and mask this level's operands.
template <int PARTY, int LEVEL, int W, bool PUT>
__device__ __forceinline__ void b_plevel(const ReluParty& p, const MsbGeom& g, size_t lo, size_t hi)
{
    constexpr int d = 1 << LEVEL, s = 2 * d;
    constexpr u64 A = sel_mask(LEVEL), B = low_mask(LEVEL);
    const size_t wlo = lo >> (LEVEL + 1), whi = (hi + s - 1) >> (LEVEL + 1);
    const size_t stride = (size_t)gridDim.x * blockDim.x * W;
    for (size_t j = wlo + ((size_t)blockIdx.x * blockDim.x + threadIdx.x) * W; j < whi; j += stride) {
        Pack<2 * W> G, P;
        if constexpr (LEVEL == 0) {
            const size_t n = p.n, e = 2 * j;
            const Pack<2 * W> rd = ld_upto<2 * W>(p.recv, e, n), rg = ld_upto<2 * W>(p.recv + n, e, n);
            const Pack<2 * W> a = ld_upto<2 * W>(p.ta, e, n), b = ld_upto<2 * W>(p.tb, e, n), c = ld_upto<2 * W>(p.tc, e, n);
            P = ld_upto<2 * W>(p.P, e, n);
            Pack<2 * W> sd, sg;
            if constexpr (PUT) {
                // own masked words of G = U & V, re-formed as in the whole-word level-0 stage
                const Pack<2 * W> x = ld_upto<2 * W>(p.x, e, n), r = ld_upto<2 * W>(p.r, e, n);
#pragma unroll
                for (int k = 0; k < 2 * W; ++k) {
                    const u64 own = x.v[k] ^ r.v[k], other = P.v[k] ^ own;
                    sd.v[k] = (PARTY == 0 ? own : other) ^ a.v[k];
                    sg.v[k] = (PARTY == 0 ? other : own) ^ b.v[k];
                }
            } else {
                sd = ld_upto<2 * W>(p.send, e, n); sg = ld_upto<2 * W>(p.send + n, e, n);
            }
#pragma unroll
            for (int k = 0; k < 2 * W; ++k)
                G.v[k] = and_finish<PARTY>(sd.v[k] ^ rd.v[k], sg.v[k] ^ rg.v[k], a.v[k], b.v[k], c.v[k]);
        } else {
            static_assert(LEVEL == 0 || W == 2, "packed levels run two output words per thread");
            constexpr int q = LEVEL - 1, t1 = 1 + 2 * q, t2 = 2 + 2 * q;
            const size_t w = 2 * j, pq = g.pw[q];
            const u64* sp = p.sendL + g.loff[q]; const u64* rp = p.recvL + g.loff[q];
            const Pack<4> gs = Pack<4>::ld(p.gsel + g.goff[q], w);
            const Pack<4> sd1 = Pack<4>::ld(sp, w), sg1 = Pack<4>::ld(sp + pq, w);
            const Pack<4> sd2 = Pack<4>::ld(sp + 2 * pq, w), sg2 = Pack<4>::ld(sp + 3 * pq, w);
            const Pack<4> rd1 = Pack<4>::ld(rp, w), rg1 = Pack<4>::ld(rp + pq, w);
            const Pack<4> rd2 = Pack<4>::ld(rp + 2 * pq, w), rg2 = Pack<4>::ld(rp + 3 * pq, w);
            const Pack<4> a1 = Pack<4>::ld(p.ta + g.toff[t1], w), b1 = Pack<4>::ld(p.tb + g.toff[t1], w),
                          c1 = Pack<4>::ld(p.tc + g.toff[t1], w);
            const Pack<4> a2 = Pack<4>::ld(p.ta + g.toff[t2], w), b2 = Pack<4>::ld(p.tb + g.toff[t2], w),
                          c2 = Pack<4>::ld(p.tc + g.toff[t2], w);
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                G.v[k] = gs.v[k] ^ and_finish<PARTY>(sd1.v[k] ^ rd1.v[k], sg1.v[k] ^ rg1.v[k], a1.v[k], b1.v[k], c1.v[k]);
                P.v[k] = and_finish<PARTY>(sd2.v[k] ^ rd2.v[k], sg2.v[k] ^ rg2.v[k], a2.v[k], b2.v[k], c2.v[k]);
            }
        }
        Pack<W> X, Gk, Y1, Y2;
#pragma unroll
        for (int k = 0; k < W; ++k) {
            const u64 Glo = G.v[2 * k], Ghi = G.v[2 * k + 1], Plo = P.v[2 * k], Phi = P.v[2 * k + 1];
            X.v[k] = (Plo & A) | rotl<d>(Phi & A);           // P[p]
            Gk.v[k] = (Glo & A) | rotl<d>(Ghi & A);          // G[p]
            Y1.v[k] = rotl<d>(Glo & B) | rotl<2 * d>(Ghi & B);   // G[p - d] moved to p
            Y2.v[k] = rotl<d>(Plo & B) | rotl<2 * d>(Phi & B);   // P[p - d] moved to p
        }
        constexpr int u1 = 1 + 2 * LEVEL, u2 = 2 + 2 * LEVEL;
        const size_t pl = g.pw[LEVEL];
        u64* so = p.sendL + g.loff[LEVEL];
        const Pack<W> na1 = Pack<W>::ld(p.ta + g.toff[u1], j), nb1 = Pack<W>::ld(p.tb + g.toff[u1], j);
        Pack<W> d1, g1;
#pragma unroll
        for (int k = 0; k < W; ++k) { d1.v[k] = X.v[k] ^ na1.v[k]; g1.v[k] = Y1.v[k] ^ nb1.v[k]; }
        u64* po = PUT ? p.putL + g.loff[LEVEL] : nullptr;
        d1.st(so, j); g1.st(so + pl, j);
        if constexpr (PUT) { d1.st(po, j); g1.st(po + pl, j); }
        if constexpr (LEVEL < 5) {
            const Pack<W> na2 = Pack<W>::ld(p.ta + g.toff[u2], j), nb2 = Pack<W>::ld(p.tb + g.toff[u2], j);
            Pack<W> d2, g2;
#pragma unroll
            for (int k = 0; k < W; ++k) { d2.v[k] = X.v[k] ^ na2.v[k]; g2.v[k] = Y2.v[k] ^ nb2.v[k]; }
            d2.st(so + 2 * pl, j); g2.st(so + 3 * pl, j);
            if constexpr (PUT) { d2.st(po + 2 * pl, j); g2.st(po + 3 * pl, j); }
        }
        Gk.st(p.gsel + g.goff[LEVEL], j);
    }
}

// Packed K_sign: finish level 5; element i's carry into bit 63 sits at bit
// (62 + i) mod 64 of word i / 64.
template <int PARTY, int V, bool PUT>
__device__ __forceinline__ void b_psign(const ReluParty& p, const MsbGeom& g, size_t lo, size_t hi)
{
    const size_t p5 = g.pw[5];
    const u64* sp = p.sendL + g.loff[5]; const u64* rp = p.recvL + g.loff[5];
    const u64* gs = p.gsel + g.goff[5];
    const u64 *a = p.ta + g.toff[11], *b = p.tb + g.toff[11], *c = p.tc + g.toff[11];
    FOR_ELEMS(V) {
        u8 top[V], rb[V], sb[V], mb[V];
        ld_bytes<V>(p.p63, i, top); ld_bytes<V>(p.rb, i, rb);
        size_t w_have = ~(size_t)0; u64 Gw = 0;
#pragma unroll
        for (int k = 0; k < V; ++k) {
            const size_t w = (i + k) >> 6;
            if (w != w_have) {
                Gw = gs[w] ^ and_finish<PARTY>(sp[w] ^ rp[w], sp[p5 + w] ^ rp[p5 + w], a[w], b[w], c[w]);
                w_have = w;
            }
            sb[k] = (u8)(top[k] ^ (u8)((Gw >> ((62 + i + k) & 63)) & 1));
            mb[k] = (u8)(sb[k] ^ rb[k]);
        }
        if (p.s_bit) st_bytes<V>(p.s_bit, i, sb);
        st_bytes<V>(p.sendb, i, mb);
        if constexpr (PUT) st_bytes<V>(p.putb, i, mb);
    }
}

// Offline helper: triple-major [12][n] words -> the packed layout (blockIdx.y = triple).
__global__ __launch_bounds__(kThreads) void k_pack_triples(const u64* __restrict__ in, u64* __restrict__ out, MsbGeom g)
{
    const int t = blockIdx.y;
    const size_t n = g.n, stride = (size_t)gridDim.x * blockDim.x;
    const size_t first = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t == 0) {
        for (size_t i = first; i < g.toff[1]; i += stride) out[i] = i < n ? in[i] : 0;
        return;
    }
    const int l = (t - 1) / 2, s = 2 << l;
    u64 m = 0;
    for (int q = s - 2; q < 63; q += s) m |= (u64)1 << q;
    for (size_t j = first; j < g.pw[l]; j += stride) {
        u64 acc = 0;
        for (int k = 0; k < s; ++k) {
            const size_t e = j * s + k;
            if (e < n) { const u64 v = in[(size_t)t * n + e] & m; acc |= k ? (v << k) | (v >> (64 - k)) : v; }
        }
        out[g.toff[t] + j] = acc;
    }
}

// rows x len words, both sides with pitch `pitch` words: the per-round wire copy
// blockIdx.y selects the direction: 0 = party 0 -> party 1, 1 = party 1 -> party 0
// All rows of a position are loaded before any is stored, so a thread keeps ROWS loads in flight.
template <int ROWS>
__global__ __launch_bounds__(kThreads) void k_wire_words(const u64* __restrict__ src0, u64* __restrict__ dst0,
                                                         const u64* __restrict__ src1, u64* __restrict__ dst1,
                                                         size_t pitch, size_t lo, size_t hi)
{
    const u64* src = blockIdx.y ? src1 : src0; u64* dst = blockIdx.y ? dst1 : dst0;
    const size_t stride = (size_t)gridDim.x * blockDim.x * 2;
    for (size_t i = lo + ((size_t)blockIdx.x * blockDim.x + threadIdx.x) * 2; i < hi; i += stride) {
        u64x2 v[ROWS];
#pragma unroll
        for (int r = 0; r < ROWS; ++r) v[r] = *reinterpret_cast<const u64x2*>(src + (size_t)r * pitch + i);
#pragma unroll
        for (int r = 0; r < ROWS; ++r) *reinterpret_cast<u64x2*>(dst + (size_t)r * pitch + i) = v[r];
    }
}
__global__ __launch_bounds__(kThreads) void k_wire_words1(const u64* __restrict__ src0, u64* __restrict__ dst0,
                                                          const u64* __restrict__ src1, u64* __restrict__ dst1,
                                                          size_t pitch, size_t lo, size_t hi, int rows)
{
    const u64* src = blockIdx.y ? src1 : src0; u64* dst = blockIdx.y ? dst1 : dst0;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (int r = 0; r < rows; ++r)
        for (size_t i = lo + (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < hi; i += stride)
            dst[(size_t)r * pitch + i] = src[(size_t)r * pitch + i];
}
__global__ __launch_bounds__(kThreads) void k_wire_bytes(const u8* __restrict__ src0, u8* __restrict__ dst0,
                                                         const u8* __restrict__ src1, u8* __restrict__ dst1,
                                                         size_t lo, size_t hi)
{
    const u8* src = blockIdx.y ? src1 : src0; u8* dst = blockIdx.y ? dst1 : dst0;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = lo + (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < hi; i += stride) dst[i] = src[i];
}

inline int grid_for(size_t items)
{
    size_t blocks = (items + kThreads - 1) / kThreads;
    if (blocks > 256 * 16) blocks = 256 * 16;
    if (blocks < 1) blocks = 1;
    return (int)blocks;
}

struct ReluWs {
    u64 *send[2], *recv[2];     // [4][n]
    u8 *sendb[2], *recvb[2];
    u64 *G[2], *P[2]; u8* p63[2];
    u64* recv2[2];                          // second receive buffer (exchange by remote store alternates)
    u64 *sendL[2], *recvL[2], *gsel[2];     // packed levels only
    size_t bytes; bool ok;
};

ReluWs carve_relu(u8* base, size_t cap, size_t n)
{
    WsAlloc w(base, cap);
    ReluWs r{};
    for (int i = 0; i < 2; ++i) {
        r.send[i] = w.take<u64>(4 * n); r.recv[i] = w.take<u64>(4 * n);
        r.sendb[i] = w.take<u8>(n); r.recvb[i] = w.take<u8>(n);
        r.G[i] = w.take<u64>(n); r.P[i] = w.take<u64>(n); r.p63[i] = w.take<u8>(n);
    }
    for (int i = 0; i < 2; ++i) r.recv2[i] = w.take<u64>(4 * n);      // only touched by the remote-store exchange
    r.bytes = w.off; r.ok = w.ok;
    return r;
}

ReluWs carve_relu_msb(u8* base, size_t cap, size_t n, const MsbGeom& g)
{
    WsAlloc w(base, cap);
    ReluWs r{};
    for (int i = 0; i < 2; ++i) {
        r.send[i] = w.take<u64>(2 * n); r.recv[i] = w.take<u64>(2 * n);
        r.sendb[i] = w.take<u8>(n); r.recvb[i] = w.take<u8>(n);
        r.P[i] = w.take<u64>(n); r.p63[i] = w.take<u8>(n);
        r.sendL[i] = w.take<u64>(g.words_level_blocks); r.recvL[i] = w.take<u64>(g.words_level_blocks);
        r.gsel[i] = w.take<u64>(g.words_gsel);
    }
    for (int i = 0; i < 2; ++i) r.recv2[i] = w.take<u64>(2 * n);
    r.bytes = w.off; r.ok = w.ok;
    return r;
}

enum Stage { ST_FIRST = 0, ST_LEVEL0 = 1, ST_SIGN = 7, ST_B2A = 8, ST_SELECT = 9, ST_COUNT = 10 };

// One launch runs a protocol stage for both parties (blockIdx.y = party) or,
// when the parties live on different streams, for party `only` alone.
template <int STAGE, int PARTY, int V, int TOPO, bool PUT>
__device__ __forceinline__ void stage_body(const ReluParty& p, size_t lo, size_t hi)
{
    if constexpr (STAGE == 0) b_first<PARTY, V, PUT>(p, lo, hi);
    else if constexpr (STAGE >= 1 && STAGE <= 6) b_level<PARTY, STAGE - 1, V, TOPO, PUT>(p, lo, hi);
    else if constexpr (STAGE == 7) b_sign<PARTY, V, TOPO, PUT>(p, lo, hi);
    else if constexpr (STAGE == 8) b_b2a<PARTY, V, PUT>(p, lo, hi);
    else b_select<PARTY, V, PUT>(p, lo, hi);
}

template <int STAGE, int V, int TOPO, bool PUT>
__global__ __launch_bounds__(kThreads) void k_relu_stage(ReluParty p0, ReluParty p1, int only, size_t lo, size_t hi)
{
    const int party = only >= 0 ? only : (int)blockIdx.y;
    if (party == 0) stage_body<STAGE, 0, V, TOPO, PUT>(p0, lo, hi);
    else            stage_body<STAGE, 1, V, TOPO, PUT>(p1, lo, hi);
}

template <int STAGE, int V>
void launch_stage_t(hipStream_t st, const ReluParty& p0, const ReluParty& p1, int only, size_t lo, size_t hi, int topo)
{
    const dim3 grid(grid_for((hi - lo + V - 1) / V), only >= 0 ? 1 : 2), block(kThreads);
    // only the carry-network stages depend on the topology; the last stage sends nothing, but with the exchange
    // by remote store it re-forms its own masked words instead of reading them back
    constexpr int T1 = (STAGE >= 1 && STAGE <= 7) ? 1 : 0;
    constexpr bool P1 = true;
    const bool put = p0.put != nullptr && P1;
    if (topo && T1) {
        if (put) hipLaunchKernelGGL((k_relu_stage<STAGE, V, T1, P1>), grid, block, 0, st, p0, p1, only, lo, hi);
        else     hipLaunchKernelGGL((k_relu_stage<STAGE, V, T1, false>), grid, block, 0, st, p0, p1, only, lo, hi);
    } else {
        if (put) hipLaunchKernelGGL((k_relu_stage<STAGE, V, 0, P1>), grid, block, 0, st, p0, p1, only, lo, hi);
        else     hipLaunchKernelGGL((k_relu_stage<STAGE, V, 0, false>), grid, block, 0, st, p0, p1, only, lo, hi);
    }
}

template <int V>
void launch_stage(int stage, hipStream_t st, const ReluParty& p0, const ReluParty& p1, int only, size_t lo, size_t hi, int topo)
{
    switch (stage) {
    case 0: launch_stage_t<0, V>(st, p0, p1, only, lo, hi, topo); break;
    case 1: launch_stage_t<1, V>(st, p0, p1, only, lo, hi, topo); break;
    case 2: launch_stage_t<2, V>(st, p0, p1, only, lo, hi, topo); break;
    case 3: launch_stage_t<3, V>(st, p0, p1, only, lo, hi, topo); break;
    case 4: launch_stage_t<4, V>(st, p0, p1, only, lo, hi, topo); break;
    case 5: launch_stage_t<5, V>(st, p0, p1, only, lo, hi, topo); break;
    case 6: launch_stage_t<6, V>(st, p0, p1, only, lo, hi, topo); break;
    case 7: launch_stage_t<7, V>(st, p0, p1, only, lo, hi, topo); break;
    case 8: launch_stage_t<8, V>(st, p0, p1, only, lo, hi, topo); break;
    case 9: launch_stage_t<9, V>(st, p0, p1, only, lo, hi, topo); break;
    default: break;
    }
}

// The packed chain: stages 1..7 work on packed words, the others are shared.
template <int STAGE, int PARTY, int V, bool PUT>
__device__ __forceinline__ void stage_body_msb(const ReluParty& p, const MsbGeom& g, size_t lo, size_t hi)
{
    if constexpr (STAGE == 0) b_first<PARTY, V, PUT>(p, lo, hi);
    else if constexpr (STAGE == 1) b_plevel<PARTY, 0, (V == 4 ? 2 : 1), PUT>(p, g, lo, hi);
    else if constexpr (STAGE >= 2 && STAGE <= 6) b_plevel<PARTY, STAGE - 1, 2, PUT>(p, g, lo, hi);
    else if constexpr (STAGE == 7) b_psign<PARTY, V, PUT>(p, g, lo, hi);
    else if constexpr (STAGE == 8) b_b2a<PARTY, V, PUT>(p, lo, hi);
    else b_select<PARTY, V, PUT>(p, lo, hi);
}

template <int STAGE, int V, bool PUT>
__global__ __launch_bounds__(kThreads) void k_relu_msb_stage(ReluParty p0, ReluParty p1, MsbGeom g, int only,
                                                             size_t lo, size_t hi)
{
    const int party = only >= 0 ? only : (int)blockIdx.y;
    if (party == 0) stage_body_msb<STAGE, 0, V, PUT>(p0, g, lo, hi);
    else            stage_body_msb<STAGE, 1, V, PUT>(p1, g, lo, hi);
}

template <int STAGE, int V>
void launch_msb_stage_t(hipStream_t st, const ReluParty& p0, const ReluParty& p1, const MsbGeom& g, int only,
                        size_t lo, size_t hi)
{
    size_t threads;
    if (STAGE >= 1 && STAGE <= 6) {
        const int level = STAGE - 1, per_thread = (STAGE == 1 && V != 4) ? 1 : 2;
        const size_t words = ((hi + ((size_t)2 << level) - 1) >> (level + 1)) - (lo >> (level + 1));
        threads = (words + per_thread - 1) / per_thread;
    } else {
        threads = (hi - lo + V - 1) / V;
    }
    const dim3 grid(grid_for(threads), only >= 0 ? 1 : 2), block(kThreads);
    constexpr bool P1 = true;
    if (p0.put != nullptr && P1) hipLaunchKernelGGL((k_relu_msb_stage<STAGE, V, P1>), grid, block, 0, st, p0, p1, g, only, lo, hi);
    else                         hipLaunchKernelGGL((k_relu_msb_stage<STAGE, V, false>), grid, block, 0, st, p0, p1, g, only, lo, hi);
}

template <int V>
void launch_msb_stage(int stage, hipStream_t st, const ReluParty& p0, const ReluParty& p1, const MsbGeom& g,
                      int only, size_t lo, size_t hi)
{
    switch (stage) {
    case 0: launch_msb_stage_t<0, V>(st, p0, p1, g, only, lo, hi); break;
    case 1: launch_msb_stage_t<1, V>(st, p0, p1, g, only, lo, hi); break;
    case 2: launch_msb_stage_t<2, V>(st, p0, p1, g, only, lo, hi); break;
    case 3: launch_msb_stage_t<3, V>(st, p0, p1, g, only, lo, hi); break;
    case 4: launch_msb_stage_t<4, V>(st, p0, p1, g, only, lo, hi); break;
    case 5: launch_msb_stage_t<5, V>(st, p0, p1, g, only, lo, hi); break;
    case 6: launch_msb_stage_t<6, V>(st, p0, p1, g, only, lo, hi); break;
    case 7: launch_msb_stage_t<7, V>(st, p0, p1, g, only, lo, hi); break;
    case 8: launch_msb_stage_t<8, V>(st, p0, p1, g, only, lo, hi); break;
    case 9: launch_msb_stage_t<9, V>(st, p0, p1, g, only, lo, hi); break;
    default: break;
    }
}

// words (rows of the [4][n] buffer) exchanged after each stage; 0 = byte exchange
inline int words_after(int stage)
{
    if (stage == ST_FIRST) return 2;
    if (stage >= ST_LEVEL0 && stage < ST_LEVEL0 + 5) return 4;
    if (stage == ST_LEVEL0 + 5) return 2;
    if (stage == ST_SIGN) return 0;
    if (stage == ST_B2A) return 2;
    return -1;  // select: nothing to send
}

// one exchange: party 0's words to party 1's receive buffer and vice versa
int wire_words(mpc_ctx* c, const u64* src0, u64* dst0, const u64* src1, u64* dst1,
               size_t pitch, size_t lo, size_t hi, int rows, bool vec)
{
    const size_t len = hi - lo;
    if (vec && rows == 4)
        hipLaunchKernelGGL(k_wire_words<4>, dim3(grid_for(len / 2), 2), dim3(kThreads), 0, c->s[2], src0, dst0, src1, dst1, pitch, lo, hi);
    else if (vec && rows == 2)
        hipLaunchKernelGGL(k_wire_words<2>, dim3(grid_for(len / 2), 2), dim3(kThreads), 0, c->s[2], src0, dst0, src1, dst1, pitch, lo, hi);
    else if (vec && rows == 1)
        hipLaunchKernelGGL(k_wire_words<1>, dim3(grid_for(len / 2), 2), dim3(kThreads), 0, c->s[2], src0, dst0, src1, dst1, pitch, lo, hi);
    else
        hipLaunchKernelGGL(k_wire_words1, dim3(grid_for(len), 2), dim3(kThreads), 0, c->s[2],
                           src0, dst0, src1, dst1, pitch, lo, hi, rows);
    MPC_HIP(c, hipGetLastError());
    return MPC_OK;
}

// The protocol on n elements whose buffers are described by parties[2].  With
// `geom` the carry chain runs on packed words (mpc_relu_msb), without it on
// whole words.
int relu_run(mpc_ctx* c, ReluParty (&pp)[2], size_t n, int n_chunks, const MsbGeom* geom = nullptr)
{
    const bool one_queue = c->s[0] == c->s[1] && c->s[1] == c->s[2];   // in-order queue: no events needed
    // chunk boundaries: multiples of four elements, and of 256 on the packed path
    // (four whole words of the deepest level)
    const size_t align = geom ? 256 : 4;
    const size_t lane_elems = c->relu_chunk[geom ? 1 : 0];
    const size_t auto_elems = lane_elems ? lane_elems : geom ? kAutoChunkElemsPacked : kAutoChunkElems;
    if (n_chunks == 0)
        // automatic: about a million elements per chunk on a single queue (the chunk's
        // state then survives in the last-level cache from round to round), one chunk otherwise
        n_chunks = one_queue ? (int)((n + auto_elems / 2) / auto_elems) : 1;
    if (n_chunks > kMaxChunks) n_chunks = kMaxChunks;
    if ((size_t)n_chunks > (n + align - 1) / align) n_chunks = (int)((n + align - 1) / align);
    if (n_chunks < 1) n_chunks = 1;
    // 16-byte accesses need even n (so that every [k][n] row stays aligned) and aligned bases;
    // four elements per thread additionally need n % 4 == 0 and 4-byte aligned byte arrays
    bool vec = (n % 2 == 0);
    for (int i = 0; i < 2 && vec; ++i) {
        const void* ptrs[] = { pp[i].x, pp[i].r, pp[i].ta, pp[i].tb, pp[i].tc, pp[i].ra, pp[i].ma,
                               pp[i].mb, pp[i].mc, pp[i].y, pp[i].s_arith };
        for (const void* q : ptrs) if (q && ((uintptr_t)q & 15)) vec = false;
    }
    bool vec4 = vec && (n % 4 == 0);
    for (int i = 0; i < 2 && vec4; ++i)
        if (((uintptr_t)pp[i].rb & 3) || (pp[i].s_bit && ((uintptr_t)pp[i].s_bit & 3))) vec4 = false;
    size_t lo[kMaxChunks], hi[kMaxChunks];
    for (int m = 0; m < n_chunks; ++m) {
        lo[m] = (n * m / n_chunks) & ~(align - 1);
        hi[m] = (m == n_chunks - 1) ? n : ((n * (m + 1) / n_chunks) & ~(align - 1));
    }
    hipStream_t P[2] = { c->s[0], c->s[1] }, Wr = c->s[2];
    hipEvent_t got[kMaxChunks];

    // stage `stage` on elements [l, h): both parties in one launch (only = -1) or party `only`
    auto launch_with = [&](const ReluParty (&q)[2], int stage, hipStream_t st, int only, size_t l, size_t h) -> int {
        if (geom) {
            if (vec4)     launch_msb_stage<4>(stage, st, q[0], q[1], *geom, only, l, h);
            else if (vec) launch_msb_stage<2>(stage, st, q[0], q[1], *geom, only, l, h);
            else          launch_msb_stage<1>(stage, st, q[0], q[1], *geom, only, l, h);
        } else {
            if (vec4)     launch_stage<4>(stage, st, q[0], q[1], only, l, h, c->adder);
            else if (vec) launch_stage<2>(stage, st, q[0], q[1], only, l, h, c->adder);
            else          launch_stage<1>(stage, st, q[0], q[1], only, l, h, c->adder);
        }
        MPC_HIP(c, hipGetLastError());
        return MPC_OK;
    };
    auto launch = [&](int stage, hipStream_t st, int only, size_t l, size_t h) -> int {
        return launch_with(pp, stage, st, only, l, h);
    };
    // the exchange that follows `stage` (-1: the A2B masks); *sent = false if the stage sends nothing
    auto exchange = [&](int stage, size_t l, size_t h, bool* sent) -> int {
        *sent = true;
        if (stage < 0)
            return wire_words(c, pp[0].r, const_cast<u64*>(pp[1].recv), pp[1].r, const_cast<u64*>(pp[0].recv),
                              n, l, h, 1, vec);
        const int rows = words_after(stage);
        if (rows < 0) { *sent = false; return MPC_OK; }
        if (rows == 0) {
            hipLaunchKernelGGL(k_wire_bytes, dim3(grid_for(h - l), 2), dim3(kThreads), 0, Wr,
                               pp[0].sendb, const_cast<u8*>(pp[1].recvb), pp[1].sendb, const_cast<u8*>(pp[0].recvb), l, h);
            MPC_HIP(c, hipGetLastError());
            return MPC_OK;
        }
        if (geom && stage >= ST_LEVEL0 && stage < ST_SIGN) {
            // packed level: `rows` rows of pw words; the range is rounded to whole 16-byte units
            const int level = stage - ST_LEVEL0;
            const size_t wl = l >> (level + 1);
            const size_t wh = ((((h + ((size_t)2 << level) - 1) >> (level + 1)) + 1) & ~(size_t)1);
            const size_t off = geom->loff[level];
            return wire_words(c, pp[0].sendL + off, const_cast<u64*>(pp[1].recvL) + off,
                              pp[1].sendL + off, const_cast<u64*>(pp[0].recvL) + off,
                              geom->pw[level], wl, wh, rows, true);
        }
        return wire_words(c, pp[0].send, const_cast<u64*>(pp[1].recv), pp[1].send, const_cast<u64*>(pp[0].recv),
                          n, l, h, rows, vec);
    };
    bool sent;

    if (one_queue) {
        // One in-order queue: chunk-major order.  A chunk runs through all ten
        // rounds before the next one starts, so its carried state and exchange
        // buffers are still in the last-level cache when the next round reads them.
        for (int m = 0; m < n_chunks; ++m) {
            if (hi[m] <= lo[m]) continue;
            MPC_TRY(exchange(-1, lo[m], hi[m], &sent));
            for (int stage = 0; stage < ST_COUNT; ++stage) {
                if (c->exchange_put) {
                    // Exchange by remote store: the stage kernel writes its masked words into the
                    // peer's receive buffer as well; the word buffers alternate so that a stage
                    // never stores where the peer's same stage still reads.
                    ReluParty q[2] = { pp[0], pp[1] };
                    for (int i = 0; i < 2; ++i) {
                        u64* mine[2] = { const_cast<u64*>(pp[i].recv), pp[i].recv_alt };
                        u64* peer[2] = { const_cast<u64*>(pp[1 - i].recv), pp[1 - i].recv_alt };
                        q[i].recv = mine[stage & 1];
                        q[i].put = peer[(stage + 1) & 1];
                        q[i].putb = const_cast<u8*>(pp[1 - i].recvb);
                        q[i].putL = const_cast<u64*>(pp[1 - i].recvL);
                    }
                    MPC_TRY(launch_with(q, stage, P[0], -1, lo[m], hi[m]));
                    continue;
                }
                MPC_TRY(launch(stage, P[0], -1, lo[m], hi[m]));
                MPC_TRY(exchange(stage, lo[m], hi[m], &sent));
            }
        }
        return MPC_OK;
    }

    // Alg. 4 order on three queues.  Alg. 2 first: each party sends the mask half
    // of the XOR sharing of its own share
    for (int m = 0; m < n_chunks; ++m) {
        if (hi[m] <= lo[m]) continue;
        MPC_TRY(exchange(-1, lo[m], hi[m], &sent));
        got[m] = next_event(c); MPC_HIP(c, hipEventRecord(got[m], Wr));
    }
    for (int stage = 0; stage < ST_COUNT; ++stage) {
        const bool sends = words_after(stage) >= 0;
        for (int m = 0; m < n_chunks; ++m) {
            if (hi[m] <= lo[m]) continue;
            for (int i = 0; i < 2; ++i) {
                MPC_HIP(c, hipStreamWaitEvent(P[i], got[m], 0));
                MPC_TRY(launch(stage, P[i], i, lo[m], hi[m]));
                if (sends) MPC_TRY(chain(c, P[i], Wr));
            }
            if (!sends) continue;
            MPC_TRY(exchange(stage, lo[m], hi[m], &sent));
            got[m] = next_event(c); MPC_HIP(c, hipEventRecord(got[m], Wr));
        }
    }
    return MPC_OK;
}

int check_material(const mpc_relu_material* m)
{
    if (!m) return MPC_EINVAL;
    for (int i = 0; i < 2; ++i)
        if (!m->r.p[i] || !m->and_a.p[i] || !m->and_b.p[i] || !m->and_c.p[i] || !m->rb[i] || !m->ra.p[i] ||
            !m->ma.p[i] || !m->mb.p[i] || !m->mc.p[i])
            return MPC_EINVAL;
    return MPC_OK;
}

void fill_party(ReluParty& p, int i, const u64* x, const mpc_relu_material* m, const ReluWs& w, u64* y,
                u8* s_bit, u64* s_arith, size_t n)
{
    p.x = x; p.r = m->r.p[i];
    p.ta = m->and_a.p[i]; p.tb = m->and_b.p[i]; p.tc = m->and_c.p[i];
    p.rb = m->rb[i]; p.ra = m->ra.p[i];
    p.ma = m->ma.p[i]; p.mb = m->mb.p[i]; p.mc = m->mc.p[i];
    p.send = w.send[i]; p.recv = w.recv[i]; p.sendb = w.sendb[i]; p.recvb = w.recvb[i];
    p.put = nullptr; p.putb = nullptr; p.putL = nullptr; p.recv_alt = w.recv2[i];
    p.G = w.G[i]; p.P = w.P[i]; p.p63 = w.p63[i];
    p.sendL = w.sendL[i]; p.recvL = w.recvL[i]; p.gsel = w.gsel[i];
    p.y = y; p.s_bit = s_bit; p.s_arith = s_arith; p.n = n;
}

// ---- max-pool gathers (local, linear) ----------------------------------------------
// level 1: d[2o] = p00 - p01, d[2o+1] = p10 - p11 for output index o (NHWC)
__global__ __launch_bounds__(kThreads) void k_pool_l1(const u64* __restrict__ x, u64* __restrict__ d,
                                                      int B, int H, int W, int C)
{
    const int Ho = H / 2, Wo = W / 2;
    const size_t n_out = (size_t)B * Ho * Wo * C;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t o = (size_t)blockIdx.x * blockDim.x + threadIdx.x; o < n_out; o += stride) {
        const int ch = (int)(o % C); size_t t = o / C;
        const int wo = (int)(t % Wo); t /= Wo;
        const int ho = (int)(t % Ho); const int b = (int)(t / Ho);
        const size_t base = (((size_t)b * H + 2 * ho) * W + 2 * wo) * C + ch;
        const size_t dw = C, dh = (size_t)W * C;
        d[2 * o + 0] = x[base] - x[base + dw];
        d[2 * o + 1] = x[base + dh] - x[base + dh + dw];
    }
}
// level 2: u = p01 + r1[2o], v = p11 + r1[2o+1]; keep v, d2 = u - v
__global__ __launch_bounds__(kThreads) void k_pool_l2(const u64* __restrict__ x, const u64* __restrict__ r1,
                                                      u64* __restrict__ v_out, u64* __restrict__ d2,
                                                      int B, int H, int W, int C)
{
    const int Ho = H / 2, Wo = W / 2;
    const size_t n_out = (size_t)B * Ho * Wo * C;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t o = (size_t)blockIdx.x * blockDim.x + threadIdx.x; o < n_out; o += stride) {
        const int ch = (int)(o % C); size_t t = o / C;
        const int wo = (int)(t % Wo); t /= Wo;
        const int ho = (int)(t % Ho); const int b = (int)(t / Ho);
        const size_t base = (((size_t)b * H + 2 * ho) * W + 2 * wo) * C + ch;
        const size_t dw = C, dh = (size_t)W * C;
        const u64 u = x[base + dw] + r1[2 * o];
        const u64 v = x[base + dh + dw] + r1[2 * o + 1];
        v_out[o] = v;
        d2[o] = u - v;
    }
}

// Shared body of the two entry points; `packed` selects the MSB-only chain.
int relu_entry(mpc_ctx* c, mpc_cshare x, const mpc_relu_material* mat, mpc_share y, size_t n, int n_chunks,
               uint8_t* const s_bit[2], uint64_t* const s_arith[2], bool packed,
               u8* ws, size_t ws_bytes, bool timed = true)
{
    if (!c || n == 0 || n_chunks < 0 || !x.p[0] || !x.p[1] || !y.p[0] || !y.p[1]) return MPC_EINVAL;
    MPC_TRY(check_material(mat));
    MsbGeom g{};
    ReluWs w;
    if (packed) {
        for (int i = 0; i < 2; ++i)
            if (((uintptr_t)mat->and_a.p[i] | (uintptr_t)mat->and_b.p[i] | (uintptr_t)mat->and_c.p[i]) & 15) return MPC_EINVAL;
        g = msb_geom(n);
        w = carve_relu_msb(ws, ws_bytes, n, g);
    } else {
        w = carve_relu(ws, ws_bytes, n);
    }
    if (!w.ok) return MPC_ENOMEM;
    MPC_TRY(lane_join(c));
    const int pi = timed ? prof_begin(c, MPC_PROF_RELU, c->s[0]) : -1;
    ReluParty pp[2];
    for (int i = 0; i < 2; ++i)
        fill_party(pp[i], i, x.p[i], mat, w, y.p[i], s_bit ? s_bit[i] : nullptr, s_arith ? s_arith[i] : nullptr, n);
    MPC_TRY(relu_run(c, pp, n, n_chunks, packed ? &g : nullptr));
    if (pi >= 0) {      // the region ends when both parties' last kernels are done
        MPC_TRY(chain(c, c->s[1], c->s[0]));
        prof_end(c, MPC_PROF_RELU, pi, c->s[0]);
    }
    return MPC_OK;
}

size_t maxpool_ws(int B, int H, int W, int C, bool packed)
{
    if (B <= 0 || H <= 0 || W <= 0 || C <= 0 || (H & 1) || (W & 1)) return 0;
    const size_t n_out = (size_t)B * (H / 2) * (W / 2) * C;
    // per party: d1 (2 n_out), r1 (2 n_out), v (n_out), d2 (n_out); then the ReLU's own scratch
    const size_t relu = packed ? carve_relu_msb(nullptr, 0, 2 * n_out, msb_geom(2 * n_out)).bytes
                               : carve_relu(nullptr, 0, 2 * n_out).bytes;
    return 2 * (align_up(2 * n_out * 8) * 2 + align_up(n_out * 8) * 2) + relu;
}

int maxpool_entry(mpc_ctx* c, mpc_cshare x, const mpc_relu_material* mat1, const mpc_relu_material* mat2,
                  mpc_share y, int B, int H, int W, int C, int n_chunks, bool packed,
                  uint64_t* const s1[2] = nullptr, uint64_t* const s2[2] = nullptr)
{
    if (!c || B <= 0 || H <= 0 || W <= 0 || C <= 0 || (H & 1) || (W & 1) || n_chunks < 0 ||
        !x.p[0] || !x.p[1] || !y.p[0] || !y.p[1])
        return MPC_EINVAL;
    MPC_TRY(check_material(mat1));
    MPC_TRY(check_material(mat2));
    if (packed)
        for (const mpc_relu_material* m : { mat1, mat2 })
            for (int i = 0; i < 2; ++i)
                if (((uintptr_t)m->and_a.p[i] | (uintptr_t)m->and_b.p[i] | (uintptr_t)m->and_c.p[i]) & 15) return MPC_EINVAL;
    const size_t n_out = (size_t)B * (H / 2) * (W / 2) * C;
    WsAlloc wa(c->ws, c->ws_bytes);
    u64 *d1[2], *r1[2], *v[2], *d2[2];
    for (int i = 0; i < 2; ++i) {
        d1[i] = wa.take<u64>(2 * n_out); r1[i] = wa.take<u64>(2 * n_out);
        v[i] = wa.take<u64>(n_out); d2[i] = wa.take<u64>(n_out);
    }
    if (!wa.ok) return MPC_ENOMEM;
    const MsbGeom g1 = msb_geom(2 * n_out), g2 = msb_geom(n_out);
    // both conversions use the scratch carved for the larger one
    const ReluWs w1 = packed ? carve_relu_msb(c->ws + wa.off, c->ws_bytes - wa.off, 2 * n_out, g1)
                             : carve_relu(c->ws + wa.off, c->ws_bytes - wa.off, 2 * n_out);
    const ReluWs w2 = packed ? carve_relu_msb(c->ws + wa.off, c->ws_bytes - wa.off, n_out, g2) : w1;
    if (!w1.ok || !w2.ok) return MPC_ENOMEM;
    MPC_TRY(lane_join(c));
    const dim3 grid(grid_for(n_out)), block(kThreads);
    ReluParty pp[2];
    // first tournament level: max(p00, p01) and max(p10, p11)
    for (int i = 0; i < 2; ++i) {
        hipLaunchKernelGGL(k_pool_l1, grid, block, 0, c->s[i], x.p[i], d1[i], B, H, W, C);
        MPC_HIP(c, hipGetLastError());
        fill_party(pp[i], i, d1[i], mat1, w1, r1[i], nullptr, s1 ? s1[i] : nullptr, 2 * n_out);
    }
    MPC_TRY(lane_join(c));
    MPC_TRY(relu_run(c, pp, 2 * n_out, n_chunks, packed ? &g1 : nullptr));
    // second level: max of the two winners; out = v + ReLU(u - v)
    for (int i = 0; i < 2; ++i) {
        hipLaunchKernelGGL(k_pool_l2, grid, block, 0, c->s[i], x.p[i], r1[i], v[i], d2[i], B, H, W, C);
        MPC_HIP(c, hipGetLastError());
        fill_party(pp[i], i, d2[i], mat2, w2, y.p[i], nullptr, s2 ? s2[i] : nullptr, n_out);
    }
    MPC_TRY(lane_join(c));
    MPC_TRY(relu_run(c, pp, n_out, n_chunks, packed ? &g2 : nullptr));
    for (int i = 0; i < 2; ++i)
        MPC_TRY(launch_add(c, c->s[i], y.p[i], v[i], y.p[i], n_out));
    return MPC_OK;
}

// ---- the entry point that allocates nothing ------------------------------------
// Its rounds exchange and carry state through a fixed array in the code object
// instead of the caller's workspace.  Layout and size are those carve_relu gives
// for kStaticMaxN elements: per party 2 x [4][n] words (sent / received), 2 x n
// bytes, G, P (n words each), n bytes; then the two alternate receive buffers.
constexpr size_t kStaticMaxN = 65536;
constexpr size_t static_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }
constexpr size_t kStaticBytes =
    2 * (2 * static_up(32 * kStaticMaxN) + 2 * static_up(kStaticMaxN) + 2 * static_up(8 * kStaticMaxN) + static_up(kStaticMaxN)) +
    2 * static_up(32 * kStaticMaxN);
static __device__ __align__(256) unsigned char scratch[kStaticBytes];

// Device address of `scratch` per device (every device holds its own copy of the
// array); resolved once per device by relu_static_setup, with that device current.
constexpr int kMaxDevices = 16;
std::atomic<u8*> g_scratch_ptr[kMaxDevices];

}  // namespace

int relu_static_setup(mpc_ctx* c)
{
    if (c->device < 0 || c->device >= kMaxDevices) return MPC_OK;     // mpc_relu_static reports it
    if (g_scratch_ptr[c->device].load(std::memory_order_acquire)) return MPC_OK;
    void* p = nullptr;
    MPC_HIP(c, hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p || ((uintptr_t)p % kAlign) != 0) return MPC_EHIP;
    g_scratch_ptr[c->device].store((u8*)p, std::memory_order_release);
    return MPC_OK;
}

extern "C" {

int mpc_ctx_set_relu_chunk(mpc_ctx* c, size_t whole_word_elems, size_t packed_elems)
{
    if (!c || (whole_word_elems && whole_word_elems < 1024) || (packed_elems && packed_elems < 1024)) return MPC_EINVAL;
    c->relu_chunk[0] = whole_word_elems; c->relu_chunk[1] = packed_elems;
    return MPC_OK;
}


size_t mpc_relu_static_max_n(void) { return kStaticMaxN; }

int mpc_relu_static(mpc_ctx* c, mpc_cshare x, const mpc_relu_material* mat, mpc_share y, size_t n, int n_chunks,
                    uint8_t* const s_bit[2], uint64_t* const s_arith[2])
{
    if (!c || c->device < 0 || c->device >= kMaxDevices) return MPC_EINVAL;
    if (n > kStaticMaxN) return MPC_ERANGE;
    u8* ws = g_scratch_ptr[c->device].load(std::memory_order_acquire);
    if (!ws) return MPC_EINVAL;          // the context was not created on this device by mpc_ctx_create
    // no timing region: its events would be created here
    return relu_entry(c, x, mat, y, n, n_chunks, s_bit, s_arith, false, ws, kStaticBytes, false);
}

size_t mpc_relu_workspace_bytes(size_t n)
{
    if (n == 0) return 0;
    return carve_relu(nullptr, 0, n).bytes;
}

size_t mpc_relu_msb_workspace_bytes(size_t n)
{
    if (n == 0) return 0;
    return carve_relu_msb(nullptr, 0, n, msb_geom(n)).bytes;
}

size_t mpc_relu_packed_words(size_t n) { return n ? msb_geom(n).words_triples : 0; }

size_t mpc_maxpool_workspace_bytes(int B, int H, int W, int C) { return maxpool_ws(B, H, W, C, false); }
size_t mpc_maxpool_msb_workspace_bytes(int B, int H, int W, int C) { return maxpool_ws(B, H, W, C, true); }

int mpc_relu(mpc_ctx* c, mpc_cshare x, const mpc_relu_material* mat, mpc_share y, size_t n, int n_chunks,
             uint8_t* const s_bit[2], uint64_t* const s_arith[2])
{
    if (!c) return MPC_EINVAL;
    return relu_entry(c, x, mat, y, n, n_chunks, s_bit, s_arith, false, c->ws, c->ws_bytes);
}

int mpc_relu_msb(mpc_ctx* c, mpc_cshare x, const mpc_relu_material* mat, mpc_share y, size_t n, int n_chunks,
                 uint8_t* const s_bit[2], uint64_t* const s_arith[2])
{
    if (!c) return MPC_EINVAL;
    return relu_entry(c, x, mat, y, n, n_chunks, s_bit, s_arith, true, c->ws, c->ws_bytes);
}

int mpc_relu_pack_triples(mpc_ctx* c, mpc_cshare words, mpc_share packed, size_t n)
{
    if (!c || n == 0 || !words.p[0] || !words.p[1] || !packed.p[0] || !packed.p[1]) return MPC_EINVAL;
    const MsbGeom g = msb_geom(n);
    MPC_TRY(lane_join(c));
    for (int i = 0; i < 2; ++i) {
        hipLaunchKernelGGL(k_pack_triples, dim3(grid_for(n), MPC_N_AND_TRIPLES), dim3(kThreads), 0, c->s[i],
                           words.p[i], packed.p[i], g);
        MPC_HIP(c, hipGetLastError());
    }
    return MPC_OK;
}

int mpc_maxpool2x2(mpc_ctx* c, mpc_cshare x, const mpc_relu_material* mat1, const mpc_relu_material* mat2,
                   mpc_share y, int B, int H, int W, int C, int n_chunks)
{
    return maxpool_entry(c, x, mat1, mat2, y, B, H, W, C, n_chunks, false);
}

int mpc_maxpool2x2_msb(mpc_ctx* c, mpc_cshare x, const mpc_relu_material* mat1, const mpc_relu_material* mat2,
                       mpc_share y, int B, int H, int W, int C, int n_chunks)
{
    return maxpool_entry(c, x, mat1, mat2, y, B, H, W, C, n_chunks, true);
}

int mpc_maxpool2x2_signs(mpc_ctx* c, mpc_cshare x, const mpc_relu_material* mat1, const mpc_relu_material* mat2,
                         mpc_share y, uint64_t* const s1[2], uint64_t* const s2[2],
                         int B, int H, int W, int C, int n_chunks, int packed)
{
    if (!s1 || !s2 || !s1[0] || !s1[1] || !s2[0] || !s2[1]) return MPC_EINVAL;
    return maxpool_entry(c, x, mat1, mat2, y, B, H, W, C, n_chunks, packed != 0, s1, s2);
}

}  // extern "C"
