// Three simulated parties (Alg. 1 and Alg. 2 are stated for N parties; Sec. 3.3,
// Sec. 5.6): opening, the masked rescale, the secure ReLU whose A2B step adds
// three binary-shared words (carry-save step, then the Kogge-Stone network) on
// whole words or on the sign's carry chain only, 2x2 max-pool by composition,
// and the element-wise steps of the backward pass (Sec. 5.3).  Everything here
// is bound by HBM; all launches go to the lane's first stream, one launch per
// step for all three parties (blockIdx.y = party), and every exchange is a copy
// kernel or, on request, a remote store by the stage kernel itself.  The linear
// layers with three parties live in linear.hip.
#include "common.h"
#include "msb_pack.h"

namespace {

constexpr int kT = 256;

inline unsigned grid3(size_t items)
{
    size_t blocks = (items + kT - 1) / kT;
    if (blocks > 256 * 16) blocks = 256 * 16;
    if (blocks < 1) blocks = 1;
    return (unsigned)blocks;
}

// ------------------------------------------------------------------- rescale
struct Trunc3Args {
    u64* z[3]; const u64* r[3]; const u64* rt[3];
    u64* send[2];            // z_i + r_i of parties 1 and 2
    const u64* recv[2];      // the same words as party 0 received them
    size_t n; int bits;
};

// parties 1, 2 (blockIdx.y + 1): mask the share with the party's share of r
__global__ __launch_bounds__(kT) void k3_trunc_mask(Trunc3Args q)
{
    const int p = blockIdx.y + 1;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < q.n; i += stride)
        q.send[p - 1][i] = q.z[p][i] + q.r[p][i];
}

// party 0 opens m = z + r + 2^62 and shifts; parties 1, 2 negate their share of r >> bits
__global__ __launch_bounds__(kT) void k3_trunc_finish(Trunc3Args q)
{
    const int p = blockIdx.y;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < q.n; i += stride) {
        if (p == 0) {
            const u64 m = q.z[0][i] + q.r[0][i] + q.recv[0][i] + q.recv[1][i] + ((u64)1 << 62);
            q.z[0][i] = (m >> q.bits) - ((u64)1 << (62 - q.bits)) - q.rt[0][i];
        } else {
            q.z[p][i] = (u64)0 - q.rt[p][i];
        }
    }
}

// ---------------------------------------------------------------------- ReLU
struct Relu3Party {
    const u64 *x, *r0, *r1;              // input share; A2B masks sent to party+1 / party+2
    const u64 *ta, *tb, *tc;             // [13][n] AND triples
    const u8* rb; const u64* ra;         // B2A
    const u64 *ma, *mb, *mc;             // select
    u64* y; u8* s_bit; u64* s_arith;     // outputs (the last two optional)
    // workspace
    u64* wrecv[2];                       // this party's shares of the words of party+1 / party+2
    u64 *S, *Wd, *P, *G; u8* p63;        // carried state (from level 0 on, P lives in the opened AND of each round)
    u64* send;                           // [4][n] masked words of the current round
    u64* recv[2];                        // [4][n] the same from party+1 / party+2
    u8* vsend; u8* vrecv[2];             // B2A round (one byte per element)
    // exchange by remote store: the stage kernel also writes its masked words where the two peers
    // read them (put[s]: the receive buffer recv[s] of party (me + 2 - s) mod 3); recv_alt is the second
    // set of receive buffers, alternating with recv from stage to stage in that mode
    u64* put[2]; u64* putL[2]; u8* vput[2]; u64* recv_alt[2];
    // sign-only chain: per level a [4][pw] block of masked packed words, and the G bits a level keeps
    u64* sendL; u64* recvL[2]; u64* gsel;
};
struct Relu3Args { Relu3Party p[3]; size_t n; size_t tn; };   // n: elements of this call or chunk; tn: row stride of the [13][tn] triples

// Words are processed one per thread, or two per thread with 16-byte accesses
// when the element count is even and every array is 16-byte aligned.
typedef u64 u64v2 __attribute__((ext_vector_type(2)));
typedef u8 u8v2 __attribute__((ext_vector_type(2)));
// four words per thread: two 16-byte accesses each (the type asks for no more than 16-byte alignment)
typedef u64 u64v4 __attribute__((ext_vector_type(4), aligned(16)));
typedef u8 u8v4 __attribute__((ext_vector_type(4)));
template <typename T> struct ByteOf { typedef u8 type; };
template <> struct ByteOf<u64v2> { typedef u8v2 type; };
template <> struct ByteOf<u64v4> { typedef u8v4 type; };
__device__ __forceinline__ u8 to_bytes(u64 v) { return (u8)v; }
__device__ __forceinline__ u8v2 to_bytes(u64v2 v) { return __builtin_convertvector(v, u8v2); }
__device__ __forceinline__ u8v4 to_bytes(u64v4 v) { return __builtin_convertvector(v, u8v4); }
__device__ __forceinline__ u64 to_words(u8 v) { return v; }
__device__ __forceinline__ u64v2 to_words(u8v2 v) { return __builtin_convertvector(v, u64v2); }
__device__ __forceinline__ u64v4 to_words(u8v4 v) { return __builtin_convertvector(v, u64v4); }

// One Beaver AND gate finished: own and received masked operands -> this party's share.
template <typename T>
__device__ __forceinline__ T and_finish(int party, T d, T g, T a, T b, T c)
{
    T t = c ^ (d & b) ^ (g & a);
    if (party == 0) t ^= d & g;
    return t;
}

// STAGE 0      : A2B words in place -> carry-save sum S, majority AND masked
//       1      : majority finished -> K = C << 1, P = S ^ K, G = S & K masked
//       2      : G finished -> level 0 masked
//       3 .. 7 : level L = STAGE - 3 finished -> level L + 1 masked
//       8      : level 5 finished -> sign share, B2A masked
//       9      : B2A finished -> m = 1 - s, select masked
//       10     : select finished -> y
template <int STAGE, typename T, bool PUT>
__global__ __launch_bounds__(kT) void k3_relu(Relu3Args q)
{
    typedef typename ByteOf<T>::type B;
    const int party = blockIdx.y;
    const Relu3Party& p = q.p[party];
    const size_t n = q.n;                                    // words per row
    const size_t units = n / (sizeof(T) / sizeof(u64));
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    // row r of a [rows][n] workspace array / of a [13][tn] triple array, as units
    const size_t tn = q.tn;
    auto in = [n](const u64* base, int r) { return reinterpret_cast<const T*>(base + (size_t)r * n); };
    auto out = [n](u64* base, int r) { return reinterpret_cast<T*>(base + (size_t)r * n); };
    auto tr = [tn](const u64* base, int r) { return reinterpret_cast<const T*>(base + (size_t)r * tn); };
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < units; i += stride) {
        // row k of this round's masked words: into the own send buffer and, by remote store, to both peers.
        // From stage 2 on a party that stores to its peers keeps no copy for itself: the stage that opens the
        // words forms the party's own ones again from the state it carries and the triples it reads anyway
        // (the level stages then also carry P).
        constexpr bool kReform = PUT && STAGE >= 3;          // the round before left no own copy
        auto send = [&](int k, T v) {
            if constexpr (!(PUT && STAGE >= 2)) out(p.send, k)[i] = v;
            if constexpr (PUT) { out(p.put[0], k)[i] = v; out(p.put[1], k)[i] = v; }
        };
        // masked words of the previous round, opened
        T o[4] = {};
        constexpr int kOpen = (STAGE == 0 || STAGE >= 9) ? 0 : (STAGE >= 3 && STAGE <= 7) ? 4 : 2;
        if constexpr (kReform && kOpen > 0) {
            // stages 3..8 finish level L = STAGE - 3, masked by the stage before from its (P, G) with shift 2^L
            constexpr int L = STAGE - 3, tg = 2 + 2 * L, tp = 3 + 2 * L;
            const T Pp = in(p.P, 0)[i], Gp = in(p.G, 0)[i];
            o[0] = Pp ^ tr(p.ta, tg)[i];  o[1] = (Gp << (1 << L)) ^ tr(p.tb, tg)[i];
            if constexpr (kOpen == 4) { o[2] = Pp ^ tr(p.ta, tp)[i];  o[3] = (Pp << (1 << L)) ^ tr(p.tb, tp)[i]; }
#pragma unroll
            for (int k = 0; k < kOpen; ++k) o[k] ^= in(p.recv[0], k)[i] ^ in(p.recv[1], k)[i];
        } else {
#pragma unroll
            for (int k = 0; k < kOpen; ++k) o[k] = in(p.send, k)[i] ^ in(p.recv[0], k)[i] ^ in(p.recv[1], k)[i];
        }

        if constexpr (STAGE == 0) {
            const T own = in(p.x, 0)[i] ^ in(p.r0, 0)[i] ^ in(p.r1, 0)[i];
            // party's shares of the words x_0, x_1, x_2
            const T w1 = in(p.wrecv[0], 0)[i], w2 = in(p.wrecv[1], 0)[i];      // words of party+1, party+2
            const T U = party == 0 ? own : party == 1 ? w2 : w1;
            const T V = party == 1 ? own : party == 2 ? w2 : w1;
            const T W = party == 2 ? own : party == 0 ? w2 : w1;
            out(p.S, 0)[i] = U ^ V ^ W; out(p.Wd, 0)[i] = W;
            send(0, (U ^ W) ^ tr(p.ta, 0)[i]);
            send(1, (V ^ W) ^ tr(p.tb, 0)[i]);
        } else if constexpr (STAGE == 1) {
            const T Tm = and_finish<T>(party, o[0], o[1], tr(p.ta, 0)[i], tr(p.tb, 0)[i], tr(p.tc, 0)[i]);
            const T S = in(p.S, 0)[i];
            const T K = (Tm ^ in(p.Wd, 0)[i]) << 1;
            const T P = S ^ K;
            out(p.P, 0)[i] = P; reinterpret_cast<B*>(p.p63)[i] = to_bytes(P >> 63);
            send(0, S ^ tr(p.ta, 1)[i]);
            send(1, K ^ tr(p.tb, 1)[i]);
        } else if constexpr (STAGE == 2) {
            const T G = and_finish<T>(party, o[0], o[1], tr(p.ta, 1)[i], tr(p.tb, 1)[i], tr(p.tc, 1)[i]);
            const T P = in(p.P, 0)[i];
            out(p.G, 0)[i] = G;
            send(0, P ^ tr(p.ta, 2)[i]);  send(1, (G << 1) ^ tr(p.tb, 2)[i]);
            send(2, P ^ tr(p.ta, 3)[i]);  send(3, (P << 1) ^ tr(p.tb, 3)[i]);
        } else if constexpr (STAGE >= 3 && STAGE <= 7) {
            constexpr int L = STAGE - 3;                 // level being finished
            constexpr int tg = 2 + 2 * L, tp = 3 + 2 * L;
            const T T1 = and_finish<T>(party, o[0], o[1], tr(p.ta, tg)[i], tr(p.tb, tg)[i], tr(p.tc, tg)[i]);
            const T P = and_finish<T>(party, o[2], o[3], tr(p.ta, tp)[i], tr(p.tb, tp)[i], tr(p.tc, tp)[i]);
            const T G = in(p.G, 0)[i] ^ T1;
            out(p.G, 0)[i] = G;
            if constexpr (PUT) out(p.P, 0)[i] = P;       // the next stage forms this party's masked words from (P, G)
            constexpr int d = 2 << L;                    // shift of level L + 1
            constexpr int ng = tg + 2, np = tp + 2;
            send(0, P ^ tr(p.ta, ng)[i]);  send(1, (G << d) ^ tr(p.tb, ng)[i]);
            if constexpr (L + 1 < 5) {                   // the last level needs no P update
                send(2, P ^ tr(p.ta, np)[i]);  send(3, (P << d) ^ tr(p.tb, np)[i]);
            }
        } else if constexpr (STAGE == 8) {
            const T T1 = and_finish<T>(party, o[0], o[1], tr(p.ta, 12)[i], tr(p.tb, 12)[i], tr(p.tc, 12)[i]);
            const T G = in(p.G, 0)[i] ^ T1;
            const B s = reinterpret_cast<const B*>(p.p63)[i] ^ to_bytes((G >> 62) & 1);
            if (p.s_bit) reinterpret_cast<B*>(p.s_bit)[i] = s;
            const B masked = s ^ reinterpret_cast<const B*>(p.rb)[i];
            reinterpret_cast<B*>(p.vsend)[i] = masked;
            if constexpr (PUT) { reinterpret_cast<B*>(p.vput[0])[i] = masked; reinterpret_cast<B*>(p.vput[1])[i] = masked; }
        } else if constexpr (STAGE == 9) {
            const T v = to_words(reinterpret_cast<const B*>(p.vsend)[i] ^ reinterpret_cast<const B*>(p.vrecv[0])[i] ^
                                 reinterpret_cast<const B*>(p.vrecv[1])[i]);
            const T ra = in(p.ra, 0)[i];
            T sa = ra - 2 * v * ra;
            if (party == 0) sa += v;
            if (p.s_arith) out(p.s_arith, 0)[i] = sa;
            const T m = (party == 0 ? (u64)1 : (u64)0) - sa;
            send(0, in(p.x, 0)[i] - in(p.ma, 0)[i]);
            send(1, m - in(p.mb, 0)[i]);
        } else {
            // additive opening of the select product's masked operands
            const T mb = in(p.mb, 0)[i], ma = in(p.ma, 0)[i];
            T e_own, f_own;
            if constexpr (PUT) {                         // formed again from x, ra and the opened sign byte
                const T v = to_words(reinterpret_cast<const B*>(p.vsend)[i] ^ reinterpret_cast<const B*>(p.vrecv[0])[i] ^
                                     reinterpret_cast<const B*>(p.vrecv[1])[i]);
                const T ra = in(p.ra, 0)[i];
                T sa = ra - 2 * v * ra;
                if (party == 0) sa += v;
                e_own = in(p.x, 0)[i] - ma;
                f_own = ((party == 0 ? (u64)1 : (u64)0) - sa) - mb;
            } else {
                e_own = in(p.send, 0)[i]; f_own = in(p.send, 1)[i];
            }
            const T e = e_own + in(p.recv[0], 0)[i] + in(p.recv[1], 0)[i];
            const T f = f_own + in(p.recv[0], 1)[i] + in(p.recv[1], 1)[i];
            T yv = in(p.mc, 0)[i] + e * mb + ma * f;
            if (party == 0) yv += e * f;
            out(p.y, 0)[i] = yv;
        }
    }
}

// Words per thread: 16-byte accesses need an even element count (rows of the [k][n] arrays stay aligned)
// and aligned arrays; four words per thread a multiple of four and 4-byte aligned byte arrays.
int relu3_vectorisable(const Relu3Args& q)
{
    if ((q.n | q.tn) & 1) return 1;
    uintptr_t w = 0, b = 0;
    for (int i = 0; i < 3; ++i) {
        const Relu3Party& p = q.p[i];
        for (const void* ptr : { (const void*)p.x, (const void*)p.r0, (const void*)p.r1, (const void*)p.ta, (const void*)p.tb,
                                 (const void*)p.tc, (const void*)p.ra, (const void*)p.ma, (const void*)p.mb, (const void*)p.mc,
                                 (const void*)p.y, (const void*)p.s_arith })
            w |= (uintptr_t)ptr;
        b |= (uintptr_t)p.rb | (uintptr_t)p.s_bit;
    }
    if ((w & 15) != 0 || (b & 1) != 0) return 1;
    return ((q.n | q.tn) & 3) == 0 && (b & 3) == 0 ? 4 : 2;
}

// ---- the sign-only chain (mpc_relu3_msb) ---------------------------------------------
// Stages 0 and 1 (carry-save step, P and the operands of G = S & K) run on whole words as
// above.  From there the Kogge-Stone levels keep only the positions bit 63 depends on
// (msb_pack.h): level l works on n / 2^(l+1) packed words, its triples arrive packed the
// same way, and the exchanges shrink by the same factor.  Triple layout of one party's
// and_a / and_b / and_c: rows 0 and 1 (majority, G) whole words, padded to a multiple of
// four; then triples 2 .. 12 packed for their level.
struct Msb3Geom {
    size_t n;
    size_t pw[6];       // words of level l's packed arrays
    size_t toff[13];    // offset of triple t inside a packed and_a / and_b / and_c buffer
    size_t loff[6];     // offset of level l's [4][pw] block inside sendL / recvL
    size_t goff[6];     // offset of level l's words inside gsel
    size_t words_triples, words_blocks, words_gsel;
};

Msb3Geom msb3_geom(size_t n)
{
    Msb3Geom g{};
    g.n = n;
    size_t lo = 0, go = 0;
    for (int l = 0; l < 6; ++l) {
        g.pw[l] = msb_level_words(n, l);
        g.loff[l] = lo; lo += 4 * g.pw[l];
        g.goff[l] = go; go += g.pw[l];
    }
    const size_t n4 = (n + 3) / 4 * 4;
    g.toff[0] = 0; g.toff[1] = n4;
    size_t to = 2 * n4;
    for (int t = 2; t < 13; ++t) { g.toff[t] = to; to += g.pw[(t - 2) / 2]; }
    g.words_triples = to; g.words_blocks = lo; g.words_gsel = go;
    return g;
}

struct W4 { u64 v[4]; };
// four consecutive words: two 16-byte loads when `vec`, else one by one with words past `n` read as zero
__device__ __forceinline__ W4 ld4(const u64* p, size_t i, size_t n, bool vec)
{
    W4 r;
    if (vec) {
        const u64v2 a = *reinterpret_cast<const u64v2*>(p + i), b = *reinterpret_cast<const u64v2*>(p + i + 2);
        r.v[0] = a.x; r.v[1] = a.y; r.v[2] = b.x; r.v[3] = b.y;
    } else {
#pragma unroll
        for (int k = 0; k < 4; ++k) r.v[k] = i + k < n ? p[i + k] : 0;
    }
    return r;
}
__device__ __forceinline__ W4 xor3(const W4& a, const W4& b, const W4& c)
{
    W4 r;
#pragma unroll
    for (int k = 0; k < 4; ++k) r.v[k] = a.v[k] ^ b.v[k] ^ c.v[k];
    return r;
}
__device__ __forceinline__ void st2(u64* p, size_t j, u64 a, u64 b)
{
    u64v2 t; t.x = a; t.y = b;
    *reinterpret_cast<u64v2*>(p + j) = t;        // packed arrays are 16-byte aligned and padded to four words
}

// Packed level LEVEL: finish the ANDs of the round before (G = S & K on whole words for
// LEVEL 0, else level LEVEL - 1 on packed words) for the four input words behind two
// output words, regroup, and mask this level's operands.  `vec0`: the whole-word arrays
// of LEVEL 0 allow 16-byte loads (n a multiple of four, aligned bases).
template <int LEVEL, bool PUT>
__global__ __launch_bounds__(kT) void k3_plevel(Relu3Args q, Msb3Geom g, bool vec0)
{
    const int party = blockIdx.y;
    const Relu3Party& p = q.p[party];
    constexpr int d = 1 << LEVEL, s = 2 * d;
    constexpr u64 A = sel_mask(LEVEL), Bm = low_mask(LEVEL);
    const size_t n = q.n;
    const size_t whi = (n + s - 1) >> (LEVEL + 1);                   // output words that hold an element
    const size_t stride = (size_t)gridDim.x * blockDim.x * 2;
    for (size_t j = ((size_t)blockIdx.x * blockDim.x + threadIdx.x) * 2; j < whi; j += stride) {
        W4 G, P;
        if constexpr (LEVEL == 0) {
            const size_t e = 2 * j;
            const bool v = vec0 && e + 3 < n;
            const W4 od = xor3(ld4(p.send, e, n, v), ld4(p.recv[0], e, n, v), ld4(p.recv[1], e, n, v));
            const W4 og = xor3(ld4(p.send + n, e, n, v), ld4(p.recv[0] + n, e, n, v), ld4(p.recv[1] + n, e, n, v));
            const W4 a = ld4(p.ta + g.toff[1], e, n, v), b = ld4(p.tb + g.toff[1], e, n, v), c = ld4(p.tc + g.toff[1], e, n, v);
            P = ld4(p.P, e, n, v);
#pragma unroll
            for (int k = 0; k < 4; ++k) G.v[k] = and_finish<u64>(party, od.v[k], og.v[k], a.v[k], b.v[k], c.v[k]);
        } else {
            constexpr int lq = LEVEL - 1, tg = 2 + 2 * lq, tp = 3 + 2 * lq;
            const size_t w = 2 * j, pq = g.pw[lq];
            const u64* sp = p.sendL + g.loff[lq];
            const u64* r0 = p.recvL[0] + g.loff[lq]; const u64* r1 = p.recvL[1] + g.loff[lq];
            const W4 gs = ld4(p.gsel + g.goff[lq], w, pq, true);
            const W4 d1 = xor3(ld4(sp, w, pq, true), ld4(r0, w, pq, true), ld4(r1, w, pq, true));
            const W4 g1 = xor3(ld4(sp + pq, w, pq, true), ld4(r0 + pq, w, pq, true), ld4(r1 + pq, w, pq, true));
            const W4 d2 = xor3(ld4(sp + 2 * pq, w, pq, true), ld4(r0 + 2 * pq, w, pq, true), ld4(r1 + 2 * pq, w, pq, true));
            const W4 g2 = xor3(ld4(sp + 3 * pq, w, pq, true), ld4(r0 + 3 * pq, w, pq, true), ld4(r1 + 3 * pq, w, pq, true));
            const W4 a1 = ld4(p.ta + g.toff[tg], w, pq, true), b1 = ld4(p.tb + g.toff[tg], w, pq, true), c1 = ld4(p.tc + g.toff[tg], w, pq, true);
            const W4 a2 = ld4(p.ta + g.toff[tp], w, pq, true), b2 = ld4(p.tb + g.toff[tp], w, pq, true), c2 = ld4(p.tc + g.toff[tp], w, pq, true);
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                G.v[k] = gs.v[k] ^ and_finish<u64>(party, d1.v[k], g1.v[k], a1.v[k], b1.v[k], c1.v[k]);
                P.v[k] = and_finish<u64>(party, d2.v[k], g2.v[k], a2.v[k], b2.v[k], c2.v[k]);
            }
        }
        u64 X[2], Gk[2], Y1[2], Y2[2];
#pragma unroll
        for (int k = 0; k < 2; ++k) {
            const u64 Glo = G.v[2 * k], Ghi = G.v[2 * k + 1], Plo = P.v[2 * k], Phi = P.v[2 * k + 1];
            X[k] = (Plo & A) | rotl<d>(Phi & A);                 // P[p]
            Gk[k] = (Glo & A) | rotl<d>(Ghi & A);                // G[p]
            Y1[k] = rotl<d>(Glo & Bm) | rotl<2 * d>(Ghi & Bm);   // G[p - d] moved to p
            Y2[k] = rotl<d>(Plo & Bm) | rotl<2 * d>(Phi & Bm);   // P[p - d] moved to p
        }
        constexpr int ng = 2 + 2 * LEVEL, np = 3 + 2 * LEVEL;
        const size_t pl = g.pw[LEVEL];
        u64* so = p.sendL + g.loff[LEVEL];
        const u64v2 na1 = *reinterpret_cast<const u64v2*>(p.ta + g.toff[ng] + j), nb1 = *reinterpret_cast<const u64v2*>(p.tb + g.toff[ng] + j);
        // row r of this level's block: own send buffer and, by remote store, both peers' receive blocks
        auto send2 = [&](int r, u64 a, u64 b) {
            st2(so + (size_t)r * pl, j, a, b);
            if constexpr (PUT) {
                st2(p.putL[0] + g.loff[LEVEL] + (size_t)r * pl, j, a, b);
                st2(p.putL[1] + g.loff[LEVEL] + (size_t)r * pl, j, a, b);
            }
        };
        send2(0, X[0] ^ na1.x, X[1] ^ na1.y);
        send2(1, Y1[0] ^ nb1.x, Y1[1] ^ nb1.y);
        if constexpr (LEVEL < 5) {                               // the last level needs no P update
            const u64v2 na2 = *reinterpret_cast<const u64v2*>(p.ta + g.toff[np] + j), nb2 = *reinterpret_cast<const u64v2*>(p.tb + g.toff[np] + j);
            send2(2, X[0] ^ na2.x, X[1] ^ na2.y);
            send2(3, Y2[0] ^ nb2.x, Y2[1] ^ nb2.y);
        }
        st2(p.gsel + g.goff[LEVEL], j, Gk[0], Gk[1]);
    }
}

// Packed sign stage: finish level 5; element i's carry into bit 63 sits at bit
// (62 + i) mod 64 of word i / 64.  Then the B2A mask as in stage 8 of the whole-word chain.
template <int V, bool PUT>
__global__ __launch_bounds__(kT) void k3_psign(Relu3Args q, Msb3Geom g)
{
    const int party = blockIdx.y;
    const Relu3Party& p = q.p[party];
    const size_t p5 = g.pw[5];
    const u64* sp = p.sendL + g.loff[5];
    const u64* r0 = p.recvL[0] + g.loff[5]; const u64* r1 = p.recvL[1] + g.loff[5];
    const u64* gs = p.gsel + g.goff[5];
    const u64 *a = p.ta + g.toff[12], *b = p.tb + g.toff[12], *c = p.tc + g.toff[12];
    const size_t stride = (size_t)gridDim.x * blockDim.x * V;
    // V consecutive elements (V = 4: n is a multiple of four, so they share word i / 64 and one 4-byte access each)
    for (size_t i = ((size_t)blockIdx.x * blockDim.x + threadIdx.x) * V; i < q.n; i += stride) {
        const size_t w = i >> 6;
        const u64 Gw = gs[w] ^ and_finish<u64>(party, sp[w] ^ r0[w] ^ r1[w], sp[p5 + w] ^ r0[p5 + w] ^ r1[p5 + w], a[w], b[w], c[w]);
        if constexpr (V == 4) {
            const uint32_t top = *reinterpret_cast<const uint32_t*>(p.p63 + i), rb = *reinterpret_cast<const uint32_t*>(p.rb + i);
            uint32_t carry = 0;
#pragma unroll
            for (int k = 0; k < 4; ++k) carry |= (uint32_t)((Gw >> ((62 + i + k) & 63)) & 1) << (8 * k);
            const uint32_t sb = top ^ carry;
            if (p.s_bit) *reinterpret_cast<uint32_t*>(p.s_bit + i) = sb;
            *reinterpret_cast<uint32_t*>(p.vsend + i) = sb ^ rb;
            if constexpr (PUT) { *reinterpret_cast<uint32_t*>(p.vput[0] + i) = sb ^ rb; *reinterpret_cast<uint32_t*>(p.vput[1] + i) = sb ^ rb; }
        } else {
            const u8 sb = (u8)(p.p63[i] ^ (u8)((Gw >> ((62 + i) & 63)) & 1));
            if (p.s_bit) p.s_bit[i] = sb;
            const u8 masked = (u8)(sb ^ p.rb[i]);
            p.vsend[i] = masked;
            if constexpr (PUT) { p.vput[0][i] = masked; p.vput[1][i] = masked; }
        }
    }
}

// Offline helper: triple-major [13][n] words -> the packed layout (blockIdx.y = triple).
__global__ __launch_bounds__(kT) void k3_pack_triples(const u64* __restrict__ in, u64* __restrict__ out, Msb3Geom g)
{
    const int t = blockIdx.y;
    const size_t n = g.n, stride = (size_t)gridDim.x * blockDim.x;
    const size_t first = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t < 2) {
        const size_t n4 = g.toff[1];
        for (size_t i = first; i < n4; i += stride) out[g.toff[t] + i] = i < n ? in[(size_t)t * n + i] : 0;
        return;
    }
    const int l = (t - 2) / 2, s = 2 << l;
    const u64 m = msb_mask(l);
    for (size_t j = first; j < g.pw[l]; j += stride) {
        u64 acc = 0;
        for (int k = 0; k < s; ++k) {
            const size_t e = j * s + k;
            if (e < n) { const u64 v = in[(size_t)t * n + e] & m; acc |= k ? (v << k) | (v >> (64 - k)) : v; }
        }
        out[g.toff[t] + j] = acc;
    }
}

// Arguments of one stage launch when the exchange is by remote store: the launch with index k
// reads the receive-buffer set (k - 1) & 1 and stores into the peers' set k & 1, so that no party
// stores where a peer's same launch still reads.  Party i's words land in recv[s] of party
// (i + 2 - s) mod 3, the buffer that party reads for its peer number s.
Relu3Args put_args(const Relu3Args& q, int k)
{
    Relu3Args a = q;
    for (int i = 0; i < 3; ++i)
        for (int s = 0; s < 2; ++s) {
            const int peer = (i + 2 - s) % 3;
            u64* const rd[2] = { q.p[i].recv[s], q.p[i].recv_alt[s] };
            u64* const wr[2] = { q.p[peer].recv[s], q.p[peer].recv_alt[s] };
            a.p[i].recv[s] = rd[(k + 1) & 1];
            a.p[i].put[s] = wr[k & 1];
            a.p[i].putL[s] = q.p[peer].recvL[s];
            a.p[i].vput[s] = q.p[peer].vrecv[s];
        }
    return a;
}

template <int STAGE, bool PUT>
int launch_stage_t(mpc_ctx* c, hipStream_t st, const Relu3Args& q, int vec)
{
    if (vec == 4)      hipLaunchKernelGGL((k3_relu<STAGE, u64v4, PUT>), dim3(grid3(q.n / 4), 3), dim3(kT), 0, st, q);
    else if (vec == 2) hipLaunchKernelGGL((k3_relu<STAGE, u64v2, PUT>), dim3(grid3(q.n / 2), 3), dim3(kT), 0, st, q);
    else               hipLaunchKernelGGL((k3_relu<STAGE, u64, PUT>), dim3(grid3(q.n), 3), dim3(kT), 0, st, q);
    MPC_HIP(c, hipGetLastError());
    return MPC_OK;
}

int exchange_words(mpc_ctx* c, hipStream_t st, const Relu3Args& q, int words);
int exchange_bytes(mpc_ctx* c, hipStream_t st, const Relu3Args& q);

// Stage STAGE for all three parties, then the exchange of what it sends: `rows` word rows,
// bytes for rows < 0, nothing for rows == 0.  By remote store the kernel itself delivers.
template <int STAGE>
int launch_stage(mpc_ctx* c, hipStream_t st, const Relu3Args& q, int vec, int rows)
{
    if (c->exchange_put) return launch_stage_t<STAGE, true>(c, st, put_args(q, STAGE), vec);
    MPC_TRY((launch_stage_t<STAGE, false>(c, st, q, vec)));
    if (rows == 0) return MPC_OK;
    return rows > 0 ? exchange_words(c, st, q, rows) : exchange_bytes(c, st, q);
}

// every party's first `words` rows of its send buffer go to both peers
int exchange_words(mpc_ctx* c, hipStream_t st, const Relu3Args& q, int words)
{
    CopySeg cp[6]; int k = 0;
    for (int i = 0; i < 3; ++i)
        for (int s = 0; s < 2; ++s)
            cp[k++] = CopySeg{ (const u8*)q.p[(i + 1 + s) % 3].send, (u8*)q.p[i].recv[s],
                               (size_t)words * q.n * sizeof(u64), 0 };
    return launch_copy_multi(c, st, cp, 6);
}

// the masked sign bytes of every party go to both peers
int exchange_bytes(mpc_ctx* c, hipStream_t st, const Relu3Args& q)
{
    CopySeg cp[6]; int k = 0;
    for (int i = 0; i < 3; ++i)
        for (int s = 0; s < 2; ++s)
            cp[k++] = CopySeg{ q.p[(i + 1 + s) % 3].vsend, q.p[i].vrecv[s], q.n, 0 };
    return launch_copy_multi(c, st, cp, 6);
}

size_t relu3_ws(u8* base, size_t cap, size_t n, Relu3Args* q, bool* ok)
{
    WsAlloc w(base, cap);
    for (int i = 0; i < 3; ++i) {
        Relu3Party& p = q->p[i];
        p.wrecv[0] = w.take<u64>(n); p.wrecv[1] = w.take<u64>(n);
        p.S = w.take<u64>(n); p.Wd = w.take<u64>(n); p.P = w.take<u64>(n); p.G = w.take<u64>(n);
        p.send = w.take<u64>(4 * n); p.recv[0] = w.take<u64>(4 * n); p.recv[1] = w.take<u64>(4 * n);
        p.p63 = w.take<u8>(n); p.vsend = w.take<u8>(n); p.vrecv[0] = w.take<u8>(n); p.vrecv[1] = w.take<u8>(n);
    }
    for (int i = 0; i < 3; ++i)      // only touched by the remote-store exchange
        for (int s = 0; s < 2; ++s) q->p[i].recv_alt[s] = w.take<u64>(4 * n);
    if (ok) *ok = w.ok;
    return w.off;
}

int check_material3(const mpc_relu3_material* m)
{
    if (!m) return MPC_EINVAL;
    for (int i = 0; i < 3; ++i)
        if (!m->r0.p[i] || !m->r1.p[i] || !m->and_a.p[i] || !m->and_b.p[i] || !m->and_c.p[i] || !m->rb[i] ||
            !m->ra.p[i] || !m->ma.p[i] || !m->mb.p[i] || !m->mc.p[i])
            return MPC_EINVAL;
    return MPC_OK;
}

void fill3(Relu3Args& q, const u64* const x[3], const mpc_relu3_material* m, u64* const y[3],
           uint8_t* const s_bit[3], uint64_t* const s_arith[3], size_t n)
{
    for (int i = 0; i < 3; ++i) {
        Relu3Party& p = q.p[i];
        p.x = x[i]; p.r0 = m->r0.p[i]; p.r1 = m->r1.p[i];
        p.ta = m->and_a.p[i]; p.tb = m->and_b.p[i]; p.tc = m->and_c.p[i];
        p.rb = m->rb[i]; p.ra = m->ra.p[i]; p.ma = m->ma.p[i]; p.mb = m->mb.p[i]; p.mc = m->mc.p[i];
        p.y = y[i];
        p.s_bit = s_bit ? s_bit[i] : nullptr; p.s_arith = s_arith ? s_arith[i] : nullptr;
    }
    q.n = n; q.tn = n;
}

// The whole chain for one chunk on one stream: A2B distribution, 11 stage kernels, 10 word exchanges, one byte exchange.
int relu3_chunk(mpc_ctx* c, hipStream_t st, const Relu3Args& q)
{
    const size_t n = q.n;
    const int vec = relu3_vectorisable(q);
    // Alg. 2: party j sends the mask r1_j to party j+2 and r0_j to party j+1, i.e. party i
    // receives its share of word i+1 (that party's r1) and of word i+2 (that party's r0)
    {
        CopySeg cp[6];
        for (int i = 0; i < 3; ++i) {
            cp[2 * i] = CopySeg{ (const u8*)q.p[(i + 1) % 3].r1, (u8*)q.p[i].wrecv[0], n * sizeof(u64), 0 };
            cp[2 * i + 1] = CopySeg{ (const u8*)q.p[(i + 2) % 3].r0, (u8*)q.p[i].wrecv[1], n * sizeof(u64), 0 };
        }
        MPC_TRY(launch_copy_multi(c, st, cp, 6));
    }
    MPC_TRY(launch_stage<0>(c, st, q, vec, 2));
    MPC_TRY(launch_stage<1>(c, st, q, vec, 2));
    MPC_TRY(launch_stage<2>(c, st, q, vec, 4));
    MPC_TRY(launch_stage<3>(c, st, q, vec, 4));
    MPC_TRY(launch_stage<4>(c, st, q, vec, 4));
    MPC_TRY(launch_stage<5>(c, st, q, vec, 4));
    MPC_TRY(launch_stage<6>(c, st, q, vec, 4));
    MPC_TRY(launch_stage<7>(c, st, q, vec, 2));
    MPC_TRY(launch_stage<8>(c, st, q, vec, -1));
    MPC_TRY(launch_stage<9>(c, st, q, vec, 2));
    MPC_TRY(launch_stage<10>(c, st, q, vec, 0));
    return MPC_OK;
}

// Chunks of about 2^19 elements: the exchanged words and the carried state of a chunk (about 0.35 GB
// for the three parties) then stay close to the last-level cache from stage to stage, and only the
// offline material streams from DRAM.  Chunk boundaries are multiples of four, so wide accesses stay possible.
// A lane whose conversion chunk has been set (mpc_ctx_set_relu_chunk: lanes that convert at the same time share the
// cache) takes half of that, a three-party element carrying about twice the exchanged words of a two-party one; a
// smaller chunk never needs more workspace than the default one the workspace queries assume.
constexpr size_t kChunk3 = (size_t)1 << 19;
inline size_t relu3_chunk_of(const mpc_ctx* c)
{
    if (!c || !c->relu_chunk[0]) return kChunk3;
    const size_t half = c->relu_chunk[0] / 2;
    return half < 4096 ? 4096 : half > kChunk3 ? kChunk3 : half;
}
inline int relu3_chunks(size_t n, size_t chunk = kChunk3) { return n <= chunk + chunk / 2 ? 1 : (int)((n + chunk - 1) / chunk); }
inline size_t relu3_chunk_cap(size_t n, size_t chunk = kChunk3)          // largest chunk of relu3_run's split
{
    const int k = relu3_chunks(n, chunk);
    return k == 1 ? n : ((n + k - 1) / k + 3) & ~(size_t)3;
}

// q: caller arrays of the whole call (q.n = q.tn = n), workspace carved for relu3_chunk_cap(n) elements.
int relu3_run(mpc_ctx* c, hipStream_t st, const Relu3Args& q)
{
    const size_t n = q.n;
    const int k = relu3_chunks(n, relu3_chunk_of(c));
    if (k == 1) return relu3_chunk(c, st, q);
    const size_t cap = relu3_chunk_cap(n, relu3_chunk_of(c));
    for (size_t lo = 0; lo < n; lo += cap) {
        Relu3Args ch = q;
        ch.n = n - lo < cap ? n - lo : cap;
        for (int i = 0; i < 3; ++i) {
            Relu3Party& p = ch.p[i];
            p.x += lo; p.r0 += lo; p.r1 += lo; p.ta += lo; p.tb += lo; p.tc += lo;
            p.rb += lo; p.ra += lo; p.ma += lo; p.mb += lo; p.mc += lo; p.y += lo;
            if (p.s_bit) p.s_bit += lo;
            if (p.s_arith) p.s_arith += lo;
        }
        MPC_TRY(relu3_chunk(c, st, ch));
    }
    return MPC_OK;
}

// ---- sign-only chain: workspace and the chain on one stream (no chunks: a call's packed
// state is a third of the whole-word chain's, and its levels halve from round to round)
size_t relu3_msb_ws(u8* base, size_t cap, size_t n, const Msb3Geom& g, Relu3Args* q, bool* ok)
{
    WsAlloc w(base, cap);
    for (int i = 0; i < 3; ++i) {
        Relu3Party& p = q->p[i];
        p.wrecv[0] = w.take<u64>(n); p.wrecv[1] = w.take<u64>(n);
        p.S = w.take<u64>(n); p.Wd = w.take<u64>(n); p.P = w.take<u64>(n); p.G = nullptr;
        p.send = w.take<u64>(2 * n); p.recv[0] = w.take<u64>(2 * n); p.recv[1] = w.take<u64>(2 * n);
        p.p63 = w.take<u8>(n); p.vsend = w.take<u8>(n); p.vrecv[0] = w.take<u8>(n); p.vrecv[1] = w.take<u8>(n);
        p.sendL = w.take<u64>(g.words_blocks); p.recvL[0] = w.take<u64>(g.words_blocks); p.recvL[1] = w.take<u64>(g.words_blocks);
        p.gsel = w.take<u64>(g.words_gsel);
    }
    for (int i = 0; i < 3; ++i)      // only touched by the remote-store exchange
        for (int s = 0; s < 2; ++s) q->p[i].recv_alt[s] = w.take<u64>(2 * n);
    if (ok) *ok = w.ok;
    return w.off;
}

template <int LEVEL>
int launch_plevel(mpc_ctx* c, hipStream_t st, const Relu3Args& q, const Msb3Geom& g, bool vec0)
{
    const size_t words = (q.n + ((size_t)2 << LEVEL) - 1) >> (LEVEL + 1);
    const dim3 grid(grid3((words + 1) / 2), 3), block(kT);
    if (c->exchange_put) {
        // level 0 reads the whole words stage 1 delivered (launch index 2); the levels' own blocks do not alternate
        hipLaunchKernelGGL((k3_plevel<LEVEL, true>), grid, block, 0, st, put_args(q, 2), g, vec0);
        MPC_HIP(c, hipGetLastError());
        return MPC_OK;
    }
    hipLaunchKernelGGL((k3_plevel<LEVEL, false>), grid, block, 0, st, q, g, vec0);
    MPC_HIP(c, hipGetLastError());
    // this level's masked packed words go to both peers
    const size_t len = (size_t)(LEVEL < 5 ? 4 : 2) * g.pw[LEVEL] * sizeof(u64);
    CopySeg cp[6]; int k = 0;
    for (int i = 0; i < 3; ++i)
        for (int s = 0; s < 2; ++s)
            cp[k++] = CopySeg{ (const u8*)(q.p[(i + 1 + s) % 3].sendL + g.loff[LEVEL]), (u8*)(q.p[i].recvL[s] + g.loff[LEVEL]), len, 0 };
    return launch_copy_multi(c, st, cp, 6);
}

// q: caller arrays (q.n = n, q.tn = the packed buffers' whole-word row stride), workspace from relu3_msb_ws
int relu3_msb_run(mpc_ctx* c, hipStream_t st, const Relu3Args& q, const Msb3Geom& g)
{
    const size_t n = q.n;
    const int vec = relu3_vectorisable(q);
    const bool vec0 = vec >= 2 && n % 4 == 0;
    {
        CopySeg cp[6];
        for (int i = 0; i < 3; ++i) {
            cp[2 * i] = CopySeg{ (const u8*)q.p[(i + 1) % 3].r1, (u8*)q.p[i].wrecv[0], n * sizeof(u64), 0 };
            cp[2 * i + 1] = CopySeg{ (const u8*)q.p[(i + 2) % 3].r0, (u8*)q.p[i].wrecv[1], n * sizeof(u64), 0 };
        }
        MPC_TRY(launch_copy_multi(c, st, cp, 6));
    }
    MPC_TRY(launch_stage<0>(c, st, q, vec, 2));
    MPC_TRY(launch_stage<1>(c, st, q, vec, 2));
    MPC_TRY(launch_plevel<0>(c, st, q, g, vec0));
    MPC_TRY(launch_plevel<1>(c, st, q, g, vec0));
    MPC_TRY(launch_plevel<2>(c, st, q, g, vec0));
    MPC_TRY(launch_plevel<3>(c, st, q, g, vec0));
    MPC_TRY(launch_plevel<4>(c, st, q, g, vec0));
    MPC_TRY(launch_plevel<5>(c, st, q, g, vec0));
    const dim3 sgrid(vec == 4 ? grid3(n / 4) : grid3(n), 3), block(kT);
    if (c->exchange_put) {
        const Relu3Args a = put_args(q, 8);
        if (vec == 4) hipLaunchKernelGGL((k3_psign<4, true>), sgrid, block, 0, st, a, g);
        else          hipLaunchKernelGGL((k3_psign<1, true>), sgrid, block, 0, st, a, g);
        MPC_HIP(c, hipGetLastError());
    } else {
        if (vec == 4) hipLaunchKernelGGL((k3_psign<4, false>), sgrid, block, 0, st, q, g);
        else          hipLaunchKernelGGL((k3_psign<1, false>), sgrid, block, 0, st, q, g);
        MPC_HIP(c, hipGetLastError());
        MPC_TRY(exchange_bytes(c, st, q));
    }
    MPC_TRY(launch_stage<9>(c, st, q, vec, 2));
    MPC_TRY(launch_stage<10>(c, st, q, vec, 0));
    return MPC_OK;
}

// the packed buffers must allow 16-byte accesses
int check_packed3(const mpc_relu3_material* m)
{
    for (int i = 0; i < 3; ++i)
        if (((uintptr_t)m->and_a.p[i] | (uintptr_t)m->and_b.p[i] | (uintptr_t)m->and_c.p[i]) & 15) return MPC_EINVAL;
    return MPC_OK;
}

// ---- 2x2 max-pool by max(p, q) = q + ReLU(p - q): the local steps (blockIdx.y = party)
struct Pool3Args { const u64* x[3]; u64* d1[3]; const u64* r1[3]; u64* v[3]; u64* d2[3]; u64* y[3]; int B, H, W, C; };

// STEP 0: d1[2o] = p00 - p01, d1[2o+1] = p10 - p11;  1: u = p01 + r1[2o], v = p11 + r1[2o+1], d2 = u - v;  2: y += v
template <int STEP>
__global__ __launch_bounds__(kT) void k3_pool(Pool3Args q)
{
    const int p = blockIdx.y;
    const int Ho = q.H / 2, Wo = q.W / 2;
    const size_t n_out = (size_t)q.B * Ho * Wo * q.C;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t o = (size_t)blockIdx.x * blockDim.x + threadIdx.x; o < n_out; o += stride) {
        if constexpr (STEP == 2) { q.y[p][o] += q.v[p][o]; continue; }
        const int ch = (int)(o % q.C); size_t t = o / q.C;
        const int wo = (int)(t % Wo); t /= Wo;
        const int ho = (int)(t % Ho); const int b = (int)(t / Ho);
        const size_t base = (((size_t)b * q.H + 2 * ho) * q.W + 2 * wo) * q.C + ch;
        const size_t dw = q.C, dh = (size_t)q.W * q.C;
        const u64* x = q.x[p];
        if constexpr (STEP == 0) {
            q.d1[p][2 * o] = x[base] - x[base + dw];
            q.d1[p][2 * o + 1] = x[base + dh] - x[base + dh + dw];
        } else {
            const u64 u = x[base + dw] + q.r1[p][2 * o];
            const u64 v = x[base + dh + dw] + q.r1[p][2 * o + 1];
            q.v[p][o] = v;
            q.d2[p][o] = u - v;
        }
    }
}

// ---- element-wise Alg. 1 with three parties, and the backward steps built on it ------
struct Mul3Args {
    const u64 *x[3], *y[3], *a[3], *b[3], *c[3];
    u64 *se[3], *sf[3];                       // own masked words
    const u64 *re[3][2], *rf[3][2];           // the masked words of party+1 / party+2
    u64* z[3];
    size_t n; int mask_from_sign;             // mask_from_sign: y holds sign shares s, the factor is 1 - s
};

__global__ __launch_bounds__(kT) void k3_mul_mask(Mul3Args q)
{
    const int i = blockIdx.y;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t k = (size_t)blockIdx.x * blockDim.x + threadIdx.x; k < q.n; k += stride) {
        u64 y = q.y[i][k];
        if (q.mask_from_sign) y = (i == 0 ? (u64)1 : (u64)0) - y;
        q.se[i][k] = q.x[i][k] - q.a[i][k];
        q.sf[i][k] = y - q.b[i][k];
    }
}

__global__ __launch_bounds__(kT) void k3_mul_finish(Mul3Args q)
{
    const int i = blockIdx.y;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t k = (size_t)blockIdx.x * blockDim.x + threadIdx.x; k < q.n; k += stride) {
        const u64 e = q.se[i][k] + q.re[i][0][k] + q.re[i][1][k], f = q.sf[i][k] + q.rf[i][0][k] + q.rf[i][1][k];
        u64 z = q.c[i][k] + e * q.b[i][k] + q.a[i][k] * f;
        if (i == 0) z += e * f;
        q.z[i][k] = z;
    }
}

size_t mul3_ws_bytes(size_t n) { return 18 * align_up(n * sizeof(u64)); }

// z = x * y element by element (no rescale); ws_off: bytes of the workspace the caller keeps for itself
int mul3_run(mpc_ctx* c, hipStream_t st, const u64* const x[3], const u64* const y[3], const u64* const a[3],
             const u64* const b[3], const u64* const cc[3], u64* const z[3], size_t n, int mask_from_sign, size_t ws_off)
{
    if (ws_off > c->ws_bytes) return MPC_ENOMEM;
    WsAlloc ws(c->ws ? c->ws + ws_off : nullptr, c->ws_bytes - ws_off);
    Mul3Args q{};
    u64 *re[3][2], *rf[3][2];
    for (int i = 0; i < 3; ++i) {
        q.se[i] = ws.take<u64>(n); q.sf[i] = ws.take<u64>(n);
        for (int k = 0; k < 2; ++k) { re[i][k] = ws.take<u64>(n); rf[i][k] = ws.take<u64>(n); q.re[i][k] = re[i][k]; q.rf[i][k] = rf[i][k]; }
    }
    if (!ws.ok) return MPC_ENOMEM;
    for (int i = 0; i < 3; ++i) { q.x[i] = x[i]; q.y[i] = y[i]; q.a[i] = a[i]; q.b[i] = b[i]; q.c[i] = cc[i]; q.z[i] = z[i]; }
    q.n = n; q.mask_from_sign = mask_from_sign;
    hipLaunchKernelGGL(k3_mul_mask, dim3(grid3(n), 3), dim3(kT), 0, st, q);
    MPC_HIP(c, hipGetLastError());
    // both masked words of every party go to both peers: two launches of six copies
    for (int what = 0; what < 2; ++what) {
        CopySeg cp[6]; int k = 0;
        for (int i = 0; i < 3; ++i)
            for (int sdx = 0; sdx < 2; ++sdx) {
                const int from = (i + 1 + sdx) % 3;
                cp[k++] = CopySeg{ (const u8*)(what ? q.sf[from] : q.se[from]), (u8*)(what ? rf[i][sdx] : re[i][sdx]), n * sizeof(u64), 0 };
            }
        MPC_TRY(launch_copy_multi(c, st, cp, 6));
    }
    hipLaunchKernelGGL(k3_mul_finish, dim3(grid3(n), 3), dim3(kT), 0, st, q);
    MPC_HIP(c, hipGetLastError());
    return MPC_OK;
}

// max-pool backward: the local steps around its two element-wise products (blockIdx.y = party)
struct PoolBwd3Args { const u64* g[3]; const u64* gu[3]; u64* pairs[3]; const u64* prod[3]; u64* gx[3]; size_t n_out; int B, H, W, C; };

// STEP 0: grad_v = g - grad_u, the pair (grad_u, grad_v) interleaved as the first tournament level stored its pairs
// STEP 1: after P = pairs * mask1 the four window positions receive P[2o], grad_u - P[2o], P[2o+1], grad_v - P[2o+1]
template <int STEP>
__global__ __launch_bounds__(kT) void k3_poolbwd(PoolBwd3Args q)
{
    const int i = blockIdx.y;
    const int Ho = q.H / 2, Wo = q.W / 2;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t o = (size_t)blockIdx.x * blockDim.x + threadIdx.x; o < q.n_out; o += stride) {
        if constexpr (STEP == 0) {
            const u64 gu = q.gu[i][o];
            q.pairs[i][2 * o] = gu;
            q.pairs[i][2 * o + 1] = q.g[i][o] - gu;
        } else {
            const int ch = (int)(o % q.C); size_t t = o / q.C;
            const int wo = (int)(t % Wo); t /= Wo;
            const int ho = (int)(t % Ho); const int b = (int)(t / Ho);
            const size_t base = (((size_t)b * q.H + 2 * ho) * q.W + 2 * wo) * q.C + ch;
            const size_t dw = q.C, dh = (size_t)q.W * q.C;
            const u64 p0 = q.prod[i][2 * o], p1 = q.prod[i][2 * o + 1];
            const u64 gu = q.pairs[i][2 * o], gv = q.pairs[i][2 * o + 1];
            u64* gx = q.gx[i];
            gx[base] = p0;            gx[base + dw] = gu - p0;
            gx[base + dh] = p1;       gx[base + dh + dw] = gv - p1;
        }
    }
}

template <int STEP>
int launch_pool(mpc_ctx* c, hipStream_t st, const Pool3Args& q, size_t n_out)
{
    hipLaunchKernelGGL(k3_pool<STEP>, dim3(grid3(n_out), 3), dim3(kT), 0, st, q);
    MPC_HIP(c, hipGetLastError());
    return MPC_OK;
}

}  // namespace

extern "C" {

int mpc_open3(mpc_ctx* c, mpc_cshare3 s, uint64_t* out, size_t n)
{
    if (!c || !s.p[0] || !s.p[1] || !s.p[2] || !out || n == 0) return MPC_EINVAL;
    WsAlloc ws(c->ws, c->ws_bytes);
    u64* r[3];
    for (int i = 0; i < 3; ++i) r[i] = ws.take<u64>(n);
    if (!ws.ok) return MPC_ENOMEM;
    hipStream_t st = c->s[0];
    MPC_TRY(lane_join(c));
    CopySeg cp[3];
    for (int i = 0; i < 3; ++i) cp[i] = CopySeg{ (const u8*)s.p[i], (u8*)r[i], n * sizeof(u64), 0 };
    MPC_TRY(launch_copy_multi(c, st, cp, 3));
    MPC_TRY(launch_sum3(c, st, r[0], r[1], r[2], out, n));
    return lane_fanout(c);
}

size_t mpc_truncate3_workspace_bytes(size_t n)
{
    return n == 0 ? 0 : 4 * align_up(n * sizeof(u64));
}

int mpc_truncate3(mpc_ctx* c, mpc_share3 z, mpc_cshare3 r, mpc_cshare3 rt, size_t n, int bits)
{
    if (!c || n == 0 || bits < 0 || bits > 62) return MPC_EINVAL;
    for (int i = 0; i < 3; ++i) if (!z.p[i] || !r.p[i] || !rt.p[i]) return MPC_EINVAL;
    WsAlloc ws(c->ws, c->ws_bytes);
    Trunc3Args q{};
    u64* recv[2];
    for (int k = 0; k < 2; ++k) { q.send[k] = ws.take<u64>(n); recv[k] = ws.take<u64>(n); q.recv[k] = recv[k]; }
    if (!ws.ok) return MPC_ENOMEM;
    for (int i = 0; i < 3; ++i) { q.z[i] = z.p[i]; q.r[i] = r.p[i]; q.rt[i] = rt.p[i]; }
    q.n = n; q.bits = bits;
    hipStream_t st = c->s[0];
    MPC_TRY(lane_join(c));
    hipLaunchKernelGGL(k3_trunc_mask, dim3(grid3(n), 2), dim3(kT), 0, st, q);
    MPC_HIP(c, hipGetLastError());
    CopySeg cp[2];
    for (int k = 0; k < 2; ++k) cp[k] = CopySeg{ (const u8*)q.send[k], (u8*)recv[k], n * sizeof(u64), 0 };
    MPC_TRY(launch_copy_multi(c, st, cp, 2));
    hipLaunchKernelGGL(k3_trunc_finish, dim3(grid3(n), 3), dim3(kT), 0, st, q);
    MPC_HIP(c, hipGetLastError());
    return lane_fanout(c);
}

size_t mpc_relu3_workspace_bytes(size_t n)
{
    if (n == 0) return 0;
    Relu3Args q{};
    return relu3_ws(nullptr, 0, relu3_chunk_cap(n), &q, nullptr);
}

int mpc_relu3(mpc_ctx* c, mpc_cshare3 x, const mpc_relu3_material* m, mpc_share3 y, size_t n,
              uint8_t* const s_bit[3], uint64_t* const s_arith[3])
{
    if (!c || n == 0) return MPC_EINVAL;
    if (n > ((size_t)1 << 40)) return MPC_ERANGE;
    MPC_TRY(check_material3(m));
    for (int i = 0; i < 3; ++i) if (!x.p[i] || !y.p[i]) return MPC_EINVAL;
    Relu3Args q{};
    bool ok = false;
    relu3_ws(c->ws, c->ws_bytes, relu3_chunk_cap(n, relu3_chunk_of(c)), &q, &ok);
    if (!ok) return MPC_ENOMEM;
    fill3(q, x.p, m, y.p, s_bit, s_arith, n);
    hipStream_t st = c->s[0];
    MPC_TRY(lane_join(c));
    const int pi = prof_begin(c, MPC_PROF_RELU, st);
    MPC_TRY(relu3_run(c, st, q));
    prof_end(c, MPC_PROF_RELU, pi, st);
    return lane_fanout(c);
}

size_t mpc_relu3_packed_words(size_t n) { return n ? msb3_geom(n).words_triples : 0; }

size_t mpc_relu3_msb_workspace_bytes(size_t n)
{
    if (n == 0) return 0;
    Relu3Args q{};
    return relu3_msb_ws(nullptr, 0, n, msb3_geom(n), &q, nullptr);
}

int mpc_relu3_pack_triples(mpc_ctx* c, mpc_cshare3 words, mpc_share3 packed, size_t n)
{
    if (!c || n == 0) return MPC_EINVAL;
    if (n > ((size_t)1 << 40)) return MPC_ERANGE;
    for (int i = 0; i < 3; ++i) if (!words.p[i] || !packed.p[i]) return MPC_EINVAL;
    const Msb3Geom g = msb3_geom(n);
    hipStream_t st = c->s[0];
    MPC_TRY(lane_join(c));
    for (int i = 0; i < 3; ++i) {
        hipLaunchKernelGGL(k3_pack_triples, dim3(grid3(n), 13), dim3(kT), 0, st, words.p[i], packed.p[i], g);
        MPC_HIP(c, hipGetLastError());
    }
    return lane_fanout(c);
}

int mpc_relu3_msb(mpc_ctx* c, mpc_cshare3 x, const mpc_relu3_material* m, mpc_share3 y, size_t n,
                  uint8_t* const s_bit[3], uint64_t* const s_arith[3])
{
    if (!c || n == 0) return MPC_EINVAL;
    if (n > ((size_t)1 << 40)) return MPC_ERANGE;
    MPC_TRY(check_material3(m));
    MPC_TRY(check_packed3(m));
    for (int i = 0; i < 3; ++i) if (!x.p[i] || !y.p[i]) return MPC_EINVAL;
    const Msb3Geom g = msb3_geom(n);
    Relu3Args q{};
    bool ok = false;
    relu3_msb_ws(c->ws, c->ws_bytes, n, g, &q, &ok);
    if (!ok) return MPC_ENOMEM;
    fill3(q, x.p, m, y.p, s_bit, s_arith, n);
    q.tn = g.toff[1];
    hipStream_t st = c->s[0];
    MPC_TRY(lane_join(c));
    const int pi = prof_begin(c, MPC_PROF_RELU, st);
    MPC_TRY(relu3_msb_run(c, st, q, g));
    prof_end(c, MPC_PROF_RELU, pi, st);
    return lane_fanout(c);
}

static size_t maxpool3_ws(int B, int H, int W, int C, bool packed)
{
    if (B <= 0 || H <= 0 || W <= 0 || C <= 0 || (H & 1) || (W & 1)) return 0;
    const size_t n_out = (size_t)B * (H / 2) * (W / 2) * C;
    // per party: d1 (2 n_out), r1 (2 n_out), v (n_out), d2 (n_out); then the larger conversion's scratch
    return 3 * (2 * align_up(2 * n_out * 8) + 2 * align_up(n_out * 8)) +
           (packed ? mpc_relu3_msb_workspace_bytes(2 * n_out) : mpc_relu3_workspace_bytes(2 * n_out));
}

size_t mpc_maxpool3_workspace_bytes(int B, int H, int W, int C) { return maxpool3_ws(B, H, W, C, false); }
size_t mpc_maxpool3_msb_workspace_bytes(int B, int H, int W, int C) { return maxpool3_ws(B, H, W, C, true); }

static int maxpool3_entry(mpc_ctx* c, mpc_cshare3 x, const mpc_relu3_material* mat1, const mpc_relu3_material* mat2,
                          mpc_share3 y, int B, int H, int W, int C, bool packed,
                          uint64_t* const s1[3] = nullptr, uint64_t* const s2[3] = nullptr)
{
    if (!c || B <= 0 || H <= 0 || W <= 0 || C <= 0 || (H & 1) || (W & 1)) return MPC_EINVAL;
    MPC_TRY(check_material3(mat1));
    MPC_TRY(check_material3(mat2));
    if (packed) { MPC_TRY(check_packed3(mat1)); MPC_TRY(check_packed3(mat2)); }
    for (int i = 0; i < 3; ++i) if (!x.p[i] || !y.p[i]) return MPC_EINVAL;
    const size_t n_out = (size_t)B * (H / 2) * (W / 2) * C;
    WsAlloc wa(c->ws, c->ws_bytes);
    Pool3Args pq{};
    u64* r1[3];
    for (int i = 0; i < 3; ++i) {
        pq.x[i] = x.p[i]; pq.y[i] = y.p[i];
        pq.d1[i] = wa.take<u64>(2 * n_out); r1[i] = wa.take<u64>(2 * n_out); pq.r1[i] = r1[i];
        pq.v[i] = wa.take<u64>(n_out); pq.d2[i] = wa.take<u64>(n_out);
    }
    pq.B = B; pq.H = H; pq.W = W; pq.C = C;
    if (!wa.ok) return MPC_ENOMEM;
    Relu3Args q1{}, q2{};
    bool ok1 = false, ok2 = false;
    const Msb3Geom g1 = msb3_geom(2 * n_out), g2 = msb3_geom(n_out);
    u8* rest = c->ws ? c->ws + wa.off : nullptr;
    const size_t room = c->ws_bytes - wa.off;
    if (packed) {
        relu3_msb_ws(rest, room, 2 * n_out, g1, &q1, &ok1);
        relu3_msb_ws(rest, room, n_out, g2, &q2, &ok2);                        // the second conversion reuses the scratch
    } else {
        relu3_ws(rest, room, relu3_chunk_cap(2 * n_out, relu3_chunk_of(c)), &q1, &ok1);
        relu3_ws(rest, room, relu3_chunk_cap(n_out, relu3_chunk_of(c)), &q2, &ok2);
    }
    if (!ok1 || !ok2) return MPC_ENOMEM;
    fill3(q1, pq.d1, mat1, r1, nullptr, s1, 2 * n_out);
    fill3(q2, pq.d2, mat2, y.p, nullptr, s2, n_out);
    if (packed) { q1.tn = g1.toff[1]; q2.tn = g2.toff[1]; }
    hipStream_t st = c->s[0];
    MPC_TRY(lane_join(c));
    MPC_TRY(launch_pool<0>(c, st, pq, n_out));       // first tournament level: max(p00, p01), max(p10, p11)
    MPC_TRY(packed ? relu3_msb_run(c, st, q1, g1) : relu3_run(c, st, q1));
    MPC_TRY(launch_pool<1>(c, st, pq, n_out));       // second level: the two winners
    MPC_TRY(packed ? relu3_msb_run(c, st, q2, g2) : relu3_run(c, st, q2));
    MPC_TRY(launch_pool<2>(c, st, pq, n_out));       // out = v + ReLU(u - v)
    return lane_fanout(c);
}

int mpc_maxpool3(mpc_ctx* c, mpc_cshare3 x, const mpc_relu3_material* mat1, const mpc_relu3_material* mat2,
                 mpc_share3 y, int B, int H, int W, int C)
{
    return maxpool3_entry(c, x, mat1, mat2, y, B, H, W, C, false);
}

int mpc_maxpool3_msb(mpc_ctx* c, mpc_cshare3 x, const mpc_relu3_material* mat1, const mpc_relu3_material* mat2,
                     mpc_share3 y, int B, int H, int W, int C)
{
    return maxpool3_entry(c, x, mat1, mat2, y, B, H, W, C, true);
}

int mpc_maxpool3_signs(mpc_ctx* c, mpc_cshare3 x, const mpc_relu3_material* mat1, const mpc_relu3_material* mat2,
                       mpc_share3 y, uint64_t* const s1[3], uint64_t* const s2[3],
                       int B, int H, int W, int C, int packed)
{
    if (!s1 || !s2) return MPC_EINVAL;
    for (int i = 0; i < 3; ++i) if (!s1[i] || !s2[i]) return MPC_EINVAL;
    return maxpool3_entry(c, x, mat1, mat2, y, B, H, W, C, packed != 0, s1, s2);
}

// local linear steps on three shares: out_i = x_i +/- y_i
static int linear3(mpc_ctx* c, mpc_cshare3 x, mpc_cshare3 y, mpc_share3 out, size_t n, bool subtract)
{
    if (!c || n == 0) return MPC_EINVAL;
    for (int i = 0; i < 3; ++i) if (!x.p[i] || !y.p[i] || !out.p[i]) return MPC_EINVAL;
    hipStream_t st = c->s[0];
    MPC_TRY(lane_join(c));
    for (int i = 0; i < 3; ++i)
        MPC_TRY(subtract ? launch_sub(c, st, x.p[i], y.p[i], out.p[i], n) : launch_add(c, st, x.p[i], y.p[i], out.p[i], n));
    return lane_fanout(c);
}

int mpc_add3(mpc_ctx* c, mpc_cshare3 x, mpc_cshare3 y, mpc_share3 out, size_t n) { return linear3(c, x, y, out, n, false); }
int mpc_sub3(mpc_ctx* c, mpc_cshare3 x, mpc_cshare3 y, mpc_share3 out, size_t n) { return linear3(c, x, y, out, n, true); }

size_t mpc_mul3_workspace_bytes(size_t n) { return n ? mul3_ws_bytes(n) : 0; }

int mpc_mul3(mpc_ctx* c, mpc_cshare3 x, mpc_cshare3 y, mpc_cshare3 a, mpc_cshare3 b, mpc_cshare3 cc, mpc_share3 z, size_t n)
{
    if (!c || n == 0) return MPC_EINVAL;
    for (int i = 0; i < 3; ++i) if (!x.p[i] || !y.p[i] || !a.p[i] || !b.p[i] || !cc.p[i] || !z.p[i]) return MPC_EINVAL;
    hipStream_t st = c->s[0];
    MPC_TRY(lane_join(c));
    MPC_TRY(mul3_run(c, st, x.p, y.p, a.p, b.p, cc.p, z.p, n, 0, 0));
    return lane_fanout(c);
}

int mpc_relu3_backward(mpc_ctx* c, mpc_cshare3 g, mpc_cshare3 s_arith, mpc_cshare3 a, mpc_cshare3 b, mpc_cshare3 cc,
                       mpc_share3 gx, size_t n)
{
    if (!c || n == 0) return MPC_EINVAL;
    for (int i = 0; i < 3; ++i) if (!g.p[i] || !s_arith.p[i] || !a.p[i] || !b.p[i] || !cc.p[i] || !gx.p[i]) return MPC_EINVAL;
    hipStream_t st = c->s[0];
    MPC_TRY(lane_join(c));
    MPC_TRY(mul3_run(c, st, g.p, s_arith.p, a.p, b.p, cc.p, gx.p, n, 1, 0));
    return lane_fanout(c);
}

size_t mpc_maxpool3_backward_workspace_bytes(int B, int H, int W, int C)
{
    if (B <= 0 || H <= 0 || W <= 0 || C <= 0 || (H & 1) || (W & 1)) return 0;
    const size_t n_out = (size_t)B * (H / 2) * (W / 2) * C;
    // per party grad_u (n_out), pairs and their product (2 n_out each); then the larger product's scratch
    return 3 * (align_up(n_out * 8) + 2 * align_up(2 * n_out * 8)) + mul3_ws_bytes(2 * n_out);
}

int mpc_maxpool3_backward(mpc_ctx* c, mpc_cshare3 g, mpc_cshare3 s1, mpc_cshare3 s2,
                          mpc_cshare3 a1, mpc_cshare3 b1, mpc_cshare3 c1,
                          mpc_cshare3 a2, mpc_cshare3 b2, mpc_cshare3 c2,
                          mpc_share3 gx, int B, int H, int W, int C)
{
    if (!c || B <= 0 || H <= 0 || W <= 0 || C <= 0 || (H & 1) || (W & 1)) return MPC_EINVAL;
    for (int i = 0; i < 3; ++i)
        if (!g.p[i] || !s1.p[i] || !s2.p[i] || !gx.p[i] || !a1.p[i] || !b1.p[i] || !c1.p[i] || !a2.p[i] || !b2.p[i] || !c2.p[i])
            return MPC_EINVAL;
    const size_t n_out = (size_t)B * (H / 2) * (W / 2) * C;
    WsAlloc ws(c->ws, c->ws_bytes);
    u64 *gu[3], *pairs[3], *prod[3];
    for (int i = 0; i < 3; ++i) { gu[i] = ws.take<u64>(n_out); pairs[i] = ws.take<u64>(2 * n_out); prod[i] = ws.take<u64>(2 * n_out); }
    if (!ws.ok) return MPC_ENOMEM;
    const size_t off = ws.off;
    hipStream_t st = c->s[0];
    MPC_TRY(lane_join(c));
    // grad_u = g * (1 - s2)
    MPC_TRY(mul3_run(c, st, g.p, s2.p, a2.p, b2.p, c2.p, gu, n_out, 1, off));
    PoolBwd3Args q{};
    for (int i = 0; i < 3; ++i) { q.g[i] = g.p[i]; q.gu[i] = gu[i]; q.pairs[i] = pairs[i]; q.prod[i] = prod[i]; q.gx[i] = gx.p[i]; }
    q.n_out = n_out; q.B = B; q.H = H; q.W = W; q.C = C;
    hipLaunchKernelGGL(k3_poolbwd<0>, dim3(grid3(n_out), 3), dim3(kT), 0, st, q);
    MPC_HIP(c, hipGetLastError());
    // (grad_p00, grad_p10) = (grad_u, grad_v) * (1 - s1)
    MPC_TRY(mul3_run(c, st, pairs, s1.p, a1.p, b1.p, c1.p, prod, 2 * n_out, 1, off));
    hipLaunchKernelGGL(k3_poolbwd<1>, dim3(grid3(n_out), 3), dim3(kT), 0, st, q);
    MPC_HIP(c, hipGetLastError());
    return lane_fanout(c);
}

}  // extern "C"
