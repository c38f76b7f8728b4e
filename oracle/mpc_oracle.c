/*
 * CPU oracle for the two-party semi-honest online phase of MPC-Pipe's secure
 * layer over the ring Z_2^64.
 *
 * THIS IS TEST INFRASTRUCTURE.  It is a plain, slow, direct statement of the
 * protocol: uint64_t wrap-around arithmetic, straight loops, no digit
 * decomposition, no tiling, no fusion.  It shares nothing with the GPU
 * library and must never be called from the product path.
 *
 * Conventions
 *   - every array is dense, row-major uint64_t in host memory;
 *   - "party 0" here is the paper's "Party #1", the one that adds the
 *     Delta*epsilon term (Alg. 1; Alg. 4);
 *   - `e` is the paper's Delta = X - A, `f` its epsilon = Y - B;
 *   - activations are NHWC, filters [KH][KW][Cin][Cout].
 *
 * What the paper fixes: Alg. 1 (Beaver multiplication), Eq. 3 (its conv form),
 * Alg. 2 (A2B), Sec. 4.2 / Eq. 4 / Alg. 4 (Beaver AND).  What it leaves open
 * (ring width, fixed-point scale, truncation, the adder's topology, B2A, the
 * ReLU formula) is stated next to each function below.
 */
#include <stdint.h>
#include <stddef.h>
#include <stdlib.h>
#include <string.h>

typedef uint64_t u64;
typedef uint8_t u8;

/* ---------------------------------------------------------------- ring ops */

/* Z[m][n] = sum_k L[m][k] * R[k][n]  (mod 2^64).  Plain definition. */
void orc_ring_matmul(const u64* L, const u64* R, u64* Z, int M, int K, int N)
{
#pragma omp parallel for schedule(static)
    for (int m = 0; m < M; ++m) {
        u64* z = Z + (size_t)m * N;
        for (int n = 0; n < N; ++n) z[n] = 0;
        for (int k = 0; k < K; ++k) {
            const u64 l = L[(size_t)m * K + k];
            const u64* r = R + (size_t)k * N;
            for (int n = 0; n < N; ++n) z[n] += l * r[n];
        }
    }
}

/* Direct convolution (cross-correlation, as in ML frameworks), zero padding:
 * z[b][ho][wo][co] = sum_{kh,kw,ci} x[b][ho*s+kh-p][wo*s+kw-p][ci] * w[kh][kw][ci][co]
 * Ho = (H + 2p - KH)/s + 1, Wo likewise.  Seven loops, nothing else. */
void orc_ring_conv2d(const u64* x, const u64* w, u64* z,
                     int B, int H, int W, int Cin, int Cout,
                     int KH, int KW, int pad, int stride)
{
    const int Ho = (H + 2 * pad - KH) / stride + 1;
    const int Wo = (W + 2 * pad - KW) / stride + 1;
#pragma omp parallel for collapse(2) schedule(static)
    for (int b = 0; b < B; ++b)
        for (int ho = 0; ho < Ho; ++ho)
            for (int wo = 0; wo < Wo; ++wo) {
                u64* zo = z + (((size_t)b * Ho + ho) * Wo + wo) * Cout;
                for (int co = 0; co < Cout; ++co) zo[co] = 0;
                for (int kh = 0; kh < KH; ++kh) {
                    const int hi = ho * stride + kh - pad;
                    if (hi < 0 || hi >= H) continue;
                    for (int kw = 0; kw < KW; ++kw) {
                        const int wi = wo * stride + kw - pad;
                        if (wi < 0 || wi >= W) continue;
                        const u64* xi = x + (((size_t)b * H + hi) * W + wi) * Cin;
                        const u64* wk = w + ((size_t)kh * KW + kw) * Cin * Cout;
                        for (int ci = 0; ci < Cin; ++ci) {
                            const u64 xv = xi[ci];
                            const u64* wr = wk + (size_t)ci * Cout;
                            for (int co = 0; co < Cout; ++co) zo[co] += xv * wr[co];
                        }
                    }
                }
            }
}

/* Gradients of that convolution, for the backward pass (Sec. 4.1 and 5.3:
 * the gradient w.r.t. the input is a convolution of the output gradients with
 * the weights, the gradient w.r.t. the weights one of the output gradients
 * with the stored activation).  Both are written as the transpose of the
 * forward sum: the same seven index ranges, the product accumulated into the
 * other operand's position.
 *   gx[b][hi][wi][ci]  = sum_{ho,wo,kh,kw,co : hi = ho*s+kh-p, wi = wo*s+kw-p} g[b][ho][wo][co] * w[kh][kw][ci][co]
 *   gw[kh][kw][ci][co] = sum_{b,ho,wo}  x[b][ho*s+kh-p][wo*s+kw-p][ci] * g[b][ho][wo][co]          */
void orc_ring_conv2d_grad_x(const u64* g, const u64* w, u64* gx,
                            int B, int H, int W, int Cin, int Cout,
                            int KH, int KW, int pad, int stride)
{
    const int Ho = (H + 2 * pad - KH) / stride + 1;
    const int Wo = (W + 2 * pad - KW) / stride + 1;
    memset(gx, 0, (size_t)B * H * W * Cin * sizeof(u64));
#pragma omp parallel for schedule(static)
    for (int b = 0; b < B; ++b)
        for (int ho = 0; ho < Ho; ++ho)
            for (int wo = 0; wo < Wo; ++wo) {
                const u64* go = g + (((size_t)b * Ho + ho) * Wo + wo) * Cout;
                for (int kh = 0; kh < KH; ++kh) {
                    const int hi = ho * stride + kh - pad;
                    if (hi < 0 || hi >= H) continue;
                    for (int kw = 0; kw < KW; ++kw) {
                        const int wi = wo * stride + kw - pad;
                        if (wi < 0 || wi >= W) continue;
                        u64* xo = gx + (((size_t)b * H + hi) * W + wi) * Cin;
                        const u64* wk = w + ((size_t)kh * KW + kw) * Cin * Cout;
                        for (int ci = 0; ci < Cin; ++ci) {
                            const u64* wr = wk + (size_t)ci * Cout;
                            u64 acc = 0;
                            for (int co = 0; co < Cout; ++co) acc += go[co] * wr[co];
                            xo[ci] += acc;
                        }
                    }
                }
            }
}

void orc_ring_conv2d_grad_w(const u64* x, const u64* g, u64* gw,
                            int B, int H, int W, int Cin, int Cout,
                            int KH, int KW, int pad, int stride)
{
    const int Ho = (H + 2 * pad - KH) / stride + 1;
    const int Wo = (W + 2 * pad - KW) / stride + 1;
#pragma omp parallel for collapse(2) schedule(static)
    for (int kh = 0; kh < KH; ++kh)
        for (int kw = 0; kw < KW; ++kw) {
            u64* wk = gw + ((size_t)kh * KW + kw) * Cin * Cout;
            for (size_t i = 0; i < (size_t)Cin * Cout; ++i) wk[i] = 0;
            for (int b = 0; b < B; ++b)
                for (int ho = 0; ho < Ho; ++ho) {
                    const int hi = ho * stride + kh - pad;
                    if (hi < 0 || hi >= H) continue;
                    for (int wo = 0; wo < Wo; ++wo) {
                        const int wi = wo * stride + kw - pad;
                        if (wi < 0 || wi >= W) continue;
                        const u64* xi = x + (((size_t)b * H + hi) * W + wi) * Cin;
                        const u64* go = g + (((size_t)b * Ho + ho) * Wo + wo) * Cout;
                        for (int ci = 0; ci < Cin; ++ci) {
                            const u64 xv = xi[ci];
                            u64* wr = wk + (size_t)ci * Cout;
                            for (int co = 0; co < Cout; ++co) wr[co] += xv * go[co];
                        }
                    }
                }
        }
}

/* Explicit im2col of an NHWC tensor: row (b,ho,wo), column (kh,kw,ci).
 * Only used by tests to pin conv == im2col-then-matmul. */
void orc_im2col(const u64* x, u64* col, int B, int H, int W, int Cin,
                int KH, int KW, int pad, int stride)
{
    const int Ho = (H + 2 * pad - KH) / stride + 1;
    const int Wo = (W + 2 * pad - KW) / stride + 1;
    const size_t Kc = (size_t)KH * KW * Cin;
    for (int b = 0; b < B; ++b)
        for (int ho = 0; ho < Ho; ++ho)
            for (int wo = 0; wo < Wo; ++wo) {
                u64* row = col + (((size_t)b * Ho + ho) * Wo + wo) * Kc;
                for (int kh = 0; kh < KH; ++kh)
                    for (int kw = 0; kw < KW; ++kw)
                        for (int ci = 0; ci < Cin; ++ci) {
                            const int hi = ho * stride + kh - pad;
                            const int wi = wo * stride + kw - pad;
                            u64 v = 0;
                            if (hi >= 0 && hi < H && wi >= 0 && wi < W)
                                v = x[(((size_t)b * H + hi) * W + wi) * Cin + ci];
                            row[((size_t)kh * KW + kw) * Cin + ci] = v;
                        }
            }
}

/* ------------------------------------------------- Alg. 1: Beaver multiply */

/* Alg. 1, "computes [x_i] - [a_i]". */
void orc_mask(const u64* x, const u64* a, u64* e, size_t n)
{
    for (size_t i = 0; i < n; ++i) e[i] = x[i] - a[i];
}

/* Alg. 1, Delta = sum_i ([x_i] - [a_i]); also the generic opening of a
 * two-party additive sharing. */
void orc_open(const u64* s0, const u64* s1, u64* out, size_t n)
{
    for (size_t i = 0; i < n; ++i) out[i] = s0[i] + s1[i];
}

/* Alg. 1 element by element (the products of the non-linear layers' backward
 * pass, Sec. 4.2 and 5.3: output gradient times the stored input mask):
 *   [z_0] = [c_0] + e*[b_0] + [a_0]*f + e*f,   [z_1] = [c_1] + e*[b_1] + [a_1]*f. */
void orc_beaver_mul(const u64* x0, const u64* x1, const u64* y0, const u64* y1,
                    const u64* a0, const u64* a1, const u64* b0, const u64* b1,
                    const u64* c0, const u64* c1, u64* z0, u64* z1, size_t n)
{
    for (size_t i = 0; i < n; ++i) {
        const u64 e = (x0[i] - a0[i]) + (x1[i] - a1[i]);
        const u64 f = (y0[i] - b0[i]) + (y1[i] - b1[i]);
        z0[i] = c0[i] + e * b0[i] + a0[i] * f + e * f;
        z1[i] = c1[i] + e * b1[i] + a1[i] * f;
    }
}

static u64* alloc_words(size_t n) { return (u64*)malloc(n * sizeof(u64)); }

/* Alg. 1 for matrices, literally: five ring products.
 *   [z_0] = [c_0] + e*[b_0] + [a_0]*f + e*f      (party that owns the e*f term)
 *   [z_1] = [c_1] + e*[b_1] + [a_1]*f
 * with e, a on the left and b, f on the right (Eq. 3's Conv(Delta,[b]),
 * Conv([a],epsilon) operand order).  e_out / f_out (optional) receive the
 * opened values. */
void orc_beaver_matmul(const u64* x0, const u64* x1, const u64* y0, const u64* y1,
                       const u64* a0, const u64* a1, const u64* b0, const u64* b1,
                       const u64* c0, const u64* c1, u64* z0, u64* z1,
                       int M, int K, int N, u64* e_out, u64* f_out)
{
    const size_t mk = (size_t)M * K, kn = (size_t)K * N, mn = (size_t)M * N;
    u64 *e0 = alloc_words(mk), *e1 = alloc_words(mk), *e = alloc_words(mk);
    u64 *f0 = alloc_words(kn), *f1 = alloc_words(kn), *f = alloc_words(kn);
    u64 *t = alloc_words(mn);
    orc_mask(x0, a0, e0, mk); orc_mask(x1, a1, e1, mk);
    orc_mask(y0, b0, f0, kn); orc_mask(y1, b1, f1, kn);
    orc_open(e0, e1, e, mk);
    orc_open(f0, f1, f, kn);

    for (size_t i = 0; i < mn; ++i) z0[i] = c0[i];
    orc_ring_matmul(e, b0, t, M, K, N);  for (size_t i = 0; i < mn; ++i) z0[i] += t[i];
    orc_ring_matmul(a0, f, t, M, K, N);  for (size_t i = 0; i < mn; ++i) z0[i] += t[i];
    orc_ring_matmul(e, f, t, M, K, N);   for (size_t i = 0; i < mn; ++i) z0[i] += t[i];

    for (size_t i = 0; i < mn; ++i) z1[i] = c1[i];
    orc_ring_matmul(e, b1, t, M, K, N);  for (size_t i = 0; i < mn; ++i) z1[i] += t[i];
    orc_ring_matmul(a1, f, t, M, K, N);  for (size_t i = 0; i < mn; ++i) z1[i] += t[i];

    if (e_out) memcpy(e_out, e, mk * sizeof(u64));
    if (f_out) memcpy(f_out, f, kn * sizeof(u64));
    free(e0); free(e1); free(e); free(f0); free(f1); free(f); free(t);
}

/* Eq. 3: the same with Conv in place of the product.  A has the shape of X,
 * B the shape of W, C = Conv(A,B) the shape of the output.  Padding pads the
 * shares with zero words (a pair of zero shares reconstructs to zero). */
void orc_beaver_conv2d(const u64* x0, const u64* x1, const u64* w0, const u64* w1,
                       const u64* a0, const u64* a1, const u64* b0, const u64* b1,
                       const u64* c0, const u64* c1, u64* z0, u64* z1,
                       int B, int H, int W, int Cin, int Cout,
                       int KH, int KW, int pad, int stride)
{
    const int Ho = (H + 2 * pad - KH) / stride + 1;
    const int Wo = (W + 2 * pad - KW) / stride + 1;
    const size_t nx = (size_t)B * H * W * Cin, nw = (size_t)KH * KW * Cin * Cout;
    const size_t nz = (size_t)B * Ho * Wo * Cout;
    u64 *e0 = alloc_words(nx), *e1 = alloc_words(nx), *e = alloc_words(nx);
    u64 *f0 = alloc_words(nw), *f1 = alloc_words(nw), *f = alloc_words(nw);
    u64 *t = alloc_words(nz);
    orc_mask(x0, a0, e0, nx); orc_mask(x1, a1, e1, nx);
    orc_mask(w0, b0, f0, nw); orc_mask(w1, b1, f1, nw);
    orc_open(e0, e1, e, nx);
    orc_open(f0, f1, f, nw);
#define CONV(in, flt) orc_ring_conv2d(in, flt, t, B, H, W, Cin, Cout, KH, KW, pad, stride)
    for (size_t i = 0; i < nz; ++i) z0[i] = c0[i];
    CONV(e, b0);  for (size_t i = 0; i < nz; ++i) z0[i] += t[i];
    CONV(a0, f);  for (size_t i = 0; i < nz; ++i) z0[i] += t[i];
    CONV(e, f);   for (size_t i = 0; i < nz; ++i) z0[i] += t[i];
    for (size_t i = 0; i < nz; ++i) z1[i] = c1[i];
    CONV(e, b1);  for (size_t i = 0; i < nz; ++i) z1[i] += t[i];
    CONV(a1, f);  for (size_t i = 0; i < nz; ++i) z1[i] += t[i];
#undef CONV
    free(e0); free(e1); free(e); free(f0); free(f1); free(f); free(t);
}

/* Fixed-point rescale after a product.  The paper only says operands are
 * fixed point (Sec. 1.1); the reading taken here is the usual two-party local
 * truncation: party 0 shifts its share right (logical), party 1 negates,
 * shifts, negates.  The reconstructed result is floor(z / 2^bits) + {0, 1}
 * unless the shares wrap, which happens with probability about |z| / 2^64. */
void orc_truncate(u64* z0, u64* z1, size_t n, int bits)
{
    for (size_t i = 0; i < n; ++i) {
        z0[i] = z0[i] >> bits;
        z1[i] = (u64)0 - (((u64)0 - z1[i]) >> bits);
    }
}

/* ------------------------------------------------ binary-share primitives */

static inline u64 width_mask(int w) { return w >= 64 ? ~(u64)0 : (((u64)1 << w) - 1); }

/* Beaver AND on one word pair, both parties at once (Sec. 3.2: Alg. 1 with
 * + -> xor and * -> and; Alg. 4 for the party that owns the d&g term).
 * X, Y are XOR-shared operands, (a, b, c) an XOR-shared triple with
 * c = a & b.  out[i] is party i's share of X & Y. */
static inline void beaver_and(const u64 X[2], const u64 Y[2],
                              const u64 a[2], const u64 b[2], const u64 c[2],
                              u64 out[2])
{
    const u64 d0 = X[0] ^ a[0], d1 = X[1] ^ a[1];   /* each party masks ...   */
    const u64 g0 = Y[0] ^ b[0], g1 = Y[1] ^ b[1];
    const u64 d = d0 ^ d1, g = g0 ^ g1;             /* ... and both open      */
    out[0] = c[0] ^ (d & b[0]) ^ (g & a[0]) ^ (d & g);
    out[1] = c[1] ^ (d & b[1]) ^ (g & a[1]);
}

/* exported scalar form for exhaustive tests */
void orc_beaver_and(const u64* X, const u64* Y, const u64* a, const u64* b,
                    const u64* c, u64* out)
{
    beaver_and(X, Y, a, b, c, out);
}

/* Alg. 2, first half: each party XOR-shares its own arithmetic share.
 * Party 0 keeps x_0 ^ r_0 and sends r_0; party 1 keeps x_1 ^ r_1 and sends
 * r_1.  U is the binary sharing of the word x_0, V of the word x_1. */
static inline void a2b_distribute(const u64 x[2], const u64 r[2], u64 U[2], u64 V[2])
{
    U[0] = x[0] ^ r[0];  U[1] = r[0];
    V[0] = r[1];         V[1] = x[1] ^ r[1];
}

/* Alg. 2, last step: add the two binary-shared words with a parallel-prefix
 * (Kogge-Stone) carry network over XOR shares, width w = 2^levels bits.
 *   P = U ^ V (local);  G = U & V               (triple 0)
 *   for l = 0 .. levels-1, d = 2^l:
 *       G <- G ^ (P & (G << d))                  (triple 1 + 2l)
 *       P <- P & (P << d)   unless last level    (triple 2 + 2l)
 * Both ANDs of a level read the P of the previous level.  Shifts are
 * share-wise with zero fill.  After the loop bit j of G is the carry out of
 * bit positions [0..j].  XOR may stand for OR because a group cannot both
 * generate and propagate.  ta/tb/tc: [2*levels][2] triple words (masked to w
 * bits by the caller).  Returns G shares; P0 (the initial U^V) in P0_out. */
static void ks_adder(const u64 U[2], const u64 V[2], int w,
                     const u64 (*ta)[2], const u64 (*tb)[2], const u64 (*tc)[2],
                     u64 G[2], u64 P0_out[2])
{
    const u64 wm = width_mask(w);
    u64 P[2] = { U[0] ^ V[0], U[1] ^ V[1] };
    P0_out[0] = P[0]; P0_out[1] = P[1];
    beaver_and(U, V, ta[0], tb[0], tc[0], G);
    int levels = 0; while ((1 << levels) < w) ++levels;
    for (int l = 0; l < levels; ++l) {
        const int d = 1 << l;
        const u64 Gs[2] = { (G[0] << d) & wm, (G[1] << d) & wm };
        const u64 Ps[2] = { (P[0] << d) & wm, (P[1] << d) & wm };
        u64 T[2], Pn[2];
        beaver_and(P, Gs, ta[1 + 2 * l], tb[1 + 2 * l], tc[1 + 2 * l], T);
        if (l < levels - 1)
            beaver_and(P, Ps, ta[2 + 2 * l], tb[2 + 2 * l], tc[2 + 2 * l], Pn);
        G[0] ^= T[0]; G[1] ^= T[1];
        if (l < levels - 1) { P[0] = Pn[0]; P[1] = Pn[1]; }
    }
}

/* The same carries by the divide-and-conquer prefix tree of the listing in
 * Sec. 4.2 (level i joins blocks of 2^i bits into blocks of 2^(i+1)); the
 * constants are not printed there and follow from that description:
 *   im_i  the top bit of every lower half,  om_i  every upper half,
 *   spread_i(w) = (w & im_i) * (2 + 4 + ... + 2^(2^i)): that bit copied over its upper half.
 *   for i = 0 .. 5:   X  = P & om_i
 *       G <- G ^ (X & spread_i(G))                        (triple 1 + 2i)
 *       P <- (P & ~om_i) ^ (X & spread_i(P))   unless last (triple 2 + 2i)
 * Masks and spreads act on each XOR share (no two copied bits meet, so the
 * multiply adds nothing).  64-bit words only. */
static void tree_adder(const u64 U[2], const u64 V[2],
                       const u64 (*ta)[2], const u64 (*tb)[2], const u64 (*tc)[2],
                       u64 G[2], u64 P0_out[2])
{
    u64 P[2] = { U[0] ^ V[0], U[1] ^ V[1] };
    P0_out[0] = P[0]; P0_out[1] = P[1];
    beaver_and(U, V, ta[0], tb[0], tc[0], G);
    for (int i = 0; i < 6; ++i) {
        const int half = 1 << i, blk = 2 << i;
        u64 im = 0, om = 0, mu = 0;
        for (int base = 0; base < 64; base += blk) {
            im |= (u64)1 << (base + half - 1);
            om |= ((half == 64 ? ~(u64)0 : (((u64)1 << half) - 1))) << (base + half);
        }
        for (int k = 1; k <= half; ++k) mu |= (u64)1 << k;
        const u64 X[2] = { P[0] & om, P[1] & om };
        const u64 Gs[2] = { (G[0] & im) * mu, (G[1] & im) * mu };
        const u64 Ps[2] = { (P[0] & im) * mu, (P[1] & im) * mu };
        u64 T[2], Pn[2];
        beaver_and(X, Gs, ta[1 + 2 * i], tb[1 + 2 * i], tc[1 + 2 * i], T);
        if (i < 5) beaver_and(X, Ps, ta[2 + 2 * i], tb[2 + 2 * i], tc[2 + 2 * i], Pn);
        G[0] ^= T[0]; G[1] ^= T[1];
        if (i < 5) { P[0] = (P[0] & ~om) ^ Pn[0]; P[1] = (P[1] & ~om) ^ Pn[1]; }
    }
}

/* Exported for tests: the tree's carry shares for one word pair, 12 triple words per party. */
void orc_tree_carries(const u64* U, const u64* V,
                      const u64* ta0, const u64* ta1, const u64* tb0, const u64* tb1,
                      const u64* tc0, const u64* tc1, u64* G)
{
    u64 ta[12][2], tb[12][2], tc[12][2], P0[2];
    for (int t = 0; t < 12; ++t) {
        ta[t][0] = ta0[t]; ta[t][1] = ta1[t];
        tb[t][0] = tb0[t]; tb[t][1] = tb1[t];
        tc[t][0] = tc0[t]; tc[t][1] = tc1[t];
    }
    tree_adder(U, V, ta, tb, tc, G, P0);
}

/* Exported for tests: XOR shares of (U + V) mod 2^w given XOR shares of U, V.
 * Triples: arrays of 2*levels words per party, ta0 = party 0's a words, ... */
void orc_ks_add(const u64* U, const u64* V, int w,
                const u64* ta0, const u64* ta1, const u64* tb0, const u64* tb1,
                const u64* tc0, const u64* tc1, u64* S)
{
    u64 ta[12][2], tb[12][2], tc[12][2], G[2], P0[2];
    int levels = 0; while ((1 << levels) < w) ++levels;
    for (int t = 0; t < 2 * levels; ++t) {
        ta[t][0] = ta0[t]; ta[t][1] = ta1[t];
        tb[t][0] = tb0[t]; tb[t][1] = tb1[t];
        tc[t][0] = tc0[t]; tc[t][1] = tc1[t];
    }
    ks_adder(U, V, w, ta, tb, tc, G, P0);
    const u64 wm = width_mask(w);
    S[0] = P0[0] ^ ((G[0] << 1) & wm);
    S[1] = P0[1] ^ ((G[1] << 1) & wm);
}

/* ------------------------------------------------------------ secure ReLU */

/* Per-party material for n elements (all "offline" inputs):
 *   r      n words       A2B masks
 *   ta/tb/tc  [12][n]    AND triples, triple-major, c = a & b when XORed
 *   rb     n bytes (0/1) XOR-shared random bit,  ra: n words additive shares
 *                        of that same bit (ra_0 + ra_1 = rb_0 ^ rb_1)
 *   ma/mb/mc  n words    element-wise multiplication triple, mc = ma*mb
 */
typedef struct {
    const u64* r[2];
    const u64* ta[2]; const u64* tb[2]; const u64* tc[2];
    const u8*  rb[2]; const u64* ra[2];
    const u64* ma[2]; const u64* mb[2]; const u64* mc[2];
} orc_relu_material;

/* ReLU(x) = x * (1 - MSB(x)) on additive shares (the paper names only "MSB"
 * and "one conversion per ReLU", Sec. 3.2 / 4.2; the rest is this reading):
 *   1. A2B distribution (Alg. 2)           -> U, V
 *   2. 64-bit prefix adder, 12 AND triples -> carries G
 *   3. sign share  s_i = bit63(U_i ^ V_i) ^ bit62(G_i)
 *   4. B2A with a shared random bit: open v = s ^ rb;
 *        [s]_0 = ra_0 + v - 2 v ra_0,   [s]_1 = ra_1 - 2 v ra_1
 *   5. m = 1 - s:  m_0 = 1 - [s]_0, m_1 = -[s]_1
 *   6. y = x * m by element-wise Alg. 1 (no rescale: m is an integer 0/1)
 * Optional outputs: s_bit[i] (n bytes), s_arith[i] (n words).
 * adder: 0 = Kogge-Stone network, 1 = the listing's prefix tree. */
void orc_relu_adder(const u64* x0, const u64* x1, const orc_relu_material* mt,
                    u64* y0, u64* y1, size_t n,
                    u8* s_bit0, u8* s_bit1, u64* s_ar0, u64* s_ar1, int adder)
{
#pragma omp parallel for schedule(static)
    for (size_t i = 0; i < n; ++i) {
        const u64 x[2] = { x0[i], x1[i] };
        const u64 r[2] = { mt->r[0][i], mt->r[1][i] };
        u64 U[2], V[2], G[2], P0[2];
        u64 ta[12][2], tb[12][2], tc[12][2];
        for (int t = 0; t < 12; ++t)
            for (int p = 0; p < 2; ++p) {
                ta[t][p] = mt->ta[p][(size_t)t * n + i];
                tb[t][p] = mt->tb[p][(size_t)t * n + i];
                tc[t][p] = mt->tc[p][(size_t)t * n + i];
            }
        a2b_distribute(x, r, U, V);
        if (adder == 1) tree_adder(U, V, ta, tb, tc, G, P0);
        else            ks_adder(U, V, 64, ta, tb, tc, G, P0);
        /* sum bit 63 = u63 ^ v63 ^ carry into 63 = P0 bit 63 ^ G bit 62 */
        const u64 s[2] = { (P0[0] >> 63) ^ ((G[0] >> 62) & 1),
                           (P0[1] >> 63) ^ ((G[1] >> 62) & 1) };
        /* B2A */
        const u64 rb[2] = { mt->rb[0][i], mt->rb[1][i] };
        const u64 ra[2] = { mt->ra[0][i], mt->ra[1][i] };
        const u64 v = (s[0] ^ rb[0]) ^ (s[1] ^ rb[1]);
        const u64 sa[2] = { ra[0] + v - 2 * v * ra[0], ra[1] - 2 * v * ra[1] };
        /* select */
        const u64 m[2] = { (u64)1 - sa[0], (u64)0 - sa[1] };
        const u64 ma[2] = { mt->ma[0][i], mt->ma[1][i] };
        const u64 mb[2] = { mt->mb[0][i], mt->mb[1][i] };
        const u64 mc[2] = { mt->mc[0][i], mt->mc[1][i] };
        const u64 e = (x[0] - ma[0]) + (x[1] - ma[1]);
        const u64 f = (m[0] - mb[0]) + (m[1] - mb[1]);
        y0[i] = mc[0] + e * mb[0] + ma[0] * f + e * f;
        y1[i] = mc[1] + e * mb[1] + ma[1] * f;
        if (s_bit0) s_bit0[i] = (u8)s[0];
        if (s_bit1) s_bit1[i] = (u8)s[1];
        if (s_ar0) s_ar0[i] = sa[0];
        if (s_ar1) s_ar1[i] = sa[1];
    }
}

void orc_relu(const u64* x0, const u64* x1, const orc_relu_material* mt,
              u64* y0, u64* y1, size_t n,
              u8* s_bit0, u8* s_bit1, u64* s_ar0, u64* s_ar1)
{
    orc_relu_adder(x0, x1, mt, y0, y1, n, s_bit0, s_bit1, s_ar0, s_ar1, 0);
}

/* B2A step alone, scalar, for exhaustive tests. */
void orc_b2a(const u8* s, const u8* rb, const u64* ra, u64* out)
{
    const u64 v = (u64)((s[0] ^ rb[0]) ^ (s[1] ^ rb[1]));
    out[0] = ra[0] + v - 2 * v * ra[0];
    out[1] = ra[1] - 2 * v * ra[1];
}

/* ---------------------------------------------------------- 2x2 max-pool */

/* Gathers for max(p,q) = q + ReLU(p - q), NHWC, 2x2 window, stride 2, on one
 * party's share (all three steps are local and linear):
 *   level 1: for every window, d[2*o+0] = p00 - p01, d[2*o+1] = p10 - p11
 *   after ReLU r1:  u = p01 + r1[2*o], v = p11 + r1[2*o+1], level 2: d2 = u - v
 *   after ReLU r2:  out = v + r2
 * o = output index in [B][H/2][W/2][C] order. */
void orc_pool_level1(const u64* x, u64* d, int B, int H, int W, int C)
{
    const int Ho = H / 2, Wo = W / 2;
    for (int b = 0; b < B; ++b) for (int ho = 0; ho < Ho; ++ho)
    for (int wo = 0; wo < Wo; ++wo) for (int c = 0; c < C; ++c) {
        const size_t o = (((size_t)b * Ho + ho) * Wo + wo) * C + c;
#define PX(dh, dw) x[(((size_t)b * H + 2 * ho + dh) * W + 2 * wo + dw) * C + c]
        d[2 * o + 0] = PX(0, 0) - PX(0, 1);
        d[2 * o + 1] = PX(1, 0) - PX(1, 1);
    }
}

void orc_pool_level2(const u64* x, const u64* r1, u64* v_out, u64* d2,
                     int B, int H, int W, int C)
{
    const int Ho = H / 2, Wo = W / 2;
    for (int b = 0; b < B; ++b) for (int ho = 0; ho < Ho; ++ho)
    for (int wo = 0; wo < Wo; ++wo) for (int c = 0; c < C; ++c) {
        const size_t o = (((size_t)b * Ho + ho) * Wo + wo) * C + c;
        const u64 u = PX(0, 1) + r1[2 * o + 0];
        const u64 v = PX(1, 1) + r1[2 * o + 1];
        v_out[o] = v;
        d2[o] = u - v;
    }
#undef PX
}

/* ========================================================= three parties
 *
 * Alg. 1 and Alg. 2 are written for N parties (Sec. 3.2; Sec. 3.3 on the
 * number of parties; Sec. 5.6 measures three).  Below, N = 3: an additive
 * sharing is x = x_0 + x_1 + x_2, a binary one X = X_0 ^ X_1 ^ X_2, and a
 * masked value is opened by summing (XORing) what all three parties
 * broadcast.  Party 0 is again the paper's "Party #1".  Arguments are arrays
 * of three pointers, one per party.
 */
#define NP 3

/* Sec. 3.1: reconstruct an additive sharing. */
void orc3_open(const u64* const s[NP], u64* out, size_t n)
{
    for (size_t i = 0; i < n; ++i) out[i] = s[0][i] + s[1][i] + s[2][i];
}

/* Alg. 1, element by element, three parties. */
void orc3_beaver_mul(const u64* const x[NP], const u64* const y[NP],
                     const u64* const a[NP], const u64* const b[NP], const u64* const c[NP],
                     u64* const z[NP], size_t n)
{
    for (size_t i = 0; i < n; ++i) {
        u64 e = 0, f = 0;
        for (int p = 0; p < NP; ++p) { e += x[p][i] - a[p][i]; f += y[p][i] - b[p][i]; }
        for (int p = 0; p < NP; ++p) {
            u64 v = c[p][i] + e * b[p][i] + a[p][i] * f;
            if (p == 0) v += e * f;
            z[p][i] = v;
        }
    }
}

/* Alg. 1 on matrices, literally: Delta and epsilon are the sums of the three
 * broadcast differences; party 0 adds Delta*epsilon (seven ring products). */
void orc3_beaver_matmul(const u64* const x[NP], const u64* const y[NP],
                        const u64* const a[NP], const u64* const b[NP], const u64* const c[NP],
                        u64* const z[NP], int M, int K, int N)
{
    const size_t mk = (size_t)M * K, kn = (size_t)K * N, mn = (size_t)M * N;
    u64 *e = alloc_words(mk), *f = alloc_words(kn), *t = alloc_words(mn);
    for (size_t i = 0; i < mk; ++i) { e[i] = 0; for (int p = 0; p < NP; ++p) e[i] += x[p][i] - a[p][i]; }
    for (size_t i = 0; i < kn; ++i) { f[i] = 0; for (int p = 0; p < NP; ++p) f[i] += y[p][i] - b[p][i]; }
    for (int p = 0; p < NP; ++p) {
        for (size_t i = 0; i < mn; ++i) z[p][i] = c[p][i];
        orc_ring_matmul(e, b[p], t, M, K, N);  for (size_t i = 0; i < mn; ++i) z[p][i] += t[i];
        orc_ring_matmul(a[p], f, t, M, K, N);  for (size_t i = 0; i < mn; ++i) z[p][i] += t[i];
        if (p == 0) { orc_ring_matmul(e, f, t, M, K, N); for (size_t i = 0; i < mn; ++i) z[p][i] += t[i]; }
    }
    free(e); free(f); free(t);
}

/* Eq. 3 with three parties. */
void orc3_beaver_conv2d(const u64* const x[NP], const u64* const w[NP],
                        const u64* const a[NP], const u64* const b[NP], const u64* const c[NP],
                        u64* const z[NP], int B, int H, int W, int Cin, int Cout,
                        int KH, int KW, int pad, int stride)
{
    const int Ho = (H + 2 * pad - KH) / stride + 1;
    const int Wo = (W + 2 * pad - KW) / stride + 1;
    const size_t nx = (size_t)B * H * W * Cin, nw = (size_t)KH * KW * Cin * Cout;
    const size_t nz = (size_t)B * Ho * Wo * Cout;
    u64 *e = alloc_words(nx), *f = alloc_words(nw), *t = alloc_words(nz);
    for (size_t i = 0; i < nx; ++i) { e[i] = 0; for (int p = 0; p < NP; ++p) e[i] += x[p][i] - a[p][i]; }
    for (size_t i = 0; i < nw; ++i) { f[i] = 0; for (int p = 0; p < NP; ++p) f[i] += w[p][i] - b[p][i]; }
#define CONV(in, flt) orc_ring_conv2d(in, flt, t, B, H, W, Cin, Cout, KH, KW, pad, stride)
    for (int p = 0; p < NP; ++p) {
        for (size_t i = 0; i < nz; ++i) z[p][i] = c[p][i];
        CONV(e, b[p]);  for (size_t i = 0; i < nz; ++i) z[p][i] += t[i];
        CONV(a[p], f);  for (size_t i = 0; i < nz; ++i) z[p][i] += t[i];
        if (p == 0) { CONV(e, f); for (size_t i = 0; i < nz; ++i) z[p][i] += t[i]; }
    }
#undef CONV
    free(e); free(f); free(t);
}

/* Fixed-point rescale with three parties.  Shifting each share locally is
 * only sound for two parties; the paper gives no rescale at all (Sec. 1.1
 * names fixed point, nothing more), so the reading taken here is the usual
 * masked one with an offline pair ([r], [r >> bits]), r uniform in [0, 2^63):
 *   parties 1 and 2 send z_i + r_i to party 0, which forms
 *       m = z + r + 2^62                 (z in [-2^62, 2^62): no wrap mod 2^64)
 *   [t_0] = (m >> bits) - 2^(62-bits) - [rt_0],   [t_i] = -[rt_i].
 * m >> bits = (z + 2^62 >> bits) + (r >> bits) + carry of the low parts, so
 * the result reconstructs to floor(z / 2^bits) + {0, 1}. */
void orc3_truncate(u64* const z[NP], const u64* const r[NP], const u64* const rt[NP],
                   size_t n, int bits)
{
    for (size_t i = 0; i < n; ++i) {
        u64 m = (u64)1 << 62;
        for (int p = 0; p < NP; ++p) m += z[p][i] + r[p][i];
        z[0][i] = (m >> bits) - ((u64)1 << (62 - bits)) - rt[0][i];
        z[1][i] = (u64)0 - rt[1][i];
        z[2][i] = (u64)0 - rt[2][i];
    }
}

/* Beaver AND with three parties (Alg. 1 with xor for + and and for *). */
static inline void beaver_and3(const u64 X[NP], const u64 Y[NP],
                               const u64 a[NP], const u64 b[NP], const u64 c[NP], u64 out[NP])
{
    u64 d = 0, g = 0;
    for (int p = 0; p < NP; ++p) { d ^= X[p] ^ a[p]; g ^= Y[p] ^ b[p]; }
    for (int p = 0; p < NP; ++p) out[p] = c[p] ^ (d & b[p]) ^ (g & a[p]);
    out[0] ^= d & g;
}

void orc3_beaver_and(const u64* X, const u64* Y, const u64* a, const u64* b, const u64* c, u64* out)
{
    beaver_and3(X, Y, a, b, c, out);
}

/* Alg. 2, first half, three parties: party j XOR-shares its own word x_j by
 * keeping x_j ^ r0_j ^ r1_j, sending r0_j to party j+1 and r1_j to party j+2
 * (indices mod 3).  Wd[j][p] = party p's share of the word x_j. */
static inline void a2b_distribute3(const u64 x[NP], const u64 r0[NP], const u64 r1[NP], u64 Wd[NP][NP])
{
    for (int j = 0; j < NP; ++j) {
        Wd[j][j] = x[j] ^ r0[j] ^ r1[j];
        Wd[j][(j + 1) % NP] = r0[j];
        Wd[j][(j + 2) % NP] = r1[j];
    }
}

/* Alg. 2, last step, three parties: "binary operations" that add the three
 * binary-shared words.  The paper names no circuit for more than two
 * addends; the reading taken here is the hardware-adder one: a carry-save
 * step turns three addends into two,
 *     S = U ^ V ^ W,   C = maj(U, V, W) = ((U ^ W) & (V ^ W)) ^ W   (triple 0)
 * and the same Kogge-Stone network as for two parties adds S and C << 1:
 *     P = S ^ K,  G = S & K with K = C << 1                          (triple 1)
 *     level l, d = 2^l:  G <- G ^ (P & (G << d))                     (triple 2 + 2l)
 *                        P <- P & (P << d)    unless last level      (triple 3 + 2l)
 * 1 + 2*levels triples for width w = 2^levels.  Returns the carries G and
 * the initial P = S ^ K. */
static void add3_carries(const u64 U[NP], const u64 V[NP], const u64 W[NP], int w,
                         const u64 (*ta)[NP], const u64 (*tb)[NP], const u64 (*tc)[NP],
                         u64 G[NP], u64 P0_out[NP])
{
    const u64 wm = width_mask(w);
    u64 X[NP], Y[NP], T[NP], S[NP], K[NP], P[NP];
    for (int p = 0; p < NP; ++p) { X[p] = U[p] ^ W[p]; Y[p] = V[p] ^ W[p]; S[p] = U[p] ^ V[p] ^ W[p]; }
    beaver_and3(X, Y, ta[0], tb[0], tc[0], T);
    for (int p = 0; p < NP; ++p) { K[p] = ((T[p] ^ W[p]) << 1) & wm; P[p] = S[p] ^ K[p]; P0_out[p] = P[p]; }
    beaver_and3(S, K, ta[1], tb[1], tc[1], G);
    int levels = 0; while ((1 << levels) < w) ++levels;
    for (int l = 0; l < levels; ++l) {
        const int d = 1 << l;
        u64 Gs[NP], Ps[NP], Pn[NP];
        for (int p = 0; p < NP; ++p) { Gs[p] = (G[p] << d) & wm; Ps[p] = (P[p] << d) & wm; }
        beaver_and3(P, Gs, ta[2 + 2 * l], tb[2 + 2 * l], tc[2 + 2 * l], T);
        if (l < levels - 1) beaver_and3(P, Ps, ta[3 + 2 * l], tb[3 + 2 * l], tc[3 + 2 * l], Pn);
        for (int p = 0; p < NP; ++p) { G[p] ^= T[p]; if (l < levels - 1) P[p] = Pn[p]; }
    }
}

/* Exported for tests: XOR shares of (U + V + W) mod 2^w.  U, V, W: three
 * share words each; ta/tb/tc: [1 + 2*levels][3] words, triple-major. */
void orc3_add3(const u64* U, const u64* V, const u64* W, int w,
               const u64* ta, const u64* tb, const u64* tc, u64* S)
{
    u64 G[NP], P0[NP];
    add3_carries(U, V, W, w, (const u64 (*)[NP])ta, (const u64 (*)[NP])tb, (const u64 (*)[NP])tc, G, P0);
    const u64 wm = width_mask(w);
    for (int p = 0; p < NP; ++p) S[p] = P0[p] ^ ((G[p] << 1) & wm);
}

/* Per-party material for n elements of the three-party ReLU:
 *   r0, r1    n words each   A2B masks (sent to the next / the second-next party)
 *   ta/tb/tc  [13][n]        AND triples, triple-major
 *   rb        n bytes (0/1)  XOR-shared random bit, ra: additive shares of that bit
 *   ma/mb/mc  n words        element-wise multiplication triple
 */
typedef struct {
    const u64* r0[NP]; const u64* r1[NP];
    const u64* ta[NP]; const u64* tb[NP]; const u64* tc[NP];
    const u8*  rb[NP]; const u64* ra[NP];
    const u64* ma[NP]; const u64* mb[NP]; const u64* mc[NP];
} orc3_relu_material;

/* B2A of one XOR-shared bit with a shared random bit, three parties:
 * open v = s ^ rb; [s]_0 = ra_0 + v - 2 v ra_0, [s]_i = ra_i - 2 v ra_i. */
static inline void b2a3(const u64 s[NP], const u64 rb[NP], const u64 ra[NP], u64 out[NP])
{
    u64 v = 0;
    for (int p = 0; p < NP; ++p) v ^= s[p] ^ rb[p];
    for (int p = 0; p < NP; ++p) out[p] = ra[p] - 2 * v * ra[p];
    out[0] += v;
}

void orc3_b2a(const u8* s, const u8* rb, const u64* ra, u64* out)
{
    const u64 s64[NP] = { s[0], s[1], s[2] }, rb64[NP] = { rb[0], rb[1], rb[2] };
    b2a3(s64, rb64, ra, out);
}

/* ReLU(x) = x * (1 - MSB(x)), three parties: A2B distribution, the
 * three-addend adder above (13 triples), sign share
 * s_p = bit63(P0_p) ^ bit62(G_p), B2A, m = 1 - s (party 0 holds the 1),
 * y = x * m by element-wise Alg. 1 without rescale. */
void orc3_relu(const u64* const x[NP], const orc3_relu_material* mt, u64* const y[NP], size_t n,
               u8* const s_bit[NP], u64* const s_ar[NP])
{
#pragma omp parallel for schedule(static)
    for (size_t i = 0; i < n; ++i) {
        u64 xs[NP], r0[NP], r1[NP], Wd[NP][NP], G[NP], P0[NP];
        u64 ta[13][NP], tb[13][NP], tc[13][NP];
        for (int p = 0; p < NP; ++p) {
            xs[p] = x[p][i]; r0[p] = mt->r0[p][i]; r1[p] = mt->r1[p][i];
            for (int t = 0; t < 13; ++t) {
                ta[t][p] = mt->ta[p][(size_t)t * n + i];
                tb[t][p] = mt->tb[p][(size_t)t * n + i];
                tc[t][p] = mt->tc[p][(size_t)t * n + i];
            }
        }
        a2b_distribute3(xs, r0, r1, Wd);
        add3_carries(Wd[0], Wd[1], Wd[2], 64, ta, tb, tc, G, P0);
        u64 s[NP], rb[NP], ra[NP], sa[NP], m[NP];
        for (int p = 0; p < NP; ++p) {
            s[p] = (P0[p] >> 63) ^ ((G[p] >> 62) & 1);
            rb[p] = mt->rb[p][i]; ra[p] = mt->ra[p][i];
        }
        b2a3(s, rb, ra, sa);
        for (int p = 0; p < NP; ++p) m[p] = (u64)(p == 0) - sa[p];
        u64 e = 0, f = 0;
        for (int p = 0; p < NP; ++p) { e += xs[p] - mt->ma[p][i]; f += m[p] - mt->mb[p][i]; }
        for (int p = 0; p < NP; ++p) {
            u64 v = mt->mc[p][i] + e * mt->mb[p][i] + mt->ma[p][i] * f;
            if (p == 0) v += e * f;
            y[p][i] = v;
            if (s_bit && s_bit[p]) s_bit[p][i] = (u8)s[p];
            if (s_ar && s_ar[p]) s_ar[p][i] = sa[p];
        }
    }
}
#undef NP
