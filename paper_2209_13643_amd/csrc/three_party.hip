// Three simulated parties (Alg. 1 and Alg. 2 are stated for N parties; Sec. 3.3,
// Sec. 5.6): opening, the masked rescale, and the secure ReLU whose A2B step
// adds three binary-shared words (carry-save step, then the Kogge-Stone
// network).  Everything here streams whole words and is bound by HBM; all
// launches go to the lane's first stream, one launch per step for all three
// parties (blockIdx.y = party), and every exchange is a copy kernel.
#include "common.h"

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
};
struct Relu3Args { Relu3Party p[3]; size_t n; };

// One Beaver AND gate finished: own and received masked operands -> this party's share.
__device__ __forceinline__ u64 and_finish(int party, u64 d, u64 g, u64 a, u64 b, u64 c)
{
    u64 t = c ^ (d & b) ^ (g & a);
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
template <int STAGE>
__global__ __launch_bounds__(kT) void k3_relu(Relu3Args q)
{
    const int party = blockIdx.y;
    const Relu3Party& p = q.p[party];
    const size_t n = q.n;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        // masked words of the previous round, opened
        u64 o[4] = { 0, 0, 0, 0 };
        constexpr int kOpen = (STAGE == 0 || STAGE >= 9) ? 0 : (STAGE >= 3 && STAGE <= 7) ? 4 : 2;
#pragma unroll
        for (int k = 0; k < kOpen; ++k) o[k] = p.send[k * n + i] ^ p.recv[0][k * n + i] ^ p.recv[1][k * n + i];

        if constexpr (STAGE == 0) {
            const u64 own = p.x[i] ^ p.r0[i] ^ p.r1[i];
            // party's shares of the words x_0, x_1, x_2
            const u64 w1 = p.wrecv[0][i], w2 = p.wrecv[1][i];        // words of party+1, party+2
            const u64 U = party == 0 ? own : party == 1 ? w2 : w1;
            const u64 V = party == 1 ? own : party == 2 ? w2 : w1;
            const u64 W = party == 2 ? own : party == 0 ? w2 : w1;
            p.S[i] = U ^ V ^ W; p.Wd[i] = W;
            p.send[i] = (U ^ W) ^ p.ta[i];
            p.send[n + i] = (V ^ W) ^ p.tb[i];
        } else if constexpr (STAGE == 1) {
            const u64 T = and_finish(party, o[0], o[1], p.ta[i], p.tb[i], p.tc[i]);
            const u64 S = p.S[i];
            const u64 K = (T ^ p.Wd[i]) << 1;
            const u64 P = S ^ K;
            p.P[i] = P; p.p63[i] = (u8)(P >> 63);
            p.send[i] = S ^ p.ta[n + i];
            p.send[n + i] = K ^ p.tb[n + i];
        } else if constexpr (STAGE == 2) {
            const u64 G = and_finish(party, o[0], o[1], p.ta[n + i], p.tb[n + i], p.tc[n + i]);
            const u64 P = p.P[i];
            p.G[i] = G;
            p.send[i] = P ^ p.ta[2 * n + i];          p.send[n + i] = (G << 1) ^ p.tb[2 * n + i];
            p.send[2 * n + i] = P ^ p.ta[3 * n + i];  p.send[3 * n + i] = (P << 1) ^ p.tb[3 * n + i];
        } else if constexpr (STAGE >= 3 && STAGE <= 7) {
            constexpr int L = STAGE - 3;                 // level being finished
            constexpr int tg = 2 + 2 * L, tp = 3 + 2 * L;
            const u64 T1 = and_finish(party, o[0], o[1], p.ta[tg * n + i], p.tb[tg * n + i], p.tc[tg * n + i]);
            const u64 P = and_finish(party, o[2], o[3], p.ta[tp * n + i], p.tb[tp * n + i], p.tc[tp * n + i]);
            const u64 G = p.G[i] ^ T1;
            p.G[i] = G;
            constexpr int d = 2 << L;                    // shift of level L + 1
            constexpr int ng = tg + 2, np = tp + 2;
            p.send[i] = P ^ p.ta[ng * n + i];  p.send[n + i] = (G << d) ^ p.tb[ng * n + i];
            if constexpr (L + 1 < 5) {                   // the last level needs no P update
                p.send[2 * n + i] = P ^ p.ta[np * n + i];  p.send[3 * n + i] = (P << d) ^ p.tb[np * n + i];
            }
        } else if constexpr (STAGE == 8) {
            const u64 T1 = and_finish(party, o[0], o[1], p.ta[12 * n + i], p.tb[12 * n + i], p.tc[12 * n + i]);
            const u64 G = p.G[i] ^ T1;
            const u8 s = (u8)(p.p63[i] ^ ((G >> 62) & 1));
            if (p.s_bit) p.s_bit[i] = s;
            p.vsend[i] = s ^ p.rb[i];
        } else if constexpr (STAGE == 9) {
            const u64 v = (u64)(p.vsend[i] ^ p.vrecv[0][i] ^ p.vrecv[1][i]);
            const u64 ra = p.ra[i];
            u64 sa = ra - 2 * v * ra;
            if (party == 0) sa += v;
            if (p.s_arith) p.s_arith[i] = sa;
            const u64 m = (party == 0 ? (u64)1 : (u64)0) - sa;
            p.send[i] = p.x[i] - p.ma[i];
            p.send[n + i] = m - p.mb[i];
        } else {
            // additive opening of the select product's masked operands
            const u64 e = p.send[i] + p.recv[0][i] + p.recv[1][i];
            const u64 f = p.send[n + i] + p.recv[0][n + i] + p.recv[1][n + i];
            u64 yv = p.mc[i] + e * p.mb[i] + p.ma[i] * f;
            if (party == 0) yv += e * f;
            p.y[i] = yv;
        }
    }
}

template <int STAGE>
int launch_stage(mpc_ctx* c, hipStream_t st, const Relu3Args& q)
{
    hipLaunchKernelGGL(k3_relu<STAGE>, dim3(grid3(q.n), 3), dim3(kT), 0, st, q);
    MPC_HIP(c, hipGetLastError());
    return MPC_OK;
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
    q.n = n;
}

// The whole chain on one stream: A2B distribution, 11 stage kernels, 10 word exchanges, one byte exchange.
int relu3_run(mpc_ctx* c, hipStream_t st, const Relu3Args& q)
{
    const size_t n = q.n;
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
    MPC_TRY(launch_stage<0>(c, st, q));  MPC_TRY(exchange_words(c, st, q, 2));
    MPC_TRY(launch_stage<1>(c, st, q));  MPC_TRY(exchange_words(c, st, q, 2));
    MPC_TRY(launch_stage<2>(c, st, q));  MPC_TRY(exchange_words(c, st, q, 4));
    MPC_TRY(launch_stage<3>(c, st, q));  MPC_TRY(exchange_words(c, st, q, 4));
    MPC_TRY(launch_stage<4>(c, st, q));  MPC_TRY(exchange_words(c, st, q, 4));
    MPC_TRY(launch_stage<5>(c, st, q));  MPC_TRY(exchange_words(c, st, q, 4));
    MPC_TRY(launch_stage<6>(c, st, q));  MPC_TRY(exchange_words(c, st, q, 4));
    MPC_TRY(launch_stage<7>(c, st, q));  MPC_TRY(exchange_words(c, st, q, 2));
    MPC_TRY(launch_stage<8>(c, st, q));
    {
        CopySeg cp[6]; int k = 0;
        for (int i = 0; i < 3; ++i)
            for (int s = 0; s < 2; ++s)
                cp[k++] = CopySeg{ q.p[(i + 1 + s) % 3].vsend, q.p[i].vrecv[s], n, 0 };
        MPC_TRY(launch_copy_multi(c, st, cp, 6));
    }
    MPC_TRY(launch_stage<9>(c, st, q));  MPC_TRY(exchange_words(c, st, q, 2));
    MPC_TRY(launch_stage<10>(c, st, q));
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
    return relu3_ws(nullptr, 0, n, &q, nullptr);
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
    relu3_ws(c->ws, c->ws_bytes, n, &q, &ok);
    if (!ok) return MPC_ENOMEM;
    fill3(q, x.p, m, y.p, s_bit, s_arith, n);
    hipStream_t st = c->s[0];
    MPC_TRY(lane_join(c));
    const int pi = prof_begin(c, MPC_PROF_RELU, st);
    MPC_TRY(relu3_run(c, st, q));
    prof_end(c, MPC_PROF_RELU, pi, st);
    return lane_fanout(c);
}

size_t mpc_maxpool3_workspace_bytes(int B, int H, int W, int C)
{
    if (B <= 0 || H <= 0 || W <= 0 || C <= 0 || (H & 1) || (W & 1)) return 0;
    const size_t n_out = (size_t)B * (H / 2) * (W / 2) * C;
    // per party: d1 (2 n_out), r1 (2 n_out), v (n_out), d2 (n_out); then the larger conversion's scratch
    return 3 * (2 * align_up(2 * n_out * 8) + 2 * align_up(n_out * 8)) + mpc_relu3_workspace_bytes(2 * n_out);
}

int mpc_maxpool3(mpc_ctx* c, mpc_cshare3 x, const mpc_relu3_material* mat1, const mpc_relu3_material* mat2,
                 mpc_share3 y, int B, int H, int W, int C)
{
    if (!c || B <= 0 || H <= 0 || W <= 0 || C <= 0 || (H & 1) || (W & 1)) return MPC_EINVAL;
    MPC_TRY(check_material3(mat1));
    MPC_TRY(check_material3(mat2));
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
    relu3_ws(c->ws + wa.off, c->ws_bytes - wa.off, 2 * n_out, &q1, &ok1);
    relu3_ws(c->ws + wa.off, c->ws_bytes - wa.off, n_out, &q2, &ok2);      // the second conversion reuses the scratch
    if (!ok1 || !ok2) return MPC_ENOMEM;
    fill3(q1, pq.d1, mat1, r1, nullptr, nullptr, 2 * n_out);
    fill3(q2, pq.d2, mat2, y.p, nullptr, nullptr, n_out);
    hipStream_t st = c->s[0];
    MPC_TRY(lane_join(c));
    MPC_TRY(launch_pool<0>(c, st, pq, n_out));       // first tournament level: max(p00, p01), max(p10, p11)
    MPC_TRY(relu3_run(c, st, q1));
    MPC_TRY(launch_pool<1>(c, st, pq, n_out));       // second level: the two winners
    MPC_TRY(relu3_run(c, st, q2));
    MPC_TRY(launch_pool<2>(c, st, pq, n_out));       // out = v + ReLU(u - v)
    return lane_fanout(c);
}

}  // extern "C"
