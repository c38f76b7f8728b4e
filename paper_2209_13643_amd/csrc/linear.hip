// Beaver-triple matmul / conv (Alg. 1, Eq. 3) and the inter-linear ordering
// of Alg. 3: host-side orchestration of mask kernels, wire copies, digit
// recoding and the limb GEMM on the lane's three streams.
#include "common.h"

namespace {

// Geometry of one secure linear layer seen as a GEMM.
struct LinearShape {
    bool conv;
    int M, K, N, batch;          // GEMM view (conv: M = B*Ho*Wo, K = KH*KW*Cin, batch = 1)
    // conv only
    int B, H, W, Cin, Cout, KH, KW, pad, stride, Ho, Wo, CB;
    // derived
    size_t nx, nw, nz;           // words in x / w / z per party (all batch items)
    bool transX, transY;         // matmul operands stored transposed ([K][M] / [N][K])
    bool wflip;                  // conv: filter stored [KH][KW][N][Cin'] and read in reverse tap order (input gradient)
    bool im2colT;                // left operand = transposed im2col of an NHWC tensor (filter gradient)
    int gB, gH, gW, gCin, gKH, gKW, gpad, gstride, gHo, gWo;    // geometry of that tensor
    int rowsL;                   // rows of a left plane (M, or B*H*W pixels + 1 zero row)
    int KB_L;                    // k blocks stored per left plane row
    int KB;                      // k blocks contracted per segment (even)
    size_t L_plane, R_plane;     // bytes of one digit plane (one batch item)
};

LinearShape shape_matmul(int M, int K, int N, int batch, int flags = 0)
{
    LinearShape s{};
    s.conv = false; s.M = M; s.K = K; s.N = N; s.batch = batch;
    s.transX = (flags & MPC_TRANS_X) != 0; s.transY = (flags & MPC_TRANS_Y) != 0;
    s.nx = (size_t)batch * M * K; s.nw = (size_t)batch * K * N; s.nz = (size_t)batch * M * N;
    s.rowsL = M; s.KB = kblocks(K); s.KB_L = s.KB;
    s.L_plane = plane_bytes(M, s.KB); s.R_plane = plane_bytes(N, s.KB);
    return s;
}

LinearShape shape_conv(int B, int H, int W, int Cin, int Cout, int KH, int KW, int pad, int stride)
{
    LinearShape s{};
    s.conv = true; s.B = B; s.H = H; s.W = W; s.Cin = Cin; s.Cout = Cout;
    s.KH = KH; s.KW = KW; s.pad = pad; s.stride = stride;
    s.Ho = (H + 2 * pad - KH) / stride + 1; s.Wo = (W + 2 * pad - KW) / stride + 1;
    s.CB = (Cin + 15) / 16;
    s.M = B * s.Ho * s.Wo; s.K = KH * KW * Cin; s.N = Cout; s.batch = 1;
    s.nx = (size_t)B * H * W * Cin; s.nw = (size_t)KH * KW * Cin * Cout; s.nz = (size_t)s.M * Cout;
    s.rowsL = B * H * W + 1; s.KB_L = s.CB;      // + the all-zero row that padding taps read
    s.KB = (KH * KW * s.CB + 1) & ~1;
    s.L_plane = plane_bytes(s.rowsL, s.KB_L); s.R_plane = plane_bytes(Cout, s.KB);
    return s;
}

// Input gradient of a stride-1 convolution with a square filter: itself a
// convolution of the output gradient [B][Ho][Wo][Cout] with the filter read
// in reverse tap order and with its channel roles swapped, padding KH-1-pad.
LinearShape shape_conv_grad_x(int B, int H, int W, int Cin, int Cout, int KH, int KW, int pad)
{
    const int Ho = H + 2 * pad - KH + 1, Wo = W + 2 * pad - KW + 1;
    LinearShape s = shape_conv(B, Ho, Wo, Cout, Cin, KH, KW, KH - 1 - pad, 1);
    s.wflip = true;
    return s;
}

// Strided convolutions: the input gradient is the stride-1 one of the output gradient
// with stride-1 zeros between its pixels (and as many zero rows / columns at the far
// edge as the forward pass left unused), so the same path serves after a scatter.
struct DilatedGeom { int Ho, Wo, Hd, Wd; size_t words; };
DilatedGeom dilated_geom(int B, int H, int W, int Cout, int KH, int KW, int pad, int stride)
{
    DilatedGeom d{};
    d.Ho = (H + 2 * pad - KH) / stride + 1; d.Wo = (W + 2 * pad - KW) / stride + 1;
    d.Hd = H + 2 * pad - KH + 1; d.Wd = W + 2 * pad - KW + 1;        // = (Ho-1)*stride + 1 + unused remainder
    d.words = (size_t)B * d.Hd * d.Wd * Cout;
    return d;
}

// Filter gradient: [KH*KW*Cin x B*Ho*Wo] (transposed im2col of x) times
// [B*Ho*Wo x Cout] (the output gradient as it is stored).
LinearShape shape_conv_grad_w(int B, int H, int W, int Cin, int Cout, int KH, int KW, int pad, int stride)
{
    const int Ho = (H + 2 * pad - KH) / stride + 1, Wo = (W + 2 * pad - KW) / stride + 1;
    LinearShape s = shape_matmul(KH * KW * Cin, B * Ho * Wo, Cout, 1);
    s.im2colT = true;
    s.gB = B; s.gH = H; s.gW = W; s.gCin = Cin; s.gKH = KH; s.gKW = KW; s.gpad = pad; s.gstride = stride;
    s.gHo = Ho; s.gWo = Wo;
    s.nx = (size_t)B * H * W * Cin;             // x and its mask keep their NHWC shape
    return s;
}

struct LinearWs {
    u64 *se[2], *re[2];        // masked x shares: sent / received
    u64 *sf[2], *rf[2];        // masked y shares
    u8 *pl_e, *pl_a[2];        // left digit planes
    u8 *pr_f, *pr_b[2];        // right digit planes
    u64* partial; int ksplit;  // split-contraction partial products
    size_t bytes; bool ok;
};

LinearWs carve(u8* base, size_t cap, const LinearShape& s, bool folded = false)
{
    WsAlloc w(base, cap);
    LinearWs r{};
    for (int i = 0; i < 2; ++i) { r.se[i] = w.take<u64>(s.nx); r.re[i] = w.take<u64>(s.nx); }
    for (int i = 0; i < 2; ++i) { r.sf[i] = w.take<u64>(s.nw); r.rf[i] = w.take<u64>(s.nw); }
    const size_t lp = 8 * s.L_plane * s.batch, rp = 8 * s.R_plane * s.batch;
    r.pl_e = w.take<u8>(lp); r.pl_a[0] = w.take<u8>(lp); r.pl_a[1] = w.take<u8>(lp);
    r.pr_f = w.take<u8>(rp); r.pr_b[0] = w.take<u8>(rp); r.pr_b[1] = w.take<u8>(rp);
    // the two-segment, two-party launch is the one that decides the split (folded: party 0 contracts one segment)
    r.ksplit = folded ? gemm_ksplit2(s.M, s.N, s.batch, s.KB / 2, 2 * s.KB / 2)
                      : gemm_ksplit(s.M, s.N, s.batch, 2, 2 * s.KB / 2);
    r.partial = r.ksplit > 1 ? w.take<u64>((size_t)r.ksplit * 2 * s.batch * s.M * s.N) : nullptr;
    r.bytes = w.off; r.ok = w.ok;
    return r;
}

RecodeArgs recode_left(const LinearShape& s, const u64* src, const u64* src2, u8* dst)
{
    RecodeArgs a{};
    a.src = src; a.src2 = src2; a.src3 = nullptr; a.dst = dst;
    a.k_stride = 1; a.tap_stride = 0; a.ntaps = 1; a.batch = s.batch;
    if (s.conv) { a.rows = s.rowsL - 1; a.plane_rows = s.rowsL; a.K = s.Cin; a.row_stride = s.Cin; a.KB_tap = s.CB; a.KB_total = s.CB; }
    else        { a.rows = s.M; a.plane_rows = s.M; a.K = s.K; a.row_stride = s.K; a.KB_tap = (s.K + 15) / 16; a.KB_total = s.KB; }
    if (s.transX) { a.row_stride = 1; a.k_stride = s.M; }       // stored [K][M]
    a.digit_stride = (long long)s.L_plane;
    a.src_batch_stride = (long long)s.M * s.K;          // unused for conv (batch == 1)
    a.dst_batch_stride = (long long)(8 * s.L_plane);
    return a;
}

// Left digit planes of up to three sources in one launch.
int launch_left(mpc_ctx* c, hipStream_t st, const LinearShape& s, int count,
                const u64* const src[], const u64* const src2[], u8* const dst[])
{
    if (s.im2colT) {
        Im2colTArgs t[3];
        for (int i = 0; i < count; ++i)
            t[i] = Im2colTArgs{ src[i], src2[i], dst[i], s.gB, s.gH, s.gW, s.gCin, s.gKH, s.gKW, s.gpad, s.gstride,
                                s.gHo, s.gWo, s.KB, (long long)s.L_plane };
        return launch_recode_im2col_t(c, st, t, count);
    }
    RecodeArgs r[3];
    for (int i = 0; i < count; ++i) r[i] = recode_left(s, src[i], src2[i], dst[i]);
    return count == 1 ? launch_recode(c, st, r[0]) : launch_recode_multi(c, st, r, count);
}
int launch_left1(mpc_ctx* c, hipStream_t st, const LinearShape& s, const u64* src, const u64* src2, u8* dst)
{
    const u64* a[1] = { src }; const u64* b[1] = { src2 }; u8* d[1] = { dst };
    return launch_left(c, st, s, 1, a, b, d);
}

RecodeArgs recode_right(const LinearShape& s, const u64* src, const u64* src2, const u64* src3, u8* dst)
{
    RecodeArgs a{};
    a.src = src; a.src2 = src2; a.src3 = src3; a.dst = dst;
    a.rows = s.N; a.plane_rows = s.N; a.row_stride = 1; a.k_stride = s.N; a.batch = s.batch;
    if (s.conv) { a.K = s.Cin; a.KB_tap = s.CB; a.ntaps = s.KH * s.KW; a.tap_stride = (long long)s.Cin * s.Cout; }
    else        { a.K = s.K; a.KB_tap = (s.K + 15) / 16; a.ntaps = 1; a.tap_stride = 0; }
    if (s.transY) { a.row_stride = s.K; a.k_stride = 1; }       // stored [N][K]
    if (s.wflip) {
        // stored [tap][n][k] (the forward filter [KH][KW][Cin][Cout] with n = Cin, k = Cout), taps reversed
        const long long tap_words = (long long)s.N * s.Cin;
        a.row_stride = s.Cin; a.k_stride = 1; a.tap_stride = -tap_words;
        const long long last = (long long)(s.KH * s.KW - 1) * tap_words;
        a.src = src + last; a.src2 = src2 ? src2 + last : nullptr; a.src3 = src3 ? src3 + last : nullptr;
    }
    a.KB_total = s.KB;
    a.digit_stride = (long long)s.R_plane;
    a.src_batch_stride = (long long)s.K * s.N;
    a.dst_batch_stride = (long long)(8 * s.R_plane);
    return a;
}

void fill_geom(const LinearShape& s, const LinearWs& w, GemmArgs& g)
{
    g.M = s.M; g.N = s.N; g.batch = s.batch;
    g.out_bstride = (long long)s.M * s.N;
    g.rows_L = s.rowsL;
    g.ksplit = w.ksplit; g.partial = w.partial;
    g.conv = ConvGeom{};
    if (s.conv) {
        g.conv.enabled = 1; g.conv.H = s.H; g.conv.W = s.W; g.conv.Ho = s.Ho; g.conv.Wo = s.Wo;
        g.conv.CB = s.CB; g.conv.KH = s.KH; g.conv.KW = s.KW; g.conv.pad = s.pad; g.conv.stride = s.stride;
        g.conv.npix = (long long)s.rowsL - 1;
    }
}

GemmSeg make_seg(const LinearShape& s, const u8* L, const u8* R)
{
    GemmSeg q{};
    q.L = L; q.R = R;
    q.L_dstride = (long long)s.L_plane; q.R_dstride = (long long)s.R_plane;
    q.L_bstride = (long long)(8 * s.L_plane); q.R_bstride = (long long)(8 * s.R_plane);
    q.KB = s.KB;
    return q;
}

int check_shape(const LinearShape& s)
{
    if (s.M <= 0 || s.K <= 0 || s.N <= 0 || s.batch <= 0) return MPC_EINVAL;
    if (s.conv) {
        if (s.B <= 0 || s.H <= 0 || s.W <= 0 || s.Cin <= 0 || s.Cout <= 0 || s.KH <= 0 || s.KW <= 0 ||
            s.pad < 0 || s.stride <= 0 || s.Ho <= 0 || s.Wo <= 0 || s.KH * s.KW > 64)
            return MPC_EINVAL;
        // the filter window must fit the padded image (C division would round a negative extent up to one output)
        if (s.H + 2 * s.pad < s.KH || s.W + 2 * s.pad < s.KW) return MPC_EINVAL;
        if ((long long)s.KH * s.KW * s.CB * 16 > MPC_MAX_K_TOTAL) return MPC_ERANGE;
    } else if (s.K > MPC_MAX_K_TOTAL) return MPC_ERANGE;
    if ((long long)s.M * s.N * s.batch > (1ll << 40)) return MPC_ERANGE;
    if ((long long)s.batch * 2 > 65535) return MPC_EINVAL;
    return MPC_OK;
}

// The whole secure linear layer.  See mpc_beaver_matmul in the public header.
int beaver_linear(mpc_ctx* c, const LinearShape& s, mpc_cshare x, mpc_cshare y,
                  mpc_cshare a, mpc_cshare b, mpc_cshare cc, mpc_share z,
                  const u64* f_public, int n_chunks, int flags, const u64* x_public = nullptr,
                  const u8* prep_right = nullptr, const u8* prep_left = nullptr, size_t ws_off = 0)
{
    if (!c) return MPC_EINVAL;
    MPC_TRY(check_shape(s));
    if (n_chunks < 1) return MPC_EINVAL;
    // prepared planes: digit planes of the input-independent operands, recoded ahead of time
    // folded triple: cc.p[0] holds c_0 - a_0 * b_0, and party 0 contracts (x_0 + e_1) against b_0 + f alone
    const bool folded = (flags & MPC_FOLDED) != 0;
    // folded product of two activations: y arrives as shares and f opens in this call, so of the right planes only
    // party 1's [b_1] can be prepared; those of f and of b_0 + f = y_0 + f_1 are recoded here
    const bool right_online = folded && prep_right != nullptr && y.p[0] != nullptr && y.p[1] != nullptr;
    const bool skip_right = prep_right != nullptr && !right_online, skip_left = prep_left != nullptr;
    if (folded && (!(skip_right || right_online) || !skip_left || x_public || (flags & MPC_TWO_PHASE))) return MPC_EINVAL;
    if (right_online && f_public) return MPC_EINVAL;
    for (int i = 0; i < 2; ++i) {
        if (!a.p[i] || !cc.p[i] || !z.p[i]) return MPC_EINVAL;
        if (!skip_right && !b.p[i]) return MPC_EINVAL;
        if (!x_public && !x.p[i]) return MPC_EINVAL;
        if (!skip_right && !f_public && !y.p[i]) return MPC_EINVAL;
    }
    if ((prep_right && ((uintptr_t)prep_right & 15)) || (skip_left && ((uintptr_t)prep_left & 15))) return MPC_EINVAL;
    if (ws_off > c->ws_bytes) return MPC_ENOMEM;
    LinearWs w = carve(c->ws ? c->ws + ws_off : nullptr, c->ws_bytes - ws_off, s, folded);
    if (!w.ok) return MPC_ENOMEM;
    if (skip_right) {
        const size_t rp = align_up(8 * s.R_plane * s.batch);
        w.pr_f = const_cast<u8*>(prep_right); w.pr_b[0] = w.pr_f + rp; w.pr_b[1] = w.pr_f + 2 * rp;
    }
    if (right_online) w.pr_b[1] = const_cast<u8*>(prep_right) + 2 * align_up(8 * s.R_plane * s.batch);
    if (skip_left) {
        const size_t lp = align_up(8 * s.L_plane * s.batch);
        // folded: the workspace slot of a_0's planes receives the planes of x_0 + e_1 instead
        if (!folded) w.pl_a[0] = const_cast<u8*>(prep_left);
        w.pl_a[1] = const_cast<u8*>(prep_left) + lp;
    }
    const bool have_f = f_public != nullptr || skip_right;     // the weight mask needs no exchange in this call

    hipStream_t P0 = c->s[0], P1 = c->s[1], Wr = c->s[2];
    hipStream_t P[2] = { P0, P1 };
    const bool two_phase = (flags & MPC_TWO_PHASE) != 0;
    const int trunc = (flags & MPC_TRUNCATE) ? c->frac_bits : 0;

    MPC_TRY(lane_join(c));
    const int pi = prof_begin(c, MPC_PROF_LINEAR, P0);

    if (P0 == P1 && P1 == Wr) {
        // One in-order queue: same steps, same order, but jobs of equal kind share a launch.
        GemmArgs g{};
        fill_geom(s, w, g);
        g.nparty = 2;
        if (folded && c->exchange_put && !s.im2colT) {
            // Folded call with the exchange by remote store: three passes over the activation, each word touched once.
            //   party 0 masks and sends:           e_0 = x_0 - a_0                  -> party 1's receive buffer
            //   party 1 masks, sends and recodes:  e_1 = x_1 - a_1 -> party 0's receive buffer; planes of e = e_1 + e_0
            //   party 0 recodes:                   planes of a_0 + e = x_0 + e_1
            // (party 1's word leaves after party 0's has arrived: on a network the two directions of this exchange
            // would follow each other; with the copy exchange they stay simultaneous.)
            // A product of two activations opens f the same way, in the same three launches:
            //   f_0 = y_0 - b_0 -> party 1;  f_1 = y_1 - b_1 -> party 0 and planes of f;  planes of b_0 + f = y_0 + f_1.
            SubSeg sub0[2] = { SubSeg{ x.p[0], a.p[0], w.re[1], s.nx, 0, nullptr },
                               SubSeg{ y.p[0], b.p[0], w.rf[1], s.nw, 0, nullptr } };
            MPC_TRY(launch_sub_multi(c, P0, sub0, right_online ? 2 : 1));
            RecodeArgs r1[2] = { recode_left(s, x.p[1], w.re[1], w.pl_e), RecodeArgs{} };
            r1[0].sub = a.p[1]; r1[0].side = w.re[0];
            RecodeArgs r0[2] = { recode_left(s, x.p[0], w.re[0], w.pl_a[0]), RecodeArgs{} };
            if (right_online) {
                r1[1] = recode_right(s, y.p[1], w.rf[1], nullptr, w.pr_f);
                r1[1].sub = b.p[1]; r1[1].side = w.rf[0];
                r0[1] = recode_right(s, y.p[0], w.rf[0], nullptr, w.pr_b[0]);
                MPC_TRY(launch_recode_any(c, P0, r1, 2));
                MPC_TRY(launch_recode_any(c, P0, r0, 2));
            } else {
                MPC_TRY(launch_recode(c, P0, r1[0]));
                MPC_TRY(launch_recode(c, P0, r0[0]));
            }
            g.nseg = 2;
            g.seg[0][0] = make_seg(s, w.pl_a[0], w.pr_b[0]); g.seg[0][1] = GemmSeg{};
            g.seg[1][0] = make_seg(s, w.pl_e, w.pr_b[1]);    g.seg[1][1] = make_seg(s, w.pl_a[1], w.pr_f);
            for (int i = 0; i < 2; ++i) { g.addend[i] = cc.p[i]; g.addend2[i] = nullptr; g.out[i] = z.p[i]; }
            g.trunc_bits = trunc;
            MPC_TRY(launch_limb_gemm(c, P0, g));
            prof_end(c, MPC_PROF_LINEAR, pi, P0);
            return MPC_OK;
        }
        if (c->exchange_put && !folded && !skip_left && !x_public && !s.im2colT && !(two_phase && have_f)) {
            // Plain call with the exchange by remote store: the pass that recodes the triple's [a_i] forms the masked
            // shares on the way (e_i = x_i - a_i, stored into the peer's receive buffer), and the opened e is recoded
            // from party 0's own shares and the word it received: every activation word is read once per use.
            if (!have_f) {
                SubSeg sub[2];
                for (int i = 0; i < 2; ++i) sub[i] = SubSeg{ y.p[i], b.p[i], w.sf[i], s.nw, 0, w.rf[1 - i] };
                MPC_TRY(launch_sub_multi(c, P0, sub, 2));
            }
            RecodeArgs k1[3]; int n1 = 0;
            for (int i = 0; i < 2; ++i) {
                k1[n1] = recode_left(s, a.p[i], nullptr, w.pl_a[i]);
                k1[n1].minuend = x.p[i]; k1[n1].side = w.re[1 - i];
                ++n1;
            }
            if (!skip_right) k1[n1++] = recode_right(s, b.p[1], nullptr, nullptr, w.pr_b[1]);
            MPC_TRY(launch_recode_any(c, P0, k1, n1));
            RecodeArgs k2[3]; int n2 = 0;
            k2[n2] = recode_left(s, x.p[0], w.re[0], w.pl_e);
            k2[n2].sub = a.p[0];
            ++n2;
            if (!skip_right) {
                const u64* f0 = f_public ? f_public : w.sf[0];
                const u64* f1 = f_public ? nullptr : w.rf[0];
                k2[n2++] = recode_right(s, f0, f1, nullptr, w.pr_f);
                k2[n2++] = recode_right(s, b.p[0], f0, f1, w.pr_b[0]);
            }
            MPC_TRY(launch_recode_any(c, P0, k2, n2));
            g.nseg = 2;
            for (int i = 0; i < 2; ++i) {
                g.seg[i][0] = make_seg(s, w.pl_e, w.pr_b[i]);
                g.seg[i][1] = make_seg(s, w.pl_a[i], w.pr_f);
                g.addend[i] = cc.p[i]; g.addend2[i] = nullptr; g.out[i] = z.p[i];
            }
            g.trunc_bits = trunc;
            MPC_TRY(launch_limb_gemm(c, P0, g));
            prof_end(c, MPC_PROF_LINEAR, pi, P0);
            return MPC_OK;
        }
        if ((size_t)n_chunks > s.nx) n_chunks = (int)s.nx;
        bool f_pending = !have_f;                            // the weight mask rides with the first launch issued
        for (int ch = 0; ch < n_chunks; ++ch) {
            size_t lo = (s.nx * ch / n_chunks) & ~(size_t)1, hi = (s.nx * (ch + 1) / n_chunks) & ~(size_t)1;
            if (ch == n_chunks - 1) hi = s.nx;
            const bool last = ch == n_chunks - 1;
            SubSeg sub[4]; CopySeg cp[4]; int ns = 0;
            for (int i = 0; i < 2 && !x_public && hi > lo; ++i) {
                sub[ns] = SubSeg{ x.p[i] + lo, a.p[i] + lo, w.se[i] + lo, hi - lo, 0,
                                  c->exchange_put ? w.re[1 - i] + lo : nullptr };
                cp[ns] = CopySeg{ (const u8*)(w.se[i] + lo), (u8*)(w.re[1 - i] + lo), (hi - lo) * sizeof(u64), 0 };
                ++ns;
            }
            // an empty chunk (fewer than two words per chunk) issues nothing; the weight mask must not depend on it
            if (f_pending && (ns > 0 || last)) {
                for (int i = 0; i < 2; ++i) {
                    sub[ns] = SubSeg{ y.p[i], b.p[i], w.sf[i], s.nw, 0, c->exchange_put ? w.rf[1 - i] : nullptr };
                    cp[ns] = CopySeg{ (const u8*)w.sf[i], (u8*)w.rf[1 - i], s.nw * sizeof(u64), 0 };
                    ++ns;
                }
                f_pending = false;
            }
            if (ns == 0) continue;                           // empty chunk, or both operands were opened ahead of time
            MPC_TRY(launch_sub_multi(c, P0, sub, ns));       // Alg. 1: mask (and, by remote store, send)
            if (!c->exchange_put) MPC_TRY(launch_copy_multi(c, P0, cp, ns));       // Alg. 1: exchange
        }
        const u64* f0 = f_public ? f_public : w.sf[0];
        const u64* f1 = f_public ? nullptr : w.rf[0];
        RecodeArgs rr[6];
        const u64* lsrc[3] = { a.p[0], a.p[1], x_public ? x_public : w.se[0] };
        const u64* lsrc2[3] = { nullptr, nullptr, x_public ? nullptr : w.re[0] };
        u8* ldst[3] = { w.pl_a[0], w.pl_a[1], w.pl_e };
        if (folded) {
            // party 0: a_0 + e = x_0 + e_1 (own share + received word); party 1: e from its own and the received word
            lsrc[1] = x.p[0]; lsrc2[1] = w.re[0]; ldst[1] = w.pl_a[0];
            lsrc[2] = w.se[1]; lsrc2[2] = w.re[1];
        }
        // all digit planes of the call in one launch (the transposed-im2col recoder is a kernel of its own)
        int nr = 0;
        const int l0 = folded ? 1 : skip_left ? 2 : 0;
        if (s.im2colT) {
            MPC_TRY(launch_left(c, P0, s, 3 - l0, lsrc + l0, lsrc2 + l0, ldst + l0));
        } else {
            for (int i = l0; i < 3; ++i) rr[nr++] = recode_left(s, lsrc[i], lsrc2[i], ldst[i]);
        }
        if (!skip_right) {
            if (!right_online) rr[nr++] = recode_right(s, b.p[1], nullptr, nullptr, w.pr_b[1]);
            rr[nr++] = recode_right(s, f0, f1, nullptr, w.pr_f);
            rr[nr++] = recode_right(s, b.p[0], f0, f1, w.pr_b[0]);
        }
        if (nr) MPC_TRY(launch_recode_any(c, P0, rr, nr));
        if (two_phase && have_f) {
            g.nseg = 1;
            for (int i = 0; i < 2; ++i) {
                g.seg[i][0] = make_seg(s, w.pl_a[i], w.pr_f);
                g.addend[i] = nullptr; g.addend2[i] = nullptr; g.out[i] = z.p[i];
            }
            g.trunc_bits = 0;
            MPC_TRY(launch_limb_gemm(c, P0, g));
            for (int i = 0; i < 2; ++i) {
                g.seg[i][0] = make_seg(s, w.pl_e, w.pr_b[i]);
                g.addend[i] = cc.p[i]; g.addend2[i] = z.p[i];
            }
            g.trunc_bits = trunc;
            MPC_TRY(launch_limb_gemm(c, P0, g));
        } else {
            g.nseg = 2;
            for (int i = 0; i < 2; ++i) {
                g.seg[i][0] = make_seg(s, w.pl_e, w.pr_b[i]);
                g.seg[i][1] = make_seg(s, w.pl_a[i], w.pr_f);
                g.addend[i] = cc.p[i]; g.addend2[i] = nullptr; g.out[i] = z.p[i];
            }
            if (folded) {
                // z_0 = (c_0 - a_0 b_0) + (a_0 + e)(b_0 + f): one product; party 1 as ever
                g.seg[0][0] = make_seg(s, w.pl_a[0], w.pr_b[0]);
                g.seg[0][1] = GemmSeg{};
            }
            g.trunc_bits = trunc;
            MPC_TRY(launch_limb_gemm(c, P0, g));
        }
        prof_end(c, MPC_PROF_LINEAR, pi, P0);
        return MPC_OK;
    }

    // -- Alg. 1 / Alg. 3, masking step: mask and start the exchange, chunk by chunk
    if (!have_f) {
        for (int i = 0; i < 2; ++i) {
            MPC_TRY(launch_sub(c, P[i], y.p[i], b.p[i], w.sf[i], s.nw));
            MPC_TRY(chain(c, P[i], Wr));
        }
        for (int i = 0; i < 2; ++i)
            MPC_TRY(launch_copy(c, Wr, w.sf[i], w.rf[1 - i], s.nw * sizeof(u64)));
    }
    if ((size_t)n_chunks > s.nx) n_chunks = (int)s.nx;
    for (int ch = 0; ch < n_chunks; ++ch) {
        // contiguous word ranges, 2-word aligned so the 16-byte paths stay usable
        size_t lo = (s.nx * ch / n_chunks) & ~(size_t)1, hi = (s.nx * (ch + 1) / n_chunks) & ~(size_t)1;
        if (ch == n_chunks - 1) hi = s.nx;
        if (hi <= lo) continue;
        if (x_public) break;
        for (int i = 0; i < 2; ++i) {
            MPC_TRY(launch_sub(c, P[i], x.p[i] + lo, a.p[i] + lo, w.se[i] + lo, hi - lo));
            MPC_TRY(chain(c, P[i], Wr));
        }
        for (int i = 0; i < 2; ++i)
            MPC_TRY(launch_copy(c, Wr, w.se[i] + lo, w.re[1 - i] + lo, (hi - lo) * sizeof(u64)));
    }
    const u64* e_src = x_public ? x_public : w.se[0];
    const u64* e_src2 = x_public ? nullptr : w.re[0];

    if (folded) {
        // after the exchange each party recodes what it contracts: party 0 the planes of x_0 + e_1,
        // party 1 those of e; then the joint launch, party 0 with one segment
        MPC_TRY(chain(c, Wr, P0));
        MPC_TRY(chain(c, Wr, P1));
        MPC_TRY(launch_left1(c, P0, s, x.p[0], w.re[0], w.pl_a[0]));
        MPC_TRY(launch_left1(c, P1, s, w.se[1], w.re[1], w.pl_e));
        if (right_online) {
            // f opened in this call: party 0 recodes b_0 + f, party 1 f, each from its own and the received word
            MPC_TRY(launch_recode(c, P0, recode_right(s, b.p[0], w.sf[0], w.rf[0], w.pr_b[0])));
            MPC_TRY(launch_recode(c, P1, recode_right(s, w.sf[1], w.rf[1], nullptr, w.pr_f)));
        }
        MPC_TRY(chain(c, P1, P0));
        GemmArgs g{};
        fill_geom(s, w, g);
        g.nparty = 2; g.nseg = 2;
        g.seg[0][0] = make_seg(s, w.pl_a[0], w.pr_b[0]); g.seg[0][1] = GemmSeg{};
        g.seg[1][0] = make_seg(s, w.pl_e, w.pr_b[1]);    g.seg[1][1] = make_seg(s, w.pl_a[1], w.pr_f);
        for (int i = 0; i < 2; ++i) { g.addend[i] = cc.p[i]; g.addend2[i] = nullptr; g.out[i] = z.p[i]; }
        g.trunc_bits = trunc;
        MPC_TRY(launch_limb_gemm(c, P0, g));
        prof_end(c, MPC_PROF_LINEAR, pi, P0);
        MPC_TRY(chain(c, P0, P1));
        return MPC_OK;
    }

    // -- digit planes that do not depend on the exchange: [a_i] (and b_1)
    for (int i = 0; i < 2 && !skip_left; ++i)
        MPC_TRY(launch_left1(c, P[i], s, a.p[i], nullptr, w.pl_a[i]));
    if (!skip_right) MPC_TRY(launch_recode(c, P1, recode_right(s, b.p[1], nullptr, nullptr, w.pr_b[1])));

    GemmArgs g{};
    fill_geom(s, w, g);
    g.nparty = 2;

    if (two_phase && have_f) {
        // Alg. 3, first product: epsilon is already here; z_i = Conv([a_i], epsilon)
        // runs while the masked inputs are still crossing the wire.
        if (!skip_right) {
            MPC_TRY(launch_recode(c, P0, recode_right(s, f_public, nullptr, nullptr, w.pr_f)));
            MPC_TRY(launch_recode(c, P0, recode_right(s, b.p[0], f_public, nullptr, w.pr_b[0])));
        }
        MPC_TRY(chain(c, P1, P0));
        g.nseg = 1;
        for (int i = 0; i < 2; ++i) {
            g.seg[i][0] = make_seg(s, w.pl_a[i], w.pr_f);
            g.addend[i] = nullptr; g.addend2[i] = nullptr; g.out[i] = z.p[i];
        }
        g.trunc_bits = 0;
        MPC_TRY(launch_limb_gemm(c, P0, g));
        // Alg. 3, after the wait for Delta: add [c_i] + Conv(Delta, [b_i]) (+ Conv(Delta, epsilon))
        MPC_TRY(chain(c, Wr, P0));
        MPC_TRY(launch_left1(c, P0, s, e_src, e_src2, w.pl_e));
        for (int i = 0; i < 2; ++i) {
            g.seg[i][0] = make_seg(s, w.pl_e, w.pr_b[i]);
            g.addend[i] = cc.p[i]; g.addend2[i] = z.p[i];
        }
        g.trunc_bits = trunc;
        MPC_TRY(launch_limb_gemm(c, P0, g));
    } else {
        // Alg. 1 after the masking step: wait for the exchange, open, one fused contraction
        // [e | a_i] x [b_i (+ f for party 0) ; f] per party.
        MPC_TRY(chain(c, Wr, P0));
        MPC_TRY(launch_left1(c, P0, s, e_src, e_src2, w.pl_e));
        if (skip_right) {
            // the right-operand planes were recoded ahead of time
        } else if (f_public) {
            MPC_TRY(launch_recode(c, P0, recode_right(s, f_public, nullptr, nullptr, w.pr_f)));
            MPC_TRY(launch_recode(c, P0, recode_right(s, b.p[0], f_public, nullptr, w.pr_b[0])));
        } else {
            MPC_TRY(launch_recode(c, P0, recode_right(s, w.sf[0], w.rf[0], nullptr, w.pr_f)));
            MPC_TRY(launch_recode(c, P0, recode_right(s, b.p[0], w.sf[0], w.rf[0], w.pr_b[0])));
        }
        MPC_TRY(chain(c, P1, P0));
        g.nseg = 2;
        for (int i = 0; i < 2; ++i) {
            g.seg[i][0] = make_seg(s, w.pl_e, w.pr_b[i]);
            g.seg[i][1] = make_seg(s, w.pl_a[i], w.pr_f);
            g.addend[i] = cc.p[i]; g.addend2[i] = nullptr; g.out[i] = z.p[i];
        }
        g.trunc_bits = trunc;
        MPC_TRY(launch_limb_gemm(c, P0, g));
    }
    prof_end(c, MPC_PROF_LINEAR, pi, P0);
    // party 1's output was produced by the joint launch on party 0's stream
    MPC_TRY(chain(c, P0, P1));
    return MPC_OK;
}

// ---- three parties -------------------------------------------------------------
struct LinearWs3 {
    u64 *se[3], *re[3][2];     // masked x shares: own, and as received from party+1 / party+2
    u64 *sf[3], *rf[3][2];     // masked y shares
    u64 *e_pub, *f_pub;        // opened e, f
    u8 *pl_e, *pl_a[3];
    u8 *pr_f, *pr_b[3];        // pr_b[0] holds b_0 + f
    LinearWs g;                // split count and partial products for the GEMM launches
    size_t bytes; bool ok;
};

LinearWs3 carve3(u8* base, size_t cap, const LinearShape& s)
{
    WsAlloc w(base, cap);
    LinearWs3 r{};
    for (int i = 0; i < 3; ++i) { r.se[i] = w.take<u64>(s.nx); r.re[i][0] = w.take<u64>(s.nx); r.re[i][1] = w.take<u64>(s.nx); }
    for (int i = 0; i < 3; ++i) { r.sf[i] = w.take<u64>(s.nw); r.rf[i][0] = w.take<u64>(s.nw); r.rf[i][1] = w.take<u64>(s.nw); }
    r.e_pub = w.take<u64>(s.nx); r.f_pub = w.take<u64>(s.nw);
    const size_t lp = 8 * s.L_plane * s.batch, rp = 8 * s.R_plane * s.batch;
    r.pl_e = w.take<u8>(lp); for (int i = 0; i < 3; ++i) r.pl_a[i] = w.take<u8>(lp);
    r.pr_f = w.take<u8>(rp); for (int i = 0; i < 3; ++i) r.pr_b[i] = w.take<u8>(rp);
    r.g.ksplit = gemm_ksplit(s.M, s.N, s.batch, 2, 2 * s.KB / 2);
    r.g.partial = r.g.ksplit > 1 ? w.take<u64>((size_t)r.g.ksplit * 2 * s.batch * s.M * s.N) : nullptr;
    r.bytes = w.off; r.ok = w.ok;
    return r;
}

// Alg. 1 / Eq. 3 with three parties, everything on the lane's first stream:
// mask, broadcast to both peers, open e and f, recode, then the two-segment
// contraction [e | a_i] x [b_i (+ f for party 0) ; f] for parties 0 and 1 in
// one launch and for party 2 in a second one.
int beaver_linear3(mpc_ctx* c, const LinearShape& s, mpc_cshare3 x, mpc_cshare3 y,
                   mpc_cshare3 a, mpc_cshare3 b, mpc_cshare3 cc, mpc_share3 z, const u64* f_public, size_t ws_off = 0,
                   const u8* prep_right = nullptr, const u8* prep_left = nullptr)
{
    if (!c) return MPC_EINVAL;
    MPC_TRY(check_shape(s));
    // prepared planes: digit planes of the input-independent operands, recoded ahead of time
    const bool skip_right = prep_right != nullptr, skip_left = prep_left != nullptr;
    for (int i = 0; i < 3; ++i) {
        if (!x.p[i] || !a.p[i] || !cc.p[i] || !z.p[i]) return MPC_EINVAL;
        if (!skip_right && !b.p[i]) return MPC_EINVAL;
        if (!skip_right && !f_public && !y.p[i]) return MPC_EINVAL;
    }
    if ((skip_right && ((uintptr_t)prep_right & 15)) || (skip_left && ((uintptr_t)prep_left & 15))) return MPC_EINVAL;
    if (ws_off > c->ws_bytes) return MPC_ENOMEM;
    LinearWs3 w = carve3(c->ws ? c->ws + ws_off : nullptr, c->ws_bytes - ws_off, s);
    if (!w.ok) return MPC_ENOMEM;
    if (skip_right) {
        const size_t rp = align_up(8 * s.R_plane * s.batch);
        w.pr_f = const_cast<u8*>(prep_right);
        for (int i = 0; i < 3; ++i) w.pr_b[i] = w.pr_f + (size_t)(i + 1) * rp;
    }
    if (skip_left) {
        const size_t lp = align_up(8 * s.L_plane * s.batch);
        for (int i = 0; i < 3; ++i) w.pl_a[i] = const_cast<u8*>(prep_left) + (size_t)i * lp;
    }
    const bool have_f = f_public != nullptr || skip_right;
    hipStream_t st = c->s[0];
    MPC_TRY(lane_join(c));
    const int pi = prof_begin(c, MPC_PROF_LINEAR, st);

    // Alg. 1: every party masks its shares ...
    SubSeg sub[6]; int ns = 0;
    for (int i = 0; i < 3; ++i) sub[ns++] = SubSeg{ x.p[i], a.p[i], w.se[i], s.nx, 0, nullptr };
    for (int i = 0; i < 3 && !have_f; ++i) sub[ns++] = SubSeg{ y.p[i], b.p[i], w.sf[i], s.nw, 0, nullptr };
    MPC_TRY(launch_sub_multi(c, st, sub, ns));
    // ... and broadcasts them: party i receives from party i+1 and party i+2
    CopySeg cp[6];
    for (int i = 0; i < 3; ++i)
        for (int k = 0; k < 2; ++k)
            cp[2 * i + k] = CopySeg{ (const u8*)w.se[(i + 1 + k) % 3], (u8*)w.re[i][k], s.nx * sizeof(u64), 0 };
    MPC_TRY(launch_copy_multi(c, st, cp, 6));
    if (!have_f) {
        for (int i = 0; i < 3; ++i)
            for (int k = 0; k < 2; ++k)
                cp[2 * i + k] = CopySeg{ (const u8*)w.sf[(i + 1 + k) % 3], (u8*)w.rf[i][k], s.nw * sizeof(u64), 0 };
        MPC_TRY(launch_copy_multi(c, st, cp, 6));
    }
    // Delta and epsilon (all parties hold the same three words; formed once, from party 0's buffers)
    MPC_TRY(launch_sum3(c, st, w.se[0], w.re[0][0], w.re[0][1], w.e_pub, s.nx));
    const u64* f = f_public;
    if (!have_f) { MPC_TRY(launch_sum3(c, st, w.sf[0], w.rf[0][0], w.rf[0][1], w.f_pub, s.nw)); f = w.f_pub; }

    // digit planes
    {
        if (!skip_left) {
            const u64* src[3] = { a.p[0], a.p[1], a.p[2] };
            const u64* none[3] = { nullptr, nullptr, nullptr };
            u8* dst[3] = { w.pl_a[0], w.pl_a[1], w.pl_a[2] };
            MPC_TRY(launch_left(c, st, s, 3, src, none, dst));
        }
        MPC_TRY(launch_left1(c, st, s, w.e_pub, nullptr, w.pl_e));
        if (!skip_right) {
            RecodeArgs rr[4];
            rr[0] = recode_right(s, b.p[1], nullptr, nullptr, w.pr_b[1]);
            rr[1] = recode_right(s, b.p[2], nullptr, nullptr, w.pr_b[2]);
            rr[2] = recode_right(s, f, nullptr, nullptr, w.pr_f);
            rr[3] = recode_right(s, b.p[0], f, nullptr, w.pr_b[0]);
            MPC_TRY(launch_recode_multi(c, st, rr, 4));
        }
    }

    GemmArgs g{};
    fill_geom(s, w.g, g);
    g.nseg = 2; g.trunc_bits = 0;
    g.nparty = 2;
    for (int i = 0; i < 2; ++i) {
        g.seg[i][0] = make_seg(s, w.pl_e, w.pr_b[i]);
        g.seg[i][1] = make_seg(s, w.pl_a[i], w.pr_f);
        g.addend[i] = cc.p[i]; g.addend2[i] = nullptr; g.out[i] = z.p[i];
    }
    MPC_TRY(launch_limb_gemm(c, st, g));
    g.nparty = 1;
    g.seg[0][0] = make_seg(s, w.pl_e, w.pr_b[2]);
    g.seg[0][1] = make_seg(s, w.pl_a[2], w.pr_f);
    g.addend[0] = cc.p[2]; g.out[0] = z.p[2];
    g.seg[1][0] = GemmSeg{}; g.seg[1][1] = GemmSeg{}; g.addend[1] = nullptr; g.out[1] = nullptr;
    MPC_TRY(launch_limb_gemm(c, st, g));
    prof_end(c, MPC_PROF_LINEAR, pi, st);
    return lane_fanout(c);
}

// Digit planes of the input-independent operands of a layer, recoded once:
// right = [f | b_0 + f | b_1] (needs the opened weight mask f), left = [a_0 | a_1].
void prepared_sizes(const LinearShape& s, size_t* right, size_t* left)
{
    if (right) *right = 3 * align_up(8 * s.R_plane * s.batch);
    if (left) *left = 2 * align_up(8 * s.L_plane * s.batch);
}

int prepare_planes(mpc_ctx* c, const LinearShape& s, mpc_cshare a, mpc_cshare b, const u64* f_public,
                   u8* right, u8* left)
{
    if (!c || (!right && !left)) return MPC_EINVAL;
    MPC_TRY(check_shape(s));
    // without f (a product of two activations, whose f opens online) only [b_1] can be recoded ahead of time
    if (right && (!b.p[1] || (f_public && !b.p[0]) || ((uintptr_t)right & 15))) return MPC_EINVAL;
    if (left && (!a.p[0] || !a.p[1] || ((uintptr_t)left & 15))) return MPC_EINVAL;
    hipStream_t P0 = c->s[0];
    MPC_TRY(lane_join(c));
    if (left) {
        const size_t lp = align_up(8 * s.L_plane * s.batch);
        const u64* src[2] = { a.p[0], a.p[1] }; const u64* src2[2] = { nullptr, nullptr };
        u8* dst[2] = { left, left + lp };
        MPC_TRY(launch_left(c, P0, s, 2, src, src2, dst));
    }
    if (right) {
        const size_t rp = align_up(8 * s.R_plane * s.batch);
        if (f_public) {
            RecodeArgs rr[3];
            rr[0] = recode_right(s, f_public, nullptr, nullptr, right);
            rr[1] = recode_right(s, b.p[0], f_public, nullptr, right + rp);
            rr[2] = recode_right(s, b.p[1], nullptr, nullptr, right + 2 * rp);
            MPC_TRY(launch_recode_multi(c, P0, rr, 3));
        } else {
            MPC_TRY(launch_recode(c, P0, recode_right(s, b.p[1], nullptr, nullptr, right + 2 * rp)));
        }
    }
    MPC_TRY(chain(c, P0, c->s[1]));
    return MPC_OK;
}

int ring_product(mpc_ctx* c, const LinearShape& s, const u64* L, const u64* R, u64* Z, size_t ws_off = 0)
{
    if (!c || !L || !R || !Z) return MPC_EINVAL;
    MPC_TRY(check_shape(s));
    if (ws_off > c->ws_bytes) return MPC_ENOMEM;
    LinearWs w = carve(c->ws ? c->ws + ws_off : nullptr, c->ws_bytes - ws_off, s);
    if (!w.ok) return MPC_ENOMEM;
    hipStream_t P0 = c->s[0];
    MPC_TRY(lane_join(c));
    MPC_TRY(launch_left1(c, P0, s, L, nullptr, w.pl_e));
    MPC_TRY(launch_recode(c, P0, recode_right(s, R, nullptr, nullptr, w.pr_f)));
    GemmArgs g{};
    fill_geom(s, w, g);
    g.nparty = 1; g.nseg = 1;
    g.seg[0][0] = make_seg(s, w.pl_e, w.pr_f);
    g.addend[0] = nullptr; g.addend2[0] = nullptr; g.out[0] = Z; g.trunc_bits = 0;
    MPC_TRY(launch_limb_gemm(c, P0, g));
    MPC_TRY(chain(c, P0, c->s[1]));
    return MPC_OK;
}

// Party 0's folded addend of a prepared layer: out = c_0 - a_0 * b_0 (a local, input-independent product).
int fold_addend(mpc_ctx* c, const LinearShape& s, const u64* a0, const u64* b0, const u64* c0, u64* out)
{
    if (!c || !a0 || !b0 || !c0 || !out) return MPC_EINVAL;
    MPC_TRY(ring_product(c, s, a0, b0, out));
    MPC_TRY(launch_sub(c, c->s[0], c0, out, out, s.nz));    // element-wise, in place: out = c_0 - out
    return chain(c, c->s[0], c->s[1]);
}

// Three parties: right = [f | b_0 + f | b_1 | b_2], left = [a_0 | a_1 | a_2].
void prepared_sizes3(const LinearShape& s, size_t* right, size_t* left)
{
    if (right) *right = 4 * align_up(8 * s.R_plane * s.batch);
    if (left) *left = 3 * align_up(8 * s.L_plane * s.batch);
}

int prepare_planes3(mpc_ctx* c, const LinearShape& s, mpc_cshare3 a, mpc_cshare3 b, const u64* f_public,
                    u8* right, u8* left)
{
    if (!c || (!right && !left)) return MPC_EINVAL;
    MPC_TRY(check_shape(s));
    if (right && (!f_public || !b.p[0] || !b.p[1] || !b.p[2] || ((uintptr_t)right & 15))) return MPC_EINVAL;
    if (left && (!a.p[0] || !a.p[1] || !a.p[2] || ((uintptr_t)left & 15))) return MPC_EINVAL;
    hipStream_t st = c->s[0];
    MPC_TRY(lane_join(c));
    if (left) {
        const size_t lp = align_up(8 * s.L_plane * s.batch);
        const u64* src[3] = { a.p[0], a.p[1], a.p[2] }; const u64* none[3] = { nullptr, nullptr, nullptr };
        u8* dst[3] = { left, left + lp, left + 2 * lp };
        MPC_TRY(launch_left(c, st, s, 3, src, none, dst));
    }
    if (right) {
        const size_t rp = align_up(8 * s.R_plane * s.batch);
        RecodeArgs rr[4];
        rr[0] = recode_right(s, f_public, nullptr, nullptr, right);
        rr[1] = recode_right(s, b.p[0], f_public, nullptr, right + rp);
        rr[2] = recode_right(s, b.p[1], nullptr, nullptr, right + 2 * rp);
        rr[3] = recode_right(s, b.p[2], nullptr, nullptr, right + 3 * rp);
        MPC_TRY(launch_recode_multi(c, st, rr, 4));
    }
    return lane_fanout(c);
}

}  // namespace

extern "C" {

size_t mpc_matmul_workspace_bytes(int M, int K, int N, int batch)
{
    LinearShape s = shape_matmul(M, K, N, batch);
    if (check_shape(s) != MPC_OK) return 0;
    // the folded prepared call may slice its contraction differently: the query covers both
    const size_t plain = carve(nullptr, 0, s).bytes, folded = carve(nullptr, 0, s, true).bytes;
    return plain > folded ? plain : folded;
}

size_t mpc_conv2d_workspace_bytes(int B, int H, int W, int Cin, int Cout, int KH, int KW, int pad, int stride)
{
    if (stride <= 0) return 0;
    LinearShape s = shape_conv(B, H, W, Cin, Cout, KH, KW, pad, stride);
    if (check_shape(s) != MPC_OK) return 0;
    const size_t plain = carve(nullptr, 0, s).bytes, folded = carve(nullptr, 0, s, true).bytes;
    return plain > folded ? plain : folded;
}

int mpc_beaver_matmul(mpc_ctx* ctx, mpc_cshare x, mpc_cshare y, mpc_cshare a, mpc_cshare b, mpc_cshare c,
                      mpc_share z, int M, int K, int N, int batch,
                      const uint64_t* f_public, int n_chunks, int flags)
{
    if (M <= 0 || K <= 0 || N <= 0 || batch <= 0) return MPC_EINVAL;
    return beaver_linear(ctx, shape_matmul(M, K, N, batch, flags), x, y, a, b, c, z, f_public, n_chunks, flags);
}

int mpc_matmul_prepared_bytes(int M, int K, int N, int batch, size_t* right, size_t* left)
{
    if (M <= 0 || K <= 0 || N <= 0 || batch <= 0) return MPC_EINVAL;
    LinearShape s = shape_matmul(M, K, N, batch);
    MPC_TRY(check_shape(s));
    prepared_sizes(s, right, left);
    return MPC_OK;
}

int mpc_conv2d_prepared_bytes(int B, int H, int W, int Cin, int Cout, int KH, int KW, int pad, int stride,
                              size_t* right, size_t* left)
{
    if (stride <= 0 || B <= 0 || H <= 0 || W <= 0 || Cin <= 0 || Cout <= 0 || KH <= 0 || KW <= 0 || pad < 0)
        return MPC_EINVAL;
    LinearShape s = shape_conv(B, H, W, Cin, Cout, KH, KW, pad, stride);
    MPC_TRY(check_shape(s));
    prepared_sizes(s, right, left);
    return MPC_OK;
}

int mpc_matmul_prepare(mpc_ctx* ctx, mpc_cshare a, mpc_cshare b, const uint64_t* f_public,
                       void* right_planes, void* left_planes, int M, int K, int N, int batch, int flags)
{
    if (M <= 0 || K <= 0 || N <= 0 || batch <= 0) return MPC_EINVAL;
    return prepare_planes(ctx, shape_matmul(M, K, N, batch, flags), a, b, f_public, (u8*)right_planes, (u8*)left_planes);
}

int mpc_conv2d_prepare(mpc_ctx* ctx, mpc_cshare a, mpc_cshare b, const uint64_t* f_public,
                       void* right_planes, void* left_planes,
                       int B, int H, int W, int Cin, int Cout, int KH, int KW, int pad, int stride)
{
    if (stride <= 0 || B <= 0 || H <= 0 || W <= 0 || Cin <= 0 || Cout <= 0 || KH <= 0 || KW <= 0 || pad < 0)
        return MPC_EINVAL;
    return prepare_planes(ctx, shape_conv(B, H, W, Cin, Cout, KH, KW, pad, stride), a, b, f_public,
                          (u8*)right_planes, (u8*)left_planes);
}

int mpc_beaver_matmul_prepared(mpc_ctx* ctx, mpc_cshare x, mpc_cshare a, mpc_cshare c, mpc_share z,
                               const void* right_planes, const void* left_planes,
                               int M, int K, int N, int batch, int n_chunks, int flags)
{
    if (M <= 0 || K <= 0 || N <= 0 || batch <= 0 || !right_planes) return MPC_EINVAL;
    const mpc_cshare none = { { nullptr, nullptr } };
    return beaver_linear(ctx, shape_matmul(M, K, N, batch, flags), x, none, a, none, c, z, nullptr, n_chunks, flags,
                         nullptr, (const u8*)right_planes, (const u8*)left_planes);
}

int mpc_beaver_matmul_folded(mpc_ctx* ctx, mpc_cshare x, mpc_cshare y, mpc_cshare a, mpc_cshare b, mpc_cshare c,
                             mpc_share z, const void* right_planes, const void* left_planes,
                             int M, int K, int N, int batch, int n_chunks, int flags)
{
    if (M <= 0 || K <= 0 || N <= 0 || batch <= 0 || !right_planes || !left_planes || !y.p[0] || !y.p[1] ||
        !b.p[0] || !b.p[1])
        return MPC_EINVAL;
    return beaver_linear(ctx, shape_matmul(M, K, N, batch, flags), x, y, a, b, c, z, nullptr, n_chunks,
                         flags | MPC_FOLDED, nullptr, (const u8*)right_planes, (const u8*)left_planes);
}

int mpc_conv2d_prepared(mpc_ctx* ctx, mpc_cshare x, mpc_cshare a, mpc_cshare c, mpc_share z,
                        const void* right_planes, const void* left_planes,
                        int B, int H, int W, int Cin, int Cout, int KH, int KW, int pad, int stride,
                        int n_chunks, int flags)
{
    if (stride <= 0 || B <= 0 || H <= 0 || W <= 0 || Cin <= 0 || Cout <= 0 || KH <= 0 || KW <= 0 || pad < 0 ||
        !right_planes || (flags & (MPC_TRANS_X | MPC_TRANS_Y)))
        return MPC_EINVAL;
    const mpc_cshare none = { { nullptr, nullptr } };
    return beaver_linear(ctx, shape_conv(B, H, W, Cin, Cout, KH, KW, pad, stride), x, none, a, none, c, z,
                         nullptr, n_chunks, flags, nullptr, (const u8*)right_planes, (const u8*)left_planes);
}

int mpc_matmul_fold(mpc_ctx* ctx, const uint64_t* a0, const uint64_t* b0, const uint64_t* c0, uint64_t* c0_folded,
                    int M, int K, int N, int batch, int flags)
{
    if (M <= 0 || K <= 0 || N <= 0 || batch <= 0 || (flags & ~(MPC_TRANS_X | MPC_TRANS_Y))) return MPC_EINVAL;
    return fold_addend(ctx, shape_matmul(M, K, N, batch, flags), a0, b0, c0, c0_folded);
}

int mpc_conv2d_fold(mpc_ctx* ctx, const uint64_t* a0, const uint64_t* b0, const uint64_t* c0, uint64_t* c0_folded,
                    int B, int H, int W, int Cin, int Cout, int KH, int KW, int pad, int stride)
{
    if (stride <= 0 || B <= 0 || H <= 0 || W <= 0 || Cin <= 0 || Cout <= 0 || KH <= 0 || KW <= 0 || pad < 0)
        return MPC_EINVAL;
    return fold_addend(ctx, shape_conv(B, H, W, Cin, Cout, KH, KW, pad, stride), a0, b0, c0, c0_folded);
}

size_t mpc_conv2d_grad_x_workspace_bytes(int B, int H, int W, int Cin, int Cout, int KH, int KW, int pad, int stride)
{
    if (stride <= 0 || KH != KW || KH <= 0 || pad < 0 || pad > KH - 1 || H + 2 * pad - KH < 0 || W + 2 * pad - KW < 0) return 0;
    LinearShape s = shape_conv_grad_x(B, H, W, Cin, Cout, KH, KW, pad);
    if (check_shape(s) != MPC_OK) return 0;
    // a strided layer first scatters g_i and its mask a_i (both parties) into the dilated grid
    const size_t extra = stride > 1 ? 4 * align_up(dilated_geom(B, H, W, Cout, KH, KW, pad, stride).words * sizeof(u64)) : 0;
    return extra + carve(nullptr, 0, s).bytes;
}

size_t mpc_conv2d_grad_w_workspace_bytes(int B, int H, int W, int Cin, int Cout, int KH, int KW, int pad, int stride)
{
    if (stride <= 0 || KH <= 0 || KW <= 0 || pad < 0 || H + 2 * pad - KH < 0 || W + 2 * pad - KW < 0) return 0;
    LinearShape s = shape_conv_grad_w(B, H, W, Cin, Cout, KH, KW, pad, stride);
    if (check_shape(s) != MPC_OK) return 0;
    return carve(nullptr, 0, s).bytes;
}

int mpc_conv2d_grad_x(mpc_ctx* ctx, mpc_cshare g, mpc_cshare w, mpc_cshare a, mpc_cshare b, mpc_cshare c,
                      mpc_share gx, int B, int H, int W, int Cin, int Cout, int KH, int KW, int pad, int stride,
                      const uint64_t* f_public, int n_chunks, int flags)
{
    if (!ctx || B <= 0 || H <= 0 || W <= 0 || Cin <= 0 || Cout <= 0 || KH <= 0 || KW <= 0 || pad < 0 || stride <= 0) return MPC_EINVAL;
    if (KH != KW || pad > KH - 1 || H + 2 * pad - KH < 0 || W + 2 * pad - KW < 0) return MPC_EINVAL;
    if (flags & (MPC_TRANS_X | MPC_TRANS_Y)) return MPC_EINVAL;
    const LinearShape s = shape_conv_grad_x(B, H, W, Cin, Cout, KH, KW, pad);
    if (stride == 1)
        return beaver_linear(ctx, s, g, w, a, b, c, gx, f_public, n_chunks, flags);
    for (int i = 0; i < 2; ++i) if (!g.p[i] || !a.p[i]) return MPC_EINVAL;
    const DilatedGeom d = dilated_geom(B, H, W, Cout, KH, KW, pad, stride);
    WsAlloc wa(ctx->ws, ctx->ws_bytes);
    u64* gd[2]; u64* ad[2];
    for (int i = 0; i < 2; ++i) { gd[i] = wa.take<u64>(d.words); ad[i] = wa.take<u64>(d.words); }
    if (!wa.ok) return MPC_ENOMEM;
    MPC_TRY(lane_join(ctx));
    DilateArgs q{};
    for (int i = 0; i < 2; ++i) { q.src[2 * i] = g.p[i]; q.dst[2 * i] = gd[i]; q.src[2 * i + 1] = a.p[i]; q.dst[2 * i + 1] = ad[i]; }
    q.B = B; q.Ho = d.Ho; q.Wo = d.Wo; q.Hd = d.Hd; q.Wd = d.Wd; q.C = Cout; q.stride = stride;
    MPC_TRY(launch_dilate(ctx, ctx->s[0], q));
    MPC_TRY(chain(ctx, ctx->s[0], ctx->s[1]));
    const mpc_cshare gs = { { gd[0], gd[1] } }, as = { { ad[0], ad[1] } };
    return beaver_linear(ctx, s, gs, w, as, b, c, gx, f_public, n_chunks, flags, nullptr, nullptr, nullptr, wa.off);
}

int mpc_conv2d_grad_w(mpc_ctx* ctx, mpc_cshare x, mpc_cshare g, mpc_cshare a, mpc_cshare b, mpc_cshare c,
                      mpc_share gw, int B, int H, int W, int Cin, int Cout, int KH, int KW, int pad, int stride,
                      const uint64_t* e_public, int n_chunks, int flags)
{
    if (stride <= 0 || B <= 0 || H <= 0 || W <= 0 || Cin <= 0 || Cout <= 0 || KH <= 0 || KW <= 0 || pad < 0)
        return MPC_EINVAL;
    if (H + 2 * pad - KH < 0 || W + 2 * pad - KW < 0 || (flags & (MPC_TRANS_X | MPC_TRANS_Y | MPC_TWO_PHASE))) return MPC_EINVAL;
    return beaver_linear(ctx, shape_conv_grad_w(B, H, W, Cin, Cout, KH, KW, pad, stride), x, g, a, b, c, gw,
                         nullptr, n_chunks, flags, e_public);
}

int mpc_conv2d(mpc_ctx* ctx, mpc_cshare x, mpc_cshare w, mpc_cshare a, mpc_cshare b, mpc_cshare c,
               mpc_share z, int B, int H, int W, int Cin, int Cout, int KH, int KW, int pad, int stride,
               const uint64_t* f_public, int n_chunks, int flags)
{
    if (stride <= 0 || B <= 0 || H <= 0 || W <= 0 || Cin <= 0 || Cout <= 0 || KH <= 0 || KW <= 0 || pad < 0)
        return MPC_EINVAL;
    if (flags & (MPC_TRANS_X | MPC_TRANS_Y)) return MPC_EINVAL;
    return beaver_linear(ctx, shape_conv(B, H, W, Cin, Cout, KH, KW, pad, stride), x, w, a, b, c, z,
                         f_public, n_chunks, flags);
}

int mpc_ring_matmul(mpc_ctx* ctx, const uint64_t* L, const uint64_t* R, uint64_t* Z,
                    int M, int K, int N, int batch)
{
    if (M <= 0 || K <= 0 || N <= 0 || batch <= 0) return MPC_EINVAL;
    return ring_product(ctx, shape_matmul(M, K, N, batch), L, R, Z);
}

int mpc_ring_conv2d(mpc_ctx* ctx, const uint64_t* x, const uint64_t* w, uint64_t* z,
                    int B, int H, int W, int Cin, int Cout, int KH, int KW, int pad, int stride)
{
    if (stride <= 0 || B <= 0 || H <= 0 || W <= 0 || Cin <= 0 || Cout <= 0 || KH <= 0 || KW <= 0 || pad < 0)
        return MPC_EINVAL;
    return ring_product(ctx, shape_conv(B, H, W, Cin, Cout, KH, KW, pad, stride), x, w, z);
}

int mpc_ring_conv2d_grad_x(mpc_ctx* ctx, const uint64_t* g, const uint64_t* w, uint64_t* gx,
                           int B, int H, int W, int Cin, int Cout, int KH, int KW, int pad, int stride)
{
    if (!ctx || !g || B <= 0 || H <= 0 || W <= 0 || Cin <= 0 || Cout <= 0 || KH <= 0 || KW <= 0 || pad < 0 || stride <= 0) return MPC_EINVAL;
    if (KH != KW || pad > KH - 1 || H + 2 * pad - KH < 0 || W + 2 * pad - KW < 0) return MPC_EINVAL;
    const LinearShape s = shape_conv_grad_x(B, H, W, Cin, Cout, KH, KW, pad);
    if (stride == 1) return ring_product(ctx, s, g, w, gx);
    const DilatedGeom d = dilated_geom(B, H, W, Cout, KH, KW, pad, stride);
    WsAlloc wa(ctx->ws, ctx->ws_bytes);
    u64* gd = wa.take<u64>(d.words);
    if (!wa.ok) return MPC_ENOMEM;
    MPC_TRY(lane_join(ctx));
    DilateArgs q{};
    q.src[0] = g; q.dst[0] = gd;
    q.B = B; q.Ho = d.Ho; q.Wo = d.Wo; q.Hd = d.Hd; q.Wd = d.Wd; q.C = Cout; q.stride = stride;
    MPC_TRY(launch_dilate(ctx, ctx->s[0], q));
    // ring_product needs 3x align of its own; the query above reserves 4 dilated buffers, one is used here
    return ring_product(ctx, s, gd, w, gx, wa.off);
}

int mpc_ring_conv2d_grad_w(mpc_ctx* ctx, const uint64_t* x, const uint64_t* g, uint64_t* gw,
                           int B, int H, int W, int Cin, int Cout, int KH, int KW, int pad, int stride)
{
    if (stride <= 0 || B <= 0 || H <= 0 || W <= 0 || Cin <= 0 || Cout <= 0 || KH <= 0 || KW <= 0 || pad < 0)
        return MPC_EINVAL;
    if (H + 2 * pad - KH < 0 || W + 2 * pad - KW < 0) return MPC_EINVAL;
    return ring_product(ctx, shape_conv_grad_w(B, H, W, Cin, Cout, KH, KW, pad, stride), x, g, gw);
}

size_t mpc_matmul3_workspace_bytes(int M, int K, int N, int batch)
{
    if (M <= 0 || K <= 0 || N <= 0 || batch <= 0) return 0;
    LinearShape s = shape_matmul(M, K, N, batch);
    if (check_shape(s) != MPC_OK) return 0;
    return carve3(nullptr, 0, s).bytes;
}

int mpc_beaver_matmul3(mpc_ctx* ctx, mpc_cshare3 x, mpc_cshare3 y, mpc_cshare3 a, mpc_cshare3 b, mpc_cshare3 c,
                       mpc_share3 z, int M, int K, int N, int batch, const uint64_t* f_public, int flags)
{
    if (M <= 0 || K <= 0 || N <= 0 || batch <= 0 || (flags & ~(MPC_TRANS_X | MPC_TRANS_Y))) return MPC_EINVAL;
    return beaver_linear3(ctx, shape_matmul(M, K, N, batch, flags), x, y, a, b, c, z, f_public);
}

size_t mpc_conv2d3_workspace_bytes(int B, int H, int W, int Cin, int Cout, int KH, int KW, int pad, int stride)
{
    if (stride <= 0) return 0;
    LinearShape s = shape_conv(B, H, W, Cin, Cout, KH, KW, pad, stride);
    if (check_shape(s) != MPC_OK) return 0;
    return carve3(nullptr, 0, s).bytes;
}

int mpc_conv2d3(mpc_ctx* ctx, mpc_cshare3 x, mpc_cshare3 w, mpc_cshare3 a, mpc_cshare3 b, mpc_cshare3 c,
                mpc_share3 z, int B, int H, int W, int Cin, int Cout, int KH, int KW, int pad, int stride,
                const uint64_t* f_public)
{
    if (stride <= 0 || B <= 0 || H <= 0 || W <= 0 || Cin <= 0 || Cout <= 0 || KH <= 0 || KW <= 0 || pad < 0)
        return MPC_EINVAL;
    return beaver_linear3(ctx, shape_conv(B, H, W, Cin, Cout, KH, KW, pad, stride), x, w, a, b, c, z, f_public);
}

int mpc_matmul3_prepared_bytes(int M, int K, int N, int batch, size_t* right, size_t* left)
{
    if (M <= 0 || K <= 0 || N <= 0 || batch <= 0) return MPC_EINVAL;
    LinearShape s = shape_matmul(M, K, N, batch);
    MPC_TRY(check_shape(s));
    prepared_sizes3(s, right, left);
    return MPC_OK;
}

int mpc_conv2d3_prepared_bytes(int B, int H, int W, int Cin, int Cout, int KH, int KW, int pad, int stride,
                               size_t* right, size_t* left)
{
    if (stride <= 0 || B <= 0 || H <= 0 || W <= 0 || Cin <= 0 || Cout <= 0 || KH <= 0 || KW <= 0 || pad < 0)
        return MPC_EINVAL;
    LinearShape s = shape_conv(B, H, W, Cin, Cout, KH, KW, pad, stride);
    MPC_TRY(check_shape(s));
    prepared_sizes3(s, right, left);
    return MPC_OK;
}

int mpc_matmul3_prepare(mpc_ctx* ctx, mpc_cshare3 a, mpc_cshare3 b, const uint64_t* f_public,
                        void* right_planes, void* left_planes, int M, int K, int N, int batch, int flags)
{
    if (M <= 0 || K <= 0 || N <= 0 || batch <= 0 || (flags & ~(MPC_TRANS_X | MPC_TRANS_Y))) return MPC_EINVAL;
    return prepare_planes3(ctx, shape_matmul(M, K, N, batch, flags), a, b, f_public, (u8*)right_planes, (u8*)left_planes);
}

int mpc_conv2d3_prepare(mpc_ctx* ctx, mpc_cshare3 a, mpc_cshare3 b, const uint64_t* f_public,
                        void* right_planes, void* left_planes,
                        int B, int H, int W, int Cin, int Cout, int KH, int KW, int pad, int stride)
{
    if (stride <= 0 || B <= 0 || H <= 0 || W <= 0 || Cin <= 0 || Cout <= 0 || KH <= 0 || KW <= 0 || pad < 0)
        return MPC_EINVAL;
    return prepare_planes3(ctx, shape_conv(B, H, W, Cin, Cout, KH, KW, pad, stride), a, b, f_public,
                           (u8*)right_planes, (u8*)left_planes);
}

int mpc_beaver_matmul3_prepared(mpc_ctx* ctx, mpc_cshare3 x, mpc_cshare3 a, mpc_cshare3 c, mpc_share3 z,
                                const void* right_planes, const void* left_planes,
                                int M, int K, int N, int batch, int flags)
{
    if (M <= 0 || K <= 0 || N <= 0 || batch <= 0 || !right_planes || (flags & ~(MPC_TRANS_X | MPC_TRANS_Y))) return MPC_EINVAL;
    const mpc_cshare3 none = { { nullptr, nullptr, nullptr } };
    return beaver_linear3(ctx, shape_matmul(M, K, N, batch, flags), x, none, a, none, c, z, nullptr, 0,
                          (const u8*)right_planes, (const u8*)left_planes);
}

int mpc_conv2d3_prepared(mpc_ctx* ctx, mpc_cshare3 x, mpc_cshare3 a, mpc_cshare3 c, mpc_share3 z,
                         const void* right_planes, const void* left_planes,
                         int B, int H, int W, int Cin, int Cout, int KH, int KW, int pad, int stride)
{
    if (stride <= 0 || B <= 0 || H <= 0 || W <= 0 || Cin <= 0 || Cout <= 0 || KH <= 0 || KW <= 0 || pad < 0 || !right_planes)
        return MPC_EINVAL;
    const mpc_cshare3 none = { { nullptr, nullptr, nullptr } };
    return beaver_linear3(ctx, shape_conv(B, H, W, Cin, Cout, KH, KW, pad, stride), x, none, a, none, c, z, nullptr, 0,
                          (const u8*)right_planes, (const u8*)left_planes);
}

size_t mpc_conv2d3_grad_x_workspace_bytes(int B, int H, int W, int Cin, int Cout, int KH, int KW, int pad, int stride)
{
    if (stride <= 0 || KH != KW || KH <= 0 || pad < 0 || pad > KH - 1 || H + 2 * pad - KH < 0 || W + 2 * pad - KW < 0) return 0;
    LinearShape s = shape_conv_grad_x(B, H, W, Cin, Cout, KH, KW, pad);
    if (check_shape(s) != MPC_OK) return 0;
    // a strided layer first scatters g_i and its mask a_i (three parties) into the dilated grid
    const size_t extra = stride > 1 ? 6 * align_up(dilated_geom(B, H, W, Cout, KH, KW, pad, stride).words * sizeof(u64)) : 0;
    return extra + carve3(nullptr, 0, s).bytes;
}

size_t mpc_conv2d3_grad_w_workspace_bytes(int B, int H, int W, int Cin, int Cout, int KH, int KW, int pad, int stride)
{
    if (stride <= 0 || KH <= 0 || KW <= 0 || pad < 0 || H + 2 * pad - KH < 0 || W + 2 * pad - KW < 0) return 0;
    LinearShape s = shape_conv_grad_w(B, H, W, Cin, Cout, KH, KW, pad, stride);
    if (check_shape(s) != MPC_OK) return 0;
    return carve3(nullptr, 0, s).bytes;
}

int mpc_conv2d3_grad_x(mpc_ctx* ctx, mpc_cshare3 g, mpc_cshare3 w, mpc_cshare3 a, mpc_cshare3 b, mpc_cshare3 c,
                       mpc_share3 gx, int B, int H, int W, int Cin, int Cout, int KH, int KW, int pad, int stride,
                       const uint64_t* f_public)
{
    if (!ctx || B <= 0 || H <= 0 || W <= 0 || Cin <= 0 || Cout <= 0 || KH <= 0 || KW <= 0 || pad < 0 || stride <= 0) return MPC_EINVAL;
    if (KH != KW || pad > KH - 1 || H + 2 * pad - KH < 0 || W + 2 * pad - KW < 0) return MPC_EINVAL;
    const LinearShape s = shape_conv_grad_x(B, H, W, Cin, Cout, KH, KW, pad);
    if (stride == 1) return beaver_linear3(ctx, s, g, w, a, b, c, gx, f_public);
    for (int i = 0; i < 3; ++i) if (!g.p[i] || !a.p[i]) return MPC_EINVAL;
    const DilatedGeom d = dilated_geom(B, H, W, Cout, KH, KW, pad, stride);
    WsAlloc wa(ctx->ws, ctx->ws_bytes);
    u64* gd[3]; u64* ad[3];
    for (int i = 0; i < 3; ++i) { gd[i] = wa.take<u64>(d.words); ad[i] = wa.take<u64>(d.words); }
    if (!wa.ok) return MPC_ENOMEM;
    MPC_TRY(lane_join(ctx));
    // the scatter kernel takes four tensors per launch: parties 0 and 1, then party 2
    for (int first = 0; first < 3; first += 2) {
        DilateArgs q{};
        for (int i = first, k = 0; i < 3 && k < 2; ++i, ++k) {
            q.src[2 * k] = g.p[i]; q.dst[2 * k] = gd[i]; q.src[2 * k + 1] = a.p[i]; q.dst[2 * k + 1] = ad[i];
        }
        q.B = B; q.Ho = d.Ho; q.Wo = d.Wo; q.Hd = d.Hd; q.Wd = d.Wd; q.C = Cout; q.stride = stride;
        MPC_TRY(launch_dilate(ctx, ctx->s[0], q));
    }
    const mpc_cshare3 gs = { { gd[0], gd[1], gd[2] } }, as = { { ad[0], ad[1], ad[2] } };
    return beaver_linear3(ctx, s, gs, w, as, b, c, gx, f_public, wa.off);
}

int mpc_conv2d3_grad_w(mpc_ctx* ctx, mpc_cshare3 x, mpc_cshare3 g, mpc_cshare3 a, mpc_cshare3 b, mpc_cshare3 c,
                       mpc_share3 gw, int B, int H, int W, int Cin, int Cout, int KH, int KW, int pad, int stride)
{
    if (stride <= 0 || B <= 0 || H <= 0 || W <= 0 || Cin <= 0 || Cout <= 0 || KH <= 0 || KW <= 0 || pad < 0)
        return MPC_EINVAL;
    if (H + 2 * pad - KH < 0 || W + 2 * pad - KW < 0) return MPC_EINVAL;
    return beaver_linear3(ctx, shape_conv_grad_w(B, H, W, Cin, Cout, KH, KW, pad, stride), x, g, a, b, c, gw, nullptr);
}

}  // extern "C"
