// Streaming element-wise kernels: masking, opening, truncation, wire copy,
// and the recoding of ring words into balanced base-256 digit planes.
// All of them are HBM-bound; they use 16-byte accesses and grid-stride loops.
#include "common.h"

#include <algorithm>

namespace {

constexpr int kThreads = 256;

inline int grid_for(size_t items, int per_thread = 1)
{
    size_t blocks = (items + (size_t)kThreads * per_thread - 1) / ((size_t)kThreads * per_thread);
    const size_t cap = 256 * 16;          // 16 workgroups per CU keep HBM busy
    if (blocks > cap) blocks = cap;
    if (blocks < 1) blocks = 1;
    return (int)blocks;
}

struct alignas(16) u64x2 { u64 a, b; };

template <int OP>  // 0: x - y, 1: x + y
__global__ __launch_bounds__(kThreads) void k_binary(const u64* __restrict__ x, const u64* __restrict__ y,
                                                     u64* __restrict__ out, size_t n)
{
    const size_t n2 = n / 2;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    const u64x2* x2 = reinterpret_cast<const u64x2*>(x);
    const u64x2* y2 = reinterpret_cast<const u64x2*>(y);
    u64x2* o2 = reinterpret_cast<u64x2*>(out);
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n2; i += stride) {
        u64x2 p = x2[i], q = y2[i], r;
        if (OP == 0) { r.a = p.a - q.a; r.b = p.b - q.b; }
        else         { r.a = p.a + q.a; r.b = p.b + q.b; }
        o2[i] = r;
    }
    if ((n & 1) && blockIdx.x == 0 && threadIdx.x == 0) {
        const size_t i = n - 1;
        out[i] = OP == 0 ? x[i] - y[i] : x[i] + y[i];
    }
}

// scalar fallback when a pointer is only 8-byte aligned
template <int OP>
__global__ __launch_bounds__(kThreads) void k_binary_scalar(const u64* __restrict__ x, const u64* __restrict__ y,
                                                            u64* __restrict__ out, size_t n)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride)
        out[i] = OP == 0 ? x[i] - y[i] : x[i] + y[i];
}

__global__ __launch_bounds__(kThreads) void k_copy16(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n16)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

__global__ __launch_bounds__(kThreads) void k_copy1(const u8* __restrict__ src, u8* __restrict__ dst, size_t n)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) dst[i] = src[i];
}

// Local two-party truncation: party 0 shifts, party 1 negates, shifts, negates.
__global__ __launch_bounds__(kThreads) void k_truncate(u64* __restrict__ z, size_t n, int bits, int party)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        const u64 v = z[i];
        z[i] = party == 0 ? (v >> bits) : (u64)0 - (((u64)0 - v) >> bits);
    }
}

// Balanced base-256 digits of x: x = sum_j d_j 2^(8j) (mod 2^64), d_j in
// [-128, 127].  Adding 0x80 to every byte position (with carries) and flipping
// the top bit of every byte yields the eight digits as two's-complement bytes.
__device__ __forceinline__ u64 balanced_digits(u64 x)
{
    const u64 h = 0x8080808080808080ull;
    return (x + h) ^ h;
}

// One thread recodes one (row, k-block): 16 ring words in, one 16-byte unit
// out per digit plane.  Consecutive lanes take consecutive rows so that the
// plane stores are contiguous.
__device__ __forceinline__ void recode_body(const RecodeArgs& a, int tap /* == ntaps: zero padding block(s) */, int b,
                                            unsigned bx, unsigned nbx)
{
    const u64* src = a.src + (size_t)b * a.src_batch_stride;
    const u64* src2 = a.src2 ? a.src2 + (size_t)b * a.src_batch_stride : nullptr;
    const u64* src3 = a.src3 ? a.src3 + (size_t)b * a.src_batch_stride : nullptr;
    const u64* sub = a.sub ? a.sub + (size_t)b * a.src_batch_stride : nullptr;
    u64* side = a.side ? a.side + (size_t)b * a.src_batch_stride : nullptr;
    const u64* minuend = (a.minuend && a.side && !a.sub) ? a.minuend + (size_t)b * a.src_batch_stride : nullptr;
    u8* dst = a.dst + (size_t)b * a.dst_batch_stride;
    const bool padtap = tap >= a.ntaps;
    const int kb_count = padtap ? a.KB_total - a.ntaps * a.KB_tap : a.KB_tap;
    const size_t items = (size_t)kb_count * a.plane_rows;
    const size_t stride = (size_t)nbx * blockDim.x;
    for (size_t it = (size_t)bx * blockDim.x + threadIdx.x; it < items; it += stride) {
        const int kbl = (int)(it / a.plane_rows);
        const int row = (int)(it - (size_t)kbl * a.plane_rows);
        const int kb_out = (padtap ? a.ntaps * a.KB_tap : tap * a.KB_tap) + kbl;
        u64 dg[16];
#pragma unroll
        for (int t = 0; t < 16; ++t) {
            const int k = kbl * 16 + t;
            u64 v = 0;
            if (!padtap && k < a.K && row < a.rows) {
                // tap_stride may be negative (filters read in reverse tap order)
                const long long idx = (long long)row * a.row_stride + (long long)k * a.k_stride + (long long)tap * a.tap_stride;
                v = src[idx];
                if (sub) { v -= sub[idx]; if (side) side[idx] = v; }
                else if (minuend) side[idx] = minuend[idx] - v;
                if (src2) v += src2[idx];
                if (src3) v += src3[idx];
            }
            dg[t] = balanced_digits(v);
        }
        u8* out = dst + ((size_t)kb_out * a.plane_rows + row) * 16;
#pragma unroll
        for (int d = 0; d < 8; ++d) {
            uint32_t w[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                uint32_t v = 0;
#pragma unroll
                for (int t = 0; t < 4; ++t)
                    v |= (uint32_t)((dg[q * 4 + t] >> (8 * d)) & 0xff) << (8 * t);
                w[q] = v;
            }
            *reinterpret_cast<uint4*>(out + (size_t)d * a.digit_stride) = make_uint4(w[0], w[1], w[2], w[3]);
        }
    }
}

__global__ __launch_bounds__(kThreads) void k_recode(RecodeArgs a)
{
    recode_body(a, blockIdx.y, blockIdx.z, blockIdx.x, gridDim.x);
}

// Recoding of a matrix whose k index is contiguous in memory (left operands,
// NHWC activations): a workgroup takes a 64-row x 64-k tile, reads it with
// lanes along k (coalesced 16-byte loads), scatters the digits into LDS in
// plane order, and writes each plane's 16-byte units with lanes along rows
// (coalesced again).  blockIdx = (row tile, group of 4 k blocks, set*batch).
__device__ __forceinline__ void recode_rows_body(const RecodeArgs& a, int b, unsigned bx, unsigned by, uint32_t (*tile)[4][64][4])
{
    const int row0 = bx * 64, kb0 = by * 4;
    if (row0 >= a.plane_rows || kb0 >= a.KB_total) return;      // uniform per workgroup
    const u64* src = a.src + (size_t)b * a.src_batch_stride;
    const u64* src2 = a.src2 ? a.src2 + (size_t)b * a.src_batch_stride : nullptr;
    const u64* src3 = a.src3 ? a.src3 + (size_t)b * a.src_batch_stride : nullptr;
    const u64* sub = a.sub ? a.sub + (size_t)b * a.src_batch_stride : nullptr;
    u64* side = a.side ? a.side + (size_t)b * a.src_batch_stride : nullptr;
    const u64* minuend = (a.minuend && a.side && !a.sub) ? a.minuend + (size_t)b * a.src_batch_stride : nullptr;
    u8* dst = a.dst + (size_t)b * a.dst_batch_stride;
    const bool vec_ok = (a.row_stride % 2 == 0) && (((uintptr_t)src & 15) == 0) &&
                        (!src2 || ((uintptr_t)src2 & 15) == 0) && (!src3 || ((uintptr_t)src3 & 15) == 0) &&
                        (!sub || ((uintptr_t)sub & 15) == 0) && (!side || ((uintptr_t)side & 15) == 0) &&
                        (!minuend || ((uintptr_t)minuend & 15) == 0);
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        const int seg = threadIdx.x + 256 * p;
        const int row = seg >> 4, s4 = seg & 15;
        const int r = row0 + row, k = kb0 * 16 + s4 * 4;
        u64 v[4] = { 0, 0, 0, 0 };
        if (r < a.rows && k < a.K) {
            const size_t idx = (size_t)r * a.row_stride + k;
            if (vec_ok && k + 3 < a.K) {
                const u64x2 p0 = *reinterpret_cast<const u64x2*>(src + idx), p1 = *reinterpret_cast<const u64x2*>(src + idx + 2);
                v[0] = p0.a; v[1] = p0.b; v[2] = p1.a; v[3] = p1.b;
                if (sub) {
                    const u64x2 q0 = *reinterpret_cast<const u64x2*>(sub + idx), q1 = *reinterpret_cast<const u64x2*>(sub + idx + 2);
                    v[0] -= q0.a; v[1] -= q0.b; v[2] -= q1.a; v[3] -= q1.b;
                    if (side) {
                        u64x2 s0, s1; s0.a = v[0]; s0.b = v[1]; s1.a = v[2]; s1.b = v[3];
                        *reinterpret_cast<u64x2*>(side + idx) = s0; *reinterpret_cast<u64x2*>(side + idx + 2) = s1;
                    }
                }
                if (minuend) {
                    const u64x2 q0 = *reinterpret_cast<const u64x2*>(minuend + idx), q1 = *reinterpret_cast<const u64x2*>(minuend + idx + 2);
                    u64x2 s0, s1; s0.a = q0.a - v[0]; s0.b = q0.b - v[1]; s1.a = q1.a - v[2]; s1.b = q1.b - v[3];
                    *reinterpret_cast<u64x2*>(side + idx) = s0; *reinterpret_cast<u64x2*>(side + idx + 2) = s1;
                }
                if (src2) { const u64x2 q0 = *reinterpret_cast<const u64x2*>(src2 + idx), q1 = *reinterpret_cast<const u64x2*>(src2 + idx + 2);
                            v[0] += q0.a; v[1] += q0.b; v[2] += q1.a; v[3] += q1.b; }
                if (src3) { const u64x2 q0 = *reinterpret_cast<const u64x2*>(src3 + idx), q1 = *reinterpret_cast<const u64x2*>(src3 + idx + 2);
                            v[0] += q0.a; v[1] += q0.b; v[2] += q1.a; v[3] += q1.b; }
            } else {
#pragma unroll
                for (int t = 0; t < 4; ++t)
                    if (k + t < a.K) {
                        v[t] = src[idx + t];
                        if (sub) { v[t] -= sub[idx + t]; if (side) side[idx + t] = v[t]; }
                        else if (minuend) side[idx + t] = minuend[idx + t] - v[t];
                        if (src2) v[t] += src2[idx + t];
                        if (src3) v[t] += src3[idx + t];
                    }
            }
        }
        u64 dg[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) dg[t] = balanced_digits(v[t]);
#pragma unroll
        for (int d = 0; d < 8; ++d) {
            uint32_t w = 0;
#pragma unroll
            for (int t = 0; t < 4; ++t) w |= (uint32_t)((dg[t] >> (8 * d)) & 0xff) << (8 * t);
            tile[d][s4 >> 2][row][s4 & 3] = w;
        }
    }
    __syncthreads();
#pragma unroll
    for (int q = 0; q < 8; ++q) {
        const int u = threadIdx.x + 256 * q;
        const int d = u >> 8, kbl = (u >> 6) & 3, row = u & 63;
        if (row0 + row < a.plane_rows && kb0 + kbl < a.KB_total) {
            const uint4 val = *reinterpret_cast<const uint4*>(&tile[d][kbl][row][0]);
            *reinterpret_cast<uint4*>(dst + (size_t)d * a.digit_stride + ((size_t)(kb0 + kbl) * a.plane_rows + row0 + row) * 16) = val;
        }
    }
}

__global__ __launch_bounds__(kThreads) void k_recode_rows(RecodeBatch rb)
{
    __shared__ uint32_t tile[8][4][64][4];
    const int set = blockIdx.z / rb.batch, b = blockIdx.z - set * rb.batch;
    recode_rows_body(rb.a[set], b, blockIdx.x, blockIdx.y, tile);
}

// Sets of both kinds in one launch over a flat list of workgroups: set q owns the
// ids [first[q], first[q+1]), decoded as (x, y, batch item) with its own extents gx, gy.
// Contiguous-k sets (rows_kind) use the tile recoder above with (x, y) = (row tile, group
// of 4 k blocks); generic sets use one thread per (row, k block) with y = tap.
struct RecodeMixed { RecodeBatch rb; unsigned first[kMaxRecodeSets + 1]; unsigned gx[kMaxRecodeSets], gy[kMaxRecodeSets];
                     bool rows_kind[kMaxRecodeSets]; int count; };
__global__ __launch_bounds__(kThreads) void k_recode_mixed(RecodeMixed m)
{
    __shared__ uint32_t tile[8][4][64][4];
    int q = 0;
    while (q + 1 < m.count && blockIdx.x >= m.first[q + 1]) ++q;       // uniform per workgroup
    const RecodeArgs& a = m.rb.a[q];
    unsigned id = blockIdx.x - m.first[q];
    const unsigned x = id % m.gx[q]; id /= m.gx[q];
    const unsigned y = id % m.gy[q]; const int b = (int)(id / m.gy[q]);
    if (m.rows_kind[q]) recode_rows_body(a, b, x, y, tile);
    else                recode_body(a, (int)y, b, x, m.gx[q]);
}

// Digit planes of the transposed im2col matrix of an NHWC tensor: plane row
// (tap, ci), contraction index = output pixel (b, ho, wo).  One thread fills
// one 16-byte unit per digit: 16 consecutive output pixels of one (tap, ci).
// Lanes run along the rows, i.e. along ci, so loads and stores are contiguous.
__global__ __launch_bounds__(kThreads) void k_recode_im2col_t(Im2colTBatch bt)
{
    const Im2colTArgs& a = bt.a[blockIdx.z];
    const int rows = a.KH * a.KW * a.Cin;
    const long long npix = (long long)a.B * a.Ho * a.Wo;
    const size_t items = (size_t)a.KB_total * rows;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t it = (size_t)blockIdx.x * blockDim.x + threadIdx.x; it < items; it += stride) {
        const int kb = (int)(it / rows);
        const int row = (int)(it - (size_t)kb * rows);
        const int tap = row / a.Cin, ci = row - tap * a.Cin;
        const int dy = tap / a.KW, dx = tap - dy * a.KW;
        long long m = (long long)kb * 16;
        int wo = (int)(m % a.Wo); long long t2 = m / a.Wo;
        int ho = (int)(t2 % a.Ho); int b = (int)(t2 / a.Ho);
        u64 dg[16];
#pragma unroll
        for (int t = 0; t < 16; ++t) {
            u64 v = 0;
            if (m + t < npix) {
                const int hi = ho * a.stride + dy - a.pad, wi = wo * a.stride + dx - a.pad;
                if (hi >= 0 && hi < a.H && wi >= 0 && wi < a.W) {
                    const size_t idx = (((size_t)b * a.H + hi) * a.W + wi) * a.Cin + ci;
                    v = a.src[idx];
                    if (a.src2) v += a.src2[idx];
                }
            }
            dg[t] = balanced_digits(v);
            if (++wo == a.Wo) { wo = 0; if (++ho == a.Ho) { ho = 0; ++b; } }
        }
        u8* out = a.dst + ((size_t)kb * rows + row) * 16;
#pragma unroll
        for (int d = 0; d < 8; ++d) {
            uint32_t w[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                uint32_t v = 0;
#pragma unroll
                for (int t = 0; t < 4; ++t)
                    v |= (uint32_t)((dg[q * 4 + t] >> (8 * d)) & 0xff) << (8 * t);
                w[q] = v;
            }
            *reinterpret_cast<uint4*>(out + (size_t)d * a.digit_stride) = make_uint4(w[0], w[1], w[2], w[3]);
        }
    }
}

// Element-wise Alg. 1 after the exchange (blockIdx.y = party): e, f from the
// own and the received masked words, z_i = c_i + e*b_i + a_i*f (+ e*f), then the
// optional local truncation.  With `mask_from_sign` the second operand is the
// ReLU input mask 1 - s formed from the additive sign shares in y.
__global__ __launch_bounds__(kThreads) void k_mul_finish(MulArgs q)
{
    const int i = blockIdx.y;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t k = (size_t)blockIdx.x * blockDim.x + threadIdx.x; k < q.n; k += stride) {
        const u64 e = q.se[i][k] + q.re[i][k], f = q.sf[i][k] + q.rf[i][k];
        u64 z = q.c[i][k] + e * q.b[i][k] + q.a[i][k] * f;
        if (i == 0) z += e * f;
        if (q.trunc_bits) z = i == 0 ? (z >> q.trunc_bits) : (u64)0 - (((u64)0 - z) >> q.trunc_bits);
        q.z[i][k] = z;
    }
}

// masks of the element-wise product (blockIdx.y = party): se = x - a, sf = y - b
__global__ __launch_bounds__(kThreads) void k_mul_mask(MulArgs q)
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

// Max-pool backward, between its two products (blockIdx.y = party):
// grad_v = g - grad_u, and the pair (grad_u, grad_v) interleaved as the first
// tournament level stored its pairs.
__global__ __launch_bounds__(kThreads) void k_poolbwd_pairs(PoolBwdArgs q)
{
    const int i = blockIdx.y;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t o = (size_t)blockIdx.x * blockDim.x + threadIdx.x; o < q.n_out; o += stride) {
        const u64 gu = q.gu[i][o];
        q.pairs[i][2 * o] = gu;
        q.pairs[i][2 * o + 1] = q.g[i][o] - gu;
    }
}

// ... and after the second product P = pairs * mask1: the four window positions
// receive P[2o], grad_u - P[2o], P[2o+1], grad_v - P[2o+1] (NHWC input layout).
__global__ __launch_bounds__(kThreads) void k_poolbwd_scatter(PoolBwdArgs q)
{
    const int i = blockIdx.y;
    const int Ho = q.H / 2, Wo = q.W / 2;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t o = (size_t)blockIdx.x * blockDim.x + threadIdx.x; o < q.n_out; o += stride) {
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

// Zero-dilation for the input gradient of a strided convolution (blockIdx.y = tensor):
// every destination word is written, a source word where its pixel is a multiple of the stride.
__global__ __launch_bounds__(kThreads) void k_dilate(DilateArgs q)
{
    const u64* src = q.src[blockIdx.y]; u64* dst = q.dst[blockIdx.y];
    if (!src) return;
    const size_t total = (size_t)q.B * q.Hd * q.Wd * q.C;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t o = (size_t)blockIdx.x * blockDim.x + threadIdx.x; o < total; o += stride) {
        const int ch = (int)(o % q.C); size_t t = o / q.C;
        const int wd = (int)(t % q.Wd); t /= q.Wd;
        const int hd = (int)(t % q.Hd); const int b = (int)(t / q.Hd);
        u64 v = 0;
        if (hd % q.stride == 0 && wd % q.stride == 0) {
            const int ho = hd / q.stride, wo = wd / q.stride;
            if (ho < q.Ho && wo < q.Wo) v = src[(((size_t)b * q.Ho + ho) * q.Wo + wo) * q.C + ch];
        }
        dst[o] = v;
    }
}

// Several recodings in one launch: blockIdx.z = set * batch + batch item.
__global__ __launch_bounds__(kThreads) void k_recode_multi(RecodeBatch rb)
{
    const int set = blockIdx.z / rb.batch, b = blockIdx.z - set * rb.batch;
    const RecodeArgs& a = rb.a[set];
    const int taps = a.ntaps + (a.KB_total > a.ntaps * a.KB_tap ? 1 : 0);
    if ((int)blockIdx.y < taps) recode_body(a, blockIdx.y, b, blockIdx.x, gridDim.x);
}

// Several element-wise subtractions / copies in one launch: blockIdx.y = segment.
// PUT: every difference is also stored into out2, the peer's receive buffer
// (exchange by remote store: the mask kernel is the sender).
template <bool PUT>
__global__ __launch_bounds__(kThreads) void k_sub_multi(SubBatch sb)
{
    const SubSeg& q = sb.s[blockIdx.y];
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    if (q.vec) {
        const size_t n2 = q.n / 2;
        const u64x2* x2 = reinterpret_cast<const u64x2*>(q.x);
        const u64x2* y2 = reinterpret_cast<const u64x2*>(q.a);
        u64x2* o2 = reinterpret_cast<u64x2*>(q.out);
        u64x2* p2 = reinterpret_cast<u64x2*>(q.out2);
        for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n2; i += stride) {
            u64x2 p = x2[i], r = y2[i];
            p.a -= r.a; p.b -= r.b;
            o2[i] = p;
            if constexpr (PUT) p2[i] = p;
        }
        if ((q.n & 1) && blockIdx.x == 0 && threadIdx.x == 0) {
            q.out[q.n - 1] = q.x[q.n - 1] - q.a[q.n - 1];
            if constexpr (PUT) q.out2[q.n - 1] = q.out[q.n - 1];
        }
    } else {
        for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < q.n; i += stride) {
            const u64 v = q.x[i] - q.a[i];
            q.out[i] = v;
            if constexpr (PUT) q.out2[i] = v;
        }
    }
}

__global__ __launch_bounds__(kThreads) void k_copy_multi(CopyBatch cb)
{
    const CopySeg& q = cb.s[blockIdx.y];
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    if (q.vec) {
        const uint4* s4 = reinterpret_cast<const uint4*>(q.src); uint4* d4 = reinterpret_cast<uint4*>(q.dst);
        const size_t n16 = q.bytes / 16;
        for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) d4[i] = s4[i];
    } else {
        for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < q.bytes; i += stride) q.dst[i] = q.src[i];
    }
}

// out = x + y + w: the opening of a three-party additive sharing.
__global__ __launch_bounds__(kThreads) void k_sum3(const u64* __restrict__ x, const u64* __restrict__ y,
                                                   const u64* __restrict__ w, u64* __restrict__ out, size_t n)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) out[i] = x[i] + y[i] + w[i];
}

inline bool aligned16(const void* p) { return ((uintptr_t)p & 15) == 0; }

template <int OP>
int launch_binary(mpc_ctx* c, hipStream_t st, const u64* x, const u64* y, u64* out, size_t n)
{
    if (aligned16(x) && aligned16(y) && aligned16(out))
        hipLaunchKernelGGL(k_binary<OP>, dim3(grid_for(n / 2 + 1)), dim3(kThreads), 0, st, x, y, out, n);
    else
        hipLaunchKernelGGL(k_binary_scalar<OP>, dim3(grid_for(n)), dim3(kThreads), 0, st, x, y, out, n);
    MPC_HIP(c, hipGetLastError());
    return MPC_OK;
}

}  // namespace

int launch_sub(mpc_ctx* c, hipStream_t st, const u64* x, const u64* a, u64* out, size_t n)
{
    return launch_binary<0>(c, st, x, a, out, n);
}

int launch_add(mpc_ctx* c, hipStream_t st, const u64* x, const u64* y, u64* out, size_t n)
{
    return launch_binary<1>(c, st, x, y, out, n);
}

// The "wire": a plain device copy kernel (kept as a kernel rather than
// hipMemcpyAsync so that the same path can be captured into a HIP graph).
int launch_copy(mpc_ctx* c, hipStream_t st, const void* src, void* dst, size_t bytes)
{
    if (bytes == 0) return MPC_OK;
    if (aligned16(src) && aligned16(dst) && bytes % 16 == 0) {
        const size_t n16 = bytes / 16;
        hipLaunchKernelGGL(k_copy16, dim3(grid_for(n16)), dim3(kThreads), 0, st,
                           (const uint4*)src, (uint4*)dst, n16);
    } else {
        hipLaunchKernelGGL(k_copy1, dim3(grid_for(bytes)), dim3(kThreads), 0, st,
                           (const u8*)src, (u8*)dst, bytes);
    }
    MPC_HIP(c, hipGetLastError());
    return MPC_OK;
}

int launch_sum3(mpc_ctx* c, hipStream_t st, const u64* x, const u64* y, const u64* w, u64* out, size_t n)
{
    if (n == 0) return MPC_OK;
    hipLaunchKernelGGL(k_sum3, dim3(grid_for(n)), dim3(kThreads), 0, st, x, y, w, out, n);
    MPC_HIP(c, hipGetLastError());
    return MPC_OK;
}

int launch_truncate(mpc_ctx* c, hipStream_t st, u64* z, size_t n, int bits, int party)
{
    hipLaunchKernelGGL(k_truncate, dim3(grid_for(n)), dim3(kThreads), 0, st, z, n, bits, party);
    MPC_HIP(c, hipGetLastError());
    return MPC_OK;
}

int launch_recode_multi(mpc_ctx* c, hipStream_t st, const RecodeArgs* sets, int count)
{
    if (count < 1 || count > kMaxRecodeSets) return MPC_EINVAL;
    bool rows_kind = true;          // every set a plain matrix with contiguous k?
    for (int i = 0; i < count; ++i)
        if (sets[i].k_stride != 1 || sets[i].ntaps != 1 || sets[i].batch != sets[0].batch) rows_kind = false;
    if (rows_kind) {
        RecodeBatch rb{};
        int rows = 0, kb = 0;
        for (int i = 0; i < count; ++i) {
            rb.a[i] = sets[i];
            if (sets[i].plane_rows > rows) rows = sets[i].plane_rows;
            if (sets[i].KB_total > kb) kb = sets[i].KB_total;
        }
        rb.batch = sets[0].batch;
        if ((size_t)count * rb.batch > 65535 || (kb + 3) / 4 > 65535) return MPC_EINVAL;
        dim3 grid((rows + 63) / 64, (kb + 3) / 4, count * rb.batch);
        hipLaunchKernelGGL(k_recode_rows, grid, dim3(kThreads), 0, st, rb);
        MPC_HIP(c, hipGetLastError());
        return MPC_OK;
    }
    RecodeBatch rb{};
    size_t items = 0; int taps = 0;
    for (int i = 0; i < count; ++i) {
        rb.a[i] = sets[i];
        if (sets[i].batch != sets[0].batch) return MPC_EINVAL;
        const size_t it = (size_t)sets[i].KB_tap * sets[i].plane_rows;
        if (it > items) items = it;
        const int t = sets[i].ntaps + (sets[i].KB_total > sets[i].ntaps * sets[i].KB_tap ? 1 : 0);
        if (t > taps) taps = t;
    }
    rb.batch = sets[0].batch;
    if ((size_t)count * rb.batch > 65535) return MPC_EINVAL;
    dim3 grid(grid_for(items), taps, count * rb.batch);
    hipLaunchKernelGGL(k_recode_multi, grid, dim3(kThreads), 0, st, rb);
    MPC_HIP(c, hipGetLastError());
    return MPC_OK;
}

// Up to kMaxRecodeSets recodings of either kind (contiguous k, or generic with taps) in one launch.
int launch_recode_any(mpc_ctx* c, hipStream_t st, const RecodeArgs* sets, int count)
{
    if (count < 1 || count > kMaxRecodeSets) return MPC_EINVAL;
    RecodeMixed m{};
    unsigned long long total = 0;
    for (int i = 0; i < count; ++i) {
        const RecodeArgs& a = sets[i];
        m.rb.a[i] = a;
        m.rows_kind[i] = a.k_stride == 1 && a.ntaps == 1;
        if (m.rows_kind[i]) {
            m.gx[i] = (unsigned)((a.plane_rows + 63) / 64); m.gy[i] = (unsigned)((a.KB_total + 3) / 4);
        } else {
            m.gx[i] = (unsigned)grid_for((size_t)a.KB_tap * a.plane_rows);
            m.gy[i] = (unsigned)(a.ntaps + (a.KB_total > a.ntaps * a.KB_tap ? 1 : 0));
        }
        if (m.gx[i] == 0 || m.gy[i] == 0 || a.batch < 1) return MPC_EINVAL;
        m.first[i] = (unsigned)total;
        total += (unsigned long long)m.gx[i] * m.gy[i] * a.batch;
        if (total >= (1ull << 31)) return MPC_EINVAL;
    }
    m.first[count] = (unsigned)total;
    m.count = count;
    hipLaunchKernelGGL(k_recode_mixed, dim3((unsigned)total), dim3(kThreads), 0, st, m);
    MPC_HIP(c, hipGetLastError());
    return MPC_OK;
}

int launch_sub_multi(mpc_ctx* c, hipStream_t st, const SubSeg* segs, int count)
{
    if (count < 1 || count > kMaxSegs) return MPC_EINVAL;
    SubBatch sb{}; size_t nmax = 0;
    for (int i = 0; i < count; ++i) {
        sb.s[i] = segs[i];
        sb.s[i].vec = aligned16(segs[i].x) && aligned16(segs[i].a) && aligned16(segs[i].out) &&
                      (!segs[i].out2 || aligned16(segs[i].out2));
        if (segs[i].n > nmax) nmax = segs[i].n;
        if ((segs[i].out2 != nullptr) != (segs[0].out2 != nullptr)) return MPC_EINVAL;    // all or none
    }
    if (segs[0].out2) hipLaunchKernelGGL(k_sub_multi<true>, dim3(grid_for(nmax / 2 + 1), count), dim3(kThreads), 0, st, sb);
    else              hipLaunchKernelGGL(k_sub_multi<false>, dim3(grid_for(nmax / 2 + 1), count), dim3(kThreads), 0, st, sb);
    MPC_HIP(c, hipGetLastError());
    return MPC_OK;
}

int launch_copy_multi(mpc_ctx* c, hipStream_t st, const CopySeg* segs, int count)
{
    if (count < 1 || count > kMaxSegs) return MPC_EINVAL;
    CopyBatch cb{}; size_t bmax = 0;
    for (int i = 0; i < count; ++i) {
        cb.s[i] = segs[i];
        cb.s[i].vec = aligned16(segs[i].src) && aligned16(segs[i].dst) && segs[i].bytes % 16 == 0;
        if (segs[i].bytes > bmax) bmax = segs[i].bytes;
    }
    hipLaunchKernelGGL(k_copy_multi, dim3(grid_for(bmax / 16 + 1), count), dim3(kThreads), 0, st, cb);
    MPC_HIP(c, hipGetLastError());
    return MPC_OK;
}

int launch_recode_im2col_t(mpc_ctx* c, hipStream_t st, const Im2colTArgs* sets, int count)
{
    if (count < 1 || count > 3) return MPC_EINVAL;
    Im2colTBatch bt{};
    for (int i = 0; i < count; ++i) bt.a[i] = sets[i];
    const size_t items = (size_t)sets[0].KB_total * sets[0].KH * sets[0].KW * sets[0].Cin;
    hipLaunchKernelGGL(k_recode_im2col_t, dim3(grid_for(items), 1, count), dim3(kThreads), 0, st, bt);
    MPC_HIP(c, hipGetLastError());
    return MPC_OK;
}

int launch_mul_mask(mpc_ctx* c, hipStream_t st, const MulArgs& q)
{
    hipLaunchKernelGGL(k_mul_mask, dim3(grid_for(q.n), 2), dim3(kThreads), 0, st, q);
    MPC_HIP(c, hipGetLastError());
    return MPC_OK;
}

int launch_mul_finish(mpc_ctx* c, hipStream_t st, const MulArgs& q)
{
    hipLaunchKernelGGL(k_mul_finish, dim3(grid_for(q.n), 2), dim3(kThreads), 0, st, q);
    MPC_HIP(c, hipGetLastError());
    return MPC_OK;
}

int launch_dilate(mpc_ctx* c, hipStream_t st, const DilateArgs& q)
{
    const size_t total = (size_t)q.B * q.Hd * q.Wd * q.C;
    hipLaunchKernelGGL(k_dilate, dim3(grid_for(total), 4), dim3(kThreads), 0, st, q);
    MPC_HIP(c, hipGetLastError());
    return MPC_OK;
}

int launch_poolbwd_pairs(mpc_ctx* c, hipStream_t st, const PoolBwdArgs& q)
{
    hipLaunchKernelGGL(k_poolbwd_pairs, dim3(grid_for(q.n_out), 2), dim3(kThreads), 0, st, q);
    MPC_HIP(c, hipGetLastError());
    return MPC_OK;
}

int launch_poolbwd_scatter(mpc_ctx* c, hipStream_t st, const PoolBwdArgs& q)
{
    hipLaunchKernelGGL(k_poolbwd_scatter, dim3(grid_for(q.n_out), 2), dim3(kThreads), 0, st, q);
    MPC_HIP(c, hipGetLastError());
    return MPC_OK;
}

int launch_recode(mpc_ctx* c, hipStream_t st, const RecodeArgs& a)
{
    if (a.k_stride == 1 && a.ntaps == 1) return launch_recode_multi(c, st, &a, 1);
    const bool has_pad = a.KB_total > a.ntaps * a.KB_tap;
    const size_t items = (size_t)a.KB_tap * a.plane_rows;
    dim3 grid(grid_for(items), a.ntaps + (has_pad ? 1 : 0), a.batch);
    hipLaunchKernelGGL(k_recode, grid, dim3(kThreads), 0, st, a);
    MPC_HIP(c, hipGetLastError());
    return MPC_OK;
}
