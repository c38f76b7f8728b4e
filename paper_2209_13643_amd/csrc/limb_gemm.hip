// Ring GEMM over Z_2^64 on the int8 matrix cores.
//
// A ring word is split into eight balanced base-256 digits d_j in [-128,127].
// Mod 2^64 only digit pairs with i + j <= 7 contribute, so one ring MAC is 36
// int8 products; products with equal s = i + j share one int32 accumulator
// (exact while (s+1) * K * 2^14 < 2^31 for s <= 3; for s >= 4 only the low
// 64 - 8s <= 32 bits matter, so wrap-around there is harmless).  The epilogue
// recombines sum_s acc_s * 2^(8s) mod 2^64, adds the party's addend (c_i or a
// partial sum), optionally truncates, and stores.
//
// Each wave owns a 32x32 output tile = 8 digit-sum groups x 16 accumulator
// registers, and issues 36 v_mfma_i32_32x32x32_i8 per 32-deep K step.  A
// workgroup of WGM x WGN waves stages the eight digit planes of its
// (32*WGM) x 32 left tile and 32 x (32*WGN) right tile through LDS, double
// buffered; the planes' [kb][row][16] layout makes both the global reads and
// the ds_read_b128 operand fetches contiguous in lane order.
//
// The contraction may run over two operand segments (party i contracts
// [e | a_i] against [b_i' ; f]) and, for convolutions, the left tile loader
// gathers filter taps from NHWC activation planes (implicit im2col).
#include "common.h"

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int KS = 2;   // 16-wide k blocks per pipeline stage = one MFMA K step

template <int WGM, int WGN>
struct Cfg {
    static constexpr int TM = 32 * WGM, TN = 32 * WGN, NW = WGM * WGN, NT = 64 * NW;
    static constexpr int L_UNITS = 8 * KS * TM, R_UNITS = 8 * KS * TN;   // 16-byte units per stage
    static constexpr int LI = L_UNITS / NT, RI = R_UNITS / NT;           // units per thread
    static constexpr int STAGE_UNITS = L_UNITS + R_UNITS;
    static constexpr size_t LDS_BYTES = 2 * (size_t)STAGE_UNITS * 16;
    static_assert(NT % TM == 0 && NT % TN == 0, "a thread keeps one row for all its units");
    static_assert(L_UNITS % NT == 0 && R_UNITS % NT == 0, "units divide evenly");
};

// Byte offset of the 16-byte unit (row-of-thread, k block kb) inside one digit
// plane of the left operand, or -1 for a zero unit (conv padding / pad taps).
struct LeftRow {
    long long base;      // plain: clamped row; conv: pixel index of tap (0,0), may be negative
    unsigned long long valid;   // conv: bit per tap
};

template <int WGM, int WGN>
__global__ __launch_bounds__(64 * WGM * WGN, (WGM * WGN == 8) ? 1 : 2)
void k_limb_gemm(GemmArgs g)
{
    using C = Cfg<WGM, WGN>;
    extern __shared__ uint4 lds[];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave % WGM, wn = wave / WGM;
    const int i32 = lane & 31, g2 = lane >> 5;
    const int party = blockIdx.z % g.nparty;
    const int bidx = blockIdx.z / g.nparty;
    const int m0 = blockIdx.x * C::TM, n0 = blockIdx.y * C::TN;

    // ---- loader geometry: this thread's row in the left / right tiles
    const int lrow = tid % C::TM, lq = tid / C::TM;     // unit j: q = lq + j * (NT/TM)
    const int rrow = tid % C::TN, rq = tid / C::TN;
    LeftRow lr;
    {
        int m = m0 + lrow; if (m > g.M - 1) m = g.M - 1;
        if (g.conv.enabled) {
            const int wo = m % g.conv.Wo; const int t = m / g.conv.Wo;
            const int ho = t % g.conv.Ho; const int b = t / g.conv.Ho;
            const int hi0 = ho * g.conv.stride - g.conv.pad, wi0 = wo * g.conv.stride - g.conv.pad;
            lr.base = ((long long)b * g.conv.H + hi0) * g.conv.W + wi0;
            unsigned long long v = 0;
            for (int kh = 0; kh < g.conv.KH; ++kh)
                for (int kw = 0; kw < g.conv.KW; ++kw) {
                    const int hi = hi0 + kh, wi = wi0 + kw;
                    if (hi >= 0 && hi < g.conv.H && wi >= 0 && wi < g.conv.W)
                        v |= 1ull << (kh * g.conv.KW + kw);
                }
            lr.valid = v;
        } else {
            lr.base = m; lr.valid = ~0ull;
        }
    }
    int nrow = n0 + rrow; if (nrow > g.N - 1) nrow = g.N - 1;

    uint4 stL[C::LI], stR[C::RI];

    auto load_stage = [&](int seg, int kb0) {
        const GemmSeg& s = g.seg[party][seg];
        const u8* Lb = s.L + (size_t)bidx * s.L_bstride;
        const u8* Rb = s.R + (size_t)bidx * s.R_bstride;
#pragma unroll
        for (int j = 0; j < C::LI; ++j) {
            const int q = lq + j * (C::NT / C::TM);
            const int kk = q % KS, d = q / KS;
            const int kb = kb0 + kk;
            const u8* p;
            if (g.conv.enabled) {
                const int tap = kb / g.conv.CB, cb = kb - tap * g.conv.CB;
                const bool ok = tap < g.conv.KH * g.conv.KW && ((lr.valid >> tap) & 1);
                const int kh = tap / g.conv.KW, kw = tap - kh * g.conv.KW;
                const long long pix = lr.base + (long long)kh * g.conv.W + kw;
                p = ok ? Lb + (size_t)d * s.L_dstride + ((size_t)cb * g.conv.npix + (size_t)pix) * 16
                       : g.zero16;
            } else {
                p = Lb + (size_t)d * s.L_dstride + ((size_t)kb * g.rows_L + (size_t)lr.base) * 16;
            }
            stL[j] = *reinterpret_cast<const uint4*>(p);
        }
#pragma unroll
        for (int j = 0; j < C::RI; ++j) {
            const int q = rq + j * (C::NT / C::TN);
            const int kk = q % KS, d = q / KS;
            const u8* p = Rb + (size_t)d * s.R_dstride + ((size_t)(kb0 + kk) * g.N + (size_t)nrow) * 16;
            stR[j] = *reinterpret_cast<const uint4*>(p);
        }
    };

    auto store_stage = [&](int buf) {
        uint4* Ls = lds + (size_t)buf * C::STAGE_UNITS;
        uint4* Rs = Ls + C::L_UNITS;
#pragma unroll
        for (int j = 0; j < C::LI; ++j) {
            const int q = lq + j * (C::NT / C::TM);       // q = d*KS + kk
            Ls[q * C::TM + lrow] = stL[j];
        }
#pragma unroll
        for (int j = 0; j < C::RI; ++j) {
            const int q = rq + j * (C::NT / C::TN);
            Rs[q * C::TN + rrow] = stR[j];
        }
    };

    v16i acc[8];
#pragma unroll
    for (int s = 0; s < 8; ++s)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[s][v] = 0;

    auto compute_stage = [&](int buf) {
        const uint4* Ls = lds + (size_t)buf * C::STAGE_UNITS;
        const uint4* Rs = Ls + C::L_UNITS;
        v4i A[8], B[8];
#pragma unroll
        for (int d = 0; d < 8; ++d) {
            const uint4 a = Ls[(d * KS + g2) * C::TM + wm * 32 + i32];
            const uint4 b = Rs[(d * KS + g2) * C::TN + wn * 32 + i32];
            A[d] = v4i{ (int)a.x, (int)a.y, (int)a.z, (int)a.w };
            B[d] = v4i{ (int)b.x, (int)b.y, (int)b.z, (int)b.w };
        }
#pragma unroll
        for (int i = 0; i < 8; ++i)
#pragma unroll
            for (int j = 0; j < 8 - i; ++j)
                acc[i + j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(A[i], B[j], acc[i + j], 0, 0, 0);
    };

    // ---- main loop over (segment, k block) stages
    int seg = 0, kb0 = 0;
    auto advance = [&]() { kb0 += KS; if (kb0 >= g.seg[party][seg].KB) { kb0 = 0; ++seg; } };
    int total = 0;
    for (int s = 0; s < g.nseg; ++s) total += g.seg[party][s].KB / KS;

    load_stage(seg, kb0); advance();
    store_stage(0);
    __syncthreads();
    for (int t = 0; t < total; ++t) {
        const bool more = t + 1 < total;
        if (more) { load_stage(seg, kb0); advance(); }
        compute_stage(t & 1);
        if (more) store_stage((t + 1) & 1);
        __syncthreads();
    }

    // ---- epilogue: recombine, add, truncate, store
    const u64* addend = g.addend[party] ? g.addend[party] + (size_t)bidx * g.out_bstride : nullptr;
    const u64* addend2 = g.addend2[party] ? g.addend2[party] + (size_t)bidx * g.out_bstride : nullptr;
    u64* out = g.out[party] + (size_t)bidx * g.out_bstride;
    const int col = n0 + wn * 32 + i32;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int row = m0 + wm * 32 + (v >> 2) * 8 + g2 * 4 + (v & 3);
        u64 z = 0;
#pragma unroll
        for (int s = 0; s < 8; ++s) z += (u64)(long long)acc[s][v] << (8 * s);
        if (row < g.M && col < g.N) {
            const size_t idx = (size_t)row * g.N + col;
            if (addend) z += addend[idx];
            if (addend2) z += addend2[idx];
            if (g.trunc_bits) z = party == 0 ? (z >> g.trunc_bits) : (u64)0 - (((u64)0 - z) >> g.trunc_bits);
            out[idx] = z;
        }
    }
}

template <int WGM, int WGN>
int launch_cfg(mpc_ctx* c, hipStream_t st, const GemmArgs& g)
{
    using C = Cfg<WGM, WGN>;
    static bool attr_set[16] = { false };
    auto kern = k_limb_gemm<WGM, WGN>;
    if (c->device >= 0 && c->device < 16 && !attr_set[c->device]) {
        MPC_HIP(c, hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)C::LDS_BYTES));
        attr_set[c->device] = true;
    }
    dim3 grid((g.M + C::TM - 1) / C::TM, (g.N + C::TN - 1) / C::TN, g.batch * g.nparty);
    hipLaunchKernelGGL(kern, grid, dim3(C::NT), C::LDS_BYTES, st, g);
    MPC_HIP(c, hipGetLastError());
    return MPC_OK;
}

}  // namespace

int launch_limb_gemm(mpc_ctx* c, hipStream_t st, const GemmArgs& g)
{
    if (g.M <= 0 || g.N <= 0 || g.batch <= 0 || g.nseg < 1 || g.nseg > 2) return MPC_EINVAL;
    if ((size_t)g.batch * g.nparty > 65535) return MPC_EINVAL;
    for (int p = 0; p < g.nparty; ++p)
        for (int s = 0; s < g.nseg; ++s)
            if (g.seg[p][s].KB <= 0 || g.seg[p][s].KB % KS) return MPC_EINVAL;
    // large problems: 128x64 workgroup tiles (8 waves); small ones: 64x64 (4 waves)
    const long long tiles_big = (long long)((g.M + 127) / 128) * ((g.N + 63) / 64) * g.batch * g.nparty;
    if (tiles_big >= 256) return launch_cfg<4, 2>(c, st, g);
    return launch_cfg<2, 2>(c, st, g);
}
