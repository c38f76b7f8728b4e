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
// One wave per SIMD, the whole register file per wave: a wave owns a 32x64
// output tile = 2 x 8 digit-sum groups x 16 accumulator registers (256 AGPRs)
// and issues 72 v_mfma_i32_32x32x32_i8 per 32-deep K step.  A workgroup of
// WGM x WGN waves streams the eight digit planes of its (32*WGM)-row left tile
// and (64*WGN)-row right tile through a three-slot LDS ring filled by direct
// global->LDS loads (no staging registers).  Every load is "scalar base +
// per-lane constant offset": the lane offsets are fixed for the whole kernel
// and the bases advance with scalar arithmetic, so the loader costs almost no
// vector ALU work.  Inside a K step an operand register is refilled from the
// next ring slot right after its last use, and the global loads for step t+3
// are issued in the same MFMA shadow.  The planes' [kb][row][16] layout makes
// the global reads and the ds_read_b128 operand fetches contiguous in lane
// order.
//
// The contraction may run over two operand segments (party i contracts
// [e | a_i] against [b_i' ; f]) and, for convolutions, the left tile loader
// gathers filter taps from NHWC activation planes (implicit im2col); taps
// that fall into the zero padding read the all-zero row that ends every
// activation plane.
#include <atomic>
#include "common.h"

#include <type_traits>
#include <utility>

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int KS = 2;   // 16-wide k blocks per pipeline stage = one MFMA K step
// LDS ring depth: three slots for the one-workgroup-per-unit tiles; two for the small tile of short
// contractions, which then fits twice on a compute unit

// NH: 32-column halves of a wave's output tile (2: 32 x 64, all 256 accumulator registers, one wave per SIMD;
// 1: 32 x 32, 128 accumulator registers, two waves per SIMD).
template <int WGM, int WGN, int NS, int NH>
struct Cfg {
    static constexpr int WN = 32 * NH;
    static constexpr int TM = 32 * WGM, TN = WN * WGN, NW = WGM * WGN, NT = 64 * NW;
    static constexpr int L_UNITS = 8 * KS * TM, R_UNITS = 8 * KS * TN;   // 16-byte units per stage
    static constexpr int STAGE_UNITS = L_UNITS + R_UNITS;
    static constexpr size_t LDS_BYTES = (size_t)NS * STAGE_UNITS * 16;
    // Tiles are loaded in chunks of 64 rows x 16 bytes (one wave-wide load).
    // Wave w loads digits w, w+NW, ... (DPW of them) of every k block and row
    // chunk: load j <-> digit w + NW*(j % DPW), k block (j / DPW) % KS,
    // row chunk j / (DPW * KS).
    static constexpr int RCM = TM / 64, RCN = TN / 64;
    static constexpr int DPW = 8 / NW;
    static constexpr int LPW = DPW * KS * RCM, RPW = DPW * KS * RCN;     // loads per wave per stage
    static_assert(TM % 64 == 0 && TN % 64 == 0, "tiles are whole numbers of 64-row chunks");
    static_assert(8 % NW == 0, "digits divide evenly over waves");
};

template <typename F, int... Is>
__device__ __forceinline__ void static_for_impl(F&& f, std::integer_sequence<int, Is...>)
{
    (f(std::integral_constant<int, Is>{}), ...);
}
template <int N, typename F>
__device__ __forceinline__ void static_for(F&& f)
{
    static_for_impl(f, std::make_integer_sequence<int, N>{});
}

// s_waitcnt immediate that waits for vmcnt <= n only (gfx9 encoding)
constexpr int vmcnt_imm(int n) { return (n & 15) | (7 << 4) | (15 << 8) | ((n >> 4) << 14); }

// One wave-wide direct global->LDS load: lane l's 16 bytes at base + voff(l)
// land at lds_slot + LDS_OFF + 16*l.  Issued through inline assembly so that
// completion is tracked by this kernel's own vmcnt waits (see the main loop).
template <int LDS_OFF>
__device__ __forceinline__ void load_lds16(const u8* base, unsigned voff, unsigned lds_slot)
{
    asm volatile("s_add_u32 m0, %0, %1\n\tglobal_load_lds_dwordx4 %2, %3"
                 :: "s"(lds_slot), "n"(LDS_OFF), "v"(voff), "s"(base) : "memory", "scc");
}

template <int WGM, int WGN, bool CONV, int NS, int NH>
__global__ __launch_bounds__(64 * WGM * WGN, NH == 1 ? 2 : 1)
void k_limb_gemm(GemmArgs g)
{
    using C = Cfg<WGM, WGN, NS, NH>;
    extern __shared__ uint4 lds[];
    const unsigned lds_base = (unsigned)(uintptr_t)(__attribute__((address_space(3))) void*)lds;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave % WGM, wn = wave / WGM;
    const int i32 = lane & 31, g2 = lane >> 5;
    // One-dimensional grid.  Workgroups go to the eight XCDs (each with its own L2) round-robin by their
    // linear id, and XCD r owns a contiguous range of the tile sequence, so that the workgroups resident on
    // an XCD at one time are neighbours in that sequence.  The sequence runs over (split, batch item), then
    // panels of GN column tiles, then row tiles, then the column tiles of the panel: what an XCD holds at a
    // time is a block of a few row tiles by up to GN column tiles of one item, whose left and right tiles
    // are fetched into that L2 once (convolutions: neighbouring pixel tiles also share the rows their filter
    // taps overlap on).  Measured with the fetch counter: the 256-wide 1x1 convolution on 56 x 56 x 64 moved
    // 983 MiB with the row tiles of one column running first, per-head Q K^T 1032 MiB with the tiles dealt
    // round-robin; in this order 547 and 539 MiB (the minimum is 539 and 528).
    //  - parties with equal work: both parties' workgroups of a tile one after the other (they share e and f);
    //  - parties that contract different lengths: party 1's workgroups (the long ones) fill the chip first,
    //    party 0's follow as units free up.
    const unsigned id = blockIdx.x;
    int party; unsigned tile;
    if (g.heavy_first) {
        const unsigned blk1 = (unsigned)((g.tiles_party[1] + 7) / 8 * 8);
        party = id < blk1 ? 1 : 0;
        const unsigned local = party ? id : id - blk1;
        const unsigned per_xcd = (unsigned)((g.tiles_party[party] + 7) / 8);
        const unsigned q = local >> 3;
        tile = q < per_xcd ? (local & 7) * per_xcd + q : 0xffffffffu;
    } else {
        const unsigned r8 = id & 7, sl = id >> 3;
        const unsigned per_xcd = (unsigned)((g.tiles_party[0] + 7) / 8);
        const unsigned q = sl / (unsigned)g.nparty;
        party = (int)(sl % (unsigned)g.nparty);
        tile = q < per_xcd ? r8 * per_xcd + q : 0xffffffffu;
    }
    if (tile >= (unsigned)g.tiles_party[party]) return;      // padding of the last group of eight
    constexpr unsigned GN = NH == 1 ? 8 : 4;
    const unsigned per_item = (unsigned)g.tiles_m * (unsigned)g.tiles_n;
    const unsigned t2 = tile / per_item, tq = tile - t2 * per_item;
    const unsigned panel = tq / (GN * (unsigned)g.tiles_m), rem = tq - panel * GN * (unsigned)g.tiles_m;
    const unsigned width = (unsigned)g.tiles_n - panel * GN < GN ? (unsigned)g.tiles_n - panel * GN : GN;
    const int mt = (int)(rem / width);
    const int nt = (int)(panel * GN + rem % width);
    const int bidx = (int)(t2 % (unsigned)g.batch);
    const int split = (int)(t2 / (unsigned)g.batch);
    const int m0 = mt * C::TM, n0 = nt * C::TN;

    // ---- per-party operands as scalars
    const GemmSeg& sg0 = party ? g.seg[1][0] : g.seg[0][0];
    const GemmSeg& sg1 = party ? g.seg[1][1] : g.seg[0][1];
    const int KB0 = sg0.KB, KB1 = g.nseg > 1 ? sg1.KB : 0;        // a party's second segment may be empty
    // K steps of this workgroup: all of them, or one slice when the contraction is split
    const int T_all = (KB0 + KB1) / KS;
    const int st0 = split * g.steps_per_split;
    const int T = T_all - st0 < g.steps_per_split ? T_all - st0 : g.steps_per_split;
    if (T <= 0) return;             // cannot happen: the launcher gives each party ceil(steps / steps_per_split) slices
    const long long krowL = (long long)g.rows_L * 16;      // bytes between k blocks of a left plane
    const long long krowR = (long long)g.N * 16;

    // ---- per-lane constant byte offsets
    // conv: pixel index of filter tap (0,0), biased so that it is never negative
    const int bias = CONV ? g.conv.pad * g.conv.W + g.conv.pad : 0;
    unsigned voffL[C::RCM];
    unsigned long long lvalid[C::RCM];      // conv: bit per filter tap that hits the image
#pragma unroll
    for (int rc = 0; rc < C::RCM; ++rc) {
        int m = m0 + rc * 64 + lane; if (m > g.M - 1) m = g.M - 1;
        if (CONV) {
            const int wo = m % g.conv.Wo; const int t = m / g.conv.Wo;
            const int ho = t % g.conv.Ho; const int b = t / g.conv.Ho;
            const int hi0 = ho * g.conv.stride - g.conv.pad, wi0 = wo * g.conv.stride - g.conv.pad;
            const long long pix00 = ((long long)b * g.conv.H + hi0) * g.conv.W + wi0;
            voffL[rc] = (unsigned)((pix00 + bias) * 16);
            unsigned long long v = 0;
            for (int kh = 0; kh < g.conv.KH; ++kh)
                for (int kw = 0; kw < g.conv.KW; ++kw) {
                    const int hi = hi0 + kh, wi = wi0 + kw;
                    if (hi >= 0 && hi < g.conv.H && wi >= 0 && wi < g.conv.W)
                        v |= 1ull << (kh * g.conv.KW + kw);
                }
            lvalid[rc] = v;
        } else {
            voffL[rc] = (unsigned)m * 16u; lvalid[rc] = ~0ull;
        }
    }
    unsigned voffR[C::RCN];
#pragma unroll
    for (int rc = 0; rc < C::RCN; ++rc) {
        int n = n0 + rc * 64 + lane; if (n > g.N - 1) n = g.N - 1;
        voffR[rc] = (unsigned)n * 16u;
    }
    const int ntaps = CONV ? g.conv.KH * g.conv.KW : 0;
    const int CB = CONV ? g.conv.CB : 1, KWf = CONV ? g.conv.KW : 1, Wimg = CONV ? g.conv.W : 0;
    const long long npix = CONV ? g.conv.npix : 0;          // the zero row of a plane has index npix

    // ---- loader state (all scalar).  segL / segR already point at this wave's
    // first digit plane; dsL / dsR are the byte strides between the digit
    // planes a wave loads (NW planes apart).
    const u8 *segL, *segR; long long dsL, dsR;
    auto set_segment = [&](int seg) {
        const GemmSeg& q = seg ? sg1 : sg0;
        segL = q.L + (size_t)bidx * q.L_bstride + (long long)wave * q.L_dstride;
        segR = q.R + (size_t)bidx * q.R_bstride + (long long)wave * q.R_dstride;
        dsL = q.L_dstride * C::NW; dsR = q.R_dstride * C::NW;
    };
    // cursor at K step st0
    int c_seg = st0 * KS >= KB0 ? 1 : 0;
    int c_kb = st0 * KS - (c_seg ? KB0 : 0);
    int c_tap = CONV ? c_kb / CB : 0, c_cb = CONV ? c_kb - c_tap * CB : 0;
    int c_kw = CONV ? c_tap % KWf : 0;
    int c_dpix = CONV ? (c_tap / KWf) * Wimg + c_kw : 0;
    long long c_offL = (long long)c_kb * krowL, c_offR = (long long)c_kb * krowR;       // c_kb * krowL / krowR
    set_segment(c_seg);
    auto cursor_next = [&]() {      // advance by one k block
        ++c_kb; c_offL += krowL; c_offR += krowR;
        if (CONV) {
            if (++c_cb == CB) {
                c_cb = 0; ++c_tap;
                if (++c_kw == KWf) { c_kw = 0; c_dpix += Wimg - (KWf - 1); } else ++c_dpix;
            }
        }
        if (c_seg == 0 && c_kb == KB0) {
            c_seg = 1; c_kb = 0; c_tap = 0; c_cb = 0; c_dpix = 0; c_kw = 0; c_offL = 0; c_offR = 0;
            set_segment(1);
        }
    };

    // State of the stage being issued, captured once per stage; the stage's
    // loads are then issued one by one between MFMAs.
    const u8* s_L[KS]; const u8* s_R[KS];
    unsigned s_zoff[KS]; int s_tap[KS];
    unsigned s_slotL, s_slotR; long long s_dsL, s_dsR;
    auto stage_begin = [&](int slot) {
        // KS divides every segment, so a stage never straddles two segments
        // (the cursor may move on to the next segment at the end of this stage)
        s_dsL = dsL; s_dsR = dsR;
        s_slotL = lds_base + (unsigned)(slot * C::STAGE_UNITS * 16) + (unsigned)(wave * KS * C::TM * 16);
        s_slotR = lds_base + (unsigned)((slot * C::STAGE_UNITS + C::L_UNITS) * 16) + (unsigned)(wave * KS * C::TN * 16);
#pragma unroll
        for (int kk = 0; kk < KS; ++kk) {
            s_R[kk] = segR + c_offR;
            if (CONV) {
                // base such that base + (pix00 + bias)*16 is the tap pixel's unit in channel block c_cb
                s_L[kk] = segL + ((long long)c_cb * (npix + 1) + c_dpix - bias) * 16;
                s_zoff[kk] = (unsigned)((npix - c_dpix + bias) * 16);   // lands on the zero row instead
                s_tap[kk] = c_tap;
            } else {
                s_L[kk] = segL + c_offL;
            }
            cursor_next();
        }
    };
    // q-th load of the stage (left tile first), q a compile-time constant
    auto issue_one = [&](auto q_tag) {
        constexpr int q = decltype(q_tag)::value;
        if constexpr (q < C::LPW) {
            constexpr int dj = q % C::DPW, kk = (q / C::DPW) % KS, rc = q / (C::DPW * KS);
            unsigned voff = voffL[rc];
            if (CONV) {
                const bool ok = s_tap[kk] < ntaps && ((lvalid[rc] >> (s_tap[kk] & 63)) & 1);
                voff = ok ? voff : s_zoff[kk];
            }
            // destination unit: ((d*KS + kk)*TM + rc*64) with d = wave + NW*dj
            load_lds16<((C::NW * dj * KS + kk) * C::TM + rc * 64) * 16>(s_L[kk] + dj * s_dsL, voff, s_slotL);
        } else {
            constexpr int r = q - C::LPW;
            constexpr int dj = r % C::DPW, kk = (r / C::DPW) % KS, rc = r / (C::DPW * KS);
            load_lds16<((C::NW * dj * KS + kk) * C::TN + rc * 64) * 16>(s_R[kk] + dj * s_dsR, voffR[rc], s_slotR);
        }
    };
    constexpr int PER_STAGE = C::LPW + C::RPW;
    auto issue_all = [&](int slot) {
        stage_begin(slot);
        static_for<PER_STAGE>([&](auto q) { issue_one(q); });
    };

    v16i acc[NH][8];
#pragma unroll
    for (int c = 0; c < NH; ++c)
#pragma unroll
        for (int s = 0; s < 8; ++s)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[c][s][v] = 0;

    v4i A[8], B[NH][8];
    auto read_A = [&](int slot, int d) {
        const uint4 a = lds[(size_t)slot * C::STAGE_UNITS + (d * KS + g2) * C::TM + wm * 32 + i32];
        A[d] = v4i{ (int)a.x, (int)a.y, (int)a.z, (int)a.w };
    };
    auto read_B = [&](int slot, int d) {
#pragma unroll
        for (int c = 0; c < NH; ++c) {
            const uint4 b = lds[(size_t)slot * C::STAGE_UNITS + C::L_UNITS + (d * KS + g2) * C::TN + wn * C::WN + c * 32 + i32];
            B[c][d] = v4i{ (int)b.x, (int)b.y, (int)b.z, (int)b.w };
        }
    };

    // ---- output pointers, and the addend c_i of the epilogue.  Its loads (indices clamped
    // into the matrix, no per-word branch) are issued all at once at the start of the
    // epilogue.  Issuing them from inside the last steps hides their latency (4 % on
    // 64-deep contractions) but keeps 64 more registers live across the main loop; the
    // kernel stays below 128 vector registers instead, so that a wave of a streaming
    // kernel from another lane (secure ReLU: at most 128) fits beside it on the same SIMD
    // and fills the issue slots the MFMAs leave free: 7-13 % on the inter-batch pipeline.
    const bool partial = g.ksplit > 1;      // raw partial products go to the workspace; a second kernel finishes
    const u64* addend = (g.addend[party] && !partial) ? g.addend[party] + (size_t)bidx * g.out_bstride : nullptr;
    const u64* addend2 = (g.addend2[party] && !partial) ? g.addend2[party] + (size_t)bidx * g.out_bstride : nullptr;
    u64* out = partial ? g.partial + (((size_t)split * g.nparty + party) * g.batch + bidx) * g.out_bstride
                       : g.out[party] + (size_t)bidx * g.out_bstride;
    const int rbase = m0 + wm * 32 + g2 * 4;
    const int shift = partial ? 0 : g.trunc_bits;
    const bool interior = m0 + C::TM <= g.M && n0 + C::TN <= g.N;   // uniform: no per-word bounds checks
    u64 addw[NH][16];
    auto load_addend = [&]() {
#pragma unroll
        for (int c = 0; c < NH; ++c) {
            const int col = n0 + wn * C::WN + c * 32 + i32;
            const int colc = col < g.N ? col : g.N - 1;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = rbase + (v >> 2) * 8 + (v & 3);
                const int rowc = row < g.M ? row : g.M - 1;
                addw[c][v] = addend ? addend[(size_t)rowc * g.N + colc] : 0;
            }
        }
    };

    // ---- main loop.  Ring slot t%NS holds K step t.  At the top of step t the
    // slot of step t+1 must have landed (this wave's loads: all but the most
    // recent PER_STAGE); the barrier makes every wave's part visible and
    // retires slot t%NS, whose operands every wave already holds in registers,
    // so the loads of step t+NS can go there.  Inside the step the MFMAs run
    // block by block over the right-operand digit j (left digits 7-j .. 0);
    // an operand register is refilled from the next slot right after its last
    // use, in an order that gives every refill at least ~14 MFMAs of cover,
    // and one global->LDS load is issued after every fourth MFMA: a wave can
    // issue one instruction per four cycles, so everything that is not an MFMA
    // has to sit in the seven free issue slots an 8-pass MFMA leaves behind.
    issue_all(0);
    if (1 < T) issue_all(1);
    if (NS > 2 && 2 < T) issue_all(2);
    // slot 0 must have landed: everything but the stages issued after it
    static_assert(NS == 2 || NS == 3, "ring depth");
    static_assert((NS - 1) * PER_STAGE <= 63, "vmcnt is a six-bit counter");
    if (NS > 2 && T > 2) __builtin_amdgcn_s_waitcnt(vmcnt_imm(2 * PER_STAGE));
    else if (T > 1)      __builtin_amdgcn_s_waitcnt(vmcnt_imm(1 * PER_STAGE));
    else                 __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
    __syncthreads();
#pragma unroll
    for (int d = 0; d < 8; ++d) { read_A(0, d); read_B(0, d); }

    int slot = 0;                        // t % NS
    // FULL: steps with both a successor to prefetch operands from and a stage to issue
    auto step = [&](auto full_tag, int t) {
        constexpr bool FULL = decltype(full_tag)::value;
        const bool have_next = FULL || t + 1 < T, fill = FULL || t + NS < T;
        // slot t+1 must have landed; with three slots the loads of step t+2 may still be in flight
        if (NS > 2 && (FULL || t + 2 < T)) __builtin_amdgcn_s_waitcnt(vmcnt_imm(PER_STAGE));
        else if (have_next)               __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
        __syncthreads();
        const int nslot = slot + 1 == NS ? 0 : slot + 1;
        if (fill) stage_begin(slot);
        // MFMA number n (0..71) <-> block j, left digit i, column half c
        static_for<8>([&](auto jt) {
            constexpr int j = decltype(jt)::value;
            static_for<8 - j>([&](auto it) {
                constexpr int i = 7 - j - decltype(it)::value;
                static_for<NH>([&](auto ct) {
                    constexpr int c = decltype(ct)::value;
                    // MFMAs before this block: sum_{j'<j} NH*(8-j') = NH*j*(17-j)/2
                    constexpr int n = NH * (j * (17 - j) / 2 + (7 - j - i)) + c;
                    acc[c][i + j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(A[i], B[c][j], acc[c][i + j], 0, 0, 0);
                    if constexpr (n % 4 == 1 && n / 4 < PER_STAGE) {
                        if (fill) issue_one(std::integral_constant<int, n / 4>{});
                    }
                });
                if (i == 7 - j && have_next) read_A(nslot, i);       // last use of A[7-j] in this step
                // keep this interleaving: without the fence the scheduler packs the
                // MFMAs back to back and everything else into one exposed cluster
                __builtin_amdgcn_sched_barrier(0);
            });
            if (have_next) read_B(nslot, j);                          // last use of B[.][j]
        });
        slot = nslot;
    };
    int t = 0;
    for (; t + NS < T; ++t) step(std::true_type{}, t);
    for (; t < T; ++t) step(std::false_type{}, t);

    load_addend();
    // The explicit accumulator reads below are opaque to the compiler's hazard
    // handling: give the last MFMA (8 passes) time to retire before the first read.
    asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 15\n\ts_nop 15" ::: "memory");

    // ---- epilogue: recombine, add, truncate, store.
    static_for<NH>([&](auto ct) {
        constexpr int c = decltype(ct)::value;
        const int col = n0 + wn * C::WN + c * 32 + i32;
        u64 (&add)[16] = addw[c];
        if (addend2) {                  // partial sums of a two-phase call: loaded here, all 16 at once
            const int colc = col < g.N ? col : g.N - 1;
            u64 more[16];
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = rbase + (v >> 2) * 8 + (v & 3);
                const int rowc = row < g.M ? row : g.M - 1;
                more[v] = addend2[(size_t)rowc * g.N + colc];
            }
#pragma unroll
            for (int v = 0; v < 16; ++v) add[v] += more[v];
        }
        // The accumulators are read out explicitly (left to itself the compiler copies all
        // 256 accumulator registers into vector registers at the loop exit, which leaves no
        // room for anything else to stay live across the main loop); the two column halves
        // are fenced from each other, inside a half the 16 words are independent chains.
        // Recombination sum_s acc_s 2^(8s) mod 2^64 in 32-bit pieces: the digit sums of weights 0..3 add up exactly
        // as 64-bit terms built from two shifts each; of weights 4..7 only the low 32 bits reach the result, and
        // those land in the high word.
        u64 z[16];
        static_for<16>([&](auto vt) {
            constexpr int v = decltype(vt)::value;
            int d[8];
            static_for<8>([&](auto st) {
                constexpr int sg = decltype(st)::value;
                int t;
                asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(t) : "a"(acc[c][sg][v]));
                d[sg] = t;
            });
            u64 acc64 = (u64)(long long)d[0];
#pragma unroll
            for (int sg = 1; sg < 4; ++sg)
                acc64 += (u64)((unsigned)d[sg] << (8 * sg)) | ((u64)(unsigned)(d[sg] >> (32 - 8 * sg)) << 32);
            const unsigned high = (unsigned)d[4] + ((unsigned)d[5] << 8) + ((unsigned)d[6] << 16) + ((unsigned)d[7] << 24);
            acc64 += (u64)high << 32;
            acc64 += add[v];
            // local truncation (party is uniform over the workgroup): party 0 shifts, party 1 negates around the shift
            if (shift == 0)      z[v] = acc64;
            else if (party == 0) z[v] = acc64 >> shift;
            else                 z[v] = (u64)0 - (((u64)0 - acc64) >> shift);
        });
        if (interior) {
#pragma unroll
            for (int v = 0; v < 16; ++v) out[(size_t)(rbase + (v >> 2) * 8 + (v & 3)) * g.N + col] = z[v];
        } else {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = rbase + (v >> 2) * 8 + (v & 3);
                if (row < g.M && col < g.N) out[(size_t)row * g.N + col] = z[v];
            }
        }
        __builtin_amdgcn_sched_barrier(0);
    });
}

// Second pass of a split contraction: out = sum over splits of the partial
// products + addends, then truncation.  One thread per output word.
__global__ __launch_bounds__(256) void k_splitk_finish(GemmArgs g)
{
    const size_t per = (size_t)g.batch * g.out_bstride;            // words per party
    const size_t total = per * g.nparty;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += stride) {
        const int party = (int)(i / per);
        const size_t w = i - (size_t)party * per;
        u64 z = 0;
        for (int sp = 0; sp < g.ksplit_p[party]; ++sp) z += g.partial[((size_t)sp * g.nparty + party) * per + w];
        if (g.addend[party]) z += g.addend[party][w];
        if (g.addend2[party]) z += g.addend2[party][w];
        if (g.trunc_bits) z = party == 0 ? (z >> g.trunc_bits) : (u64)0 - (((u64)0 - z) >> g.trunc_bits);
        g.out[party][w] = z;
    }
}

template <int WGM, int WGN, bool CONV, int NS = 3, int NH = 2>
int launch_cfg(mpc_ctx* c, hipStream_t st, const GemmArgs& g)
{
    using C = Cfg<WGM, WGN, NS, NH>;
    // once per device and kernel: allow the large dynamic LDS allocation (lanes may live on several host threads)
    static std::atomic<bool> attr_set[16];
    auto kern = k_limb_gemm<WGM, WGN, CONV, NS, NH>;
    if (c->device < 0 || c->device >= 16) return MPC_EINVAL;
    if (!attr_set[c->device].load(std::memory_order_acquire)) {
        MPC_HIP(c, hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)C::LDS_BYTES));
        attr_set[c->device].store(true, std::memory_order_release);
    }
    GemmArgs ga = g;
    ga.tiles_m = (g.M + C::TM - 1) / C::TM; ga.tiles_n = (g.N + C::TN - 1) / C::TN;
    long long wgs = 0;
    for (int p = 0; p < 2; ++p) {
        const long long tiles = p < g.nparty ? (long long)ga.tiles_m * ga.tiles_n * g.batch * g.ksplit_p[p] : 0;
        if (tiles >= (1ll << 30)) return MPC_EINVAL;
        ga.tiles_party[p] = (int)tiles;
        wgs += (tiles + 7) / 8 * 8;
    }
    // equal slice counts: the interleaved / party-major orders of the kernel assume equal blocks
    if (!ga.heavy_first && g.nparty == 2 && ga.tiles_party[0] != ga.tiles_party[1]) return MPC_EINVAL;
    if (wgs >= (1ll << 31)) return MPC_EINVAL;
    dim3 grid((unsigned)wgs, 1, 1);
    const int pi = prof_begin(c, MPC_PROF_GEMM_KERNEL, st);
    hipLaunchKernelGGL(kern, grid, dim3(C::NT), C::LDS_BYTES, st, ga);
    if (g.ksplit > 1) {
        const size_t total = (size_t)g.batch * g.out_bstride * g.nparty;
        size_t blocks = (total + 255) / 256; if (blocks > 4096) blocks = 4096;
        hipLaunchKernelGGL(k_splitk_finish, dim3((unsigned)blocks), dim3(256), 0, st, ga);
    }
    prof_end(c, MPC_PROF_GEMM_KERNEL, pi, st);
    MPC_HIP(c, hipGetLastError());
    return MPC_OK;
}

}  // namespace

// How many ways to split the contraction so that a small output still fills
// the chip: aim for about 256 workgroups, keep at least 4 K steps per slice.
// 32 k per step; with balanced digits (|d| <= 128) the digit-sum groups that
// matter beyond their low 32 bits hold at most four pairs, so 4 * 2^14 * k < 2^31.
constexpr int kMaxStepsExact = 1023;

// Output tile of a workgroup: 0 = 64 x 128 (2 x 2 waves), 1 = 128 x 64 (4 x 1 waves) when a second 64-column half
// would be empty, 2 = 64 x 64 (2 x 2 waves of 32 x 32 with half the accumulator registers, two-slot ring: two
// workgroups per compute unit, two waves per SIMD) for short contractions, where a workgroup's life is mostly
// pipeline fill and epilogue and a second resident wave hides them.
// Tile 2 is chosen when the longest contraction of the launch has at most g_small_max_steps K steps (32 terms each)
// and the output has at least g_small_min_tiles tiles of 64 x 64 (mpc_set_gemm_small_tile changes both).
// A launch whose parties contract different lengths (the folded calls: party 0 one segment, party 1 two) also takes
// tile 2 at any contraction length once the output has kAsymMinTiles tiles of 64 x 64: short and long workgroups then
// mix two to a compute unit, and the launch loses less to the imbalance (BERT-base layers 2-9 % faster; at 512 tiles,
// configs[1]'s convolution, the two tilings are even, and the wide tile keeps room for another lane's streaming waves).
static std::atomic<int> g_small_max_steps{ 16 }, g_small_min_tiles{ 512 };
constexpr long long kAsymMinTiles = 768;
static int tile_kind(int M, int N, int batch, int longest_steps, bool asymmetric)
{
    const long long tiles64 = (long long)((M + 63) / 64) * ((N + 63) / 64) * batch;
    const int max_steps = g_small_max_steps.load(std::memory_order_relaxed);
    if (longest_steps <= max_steps && tiles64 >= g_small_min_tiles.load(std::memory_order_relaxed)) return 2;
    // (not the batched products one 64-column tile wide, per-head A*V: those are 5 % faster on the 128 x 64 tile)
    if (asymmetric && max_steps > 0 && tiles64 >= kAsymMinTiles && !(batch > 1 && N <= 64)) return 2;
    return (((N - 1) % 128) < 64 && (N <= 64 || M >= 4096)) ? 1 : 0;
}

// steps[p]: K steps party p contracts (steps[1] = 0 for a one-party launch).  Returns the number of slices
// of the longer contraction; a party with fewer steps gets ceil(its steps / slice length) slices.
static int ksplit_for(int M, int N, int batch, const int steps[2])
{
    const int nparty = steps[1] > 0 ? 2 : 1;
    const int longest = steps[0] > steps[1] ? steps[0] : steps[1];
    const int kind = tile_kind(M, N, batch, longest, nparty == 2 && steps[0] != steps[1]);
    const int tm = kind == 1 ? 128 : 64, tn = kind == 0 ? 128 : 64;
    const long long tiles_pp = (long long)((M + tm - 1) / tm) * ((N + tn - 1) / tn) * batch;      // per party
    // the int32 digit sums of one workgroup stay exact for at most kMaxStepsExact steps
    const int s_exact = (longest + kMaxStepsExact - 1) / kMaxStepsExact;
    int s = s_exact;
    if (tiles_pp * nparty < 160 && longest >= 8) {
        // One workgroup per compute unit at a time: pick the slice count that minimises
        // (rounds of workgroups over the 256 units) x (steps per slice + fixed cost per
        // workgroup: pipeline fill, epilogue, its share of the finishing pass).
        long long best = -1;
        const int s_max = longest / 4 < 32 ? longest / 4 : 32;
        for (int q = s_exact < 1 ? 1 : s_exact; q <= s_max; ++q) {
            const int per = (longest + q - 1) / q;
            long long wgs = 0;
            for (int p = 0; p < nparty; ++p) wgs += tiles_pp * ((steps[p] + per - 1) / per);
            const long long rounds = (wgs + 255) / 256;
            const long long cost = rounds * (per + 6);
            if (best < 0 || cost < best) { best = cost; s = q; }
        }
    }
    if (s <= 1) return 1;
    const int per = (longest + s - 1) / s;
    return (longest + per - 1) / per;          // no empty slice
}

int gemm_ksplit(int M, int N, int batch, int nparty, int total_steps)
{
    const int steps[2] = { total_steps, nparty > 1 ? total_steps : 0 };
    return ksplit_for(M, N, batch, steps);
}

int gemm_ksplit2(int M, int N, int batch, int steps0, int steps1)
{
    const int steps[2] = { steps0, steps1 };
    return ksplit_for(M, N, batch, steps);
}

extern "C" int mpc_set_gemm_small_tile(int max_steps, int min_tiles)
{
    if (max_steps < 0 || min_tiles < 1) return MPC_EINVAL;
    g_small_max_steps.store(max_steps, std::memory_order_relaxed);
    g_small_min_tiles.store(min_tiles, std::memory_order_relaxed);
    return MPC_OK;
}

int launch_limb_gemm(mpc_ctx* c, hipStream_t st, const GemmArgs& g_in)
{
    GemmArgs g = g_in;
    if (g.nparty < 1 || g.nparty > 2 || g.nseg < 1 || g.nseg > 2) return MPC_EINVAL;
    int longest_steps = 0;
    {
        int steps[2] = { 0, 0 };
        for (int p = 0; p < g.nparty; ++p)
            for (int s = 0; s < g.nseg; ++s) steps[p] += g.seg[p][s].KB / KS;
        const int longest = steps[0] > steps[1] ? steps[0] : steps[1];
        longest_steps = longest;
        if (g.ksplit < 1 || !g.partial) g.ksplit = 1;
        g.steps_per_split = (longest + g.ksplit - 1) / g.ksplit;
        if (g.steps_per_split < 1 || g.steps_per_split > kMaxStepsExact) return MPC_ERANGE;
        g.ksplit = 1;
        for (int p = 0; p < 2; ++p) {
            g.ksplit_p[p] = p < g.nparty ? (steps[p] + g.steps_per_split - 1) / g.steps_per_split : 0;      // no empty slice
            if (g.ksplit_p[p] > g.ksplit) g.ksplit = g.ksplit_p[p];
        }
        // the longer contraction first (party 1's by construction of the callers)
        g.heavy_first = g.nparty == 2 && steps[1] > steps[0];
        if (g.nparty == 2 && steps[1] < steps[0]) return MPC_EINVAL;
    }
    if (g.M <= 0 || g.N <= 0 || g.batch <= 0 || g.nseg < 1 || g.nseg > 2) return MPC_EINVAL;
    for (int p = 0; p < g.nparty; ++p)
        for (int s = 0; s < g.nseg; ++s)
            if (g.seg[p][s].KB < (s == 0 ? 1 : 0) || g.seg[p][s].KB % KS) return MPC_EINVAL;     // a second segment may be empty
    // per-lane byte offsets inside one k block of a plane are 32-bit
    if ((long long)g.rows_L * 16 >= (1ll << 32) || (long long)g.N * 16 >= (1ll << 32)) return MPC_EINVAL;
    // 64x128 workgroup tiles, or 128x64 when a second 64-column half would be empty
    const int kind = g.ksplit > 1 ? tile_kind(g.M, g.N, g.batch, 1 << 30, false) : tile_kind(g.M, g.N, g.batch, longest_steps, g.heavy_first != 0);
    if (g.conv.enabled)
        return kind == 2 ? launch_cfg<2, 2, true, 2, 1>(c, st, g) : kind == 1 ? launch_cfg<4, 1, true>(c, st, g) : launch_cfg<2, 2, true>(c, st, g);
    return kind == 2 ? launch_cfg<2, 2, false, 2, 1>(c, st, g) : kind == 1 ? launch_cfg<4, 1, false>(c, st, g) : launch_cfg<2, 2, false>(c, st, g);
}
