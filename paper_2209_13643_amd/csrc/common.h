// Internal declarations shared by the translation units of libmpcpipe.
// Nothing here is part of the C ABI (that is include/mpcpipe.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <utility>
#include <vector>

#include "../../include/mpcpipe.h"

typedef uint64_t u64;
typedef uint8_t u8;

constexpr int kEventPool = 256;
constexpr size_t kAlign = 256;

struct mpc_ctx {
    int device;
    int frac_bits;
    hipStream_t s[3];        // 0, 1: party streams; 2: wire
    bool own_stream[3];
    bool pooled_stream;      // single-queue lane: `pooled` came from the device's fixed set of lane streams
    hipStream_t pooled;
    hipEvent_t ev[kEventPool];
    int ev_next;
    u8* ws;                  // caller-owned workspace
    size_t ws_bytes;
    int last_hip;
    int adder;               // carry network of mpc_relu / mpc_maxpool2x2: MPC_ADDER_*
    bool exchange_put;       // secure ReLU on a single queue: exchange by remote store instead of copy kernels
    size_t relu_chunk[2];    // elements per chunk when n_chunks = 0 (whole words, packed chain); 0: the library's default
    bool capturing;          // between mpc_ctx_capture_begin and mpc_ctx_capture_end
    bool profiling;
    std::vector<std::pair<hipEvent_t, hipEvent_t>> prof[3];   // timing event pairs per region kind
};

static inline size_t align_up(size_t v, size_t a = kAlign) { return (v + a - 1) / a * a; }

// Event pool: an event may be re-recorded once every wait on its previous
// record has been enqueued, which host program order guarantees here because
// each record is followed at once by the waits that consume it.
static inline hipEvent_t next_event(mpc_ctx* c)
{
    hipEvent_t e = c->ev[c->ev_next];
    c->ev_next = (c->ev_next + 1) % kEventPool;
    return e;
}

#define MPC_HIP(ctx, call)                                   \
    do {                                                     \
        hipError_t _e = (call);                              \
        if (_e != hipSuccess) {                              \
            (ctx)->last_hip = (int)_e;                       \
            return MPC_EHIP;                                 \
        }                                                    \
    } while (0)

#define MPC_TRY(expr)                                        \
    do {                                                     \
        int _rc = (expr);                                    \
        if (_rc != MPC_OK) return _rc;                       \
    } while (0)

// record on `from`, make `to` wait for it
static inline int chain(mpc_ctx* c, hipStream_t from, hipStream_t to)
{
    if (from == to) return MPC_OK;
    hipEvent_t e = next_event(c);
    MPC_HIP(c, hipEventRecord(e, from));
    MPC_HIP(c, hipStreamWaitEvent(to, e, 0));
    return MPC_OK;
}

// Start of an entry point: every stream of the lane waits for the work already
// enqueued on the other two, so a call may reuse the workspace and may read the
// previous call's outputs of either party.
static inline int lane_join(mpc_ctx* c)
{
    if (c->s[0] == c->s[1] && c->s[1] == c->s[2]) return MPC_OK;   // one in-order queue: nothing to join
    hipEvent_t e[3];
    for (int i = 0; i < 3; ++i) {
        e[i] = next_event(c);
        MPC_HIP(c, hipEventRecord(e[i], c->s[i]));
    }
    for (int i = 0; i < 3; ++i)
        for (int j = 0; j < 3; ++j)
            if (i != j && c->s[i] != c->s[j]) MPC_HIP(c, hipStreamWaitEvent(c->s[i], e[j], 0));
    return MPC_OK;
}

// End of an entry point that issued everything on the lane's first stream: the
// other two streams wait for it, so whichever stream the caller synchronises
// sees the outputs.
static inline int lane_fanout(mpc_ctx* c)
{
    MPC_TRY(chain(c, c->s[0], c->s[1]));
    if (c->s[2] != c->s[1]) MPC_TRY(chain(c, c->s[0], c->s[2]));
    return MPC_OK;
}

// Timing regions (no-ops unless profiling is on): prof_begin records a start
// event on `st` and returns its index, prof_end records the matching stop.
static inline int prof_begin(mpc_ctx* c, int which, hipStream_t st)
{
    if (!c->profiling) return -1;
    hipEvent_t a, b;
    if (hipEventCreate(&a) != hipSuccess) return -1;
    if (hipEventCreate(&b) != hipSuccess) { (void)hipEventDestroy(a); return -1; }
    (void)hipEventRecord(a, st);
    c->prof[which].push_back({ a, b });
    return (int)c->prof[which].size() - 1;
}
static inline void prof_end(mpc_ctx* c, int which, int idx, hipStream_t st)
{
    if (idx >= 0) (void)hipEventRecord(c->prof[which][idx].second, st);
}

// Bump allocator over the workspace.
struct WsAlloc {
    u8* base; size_t cap; size_t off; bool ok;
    WsAlloc(u8* b, size_t c) : base(b), cap(c), off(0), ok(true) {}
    template <typename T> T* take(size_t count)
    {
        size_t bytes = align_up(count * sizeof(T));
        if (!base || off + bytes > cap) { ok = false; off += bytes; return nullptr; }
        T* p = reinterpret_cast<T*>(base + off);
        off += bytes;
        return p;
    }
};

// resolves, once per device, the address of the fixed scratch array of mpc_relu_static (relu.hip);
// called by mpc_ctx_create with the context's device current
int relu_static_setup(mpc_ctx* c);

// ---- element-wise launchers (elementwise.hip) --------------------------------
int launch_sub(mpc_ctx* c, hipStream_t st, const u64* x, const u64* a, u64* out, size_t n);
int launch_add(mpc_ctx* c, hipStream_t st, const u64* x, const u64* y, u64* out, size_t n);
int launch_copy(mpc_ctx* c, hipStream_t st, const void* src, void* dst, size_t bytes);
int launch_truncate(mpc_ctx* c, hipStream_t st, u64* z, size_t n, int bits, int party);
int launch_sum3(mpc_ctx* c, hipStream_t st, const u64* x, const u64* y, const u64* w, u64* out, size_t n);

// ---- digit planes -------------------------------------------------------------
// A digit-plane tensor stores a [rows][K] ring matrix as eight int8 planes,
// one per balanced base-256 digit, each laid out [kb][row][16]: 16 consecutive
// k of one row are one 16-byte unit, units of consecutive rows are adjacent.
// KB is padded to an even number of blocks; digits beyond K are zero.
static inline int kblocks(int K) { int kb = (K + 15) / 16; return (kb + 1) & ~1; }
static inline size_t plane_bytes(int rows, int KB) { return (size_t)KB * rows * 16; }

struct RecodeArgs {
    const u64* src;       // element (row r, k) at src[r*row_stride + k*k_stride (+ tap*tap_stride)]
    const u64* src2;      // optional addends with the same indexing (nullptr: none)
    const u64* src3;
    const u64* sub;       // optional: subtracted from src first (v = src - sub), same indexing
    u64* side;            // optional: v is also stored here, same indexing (a mask kernel's output, formed on the way)
    const u64* minuend;   // optional, with side and without sub: side = minuend - src instead (src itself is recoded)
    u8* dst;              // plane base
    long long row_stride, k_stride, tap_stride;
    int plane_rows;       // rows of the plane tensor (>= rows); rows beyond `rows` are zero-filled
    int rows, K;          // valid extent per tap
    int KB_tap;           // k-blocks per tap (ceil(K/16))
    int ntaps;            // filter taps (1 for a plain matrix)
    int KB_total;         // padded k-blocks of the plane tensor (>= ntaps*KB_tap)
    long long digit_stride;   // bytes between digit planes
    long long src_batch_stride, dst_batch_stride;  // elements / bytes
    int batch;
};
int launch_recode(mpc_ctx* c, hipStream_t st, const RecodeArgs& a);
constexpr int kMaxRecodeSets = 6;
struct RecodeBatch { RecodeArgs a[kMaxRecodeSets]; int batch; };
int launch_recode_multi(mpc_ctx* c, hipStream_t st, const RecodeArgs* sets, int count);
int launch_recode_any(mpc_ctx* c, hipStream_t st, const RecodeArgs* sets, int count);

// transposed im2col planes of an NHWC tensor (left operand of the filter-gradient product)
struct Im2colTArgs {
    const u64* src; const u64* src2;      // [B][H][W][Cin]; optional addend with the same indexing
    u8* dst;                              // planes: rows = KH*KW*Cin, k = output pixel
    int B, H, W, Cin, KH, KW, pad, stride, Ho, Wo;
    int KB_total;                         // padded k blocks (>= ceil(B*Ho*Wo / 16))
    long long digit_stride;
};
struct Im2colTBatch { Im2colTArgs a[3]; };
int launch_recode_im2col_t(mpc_ctx* c, hipStream_t st, const Im2colTArgs* sets, int count);

// element-wise Alg. 1 (mask kernel, then finish kernel after the exchange)
struct MulArgs {
    const u64 *x[2], *y[2], *a[2], *b[2], *c[2];
    u64 *se[2], *sf[2];                   // own masked words
    const u64 *re[2], *rf[2];             // received masked words
    u64* z[2];
    size_t n; int trunc_bits; int mask_from_sign;
};
int launch_mul_mask(mpc_ctx* c, hipStream_t st, const MulArgs& q);
int launch_mul_finish(mpc_ctx* c, hipStream_t st, const MulArgs& q);

// max-pool backward: the local steps around its two element-wise products
struct PoolBwdArgs {
    const u64* g[2]; const u64* gu[2];    // output gradient, grad_u = g * mask2
    u64* pairs[2];                        // [2*n_out] (grad_u, grad_v) interleaved
    const u64* prod[2];                   // pairs * mask1
    u64* gx[2];                           // [B][H][W][C]
    size_t n_out; int B, H, W, C;
};
int launch_poolbwd_pairs(mpc_ctx* c, hipStream_t st, const PoolBwdArgs& q);
int launch_poolbwd_scatter(mpc_ctx* c, hipStream_t st, const PoolBwdArgs& q);

// scatter of up to four [B][Ho][Wo][C] tensors into zero-filled [B][Hd][Wd][C] grids at pixel (ho*stride, wo*stride)
struct DilateArgs { const u64* src[4]; u64* dst[4]; int B, Ho, Wo, Hd, Wd, C, stride; };
int launch_dilate(mpc_ctx* c, hipStream_t st, const DilateArgs& q);

// several element-wise jobs in one launch (single-queue lanes)
constexpr int kMaxSegs = 6;
struct SubSeg { const u64* x; const u64* a; u64* out; size_t n; int vec; u64* out2; };   // out2: optional second destination
struct SubBatch { SubSeg s[kMaxSegs]; };
struct CopySeg { const u8* src; u8* dst; size_t bytes; int vec; };
struct CopyBatch { CopySeg s[kMaxSegs]; };
int launch_sub_multi(mpc_ctx* c, hipStream_t st, const SubSeg* segs, int count);
int launch_copy_multi(mpc_ctx* c, hipStream_t st, const CopySeg* segs, int count);

// ---- limb GEMM (limb_gemm.hip) --------------------------------------------------
struct GemmSeg {
    const u8* L; const u8* R;         // digit planes (left: rows = M or pixels; right: rows = N)
    long long L_dstride, R_dstride;   // bytes between digit planes
    long long L_bstride, R_bstride;   // bytes between batch items
    int KB;                           // 16-wide k blocks to contract (even)
};
struct ConvGeom {
    int enabled;
    int H, W, Ho, Wo, CB, KH, KW, pad, stride;
    long long npix;                   // B*H*W: rows of the activation planes
};
struct GemmArgs {
    GemmSeg seg[2][2];                // [party][segment]
    int nseg, nparty;
    const u64* addend[2];             // c_i, may be nullptr
    const u64* addend2[2];            // partial sums of an earlier phase, may be nullptr
    u64* out[2];
    int M, N, batch;
    long long out_bstride;            // elements between batch items of addend/out
    int trunc_bits;                   // 0: none
    int rows_L;                       // rows of the left planes (plain: M)
    ConvGeom conv;
    int ksplit;                       // > 1: split the (longest party's) contraction over this many workgroups per tile
    int steps_per_split;              // filled by the launcher
    int tiles_m, tiles_n;             // filled by the launcher: output tiles per matrix
    int ksplit_p[2];                  // filled by the launcher: slices of each party's contraction (equal unless the
                                      // parties contract different lengths: a party's second segment may have KB = 0)
    int tiles_party[2];               // filled by the launcher: tiles x batch x ksplit_p
    int heavy_first;                  // filled by the launcher: 1 = all workgroups of party 1 (the longer contraction)
                                      // come before party 0's in the grid, so the long ones start first
    u64* partial;                     // [ksplit][nparty][batch][M][N] partial products (ksplit > 1)
};
int gemm_ksplit(int M, int N, int batch, int nparty, int total_steps);
// the same choice when party 0 contracts steps0 and party 1 steps1 K steps (slices of the longer one)
int gemm_ksplit2(int M, int N, int batch, int steps0, int steps1);
int launch_limb_gemm(mpc_ctx* c, hipStream_t st, const GemmArgs& g);
