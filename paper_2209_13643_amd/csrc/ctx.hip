// Context (execution lane), opening and truncation entry points.
#include "common.h"

#include <mutex>
#include <new>

namespace {

// Streams of the single-queue lanes.  The runtime multiplexes streams onto a small number of hardware queues (four
// by default), and how well lanes overlap was found to depend on how many distinct streams the process has used
// before: four lanes made after one other lane had run lost half of their overlap.  Single-queue lanes therefore
// draw their stream from a fixed set of four per device, made once and kept until the process ends; a lane takes the
// least used one, a fifth concurrent lane shares a stream with another (the two are then ordered with each other,
// as two streams on one hardware queue would be).
constexpr int kLaneStreams = 4, kPoolDevices = 16;
struct LaneStreamPool {
    std::mutex mu;
    bool made[kPoolDevices] = {};
    hipStream_t s[kPoolDevices][kLaneStreams] = {};
    int users[kPoolDevices][kLaneStreams] = {};
} g_lane_streams;

hipError_t lane_stream_acquire(int device, hipStream_t* out)
{
    if (device < 0 || device >= kPoolDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_lane_streams.mu);
    if (!g_lane_streams.made[device]) {
        for (int i = 0; i < kLaneStreams; ++i) {
            const hipError_t e = hipStreamCreateWithFlags(&g_lane_streams.s[device][i], hipStreamNonBlocking);
            if (e != hipSuccess) {
                for (int j = 0; j < i; ++j) { (void)hipStreamDestroy(g_lane_streams.s[device][j]); g_lane_streams.s[device][j] = nullptr; }
                return e;
            }
        }
        g_lane_streams.made[device] = true;
    }
    int best = 0;
    for (int i = 1; i < kLaneStreams; ++i)
        if (g_lane_streams.users[device][i] < g_lane_streams.users[device][best]) best = i;
    ++g_lane_streams.users[device][best];
    *out = g_lane_streams.s[device][best];
    return hipSuccess;
}

int lane_stream_users(int device, hipStream_t st)
{
    if (device < 0 || device >= kPoolDevices) return 0;
    std::lock_guard<std::mutex> lock(g_lane_streams.mu);
    for (int i = 0; i < kLaneStreams; ++i)
        if (g_lane_streams.s[device][i] == st) return g_lane_streams.users[device][i];
    return 0;
}

void lane_stream_release(int device, hipStream_t st)
{
    if (device < 0 || device >= kPoolDevices) return;
    std::lock_guard<std::mutex> lock(g_lane_streams.mu);
    for (int i = 0; i < kLaneStreams; ++i)
        if (g_lane_streams.s[device][i] == st && g_lane_streams.users[device][i] > 0) { --g_lane_streams.users[device][i]; return; }
}

}  // namespace

extern "C" {

static int ctx_create(mpc_ctx** out, int device, int frac_bits, int n_streams)
{
    if (!out || frac_bits < 0 || frac_bits > 62) return MPC_EINVAL;
    mpc_ctx* c = new (std::nothrow) mpc_ctx();
    if (!c) return MPC_ENOMEM;
    c->device = device; c->frac_bits = frac_bits; c->ev_next = 0;
    c->ws = nullptr; c->ws_bytes = 0; c->last_hip = 0; c->profiling = false;
    c->relu_chunk[0] = c->relu_chunk[1] = 0;
    for (int i = 0; i < 3; ++i) { c->s[i] = nullptr; c->own_stream[i] = false; }
    for (int i = 0; i < kEventPool; ++i) c->ev[i] = nullptr;
    hipError_t e = hipSetDevice(device);
    c->pooled_stream = false;
    if (n_streams == 1) {
        // one in-order queue for everything, drawn from the device's fixed set
        if (e == hipSuccess) e = lane_stream_acquire(device, &c->s[0]);
        if (e == hipSuccess) { c->pooled_stream = true; c->pooled = c->s[0]; c->s[1] = c->s[2] = c->s[0]; }
    } else {
        for (int i = 0; i < 3 && e == hipSuccess; ++i) {
            e = hipStreamCreateWithFlags(&c->s[i], hipStreamNonBlocking);
            c->own_stream[i] = (e == hipSuccess);
        }
    }
    for (int i = 0; i < kEventPool && e == hipSuccess; ++i)
        e = hipEventCreateWithFlags(&c->ev[i], hipEventDisableTiming);
    if (e != hipSuccess) {
        (void)mpc_ctx_destroy(c);       // releases whatever was created; the HIP code is lost with the context
        return MPC_EHIP;
    }
    if (relu_static_setup(c) != MPC_OK) { (void)mpc_ctx_destroy(c); return MPC_EHIP; }
    *out = c;
    return MPC_OK;
}

int mpc_ctx_create(mpc_ctx** out, int device, int frac_bits) { return ctx_create(out, device, frac_bits, 3); }

int mpc_ctx_create_single_queue(mpc_ctx** out, int device, int frac_bits) { return ctx_create(out, device, frac_bits, 1); }

int mpc_ctx_destroy(mpc_ctx* c)
{
    if (!c) return MPC_EINVAL;
    for (int i = 0; i < 3; ++i)
        if (c->s[i]) (void)hipStreamSynchronize(c->s[i]);
    for (int i = 0; i < kEventPool; ++i)
        if (c->ev[i]) (void)hipEventDestroy(c->ev[i]);
    (void)mpc_ctx_profile_reset(c);
    for (int i = 0; i < 3; ++i)
        if (c->own_stream[i] && c->s[i]) (void)hipStreamDestroy(c->s[i]);
    if (c->pooled_stream) lane_stream_release(c->device, c->pooled);
    delete c;
    return MPC_OK;
}

int mpc_ctx_set_streams(mpc_ctx* c, void* s0, void* s1, void* sw)
{
    if (!c || c->capturing) return MPC_EINVAL;
    void* in[3] = { s0, s1, sw };
    for (int i = 0; i < 3; ++i) {
        if (!in[i] || in[i] == (void*)c->s[i]) continue;
        if (c->own_stream[i]) {
            MPC_HIP(c, hipStreamSynchronize(c->s[i]));
            MPC_HIP(c, hipStreamDestroy(c->s[i]));
            c->own_stream[i] = false;
        }
        c->s[i] = (hipStream_t)in[i];
    }
    return MPC_OK;
}

void* mpc_ctx_stream(mpc_ctx* c, int which)
{
    if (!c || which < 0 || which > 2) return nullptr;
    return (void*)c->s[which];
}

int mpc_ctx_set_workspace(mpc_ctx* c, void* p, size_t bytes)
{
    if (!c || c->capturing) return MPC_EINVAL;
    if (p && ((uintptr_t)p % kAlign) != 0) return MPC_EINVAL;
    c->ws = (u8*)p;
    c->ws_bytes = p ? bytes : 0;
    return MPC_OK;
}

int mpc_ctx_sync(mpc_ctx* c)
{
    if (!c || c->capturing) return MPC_EINVAL;      // a capturing queue cannot be waited for
    for (int i = 0; i < 3; ++i) MPC_HIP(c, hipStreamSynchronize(c->s[i]));
    return MPC_OK;
}

int mpc_ctx_wait(mpc_ctx* c, mpc_ctx* after)
{
    if (!c || !after) return MPC_EINVAL;
    for (int i = 0; i < 2; ++i) {
        hipEvent_t e = next_event(after);
        MPC_HIP(after, hipEventRecord(e, after->s[i]));
        for (int j = 0; j < 2; ++j) MPC_HIP(c, hipStreamWaitEvent(c->s[j], e, 0));
    }
    return MPC_OK;
}

// ---- graph capture: a sequence of calls on a single-queue lane recorded once, replayed many times
struct mpc_graph { hipGraph_t graph; hipGraphExec_t exec; };

int mpc_ctx_capture_begin(mpc_ctx* c)
{
    if (!c || c->capturing || c->profiling) return MPC_EINVAL;
    if (!(c->s[0] == c->s[1] && c->s[1] == c->s[2])) return MPC_EINVAL;      // events between streams are not recorded
    // a stream shared with another lane (more than four single-queue lanes alive) would record that lane's calls too
    if (c->pooled_stream && c->s[0] == c->pooled && lane_stream_users(c->device, c->pooled) > 1) return MPC_EINVAL;
    MPC_HIP(c, hipStreamBeginCapture(c->s[0], hipStreamCaptureModeRelaxed));
    c->capturing = true;
    return MPC_OK;
}

int mpc_ctx_capture_end(mpc_ctx* c, mpc_graph** out)
{
    if (!c || !out || !c->capturing) return MPC_EINVAL;
    c->capturing = false;
    hipGraph_t g = nullptr;
    MPC_HIP(c, hipStreamEndCapture(c->s[0], &g));
    if (!g) return MPC_EHIP;
    hipGraphExec_t e = nullptr;
    const hipError_t err = hipGraphInstantiate(&e, g, nullptr, nullptr, 0);
    if (err != hipSuccess) { c->last_hip = (int)err; (void)hipGraphDestroy(g); return MPC_EHIP; }
    mpc_graph* mg = new (std::nothrow) mpc_graph{ g, e };
    if (!mg) { (void)hipGraphExecDestroy(e); (void)hipGraphDestroy(g); return MPC_ENOMEM; }
    *out = mg;
    return MPC_OK;
}

int mpc_graph_launch(mpc_graph* g, mpc_ctx* c)
{
    if (!g || !c || c->capturing) return MPC_EINVAL;
    MPC_TRY(lane_join(c));
    MPC_HIP(c, hipGraphLaunch(g->exec, c->s[0]));
    MPC_TRY(chain(c, c->s[0], c->s[1]));
    return MPC_OK;
}

int mpc_graph_destroy(mpc_graph* g)
{
    if (!g) return MPC_EINVAL;
    (void)hipGraphExecDestroy(g->exec);
    (void)hipGraphDestroy(g->graph);
    delete g;
    return MPC_OK;
}

int mpc_ctx_set_exchange(mpc_ctx* c, int mode)
{
    if (!c || (mode != MPC_EXCHANGE_COPY && mode != MPC_EXCHANGE_PUT)) return MPC_EINVAL;
    c->exchange_put = mode == MPC_EXCHANGE_PUT;
    return MPC_OK;
}

int mpc_ctx_set_adder(mpc_ctx* c, int adder)
{
    if (!c || (adder != MPC_ADDER_KOGGE_STONE && adder != MPC_ADDER_TREE)) return MPC_EINVAL;
    c->adder = adder;
    return MPC_OK;
}

int mpc_ctx_set_profiling(mpc_ctx* c, int enable)
{
    if (!c || c->capturing) return MPC_EINVAL;
    c->profiling = enable != 0;
    return MPC_OK;
}

int mpc_ctx_profile(mpc_ctx* c, int which, double* total_ms, int* count)
{
    if (!c || which < 0 || which > 2 || !total_ms || !count) return MPC_EINVAL;
    MPC_TRY(mpc_ctx_sync(c));
    double sum = 0.0;
    for (auto& pr : c->prof[which]) {
        float ms = 0.f;
        MPC_HIP(c, hipEventElapsedTime(&ms, pr.first, pr.second));
        sum += ms;
    }
    *total_ms = sum;
    *count = (int)c->prof[which].size();
    return MPC_OK;
}

int mpc_ctx_profile_samples(mpc_ctx* c, int which, double* ms_out, int capacity, int* count)
{
    if (!c || which < 0 || which > 2 || !count || capacity < 0 || (capacity > 0 && !ms_out)) return MPC_EINVAL;
    MPC_TRY(mpc_ctx_sync(c));
    const int n = (int)c->prof[which].size();
    for (int i = 0; i < n && i < capacity; ++i) {
        float ms = 0.f;
        MPC_HIP(c, hipEventElapsedTime(&ms, c->prof[which][i].first, c->prof[which][i].second));
        ms_out[i] = ms;
    }
    *count = n;
    return MPC_OK;
}

int mpc_ctx_profile_reset(mpc_ctx* c)
{
    if (!c) return MPC_EINVAL;
    for (int k = 0; k < 3; ++k) {
        for (auto& pr : c->prof[k]) { (void)hipEventDestroy(pr.first); (void)hipEventDestroy(pr.second); }
        c->prof[k].clear();
    }
    return MPC_OK;
}

int mpc_last_hip_error(const mpc_ctx* c) { return c ? c->last_hip : 0; }

const char* mpc_strerror(int code)
{
    switch (code) {
    case MPC_OK: return "success";
    case MPC_EINVAL: return "invalid argument (null pointer, non-positive size or unsupported shape)";
    case MPC_ENOMEM: return "workspace missing or too small for this call";
    case MPC_EHIP: return "a HIP runtime call failed (see mpc_last_hip_error)";
    case MPC_ERANGE: return "size out of range: contraction beyond the exact int32 digit-sum bound, or more elements than a fixed-size entry point holds";
    default: return "unknown mpcpipe error code";
    }
}

// out = s0 + s1.  Each share is copied once over the wire stream into the
// workspace ("received"), then party 0's stream adds the two.
int mpc_open(mpc_ctx* c, mpc_cshare s, uint64_t* out, size_t n)
{
    if (!c || !s.p[0] || !s.p[1] || !out || n == 0) return MPC_EINVAL;
    WsAlloc ws(c->ws, c->ws_bytes);
    u64* r0 = ws.take<u64>(n);
    u64* r1 = ws.take<u64>(n);
    if (!ws.ok) return MPC_ENOMEM;
    MPC_TRY(lane_join(c));
    MPC_TRY(launch_copy(c, c->s[2], s.p[0], r0, n * sizeof(u64)));
    MPC_TRY(launch_copy(c, c->s[2], s.p[1], r1, n * sizeof(u64)));
    MPC_TRY(chain(c, c->s[2], c->s[0]));
    MPC_TRY(launch_add(c, c->s[0], r0, r1, out, n));
    // the workspace may be reused by party 1's next call only after the add
    MPC_TRY(chain(c, c->s[0], c->s[1]));
    return MPC_OK;
}

int mpc_sub(mpc_ctx* c, mpc_cshare x, mpc_cshare a, mpc_share out, size_t n)
{
    if (!c || n == 0) return MPC_EINVAL;
    for (int i = 0; i < 2; ++i) if (!x.p[i] || !a.p[i] || !out.p[i]) return MPC_EINVAL;
    MPC_TRY(lane_join(c));
    for (int i = 0; i < 2; ++i) MPC_TRY(launch_sub(c, c->s[i], x.p[i], a.p[i], out.p[i], n));
    return MPC_OK;
}

int mpc_add(mpc_ctx* c, mpc_cshare x, mpc_cshare y, mpc_share out, size_t n)
{
    if (!c || n == 0) return MPC_EINVAL;
    for (int i = 0; i < 2; ++i) if (!x.p[i] || !y.p[i] || !out.p[i]) return MPC_EINVAL;
    MPC_TRY(lane_join(c));
    for (int i = 0; i < 2; ++i) MPC_TRY(launch_add(c, c->s[i], x.p[i], y.p[i], out.p[i], n));
    return MPC_OK;
}

size_t mpc_mul_workspace_bytes(size_t n) { return n ? 8 * align_up(n * sizeof(u64)) : 0; }

// Element-wise Alg. 1.  Both parties' mask and finish kernels share a launch on
// party 0's stream; the exchange of the masked words runs on the wire stream.
static int mul_entry(mpc_ctx* c, mpc_cshare x, mpc_cshare y, mpc_cshare a, mpc_cshare b, mpc_cshare cc,
                     mpc_share z, size_t n, int flags, int mask_from_sign, size_t ws_off = 0)
{
    if (!c || n == 0 || (flags & ~MPC_TRUNCATE)) return MPC_EINVAL;
    for (int i = 0; i < 2; ++i)
        if (!x.p[i] || !y.p[i] || !a.p[i] || !b.p[i] || !cc.p[i] || !z.p[i]) return MPC_EINVAL;
    if (ws_off > c->ws_bytes) return MPC_ENOMEM;
    WsAlloc ws(c->ws ? c->ws + ws_off : nullptr, c->ws_bytes - ws_off);
    MulArgs q{};
    u64 *re[2], *rf[2];
    for (int i = 0; i < 2; ++i) {
        q.se[i] = ws.take<u64>(n); q.sf[i] = ws.take<u64>(n);
        re[i] = ws.take<u64>(n); rf[i] = ws.take<u64>(n);
    }
    if (!ws.ok) return MPC_ENOMEM;
    for (int i = 0; i < 2; ++i) {
        q.x[i] = x.p[i]; q.y[i] = y.p[i]; q.a[i] = a.p[i]; q.b[i] = b.p[i]; q.c[i] = cc.p[i]; q.z[i] = z.p[i];
        q.re[i] = re[i]; q.rf[i] = rf[i];
    }
    q.n = n; q.trunc_bits = (flags & MPC_TRUNCATE) ? c->frac_bits : 0; q.mask_from_sign = mask_from_sign;
    MPC_TRY(lane_join(c));
    MPC_TRY(launch_mul_mask(c, c->s[0], q));
    MPC_TRY(chain(c, c->s[0], c->s[2]));
    CopySeg cp[4];
    for (int i = 0; i < 2; ++i) {
        cp[2 * i] = CopySeg{ (const u8*)q.se[i], (u8*)re[1 - i], n * sizeof(u64), 0 };
        cp[2 * i + 1] = CopySeg{ (const u8*)q.sf[i], (u8*)rf[1 - i], n * sizeof(u64), 0 };
    }
    MPC_TRY(launch_copy_multi(c, c->s[2], cp, 4));
    MPC_TRY(chain(c, c->s[2], c->s[0]));
    MPC_TRY(launch_mul_finish(c, c->s[0], q));
    MPC_TRY(chain(c, c->s[0], c->s[1]));
    return MPC_OK;
}

int mpc_mul(mpc_ctx* c, mpc_cshare x, mpc_cshare y, mpc_cshare a, mpc_cshare b, mpc_cshare cc, mpc_share z,
            size_t n, int flags)
{
    return mul_entry(c, x, y, a, b, cc, z, n, flags, 0);
}

int mpc_relu_backward(mpc_ctx* c, mpc_cshare g, mpc_cshare s_arith, mpc_cshare a, mpc_cshare b, mpc_cshare cc,
                      mpc_share gx, size_t n)
{
    return mul_entry(c, g, s_arith, a, b, cc, gx, n, 0, 1);
}

size_t mpc_maxpool_backward_workspace_bytes(int B, int H, int W, int C)
{
    if (B <= 0 || H <= 0 || W <= 0 || C <= 0 || (H & 1) || (W & 1)) return 0;
    const size_t n_out = (size_t)B * (H / 2) * (W / 2) * C;
    // per party grad_u (n_out), pairs and their product (2 n_out each); then the larger product's scratch
    return 2 * (align_up(n_out * 8) + 2 * align_up(2 * n_out * 8)) + mpc_mul_workspace_bytes(2 * n_out);
}

// Backward of mpc_maxpool2x2: two element-wise products with the masks of the
// two conversions and local sums around them.
int mpc_maxpool2x2_backward(mpc_ctx* c, mpc_cshare g, mpc_cshare s1, mpc_cshare s2,
                            mpc_cshare a1, mpc_cshare b1, mpc_cshare c1,
                            mpc_cshare a2, mpc_cshare b2, mpc_cshare c2,
                            mpc_share gx, int B, int H, int W, int C)
{
    if (!c || B <= 0 || H <= 0 || W <= 0 || C <= 0 || (H & 1) || (W & 1)) return MPC_EINVAL;
    for (int i = 0; i < 2; ++i)
        if (!g.p[i] || !s1.p[i] || !s2.p[i] || !gx.p[i]) return MPC_EINVAL;
    const size_t n_out = (size_t)B * (H / 2) * (W / 2) * C;
    WsAlloc ws(c->ws, c->ws_bytes);
    mpc_share gu, pairs, prod;
    for (int i = 0; i < 2; ++i) {
        gu.p[i] = ws.take<u64>(n_out); pairs.p[i] = ws.take<u64>(2 * n_out); prod.p[i] = ws.take<u64>(2 * n_out);
    }
    if (!ws.ok) return MPC_ENOMEM;
    const size_t off = ws.off;
    const mpc_cshare pairs_c = { { pairs.p[0], pairs.p[1] } };
    // grad_u = g * (1 - s2)
    MPC_TRY(mul_entry(c, g, s2, a2, b2, c2, gu, n_out, 0, 1, off));
    PoolBwdArgs q{};
    for (int i = 0; i < 2; ++i) { q.g[i] = g.p[i]; q.gu[i] = gu.p[i]; q.pairs[i] = pairs.p[i]; q.prod[i] = prod.p[i]; q.gx[i] = gx.p[i]; }
    q.n_out = n_out; q.B = B; q.H = H; q.W = W; q.C = C;
    MPC_TRY(launch_poolbwd_pairs(c, c->s[0], q));
    MPC_TRY(chain(c, c->s[0], c->s[1]));
    // (grad_p00, grad_p10) = (grad_u, grad_v) * (1 - s1)
    MPC_TRY(mul_entry(c, pairs_c, s1, a1, b1, c1, prod, 2 * n_out, 0, 1, off));
    MPC_TRY(launch_poolbwd_scatter(c, c->s[0], q));
    MPC_TRY(chain(c, c->s[0], c->s[1]));
    return MPC_OK;
}

int mpc_truncate(mpc_ctx* c, mpc_share z, size_t n, int bits)
{
    if (!c || !z.p[0] || !z.p[1] || n == 0 || bits < 0 || bits > 63) return MPC_EINVAL;
    MPC_TRY(lane_join(c));
    MPC_TRY(launch_truncate(c, c->s[0], z.p[0], n, bits, 0));
    MPC_TRY(launch_truncate(c, c->s[1], z.p[1], n, bits, 1));
    return MPC_OK;
}

}  // extern "C"
