// Measurement aid: the int8 matrix-core rate this device sustains on register-resident operands, in the
// instruction order of the GEMM's K step (72 v_mfma_i32_32x32x32_i8 into 16 accumulator tiles, one wave per
// SIMD), with no memory traffic at all.  The chip is power-limited: the clock it holds, and with it the rate,
// depends on how much the operand bits toggle, so the ceiling for uniformly random digits (what secret shares
// are) lies well below the one for constant operands and below the published peak.
#include "common.h"

#include <type_traits>

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int kRateThreads = 256;          // four waves: one per SIMD, as the GEMM's workgroups
constexpr int kRateGroupsPerCu = 1;
constexpr int kMfmaPerIter = 72;

template <typename F, int... Is>
__device__ __forceinline__ void unroll_impl(F&& f, std::integer_sequence<int, Is...>) { (f(std::integral_constant<int, Is>{}), ...); }
template <int N, typename F>
__device__ __forceinline__ void unroll(F&& f) { unroll_impl(f, std::make_integer_sequence<int, N>{}); }

__global__ __launch_bounds__(kRateThreads, 1) void k_mfma_rate(int* __restrict__ out, int iters, unsigned seed)
{
    // seed 0: all-zero operands; otherwise every byte of every operand register is a uniform pseudo-random digit
    unsigned s = (seed ^ ((unsigned)blockIdx.x * kRateThreads + threadIdx.x)) * 2654435761u + 12345u;
    auto word = [&]() -> int {
        s = s * 1664525u + 1013904223u;
        const unsigned r = s ^ (s >> 13) ^ (s << 7);
        return seed ? (int)r : 0;
    };
    v4i A[8], B[2][8];
#pragma unroll
    for (int d = 0; d < 8; ++d) {
        A[d] = v4i{ word(), word(), word(), word() };
        B[0][d] = v4i{ word(), word(), word(), word() };
        B[1][d] = v4i{ word(), word(), word(), word() };
    }
    v16i acc[2][8];
#pragma unroll
    for (int c = 0; c < 2; ++c)
#pragma unroll
        for (int q = 0; q < 8; ++q)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[c][q][v] = 0;
    for (int it = 0; it < iters; ++it) {
        // the GEMM's order: blocks over the right-operand digit j, left digits 7-j .. 0, both column halves
        unroll<8>([&](auto jt) {
            constexpr int j = decltype(jt)::value;
            unroll<8 - j>([&](auto it2) {
                constexpr int i = 7 - j - decltype(it2)::value;
                acc[0][i + j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(A[i], B[0][j], acc[0][i + j], 0, 0, 0);
                acc[1][i + j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(A[i], B[1][j], acc[1][i + j], 0, 0, 0);
            });
        });
    }
    int r = 0;
#pragma unroll
    for (int c = 0; c < 2; ++c)
#pragma unroll
        for (int q = 0; q < 8; ++q)
#pragma unroll
            for (int v = 0; v < 16; ++v) r ^= acc[c][q][v];
    out[(size_t)blockIdx.x * kRateThreads + threadIdx.x] = r;
}

}  // namespace

extern "C" int mpc_mfma_rate(mpc_ctx* c, int random_operands, int iters, int launches, double* int8_ops_per_s)
{
    if (!c || !int8_ops_per_s || iters < 1 || iters > (1 << 20) || launches < 1 || launches > 1024) return MPC_EINVAL;
    if (c->capturing) return MPC_EINVAL;
    hipDeviceProp_t prop;
    MPC_HIP(c, hipGetDeviceProperties(&prop, c->device));
    const int groups = prop.multiProcessorCount * kRateGroupsPerCu;
    const size_t need = (size_t)groups * kRateThreads * sizeof(int);
    if (!c->ws || c->ws_bytes < need) return MPC_ENOMEM;
    hipStream_t st = c->s[0];
    MPC_TRY(lane_join(c));
    hipEvent_t t0, t1;
    MPC_HIP(c, hipEventCreate(&t0));
    if (hipEventCreate(&t1) != hipSuccess) { (void)hipEventDestroy(t0); return MPC_EHIP; }
    int rc = MPC_OK;
    float ms = 0.f;
    hipError_t e = hipEventRecord(t0, st);
    for (int l = 0; l < launches && e == hipSuccess; ++l) {
        hipLaunchKernelGGL(k_mfma_rate, dim3(groups), dim3(kRateThreads), 0, st, (int*)c->ws, iters,
                           random_operands ? 0x9e3779b9u + (unsigned)l : 0u);
        e = hipGetLastError();
    }
    if (e == hipSuccess) e = hipEventRecord(t1, st);
    if (e == hipSuccess) e = hipEventSynchronize(t1);
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, t0, t1);
    if (e != hipSuccess) { c->last_hip = (int)e; rc = MPC_EHIP; }
    (void)hipEventDestroy(t0); (void)hipEventDestroy(t1);
    if (rc != MPC_OK) return rc;
    // waves x iterations x 72 instructions x 32*32*32 multiply-accumulates x 2
    const double ops = (double)groups * (kRateThreads / 64) * (double)iters * kMfmaPerIter * 65536.0 * launches;
    *int8_ops_per_s = ms > 0.f ? ops / (ms * 1e-3) : 0.0;
    return MPC_OK;
}
