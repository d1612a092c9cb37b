// selective_state_update: one generated token, i.e. the scan's recurrence taken for a single step from the carried
// state (the state selective_scan_fwd leaves in last_state), updated in place.
//
// A (sequence, channel) row owns N consecutive binary32 states.  A row is spread over LPR = 2^k lanes, each lane
// taking 16-byte groups of four states (LPR = ceil(N / 4) rounded up to a power of two, at most 64), so a wave reads
// and writes whole contiguous stretches of the state tensor; the row's readout sum_n C[n] h'[n] is folded across
// its lanes with butterfly shuffles and its first lane applies the skip term and the gate.  The arithmetic is the
// scan kernel's: softplus, exp2(dl * (A * log2 e)), one fused multiply-add per state.
// Work bound by the state traffic (8 bytes per state); nothing here is a contraction.
#include <hip/hip_runtime.h>

#include "corey_internal.h"
#include "corey_scan_impl.h"

namespace {

using corey_scan::fast_exp2;
using corey_scan::Io;
using corey_scan::kLog2e;
using corey_scan::silu;
using corey_scan::softplus;

constexpr int kThreads = 256;
typedef float float4v __attribute__((ext_vector_type(4)));

template <typename T>
__global__ __launch_bounds__(kThreads) void k_state_update(float* __restrict__ state, const T* __restrict__ x,
                                                           const T* __restrict__ delta, const float* __restrict__ A,
                                                           const T* __restrict__ Bt, const T* __restrict__ Ct,
                                                           const float* __restrict__ Dv, const T* __restrict__ z,
                                                           const float* __restrict__ dbias, T* __restrict__ y, uint32_t rows,
                                                           uint32_t D, int N, int lpr_log2, int use_softplus, int vector_ok)
{
    const uint64_t gid = (uint64_t)blockIdx.x * kThreads + threadIdx.x;
    const uint32_t row = (uint32_t)(gid >> lpr_log2);
    const int LPR = 1 << lpr_log2;
    const int j = (int)(gid & (uint64_t)(LPR - 1));
    const bool active = row < rows;                         // whole rows are active or not: LPR divides the wave
    float acc = 0.f, xv = 0.f;
    uint32_t d = 0;
    if (active) {
        const uint32_t b = row / D;
        d = row - b * D;
        xv = Io<T>::ld(x + row);
        float dl = Io<T>::ld(delta + row) + (dbias ? dbias[d] : 0.f);
        if (use_softplus) dl = softplus(dl);
        const float dx = dl * xv;
        float* hrow = state + (size_t)row * N;
        const float* arow = A + (size_t)d * N;
        const T* brow = Bt + (size_t)b * N;
        const T* crow = Ct + (size_t)b * N;
        for (int n = 4 * j; n < N; n += 4 * LPR) {
            if (vector_ok && n + 4 <= N) {
                float4v h = *reinterpret_cast<const float4v*>(hrow + n);
                const float4v a = *reinterpret_cast<const float4v*>(arow + n);
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const float hn = fmaf(fast_exp2(dl * (a[i] * kLog2e)), h[i], dx * Io<T>::ld(brow + n + i));
                    h[i] = hn;
                    acc = fmaf(Io<T>::ld(crow + n + i), hn, acc);
                }
                *reinterpret_cast<float4v*>(hrow + n) = h;
            } else {
                for (int i = n; i < N && i < n + 4; ++i) {
                    const float hn = fmaf(fast_exp2(dl * (arow[i] * kLog2e)), hrow[i], dx * Io<T>::ld(brow + i));
                    hrow[i] = hn;
                    acc = fmaf(Io<T>::ld(crow + i), hn, acc);
                }
            }
        }
    }
    for (int m = LPR >> 1; m >= 1; m >>= 1) acc += __shfl_xor(acc, m);
    if (active && j == 0) {
        float yv = acc + (Dv ? Dv[d] * xv : 0.f);
        if (z) yv *= silu(Io<T>::ld(z + row));
        Io<T>::st(y + row, yv);
    }
}

template <typename T>
void launch(void* state, const void* x, const void* delta, const float* A, const void* Bt, const void* Ct, const float* Dv,
            const void* z, const float* dbias, void* y, int64_t B, int64_t D, int64_t N, int softplus_on, hipStream_t stream)
{
    int lpr_log2 = 0;
    while ((1 << lpr_log2) < (N + 3) / 4 && lpr_log2 < 6) ++lpr_log2;
    const bool vector_ok = (N % 4) == 0 && reinterpret_cast<uintptr_t>(state) % 16 == 0 && reinterpret_cast<uintptr_t>(A) % 16 == 0;
    const uint64_t lanes = (uint64_t)(B * D) << lpr_log2;
    const uint64_t blocks = (lanes + kThreads - 1) / kThreads;
    k_state_update<T><<<dim3((unsigned)blocks), dim3(kThreads), 0, stream>>>(
        static_cast<float*>(state), static_cast<const T*>(x), static_cast<const T*>(delta), A, static_cast<const T*>(Bt),
        static_cast<const T*>(Ct), Dv, static_cast<const T*>(z), dbias, static_cast<T*>(y), (uint32_t)(B * D), (uint32_t)D, (int)N,
        lpr_log2, softplus_on, vector_ok ? 1 : 0);
}

}  // namespace

extern "C" int selective_state_update(void* state, const void* x, const void* delta, const float* A, const void* Bt,
                                      const void* Ct, const float* Dv, const void* z, const float* delta_bias,
                                      int32_t delta_softplus, void* y, corey_dtype dt, int64_t B, int64_t D, int64_t N,
                                      void* hip_stream)
{
    using corey::fail;
    if (!state || !x || !delta || !A || !Bt || !Ct || !y)
        return fail(COREY_ENULL, "selective_state_update: state, x, delta, A, Bt, Ct and y are required");
    if (dt != COREY_F32 && dt != COREY_BF16 && dt != COREY_F16) return fail(COREY_EINVAL, "selective_state_update: unknown dtype %d", (int)dt);
    if (B < 1 || D < 1 || N < 1 || N > COREY_MAX_STATE)
        return fail(COREY_ESHAPE, "selective_state_update: B, D >= 1 and 1 <= N <= %d required", COREY_MAX_STATE);
    if ((double)B * (double)D >= 33554432.0)                // 2^25 rows: every index below stays far inside 32 / 64 bits
        return fail(COREY_ESHAPE, "selective_state_update: B*D must stay below 2^25");
    if (reinterpret_cast<uintptr_t>(state) % 4 != 0) return fail(COREY_EINVAL, "selective_state_update: state must be 4-byte aligned");
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const int sp = delta_softplus ? 1 : 0;
    if (dt == COREY_F32) launch<float>(state, x, delta, A, Bt, Ct, Dv, z, delta_bias, y, B, D, N, sp, stream);
    else if (dt == COREY_F16) launch<_Float16>(state, x, delta, A, Bt, Ct, Dv, z, delta_bias, y, B, D, N, sp, stream);
    else launch<uint16_t>(state, x, delta, A, Bt, Ct, Dv, z, delta_bias, y, B, D, N, sp, stream);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return corey::hip_fail(e, "selective_state_update launch");
    return COREY_OK;
}
