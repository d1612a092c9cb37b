// corey_entropy_hist: fixed-bin histogram entropy (Eq. 1) and r = H / log K on gfx950.
//
// Three sweeps, as the paper's estimation protocol states them (a min/max pass, a bin-count pass, an
// O(K) reduction):
//   k_entropy_init      clears counts and the range keys (a kernel, not a memset, so a caller may capture it)
//   k_entropy_range     lo/hi per histogram: 16-byte loads, wave + workgroup reduction, one pair of integer
//                       atomics per workgroup on order-preserving keys
//   k_entropy_count     bin index per value in binary32 (subtract, multiply, truncate: the ABI's definition),
//                       counts privatised in LDS (one copy per wave) and merged with integer atomics, so the
//                       result is exact and independent of scheduling
//   k_entropy_finalise  p_k, H = -sum p log(p + eps) and r in double, one workgroup per histogram
// All of it is bandwidth work: no matrix instructions.
#include <hip/hip_runtime.h>

#include <cmath>

#include "corey_internal.h"

namespace {

using corey::bf16_to_f32;

constexpr int kThreads = 256;
constexpr int kVecBytes = 16;

struct RangeSlot {        // one per histogram, in the caller's workspace
    uint32_t lo_key;      // order-preserving image of the minimum (0xffffffff: nothing seen)
    uint32_t hi_key;      // order-preserving image of the maximum (0: nothing seen)
    uint32_t saw_nan;
    uint32_t pad;
};

__device__ __forceinline__ uint32_t order_key(float f)
{
    const uint32_t u = __float_as_uint(f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__device__ __forceinline__ float key_value(uint32_t k)
{
    return __uint_as_float((k & 0x80000000u) ? (k & 0x7fffffffu) : ~k);
}

template <typename T> struct Elem;
template <> struct Elem<float> {
    static constexpr int kVec = 4;
    static __device__ __forceinline__ float widen(float v) { return v; }
};
template <> struct Elem<uint16_t> {
    static constexpr int kVec = 8;
    static __device__ __forceinline__ float widen(uint16_t v) { return bf16_to_f32(v); }
};

// Geometry of one histogram: `rows` rows of `len` valid values, `row_stride` apart, starting at `base`.
struct Geometry {
    int64_t base, rows, len, row_stride;
};

__device__ __forceinline__ Geometry geometry(int h, int64_t B, int64_t D, int64_t L, const int32_t* seqlens)
{
    Geometry g;
    if (seqlens) {
        int64_t len = seqlens[h];
        len = len < 0 ? 0 : (len > L ? L : len);
        g.base = (int64_t)h * D * L;
        g.rows = D;
        g.len = len;
    } else {
        g.base = 0;
        g.rows = B * D;
        g.len = L;
    }
    g.row_stride = L;
    return g;
}

// Visit every sampled value of histogram `h` once: f(value).  A workgroup takes (row, segment) units
// grid-stride; inside a unit every thread owns one 16-byte vector.  `vector_ok` says rows are 16-byte
// aligned (pointer and L), otherwise values are fetched one by one.
template <typename T, typename F>
__device__ __forceinline__ void for_each_value(const T* x, const Geometry& g, int64_t stride, bool vector_ok, F&& f)
{
    constexpr int V = Elem<T>::kVec;
    constexpr int64_t kSeg = (int64_t)kThreads * V;
    if (g.len == 0) return;
    const int64_t nseg = (g.len + kSeg - 1) / kSeg;
    const int64_t units = g.rows * nseg;
    for (int64_t unit = blockIdx.x; unit < units; unit += gridDim.x) {
        const int64_t r = unit / nseg;
        const int64_t t0 = (unit - r * nseg) * kSeg + (int64_t)threadIdx.x * V;
        if (t0 >= g.len) continue;
        const T* p = x + g.base + r * g.row_stride + t0;
        const int nvalid = (g.len - t0 < V) ? (int)(g.len - t0) : V;
        T v[V];
        if (vector_ok && nvalid == V) {
            typedef uint32_t vec4 __attribute__((ext_vector_type(4)));
            const vec4 raw = *reinterpret_cast<const vec4*>(p);
            __builtin_memcpy(v, &raw, kVecBytes);
        } else {
            for (int e = 0; e < V; ++e) v[e] = (e < nvalid) ? p[e] : T(0);
        }
        if (stride == 1) {
#pragma unroll
            for (int e = 0; e < V; ++e)
                if (e < nvalid) f(Elem<T>::widen(v[e]));
        } else {
            int64_t phase = (r * g.len + t0) % stride;   // index of v[0] in memory order, modulo stride
#pragma unroll
            for (int e = 0; e < V; ++e) {
                if (e < nvalid && phase == 0) f(Elem<T>::widen(v[e]));
                if (++phase == stride) phase = 0;
            }
        }
    }
}

__global__ void k_entropy_init(uint32_t* counts, int64_t ncounts, RangeSlot* slots, int nh)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < ncounts) counts[i] = 0u;
    if (i < nh) {
        slots[i].lo_key = 0xffffffffu;
        slots[i].hi_key = 0u;
        slots[i].saw_nan = 0u;
        slots[i].pad = 0u;
    }
}

template <typename T>
__global__ __launch_bounds__(kThreads) void k_entropy_range(const T* __restrict__ x, int64_t B, int64_t D, int64_t L,
                                                            const int32_t* __restrict__ seqlens, int64_t stride,
                                                            int vector_ok, RangeSlot* slots)
{
    const int h = blockIdx.y;
    const Geometry g = geometry(h, B, D, L, seqlens);
    float lo = INFINITY, hi = -INFINITY;
    bool nan = false;
    for_each_value(x, g, stride, vector_ok != 0, [&](float v) {
        nan |= (v != v);
        lo = fminf(lo, v);       // fminf/fmaxf drop a NaN operand; NaNs are flagged separately
        hi = fmaxf(hi, v);
    });
    uint32_t klo = (lo <= hi) ? order_key(lo) : 0xffffffffu;
    uint32_t khi = (lo <= hi) ? order_key(hi) : 0u;
    uint32_t knan = nan ? 1u : 0u;
    for (int off = 32; off > 0; off >>= 1) {
        klo = min(klo, (uint32_t)__shfl_xor((int)klo, off));
        khi = max(khi, (uint32_t)__shfl_xor((int)khi, off));
        knan |= (uint32_t)__shfl_xor((int)knan, off);
    }
    __shared__ uint32_t s_lo[kThreads / 64], s_hi[kThreads / 64], s_nan[kThreads / 64];
    const int wave = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) { s_lo[wave] = klo; s_hi[wave] = khi; s_nan[wave] = knan; }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < kThreads / 64; ++w) {
            klo = min(klo, s_lo[w]);
            khi = max(khi, s_hi[w]);
            knan |= s_nan[w];
        }
        if (klo != 0xffffffffu) atomicMin(&slots[h].lo_key, klo);
        if (khi != 0u) atomicMax(&slots[h].hi_key, khi);
        if (knan) atomicOr(&slots[h].saw_nan, 1u);
    }
}

__device__ __forceinline__ bool usable_range(const RangeSlot& s, float* lo, float* hi)
{
    if (s.saw_nan || s.lo_key == 0xffffffffu || s.hi_key == 0u) return false;
    *lo = key_value(s.lo_key);
    *hi = key_value(s.hi_key);
    return isfinite(*lo) && isfinite(*hi);
}

constexpr int kMaxLdsBins = 4096;

template <typename T>
__global__ __launch_bounds__(kThreads) void k_entropy_count(const T* __restrict__ x, int64_t B, int64_t D, int64_t L,
                                                            const int32_t* __restrict__ seqlens, int64_t stride,
                                                            int vector_ok, int K, const RangeSlot* __restrict__ slots,
                                                            uint32_t* counts)
{
    __shared__ uint32_t s_bins[kMaxLdsBins];
    const int h = blockIdx.y;
    float lo, hi;
    if (!usable_range(slots[h], &lo, &hi)) return;            // counts stay zero, H and r become NaN
    const Geometry g = geometry(h, B, D, L, seqlens);
    // one private copy per wave while they fit, to spread same-bin collisions
    const int copies = (K * (kThreads / 64) <= kMaxLdsBins) ? kThreads / 64 : 1;
    for (int i = threadIdx.x; i < K * copies; i += kThreads) s_bins[i] = 0u;
    __syncthreads();
    uint32_t* mine = s_bins + ((copies > 1) ? (threadIdx.x >> 6) * K : 0);

    if (hi == lo) {
        uint32_t n = 0;
        for_each_value(x, g, stride, vector_ok != 0, [&](float) { ++n; });
        if (n) atomicAdd(&mine[0], n);
    } else {
        const float scale = (float)((double)K / ((double)hi - (double)lo));
        const int top = K - 1;
        for_each_value(x, g, stride, vector_ok != 0, [&](float v) {
            const float q = __fmul_rn(__fsub_rn(v, lo), scale);   // two separate binary32 roundings
            int k = (int)q;                                        // truncation; q >= 0
            k = k > top ? top : (k < 0 ? 0 : k);
            atomicAdd(&mine[k], 1u);
        });
    }
    __syncthreads();
    uint32_t* out = counts + (int64_t)h * K;
    for (int k = threadIdx.x; k < K; k += kThreads) {
        uint32_t c = 0;
        for (int w = 0; w < copies; ++w) c += s_bins[w * K + k];
        if (c) atomicAdd(&out[k], c);
    }
}

__global__ __launch_bounds__(kThreads) void k_entropy_finalise(const uint32_t* __restrict__ counts, int K, double eps,
                                                               const RangeSlot* __restrict__ slots, double* H_out,
                                                               double* r_out, float* range_out)
{
    const int h = blockIdx.x;
    const uint32_t* c = counts + (int64_t)h * K;
    float lo = 0.f, hi = 0.f;
    const bool ok = usable_range(slots[h], &lo, &hi);
    __shared__ double s_red[kThreads];
    __shared__ unsigned long long s_n[kThreads];

    unsigned long long n_part = 0;
    for (int k = threadIdx.x; k < K; k += kThreads) n_part += c[k];
    s_n[threadIdx.x] = n_part;
    __syncthreads();
    for (int off = kThreads / 2; off > 0; off >>= 1) {
        if ((int)threadIdx.x < off) s_n[threadIdx.x] += s_n[threadIdx.x + off];
        __syncthreads();
    }
    const double n = (double)s_n[0];

    double part = 0.0;
    if (ok && n > 0.0)
        for (int k = threadIdx.x; k < K; k += kThreads) {
            const double p = (double)c[k] / n;
            part += p * log(p + eps);
        }
    s_red[threadIdx.x] = part;
    __syncthreads();
    for (int off = kThreads / 2; off > 0; off >>= 1) {
        if ((int)threadIdx.x < off) s_red[threadIdx.x] += s_red[threadIdx.x + off];
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        double H = NAN, r = NAN;
        if (ok && n > 0.0) {
            H = -s_red[0];
            r = H / log((double)K);
            r = r < 0.0 ? 0.0 : (r > 1.0 ? 1.0 : r);
        }
        H_out[h] = H;
        r_out[h] = r;
        if (range_out) {
            range_out[2 * h] = (slots[h].lo_key == 0xffffffffu) ? INFINITY : key_value(slots[h].lo_key);
            range_out[2 * h + 1] = (slots[h].hi_key == 0u) ? -INFINITY : key_value(slots[h].hi_key);
        }
    }
}

size_t workspace_bytes(int64_t nh)
{
    const size_t raw = (size_t)nh * sizeof(RangeSlot);
    return (raw + 255) / 256 * 256;
}

template <typename T>
int launch(const void* x, int64_t B, int64_t D, int64_t L, const int32_t* seqlens, int32_t K, double eps, int64_t stride,
           uint32_t* counts, double* H_out, double* r_out, float* range_out, RangeSlot* slots, hipStream_t stream)
{
    const int nh = seqlens ? (int)B : 1;
    const int64_t ncounts = (int64_t)nh * K;
    const int64_t init_items = ncounts > nh ? ncounts : nh;
    k_entropy_init<<<dim3((unsigned)((init_items + kThreads - 1) / kThreads)), dim3(kThreads), 0, stream>>>(
        counts, ncounts, slots, nh);

    constexpr int V = Elem<T>::kVec;
    const bool vector_ok = (reinterpret_cast<uintptr_t>(x) % kVecBytes == 0) && (L % V == 0);
    const int64_t rows = seqlens ? D : B * D;
    const int64_t units = rows * ((L + (int64_t)kThreads * V - 1) / ((int64_t)kThreads * V));
    int64_t blocks = units < 1 ? 1 : units;
    const int64_t cap = 256 * 8;                       // a few workgroups per compute unit
    if (blocks > cap) blocks = cap;
    const dim3 grid((unsigned)blocks, (unsigned)nh);
    k_entropy_range<T><<<grid, dim3(kThreads), 0, stream>>>(static_cast<const T*>(x), B, D, L, seqlens, stride,
                                                           vector_ok ? 1 : 0, slots);
    k_entropy_count<T><<<grid, dim3(kThreads), 0, stream>>>(static_cast<const T*>(x), B, D, L, seqlens, stride,
                                                           vector_ok ? 1 : 0, K, slots, counts);
    k_entropy_finalise<<<dim3((unsigned)nh), dim3(kThreads), 0, stream>>>(counts, K, eps, slots, H_out, r_out, range_out);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return corey::hip_fail(e, "corey_entropy_hist launch");
    return COREY_OK;
}

}  // namespace

extern "C" size_t corey_entropy_hist_workspace(int64_t B, int32_t K)
{
    if (B < 1 || K < 2 || K > COREY_MAX_BINS) return 0;
    return workspace_bytes(B);
}

extern "C" int corey_entropy_hist(const void* x, corey_dtype dt, int64_t B, int64_t D, int64_t L, const int32_t* seqlens,
                                  int32_t K, double eps, int64_t stride, uint32_t* counts_out, double* H_out, double* r_out,
                                  float* range_out, void* workspace, size_t workspace_bytes_given, void* hip_stream)
{
    using corey::fail;
    if (!x || !counts_out || !H_out || !r_out) return fail(COREY_ENULL, "corey_entropy_hist: x, counts_out, H_out and r_out are required");
    if (dt != COREY_F32 && dt != COREY_BF16) return fail(COREY_EINVAL, "corey_entropy_hist: unknown dtype %d", (int)dt);
    if (B < 1 || D < 1 || L < 1) return fail(COREY_ESHAPE, "corey_entropy_hist: B, D, L must be >= 1");
    if (B > 65535) return fail(COREY_ESHAPE, "corey_entropy_hist: B = %lld exceeds 65535", (long long)B);
    if ((double)B * (double)D * (double)L >= 9.0e18) return fail(COREY_ESHAPE, "corey_entropy_hist: B*D*L overflows");
    if ((double)B * (double)D * (double)L >= 4294967296.0 && stride == 1)
        return fail(COREY_ESHAPE, "corey_entropy_hist: more than 2^32-1 samples would overflow the 32-bit counts");
    if (K < 2 || K > COREY_MAX_BINS) return fail(COREY_EINVAL, "corey_entropy_hist: K = %d outside [2, %d]", K, COREY_MAX_BINS);
    if (!(eps >= 0.0)) return fail(COREY_EINVAL, "corey_entropy_hist: eps must be >= 0");
    if (stride < 1) return fail(COREY_EINVAL, "corey_entropy_hist: stride must be >= 1");
    const size_t need = workspace_bytes(B);
    if (!workspace || workspace_bytes_given < need)
        return fail(COREY_EWORKSPACE, "corey_entropy_hist: workspace of %zu bytes required", need);
    if (reinterpret_cast<uintptr_t>(workspace) % 16 != 0) return fail(COREY_EWORKSPACE, "corey_entropy_hist: workspace must be 16-byte aligned");
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    RangeSlot* slots = static_cast<RangeSlot*>(workspace);
    if (dt == COREY_F32)
        return launch<float>(x, B, D, L, seqlens, K, eps, stride, counts_out, H_out, r_out, range_out, slots, stream);
    return launch<uint16_t>(x, B, D, L, seqlens, K, eps, stride, counts_out, H_out, r_out, range_out, slots, stream);
}
