// corey_entropy_hist: fixed-bin histogram entropy (Eq. 1) and r = H / log K on gfx950.
//
// Three sweeps, as the paper's estimation protocol states them (a min/max pass, a bin-count pass, an
// O(K) reduction):
//   k_entropy_init      clears the partial counts and the range keys (a kernel, not a memset, so a caller may
//                       capture it); only the general path needs it
//   k_entropy_range     lo/hi per histogram: 16-byte loads, wave + workgroup reduction, one pair of integer
//                       atomics per workgroup on order-preserving keys
//   k_entropy_count     bin index per value in binary32 (subtract, multiply, truncate: the ABI's definition),
//                       counts privatised in LDS (several copies per workgroup) and merged with integer atomics, so the
//                       result is exact and independent of scheduling
//                       (merged into kParts partial histograms in the workspace, so that the merging atomics
//                       of many workgroups do not all queue on the same few cache lines)
//   k_entropy_finalise  sums the partial histograms into counts, then p_k, H = -sum p log(p + eps) and r in
//                       double, one workgroup per histogram
// The common call (one histogram over the whole tensor, aligned, every value or every stride-th block of a
// power-of-two number of 16-byte words) takes the *_flat kernels: the range sweep leaves one partial range per
// workgroup (no atomics, so nothing has to be cleared first; it also clears the partial counts), the count sweep
// starts by reducing those partials, and only the sampled 16-byte words are fetched at all.  When the producer of the
// tensor hands over its partial ranges (and, beside them, partial histograms it cleared) the statistic is ONE launch,
// the count sweep, plus the reduction; the reduction leaves those partial histograms cleared for the next call.  The
// reduction itself (corey_finalise.h) can also be left to the first kernel of a routed scan (corey_route_device_deferred).
// All of it is bandwidth work: no matrix instructions.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstring>
#include <mutex>

#include "corey_finalise.h"
#include "corey_internal.h"
#include "corey_range.h"

namespace {

using corey::bf16_to_f32;

using corey_range::kThreads;
using corey_range::key_value;
using corey_range::order_key;
using corey_range::Handoff;
using corey_range::RangePart;
using corey_range::RangeSlot;
using corey_range::RangeFold;
using corey_range::usable_range;
using corey_range::word4;
using corey_range::reduce_range_keys;
constexpr int kVecBytes = 16;
using corey_range::kParts;     // partial histograms per histogram in the workspace
constexpr int kMaxBlocks = COREY_RANGE_PARTS;  // most workgroups per sweep (four per compute unit) and partial ranges kept
constexpr int kFlatBlocks = 512;               // workgroups of a flat sweep: two per compute unit measured 4 % (exact) to
                                               // 11 % (sampled) faster than four (fewer LDS clears, merges and range folds)

template <typename T> struct Elem;
template <> struct Elem<float> {
    static constexpr int kVec = 4;
    static __device__ __forceinline__ float widen(float v) { return v; }
};
template <> struct Elem<uint16_t> {                       // bfloat16 bit patterns
    static constexpr int kVec = 8;
    static __device__ __forceinline__ float widen(uint16_t v) { return bf16_to_f32(v); }
    static __device__ __forceinline__ void widen2(uint32_t w, float& a, float& b)
    {
        a = __uint_as_float(w << 16);
        b = __uint_as_float(w & 0xffff0000u);
    }
};
template <> struct Elem<_Float16> {                       // IEEE binary16
    static constexpr int kVec = 8;
    static __device__ __forceinline__ float widen(_Float16 v) { return (float)v; }
    static __device__ __forceinline__ void widen2(uint32_t w, float& a, float& b)
    {
        typedef _Float16 h2 __attribute__((ext_vector_type(2)));
        h2 h;
        __builtin_memcpy(&h, &w, 4);
        a = (float)h.x;
        b = (float)h.y;
    }
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

constexpr int kUnroll = 4;   // 16-byte loads a thread keeps in flight

// Which of the values numbered idx, idx + 1, ... (memory order within one histogram) are sampled: every stride-th
// block of `block` consecutive values.
struct SamplePhase {
    int64_t pos, bph, block, stride;
    __device__ __forceinline__ SamplePhase(int64_t idx, int64_t block_, int64_t stride_) : block(block_), stride(stride_)
    {
        if (((block & (block - 1)) | (stride & (stride - 1))) == 0) {   // powers of two (uniform): no division
            const int lb = 63 - __clzll((long long)block);
            pos = idx & (block - 1);
            bph = (idx >> lb) & (stride - 1);
        } else {
            const int64_t blk = idx / block;
            pos = idx - blk * block;
            bph = blk % stride;
        }
    }
    __device__ __forceinline__ bool take_and_advance()
    {
        const bool take = bph == 0;
        if (++pos == block) {
            pos = 0;
            if (++bph == stride) bph = 0;
        }
        return take;
    }
};

// Visit every sampled value of histogram `h` once: f(value).  A row is cut into slabs of kThreads 16-byte vectors
// (one vector per thread); a workgroup takes kUnroll consecutive slabs at a time, grid-stride, whichever rows they
// fall in (short rows: several rows per turn), and loads all of them before any is consumed so that enough bytes
// are in flight to cover HBM latency.  The (row, slab) cursor is stepped, never divided, inside the loop.
// `vector_ok` says rows are 16-byte aligned (pointer and L); otherwise, and in the ragged last slab of a row,
// values are fetched one by one where no whole vector fits.
// Apply a per-value function to the values of one 16-byte vector.
template <typename T, typename F>
__device__ __forceinline__ void each_of_vector(const uint32_t __attribute__((ext_vector_type(4)))& raw, F&& f)
{
    T v[Elem<T>::kVec];
    __builtin_memcpy(v, &raw, kVecBytes);
#pragma unroll
    for (int e = 0; e < Elem<T>::kVec; ++e) f(Elem<T>::widen(v[e]));
}

// The grid is sized on the host from L; the valid lengths are only known here.  active_groups says how many of the
// launched workgroups a histogram keeps busy (about kTurns turns each): the others leave at once instead of paying a
// workgroup's fixed costs (clearing and merging the LDS counters) for a sliver of data.
constexpr int kTurns = 2;
template <typename T>
__device__ __forceinline__ int64_t active_groups(const Geometry& g)
{
    constexpr int64_t kSlab = (int64_t)kThreads * Elem<T>::kVec;
    const int64_t nslab = g.rows * ((g.len + kSlab - 1) / kSlab);
    const int64_t n = (nslab + kUnroll * kTurns - 1) / (kUnroll * kTurns);
    return n < 1 ? 1 : (n > (int64_t)gridDim.x ? (int64_t)gridDim.x : n);
}

// `fv` takes a whole 16-byte vector of values that are all used (stride 1); `f` one value.
template <typename T, typename F, typename FV>
__device__ __forceinline__ void for_each_value(const T* x, const Geometry& g, int64_t stride, int64_t block, bool vector_ok,
                                               int64_t nwg, F&& f, FV&& fv)
{
    constexpr int V = Elem<T>::kVec;
    constexpr int64_t kSlab = (int64_t)kThreads * V;
    typedef uint32_t vec4 __attribute__((ext_vector_type(4)));
    if (g.len == 0) return;
    const bool all = stride == 1;
    const int64_t spr = (g.len + kSlab - 1) / kSlab;           // slabs per row
    const int64_t nslab = g.rows * spr;
    const int64_t step = nwg * kUnroll;                         // nwg workgroups (blockIdx.x < nwg) share the histogram
    const int64_t step_r = step / spr, step_o = step - step_r * spr;
    int64_t s = (int64_t)blockIdx.x * kUnroll;
    int64_t r = s / spr, o = s - r * spr;                       // row and slab within the row of slab s
    const int64_t tid_off = (int64_t)threadIdx.x * V;
    // sampling in power-of-two blocks of whole vectors, every power-of-two-th block, rows of whole vectors
    const bool vec_blocks = !all && ((block & (block - 1)) | (stride & (stride - 1))) == 0 && block % V == 0 && g.len % V == 0;
    const int block_log2 = 63 - __clzll((long long)block);
    for (; s < nslab; s += step) {                              // everything about the cursor is uniform
        int64_t row_k[kUnroll], t0_k[kUnroll];
        int nk = 0;
        bool fast = vector_ok;
        {
            int64_t rk = r, ok = o;
#pragma unroll
            for (int k = 0; k < kUnroll; ++k) {
                row_k[k] = rk;
                t0_k[k] = ok * kSlab;
                if (s + k < nslab) {
                    ++nk;
                    fast = fast && (t0_k[k] + kSlab <= g.len);
                }
                if (++ok == spr) {
                    ok = 0;
                    ++rk;
                }
            }
        }
        if (fast && nk == kUnroll && vec_blocks) {              // whole slabs, sampled in blocks of whole vectors:
            vec4 raw[kUnroll];                                  // a vector is used or skipped (not even fetched) as one
            bool take[kUnroll];
#pragma unroll
            for (int k = 0; k < kUnroll; ++k) {
                const int64_t idx = row_k[k] * g.len + t0_k[k] + tid_off;
                take[k] = ((idx >> block_log2) & (stride - 1)) == 0;
                if (take[k]) raw[k] = *reinterpret_cast<const vec4*>(x + g.base + row_k[k] * g.row_stride + t0_k[k] + tid_off);
            }
#pragma unroll
            for (int k = 0; k < kUnroll; ++k)
                if (take[k]) fv(raw[k]);
        } else if (fast && nk == kUnroll) {                     // kUnroll whole slabs
            vec4 raw[kUnroll];
#pragma unroll
            for (int k = 0; k < kUnroll; ++k)
                raw[k] = *reinterpret_cast<const vec4*>(x + g.base + row_k[k] * g.row_stride + t0_k[k] + tid_off);
#pragma unroll
            for (int k = 0; k < kUnroll; ++k) {
                if (all) {
                    fv(raw[k]);
                    continue;
                }
                T v[V];
                __builtin_memcpy(v, &raw[k], kVecBytes);
                {
                    SamplePhase ph(row_k[k] * g.len + t0_k[k] + tid_off, block, stride);   // index of v[0] in memory order
#pragma unroll
                    for (int e = 0; e < V; ++e)
                        if (ph.take_and_advance()) f(Elem<T>::widen(v[e]));
                }
            }
        } else if (vector_ok) {                                 // a ragged slab among them, or the last turn: every thread
            vec4 raw[kUnroll];                                  // still fetches its whole vectors before it uses any
            int nvalid[kUnroll];
#pragma unroll
            for (int k = 0; k < kUnroll; ++k) {
                const int64_t left = g.len - (t0_k[k] + tid_off);
                nvalid[k] = (k < nk && left > 0) ? (left < V ? (int)left : V) : 0;
                if (nvalid[k] == V)
                    raw[k] = *reinterpret_cast<const vec4*>(x + g.base + row_k[k] * g.row_stride + t0_k[k] + tid_off);
            }
#pragma unroll
            for (int k = 0; k < kUnroll; ++k) {
                if (nvalid[k] == 0) continue;
                const int64_t t0 = t0_k[k] + tid_off;
                const T* row = x + g.base + row_k[k] * g.row_stride;
                if (nvalid[k] == V) {
                    if (all) {
                        fv(raw[k]);
                    } else {
                        T v[V];
                        __builtin_memcpy(v, &raw[k], kVecBytes);
                        SamplePhase ph(row_k[k] * g.len + t0, block, stride);
#pragma unroll
                        for (int e = 0; e < V; ++e)
                            if (ph.take_and_advance()) f(Elem<T>::widen(v[e]));
                    }
                } else if (all) {                              // the thread that straddles the end of the row
                    for (int e = 0; e < nvalid[k]; ++e) f(Elem<T>::widen(row[t0 + e]));
                } else {
                    SamplePhase ph(row_k[k] * g.len + t0, block, stride);
                    for (int e = 0; e < nvalid[k]; ++e)
                        if (ph.take_and_advance()) f(Elem<T>::widen(row[t0 + e]));
                }
            }
        } else {                                                // unaligned rows: value by value
            for (int k = 0; k < nk; ++k) {
                const T* row = x + g.base + row_k[k] * g.row_stride;
                const int64_t t0 = t0_k[k] + tid_off;
                if (t0 >= g.len) continue;
                const int nv = (g.len - t0 < V) ? (int)(g.len - t0) : V;
                if (all) {
                    for (int e = 0; e < nv; ++e) f(Elem<T>::widen(row[t0 + e]));
                } else {
                    SamplePhase ph(row_k[k] * g.len + t0, block, stride);
                    for (int e = 0; e < nv; ++e)
                        if (ph.take_and_advance()) f(Elem<T>::widen(row[t0 + e]));
                }
            }
        }
        r += step_r;
        o += step_o;
        if (o >= spr) {
            o -= spr;
            ++r;
        }
    }
}

// Range slots of the general sweeps: every histogram has kSubSlots of them and a workgroup publishes into slot
// blockIdx.x % kSubSlots (a thousand workgroups that finish together would otherwise queue their atomics on one
// address: that queue, not the data, set the time of the range sweep); the count sweep folds them.
constexpr int kSubSlots = 32;

__global__ __launch_bounds__(kThreads) void k_entropy_init(uint32_t* parts, int64_t nparts, RangeSlot* slots, int nh, RangeSlot* subs)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const RangeSlot empty = {0xffffffffu, 0u, 0u, 0u};
    if (i < nparts) parts[i] = 0u;
    if (i < nh) slots[i] = empty;
    if (i < (int64_t)nh * kSubSlots) subs[i] = empty;
}

// ... and the integer atomics that publish it.  The slot is read first and an atomic is issued only if it
// would change it: extremes only move one way, so a stale read can cost a redundant atomic but never lose an
// update, and almost all workgroups skip the contended atomics.
__device__ __forceinline__ void publish_range(float lo, float hi, bool nan, RangeSlot* slot)
{
    uint32_t klo = (lo <= hi) ? order_key(lo) : 0xffffffffu;
    uint32_t khi = (lo <= hi) ? order_key(hi) : 0u;
    uint32_t knan = nan ? 1u : 0u;
    reduce_range_keys(klo, khi, knan);
    if (threadIdx.x == 0) {
        if (klo < __atomic_load_n(&slot->lo_key, __ATOMIC_RELAXED)) atomicMin(&slot->lo_key, klo);
        if (khi > __atomic_load_n(&slot->hi_key, __ATOMIC_RELAXED)) atomicMax(&slot->hi_key, khi);
        if (knan) atomicOr(&slot->saw_nan, 1u);
    }
}

// ---------------------------------------------------------------------------------------------------------
// Fast path for the common call: one histogram over the whole tensor, every value used, 16-byte aligned.
// The tensor is then a flat array of 16-byte words; a workgroup walks it grid-stride with kUnroll loads in
// flight per lane and nothing but straight-line code in between.

template <typename T>
__global__ __launch_bounds__(kThreads) void k_entropy_range(const T* __restrict__ x, int64_t B, int64_t D, int64_t L,
                                                            const int32_t* __restrict__ seqlens, int64_t stride, int64_t block,
                                                            int vector_ok, RangeSlot* subs)
{
    const int h = blockIdx.y;
    const Geometry g = geometry(h, B, D, L, seqlens);
    const int64_t nwg = active_groups<T>(g);
    if ((int64_t)blockIdx.x >= nwg) return;                     // uniform
    float lo = INFINITY, hi = -INFINITY;
    uint32_t mag = 0u;                                          // whole vectors: NaN is read off the largest magnitude pattern
    bool nan = false;
    for_each_value(
        x, g, stride, block, vector_ok != 0, nwg,
        [&](float v) {
            nan |= (v != v);
            lo = fminf(lo, v);       // fminf/fmaxf drop a NaN operand; NaNs are flagged separately
            hi = fmaxf(hi, v);
        },
        [&](const word4& q) { RangeFold<T>::fold(q, lo, hi, mag); });
    nan |= RangeFold<T>::saw_nan(mag);
    publish_range(lo, hi, nan, &subs[h * kSubSlots + blockIdx.x % kSubSlots]);
}

// The 16-byte words of a flat sweep.  Unsampled: word i is word i.  Sampled: the tensor is cut into blocks of
// 2^bw_log2 words and every stride-th block is used; the sampled words are numbered consecutively.
template <bool SAMPLED> struct WordMap {
    int bw_log2;
    int64_t stride;
    __device__ __forceinline__ int64_t operator()(int64_t i) const
    {
        if constexpr (!SAMPLED) return i;
        const int64_t sb = i >> bw_log2;
        return ((sb * stride) << bw_log2) + (i - (sb << bw_log2));
    }
};

template <typename T, bool SAMPLED>
__global__ __launch_bounds__(kThreads) void k_entropy_range_flat(const word4* __restrict__ x, int64_t nwords, WordMap<SAMPLED> map,
                                                                 RangePart* __restrict__ rparts, uint32_t* __restrict__ parts,
                                                                 int nparts)
{
    // the partial counts the next sweep adds into
    for (int i = blockIdx.x * kThreads + threadIdx.x; i < nparts; i += gridDim.x * kThreads) parts[i] = 0u;
    float lo = INFINITY, hi = -INFINITY;
    uint32_t mag = 0u;
    const int64_t step = (int64_t)gridDim.x * kThreads * kUnroll;
    int64_t base = (int64_t)blockIdx.x * kThreads * kUnroll;
    for (; base + kThreads * kUnroll <= nwords; base += step) {
        word4 q[kUnroll];
#pragma unroll
        for (int k = 0; k < kUnroll; ++k) q[k] = x[map(base + k * kThreads + threadIdx.x)];
#pragma unroll
        for (int k = 0; k < kUnroll; ++k) RangeFold<T>::fold(q[k], lo, hi, mag);
    }
    for (int64_t i = base + threadIdx.x; i < nwords; i += kThreads) {     // ragged end: at most one workgroup gets here
        const word4 q = x[map(i)];
        RangeFold<T>::fold(q, lo, hi, mag);
    }
    uint32_t klo = (lo <= hi) ? order_key(lo) : 0xffffffffu;
    uint32_t khi = (lo <= hi) ? order_key(hi) : 0u;
    uint32_t knan = RangeFold<T>::saw_nan(mag) ? 1u : 0u;
    reduce_range_keys(klo, khi, knan);
    if (threadIdx.x == 0) {
        RangePart rp;
        rp.lo_key = klo; rp.hi_key = khi; rp.saw_nan = knan; rp.pad = 0u;
        rparts[blockIdx.x] = rp;
    }
}

constexpr int kMaxLdsBins = 8192;   // uint32 counters in LDS (32 KiB)

// Private copies of the K counters a workgroup keeps in LDS: as many as fit, up to one per pair of lanes of a wave,
// so that lanes of a wave that hit the same bin mostly land on different addresses (same-address LDS atomics
// serialise).  Copies are K + 1 words apart: with a stride that is a multiple of the bank count (K = 256) the same
// bin of every copy would sit in one bank and the atomics would serialise all the same.
__device__ __forceinline__ int lds_copies(int K)
{
    const int c = kMaxLdsBins / (K + 1);
    return c > 32 ? 32 : (c < 1 ? 1 : c);
}

template <typename T>
__global__ __launch_bounds__(kThreads) void k_entropy_count(const T* __restrict__ x, int64_t B, int64_t D, int64_t L,
                                                            const int32_t* __restrict__ seqlens, int64_t stride, int64_t block,
                                                            int vector_ok, int K, const RangeSlot* __restrict__ subs,
                                                            RangeSlot* __restrict__ slots, uint32_t* parts)
{
    __shared__ uint32_t s_bins[kMaxLdsBins];
    __shared__ RangeSlot s_slot;
    const int h = blockIdx.y;
    const Geometry g = geometry(h, B, D, L, seqlens);
    const int64_t nwg = active_groups<T>(g);
    if ((int64_t)blockIdx.x >= nwg) return;                     // uniform; workgroup 0 always stays
    {   // the range: every workgroup folds the histogram's sub-slots (half a KB from L2)
        uint32_t klo = 0xffffffffu, khi = 0u, knan = 0u;
        if (threadIdx.x < kSubSlots) {
            const RangeSlot rs = subs[h * kSubSlots + threadIdx.x];
            klo = rs.lo_key;
            khi = rs.hi_key;
            knan = rs.saw_nan;
        }
        reduce_range_keys(klo, khi, knan);
        if (threadIdx.x == 0) {
            s_slot.lo_key = klo; s_slot.hi_key = khi; s_slot.saw_nan = knan; s_slot.pad = 0u;
            if (blockIdx.x == 0) slots[h] = s_slot;           // for the reduction kernel
        }
        __syncthreads();
    }
    float lo, hi;
    if (!usable_range(s_slot, &lo, &hi)) return;              // counts stay zero, H and r become NaN
    // as many private copies as fit (up to one per pair of lanes of a wave): lanes of a wave that hit the same
    // bin then mostly land on different addresses, which is what serialises LDS atomics
    const int cs = K + 1;                                     // copy stride: odd offset between copies, see lds_copies
    const int copies = lds_copies(K);
    for (int i = threadIdx.x; i < cs * copies; i += kThreads) s_bins[i] = 0u;
    __syncthreads();
    uint32_t* mine = s_bins + (threadIdx.x % copies) * cs;

    if (hi == lo) {
        uint32_t n = 0;
        for_each_value(x, g, stride, block, vector_ok != 0, nwg, [&](float) { ++n; },
                       [&](const word4&) { n += Elem<T>::kVec; });
        if (n) atomicAdd(&mine[0], n);
    } else {
        const float scale = (float)((double)K / ((double)hi - (double)lo));
        const int top = K - 1;
        auto bin = [&](float v) {
            const float q = __fmul_rn(__fsub_rn(v, lo), scale);   // two separate binary32 roundings
            int k = (int)q;                                        // truncation; q >= 0
            k = k > top ? top : (k < 0 ? 0 : k);
            atomicAdd(&mine[k], 1u);
        };
        for_each_value(x, g, stride, block, vector_ok != 0, nwg, bin, [&](const word4& q) { each_of_vector<T>(q, bin); });
    }
    __syncthreads();
    uint32_t* out = parts + ((int64_t)h * kParts + blockIdx.x % kParts) * K;
    for (int k = threadIdx.x; k < K; k += kThreads) {
        uint32_t c = 0;
        for (int w = 0; w < copies; ++w) c += s_bins[w * cs + k];
        if (c) atomicAdd(&out[k], c);
    }
}

template <typename T, bool SAMPLED>
__global__ __launch_bounds__(kThreads) void k_entropy_count_flat(const word4* __restrict__ x, int64_t nwords, WordMap<SAMPLED> map, int K,
                                                                 const RangePart* __restrict__ rparts, int nrparts,
                                                                 RangeSlot* __restrict__ slots, uint32_t* parts)
{
    __shared__ uint32_t s_bins[kMaxLdsBins];
    __shared__ RangeSlot s_slot;
    // the first words are requested before anything else, so that their trip from HBM overlaps the range fold and the
    // clearing of the counters below (a sampled sweep is only two or three such turns long: their latency is its time)
    const int64_t step = (int64_t)gridDim.x * kThreads * kUnroll;
    int64_t base = (int64_t)blockIdx.x * kThreads * kUnroll;
    word4 q[kUnroll], qn[kUnroll];
    bool have = base + kThreads * kUnroll <= nwords;
    if (have) {
#pragma unroll
        for (int k = 0; k < kUnroll; ++k) q[k] = x[map(base + k * kThreads + threadIdx.x)];
    }
    {   // the range: every workgroup reduces the partial ranges of the sweep before, or of the tensor's producer (a few KB
        // from L2)
        uint32_t klo = 0xffffffffu, khi = 0u, knan = 0u;
        for (int i = threadIdx.x; i < nrparts; i += kThreads) {
            const RangePart rp = rparts[i];
            klo = min(klo, rp.lo_key);
            khi = max(khi, rp.hi_key);
            knan |= rp.saw_nan;
        }
        reduce_range_keys(klo, khi, knan);
        if (threadIdx.x == 0) {
            s_slot.lo_key = klo; s_slot.hi_key = khi; s_slot.saw_nan = knan; s_slot.pad = 0u;
            if (blockIdx.x == 0) slots[0] = s_slot;           // for the reduction
        }
        __syncthreads();
    }
    float lo, hi;
    if (!usable_range(s_slot, &lo, &hi)) return;              // counts stay zero, H and r become NaN
    const int cs = K + 1;                                     // copy stride: odd offset between copies, see lds_copies
    const int copies = lds_copies(K);
    for (int i = threadIdx.x; i < cs * copies; i += kThreads) s_bins[i] = 0u;
    __syncthreads();
    uint32_t* mine = s_bins + (threadIdx.x % copies) * cs;
    const float scale = hi == lo ? 0.f : (float)((double)K / ((double)hi - (double)lo));     // degenerate range: everything in bin 0
    const uint32_t top = (uint32_t)K - 1u;
    auto bin = [&](float v) {
        const float q = __fmul_rn(__fsub_rn(v, lo), scale);    // two separate binary32 roundings
        // truncation; q >= 0 (a degenerate range has scale 0: bin 0).  The conversion to unsigned saturates, so a value
        // outside a stale range still lands inside the counters.
        const uint32_t k = min(__float2uint_rz(q), top);
        atomicAdd(&mine[k], 1u);
    };
    auto fold = [&](const word4& q) {
        const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            if constexpr (sizeof(T) == 2) {
                float a, b;
                Elem<T>::widen2(w[k], a, b);
                bin(a);
                bin(b);
            } else {
                bin(__uint_as_float(w[k]));
            }
        }
    };
    while (have) {                                            // the next turn's words are requested before this turn's are counted;
        base += step;                                         // two turns per iteration, so the two sets of registers swap roles
        have = base + kThreads * kUnroll <= nwords;           // without being copied
        if (have) {
#pragma unroll
            for (int k = 0; k < kUnroll; ++k) qn[k] = x[map(base + k * kThreads + threadIdx.x)];
        }
#pragma unroll
        for (int k = 0; k < kUnroll; ++k) fold(q[k]);
        if (!have) break;
        base += step;
        have = base + kThreads * kUnroll <= nwords;
        if (have) {
#pragma unroll
            for (int k = 0; k < kUnroll; ++k) q[k] = x[map(base + k * kThreads + threadIdx.x)];
        }
#pragma unroll
        for (int k = 0; k < kUnroll; ++k) fold(qn[k]);
    }
    for (int64_t i = base + threadIdx.x; i < nwords; i += kThreads) fold(x[map(i)]);     // ragged end: at most one workgroup
    __syncthreads();
    for (int k = threadIdx.x; k < K; k += kThreads) {
        uint32_t c = 0;
        for (int w = 0; w < copies; ++w) c += s_bins[w * cs + k];
        if (c) atomicAdd(&parts[(size_t)(blockIdx.x % kParts) * K + k], c);
    }
}

// The O(K) reduction and the chunk rule (corey_finalise.h), one workgroup per histogram.
__global__ __launch_bounds__(kThreads) void k_entropy_finalise(const corey_finalise::Args a)
{
    corey_finalise::finalise(a, (int)blockIdx.x, true);
}

// One thread per histogram.
__global__ void k_select_chunk(const double* __restrict__ r, const int32_t* __restrict__ seqlens, int64_t L_all, int nh,
                               corey_policy p, int32_t* __restrict__ chunks)
{
    const int h = blockIdx.x * blockDim.x + threadIdx.x;
    if (h >= nh) return;
    chunks[h] = corey_finalise::chunk_rule(r[h], seqlens ? (int64_t)seqlens[h] : L_all, p);
}

size_t slots_bytes(int64_t nh)
{
    const size_t raw = (size_t)nh * sizeof(RangeSlot);
    return (raw + 255) / 256 * 256;
}

size_t parts_bytes(int64_t nh, int32_t K) { return ((size_t)nh * kParts * K * sizeof(uint32_t) + 255) / 256 * 256; }

size_t workspace_bytes(int64_t nh, int32_t K)
{
    return slots_bytes(nh) + parts_bytes(nh, K) + (size_t)kMaxBlocks * sizeof(RangePart) + slots_bytes(nh * kSubSlots);
}

// Fold given partial ranges into the first sub-slot of the (single) histogram (the others stay empty).
__global__ __launch_bounds__(kThreads) void k_entropy_fold_parts(const RangePart* __restrict__ rparts, int nrparts, RangeSlot* slots)
{
    uint32_t klo = 0xffffffffu, khi = 0u, knan = 0u;
    for (int i = threadIdx.x; i < nrparts; i += kThreads) {
        const RangePart rp = rparts[i];
        klo = min(klo, rp.lo_key);
        khi = max(khi, rp.hi_key);
        knan |= rp.saw_nan;
    }
    reduce_range_keys(klo, khi, knan);
    if (threadIdx.x == 0) {
        slots[0].lo_key = klo; slots[0].hi_key = khi; slots[0].saw_nan = knan; slots[0].pad = 0u;
    }
}

template <typename T, bool SAMPLED>
void launch_flat(const word4* x, int64_t nwords, WordMap<SAMPLED> map, int32_t K, RangeSlot* slots, uint32_t* parts,
                 RangePart* rparts, hipStream_t stream)
{
    int64_t blocks = (nwords + (int64_t)kThreads * kUnroll - 1) / ((int64_t)kThreads * kUnroll);
    blocks = blocks < 1 ? 1 : (blocks > kFlatBlocks ? kFlatBlocks : blocks);
    k_entropy_range_flat<T, SAMPLED><<<dim3((unsigned)blocks), dim3(kThreads), 0, stream>>>(x, nwords, map, rparts, parts, kParts * K);
    k_entropy_count_flat<T, SAMPLED><<<dim3((unsigned)blocks), dim3(kThreads), 0, stream>>>(x, nwords, map, K, rparts, (int)blocks,
                                                                                          slots, parts);
}

// What the caller wants done with the partial histograms once the sweeps are enqueued.
struct Tail {
    const corey_policy* pol;            // NULL: statistic only
    int32_t* chunks_out;
    double ema_lambda;
    double* ema_state;
    uint32_t* chunk_calls;
    corey_finalise::Args* defer;        // not NULL: do not launch the reduction, describe it here instead
};

template <typename T>
int launch(const void* x, int64_t B, int64_t D, int64_t L, const int32_t* seqlens, int32_t K, double eps, int64_t stride,
           int64_t block, uint32_t* counts, double* H_out, double* r_out, float* range_out, RangeSlot* slots, hipStream_t stream,
           const Tail& tail, Handoff* handoff)
{
    const int nh = seqlens ? (int)B : 1;
    uint32_t* parts = reinterpret_cast<uint32_t*>(reinterpret_cast<char*>(slots) + slots_bytes(B));
    RangePart* rparts = reinterpret_cast<RangePart*>(reinterpret_cast<char*>(parts) + parts_bytes(B, K));
    RangeSlot* subs = reinterpret_cast<RangeSlot*>(rparts + kMaxBlocks);
    const int64_t nparts = (int64_t)nh * kParts * K;
    uint32_t* final_parts = parts;                              // where the reduction finds the partial histograms
    bool rezero = false;

    constexpr int V = Elem<T>::kVec;
    const int64_t E = B * D * L;
    const bool flat_ok = !seqlens && reinterpret_cast<uintptr_t>(x) % kVecBytes == 0 && E % V == 0;
    const int64_t bw = block / V;                              // 16-byte words per sampling block
    const bool flat_blocks = flat_ok && block % V == 0 && corey::is_pow2(bw);    // sampled runs are whole 16-byte words
    if (handoff && flat_ok && (stride == 1 || flat_blocks)) {
        // the producer of x left its partial ranges and cleared partial histograms beside them: one launch, the count sweep
        // (over every word, or over the words of every stride-th block), whose workgroups fold the partial ranges themselves
        int64_t nwords = E / V;
        int bw_log2 = 0;
        if (stride > 1) {
            const int64_t nb = (nwords + bw - 1) / bw;
            const int64_t ns = (nb + stride - 1) / stride;
            const int64_t last_first = (ns - 1) * stride * bw;
            const int64_t last_words = nwords - last_first < bw ? nwords - last_first : bw;
            while (((int64_t)1 << bw_log2) < bw) ++bw_log2;
            nwords = (ns - 1) * bw + last_words;
        }
        int64_t blocks = (nwords + (int64_t)kThreads * kUnroll - 1) / ((int64_t)kThreads * kUnroll);
        blocks = blocks < 1 ? 1 : (blocks > kFlatBlocks ? kFlatBlocks : blocks);
        if (stride == 1)
            k_entropy_count_flat<T, false><<<dim3((unsigned)blocks), dim3(kThreads), 0, stream>>>(
                static_cast<const word4*>(x), nwords, WordMap<false>{0, 1}, K, handoff->parts, COREY_RANGE_PARTS, slots, handoff->counts);
        else
            k_entropy_count_flat<T, true><<<dim3((unsigned)blocks), dim3(kThreads), 0, stream>>>(
                static_cast<const word4*>(x), nwords, WordMap<true>{bw_log2, stride}, K, handoff->parts, COREY_RANGE_PARTS, slots,
                handoff->counts);
        final_parts = handoff->counts;
        rezero = true;                                          // left cleared for the next statistic on this buffer
    } else if (handoff) {
        // unaligned tensor: one workgroup folds the partial ranges into the slot, then the general count sweep
        k_entropy_init<<<dim3((unsigned)((nparts + kThreads - 1) / kThreads)), dim3(kThreads), 0, stream>>>(parts, nparts, slots, nh, subs);
        k_entropy_fold_parts<<<dim3(1), dim3(kThreads), 0, stream>>>(handoff->parts, COREY_RANGE_PARTS, subs);
        const bool vector_ok = (reinterpret_cast<uintptr_t>(x) % kVecBytes == 0) && (L % V == 0);
        const int64_t seg = (int64_t)kThreads * V * kUnroll;
        int64_t blocks = B * D * ((L + seg - 1) / seg);
        blocks = blocks < 1 ? 1 : (blocks > kMaxBlocks ? kMaxBlocks : blocks);
        k_entropy_count<T><<<dim3((unsigned)blocks, 1), dim3(kThreads), 0, stream>>>(static_cast<const T*>(x), B, D, L, nullptr, stride,
                                                                                   block, vector_ok ? 1 : 0, K, subs, slots, parts);
    } else if (flat_ok && stride == 1) {
        // whole tensor, every value, aligned: flat sweeps
        launch_flat<T, false>(static_cast<const word4*>(x), E / V, WordMap<false>{0, 1}, K, slots, parts, rparts, stream);
    } else if (flat_blocks) {
        // whole tensor, every stride-th block of a power-of-two number of words: flat sweeps over the sampled words only
        const int64_t nwords_all = E / V;
        const int64_t nb = (nwords_all + bw - 1) / bw;          // blocks in the tensor (the last may be short)
        const int64_t ns = (nb + stride - 1) / stride;          // sampled blocks
        const int64_t last_first = (ns - 1) * stride * bw;      // first word of the last sampled block
        const int64_t last_words = nwords_all - last_first < bw ? nwords_all - last_first : bw;
        int bw_log2 = 0;
        while (((int64_t)1 << bw_log2) < bw) ++bw_log2;
        launch_flat<T, true>(static_cast<const word4*>(x), (ns - 1) * bw + last_words, WordMap<true>{bw_log2, stride}, K, slots,
                             parts, rparts, stream);
    } else {
        k_entropy_init<<<dim3((unsigned)((nparts + kThreads - 1) / kThreads)), dim3(kThreads), 0, stream>>>(parts, nparts, slots, nh, subs);
        const bool vector_ok = (reinterpret_cast<uintptr_t>(x) % kVecBytes == 0) && (L % V == 0);
        const int64_t rows = seqlens ? D : B * D;
        const int64_t seg = (int64_t)kThreads * V * kUnroll;
        const int64_t units = rows * ((L + seg - 1) / seg);
        // about kMaxBlocks workgroups over all histograms (each pays for clearing and merging its LDS counters), at
        // least 8 per histogram
        const int64_t cap = kMaxBlocks / nh > 8 ? kMaxBlocks / nh : 8;
        int64_t blocks = units < 1 ? 1 : units;
        if (blocks > cap) blocks = cap;
        const dim3 grid((unsigned)blocks, (unsigned)nh);
        k_entropy_range<T><<<grid, dim3(kThreads), 0, stream>>>(static_cast<const T*>(x), B, D, L, seqlens, stride, block,
                                                               vector_ok ? 1 : 0, subs);
        k_entropy_count<T><<<grid, dim3(kThreads), 0, stream>>>(static_cast<const T*>(x), B, D, L, seqlens, stride, block,
                                                               vector_ok ? 1 : 0, K, subs, slots, parts);
    }
    corey_finalise::Args fa = {};
    fa.parts = final_parts; fa.slots = slots; fa.counts = counts; fa.H_out = H_out; fa.r_out = r_out; fa.range_out = range_out;
    fa.chunks_out = tail.pol ? tail.chunks_out : nullptr; fa.seqlens = seqlens; fa.ema_state = tail.ema_state;
    fa.chunk_calls = tail.chunk_calls; fa.L_all = L; fa.eps = eps; fa.ema_lambda = tail.ema_lambda;
    if (tail.pol) fa.pol = *tail.pol;
    fa.K = K; fa.nh = nh; fa.rezero = rezero ? 1 : 0;
    if (tail.defer) *tail.defer = fa;                           // the scan's first kernel will do it
    else k_entropy_finalise<<<dim3((unsigned)nh), dim3(kThreads), 0, stream>>>(fa);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return corey::hip_fail(e, "corey_entropy_hist launch");
    return COREY_OK;
}

}  // namespace

namespace corey {

// The policy as the GPU rule will apply it: the host rule's checks (r = 0.5 is a placeholder that no mode rejects), and
// no chunk the scan cannot run (the rule's result goes straight into selective_scan_fwd's chunks_dev and into the
// chunk-distribution counters, which have a slot per power of two up to COREY_MAX_CHUNK).
int check_device_policy(const char* who, const corey_policy* p, int64_t L)
{
    using corey::fail;
    int32_t probe = 0;
    const int st = corey_select_chunk(0.5, L < 1 ? 1 : L, p, &probe);
    if (st != COREY_OK) return st;
    if (p->mode == 1 && !corey::is_pow2(p->short_chunk)) return fail(COREY_EINVAL, "%s: short_chunk = %d", who, p->short_chunk);
    const bool entropy = p->mode == 0 || p->mode == 1 || p->mode == 4;
    const bool table = p->mode == 1 || p->mode == 2;
    if ((entropy && p->c_max > COREY_MAX_CHUNK) || (table && p->short_chunk > COREY_MAX_CHUNK) ||
        (p->mode == 2 && p->long_chunk > COREY_MAX_CHUNK) || (p->mode == 3 && p->static_chunk > COREY_MAX_CHUNK) ||
        (p->mode == 4 && p->safe_chunk > COREY_MAX_CHUNK))
        return fail(COREY_EINVAL, "%s: the policy can select a chunk above %d", who, COREY_MAX_CHUNK);
    return COREY_OK;
}

int launch_entropy_finalise(const uint32_t* parts, uint32_t* counts, int32_t K, double eps, const void* slot, double* H_out,
                            double* r_out, float* range_out, const corey_policy* pol, int32_t* chunks_out, int64_t L,
                            hipStream_t stream)
{
    corey_finalise::Args fa = {};
    fa.parts = const_cast<uint32_t*>(parts); fa.slots = static_cast<const RangeSlot*>(slot); fa.counts = counts; fa.H_out = H_out;
    fa.r_out = r_out; fa.range_out = range_out; fa.chunks_out = pol ? chunks_out : nullptr; fa.L_all = L; fa.eps = eps;
    if (pol) fa.pol = *pol;
    fa.K = K; fa.nh = 1;
    fa.rezero = 1;                                              // the next statistic from the same table adds into them again
    k_entropy_finalise<<<dim3(1), dim3(kThreads), 0, stream>>>(fa);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(e, "entropy reduction launch");
    return COREY_OK;
}

}  // namespace corey

using corey::check_device_policy;

extern "C" int corey_select_chunk_device(const double* r_dev, const int32_t* seqlens, int64_t L, int32_t nh,
                                         const corey_policy* p, int32_t* chunks_out, void* hip_stream)
{
    using corey::fail;
    if (!r_dev || !p || !chunks_out) return fail(COREY_ENULL, "corey_select_chunk_device: r_dev, p and chunks_out are required");
    if (nh < 1) return fail(COREY_EINVAL, "corey_select_chunk_device: nh = %d < 1", nh);
    if (!seqlens && L < 1) return fail(COREY_EINVAL, "corey_select_chunk_device: L = %lld < 1", (long long)L);
    const int st = check_device_policy("corey_select_chunk_device", p, L);
    if (st != COREY_OK) return st;
    k_select_chunk<<<dim3((unsigned)((nh + 63) / 64)), dim3(64), 0, static_cast<hipStream_t>(hip_stream)>>>(r_dev, seqlens, L, nh, *p, chunks_out);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return corey::hip_fail(e, "corey_select_chunk_device launch");
    return COREY_OK;
}

extern "C" size_t corey_entropy_hist_workspace(int64_t B, int32_t K)
{
    if (B < 1 || K < 2 || K > COREY_MAX_BINS) return 0;
    return workspace_bytes(B, K);
}

namespace {

int entropy_hist_impl(const char* who, const void* x, corey_dtype dt, int64_t B, int64_t D, int64_t L, const int32_t* seqlens, int32_t K,
                      double eps, int64_t stride, int64_t block, uint32_t* counts_out, double* H_out, double* r_out, float* range_out,
                      void* workspace, size_t workspace_bytes_given, void* hip_stream, const Tail& tail, void* range_parts)
{
    using corey::fail;
    if (!x || !counts_out || !H_out || !r_out) return fail(COREY_ENULL, "%s: x, counts_out, H_out and r_out are required", who);
    if (dt != COREY_F32 && dt != COREY_BF16 && dt != COREY_F16) return fail(COREY_EINVAL, "%s: unknown dtype %d", who, (int)dt);
    if (B < 1 || D < 1 || L < 1) return fail(COREY_ESHAPE, "%s: B, D, L must be >= 1", who);
    if (B > 65535) return fail(COREY_ESHAPE, "%s: B = %lld exceeds 65535", who, (long long)B);
    if ((double)B * (double)D * (double)L >= 9.0e18) return fail(COREY_ESHAPE, "%s: B*D*L overflows", who);
    if ((double)B * (double)D * (double)L >= 4294967296.0 && stride == 1)
        return fail(COREY_ESHAPE, "%s: more than 2^32-1 samples would overflow the 32-bit counts", who);
    if (K < 2 || K > COREY_MAX_BINS) return fail(COREY_EINVAL, "%s: K = %d outside [2, %d]", who, K, COREY_MAX_BINS);
    if (!(eps >= 0.0)) return fail(COREY_EINVAL, "%s: eps must be >= 0", who);
    if (stride < 1 || block < 1) return fail(COREY_EINVAL, "%s: stride and block must be >= 1", who);
    if (range_parts && seqlens)
        return fail(COREY_EINVAL, "%s: range_parts needs the whole-tensor statistic (seqlens NULL)", who);
    if (range_parts && reinterpret_cast<uintptr_t>(range_parts) % 16 != 0) return fail(COREY_EINVAL, "%s: range_parts must be 16-byte aligned", who);
    const size_t need = workspace_bytes(B, K);
    if (!workspace || workspace_bytes_given < need) return fail(COREY_EWORKSPACE, "%s: workspace of %zu bytes required", who, need);
    if (reinterpret_cast<uintptr_t>(workspace) % 16 != 0) return fail(COREY_EWORKSPACE, "%s: workspace must be 16-byte aligned", who);
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    RangeSlot* slots = static_cast<RangeSlot*>(workspace);
    Handoff* handoff = static_cast<Handoff*>(range_parts);
    if (dt == COREY_F32)
        return launch<float>(x, B, D, L, seqlens, K, eps, stride, block, counts_out, H_out, r_out, range_out, slots, stream, tail, handoff);
    if (dt == COREY_F16)
        return launch<_Float16>(x, B, D, L, seqlens, K, eps, stride, block, counts_out, H_out, r_out, range_out, slots, stream, tail, handoff);
    return launch<uint16_t>(x, B, D, L, seqlens, K, eps, stride, block, counts_out, H_out, r_out, range_out, slots, stream, tail, handoff);
}

}  // namespace

extern "C" int corey_entropy_hist(const void* x, corey_dtype dt, int64_t B, int64_t D, int64_t L, const int32_t* seqlens,
                                  int32_t K, double eps, int64_t stride, int64_t block, uint32_t* counts_out, double* H_out,
                                  double* r_out, float* range_out, void* range_parts, void* workspace,
                                  size_t workspace_bytes_given, void* hip_stream)
{
    return entropy_hist_impl("corey_entropy_hist", x, dt, B, D, L, seqlens, K, eps, stride, block, counts_out, H_out, r_out, range_out,
                             workspace, workspace_bytes_given, hip_stream, Tail{}, range_parts);
}

// ---------------------------------------------------------------------------------------------------------
// corey_entropy_hist_static: the same statistic for callers that cannot allocate (HIP graph capture, serving loops
// that may not call hipMalloc).  The workspace of corey_entropy_hist lives in an array in the GPU's global memory that is
// part of the library's code object: every GPU the library runs on holds its own copy at its own address until the
// process ends.  On the host the array's name is only a handle: the address kernels can use is asked for once per
// device (hipGetSymbolAddress, with that device current) and kept.
static __device__ __align__(256) unsigned char scratch[COREY_STATIC_SCRATCH_BYTES];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};      // address of `scratch` on each device, filled on first use

// The current device's copy of `scratch` (NULL after recording the error).
void* static_scratch(const char* who)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) {
        corey::hip_fail(e, who);
        return nullptr;
    }
    if (dev < 0 || dev >= kMaxDevices) {
        corey::fail(COREY_EUNSUPPORTED, "%s: device index %d beyond the %d this entry point keeps an address for", who, dev, kMaxDevices);
        return nullptr;
    }
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !ptr) {
            corey::hip_fail(e, "hipGetSymbolAddress(scratch)");
            return nullptr;
        }
        g_scratch_ptr[dev] = ptr;
    }
    return g_scratch_ptr[dev];
}

}  // namespace

extern "C" int corey_entropy_hist_static(const void* x, corey_dtype dt, int64_t B, int64_t D, int64_t L, const int32_t* seqlens,
                                         int32_t K, double eps, int64_t stride, int64_t block, uint32_t* counts_out, double* H_out,
                                         double* r_out, float* range_out, void* range_parts, void* hip_stream)
{
    const size_t need = corey_entropy_hist_workspace(B, K);     // 0 for invalid B or K: the common checks below name those
    if (need > COREY_STATIC_SCRATCH_BYTES)
        return corey::fail(COREY_EWORKSPACE, "corey_entropy_hist_static: B = %lld with K = %d needs %zu bytes of scratch, the built-in "
                           "buffer holds %d (use corey_entropy_hist with a workspace of your own)", (long long)B, K, need,
                           COREY_STATIC_SCRATCH_BYTES);
    void* ws = static_scratch("corey_entropy_hist_static");
    if (!ws) return COREY_EHIP;
    return entropy_hist_impl("corey_entropy_hist_static", x, dt, B, D, L, seqlens, K, eps, stride, block, counts_out, H_out, r_out,
                             range_out, ws, COREY_STATIC_SCRATCH_BYTES, hip_stream, Tail{}, range_parts);
}

extern "C" int corey_route_device(const void* x, corey_dtype dt, int64_t B, int64_t D, int64_t L, const int32_t* seqlens,
                                  int32_t K, double eps, int64_t stride, int64_t block, const corey_policy* p,
                                  double ema_lambda, double* ema_state, uint32_t* chunk_calls,
                                  uint32_t* counts_out, double* H_out, double* r_out, float* range_out, void* range_parts,
                                  int32_t* chunks_out, void* workspace, size_t workspace_bytes_given, void* hip_stream)
{
    using corey::fail;
    if (!p || !chunks_out) return fail(COREY_ENULL, "corey_route_device: p and chunks_out are required");
    if (ema_state && !(ema_lambda >= 0.0 && ema_lambda < 1.0))
        return fail(COREY_EINVAL, "corey_route_device: ema_lambda = %g outside [0, 1)", ema_lambda);
    const int st = check_device_policy("corey_route_device", p, L);
    if (st != COREY_OK) return st;
    Tail tail = {};
    tail.pol = p; tail.chunks_out = chunks_out; tail.ema_lambda = ema_lambda; tail.ema_state = ema_state; tail.chunk_calls = chunk_calls;
    return entropy_hist_impl("corey_route_device", x, dt, B, D, L, seqlens, K, eps, stride, block, counts_out, H_out, r_out, range_out,
                             workspace, workspace_bytes_given, hip_stream, tail, range_parts);
}

static_assert(sizeof(corey_finalise::Args) <= sizeof(corey_deferred_route), "the opaque ticket holds the reduction's arguments");

extern "C" int corey_route_device_deferred(const void* x, corey_dtype dt, int64_t B, int64_t D, int64_t L, const int32_t* seqlens,
                                           int32_t K, double eps, int64_t stride, int64_t block, const corey_policy* p,
                                           uint32_t* chunk_calls, uint32_t* counts_out, double* H_out, double* r_out,
                                           float* range_out, void* range_parts, int32_t* chunks_out, void* workspace,
                                           size_t workspace_bytes_given, corey_deferred_route* route, void* hip_stream)
{
    using corey::fail;
    if (!p || !chunks_out || !route) return fail(COREY_ENULL, "corey_route_device_deferred: p, chunks_out and route are required");
    const int st = check_device_policy("corey_route_device_deferred", p, L);
    if (st != COREY_OK) return st;
    corey_finalise::Args fa = {};
    Tail tail = {};
    tail.pol = p; tail.chunks_out = chunks_out; tail.chunk_calls = chunk_calls; tail.defer = &fa;
    const int rc = entropy_hist_impl("corey_route_device_deferred", x, dt, B, D, L, seqlens, K, eps, stride, block, counts_out, H_out, r_out,
                                     range_out, workspace, workspace_bytes_given, hip_stream, tail, range_parts);
    if (rc != COREY_OK) return rc;
    memset(route, 0, sizeof(*route));
    memcpy(route, &fa, sizeof(fa));
    return COREY_OK;
}
