// The O(K) end of the entropy statistic as a device function: partial histograms -> counts, H = -sum p log(p + eps)
// (Eq. 1), r = H / log K, and Eq. 2 with the scheduler family around it.  It runs as a kernel of its own
// (k_entropy_finalise) or, for a routed scan, at the start of the kernel that lays out B and C for the scan (every
// workgroup of that kernel evaluates it for its sequence and arrives at the same chunk; the first one publishes the
// results), which takes one dependent launch out of the routed path.
#ifndef COREY_FINALISE_H
#define COREY_FINALISE_H

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "corey.h"
#include "corey_range.h"

namespace corey_finalise {

constexpr int kThreads = 256;          // lanes of a workgroup that calls finalise()

// Everything the reduction of one call needs.  Pointers are device pointers owned by the caller.
struct Args {
    uint32_t* parts;                   // [nh][kParts][K] partial histograms (NULL: nothing to do)
    const corey_range::RangeSlot* slots;   // [nh] range of each histogram
    uint32_t* counts;                  // [nh][K] out
    double* H_out;                     // [nh] out
    double* r_out;                     // [nh] out
    float* range_out;                  // [nh][2] out or NULL
    int32_t* chunks_out;               // [nh] out or NULL (no rule)
    const int32_t* seqlens;            // [nh] or NULL: the sequence length each decision is taken for (else L_all)
    double* ema_state;                 // [nh] or NULL
    uint32_t* chunk_calls;             // [COREY_CHUNK_SLOTS] or NULL
    int64_t L_all;
    double eps, ema_lambda;
    corey_policy pol;
    int32_t K, nh;
    int32_t rezero;                    // clear the partial histograms after reading them (they live in a buffer that the next
                                       // count sweep adds into without a clearing launch of its own)
};

// Eq. 2 and the scheduler family around it for one histogram (see corey_select_chunk for the rule); 0 when r is NaN
// in an entropy mode.
__device__ __forceinline__ int32_t chunk_rule(double rv, int64_t L, const corey_policy& p)
{
    if (L < 1) L = 1;
    const bool short_seq = L <= p.short_len;
    int64_t c;
    if (p.mode == 3) {
        c = p.static_chunk;
    } else if (p.mode == 2) {
        c = short_seq ? p.short_chunk : p.long_chunk;
    } else if (p.mode == 1 && short_seq) {
        c = p.short_chunk;
    } else {
        if (rv != rv) return 0;
        double re = rv * p.h_ref_scale;
        re = re < 0.0 ? 0.0 : (re > 1.0 ? 1.0 : re);
        const double target = (double)p.c_min + re * (double)(p.c_max - p.c_min);
        const double k = floor(log2(target) + 0.5);
        c = (int64_t)1 << (int)k;
        c = c < p.c_min ? p.c_min : (c > p.c_max ? p.c_max : c);
        if (p.mode == 4) {
            int away = (63 - __clzll((long long)c)) - (63 - __clzll((long long)p.safe_chunk));
            away = away < 0 ? -away : away;
            if (away < p.guard_buckets) c = p.safe_chunk;
        }
        int64_t cap = 1;
        while (cap < L) cap <<= 1;
        if (cap < p.c_min) cap = p.c_min;
        if (c > cap) c = cap;
    }
    return (int32_t)c;
}

// Histogram h of the call, by all kThreads lanes of a workgroup.  Returns the chunk the rule selects (0: no rule, or r is
// NaN in an entropy mode) in every lane; with `publish` the workgroup also writes counts, H, r, range and chunk, updates
// the moving average and the chunk counters.  Two workgroups that evaluate the same histogram add the same numbers in
// the same order and get the same bits.
__device__ __forceinline__ int32_t finalise(const Args& a, int h, bool publish)
{
    using corey_range::kParts;
    constexpr int kPer = COREY_MAX_BINS / kThreads;             // bins a lane owns at most
    const int K = a.K;
    uint32_t* ph = a.parts + (int64_t)h * kParts * K;
    uint32_t c[kPer];
    unsigned long long n_part = 0;
#pragma unroll
    for (int i = 0; i < kPer; ++i) {
        const int k = (int)threadIdx.x + i * kThreads;
        uint32_t sum = 0;
        if (k < K)
            for (int q = 0; q < kParts; ++q) sum += ph[(size_t)q * K + k];
        c[i] = sum;
        n_part += sum;
    }
    if (publish) {
#pragma unroll
        for (int i = 0; i < kPer; ++i) {
            const int k = (int)threadIdx.x + i * kThreads;
            if (k < K) a.counts[(int64_t)h * K + k] = c[i];
        }
        if (a.rezero) {
#pragma unroll
            for (int i = 0; i < kPer; ++i) {
                const int k = (int)threadIdx.x + i * kThreads;
                if (k < K)
                    for (int q = 0; q < kParts; ++q) ph[(size_t)q * K + k] = 0u;
            }
        }
    }
    float lo = 0.f, hi = 0.f;
    const corey_range::RangeSlot slot = a.slots[h];
    const bool ok = corey_range::usable_range(slot, &lo, &hi);
    // two workgroup sums (the sample count, then the entropy terms): butterfly inside each wave, the waves' totals
    // through LDS; every lane ends up with the same total, added in the same order
    __shared__ double s_red[kThreads / 64];
    __shared__ unsigned long long s_n[kThreads / 64];
    __shared__ int32_t s_chunk;
    const int wave = threadIdx.x >> 6;

    for (int off = 32; off > 0; off >>= 1) n_part += __shfl_xor(n_part, off);
    if ((threadIdx.x & 63) == 0) s_n[wave] = n_part;
    __syncthreads();
    unsigned long long n_all = 0;
    for (int w = 0; w < kThreads / 64; ++w) n_all += s_n[w];
    const double n = (double)n_all;

    double part = 0.0;
    if (ok && n > 0.0) {
#pragma unroll
        for (int i = 0; i < kPer; ++i) {
            if (c[i] == 0u) continue;                          // an empty bin adds nothing (0 log 0 = 0 when eps = 0)
            const double p = (double)c[i] / n;
            part += p * log(p + a.eps);
        }
    }
    for (int off = 32; off > 0; off >>= 1) part += __shfl_xor(part, off);
    if ((threadIdx.x & 63) == 0) s_red[wave] = part;
    __syncthreads();
    if (threadIdx.x == 0) {
        double H = NAN, r = NAN;
        if (ok && n > 0.0) {
            double acc = 0.0;
            for (int w = 0; w < kThreads / 64; ++w) acc += s_red[w];
            H = -acc;
            r = H / log((double)K);
            r = r < 0.0 ? 0.0 : (r > 1.0 ? 1.0 : r);
        }
        int32_t chunk = 0;
        if (a.chunks_out) {
            double r_rule = r;
            if (a.ema_state) {                                 // the rule sees the entropy smoothed across calls
                const double prev = a.ema_state[h];
                double Hs = prev;
                if (H == H) Hs = (prev != prev) ? H : a.ema_lambda * prev + (1.0 - a.ema_lambda) * H;
                if (publish) a.ema_state[h] = Hs;
                r_rule = Hs / log((double)K);
                r_rule = r_rule < 0.0 ? 0.0 : (r_rule > 1.0 ? 1.0 : r_rule);
            }
            chunk = chunk_rule(r_rule, a.seqlens ? (int64_t)a.seqlens[h] : a.L_all, a.pol);
        }
        s_chunk = chunk;
        if (publish) {
            a.H_out[h] = H;
            a.r_out[h] = r;
            if (a.chunks_out) {
                a.chunks_out[h] = chunk;
                if (a.chunk_calls && chunk > 0 && 31 - __clz(chunk) < COREY_CHUNK_SLOTS) atomicAdd(&a.chunk_calls[31 - __clz(chunk)], 1u);
            }
            if (a.range_out) {
                a.range_out[2 * h] = (slot.lo_key == 0xffffffffu) ? INFINITY : corey_range::key_value(slot.lo_key);
                a.range_out[2 * h + 1] = (slot.hi_key == 0u) ? -INFINITY : corey_range::key_value(slot.hi_key);
            }
        }
    }
    __syncthreads();
    return s_chunk;
}

}  // namespace corey_finalise
#endif
