// causal_conv1d_silu_fwd: the causal depthwise convolution and SiLU that produce the scan input u, with the range of
// u (what the histogram's first sweep would compute) taken in the same pass.
//
// One kernel.  A workgroup of 256 lanes takes (row, segment) units grid-stride, two at a time so that their loads are
// in flight together; per unit a lane owns one 16-byte vector of consecutive time steps, loads it and the vector
// before it (the W - 1 <= 3 earlier inputs the taps reach back to;
// at the start of a row they come from state_in or are zero), accumulates the taps oldest first with fused
// multiply-adds in binary32, applies v * sigmoid(v), rounds to the storage type and stores 16 bytes.  The minimum
// and maximum are taken over the values as stored (the histogram will see those bits), kept per lane and reduced
// once per workgroup into a partial range; corey_entropy_hist reduces the COREY_RANGE_PARTS partials.
// Bandwidth work (x in, u out): no matrix instructions.
#include <hip/hip_runtime.h>

#include <cmath>

#include "corey_internal.h"
#include "corey_range.h"
#include "corey_table.h"

namespace {

using corey::bf16_to_f32;
using corey_range::kThreads;
using corey_range::order_key;
using corey_range::Handoff;
using corey_range::RangePart;
using corey_range::reduce_range_keys;

#ifndef COREY_CONV_UNITS
#define COREY_CONV_UNITS 2
#endif

constexpr float kLog2e = 1.4426950408889634f;
typedef uint32_t word4 __attribute__((ext_vector_type(4)));
typedef float float2v __attribute__((ext_vector_type(2)));

// Storage type: widen one element, round a vector of values (to nearest even), elements per 16-byte vector.
template <typename T> struct St;
template <> struct St<float> {
    static constexpr int kVec = 4;
    static __device__ __forceinline__ float widen(float v) { return v; }
    static __device__ __forceinline__ void narrow(const float (&v)[4], float (&out)[4])
    {
#pragma unroll
        for (int e = 0; e < 4; ++e) out[e] = v[e];
    }
};
template <> struct St<uint16_t> {                       // bfloat16 bit patterns
    static constexpr int kVec = 8;
    static __device__ __forceinline__ float widen(uint16_t v) { return bf16_to_f32(v); }
    static __device__ __forceinline__ void narrow(const float (&v)[8], uint16_t (&out)[8])
    {
        typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
#pragma unroll
        for (int e = 0; e < 8; e += 2) {
            float2v f;
            f.x = v[e]; f.y = v[e + 1];
            const bf16x2 h = __builtin_convertvector(f, bf16x2);    // v_cvt_pk_bf16_f32
            __builtin_memcpy(&out[e], &h, 4);
        }
    }
};
template <> struct St<_Float16> {
    static constexpr int kVec = 8;
    static __device__ __forceinline__ float widen(_Float16 v) { return (float)v; }
    static __device__ __forceinline__ void narrow(const float (&v)[8], _Float16 (&out)[8])
    {
#pragma unroll
        for (int e = 0; e < 8; ++e) out[e] = (_Float16)v[e];
    }
};

// min / max that return the other operand when one is NaN (the hardware's IEEE-mode behaviour), without the
// canonicalising extra instruction the generic fminf / fmaxf lowering adds per call
__device__ __forceinline__ float vmin(float a, float b)
{
    float r;
    asm("v_min_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
    return r;
}
__device__ __forceinline__ float vmax(float a, float b)
{
    float r;
    asm("v_max_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
    return r;
}

constexpr int H = COREY_MAX_CONV - 1;                     // most earlier inputs a tap reaches back to

// The inputs one lane needs for one vector of outputs: xs[H + e] = x[t0 + e] and the H inputs before them
// (xs[H - k] = x[t0 - k]), from the previous vector of the row, from state_in before the row starts, or zero.
template <typename T>
__device__ __forceinline__ void load_inputs(const T* __restrict__ xr, const T* __restrict__ state_row, int64_t t0, int nvalid,
                                            int W, bool vector_ok, float (&xs)[H + St<T>::kVec])
{
    constexpr int V = St<T>::kVec;
    if (vector_ok && nvalid == V) {
        T cur[V];
        const word4 q = *reinterpret_cast<const word4*>(xr + t0);
        __builtin_memcpy(cur, &q, 16);
#pragma unroll
        for (int e = 0; e < V; ++e) xs[H + e] = St<T>::widen(cur[e]);
    } else {
#pragma unroll
        for (int e = 0; e < V; ++e) xs[H + e] = (e < nvalid) ? St<T>::widen(xr[t0 + e]) : 0.f;
    }
    if (t0 >= V && vector_ok) {
        T prev[V];
        const word4 q = *reinterpret_cast<const word4*>(xr + t0 - V);
        __builtin_memcpy(prev, &q, 16);
#pragma unroll
        for (int k = 1; k <= H; ++k) xs[H - k] = St<T>::widen(prev[V - k]);
    } else {
#pragma unroll
        for (int k = 1; k <= H; ++k) {
            const int64_t t = t0 - k;
            float v = 0.f;
            if (t >= 0) v = St<T>::widen(xr[t]);
            else if (state_row && t + (W - 1) >= 0) v = St<T>::widen(state_row[t + (W - 1)]);
            xs[H - k] = v;
        }
    }
}

// One vector of outputs from its inputs: taps oldest first with fused multiply-adds, v * sigmoid(v), one rounding to
// the storage type.  Rounding to nearest is monotonic, so the range of the stored values is the rounded range of the
// unrounded ones: lo / hi follow the binary32 results and are rounded once at the end of the kernel.
template <typename T, int W, bool FULL>
__device__ __forceinline__ void conv_vector(const float (&xs)[H + St<T>::kVec], const float (&w)[W], float bs, int nvalid,
                                            T (&out)[St<T>::kVec], float& lo, float& hi, bool& nan)
{
    constexpr int V = St<T>::kVec;
    float val[V];
#pragma unroll
    for (int e = 0; e < V; ++e) {
        float acc = bs;
#pragma unroll
        for (int k = 0; k < W; ++k) acc = fmaf(w[k], xs[H + e - (W - 1) + k], acc);
        val[e] = acc * __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(-acc * kLog2e));
        if (FULL || e < nvalid) {
            nan |= (val[e] != val[e]);
            lo = vmin(lo, val[e]);
            hi = vmax(hi, val[e]);
        }
    }
    St<T>::narrow(val, out);
}

// Position of a workgroup's next unit: row, segment within the row, channel of the row.  Units are numbered
// row * nseg + seg and a workgroup visits every gridDim.x-th one; stepping the three coordinates by the quotient and
// remainder of that stride keeps the 64-bit divisions out of the loop.
struct Cursor {
    int64_t row, seg, d;
};
struct Stride {
    int64_t q, rem, qd, nseg, D;
};
__device__ __forceinline__ Cursor advance(Cursor c, const Stride& s)
{
    c.seg += s.rem;
    const int64_t carry = (c.seg >= s.nseg) ? 1 : 0;
    c.seg -= carry ? s.nseg : 0;
    c.row += s.q + carry;
    c.d += s.qd + carry;
    c.d -= (c.d >= s.D) ? s.D : 0;
    return c;
}

// Count the stored values of one vector in the workgroup's bit-pattern table (16-bit storage).
template <typename T>
__device__ __forceinline__ void table_add_vector(uint32_t* s_tab, corey_table::Shared& sh, const T (&out)[St<T>::kVec], int nvalid)
{
    if constexpr (sizeof(T) == 2) {
        if (nvalid == St<T>::kVec) {
            uint32_t w[4];
            __builtin_memcpy(w, out, 16);
            corey_table::add_word4(s_tab, sh, w);
        } else {
#pragma unroll
            for (int e = 0; e < St<T>::kVec; ++e) {
                if (e < nvalid) {
                    uint16_t bits;
                    __builtin_memcpy(&bits, &out[e], 2);
                    corey_table::add(s_tab, sh, bits);
                }
            }
        }
    }
}

// NT lanes per workgroup.  TABLE: the workgroup also counts the bit patterns of the values it stores (corey_table.h:
// NT = corey_table::kLanes, at most corey_table::kMaxSlabs workgroups, 16-bit storage); a turn of the unit loop adds at
// most U * NT * 8 = 16384 values and ends at a barrier, inside the table's bound of 32768 per round.
template <typename T, int W, int NT, bool TABLE>
__global__ __launch_bounds__(NT) void k_conv1d_silu(const T* __restrict__ x, const float* __restrict__ weight,
                                                    const float* __restrict__ bias, const T* __restrict__ state_in,
                                                    T* __restrict__ u, T* __restrict__ state_out, Handoff* __restrict__ handoff,
                                                    void* table_ws, int64_t rows, int64_t D, int64_t L, int vector_ok)
{
    RangePart* rparts = handoff ? handoff->parts : nullptr;
    if (handoff) corey_range::clear_handoff_counts(handoff);   // the statistic's count sweep adds into them
    constexpr int kThreads = NT;                              // (shadows the 256 of the other kernels in this file)
    constexpr int V = St<T>::kVec;
    constexpr int U = COREY_CONV_UNITS;                       // units in flight per lane: their loads go out together
    static_assert(!TABLE || (NT == corey_table::kLanes && U * NT * 8 <= corey_table::kRoundAdds && sizeof(T) == 2),
                  "a turn must stay inside the table's round");
    __shared__ uint32_t s_tab[TABLE ? corey_table::kWords : 1];
    __shared__ corey_table::Shared sh;
    corey_table::Workspace tws = {};
    if constexpr (TABLE) {
        tws = corey_table::carve(table_ws);
        corey_table::begin(s_tab, sh, tws);
    }
    constexpr int64_t kSeg = (int64_t)kThreads * V;
    const int64_t nseg = (L + kSeg - 1) / kSeg;
    const int64_t nfull = vector_ok ? L / kSeg : 0;           // segments of a row that are whole and aligned
    Stride st;
    st.nseg = nseg;
    st.D = D;
    st.q = (int64_t)gridDim.x / nseg;
    st.rem = (int64_t)gridDim.x - st.q * nseg;
    st.qd = st.q % D;
    Cursor cur;
    cur.row = (int64_t)blockIdx.x / nseg;
    cur.seg = (int64_t)blockIdx.x - cur.row * nseg;
    cur.d = cur.row % D;
    float lo = INFINITY, hi = -INFINITY;
    bool nan = false;

    while (cur.row < rows) {
        Cursor c[U];
        c[0] = cur;
        bool all_full = cur.seg < nfull;
#pragma unroll
        for (int j = 1; j < U; ++j) {
            c[j] = advance(c[j - 1], st);
            all_full = all_full && c[j].row < rows && c[j].seg < nfull;
        }
        cur = advance(c[U - 1], st);
        if (all_full) {                                       // uniform over the workgroup
            float xs[U][H + V], w[U][W], bs[U];
            word4 qc[U], qp[U];
#pragma unroll
            for (int j = 0; j < U; ++j) {                     // every load of these units before any use
                const T* xr = x + c[j].row * L;
                const int64_t t0 = c[j].seg * kSeg + (int64_t)threadIdx.x * V;
                qc[j] = *reinterpret_cast<const word4*>(xr + t0);
                qp[j] = *reinterpret_cast<const word4*>(xr + (t0 >= V ? t0 - V : 0));
#pragma unroll
                for (int k = 0; k < W; ++k) w[j][k] = weight[c[j].d * W + k];
                bs[j] = bias ? bias[c[j].d] : 0.f;
            }
#pragma unroll
            for (int j = 0; j < U; ++j) {
                T curv[V], prev[V];
                __builtin_memcpy(curv, &qc[j], 16);
                __builtin_memcpy(prev, &qp[j], 16);
#pragma unroll
                for (int e = 0; e < V; ++e) xs[j][H + e] = St<T>::widen(curv[e]);
#pragma unroll
                for (int k = 1; k <= H; ++k) xs[j][H - k] = St<T>::widen(prev[V - k]);
                if (c[j].seg == 0) {                          // the row starts in this unit: its first lane looks before t = 0
#pragma unroll
                    for (int k = 1; k <= H; ++k) {
                        float head = 0.f;
                        if (state_in && k <= W - 1) head = St<T>::widen(state_in[c[j].row * (W - 1) + (W - 1 - k)]);
                        xs[j][H - k] = (threadIdx.x == 0) ? head : xs[j][H - k];
                    }
                }
            }
#pragma unroll
            for (int j = 0; j < U; ++j) {
                T out[V];
                conv_vector<T, W, true>(xs[j], w[j], bs[j], V, out, lo, hi, nan);
                word4 q;
                __builtin_memcpy(&q, out, 16);
                // streaming store: u is written once and far exceeds the caches; leaving them to the loads measured 9 %
                // faster (5.4 against 4.9 TB/s, what a device copy reaches) with the next kernel's reads no slower
                __builtin_nontemporal_store(q, reinterpret_cast<word4*>(u + c[j].row * L + c[j].seg * kSeg + (int64_t)threadIdx.x * V));
                if constexpr (TABLE) table_add_vector<T>(s_tab, sh, out, V);
            }
            if constexpr (TABLE) __syncthreads();             // end of the table's round
            continue;
        }
#pragma unroll
        for (int j = 0; j < U; ++j) {                         // ragged or unaligned units, one at a time
            if (c[j].row >= rows) break;
            const int64_t t0 = c[j].seg * kSeg + (int64_t)threadIdx.x * V;
            if (t0 >= L) continue;
            const int nvalid = (L - t0 < V) ? (int)(L - t0) : V;
            float xs[H + V], w[W];
            load_inputs<T>(x + c[j].row * L, state_in ? state_in + c[j].row * (W - 1) : nullptr, t0, nvalid, W, vector_ok != 0, xs);
#pragma unroll
            for (int k = 0; k < W; ++k) w[k] = weight[c[j].d * W + k];
            T out[V];
            conv_vector<T, W, false>(xs, w, bias ? bias[c[j].d] : 0.f, nvalid, out, lo, hi, nan);
            T* ur = u + c[j].row * L + t0;
            if (vector_ok && nvalid == V) {
                word4 q;
                __builtin_memcpy(&q, out, 16);
                *reinterpret_cast<word4*>(ur) = q;
            } else {
#pragma unroll
                for (int e = 0; e < V; ++e)
                    if (e < nvalid) ur[e] = out[e];
            }
            if constexpr (TABLE) table_add_vector<T>(s_tab, sh, out, nvalid);
        }
        if constexpr (TABLE) __syncthreads();                 // end of the table's round (the loop condition is uniform)
    }
    if (lo <= hi) {                                           // the stored extremes: one rounding each
        float pad[V], two[V];
        T st[V];
#pragma unroll
        for (int e = 0; e < V; ++e) pad[e] = (e == 0) ? lo : hi;
        St<T>::narrow(pad, st);
        two[0] = St<T>::widen(st[0]);
        two[1] = St<T>::widen(st[1]);
        lo = two[0];
        hi = two[1];
    }

    if (state_out && W > 1) {                                 // the last W - 1 inputs of every row, oldest first
        const int64_t n = rows * (W - 1);
        for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < n; i += (int64_t)gridDim.x * kThreads) {
            const int64_t r = i / (W - 1);
            const int k = (int)(i - r * (W - 1));
            const int64_t t = L - (W - 1) + k;
            T v = T(0);
            if (t >= 0) v = x[r * L + t];
            else if (state_in) v = state_in[r * (W - 1) + (t + (W - 1))];
            state_out[i] = v;
        }
    }

    if (rparts || TABLE) {
        uint32_t klo = (lo <= hi) ? order_key(lo) : 0xffffffffu;
        uint32_t khi = (lo <= hi) ? order_key(hi) : 0u;
        uint32_t knan = nan ? 1u : 0u;
        if constexpr (TABLE) corey_table::end(s_tab, sh, tws, klo, khi, knan);     // also reduces the keys into thread 0
        else reduce_range_keys<NT>(klo, khi, knan);
        if (rparts && threadIdx.x == 0) {
            RangePart rp;
            rp.lo_key = klo; rp.hi_key = khi; rp.saw_nan = knan; rp.pad = 0u;
            rparts[blockIdx.x] = rp;
        }
        // entries no workgroup owns say "nothing seen"
        if (rparts && blockIdx.x == 0)
            for (int i = gridDim.x + threadIdx.x; i < COREY_RANGE_PARTS; i += kThreads) {
                RangePart rp;
                rp.lo_key = 0xffffffffu; rp.hi_key = 0u; rp.saw_nan = 0u; rp.pad = 0u;
                rparts[i] = rp;
            }
    }
}

// Sequences of a few steps (generation: L = 1 with the carried state): one lane per row instead of one workgroup
// per row segment.  A lane keeps the row's window of W - 1 earlier inputs in registers and walks its L steps.
constexpr int kShortL = 16;

template <typename T, int W>
__global__ __launch_bounds__(kThreads) void k_conv1d_silu_short(const T* __restrict__ x, const float* __restrict__ weight,
                                                                const float* __restrict__ bias, const T* __restrict__ state_in,
                                                                T* __restrict__ u, T* __restrict__ state_out,
                                                                Handoff* __restrict__ handoff, int64_t rows, int64_t D, int L)
{
    RangePart* rparts = handoff ? handoff->parts : nullptr;
    if (handoff) corey_range::clear_handoff_counts(handoff);
    float lo = INFINITY, hi = -INFINITY;
    bool nan = false;
    for (int64_t r = (int64_t)blockIdx.x * kThreads + threadIdx.x; r < rows; r += (int64_t)gridDim.x * kThreads) {
        const int64_t d = r % D;
        float w[W], win[W];                                   // win[k]: the input the tap w[k] multiplies at the current step
#pragma unroll
        for (int k = 0; k < W; ++k) w[k] = weight[d * W + k];
#pragma unroll
        for (int k = 0; k < W - 1; ++k) win[k + 1] = state_in ? St<T>::widen(state_in[r * (W - 1) + k]) : 0.f;
        const float bs = bias ? bias[d] : 0.f;
        T raw[W > 1 ? W - 1 : 1];                             // the stored form of the window, for state_out
#pragma unroll
        for (int k = 0; k < W - 1; ++k) raw[k] = state_in ? state_in[r * (W - 1) + k] : T(0);
        for (int t = 0; t < L; ++t) {
#pragma unroll
            for (int k = 0; k < W - 1; ++k) win[k] = win[k + 1];
#pragma unroll
            for (int k = 0; k + 1 < W - 1; ++k) raw[k] = raw[k + 1];
            const T xt = x[r * L + t];
            win[W - 1] = St<T>::widen(xt);
            if constexpr (W > 1) raw[W - 2] = xt;
            float acc = bs;
#pragma unroll
            for (int k = 0; k < W; ++k) acc = fmaf(w[k], win[k], acc);
            const float val = acc * __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(-acc * kLog2e));
            nan |= (val != val);
            lo = vmin(lo, val);
            hi = vmax(hi, val);
            float one[St<T>::kVec];
            T st[St<T>::kVec];
#pragma unroll
            for (int e = 0; e < St<T>::kVec; ++e) one[e] = val;
            St<T>::narrow(one, st);
            u[r * L + t] = st[0];
        }
        if (state_out)
#pragma unroll
            for (int k = 0; k < W - 1; ++k) state_out[r * (W - 1) + k] = raw[k];
    }
    if (lo <= hi) {                                           // the stored extremes: one rounding each
        float pad[St<T>::kVec];
        T st[St<T>::kVec];
#pragma unroll
        for (int e = 0; e < St<T>::kVec; ++e) pad[e] = (e == 0) ? lo : hi;
        St<T>::narrow(pad, st);
        lo = St<T>::widen(st[0]);
        hi = St<T>::widen(st[1]);
    }
    if (rparts) {
        uint32_t klo = (lo <= hi) ? order_key(lo) : 0xffffffffu;
        uint32_t khi = (lo <= hi) ? order_key(hi) : 0u;
        uint32_t knan = nan ? 1u : 0u;
        reduce_range_keys(klo, khi, knan);
        if (threadIdx.x == 0) {
            RangePart rp;
            rp.lo_key = klo; rp.hi_key = khi; rp.saw_nan = knan; rp.pad = 0u;
            rparts[blockIdx.x] = rp;
        }
        if (blockIdx.x == 0)                                  // entries no workgroup owns say "nothing seen"
            for (int i = gridDim.x + threadIdx.x; i < COREY_RANGE_PARTS; i += kThreads) {
                RangePart rp;
                rp.lo_key = 0xffffffffu; rp.hi_key = 0u; rp.saw_nan = 0u; rp.pad = 0u;
                rparts[i] = rp;
            }
    }
}

template <typename T>
void launch(const void* x, const float* weight, const float* bias, const void* state_in, void* u, void* state_out, void* rparts,
            void* table_ws, int64_t B, int64_t D, int64_t L, int W, hipStream_t stream)
{
    constexpr int V = St<T>::kVec;
    bool vector_ok = (L % V) == 0;
    for (const void* p : {x, (const void*)u})
        if (reinterpret_cast<uintptr_t>(p) % 16 != 0) vector_ok = false;
    const int64_t rows = B * D;
    if constexpr (sizeof(T) == 2) {
        if (table_ws) {                                       // one workgroup of 1024 lanes per compute unit, each with a table
            constexpr int NT = corey_table::kLanes;
            const int64_t seg = (int64_t)NT * V;
            int64_t blocks = rows * ((L + seg - 1) / seg);
            blocks = blocks < 1 ? 1 : (blocks > corey_table::kMaxSlabs ? corey_table::kMaxSlabs : blocks);
            auto go_table = [&](auto kernel) {
                kernel<<<dim3((unsigned)blocks), dim3(NT), 0, stream>>>(
                    static_cast<const T*>(x), weight, bias, static_cast<const T*>(state_in), static_cast<T*>(u), static_cast<T*>(state_out),
                    static_cast<Handoff*>(rparts), table_ws, rows, D, L, vector_ok ? 1 : 0);
            };
            switch (W) {
            case 1: go_table(k_conv1d_silu<T, 1, NT, true>); break;
            case 2: go_table(k_conv1d_silu<T, 2, NT, true>); break;
            case 3: go_table(k_conv1d_silu<T, 3, NT, true>); break;
            default: go_table(k_conv1d_silu<T, 4, NT, true>); break;
            }
            return;
        }
    }
    if (L <= kShortL) {
        int64_t nb = (rows + kThreads - 1) / kThreads;
        nb = nb > COREY_RANGE_PARTS ? COREY_RANGE_PARTS : nb;
        auto go_short = [&](auto kernel) {
            kernel<<<dim3((unsigned)nb), dim3(kThreads), 0, stream>>>(
                static_cast<const T*>(x), weight, bias, static_cast<const T*>(state_in), static_cast<T*>(u), static_cast<T*>(state_out),
                static_cast<Handoff*>(rparts), rows, D, (int)L);
        };
        switch (W) {
        case 1: go_short(k_conv1d_silu_short<T, 1>); break;
        case 2: go_short(k_conv1d_silu_short<T, 2>); break;
        case 3: go_short(k_conv1d_silu_short<T, 3>); break;
        default: go_short(k_conv1d_silu_short<T, 4>); break;
        }
        return;
    }
    const int64_t seg = (int64_t)kThreads * V;
    int64_t blocks = rows * ((L + seg - 1) / seg);
    blocks = blocks < 1 ? 1 : (blocks > COREY_RANGE_PARTS ? COREY_RANGE_PARTS : blocks);
    auto go = [&](auto kernel) {
        kernel<<<dim3((unsigned)blocks), dim3(kThreads), 0, stream>>>(
            static_cast<const T*>(x), weight, bias, static_cast<const T*>(state_in), static_cast<T*>(u), static_cast<T*>(state_out),
            static_cast<Handoff*>(rparts), nullptr, rows, D, L, vector_ok ? 1 : 0);
    };
    switch (W) {                                              // the tap count is a compile-time constant of the kernel
    case 1: go(k_conv1d_silu<T, 1, kThreads, false>); break;
    case 2: go(k_conv1d_silu<T, 2, kThreads, false>); break;
    case 3: go(k_conv1d_silu<T, 3, kThreads, false>); break;
    default: go(k_conv1d_silu<T, 4, kThreads, false>); break;
    }
}

}  // namespace

extern "C" int causal_conv1d_silu_fwd(const void* x, const float* weight, const float* bias, const void* state_in, void* u,
                                      void* state_out, void* range_parts, void* pattern_table, size_t pattern_table_bytes,
                                      corey_dtype dt, int64_t B, int64_t D, int64_t L, int32_t W, void* hip_stream)
{
    using corey::fail;
    if (!x || !weight || !u) return fail(COREY_ENULL, "causal_conv1d_silu_fwd: x, weight and u are required");
    if (dt != COREY_F32 && dt != COREY_BF16 && dt != COREY_F16) return fail(COREY_EINVAL, "causal_conv1d_silu_fwd: unknown dtype %d", (int)dt);
    if (W < 1 || W > COREY_MAX_CONV) return fail(COREY_EINVAL, "causal_conv1d_silu_fwd: W = %d outside [1, %d]", W, COREY_MAX_CONV);
    if (B < 1 || D < 1 || L < 1) return fail(COREY_ESHAPE, "causal_conv1d_silu_fwd: B, D, L must be >= 1");
    if ((double)B * (double)D * (double)L >= 4.0e18) return fail(COREY_ESHAPE, "causal_conv1d_silu_fwd: B*D*L overflows");
    if (x == u) return fail(COREY_EINVAL, "causal_conv1d_silu_fwd: u may not alias x");
    if (range_parts && reinterpret_cast<uintptr_t>(range_parts) % 16 != 0)
        return fail(COREY_EINVAL, "causal_conv1d_silu_fwd: range_parts must be 16-byte aligned");
    if (pattern_table) {
        if (dt == COREY_F32) return fail(COREY_EUNSUPPORTED, "causal_conv1d_silu_fwd: the bit-pattern table exists for 16-bit storage only");
        if (pattern_table_bytes < corey_table::kWorkspaceBytes || reinterpret_cast<uintptr_t>(pattern_table) % 256 != 0)
            return fail(COREY_EWORKSPACE, "causal_conv1d_silu_fwd: pattern_table needs %zu bytes, 256-byte aligned", corey_table::kWorkspaceBytes);
        if ((double)B * (double)D * (double)L >= 4294967296.0)
            return fail(COREY_ESHAPE, "causal_conv1d_silu_fwd: more than 2^32-1 values would overflow the table's 32-bit totals");
    }
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    if (dt == COREY_F32) launch<float>(x, weight, bias, state_in, u, state_out, range_parts, nullptr, B, D, L, W, stream);
    else if (dt == COREY_F16) launch<_Float16>(x, weight, bias, state_in, u, state_out, range_parts, pattern_table, B, D, L, W, stream);
    else launch<uint16_t>(x, weight, bias, state_in, u, state_out, range_parts, pattern_table, B, D, L, W, stream);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return corey::hip_fail(e, "causal_conv1d_silu_fwd launch");
    return COREY_OK;
}
