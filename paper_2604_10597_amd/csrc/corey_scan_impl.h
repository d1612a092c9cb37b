// Kernels of selective_scan_fwd (Mamba-1 selective-scan forward with a run-time chunk) for gfx950, as templates
// over the storage type.  Each storage type is instantiated in a translation unit of its own (corey_scan_f32.hip,
// corey_scan_bf16.hip, corey_scan_f16.hip) so that they compile in parallel; corey_scan.hip holds the host entry.
//
// Two kernels per call.
//
// k_relayout_bc   converts B and C ([B, N, L]) once to fp32 in the caller's workspace, tile by tile, in exactly
//                 the order the scan's lanes read them.  B and C are shared by every channel of a sequence, so
//                 doing this once per call removes all conversion work from the scan (a few MB of traffic against
//                 the scan's hundreds).
//
// k_scan          A workgroup of 256 lanes owns ROWS channels of one sequence and walks the time axis in tiles of
//                 CHUNK steps.  The tile geometry is a compile-time constant (one instantiation per chunk, chosen at
//                 launch from the run-time chunk), so every LDS address in the inner loop is an immediate offset.
//                 Inside a tile a row is spread over LPR = CHUNK / K consecutive lanes, each lane owning K (16, 8 or
//                 4) consecutive time steps: loads of u / delta / z and the store of y are one vector per lane (16 bytes
//                 or more; 8 for four 16-bit values), contiguous along L.  The fp32 B / C values of a few states at a time are copied from the
//                 workspace straight into LDS (global_load_lds, no registers), double buffered.  For every state
//                 index n a lane
//   1. discretises its K steps (a_i = exp2(dl_i A log2e), b_i = dl_i B_i u_i) and folds them, from a zero state,
//      into the pair (P, h) of the affine map  x -> P x + h  of its sub-block (P is one exp2 of the summed dl);
//      the first lane of the row also applies its map to the state carried from the previous tile;
//   2. takes part in an inclusive scan of the pairs across the lanes of the row (the pair operator is associative),
//      written as single DPP instructions; h then is the true state at the end of the lane's sub-block.  Rows
//      wider than a wave pass the wave totals through LDS;
//   3. receives the state entering its sub-block from the lane to its left, replays its K steps from it and
//      accumulates y_i += C_i h_i.
// The fp32 state carried from tile to tile lives in LDS; the last lane of a row refreshes it.
// The work is a recurrence plus elementwise maths: no matrix instructions.
#ifndef COREY_SCAN_IMPL_H
#define COREY_SCAN_IMPL_H

#include <hip/hip_runtime.h>

#include "corey_finalise.h"
#include "corey_internal.h"

namespace corey_scan {

using corey::bf16_to_f32;
using corey::f32_to_bf16;

#ifndef COREY_BLOCK
#define COREY_BLOCK 256
#endif
constexpr int kBlock = COREY_BLOCK;   // lanes per workgroup: four waves, one per SIMD of a compute unit
constexpr int kWaves = kBlock / 64;
// Build-time tuning knobs (defaults are the measured best on MI355X).
#ifndef COREY_STAGE_FLOATS_K16
#define COREY_STAGE_FLOATS_K16 2048   // fp32 values of B (and of C) per LDS staging buffer (two buffers), 16 steps per lane
#endif
#ifndef COREY_STAGE_FLOATS_K8
#define COREY_STAGE_FLOATS_K8 2048    // the same for 8 or 4 steps per lane
#endif
#ifndef COREY_WAVES_K16
#define COREY_WAVES_K16 4             // waves per SIMD the register allocation of the 16-step kernels leaves room for
#endif
#ifndef COREY_WAVES_K8
#define COREY_WAVES_K8 4              // the same for 8 or 4 steps per lane (the spare registers hold the tile fetched ahead)
#endif
#ifndef COREY_CPREFETCH_MAXK
#define COREY_CPREFETCH_MAXK 8        // geometries with at most this many steps per lane fetch C before the lane scan
#endif
#ifndef COREY_SPLIT_WAVES
#define COREY_SPLIT_WAVES 1536        // a launch with at most this many waves splits the states of a row between two rows
#endif
constexpr int kMaxGroup = 4;          // most states staged (and unrolled) per group
constexpr int kPad = COREY_MAX_CHUNK; // the relaid-out time axis is padded to whole tiles
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

typedef float float4v __attribute__((ext_vector_type(4)));
typedef float float2v __attribute__((ext_vector_type(2)));
typedef uint32_t uint4v __attribute__((ext_vector_type(4)));
typedef uint32_t uint2v __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

// Geometry of one (K, CHUNK) instantiation.
template <int K, int CHUNK> struct Geo {
    static_assert(CHUNK >= K && CHUNK / K <= kBlock, "a tile row must fit one workgroup");
    static constexpr int LPR = CHUNK / K;                       // lanes per row
    static constexpr int SEG = LPR < 64 ? LPR : 64;             // lanes of a row inside one wave
    static constexpr int WPR = LPR > 64 ? LPR / 64 : 1;         // waves per row
    static constexpr int ROWS = kBlock / LPR;                   // rows per workgroup
    static constexpr int kStageFloats = K < 16 ? COREY_STAGE_FLOATS_K8 : COREY_STAGE_FLOATS_K16;
    static constexpr int G = kStageFloats / CHUNK < 1 ? 1 : (kStageFloats / CHUNK > kMaxGroup ? kMaxGroup : kStageFloats / CHUNK);
    static_assert(kMaxGroup % G == 0, "the padded state count must be whole groups");
    static constexpr int STAGE = G * CHUNK;                     // floats per operand per staging buffer
};

// Time steps per lane, chosen per channel range.  16 steps halve the lane-scan work per value and stage B / C once for
// twice as many rows of a workgroup; 8 steps double the waves per row and need fewer registers.  Measured on channel
// counts 1024 ... 16384 at chunks 128 ... 512: while every row can have a wave of its own with all of them resident
// (four waves per SIMD: 4096 waves), 8 steps win.  Beyond that the fastest launch gives the channels below d16 sixteen
// steps, in whole layers of one workgroup per compute unit, and the remaining channels (less than one such layer)
// eight: the two kinds of workgroups then fill the SIMDs evenly (e.g. 5120 rows at chunk 512: 4096 rows as two
// 16-step waves per SIMD plus 1024 rows as one 8-step wave, 10 % faster than either geometry alone).
// plan_d16 returns d16: channels [0, d16) of every sequence take 16 steps per lane, [d16, D) take 8; 0 and D are the
// pure launches.  It runs on the host (known chunk) and on the device (chunk read from memory) with the same inputs.
__host__ __device__ inline int64_t plan_d16(int64_t B, int64_t D, int chunk, int rows_cap)
{
    if (chunk > 512) return D;                                   // a row of 8-step lanes would no longer fit one wave
    if (chunk < 128)                                             // 16-step rows would leave workgroup lanes idle here
        return (B * D * (chunk / 16) < 172032) ? 0 : D;
    const int64_t waves8 = B * D * (chunk / 8) / 64;
    if (waves8 <= 4096) return 0;
    int rows16 = kBlock * 16 / chunk;                            // rows of a 16-step workgroup
    rows16 = rows16 < rows_cap ? rows16 : rows_cap;
    const int64_t layer = (int64_t)256 * rows16 / B / 32 * 32;   // channels per sequence in one workgroup per compute unit
    if (layer < 32) return D;
    return D / layer * layer;
}

// Steps per lane of the channels that do not take 16 (all of them when d16 = 0): 8, or 4 when even 8-step rows leave
// most SIMDs without a wave (short tiles or few channels: a row is only chunk / 8 lanes wide).  Halving the steps doubles
// the lanes at the price of a longer lane scan per value.  Measured on 1024 ... 8192 channels at chunks 16 ... 512:
// 4 steps win by 10 ... 35 % while the 8-step launch has at most about 1500 waves (1.5 per SIMD) and a 4-step row still
// fits one wave (chunk <= 256); with 2 steps the lane scan costs more than the extra waves bring at chunks of 64 and up.
constexpr int64_t kFewWaves = 1536;
__host__ __device__ inline int plan_klo(int64_t B, int64_t D, int chunk, int64_t d16)
{
    if (d16 != 0 || chunk > 256) return 8;
    return B * D * (chunk / 8) / 64 <= kFewWaves ? 4 : 8;
}

// A launch of one kind of row that still leaves the SIMDs short of waves (small layers, short tiles) gives every channel
// TWO rows in the same workgroup, each with half of the states: twice the waves, each with half the per-state work and
// all of the per-token work, and one exchange of partial y per tile through LDS.  The staging group must hold at least
// one state of each half (tiles up to 1024 steps), and only the geometries such a launch can have are built.
constexpr int64_t kSplitWaves = COREY_SPLIT_WAVES;
template <int K, int CHUNK> constexpr bool split_exists()
{
    return (K == 16 && CHUNK == 1024) || (K == 8 && CHUNK == 512) || (K == 4 && CHUNK >= 4 && CHUNK <= 256);
}
__host__ __device__ inline int plan_split(int64_t B, int64_t D, int N, int chunk, int64_t d16, int klo, int allow)
{
    if (!allow || N < 4 || (d16 > 0 && d16 < D)) return 0;    // (fewer than four states: the second row would hold padding only)
    const int K = d16 >= D ? 16 : klo;
    if (!((K == 16 && chunk == 1024) || (K == 8 && chunk == 512) || (K == 4 && chunk <= 256))) return 0;
    const int lpr = chunk / K < 1 ? 1 : chunk / K;
    return B * D * lpr / 64 <= kSplitWaves ? 1 : 0;
}

// ------------------------------------------------------------------------------------------- storage types
// A lane keeps its K consecutive stored values as raw 16-byte words (Raw) and widens them when needed.
template <typename T> struct Io;
template <> struct Io<float> {
    static constexpr int kVec = 4;     // elements per 16-byte word
    static __device__ __forceinline__ float ld(const float* p) { return *p; }
    static __device__ __forceinline__ void st(float* p, float v) { *p = v; }
    static __device__ __forceinline__ void unpack(const uint4v& q, float* out)
    {
        out[0] = __uint_as_float(q.x); out[1] = __uint_as_float(q.y);
        out[2] = __uint_as_float(q.z); out[3] = __uint_as_float(q.w);
    }
    static __device__ __forceinline__ uint4v pack(const float* v)
    {
        uint4v q;
        q.x = __float_as_uint(v[0]); q.y = __float_as_uint(v[1]); q.z = __float_as_uint(v[2]); q.w = __float_as_uint(v[3]);
        return q;
    }
};
template <> struct Io<uint16_t> {                         // bfloat16 storage
    static constexpr int kVec = 8;
    static __device__ __forceinline__ float ld(const uint16_t* p) { return bf16_to_f32(*p); }
    static __device__ __forceinline__ void st(uint16_t* p, float v) { *p = f32_to_bf16(v); }
    static __device__ __forceinline__ void unpack(const uint4v& q, float* out)
    {
        const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            out[2 * k] = __uint_as_float(w[k] << 16);
            out[2 * k + 1] = __uint_as_float(w[k] & 0xffff0000u);
        }
    }
    // round to nearest even in hardware (v_cvt_pk_bf16_f32)
    static __device__ __forceinline__ uint32_t pack2(float lo, float hi)
    {
        float2v f;
        f.x = lo; f.y = hi;
        const bf16x2 h = __builtin_convertvector(f, bf16x2);
        uint32_t r;
        __builtin_memcpy(&r, &h, 4);
        return r;
    }
    static __device__ __forceinline__ uint4v pack(const float* v)
    {
        uint4v q;
        q.x = pack2(v[0], v[1]); q.y = pack2(v[2], v[3]); q.z = pack2(v[4], v[5]); q.w = pack2(v[6], v[7]);
        return q;
    }
};
template <> struct Io<_Float16> {                         // IEEE binary16 storage
    static constexpr int kVec = 8;
    typedef _Float16 h2 __attribute__((ext_vector_type(2)));
    static __device__ __forceinline__ float ld(const _Float16* p) { return (float)*p; }
    static __device__ __forceinline__ void st(_Float16* p, float v) { *p = (_Float16)v; }
    static __device__ __forceinline__ void unpack(const uint4v& q, float* out)
    {
        const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            h2 h;
            __builtin_memcpy(&h, &w[k], 4);
            out[2 * k] = (float)h.x;
            out[2 * k + 1] = (float)h.y;
        }
    }
    static __device__ __forceinline__ uint32_t pack2(float lo, float hi)    // round to nearest even
    {
        float2v f;
        f.x = lo; f.y = hi;
        const h2 h = __builtin_convertvector(f, h2);
        uint32_t r;
        __builtin_memcpy(&r, &h, 4);
        return r;
    }
    static __device__ __forceinline__ uint4v pack(const float* v)
    {
        uint4v q;
        q.x = pack2(v[0], v[1]); q.y = pack2(v[2], v[3]); q.z = pack2(v[4], v[5]); q.w = pack2(v[6], v[7]);
        return q;
    }
};

template <typename T, int K> struct Raw {
    static constexpr int kBytes = K * (int)sizeof(T);           // 4 or 8 (short runs: one load), else whole 16-byte words
    static constexpr int kWords = kBytes / 16 > 0 ? kBytes / 16 : 1;
    uint4v w[kWords];                                          // a short run uses the first kBytes of w[0]
};

// K consecutive stored values starting at p (the first nvalid exist); missing ones read as zero bits.
template <typename T, int K>
__device__ __forceinline__ Raw<T, K> load_raw(const T* p, int nvalid, bool vector_ok)
{
    constexpr int V = Io<T>::kVec;
    Raw<T, K> r;
    if constexpr (Raw<T, K>::kBytes < 16) {                    // 2 or 4 values of a 16-bit type, 2 of binary32
        r.w[0] = uint4v{0u, 0u, 0u, 0u};
        if (vector_ok && nvalid == K) {
            if constexpr (Raw<T, K>::kBytes == 8) {
                const uint2v q = *reinterpret_cast<const uint2v*>(p);
                r.w[0].x = q.x;
                r.w[0].y = q.y;
            } else {
                r.w[0].x = *reinterpret_cast<const uint32_t*>(p);
            }
        } else {
            T tmp[V];
#pragma unroll
            for (int i = 0; i < V; ++i) tmp[i] = (i < K && i < nvalid) ? p[i < K ? i : 0] : T(0);
            __builtin_memcpy(&r.w[0], tmp, 16);
        }
    } else if (vector_ok && nvalid == K) {
        const uint4v* pv = reinterpret_cast<const uint4v*>(p);
#pragma unroll
        for (int v = 0; v < Raw<T, K>::kWords; ++v) r.w[v] = pv[v];
    } else {
        T tmp[K];
#pragma unroll
        for (int i = 0; i < K; ++i) tmp[i] = (i < nvalid) ? p[i] : T(0);
#pragma unroll
        for (int v = 0; v < Raw<T, K>::kWords; ++v) __builtin_memcpy(&r.w[v], &tmp[v * V], 16);
    }
    return r;
}

template <typename T, int K>
__device__ __forceinline__ void widen(const Raw<T, K>& r, float (&out)[K])
{
    if constexpr (Raw<T, K>::kBytes < 16) {
        float all[Io<T>::kVec];
        Io<T>::unpack(r.w[0], all);
#pragma unroll
        for (int i = 0; i < K; ++i) out[i] = all[i];
    } else {
#pragma unroll
        for (int v = 0; v < Raw<T, K>::kWords; ++v) Io<T>::unpack(r.w[v], &out[v * Io<T>::kVec]);
    }
}

template <typename T, int K>
__device__ __forceinline__ void store_items(T* p, int nstore, bool vector_ok, const float (&v)[K])
{
    constexpr int V = Io<T>::kVec;
    if constexpr (Raw<T, K>::kBytes < 16) {
        if (vector_ok && nstore == K) {
            float all[V];
#pragma unroll
            for (int i = 0; i < V; ++i) all[i] = i < K ? v[i < K ? i : 0] : 0.f;
            const uint4v q = Io<T>::pack(all);
            if constexpr (Raw<T, K>::kBytes == 8) {
                uint2v o;
                o.x = q.x;
                o.y = q.y;
                *reinterpret_cast<uint2v*>(p) = o;
            } else {
                *reinterpret_cast<uint32_t*>(p) = q.x;
            }
        } else {
#pragma unroll
            for (int i = 0; i < K; ++i)
                if (i < nstore) Io<T>::st(p + i, v[i]);
        }
    } else if (vector_ok && nstore == K) {
        uint4v* pv = reinterpret_cast<uint4v*>(p);
#pragma unroll
        for (int k = 0; k < K / V; ++k) pv[k] = Io<T>::pack(&v[k * V]);
    } else {
#pragma unroll
        for (int i = 0; i < K; ++i)
            if (i < nstore) Io<T>::st(p + i, v[i]);
    }
}

// ------------------------------------------------------------------------------------------- elementwise maths
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// log(1 + e^x) = max(x, 0) + log1p(e^{-|x|}).  log1p(e) is taken as log(w), w = fl(1 + e), plus the repair
// e - (w - 1) of the rounding in w (its 1/w factor lies in [1/2, 1] and the repair is below one ulp of w, so
// dropping the factor costs < 3e-8 absolute): the small tail e << 1 stays accurate to binary32 relative precision.
__device__ __forceinline__ float softplus(float x)
{
    const float e = fast_exp2(-fabsf(x) * kLog2e);
    const float w = 1.f + e;
    const float fix = e - (w - 1.f);
    float pos;                                             // max(x, 0) in one instruction: fmaxf would first quiet a signalling
    asm("v_max_f32_e32 %0, 0, %1" : "=v"(pos) : "v"(x));   // NaN with a second one, which x (a sum) cannot be
    return pos + fmaf(__builtin_amdgcn_logf(w), kLn2, fix);
}

// z * sigmoid(z)
__device__ __forceinline__ float silu(float z)
{
    return z * __builtin_amdgcn_rcpf(1.f + fast_exp2(-z * kLog2e));
}

// ------------------------------------------------------------------------------------------- lane scan (DPP)
// Inclusive scan, over the SEG consecutive lanes of a row inside one wave, of the per-lane affine maps
// x -> P x + h (oldest lane first): a Hillis-Steele scan whose steps are single DPP instructions,
//     h += h[lane - s] * P ;  P *= P[lane - s] ;
// lanes without a source (DPP bound control off) keep their value, which is composing with the identity.
// The instructions are written out because the hazard rules matter: a DPP source register needs two wait
// states after the VALU write that produced it (inside a step pair: the other instruction plus s_nop 0), and
// five after a VALU write of EXEC (s_nop 4 up front).  With NEED_P false the last step leaves P stale
// (only h is wanted afterwards).
#define COREY_DPP_H(ctrl) "v_fmac_f32_dpp %0, %0, %1 " ctrl " bank_mask:0xf\n\t"
#define COREY_DPP_P(ctrl) "v_mul_f32_dpp %1, %1, %1 " ctrl " bank_mask:0xf\n\t"
#define COREY_DPP_STEP(ctrl) COREY_DPP_H(ctrl) COREY_DPP_P(ctrl) "s_nop 0\n\t"
#define COREY_ROW_STEPS3                                                                   \
    COREY_DPP_STEP("row_shr:1 row_mask:0xf") COREY_DPP_STEP("row_shr:2 row_mask:0xf")      \
    COREY_DPP_STEP("row_shr:4 row_mask:0xf")

template <int CTRL>
__device__ __forceinline__ float dpp_move(float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, true));
}

template <int SEG, bool NEED_P>
__device__ __forceinline__ void scan_inclusive(int jseg, float& P, float& h)
{
    if constexpr (SEG == 64) {
        if constexpr (NEED_P)
            asm volatile("s_nop 4\n\t" COREY_ROW_STEPS3 COREY_DPP_STEP("row_shr:8 row_mask:0xf")
                         COREY_DPP_STEP("row_bcast:15 row_mask:0xa") COREY_DPP_STEP("row_bcast:31 row_mask:0xc")
                         : "+v"(h), "+v"(P));
        else
            asm volatile("s_nop 4\n\t" COREY_ROW_STEPS3 COREY_DPP_STEP("row_shr:8 row_mask:0xf")
                         COREY_DPP_STEP("row_bcast:15 row_mask:0xa") COREY_DPP_H("row_bcast:31 row_mask:0xc") "s_nop 1\n\t"
                         : "+v"(h), "+v"(P));
    } else if constexpr (SEG == 32) {
        asm volatile("s_nop 4\n\t" COREY_ROW_STEPS3 COREY_DPP_STEP("row_shr:8 row_mask:0xf")
                     COREY_DPP_H("row_bcast:15 row_mask:0xa") "s_nop 1\n\t" : "+v"(h), "+v"(P));
    } else if constexpr (SEG == 16) {
        asm volatile("s_nop 4\n\t" COREY_ROW_STEPS3 COREY_DPP_H("row_shr:8 row_mask:0xf") "s_nop 1\n\t" : "+v"(h), "+v"(P));
    } else if constexpr (SEG > 1) {
        // segments shorter than a DPP row: the shifted-in partner must come from the same segment
        {
            const float ho = dpp_move<0x111>(h), Po = dpp_move<0x111>(P);        // row_shr:1
            const bool take = jseg >= 1;
            h = take ? fmaf(P, ho, h) : h;
            P = take ? P * Po : P;
        }
        if constexpr (SEG > 2) {
            const float ho = dpp_move<0x112>(h), Po = dpp_move<0x112>(P);        // row_shr:2
            const bool take = jseg >= 2;
            h = take ? fmaf(P, ho, h) : h;
            P = take ? P * Po : P;
        }
        if constexpr (SEG > 4) {
            const float ho = dpp_move<0x114>(h), Po = dpp_move<0x114>(P);        // row_shr:4
            const bool take = jseg >= 4;
            h = take ? fmaf(P, ho, h) : h;
            P = take ? P * Po : P;
        }
    }
}

// The value of the lane to the left inside the wave (lane 0 keeps `first`).
__device__ __forceinline__ float from_left_lane(float v, float first)
{
    float r = first;
    asm volatile("s_nop 1\n\tv_mov_b32_dpp %0, %1 wave_shr:1 row_mask:0xf bank_mask:0xf\n\ts_nop 0" : "+v"(r) : "v"(v));
    return r;
}

// The value of the lane to the left inside a segment of SEG = 16 or 32 lanes (segments start at multiples of SEG); the
// first lane of every segment keeps `first`.  DPP rows are 16 lanes: a shift by one inside every row leaves the rows'
// first lanes alone, and for 32-lane segments the odd rows' first lanes (16, 48) take the last lane of the row before
// them first (row_bcast:15 on rows 1 and 3, limited by the bank mask to lanes 0..3 of the row, of which 1..3 are
// overwritten by the shift that follows).
template <int SEG>
__device__ __forceinline__ float from_left_in_segment(float v, float first)
{
    static_assert(SEG == 16 || SEG == 32, "segments of one or two DPP rows");
    float r = first;
    if constexpr (SEG == 32)
        asm volatile("s_nop 1\n\tv_mov_b32_dpp %0, %1 row_bcast:15 row_mask:0xa bank_mask:0x1\n\t"
                     "v_mov_b32_dpp %0, %1 row_shr:1 row_mask:0xf bank_mask:0xf\n\ts_nop 0" : "+v"(r) : "v"(v));
    else
        asm volatile("s_nop 1\n\tv_mov_b32_dpp %0, %1 row_shr:1 row_mask:0xf bank_mask:0xf\n\ts_nop 0" : "+v"(r) : "v"(v));
    return r;
}

// ------------------------------------------------------------------------------------------- kernel arguments
struct ScanArgs {
    const void* u;
    const void* delta;
    const float* A;
    const void* Bm;
    const void* Cm;
    const float* Dv;
    const void* z;
    const float* dbias;
    const float* h0;
    const int32_t* seqlens;
    const int32_t* chunks_dev;
    void* y;
    float* last_state;
    float* ws_B;            // relaid-out fp32 B, [B][N * Lpad]
    float* ws_C;
    float* ws_B8;           // the same operands in the order of the 8- or 4-step rows of this launch (ws_B / ws_C: the 16-step ones)
    float* ws_C8;
    int64_t d16;            // channels below d16 take 16 steps per lane, the others klo (host chunk; see plan_d16)
    int32_t klo;            // 8 or 4 (host chunk; see plan_klo)
    int32_t split;          // the states of a channel are shared by two rows (host chunk; see plan_split)
    int32_t allow_split;    // 0: every channel keeps one row whatever the size of the launch
    int64_t L, Lpad;
    int64_t rows_total;     // B * D (input of the items-per-lane rule)
    int32_t D, N;
    int32_t Np;             // N rounded up to whole staging groups (a multiple of 4); states N..Np-1 are zero padding
    int32_t chunk;          // host chunk (also the fallback for invalid device entries)
    int32_t rows_cap;       // most rows a workgroup may hold (LDS budget for the carried state)
    int32_t softplus;
    int32_t allow_structured;   // take the power-chain path when A[d, n] = (n + 1) A[d, 0] (16-bit storage only)
    int32_t vector_ok;      // rows of the [.., L] tensors are 16-byte aligned
    int32_t one_chunk;      // chunks_dev holds a single entry that applies to every sequence
    corey_finalise::Args route;   // route.parts != NULL: the statistic's reduction and the chunk rule run at the start of this call
};

__device__ __forceinline__ int resolve_chunk(const ScanArgs& a, int b)
{
    int chunk = a.chunk;
    if (a.chunks_dev) {
        const int c = a.chunks_dev[a.one_chunk ? 0 : b];
        if (c >= COREY_MIN_CHUNK && c <= COREY_MAX_CHUNK && (c & (c - 1)) == 0) chunk = c;
    }
    return chunk;
}

// Workspace layout of one operand for sequence b, chunk c (lpr = c / K lanes per row): value (n, t) of tile
// tau = t / c lives at   b*N*Lpad + tau*N*c + ((n*(K/4) + q) * lpr + j) * 4 + e,   t - tau*c = j*K + q*4 + e.
// For a fixed quarter q of a lane's K steps consecutive lanes j read consecutive 16-byte words, the values
// of one state are c consecutive floats and a group of states of one tile is one contiguous block, so a
// workgroup stages it with straight 16-byte copies.  Steps at or beyond the sequence length are written as 0, and so
// are the padding states N..Np-1 (N here is the padded count Np): with B = C = 0 they contribute nothing.
template <typename T>
__global__ __launch_bounds__(256) void k_relayout_bc(const T* __restrict__ Bm, const T* __restrict__ Cm, float* __restrict__ ws_B,
                                                     float* __restrict__ ws_C, float* __restrict__ ws_B8, float* __restrict__ ws_C8,
                                                     const int32_t* __restrict__ seqlens, const int32_t* __restrict__ chunks_dev,
                                                     int one_chunk, int chunk_host, int64_t d16_host, int klo_host, int64_t Bn, int64_t D, int rows_cap,
                                                     int Nreal, int N, int64_t L, int64_t Lpad, corey_finalise::Args route)
{
    const int b = blockIdx.y;
    int chunk = chunk_host;
    int64_t d16 = d16_host;
    int klo = klo_host;
    if (route.parts) {
        // the end of the entropy statistic, left to this kernel: every workgroup reduces the partial histograms of its
        // sequence's statistic and applies the chunk rule (all arrive at the same chunk); the first one publishes counts, H,
        // r and the chunk, which is where the scan kernel that follows reads it.  The partial histograms are read by all
        // workgroups here, so clearing them for the next call is left to that scan kernel.
        route.rezero = 0;
        const bool first = blockIdx.x == 0 && (route.nh > 1 || b == 0);
        const int c = corey_finalise::finalise(route, route.nh > 1 ? b : 0, first);
        if (c >= COREY_MIN_CHUNK && c <= COREY_MAX_CHUNK && (c & (c - 1)) == 0) chunk = c;
        d16 = plan_d16(Bn, D, chunk, rows_cap);
        klo = plan_klo(Bn, D, chunk, d16);
    } else if (chunks_dev) {
        const int c = chunks_dev[one_chunk ? 0 : b];
        if (c >= COREY_MIN_CHUNK && c <= COREY_MAX_CHUNK && (c & (c - 1)) == 0) chunk = c;
        d16 = plan_d16(Bn, D, chunk, rows_cap);
        klo = plan_klo(Bn, D, chunk, d16);
    }
    int64_t len = L;
    if (seqlens) {
        const int64_t sl = seqlens[b];
        len = sl < 0 ? 0 : (sl > L ? L : sl);
    }
    const int slots_log2 = __ffs(chunk / 4) - 1;                 // 16-byte slots per (tile, state)
    const int64_t ntiles = (len + chunk - 1) / chunk;            // tiles the scan will actually visit
    const int64_t total = (ntiles * N) << slots_log2;
    const T* Bs = Bm + (int64_t)b * Nreal * L;
    const T* Cs = Cm + (int64_t)b * Nreal * L;
    struct alignas(4 * sizeof(T)) Quad { T v[4]; };
    // t is always a multiple of 4: rows of whole, aligned quads can be fetched four values at a time
    const bool quads_ok = L % 4 == 0 && reinterpret_cast<uintptr_t>(Bm) % sizeof(Quad) == 0 && reinterpret_cast<uintptr_t>(Cm) % sizeof(Quad) == 0;
    for (int pass = 0; pass < 2; ++pass) {                       // the order of the 16-step rows, then that of the others
        const int K = pass == 0 ? 16 : (klo == 8 ? 8 : 4);       // 4 or fewer steps per lane read B / C in time order
        if (pass == 0 ? d16 <= 0 : d16 >= D) continue;           // no channel of this sequence uses it
        if (chunk < K) continue;
        const int lpr = chunk / K;
        const int lpr_log2 = __ffs(lpr) - 1;
        float4v* oB = reinterpret_cast<float4v*>((pass == 0 ? ws_B : ws_B8) + (int64_t)b * N * Lpad);
        float4v* oC = reinterpret_cast<float4v*>((pass == 0 ? ws_C : ws_C8) + (int64_t)b * N * Lpad);
        for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
            const int slot = (int)(i & ((1 << slots_log2) - 1));
            const int64_t tn = i >> slots_log2;                  // tau * N + n
            const int64_t tau = tn / N;
            const int n = (int)(tn - tau * N);
            const int j = slot & (lpr - 1);
            const int q = slot >> lpr_log2;
            const int64_t t = n < Nreal ? tau * chunk + (int64_t)j * K + q * 4 : len;     // padding states read nothing
            const T* pb = Bs + (int64_t)n * L + t;
            const T* pc = Cs + (int64_t)n * L + t;
            float4v vb, vc;
            if (quads_ok && t + 4 <= len) {                      // four values of each operand in one load
                Quad qb, qc;
                __builtin_memcpy(&qb, __builtin_assume_aligned(pb, sizeof(Quad)), sizeof(Quad));
                __builtin_memcpy(&qc, __builtin_assume_aligned(pc, sizeof(Quad)), sizeof(Quad));
                vb.x = Io<T>::ld(&qb.v[0]); vb.y = Io<T>::ld(&qb.v[1]); vb.z = Io<T>::ld(&qb.v[2]); vb.w = Io<T>::ld(&qb.v[3]);
                vc.x = Io<T>::ld(&qc.v[0]); vc.y = Io<T>::ld(&qc.v[1]); vc.z = Io<T>::ld(&qc.v[2]); vc.w = Io<T>::ld(&qc.v[3]);
            } else {
                vb.x = (t + 0 < len) ? Io<T>::ld(pb + 0) : 0.f; vb.y = (t + 1 < len) ? Io<T>::ld(pb + 1) : 0.f;
                vb.z = (t + 2 < len) ? Io<T>::ld(pb + 2) : 0.f; vb.w = (t + 3 < len) ? Io<T>::ld(pb + 3) : 0.f;
                vc.x = (t + 0 < len) ? Io<T>::ld(pc + 0) : 0.f; vc.y = (t + 1 < len) ? Io<T>::ld(pc + 1) : 0.f;
                vc.z = (t + 2 < len) ? Io<T>::ld(pc + 2) : 0.f; vc.w = (t + 3 < len) ? Io<T>::ld(pc + 3) : 0.f;
            }
            oB[i] = vb;
            oC[i] = vc;
        }
    }
}

// Start the copy of NFLOAT consecutive floats (a multiple of 4) of each operand from the workspace into an LDS
// staging buffer.  Every wave copies 64 sixteen-byte words per instruction; the words go from global memory to
// LDS without passing through registers and are complete when the wave's vmcnt reaches zero.
template <int NFLOAT, bool SCALAR_BASE>
__device__ __forceinline__ void stage_async(const float* __restrict__ srcB, const float* __restrict__ srcC, float* dstB,
                                            float* dstC, int wave, int lane)
{
    constexpr int SLOTS = NFLOAT / 4;
#pragma unroll
    for (int s0 = 0; s0 < SLOTS; s0 += kBlock) {
        const int s = s0 + wave * 64;
        if (SLOTS % kBlock == 0 || s + lane < SLOTS) {
            // uniform base + 32-bit lane offset in bytes
            uint32_t voff = (uint32_t)(s + lane) * 16u;
            // SCALAR_BASE: the empty asm keeps the offset from being widened to 64 bits outside the tile loop, so that the
            // copy uses its scalar-base addressing mode; otherwise the compiler adds base and offset with one vector
            // instruction per copy.  Long tiles stage few states per group and gain from it (chunk 1024: -7 %, 2048:
            // -5 % on 5120 channels); at chunk 512 and below the other schedule measured 1 % faster.
            if constexpr (SCALAR_BASE) asm volatile("" : "+v"(voff));
            __builtin_amdgcn_global_load_lds(reinterpret_cast<const char*>(srcB) + voff, dstB + (size_t)s * 4, 16, 0, 0);
            __builtin_amdgcn_global_load_lds(reinterpret_cast<const char*>(srcC) + voff, dstC + (size_t)s * 4, 16, 0, 0);
        }
    }
}

// Floats of dynamic LDS one workgroup of the (K, CHUNK) geometry needs for `rows` rows of N states.
template <int K, int CHUNK>
__host__ __device__ constexpr int lds_floats(int rows, int N, bool split = false)
{
    // N: padded state count; a split launch adds the partial y of the rows that hold the second half of the states
    return 4 * Geo<K, CHUNK>::STAGE + 2 * rows * N + N + 4 * kWaves + kBlock + N + (split ? kBlock / 2 * K : 0);
}

// ------------------------------------------------------------------------------------------- the scan
// The rows d0 .. d0 + rows - 1 of sequence blockIdx.y, start to end.
//
// STRUCT: every row of the group has A[d, n] = (n + 1) A[d, 0] (the S4D-real initialisation Mamba starts from, and
// the benchmark's A = -(n + 1)).  Then exp(dl A[d, n]) = exp(dl A[d, 0])^(n + 1): one exponential per time step
// instead of one per (time step, state), the decay of state n following from that of state n - 1 by one multiply
// (likewise the sub-block product P).  The chain adds at most n roundings (about (n + 1) 2^-24 relative) to a decay.
//
// SPLIT: a channel has two rows of the workgroup (neighbours), the first with states [0, N/2), the second with
// [N/2, N); `rows` counts channels.  Both do the per-token work; the second hands its partial y to the first through
// LDS at the end of every tile, and the first adds the skip term, gates and stores.
template <typename T, int K, int CHUNK, bool STRUCT, bool SPLIT>
__device__ __forceinline__ void scan_group(const ScanArgs& a, float* s_mem, const int rows, const int d0)
{
    using Gm = Geo<K, CHUNK>;
    constexpr int LPR = Gm::LPR, SEG = Gm::SEG, WPR = Gm::WPR, G = Gm::G, STAGE = Gm::STAGE;
    constexpr int NS = SPLIT ? 2 : 1;                       // rows per channel
    constexpr int GH = G / NS;                              // states of one row per staging group
    static_assert(!SPLIT || (G >= 2 && WPR == 1 && Gm::ROWS >= 2), "a split row needs a state of its own in every staging group");
    constexpr int E = K < 4 ? K : 4;                        // staged B / C values a lane reads per LDS instruction
    constexpr int KQ = K / E;
    typedef float BCv __attribute__((ext_vector_type(E)));

    const int b = blockIdx.y;
    const int tid = threadIdx.x;
    const int row_local = tid / LPR;
    const int j = tid % LPR;                                // sub-block of this lane inside the tile
    const int ch_local = SPLIT ? row_local >> 1 : row_local; // channel of this lane inside the group
    const int half = SPLIT ? row_local & 1 : 0;             // which half of the states its row holds
    const int d = d0 + ch_local;
    const bool active = ch_local < rows && d < a.D;
    const int rl = active ? ch_local : 0;                   // safe LDS row for idle lanes
    const int N = a.Np;                                     // padded state count: whole staging groups, no tail group
    const int NH = N / NS;                                  // states per row (N is a multiple of 4: whole half-groups)
    const int n_first = half * NH;                          // first state of this lane's row
    const int Nreal = a.N;
    const int64_t L = a.L;
    int64_t len = L;
    if (a.seqlens) {
        const int64_t s = a.seqlens[b];
        len = s < 0 ? 0 : (s > L ? L : s);
    }

    float* s_stage = s_mem;                                 // [2 buffers][B, C][STAGE] staged fp32 operands
    float* s_carry = s_stage + 4 * STAGE;                   // [rows][N] state carried tile to tile
    float* s_A2 = s_carry + rows * N;                       // [rows][N] A * log2(e)
    float* s_zero = s_A2 + rows * N;                        // [N] zeros: the "carried state" of lanes that are not first in their row
    float* s_xchg = s_zero + N;                             // [2][kWaves][2] wave totals when a row spans several waves
    float* s_sink = s_xchg + 4 * kWaves;                    // [kBlock + N] where lanes that are not last in their row "store" the state
    float* s_ypart = s_sink + kBlock + N;                   // SPLIT: [K][kBlock / 2] partial y of the second rows
    for (int i = tid; i < rows * N; i += kBlock) {
        const int r = i / N, n = i - r * N;
        const int dd = d0 + r;
        const bool ok = dd < a.D && n < Nreal;
        s_carry[i] = (a.h0 && ok) ? a.h0[((int64_t)b * a.D + dd) * Nreal + n] : 0.f;
        s_A2[i] = ok ? a.A[(int64_t)dd * Nreal + n] * kLog2e : 0.f;
    }
    for (int i = tid; i < N; i += kBlock) s_zero[i] = 0.f;
    __syncthreads();                                        // the first tile reads A before any other barrier (STRUCT)

    // u, delta, z and y are addressed as a base that is uniform over the workgroup (the group's first row; it lives in
    // scalar registers and advances by a tile per iteration) plus ONE 32-bit byte offset per lane that never changes
    // (the lane's row inside the group and its sub-block inside a tile): four 64-bit pointers per lane would not fit the
    // register budget of the 16-step geometries.  The host limits the rows of a group so that the offset fits 32 bits.
    const int64_t row0 = ((int64_t)b * a.D + d0) * L;
    const T* u_grp = static_cast<const T*>(a.u) + row0;
    const T* dl_grp = static_cast<const T*>(a.delta) + row0;
    const T* z_grp = a.z ? static_cast<const T*>(a.z) + row0 : nullptr;
    T* y_grp = static_cast<T*>(a.y) + row0;
    const uint32_t lane_off = (uint32_t)(((int64_t)rl * L + (int64_t)j * K) * (int64_t)sizeof(T));
    auto at = [lane_off](const T* uniform_base) __attribute__((always_inline)) {
        return reinterpret_cast<const T*>(reinterpret_cast<const char*>(uniform_base) + lane_off);
    };
    const bool z_on = z_grp != nullptr;
    const float* wsB = (K < 16 ? a.ws_B8 : a.ws_B) + (int64_t)b * N * a.Lpad;    // each kind of row has its own order of B / C
    const float* wsC = (K < 16 ? a.ws_C8 : a.ws_C) + (int64_t)b * N * a.Lpad;
    const float bias = (a.dbias && active) ? a.dbias[d] : 0.f;
    const float Dd = (a.Dv && active && half == 0) ? a.Dv[d] : 0.f;      // the skip term enters once per channel
    const bool vec = a.vector_ok != 0;
    const bool sp = a.softplus != 0;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);    // uniform: addresses built from it stay in scalar registers
    const int jseg = lane & (SEG - 1);
    const int wpos = wave & (WPR - 1);                      // this wave's position inside its row
    // per-state arrays are indexed with the state's number inside the row: the row's first state is folded into the bases
    const float* A2_row = s_A2 + rl * N + n_first;
    const float* carry_rd = ((active && j == 0) ? s_carry + rl * N : s_zero) + n_first;
    // every lane stores its end-of-sub-block state each step (no branch in the inner loop): the row's last lane into
    // the carried state, all others into a scratch slot of their own
    float* carry_wr = (active && j == LPR - 1) ? s_carry + rl * N + n_first : s_sink + tid;
    // staging: one block of GH states per row kind and operand, [half][GH][CHUNK]
    auto stage_group = [&](const int64_t tau_s, const int n_s, float* dst) __attribute__((always_inline)) {
        constexpr bool kScalarBase = CHUNK >= 1024;
#pragma unroll
        for (int hs = 0; hs < NS; ++hs) {
            const int64_t off = (tau_s * N + hs * NH + n_s) * CHUNK;
            stage_async<GH * CHUNK, kScalarBase>(wsB + off, wsC + off, dst + hs * GH * CHUNK, dst + STAGE + hs * GH * CHUNK, wave, lane);
        }
    };

    int buf = 0;                                            // staging buffer holding the group about to be used
    if (len > 0) stage_group(0, 0, s_stage);

    // Geometries with at most 8 steps per lane have the registers to fetch the next tile's u / delta / z while the last
    // group of states of the current tile is computed, which takes the HBM latency out of every tile's start.
    constexpr bool kTileAhead = K <= 8;
    Raw<T, K> u_nx, d_nx, z_nx;
    bool have_nx = false;                                   // uniform over the workgroup
    const int64_t ntiles = (len + CHUNK - 1) / CHUNK;
    for (int64_t tau = 0; tau < ntiles; ++tau) {
        const int64_t tile = tau * CHUNK;
        const int64_t t0 = tile + (int64_t)j * K;
        // A full tile lies inside the sequence with aligned rows: no masks anywhere (idle lanes read row d0).
        const bool full = vec && tile + CHUNK <= len;       // uniform over the workgroup
        // otherwise: valid steps of this lane (within the sequence) and steps that get a y written (within L)
        int nvalid = K, nstore = K;
        if (!full) {
            nvalid = nstore = 0;
            if (active) {
                nvalid = (t0 >= len) ? 0 : (len - t0 < K ? (int)(len - t0) : K);
                nstore = (t0 >= L) ? 0 : (L - t0 < K ? (int)(L - t0) : K);
            }
        }
        float dl[K], du[K], yv[K];
        Raw<T, K> z_raw;                                    // the gate is fetched with the tile and used after the last state
        if (kTileAhead && have_nx) {                        // a full tile fetched one tile ago
            z_raw = z_nx;
            widen<T, K>(d_nx, dl);
            widen<T, K>(u_nx, du);
        } else {
            const Raw<T, K> u_raw = load_raw<T, K>(at(u_grp + tile), nvalid, vec);
            const Raw<T, K> d_raw = load_raw<T, K>(at(dl_grp + tile), nvalid, vec);
            if (z_on) z_raw = load_raw<T, K>(at(z_grp + tile), nvalid, vec);
            widen<T, K>(d_raw, dl);
            widen<T, K>(u_raw, du);
        }
        have_nx = false;
        float S = 0.f;
#pragma unroll
        for (int i = 0; i < K; ++i) dl[i] = dl[i] + bias;
        if (sp) {
#pragma unroll
            for (int i = 0; i < K; ++i) dl[i] = softplus(dl[i]);
        }
        if (!full) {
#pragma unroll
            for (int i = 0; i < K; ++i) dl[i] = (i < nvalid) ? dl[i] : 0.f;   // padded steps: dl = 0 -> a = 1, b = 0 (identity)
        }
#pragma unroll
        for (int i = 0; i < K; ++i) {
            yv[i] = Dd * du[i];                             // the skip term D u opens the sum over states
            du[i] = dl[i] * du[i];
            S += dl[i];
        }
        float av_chain[K], P_chain = 1.f, P_base = 1.f;      // STRUCT: decay of the current state, built up state by state
        if constexpr (STRUCT) {
            const float A20 = s_A2[rl * N];
#pragma unroll
            for (int i = 0; i < K; ++i) {
                // a row that starts at state n_first starts its chain at the decay of state 0 to the power n_first
                av_chain[i] = SPLIT ? fast_exp2(dl[i] * A20 * (float)n_first) : 1.f;
                dl[i] = fast_exp2(dl[i] * A20);             // from here on dl holds the decay of state 0
            }
            P_base = fast_exp2(S * A20);
            if constexpr (SPLIT) P_chain = fast_exp2(S * A20 * (float)n_first);
        }

        for (int n0 = 0; n0 < NH; n0 += GH) {                 // n0: number inside the row of the group's first state
            const float* s_B = s_stage + buf * 2 * STAGE;
            const float* s_C = s_B + STAGE;
            // this group's copy (started one group earlier) has landed; every wave is past the previous group
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __syncthreads();
            {   // start the copy of the next group: same tile, or the first group of the next tile
                int nn0 = n0 + GH;
                int64_t ntau = tau;
                if (nn0 >= NH) { nn0 = 0; ntau = tau + 1; }
                if (ntau < ntiles) stage_group(ntau, nn0, s_stage + (buf ^ 1) * 2 * STAGE);
                if constexpr (kTileAhead) {                 // last group of this tile: fetch the next tile if it is a full one
                    if (nn0 == 0 && vec && tile + 2 * CHUNK <= len) {
                        u_nx = load_raw<T, K>(at(u_grp + tile + CHUNK), K, true);
                        d_nx = load_raw<T, K>(at(dl_grp + tile + CHUNK), K, true);
                        if (z_on) z_nx = load_raw<T, K>(at(z_grp + tile + CHUNK), K, true);
                        have_nx = true;
                    }
                }
            }
            buf ^= 1;
            const BCv* bq0 = reinterpret_cast<const BCv*>(s_B + half * GH * CHUNK) + j;
            const BCv* cq0 = reinterpret_cast<const BCv*>(s_C + half * GH * CHUNK) + j;
            constexpr bool kEarlyC = K <= COREY_CPREFETCH_MAXK;   // C is requested before the lane scan, which covers the LDS latency
            auto one_state = [&](const int nl, const int n) __attribute__((always_inline)) {
                const float cin = carry_rd[n];              // carried state for the first lane of the row, 0 elsewhere
                const BCv* bq = bq0 + nl * KQ * LPR;
                const BCv* cq = cq0 + nl * KQ * LPR;
                float A2 = 0.f;
                if constexpr (!STRUCT) A2 = A2_row[n];

                float av_local[K], bv[K];
                float (&av)[K] = STRUCT ? av_chain : av_local;
                float h = 0.f, P;
                if constexpr (STRUCT) {
#pragma unroll
                    for (int q = 0; q < KQ; ++q) {
                        const BCv b4 = bq[q * LPR];
#pragma unroll
                        for (int e = 0; e < E; ++e) {
                            const int i = E * q + e;
                            av[i] *= dl[i];                 // decay of state n from that of state n - 1
                            bv[i] = du[i] * b4[e];
                            h = i == 0 ? bv[i] : fmaf(av[i], h, bv[i]);
                        }
                    }
                    P_chain *= P_base;
                    P = P_chain;
                } else {
#pragma unroll
                    for (int q = 0; q < KQ; ++q) {
                        const BCv b4 = bq[q * LPR];
#pragma unroll
                        for (int e = 0; e < E; ++e) {
                            const int i = E * q + e;
                            av[i] = fast_exp2(dl[i] * A2);
                            bv[i] = du[i] * b4[e];
                            h = i == 0 ? bv[i] : fmaf(av[i], h, bv[i]);      // the fold starts from a zero state
                        }
                    }
                    P = fast_exp2(S * A2);
                }
                BCv cv[KQ];
                if constexpr (kEarlyC) {
#pragma unroll
                    for (int q = 0; q < KQ; ++q) cv[q] = cq[q * LPR];
                }
                h = fmaf(P, cin, h);                        // the row's first lane starts from the carried state
                scan_inclusive<SEG, (WPR > 1)>(jseg, P, h); // h: state at the end of this lane's sub-block (within the wave)
                float first = cin;                          // state entering the first lane of this wave's part of the row
                if constexpr (WPR > 1) {                    // a row spans several waves: add what the waves before it did
                    float* xc = s_xchg + (n & 1) * (2 * kWaves);
                    if (lane == 63) { xc[2 * wave] = P; xc[2 * wave + 1] = h; }
                    __syncthreads();
                    float hw = 0.f;                         // state at the end of the wave to the left
                    for (int w = 0; w < wpos; ++w) hw = fmaf(xc[2 * (wave - wpos + w)], hw, xc[2 * (wave - wpos + w) + 1]);
                    h = fmaf(P, hw, h);
                    if (wpos > 0) first = hw;
                }
                carry_wr[n] = h;
                float hh;                                   // true state entering this lane's sub-block
                if constexpr (LPR == 1) {
                    hh = cin;
                } else if constexpr (SEG == 16 || SEG == 32) {
                    hh = from_left_in_segment<SEG>(h, cin);  // a row inside one wave: its first lane enters with the carried state
                } else {
                    hh = from_left_lane(h, first);
                    if constexpr (SEG < 64) hh = (jseg == 0) ? cin : hh;
                }
#pragma unroll
                for (int q = 0; q < KQ; ++q) {
                    const BCv c4 = kEarlyC ? cv[q] : cq[q * LPR];
#pragma unroll
                    for (int e = 0; e < E; ++e) {
                        const int i = E * q + e;
                        hh = fmaf(av[i], hh, bv[i]);
                        yv[i] = fmaf(c4[e], hh, yv[i]);
                    }
                }
            };
#pragma unroll
            for (int nl = 0; nl < GH; ++nl) one_state(nl, n0 + nl);      // straight-line code for the whole group
        }

        if constexpr (SPLIT) {                              // the second row of a channel hands over its part of the sum over states
            float* yp = s_ypart + ch_local * LPR + j;
            if (half == 1 && active) {
#pragma unroll
                for (int i = 0; i < K; ++i) yp[i * (kBlock / 2)] = yv[i];
            }
            __syncthreads();                                // (the next tile's barriers separate these reads from its writes)
            if (half == 0 && active) {
#pragma unroll
                for (int i = 0; i < K; ++i) yv[i] += yp[i * (kBlock / 2)];
            }
        }
        const bool writer = active && half == 0;            // the row that gates and stores y

        T* y_lane = const_cast<T*>(at(y_grp + tile));
        if (full) {
            if (!SPLIT || writer) {
                if (z_on) {
                    float zz[K];
                    widen<T, K>(z_raw, zz);
#pragma unroll
                    for (int i = 0; i < K; ++i) yv[i] *= silu(zz[i]);
                }
                if (active) store_items<T, K>(y_lane, K, true, yv);
            }
        } else if (nstore > 0 && (!SPLIT || writer)) {
            if (nvalid > 0 && z_on) {
                float zz[K];
                widen<T, K>(z_raw, zz);
#pragma unroll
                for (int i = 0; i < K; ++i) yv[i] *= silu(zz[i]);
            }
#pragma unroll
            for (int i = 0; i < K; ++i)
                if (i >= nvalid) yv[i] = 0.f;                // padded positions are written as zero
            store_items<T, K>(y_lane, nstore, vec, yv);
        }
    }

    // tiles wholly beyond the sequence: y is written as zero
    if (active && half == 0) {
        float zero[K];
#pragma unroll
        for (int i = 0; i < K; ++i) zero[i] = 0.f;
        for (int64_t tile = ntiles * CHUNK; tile < L; tile += CHUNK) {
            const int64_t t0 = tile + (int64_t)j * K;
            const int nstore = (t0 >= L) ? 0 : (L - t0 < K ? (int)(L - t0) : K);
            if (nstore > 0) store_items<T, K>(const_cast<T*>(at(y_grp + tile)), nstore, vec, zero);
        }
    }
    __syncthreads();                                         // last writes of the carried state are visible

    for (int i = tid; i < rows * N; i += kBlock) {
        const int r = i / N, n = i - r * N;
        const int dd = d0 + r;
        if (dd < a.D && n < Nreal) a.last_state[((int64_t)b * a.D + dd) * Nreal + n] = s_carry[i];
    }
}

// A workgroup takes groups of `rows` rows of its sequence, grid-stride.  A launch whose grid was sized from the
// run-time chunk gives every workgroup exactly one group; a launch that reads the chunk from device memory sizes
// its grid from the host's hint and is correct for any chunk (more groups than workgroups: some take several in
// turn; fewer: the surplus leaves at once).
template <typename T, int K, int CHUNK, bool SPLIT = false>
__device__ __forceinline__ void scan_rows(const ScanArgs& a, float* s_mem, const int64_t d_first, const int64_t d_end,
                                          const int64_t wg, const int64_t nwg)
{
    constexpr int kChannels = Geo<K, CHUNK>::ROWS / (SPLIT ? 2 : 1);                  // channels of a full group
    const int rows_full = kChannels < a.rows_cap ? kChannels : a.rows_cap;
    for (int64_t d0 = d_first + wg * rows_full; d0 < d_end; d0 += nwg * rows_full) {   // uniform over the workgroup
        const int rows = d_end - d0 < rows_full ? (int)(d_end - d0) : rows_full;     // the range's last group may be short
        bool structured = false;
        if constexpr (sizeof(T) == 2) {                      // fp32 storage keeps the one-exponential-per-state path
            if (a.allow_structured) {
                int ok = 1;
                for (int i = threadIdx.x; i < rows * a.N; i += kBlock) {
                    const int r = i / a.N, n = i - r * a.N;
                    const int64_t dd = d0 + r;
                    if (dd < a.D) ok &= a.A[dd * a.N + n] == (float)(n + 1) * a.A[dd * a.N];
                }
                structured = __syncthreads_and(ok) != 0;
            }
        }
        if (structured) scan_group<T, K, CHUNK, true, SPLIT>(a, s_mem, rows, (int)d0);
        else scan_group<T, K, CHUNK, false, SPLIT>(a, s_mem, rows, (int)d0);
        __syncthreads();                                     // the LDS arrays are set up afresh for the next group
    }
}

// Register budget: K = 16 keeps 16 x (dl, du, y, a, b) per lane and is built for four waves per SIMD (128 VGPRs), and
// so are the shorter lanes (their spare registers hold the tile fetched ahead).
template <int K> constexpr int waves_target() { return K < 16 ? COREY_WAVES_K8 : COREY_WAVES_K16; }

// One geometry, chosen on the host from the run-time chunk.
template <typename T, int K, int CHUNK>
__global__ __launch_bounds__(kBlock) __attribute__((amdgpu_waves_per_eu(waves_target<K>()))) void k_scan(const ScanArgs a)
{
    extern __shared__ float s_mem[];
    if constexpr (split_exists<K, CHUNK>()) {
        if (a.split) {
            scan_rows<T, K, CHUNK, true>(a, s_mem, 0, a.D, blockIdx.x, gridDim.x);
            return;
        }
    }
    scan_rows<T, K, CHUNK>(a, s_mem, 0, a.D, blockIdx.x, gridDim.x);
}

// Workgroup `wg` of `nwg` takes its share of one sequence's channels: those below d16 with 16 steps per lane (the first
// g16 workgroups), the others with 8.  With a grid sized for exactly these two kinds every workgroup has one row group;
// any other grid is still correct (row groups are taken grid-stride within each kind).
template <int K, int CHUNK> constexpr bool geometry_exists()
{
    return CHUNK >= K && (K == 16 || (K == 8 && CHUNK <= 512) || (K == 4 && CHUNK <= 256));
}

template <int CHUNK> __host__ __device__ inline int rows_of(int K, int rows_cap, int split = 0)
{
    const int lpr = CHUNK / K < 1 ? 1 : CHUNK / K;
    const int rows = kBlock / lpr / (split ? 2 : 1);        // channels of a workgroup
    return rows < rows_cap ? rows : rows_cap;
}

template <typename T, int CHUNK>
__device__ __forceinline__ void scan_by_kind(const ScanArgs& a, float* s_mem, const int64_t d16, const int klo, const int split)
{
    if (split) {                                                 // one kind of row, two rows per channel
        if (d16 >= a.D) {
            if constexpr (split_exists<16, CHUNK>()) scan_rows<T, 16, CHUNK, true>(a, s_mem, 0, a.D, blockIdx.x, gridDim.x);
        } else if (klo == 8) {
            if constexpr (split_exists<8, CHUNK>()) scan_rows<T, 8, CHUNK, true>(a, s_mem, 0, a.D, blockIdx.x, gridDim.x);
        } else {
            if constexpr (split_exists<4, CHUNK>()) scan_rows<T, 4, CHUNK, true>(a, s_mem, 0, a.D, blockIdx.x, gridDim.x);
        }
        return;
    }
    const int rows16 = rows_of<CHUNK>(16, a.rows_cap);
    const int64_t n16 = (d16 + rows16 - 1) / rows16;
    const int64_t nwg = gridDim.x;
    if constexpr (CHUNK <= 512) {
        const int rows8 = rows_of<CHUNK>(klo, a.rows_cap);
        const int64_t n8 = (a.D - d16 + rows8 - 1) / rows8;
        int64_t g16 = n16;                                       // workgroups of the 16-step kind
        if (n16 + n8 != nwg) {                                   // a grid sized for another chunk: share it in proportion
            g16 = n8 == 0 ? nwg : (n16 == 0 ? 0 : (nwg * n16 + (n16 + n8) / 2) / (n16 + n8));
            if (n16 > 0 && g16 < 1) g16 = 1;
            if (n8 > 0 && g16 > nwg - 1) g16 = nwg - 1;
        }
        const int64_t wg = (int64_t)blockIdx.x - g16;
        if ((int64_t)blockIdx.x < g16) {
            if constexpr (geometry_exists<16, CHUNK>()) scan_rows<T, 16, CHUNK>(a, s_mem, 0, d16, blockIdx.x, g16);
        } else if (klo == 8) {
            if constexpr (geometry_exists<8, CHUNK>()) scan_rows<T, 8, CHUNK>(a, s_mem, d16, a.D, wg, nwg - g16);
        } else {
            if constexpr (geometry_exists<4, CHUNK>()) scan_rows<T, 4, CHUNK>(a, s_mem, d16, a.D, wg, nwg - g16);
        }
    } else {
        scan_rows<T, 16, CHUNK>(a, s_mem, 0, a.D, blockIdx.x, nwg);
    }
}

// Both kinds of workgroups in one launch (host chunk, 0 < d16 < D).
template <typename T, int CHUNK>
__global__ __launch_bounds__(kBlock) __attribute__((amdgpu_waves_per_eu(COREY_WAVES_K16))) void k_scan_mix(const ScanArgs a)
{
    extern __shared__ float s_mem[];
    scan_by_kind<T, CHUNK>(a, s_mem, a.d16, a.klo, 0);
}

// Per-sequence chunk read from device memory: every geometry in one kernel, selected per workgroup (register budget
// of the 16-step geometries).
template <typename T>
__global__ __launch_bounds__(kBlock) __attribute__((amdgpu_waves_per_eu(COREY_WAVES_K16))) void k_scan_any(const ScanArgs a)
{
    extern __shared__ float s_mem[];
    const int chunk = resolve_chunk(a, blockIdx.y);
    if (a.route.parts && a.route.rezero && blockIdx.x == 0 && blockIdx.y == 0) {
        // the statistic's partial histograms live in the buffer its producer handed over and have been reduced by the kernel
        // before this one: leave them cleared for the next count sweep, which adds into them without a clearing launch
        const int n = a.route.nh * corey_range::kParts * a.route.K;
        for (int i = threadIdx.x; i < n; i += kBlock) a.route.parts[i] = 0u;
    }
    const int64_t d16 = plan_d16(gridDim.y, a.D, chunk, a.rows_cap);
    const int klo = plan_klo(gridDim.y, a.D, chunk, d16);
    const int split = plan_split(gridDim.y, a.D, a.N, chunk, d16, klo, a.allow_split);
#define COREY_CASE(C)                                                                       \
    case C:                                                                                 \
        scan_by_kind<T, C>(a, s_mem, d16, klo, split);                                      \
        break;
    switch (chunk) {
        COREY_CASE(16) COREY_CASE(32) COREY_CASE(64) COREY_CASE(128) COREY_CASE(256) COREY_CASE(512) COREY_CASE(1024)
        COREY_CASE(2048)
    default: break;
    }
#undef COREY_CASE
}

// ------------------------------------------------------------------------------------------- launch
struct LaunchPlan {
    int chunk;              // host chunk
    bool routed;            // per-sequence device chunks
    int64_t B, D, N;
    hipStream_t stream;
};

inline int a_np(int64_t N) { return (int)((N + kMaxGroup - 1) / kMaxGroup * kMaxGroup); }

template <int K, int CHUNK>
inline void geometry(int64_t nrows, int64_t N, int rows_cap, int split, int64_t& gx, size_t& lds)
{
    gx = 0;
    lds = 0;
    if constexpr (geometry_exists<K, CHUNK>()) {
        const int full = Geo<K, CHUNK>::ROWS / (split ? 2 : 1);
        int rows = full < rows_cap ? full : rows_cap;
        gx = (nrows + rows - 1) / rows;
        lds = (size_t)lds_floats<K, CHUNK>(rows, a_np(N), split != 0) * sizeof(float);
    }
}

// Grid and LDS of a launch whose channels below d16 take 16 steps per lane and the others klo.
template <int CHUNK>
inline void launch_geometry(const LaunchPlan& p, int rows_cap, int64_t d16, int klo, int split, int64_t& gx, size_t& lds)
{
    gx = 0;
    lds = 0;
    int64_t g = 0;
    size_t l = 0;
    if (d16 > 0) {
        geometry<16, CHUNK>(d16, p.N, rows_cap, split, g, l);
        gx += g;
        lds = l > lds ? l : lds;
    }
    if (d16 < p.D) {
        if (klo == 8) geometry<8, CHUNK>(p.D - d16, p.N, rows_cap, split, g, l);
        else geometry<4, CHUNK>(p.D - d16, p.N, rows_cap, split, g, l);
        gx += g;
        lds = l > lds ? l : lds;
    }
}

template <typename T>
inline void launch_scan(const ScanArgs& a, const LaunchPlan& p)
{
    // relayout of B and C: one 16-byte word per lane, enough workgroups to cover the operand a few times over
    int64_t rb = (a.Np * a.Lpad / 4 + 255) / 256;
    rb = rb < 1 ? 1 : (rb > 2048 ? 2048 : rb);
    k_relayout_bc<T><<<dim3((unsigned)rb, (unsigned)p.B), dim3(256), 0, p.stream>>>(
        static_cast<const T*>(a.Bm), static_cast<const T*>(a.Cm), a.ws_B, a.ws_C, a.ws_B8, a.ws_C8, a.seqlens, a.chunks_dev,
        a.one_chunk, p.chunk, a.d16, a.klo, p.B, p.D, a.rows_cap, (int)p.N, a.Np, a.L, a.Lpad, a.route);
    int64_t gx = 0, g;
    size_t lds = 0, l;
    if (p.routed) {
        // grid from the host's chunk (the caller's hint: workgroups take row groups grid-stride, so any grid is correct),
        // LDS for the largest need of any geometry the device-side plan can pick
#define COREY_GEO(C)                                                                        \
        {                                                                                   \
            const int64_t d16_c = plan_d16(p.B, p.D, C, a.rows_cap);                        \
            const int klo_c = plan_klo(p.B, p.D, C, d16_c);                                 \
            launch_geometry<C>(p, a.rows_cap, d16_c, klo_c, plan_split(p.B, p.D, (int)p.N, C, d16_c, klo_c, a.allow_split), g, l);    \
        }                                                                                   \
        lds = l > lds ? l : lds;                                                            \
        if (C == p.chunk) gx = g;
        COREY_GEO(16) COREY_GEO(32) COREY_GEO(64) COREY_GEO(128) COREY_GEO(256) COREY_GEO(512) COREY_GEO(1024) COREY_GEO(2048)
#undef COREY_GEO
        if (gx < 2) gx = 2;     // two kinds of rows decided on the device need a workgroup for each kind (a surplus one leaves at once)
        k_scan_any<T><<<dim3((unsigned)gx, (unsigned)p.B), dim3(kBlock), lds, p.stream>>>(a);
        return;
    }
#define COREY_LAUNCH(K, C)                                                                  \
    if constexpr (geometry_exists<K, C>())                                                  \
        k_scan<T, K, C><<<dim3((unsigned)gx, (unsigned)p.B), dim3(kBlock), lds, p.stream>>>(a)
#define COREY_CASE(C)                                                                       \
    case C:                                                                                 \
        launch_geometry<C>(p, a.rows_cap, a.d16, a.klo, a.split, gx, lds);                   \
        if (a.d16 >= p.D) { COREY_LAUNCH(16, C); }                                          \
        else if constexpr (C <= 512) {                                                      \
            if (a.d16 > 0) k_scan_mix<T, C><<<dim3((unsigned)gx, (unsigned)p.B), dim3(kBlock), lds, p.stream>>>(a);                 \
            else if (a.klo == 8) { COREY_LAUNCH(8, C); }                                    \
            else { COREY_LAUNCH(4, C); }                                                    \
        }                                                                                   \
        break;
    switch (p.chunk) {
        COREY_CASE(16) COREY_CASE(32) COREY_CASE(64) COREY_CASE(128) COREY_CASE(256) COREY_CASE(512) COREY_CASE(1024)
        COREY_CASE(2048)
    default: break;
    }
#undef COREY_CASE
#undef COREY_LAUNCH
}

}  // namespace corey_scan
#endif
