// selective_scan_fwd: Mamba-1 selective-scan forward with a run-time chunk on gfx950.
//
// Two kernels per call.
//
// k_relayout_bc   converts B and C ([B, N, L], bf16 or fp32) once to fp32 in the caller's workspace, tile by
//                 tile, in exactly the order the scan's lanes read them.  B and C are shared by every channel of
//                 a sequence, so doing this once per call instead of once per workgroup removes all conversion
//                 work from the scan (a few MB of traffic against the scan's hundreds).
//
// k_selective_scan   A workgroup of 256 lanes owns `rows` channels of one sequence and walks the time axis in
//                 tiles of `chunk` steps.  Inside a tile a row is spread over chunk/K consecutive lanes, each lane
//                 owning K (16 or 8) consecutive time steps, so loads of u/delta/z and the store of y are
//                 contiguous along L (16-byte vectors per lane).  The fp32 B/C values of a few states at a time
//                 are copied from the workspace straight into LDS (global_load_lds, no registers), double
//                 buffered: the copy for the next group of states is in flight while the current one is
//                 computed.  For every state index n a lane
//   1. discretises its K steps (a_i = exp2(dl_i A log2e), b_i = dl_i B_i u_i) and folds them, from a zero
//      state, into the pair (P, h) that represents the affine map  x -> P x + h  of its sub-block
//      (P itself comes from one exp2 of the summed dl);
//   2. obtains the composition of all pairs to its left in the row by a DPP scan across lanes (the pair
//      operator is associative); rows wider than a wave cross the wave boundary through LDS;
//   3. replays its K steps from the true incoming state (prefix pair applied to the state carried from
//      the previous tile) and accumulates y_i += C_i h_i.
// The fp32 state carried from tile to tile lives in LDS; the last lane of a row refreshes it.
// The work is a recurrence plus elementwise maths: no matrix instructions.
#include <hip/hip_runtime.h>

#include "corey_internal.h"

namespace {

using corey::bf16_to_f32;
using corey::f32_to_bf16;

constexpr int kMaxBlock = 256;    // lanes per workgroup: four waves, one per SIMD of a compute unit (workgroups whose
                                  // wave count is not a multiple of four were measured to place badly)
constexpr int kMaxWaves = kMaxBlock / 64;
constexpr int kStageElems = 2048; // fp32 values of B (and of C) per LDS staging buffer (two buffers)
// waves per SIMD the register allocation must leave room for: K = 16 needs about 156 VGPRs, K = 8 about 95
// (a four-wave target for K = 16 was measured: it spills a little and is slower at the routed chunk)
template <int K> constexpr int min_waves() { return K == 8 ? 5 : 3; }
constexpr int kPad = COREY_MAX_CHUNK;  // the relaid-out time axis is padded to whole tiles
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

typedef float float4v __attribute__((ext_vector_type(4)));
typedef float float2v __attribute__((ext_vector_type(2)));
typedef uint32_t uint4v __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

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
template <> struct Io<uint16_t> {
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
    static constexpr int kWords = K / Io<T>::kVec;
    uint4v w[kWords];
};

// K consecutive stored values starting at p (the first nvalid exist); missing ones read as zero bits.
template <typename T, int K>
__device__ __forceinline__ Raw<T, K> load_raw(const T* p, int nvalid, bool vector_ok)
{
    constexpr int V = Io<T>::kVec;
    Raw<T, K> r;
    if (vector_ok && nvalid == K) {
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
#pragma unroll
    for (int v = 0; v < Raw<T, K>::kWords; ++v) Io<T>::unpack(r.w[v], &out[v * Io<T>::kVec]);
}

template <typename T, int K>
__device__ __forceinline__ void store_items(T* p, int nstore, bool vector_ok, const float (&v)[K])
{
    constexpr int V = Io<T>::kVec;
    if (vector_ok && nstore == K) {
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
    return fmaxf(x, 0.f) + fmaf(__builtin_amdgcn_logf(w), kLn2, fix);
}

// z * sigmoid(z)
__device__ __forceinline__ float silu(float z)
{
    return z * __builtin_amdgcn_rcpf(1.f + fast_exp2(-z * kLog2e));
}

// ------------------------------------------------------------------------------------------- lane scan (DPP)
// Exclusive prefix, over the `seg` consecutive lanes of a row inside one wave, of the per-lane affine maps
// x -> P x + h: on return (P, h) is the composition of the maps of all lanes to the left (identity for the
// first lane of a segment).  The pairs are first moved one lane to the right, then combined by a
// Hillis-Steele scan whose steps are single DPP instructions:  h += h[lane - s] * P ;  P *= P[lane - s];
// lanes without a source (DPP bound control off) keep their value, which is composing with the identity.
// The instructions are written out because the hazard rules matter: a DPP source register needs two wait
// states after the VALU write that produced it (here: one other instruction plus s_nop 0), and five after a
// VALU write of EXEC (s_nop 4 up front).
#define COREY_DPP_STEP(ctrl)                                                               \
    "s_nop 0\n\tv_fmac_f32_dpp %0, %0, %1 " ctrl " bank_mask:0xf\n\t"                      \
    "s_nop 0\n\tv_mul_f32_dpp %1, %1, %1 " ctrl " bank_mask:0xf\n\t"
#define COREY_ROW_STEPS                                                                    \
    COREY_DPP_STEP("row_shr:1 row_mask:0xf") COREY_DPP_STEP("row_shr:2 row_mask:0xf")      \
    COREY_DPP_STEP("row_shr:4 row_mask:0xf") COREY_DPP_STEP("row_shr:8 row_mask:0xf")

__device__ __forceinline__ void exclusive_scan_pairs(int seg, int jseg, float& P, float& h)
{
    float hs = 0.f, Ps = 1.f;
    asm volatile("s_nop 4\n\t"
                 "v_mov_b32_dpp %0, %2 wave_shr:1 row_mask:0xf bank_mask:0xf\n\t"
                 "v_mov_b32_dpp %1, %3 wave_shr:1 row_mask:0xf bank_mask:0xf\n\t"
                 : "+v"(hs), "+v"(Ps)
                 : "v"(h), "v"(P));
    if (jseg == 0) { hs = 0.f; Ps = 1.f; }
    h = hs;
    P = Ps;
    if (seg == 64) {
        asm volatile("s_nop 4\n\t" COREY_ROW_STEPS COREY_DPP_STEP("row_bcast:15 row_mask:0xa")
                     COREY_DPP_STEP("row_bcast:31 row_mask:0xc") : "+v"(h), "+v"(P));
    } else if (seg == 32) {
        asm volatile("s_nop 4\n\t" COREY_ROW_STEPS COREY_DPP_STEP("row_bcast:15 row_mask:0xa") : "+v"(h), "+v"(P));
    } else if (seg == 16) {
        asm volatile("s_nop 4\n\t" COREY_ROW_STEPS : "+v"(h), "+v"(P));
    } else if (seg > 1) {
        // segments shorter than a DPP row: the shifted-in partner must come from the same segment
        for (int off = 1; off < seg; off <<= 1) {
            float ho = 0.f, Po = 1.f;
            if (off == 1)
                asm volatile("s_nop 4\n\tv_mov_b32_dpp %0, %2 row_shr:1 row_mask:0xf bank_mask:0xf\n\t"
                             "v_mov_b32_dpp %1, %3 row_shr:1 row_mask:0xf bank_mask:0xf\n\t" : "+v"(ho), "+v"(Po) : "v"(h), "v"(P));
            else if (off == 2)
                asm volatile("s_nop 4\n\tv_mov_b32_dpp %0, %2 row_shr:2 row_mask:0xf bank_mask:0xf\n\t"
                             "v_mov_b32_dpp %1, %3 row_shr:2 row_mask:0xf bank_mask:0xf\n\t" : "+v"(ho), "+v"(Po) : "v"(h), "v"(P));
            else
                asm volatile("s_nop 4\n\tv_mov_b32_dpp %0, %2 row_shr:4 row_mask:0xf bank_mask:0xf\n\t"
                             "v_mov_b32_dpp %1, %3 row_shr:4 row_mask:0xf bank_mask:0xf\n\t" : "+v"(ho), "+v"(Po) : "v"(h), "v"(P));
            const bool take = jseg >= off;
            ho = take ? ho : 0.f;
            Po = take ? Po : 1.f;
            h = fmaf(P, ho, h);
            P = P * Po;
        }
    }
}

// ------------------------------------------------------------------------------------------- kernel
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
    int64_t L, Lpad;
    int32_t D, N;
    int32_t chunk;          // host chunk (also the fallback for invalid device entries)
    int32_t rows_cap;       // most rows a workgroup may hold (LDS budget for the carried state)
    int32_t rows_alloc;     // rows the LDS arrays are sized for
    int32_t softplus;
    int32_t vector_ok;      // rows of the [.., L] tensors are 16-byte aligned
};

// Workspace layout of one operand for sequence b, chunk c (lpr = c / K lanes per row): value (n, t) of tile
// tau = t / c lives at   b*N*Lpad + tau*N*c + ((n*(K/4) + q) * lpr + j) * 4 + e,   t - tau*c = j*K + q*4 + e.
// For a fixed quarter q of a lane's K steps consecutive lanes j read consecutive 16-byte words, the values
// of one state are c consecutive floats and a group of states of one tile is one contiguous block, so a
// workgroup stages it with straight 16-byte copies.  Steps at or beyond the sequence length are written as 0.
template <typename T, int K>
__global__ __launch_bounds__(256) void k_relayout_bc(const T* __restrict__ Bm, const T* __restrict__ Cm, float* __restrict__ ws_B,
                                                     float* __restrict__ ws_C, const int32_t* __restrict__ seqlens,
                                                     const int32_t* __restrict__ chunks_dev, int chunk_host, int N, int64_t L,
                                                     int64_t Lpad)
{
    const int b = blockIdx.y;
    int chunk = chunk_host;
    if (chunks_dev) {
        const int c = chunks_dev[b];
        if (c >= COREY_MIN_CHUNK && c <= COREY_MAX_CHUNK && (c & (c - 1)) == 0) chunk = c;
    }
    int64_t len = L;
    if (seqlens) {
        const int64_t sl = seqlens[b];
        len = sl < 0 ? 0 : (sl > L ? L : sl);
    }
    const int lpr = chunk / K;
    const int slots_log2 = __ffs(chunk / 4) - 1;                 // 16-byte slots per (tile, state)
    const int lpr_log2 = __ffs(lpr) - 1;
    const int64_t ntiles = (len + chunk - 1) / chunk;            // tiles the scan will actually visit
    const int64_t total = (ntiles * N) << slots_log2;
    const T* Bs = Bm + (int64_t)b * N * L;
    const T* Cs = Cm + (int64_t)b * N * L;
    float4v* oB = reinterpret_cast<float4v*>(ws_B + (int64_t)b * N * Lpad);
    float4v* oC = reinterpret_cast<float4v*>(ws_C + (int64_t)b * N * Lpad);
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
        const int slot = (int)(i & ((1 << slots_log2) - 1));
        const int64_t tn = i >> slots_log2;                      // tau * N + n
        const int64_t tau = tn / N;
        const int n = (int)(tn - tau * N);
        const int j = slot & (lpr - 1);
        const int q = slot >> lpr_log2;
        const int64_t t = tau * chunk + (int64_t)j * K + q * 4;
        const T* pb = Bs + (int64_t)n * L + t;
        const T* pc = Cs + (int64_t)n * L + t;
        float4v vb, vc;
        vb.x = (t + 0 < len) ? Io<T>::ld(pb + 0) : 0.f; vb.y = (t + 1 < len) ? Io<T>::ld(pb + 1) : 0.f;
        vb.z = (t + 2 < len) ? Io<T>::ld(pb + 2) : 0.f; vb.w = (t + 3 < len) ? Io<T>::ld(pb + 3) : 0.f;
        vc.x = (t + 0 < len) ? Io<T>::ld(pc + 0) : 0.f; vc.y = (t + 1 < len) ? Io<T>::ld(pc + 1) : 0.f;
        vc.z = (t + 2 < len) ? Io<T>::ld(pc + 2) : 0.f; vc.w = (t + 3 < len) ? Io<T>::ld(pc + 3) : 0.f;
        oB[i] = vb;
        oC[i] = vc;
    }
}

// Start the copy of `nfloat` consecutive floats (a multiple of 4) of each operand from the workspace into an
// LDS staging buffer.  Every wave copies 64 sixteen-byte words per instruction; the words go from global
// memory to LDS without passing through registers and are complete when the wave's vmcnt reaches zero.
__device__ __forceinline__ void stage_async(const float* __restrict__ srcB, const float* __restrict__ srcC, float* dstB,
                                            float* dstC, int nfloat, int wave, int lane)
{
    const int slots = nfloat >> 2;
    for (int s0 = wave * 64; s0 < slots; s0 += (int)blockDim.x) {
        if (s0 + lane < slots) {
            __builtin_amdgcn_global_load_lds(srcB + (size_t)(s0 + lane) * 4, dstB + (size_t)s0 * 4, 16, 0, 0);
            __builtin_amdgcn_global_load_lds(srcC + (size_t)(s0 + lane) * 4, dstC + (size_t)s0 * 4, 16, 0, 0);
        }
    }
}

template <typename T, int K, bool SOFTPLUS>
__global__ __launch_bounds__(kMaxBlock) __attribute__((amdgpu_waves_per_eu(min_waves<K>()))) void k_selective_scan(const ScanArgs a)
{
    extern __shared__ float s_mem[];
    const int b = blockIdx.y;
    int chunk = a.chunk;
    if (a.chunks_dev) {
        const int c = a.chunks_dev[b];
        if (c >= COREY_MIN_CHUNK && c <= COREY_MAX_CHUNK && (c & (c - 1)) == 0) chunk = c;
    }
    const int lpr = chunk / K;                              // lanes per row
    const int nthreads = blockDim.x;                        // whole waves; a multiple of lpr when lpr > 64
    int rows = lpr >= nthreads ? 1 : nthreads / lpr;        // rows per workgroup
    if (rows > a.rows_cap) rows = a.rows_cap;
    const int d0 = blockIdx.x * rows;
    if (d0 >= a.D) return;                                  // whole workgroup leaves together

    const int tid = threadIdx.x;
    const int row_local = tid / lpr;
    const int j = tid - row_local * lpr;                    // sub-block of this lane inside the tile
    const int d = d0 + row_local;
    const bool active = row_local < rows && d < a.D;
    const int rl = active ? row_local : 0;                  // safe LDS row for idle lanes
    const int N = a.N;
    const int64_t L = a.L;
    int64_t len = L;
    if (a.seqlens) {
        const int64_t s = a.seqlens[b];
        len = s < 0 ? 0 : (s > L ? L : s);
    }

    float* s_stage = s_mem;                                 // [2 buffers][B, C][kStageElems] staged fp32 operands
    float* s_carry = s_stage + 4 * kStageElems;             // [rows][N] state carried tile to tile
    float* s_A2 = s_carry + (size_t)a.rows_alloc * N;       // [rows][N] A * log2(e)
    float* s_xchg = s_A2 + (size_t)a.rows_alloc * N;        // [kMaxWaves][2] wave totals when a row spans several waves
    for (int i = tid; i < rows * N; i += nthreads) {
        const int r = i / N, n = i - r * N;
        const int dd = d0 + r;
        const bool ok = dd < a.D;
        s_carry[i] = (a.h0 && ok) ? a.h0[((int64_t)b * a.D + dd) * N + n] : 0.f;
        s_A2[i] = ok ? a.A[(int64_t)dd * N + n] * kLog2e : 0.f;
    }

    const int64_t row = (int64_t)b * a.D + (active ? d : d0);
    const T* u_row = static_cast<const T*>(a.u) + row * L;
    const T* dl_row = static_cast<const T*>(a.delta) + row * L;
    const T* z_row = a.z ? static_cast<const T*>(a.z) + row * L : nullptr;
    T* y_row = static_cast<T*>(a.y) + row * L;
    const float* wsB = a.ws_B + (int64_t)b * N * a.Lpad;
    const float* wsC = a.ws_C + (int64_t)b * N * a.Lpad;
    const float bias = (a.dbias && active) ? a.dbias[d] : 0.f;
    const float Dd = (a.Dv && active) ? a.Dv[d] : 0.f;
    const bool vec = a.vector_ok != 0;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int seg = lpr < 64 ? lpr : 64;                    // scan segment inside a wave
    const int jseg = lane & (seg - 1);
    const int wpr = lpr > 64 ? lpr / 64 : 1;                // waves per row
    const int wpos = wave & (wpr - 1);                      // this wave's position inside its row
    int nsub = kStageElems / chunk;                         // states staged per group
    nsub = nsub < 1 ? 1 : (nsub > N ? N : nsub);
    int buf = 0;                                            // staging buffer holding the group about to be used
    if (len > 0) {                                          // first group of the first tile
        const int ns0 = N < nsub ? N : nsub;
        stage_async(wsB, wsC, s_stage, s_stage + kStageElems, ns0 * chunk, wave, lane);
    }

    for (int64_t tile = 0; tile < L; tile += chunk) {
        const int64_t t0 = tile + (int64_t)j * K;
        // A full tile lies inside the sequence with aligned rows: no masks anywhere (idle lanes read row d0).
        const bool full = vec && tile + chunk <= len;       // uniform over the workgroup
        // otherwise: valid steps of this lane (within the sequence) and steps that get a y written (within L)
        int nvalid = K, nstore = K;
        if (!full) {
            nvalid = nstore = 0;
            if (active) {
                nvalid = (t0 >= len) ? 0 : (len - t0 < K ? (int)(len - t0) : K);
                nstore = (t0 >= L) ? 0 : (L - t0 < K ? (int)(L - t0) : K);
            }
        }
        const Raw<T, K> u_raw = load_raw<T, K>(u_row + t0, nvalid, vec);
        float dl[K], du[K], yv[K];
        {
            const Raw<T, K> d_raw = load_raw<T, K>(dl_row + t0, nvalid, vec);
            widen<T, K>(d_raw, dl);
            widen<T, K>(u_raw, du);
        }
        float S = 0.f;
#pragma unroll
        for (int i = 0; i < K; ++i) {
            float v = dl[i] + bias;
            if (SOFTPLUS) v = softplus(v);
            if (!full) v = (i < nvalid) ? v : 0.f;          // padded steps: dl = 0 -> a = 1, b = 0 (identity)
            dl[i] = v;
            du[i] = v * du[i];
            S += v;
            yv[i] = 0.f;
        }

        if (tile < len) {                                   // uniform over the workgroup
            for (int n0 = 0; n0 < N; n0 += nsub) {
                const int ns = (N - n0 < nsub) ? N - n0 : nsub;
                float* s_B = s_stage + buf * 2 * kStageElems;
                float* s_C = s_B + kStageElems;
                // this group's copy (started one group earlier) has landed; every wave is past the previous group
                asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
                __syncthreads();
                {   // start the copy of the next group: same tile, or the first group of the next tile
                    int nn0 = n0 + nsub;
                    int64_t ntile = tile;
                    if (nn0 >= N) { nn0 = 0; ntile = tile + chunk; }
                    if (ntile < len) {
                        const int nns = (N - nn0 < nsub) ? N - nn0 : nsub;
                        const int64_t off = (ntile / chunk * N + nn0) * chunk;
                        float* d_B = s_stage + (buf ^ 1) * 2 * kStageElems;
                        stage_async(wsB + off, wsC + off, d_B, d_B + kStageElems, nns * chunk, wave, lane);
                    }
                }
                buf ^= 1;
                for (int nl = 0; nl < ns; ++nl) {
                    const int n = n0 + nl;
                    const float A2 = s_A2[rl * N + n];
                    const float carry = s_carry[rl * N + n];
                    const float4v* bq = reinterpret_cast<const float4v*>(s_B) + (size_t)(nl * (K / 4)) * lpr + j;
                    const float4v* cq = reinterpret_cast<const float4v*>(s_C) + (size_t)(nl * (K / 4)) * lpr + j;

                    float av[K], bv[K];
                    float h = 0.f;
#pragma unroll
                    for (int q = 0; q < K / 4; ++q) {
                        const float4v b4 = bq[q * lpr];
                        const float be[4] = {b4.x, b4.y, b4.z, b4.w};
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const int i = 4 * q + e;
                            av[i] = fast_exp2(dl[i] * A2);
                            bv[i] = du[i] * be[e];
                            h = fmaf(av[i], h, bv[i]);
                        }
                    }
                    const float P = fast_exp2(S * A2);
                    float Pex = P, hex = h;
                    exclusive_scan_pairs(seg, jseg, Pex, hex);
                    if (wpr > 1) {                           // a row spans several waves: add the totals of the waves before
                        if (lane == 63) { s_xchg[2 * wave] = P * Pex; s_xchg[2 * wave + 1] = fmaf(P, hex, h); }
                        __syncthreads();
                        float Pw = 1.f, hw = 0.f;            // composition of the row's earlier waves, oldest first
                        for (int w = 0; w < wpos; ++w) {
                            const float Pi = s_xchg[2 * (wave - wpos + w)], hi = s_xchg[2 * (wave - wpos + w) + 1];
                            hw = fmaf(Pi, hw, hi);
                            Pw = Pw * Pi;
                        }
                        hex = fmaf(Pex, hw, hex);
                        Pex = Pex * Pw;
                    }
                    float hh = fmaf(Pex, carry, hex);        // true state entering this lane's sub-block
#pragma unroll
                    for (int q = 0; q < K / 4; ++q) {
                        const float4v c4 = cq[q * lpr];
                        const float ce[4] = {c4.x, c4.y, c4.z, c4.w};
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const int i = 4 * q + e;
                            hh = fmaf(av[i], hh, bv[i]);
                            yv[i] = fmaf(ce[e], hh, yv[i]);
                        }
                    }
                    if (wpr > 1) __syncthreads();            // exchange slots are reused by the next state
                    if (active && j == lpr - 1) s_carry[rl * N + n] = hh;
                }
            }
        }

        if (full) {
            float uu[K];
            widen<T, K>(u_raw, uu);
            if (z_row) {
                float zz[K];
                widen<T, K>(load_raw<T, K>(z_row + t0, K, true), zz);
#pragma unroll
                for (int i = 0; i < K; ++i) yv[i] = fmaf(Dd, uu[i], yv[i]) * silu(zz[i]);
            } else {
#pragma unroll
                for (int i = 0; i < K; ++i) yv[i] = fmaf(Dd, uu[i], yv[i]);
            }
            if (active) store_items<T, K>(y_row + t0, K, true, yv);
        } else if (nstore > 0) {
            float uu[K];
            widen<T, K>(u_raw, uu);
            if (nvalid > 0 && z_row) {
                float zz[K];
                widen<T, K>(load_raw<T, K>(z_row + t0, nvalid, vec), zz);
#pragma unroll
                for (int i = 0; i < K; ++i) yv[i] = fmaf(Dd, uu[i], yv[i]) * silu(zz[i]);
            } else {
#pragma unroll
                for (int i = 0; i < K; ++i) yv[i] = fmaf(Dd, uu[i], yv[i]);
            }
#pragma unroll
            for (int i = 0; i < K; ++i)
                if (i >= nvalid) yv[i] = 0.f;                // padded positions are written as zero
            store_items<T, K>(y_row + t0, nstore, vec, yv);
        }
    }
    __syncthreads();                                         // last writes of the carried state are visible

    for (int i = tid; i < rows * N; i += nthreads) {
        const int r = i / N, n = i - r * N;
        const int dd = d0 + r;
        if (dd < a.D) a.last_state[((int64_t)b * a.D + dd) * N + n] = s_carry[i];
    }
}

int64_t padded_len(int64_t L) { return (L + kPad + 3) / 4 * 4; }

}  // namespace

extern "C" size_t selective_scan_fwd_workspace(int64_t B, int64_t N, int64_t L)
{
    if (B < 1 || N < 1 || N > COREY_MAX_STATE || L < 1) return 0;
    return (size_t)2 * B * N * padded_len(L) * sizeof(float);
}

extern "C" int selective_scan_fwd(const void* u, const void* delta, const float* A, const void* Bm, const void* Cm,
                                  const float* Dv, const void* z, const float* delta_bias, int delta_softplus,
                                  const float* h0, const int32_t* seqlens, int32_t chunk, const int32_t* chunks_dev,
                                  void* y, float* last_state, corey_dtype dt, int64_t B, int64_t D, int64_t N, int64_t L,
                                  void* workspace, size_t workspace_bytes, void* hip_stream)
{
    using corey::fail;
    if (!u || !delta || !A || !Bm || !Cm || !y || !last_state)
        return fail(COREY_ENULL, "selective_scan_fwd: u, delta, A, Bm, Cm, y and last_state are required");
    if (dt != COREY_F32 && dt != COREY_BF16 && dt != COREY_F16) return fail(COREY_EINVAL, "selective_scan_fwd: unknown dtype %d", (int)dt);
    if (B < 1 || D < 1 || L < 1) return fail(COREY_ESHAPE, "selective_scan_fwd: B, D, L must be >= 1");
    if (N < 1 || N > COREY_MAX_STATE) return fail(COREY_ESHAPE, "selective_scan_fwd: N = %lld outside [1, %d]", (long long)N, COREY_MAX_STATE);
    if (B > 65535) return fail(COREY_ESHAPE, "selective_scan_fwd: B = %lld exceeds 65535", (long long)B);
    if ((double)B * (double)D >= 2147483647.0 || (double)B * (double)D * (double)L >= 4.0e18 ||
        (double)B * (double)N * (double)L >= 4.0e18)
        return fail(COREY_ESHAPE, "selective_scan_fwd: tensor sizes overflow the kernel's indexing");
    if (chunk < COREY_MIN_CHUNK || chunk > COREY_MAX_CHUNK || !corey::is_pow2(chunk))
        return fail(COREY_EINVAL, "selective_scan_fwd: chunk = %d must be a power of two in [%d, %d]", chunk, COREY_MIN_CHUNK, COREY_MAX_CHUNK);

    const size_t need = selective_scan_fwd_workspace(B, N, L);
    if (!workspace || workspace_bytes < need)
        return fail(COREY_EWORKSPACE, "selective_scan_fwd: workspace of %zu bytes required", need);
    if (reinterpret_cast<uintptr_t>(workspace) % 16 != 0) return fail(COREY_EWORKSPACE, "selective_scan_fwd: workspace must be 16-byte aligned");

    const size_t esz = dt == COREY_F32 ? 4 : 2;
    bool vector_ok = (L * (int64_t)esz) % 16 == 0;
    for (const void* p : {u, delta, Bm, Cm, z, (const void*)y})
        if (p && reinterpret_cast<uintptr_t>(p) % 16 != 0) vector_ok = false;

    ScanArgs a;
    a.u = u; a.delta = delta; a.A = A; a.Bm = Bm; a.Cm = Cm; a.Dv = Dv; a.z = z; a.dbias = delta_bias; a.h0 = h0;
    a.seqlens = seqlens; a.chunks_dev = chunks_dev; a.y = y; a.last_state = last_state;
    a.Lpad = padded_len(L);
    a.ws_B = static_cast<float*>(workspace);
    a.ws_C = a.ws_B + (size_t)B * N * a.Lpad;
    a.L = L; a.D = (int32_t)D; a.N = (int32_t)N; a.chunk = chunk; a.softplus = delta_softplus ? 1 : 0;
    a.vector_ok = vector_ok ? 1 : 0;
    // LDS budget for the per-row arrays (carried state and A): at most 64 rows and 16 KiB each.  64 rows fill
    // the workgroup for every chunk >= 64; shorter chunks run with idle lanes.
    int rows_cap = (int)(4096 / N);
    if (rows_cap < 1) rows_cap = 1;
    if (rows_cap > 64) rows_cap = 64;
    a.rows_cap = rows_cap;

    // Time steps per lane.  16 halves the lane-scan work per value; 8 doubles the lanes and needs fewer registers,
    // which pays only when 16 would leave the chip short of waves (fewer than two per SIMD: 256 CUs x 4 SIMDs x
    // 64 lanes x 2).  Measured on the 2.8B-shaped layer: 8 wins for chunks up to 256, 16 from 512 on.
    const int64_t chunk_for_plan = chunks_dev ? COREY_MAX_CHUNK : chunk;
    const int items = (B * D * (chunk_for_plan / 16) < 131072) ? 8 : 16;
    const int nthreads = kMaxBlock;
    // Rows per workgroup follow from the chunk.  With per-sequence device chunks the grid is sized for the
    // fewest rows any legal chunk gives (surplus workgroups leave at once) and LDS for the most.
    const int lpr_grid = (chunks_dev ? COREY_MAX_CHUNK : chunk) / items;
    const int lpr_lds = (chunks_dev ? COREY_MIN_CHUNK : chunk) / items;
    int rows_min = lpr_grid >= nthreads ? 1 : nthreads / lpr_grid;
    if (rows_min > rows_cap) rows_min = rows_cap;
    int rows_alloc = lpr_lds >= nthreads ? 1 : nthreads / lpr_lds;
    if (rows_alloc > rows_cap) rows_alloc = rows_cap;
    a.rows_alloc = rows_alloc;
    const int64_t gx = (D + rows_min - 1) / rows_min;
    const size_t lds = ((size_t)4 * kStageElems + (size_t)2 * rows_alloc * N + 2 * kMaxWaves) * sizeof(float);
    const dim3 grid((unsigned)gx, (unsigned)B);
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const dim3 block((unsigned)nthreads);
    // relayout of B and C: one 16-byte word per lane, enough workgroups to cover the operand a few times over
    int64_t rb = (N * a.Lpad / 4 + 255) / 256;
    rb = rb < 1 ? 1 : (rb > 2048 ? 2048 : rb);
    const dim3 rgrid((unsigned)rb, (unsigned)B);
#define COREY_LAUNCH(T, K, SP)                                                                                       \
    do {                                                                                                             \
        k_relayout_bc<T, K><<<rgrid, dim3(256), 0, stream>>>(static_cast<const T*>(Bm), static_cast<const T*>(Cm), a.ws_B, \
                                                         a.ws_C, seqlens, chunks_dev, chunk, (int)N, L, a.Lpad);     \
        k_selective_scan<T, K, SP><<<grid, block, lds, stream>>>(a);                                                 \
    } while (0)
#define COREY_LAUNCH_SP(T, K) do { if (a.softplus) COREY_LAUNCH(T, K, true); else COREY_LAUNCH(T, K, false); } while (0)
    if (dt == COREY_F32) {
        if (items == 8) COREY_LAUNCH_SP(float, 8); else COREY_LAUNCH_SP(float, 16);
    } else if (dt == COREY_F16) {
        if (items == 8) COREY_LAUNCH_SP(_Float16, 8); else COREY_LAUNCH_SP(_Float16, 16);
    } else {
        if (items == 8) COREY_LAUNCH_SP(uint16_t, 8); else COREY_LAUNCH_SP(uint16_t, 16);
    }
#undef COREY_LAUNCH_SP
#undef COREY_LAUNCH
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return corey::hip_fail(e, "selective_scan_fwd launch");
    return COREY_OK;
}
