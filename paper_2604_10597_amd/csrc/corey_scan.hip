// selective_scan_fwd: Mamba-1 selective-scan forward with a run-time chunk on gfx950.
//
// Mapping.  A workgroup of 256 lanes owns `rows` channels of one sequence and walks the time axis in
// tiles of `chunk` steps.  Inside a tile a row is spread over chunk/16 consecutive lanes, each lane owning
// 16 consecutive time steps, so loads of u/delta/z and the store of y are contiguous along L.  For every
// state index n a lane
//   1. discretises its 16 steps (a_i = exp(dl_i A), b_i = dl_i B_i u_i) and folds them, from a zero state,
//      into the pair (P, h) that represents the affine map  x -> P x + h  of its sub-block;
//   2. takes part in a segmented inclusive scan of those pairs over the lanes of its row (the pair
//      operator is associative), crossing the wave boundary through LDS when a row needs 128 lanes;
//   3. replays its 16 steps from the true incoming state (prefix pair applied to the state carried from
//      the previous tile) and accumulates y_i += C_i h_i.
// The fp32 state carried from tile to tile lives in LDS; the last lane of a row refreshes it.
// The work is a recurrence plus elementwise maths: no matrix instructions.
#include <hip/hip_runtime.h>

#include "corey_internal.h"

namespace {

using corey::bf16_to_f32;
using corey::f32_to_bf16;

constexpr int kItems = 16;      // time steps per lane per tile
constexpr int kBlock = 256;     // lanes per workgroup
constexpr float kLog2e = 1.4426950408889634f;

template <typename T> struct Io;
template <> struct Io<float> {
    static __device__ __forceinline__ float ld(const float* p) { return *p; }
    static __device__ __forceinline__ void st(float* p, float v) { *p = v; }
};
template <> struct Io<uint16_t> {
    static __device__ __forceinline__ float ld(const uint16_t* p) { return bf16_to_f32(*p); }
    static __device__ __forceinline__ void st(uint16_t* p, float v) { *p = f32_to_bf16(v); }
};

// Load kItems consecutive values starting at p (valid: the first nvalid), widened to fp32; the rest are 0.
template <typename T>
__device__ __forceinline__ void load_items(const T* p, int nvalid, bool vector_ok, float (&out)[kItems])
{
    if (vector_ok && nvalid == kItems) {
        typedef uint32_t vec4 __attribute__((ext_vector_type(4)));
        constexpr int kVecs = kItems * (int)sizeof(T) / 16;
        T raw[kItems];
        const vec4* pv = reinterpret_cast<const vec4*>(p);
#pragma unroll
        for (int v = 0; v < kVecs; ++v) {
            const vec4 q = pv[v];
            __builtin_memcpy(reinterpret_cast<char*>(raw) + 16 * v, &q, 16);
        }
#pragma unroll
        for (int i = 0; i < kItems; ++i) out[i] = Io<T>::ld(&raw[i]);
    } else {
#pragma unroll
        for (int i = 0; i < kItems; ++i) out[i] = (i < nvalid) ? Io<T>::ld(p + i) : 0.f;
    }
}

template <typename T>
__device__ __forceinline__ void store_items(T* p, int nstore, bool vector_ok, const float (&v)[kItems])
{
    if (vector_ok && nstore == kItems) {
        typedef uint32_t vec4 __attribute__((ext_vector_type(4)));
        constexpr int kVecs = kItems * (int)sizeof(T) / 16;
        T raw[kItems];
#pragma unroll
        for (int i = 0; i < kItems; ++i) Io<T>::st(&raw[i], v[i]);
        vec4* pv = reinterpret_cast<vec4*>(p);
#pragma unroll
        for (int k = 0; k < kVecs; ++k) {
            vec4 q;
            __builtin_memcpy(&q, reinterpret_cast<const char*>(raw) + 16 * k, 16);
            pv[k] = q;
        }
    } else {
#pragma unroll
        for (int i = 0; i < kItems; ++i)
            if (i < nstore) Io<T>::st(p + i, v[i]);
    }
}

// log(1 + e^x) without losing the small tail: log1p on e^{-|x|}.
__device__ __forceinline__ float softplus(float x)
{
    return fmaxf(x, 0.f) + log1pf(expf(-fabsf(x)));
}

__device__ __forceinline__ float silu(float z) { return z / (1.f + expf(-z)); }

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
    int64_t L;
    int32_t D, N;
    int32_t chunk;          // host chunk (also the fallback for invalid device entries)
    int32_t rows_cap;       // most rows a workgroup may hold (LDS budget for the carried state)
    int32_t softplus;
    int32_t vector_ok;      // rows of the [.., L] tensors are 16-byte aligned
};

template <typename T>
__global__ __launch_bounds__(kBlock) void k_selective_scan(const ScanArgs a)
{
    extern __shared__ float s_mem[];
    const int b = blockIdx.y;
    int chunk = a.chunk;
    if (a.chunks_dev) {
        const int c = a.chunks_dev[b];
        if (c >= COREY_MIN_CHUNK && c <= COREY_MAX_CHUNK && (c & (c - 1)) == 0) chunk = c;
    }
    const int lpr = chunk / kItems;                         // lanes per row (1 .. 128)
    int rows = kBlock / lpr;                                // rows per workgroup
    if (rows > a.rows_cap) rows = a.rows_cap;
    const int d0 = blockIdx.x * rows;
    if (d0 >= a.D) return;                                  // whole workgroup leaves together

    const int tid = threadIdx.x;
    const int row_local = tid / lpr;
    const int j = tid - row_local * lpr;                    // sub-block of this lane inside the tile
    const int d = d0 + row_local;
    const bool active = row_local < rows && d < a.D;
    const int N = a.N;
    const int64_t L = a.L;
    int64_t len = L;
    if (a.seqlens) {
        const int64_t s = a.seqlens[b];
        len = s < 0 ? 0 : (s > L ? L : s);
    }

    float* s_carry = s_mem;                                 // [rows][N] state carried tile to tile
    float* s_xchg = s_mem + (size_t)a.rows_cap * N;         // [waves][2] wave totals when a row spans two waves
    const int64_t row = (int64_t)b * a.D + (active ? d : d0);
    for (int i = tid; i < rows * N; i += kBlock) {
        const int rl = i / N, n = i - rl * N;
        const int dd = d0 + rl;
        s_carry[i] = (a.h0 && dd < a.D) ? a.h0[((int64_t)b * a.D + dd) * N + n] : 0.f;
    }
    __syncthreads();

    const T* u_row = static_cast<const T*>(a.u) + row * L;
    const T* dl_row = static_cast<const T*>(a.delta) + row * L;
    const T* z_row = a.z ? static_cast<const T*>(a.z) + row * L : nullptr;
    T* y_row = static_cast<T*>(a.y) + row * L;
    const T* B_seq = static_cast<const T*>(a.Bm) + (int64_t)b * N * L;
    const T* C_seq = static_cast<const T*>(a.Cm) + (int64_t)b * N * L;
    const float bias = (a.dbias && active) ? a.dbias[d] : 0.f;
    const float Dd = (a.Dv && active) ? a.Dv[d] : 0.f;
    const bool vec = a.vector_ok != 0;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int seg = lpr < 64 ? lpr : 64;                    // scan segment inside a wave

    for (int64_t tile = 0; tile < L; tile += chunk) {
        const int64_t t0 = tile + (int64_t)j * kItems;
        // valid steps of this lane (within the sequence) and steps that get a y written (within L)
        int nvalid = 0, nstore = 0;
        if (active) {
            nvalid = (t0 >= len) ? 0 : (len - t0 < kItems ? (int)(len - t0) : kItems);
            nstore = (t0 >= L) ? 0 : (L - t0 < kItems ? (int)(L - t0) : kItems);
        }
        float dl[kItems], du[kItems], uu[kItems], yv[kItems];
        if (tile < len || nstore > 0) {
            load_items<T>(u_row + t0, nvalid, vec, uu);
            load_items<T>(dl_row + t0, nvalid, vec, dl);
        }
        float S = 0.f;
#pragma unroll
        for (int i = 0; i < kItems; ++i) {
            float v = 0.f;
            if (i < nvalid) {
                v = dl[i] + bias;
                if (a.softplus) v = softplus(v);
            }
            dl[i] = v;                                      // padded steps: dl = 0 -> a = 1, b = 0 (identity)
            du[i] = v * uu[i];
            S += v;
            yv[i] = 0.f;
        }

        if (tile < len) {                                   // uniform over the workgroup
            for (int n = 0; n < N; ++n) {
                const float A2 = active ? a.A[(int64_t)d * N + n] * kLog2e : 0.f;
                float Bv[kItems], Cv[kItems];
                load_items<T>(B_seq + (int64_t)n * L + t0, nvalid, vec, Bv);
                load_items<T>(C_seq + (int64_t)n * L + t0, nvalid, vec, Cv);
                const float carry = active ? s_carry[row_local * N + n] : 0.f;

                float av[kItems], bv[kItems];
                float h = 0.f;
#pragma unroll
                for (int i = 0; i < kItems; ++i) {
                    av[i] = __builtin_amdgcn_exp2f(dl[i] * A2);
                    bv[i] = du[i] * Bv[i];
                    h = fmaf(av[i], h, bv[i]);
                }
                float P = __builtin_amdgcn_exp2f(S * A2);

                // segmented inclusive scan of (P, h) over the lanes of the row inside this wave
                for (int off = 1; off < seg; off <<= 1) {
                    const float Po = __shfl_up(P, off, seg);
                    const float ho = __shfl_up(h, off, seg);
                    if ((lane & (seg - 1)) >= off) {
                        h = fmaf(P, ho, h);
                        P = P * Po;
                    }
                }
                // exclusive prefix = inclusive value of the lane to the left
                float Pex = __shfl_up(P, 1, seg);
                float hex = __shfl_up(h, 1, seg);
                if ((lane & (seg - 1)) == 0) { Pex = 1.f; hex = 0.f; }
                if (lpr > 64) {                              // a row spans two waves: second wave adds the first's total
                    if (lane == 63) { s_xchg[2 * wave] = P; s_xchg[2 * wave + 1] = h; }
                    __syncthreads();
                    if (wave & 1) {
                        const float Pw = s_xchg[2 * (wave - 1)], hw = s_xchg[2 * (wave - 1) + 1];
                        hex = fmaf(Pex, hw, hex);
                        Pex = Pex * Pw;
                    }
                }
                float hh = fmaf(Pex, carry, hex);            // true state entering this lane's sub-block
#pragma unroll
                for (int i = 0; i < kItems; ++i) {
                    hh = fmaf(av[i], hh, bv[i]);
                    yv[i] = fmaf(Cv[i], hh, yv[i]);
                }
                if (lpr > 64) __syncthreads();               // exchange slots are reused by the next state
                if (active && j == lpr - 1) s_carry[row_local * N + n] = hh;
            }
        }

        if (nstore > 0) {
            if (nvalid > 0 && z_row) {
                float zz[kItems];
                load_items<T>(z_row + t0, nvalid, vec, zz);
#pragma unroll
                for (int i = 0; i < kItems; ++i) yv[i] = (yv[i] + Dd * uu[i]) * silu(zz[i]);
            } else {
#pragma unroll
                for (int i = 0; i < kItems; ++i) yv[i] = yv[i] + Dd * uu[i];
            }
#pragma unroll
            for (int i = 0; i < kItems; ++i)
                if (i >= nvalid) yv[i] = 0.f;                // padded positions are written as zero
            store_items<T>(y_row + t0, nstore, vec, yv);
        }
        __syncthreads();                                     // carried state visible to every lane of the row
    }

    for (int i = tid; i < rows * N; i += kBlock) {
        const int rl = i / N, n = i - rl * N;
        const int dd = d0 + rl;
        if (dd < a.D) a.last_state[((int64_t)b * a.D + dd) * N + n] = s_carry[i];
    }
}

}  // namespace

extern "C" int selective_scan_fwd(const void* u, const void* delta, const float* A, const void* Bm, const void* Cm,
                                  const float* Dv, const void* z, const float* delta_bias, int delta_softplus,
                                  const float* h0, const int32_t* seqlens, int32_t chunk, const int32_t* chunks_dev,
                                  void* y, float* last_state, corey_dtype dt, int64_t B, int64_t D, int64_t N, int64_t L,
                                  void* hip_stream)
{
    using corey::fail;
    if (!u || !delta || !A || !Bm || !Cm || !y || !last_state)
        return fail(COREY_ENULL, "selective_scan_fwd: u, delta, A, Bm, Cm, y and last_state are required");
    if (dt != COREY_F32 && dt != COREY_BF16) return fail(COREY_EINVAL, "selective_scan_fwd: unknown dtype %d", (int)dt);
    if (B < 1 || D < 1 || L < 1) return fail(COREY_ESHAPE, "selective_scan_fwd: B, D, L must be >= 1");
    if (N < 1 || N > COREY_MAX_STATE) return fail(COREY_ESHAPE, "selective_scan_fwd: N = %lld outside [1, %d]", (long long)N, COREY_MAX_STATE);
    if (B > 65535) return fail(COREY_ESHAPE, "selective_scan_fwd: B = %lld exceeds 65535", (long long)B);
    if ((double)B * (double)D >= 2147483647.0 || (double)B * (double)D * (double)L >= 4.0e18 ||
        (double)B * (double)N * (double)L >= 4.0e18)
        return fail(COREY_ESHAPE, "selective_scan_fwd: tensor sizes overflow the kernel's indexing");
    if (chunk < COREY_MIN_CHUNK || chunk > COREY_MAX_CHUNK || !corey::is_pow2(chunk))
        return fail(COREY_EINVAL, "selective_scan_fwd: chunk = %d must be a power of two in [%d, %d]", chunk, COREY_MIN_CHUNK, COREY_MAX_CHUNK);

    const size_t esz = dt == COREY_F32 ? 4 : 2;
    bool vector_ok = (L * (int64_t)esz) % 16 == 0;
    for (const void* p : {u, delta, Bm, Cm, z, (const void*)y})
        if (p && reinterpret_cast<uintptr_t>(p) % 16 != 0) vector_ok = false;

    ScanArgs a;
    a.u = u; a.delta = delta; a.A = A; a.Bm = Bm; a.Cm = Cm; a.Dv = Dv; a.z = z; a.dbias = delta_bias; a.h0 = h0;
    a.seqlens = seqlens; a.chunks_dev = chunks_dev; a.y = y; a.last_state = last_state;
    a.L = L; a.D = (int32_t)D; a.N = (int32_t)N; a.chunk = chunk; a.softplus = delta_softplus ? 1 : 0;
    a.vector_ok = vector_ok ? 1 : 0;
    // LDS budget for the carried state: rows * N floats, at most 32 KiB
    int rows_cap = (int)(8192 / N);
    if (rows_cap < 1) rows_cap = 1;
    if (rows_cap > kBlock) rows_cap = kBlock;
    a.rows_cap = rows_cap;

    // Rows per workgroup follow from the chunk; with per-sequence device chunks the grid is sized for the
    // fewest rows any legal chunk gives, and surplus workgroups leave at once.
    const int lpr_host = (chunks_dev ? COREY_MAX_CHUNK : chunk) / kItems;
    int rows_min = kBlock / lpr_host;
    if (rows_min > rows_cap) rows_min = rows_cap;
    const int64_t gx = (D + rows_min - 1) / rows_min;
    const size_t lds = ((size_t)rows_cap * N + 2 * (kBlock / 64)) * sizeof(float);
    const dim3 grid((unsigned)gx, (unsigned)B);
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    if (dt == COREY_F32)
        k_selective_scan<float><<<grid, dim3(kBlock), lds, stream>>>(a);
    else
        k_selective_scan<uint16_t><<<grid, dim3(kBlock), lds, stream>>>(a);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return corey::hip_fail(e, "selective_scan_fwd launch");
    return COREY_OK;
}
