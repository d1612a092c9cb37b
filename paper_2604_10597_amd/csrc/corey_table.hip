// corey_entropy_hist_onesweep / corey_entropy_hist_from_table: the fixed-bin histogram entropy (Eq. 1, r = H / log K)
// of a 16-bit tensor from ONE pass over it, or from none when the tensor's producer filled the table.
//
//   k_table_count   one pass over x: every workgroup counts the 65536 bit patterns of its share in LDS (corey_table.h)
//                   and writes its table, a small tail and its partial range to a slab of the workspace
//   k_table_bin     adds the slabs up, pattern by pattern; the range is the fold of the partial ranges; every pattern that
//                   occurs is binned once, with its multiplicity, by the very binary32 expression the two-pass kernels
//                   apply to every element, so the K counts are bit-identical to theirs
//   k_entropy_finalise (corey_entropy.hip)  H, r and the chunk rule from the counts
// Bandwidth and LDS-atomic work: no matrix instructions.
#include <hip/hip_runtime.h>

#include <cmath>

#include "corey_internal.h"
#include "corey_range.h"
#include "corey_table.h"

namespace {

using corey_range::key_value;
using corey_range::order_key;
using corey_range::RangeFold;
using corey_range::RangePart;
using corey_range::RangeSlot;
using corey_range::usable_range;
using corey_range::word4;
using corey_table::kLanes;
using corey_table::kWords;

constexpr int kRoundWords = corey_table::kRoundAdds / 8 / kLanes;      // 16-byte words per lane and round: 4

__device__ __forceinline__ float pattern_value(uint32_t p, uint16_t) { return __uint_as_float(p << 16); }     // bfloat16
__device__ __forceinline__ float pattern_value(uint32_t p, _Float16)
{
    const uint16_t b = (uint16_t)p;
    _Float16 h;
    __builtin_memcpy(&h, &b, 2);
    return (float)h;
}

// x: the tensor as `nwords` aligned 16-byte words starting at `body`, plus up to 7 single elements before and after
// them (an unaligned or ragged tensor), which workgroup 0 counts in a round of their own.
template <typename T>
__global__ __launch_bounds__(kLanes) void k_table_count(const T* __restrict__ x, int64_t head, const word4* __restrict__ body,
                                                        int64_t nwords, int64_t tail, void* workspace)
{
    __shared__ uint32_t s_tab[kWords];
    __shared__ corey_table::Shared sh;
    const corey_table::Workspace ws = corey_table::carve(workspace);
    corey_table::begin(s_tab, sh, ws);
    float lo = INFINITY, hi = -INFINITY;
    uint32_t mag = 0u;

    bool nan_single = false;
    if (blockIdx.x == 0 && head + tail > 0) {                   // uniform over the workgroup: a round of its own
        if ((int64_t)threadIdx.x < head + tail) {
            const int64_t i = (int64_t)threadIdx.x < head ? (int64_t)threadIdx.x : head + nwords * 8 + ((int64_t)threadIdx.x - head);
            uint16_t bits;
            __builtin_memcpy(&bits, &x[i], 2);
            const float v = pattern_value(bits, T());
            nan_single = v != v;
            lo = fminf(lo, v);                                  // fminf / fmaxf drop a NaN operand; NaN is flagged separately
            hi = fmaxf(hi, v);
            corey_table::add(s_tab, sh, bits);
        }
        __syncthreads();
    }

    // rounds of kRoundWords words per lane; the next round's words are requested before this round's are counted
    const int64_t step = (int64_t)gridDim.x * kLanes * kRoundWords;
    int64_t base = (int64_t)blockIdx.x * kLanes * kRoundWords;
    word4 q[kRoundWords], qn[kRoundWords];
    auto fetch = [&](int64_t b, word4 (&dst)[kRoundWords]) {
#pragma unroll
        for (int k = 0; k < kRoundWords; ++k) {
            const int64_t i = b + (int64_t)k * kLanes + threadIdx.x;
            dst[k] = i < nwords ? body[i] : word4{0u, 0u, 0u, 0u};
        }
    };
    if (base < nwords) fetch(base, q);
    for (; base < nwords; base += step) {                        // uniform over the workgroup
        if (base + step < nwords) fetch(base + step, qn);
#pragma unroll
        for (int k = 0; k < kRoundWords; ++k) {
            if (base + (int64_t)k * kLanes + threadIdx.x < nwords) {
                RangeFold<T>::fold(q[k], lo, hi, mag);
                const uint32_t w[4] = {q[k].x, q[k].y, q[k].z, q[k].w};
                corey_table::add_word4(s_tab, sh, w);
            }
        }
#pragma unroll
        for (int k = 0; k < kRoundWords; ++k) q[k] = qn[k];
        __syncthreads();                                         // round boundary: every guard crossing has been undone
    }
    uint32_t klo = (lo <= hi) ? order_key(lo) : 0xffffffffu;
    uint32_t khi = (lo <= hi) ? order_key(hi) : 0u;
    uint32_t knan = (RangeFold<T>::saw_nan(mag) || nan_single) ? 1u : 0u;
    corey_table::end(s_tab, sh, ws, klo, khi, knan);
}

// Grid: (kWords / 1024 blocks of 1024 table words) x kSlabGroups; a workgroup adds up, for its 1024 words (2048
// patterns), the slabs s = group, group + kSlabGroups, ...: a lane owns 4 consecutive words (8 patterns).
constexpr int kBinLanes = 256;
constexpr int kWordBlock = kBinLanes * 4;
constexpr int kSlabGroups = 8;
constexpr int kBinBatch = 8;        // slab loads a lane keeps in flight

template <typename T>
__global__ __launch_bounds__(kBinLanes) void k_table_bin(void* workspace, int K)
{
    __shared__ uint32_t s_extra[2 * kWordBlock];                // overflow entries and zeros that belong to this block's patterns
    __shared__ uint32_t s_bins[COREY_MAX_BINS];
    __shared__ RangeSlot s_slot;
    const corey_table::Workspace ws = corey_table::carve(workspace);
    const int nslabs = (int)min(*ws.nslabs, (uint32_t)corey_table::kMaxSlabs);
    const int wb = blockIdx.x, group = blockIdx.y;
    const int wg = blockIdx.y * gridDim.x + blockIdx.x;
    for (int i = threadIdx.x; i < 2 * kWordBlock; i += kBinLanes) s_extra[i] = 0u;
    for (int i = threadIdx.x; i < K; i += kBinLanes) s_bins[i] = 0u;
    {   // the range: fold of the partial ranges of the workgroups that filled the tables
        uint32_t klo = 0xffffffffu, khi = 0u, knan = 0u;
        for (int i = threadIdx.x; i < nslabs; i += kBinLanes) {
            const RangePart rp = ws.rparts[i];
            klo = min(klo, rp.lo_key);
            khi = max(khi, rp.hi_key);
            knan |= rp.saw_nan;
        }
        corey_range::reduce_range_keys<kBinLanes>(klo, khi, knan);
        if (threadIdx.x == 0) {
            s_slot.lo_key = klo; s_slot.hi_key = khi; s_slot.saw_nan = knan; s_slot.pad = 0u;
            if (wg == 0) ws.slots[0] = s_slot;                  // for the reduction kernel
        }
        __syncthreads();
    }
    float lo, hi;
    if (!usable_range(s_slot, &lo, &hi)) return;                // counts stay zero, H and r become NaN

    uint32_t tot_lo[4] = {0u, 0u, 0u, 0u}, tot_hi[4] = {0u, 0u, 0u, 0u};
    const size_t my = (size_t)wb * kWordBlock + (size_t)threadIdx.x * 4;
    for (int s0 = group; s0 < nslabs; s0 += kSlabGroups * kBinBatch) {
        word4 q[kBinBatch];
#pragma unroll
        for (int k = 0; k < kBinBatch; ++k) {
            const int s = s0 + k * kSlabGroups;
            q[k] = s < nslabs ? *reinterpret_cast<const word4*>(ws.slabs + (size_t)s * kWords + my) : word4{0u, 0u, 0u, 0u};
        }
#pragma unroll
        for (int k = 0; k < kBinBatch; ++k) {
            const uint32_t w[4] = {q[k].x, q[k].y, q[k].z, q[k].w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                tot_lo[e] += w[e] & 0xffffu;
                tot_hi[e] += w[e] >> 16;
            }
        }
    }
    {   // what the same slabs keep outside their tables: the zero pattern's count and the overflow lists (usually empty)
        constexpr int kGroupSlabs = (corey_table::kMaxSlabs + kSlabGroups - 1) / kSlabGroups;
        __shared__ uint32_t s_nover[kGroupSlabs];
        if (threadIdx.x < kGroupSlabs) {                         // one slab of the group per lane: the heads in one go
            const int s = group + (int)threadIdx.x * kSlabGroups;
            uint32_t n_over = 0u;
            if (s < nslabs) {
                const corey_table::Head h = ws.heads[s];
                n_over = min(h.n_over, (uint32_t)corey_table::kMaxOver);
                if (wb == 0 && h.zeros) atomicAdd(&s_extra[0], h.zeros);      // pattern 0x0000 is the low half of word 0
            }
            s_nover[threadIdx.x] = n_over;
        }
        __syncthreads();
        for (int t = 0; t < kGroupSlabs; ++t) {                  // uniform
            const uint32_t n = s_nover[t];
            const corey_table::Tail* tail = ws.tails + (group + t * kSlabGroups);
            for (uint32_t i = threadIdx.x; i < n; i += kBinLanes) {
                const uint32_t p = tail->over[i];
                const uint32_t m = p & 0x7fffu;
                if ((int)(m / kWordBlock) == wb) atomicAdd(&s_extra[(m % kWordBlock) * 2 + (p >> 15)], 32768u);
            }
        }
    }
    __syncthreads();

    const bool flat = hi == lo;                                  // degenerate range: everything in bin 0
    const float scale = flat ? 0.f : (float)((double)K / ((double)hi - (double)lo));
    const int top = K - 1;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const uint32_t m = (uint32_t)my + e;
        const uint32_t local = (uint32_t)threadIdx.x * 4 + e;
#pragma unroll
        for (int sign = 0; sign < 2; ++sign) {
            const uint32_t total = (sign ? tot_hi[e] : tot_lo[e]) + s_extra[local * 2 + sign];
            if (total == 0u) continue;
            const float v = pattern_value(m | (sign ? 0x8000u : 0u), T());
            const float qv = __fmul_rn(__fsub_rn(v, lo), scale);          // two separate binary32 roundings
            int k = (int)qv;                                             // truncation; qv >= 0
            k = flat ? 0 : (k > top ? top : (k < 0 ? 0 : k));
            atomicAdd(&s_bins[k], total);
        }
    }
    __syncthreads();
    uint32_t* out = ws.parts + (size_t)(wg % corey_table::kParts) * K;
    for (int k = threadIdx.x; k < K; k += kBinLanes) {
        const uint32_t c = s_bins[k];
        if (c) atomicAdd(&out[k], c);
    }
}

int check_common(const char* who, corey_dtype dt, int64_t L, int32_t K, double eps, const corey_policy* p, const int32_t* chunks_out,
                 const uint32_t* counts_out, const double* H_out, const double* r_out, const void* ws, size_t ws_bytes)
{
    using corey::fail;
    if (!counts_out || !H_out || !r_out) return fail(COREY_ENULL, "%s: counts_out, H_out and r_out are required", who);
    if (dt != COREY_BF16 && dt != COREY_F16)
        return fail(dt == COREY_F32 ? COREY_EUNSUPPORTED : COREY_EINVAL, "%s: the bit-pattern table exists for 16-bit storage only", who);
    if (L < 1) return fail(COREY_ESHAPE, "%s: L must be >= 1", who);
    if (K < 2 || K > COREY_MAX_BINS) return fail(COREY_EINVAL, "%s: K = %d outside [2, %d]", who, K, COREY_MAX_BINS);
    if (!(eps >= 0.0)) return fail(COREY_EINVAL, "%s: eps must be >= 0", who);
    if (p && !chunks_out) return fail(COREY_ENULL, "%s: a policy needs chunks_out", who);
    if (p) {
        const int st = corey::check_device_policy(who, p, L);
        if (st != COREY_OK) return st;
    }
    if (!ws || ws_bytes < corey_table::kWorkspaceBytes)
        return fail(COREY_EWORKSPACE, "%s: table workspace of %zu bytes required", who, corey_table::kWorkspaceBytes);
    if (reinterpret_cast<uintptr_t>(ws) % 256 != 0) return fail(COREY_EWORKSPACE, "%s: table workspace must be 256-byte aligned", who);
    return COREY_OK;
}

int bin_and_finalise(corey_dtype dt, int64_t L, int32_t K, double eps, const corey_policy* p, int32_t* chunks_out, uint32_t* counts_out,
                     double* H_out, double* r_out, float* range_out, void* table_ws, hipStream_t stream)
{
    const dim3 grid(kWords / kWordBlock, kSlabGroups);
    if (dt == COREY_F16) k_table_bin<_Float16><<<grid, dim3(kBinLanes), 0, stream>>>(table_ws, K);
    else k_table_bin<uint16_t><<<grid, dim3(kBinLanes), 0, stream>>>(table_ws, K);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return corey::hip_fail(e, "pattern-table binning launch");
    const corey_table::Workspace ws = corey_table::carve(table_ws);
    return corey::launch_entropy_finalise(ws.parts, counts_out, K, eps, ws.slots, H_out, r_out, range_out, p, chunks_out, L, stream);
}

}  // namespace

extern "C" size_t corey_pattern_table_workspace(void) { return corey_table::kWorkspaceBytes; }

extern "C" int corey_entropy_hist_onesweep(const void* x, corey_dtype dt, int64_t B, int64_t D, int64_t L, int32_t K, double eps,
                                           const corey_policy* p, int32_t* chunks_out, uint32_t* counts_out, double* H_out,
                                           double* r_out, float* range_out, void* table_ws, size_t table_ws_bytes, void* hip_stream)
{
    using corey::fail;
    const char* who = "corey_entropy_hist_onesweep";
    if (!x) return fail(COREY_ENULL, "%s: x is required", who);
    if (B < 1 || D < 1 || L < 1) return fail(COREY_ESHAPE, "%s: B, D, L must be >= 1", who);
    if ((double)B * (double)D * (double)L >= 4294967296.0) return fail(COREY_ESHAPE, "%s: more than 2^32-1 values would overflow the 32-bit counts", who);
    const int st = check_common(who, dt, L, K, eps, p, chunks_out, counts_out, H_out, r_out, table_ws, table_ws_bytes);
    if (st != COREY_OK) return st;
    if (reinterpret_cast<uintptr_t>(x) % 2 != 0) return fail(COREY_EINVAL, "%s: x must be 2-byte aligned", who);
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const int64_t E = B * D * L;
    int64_t head = (int64_t)((16 - reinterpret_cast<uintptr_t>(x) % 16) % 16) / 2;      // single elements before the first aligned word
    if (head > E) head = E;
    const int64_t nwords = (E - head) / 8;
    const int64_t tail = E - head - nwords * 8;
    const word4* body = reinterpret_cast<const word4*>(static_cast<const char*>(x) + head * 2);
    int64_t blocks = (nwords + (int64_t)kLanes * kRoundWords - 1) / ((int64_t)kLanes * kRoundWords);
    blocks = blocks < 1 ? 1 : (blocks > corey_table::kMaxSlabs ? corey_table::kMaxSlabs : blocks);
    // a workgroup records one overflow entry per 32768 occurrences of a pattern: its share must stay below kMaxOver of them
    if ((E + blocks - 1) / blocks / 32768 >= corey_table::kMaxOver) return fail(COREY_ESHAPE, "%s: too many values per workgroup", who);
    if (dt == COREY_F16)
        k_table_count<_Float16><<<dim3((unsigned)blocks), dim3(kLanes), 0, stream>>>(static_cast<const _Float16*>(x), head, body, nwords, tail, table_ws);
    else
        k_table_count<uint16_t><<<dim3((unsigned)blocks), dim3(kLanes), 0, stream>>>(static_cast<const uint16_t*>(x), head, body, nwords, tail, table_ws);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return corey::hip_fail(e, "corey_entropy_hist_onesweep launch");
    return bin_and_finalise(dt, L, K, eps, p, chunks_out, counts_out, H_out, r_out, range_out, table_ws, stream);
}

extern "C" int corey_entropy_hist_from_table(corey_dtype dt, int64_t L, int32_t K, double eps, const corey_policy* p,
                                             int32_t* chunks_out, uint32_t* counts_out, double* H_out, double* r_out,
                                             float* range_out, void* table_ws, size_t table_ws_bytes, void* hip_stream)
{
    const int st = check_common("corey_entropy_hist_from_table", dt, L, K, eps, p, chunks_out, counts_out, H_out, r_out, table_ws,
                                table_ws_bytes);
    if (st != COREY_OK) return st;
    return bin_and_finalise(dt, L, K, eps, p, chunks_out, counts_out, H_out, r_out, range_out, table_ws, static_cast<hipStream_t>(hip_stream));
}
