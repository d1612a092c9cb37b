// selective_scan_fwd: host entry.  Validates the arguments, lays out the launch and hands over to the kernels of
// the storage type (corey_scan_impl.h, instantiated per type in corey_scan_f32/bf16/f16.hip).
#include <hip/hip_runtime.h>

#include <cstring>

#include "corey_scan_impl.h"

namespace corey_scan {
void launch_scan_f32(const ScanArgs& a, const LaunchPlan& p);
void launch_scan_bf16(const ScanArgs& a, const LaunchPlan& p);
void launch_scan_f16(const ScanArgs& a, const LaunchPlan& p);
}  // namespace corey_scan

namespace {
int64_t padded_len(int64_t L) { return (L + corey_scan::kPad + 3) / 4 * 4; }
}  // namespace

extern "C" size_t selective_scan_fwd_workspace(int64_t B, int64_t N, int64_t L)
{
    if (B < 1 || N < 1 || N > COREY_MAX_STATE || L < 1) return 0;
    return (size_t)4 * B * corey_scan::a_np(N) * padded_len(L) * sizeof(float);     // B and C, in two orders
}

extern "C" int64_t selective_scan_fwd_plan(int64_t B, int64_t D, int64_t N, int32_t chunk)
{
    if (B < 1 || D < 1 || N < 1 || N > COREY_MAX_STATE || chunk < COREY_MIN_CHUNK || chunk > COREY_MAX_CHUNK || !corey::is_pow2(chunk))
        return -1;
    int rows_cap = (int)(2048 / corey_scan::a_np(N));
    rows_cap = rows_cap < 1 ? 1 : (rows_cap > 32 ? 32 : rows_cap);
    return corey_scan::plan_d16(B, D, chunk, rows_cap);
}

extern "C" int32_t selective_scan_fwd_plan_steps(int64_t B, int64_t D, int64_t N, int32_t chunk)
{
    const int64_t d16 = selective_scan_fwd_plan(B, D, N, chunk);
    if (d16 < 0) return -1;
    return corey_scan::plan_klo(B, D, chunk, d16);
}

extern "C" int32_t selective_scan_fwd_plan_split(int64_t B, int64_t D, int64_t N, int32_t chunk)
{
    const int64_t d16 = selective_scan_fwd_plan(B, D, N, chunk);
    if (d16 < 0) return -1;
    return corey_scan::plan_split(B, D, (int)N, chunk, d16, corey_scan::plan_klo(B, D, chunk, d16), 1);
}

namespace {

int scan_impl(const char* who, const void* u, const void* delta, const float* A, const void* Bm, const void* Cm,
              const float* Dv, const void* z, const float* delta_bias, int delta_softplus,
              const float* h0, const int32_t* seqlens, int32_t chunk, const int32_t* chunks_dev, const corey_finalise::Args* route,
              void* y, float* last_state, corey_dtype dt, int64_t B, int64_t D, int64_t N, int64_t L,
              uint32_t flags, void* workspace, size_t workspace_bytes, void* hip_stream)
{
    using corey::fail;
    if (!u || !delta || !A || !Bm || !Cm || !y || !last_state)
        return fail(COREY_ENULL, "%s: u, delta, A, Bm, Cm, y and last_state are required", who);
    if (dt != COREY_F32 && dt != COREY_BF16 && dt != COREY_F16) return fail(COREY_EINVAL, "%s: unknown dtype %d", who, (int)dt);
    if (B < 1 || D < 1 || L < 1) return fail(COREY_ESHAPE, "%s: B, D, L must be >= 1", who);
    if (N < 1 || N > COREY_MAX_STATE) return fail(COREY_ESHAPE, "%s: N = %lld outside [1, %d]", who, (long long)N, COREY_MAX_STATE);
    if (B > 65535) return fail(COREY_ESHAPE, "%s: B = %lld exceeds 65535", who, (long long)B);
    if ((double)B * (double)D >= 2147483647.0 || (double)B * (double)D * (double)L >= 4.0e18 ||
        (double)B * (double)N * (double)L >= 4.0e18)
        return fail(COREY_ESHAPE, "%s: tensor sizes overflow the kernel's indexing", who);
    if (chunk < COREY_MIN_CHUNK || chunk > COREY_MAX_CHUNK || !corey::is_pow2(chunk))
        return fail(COREY_EINVAL, "%s: chunk = %d must be a power of two in [%d, %d]", who, chunk, COREY_MIN_CHUNK, COREY_MAX_CHUNK);
    if (flags & ~(COREY_SCAN_GENERAL_A | COREY_SCAN_ONE_CHUNK | COREY_SCAN_WHOLE_ROWS)) return fail(COREY_EINVAL, "%s: unknown flags 0x%x", who, flags);

    const size_t need = selective_scan_fwd_workspace(B, N, L);
    if (!workspace || workspace_bytes < need)
        return fail(COREY_EWORKSPACE, "%s: workspace of %zu bytes required", who, need);
    if (reinterpret_cast<uintptr_t>(workspace) % 16 != 0) return fail(COREY_EWORKSPACE, "%s: workspace must be 16-byte aligned", who);

    const size_t esz = dt == COREY_F32 ? 4 : 2;
    bool vector_ok = (L * (int64_t)esz) % 16 == 0;
    for (const void* p : {u, delta, Bm, Cm, z, (const void*)y})
        if (p && reinterpret_cast<uintptr_t>(p) % 16 != 0) vector_ok = false;

    corey_scan::ScanArgs a;
    a.u = u; a.delta = delta; a.A = A; a.Bm = Bm; a.Cm = Cm; a.Dv = Dv; a.z = z; a.dbias = delta_bias; a.h0 = h0;
    a.seqlens = seqlens; a.chunks_dev = chunks_dev; a.y = y; a.last_state = last_state;
    a.Lpad = padded_len(L);
    a.ws_B = static_cast<float*>(workspace);
    a.Np = corey_scan::a_np(N);
    a.ws_C = a.ws_B + (size_t)B * a.Np * a.Lpad;
    a.ws_B8 = a.ws_C + (size_t)B * a.Np * a.Lpad;
    a.ws_C8 = a.ws_B8 + (size_t)B * a.Np * a.Lpad;
    a.L = L; a.rows_total = B * D; a.D = (int32_t)D; a.N = (int32_t)N; a.chunk = chunk; a.softplus = delta_softplus ? 1 : 0;
    a.vector_ok = vector_ok ? 1 : 0;
    a.allow_structured = (flags & COREY_SCAN_GENERAL_A) ? 0 : 1;
    a.one_chunk = (flags & COREY_SCAN_ONE_CHUNK) ? 1 : 0;
    a.allow_split = (flags & COREY_SCAN_WHOLE_ROWS) ? 0 : 1;
    a.route = corey_finalise::Args{};
    if (route) {
        if (!route->parts || !route->chunks_out || route->K < 2 || route->K > COREY_MAX_BINS || (route->nh != 1 && route->nh != B))
            return fail(COREY_EINVAL, "%s: route was not filled by corey_route_device_deferred for this batch", who);
        a.route = *route;
        a.chunks_dev = route->chunks_out;                       // written by this call's first kernel, read by its second
        a.one_chunk = route->nh == 1 ? 1 : 0;
    }
    // LDS budget for the per-row arrays (carried state and A): at most 32 rows and 8 KiB each, so that the staging
    // buffers and the rows of a workgroup stay below what a compute unit gives four workgroups (chunks below 64,
    // which would put more than 32 rows into a workgroup, run with idle lanes).
    int rows_cap = (int)(2048 / a.Np);
    a.rows_cap = rows_cap < 1 ? 1 : (rows_cap > 32 ? 32 : rows_cap);
    // a lane addresses its row inside a group by a 32-bit byte offset from the group's first row
    const int64_t row_bytes = L * (int64_t)esz;
    if (row_bytes >= ((int64_t)1 << 31)) return fail(COREY_ESHAPE, "%s: a row of %lld bytes exceeds the kernels' 2 GiB", who, (long long)row_bytes);
    const int64_t fit = (((int64_t)1 << 32) - 1) / row_bytes;
    if (a.rows_cap > fit) a.rows_cap = (int)fit;

    corey_scan::LaunchPlan p;
    a.d16 = corey_scan::plan_d16(B, D, chunk, a.rows_cap);
    a.klo = corey_scan::plan_klo(B, D, chunk, a.d16);
    a.split = corey_scan::plan_split(B, D, (int)N, chunk, a.d16, a.klo, a.allow_split);
    p.chunk = chunk;
    p.routed = a.chunks_dev != nullptr;
    p.B = B; p.D = D; p.N = N;
    p.stream = static_cast<hipStream_t>(hip_stream);
    if (dt == COREY_F32) corey_scan::launch_scan_f32(a, p);
    else if (dt == COREY_F16) corey_scan::launch_scan_f16(a, p);
    else corey_scan::launch_scan_bf16(a, p);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return corey::hip_fail(e, "selective_scan_fwd launch");
    return COREY_OK;
}

}  // namespace

extern "C" int selective_scan_fwd(const void* u, const void* delta, const float* A, const void* Bm, const void* Cm,
                                  const float* Dv, const void* z, const float* delta_bias, int delta_softplus,
                                  const float* h0, const int32_t* seqlens, int32_t chunk, const int32_t* chunks_dev,
                                  void* y, float* last_state, corey_dtype dt, int64_t B, int64_t D, int64_t N, int64_t L,
                                  uint32_t flags, void* workspace, size_t workspace_bytes, void* hip_stream)
{
    return scan_impl("selective_scan_fwd", u, delta, A, Bm, Cm, Dv, z, delta_bias, delta_softplus, h0, seqlens, chunk, chunks_dev, nullptr,
                     y, last_state, dt, B, D, N, L, flags, workspace, workspace_bytes, hip_stream);
}

extern "C" int selective_scan_fwd_routed(const void* u, const void* delta, const float* A, const void* Bm, const void* Cm,
                                         const float* Dv, const void* z, const float* delta_bias, int delta_softplus,
                                         const float* h0, const int32_t* seqlens, int32_t chunk, const corey_deferred_route* route,
                                         void* y, float* last_state, corey_dtype dt, int64_t B, int64_t D, int64_t N, int64_t L,
                                         uint32_t flags, void* workspace, size_t workspace_bytes, void* hip_stream)
{
    if (!route) return corey::fail(COREY_ENULL, "selective_scan_fwd_routed: route is required");
    if (flags & COREY_SCAN_ONE_CHUNK) return corey::fail(COREY_EINVAL, "selective_scan_fwd_routed: COREY_SCAN_ONE_CHUNK follows from the route");
    corey_finalise::Args fa;
    memcpy(&fa, route, sizeof(fa));
    return scan_impl("selective_scan_fwd_routed", u, delta, A, Bm, Cm, Dv, z, delta_bias, delta_softplus, h0, seqlens, chunk, nullptr, &fa,
                     y, last_state, dt, B, D, N, L, flags, workspace, workspace_bytes, hip_stream);
}
