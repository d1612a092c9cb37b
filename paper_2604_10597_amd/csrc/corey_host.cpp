// Host-only part of libcorey: error reporting, the scheduler policy and the chunk rule (Eq. 2).
#include <cmath>
#include <cstdarg>
#include <cstdio>

#include "corey_internal.h"

namespace corey {

static thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

void clear_error() { g_err[0] = '\0'; }

}  // namespace corey

using corey::fail;
using corey::is_pow2;

extern "C" const char* corey_last_error(void) { return corey::g_err; }

extern "C" const char* corey_version(void) { return "0.1"; }

extern "C" int corey_policy_default(corey_policy* p)
{
    if (!p) return fail(COREY_ENULL, "corey_policy_default: p is NULL");
    p->mode = 0;
    p->c_min = 64;
    p->c_max = 2048;
    p->h_ref_scale = 1.0;
    p->short_len = 50;
    p->short_chunk = 128;
    p->long_chunk = 512;
    p->static_chunk = 512;
    p->safe_chunk = 512;
    p->guard_buckets = 2;
    return COREY_OK;
}

extern "C" int corey_ema_update(double lambda, double* state, double H)
{
    if (!state) return fail(COREY_ENULL, "corey_ema_update: state is NULL");
    if (!(lambda >= 0.0 && lambda < 1.0)) return fail(COREY_EINVAL, "corey_ema_update: lambda = %g outside [0, 1)", lambda);
    if (std::isnan(H)) return COREY_OK;
    *state = std::isnan(*state) ? H : lambda * *state + (1.0 - lambda) * H;
    return COREY_OK;
}

namespace {

int log2_of_pow2(int64_t v)
{
    int e = 0;
    while ((int64_t(1) << e) < v) ++e;
    return e;
}

// Eq. 2: the power of two nearest (in log2) to c_min + r (c_max - c_min), clipped to [c_min, c_max].
int64_t entropy_rule(double r, const corey_policy& p)
{
    double re = r * p.h_ref_scale;
    re = re < 0.0 ? 0.0 : (re > 1.0 ? 1.0 : re);
    const double target = double(p.c_min) + re * double(p.c_max - p.c_min);
    const double k = std::floor(std::log2(target) + 0.5);
    int64_t c = int64_t(1) << int(k);
    if (c < p.c_min) c = p.c_min;
    if (c > p.c_max) c = p.c_max;
    return c;
}

}  // namespace

extern "C" int corey_select_chunk(double r, int64_t L, const corey_policy* p, int32_t* chunk_out)
{
    if (!p || !chunk_out) return fail(COREY_ENULL, "corey_select_chunk: NULL policy or output");
    if (L < 1) return fail(COREY_EINVAL, "corey_select_chunk: L = %lld < 1", (long long)L);
    if (!is_pow2(p->c_min) || !is_pow2(p->c_max) || p->c_min > p->c_max)
        return fail(COREY_EINVAL, "corey_select_chunk: c_min = %d, c_max = %d must be powers of two, c_min <= c_max",
                    p->c_min, p->c_max);

    const bool short_seq = L <= p->short_len;
    int64_t c = 0;
    switch (p->mode) {
    case 3:
        if (!is_pow2(p->static_chunk)) return fail(COREY_EINVAL, "corey_select_chunk: static_chunk = %d", p->static_chunk);
        *chunk_out = p->static_chunk;
        return COREY_OK;
    case 2:
        if (!is_pow2(p->short_chunk) || !is_pow2(p->long_chunk))
            return fail(COREY_EINVAL, "corey_select_chunk: table chunks %d / %d", p->short_chunk, p->long_chunk);
        *chunk_out = short_seq ? p->short_chunk : p->long_chunk;
        return COREY_OK;
    case 1:
        if (short_seq) {
            if (!is_pow2(p->short_chunk)) return fail(COREY_EINVAL, "corey_select_chunk: short_chunk = %d", p->short_chunk);
            *chunk_out = p->short_chunk;
            return COREY_OK;
        }
        [[fallthrough]];
    case 0:
    case 4:
        if (std::isnan(r)) return fail(COREY_ENONFINITE, "corey_select_chunk: r is NaN");
        c = entropy_rule(r, *p);
        if (p->mode == 4) {
            if (!is_pow2(p->safe_chunk) || p->guard_buckets < 0)
                return fail(COREY_EINVAL, "corey_select_chunk: safe_chunk = %d, guard_buckets = %d", p->safe_chunk,
                            p->guard_buckets);
            const int away = std::abs(log2_of_pow2(c) - log2_of_pow2(p->safe_chunk));
            if (away < p->guard_buckets) c = p->safe_chunk;
        }
        break;
    default:
        return fail(COREY_EINVAL, "corey_select_chunk: unknown mode %d", p->mode);
    }
    // a tile longer than the sequence cannot be filled: cap at the next power of two >= L
    int64_t cap = 1;
    while (cap < L) cap <<= 1;
    if (cap < p->c_min) cap = p->c_min;
    if (c > cap) c = cap;
    *chunk_out = int32_t(c);
    return COREY_OK;
}
