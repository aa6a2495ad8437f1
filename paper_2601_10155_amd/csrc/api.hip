// Error reporting, version and the argument checks shared by the entry points.
#include <cstdarg>
#include <cstdio>

#include "common.h"

namespace lookat {

static thread_local char g_err[512] = "";

int fail(int status, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return status;
}

void clear_error() { g_err[0] = '\0'; }

int check_shape(const lookat_shape *s)
{
    if (!s)
        return fail(LOOKAT_ERR_NULL, "shape is NULL");
    if (s->B <= 0 || s->H <= 0 || s->d_k <= 0 || s->m <= 0)
        return fail(LOOKAT_ERR_SHAPE, "B, H, d_k and m must be positive (B=%d H=%d d_k=%d m=%d)", s->B, s->H,
                    s->d_k, s->m);
    if (s->K != kCentroids)
        return fail(LOOKAT_ERR_SHAPE, "K must be 256 (one byte per code), got %d", s->K);
    if (s->d_k % s->m)
        return fail(LOOKAT_ERR_SHAPE, "m=%d does not divide d_k=%d", s->m, s->d_k);
    if (s->d_k % 8 || s->d_k > 256)
        return fail(LOOKAT_ERR_UNSUPPORTED, "d_k=%d: need a multiple of 8 in [8,256]", s->d_k);
    if (s->m > 32)
        return fail(LOOKAT_ERR_UNSUPPORTED, "m=%d: at most 32 subspaces are supported", s->m);
    return LOOKAT_OK;
}

int check_launch(const char *what)
{
    hipError_t e = hipGetLastError();
    if (e != hipSuccess)
        return fail(LOOKAT_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
    return LOOKAT_OK;
}

}  // namespace lookat

extern "C" const char *lookat_last_error(void) { return lookat::g_err; }

extern "C" int lookat_version(void) { return 100; }
