// Error text, contexts (dry-run flag, asynchronous status words) and the small host-only entry points.
#include <cmath>
#include <cstdarg>
#include <new>

#include "cr_common.h"

namespace cr {

static thread_local char g_err[512] = "";
static thread_local cr_ctx *g_current = nullptr;      // the calling thread's current context, or none

void set_error(const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}

bool dry_run() { return g_current != nullptr && (g_current->flags & CR_CTX_DRY_RUN) != 0; }
int64_t *async_status() { return (g_current != nullptr && !(g_current->flags & CR_CTX_DRY_RUN)) ? g_current->status : nullptr; }

__global__ void clear_status_kernel(int64_t *status)
{
    if (threadIdx.x < CR_CTX_STATUS_WORDS) status[threadIdx.x] = 0;
}

}  // namespace cr

extern "C" const char *cr_last_error(void) { return cr::g_err; }
extern "C" const char *cr_version(void) { return "commrand-gfx950 0.1"; }

extern "C" cr_status cr_ctx_create(cr_ctx **ctx, int32_t device, uint32_t flags, int64_t *status)
{
    CR_REQUIRE(ctx != nullptr, CR_ERR_INVALID_ARG, "ctx is NULL");
    *ctx = nullptr;
    CR_REQUIRE(device >= 0, CR_ERR_INVALID_ARG, "device = %d must not be negative", device);
    CR_REQUIRE((flags & ~CR_CTX_DRY_RUN) == 0, CR_ERR_INVALID_ARG, "unknown context flags 0x%x", flags);
    CR_REQUIRE((reinterpret_cast<uintptr_t>(status) & 7u) == 0, CR_ERR_INVALID_ARG, "status must be 8-byte aligned");
    cr_ctx *c = new (std::nothrow) cr_ctx{device, flags, status};
    CR_REQUIRE(c != nullptr, CR_ERR_INVALID_ARG, "out of host memory");
    *ctx = c;
    return CR_OK;
}

extern "C" cr_status cr_ctx_destroy(cr_ctx *ctx)
{
    if (ctx == nullptr) return CR_OK;
    if (cr::g_current == ctx) cr::g_current = nullptr;
    delete ctx;
    return CR_OK;
}

extern "C" cr_status cr_ctx_make_current(cr_ctx *ctx)
{
    cr::g_current = ctx;
    return CR_OK;
}

extern "C" cr_status cr_ctx_poll_error(cr_ctx *ctx, int64_t *required, int32_t clear, void *stream)
{
    CR_REQUIRE(ctx != nullptr, CR_ERR_INVALID_ARG, "ctx is NULL");
    if (required) *required = 0;
    if ((ctx->flags & CR_CTX_DRY_RUN) || ctx->status == nullptr) return CR_OK;
    hipStream_t s = static_cast<hipStream_t>(stream);
    int64_t words[CR_CTX_STATUS_WORDS] = {0, 0};
    CR_HIP_CHECK(hipMemcpyAsync(words, ctx->status, sizeof(words), hipMemcpyDeviceToHost, s));
    CR_HIP_CHECK(hipStreamSynchronize(s));
    if (words[0] == 0) return CR_OK;
    if (required) *required = words[1];
    if (clear) {
        hipLaunchKernelGGL(cr::clear_status_kernel, dim3(1), dim3(64), 0, s, ctx->status);
        CR_LAUNCH_CHECK();
    }
    cr::set_error("a sampled block did not fit its arrays (status 0x%llx): %s; the affected blocks carry a non-zero CR_HDR_STATUS and "
                  "must not be used", (unsigned long long)words[0],
                  (words[0] & CR_ASYNC_FRONTIER_OVERFLOW) ? "a frontier needs more entries than cap_src (see `required`)"
                                                          : "a de-duplication table ran full");
    return CR_ERR_ASYNC_OVERFLOW;
}

extern "C" int32_t cr_mix_count_from_percent(double k_percent, int32_t n_comm_in_train)
{
    if (!(k_percent >= 0.0) || n_comm_in_train < 1) return 1;
    const double m = std::floor(k_percent * (double)n_comm_in_train / 100.0 + 0.5);
    if (m < 1.0) return 1;
    if (m > (double)n_comm_in_train) return n_comm_in_train;
    return (int32_t)m;
}
