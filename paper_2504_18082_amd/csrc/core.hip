// Error text, dry-run switch and the small host-only entry points.
#include <atomic>
#include <cmath>
#include <cstdarg>

#include "cr_common.h"

namespace cr {

static thread_local char g_err[512] = "";
static std::atomic<int> g_dry{0};

void set_error(const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}

bool dry_run() { return g_dry.load(std::memory_order_relaxed) != 0; }

}  // namespace cr

extern "C" const char *cr_last_error(void) { return cr::g_err; }
extern "C" const char *cr_version(void) { return "commrand-gfx950 0.1"; }
extern "C" void cr_set_dry_run(int on) { cr::g_dry.store(on ? 1 : 0, std::memory_order_relaxed); }

extern "C" int32_t cr_mix_count_from_percent(double k_percent, int32_t n_comm_in_train)
{
    if (!(k_percent >= 0.0) || n_comm_in_train < 1) return 1;
    const double m = std::floor(k_percent * (double)n_comm_in_train / 100.0 + 0.5);
    if (m < 1.0) return 1;
    if (m > (double)n_comm_in_train) return n_comm_in_train;
    return (int32_t)m;
}
