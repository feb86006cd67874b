// Error string, options and device queries shared by the entry points.
#include "common.h"
#include <cstdio>
#include <mutex>

namespace easgd {

static thread_local char g_err[512] = "";

int fail(int code, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

void clear_error() { g_err[0] = '\0'; }

int num_cus()
{
    static int cus[64] = {0};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
    if (cus[dev] == 0) {
        int n = 0;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
        cus[dev] = n;
    }
    return cus[dev];
}

Options &options()
{
    static Options o;
    return o;
}

UpdateShape update_shape(size_t N, bool wide)
{
    const Options &opt = options();
    const size_t n4 = N / 4, cus = (size_t)num_cus();
    long g = opt.update_groups;
    if (g == 0) g = 4;
    (void)wide;
    // fewer groups per thread for small N, so that the grid still covers the chip several times
    while (g > 1 && n4 / ((size_t)g * 256) < 4 * cus) g /= 2;
    const long layout = opt.update_layout;
    UpdateShape sh;
    sh.groups = (int)g;
    sh.dies = layout == 1 || (layout == 2 && g >= 4);
    const size_t super = (size_t)8 * g * 256;
    sh.blocks = sh.dies ? 8 * ((n4 + super - 1) / super) : (n4 + (size_t)g * 256 - 1) / ((size_t)g * 256);
    if (sh.blocks == 0) sh.blocks = sh.dies ? 8 : 1;
    if (opt.update_blocks_per_cu > 0) {
        // a persistent grid; a multiple of 8 blocks, so that a block stays on the same die for all its tiles
        const size_t persistent = ((size_t)opt.update_blocks_per_cu * cus + 7) / 8 * 8;
        if (sh.blocks > persistent) sh.blocks = persistent;
    }
    if (sh.blocks > 0x7ffffff8u) sh.blocks = 0x7ffffff8u;    // the kernels' grid-stride loops cover the rest
    return sh;
}

bool update_nontemporal(size_t bytes)
{
    const long v = options().update_nontemporal;
    return v == 2 ? bytes > ((size_t)512 << 20) : v != 0;
}

std::atomic<unsigned long long> &launch_counter()
{
    static std::atomic<unsigned long long> n{0};
    return n;
}

}  // namespace easgd

extern "C" {

const char *easgd_last_error(void) { return easgd::g_err; }

int easgd_version(void) { return 500; }

unsigned long long easgd_launch_count(void) { return easgd::launch_counter().load(std::memory_order_relaxed); }

int easgd_set_option(int option, long value)
{
    easgd::Options &o = easgd::options();
    switch (option) {
    case EASGD_OPT_UPDATE_BLOCKS_PER_CU:
        if (value < 0 || value > 64) return easgd::fail(EASGD_EINVAL, "blocks per CU must be in [0,64], got %ld", value);
        o.update_blocks_per_cu = value;
        return EASGD_OK;
    case EASGD_OPT_UPDATE_NONTEMPORAL:
        if (value < 0 || value > 2) return easgd::fail(EASGD_EINVAL, "nontemporal must be 0, 1 or 2 (chosen per call), got %ld", value);
        o.update_nontemporal = value;
        return EASGD_OK;
    case EASGD_OPT_UPDATE_GROUPS:
        if (value != 0 && value != 1 && value != 2 && value != 4 && value != 8)
            return easgd::fail(EASGD_EINVAL, "groups must be 0 (chosen per call), 1, 2, 4 or 8, got %ld", value);
        o.update_groups = value;
        return EASGD_OK;
    case EASGD_OPT_GEMM_TILE:
        if (value < 0 || value > 4) return easgd::fail(EASGD_EINVAL, "gemm tile must be in [0,4], got %ld", value);
        o.gemm_tile = value;
        return EASGD_OK;
    case EASGD_OPT_ROUND_OVERLAP:
        if (value < 0 || value > 3) return easgd::fail(EASGD_EINVAL, "round overlap must be in [0,3], got %ld", value);
        o.round_overlap = value;
        return EASGD_OK;
    case EASGD_OPT_GEMM_XCD:
        if (value < 0 || value > 3) return easgd::fail(EASGD_EINVAL, "gemm xcd must be in [0,3], got %ld", value);
        o.gemm_xcd = value;
        return EASGD_OK;
    case EASGD_OPT_GEMM_PAIR:
        if (value != 0 && value != 1) return easgd::fail(EASGD_EINVAL, "gemm pair must be 0 or 1, got %ld", value);
        o.gemm_pair = value;
        return EASGD_OK;
    case EASGD_OPT_MLP_HEAD:
        if (value != 0 && value != 1) return easgd::fail(EASGD_EINVAL, "mlp head must be 0 or 1, got %ld", value);
        o.mlp_head = value;
        return EASGD_OK;
    case EASGD_OPT_UPDATE_LAYOUT:
        if (value < 0 || value > 2) return easgd::fail(EASGD_EINVAL, "update layout must be 0, 1 or 2, got %ld", value);
        o.update_layout = value;
        return EASGD_OK;
    case EASGD_OPT_ROUND_SINGLE_LAUNCH:
        if (value != 0 && value != 1) return easgd::fail(EASGD_EINVAL, "round single launch must be 0 or 1, got %ld", value);
        o.round_single_launch = value;
        return EASGD_OK;
    case EASGD_OPT_ROUND_SPIN_LIMIT:
        if (value < 0 || value > 0x7fffffffL) return easgd::fail(EASGD_EINVAL, "round spin limit must be in [0, 2^31), got %ld", value);
        o.round_spin_limit = value;
        return EASGD_OK;
    default:
        return easgd::fail(EASGD_EINVAL, "unknown option %d", option);
    }
}

long easgd_get_option(int option)
{
    const easgd::Options &o = easgd::options();
    switch (option) {
    case EASGD_OPT_UPDATE_BLOCKS_PER_CU: return o.update_blocks_per_cu;
    case EASGD_OPT_UPDATE_NONTEMPORAL: return o.update_nontemporal;
    case EASGD_OPT_UPDATE_GROUPS: return o.update_groups;
    case EASGD_OPT_GEMM_TILE: return o.gemm_tile;
    case EASGD_OPT_ROUND_OVERLAP: return o.round_overlap;
    case EASGD_OPT_GEMM_XCD: return o.gemm_xcd;
    case EASGD_OPT_GEMM_PAIR: return o.gemm_pair;
    case EASGD_OPT_MLP_HEAD: return o.mlp_head;
    case EASGD_OPT_UPDATE_LAYOUT: return o.update_layout;
    case EASGD_OPT_ROUND_SINGLE_LAUNCH: return o.round_single_launch;
    case EASGD_OPT_ROUND_SPIN_LIMIT: return o.round_spin_limit;
    default: return -1;
    }
}

}  // extern "C"
