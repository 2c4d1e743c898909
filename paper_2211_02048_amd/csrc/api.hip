// Error reporting and the argument checks shared by the entry points.
#include "common.h"

namespace sige {

static thread_local char g_err[512] = "";
int g_knobs[SIGE_KNOB_COUNT] = {-1, -1, -1, -1, -1, -1, -1, -1, -1, -1, -1, -1, -1};
static_assert(SIGE_KNOB_COUNT == 13, "one initialiser per knob");

int fail(int code, const char* fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

void clear_error() { g_err[0] = '\0'; }

int check_geom(const sige_geom* g, const char* who, int* tile_h, int* tile_w)
{
    SIGE_REQUIRE(g != nullptr, SIGE_ERR_INVALID_ARG, "%s: geometry is NULL", who);
    SIGE_REQUIRE(g->H_in > 0 && g->W_in > 0 && g->H_out > 0 && g->W_out > 0, SIGE_ERR_INVALID_ARG,
                 "%s: non-positive spatial size", who);
    SIGE_REQUIRE(g->block_h > 0 && g->block_w > 0, SIGE_ERR_INVALID_ARG,
                 "%s: block size must be positive (got %d x %d)", who, g->block_h, g->block_w);
    SIGE_REQUIRE(g->k > 0 && (g->k & 1) == 1, SIGE_ERR_INVALID_ARG,
                 "%s: kernel size must be odd and positive (got %d)", who, g->k);
    SIGE_REQUIRE(g->stride >= 1 && g->pad >= 0, SIGE_ERR_INVALID_ARG,
                 "%s: stride must be >= 1 and pad >= 0", who);
    SIGE_REQUIRE(g->H_in + 2 * g->pad >= g->k && g->W_in + 2 * g->pad >= g->k, SIGE_ERR_INVALID_ARG,
                 "%s: kernel larger than the padded input", who);
    SIGE_REQUIRE(g->H_out == (g->H_in + 2 * g->pad - g->k) / g->stride + 1 &&
                     g->W_out == (g->W_in + 2 * g->pad - g->k) / g->stride + 1,
                 SIGE_ERR_INVALID_ARG, "%s: H_out/W_out do not match (H_in + 2*pad - k)/stride + 1", who);
    SIGE_REQUIRE(g->block_h <= 4096 && g->block_w <= 4096 && g->k <= 15 && g->stride <= 8,
                 SIGE_ERR_UNSUPPORTED, "%s: block, kernel or stride beyond the supported range", who);
    if (tile_h) *tile_h = (g->block_h - 1) * g->stride + g->k;
    if (tile_w) *tile_w = (g->block_w - 1) * g->stride + g->k;
    return SIGE_OK;
}

int check_blocks(const int32_t* count, int32_t max_blocks, int32_t n_blocks, const char* who,
                 int* launch_blocks)
{
    SIGE_REQUIRE(max_blocks >= 0, SIGE_ERR_INVALID_ARG, "%s: max_blocks is negative", who);
    SIGE_REQUIRE(n_blocks >= -1, SIGE_ERR_INVALID_ARG, "%s: n_blocks must be >= -1", who);
    SIGE_REQUIRE(n_blocks <= max_blocks, SIGE_ERR_CAPACITY,
                 "%s: n_blocks (%d) exceeds max_blocks (%d)", who, n_blocks, max_blocks);
    SIGE_REQUIRE(n_blocks >= 0 || count != nullptr, SIGE_ERR_INVALID_ARG,
                 "%s: count is NULL and no host n_blocks was given", who);
    *launch_blocks = n_blocks >= 0 ? n_blocks : max_blocks;
    return SIGE_OK;
}

}  // namespace sige

extern "C" const char* sige_last_error(void) { return sige::g_err; }
extern "C" int sige_version(void) { return 2; }

extern "C" int sige_set_knob(sige_knob k, int32_t value)
{
    sige::clear_error();
    SIGE_REQUIRE((int)k >= 0 && (int)k < SIGE_KNOB_COUNT, SIGE_ERR_INVALID_ARG, "sige_set_knob: unknown knob %d", (int)k);
    sige::g_knobs[k] = value < 0 ? -1 : value;
    return SIGE_OK;
}

extern "C" int32_t sige_get_knob(sige_knob k)
{
    return ((int)k >= 0 && (int)k < SIGE_KNOB_COUNT) ? sige::g_knobs[k] : -1;
}
