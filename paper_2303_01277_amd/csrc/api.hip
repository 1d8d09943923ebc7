// Status / error plumbing of the C ABI.
#include <stdarg.h>
#include <string.h>

#include "common.hpp"
#include "rounding.hpp"

namespace sylvie {

static thread_local char g_err[512] = "";

void set_error(const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}

int32_t fail(int32_t code, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

// Device-resident seed offset of this thread's quantizing calls (sylvie_seed_offset_source).
static thread_local const uint64_t *g_seed_offset = nullptr;

CallKey make_call_key(uint64_t seed, uint32_t stream_id)
{
    return CallKey{call_key(seed, stream_id), stream_id, seed, g_seed_offset};
}

}  // namespace sylvie

extern "C" int32_t sylvie_seed_offset_source(const uint64_t *offset)
{
    if (offset && !sylvie::aligned(offset, 8))
        return sylvie::fail(SYLVIE_ERR_BAD_ALIGNMENT, "sylvie_seed_offset_source: the offset needs 8-byte alignment");
    sylvie::g_seed_offset = offset;
    return SYLVIE_OK;
}

extern "C" int32_t sylvie_version(void) { return 100; }

extern "C" const char *sylvie_status_string(int32_t status)
{
    switch (status) {
    case SYLVIE_OK: return "ok";
    case SYLVIE_ERR_INVALID_ARG: return "invalid argument";
    case SYLVIE_ERR_BAD_ALIGNMENT: return "bad alignment";
    case SYLVIE_ERR_HIP: return "HIP runtime error";
    case SYLVIE_ERR_UNIMPLEMENTED: return "not implemented";
    case SYLVIE_ERR_WORKSPACE: return "workspace too small";
    default: return "unknown status";
    }
}

extern "C" const char *sylvie_last_error(void) { return sylvie::g_err; }

extern "C" int64_t sylvie_wire_row_words(int32_t d) { return (static_cast<int64_t>(d) + 63) / 64 + 1; }
