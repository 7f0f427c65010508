// Handle lifecycle, error reporting.
#include "ops.h"

namespace alt {

alt_status_t fail(alt_handle_t h, alt_status_t s, const char *fmt, ...)
{
    if (h) {
        char buf[512];
        va_list ap;
        va_start(ap, fmt);
        std::vsnprintf(buf, sizeof buf, fmt, ap);
        va_end(ap);
        h->last_error = buf;
    }
    return s;
}

}  // namespace alt

extern "C" {

alt_status_t alt_create(alt_handle_t *out)
{
    if (!out) return ALT_INVALID_ARG;
    alt_context *c = new alt_context();
    int n = 0;
    if (hipGetDeviceCount(&n) == hipSuccess && n > 0) {
        int dev = 0;
        hipDeviceProp_t prop;
        if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess) {
            c->device = dev;
            c->has_gpu = true;
            c->compute_units = prop.multiProcessorCount;
            c->clock_mhz = prop.clockRate / 1000;
            c->arch = prop.gcnArchName;
            size_t colon = c->arch.find(':');
            if (colon != std::string::npos) c->arch.resize(colon);
        }
    } else {
        (void)hipGetLastError();
    }
    if (!c->has_gpu) c->arch = "none";
    else {
        void *ws = nullptr;
        (void)alt::static_scratch(&ws);            // address of alt_conv2d_static's array on this device (kept per device)
    }
    *out = c;
    return ALT_OK;
}

alt_status_t alt_destroy(alt_handle_t h)
{
    if (!h) return ALT_INVALID_ARG;
    alt::launch_memo_free(h);
    alt::transform_memo_free(h);
    delete h;
    return ALT_OK;
}

const char *alt_last_error(alt_handle_t h) { return h ? h->last_error.c_str() : "null handle"; }

const char *alt_status_string(alt_status_t s)
{
    switch (s) {
        case ALT_OK: return "ok";
        case ALT_INVALID_ARG: return "invalid argument";
        case ALT_INVALID_LAYOUT: return "invalid layout";
        case ALT_SHAPE_MISMATCH: return "shape mismatch";
        case ALT_UNSUPPORTED: return "unsupported";
        case ALT_WORKSPACE_TOO_SMALL: return "workspace too small";
        case ALT_HIP_ERROR: return "HIP error";
        case ALT_NOT_TUNED: return "not tuned";
    }
    return "unknown status";
}

const char *alt_version(void) { return "0.1"; }

}  // extern "C"
