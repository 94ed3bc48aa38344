// Version, status strings and option defaults.
#include "common.h"

extern "C" int asteria_version(void) { return 100; }

extern "C" const char *asteria_status_string(asteria_status s)
{
    switch (s) {
        case ASTERIA_OK: return "ok";
        case ASTERIA_INVALID_ARG: return "invalid argument";
        case ASTERIA_UNSUPPORTED: return "unsupported";
        case ASTERIA_WORKSPACE_TOO_SMALL: return "workspace too small";
        case ASTERIA_HIP_ERROR: return "HIP runtime error";
    }
    return "unknown status";
}

extern "C" void asteria_root_opts_default(asteria_root_opts *o)
{
    if (!o) return;
    o->max_iters = 40;
    o->fp64_iters = -1;
    o->power_iters = 256;
    o->schedule = 0;
    o->stop_resid = 1e-2f;
    o->power_tol = 1e-3f;
    o->lambda_margin = 0.01f;
    o->reserved = 0;
}
