// lp_strerror: text for the status codes of the C ABI; lp_abi_version: the header version the library was built with.
#include "lp.h"

extern "C" const char *lp_strerror(int status) {
    switch (status) {
        case LP_OK: return "ok";
        case LP_ERR_INVALID_ARG: return "invalid argument (null pointer, negative size, misaligned matrix or bad layer count)";
        case LP_ERR_OUT_OF_RANGE: return "node id outside [0, n_nodes) or size beyond 32-bit indexing";
        case LP_ERR_WORKSPACE: return "workspace missing or smaller than *_workspace_bytes()";
        case LP_ERR_UNSUPPORTED: return "unsupported dtype or a width that is not a multiple of 4 (or above 1024)";
        case LP_ERR_HIP: return "HIP runtime error";
        default: return "unknown status";
    }
}

extern "C" int lp_abi_version(void) { return LP_ABI_VERSION; }
