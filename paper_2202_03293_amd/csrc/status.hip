#include "lg_common.hpp"

extern "C" int lg_version(void) { return 100; }

extern "C" const char* lg_status_string(int status) {
    switch (status) {
        case LG_OK: return "LG_OK";
        case LG_ERR_INVALID_ARG: return "LG_ERR_INVALID_ARG";
        case LG_ERR_UNSUPPORTED: return "LG_ERR_UNSUPPORTED";
        case LG_ERR_WORKSPACE: return "LG_ERR_WORKSPACE";
        case LG_ERR_RUNTIME: return "LG_ERR_RUNTIME";
        default: return "LG_ERR_UNKNOWN";
    }
}

extern "C" int64_t lg_conv_out_extent(int64_t in, int64_t k, int64_t stride, int64_t dilation) {
    if (in <= 0 || k <= 0 || stride <= 0 || dilation <= 0) return 0;
    const int64_t span = dilation * (k - 1) + 1;
    return span > in ? 0 : (in - span) / stride + 1;
}
