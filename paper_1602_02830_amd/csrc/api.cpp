// Version, status strings and size helpers of the C ABI.
#include "bnn.h"

extern "C" int bnn_version(void) { return BNN_VERSION; }

extern "C" const char* bnn_status_string(int status) {
    switch (status) {
        case BNN_OK: return "ok";
        case BNN_ERR_INVALID_ARG: return "invalid argument";
        case BNN_ERR_ALIGNMENT: return "misaligned pointer or leading dimension";
        case BNN_ERR_UNSUPPORTED: return "unsupported configuration";
        case BNN_ERR_LAUNCH: return "kernel launch failed";
        default: return "unknown status";
    }
}

extern "C" int64_t bnn_words_per_row(int64_t K) { return K < 0 ? -1 : (K + 31) / 32; }
