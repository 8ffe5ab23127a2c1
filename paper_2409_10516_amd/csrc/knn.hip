#include "common.h"
ra_status ra_launch_knn(const void*, const void*, ra_dtype, int, int, int, int64_t, int64_t, int,
                        hipStream_t, int32_t*) {
    RA_FAIL(RA_EUNSUP, "ra_knn not built yet");
}
