// libshiftadd: error reporting, version, row-selection validation.
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include "common.h"

namespace sa {

static thread_local char g_err[512] = "";

int fail(int code, const char *fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

void clear_error() { g_err[0] = '\0'; }

int check_launch(const char *what) {
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(SA_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
    return SA_OK;
}

__global__ void zero_kernel(uint32_t *p, size_t n) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0u;
}

int launch_zero(void *p, size_t bytes, hipStream_t st) {
    const size_t n = bytes / 4;
    if (n == 0) return SA_OK;
    const size_t blocks = (n + 255) / 256;
    if (blocks >= (1ull << 31)) return fail(SA_ERR_SHAPE, "zero fill too large");
    zero_kernel<<<dim3((unsigned)blocks), dim3(256), 0, st>>>(static_cast<uint32_t *>(p), n);
    return check_launch("zero fill");
}

int validate_rows(const sa_rows *rows, RowSel *out) {
    SA_REQUIRE(rows != nullptr, SA_ERR_INVALID, "rows descriptor is NULL");
    SA_REQUIRE(rows->max_rows >= 0, SA_ERR_INVALID, "max_rows < 0");
    SA_REQUIRE(rows->max_rows < (1L << 31), SA_ERR_SHAPE, "max_rows >= 2^31");
    if (rows->counts_or_null != nullptr) {
        SA_REQUIRE(rows->rows_or_null != nullptr, SA_ERR_INVALID,
                   "counts given without the perm list");
        SA_REQUIRE(rows->expert >= 0 && rows->expert < 8, SA_ERR_INVALID, "expert out of range");
    }
    out->rows = rows->rows_or_null;
    out->counts = rows->counts_or_null;
    out->expert = rows->expert;
    out->max_rows = rows->max_rows;
    return SA_OK;
}

}  // namespace sa

extern "C" int sa_version(void) { return 100; }

extern "C" const char *sa_last_error(void) { return sa::g_err; }
