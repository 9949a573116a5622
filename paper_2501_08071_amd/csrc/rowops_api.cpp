// C ABI of the row kernels (include/rowops.h): argument checks, then one launch.
#include <cmath>
#include <cstdint>

#include "../../include/rowops.h"
#include "rowops_launch.h"

namespace {

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int check_common(const void* x, const void* y, long long n_rows, int n, int dtype) {
    if (dtype != ROWOPS_F16 && dtype != ROWOPS_BF16) return ROWOPS_ERR_DTYPE;
    if (n_rows < 0 || n <= 0 || n > (1 << 24)) return ROWOPS_ERR_SHAPE;
    if ((double)n_rows * (double)n > 1099511627776.0) return ROWOPS_ERR_SHAPE;
    if (n_rows > 0 && (x == nullptr || y == nullptr)) return ROWOPS_ERR_NULL;
    if (!aligned16(x) || !aligned16(y)) return ROWOPS_ERR_ALIGN;
    return ROWOPS_OK;
}

}  // namespace

extern "C" int softmax_rows_fwd(const void* x, void* y, long long n_rows, int n_cols, int dtype, void* stream) {
    const int st = check_common(x, y, n_rows, n_cols, dtype);
    if (st != ROWOPS_OK) return st;
    if (n_rows == 0) return ROWOPS_OK;
    const RowopLaunch a{0, x, nullptr, y, n_rows, n_cols, 0.f, dtype, stream};
    return rowop_launch(a) == hipSuccess ? ROWOPS_OK : ROWOPS_ERR_LAUNCH;
}

extern "C" int rmsnorm_fwd(const void* x, const void* w, void* y, long long n_rows, int d, float eps, int dtype,
                           void* stream) {
    const int st = check_common(x, y, n_rows, d, dtype);
    if (st != ROWOPS_OK) return st;
    if (!(eps >= 0.f) || std::isinf(eps)) return ROWOPS_ERR_EPS;
    if (n_rows == 0) return ROWOPS_OK;
    if (w == nullptr) return ROWOPS_ERR_NULL;
    if (!aligned16(w)) return ROWOPS_ERR_ALIGN;
    const RowopLaunch a{1, x, w, y, n_rows, d, eps, dtype, stream};
    return rowop_launch(a) == hipSuccess ? ROWOPS_OK : ROWOPS_ERR_LAUNCH;
}

extern "C" int rowops_path(int op, int row_len, int dtype) {
    if ((op != 0 && op != 1) || (dtype != ROWOPS_F16 && dtype != ROWOPS_BF16)) return 0;
    if (row_len <= 0 || row_len > (1 << 24)) return 0;
    return rowop_path_of(row_len);
}

extern "C" const char* rowops_status_str(int status) {
    switch (status) {
        case ROWOPS_OK: return "ok";
        case ROWOPS_ERR_NULL: return "x, y (or w) is a null pointer";
        case ROWOPS_ERR_SHAPE: return "n_rows must be >= 0, the row length 1 .. 2^24, the tensor at most 2^40 elements";
        case ROWOPS_ERR_DTYPE: return "dtype must be ROWOPS_F16 (0) or ROWOPS_BF16 (1)";
        case ROWOPS_ERR_EPS: return "eps must be finite and >= 0";
        case ROWOPS_ERR_ALIGN: return "every pointer must be 16-byte aligned";
        case ROWOPS_ERR_LAUNCH: return "the HIP runtime refused the kernel launch";
        default: return "unknown status";
    }
}
