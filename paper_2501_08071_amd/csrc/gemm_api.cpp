// C ABI of the fused GEMM + LeakyReLU (include/gemm.h): argument checks, then one launch.
#include <cmath>
#include <cstdint>

#include "../../include/gemm.h"
#include "gemm_launch.h"

namespace {
bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
bool shape_ok(int batch, int M, int N, int K) {
    if (batch < 0 || M < 0 || N < 0 || K < 0) return false;
    const double lim = 2147483648.0;   // 32-bit offsets inside one matrix
    return (double)M * K <= lim && (double)K * N <= lim && (double)M * N <= lim && (double)batch <= 65535.0;
}
}  // namespace

extern "C" int gemm_leakyrelu_fwd(const void* a, const void* b, void* c, int batch, int M, int N, int K, float slope,
                                  int dtype, void* stream) {
    if (dtype != GEMM_F16 && dtype != GEMM_BF16) return GEMM_ERR_DTYPE;
    if (!shape_ok(batch, M, N, K)) return GEMM_ERR_SHAPE;
    if (std::isnan(slope) || std::isinf(slope)) return GEMM_ERR_SLOPE;
    if (batch == 0 || M == 0 || N == 0) return GEMM_OK;
    if (c == nullptr || (K > 0 && (a == nullptr || b == nullptr))) return GEMM_ERR_NULL;
    if (!aligned16(a) || !aligned16(b) || !aligned16(c)) return GEMM_ERR_ALIGN;
    const GemmLaunch g{a, b, c, batch, M, N, K, slope, dtype, stream};
    return gemm_launch(g) == hipSuccess ? GEMM_OK : GEMM_ERR_LAUNCH;
}

extern "C" int gemm_path(int batch, int M, int N, int K, int dtype) {
    if ((dtype != GEMM_F16 && dtype != GEMM_BF16) || !shape_ok(batch, M, N, K)) return 0;
    return gemm_path_of(batch, M, N, K);
}

extern "C" const char* gemm_status_str(int status) {
    switch (status) {
        case GEMM_OK: return "ok";
        case GEMM_ERR_NULL: return "a, b or c is a null pointer";
        case GEMM_ERR_SHAPE: return "batch (at most 65535), M, N, K must be >= 0 and every matrix at most 2^31 elements";
        case GEMM_ERR_DTYPE: return "dtype must be GEMM_F16 (0) or GEMM_BF16 (1)";
        case GEMM_ERR_SLOPE: return "slope must be finite";
        case GEMM_ERR_ALIGN: return "every pointer must be 16-byte aligned";
        case GEMM_ERR_LAUNCH: return "the HIP runtime refused the kernel launch";
        default: return "unknown status";
    }
}
