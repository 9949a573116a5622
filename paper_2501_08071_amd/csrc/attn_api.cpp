// C-ABI layer of the gfx950 attention forward: argument validation (no HIP call before every
// check has passed), then one asynchronous kernel launch on the caller's stream.
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>

#include "../../include/attn.h"
#include "attn_launch.h"

namespace {
bool d_supported(int D) { return D == 32 || D == 64 || D == 128; }
bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
}  // namespace

extern "C" int attn_supported(int S, int D, int dtype, int causal) {
    (void)causal;
    return (S >= 1 && d_supported(D) && (dtype == ATTN_F16 || dtype == ATTN_BF16)) ? 1 : 0;
}

extern "C" const char* attn_status_str(int status) {
    switch (status) {
        case ATTN_OK: return "ok";
        case ATTN_ERR_NULL: return "q, k, v or o is a null pointer";
        case ATTN_ERR_SHAPE: return "B, H, S and D must be positive (and a tensor at most 2^40 elements)";
        case ATTN_ERR_DTYPE: return "dtype must be ATTN_F16 (0) or ATTN_BF16 (1)";
        case ATTN_ERR_SCALE: return "scale must be finite";
        case ATTN_ERR_UNSUPPORTED: return "no kernel instance for this head dimension (D must be 32, 64 or 128)";
        case ATTN_ERR_ALIGN: return "every pointer must be 16-byte aligned";
        case ATTN_ERR_LAUNCH: return "the HIP runtime refused the kernel launch";
        default: return "unknown status";
    }
}

// The names a profiler reports, one string constant per instance (nothing is built at run time).
#define ATTN_STR2(x) #x
#define ATTN_STR(x) ATTN_STR2(x)
#define ATTN_NAME(DT, DD, CZ, NWS) "attn_fwd_kernel<" #DT ", " #DD ", " #CZ ", " NWS ">"
#define ATTN_NAMES_NW(NWS)                                                                              \
    {{{ATTN_NAME(0, 32, false, NWS), ATTN_NAME(0, 32, true, NWS)},                                      \
      {ATTN_NAME(0, 64, false, NWS), ATTN_NAME(0, 64, true, NWS)},                                      \
      {ATTN_NAME(0, 128, false, NWS), ATTN_NAME(0, 128, true, NWS)}},                                   \
     {{ATTN_NAME(1, 32, false, NWS), ATTN_NAME(1, 32, true, NWS)},                                      \
      {ATTN_NAME(1, 64, false, NWS), ATTN_NAME(1, 64, true, NWS)},                                      \
      {ATTN_NAME(1, 128, false, NWS), ATTN_NAME(1, 128, true, NWS)}}}
#if ATTN_NW == 8
#define ATTN_NW_FULL_STR "8"
#define ATTN_NW_HALF_STR "4"
#elif ATTN_NW == 4
#define ATTN_NW_FULL_STR "4"
#define ATTN_NW_HALF_STR "2"
#else
#error "attn_kernel_name: add the strings for this ATTN_NW"
#endif
namespace {
const char* const kKernelNames[2][2][3][2] = {ATTN_NAMES_NW(ATTN_NW_FULL_STR), ATTN_NAMES_NW(ATTN_NW_HALF_STR)};
const char* const kRows64Names[2][2] = {{"attn_fwd_rows64_kernel<0, 128, false>", "attn_fwd_rows64_kernel<0, 128, true>"},
                                        {"attn_fwd_rows64_kernel<1, 128, false>", "attn_fwd_rows64_kernel<1, 128, true>"}};
}  // namespace

extern "C" const char* attn_kernel_name(int B, int H, int S, int D, int dtype, int causal) {
    if (B <= 0 || H <= 0 || !attn_supported(S, D, dtype, causal)) return nullptr;
    if (attn_takes_rows64((long long)B * H, S, D)) return kRows64Names[dtype][causal != 0];
    const int half = attn_pick_nw((long long)B * H, S) == ATTN_NW ? 0 : 1;
    return kKernelNames[half][dtype][D == 32 ? 0 : D == 64 ? 1 : 2][causal != 0];
}

extern "C" int attn_tile_rows(int D, int dtype, int causal) {
    return attn_supported(1, D, dtype, causal) ? ATTN_NW * 32 : 0;
}

extern "C" int attn_launch_rows(int B, int H, int S, int D, int dtype, int causal) {
    if (B <= 0 || H <= 0 || !attn_supported(S, D, dtype, causal)) return 0;
    return 32 * attn_pick_nw((long long)B * H, S);
}

extern "C" int attn_tile_keys(int D, int dtype, int causal) {
    return attn_supported(1, D, dtype, causal) ? attn_block_keys(D) : 0;
}

namespace {
int fwd(const void* q, const void* k, const void* v, void* o, int o16, float* lse, int B, int H, int S, int D, int causal,
        float scale, int dtype, void* stream) {
    if (!q || !k || !v || !o) return ATTN_ERR_NULL;
    if (B <= 0 || H <= 0 || S <= 0 || D <= 0) return ATTN_ERR_SHAPE;
    const long long bh = (long long)B * H;
    if (bh > 0x7fffffffLL || (double)bh * S * D > 1099511627776.0) return ATTN_ERR_SHAPE;
    if (dtype != ATTN_F16 && dtype != ATTN_BF16) return ATTN_ERR_DTYPE;
    if (!std::isfinite(scale)) return ATTN_ERR_SCALE;
    if (!d_supported(D)) return ATTN_ERR_UNSUPPORTED;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o)) return ATTN_ERR_ALIGN;

    AttnLaunch a;
    a.q = q; a.k = k; a.v = v; a.o = o; a.lse = lse;
    a.BH = (int)bh; a.S = S; a.D = D;
    a.causal = causal != 0;
    a.dtype = dtype;
    // |scale| * log2(e), kept off zero: the kernel masks logits with a huge finite number, which has
    // to stay far below the real ones after the multiplication (at 1e-30 every real logit is still 0
    // to fp32, so scale == 0 keeps its meaning)
    a.c = std::fmax(std::fabs(scale) * 1.4426950408889634f, 1e-30f);
    a.qsign = std::signbit(scale) && scale != 0.f ? 0x80008000u : 0u;
    a.o16 = o16;
    a.stream = stream;
    const hipError_t err = attn_launch(a);
    if (err != hipSuccess) {
        if (std::getenv("ATTN_DEBUG")) std::fprintf(stderr, "attn_fwd: launch failed: %s\n", hipGetErrorString(err));
        return ATTN_ERR_LAUNCH;
    }
    return ATTN_OK;
}
}  // namespace

extern "C" int attn_fwd(const void* q, const void* k, const void* v, float* o, float* lse, int B, int H, int S, int D,
                        int causal, float scale, int dtype, void* stream) {
    return fwd(q, k, v, o, 0, lse, B, H, S, D, causal, scale, dtype, stream);
}

extern "C" int attn_fwd_o16(const void* q, const void* k, const void* v, void* o, float* lse, int B, int H, int S, int D,
                            int causal, float scale, int dtype, void* stream) {
    return fwd(q, k, v, o, 1, lse, B, H, S, D, causal, scale, dtype, stream);
}
