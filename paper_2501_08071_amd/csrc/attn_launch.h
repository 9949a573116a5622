// Internal: validated launch request handed from the C-ABI layer to the kernel dispatcher.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#ifndef ATTN_NW
#define ATTN_NW 4   // wavefronts per workgroup; each owns 32 query rows
#endif
#define ATTN_BC 64  // keys per inner-loop tile
#ifndef ATTN_WPE
#define ATTN_WPE 2  // wavefronts per SIMD the register budget is sized for
#endif

struct AttnLaunch {
    const void* q;
    const void* k;
    const void* v;
    float* o;
    float* lse;       // may be null
    int BH, S, D;
    int causal;
    int dtype;        // 0 binary16, 1 bfloat16
    float c;          // |scale| * log2(e)
    uint32_t qsign;   // 0x80008000 when scale < 0 (sign folded into q), else 0
    void* stream;
};

hipError_t attn_launch(const AttnLaunch& a);
