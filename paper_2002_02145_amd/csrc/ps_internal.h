// Internal helpers shared by the translation units of the GPU library (never installed).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "polysci_conv.h"

namespace ps {

constexpr int kBlock = 16;  // channel block B of the blocked layouts

struct Dims {
    int N, C, H, W, K, R, S, stride, pad;
    int P, Q;    // output size
    int Cb, Kb;  // channel blocks
    int NB;      // batch-reduce length Cb*R*S
    long long M; // flattened output pixels N*P*Q
    int es;      // element size of input/filter in bytes
    int dtype;
};

// Validates a descriptor and derives the sizes every entry point needs.
int make_dims(const ps_conv_desc *d, Dims *out);

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Remembers the runtime's own description of the last failure for ps_last_hip_error().
inline const char *&last_hip_error_text()
{
    static thread_local const char *text = "";
    return text;
}
inline int hip_status(hipError_t e)
{
    if (e == hipSuccess) return PS_OK;
    last_hip_error_text() = hipGetErrorString(e);
    return PS_EHIP;
}

// api.hip / conv_fwd_f32.hip
bool packs_taps(const Dims &dm);
int launch_fill_zero(float *p, size_t n, hipStream_t stream);
int launch_reduce_planes(const float *partial, void *out, size_t n, int planes, const float *bias, int epi, int PQ, int Kb,
                         hipStream_t stream);

}  // namespace ps
