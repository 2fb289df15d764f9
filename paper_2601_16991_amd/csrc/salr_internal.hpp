// Host-side declarations shared between the C boundary and the kernel files.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace salr {

hipError_t launch_encode(const uint16_t* w, int64_t rows, int64_t cols, uint32_t* bitmap, uint16_t* values,
                         int64_t capacity, uint32_t* row_offsets, hipStream_t stream);

hipError_t launch_decode(const uint32_t* bitmap, const uint16_t* values, const uint32_t* row_offsets, int64_t rows,
                         int64_t cols, uint16_t* out, hipStream_t stream);

// Columns of the bf16 workspace matrix T = X * A_cat: R rounded up to the MFMA k-step.
inline int64_t adapter_rank_padded(int64_t R) { return (R + 31) / 32 * 32; }

struct LinearArgs {
    const uint16_t* x;
    int64_t M, K, N;
    const uint32_t* bitmap;
    const uint16_t* values;
    const uint32_t* row_offsets;
    const uint16_t* a_cat;
    const uint16_t* b_cat;
    int64_t R;
    uint16_t* y;
    uint16_t* t;  // workspace: [M, adapter_rank_padded(R)] bf16
};

hipError_t launch_linear(const LinearArgs& args, hipStream_t stream);

// Optional events recorded around the fused kernel's launch (measurement hook of the boundary).
struct TimingEvents {
    hipEvent_t start = nullptr;
    hipEvent_t stop = nullptr;
};
extern thread_local TimingEvents g_timing_events;

}  // namespace salr
