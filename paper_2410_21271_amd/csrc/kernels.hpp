// Internal launch interface between the C-ABI entry points (api.hip) and the kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace eora {

// stored formats a contraction segment can read
enum SegFmt { S_NONE = 0, S_Q4 = 1, S_Q3 = 2, S_Q4S128 = 3, S_Q4S64 = 4, S_F16 = 5 };

struct DecodeArgs {
    const _Float16* x;        // M x d_in fp16 row-major
    const void* w;            // main operand tiles (backbone, or A for the down-projection)
    const _Float16* w_scales;
    const uint32_t* w_zeros;
    const void* B;            // extension operand tiles (d_out x r) or nullptr
    const _Float16* B_scales;
    const float* t;           // M x r fp32 row-major (down-projection result)
    void* y;                  // M x d_out, fp16 or fp32
    int M, d_in, d_out, r, group;
};

hipError_t launch_decode(const DecodeArgs& a, int fm, int fe, hipStream_t stream);
hipError_t launch_downproj(const DecodeArgs& a, int fa, hipStream_t stream);

hipError_t launch_unpack_q(const uint32_t* qweight, const uint32_t* qzeros, uint8_t* codes, uint8_t* zeros,
                           int d_in, int d_out, int w_bits, int group, hipStream_t stream);
hipError_t launch_dequant_q(const uint32_t* qweight, const _Float16* scales, const uint32_t* qzeros, float* W,
                            int d_in, int d_out, int w_bits, int group, hipStream_t stream);
hipError_t launch_expand_sp24(const _Float16* values, const uint32_t* indices, _Float16* W,
                              int d_in, int d_out, hipStream_t stream);

}  // namespace eora
