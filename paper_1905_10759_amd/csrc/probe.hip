// Diagnostic: the rate at which this machine sustains the matrix-core instruction that the fp32-as-bf16-pieces
// kernels are built on (v_mfma_f32_32x32x16_bf16), with nothing else in the loop.  Every compute unit runs
// eight waves, each `steps` x 24 MFMAs on four independent accumulators, operands held in registers and
// filled with pseudo-random bf16 values (all-equal operands toggle fewer wires and run faster than any real
// input).  The published peak assumes the top clock; under this load on all compute units the clock is
// lower, and this number is what a perfect kernel could reach.  Not part of the method.
#include "bf16_pieces.h"
#include "kernels.h"

namespace hbmm {
namespace {

__global__ __launch_bounds__(512) void probe_mfma_kernel(int steps, float *sink)
{
    u32x4 ua[6];
    uint32_t h = (blockIdx.x * 512u + threadIdx.x) * 2654435761u + 12345u;
#pragma unroll
    for (int i = 0; i < 6; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            h = h * 1664525u + 1013904223u;
            ua[i][j] = (h & 0x807f807fu) | 0x3f003f00u;   // two bf16 values of magnitude 0.5 .. 1, either sign
        }
    f32x16 acc[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 16; ++j) acc[i][j] = 0.f;
    for (int s = 0; s < steps; ++s) {
#pragma unroll
        for (int q = 0; q < 6; ++q) {
            const bf16x8 x = __builtin_bit_cast(bf16x8, ua[q]), y = __builtin_bit_cast(bf16x8, ua[(q + 1) % 6]);
            acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x, y, acc[0], 0, 0, 0);
            acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(y, x, acc[1], 0, 0, 0);
            acc[2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x, x, acc[2], 0, 0, 0);
            acc[3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(y, y, acc[3], 0, 0, 0);
        }
        // keep the sums finite without leaving the loop body empty of data dependence
        if ((s & 63) == 63) {
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 16; ++j) acc[i][j] *= 0.0009765625f;
        }
    }
    float sum = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 16; ++j) sum += acc[i][j];
    sink[blockIdx.x * 512 + threadIdx.x] = sum;
}

}  // namespace

hipError_t launch_probe_mfma(int steps, int blocks, float *sink, hipStream_t s)
{
    probe_mfma_kernel<<<dim3((unsigned)blocks), dim3(512), 0, s>>>(steps, sink);
    return hipGetLastError();
}

}  // namespace hbmm
