// Diagnostic: what the fp16 matrix core returns for given operands.
//
// The fp16 E-step (Section 3.1's argmin, scored as ||c||^2 - 2 x.c on v_mfma_f32_32x32x16_f16) relies on one
// property of that instruction which no manual states: how far its fp32 result can be from the exact sum of its
// (exact) products and its C operand. The guard band of assign_mfma_f16.hip assumes a multiple of 2^-24 times an
// inflated sum of |terms|. This kernel runs the instruction - chained exactly as the E-step chains it, the C
// operand preset per output row - on operands the caller chooses, so that a test can pin that assumption on
// adversarial inputs against exact arithmetic.
#include "common.h"

namespace cc {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));

// One wave per tile. A [tiles][32][16*KM], B [tiles][32][16*KM] (fp16 bit patterns; row m of A against row n of B
// gives D[m][n]), C [tiles][32] (fp32, the accumulator's start value for output row m), D [tiles][32][32].
template <int KM>
__global__ __launch_bounds__(64) void mfma_f16_probe_kernel(const uint16_t* __restrict__ A, const uint16_t* __restrict__ B,
                                                            const float* __restrict__ C, float* __restrict__ D)
{
    const int lane = threadIdx.x, h = lane >> 5, n = lane & 31;
    const size_t t = blockIdx.x;
    f16x8 a[KM], b[KM];
#pragma unroll
    for (int mi = 0; mi < KM; ++mi)
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            // lane (n, h) supplies k slots 16*mi + 8h .. +7 of A row n and of B row n
            a[mi][q] = __builtin_bit_cast(_Float16, A[(t * 32 + n) * (16 * KM) + 16 * mi + 8 * h + q]);
            b[mi][q] = __builtin_bit_cast(_Float16, B[(t * 32 + n) * (16 * KM) + 16 * mi + 8 * h + q]);
        }
    f32x16 acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = C[t * 32 + (r % 4) + 8 * (r / 4) + 4 * h];
#pragma unroll
    for (int mi = 0; mi < KM; ++mi) acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[mi], b[mi], acc, 0, 0, 0);
#pragma unroll
    for (int r = 0; r < 16; ++r) D[(t * 32 + (r % 4) + 8 * (r / 4) + 4 * h) * 32 + n] = acc[r];
}

hipError_t launch_mfma_f16_probe(const uint16_t* A, const uint16_t* B, const float* C, float* D, uint32_t tiles, uint32_t km,
                                 hipStream_t s)
{
    if (km == 1) hipLaunchKernelGGL(mfma_f16_probe_kernel<1>, dim3(tiles), dim3(64), 0, s, A, B, C, D);
    else if (km == 2) hipLaunchKernelGGL(mfma_f16_probe_kernel<2>, dim3(tiles), dim3(64), 0, s, A, B, C, D);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

}  // namespace cc
