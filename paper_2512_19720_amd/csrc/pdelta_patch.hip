// pdelta_patch: W_out = round(W_b + v (.) B)  (paper Eq. 1), the merge the paper deploys with
// ("add all residual terms at once", Limitations; "Model-wide application from a saved delta
// file").  Streaming, HBM-bound: 2 + 1/8 bytes read and 2 bytes written per weight.
//
// Rounding: both operands are 16-bit floats, so their sum is exact in fp64; it is narrowed to
// fp32 with round-to-odd and then to the weight dtype with round-to-nearest-even, which equals
// one nearest-even rounding of the exact sum.
#include "pdelta_device.h"
#include "pdelta_host.h"

namespace pdelta {

constexpr int kPatchThreads = 256;
constexpr int kPatchRows = 8;   // rows per workgroup: column-mode scales are loaded once for all

// grid.x = block of kPatchRows rows, grid.y = column segment of 256 * 8 = 2048 weights.
// A thread owns 8 consecutive weights of a row (one 16-byte load / store) and the matching
// sign byte.
template <int DT, int AXIS>
__global__ void __launch_bounds__(kPatchThreads)
patch_kernel(const uint16_t* W_b, const uint8_t* __restrict__ B_bytes,
             const uint16_t* __restrict__ v, uint16_t* W_out, int d_out, int d_in)
{
    const int col = (blockIdx.y * kPatchThreads + threadIdx.x) * 8;
    if (col >= d_in) return;
    const int row0 = blockIdx.x * kPatchRows;

    double vc[8];
    if constexpr (AXIS == 1) {
        const uint4v vv = *(const uint4v*)(v + col);
#pragma unroll
        for (int e = 0; e < 8; ++e)
            vc[e] = (double)f16_bits_to_f32((vv[e >> 1] >> ((e & 1) * 16)) & 0xFFFFu);
    }

#pragma unroll 4
    for (int r = 0; r < kPatchRows; ++r) {
        const int row = row0 + r;
        if (row >= d_out) break;
        const int64_t off = (int64_t)row * d_in + col;
        const uint4v w = *(const uint4v*)(W_b + off);
        const uint32_t byte = B_bytes[off >> 3];
        double vr = 0.0;
        if constexpr (AXIS == 0) vr = (double)f16_bits_to_f32(v[row]);
        uint4v out;
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            uint32_t packed = 0;
#pragma unroll
            for (int q = 0; q < 2; ++q) {
                const int e = p * 2 + q;
                const double wb = (double)bits_to_f32<DT>((w[p] >> (q * 16)) & 0xFFFFu);
                const double scale = AXIS == 0 ? vr : vc[e];
                const double sum = ((byte >> e) & 1u) ? wb + scale : wb - scale;
                const uint32_t bits = DT == kBF16 ? f64_to_bf16_bits_rne(sum) : f64_to_f16_bits_rne(sum);
                packed |= bits << (q * 16);
            }
            out[p] = packed;
        }
        *(uint4v*)(W_out + off) = out;
    }
}

template <int DT, int AXIS>
static int launch_patch(const void* W_b, const uint32_t* B_packed, const uint16_t* v, void* W_out,
                        int64_t d_out, int64_t d_in, hipStream_t stream)
{
    dim3 grid((unsigned)((d_out + kPatchRows - 1) / kPatchRows),
              (unsigned)((d_in / 8 + kPatchThreads - 1) / kPatchThreads));
    hipLaunchKernelGGL((patch_kernel<DT, AXIS>), grid, dim3(kPatchThreads), 0, stream,
                       (const uint16_t*)W_b, (const uint8_t*)B_packed, v, (uint16_t*)W_out,
                       (int)d_out, (int)d_in);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

int launch_patch_dispatch(int w_dtype, int axis, const void* W_b, const uint32_t* B_packed,
                          const uint16_t* v, void* W_out, int64_t d_out, int64_t d_in,
                          hipStream_t stream)
{
    if (w_dtype == kBF16)
        return axis == 0 ? launch_patch<kBF16, 0>(W_b, B_packed, v, W_out, d_out, d_in, stream)
                         : launch_patch<kBF16, 1>(W_b, B_packed, v, W_out, d_out, d_in, stream);
    return axis == 0 ? launch_patch<kF16, 0>(W_b, B_packed, v, W_out, d_out, d_in, stream)
                     : launch_patch<kF16, 1>(W_b, B_packed, v, W_out, d_out, d_in, stream);
}

}  // namespace pdelta
