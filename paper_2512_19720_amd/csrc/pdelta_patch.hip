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

// Batched merge: workgroup b patches 16 consecutive rows (all columns) of the last layer whose
// first_block is <= b; the layer's Y field is W_out.  Loads are unconditional, four rows at a
// time (row indices clamped into the matrix, stores of clamped rows skipped).
constexpr int kPatchBatchRows = 16;

template <int DT, int AXIS>
__device__ __forceinline__ void
patch_rows(const uint16_t* W_b, const uint8_t* __restrict__ B_bytes, const uint16_t* __restrict__ v,
           uint16_t* W_out, int d_out, int d_in, int row0)
{
    for (int col = threadIdx.x * 8; col < d_in; col += kPatchThreads * 8) {
        double vc[8];
        if constexpr (AXIS == 1) {
            const uint4v vv = *(const uint4v*)(v + col);
#pragma unroll
            for (int e = 0; e < 8; ++e)
                vc[e] = (double)f16_bits_to_f32((vv[e >> 1] >> ((e & 1) * 16)) & 0xFFFFu);
        }
        for (int r4 = 0; r4 < kPatchBatchRows; r4 += 4) {
            uint4v w[4];
            uint32_t byte[4];
            double vr[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int row = min(row0 + r4 + k, d_out - 1);
                const int64_t off = (int64_t)row * d_in + col;
                w[k] = *(const uint4v*)(W_b + off);
                byte[k] = B_bytes[off >> 3];
                vr[k] = AXIS == 0 ? (double)f16_bits_to_f32(v[row]) : 0.0;
            }
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                uint4v out;
#pragma unroll
                for (int p = 0; p < 4; ++p) {
                    uint32_t packed = 0;
#pragma unroll
                    for (int q = 0; q < 2; ++q) {
                        const int e = p * 2 + q;
                        const double wb = (double)bits_to_f32<DT>((w[k][p] >> (q * 16)) & 0xFFFFu);
                        const double scale = AXIS == 0 ? vr[k] : vc[e];
                        const double sum = ((byte[k] >> e) & 1u) ? wb + scale : wb - scale;
                        const uint32_t bits = DT == kBF16 ? f64_to_bf16_bits_rne(sum) : f64_to_f16_bits_rne(sum);
                        packed |= bits << (q * 16);
                    }
                    out[p] = packed;
                }
                const int row = row0 + r4 + k;
                if (row < d_out) *(uint4v*)(W_out + (int64_t)row * d_in + col) = out;
            }
        }
    }
}

template <int DT>
__global__ void __launch_bounds__(kPatchThreads)
patch_batch_kernel(const pdelta_layer* __restrict__ layers, int n_layers)
{
    const int b = (int)blockIdx.x;
    int lo = 0, hi = n_layers - 1;
    while (lo < hi) {                                 // workgroup-uniform
        const int mid = (lo + hi + 1) >> 1;
        if (layers[mid].first_block <= b) lo = mid; else hi = mid - 1;
    }
    const pdelta_layer L = layers[lo];
    const int row0 = (b - L.first_block) * kPatchBatchRows;
    if (L.axis == 0)
        patch_rows<DT, 0>((const uint16_t*)L.W_b, (const uint8_t*)L.B_packed, L.v, (uint16_t*)L.Y,
                          (int)L.d_out, (int)L.d_in, row0);
    else
        patch_rows<DT, 1>((const uint16_t*)L.W_b, (const uint8_t*)L.B_packed, L.v, (uint16_t*)L.Y,
                          (int)L.d_out, (int)L.d_in, row0);
}

int launch_patch_batch(int w_dtype, const pdelta_layer* layers_host, const pdelta_layer* layers_device,
                       int n_layers, hipStream_t stream)
{
    const pdelta_layer& last = layers_host[n_layers - 1];
    const int64_t total = last.first_block + (last.d_out + kPatchBatchRows - 1) / kPatchBatchRows;
    if (w_dtype == kBF16)
        hipLaunchKernelGGL(patch_batch_kernel<kBF16>, dim3((unsigned)total), dim3(kPatchThreads), 0, stream,
                           layers_device, n_layers);
    else
        hipLaunchKernelGGL(patch_batch_kernel<kF16>, dim3((unsigned)total), dim3(kPatchThreads), 0, stream,
                           layers_device, n_layers);
    return hipGetLastError() == hipSuccess ? 0 : -1;
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
