// pdelta_pack_group: B = sign(W_f - W_b) bit-packed along the input axis (as pdelta_pack) plus
// blockwise initial scales: v[r, g] = mean |W_f - W_b| over output row r (or over all rows) and
// inputs g * group .. (g + 1) * group - 1.  Blockwise per-group scales are the first extension the
// paper's conclusion names; one scale for the whole matrix (rows shared, group = d_in) is the
// single learned scalar of its BitDelta comparison (Experiments section).  The initial value is
// the per-layer compression algorithm's mean |dW|, taken per block.
//
// One streaming pass: a wave walks one output row in chunks of 512 inputs (a lane owns 8
// consecutive weights: one 16-byte load from each matrix, one sign byte), the loads of the next
// chunk in flight while the current one is compared and summed.  |dW| is formed exactly in fp64;
// a block's sum is a butterfly over the lanes of the block (blocks up to 512 inputs) or the
// wave's running total (longer blocks), so for fp16 inputs it is the exact sum whatever the
// order, and the mean is rounded once to fp16: bit-equal to the fp64 reference while the sum of
// |dW| of a block stays below 2^29.  When the rows share the scales every row leaves one fp64
// partial per group in the workspace and a second kernel adds them in a fixed order (as 64-bit
// integers in units of 2^-24 for fp16).  bf16 sums are fp64 sums: exact while fp64 holds them.
#include <type_traits>

#include "pdelta_device.h"
#include "pdelta_host.h"

namespace pdelta {

constexpr int kPgWaves = 4;

template <int DT>
__global__ void __launch_bounds__(kPgWaves * kWave)
pack_group_kernel(const uint16_t* __restrict__ W_f, const uint16_t* __restrict__ W_b, int d_out, int d_in,
                  uint32_t* __restrict__ B_packed, uint16_t* __restrict__ v, double* __restrict__ partial,
                  int group, int n_groups)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int row = blockIdx.x * kPgWaves + wave;
    if (row >= d_out) return;                                   // whole wave
    const uint16_t* f_row = W_f + (int64_t)row * d_in;
    const uint16_t* b_row = W_b + (int64_t)row * d_in;
    uint32_t* sign_row = B_packed + (int64_t)row * (d_in >> 5);
    const int n_chunks = (d_in + 511) >> 9;
    const int lanes_per_group = group >> 3;                      // 4 .. 64 for groups inside a chunk
    const bool inside_chunk = group <= 512 && (group & (group - 1)) == 0;   // wave-uniform; else: a whole short row

    // a lane past the end of the row reads a clamped address of W_b for both operands: its
    // differences are exactly zero and nothing of it is stored (loads stay unconditional)
    auto load = [&](uint4v& a, uint4v& b, int chunk) {
        const int col = (chunk << 9) + lane * 8;
        const int cc = min(col, d_in - 8);
        const uint16_t* f_or_b = col < d_in ? f_row : b_row;
        b = *(const uint4v*)(b_row + cc);
        a = *(const uint4v*)(f_or_b + cc);
    };
    uint4v a0, b0, a1, b1;
    load(a0, b0, 0);
    double running = 0.0;                                        // blocks longer than a chunk
    for (int c = 0; c < n_chunks; ++c) {
        load(a1, b1, min(c + 1, n_chunks - 1));
        const int col = (c << 9) + lane * 8;
        uint32_t bits = 0;
        double sum = 0.0;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float fa = bits_to_f32<DT>((a0[e >> 1] >> ((e & 1) * 16)) & 0xFFFFu);
            const float fb = bits_to_f32<DT>((b0[e >> 1] >> ((e & 1) * 16)) & 0xFFFFu);
            bits |= (fa < fb ? 0u : 1u) << e;                    // a compare: +0, -0 and ties give +1
            sum += fabs((double)fa - (double)fb);                // exact for fp16
        }
        // four lanes' sign bytes make one word; lane 4k stores it
        uint32_t word = bits;
        word |= (uint32_t)__shfl_down((int)bits, 1, kWave) << 8;
        word |= (uint32_t)__shfl_down((int)bits, 2, kWave) << 16;
        word |= (uint32_t)__shfl_down((int)bits, 3, kWave) << 24;
        if ((lane & 3) == 0 && col < d_in) sign_row[col >> 5] = word;
        // block sums
        if (inside_chunk) {
            for (int off = 1; off < lanes_per_group; off <<= 1) sum += __shfl_xor(sum, off, kWave);
            if ((lane & (lanes_per_group - 1)) == 0 && col < d_in) {
                const int g = col / group;
                if (partial != nullptr) partial[(int64_t)row * n_groups + g] = sum;
                else v[(int64_t)row * n_groups + g] = (uint16_t)f64_to_f16_bits_rne(sum / (double)group);
            }
        } else {
            running += wave_sum_f64(sum);
            const int end = min((c + 1) << 9, d_in);             // first input after this chunk
            if (end % group == 0 || end == d_in) {               // wave-uniform: a block ends here
                if (lane == 0) {
                    const int g = (end - 1) / group;
                    if (partial != nullptr) partial[(int64_t)row * n_groups + g] = running;
                    else v[(int64_t)row * n_groups + g] = (uint16_t)f64_to_f16_bits_rne(running / (double)group);
                }
                running = 0.0;
            }
        }
        a0 = a1;
        b0 = b1;
    }
}

// Rows share the scales: v[g] = mean over all rows of the rows' partial sums.  One workgroup per
// group; thread t adds rows t, t + 256, ... and the 256 totals meet in LDS, always in the same order.
template <int DT>
__global__ void __launch_bounds__(256)
pack_group_shared_finalize_kernel(const double* __restrict__ partial, int d_out, int n_groups, double count,
                                  uint16_t* __restrict__ v)
{
    typedef typename std::conditional<DT == kF16, unsigned long long, double>::type acc_t;
    __shared__ acc_t part[256];
    const int g = blockIdx.x;
    acc_t s = 0;
    for (int row = threadIdx.x; row < d_out; row += 256) {
        const double p = partial[(int64_t)row * n_groups + g];
        if constexpr (DT == kF16) s += (unsigned long long)(p * 16777216.0);   // units of 2^-24: exact
        else s += p;
    }
    part[threadIdx.x] = s;
    __syncthreads();
    if (threadIdx.x == 0) {
        acc_t total = part[0];
        for (int k = 1; k < 256; ++k) total += part[k];
        const double sum = DT == kF16 ? (double)total * (1.0 / 16777216.0) : (double)total;
        v[g] = (uint16_t)f64_to_f16_bits_rne(sum / count);
    }
}

size_t pack_group_workspace_bytes(int64_t d_out, int64_t d_in, int64_t group, int shared_rows)
{
    return shared_rows ? (size_t)d_out * (size_t)(d_in / group) * sizeof(double) : 0;
}

template <int DT>
static int launch_pack_group_dt(const void* W_f, const void* W_b, int64_t d_out, int64_t d_in, int64_t group,
                                int shared_rows, uint32_t* B_packed, uint16_t* v, void* workspace,
                                hipStream_t stream)
{
    const int n_groups = (int)(d_in / group);
    double* partial = shared_rows ? (double*)workspace : nullptr;
    hipLaunchKernelGGL(pack_group_kernel<DT>, dim3((unsigned)((d_out + kPgWaves - 1) / kPgWaves)),
                       dim3(kPgWaves * kWave), 0, stream, (const uint16_t*)W_f, (const uint16_t*)W_b, (int)d_out,
                       (int)d_in, B_packed, v, partial, (int)group, n_groups);
    if (shared_rows)
        hipLaunchKernelGGL(pack_group_shared_finalize_kernel<DT>, dim3((unsigned)n_groups), dim3(256), 0, stream,
                           (const double*)partial, (int)d_out, n_groups, (double)d_out * (double)group, v);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

int launch_pack_group(int w_dtype, const void* W_f, const void* W_b, int64_t d_out, int64_t d_in,
                      int64_t group, int shared_rows, uint32_t* B_packed, uint16_t* v, void* workspace,
                      hipStream_t stream)
{
    if (w_dtype == kBF16)
        return launch_pack_group_dt<kBF16>(W_f, W_b, d_out, d_in, group, shared_rows, B_packed, v, workspace, stream);
    return launch_pack_group_dt<kF16>(W_f, W_b, d_out, d_in, group, shared_rows, B_packed, v, workspace, stream);
}

}  // namespace pdelta
