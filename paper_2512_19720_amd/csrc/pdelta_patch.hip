// pdelta_patch: W_out = round(W_b + v (.) B)  (paper Eq. 1): the one-time merge of the delta into
// the weights that the paper deploys with (Limitations section; algorithm for applying a saved
// delta file model-wide).  Streaming, HBM-bound: 2 + 1/8 bytes read and 2 bytes written per weight.
//
// Rounding.  The result is the exact sum of two 16-bit floats rounded ONCE to the weight dtype
// (nearest-even).  The sum is formed twice in fp32, rounded down and rounded up (the fp32
// rounding mode of the wave is switched around groups of adds).  The two results are equal when
// the sum is exact in fp32 and adjacent fp32 numbers otherwise; taking the one whose last bit is
// 1 is "round to odd", and rounding that to a format with at most 22 significant bits
// (fp16: 11, bf16: 8) with nearest-even equals a single nearest-even rounding of the exact sum.
// Every nonzero sum of two such numbers is a normal fp32 number, so nothing is flushed.
#include "pdelta_device.h"
#include "pdelta_host.h"

namespace pdelta {

constexpr int kPatchThreads = 256;
constexpr int kPatchRows = 8;        // rows per workgroup of the single-layer kernel
constexpr int kPatchBatchRows = 16;  // rows per workgroup of the batched kernel (= the plan's block)

// fp32 rounding mode of this wave (bits 1:0 of the MODE register): 0 nearest-even, 1 toward
// +inf, 2 toward -inf.  The fp16 / fp64 rounding mode (bits 3:2) is left at nearest-even, which
// is what the conversions to fp16 below use.
template <int MODE>
__device__ __forceinline__ void set_f32_rounding()
{
    asm volatile("s_setreg_imm32_b32 hwreg(HW_REG_MODE, 0, 2), %0\n\ts_nop 1" ::"n"(MODE));
}
// An fp32 add that stays where it is written relative to the mode switches (volatile asm
// statements keep their order).
__device__ __forceinline__ float add_in_current_mode(float a, float b)
{
    float r;
    asm volatile("v_add_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
    return r;
}

// Of the round-down and round-up sums, the one with an odd last bit (either, when equal).
__device__ __forceinline__ float pick_odd(float down, float up)
{
    const uint32_t d = __builtin_bit_cast(uint32_t, down), u = __builtin_bit_cast(uint32_t, up);
    const uint32_t odd = (uint32_t)-(int32_t)(d & 1u);        // all ones when `down` is odd
    return __builtin_bit_cast(float, (d & odd) | (u & ~odd));
}

template <int DT>
__device__ __forceinline__ uint32_t f32_to_weight_bits(float x)
{
    return DT == kBF16 ? f32_to_bf16_bits(x) : f32_to_f16_bits(x);
}

// ROWS rows x 8 consecutive weights of one thread.  wf[r][e]: base weights as fp32; sf[r][e]:
// the signed scale +-v as fp32.  Returns the patched weights packed as stored.
template <int DT, int ROWS>
__device__ __forceinline__ void round_sums(const float (&wf)[ROWS][8], const float (&sf)[ROWS][8],
                                           uint4v (&out)[ROWS])
{
    float down[ROWS][8], up[ROWS][8];
    set_f32_rounding<2>();
#pragma unroll
    for (int r = 0; r < ROWS; ++r)
#pragma unroll
        for (int e = 0; e < 8; ++e) down[r][e] = add_in_current_mode(wf[r][e], sf[r][e]);
    set_f32_rounding<1>();
#pragma unroll
    for (int r = 0; r < ROWS; ++r)
#pragma unroll
        for (int e = 0; e < 8; ++e) up[r][e] = add_in_current_mode(wf[r][e], sf[r][e]);
    set_f32_rounding<0>();
#pragma unroll
    for (int r = 0; r < ROWS; ++r)
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            const uint32_t lo = f32_to_weight_bits<DT>(pick_odd(down[r][2 * p], up[r][2 * p]));
            const uint32_t hi = f32_to_weight_bits<DT>(pick_odd(down[r][2 * p + 1], up[r][2 * p + 1]));
            out[r][p] = lo | (hi << 16);
        }
}

// Patches rows row0 .. row0 + ROWS*GROUPS - 1 at columns col .. col + 7.  Loads are
// unconditional, ROWS rows at a time (row indices clamped into the matrix; stores of clamped
// rows are skipped), so that they are all in flight together.
// AXIS 2: blockwise scales v[row * v_stride + (col >> g_shift)] (groups are multiples of 8 inputs,
// so the eight weights of a thread share one scale).
template <int DT, int AXIS, int ROWS, int GROUPS>
__device__ __forceinline__ void
patch_column_strip(const uint16_t* W_b, const uint8_t* __restrict__ B_bytes,
                   const uint16_t* __restrict__ v, uint16_t* W_out, int d_out, int d_in, int row0, int col,
                   int v_stride = 0, int g_shift = 31)
{
    float vc[8];
    if constexpr (AXIS == 1) {
        const uint4v vv = *(const uint4v*)(v + col);
#pragma unroll
        for (int e = 0; e < 8; ++e) vc[e] = f16_bits_to_f32((vv[e >> 1] >> ((e & 1) * 16)) & 0xFFFFu);
    }
#pragma unroll 1
    for (int g = 0; g < GROUPS; ++g) {
        const int first = row0 + g * ROWS;
        if (first >= d_out) break;                                   // no loads are in flight here
        uint4v w[ROWS];
        uint32_t byte[ROWS];
        float vr[ROWS];
#pragma unroll
        for (int r = 0; r < ROWS; ++r) {
            const int row = min(first + r, d_out - 1);
            const int64_t off = (int64_t)row * d_in + col;
            w[r] = *(const uint4v*)(W_b + off);
            byte[r] = B_bytes[off >> 3];
            vr[r] = AXIS == 0   ? f16_bits_to_f32(v[row])
                    : AXIS == 2 ? f16_bits_to_f32(v[(int64_t)row * v_stride + (col >> g_shift)])
                                : 0.0f;
        }
        uint4v out[ROWS];
#pragma unroll
        for (int r2 = 0; r2 < ROWS; r2 += 2) {                       // two rows per pair of mode switches
            float wf[2][8], sf[2][8];
#pragma unroll
            for (int k = 0; k < 2; ++k)
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    wf[k][e] = bits_to_f32<DT>((w[r2 + k][e >> 1] >> ((e & 1) * 16)) & 0xFFFFu);
                    const float scale = AXIS == 1 ? vc[e] : vr[r2 + k];
                    // bit 1 -> +scale, bit 0 -> -scale: flip the sign where the sign bit is clear
                    const uint32_t flip = (~byte[r2 + k] << (31 - e)) & 0x80000000u;
                    sf[k][e] = __builtin_bit_cast(float, __builtin_bit_cast(uint32_t, scale) ^ flip);
                }
            uint4v o2[2];
            round_sums<DT, 2>(wf, sf, o2);
            out[r2] = o2[0];
            out[r2 + 1] = o2[1];
        }
#pragma unroll
        for (int r = 0; r < ROWS; ++r)
            if (first + r < d_out) *(uint4v*)(W_out + (int64_t)(first + r) * d_in + col) = out[r];
    }
}

// Workgroup = kPatchRows rows x one column segment of 256 * 8 = 2048 weights; consecutive
// workgroups take the segments of one block of rows, so that rows are streamed end to end.
// A thread owns 8 consecutive weights of a row (one 16-byte load / store) and the matching
// sign byte.
template <int DT, int AXIS>
__global__ void __launch_bounds__(kPatchThreads)
patch_kernel(const uint16_t* W_b, const uint8_t* __restrict__ B_bytes,
             const uint16_t* __restrict__ v, uint16_t* W_out, int d_out, int d_in, int n_seg,
             int v_stride, int g_shift)
{
    const int seg = (int)blockIdx.x % n_seg, row_block = (int)blockIdx.x / n_seg;
    const int col = (seg * kPatchThreads + threadIdx.x) * 8;
    if (col >= d_in) return;
    patch_column_strip<DT, AXIS, 4, kPatchRows / 4>(W_b, B_bytes, v, W_out, d_out, d_in,
                                                    row_block * kPatchRows, col, v_stride, g_shift);
}

// Batched merge: workgroup b patches 16 consecutive rows (all columns) of the last layer whose
// first_block is <= b; the layer's Y field is W_out.
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
    const int d_out = (int)L.d_out, d_in = (int)L.d_in;
    for (int col = threadIdx.x * 8; col < d_in; col += kPatchThreads * 8) {
        if (L.axis == 0)
            patch_column_strip<DT, 0, 4, kPatchBatchRows / 4>((const uint16_t*)L.W_b, (const uint8_t*)L.B_packed,
                                                              L.v, (uint16_t*)L.Y, d_out, d_in, row0, col);
        else
            patch_column_strip<DT, 1, 4, kPatchBatchRows / 4>((const uint16_t*)L.W_b, (const uint8_t*)L.B_packed,
                                                              L.v, (uint16_t*)L.Y, d_out, d_in, row0, col);
    }
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
                        int64_t d_out, int64_t d_in, hipStream_t stream, int v_stride = 0, int g_shift = 31)
{
    const int64_t n_seg = (d_in / 8 + kPatchThreads - 1) / kPatchThreads;
    const int64_t n_blocks = (d_out + kPatchRows - 1) / kPatchRows;          // <= 2^19 x 2^11
    hipLaunchKernelGGL((patch_kernel<DT, AXIS>), dim3((unsigned)(n_blocks * n_seg)), dim3(kPatchThreads), 0,
                       stream, (const uint16_t*)W_b, (const uint8_t*)B_packed, v, (uint16_t*)W_out,
                       (int)d_out, (int)d_in, (int)n_seg, v_stride, g_shift);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

int launch_patch_group(int w_dtype, const void* W_b, const uint32_t* B_packed, const uint16_t* v,
                       void* W_out, int64_t d_out, int64_t d_in, int v_stride, int g_shift,
                       hipStream_t stream)
{
    if (w_dtype == kBF16)
        return launch_patch<kBF16, 2>(W_b, B_packed, v, W_out, d_out, d_in, stream, v_stride, g_shift);
    return launch_patch<kF16, 2>(W_b, B_packed, v, W_out, d_out, d_in, stream, v_stride, g_shift);
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
