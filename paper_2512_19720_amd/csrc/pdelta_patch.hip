// pdelta_patch: W_out = round(W_b + v (.) B)  (paper Eq. 1): the one-time merge of the delta into
// the weights that the paper deploys with (Limitations section; algorithm for applying a saved
// delta file model-wide).  Streaming, HBM-bound: 2 + 1/8 bytes read and 2 bytes written per weight.
//
// Rounding.  The result is the exact sum of two 16-bit floats rounded ONCE to the weight dtype
// (nearest-even).  For fp16 weights that is what the hardware's fp16 addition returns (IEEE add,
// subnormals kept): one packed add per two weights.  For bf16 weights the sum is formed twice in
// fp32, rounded down and rounded up (the fp32 rounding mode of the wave is switched around groups
// of adds).  The two results are equal when
// the sum is exact in fp32 and adjacent fp32 numbers otherwise; taking the one whose last bit is
// 1 is "round to odd", and rounding that to a format with at most 22 significant bits
// (fp16: 11, bf16: 8) with nearest-even equals a single nearest-even rounding of the exact sum.
// Every nonzero sum of two such numbers is a normal fp32 number, so nothing is flushed.
#include "pdelta_device.h"
#include "pdelta_host.h"

namespace pdelta {

constexpr int kPatchThreads = 256;
constexpr int kPatchUnits = 4;                               // 16-byte units per thread and chunk
constexpr int kPatchChunk = kPatchThreads * kPatchUnits;     // 1024 units = 16 KB of weights per workgroup pass
constexpr int kPatchBatchRows = 16;                          // rows per block of the batched plan
constexpr int kPatchBatchParts = 8;                          // workgroups per block of the batched kernel

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

// N 16-byte units of a thread (8 consecutive weights of one row each) with the matching sign
// bytes and scales, as loaded.
template <int N>
struct PatchUnits {
    uint4v w[N];
    uint32_t byte[N];
    uint32_t v16[N];     // row mode / blockwise: the scale of the unit's row (block) as stored
    uint4v vc2[N];       // column mode: the unit's eight column scales as stored (fp16 pairs)
};

// The patched weights of the units, packed as stored.
template <int DT, int AXIS, int N>
__device__ __forceinline__ void patch_values(const PatchUnits<N>& S, uint4v (&out)[N])
{
    if constexpr (DT == kF16) {
        // fp16 weights: the packed fp16 add IS the single nearest-even rounding of the exact sum
        // (IEEE addition, fp16 subnormals kept), two weights per instruction
#pragma unroll
        for (int r = 0; r < N; ++r) {
            const uint32_t neg = ~S.byte[r];
            const uint32_t vr2 = AXIS == 1 ? 0u : (S.v16[r] | (S.v16[r] << 16));
#pragma unroll
            for (int p = 0; p < 4; ++p) {
                const uint32_t t = neg >> (2 * p);
                const uint32_t flip = ((t & 1u) << 15) | ((t & 2u) << 30);   // clear sign bit -> minus
                const uint32_t sv = (AXIS == 1 ? S.vc2[r][p] : vr2) ^ flip;
                out[r][p] = as_u32(as_half2(S.w[r][p]) + as_half2(sv));
            }
        }
    } else {
        static_assert(N % 2 == 0, "units are rounded two at a time");
#pragma unroll
        for (int r2 = 0; r2 < N; r2 += 2) {                          // two units per pair of mode switches
            float wf[2][8], sf[2][8];
#pragma unroll
            for (int k = 0; k < 2; ++k) {
                const float vr = f16_bits_to_f32(S.v16[r2 + k]);
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    wf[k][e] = bits_to_f32<DT>((S.w[r2 + k][e >> 1] >> ((e & 1) * 16)) & 0xFFFFu);
                    const float scale =
                        AXIS == 1 ? f16_bits_to_f32((S.vc2[r2 + k][e >> 1] >> ((e & 1) * 16)) & 0xFFFFu) : vr;
                    // bit 1 -> +scale, bit 0 -> -scale: flip the sign where the sign bit is clear
                    const uint32_t flip = (~S.byte[r2 + k] << (31 - e)) & 0x80000000u;
                    sf[k][e] = __builtin_bit_cast(float, __builtin_bit_cast(uint32_t, scale) ^ flip);
                }
            }
            uint4v o2[2];
            round_sums<DT, 2>(wf, sf, o2);
            out[r2] = o2[0];
            out[r2 + 1] = o2[1];
        }
    }
}

// Patches 16-byte units of the matrix taken as one flat array (unit u = row u / (d_in / 8), columns
// 8 (u % (d_in / 8)) .. + 7; rows are contiguous, so W_b, W_out and the sign bytes are all indexed
// by u).  Units are counted from the start of row `row_base`: the passes that start at first_rel,
// first_rel + stride, ... below last_rel, each clipped at last_rel.  A pass covers 1024
// consecutive units: thread t takes units t, t + 256, t + 512, t + 768 of it, issues all its loads,
// sums, stores.  Measured on MI355X this plain shape (what a library elementwise kernel does)
// streams 5-8 % faster than walking rows with the next step's loads in flight, and equals the
// box's in-place update rate.  Loads are unconditional (unit index clamped to last_rel - 1); only
// stores are guarded.
// AXIS 2: blockwise scales v[row * v_stride + (col >> g_shift)] (groups are multiples of 8 inputs,
// so the eight weights of a unit share one scale).
template <int DT, int AXIS>
__device__ __forceinline__ void
patch_units(const uint16_t* W_b, const uint8_t* __restrict__ B_bytes, const uint16_t* __restrict__ v,
            uint16_t* W_out, int d_in, int row_base, int first_rel, int last_rel, int stride, int v_stride = 0,
            int g_shift = 31)
{
    const int upr = d_in >> 3;                                       // units per row
    const int64_t unit0 = (int64_t)row_base * upr;
    const uint16_t* w_base = W_b + unit0 * 8;
    const uint8_t* b_base = B_bytes + unit0;
    uint16_t* out_base = W_out + unit0 * 8;
    for (int base = first_rel; base < last_rel; base += stride) {
        PatchUnits<kPatchUnits> S;
        int rel[kPatchUnits];
#pragma unroll
        for (int j = 0; j < kPatchUnits; ++j) {
            rel[j] = base + j * kPatchThreads + (int)threadIdx.x;
            const int rc = min(rel[j], last_rel - 1);
            const int r = rc / upr;
            const int col = (rc - r * upr) * 8;
            const int row = row_base + r;
            S.w[j] = *(const uint4v*)(w_base + (int64_t)rc * 8);
            S.byte[j] = b_base[rc];
            S.v16[j] = AXIS == 0   ? (uint32_t)v[row]
                       : AXIS == 2 ? (uint32_t)v[(int64_t)row * v_stride + (col >> g_shift)]
                                   : 0u;
            if constexpr (AXIS == 1) S.vc2[j] = *(const uint4v*)(v + col);
        }
        uint4v out[kPatchUnits];
        patch_values<DT, AXIS, kPatchUnits>(S, out);
#pragma unroll
        for (int j = 0; j < kPatchUnits; ++j)
            if (rel[j] < last_rel) *(uint4v*)(out_base + (int64_t)rel[j] * 8) = out[j];
    }
}

// One layer: workgroup b patches units 1024 b .. 1024 b + 1023.
template <int DT, int AXIS>
__global__ void __launch_bounds__(kPatchThreads)
patch_kernel(const uint16_t* W_b, const uint8_t* __restrict__ B_bytes, const uint16_t* __restrict__ v,
             uint16_t* W_out, int d_in, int64_t total_units, int v_stride, int g_shift)
{
    const int upr = d_in >> 3;
    const int64_t first = (int64_t)blockIdx.x * kPatchChunk;         // workgroup-uniform
    const int64_t last = min(first + kPatchChunk, total_units);
    const int row_base = (int)(first / upr);
    const int64_t unit0 = (int64_t)row_base * upr;
    patch_units<DT, AXIS>(W_b, B_bytes, v, W_out, d_in, row_base, (int)(first - unit0), (int)(last - unit0),
                          kPatchChunk, v_stride, g_shift);
}

// Batched merge: the plan counts blocks of 16 rows; block b belongs to the last layer whose
// first_block is <= b, and kPatchBatchParts workgroups share its units in equal contiguous parts
// (at d_in = 4096 a part is exactly one pass; dealing the passes out round-robin instead was
// measured slower, 5.15 against 5.33 TB/s on a 7B-shaped stack).  The layer's Y field is W_out.
template <int DT>
__global__ void __launch_bounds__(kPatchThreads)
patch_batch_kernel(const pdelta_layer* __restrict__ layers, int n_layers)
{
    const int b = (int)(blockIdx.x / kPatchBatchParts), part = (int)(blockIdx.x % kPatchBatchParts);
    int lo = 0, hi = n_layers - 1;
    while (lo < hi) {                                 // workgroup-uniform
        const int mid = (lo + hi + 1) >> 1;
        if (layers[mid].first_block <= b) lo = mid; else hi = mid - 1;
    }
    const pdelta_layer L = layers[lo];
    const int d_out = (int)L.d_out, d_in = (int)L.d_in;
    const int row0 = (b - L.first_block) * kPatchBatchRows;
    const int block_units = min(kPatchBatchRows, d_out - row0) * (d_in >> 3);
    const uint16_t* W_b = as_global((const uint16_t*)L.W_b);
    const uint8_t* B_bytes = as_global((const uint8_t*)L.B_packed);
    const uint16_t* v = as_global(L.v);
    uint16_t* W_out = as_global((uint16_t*)L.Y);
    const int per_part = (block_units + kPatchBatchParts - 1) / kPatchBatchParts;
    const int first = part * per_part, last = min(first + per_part, block_units);
    if (L.axis == 0) patch_units<DT, 0>(W_b, B_bytes, v, W_out, d_in, row0, first, last, kPatchChunk);
    else patch_units<DT, 1>(W_b, B_bytes, v, W_out, d_in, row0, first, last, kPatchChunk);
}

// Returns 1 when the batch has too many blocks for one grid (the caller then patches layer by layer).
int launch_patch_batch(int w_dtype, const pdelta_layer* layers_host, const pdelta_layer* layers_device,
                       int n_layers, hipStream_t stream)
{
    const pdelta_layer& last = layers_host[n_layers - 1];
    const int64_t total = last.first_block + (last.d_out + kPatchBatchRows - 1) / kPatchBatchRows;
    if (total * kPatchBatchParts > 0x7FFFFFFF) return 1;
    const dim3 grid((unsigned)(total * kPatchBatchParts));
    if (w_dtype == kBF16)
        hipLaunchKernelGGL(patch_batch_kernel<kBF16>, grid, dim3(kPatchThreads), 0, stream, layers_device, n_layers);
    else
        hipLaunchKernelGGL(patch_batch_kernel<kF16>, grid, dim3(kPatchThreads), 0, stream, layers_device, n_layers);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

template <int DT, int AXIS>
static int launch_patch(const void* W_b, const uint32_t* B_packed, const uint16_t* v, void* W_out,
                        int64_t d_out, int64_t d_in, hipStream_t stream, int v_stride = 0, int g_shift = 31)
{
    const int64_t total_units = d_out * (d_in / 8);
    const int64_t n_blocks = (total_units + kPatchChunk - 1) / kPatchChunk;
    if (n_blocks > 0x7FFFFFFF) return -1;             // 2^41 weights and more: not a layer
    hipLaunchKernelGGL((patch_kernel<DT, AXIS>), dim3((unsigned)n_blocks), dim3(kPatchThreads), 0, stream,
                       (const uint16_t*)W_b, (const uint8_t*)B_packed, v, (uint16_t*)W_out, (int)d_in, total_units,
                       v_stride, g_shift);
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
