// Decode-shaped delta linear layer (M <= 64 tokens):
//   row:  Y[m,o] = sum_i X[m,i] W_b[o,i] + v[o] * sum_i X[m,i] B[o,i]
//   col:  Y[m,o] = sum_i X[m,i] W_b[o,i] +        sum_i (X[m,i] v[i]) B[o,i]
// (paper Eq. 1 applied inside the layer forward, never forming W_hat in memory).
//
// The layer is HBM-bound: every weight (2 B) and every sign bit (1/8 B) is read exactly once
// and nothing else of size is touched.  The arithmetic rides on the matrix cores, which are
// otherwise idle: a 16x16x32 MFMA takes 16 tokens x 16 output rows x 32 inputs, so even one
// token costs the same handful of issue slots as sixteen and the vector ALUs only have to turn
// sign bits into +-1 operands.  Two accumulators are kept (base and sign part); the per-row
// scale multiplies the sign accumulator once, in the epilogue, in fp32.
//
// Work split: a workgroup owns 16 consecutive output rows (a contiguous 16 * d_in * 2 byte
// slab of W_b) and all of d_in; its waves take 128-input steps round-robin and their partial
// accumulators meet in LDS.  Within a step lane (n = lane % 16, g = lane / 16) loads, for
// j = 0..3, the 16 bytes W_b[row n][k0 + 32 j + 8 g .. +7]: this is exactly the B-operand
// layout of the MFMA (no shuffles), and the four 32-bit sign words of that row and step are
// one 16-byte load from which the lane keeps byte g of word j.
#include "pdelta_device.h"
#include "pdelta_host.h"

namespace pdelta {

template <int DT>
__device__ __forceinline__ float4v mfma16(uint4v a, uint4v b, float4v c) {
    if constexpr (DT == kBF16)
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a),
                                                       __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8, a),
                                                      __builtin_bit_cast(half8, b), c, 0, 0, 0);
}

// Eight sign bits (bit e <-> element e, 1 = +1) to eight +-1.0 values of dtype DT.
template <int DT>
__device__ __forceinline__ uint4v expand_signs(uint32_t byte) {
    constexpr uint32_t one2 = DT == kBF16 ? 0x3F803F80u : 0x3C003C00u;
    const uint32_t neg = ~byte;
    uint4v r;
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        const uint32_t t = neg >> (2 * p);
        r[p] = one2 | ((t & 1u) << 15) | ((t & 2u) << 30);
    }
    return r;
}

// Column mode: the sign-part operand is fp16(X * v_col), whatever the dtype of X.
template <int XDT>
__device__ __forceinline__ uint4v scale_x(uint4v x, uint4v v) {
    uint4v r;
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        if constexpr (XDT == kF16) {
            const uint32_t xp = x[p], vp = v[p];
            r[p] = as_u32(as_half2(xp) * as_half2(vp));                        // v_pk_mul_f16
        } else {
            const float lo = bf16_bits_to_f32(x[p] & 0xFFFFu) * f16_bits_to_f32(v[p] & 0xFFFFu);
            const float hi = bf16_bits_to_f32(x[p] >> 16) * f16_bits_to_f32(v[p] >> 16);
            r[p] = f32_to_f16_bits(lo) | (f32_to_f16_bits(hi) << 16);
        }
    }
    return r;
}

template <int MT, int AXIS>
struct SkinnyStep {
    uint4v w[4];        // W_b operand, one per 32-input block
    uint4v sw;          // the step's four sign words of this lane's row
    uint4v x[MT][4];    // X operand per 16-token tile
    uint4v vc[4];       // v_col (column mode only)
};

template <int MT, int AXIS, bool K128>
__device__ __forceinline__ void skinny_load(SkinnyStep<MT, AXIS>& r, const uint16_t* wrow,
                                            const uint32_t* brow, const uint16_t* const (&xrow)[MT],
                                            const uint16_t* vcol, int kb, int K)
{
    const uint4v zero = {0, 0, 0, 0};
    if constexpr (K128) {
        r.sw = *(const uint4v*)(brow + (kb >> 5));
    } else {
#pragma unroll
        for (int j = 0; j < 4; ++j) r.sw[j] = kb + j * 32 < K ? brow[(kb >> 5) + j] : 0u;
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int k = kb + j * 32;
        const bool live = K128 || k < K;
        r.w[j] = live ? *(const uint4v*)(wrow + k) : zero;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
            r.x[mt][j] = (live && xrow[mt] != nullptr) ? *(const uint4v*)(xrow[mt] + k) : zero;
        if constexpr (AXIS == 1) r.vc[j] = live ? *(const uint4v*)(vcol + k) : zero;
    }
}

template <int XDT, int MT, int AXIS>
__device__ __forceinline__ void skinny_compute(const SkinnyStep<MT, AXIS>& r, int g,
                                               float4v (&accb)[MT], float4v (&accs)[MT])
{
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const uint32_t byte = (r.sw[j] >> (g * 8)) & 0xFFu;
        if constexpr (AXIS == 0) {
            const uint4v s = expand_signs<XDT>(byte);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                accb[mt] = mfma16<XDT>(r.x[mt][j], r.w[j], accb[mt]);
                accs[mt] = mfma16<XDT>(r.x[mt][j], s, accs[mt]);
            }
        } else {
            const uint4v s = expand_signs<kF16>(byte);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                accb[mt] = mfma16<XDT>(r.x[mt][j], r.w[j], accb[mt]);
                accs[mt] = mfma16<kF16>(scale_x<XDT>(r.x[mt][j], r.vc[j]), s, accs[mt]);
            }
        }
    }
}

// grid.x = ceil(d_out / 16); block = WAVES * 64; dynamic LDS = WAVES * MT * 256 floats.
template <int XDT, int AXIS, int MT, int WAVES, bool K128>
__global__ void __launch_bounds__(WAVES * 64)
linear_skinny_kernel(const uint16_t* __restrict__ X, const uint16_t* __restrict__ W_b,
                     const uint32_t* __restrict__ B_packed, const uint16_t* __restrict__ v,
                     void* __restrict__ Y, int M, int d_out, int d_in, int y_dtype)
{
    extern __shared__ float red[];                    // [WAVES][MT][4][64]
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n = lane & 15, g = lane >> 4;
    const int n0 = blockIdx.x * 16;
    const int o = min(n0 + n, d_out - 1);             // rows past the end repeat the last one
    const int K = d_in;

    const uint16_t* wrow = W_b + (int64_t)o * K + g * 8;
    const uint32_t* brow = B_packed + (int64_t)o * (K >> 5);
    const uint16_t* vcol = AXIS == 1 ? v + g * 8 : nullptr;
    const uint16_t* xrow[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const int t = mt * 16 + n;                    // A operand: lane % 16 is the token
        xrow[mt] = t < M ? X + (int64_t)t * K + g * 8 : nullptr;
    }

    float4v accb[MT], accs[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        accb[mt] = (float4v){0.f, 0.f, 0.f, 0.f};
        accs[mt] = (float4v){0.f, 0.f, 0.f, 0.f};
    }

    const int nsteps = (K + 127) >> 7;
    SkinnyStep<MT, AXIS> cur, nxt;
    int s = wave;
    if (s < nsteps) skinny_load<MT, AXIS, K128>(cur, wrow, brow, xrow, vcol, s << 7, K);
    while (s < nsteps) {
        const int s2 = s + WAVES;
        if (s2 < nsteps) skinny_load<MT, AXIS, K128>(nxt, wrow, brow, xrow, vcol, s2 << 7, K);
        skinny_compute<XDT, MT, AXIS>(cur, g, accb, accs);
        cur = nxt;
        s = s2;
    }

    // Accumulator layout: element r of lane (n, g) is token g*4 + r, output row n0 + n.
    float vr = 1.0f;
    if constexpr (AXIS == 0) vr = f16_bits_to_f32(v[o]);
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int r = 0; r < 4; ++r)
            red[((wave * MT + mt) * 4 + r) * 64 + lane] = accb[mt][r] + vr * accs[mt][r];
    __syncthreads();

    for (int idx = threadIdx.x; idx < MT * 256; idx += WAVES * 64) {
        float sum = 0.f;
#pragma unroll
        for (int w = 0; w < WAVES; ++w) sum += red[w * (MT * 256) + idx];
        const int ln = idx & 63, r = (idx >> 6) & 3, mt = idx >> 8;
        const int t = mt * 16 + (ln >> 4) * 4 + r;
        const int oo = n0 + (ln & 15);
        if (t < M && oo < d_out) {
            const int64_t yi = (int64_t)t * d_out + oo;
            if (y_dtype == kF32) store_y<kF32>(Y, yi, sum);
            else if (y_dtype == kBF16) store_y<kBF16>(Y, yi, sum);
            else store_y<kF16>(Y, yi, sum);
        }
    }
}

template <int XDT, int AXIS, int MT, int WAVES, bool K128>
static int launch_one(const void* X, const void* W_b, const uint32_t* B_packed, const uint16_t* v,
                      void* Y, int64_t M, int64_t d_out, int64_t d_in, int y_dtype,
                      hipStream_t stream)
{
    const dim3 grid((unsigned)((d_out + 15) / 16));
    const size_t lds = (size_t)WAVES * MT * 256 * sizeof(float);
    hipLaunchKernelGGL((linear_skinny_kernel<XDT, AXIS, MT, WAVES, K128>), grid, dim3(WAVES * 64), lds,
                       stream, (const uint16_t*)X, (const uint16_t*)W_b, B_packed, v, Y, (int)M,
                       (int)d_out, (int)d_in, y_dtype);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

template <int XDT, int AXIS, bool K128>
static int launch_by_tokens(const void* X, const void* W_b, const uint32_t* B_packed,
                            const uint16_t* v, void* Y, int64_t M, int64_t d_out, int64_t d_in,
                            int y_dtype, hipStream_t stream)
{
#define PDELTA_GO(MT, WAVES) \
    return launch_one<XDT, AXIS, MT, WAVES, K128>(X, W_b, B_packed, v, Y, M, d_out, d_in, y_dtype, stream)
    const int waves = tune_value("skinny_waves", 8);
    if (M <= 16) {
        if (waves == 4) PDELTA_GO(1, 4);
        if (waves == 16) PDELTA_GO(1, 16);
        PDELTA_GO(1, 8);
    }
    if (M <= 32) {
        if (waves == 4) PDELTA_GO(2, 4);
        PDELTA_GO(2, 8);
    }
    if (M <= 48) PDELTA_GO(3, 8);
    PDELTA_GO(4, 8);
#undef PDELTA_GO
}

int launch_linear_skinny(int x_dtype, int y_dtype, int axis, const void* X, const void* W_b,
                         const uint32_t* B_packed, const uint16_t* v, void* Y, int64_t M,
                         int64_t d_out, int64_t d_in, hipStream_t stream)
{
    const bool k128 = d_in % 128 == 0;
#define PDELTA_SEL(XDT, AXIS)                                                                      \
    return k128 ? launch_by_tokens<XDT, AXIS, true>(X, W_b, B_packed, v, Y, M, d_out, d_in, y_dtype, stream) \
                : launch_by_tokens<XDT, AXIS, false>(X, W_b, B_packed, v, Y, M, d_out, d_in, y_dtype, stream)
    if (x_dtype == kBF16) {
        if (axis == 0) PDELTA_SEL(kBF16, 0);
        PDELTA_SEL(kBF16, 1);
    }
    if (axis == 0) PDELTA_SEL(kF16, 0);
    PDELTA_SEL(kF16, 1);
#undef PDELTA_SEL
}

}  // namespace pdelta
