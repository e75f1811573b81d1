// Prefill-shaped delta linear layer (many tokens): Y = X * W_hat^T with
// W_hat = W_b + v (.) B (paper Eq. 1) built tile by tile on the way into LDS and never written
// to memory.  One MFMA stream: the tile of W_hat is formed as fp16(W_b +- v) with a packed fp16
// add (one rounding of the exact sum), X is used as fp16, products accumulate in fp32.
// bf16 operands are converted to fp16 while they are staged; this is exact for magnitudes in
// [2^-14, 65504] (bf16 carries 8 significant bits, fp16 11) and is the reason for the stated
// operand range of the prefill path.
//
// Tile: 128 tokens x 128 output rows x 64 inputs per step, 256 threads = 4 waves in a 2 x 2
// arrangement, each wave 64 x 64 outputs as 2 x 2 MFMA 32x32x16 tiles.  Global loads for step
// s+1 are in flight while step s is multiplied out of LDS.
#include "pdelta_device.h"
#include "pdelta_host.h"

namespace pdelta {

constexpr int kGemmBM = 128, kGemmBN = 128, kGemmBK = 64;
constexpr int kGemmLDK = kGemmBK + 8;   // padded LDS row (halves): 144 B stride, conflict-free b128 reads
constexpr int kGemmThreads = 256;

__device__ __forceinline__ uint32_t bf16pair_to_f16pair(uint32_t d) {
    const float lo = __builtin_bit_cast(float, d << 16);
    const float hi = __builtin_bit_cast(float, d & 0xFFFF0000u);
    return __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(lo, hi));
}

template <int XDT>
__device__ __forceinline__ uint4v to_f16x8(uint4v a) {
    if constexpr (XDT == kBF16) {
        uint4v r;
#pragma unroll
        for (int p = 0; p < 4; ++p) r[p] = bf16pair_to_f16pair(a[p]);
        return r;
    } else {
        return a;
    }
}

// Eight fp16 weights + eight sign bits + packed scales -> eight fp16 values of W_hat.
// vv[p] holds the fp16 scales of elements 2p (low half) and 2p+1 (high half).
__device__ __forceinline__ uint4v apply_delta(uint4v w, uint32_t byte, uint4v vv) {
    const uint32_t neg = ~byte;
    uint4v r;
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        const uint32_t t = neg >> (2 * p);
        const uint32_t flip = ((t & 1u) << 15) | ((t & 2u) << 30);
        const uint32_t wp = w[p], sv = vv[p] ^ flip;                            // sv = +-v
        r[p] = as_u32(as_half2(wp) + as_half2(sv));                             // v_pk_add_f16
    }
    return r;
}

template <int XDT, int AXIS>
__global__ void __launch_bounds__(kGemmThreads)
linear_gemm_kernel(const uint16_t* __restrict__ X, const uint16_t* __restrict__ W_b,
                   const uint32_t* __restrict__ B_packed, const uint16_t* __restrict__ v,
                   void* __restrict__ Y, int M, int d_out, int d_in, int y_dtype)
{
    __shared__ __attribute__((aligned(16))) uint16_t Xs[kGemmBM * kGemmLDK];
    __shared__ __attribute__((aligned(16))) uint16_t Ws[kGemmBN * kGemmLDK];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int n0 = blockIdx.x * kGemmBN;
    const int m0 = blockIdx.y * kGemmBM;
    const int K = d_in;
    const uint8_t* B_bytes = (const uint8_t*)B_packed;

    // staging role: thread covers 8 inputs (16 bytes) at column ld_c of rows ld_row + 32 q
    const int ld_row = tid >> 3, ld_c = (tid & 7) * 8;

    uint4v vrow[4];
    if constexpr (AXIS == 0) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int o = n0 + ld_row + 32 * q;
            const uint32_t h = o < d_out ? v[o] : 0u;
            const uint32_t hh = h | (h << 16);
            vrow[q] = (uint4v){hh, hh, hh, hh};
        }
    }

    uint4v xg[4], wg[4], vcg;
    uint32_t sb[4];
    const uint4v zero = {0, 0, 0, 0};

    auto load_global = [&](int kb) {
        const int col = kb + ld_c;
        const bool col_ok = col < K;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int tok = m0 + ld_row + 32 * q;
            xg[q] = (col_ok && tok < M) ? *(const uint4v*)(X + (int64_t)tok * K + col) : zero;
            const int o = n0 + ld_row + 32 * q;
            if (col_ok && o < d_out) {
                const int64_t off = (int64_t)o * K + col;
                wg[q] = *(const uint4v*)(W_b + off);
                sb[q] = B_bytes[off >> 3];
            } else {
                wg[q] = zero;
                sb[q] = 0xFFu;
            }
        }
        if constexpr (AXIS == 1) vcg = col_ok ? *(const uint4v*)(v + col) : zero;
    };

    auto store_lds = [&]() {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int r = ld_row + 32 * q;
            *(uint4v*)(Xs + r * kGemmLDK + ld_c) = to_f16x8<XDT>(xg[q]);
            const uint4v w16 = to_f16x8<XDT>(wg[q]);
            *(uint4v*)(Ws + r * kGemmLDK + ld_c) = apply_delta(w16, sb[q], AXIS == 0 ? vrow[q] : vcg);
        }
    };

    float16v acc[2][2];
#pragma unroll
    for (int f = 0; f < 2; ++f)
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[f][h][r] = 0.f;

    const int frag_row = lane & 31, frag_k = (lane >> 5) * 8;

    load_global(0);
    store_lds();
    __syncthreads();
    for (int kb = 0; kb < K; kb += kGemmBK) {
        const bool more = kb + kGemmBK < K;
        if (more) load_global(kb + kGemmBK);
#pragma unroll
        for (int ks = 0; ks < kGemmBK / 16; ++ks) {
            half8 a[2], b[2];
#pragma unroll
            for (int f = 0; f < 2; ++f)
                a[f] = *(const half8*)(Xs + (wm * 64 + f * 32 + frag_row) * kGemmLDK + ks * 16 + frag_k);
#pragma unroll
            for (int h = 0; h < 2; ++h)
                b[h] = *(const half8*)(Ws + (wn * 64 + h * 32 + frag_row) * kGemmLDK + ks * 16 + frag_k);
#pragma unroll
            for (int f = 0; f < 2; ++f)
#pragma unroll
                for (int h = 0; h < 2; ++h)
                    acc[f][h] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[f], b[h], acc[f][h], 0, 0, 0);
        }
        __syncthreads();
        if (more) {
            store_lds();
            __syncthreads();
        }
    }

    // 32x32 accumulator: element r of lane l is row (r/4)*8 + (l/32)*4 + r%4, column l%32.
#pragma unroll
    for (int f = 0; f < 2; ++f)
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int o = n0 + wn * 64 + h * 32 + (lane & 31);
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int tok = m0 + wm * 64 + f * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
                if (tok < M && o < d_out) {
                    const int64_t yi = (int64_t)tok * d_out + o;
                    const float val = acc[f][h][r];
                    if (y_dtype == kF32) store_y<kF32>(Y, yi, val);
                    else if (y_dtype == kBF16) store_y<kBF16>(Y, yi, val);
                    else store_y<kF16>(Y, yi, val);
                }
            }
        }
}

template <int XDT, int AXIS>
static int launch_gemm(const void* X, const void* W_b, const uint32_t* B_packed, const uint16_t* v,
                       void* Y, int64_t M, int64_t d_out, int64_t d_in, int y_dtype,
                       hipStream_t stream)
{
    const dim3 grid((unsigned)((d_out + kGemmBN - 1) / kGemmBN), (unsigned)((M + kGemmBM - 1) / kGemmBM));
    hipLaunchKernelGGL((linear_gemm_kernel<XDT, AXIS>), grid, dim3(kGemmThreads), 0, stream,
                       (const uint16_t*)X, (const uint16_t*)W_b, B_packed, v, Y, (int)M, (int)d_out,
                       (int)d_in, y_dtype);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

int launch_linear_gemm(int x_dtype, int y_dtype, int axis, const void* X, const void* W_b,
                       const uint32_t* B_packed, const uint16_t* v, void* Y, int64_t M,
                       int64_t d_out, int64_t d_in, hipStream_t stream)
{
    if (x_dtype == kBF16)
        return axis == 0 ? launch_gemm<kBF16, 0>(X, W_b, B_packed, v, Y, M, d_out, d_in, y_dtype, stream)
                         : launch_gemm<kBF16, 1>(X, W_b, B_packed, v, Y, M, d_out, d_in, y_dtype, stream);
    return axis == 0 ? launch_gemm<kF16, 0>(X, W_b, B_packed, v, Y, M, d_out, d_in, y_dtype, stream)
                     : launch_gemm<kF16, 1>(X, W_b, B_packed, v, Y, M, d_out, d_in, y_dtype, stream);
}

}  // namespace pdelta
