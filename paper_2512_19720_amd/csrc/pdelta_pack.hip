// pdelta_pack: B = sign(W_f - W_b) bit-packed along the input axis, plus the per-axis
// mean |W_f - W_b| that initialises the scale vectors (paper Section 2; per-layer compression
// algorithm: "B <- Pack(sign(dW)^T)", "v_c <- mean(|dW|, axis=1)", "v_r <- mean(|dW|, axis=0)").
//
// One streaming pass over both matrices (4 B read, 1/8 B written per weight): HBM-bound.
//   pack_zero_kernel      clears the d_out + d_in partial sums in the workspace
//   pack_main_kernel      signs -> words, |dW| -> per-row / per-column partial sums (atomics)
//   pack_finalize_kernel  sum / count, rounded once to fp16
//
// Exact sums.  fp16 values are integer multiples of 2^-24 below 2^16, so W_f - W_b is exact in
// fp64 and every |dW| * 2^24 is an integer below 2^41.  Lanes add a handful of them in fp64
// (still exact), convert to uint64 and from there on all adding is integer: the result does
// not depend on the order in which waves and workgroups arrive.  bf16 has no such grid, so its
// sums stay in fp64 (hardware fp64 atomics) and are exact only while fp64 holds them exactly.
#include "pdelta_device.h"
#include "pdelta_host.h"

namespace pdelta {

constexpr int kPackThreads = 256;              // 4 waves
constexpr int kPackWaves = kPackThreads / kWave;
constexpr int kPackChunk = kWave * 8;          // 512 columns: one 16-byte load per lane
constexpr int kPackChunks = 2;                 // column tile = 1024
constexpr int kPackTileCols = kPackChunk * kPackChunks;
constexpr int kPackRowsPerWave = 8;
constexpr int kPackTileRows = kPackWaves * kPackRowsPerWave;   // 32

template <int DT> struct PackAcc;
template <> struct PackAcc<kF16> {
    typedef unsigned long long type;                                      // units of 2^-24
    static __device__ __forceinline__ type from_partial(double s) { return (type)(s * 16777216.0); }
    static __device__ __forceinline__ double to_double(type s) { return (double)s * (1.0 / 16777216.0); }
    static __device__ __forceinline__ type wave_total(type x) { return wave_sum_u64(x); }
    static __device__ __forceinline__ void atomic_add(type* p, type x) { atomicAdd(p, x); }
};
template <> struct PackAcc<kBF16> {
    typedef double type;
    static __device__ __forceinline__ type from_partial(double s) { return s; }
    static __device__ __forceinline__ double to_double(type s) { return s; }
    static __device__ __forceinline__ type wave_total(type x) { return wave_sum_f64(x); }
    static __device__ __forceinline__ void atomic_add(type* p, type x) { unsafeAtomicAdd(p, x); }
};

__global__ void __launch_bounds__(256) pack_zero_kernel(unsigned long long* ws, int64_t n) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) ws[i] = 0ull;                   // all-zero bits are also +0.0
}

// Workgroup tile: 32 rows x 1024 columns.  Wave w owns rows w*8 .. w*8+7 of the tile; lane l
// owns columns chunk*512 + l*8 .. +7 of each chunk, i.e. one 16-byte load per matrix, and so the
// sign byte number l of that chunk.  Four lanes make one output word.
template <int DT>
__global__ void __launch_bounds__(kPackThreads)
pack_main_kernel(const uint16_t* __restrict__ W_f, const uint16_t* __restrict__ W_b,
                 int d_out, int d_in, uint32_t* __restrict__ B_packed,
                 typename PackAcc<DT>::type* __restrict__ row_sum,     // [d_out] or nullptr
                 typename PackAcc<DT>::type* __restrict__ col_sum)     // [d_in]  or nullptr
{
    typedef typename PackAcc<DT>::type acc_t;
    __shared__ double col_part[kPackWaves][kPackTileCols];               // 32 KB

    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const int col0 = blockIdx.y * kPackTileCols;                          // few column tiles
    const int row0 = blockIdx.x * kPackTileRows + wave * kPackRowsPerWave;
    const int words_per_row = d_in / 32;

    double csum[kPackChunks][8];
#pragma unroll
    for (int c = 0; c < kPackChunks; ++c)
#pragma unroll
        for (int e = 0; e < 8; ++e) csum[c][e] = 0.0;

#pragma unroll 2
    for (int r = 0; r < kPackRowsPerWave; ++r) {
        const int row = row0 + r;
        if (row >= d_out) break;                                         // wave-uniform
        double rsum = 0.0;
#pragma unroll
        for (int c = 0; c < kPackChunks; ++c) {
            const int col = col0 + c * kPackChunk + lane * 8;
            const bool live = col < d_in;                                // d_in % 8 == 0
            uint4v a = {0, 0, 0, 0}, b = {0, 0, 0, 0};
            if (live) {
                const int64_t off = (int64_t)row * d_in + col;
                a = *(const uint4v*)(W_f + off);
                b = *(const uint4v*)(W_b + off);
            }
            uint32_t byte = 0;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const uint32_t ha = (a[e >> 1] >> ((e & 1) * 16)) & 0xFFFFu;
                const uint32_t hb = (b[e >> 1] >> ((e & 1) * 16)) & 0xFFFFu;
                const float fa = bits_to_f32<DT>(ha), fb = bits_to_f32<DT>(hb);
                byte |= (fa < fb ? 0u : 1u) << e;                        // sign(0) -> +1
                const double d = fabs((double)fa - (double)fb);          // exact for fp16
                rsum += d;
                csum[c][e] += d;
            }
            // gather the four bytes of a word in its first lane
            uint32_t word = byte << ((lane & 3) * 8);
            word |= __shfl_xor(word, 1, kWave);
            word |= __shfl_xor(word, 2, kWave);
            if (live && (lane & 3) == 0)
                B_packed[(int64_t)row * words_per_row + (col >> 5)] = word;
        }
        if (row_sum != nullptr) {
            const acc_t total = PackAcc<DT>::wave_total(PackAcc<DT>::from_partial(rsum));
            if (lane == 0) PackAcc<DT>::atomic_add(row_sum + row, total);
        }
    }

    if (col_sum != nullptr) {                                            // grid-uniform
#pragma unroll
        for (int c = 0; c < kPackChunks; ++c)
#pragma unroll
            for (int e = 0; e < 8; ++e) col_part[wave][c * kPackChunk + lane * 8 + e] = csum[c][e];
        __syncthreads();
        for (int j = threadIdx.x; j < kPackTileCols; j += kPackThreads) {
            const int col = col0 + j;
            if (col < d_in) {
                // each term is an exact fp64 sum of <= 8 values; add them as accumulator units
                acc_t s = PackAcc<DT>::from_partial(col_part[0][j]);
#pragma unroll
                for (int w = 1; w < kPackWaves; ++w) s += PackAcc<DT>::from_partial(col_part[w][j]);
                PackAcc<DT>::atomic_add(col_sum + col, s);
            }
        }
    }
}

template <int DT>
__global__ void __launch_bounds__(256)
pack_finalize_kernel(const typename PackAcc<DT>::type* __restrict__ sums, int64_t n_row,
                     int64_t n_col, double row_count, double col_count,
                     uint16_t* __restrict__ v_row, uint16_t* __restrict__ v_col)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n_row) {
        if (v_row != nullptr)
            v_row[i] = (uint16_t)f64_to_f16_bits_rne(PackAcc<DT>::to_double(sums[i]) / row_count);
    } else if (i < n_row + n_col) {
        if (v_col != nullptr)
            v_col[i - n_row] =
                (uint16_t)f64_to_f16_bits_rne(PackAcc<DT>::to_double(sums[i]) / col_count);
    }
}

template <int DT>
static int launch_pack(const void* W_f, const void* W_b, int64_t d_out, int64_t d_in,
                       uint32_t* B_packed, uint16_t* v_row, uint16_t* v_col, void* workspace,
                       hipStream_t stream)
{
    typedef typename PackAcc<DT>::type acc_t;
    acc_t* sums = (acc_t*)workspace;                 // [d_out] row sums, then [d_in] column sums
    const int64_t n = d_out + d_in;
    const bool want_any = v_row != nullptr || v_col != nullptr;
    if (want_any)
        hipLaunchKernelGGL(pack_zero_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream,
                           (unsigned long long*)workspace, n);
    dim3 grid((unsigned)((d_out + kPackTileRows - 1) / kPackTileRows),
              (unsigned)((d_in + kPackTileCols - 1) / kPackTileCols));
    hipLaunchKernelGGL(pack_main_kernel<DT>, grid, dim3(kPackThreads), 0, stream,
                       (const uint16_t*)W_f, (const uint16_t*)W_b, (int)d_out, (int)d_in, B_packed,
                       v_row ? sums : (acc_t*)nullptr, v_col ? sums + d_out : (acc_t*)nullptr);
    if (want_any)
        hipLaunchKernelGGL(pack_finalize_kernel<DT>, dim3((unsigned)((n + 255) / 256)), dim3(256), 0,
                           stream, (const acc_t*)sums, d_out, d_in, (double)d_in, (double)d_out,
                           v_row, v_col);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

int launch_pack_dispatch(int w_dtype, const void* W_f, const void* W_b, int64_t d_out,
                         int64_t d_in, uint32_t* B_packed, uint16_t* v_row, uint16_t* v_col,
                         void* workspace, hipStream_t stream)
{
    if (w_dtype == kBF16)
        return launch_pack<kBF16>(W_f, W_b, d_out, d_in, B_packed, v_row, v_col, workspace, stream);
    return launch_pack<kF16>(W_f, W_b, d_out, d_in, B_packed, v_row, v_col, workspace, stream);
}

}  // namespace pdelta
