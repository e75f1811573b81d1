// Gradient of a loss with respect to the scale vector v, given dY = dL/dY (paper, algorithm
// "Train per-row/column scaling vectors via activation matching": the loss is backpropagated
// through v only).  With Y[m,o] = sum_i X[m,i] (W_b[o,i] + v. B[o,i])  (Eq. 1 in the layer):
//   row:  dL/dv[o] = sum_m dY[m,o] * (X B^T)[m,o]
//   col:  dL/dv[i] = sum_m X[m,i]  * (dY B)[m,i]
// Both are one matrix product with the +-1 matrix followed by an elementwise product and a sum
// over the tokens; W_b is not needed.  Column mode is row mode with the roles of X and dY
// swapped and the sign matrix transposed, so the library transposes the packed bits once into
// the workspace and runs the same kernel.
//
// Kernel: the prefill tile (256 tokens x 128 outputs x 64 inputs, 8 waves of 64 x 64, MFMA
// 32x32x16 in the operands' own dtype: +-1 is exact in fp16 and bf16, so nothing is converted).
// The epilogue multiplies each accumulator by its G entry and sums the tile's 256 tokens; tiles
// write one partial per (token tile, output) to the workspace and a second kernel adds the
// partials in a fixed order: no atomics, reproducible.
#include <type_traits>

#include "pdelta.h"
#include "pdelta_device.h"
#include "pdelta_host.h"

namespace pdelta {

constexpr int kGradBM = 256, kGradBN = 128, kGradBK = 64;
constexpr int kGradLDK = kGradBK + 8;                 // LDS row in halves (144 bytes)

template <int DT>
__device__ __forceinline__ float16v grad_mfma(uint4v a, uint4v b, float16v c) {
    if constexpr (DT == kBF16)
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a),
                                                       __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(half8, a),
                                                      __builtin_bit_cast(half8, b), c, 0, 0, 0);
}

// Eight sign bits (bit e <-> element e, 1 = +1) to eight +-1.0 values of dtype DT.
template <int DT>
__device__ __forceinline__ uint4v grad_expand(uint32_t byte) {
    constexpr uint32_t one2 = DT == kBF16 ? 0x3F803F80u : 0x3C003C00u;
    const uint32_t neg = ~byte & 0xFFu;               // higher bits would leak into bit 31 below
    uint4v r;
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        const uint32_t spread = (neg << (30 - 2 * p)) | (neg << (15 - 2 * p));
        r[p] = (spread & 0x80008000u) | one2;
    }
    return r;
}

// partial[tile_m][n] = sum over the tile's tokens m of G[m,n] * sum_k A[m,k] S[n,k],
// A [M, Kc], G [M, Nc], S = +-1 from bits [Nc][Kc/32]; Kc % 32 == 0.
template <int DT>
__global__ void __launch_bounds__(512, 4)
grad_tile_kernel(const uint16_t* __restrict__ A, const uint16_t* __restrict__ G,
                 const uint32_t* __restrict__ bits, float* __restrict__ partial, int M, int Nc, int Kc,
                 int m_tiles)
{
    constexpr int BM = kGradBM, BN = kGradBN, BK = kGradBK, LDK = kGradLDK, ROWS = 64, XQ = 4, WQ = 2;
    __shared__ __attribute__((aligned(16))) uint16_t As[BM * LDK];
    __shared__ __attribute__((aligned(16))) uint16_t Ss[BN * LDK];

    const int tile_m = blockIdx.x % m_tiles, tile_n = blockIdx.x / m_tiles;
    const int m0 = tile_m * BM, n0 = tile_n * BN;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;

    // staging role: 8 inputs (16 bytes of A, one sign byte) at column ld_c of rows ld_row + 64 q;
    // rows past the end are clamped (they only feed results that are never used)
    const int ld_row = tid >> 3, ld_c = (tid & 7) * 8;
    const char* abase = (const char*)(A + (int64_t)m0 * Kc);
    const char* sbase = (const char*)bits + (((int64_t)n0 * Kc) >> 3);
    uint32_t aoff[XQ], soff[WQ];
#pragma unroll
    for (int q = 0; q < XQ; ++q) {
        const int row = min(m0 + ld_row + ROWS * q, M - 1) - m0;
        aoff[q] = ((uint32_t)row * (uint32_t)Kc + (uint32_t)ld_c) * 2u;
    }
#pragma unroll
    for (int q = 0; q < WQ; ++q) {
        const int row = min(n0 + ld_row + ROWS * q, Nc - 1) - n0;
        soff[q] = (uint32_t)row * (uint32_t)(Kc >> 3) + (uint32_t)(tid & 7);
    }
    uint4v ag[XQ];
    uint32_t sb[WQ];
    const uint4v zero = {0, 0, 0, 0};
    auto load_global = [&](int kb, auto guard) {
        constexpr bool GUARD = decltype(guard)::value;
        const bool col_ok = !GUARD || kb + ld_c < Kc;
        const char* ab = abase + (int64_t)kb * 2;
        const char* sp = sbase + (kb >> 3);
#pragma unroll
        for (int q = 0; q < XQ; ++q) ag[q] = col_ok ? *(const uint4v*)(ab + aoff[q]) : zero;
#pragma unroll
        for (int q = 0; q < WQ; ++q) sb[q] = col_ok ? (uint32_t) * (const uint8_t*)(sp + soff[q]) : 0xFFu;
    };
    auto store_lds = [&]() {
#pragma unroll
        for (int q = 0; q < XQ; ++q) *(uint4v*)(As + (ld_row + ROWS * q) * LDK + ld_c) = ag[q];
#pragma unroll
        for (int q = 0; q < WQ; ++q) *(uint4v*)(Ss + (ld_row + ROWS * q) * LDK + ld_c) = grad_expand<DT>(sb[q]);
    };

    float16v acc[2][2];
#pragma unroll
    for (int f = 0; f < 2; ++f)
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[f][h][r] = 0.f;

    const int frag_row = lane & 31, frag_k = (lane >> 5) * 8;
    const uint16_t* a_base = As + (wm * 64 + frag_row) * LDK + frag_k;
    const uint16_t* b_base = Ss + (wn * 64 + frag_row) * LDK + frag_k;
    auto multiply_stage = [&]() {
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            uint4v a[2], b[2];
#pragma unroll
            for (int f = 0; f < 2; ++f) a[f] = *(const uint4v*)(a_base + f * 32 * LDK + ks * 16);
#pragma unroll
            for (int h = 0; h < 2; ++h) b[h] = *(const uint4v*)(b_base + h * 32 * LDK + ks * 16);
#pragma unroll
            for (int f = 0; f < 2; ++f)
#pragma unroll
                for (int h = 0; h < 2; ++h) acc[f][h] = grad_mfma<DT>(a[f], b[h], acc[f][h]);
        }
    };

    const int full_steps = Kc / BK;
    const bool tail = (Kc % BK) != 0;                 // then one more step of 32 inputs
    if (full_steps > 0) load_global(0, std::false_type{});
    else load_global(0, std::true_type{});
    for (int i = 0; i + 1 < full_steps; ++i) {
        store_lds();
        __syncthreads();
        load_global((i + 1) * BK, std::false_type{});
        __builtin_amdgcn_sched_barrier(0);            // keep the loads above the multiplication
        multiply_stage();
        __syncthreads();
    }
    if (full_steps > 0) {
        store_lds();
        __syncthreads();
        if (tail) load_global(full_steps * BK, std::true_type{});
        multiply_stage();
        __syncthreads();
    }
    if (tail) {
        store_lds();
        __syncthreads();
        multiply_stage();
        __syncthreads();
    }

    // epilogue: acc[f][h][r] is token m0 + 64 wm + 32 f + 8 (r / 4) + 4 (lane / 32) + r % 4,
    // output n0 + 64 wn + 32 h + lane % 32.  Multiply by G, sum the wave's 64 tokens, then the
    // four token groups of the tile in LDS (As is free now).
    float* red = (float*)As;                           // [4 wm][128]
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int n = n0 + wn * 64 + h * 32 + (lane & 31);
        const int nc = min(n, Nc - 1);
        float s = 0.f;
#pragma unroll
        for (int f = 0; f < 2; ++f)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int tok = m0 + wm * 64 + f * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
                const uint32_t gbits = G[(int64_t)min(tok, M - 1) * Nc + nc];
                const float gval = tok < M ? bits_to_f32<DT>(gbits) : 0.f;
                s += gval * acc[f][h][r];
            }
        s += __shfl_xor(s, 32, kWave);
        if (lane < 32) red[wm * BN + wn * 64 + h * 32 + lane] = s;
    }
    __syncthreads();
    if (tid < BN) {
        const int n = n0 + tid;
        if (n < Nc) partial[(int64_t)tile_m * Nc + n] = (red[tid] + red[BN + tid]) + (red[2 * BN + tid] + red[3 * BN + tid]);
    }
}

// Pipelined form of grad_tile_kernel, organised like the prefill kernel of the same tile: one
// workgroup per CU, two LDS stages and two register sets.  During step s a wave multiplies stage
// s % 2 and, between its groups of four MFMAs, stages the operands of step s+1 (loaded one step
// earlier) into the other stage while the loads of step s+2 are in flight: one barrier per step.
struct GradRegs {
    uint4v ag[4];
    uint32_t sb[2];
};

template <int DT>
__global__ void __launch_bounds__(512, 2)
grad_tile_pipe_kernel(const uint16_t* __restrict__ A, const uint16_t* __restrict__ G,
                      const uint32_t* __restrict__ bits, float* __restrict__ partial, int M, int Nc, int Kc,
                      int m_tiles)
{
    constexpr int BM = kGradBM, BN = kGradBN, BK = kGradBK, LDK = kGradLDK, ROWS = 64, XQ = 4, WQ = 2;
    constexpr int AS = BM * LDK, STAGE = (BM + BN) * LDK;                 // halves
    extern __shared__ __attribute__((aligned(16))) unsigned char grad_smem[];
    uint16_t* lds = (uint16_t*)grad_smem;                                 // [2][STAGE]: A tile then sign tile

    const int tile_m = blockIdx.x % m_tiles, tile_n = blockIdx.x / m_tiles;
    const int m0 = tile_m * BM, n0 = tile_n * BN;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;

    const int ld_row = tid >> 3, ld_c = (tid & 7) * 8;
    const char* abase = (const char*)(A + (int64_t)m0 * Kc);
    const char* sbase = (const char*)bits + (((int64_t)n0 * Kc) >> 3);
    uint32_t aoff[XQ], soff[WQ];
#pragma unroll
    for (int q = 0; q < XQ; ++q) {
        const int row = min(m0 + ld_row + ROWS * q, M - 1) - m0;
        aoff[q] = ((uint32_t)row * (uint32_t)Kc + (uint32_t)ld_c) * 2u;
    }
#pragma unroll
    for (int q = 0; q < WQ; ++q) {
        const int row = min(n0 + ld_row + ROWS * q, Nc - 1) - n0;
        soff[q] = (uint32_t)row * (uint32_t)(Kc >> 3) + (uint32_t)(tid & 7);
    }
    const uint4v zero = {0, 0, 0, 0};
    auto load_global = [&](GradRegs& R, int kb, auto guard) {
        constexpr bool GUARD = decltype(guard)::value;
        const bool col_ok = !GUARD || kb + ld_c < Kc;
        const char* ab = abase + (int64_t)kb * 2;
        const char* sp = sbase + (kb >> 3);
#pragma unroll
        for (int q = 0; q < XQ; ++q) R.ag[q] = col_ok ? *(const uint4v*)(ab + aoff[q]) : zero;
#pragma unroll
        for (int q = 0; q < WQ; ++q) R.sb[q] = col_ok ? (uint32_t) * (const uint8_t*)(sp + soff[q]) : 0xFFu;
    };
    // quarter c of the staging work of one step
    auto stage_part = [&](const GradRegs& R, uint16_t* stage, int c) {
        if (c < 2) {
            *(uint4v*)(stage + AS + (ld_row + ROWS * c) * LDK + ld_c) = grad_expand<DT>(R.sb[c]);
            *(uint4v*)(stage + (ld_row + ROWS * c) * LDK + ld_c) = R.ag[c];
        } else {
            *(uint4v*)(stage + (ld_row + ROWS * c) * LDK + ld_c) = R.ag[c];
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
    const int a_off = (wm * 64 + frag_row) * LDK + frag_k;
    const int b_off = AS + (wn * 64 + frag_row) * LDK + frag_k;
    auto step = [&](const uint16_t* rd, uint16_t* wr, const GradRegs& Rnext, bool stage_next) {
        uint4v a[2][2], b[2][2];
#pragma unroll
        for (int f = 0; f < 2; ++f) a[0][f] = *(const uint4v*)(rd + a_off + f * 32 * LDK);
#pragma unroll
        for (int h = 0; h < 2; ++h) b[0][h] = *(const uint4v*)(rd + b_off + h * 32 * LDK);
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            const int cur = ks & 1, nxt = cur ^ 1;
#pragma unroll
            for (int f = 0; f < 2; ++f)
#pragma unroll
                for (int h = 0; h < 2; ++h) acc[f][h] = grad_mfma<DT>(a[cur][f], b[cur][h], acc[f][h]);
            if (ks + 1 < BK / 16) {
#pragma unroll
                for (int f = 0; f < 2; ++f) a[nxt][f] = *(const uint4v*)(rd + a_off + f * 32 * LDK + (ks + 1) * 16);
#pragma unroll
                for (int h = 0; h < 2; ++h) b[nxt][h] = *(const uint4v*)(rd + b_off + h * 32 * LDK + (ks + 1) * 16);
            }
            if (stage_next) stage_part(Rnext, wr, ks);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    const int full_steps = Kc / BK;
    const int n_steps = full_steps + ((Kc % BK) != 0 ? 1 : 0);
    auto load_any = [&](GradRegs& R, int s) {
        if (s < full_steps) load_global(R, s * BK, std::false_type{});
        else load_global(R, s * BK, std::true_type{});
    };
    uint16_t* st0 = lds;
    uint16_t* st1 = lds + STAGE;
    GradRegs R0, R1;
    load_any(R0, 0);
    if (n_steps > 1) load_any(R1, 1);
#pragma unroll
    for (int c = 0; c < 4; ++c) stage_part(R0, st0, c);
    __syncthreads();

    int s = 0;
    // steady state, two steps per iteration (stages and register sets static); the loads are
    // unconditional and unguarded, so that their waits stay as deep as the pipeline
    for (; s + 3 < full_steps; s += 2) {
        load_global(R0, (s + 2) * BK, std::false_type{});
        __builtin_amdgcn_sched_barrier(0);
        step(st0, st1, R1, true);
        __syncthreads();
        load_global(R1, (s + 3) * BK, std::false_type{});
        __builtin_amdgcn_sched_barrier(0);
        step(st1, st0, R0, true);
        __syncthreads();
    }
    // the last (up to three, possibly one partial) steps
    for (; s < n_steps; ++s) {
        const bool even = (s & 1) == 0;
        if (s + 2 < n_steps) {
            if (even) load_any(R0, s + 2); else load_any(R1, s + 2);
        }
        const bool more = s + 1 < n_steps;
        if (even) step(st0, st1, R1, more); else step(st1, st0, R0, more);
        __syncthreads();
    }

    // epilogue as in grad_tile_kernel (every step ended with a barrier: the stages are free)
    float* red = (float*)lds;                          // [4 wm][128]
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int n = n0 + wn * 64 + h * 32 + (lane & 31);
        const int nc = min(n, Nc - 1);
        float sum = 0.f;
#pragma unroll
        for (int f = 0; f < 2; ++f)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int tok = m0 + wm * 64 + f * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
                const uint32_t gbits = G[(int64_t)min(tok, M - 1) * Nc + nc];
                const float gval = tok < M ? bits_to_f32<DT>(gbits) : 0.f;
                sum += gval * acc[f][h][r];
            }
        sum += __shfl_xor(sum, 32, kWave);
        if (lane < 32) red[wm * BN + wn * 64 + h * 32 + lane] = sum;
    }
    __syncthreads();
    if (tid < BN) {
        const int n = n0 + tid;
        if (n < Nc) partial[(int64_t)tile_m * Nc + n] = (red[tid] + red[BN + tid]) + (red[2 * BN + tid] + red[3 * BN + tid]);
    }
}

template <int DT>
static int launch_grad_tile_pipe(const uint16_t* A, const uint16_t* G, const uint32_t* bits, float* partial,
                                 int M, int Nc, int Kc, int m_tiles, unsigned grid, hipStream_t stream)
{
    constexpr size_t lds = (size_t)2 * (kGradBM + kGradBN) * kGradLDK * sizeof(uint16_t);   // 110,592 bytes
    auto kernel = grad_tile_pipe_kernel<DT>;
    static unsigned lds_opted_in = 0;                 // per template instance: one kernel
    if (opt_in_dynamic_lds((const void*)kernel, (int)lds, &lds_opted_in) != 0) return -1;
    hipLaunchKernelGGL(kernel, dim3(grid), dim3(512), lds, stream, A, G, bits, partial, M, Nc, Kc, m_tiles);
    return 0;
}

__global__ void __launch_bounds__(256)
grad_reduce_kernel(const float* __restrict__ partial, float* __restrict__ grad, int n, int m_tiles)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    float s = 0.f;
    for (int t = 0; t < m_tiles; ++t) s += partial[(int64_t)t * n + i];
    grad[i] = s;
}

// Bt[i][o / 32] bit (o % 32) = B[o][i / 32] bit (i % 32); d_out % 32 == 0.  A wave takes 64 rows
// o and one word column: 32 ballots turn the lanes' words into the 64-bit columns.
__global__ void __launch_bounds__(256)
transpose_bits_kernel(const uint32_t* __restrict__ B, uint32_t* __restrict__ Bt, int d_out, int d_in)
{
    const int lane = threadIdx.x & 63;
    const int wcol = blockIdx.x * 4 + (threadIdx.x >> 6);            // word column of B
    const int wpr = d_in >> 5;
    if (wcol >= wpr) return;                                        // whole wave
    const int o = blockIdx.y * 64 + lane;
    const uint32_t word = o < d_out ? B[(int64_t)o * wpr + wcol] : 0u;
    unsigned long long mine = 0;
#pragma unroll
    for (int b = 0; b < 32; ++b) {
        const unsigned long long m = __ballot((word >> b) & 1u);
        if (lane == b) mine = m;
    }
    if (lane < 32) {
        const int i = wcol * 32 + lane;
        const int wpr_t = d_out >> 5;
        const int w0 = blockIdx.y * 2;
        Bt[(int64_t)i * wpr_t + w0] = (uint32_t)mine;
        if (w0 + 1 < wpr_t) Bt[(int64_t)i * wpr_t + w0 + 1] = (uint32_t)(mine >> 32);
    }
}

size_t grad_v_workspace_bytes(int64_t M, int64_t d_out, int64_t d_in, int axis)
{
    const int64_t m_tiles = (M + kGradBM - 1) / kGradBM;
    const int64_t n = axis == 0 ? d_out : d_in;
    size_t bytes = (size_t)(m_tiles > 0 ? m_tiles : 1) * n * sizeof(float);
    bytes = (bytes + 255) & ~(size_t)255;
    if (axis == 1) bytes += (size_t)d_in * (d_out / 8);            // transposed sign bits
    return bytes;
}

int launch_grad_v(int dtype, int axis, const void* X, const void* dY, const uint32_t* B_packed, float* grad,
                  int64_t M, int64_t d_out, int64_t d_in, void* workspace, hipStream_t stream)
{
    const int64_t m_tiles = (M + kGradBM - 1) / kGradBM;
    const int64_t Nc = axis == 0 ? d_out : d_in, Kc = axis == 0 ? d_in : d_out;
    float* partial = (float*)workspace;
    const uint16_t* A = (const uint16_t*)(axis == 0 ? X : dY);
    const uint16_t* G = (const uint16_t*)(axis == 0 ? dY : X);
    const uint32_t* bits = B_packed;
    if (axis == 1 && m_tiles > 0) {
        size_t off = (size_t)m_tiles * Nc * sizeof(float);
        off = (off + 255) & ~(size_t)255;
        uint32_t* Bt = (uint32_t*)((char*)workspace + off);
        const dim3 grid((unsigned)((d_in / 32 + 3) / 4), (unsigned)((d_out + 63) / 64));
        hipLaunchKernelGGL(transpose_bits_kernel, grid, dim3(256), 0, stream, B_packed, Bt, (int)d_out, (int)d_in);
        bits = Bt;
    }
    const int64_t n_tiles = (Nc + kGradBN - 1) / kGradBN;
    const dim3 grid((unsigned)(m_tiles * n_tiles));
    if (m_tiles == 0) {
        // no tokens: the reduction below writes zeros
    } else if (tune_value("grad_pipe", 1) != 0) {
        // the pipelined kernel is the default (grad_pipe=0: the two-workgroups-per-CU kernel)
        const int rc = dtype == kBF16
            ? launch_grad_tile_pipe<kBF16>(A, G, bits, partial, (int)M, (int)Nc, (int)Kc, (int)m_tiles, grid.x, stream)
            : launch_grad_tile_pipe<kF16>(A, G, bits, partial, (int)M, (int)Nc, (int)Kc, (int)m_tiles, grid.x, stream);
        if (rc != 0) return rc;
    } else if (dtype == kBF16)
        hipLaunchKernelGGL(grad_tile_kernel<kBF16>, grid, dim3(512), 0, stream, A, G, bits, partial, (int)M, (int)Nc,
                           (int)Kc, (int)m_tiles);
    else
        hipLaunchKernelGGL(grad_tile_kernel<kF16>, grid, dim3(512), 0, stream, A, G, bits, partial, (int)M, (int)Nc,
                           (int)Kc, (int)m_tiles);
    hipLaunchKernelGGL(grad_reduce_kernel, dim3((unsigned)((Nc + 255) / 256)), dim3(256), 0, stream,
                       (const float*)partial, grad, (int)Nc, (int)m_tiles);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

}  // namespace pdelta
