// Prefill-shaped delta linear layer (many tokens): Y = X * W_hat^T with
// W_hat = W_b + v (.) B (paper Eq. 1) built tile by tile on the way into LDS and never written
// to memory.  One MFMA stream: the tile of W_hat is formed as fp16(W_b +- v) with a packed fp16
// add (one rounding of the exact sum), X is used as fp16, products accumulate in fp32.
// bf16 operands are converted to fp16 while they are staged; this is exact for magnitudes in
// [2^-14, 65504] (bf16 carries 8 significant bits, fp16 11) and is the reason for the stated
// operand range of the prefill path.
//
// Tile: BM tokens x 128 output rows x 64 inputs per step (BM = 256, or 128 for short batches),
// WM x 2 waves (8 waves of 64 x 64 outputs for BM = 256), each wave's outputs as MFMA 32x32x16
// tiles; LDS rows padded to 144 bytes so that 16-byte fragment reads of 16 consecutive rows touch
// all 64 banks once.  Three kernels share the tile:
//   linear_gemm_pipe_kernel   the default above 128 tokens: one workgroup per CU, two LDS stages,
//                             two register sets, one barrier per step (described at the kernel);
//   linear_gemm_kernel        one LDS stage, the loads of step s+1 in flight while step s is
//                             multiplied, two workgroups per CU so that one stages while the
//                             other multiplies: short batches (BM = 128) and the second
//                             implementation behind the gemm_pipe=0 switch;
//   linear_gemm_small_kernel  64 x 64 tiles with a ring of steps in flight, for grids that the
//                             big tile cannot fill.
//
// Workgroup -> tile map.  Hardware deals consecutive workgroups round-robin to the 8 XCDs, each
// with its own L2.  Workgroup w therefore belongs to XCD x = w % 8; its x-local index j = w / 8
// walks all token tiles of one output-row tile before moving to the next, and the output-row
// tiles of XCD x are x, x + 8, x + 16, ...  The tiles resident on one XCD at a time then share
// a few W_b panels and all advance through d_in together, so the live slice of X and W_b stays
// inside that XCD's 4 MB L2.
#include <type_traits>

#include "pdelta_device.h"
#include "pdelta_host.h"

namespace pdelta {

constexpr int kGemmBN = 128, kGemmBK = 64;
constexpr int kGemmLDK = kGemmBK + 8;   // padded LDS row in halves (144 bytes)
constexpr int kXcds = 8;

__device__ __forceinline__ uint32_t bf16pair_to_f16pair(uint32_t d) {
    const float lo = __builtin_bit_cast(float, d << 16);
    const float hi = __builtin_bit_cast(float, d & 0xFFFF0000u);
    return as_u32(__builtin_bit_cast(half2v, __builtin_amdgcn_cvt_pkrtz(lo, hi)));
}

template <int XDT>
__device__ __forceinline__ uint4v to_f16x8(uint4v a) {
    if constexpr (XDT == kBF16) {
        uint4v r;
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            const uint32_t ap = a[p];
            r[p] = bf16pair_to_f16pair(ap);
        }
        return r;
    } else {
        return a;
    }
}

// Eight fp16 weights and eight "negate" bits (bit e set: element e gets -|v|, clear: +|v|) with
// the packed magnitudes |v| of elements 2p (low half) and 2p+1 (high half) in vabs[p].
// Row mode: |v| is one value per row and the sign of v is folded into the bits by the caller.
__device__ __forceinline__ uint4v add_signed_scale(uint4v w, uint32_t negbits, uint4v vabs) {
    uint4v r;
    negbits &= 0xFFu;
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        // bit 2p -> position 15, bit 2p+1 -> position 31; everything else is masked by the insert
        const uint32_t spread = (negbits << (30 - 2 * p)) | (negbits << (15 - 2 * p));
        const uint32_t va = vabs[p], wp = w[p];
        const uint32_t sv = (spread & 0x80008000u) | (va & 0x7FFF7FFFu);        // v_bfi_b32
        r[p] = as_u32(as_half2(wp) + as_half2(sv));                              // v_pk_add_f16
    }
    return r;
}

// Epilogue of the 64 x 64 wave tile for 16-bit outputs: the accumulators go through a wave-private
// LDS region (32 rows x 64 columns at a time, rows padded to 144 bytes) and leave as 16-byte
// stores, eight lanes per 128-byte line of Y, instead of 64 two-byte store instructions per
// accumulator tile (measured 2-3 % of the run time).  `region` holds 32 * kGemmLDK halves of this wave.
// Returns false (nothing stored) when the tile is not fully inside Y or rows of Y are not
// 16-byte aligned; the caller then stores element by element.
template <int FM>
__device__ __forceinline__ bool store_tile_16bit(const float16v (&acc)[FM][2], uint16_t* region, void* Y,
                                                 int y_dtype, int tok0, int o0, int M, int d_out, int lane)
{
    if (y_dtype == kF32 || (d_out & 7) != 0 || o0 + 64 > d_out || tok0 + FM * 32 > M) return false;   // wave-uniform
    uint16_t* Yh = (uint16_t*)Y;
#pragma unroll
    for (int f = 0; f < FM; ++f) {
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3), col = h * 32 + (lane & 31);
                const float val = acc[f][h][r];
                region[row * kGemmLDK + col] =
                    (uint16_t)(y_dtype == kBF16 ? f32_to_bf16_bits(val) : f32_to_f16_bits(val));
            }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            const int row = it * 8 + (lane >> 3), chunk = lane & 7;
            const uint4v vals = *(const uint4v*)(region + row * kGemmLDK + chunk * 8);
            *(uint4v*)(Yh + (int64_t)(tok0 + f * 32 + row) * d_out + o0 + chunk * 8) = vals;
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
    }
    return true;
}

// WM x 2 waves; a wave owns (BM / WM) tokens x 64 output rows.
template <int XDT, int AXIS, int BM, int WM>
__global__ void __launch_bounds__(WM * 128, (WM * 128) / 128)
linear_gemm_kernel(const uint16_t* __restrict__ X, const uint16_t* __restrict__ W_b,
                   const uint32_t* __restrict__ B_packed, const uint16_t* __restrict__ v,
                   void* __restrict__ Y, int M, int d_out, int d_in, int y_dtype, int m_tiles,
                   int n_tiles, int v_stride, int g_shift)
{
    constexpr int THREADS = WM * 128;
    constexpr int ROWS = THREADS / 8;    // tile rows covered by one staging pass
    constexpr int FM = BM / WM / 32;     // 32-row MFMA tiles per wave along tokens
    constexpr int FN = 2;                // ... along output rows (wave covers 64)
    constexpr int XQ = BM / ROWS;        // 16-byte vectors of X per thread and step
    constexpr int WQ = kGemmBN / ROWS;   // ... of W_b
    __shared__ __attribute__((aligned(16))) uint16_t Xs[BM * kGemmLDK];
    __shared__ __attribute__((aligned(16))) uint16_t Ws[kGemmBN * kGemmLDK];

    // tile of this workgroup (see the map in the header comment)
    const int xcd = blockIdx.x % kXcds, local = blockIdx.x / kXcds;
    const int tile_n = (local / m_tiles) * kXcds + xcd;
    const int tile_m = local % m_tiles;
    if (tile_n >= n_tiles) return;       // whole workgroup
    const int n0 = tile_n * kGemmBN, m0 = tile_m * BM;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int K = d_in;
    constexpr int WROWS = BM / WM;       // tokens per wave

    // Staging role: the thread covers 8 inputs (16 bytes) at column ld_c of tile rows
    // ld_row + ROWS q.  Addresses are a workgroup-uniform base that advances with the step plus a
    // fixed 32-bit per-thread byte offset, so the loop spends no vector ALU work on them.  Rows
    // past the end of X or W_b are clamped to the last real row: such rows only feed outputs
    // that are never stored, and every load stays unconditional (a load behind a branch makes
    // the compiler drain all outstanding loads at the join).
    const int ld_row = tid >> 3, ld_c = (tid & 7) * 8;
    const char* xbase = (const char*)(X + (int64_t)m0 * K);
    const char* wbase = (const char*)(W_b + (int64_t)n0 * K);
    const char* sbase = (const char*)B_packed + (((int64_t)n0 * K) >> 3);
    uint32_t xoff[XQ], woff[WQ], soff[WQ];
#pragma unroll
    for (int q = 0; q < XQ; ++q) {
        const int row = min(m0 + ld_row + ROWS * q, M - 1) - m0;
        xoff[q] = ((uint32_t)row * (uint32_t)K + (uint32_t)ld_c) * 2u;
    }
    uint32_t vabs_row[WQ];               // row mode: |v| of the thread's W rows, in both halves
    uint32_t vneg_row[WQ];               // row mode: 0xFF if v < 0 (flips every sign bit)
    const uint16_t* vgrow[WQ];           // grouped mode: the scales of the thread's W rows
#pragma unroll
    for (int q = 0; q < WQ; ++q) {
        const int row = min(n0 + ld_row + ROWS * q, d_out - 1) - n0;
        woff[q] = ((uint32_t)row * (uint32_t)K + (uint32_t)ld_c) * 2u;
        soff[q] = (uint32_t)row * (uint32_t)(K >> 3) + (uint32_t)(tid & 7);
        if constexpr (AXIS == 0) {
            const uint32_t h = v[n0 + row];
            const uint32_t a = h & 0x7FFFu, aa = a | (a << 16);
            vabs_row[q] = aa;
            vneg_row[q] = (h & 0x8000u) ? 0xFFu : 0u;
        }
        if constexpr (AXIS == 2) vgrow[q] = v + (int64_t)(n0 + row) * v_stride;
    }

    uint4v xg[XQ], wg[WQ], vcg;
    uint32_t sb[WQ], vgq[WQ];            // vgq: grouped mode, the step's scale per W row
    const uint4v zero = {0, 0, 0, 0};

    // GUARD: the last, partial step of a d_in that is not a multiple of 64 (it is one of 32).
    auto load_global = [&](int kb, auto guard) {
        constexpr bool GUARD = decltype(guard)::value;
        const bool col_ok = !GUARD || kb + ld_c < K;
        const char* xb = xbase + (int64_t)kb * 2;
        const char* wb = wbase + (int64_t)kb * 2;
        const char* sp = sbase + (kb >> 3);
#pragma unroll
        for (int q = 0; q < XQ; ++q) xg[q] = col_ok ? *(const uint4v*)(xb + xoff[q]) : zero;
#pragma unroll
        for (int q = 0; q < WQ; ++q) {
            wg[q] = col_ok ? *(const uint4v*)(wb + woff[q]) : zero;
            sb[q] = col_ok ? (uint32_t) * (const uint8_t*)(sp + soff[q]) : 0xFFu;
            if constexpr (AXIS == 2) vgq[q] = col_ok ? (uint32_t)vgrow[q][(kb + ld_c) >> g_shift] : 0u;
        }
        if constexpr (AXIS == 1) vcg = col_ok ? *(const uint4v*)(v + kb + ld_c) : zero;
    };

    auto store_lds = [&]() {
#pragma unroll
        for (int q = 0; q < XQ; ++q)
            *(uint4v*)(Xs + (ld_row + ROWS * q) * kGemmLDK + ld_c) = to_f16x8<XDT>(xg[q]);
#pragma unroll
        for (int q = 0; q < WQ; ++q) {
            const uint4v w16 = to_f16x8<XDT>(wg[q]);
            uint4v what;
            if constexpr (AXIS == 0) {
                const uint32_t aa = vabs_row[q];
                what = add_signed_scale(w16, ~sb[q] ^ vneg_row[q], (uint4v){aa, aa, aa, aa});
            } else if constexpr (AXIS == 2) {
                const uint32_t h = vgq[q], a = h & 0x7FFFu, aa = a | (a << 16);
                what = add_signed_scale(w16, ~sb[q] ^ ((h & 0x8000u) ? 0xFFu : 0u), (uint4v){aa, aa, aa, aa});
            } else {
                // per-input scales: fold each scale's own sign into its negate bit
                uint32_t vsign = 0;
#pragma unroll
                for (int p = 0; p < 4; ++p) {
                    const uint32_t vp = vcg[p];
                    vsign |= ((vp >> 15) & 1u) << (2 * p) | ((vp >> 31) & 1u) << (2 * p + 1);
                }
                what = add_signed_scale(w16, ~sb[q] ^ vsign, vcg);
            }
            *(uint4v*)(Ws + (ld_row + ROWS * q) * kGemmLDK + ld_c) = what;
        }
    };

    float16v acc[FM][FN];
#pragma unroll
    for (int f = 0; f < FM; ++f)
#pragma unroll
        for (int h = 0; h < FN; ++h)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[f][h][r] = 0.f;

    const int frag_row = lane & 31, frag_k = (lane >> 5) * 8;
    const uint16_t* a_base = Xs + (wm * WROWS + frag_row) * kGemmLDK + frag_k;
    const uint16_t* b_base = Ws + (wn * 64 + frag_row) * kGemmLDK + frag_k;

    auto multiply_stage = [&]() {
#pragma unroll
        for (int ks = 0; ks < kGemmBK / 16; ++ks) {
            half8 a[FM], b[FN];
#pragma unroll
            for (int f = 0; f < FM; ++f) a[f] = *(const half8*)(a_base + f * 32 * kGemmLDK + ks * 16);
#pragma unroll
            for (int h = 0; h < FN; ++h) b[h] = *(const half8*)(b_base + h * 32 * kGemmLDK + ks * 16);
#pragma unroll
            for (int f = 0; f < FM; ++f)
#pragma unroll
                for (int h = 0; h < FN; ++h)
                    acc[f][h] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[f], b[h], acc[f][h], 0, 0, 0);
        }
    };

    const int full_steps = K / kGemmBK;              // unguarded steps
    const bool tail = (K % kGemmBK) != 0;            // then one more step of 32 inputs
    if (full_steps > 0) load_global(0, std::false_type{});
    else load_global(0, std::true_type{});
    for (int i = 0; i + 1 < full_steps; ++i) {       // steady state: always another full step
        store_lds();
        __syncthreads();
        load_global((i + 1) * kGemmBK, std::false_type{});
        // Keep the loads above the multiplication.  Left alone, the compiler sinks them below it
        // (shorter live ranges), which issues them just before they are needed: no overlap of
        // memory latency with the MFMA phase, measured 10-20 % slower.
        __builtin_amdgcn_sched_barrier(0);
        multiply_stage();
        __syncthreads();
    }
    if (full_steps > 0) {                            // last full step
        store_lds();
        __syncthreads();
        if (tail) load_global(full_steps * kGemmBK, std::true_type{});
        multiply_stage();
        __syncthreads();
    }
    if (tail) {
        store_lds();
        __syncthreads();
        multiply_stage();
        __syncthreads();
    }

    // 32x32 accumulator: element r of lane l is row (r/4)*8 + (l/32)*4 + r%4, column l%32.
    // (the loop ended with a barrier: the operand tiles in LDS are free)
    if (store_tile_16bit<FM>(acc, Xs + wave * 32 * kGemmLDK, Y, y_dtype, m0 + wm * WROWS, n0 + wn * 64, M, d_out, lane))
        return;
#pragma unroll
    for (int f = 0; f < FM; ++f)
#pragma unroll
        for (int h = 0; h < FN; ++h) {
            const int o = n0 + wn * 64 + h * 32 + (lane & 31);
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int tok = m0 + wm * WROWS + f * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
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

// ---------------------------------------------------------------------------------------------
// Pipelined variant of the 256 x 128 x 64 tile: one workgroup per CU (8 waves, up to 256
// registers each), two LDS stages and two register sets.  During step s a wave multiplies stage
// s % 2 and, between its groups of four MFMAs, converts one quarter of the operands of step s+1
// into the other stage and at once requests the same quarter of step s+3 into the registers
// just freed: one barrier per step, every load has two whole steps to arrive, and the matrix
// cores keep running while the vector ALU converts (MFMAs execute asynchronously to the wave's
// next instructions).  The scheduling fences pin that interleaving.
struct GemmRegs {                         // one step of one thread: 4 x 16 B of X, 2 x 16 B of W_b, ...
    uint4v xg[4], wg[2], vcg;
    uint32_t sb[2], vg[2];                // sign bytes; blockwise mode: the step's scale per W row
};

// PARTS (measurement builds only; 15 = the product kernel): bit 0 the global loads of the steady
// loop, bit 1 conversion and LDS writes, bit 2 fragment reads, bit 3 the MFMAs.  A part that is
// switched off is compiled out with its inputs kept alive (loads are still waited for where the
// conversion would use them, fragments where the MFMAs would), every access stays in bounds and
// Y is still written (with meaningless values unless PARTS == 15).
template <int XDT, int AXIS, int PARTS = 15>
__global__ void __launch_bounds__(512, 2)
linear_gemm_pipe_kernel(const uint16_t* __restrict__ X, const uint16_t* __restrict__ W_b,
                        const uint32_t* __restrict__ B_packed, const uint16_t* __restrict__ v,
                        void* __restrict__ Y, int M, int d_out, int d_in, int y_dtype, int m_tiles,
                        int n_tiles, int v_stride, int g_shift)
{
    constexpr int BM = 256, WM = 4, ROWS = 64, XQ = 4, WQ = 2, FM = 2, FN = 2;
    constexpr int XS = BM * kGemmLDK, WS = kGemmBN * kGemmLDK, STAGE = XS + WS;   // halves
    constexpr bool P_LOAD = (PARTS & 1) != 0, P_CONV = (PARTS & 2) != 0, P_FRAG = (PARTS & 4) != 0,
                   P_MFMA = (PARTS & 8) != 0;
    extern __shared__ __attribute__((aligned(16))) unsigned char gemm_smem[];
    uint16_t* lds = (uint16_t*)gemm_smem;                 // [2][STAGE]: X tile then W_hat tile

    const int xcd = blockIdx.x % kXcds, local = blockIdx.x / kXcds;
    const int tile_n = (local / m_tiles) * kXcds + xcd;
    const int tile_m = local % m_tiles;
    if (tile_n >= n_tiles) return;       // whole workgroup
    const int n0 = tile_n * kGemmBN, m0 = tile_m * BM;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int K = d_in;
    constexpr int WROWS = BM / WM;

    // staging role and addresses: as in linear_gemm_kernel
    const int ld_row = tid >> 3, ld_c = (tid & 7) * 8;
    const char* xbase = (const char*)(X + (int64_t)m0 * K);
    const char* wbase = (const char*)(W_b + (int64_t)n0 * K);
    const char* sbase = (const char*)B_packed + (((int64_t)n0 * K) >> 3);
    uint32_t xoff[XQ], woff[WQ], soff[WQ];
#pragma unroll
    for (int q = 0; q < XQ; ++q) {
        const int row = min(m0 + ld_row + ROWS * q, M - 1) - m0;
        xoff[q] = ((uint32_t)row * (uint32_t)K + (uint32_t)ld_c) * 2u;
    }
    uint32_t vabs_row[WQ], vneg_row[WQ];
    const uint16_t* vgrow[WQ];           // blockwise mode: the scales of the thread's W rows
#pragma unroll
    for (int q = 0; q < WQ; ++q) {
        const int row = min(n0 + ld_row + ROWS * q, d_out - 1) - n0;
        woff[q] = ((uint32_t)row * (uint32_t)K + (uint32_t)ld_c) * 2u;
        soff[q] = (uint32_t)row * (uint32_t)(K >> 3) + (uint32_t)(tid & 7);
        if constexpr (AXIS == 0) {
            const uint32_t h = v[n0 + row];
            const uint32_t a = h & 0x7FFFu, aa = a | (a << 16);
            vabs_row[q] = aa;
            vneg_row[q] = (h & 0x8000u) ? 0xFFu : 0u;
        }
        if constexpr (AXIS == 2) vgrow[q] = v + (int64_t)(n0 + row) * v_stride;
    }
    const uint4v zero = {0, 0, 0, 0};

    auto load_global = [&](GemmRegs& G, int kb, auto guard) {
        constexpr bool GUARD = decltype(guard)::value;
        const bool col_ok = !GUARD || kb + ld_c < K;
        const char* xb = xbase + (int64_t)kb * 2;
        const char* wb = wbase + (int64_t)kb * 2;
        const char* sp = sbase + (kb >> 3);
#pragma unroll
        for (int q = 0; q < XQ; ++q) G.xg[q] = col_ok ? *(const uint4v*)(xb + xoff[q]) : zero;
#pragma unroll
        for (int q = 0; q < WQ; ++q) {
            G.wg[q] = col_ok ? *(const uint4v*)(wb + woff[q]) : zero;
            G.sb[q] = col_ok ? (uint32_t) * (const uint8_t*)(sp + soff[q]) : 0xFFu;
            if constexpr (AXIS == 2) G.vg[q] = col_ok ? (uint32_t)vgrow[q][(kb + ld_c) >> g_shift] : 0u;
        }
        if constexpr (AXIS == 1) G.vcg = col_ok ? *(const uint4v*)(v + kb + ld_c) : zero;
    };
    // quarter c of an unguarded step's loads (the quarters of convert_part below)
    auto load_part = [&](GemmRegs& G, int kb, int c) {
        if (c < 2) {
            G.wg[c] = *(const uint4v*)(wbase + (int64_t)kb * 2 + woff[c]);
            G.sb[c] = (uint32_t) * (const uint8_t*)(sbase + (kb >> 3) + soff[c]);
            if constexpr (AXIS == 2) G.vg[c] = (uint32_t)vgrow[c][(kb + ld_c) >> g_shift];
            if constexpr (AXIS == 1) { if (c == 1) G.vcg = *(const uint4v*)(v + kb + ld_c); }
        } else {
            const char* xb = xbase + (int64_t)kb * 2;
            G.xg[2 * c - 4] = *(const uint4v*)(xb + xoff[2 * c - 4]);
            G.xg[2 * c - 3] = *(const uint4v*)(xb + xoff[2 * c - 3]);
        }
    };
    auto store_x = [&](const GemmRegs& G, uint16_t* stage, int q) {
        *(uint4v*)(stage + (ld_row + ROWS * q) * kGemmLDK + ld_c) = to_f16x8<XDT>(G.xg[q]);
    };
    auto store_w = [&](const GemmRegs& G, uint16_t* stage, int q) {
        const uint4v w16 = to_f16x8<XDT>(G.wg[q]);
        uint4v what;
        if constexpr (AXIS == 0) {
            const uint32_t aa = vabs_row[q];
            what = add_signed_scale(w16, ~G.sb[q] ^ vneg_row[q], (uint4v){aa, aa, aa, aa});
        } else if constexpr (AXIS == 2) {
            const uint32_t h = G.vg[q], a = h & 0x7FFFu, aa = a | (a << 16);
            what = add_signed_scale(w16, ~G.sb[q] ^ ((h & 0x8000u) ? 0xFFu : 0u), (uint4v){aa, aa, aa, aa});
        } else {
            uint32_t vsign = 0;
#pragma unroll
            for (int p = 0; p < 4; ++p) {
                const uint32_t vp = G.vcg[p];
                vsign |= ((vp >> 15) & 1u) << (2 * p) | ((vp >> 31) & 1u) << (2 * p + 1);
            }
            what = add_signed_scale(w16, ~G.sb[q] ^ vsign, G.vcg);
        }
        *(uint4v*)(stage + XS + (ld_row + ROWS * q) * kGemmLDK + ld_c) = what;
    };
    // (measurement builds) the loaded registers of quarter c are consumed without being converted;
    // a register set is made opaque so that its conversion cannot be hoisted out of the loop
    auto touch4 = [&](const uint4v& r) { asm volatile("" :: "v"(r[0]), "v"(r[1]), "v"(r[2]), "v"(r[3])); };
    auto keep_part = [&](const GemmRegs& G, int c) {
        if (c < 2) { touch4(G.wg[c]); asm volatile("" :: "v"(G.sb[c])); }
        else { touch4(G.xg[2 * c - 4]); touch4(G.xg[2 * c - 3]); }
    };
    auto opaque = [&](GemmRegs& G) {
#pragma unroll
        for (int q = 0; q < XQ; ++q) asm volatile("" : "+v"(G.xg[q][0]), "+v"(G.xg[q][1]), "+v"(G.xg[q][2]), "+v"(G.xg[q][3]));
#pragma unroll
        for (int q = 0; q < WQ; ++q) asm volatile("" : "+v"(G.wg[q][0]), "+v"(G.wg[q][1]), "+v"(G.wg[q][2]), "+v"(G.wg[q][3]), "+v"(G.sb[q]));
    };
    // quarter c of the conversion work of one step
    auto convert_part = [&](const GemmRegs& G, uint16_t* stage, int c) {
        if constexpr (!P_CONV) { keep_part(G, c); return; }
        if (c == 0) store_w(G, stage, 0);
        else if (c == 1) store_w(G, stage, 1);
        else if (c == 2) { store_x(G, stage, 0); store_x(G, stage, 1); }
        else { store_x(G, stage, 2); store_x(G, stage, 3); }
    };

    float16v acc[FM][FN];
#pragma unroll
    for (int f = 0; f < FM; ++f)
#pragma unroll
        for (int h = 0; h < FN; ++h)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[f][h][r] = 0.f;

    const int frag_row = lane & 31, frag_k = (lane >> 5) * 8;
    const int a_off = (wm * WROWS + frag_row) * kGemmLDK + frag_k;
    const int b_off = XS + (wn * 64 + frag_row) * kGemmLDK + frag_k;

    // One step.  convert: the operands of the next step are in Gnext and go to `wr`; refill_kb >= 0:
    // each quarter of Gnext is loaded again, with the inputs from refill_kb on (two steps later
    // than what it held), as soon as it has been converted.
    half8 afix[FM], bfix[FN];             // (measurement builds without fragment reads)
    auto step = [&](const uint16_t* rd, uint16_t* wr, GemmRegs& Gnext, bool convert, int refill_kb) {
        half8 a[2][FM], b[2][FN];
        if constexpr (P_FRAG) {
#pragma unroll
            for (int f = 0; f < FM; ++f) a[0][f] = *(const half8*)(rd + a_off + f * 32 * kGemmLDK);
#pragma unroll
            for (int h = 0; h < FN; ++h) b[0][h] = *(const half8*)(rd + b_off + h * 32 * kGemmLDK);
        } else {
#pragma unroll
            for (int f = 0; f < FM; ++f) a[0][f] = a[1][f] = afix[f];
#pragma unroll
            for (int h = 0; h < FN; ++h) b[0][h] = b[1][h] = bfix[h];
        }
#pragma unroll
        for (int ks = 0; ks < kGemmBK / 16; ++ks) {
            const int cur = ks & 1, nxt = cur ^ 1;
            if constexpr (P_MFMA) {
#pragma unroll
                for (int f = 0; f < FM; ++f)
#pragma unroll
                    for (int h = 0; h < FN; ++h)
                        acc[f][h] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[cur][f], b[cur][h], acc[f][h], 0, 0, 0);
            } else {
#pragma unroll
                for (int f = 0; f < FM; ++f) touch4(__builtin_bit_cast(uint4v, a[cur][f]));
#pragma unroll
                for (int h = 0; h < FN; ++h) touch4(__builtin_bit_cast(uint4v, b[cur][h]));
            }
            if constexpr (P_FRAG) {
                if (ks + 1 < kGemmBK / 16) {
#pragma unroll
                    for (int f = 0; f < FM; ++f)
                        a[nxt][f] = *(const half8*)(rd + a_off + f * 32 * kGemmLDK + (ks + 1) * 16);
#pragma unroll
                    for (int h = 0; h < FN; ++h)
                        b[nxt][h] = *(const half8*)(rd + b_off + h * 32 * kGemmLDK + (ks + 1) * 16);
                }
            }
            if (convert) convert_part(Gnext, wr, ks);
            if constexpr (P_LOAD) { if (refill_kb >= 0) load_part(Gnext, refill_kb, ks); }
            __builtin_amdgcn_sched_barrier(0);
        }
        if constexpr (!P_LOAD) opaque(Gnext);
    };

    const int full_steps = K / kGemmBK;
    const int n_steps = full_steps + ((K % kGemmBK) != 0 ? 1 : 0);
    auto load_any = [&](GemmRegs& G, int s) {
        if (s < full_steps) load_global(G, s * kGemmBK, std::false_type{});
        else load_global(G, s * kGemmBK, std::true_type{});
    };
    uint16_t* st0 = lds;
    uint16_t* st1 = lds + STAGE;
    GemmRegs G0, G1;
    load_any(G0, 0);
    if (n_steps > 1) load_any(G1, 1);
#pragma unroll
    for (int c = 0; c < 4; ++c) convert_part(G0, st0, c);
    if (n_steps > 2) load_any(G0, 2);
    __syncthreads();
    if constexpr (!P_FRAG) {
#pragma unroll
        for (int f = 0; f < FM; ++f) afix[f] = *(const half8*)(st0 + a_off + f * 32 * kGemmLDK);
#pragma unroll
        for (int h = 0; h < FN; ++h) bfix[h] = *(const half8*)(st0 + b_off + h * 32 * kGemmLDK);
    }

    // On entry to step s the set of parity (s + 1) holds step s+1 and the other one step s+2 (in
    // flight).  Steady state, two steps per iteration so that stages and register sets are static;
    // every load is unconditional and unguarded, and a quarter of a register set is requested
    // again (for two steps later) right after it has been converted: two steps of lead time with
    // two register sets.
    int s = 0;
    for (; s + 4 < full_steps; s += 2) {
        step(st0, st1, G1, true, (s + 3) * kGemmBK);
        __syncthreads();
        step(st1, st0, G0, true, (s + 4) * kGemmBK);
        __syncthreads();
    }
    // the last (up to four, possibly one partial) steps: whole-set loads after the step
    for (; s < n_steps; ++s) {
        const bool even = (s & 1) == 0;
        const bool conv = s + 1 < n_steps;
        if (even) step(st0, st1, G1, conv, -1); else step(st1, st0, G0, conv, -1);
        if (s + 3 < n_steps) {
            if constexpr (P_LOAD) { if (even) load_any(G1, s + 3); else load_any(G0, s + 3); }
        }
        __syncthreads();
    }

    // (every step ended with a barrier: both LDS stages are free)
    if (store_tile_16bit<FM>(acc, lds + wave * 32 * kGemmLDK, Y, y_dtype, m0 + wm * WROWS, n0 + wn * 64, M, d_out, lane))
        return;
#pragma unroll
    for (int f = 0; f < FM; ++f)
#pragma unroll
        for (int h = 0; h < FN; ++h) {
            const int o = n0 + wn * 64 + h * 32 + (lane & 31);
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int tok = m0 + wm * WROWS + f * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
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

template <int XDT, int AXIS, int PARTS = 15>
static int launch_gemm_pipe(const void* X, const void* W_b, const uint32_t* B_packed, const uint16_t* v,
                            void* Y, int64_t M, int64_t d_out, int64_t d_in, int y_dtype,
                            hipStream_t stream, int v_stride = 0, int g_shift = 31)
{
    constexpr int BM = 256;
    constexpr size_t lds = (size_t)2 * (BM + kGemmBN) * kGemmLDK * sizeof(uint16_t);   // 110,592 bytes
    const int m_tiles = (int)((M + BM - 1) / BM);
    const int n_tiles = (int)((d_out + kGemmBN - 1) / kGemmBN);
    const int n_groups = (n_tiles + kXcds - 1) / kXcds;
    const dim3 grid((unsigned)((int64_t)n_groups * kXcds * m_tiles));
    auto kernel = linear_gemm_pipe_kernel<XDT, AXIS, PARTS>;
    static unsigned lds_opted_in = 0;                 // per template instance: one kernel
    if (opt_in_dynamic_lds((const void*)kernel, (int)lds, &lds_opted_in) != 0) return -1;
    hipLaunchKernelGGL(kernel, grid, dim3(512), lds, stream, (const uint16_t*)X, (const uint16_t*)W_b,
                       B_packed, v, Y, (int)M, (int)d_out, (int)d_in, y_dtype, m_tiles, n_tiles, v_stride, g_shift);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

// ---------------------------------------------------------------------------------------------
// Small-tile variant for grids that the 256 x 128 tile cannot fill (a few hundred tokens): a
// workgroup of 4 waves owns 64 tokens x 64 outputs, so even 256 tokens x 4096 outputs give one
// workgroup per CU.  With so few tiles the run time of the big-tile kernels is the d_in / 64
// sequential steps times the latency of one step (load, convert, barrier: over a microsecond),
// whatever the batch.  Here a step's operands are 16 bytes of X and of W_b per thread, which
// leaves registers for a ring of DEPTH steps in flight: the loads of step s + DEPTH are issued
// while step s is multiplied, and a step costs its LDS traffic and barrier only.
// Requires d_in % 64 == 0.
struct SmallRegs {
    uint4v xg[2], wg[2], vcg;
    uint32_t sb[2], vg[2];               // vg: grouped mode, the step's scale per W row
};

template <int XDT, int AXIS, int DEPTH>
__global__ void __launch_bounds__(256, 2)
linear_gemm_small_kernel(const uint16_t* __restrict__ X, const uint16_t* __restrict__ W_b,
                         const uint32_t* __restrict__ B_packed, const uint16_t* __restrict__ v,
                         void* __restrict__ Y, int M, int d_out, int d_in, int y_dtype, int m_tiles,
                         int n_tiles, int v_stride, int g_shift)
{
    constexpr int BM = 64, BN = 64, ROWS = 32, Q = 2;
    constexpr int XS = BM * kGemmLDK, STAGE = (BM + BN) * kGemmLDK;               // halves
    __shared__ __attribute__((aligned(16))) uint16_t lds[2 * STAGE];              // 36,864 bytes

    const int xcd = blockIdx.x % kXcds, local = blockIdx.x / kXcds;
    const int tile_n = (local / m_tiles) * kXcds + xcd;
    const int tile_m = local % m_tiles;
    if (tile_n >= n_tiles) return;       // whole workgroup
    const int n0 = tile_n * BN, m0 = tile_m * BM;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int K = d_in;

    const int ld_row = tid >> 3, ld_c = (tid & 7) * 8;
    const char* xbase = (const char*)(X + (int64_t)m0 * K);
    const char* wbase = (const char*)(W_b + (int64_t)n0 * K);
    const char* sbase = (const char*)B_packed + (((int64_t)n0 * K) >> 3);
    uint32_t xoff[Q], woff[Q], soff[Q], vabs_row[Q], vneg_row[Q];
    const uint16_t* vgrow[Q];
#pragma unroll
    for (int q = 0; q < Q; ++q) {
        const int xr = min(m0 + ld_row + ROWS * q, M - 1) - m0;
        xoff[q] = ((uint32_t)xr * (uint32_t)K + (uint32_t)ld_c) * 2u;
        const int wr = min(n0 + ld_row + ROWS * q, d_out - 1) - n0;
        woff[q] = ((uint32_t)wr * (uint32_t)K + (uint32_t)ld_c) * 2u;
        soff[q] = (uint32_t)wr * (uint32_t)(K >> 3) + (uint32_t)(tid & 7);
        if constexpr (AXIS == 0) {
            const uint32_t h = v[n0 + wr];
            const uint32_t a = h & 0x7FFFu;
            vabs_row[q] = a | (a << 16);
            vneg_row[q] = (h & 0x8000u) ? 0xFFu : 0u;
        }
        if constexpr (AXIS == 2) vgrow[q] = v + (int64_t)(n0 + wr) * v_stride;
    }

    auto load_global = [&](SmallRegs& G, int step) {
        const int kb = step * kGemmBK;
        const char* xb = xbase + (int64_t)kb * 2;
        const char* wb = wbase + (int64_t)kb * 2;
        const char* sp = sbase + (kb >> 3);
#pragma unroll
        for (int q = 0; q < Q; ++q) {
            G.xg[q] = *(const uint4v*)(xb + xoff[q]);
            G.wg[q] = *(const uint4v*)(wb + woff[q]);
            G.sb[q] = (uint32_t) * (const uint8_t*)(sp + soff[q]);
            if constexpr (AXIS == 2) G.vg[q] = (uint32_t)vgrow[q][(kb + ld_c) >> g_shift];
        }
        if constexpr (AXIS == 1) G.vcg = *(const uint4v*)(v + kb + ld_c);
    };
    auto convert = [&](const SmallRegs& G, uint16_t* stage) {
#pragma unroll
        for (int q = 0; q < Q; ++q) {
            *(uint4v*)(stage + (ld_row + ROWS * q) * kGemmLDK + ld_c) = to_f16x8<XDT>(G.xg[q]);
            const uint4v w16 = to_f16x8<XDT>(G.wg[q]);
            uint4v what;
            if constexpr (AXIS == 0) {
                const uint32_t aa = vabs_row[q];
                what = add_signed_scale(w16, ~G.sb[q] ^ vneg_row[q], (uint4v){aa, aa, aa, aa});
            } else if constexpr (AXIS == 2) {
                const uint32_t h = G.vg[q], a = h & 0x7FFFu, aa = a | (a << 16);
                what = add_signed_scale(w16, ~G.sb[q] ^ ((h & 0x8000u) ? 0xFFu : 0u), (uint4v){aa, aa, aa, aa});
            } else {
                uint32_t vsign = 0;
#pragma unroll
                for (int p = 0; p < 4; ++p) {
                    const uint32_t vp = G.vcg[p];
                    vsign |= ((vp >> 15) & 1u) << (2 * p) | ((vp >> 31) & 1u) << (2 * p + 1);
                }
                what = add_signed_scale(w16, ~G.sb[q] ^ vsign, G.vcg);
            }
            *(uint4v*)(stage + XS + (ld_row + ROWS * q) * kGemmLDK + ld_c) = what;
        }
    };

    float16v acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;
    const int frag_row = lane & 31, frag_k = (lane >> 5) * 8;
    const int a_off = (wm * 32 + frag_row) * kGemmLDK + frag_k;
    const int b_off = XS + (wn * 32 + frag_row) * kGemmLDK + frag_k;
    auto multiply = [&](const uint16_t* rd) {
        half8 a[4], b[4];
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            a[ks] = *(const half8*)(rd + a_off + ks * 16);
            b[ks] = *(const half8*)(rd + b_off + ks * 16);
        }
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[ks], b[ks], acc, 0, 0, 0);
    };

    const int n_steps = K / kGemmBK;
    SmallRegs G[DEPTH];
#pragma unroll
    for (int d = 0; d < DEPTH; ++d) load_global(G[d], min(d, n_steps - 1));
    convert(G[0], lds);
    __syncthreads();
    // Every iteration refills the slot it has just consumed with step s + DEPTH (clamped to the
    // last step near the end: a redundant load of valid memory keeps every load unconditional).
    for (int s0 = 0; s0 < n_steps; s0 += DEPTH) {
#pragma unroll
        for (int d = 0; d < DEPTH; ++d) {
            const int s = s0 + d;
            load_global(G[d], min(s + DEPTH, n_steps - 1));
            __builtin_amdgcn_sched_barrier(0);
            if (s < n_steps) {                                        // workgroup-uniform
                uint16_t* rd = lds + (s & 1) * STAGE;
                uint16_t* wr = lds + ((s + 1) & 1) * STAGE;
                multiply(rd);
                if (s + 1 < n_steps) convert(G[(d + 1) % DEPTH], wr);
            }
            __syncthreads();
        }
    }

    const int o = n0 + wn * 32 + (lane & 31);
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int tok = m0 + wm * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
        if (tok < M && o < d_out) {
            const int64_t yi = (int64_t)tok * d_out + o;
            if (y_dtype == kF32) store_y<kF32>(Y, yi, acc[r]);
            else if (y_dtype == kBF16) store_y<kBF16>(Y, yi, acc[r]);
            else store_y<kF16>(Y, yi, acc[r]);
        }
    }
}

template <int XDT, int AXIS>
static int launch_gemm_small(const void* X, const void* W_b, const uint32_t* B_packed, const uint16_t* v,
                             void* Y, int64_t M, int64_t d_out, int64_t d_in, int y_dtype,
                             hipStream_t stream, int v_stride = 0, int g_shift = 31)
{
    const int m_tiles = (int)((M + 63) / 64), n_tiles = (int)((d_out + 63) / 64);
    const int n_groups = (n_tiles + kXcds - 1) / kXcds;
    const dim3 grid((unsigned)((int64_t)n_groups * kXcds * m_tiles));
    // four steps in flight (eight were measured too: 3-10 % slower, they halve the occupancy)
    hipLaunchKernelGGL((linear_gemm_small_kernel<XDT, AXIS, 4>), grid, dim3(256), 0, stream,
                       (const uint16_t*)X, (const uint16_t*)W_b, B_packed, v, Y, (int)M, (int)d_out,
                       (int)d_in, y_dtype, m_tiles, n_tiles, v_stride, g_shift);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

template <int XDT, int AXIS, int BM, int WM>
static int launch_gemm(const void* X, const void* W_b, const uint32_t* B_packed, const uint16_t* v,
                       void* Y, int64_t M, int64_t d_out, int64_t d_in, int y_dtype,
                       hipStream_t stream, int v_stride = 0, int g_shift = 31)
{
    const int m_tiles = (int)((M + BM - 1) / BM);
    const int n_tiles = (int)((d_out + kGemmBN - 1) / kGemmBN);
    const int n_groups = (n_tiles + kXcds - 1) / kXcds;
    const dim3 grid((unsigned)((int64_t)n_groups * kXcds * m_tiles));
    hipLaunchKernelGGL((linear_gemm_kernel<XDT, AXIS, BM, WM>), grid, dim3(WM * 128), 0, stream,
                       (const uint16_t*)X, (const uint16_t*)W_b, B_packed, v, Y, (int)M, (int)d_out,
                       (int)d_in, y_dtype, m_tiles, n_tiles, v_stride, g_shift);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

template <int XDT, int AXIS>
static int launch_gemm_bm(const void* X, const void* W_b, const uint32_t* B_packed, const uint16_t* v,
                          void* Y, int64_t M, int64_t d_out, int64_t d_in, int y_dtype,
                          hipStream_t stream)
{
    // Under-filled grids (at most 128 tiles of 256 x 128, i.e. a few hundred tokens): the
    // small-tile kernel is 2-3x faster there; from about 1000 tokens on the big tiles win.
    const int64_t big_tiles = ((M + 255) / 256) * ((d_out + kGemmBN - 1) / kGemmBN);
    const int small = tune_value("gemm_small", -1);
    if (d_in % 64 == 0 && (small == 1 || (small < 0 && big_tiles <= 128)))
        return launch_gemm_small<XDT, AXIS>(X, W_b, B_packed, v, Y, M, d_out, d_in, y_dtype, stream);
    if (M <= 128 || tune_value("gemm_bm", 256) == 128)
        return launch_gemm<XDT, AXIS, 128, 2>(X, W_b, B_packed, v, Y, M, d_out, d_in, y_dtype, stream);
    // The pipelined kernel (one workgroup per CU) is the default: measured 6 % faster on
    // 11008 x 4096, 2 % on 14336 x 4096 and 27 % on 4096 x 11008 (M = 2048) than the two-per-CU
    // kernel, whose finer granularity does not make up for its second barrier per step, and it
    // writes exactly Y (no register spills).  gemm_pipe=0 selects the two-per-CU kernel.
    if (tune_value("gemm_pipe", 1) != 0)
        return launch_gemm_pipe<XDT, AXIS>(X, W_b, B_packed, v, Y, M, d_out, d_in, y_dtype, stream);
    return launch_gemm<XDT, AXIS, 256, 4>(X, W_b, B_packed, v, Y, M, d_out, d_in, y_dtype, stream);
}

// Blockwise scales: the small-tile kernel for under-filled grids, the 128 x 128 tile kernel for
// short batches, else the pipelined 256 x 128 kernel (gemm_pipe=0: two workgroups per compute unit).
template <int XDT>
static int launch_gemm_group(const void* X, const void* W_b, const uint32_t* B_packed, const uint16_t* v, void* Y,
                             int64_t M, int64_t d_out, int64_t d_in, int y_dtype, int v_stride, int g_shift,
                             hipStream_t stream)
{
    const int64_t big_tiles = ((M + 255) / 256) * ((d_out + kGemmBN - 1) / kGemmBN);
    const int small = tune_value("gemm_small", -1);
    if (d_in % 64 == 0 && (small == 1 || (small < 0 && big_tiles <= 128)))
        return launch_gemm_small<XDT, 2>(X, W_b, B_packed, v, Y, M, d_out, d_in, y_dtype, stream, v_stride, g_shift);
    if (M <= 128)
        return launch_gemm<XDT, 2, 128, 2>(X, W_b, B_packed, v, Y, M, d_out, d_in, y_dtype, stream, v_stride, g_shift);
    if (tune_value("gemm_pipe", 1) != 0)
        return launch_gemm_pipe<XDT, 2>(X, W_b, B_packed, v, Y, M, d_out, d_in, y_dtype, stream, v_stride, g_shift);
    return launch_gemm<XDT, 2, 256, 4>(X, W_b, B_packed, v, Y, M, d_out, d_in, y_dtype, stream, v_stride, g_shift);
}

int launch_linear_gemm_group(int x_dtype, int y_dtype, const void* X, const void* W_b,
                             const uint32_t* B_packed, const uint16_t* v, void* Y, int64_t M,
                             int64_t d_out, int64_t d_in, int v_stride, int g_shift, hipStream_t stream)
{
    if (x_dtype == kBF16)
        return launch_gemm_group<kBF16>(X, W_b, B_packed, v, Y, M, d_out, d_in, y_dtype, v_stride, g_shift, stream);
    return launch_gemm_group<kF16>(X, W_b, B_packed, v, Y, M, d_out, d_in, y_dtype, v_stride, g_shift, stream);
}

int launch_linear_gemm(int x_dtype, int y_dtype, int axis, const void* X, const void* W_b,
                       const uint32_t* B_packed, const uint16_t* v, void* Y, int64_t M,
                       int64_t d_out, int64_t d_in, hipStream_t stream)
{
    if (x_dtype == kBF16)
        return axis == 0 ? launch_gemm_bm<kBF16, 0>(X, W_b, B_packed, v, Y, M, d_out, d_in, y_dtype, stream)
                         : launch_gemm_bm<kBF16, 1>(X, W_b, B_packed, v, Y, M, d_out, d_in, y_dtype, stream);
    return axis == 0 ? launch_gemm_bm<kF16, 0>(X, W_b, B_packed, v, Y, M, d_out, d_in, y_dtype, stream)
                     : launch_gemm_bm<kF16, 1>(X, W_b, B_packed, v, Y, M, d_out, d_in, y_dtype, stream);
}

// Measurement builds of the pipelined kernel (bf16 operands, row scales) with parts of its loop
// compiled out; parts = 15 is the product kernel.
int launch_linear_gemm_parts(int parts, int y_dtype, const void* X, const void* W_b, const uint32_t* B_packed,
                             const uint16_t* v, void* Y, int64_t M, int64_t d_out, int64_t d_in,
                             hipStream_t stream)
{
    switch (parts) {
#define PDELTA_PARTS_CASE(P) \
        case P: return launch_gemm_pipe<kBF16, 0, P>(X, W_b, B_packed, v, Y, M, d_out, d_in, y_dtype, stream);
        PDELTA_PARTS_CASE(0) PDELTA_PARTS_CASE(1) PDELTA_PARTS_CASE(2) PDELTA_PARTS_CASE(3) PDELTA_PARTS_CASE(4)
        PDELTA_PARTS_CASE(8) PDELTA_PARTS_CASE(12) PDELTA_PARTS_CASE(13) PDELTA_PARTS_CASE(14) PDELTA_PARTS_CASE(15)
#undef PDELTA_PARTS_CASE
        default: return -2;
    }
}

}  // namespace pdelta
