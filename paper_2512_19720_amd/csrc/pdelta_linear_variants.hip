// Multi-variant decode: R requests share the base weights W_b and each brings its own 1-bit
// delta (B_r, v_r) - many fine-tuned variants of one base served together, the setting the
// paper's introduction motivates.  Request r is one token:
//   row:  Y[r,o] = sum_i X[r,i] W_b[o,i] + v_r[o] * sum_i X[r,i] B_r[o,i]
//   col:  Y[r,o] = sum_i X[r,i] W_b[o,i] +          sum_i (X[r,i] v_r[i]) B_r[o,i]
// (paper Eq. 1 per request inside the layer forward).  W_b is read ONCE for all requests:
// 2 + R/8 bytes per weight instead of R (2 + 1/8).
//
// Work split as in the decode kernel: a workgroup (8 waves) owns 16 consecutive output rows and
// all of d_in; a wave takes 128-input steps, one step of W_b / X loads in flight ahead of the
// arithmetic.  The base part is one MFMA stream with the R tokens as the rows of the A operand.
// The delta part cannot be one matrix product (the matrix depends on the token), so request r
// gets its own accumulator: acc_r += A x signs(B_r), of which only token row r is kept at the
// end.  The matrix cores are idle anyway; what would bind is turning sign bits into +-1 operands
// R times per weight on the vector ALU, so that goes through a 16-entry table in LDS (two
// conflict-free 8-byte reads per sign byte), with the reads of the next input block issued
// before the MFMAs of the current one.  The sign slabs of all requests for the workgroup's 16 rows (contiguous in
// each B_packed) are copied to LDS first with coalesced loads that are all in flight together;
// when they do not fit (large d_in x R) the requests go in several passes, or, for very large
// d_in, with their sign words in registers, 8 requests per pass.
#include "pdelta.h"
#include "pdelta_device.h"
#include "pdelta_host.h"

namespace pdelta {

constexpr int kVarMaxR = 16;     // requests per launch (rows of the MFMA's A operand)

template <int DT>
__device__ __forceinline__ float4v var_mfma(uint4v a, uint4v b, float4v c) {
    if constexpr (DT == kBF16)
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a),
                                                       __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8, a),
                                                      __builtin_bit_cast(half8, b), c, 0, 0, 0);
}

struct VarStep {
    uint4v w[4];                 // W_b operand per 32-input block (group 0 only uses it)
    uint4v x[4];                 // A operand: lane % 16 = request
    uint4v vc[4];                // v_r slice of this lane's request (column mode)
    uint4v sw[8];                // four sign words of this lane's row per request (not staged: <= 8)
};

// XDT: dtype of X and W_b.  AXIS as in the single-variant kernels, or 2: each request brings its
// own axis (variants[r].axis); the sign part then runs in fp16 with the operand fp16(x * v_r) for
// column-mode requests and fp16(x * 1) for row-mode ones.  NQ = 8 or 16 request slots
// (R <= NQ).  STAGE: the sign slabs of all requests are copied to LDS first.
template <int XDT, int AXIS, int NQ, bool STAGE>
__global__ void __launch_bounds__(512, 2)
linear_variants_kernel(const uint16_t* __restrict__ X, const uint16_t* __restrict__ W_b,
                       const pdelta_variant* __restrict__ variants, int R, void* __restrict__ Y,
                       int d_out, int d_in, int y_dtype)
{
    constexpr int SDT = AXIS == 0 ? XDT : kF16;       // dtype of the sign-part operands
    __shared__ __attribute__((aligned(16))) uint32_t lut4[16 * 2];          // nibble -> four +-1.0
    __shared__ float red_b[8][16][16];                                       // [k-wave][token][row]
    __shared__ float red_s[8][NQ][16];                                       // [k-wave][request][row]
    extern __shared__ __attribute__((aligned(16))) uint32_t s_sign[];        // STAGE: [slot][16][spr]

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int kw = wave;
    const int n = lane & 15, g = lane >> 4;
    const int n0 = blockIdx.x * 16;
    const int o = min(n0 + n, d_out - 1);
    const int K = d_in, wpr = K >> 5;

    // table of +-1 operands: entry b holds, for e = 0..3, +1.0 if bit e of b is set, else -1.0
    if (tid < 16) {
        constexpr uint32_t one2 = SDT == kBF16 ? 0x3F803F80u : 0x3C003C00u;
        const uint32_t neg = ~(uint32_t)tid;
        lut4[tid * 2 + 0] = one2 | ((neg & 1u) << 15) | ((neg & 2u) << 30);
        lut4[tid * 2 + 1] = one2 | (((neg >> 2) & 1u) << 15) | (((neg >> 2) & 2u) << 30);
    }

    // operands: this lane's W_b row, its request's X row and (column mode) scale row; requests
    // past R repeat the last real one (their results are never stored)
    const int req = min(n, R - 1);
    const uint16_t* wrow = W_b + (int64_t)o * K + g * 8;
    const uint16_t* xrow = X + (int64_t)req * K + g * 8;
    // per-request axis: a row-mode request has no scale per input; its loads of "v" read its own
    // X row instead (valid memory of the right length) and the value is replaced by 1.0
    const bool col = AXIS == 1 || (AXIS == 2 && variants[req].axis == PDELTA_COL);
    const uint16_t* vrow = AXIS == 0 ? nullptr : (col ? as_global_per_lane(variants[req].v) + g * 8 : xrow);
    static_assert(STAGE || NQ == 8, "without staging a step keeps the sign words of 8 requests in registers");
    const uint32_t* brow[NQ];                         // this lane's sign row per request
    const int spr = wpr + 4;                          // LDS row stride in words (STAGE)
#pragma unroll
    for (int q = 0; q < NQ; ++q) {
        const int r = min(q, R - 1);
        if constexpr (STAGE) brow[q] = s_sign + (r * 16 + n) * spr;
        else brow[q] = as_global(variants[r].B_packed) + (int64_t)o * wpr;
    }

    auto load = [&](VarStep& S, int kb) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            S.w[j] = *(const uint4v*)(wrow + kb + j * 32);
            S.x[j] = *(const uint4v*)(xrow + kb + j * 32);
            if constexpr (AXIS != 0) S.vc[j] = *(const uint4v*)(vrow + kb + j * 32);
        }
        if constexpr (!STAGE) {
#pragma unroll
            for (int q = 0; q < NQ; ++q) S.sw[q] = *(const uint4v*)(brow[q] + (kb >> 5));
        }
    };

    float4v accb = {0.f, 0.f, 0.f, 0.f};
    float4v acc[NQ];
#pragma unroll
    for (int q = 0; q < NQ; ++q) acc[q] = (float4v){0.f, 0.f, 0.f, 0.f};

    // One step.  Requests go in halves of 8; within a half the table reads of input block j+1 are
    // issued before the 8 MFMAs of block j, so that the LDS latency hides behind the matrix
    // instructions (left alone the compiler issues read, wait, MFMA one at a time).
    auto compute = [&](const VarStep& S, int kb) {
        uint4v xs[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            xs[j] = S.x[j];
            if constexpr (AXIS != 0) {                // sign-part operand: fp16(x * v_r)
#pragma unroll
                for (int p = 0; p < 4; ++p) {
                    const uint32_t vp = col ? (uint32_t)S.vc[j][p] : 0x3C003C00u;      // row-mode request: 1.0
                    if constexpr (XDT == kF16) {
                        const uint32_t xp = S.x[j][p];
                        xs[j][p] = as_u32(as_half2(xp) * as_half2(vp));
                    } else {
                        const float lo = bf16_bits_to_f32(S.x[j][p] & 0xFFFFu) * f16_bits_to_f32(vp & 0xFFFFu);
                        const float hi = bf16_bits_to_f32(S.x[j][p] >> 16) * f16_bits_to_f32(vp >> 16);
                        xs[j][p] = f32_to_f16_bits(lo) | (f32_to_f16_bits(hi) << 16);
                    }
                }
            }
            accb = var_mfma<XDT>(S.x[j], S.w[j], accb);
        }
        constexpr int HQ = NQ < 8 ? NQ : 8;           // requests per half
#pragma unroll
        for (int h = 0; h < NQ / HQ; ++h) {
            uint4v sw[HQ];
#pragma unroll
            for (int q = 0; q < HQ; ++q) {
                if constexpr (STAGE) sw[q] = *(const uint4v*)(brow[h * HQ + q] + (kb >> 5));
                else sw[q] = S.sw[q];
            }
            uint4v cur[HQ], nxt[HQ];
            auto lookups = [&](uint4v (&dst)[HQ], int j) {
#pragma unroll
                for (int q = 0; q < HQ; ++q) {
                    const uint32_t byte = (sw[q][j] >> (g * 8)) & 0xFFu;
                    // two 8-byte reads from a 16-entry table: lanes that read the same entry are
                    // served by one broadcast and the 16 entries lie in distinct banks, so the
                    // gather is free of bank conflicts (a 256-entry table of 16-byte entries is not:
                    // measured 6-8 % slower)
                    typedef uint32_t uint2v __attribute__((ext_vector_type(2)));
                    const uint2v lo = *(const uint2v*)((const unsigned char*)lut4 + (byte & 15u) * 8);
                    const uint2v hi = *(const uint2v*)((const unsigned char*)lut4 + (byte >> 4) * 8);
                    dst[q] = (uint4v){lo[0], lo[1], hi[0], hi[1]};
                }
            };
            lookups(cur, 0);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if (j + 1 < 4) lookups(nxt, j + 1);
#pragma unroll
                for (int q = 0; q < HQ; ++q) acc[h * HQ + q] = var_mfma<SDT>(xs[j], cur[q], acc[h * HQ + q]);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int q = 0; q < HQ; ++q) cur[q] = nxt[q];
            }
        }
    };

    // STAGE: every request's sign slab of these 16 rows (contiguous in its B_packed) goes to LDS
    // with coalesced 16-byte loads, all in flight at once, behind the first W_b / X loads
    VarStep A, B;
    const int nsteps = K >> 7;
    if (kw < nsteps) load(A, kw << 7);
    if constexpr (STAGE) {
        // unit i of a slab = 16 bytes: row i / upr, words 4 (i % upr) ..; the loads of all slots
        // are issued together (slots past R repeat the last request and are not stored)
        const int upr = wpr >> 2, per_slot = 16 * upr;
        const uint32_t* slab[NQ];
#pragma unroll
        for (int q = 0; q < NQ; ++q) slab[q] = as_global(variants[min(q, R - 1)].B_packed);     // uniform
        for (int first = 0; first < per_slot; first += 512) {
            const int i = first + tid;
            const int ic = min(i, per_slot - 1);
            const int row = ic / upr, u = ic - row * upr;
            const int64_t src = (int64_t)min(n0 + row, d_out - 1) * wpr + u * 4;
            uint4v tmp[NQ];
#pragma unroll
            for (int q = 0; q < NQ; ++q) tmp[q] = *(const uint4v*)(slab[q] + src);
#pragma unroll
            for (int q = 0; q < NQ; ++q)
                if (i < per_slot && q < R) *(uint4v*)(s_sign + (q * 16 + row) * spr + u * 4) = tmp[q];
        }
    }
    __syncthreads();                                  // table and slabs are complete

    // steps kw, kw + 8, ...: one step of loads in flight ahead of the arithmetic
    {
        int s = kw;
        for (; s + 16 < nsteps; s += 16) {            // steady state: unconditional loads
            load(B, (s + 8) << 7);
            compute(A, s << 7);
            load(A, (s + 16) << 7);
            compute(B, (s + 8) << 7);
        }
        if (s < nsteps) {
            if (s + 8 < nsteps) {
                load(B, (s + 8) << 7);
                compute(A, s << 7);
                compute(B, (s + 8) << 7);
            } else {
                compute(A, s << 7);
            }
        }
    }

    // accumulator element c of lane (n, g) is token 4g + c, output row n0 + n
#pragma unroll
    for (int c = 0; c < 4; ++c) red_b[kw][g * 4 + c][n] = accb[c];
#pragma unroll
    for (int q = 0; q < NQ; ++q) {                    // request q = token q: keep that row only
        if (g == (q >> 2)) red_s[kw][q][n] = acc[q][q & 3];
    }
    __syncthreads();
    if (tid < 256) {
        const int t = tid >> 4, nn = tid & 15;
        const int oo = n0 + nn;
        if (t < R && oo < d_out) {
            float base = 0.f, delta = 0.f;
#pragma unroll
            for (int w = 0; w < 8; ++w) {
                base += red_b[w][t][nn];
                delta += red_s[w][t < NQ ? t : 0][nn];
            }
            float scale = 1.0f;
            if (AXIS == 0 || (AXIS == 2 && variants[t].axis == PDELTA_ROW)) scale = f16_bits_to_f32(as_global_per_lane(variants[t].v)[oo]);
            const float sum = base + scale * delta;
            const int64_t yi = (int64_t)t * d_out + oo;
            if (y_dtype == kF32) store_y<kF32>(Y, yi, sum);
            else if (y_dtype == kBF16) store_y<kBF16>(Y, yi, sum);
            else store_y<kF16>(Y, yi, sum);
        }
    }
}

constexpr size_t kVarStageBytes = 136 * 1024;    // LDS for sign slabs, next to 24 KB of tables

template <int XDT, int AXIS, int NQ, bool STAGE>
static int launch_variants_one(const void* X, const void* W_b, const pdelta_variant* variants_device, int R,
                               void* Y, int64_t d_out, int64_t d_in, int y_dtype, hipStream_t stream)
{
    const size_t lds = STAGE ? (size_t)R * 16 * (d_in / 8 + 16) : 0;
    auto kernel = linear_variants_kernel<XDT, AXIS, NQ, STAGE>;
    static unsigned lds_opted_in = 0;                 // per template instance: one kernel
    if (lds > 32 * 1024 && opt_in_dynamic_lds((const void*)kernel, (int)kVarStageBytes, &lds_opted_in) != 0)
        return -1;
    hipLaunchKernelGGL(kernel, dim3((unsigned)((d_out + 15) / 16)), dim3(512), lds, stream, (const uint16_t*)X,
                       (const uint16_t*)W_b, variants_device, R, Y, (int)d_out, (int)d_in, y_dtype);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

// Requests go in chunks that share one pass over W_b: up to 16 when their sign slabs (16 rows x
// d_in / 8 bytes each) fit in LDS together, else up to 8 with the sign words in registers.
template <int XDT, int AXIS>
static int launch_variants(const void* X, const void* W_b, const pdelta_variant* variants_device, int R,
                           void* Y, int64_t d_out, int64_t d_in, int y_dtype, hipStream_t stream)
{
    const size_t per_request = (size_t)16 * (d_in / 8 + 16);
    int cap = (int)(kVarStageBytes / per_request);
    if (tune_value("var_stage", 1) == 0) cap = 0;
    const bool stage = cap >= 1;
    const int chunk = stage ? (cap < kVarMaxR ? cap : kVarMaxR) : 8;
    const size_t ysz = y_dtype == kF32 ? 4 : 2;
    for (int r0 = 0; r0 < R; r0 += chunk) {
        const int n = R - r0 < chunk ? R - r0 : chunk;
        const void* Xc = (const char*)X + (size_t)r0 * d_in * 2;
        void* Yc = (char*)Y + (size_t)r0 * d_out * ysz;
        const pdelta_variant* vc = variants_device + r0;
        int rc;
        if (!stage) rc = launch_variants_one<XDT, AXIS, 8, false>(Xc, W_b, vc, n, Yc, d_out, d_in, y_dtype, stream);
        else if (n <= 4) rc = launch_variants_one<XDT, AXIS, 4, true>(Xc, W_b, vc, n, Yc, d_out, d_in, y_dtype, stream);
        else if (n <= 8) rc = launch_variants_one<XDT, AXIS, 8, true>(Xc, W_b, vc, n, Yc, d_out, d_in, y_dtype, stream);
        else rc = launch_variants_one<XDT, AXIS, 16, true>(Xc, W_b, vc, n, Yc, d_out, d_in, y_dtype, stream);
        if (rc != 0) return rc;
    }
    return 0;
}

// Returns 1 when the fused kernel does not apply (the caller then runs the requests one by
// one), else 0 / -1.
int launch_linear_variants(int x_dtype, int y_dtype, int axis, const void* X, const void* W_b,
                           const pdelta_variant* variants_device, int R, void* Y, int64_t d_out,
                           int64_t d_in, hipStream_t stream)
{
    if (d_in % 128 != 0 || tune_value("variants_fused", 1) == 0) return 1;
#define PDELTA_VAR(XDT)                                                                                         \
    return axis == 0   ? launch_variants<XDT, 0>(X, W_b, variants_device, R, Y, d_out, d_in, y_dtype, stream)  \
           : axis == 1 ? launch_variants<XDT, 1>(X, W_b, variants_device, R, Y, d_out, d_in, y_dtype, stream)  \
                       : launch_variants<XDT, 2>(X, W_b, variants_device, R, Y, d_out, d_in, y_dtype, stream)
    if (x_dtype == kBF16) PDELTA_VAR(kBF16);
    PDELTA_VAR(kF16);
#undef PDELTA_VAR
}

}  // namespace pdelta
