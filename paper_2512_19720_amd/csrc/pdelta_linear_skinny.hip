// Decode-shaped delta linear layer (M <= 64 tokens):
//   row:  Y[m,o] = sum_i X[m,i] W_b[o,i] + v[o] * sum_i X[m,i] B[o,i]
//   col:  Y[m,o] = sum_i X[m,i] W_b[o,i] +        sum_i (X[m,i] v[i]) B[o,i]
//   grouped (AXIS 2): Y[m,o] = sum_i X[m,i] W_b[o,i] + sum_i X[m,i] (v[o, i / g] B[o,i])
//         with v[row * v_stride + (i >> g_shift)]; v_stride = 0 shares the scales between rows
//         (one scalar for the whole matrix when the group is all of d_in)
// (paper Eq. 1 applied inside the layer forward, never forming W_hat in memory; the grouped form
// is the blockwise extension the paper's conclusion names, its scalar case the BitDelta baseline).
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
#include "pdelta.h"
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

// Grouped scales: the sign-part operands are fp16 whatever the dtype of X: A = fp16(X) and
// B = +-v (the exact product of the +-1 pattern and the group's scale).
template <int XDT>
__device__ __forceinline__ uint4v x_as_f16(uint4v x) {
    if constexpr (XDT == kF16) return x;
    else return scale_x<XDT>(x, (uint4v){0x3C003C00u, 0x3C003C00u, 0x3C003C00u, 0x3C003C00u});
}
__device__ __forceinline__ uint4v signs_times_scale(uint4v pm, uint32_t v_half) {
    const uint32_t vv = v_half | (v_half << 16);
    uint4v r;
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        const uint32_t sp = pm[p];
        r[p] = as_u32(as_half2(sp) * as_half2(vv));                              // v_pk_mul_f16, exact
    }
    return r;
}

template <int MT, int AXIS>
struct SkinnyStep {
    uint4v w[4];        // W_b operand, one per 32-input block
    uint4v sw;          // the step's four sign words of this lane's row
    uint4v x[MT][4];    // X operand per 16-token tile
    uint4v vc[4];       // v_col (column mode only)
    uint32_t vg[4];     // grouped mode: the scale of this lane's row for each 32-input block
};

template <int MT, int AXIS, bool K128>
__device__ __forceinline__ void skinny_load(SkinnyStep<MT, AXIS>& r, const uint16_t* wrow,
                                            const uint32_t* brow, const uint16_t* const (&xrow)[MT],
                                            const uint16_t* vcol, int kb, int K, int g_shift = 31)
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
            r.x[mt][j] = live ? *(const uint4v*)(xrow[mt] + k) : zero;
        if constexpr (AXIS == 1) r.vc[j] = live ? *(const uint4v*)(vcol + k) : zero;
        if constexpr (AXIS == 2) r.vg[j] = live ? (uint32_t)vcol[k >> g_shift] : 0u;   // vcol: this row's scales
    }
}

// W_b and X arrive in the load mapping (lane = 4 row + chunk: four lanes share one L1 access) and
// are moved to the MFMA mapping (lane = 16 chunk + row) by a lane permutation; `perm` is the
// byte address of the lane that loaded this lane's operand.
__device__ __forceinline__ uint4v lanes_to_mfma(uint4v a, int perm)
{
    uint4v r;
#pragma unroll
    for (int p = 0; p < 4; ++p) r[p] = (uint32_t)__builtin_amdgcn_ds_bpermute(perm, (int)a[p]);
    return r;
}

template <int XDT, int MT, int AXIS>
__device__ __forceinline__ void skinny_compute(const SkinnyStep<MT, AXIS>& r, int g, int perm,
                                               float4v (&accb)[MT], float4v (&accs)[MT])
{
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const uint32_t byte = (r.sw[j] >> (g * 8)) & 0xFFu;
        const uint4v wj = lanes_to_mfma(r.w[j], perm);
        uint4v xj[MT];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) xj[mt] = lanes_to_mfma(r.x[mt][j], perm);
        if constexpr (AXIS == 0) {
            const uint4v s = expand_signs<XDT>(byte);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                accb[mt] = mfma16<XDT>(xj[mt], wj, accb[mt]);
                accs[mt] = mfma16<XDT>(xj[mt], s, accs[mt]);
            }
        } else if constexpr (AXIS == 1) {
            const uint4v s = expand_signs<kF16>(byte);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                accb[mt] = mfma16<XDT>(xj[mt], wj, accb[mt]);
                accs[mt] = mfma16<kF16>(scale_x<XDT>(xj[mt], r.vc[j]), s, accs[mt]);
            }
        } else {
            const uint4v s = signs_times_scale(expand_signs<kF16>(byte), r.vg[j]);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                accb[mt] = mfma16<XDT>(xj[mt], wj, accb[mt]);
                accs[mt] = mfma16<kF16>(x_as_f16<XDT>(xj[mt]), s, accs[mt]);
            }
        }
    }
}

// grid.x = ceil(d_out / 16); block = WAVES * 64; dynamic LDS = WAVES * MT * 256 floats.
// DEPTH steps per wave are kept in flight (a ring of register buffers).
template <int XDT, int AXIS, int MT, int WAVES, int DEPTH, bool K128>
__global__ void __launch_bounds__(WAVES * 64)
linear_skinny_kernel(const uint16_t* __restrict__ X, const uint16_t* __restrict__ W_b,
                     const uint32_t* __restrict__ B_packed, const uint16_t* __restrict__ v,
                     void* __restrict__ Y, int M, int d_out, int d_in, int y_dtype, int v_stride, int g_shift)
{
    extern __shared__ float red[];                    // [WAVES][MT][4][64]
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n = lane & 15, g = lane >> 4;
    const int n0 = blockIdx.x * 16;
    const int o = min(n0 + n, d_out - 1);             // rows past the end repeat the last one
    const int K = d_in;

    const int ln = lane >> 2, lg = lane & 3;          // load mapping of W_b and X: row / token, chunk
    const int perm = (n * 4 + g) * 4;
    const uint16_t* wrow = W_b + (int64_t)min(n0 + ln, d_out - 1) * K + lg * 8;
    const uint32_t* brow = B_packed + (int64_t)o * (K >> 5);
    const uint16_t* vcol = AXIS == 1 ? v + g * 8 : (AXIS == 2 ? v + (int64_t)o * v_stride : nullptr);
    const uint16_t* xrow[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        // A operand: lane % 16 is the token.  Tokens past the batch re-read the last real one:
        // MFMA output rows are independent and those rows are never stored, and a load that
        // every lane performs keeps the loop free of divergent branches and of the waits on
        // all outstanding loads that come with them.
        const int t = min(mt * 16 + ln, M - 1);
        xrow[mt] = X + (int64_t)t * K + lg * 8;
    }

    float vr = 1.0f;                                  // row scale: fetched with the first loads
    if constexpr (AXIS == 0) vr = f16_bits_to_f32(v[o]);

    float4v accb[MT], accs[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        accb[mt] = (float4v){0.f, 0.f, 0.f, 0.f};
        accs[mt] = (float4v){0.f, 0.f, 0.f, 0.f};
    }

    // This wave owns steps wave, wave + WAVES, ...  The ring keeps DEPTH of them in flight.  In
    // the steady-state loop every load is unconditional: a load behind a branch makes the
    // compiler wait for all outstanding loads at the join, which would serialise the ring.
    const int nsteps = (K + 127) >> 7;
    const int mine = nsteps > wave ? (nsteps - wave + WAVES - 1) / WAVES : 0;
    SkinnyStep<MT, AXIS> buf[DEPTH];
    auto kb_of = [&](int i) { return (wave + i * WAVES) << 7; };
    if (mine >= DEPTH) {
#pragma unroll
        for (int d = 0; d < DEPTH; ++d) skinny_load<MT, AXIS, K128>(buf[d], wrow, brow, xrow, vcol, kb_of(d), K, g_shift);
        int i = 0;
        for (; i + 2 * DEPTH <= mine; i += DEPTH) {
#pragma unroll
            for (int d = 0; d < DEPTH; ++d) {
                skinny_compute<XDT, MT, AXIS>(buf[d], g, perm, accb, accs);
                skinny_load<MT, AXIS, K128>(buf[d], wrow, brow, xrow, vcol, kb_of(i + DEPTH + d), K, g_shift);
            }
        }
        const int rest = mine - i - DEPTH;            // loads still to issue, 0 <= rest < DEPTH
#pragma unroll
        for (int d = 0; d < DEPTH; ++d) {
            skinny_compute<XDT, MT, AXIS>(buf[d], g, perm, accb, accs);
            if (d < rest) skinny_load<MT, AXIS, K128>(buf[d], wrow, brow, xrow, vcol, kb_of(i + DEPTH + d), K, g_shift);
        }
#pragma unroll
        for (int d = 0; d < DEPTH; ++d)
            if (d < rest) skinny_compute<XDT, MT, AXIS>(buf[d], g, perm, accb, accs);
    } else {
        for (int i = 0; i < mine; ++i) {              // fewer steps than the ring is deep
            skinny_load<MT, AXIS, K128>(buf[0], wrow, brow, xrow, vcol, kb_of(i), K, g_shift);
            skinny_compute<XDT, MT, AXIS>(buf[0], g, perm, accb, accs);
        }
    }

    // Accumulator layout: element r of lane (n, g) is token g*4 + r, output row n0 + n.
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

// ---- staged variant (M <= 16, d_in % 128 == 0, slabs fit in LDS) ---------------------------
// What the plain kernel above loads besides W_b is small but awkward: the sign words of a step
// are a 16-byte piece from each of 16 rows, and at one token X is 64 useful bytes per load
// instruction.  Here the workgroup copies its whole sign slab (16 rows x d_in/8 bytes, one
// contiguous region of B_packed) into LDS with coalesced 16-byte loads while the first W_b
// loads are already in flight, and, when the batch is small enough, X as well (in column mode
// together with fp16(X * v_col), computed once).  The steady-state loop then issues global
// loads for W_b only and reads everything else from LDS.
template <int AXIS, bool STAGE_X>
struct StagedStep {
    uint4v w[4];
    uint4v x[STAGE_X ? 1 : 4];
    uint4v vc[(!STAGE_X && AXIS == 1) ? 4 : 1];
};

// Work of one workgroup: output rows 16 * block .. + 15 of one layer.
template <int XDT, int AXIS, int WAVES, int DEPTH, bool STAGE_X>
__device__ __forceinline__ void
staged_body(const uint16_t* __restrict__ X, const uint16_t* __restrict__ W_b,
            const uint32_t* __restrict__ B_packed, const uint16_t* __restrict__ v,
            void* __restrict__ Y, int M, int d_out, int d_in, int y_dtype, int block,
            int v_stride = 0, int g_shift = 31)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    // nibble -> four +-1.0 values (of the sign operand's dtype): two conflict-free 8-byte LDS
    // reads per sign byte instead of a dozen vector instructions
    __shared__ __attribute__((aligned(16))) uint32_t lut4[16 * 2];
    const int K = d_in;
    const int wpr = K >> 5;                           // sign words per row
    const int spr = wpr + 4;                          // LDS row stride in words: rows 16 B apart in banks
    const int xpr = K + 8;                            // LDS row stride of X in halves
    float* red = (float*)smem;                                        // [WAVES][4][64]
    uint32_t* s_sign = (uint32_t*)(smem + WAVES * 1024);              // [16][spr]
    uint16_t* s_x = (uint16_t*)(s_sign + 16 * spr);                   // [M][xpr]      (STAGE_X)
    uint16_t* s_xv = s_x + (STAGE_X ? M * xpr : 0);                   // [M][xpr]      (STAGE_X: col, or grouped with bf16 X)
    // grouped mode: the scales of the workgroup's 16 rows, [16][ngrp] fp16, behind the X copies
    constexpr bool XV = STAGE_X && (AXIS == 1 || (AXIS == 2 && XDT == kBF16));
    const int ngrp = g_shift >= 31 ? 1 : (K >> g_shift);
    uint16_t* s_v = s_xv + (XV ? M * xpr : 0);

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int n = lane & 15, g = lane >> 4;
    const int n0 = block * 16;
    const int o = min(n0 + n, d_out - 1);

    // When X is not staged (larger batches) the loads of W_b and X use a lane mapping in which
    // four consecutive lanes read 64 consecutive bytes of one row (lane = 4 row + chunk), so that
    // the texture unit merges them into one L1 access; the MFMA wants lane = 16 chunk + row, and
    // a lane permutation (ds_bpermute, LDS crossbar only) puts each 16 bytes where it belongs.
    // In the MFMA's own mapping every lane is its own 16-byte L1 access, and with X as large as
    // the W_b slab the L1 was the limit (measured: TA busy 64 % of the kernel, stalled by the
    // cache for 47 %): -8 % row, -13 % col at M = 16 on 4096 x 4096, -28 % on 4096 x 11008 col.
    // At small batches W_b alone does not load the L1 and the extra hop costs 5-10 %, so there
    // the loads use the MFMA mapping directly.
    constexpr bool COAL = !STAGE_X;
    const int ln = COAL ? lane >> 2 : n, lg = COAL ? lane & 3 : g;   // load mapping: row / token, chunk
    const int perm = (n * 4 + g) * 4;                 // byte address of the lane that loaded (n, g)
    const uint16_t* wrow = W_b + (int64_t)min(n0 + ln, d_out - 1) * K + lg * 8;
    const int tok = min(n, M - 1);                    // A operand: lane % 16 = token (clamped, see above)
    const uint16_t* xrow = X + (int64_t)min(ln, M - 1) * K + lg * 8;
    const uint16_t* vcol = v + g * 8;
    auto to_mfma_layout = [&](uint4v a) {
        if constexpr (!COAL) return a;
        uint4v r;
#pragma unroll
        for (int p = 0; p < 4; ++p) r[p] = (uint32_t)__builtin_amdgcn_ds_bpermute(perm, (int)a[p]);
        return r;
    };

    auto load = [&](StagedStep<AXIS, STAGE_X>& r, int kb) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            r.w[j] = *(const uint4v*)(wrow + kb + j * 32);
            if constexpr (!STAGE_X) {
                r.x[j] = *(const uint4v*)(xrow + kb + j * 32);
                if constexpr (AXIS == 1) r.vc[j] = *(const uint4v*)(vcol + kb + j * 32);
            }
        }
    };

    const int nsteps = K >> 7;
    const int mine = nsteps > wave ? (nsteps - wave + WAVES - 1) / WAVES : 0;   // steps of this wave
    auto kb_of = [&](int i) { return (wave + i * WAVES) << 7; };
    StagedStep<AXIS, STAGE_X> buf[DEPTH];
    const bool ring = mine >= DEPTH;                  // wave-uniform
    if (ring) {
#pragma unroll
        for (int d = 0; d < DEPTH; ++d) load(buf[d], kb_of(d));
    }
    float vr = 1.0f;
    if constexpr (AXIS == 0) vr = f16_bits_to_f32(v[o]);

    if (threadIdx.x < 16) {
        constexpr uint32_t one2 = (AXIS == 0 && XDT == kBF16) ? 0x3F803F80u : 0x3C003C00u;
        const uint32_t neg = ~(uint32_t)threadIdx.x;
        lut4[threadIdx.x * 2 + 0] = one2 | ((neg & 1u) << 15) | ((neg & 2u) << 30);
        lut4[threadIdx.x * 2 + 1] = one2 | (((neg >> 2) & 1u) << 15) | (((neg >> 2) & 2u) << 30);
    }
    // stage the sign slab (and X) while those loads fly
    {
        const int upr = wpr >> 2;                     // 16-byte units per sign row
        for (int i = tid; i < 16 * upr; i += WAVES * 64) {
            const int row = i / upr, u = i - row * upr;
            const int src_row = min(n0 + row, d_out - 1);
            *(uint4v*)(s_sign + row * spr + u * 4) =
                *(const uint4v*)(B_packed + (int64_t)src_row * wpr + u * 4);
        }
        if constexpr (STAGE_X) {
            const int upt = K >> 3;                   // 16-byte units per token
            for (int i = tid; i < M * upt; i += WAVES * 64) {
                const int t = i / upt, u = i - t * upt;
                const uint4v xv = *(const uint4v*)(X + (int64_t)t * K + u * 8);
                *(uint4v*)(s_x + t * xpr + u * 8) = xv;
                if constexpr (AXIS == 1)
                    *(uint4v*)(s_xv + t * xpr + u * 8) = scale_x<XDT>(xv, *(const uint4v*)(v + u * 8));
                if constexpr (AXIS == 2 && XDT == kBF16)
                    *(uint4v*)(s_xv + t * xpr + u * 8) = x_as_f16<XDT>(xv);
            }
        }
        if constexpr (AXIS == 2) {
            for (int i = tid; i < 16 * ngrp; i += WAVES * 64) {
                const int row = i / ngrp, c = i - row * ngrp;
                s_v[i] = v[(int64_t)min(n0 + row, d_out - 1) * v_stride + c];
            }
        }
    }
    __syncthreads();

    float4v accb = {0.f, 0.f, 0.f, 0.f}, accs = {0.f, 0.f, 0.f, 0.f};
    const uint32_t* my_sign = s_sign + n * spr;
    const uint16_t* my_x = s_x + tok * xpr + g * 8;
    const uint16_t* my_xv = s_xv + tok * xpr + g * 8;
    const uint16_t* my_v = s_v + n * ngrp;

    auto compute = [&](const StagedStep<AXIS, STAGE_X>& r, int kb) {
        const uint4v sw = *(const uint4v*)(my_sign + (kb >> 5));
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint32_t byte = (sw[j] >> (g * 8)) & 0xFFu;
            uint4v xa, xs;
            if constexpr (STAGE_X) {
                xa = *(const uint4v*)(my_x + kb + j * 32);
                if constexpr (XV) xs = *(const uint4v*)(my_xv + kb + j * 32);
                else if constexpr (AXIS == 2) xs = xa;
            } else {
                xa = to_mfma_layout(r.x[j]);
                if constexpr (AXIS == 1) xs = scale_x<XDT>(xa, r.vc[j]);
                if constexpr (AXIS == 2) xs = x_as_f16<XDT>(xa);
            }
            const uint4v wj = to_mfma_layout(r.w[j]);
            uint4v sg;
            if constexpr (STAGE_X) {                  // measured: the table wins at small batches (-6 %
                                                      // at M = 1), the vector ALU at M = 16
                typedef uint32_t uint2v __attribute__((ext_vector_type(2)));
                const uint2v lo = *(const uint2v*)((const unsigned char*)lut4 + (byte & 15u) * 8);
                const uint2v hi = *(const uint2v*)((const unsigned char*)lut4 + (byte >> 4) * 8);
                sg = (uint4v){lo[0], lo[1], hi[0], hi[1]};
            } else {
                sg = expand_signs<(AXIS == 0 ? XDT : kF16)>(byte);
            }
            if constexpr (AXIS == 2) sg = signs_times_scale(sg, my_v[(kb + j * 32) >> g_shift]);
            accb = mfma16<XDT>(xa, wj, accb);
            if constexpr (AXIS == 0) accs = mfma16<XDT>(xa, sg, accs);
            else accs = mfma16<kF16>(xs, sg, accs);
        }
    };

    if (ring) {
        int i = 0;
        for (; i + 2 * DEPTH <= mine; i += DEPTH) {   // steady state: unconditional loads only
#pragma unroll
            for (int d = 0; d < DEPTH; ++d) {
                compute(buf[d], kb_of(i + d));
                load(buf[d], kb_of(i + DEPTH + d));
            }
        }
        const int rest = mine - i - DEPTH;            // loads still to issue, 0 <= rest < DEPTH
#pragma unroll
        for (int d = 0; d < DEPTH; ++d) {
            compute(buf[d], kb_of(i + d));
            if (d < rest) load(buf[d], kb_of(i + DEPTH + d));
        }
#pragma unroll
        for (int d = 0; d < DEPTH; ++d)
            if (d < rest) compute(buf[d], kb_of(i + DEPTH + d));
    } else {
        for (int i = 0; i < mine; ++i) {
            load(buf[0], kb_of(i));
            compute(buf[0], kb_of(i));
        }
    }

#pragma unroll
    for (int r = 0; r < 4; ++r) red[(wave * 4 + r) * 64 + lane] = accb[r] + vr * accs[r];
    __syncthreads();
    for (int idx = tid; idx < 256; idx += WAVES * 64) {
        float sum = 0.f;
#pragma unroll
        for (int w = 0; w < WAVES; ++w) sum += red[w * 256 + idx];
        const int ln = idx & 63, r = idx >> 6;
        const int t = (ln >> 4) * 4 + r;
        const int oo = n0 + (ln & 15);
        if (t < M && oo < d_out) {
            const int64_t yi = (int64_t)t * d_out + oo;
            if (y_dtype == kF32) store_y<kF32>(Y, yi, sum);
            else if (y_dtype == kBF16) store_y<kBF16>(Y, yi, sum);
            else store_y<kF16>(Y, yi, sum);
        }
    }
}

template <int XDT, int AXIS, int WAVES, int DEPTH, bool STAGE_X>
__global__ void __launch_bounds__(WAVES * 64)
linear_skinny_staged_kernel(const uint16_t* __restrict__ X, const uint16_t* __restrict__ W_b,
                            const uint32_t* __restrict__ B_packed, const uint16_t* __restrict__ v,
                            void* __restrict__ Y, int M, int d_out, int d_in, int y_dtype, int v_stride,
                            int g_shift)
{
    staged_body<XDT, AXIS, WAVES, DEPTH, STAGE_X>(X, W_b, B_packed, v, Y, M, d_out, d_in, y_dtype,
                                                  (int)blockIdx.x, v_stride, g_shift);
}

// Many layers in one launch (all with the same batch M and dtypes; shapes and axis per layer).
// Workgroup b belongs to the last layer whose first_block is <= b.  One launch instead of one
// per layer removes the per-kernel ramp-up and drain (about 2.4 us each on MI355X, a third of a
// 4096 x 4096 decode layer) for layers that do not depend on each other.
template <int XDT, int WAVES, int DEPTH, bool STAGE_X>
__global__ void __launch_bounds__(WAVES * 64)
linear_skinny_batch_kernel(const pdelta_layer* __restrict__ layers, int n_layers, int M, int y_dtype)
{
    const int b = (int)blockIdx.x;
    int lo = 0, hi = n_layers - 1;
    while (lo < hi) {                                 // workgroup-uniform: scalar loads
        const int mid = (lo + hi + 1) >> 1;
        if (layers[mid].first_block <= b) lo = mid; else hi = mid - 1;
    }
    const pdelta_layer L = layers[lo];
    const int block = b - L.first_block;
    if (L.axis == 0)
        staged_body<XDT, 0, WAVES, DEPTH, STAGE_X>(as_global((const uint16_t*)L.X), as_global((const uint16_t*)L.W_b),
                                                as_global(L.B_packed), as_global(L.v), as_global(L.Y), M,
                                                (int)L.d_out, (int)L.d_in, y_dtype, block);
    else
        staged_body<XDT, 1, WAVES, DEPTH, STAGE_X>(as_global((const uint16_t*)L.X), as_global((const uint16_t*)L.W_b),
                                                as_global(L.B_packed), as_global(L.v), as_global(L.Y), M,
                                                (int)L.d_out, (int)L.d_in, y_dtype, block);
}

constexpr size_t kStagedLdsLimit = 96 * 1024;

// LDS bytes of the staged kernel, or 0 when the slabs do not fit.
// `x_copies`: LDS copies of X (2 when the sign part needs its own fp16 operand: column mode, or
// grouped mode with bf16 X); `scale_halves`: grouped mode's 16 rows of scales.
static size_t staged_lds_bytes(int waves, int x_copies, bool stage_x, int64_t M, int64_t K, int64_t scale_halves = 0)
{
    size_t bytes = (size_t)waves * 1024 + (size_t)16 * (K / 32 + 4) * 4 + (size_t)scale_halves * 2 + 16;
    if (stage_x) bytes += (size_t)M * (K + 8) * 2 * x_copies;
    return bytes <= kStagedLdsLimit ? bytes : 0;
}
static int x_copies_of(int axis, int x_dtype) { return axis == 1 || (axis == 2 && x_dtype == kBF16) ? 2 : 1; }

template <int XDT, int AXIS, int WAVES, int DEPTH, bool STAGE_X>
static int launch_staged(const void* X, const void* W_b, const uint32_t* B_packed, const uint16_t* v,
                         void* Y, int64_t M, int64_t d_out, int64_t d_in, int y_dtype, size_t lds,
                         hipStream_t stream, int v_stride = 0, int g_shift = 31)
{
    const dim3 grid((unsigned)((d_out + 15) / 16));
    auto kernel = linear_skinny_staged_kernel<XDT, AXIS, WAVES, DEPTH, STAGE_X>;
    static unsigned lds_opted_in = 0;                 // per template instance: one kernel
    if (lds > 48 * 1024 && opt_in_dynamic_lds((const void*)kernel, (int)kStagedLdsLimit, &lds_opted_in) != 0)
        return -1;           // above the default dynamic-LDS limit the kernel has to opt in (once)
    hipLaunchKernelGGL(kernel, grid, dim3(WAVES * 64), lds, stream, (const uint16_t*)X,
                       (const uint16_t*)W_b, B_packed, v, Y, (int)M, (int)d_out, (int)d_in, y_dtype, v_stride,
                       g_shift);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

// Returns 1 if the staged kernel does not apply, else the launch result (0 / -1).
template <int XDT, int AXIS>
static int try_staged(const void* X, const void* W_b, const uint32_t* B_packed, const uint16_t* v,
                      void* Y, int64_t M, int64_t d_out, int64_t d_in, int y_dtype,
                      hipStream_t stream)
{
    if (M > 16 || d_in % 128 != 0) return 1;
    // Measured on MI355X (4096 x 4096, 11008 x 4096, 4096 x 11008; 1 and 16 tokens): with the plain
    // kernel's loads in the coalesced lane mapping the staged kernel only wins where it saves real
    // work, in column mode with X small enough for LDS (fp16(X * v_col) is then formed once per
    // workgroup instead of once per step: 18.8 against 22.1 us on 11008 x 4096).  Everywhere else
    // the plain kernel is as fast or up to 6 % faster (no staging phase before the first MFMA).
    const bool staged_pays = AXIS == 1 && M * d_in <= 24576;
    if (tune_value("skinny_staged", staged_pays ? 1 : 0) == 0) return 1;
    // Measured on MI355X: 8 waves with 2 steps in flight each is the best general choice; when a
    // layer is wide (d_in >= 8192) but has few workgroups (<= 2 per CU) 16 waves fill the CU better.
    const bool wide_few = d_in >= 8192 && (d_out + 15) / 16 <= 512;
    // (not in column mode with X read through L2: that variant needs more than the 128 registers
    // a 16-wave workgroup leaves per lane and spills - measured 37 us against 24 us with 8 waves)
    const bool x_small = M * d_in <= 24576;
    constexpr int XC = AXIS == 1 ? 2 : 1;             // LDS copies of X
    const bool col16_ok = x_small && staged_lds_bytes(16, XC, true, M, d_in) != 0;   // X fits LDS at 16 waves
    const int waves = tune_value("stg_waves", wide_few && (AXIS == 0 || col16_ok) ? 16 : 8);
    const bool want_x = tune_value("stg_x", 1) != 0;
    size_t lds = want_x ? staged_lds_bytes(waves, XC, true, M, d_in) : 0;
    const bool stage_x = lds != 0 && x_small;
    if (!stage_x) lds = staged_lds_bytes(waves, XC, false, M, d_in);
    // Row mode, small batch, exactly four steps per wave (d_in = 4096 at 8 waves): all four in
    // flight from the start is 3 % faster than a ring of two (same-run A/B); elsewhere it makes no
    // difference or loses (column mode and larger batches carry more registers per step).
    const int depth = tune_value("stg_depth", (AXIS == 0 && stage_x && d_in / 128 == 4 * waves) ? 4 : 2);
    if (lds == 0) return 1;
#define PDELTA_STG(WAVES, DEPTH)                                                                        \
    return stage_x ? launch_staged<XDT, AXIS, WAVES, DEPTH, true>(X, W_b, B_packed, v, Y, M, d_out, d_in, \
                                                                   y_dtype, lds, stream)                  \
                   : launch_staged<XDT, AXIS, WAVES, DEPTH, false>(X, W_b, B_packed, v, Y, M, d_out, d_in, \
                                                                    y_dtype, lds, stream)
    if (waves == 4) {
        if (depth == 8) PDELTA_STG(4, 8);
        PDELTA_STG(4, 4);
    }
    if (waves == 16) PDELTA_STG(16, 2);
    if (depth == 2) PDELTA_STG(8, 2);
    if (depth == 6) PDELTA_STG(8, 6);
    PDELTA_STG(8, 4);
#undef PDELTA_STG
}

template <int XDT, int AXIS, int MT, int WAVES, int DEPTH, bool K128>
static int launch_one(const void* X, const void* W_b, const uint32_t* B_packed, const uint16_t* v,
                      void* Y, int64_t M, int64_t d_out, int64_t d_in, int y_dtype,
                      hipStream_t stream, int v_stride = 0, int g_shift = 31)
{
    const dim3 grid((unsigned)((d_out + 15) / 16));
    const size_t lds = (size_t)WAVES * MT * 256 * sizeof(float);
    hipLaunchKernelGGL((linear_skinny_kernel<XDT, AXIS, MT, WAVES, DEPTH, K128>), grid, dim3(WAVES * 64), lds,
                       stream, (const uint16_t*)X, (const uint16_t*)W_b, B_packed, v, Y, (int)M,
                       (int)d_out, (int)d_in, y_dtype, v_stride, g_shift);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

template <int XDT, int AXIS, bool K128>
static int launch_by_tokens(const void* X, const void* W_b, const uint32_t* B_packed,
                            const uint16_t* v, void* Y, int64_t M, int64_t d_out, int64_t d_in,
                            int y_dtype, hipStream_t stream)
{
#define PDELTA_GO(MT, WAVES, DEPTH) \
    return launch_one<XDT, AXIS, MT, WAVES, DEPTH, K128>(X, W_b, B_packed, v, Y, M, d_out, d_in, y_dtype, stream)
    const int waves = tune_value("skinny_waves", 8);
    // steps in flight per wave: two, except row mode at more than 8 tokens, where one is 3-4 %
    // faster (measured; the X loads double the bytes in flight per step)
    const int depth = tune_value("skinny_depth", (AXIS == 0 && M > 8) ? 1 : 2);
    if (M <= 16) {
        if (waves == 4) {
            if (depth == 4) PDELTA_GO(1, 4, 4);
            if (depth == 6) PDELTA_GO(1, 4, 6);
            PDELTA_GO(1, 4, 2);
        }
        if (waves == 16) PDELTA_GO(1, 16, 2);
        if (depth == 1) PDELTA_GO(1, 8, 1);
        if (depth == 3) PDELTA_GO(1, 8, 3);
        if (depth == 4) PDELTA_GO(1, 8, 4);
        PDELTA_GO(1, 8, 2);
    }
    if (M <= 32) PDELTA_GO(2, 8, 2);
    if (M <= 48) PDELTA_GO(3, 8, 1);
    PDELTA_GO(4, 8, 1);
#undef PDELTA_GO
}

int launch_linear_skinny_batch(int x_dtype, int y_dtype, const pdelta_layer* layers_host,
                               const pdelta_layer* layers_device, int n_layers, int64_t M,
                               hipStream_t stream)
{
    // applicable when every layer can use the staged kernel (sign slab in LDS); X goes to LDS too
    // when it is small enough in every layer, else all layers read it through L2
    if (M > 16 || tune_value("skinny_batch", 1) == 0) return 1;
    bool stage_x = true;
    for (int l = 0; l < n_layers; ++l) {
        const pdelta_layer& L = layers_host[l];
        if (L.d_in % 128 != 0) return 1;
        if (M * L.d_in > 24576 || staged_lds_bytes(8, L.axis == 1 ? 2 : 1, true, M, L.d_in) == 0) stage_x = false;
    }
    int64_t total = 0;
    size_t lds = 0;
    for (int l = 0; l < n_layers; ++l) {
        const pdelta_layer& L = layers_host[l];
        const size_t need = staged_lds_bytes(8, L.axis == 1 ? 2 : 1, stage_x, M, L.d_in);
        if (need == 0) return 1;
        if (need > lds) lds = need;
        total += (L.d_out + 15) / 16;
    }
    if (total > 0x7FFFFFFF) return 1;
    void (*kernel)(const pdelta_layer*, int, int, int);
    if (x_dtype == kBF16) kernel = stage_x ? linear_skinny_batch_kernel<kBF16, 8, 2, true> : linear_skinny_batch_kernel<kBF16, 8, 2, false>;
    else kernel = stage_x ? linear_skinny_batch_kernel<kF16, 8, 2, true> : linear_skinny_batch_kernel<kF16, 8, 2, false>;
    static unsigned lds_opted_in[4] = {0, 0, 0, 0};   // one word per kernel chosen above
    unsigned* done = &lds_opted_in[(x_dtype == kBF16 ? 2 : 0) + (stage_x ? 1 : 0)];
    if (lds > 48 * 1024 && opt_in_dynamic_lds((const void*)kernel, (int)kStagedLdsLimit, done) != 0) return -1;
    hipLaunchKernelGGL(kernel, dim3((unsigned)total), dim3(8 * 64), lds, stream, layers_device,
                       n_layers, (int)M, y_dtype);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

// Grouped (blockwise / scalar) scales, M <= kSkinnyMaxM: the staged kernel when it applies (up to
// 16 tokens, d_in a multiple of 128, slabs fit LDS), else the plain kernel.
template <int XDT>
static int launch_group(int y_dtype, const void* X, const void* W_b, const uint32_t* B_packed, const uint16_t* v,
                        void* Y, int64_t M, int64_t d_out, int64_t d_in, int v_stride, int g_shift,
                        hipStream_t stream)
{
    if (M <= 16 && d_in % 128 == 0 && tune_value("skinny_staged", 1) != 0) {
        const int64_t scale_halves = 16 * (g_shift >= 31 ? 1 : (d_in >> g_shift));
        const int xc = x_copies_of(2, XDT);
        size_t lds = M * d_in <= 24576 ? staged_lds_bytes(8, xc, true, M, d_in, scale_halves) : 0;
        const bool stage_x = lds != 0;
        if (!stage_x) lds = staged_lds_bytes(8, xc, false, M, d_in, scale_halves);
        if (lds != 0)
            return stage_x ? launch_staged<XDT, 2, 8, 2, true>(X, W_b, B_packed, v, Y, M, d_out, d_in, y_dtype, lds,
                                                               stream, v_stride, g_shift)
                           : launch_staged<XDT, 2, 8, 2, false>(X, W_b, B_packed, v, Y, M, d_out, d_in, y_dtype, lds,
                                                                stream, v_stride, g_shift);
    }
#define PDELTA_GO(MT, DEPTH)                                                                                   \
    return d_in % 128 == 0                                                                                     \
               ? launch_one<XDT, 2, MT, 8, DEPTH, true>(X, W_b, B_packed, v, Y, M, d_out, d_in, y_dtype, stream, \
                                                        v_stride, g_shift)                                     \
               : launch_one<XDT, 2, MT, 8, DEPTH, false>(X, W_b, B_packed, v, Y, M, d_out, d_in, y_dtype, stream, \
                                                         v_stride, g_shift)
    if (M <= 16) PDELTA_GO(1, 2);
    if (M <= 32) PDELTA_GO(2, 2);
    if (M <= 48) PDELTA_GO(3, 1);
    PDELTA_GO(4, 1);
#undef PDELTA_GO
}

int launch_linear_skinny_group(int x_dtype, int y_dtype, const void* X, const void* W_b,
                               const uint32_t* B_packed, const uint16_t* v, void* Y, int64_t M,
                               int64_t d_out, int64_t d_in, int v_stride, int g_shift, hipStream_t stream)
{
    if (x_dtype == kBF16)
        return launch_group<kBF16>(y_dtype, X, W_b, B_packed, v, Y, M, d_out, d_in, v_stride, g_shift, stream);
    return launch_group<kF16>(y_dtype, X, W_b, B_packed, v, Y, M, d_out, d_in, v_stride, g_shift, stream);
}

int launch_linear_skinny(int x_dtype, int y_dtype, int axis, const void* X, const void* W_b,
                         const uint32_t* B_packed, const uint16_t* v, void* Y, int64_t M,
                         int64_t d_out, int64_t d_in, hipStream_t stream)
{
    const bool k128 = d_in % 128 == 0;
    {
        int rc = 1;
        if (x_dtype == kBF16)
            rc = axis == 0 ? try_staged<kBF16, 0>(X, W_b, B_packed, v, Y, M, d_out, d_in, y_dtype, stream)
                           : try_staged<kBF16, 1>(X, W_b, B_packed, v, Y, M, d_out, d_in, y_dtype, stream);
        else
            rc = axis == 0 ? try_staged<kF16, 0>(X, W_b, B_packed, v, Y, M, d_out, d_in, y_dtype, stream)
                           : try_staged<kF16, 1>(X, W_b, B_packed, v, Y, M, d_out, d_in, y_dtype, stream);
        if (rc != 1) return rc;
    }
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
