// Multi-variant decode: R requests share the base weights W_b and each brings its own 1-bit
// delta (B_r, v_r) - many fine-tuned variants of one base served together, the setting the
// paper's introduction motivates.  Request r is one token:
//   row:  Y[r,o] = sum_i X[r,i] W_b[o,i] + v_r[o] * sum_i X[r,i] B_r[o,i]
//   col:  Y[r,o] = sum_i X[r,i] W_b[o,i] +          sum_i (X[r,i] v_r[i]) B_r[o,i]
// (paper Eq. 1 per request inside the layer forward).  W_b is read ONCE for all requests:
// 2 + R/8 bytes per weight instead of R (2 + 1/8).
//
// Work split as in the decode kernel: a workgroup (8 waves) owns 16 consecutive output rows and
// all of d_in; a wave takes 128-input steps round-robin, one step of loads in flight ahead of the
// arithmetic.  The base part is one MFMA stream with the R tokens as the rows of the A operand.
// The delta part cannot be one matrix product (the matrix depends on the token), so request r
// gets its own accumulator: acc_r += A x signs(B_r), of which only token row r is kept at the
// end.  The matrix cores have the time; what binds is turning sign bits into +-1 operands R
// times per weight, so the layout is chosen to make that two vector instructions per operand
// register and the sign traffic one 4-byte load per lane, request and step:
//   - lane (n = lane % 16, g = lane / 16) owns the 32 inputs k0 .. k0 + 31, k0 = step + 32 g, of
//     output row n (W_b, signs) or of token n (X): 64 contiguous bytes of W_b / X (four 16-byte
//     loads) and exactly ONE 32-bit sign word per request;
//   - MFMA block j (j = 0..3) multiplies, in operand register p, the input pair
//     (k0 + 4j + p, k0 + 16 + 4j + p).  Which 32 of the step's 128 inputs form a block is free as
//     long as A and B agree; with THIS pairing the two sign bits of a register are 16 bits apart,
//     like the two sign positions of a pair of 16-bit floats, so
//         operand = ((~word << (15 - 4j - p)) & 0x80008000) | (1.0, 1.0)
//     (one shift, one and-or); W_b and X get into the same order with one byte permute per register.
// Nothing goes through LDS but the final cross-wave sums.
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

// The lane's 32 consecutive 16-bit values as loaded (l[i] = values 8i .. 8i+7) -> the operand of
// MFMA block j: register p = (value 4j + p, value 16 + 4j + p).
__device__ __forceinline__ uint4v var_block_operand(const uint4v (&l)[4], int j)
{
    const uint4v a = l[j >> 1], b = l[2 + (j >> 1)];
    const int r0 = (j & 1) * 2;                       // registers r0, r0 + 1 of a and b hold values 4 (j & 1) .. + 3
    uint4v o;
    o[0] = __builtin_amdgcn_perm(b[r0], a[r0], 0x05040100u);          // low halves
    o[1] = __builtin_amdgcn_perm(b[r0], a[r0], 0x07060302u);          // high halves
    o[2] = __builtin_amdgcn_perm(b[r0 + 1], a[r0 + 1], 0x05040100u);
    o[3] = __builtin_amdgcn_perm(b[r0 + 1], a[r0 + 1], 0x07060302u);
    return o;
}

// +-1.0 operand of block j from the complement of the lane's sign word (bit set = minus).
// sign_bits = 0x80008000 and one2 = (1.0, 1.0) are passed in registers: with both as literals the
// and-or would be two instructions (one literal per instruction on this target).
__device__ __forceinline__ uint4v var_sign_operand(uint32_t minus, int j, uint32_t sign_bits, uint32_t one2)
{
    uint4v o;
#pragma unroll
    for (int p = 0; p < 4; ++p) o[p] = ((minus << (15 - 4 * j - p)) & sign_bits) | one2;
    return o;
}

// ---- stride kernel ---------------------------------------------------------------------------

template <int AXIS>
struct VarStep {
    uint4v w[4];                 // this lane's 32 inputs of its W_b row
    uint4v x[4];                 // ... of its token (lane % 16 = request)
    uint4v vc[AXIS != 0 ? 4 : 1];   // ... of its request's column scales (column mode)
};

constexpr int kVarRowWords = 36;     // LDS stride of a staged sign row: 32 words + 4 (conflict-free reads)

// XDT: dtype of X and W_b.  AXIS as in the single-variant kernels, or 2: each request brings its
// own axis (variants[r].axis); the sign part then runs in fp16 with the operand fp16(x * v_r) for
// column-mode requests and fp16(x * 1) for row-mode ones.  NQ = 4, 8 or 16 request slots (R <= NQ).
//
// Sign traffic.  A 128-byte line of a sign row covers 1024 inputs = 8 steps, and with R sign
// matrices streaming next to W_b no line survives in the 32 KB L1 from one step to the next:
// loading the sign words step by step fetched every line 8 times (measured: 285 MB through L2 for
// 67 MB of operands at R = 16).  So the workgroup moves in strides of 1024 inputs: all waves copy
// the stride's sign lines (R x 16 rows x 128 B, each fetched exactly once, coalesced) to LDS, one
// stride ahead (two LDS buffers, one barrier per stride), and wave w computes step w of the stride,
// reading its R sign words from LDS.
template <int XDT, int AXIS, int NQ>
__global__ void __launch_bounds__(512, 2)
linear_variants_kernel(const uint16_t* __restrict__ X, const uint16_t* __restrict__ W_b,
                       const pdelta_variant* __restrict__ variants, int R, void* __restrict__ Y,
                       int d_out, int d_in, int y_dtype)
{
    constexpr int SDT = AXIS == 0 ? XDT : kF16;       // dtype of the sign-part operands
    constexpr int kUnits = NQ * 16 * 8 / 512;         // 16-byte units of a stride's sign block per thread
    __shared__ float red_b[8][16][16];                                       // [k-wave][token][row]
    __shared__ float red_s[8][NQ][16];                                       // [k-wave][request][row]
    __shared__ __attribute__((aligned(16))) uint32_t s_sign[2][NQ * 16 * kVarRowWords];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int kw = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = lane & 15, g = lane >> 4;
    const int n0 = blockIdx.x * 16;
    const int o = min(n0 + n, d_out - 1);
    const int K = d_in, wpr = K >> 5;

    // operands: this lane's W_b row, its request's X row and (column mode) scale row; requests
    // past R repeat the last real one (their results are never stored)
    const int req = min(n, R - 1);
    const uint16_t* wrow = W_b + (int64_t)o * K + g * 32;
    const uint16_t* xrow = X + (int64_t)req * K + g * 32;
    // per-request axis: a row-mode request has no scale per input; its loads of "v" read its own
    // X row instead (valid memory of the right length) and the value is replaced by 1.0
    const bool col = AXIS == 1 || (AXIS == 2 && variants[req].axis == PDELTA_COL);
    const uint16_t* vrow = AXIS == 0 ? nullptr : (col ? as_global_per_lane(variants[req].v) + g * 32 : xrow);

    // staging of sign lines: unit u = tid + 512 i of a stride's block is request u / 128 (uniform
    // in a wave), row (u % 128) / 8, 16-byte piece u % 8 of the row's 128 bytes
    const uint32_t* stage_src[kUnits];
    int stage_dst[kUnits];
    const int s_row = (tid & 127) >> 3, s_piece = tid & 7;
#pragma unroll
    for (int i = 0; i < kUnits; ++i) {
        const int q = (kw >> 1) + 4 * i;              // wave-uniform
        stage_src[i] = as_global(variants[min(q, R - 1)].B_packed) + (int64_t)min(n0 + s_row, d_out - 1) * wpr;
        stage_dst[i] = (q * 16 + s_row) * kVarRowWords + s_piece * 4;
    }
    auto stage_load = [&](uint4v (&t)[kUnits], int stride) {
        // pieces past the end of the row (last stride of a d_in that is not a multiple of 1024)
        // re-read the row's last 16 bytes; the steps that would use them do not exist
        const int word = min(stride * 32 + s_piece * 4, wpr - 4);
#pragma unroll
        for (int i = 0; i < kUnits; ++i) t[i] = *(const uint4v*)(stage_src[i] + word);
    };
    auto stage_store = [&](const uint4v (&t)[kUnits], int buf) {
#pragma unroll
        for (int i = 0; i < kUnits; ++i) *(uint4v*)(&s_sign[buf][stage_dst[i]]) = t[i];
    };

    auto load = [&](VarStep<AXIS>& S, int kb) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            S.w[i] = *(const uint4v*)(wrow + kb + i * 8);
            S.x[i] = *(const uint4v*)(xrow + kb + i * 8);
            if constexpr (AXIS != 0) S.vc[i] = *(const uint4v*)(vrow + kb + i * 8);
        }
    };

    uint32_t sign_bits = 0x80008000u, one2 = SDT == kBF16 ? 0x3F803F80u : 0x3C003C00u;
    asm volatile("" : "+v"(sign_bits), "+v"(one2));   // keep them in vector registers (see var_sign_operand)

    float4v accb = {0.f, 0.f, 0.f, 0.f};
    float4v acc[NQ];
#pragma unroll
    for (int q = 0; q < NQ; ++q) acc[q] = (float4v){0.f, 0.f, 0.f, 0.f};

    // this lane's sign word of step kw of the staged stride, request q
    const int my_word = n * kVarRowWords + 4 * kw + g;
    auto compute = [&](const VarStep<AXIS>& S, int buf) {
        uint32_t minus[NQ];
#pragma unroll
        for (int q = 0; q < NQ; ++q) minus[q] = ~s_sign[buf][q * 16 * kVarRowWords + my_word];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint4v xa = var_block_operand(S.x, j);
            accb = var_mfma<XDT>(xa, var_block_operand(S.w, j), accb);
            uint4v xs = xa;
            if constexpr (AXIS != 0) {                // fp16(x * v_r); a row-mode request: fp16(x * 1.0)
                const uint4v va = var_block_operand(S.vc, j);
#pragma unroll
                for (int p = 0; p < 4; ++p) {
                    const uint32_t vp = col ? (uint32_t)va[p] : 0x3C003C00u;
                    if constexpr (XDT == kF16) {
                        const uint32_t xp = xa[p];
                        xs[p] = as_u32(as_half2(xp) * as_half2(vp));
                    } else {
                        const float lo = bf16_bits_to_f32(xa[p] & 0xFFFFu) * f16_bits_to_f32(vp & 0xFFFFu);
                        const float hi = bf16_bits_to_f32(xa[p] >> 16) * f16_bits_to_f32(vp >> 16);
                        xs[p] = f32_to_f16_bits(lo) | (f32_to_f16_bits(hi) << 16);
                    }
                }
            }
            // four requests at a time: left alone the compiler forms the operands of all requests
            // first and runs out of registers
#pragma unroll
            for (int q = 0; q < NQ; ++q) {
                if ((q & 3) == 0) __builtin_amdgcn_sched_barrier(0);
                acc[q] = var_mfma<SDT>(xs, var_sign_operand(minus[q], j, sign_bits, one2), acc[q]);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // Stride h = inputs 1024 h .. + 1023; wave kw computes step 8 h + kw.  The sign block and the
    // W_b / X step of stride h + 1 are loaded (into registers) while stride h is computed.
    const int nsteps = K >> 7;
    const int nstrides = (nsteps + 7) >> 3;
    uint4v staged[kUnits];
    VarStep<AXIS> A, B;                               // strides alternate between them (no indexing: registers)
    stage_load(staged, 0);
    load(A, min(kw, nsteps - 1) << 7);
    auto stride = [&](const VarStep<AXIS>& cur, VarStep<AXIS>& nxt, int h) {
        const int buf = h & 1;
        stage_store(staged, buf);
        __syncthreads();                              // block h complete; block h - 1 (other buffer) no longer read
        const int hn = min(h + 1, nstrides - 1);      // clamped: loads stay unconditional
        stage_load(staged, hn);
        load(nxt, min(8 * hn + kw, nsteps - 1) << 7);
        if (8 * h + kw < nsteps) compute(cur, buf);
    };
    for (int h = 0; h < nstrides; h += 2) {
        stride(A, B, h);
        if (h + 1 >= nstrides) break;
        stride(B, A, h + 1);
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
            if (AXIS == 0 || (AXIS == 2 && variants[t].axis == PDELTA_ROW))
                scale = f16_bits_to_f32(as_global_per_lane(variants[t].v)[oo]);
            const float sum = base + scale * delta;
            const int64_t yi = (int64_t)t * d_out + oo;
            if (y_dtype == kF32) store_y<kF32>(Y, yi, sum);
            else if (y_dtype == kBF16) store_y<kBF16>(Y, yi, sum);
            else store_y<kF16>(Y, yi, sum);
        }
    }
}

// ---- slab kernel: whole sign slabs in LDS, +-1 operands from a 16-entry table -------------------
// Same work split, with the 128-input steps in the order (block j, group g) -> inputs 32 j + 8 g .. + 7;
// the sign slabs of all requests for the workgroup's 16 rows (contiguous in each B_packed) are
// copied to LDS first with coalesced loads that are all in flight together, and the sign bits turn
// into +-1 operands through a 16-entry table in LDS (two conflict-free 8-byte reads per sign byte),
// the reads of the next input block issued before the MFMAs of the current one.

struct SlabStep {
    uint4v w[4];                 // W_b operand per 32-input block (group 0 only uses it)
    uint4v x[4];                 // A operand: lane % 16 = request
    uint4v vc[4];                // v_r slice of this lane's request (column mode)
};

// XDT: dtype of X and W_b.  AXIS as in the single-variant kernels, or 2: each request brings its
// own axis (variants[r].axis); the sign part then runs in fp16 with the operand fp16(x * v_r) for
// column-mode requests and fp16(x * 1) for row-mode ones.  NQ = 8 or 16 request slots
// (R <= NQ).
template <int XDT, int AXIS, int NQ>
__global__ void __launch_bounds__(512, 2)
linear_variants_slab_kernel(const uint16_t* __restrict__ X, const uint16_t* __restrict__ W_b,
                       const pdelta_variant* __restrict__ variants, int R, void* __restrict__ Y,
                       int d_out, int d_in, int y_dtype)
{
    constexpr int SDT = AXIS == 0 ? XDT : kF16;       // dtype of the sign-part operands
    __shared__ __attribute__((aligned(16))) uint32_t lut4[16 * 2];          // nibble -> four +-1.0
    __shared__ float red_b[8][16][16];                                       // [k-wave][token][row]
    __shared__ float red_s[8][NQ][16];                                       // [k-wave][request][row]
    extern __shared__ __attribute__((aligned(16))) uint32_t s_sign[];        // [slot][16][spr]

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
    const uint32_t* brow[NQ];                         // this lane's sign row per request
    const int spr = wpr + 4;                          // LDS row stride in words
#pragma unroll
    for (int q = 0; q < NQ; ++q) {
        const int r = min(q, R - 1);
        brow[q] = s_sign + (r * 16 + n) * spr;
    }

    auto load = [&](SlabStep& S, int kb) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            S.w[j] = *(const uint4v*)(wrow + kb + j * 32);
            S.x[j] = *(const uint4v*)(xrow + kb + j * 32);
            if constexpr (AXIS != 0) S.vc[j] = *(const uint4v*)(vrow + kb + j * 32);
        }
    };

    float4v accb = {0.f, 0.f, 0.f, 0.f};
    float4v acc[NQ];
#pragma unroll
    for (int q = 0; q < NQ; ++q) acc[q] = (float4v){0.f, 0.f, 0.f, 0.f};

    // One step.  Requests go in halves of 8; within a half the table reads of input block j+1 are
    // issued before the 8 MFMAs of block j, so that the LDS latency hides behind the matrix
    // instructions (left alone the compiler issues read, wait, MFMA one at a time).
    auto compute = [&](const SlabStep& S, int kb) {
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
                sw[q] = *(const uint4v*)(brow[h * HQ + q] + (kb >> 5));
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

    // Every request's sign slab of these 16 rows (contiguous in its B_packed) goes to LDS
    // with coalesced 16-byte loads, all in flight at once, behind the first W_b / X loads
    SlabStep A, B;
    const int nsteps = K >> 7;
    if (kw < nsteps) load(A, kw << 7);
    {
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

constexpr size_t kVarStageBytes = 136 * 1024;    // LDS for whole sign slabs, next to 24 KB of tables

template <int XDT, int AXIS, int NQ>
static int launch_variants_slab(const void* X, const void* W_b, const pdelta_variant* variants_device, int R,
                                void* Y, int64_t d_out, int64_t d_in, int y_dtype, hipStream_t stream)
{
    const size_t lds = (size_t)R * 16 * (d_in / 8 + 16);
    auto kernel = linear_variants_slab_kernel<XDT, AXIS, NQ>;
    static unsigned lds_opted_in = 0;                 // per template instance: one kernel
    if (lds > 32 * 1024 && opt_in_dynamic_lds((const void*)kernel, (int)kVarStageBytes, &lds_opted_in) != 0)
        return -1;
    hipLaunchKernelGGL(kernel, dim3((unsigned)((d_out + 15) / 16)), dim3(512), lds, stream, (const uint16_t*)X,
                       (const uint16_t*)W_b, variants_device, R, Y, (int)d_out, (int)d_in, y_dtype);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

template <int XDT, int AXIS, int NQ>
static int launch_variants_stride(const void* X, const void* W_b, const pdelta_variant* variants_device, int R,
                                  void* Y, int64_t d_out, int64_t d_in, int y_dtype, hipStream_t stream)
{
    hipLaunchKernelGGL((linear_variants_kernel<XDT, AXIS, NQ>), dim3((unsigned)((d_out + 15) / 16)), dim3(512), 0,
                       stream, (const uint16_t*)X, (const uint16_t*)W_b, variants_device, R, Y, (int)d_out,
                       (int)d_in, y_dtype);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

// Requests go in chunks of up to 16 that share one pass over W_b.  Two kernels (measured on
// MI355X, fp16, R = 4 / 8 / 16): when the whole sign slabs of a chunk (16 rows x d_in / 8 bytes per
// request) fit in LDS the slab kernel is 4-15 % faster (4096 x 4096: 11.2 / 14.3 / 25.1 us against
// 13.2 / 15.7 / 26.1); when they do not (d_in = 11008 from 7 requests on) the stride kernel, which
// needs 90 KB of LDS whatever d_in, does them in one pass (16 requests: 62 us against 81 us in
// three passes).
template <int XDT, int AXIS>
static int launch_variants(const void* X, const void* W_b, const pdelta_variant* variants_device, int R,
                           void* Y, int64_t d_out, int64_t d_in, int y_dtype, hipStream_t stream)
{
    const size_t per_request = (size_t)16 * (d_in / 8 + 16);
    const int which = tune_value("var_kernel", 0);    // 0: by size, 1: slab kernel when it can, 2: stride kernel
    const size_t ysz = y_dtype == kF32 ? 4 : 2;
    for (int r0 = 0; r0 < R; r0 += kVarMaxR) {
        const int n = R - r0 < kVarMaxR ? R - r0 : kVarMaxR;
        const void* Xc = (const char*)X + (size_t)r0 * d_in * 2;
        void* Yc = (char*)Y + (size_t)r0 * d_out * ysz;
        const pdelta_variant* vc = variants_device + r0;
        const bool slab = which != 2 && per_request * (size_t)n <= kVarStageBytes;
        int rc;
#define PDELTA_VAR_GO(FN)                                                                        \
        if (n <= 4) rc = FN<XDT, AXIS, 4>(Xc, W_b, vc, n, Yc, d_out, d_in, y_dtype, stream);      \
        else if (n <= 8) rc = FN<XDT, AXIS, 8>(Xc, W_b, vc, n, Yc, d_out, d_in, y_dtype, stream); \
        else rc = FN<XDT, AXIS, 16>(Xc, W_b, vc, n, Yc, d_out, d_in, y_dtype, stream)
        if (slab) { PDELTA_VAR_GO(launch_variants_slab); }
        else { PDELTA_VAR_GO(launch_variants_stride); }
#undef PDELTA_VAR_GO
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
