// pdelta_pack: B = sign(W_f - W_b) bit-packed along the input axis, plus the per-axis
// mean |W_f - W_b| that initialises the scale vectors (paper Section 2; per-layer compression
// algorithm: the packing step and the initial values of the Row and Col scale vectors).
//
// One streaming pass over both matrices (4 B read, 1/8 B written per weight): HBM-bound.
//   pack_main_kernel      signs -> words; |dW| -> one partial sum per (row, column tile) and
//                         per (row tile, column), written with plain stores to the workspace
//   pack_finalize_kernel  adds the partials of each row / column, divides by the count and
//                         rounds once to fp16
// No atomics and nothing to clear beforehand: every workspace slot that is read has been
// written by exactly one workgroup, and the partials are added in a fixed order, so the result
// is bit-reproducible for both dtypes.
//
// Exact sums.  fp16 values are integer multiples of 2^-24 below 2^16, so W_f - W_b is exact in
// fp64 and every |dW| * 2^24 is an integer below 2^41.  A workgroup adds at most 1024 of them
// per row and 512 per column in fp64 (below 2^51 units: still exact).  The finalize kernel
// converts each partial to uint64 units of 2^-24 and adds integers.  bf16 has no such grid; its
// partials are added in fp64 and are exact only while fp64 holds them exactly.
#include <type_traits>

#include "pdelta_device.h"
#include "pdelta_host.h"

namespace pdelta {

constexpr int kPackChunk = kWave * 8;                        // 512 columns: one 16-byte load per lane
constexpr int kPackChunks = 2;
constexpr int kPackTileCols = kPackChunk * kPackChunks;      // 1024: 128 B of sign bits per row
constexpr int kPackTileRows = 64;                            // smallest tile height: bounds the workspace
constexpr int kPackSignWords = kPackTileCols / 32;           // 32 words per tile row
// Measured on MI355X (fp16, 7B-shaped layers): the rate of this kernel does not depend on how far
// ahead a wave loads (1, 2 or 4 rows: 4.4-4.8, 4.3-4.8, 3.7-3.9 TB/s, the last at 3 waves per SIMD),
// on the tile width (512 or 1024 columns at 4-7 waves per SIMD), on the tile height (64 to 512
// rows) or on the arithmetic (with the sums and compares taken out it streams at the same
// 4.5 TB/s; the vector ALUs are 36-42 % busy).  Two rows ahead at 4 waves per SIMD it is.
constexpr int kPackAhead = 2;                                // rows in flight per wave
constexpr int kPackOcc = 4;                                  // waves per SIMD the registers allow
constexpr int kPackBatchWaves = 4;                           // waves per workgroup of the batched kernel

static inline int64_t pack_row_tiles(int64_t d_out) { return (d_out + kPackTileRows - 1) / kPackTileRows; }
static inline int64_t pack_col_tiles(int64_t d_in) { return (d_in + kPackTileCols - 1) / kPackTileCols; }

size_t pack_workspace_bytes(int64_t d_out, int64_t d_in)
{
    // row partials [column tiles][d_out], then column partials [row tiles][d_in], fp64
    return (size_t)(pack_col_tiles(d_in) * d_out + pack_row_tiles(d_out) * d_in) * sizeof(double);
}

// acc * 2 + (a < b): the compare leaves its result in the carry input of the add.
__device__ __forceinline__ uint32_t shift_in_less(uint32_t acc, float a, float b)
{
    asm("v_cmp_lt_f32 vcc, %1, %2\n\tv_addc_co_u32 %0, vcc, %0, %0, vcc" : "+v"(acc) : "v"(a), "v"(b) : "vcc");
    return acc;
}

struct PackRow {          // both matrices' 16 bytes per lane for the two chunks of one row
    uint4v a[kPackChunks], b[kPackChunks];
};

// Work of one workgroup of WAVES waves: a tile of WAVES * 8 * blocks rows x 1024 columns.
// Wave w owns 8 * blocks consecutive rows and walks them in blocks of 8; lane l owns columns
// chunk*512 + 8l .. 8l+7 of each chunk: one 16-byte load per matrix, one sign byte.  Loads are
// unconditional, two rows ahead of the arithmetic, across block boundaries.  After each block
// the wave writes its 8 x 128 bytes of sign words and its 8 row sums; column sums stay in
// registers until the end of the tile, where the waves meet once in LDS.
template <int DT, int WAVES>
__device__ __forceinline__ void
pack_tile(const uint16_t* __restrict__ W_f, const uint16_t* __restrict__ W_b, int d_out, int d_in,
          uint32_t* __restrict__ B_packed,
          double* __restrict__ row_part,      // [column tiles][d_out] or nullptr
          double* __restrict__ col_part,      // [row tiles][d_in]     or nullptr
          int row_tile, int col_tile, int blocks)
{
    __shared__ double s_col[WAVES][kPackChunks * 8][kWave + 1];
    __shared__ __attribute__((aligned(16))) uint32_t s_sign[WAVES][8][kPackSignWords];

    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);               // scalar: row indices stay uniform
    const int col0 = col_tile * kPackTileCols;
    const int wave_rows = 8 * blocks;
    const int row0 = (row_tile * WAVES + wave) * wave_rows;                     // first row of this wave

    // A lane whose columns lie beyond d_in, and every lane of a row beyond d_out, reads a clamped
    // address of W_b for BOTH operands: its differences are exactly zero, so it adds nothing to
    // the sums, and its own column sums and sign bytes are never stored.  This keeps the loop
    // free of branches around loads, which would make the compiler drain the loads in flight.
    const uint16_t* lane_f[kPackChunks];
    const uint16_t* lane_b[kPackChunks];
#pragma unroll
    for (int c = 0; c < kPackChunks; ++c) {
        const int col = col0 + c * kPackChunk + lane * 8;
        lane_b[c] = W_b + min(col, d_in - 8);                                   // d_in % 8 == 0
        lane_f[c] = col < d_in ? W_f + col : lane_b[c];
    }
    auto load = [&](PackRow& R, int row) {
        const bool row_live = row < d_out;
        const int64_t base = (int64_t)min(row, d_out - 1) * d_in;
#pragma unroll
        for (int c = 0; c < kPackChunks; ++c) {
            R.a[c] = *(const uint4v*)((row_live ? lane_f[c] : lane_b[c]) + base);
            R.b[c] = *(const uint4v*)(lane_b[c] + base);
        }
    };

    double csum[kPackChunks][8];
#pragma unroll
    for (int c = 0; c < kPackChunks; ++c)
#pragma unroll
        for (int e = 0; e < 8; ++e) csum[c][e] = 0.0;

    unsigned char* sign_bytes = (unsigned char*)&s_sign[wave][0][0];
    // Until the column sums are handed over, this wave's slice of s_col holds the row sums of
    // the current block: [8 rows][64 lanes], one fp64 per lane and row.
    double* s_row = &s_col[wave][0][0];
    auto compute = [&](PackRow& R, int r) {
        double rsum = 0.0;
#pragma unroll
        for (int c = 0; c < kPackChunks; ++c) {
            const uint4v a = R.a[c], b = R.b[c];
            // "W_f < W_b" is shifted into `neg`, entry 7 first so that entry e ends up in bit e
            // (a compare, not the sign bit of the difference: (-0) - (+0) is -0 but not "less")
            uint32_t neg = 0;
#pragma unroll
            for (int e = 7; e >= 0; --e) {
                const uint32_t ha = (a[e >> 1] >> ((e & 1) * 16)) & 0xFFFFu;
                const uint32_t hb = (b[e >> 1] >> ((e & 1) * 16)) & 0xFFFFu;
                const float fa = bits_to_f32<DT>(ha), fb = bits_to_f32<DT>(hb);
                neg = shift_in_less(neg, fa, fb);
                const double d = fabs((double)fa - (double)fb);                 // exact for fp16
                rsum += d;
                csum[c][e] += d;
                if (e & 1) __builtin_amdgcn_sched_barrier(0);
            }
            const uint32_t byte = ~neg;
            sign_bytes[r * (kPackSignWords * 4) + c * kWave + lane] = (unsigned char)byte;
            __builtin_amdgcn_sched_barrier(0);
        }
        s_row[r * kWave + lane] = rsum;
    };

    // The slices are private to the wave and LDS operations of one wave complete in order; the
    // fences only stop the compiler from moving accesses across them.
    auto wave_sync = [] {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    };
    // After a block: lane l adds the row sums of lanes 8 (l % 8) .. + 7 for row l / 8 and three
    // exchanges finish the row (fp64 adds stay exact for fp16, see above); the same lane writes
    // the 16-byte piece l % 8 of that row's 128 bytes of sign words: whole lines per row.
    const bool rows_aligned = (d_in & 127) == 0;
    auto flush = [&](int first_row) {
        // pin the column sums here: with their next use behind the branches below, the compiler
        // would otherwise sink the block's column arithmetic past them and keep (spill) every
        // difference until then
#pragma unroll
        for (int c = 0; c < kPackChunks; ++c)
#pragma unroll
            for (int e = 0; e < 8; ++e) asm volatile("" : "+v"(csum[c][e]));
        wave_sync();
        const double* src = s_row + (lane >> 3) * kWave + (lane & 7) * 8;
        double t = src[0];
#pragma unroll
        for (int k = 1; k < 8; ++k) t += src[k];
        t += __shfl_xor(t, 4, kWave);
        t += __shfl_xor(t, 2, kWave);
        t += __shfl_xor(t, 1, kWave);
        const int r = lane >> 3, piece = lane & 7;
        constexpr int kPieces = kPackSignWords / 4;                  // 16-byte pieces of sign words per tile row
        const uint4v words = *(const uint4v*)&s_sign[wave][r][min(piece, kPieces - 1) * 4];
        wave_sync();
        const int row = first_row + r;
        const int colp = col0 + piece * 128;
        if (row < d_out) {
            if (row_part != nullptr && piece == 0) row_part[(int64_t)col_tile * d_out + row] = t;
            if (piece < kPieces && colp < d_in) {
                uint32_t* dst = B_packed + (int64_t)row * (d_in >> 5) + (colp >> 5);
                if (rows_aligned) {
                    *(uint4v*)dst = words;
                } else {                             // rows are not 16-byte aligned, or a ragged end
#pragma unroll
                    for (int w = 0; w < 4; ++w)
                        if (colp + w * 32 < d_in) dst[w] = words[w];
                }
            }
        }
    };

    // two rows in flight; the scheduling fences keep the compiler from interleaving the
    // arithmetic of different rows (which costs registers and gains nothing: HBM-bound)
    PackRow buf[kPackAhead];
#pragma unroll
    for (int a = 0; a < kPackAhead; ++a) load(buf[a], row0 + a);
    __builtin_amdgcn_sched_barrier(0);
    int row = row0;
    for (int blk = 0; blk + 1 < blocks; ++blk, row += 8) {
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            compute(buf[r % kPackAhead], r);
            load(buf[r % kPackAhead], row + r + kPackAhead);
            __builtin_amdgcn_sched_barrier(0);
        }
        flush(row);
    }
#pragma unroll
    for (int r = 0; r < 8; ++r) {                    // last block: nothing left to load near its end
        compute(buf[r % kPackAhead], r);
        if (r < 8 - kPackAhead) load(buf[r % kPackAhead], row + r + kPackAhead);
        __builtin_amdgcn_sched_barrier(0);
    }
    flush(row);

    // hand the column sums over
#pragma unroll
    for (int c = 0; c < kPackChunks; ++c)
#pragma unroll
        for (int e = 0; e < 8; ++e) s_col[wave][c * 8 + e][lane] = csum[c][e];
    __syncthreads();
    if (col_part != nullptr) {
        for (int j = tid; j < kPackTileCols; j += WAVES * kWave) {
            const int col = col0 + j;
            const int c = j / kPackChunk, l = (j % kPackChunk) >> 3, e = j & 7;
            double s = s_col[0][c * 8 + e][l];
#pragma unroll
            for (int w = 1; w < WAVES; ++w) s += s_col[w][c * 8 + e][l];
            if (col < d_in) col_part[(int64_t)row_tile * d_in + col] = s;
        }
    }
}

template <int DT, int WAVES>
__global__ void __launch_bounds__(WAVES * kWave, kPackOcc)
pack_main_kernel(const uint16_t* __restrict__ W_f, const uint16_t* __restrict__ W_b,
                 int d_out, int d_in, uint32_t* __restrict__ B_packed,
                 double* __restrict__ row_part, double* __restrict__ col_part, int blocks,
                 int n_col_tiles)
{
    // consecutive workgroups take the column tiles of one row tile: rows are read end to end
    const int id = (int)blockIdx.x;
    pack_tile<DT, WAVES>(W_f, W_b, d_out, d_in, B_packed, row_part, col_part, id / n_col_tiles,
                         id % n_col_tiles, blocks);
}

// Many layers in one launch: workgroup b works on the last job whose first_tile is <= b.
template <int DT>
__global__ void __launch_bounds__(kPackBatchWaves * kWave, kPackOcc)
pack_main_batch_kernel(const pdelta_pack_job* __restrict__ jobs, int n_jobs)
{
    const int b = (int)blockIdx.x;
    int lo = 0, hi = n_jobs - 1;
    while (lo < hi) {                                 // workgroup-uniform
        const int mid = (lo + hi + 1) >> 1;
        if (jobs[mid].first_tile <= b) lo = mid; else hi = mid - 1;
    }
    const pdelta_pack_job J = jobs[lo];
    const int id = b - J.first_tile;
    const int d_out = (int)J.d_out, d_in = (int)J.d_in;
    const int n_ct = (d_in + kPackTileCols - 1) / kPackTileCols;
    double* row_part = as_global((double*)J.workspace);
    double* col_part = row_part + (int64_t)n_ct * d_out;
    pack_tile<DT, kPackBatchWaves>(as_global((const uint16_t*)J.W_f), as_global((const uint16_t*)J.W_b), d_out, d_in,
                     as_global(J.B_packed),
                     J.v_row ? row_part : (double*)nullptr, J.v_col ? col_part : (double*)nullptr,
                     id / n_ct, id % n_ct, J.tile_blocks);
}

// 64 rows or columns per workgroup; 16 groups of threads share the partials of one of them
// (four loads in flight each) and meet in LDS, always in the same order.
constexpr int kFinGroups = 16;

template <int DT>
__device__ __forceinline__ void
pack_finalize_block(const double* __restrict__ row_part, const double* __restrict__ col_part,
                    int n_col_tiles, int n_row_tiles, int d_out, int d_in,
                    uint16_t* __restrict__ v_row, uint16_t* __restrict__ v_col, int block)
{
    typedef typename std::conditional<DT == kF16, unsigned long long, double>::type acc_t;
    __shared__ acc_t part[kFinGroups][64];
    const int x = threadIdx.x & 63, g = threadIdx.x >> 6;
    const int row_blocks = (d_out + 63) / 64;
    const bool is_row = block < row_blocks;                                     // workgroup-uniform
    const int n = is_row ? d_out : d_in;
    const int n_part = is_row ? n_col_tiles : n_row_tiles;
    const double* src = is_row ? row_part : col_part;
    uint16_t* dst = is_row ? v_row : v_col;
    if (dst == nullptr) return;                                                 // workgroup-uniform
    const int idx = (block - (is_row ? 0 : row_blocks)) * 64 + x;
    const int idc = min(idx, n - 1);                                            // clamped: loads unconditional
    auto units = [](double v) -> acc_t {
        if constexpr (DT == kF16) return (unsigned long long)(v * 16777216.0);  // units of 2^-24
        else return v;
    };
    acc_t s = 0;
    int p = g;
    for (; p + 3 * kFinGroups < n_part; p += 4 * kFinGroups) {
        const double v0 = src[(int64_t)p * n + idc];
        const double v1 = src[(int64_t)(p + kFinGroups) * n + idc];
        const double v2 = src[(int64_t)(p + 2 * kFinGroups) * n + idc];
        const double v3 = src[(int64_t)(p + 3 * kFinGroups) * n + idc];
        s += units(v0);
        s += units(v1);
        s += units(v2);
        s += units(v3);
    }
    for (; p < n_part; p += kFinGroups) s += units(src[(int64_t)p * n + idc]);
    part[g][x] = s;
    __syncthreads();
    if (g == 0 && idx < n) {
#pragma unroll
        for (int k = 1; k < kFinGroups; ++k) s += part[k][x];
        const double total = DT == kF16 ? (double)s * (1.0 / 16777216.0) : (double)s;
        const double count = is_row ? (double)d_in : (double)d_out;
        dst[idx] = (uint16_t)f64_to_f16_bits_rne(total / count);
    }
}

template <int DT>
__global__ void __launch_bounds__(64 * kFinGroups)
pack_finalize_kernel(const double* __restrict__ row_part, const double* __restrict__ col_part,
                     int n_col_tiles, int n_row_tiles, int d_out, int d_in,
                     uint16_t* __restrict__ v_row, uint16_t* __restrict__ v_col)
{
    pack_finalize_block<DT>(row_part, col_part, n_col_tiles, n_row_tiles, d_out, d_in, v_row, v_col,
                            (int)blockIdx.x);
}

template <int DT>
__global__ void __launch_bounds__(64 * kFinGroups)
pack_finalize_batch_kernel(const pdelta_pack_job* __restrict__ jobs, int n_jobs)
{
    const int b = (int)blockIdx.x;
    int lo = 0, hi = n_jobs - 1;
    while (lo < hi) {                                 // workgroup-uniform
        const int mid = (lo + hi + 1) >> 1;
        if (jobs[mid].first_fin_block <= b) lo = mid; else hi = mid - 1;
    }
    const pdelta_pack_job J = jobs[lo];
    const int d_out = (int)J.d_out, d_in = (int)J.d_in;
    const int n_ct = (d_in + kPackTileCols - 1) / kPackTileCols;
    const int tile_rows = kPackBatchWaves * 8 * J.tile_blocks;
    const int n_rt = (d_out + tile_rows - 1) / tile_rows;
    const double* row_part = as_global((const double*)J.workspace);
    const double* col_part = row_part + (int64_t)n_ct * d_out;
    pack_finalize_block<DT>(row_part, col_part, n_ct, n_rt, d_out, d_in, as_global(J.v_row), as_global(J.v_col),
                            b - J.first_fin_block);
}

template <int DT>
static int launch_pack(const void* W_f, const void* W_b, int64_t d_out, int64_t d_in,
                       uint32_t* B_packed, uint16_t* v_row, uint16_t* v_col, void* workspace,
                       hipStream_t stream)
{
    // Tile height: 8 rows per wave and block.  Small layers take 8 waves x 1 block (64 rows, the
    // most workgroups); larger ones 4 waves and as many blocks as still leave >= 8 workgroups
    // per CU, up to 256-row tiles (fewer column partials, fewer pipeline refills).
    const int64_t n_ct = pack_col_tiles(d_in);
    int waves = 8, blocks = 1;
    if (pack_row_tiles(d_out) * n_ct >= 2 * 2048) {
        waves = 4;
        blocks = 2;
        while (blocks < 8 && ((d_out + 32 * blocks * 2 - 1) / (32 * blocks * 2)) * n_ct >= 2048) blocks *= 2;
    }
    waves = tune_value("pack_waves", waves);
    blocks = tune_value("pack_blocks", blocks);
    if (waves != 4) waves = 8;
    if (blocks < 1 || waves * 8 * blocks < kPackTileRows) blocks = kPackTileRows / (waves * 8);   // >= 64-row tiles
    const int tile_rows = waves * 8 * blocks;
    const int64_t n_rt = (d_out + tile_rows - 1) / tile_rows;
    double* row_part = (double*)workspace;
    double* col_part = row_part + n_ct * d_out;
    const bool want_any = v_row != nullptr || v_col != nullptr;
    auto main_kernel = waves == 4 ? pack_main_kernel<DT, 4> : pack_main_kernel<DT, 8>;
    hipLaunchKernelGGL(main_kernel, dim3((unsigned)(n_rt * n_ct)), dim3(waves * kWave), 0,
                       stream, (const uint16_t*)W_f, (const uint16_t*)W_b, (int)d_out, (int)d_in, B_packed,
                       v_row ? row_part : (double*)nullptr, v_col ? col_part : (double*)nullptr, blocks,
                       (int)n_ct);
    if (want_any) {
        const unsigned blocks = (unsigned)((d_out + 63) / 64 + (d_in + 63) / 64);
        hipLaunchKernelGGL(pack_finalize_kernel<DT>, dim3(blocks), dim3(64 * kFinGroups), 0, stream,
                           (const double*)row_part, (const double*)col_part, (int)n_ct, (int)n_rt,
                           (int)d_out, (int)d_in, v_row, v_col);
    }
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

// Tiles of a job in the batched kernels: 4 waves x tile_blocks blocks of 8 rows, 1024 columns
// (512-row tiles for tall layers: fewest column partials, measured 5 % faster than 128 rows).
int pack_batch_tile_blocks(int64_t d_out)
{
    const int blocks = tune_value("pack_batch_blocks", d_out >= 2048 ? 16 : (d_out >= 512 ? 4 : 2));
    const int least = kPackTileRows / (kPackBatchWaves * 8);        // 64-row tiles at least: the workspace is sized for them
    return blocks < least ? least : blocks;
}
int64_t pack_batch_tiles(int64_t d_out, int64_t d_in, int tile_blocks)
{
    const int64_t tile_rows = kPackBatchWaves * 8 * tile_blocks;
    return ((d_out + tile_rows - 1) / tile_rows) * pack_col_tiles(d_in);
}
int64_t pack_batch_fin_blocks(int64_t d_out, int64_t d_in) { return (d_out + 63) / 64 + (d_in + 63) / 64; }

int launch_pack_batch(int w_dtype, const pdelta_pack_job* jobs_host, const pdelta_pack_job* jobs_device,
                      int n_jobs, hipStream_t stream)
{
    const pdelta_pack_job& last = jobs_host[n_jobs - 1];
    const int64_t tiles = last.first_tile + pack_batch_tiles(last.d_out, last.d_in, last.tile_blocks);
    const int64_t fin = last.first_fin_block + pack_batch_fin_blocks(last.d_out, last.d_in);
    bool want_any = false;
    for (int j = 0; j < n_jobs; ++j) want_any = want_any || jobs_host[j].v_row || jobs_host[j].v_col;
    if (w_dtype == kBF16)
        hipLaunchKernelGGL(pack_main_batch_kernel<kBF16>, dim3((unsigned)tiles), dim3(kPackBatchWaves * kWave), 0, stream,
                           jobs_device, n_jobs);
    else
        hipLaunchKernelGGL(pack_main_batch_kernel<kF16>, dim3((unsigned)tiles), dim3(kPackBatchWaves * kWave), 0, stream,
                           jobs_device, n_jobs);
    if (want_any) {
        if (w_dtype == kBF16)
            hipLaunchKernelGGL(pack_finalize_batch_kernel<kBF16>, dim3((unsigned)fin), dim3(64 * kFinGroups), 0,
                               stream, jobs_device, n_jobs);
        else
            hipLaunchKernelGGL(pack_finalize_batch_kernel<kF16>, dim3((unsigned)fin), dim3(64 * kFinGroups), 0,
                               stream, jobs_device, n_jobs);
    }
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

// ---- scratch owned by the library, for callers that cannot allocate --------------------------
// pdelta_pack_noalloc runs the kernels above with their partial sums in this array instead of a
// caller's workspace.  Each GPU the library runs on holds its own copy at its own address until
// the process ends.  The name below is a host-side stand-in, not a device address: the address is
// asked for once per device (with that device current) and only that pointer is ever handed to
// a kernel.  Nothing has to be cleared between calls: every slot a finalize kernel reads has been
// written by the main kernel of the same call.
static __device__ __align__(256) unsigned char scratch[kPackScratchBytes];

int pack_static_scratch(void** ptr)
{
    constexpr int kMaxDevices = 64;
    static void* address_on_device[kMaxDevices] = {};
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return -1;
    void* p = __atomic_load_n(&address_on_device[dev], __ATOMIC_ACQUIRE);
    if (p == nullptr) {
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) {
            (void)hipGetLastError();
            return -1;
        }
        __atomic_store_n(&address_on_device[dev], p, __ATOMIC_RELEASE);
    }
    *ptr = p;
    return 0;
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
