// Host-side launch functions, one per kernel family.  Each returns 0 when every launch was
// accepted and -1 otherwise.  Arguments have been validated by the C-ABI layer (pdelta_api.hip).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "pdelta.h"

namespace pdelta {

// Bytes of fp64 partial sums pdelta_pack writes for these dimensions.
size_t pack_workspace_bytes(int64_t d_out, int64_t d_in);

int launch_pack_dispatch(int w_dtype, const void* W_f, const void* W_b, int64_t d_out,
                         int64_t d_in, uint32_t* B_packed, uint16_t* v_row, uint16_t* v_col,
                         void* workspace, hipStream_t stream);

// Device address of the library's own scratch array (kPackScratchBytes, one copy per GPU) on the
// current device; looked up once per device.  Returns 0, or -1 when the runtime refuses.
constexpr size_t kPackScratchBytes = (size_t)16 << 20;
int pack_static_scratch(void** ptr);

// Batched pack: geometry helpers shared by the plan (host) and the launcher.
int pack_batch_tile_blocks(int64_t d_out);
int64_t pack_batch_tiles(int64_t d_out, int64_t d_in, int tile_blocks);
int64_t pack_batch_fin_blocks(int64_t d_out, int64_t d_in);
int launch_pack_batch(int w_dtype, const ::pdelta_pack_job* jobs_host, const ::pdelta_pack_job* jobs_device,
                      int n_jobs, hipStream_t stream);

int launch_patch_batch(int w_dtype, const ::pdelta_layer* layers_host, const ::pdelta_layer* layers_device,
                       int n_layers, hipStream_t stream);

int launch_patch_dispatch(int w_dtype, int axis, const void* W_b, const uint32_t* B_packed,
                          const uint16_t* v, void* W_out, int64_t d_out, int64_t d_in,
                          hipStream_t stream);

// Decode-shaped layer (few tokens): HBM-bound streaming kernel.  M <= kSkinnyMaxM.
constexpr int kSkinnyMaxM = 64;
int launch_linear_skinny(int x_dtype, int y_dtype, int axis, const void* X, const void* W_b,
                         const uint32_t* B_packed, const uint16_t* v, void* Y, int64_t M,
                         int64_t d_out, int64_t d_in, hipStream_t stream);

// The same with blockwise scales v[row * v_stride + (input >> g_shift)] (v_stride = 0: the rows
// share the scales; g_shift = 31: one group spans all of d_in).
int launch_linear_skinny_group(int x_dtype, int y_dtype, const void* X, const void* W_b,
                               const uint32_t* B_packed, const uint16_t* v, void* Y, int64_t M,
                               int64_t d_out, int64_t d_in, int v_stride, int g_shift, hipStream_t stream);
int launch_linear_gemm_group(int x_dtype, int y_dtype, const void* X, const void* W_b,
                             const uint32_t* B_packed, const uint16_t* v, void* Y, int64_t M,
                             int64_t d_out, int64_t d_in, int v_stride, int g_shift, hipStream_t stream);
int launch_patch_group(int w_dtype, const void* W_b, const uint32_t* B_packed, const uint16_t* v,
                       void* W_out, int64_t d_out, int64_t d_in, int v_stride, int g_shift,
                       hipStream_t stream);
// pack with blockwise scales: signs + fp64 block sums (per row), then the scales; `workspace` is
// needed only when the rows share the scales (one partial sum per row and group).
size_t pack_group_workspace_bytes(int64_t d_out, int64_t d_in, int64_t group, int shared_rows);
int launch_pack_group(int w_dtype, const void* W_f, const void* W_b, int64_t d_out, int64_t d_in,
                      int64_t group, int shared_rows, uint32_t* B_packed, uint16_t* v, void* workspace,
                      hipStream_t stream);

// Several decode-shaped layers in one launch.  Returns 1 when the batched kernel does not apply
// (the caller then launches layer by layer), else 0 / -1.
int launch_linear_skinny_batch(int x_dtype, int y_dtype, const ::pdelta_layer* layers_host,
                               const ::pdelta_layer* layers_device, int n_layers, int64_t M,
                               hipStream_t stream);

// R requests (one token each) that share W_b and each have their own delta (more than 16 requests
// run in chunks of 16).  axis 0 / 1: one mode for all requests; 2: variants[r].axis per request.
// Returns 1 when the fused kernel does not apply (d_in % 128 != 0), else 0 / -1.
int launch_linear_variants(int x_dtype, int y_dtype, int axis, const void* X, const void* W_b,
                           const ::pdelta_variant* variants_device, int R, void* Y, int64_t d_out,
                           int64_t d_in, hipStream_t stream);

// dL/dv from dY (training of the scale vectors).  Workspace: partial sums per token tile, plus
// the transposed sign bits in column mode.
size_t grad_v_workspace_bytes(int64_t M, int64_t d_out, int64_t d_in, int axis);
int launch_grad_v(int dtype, int axis, const void* X, const void* dY, const uint32_t* B_packed, float* grad,
                  int64_t M, int64_t d_out, int64_t d_in, void* workspace, hipStream_t stream);

// Prefill-shaped layer (many tokens): MFMA tile kernel.
int launch_linear_gemm(int x_dtype, int y_dtype, int axis, const void* X, const void* W_b,
                       const uint32_t* B_packed, const uint16_t* v, void* Y, int64_t M,
                       int64_t d_out, int64_t d_in, hipStream_t stream);

// Measurement builds of the pipelined prefill kernel (bf16 operands, row scales): bit 0 of `parts`
// keeps the steady loop's global loads, bit 1 conversion and LDS writes, bit 2 fragment reads,
// bit 3 the MFMAs; 15 is the product kernel.  Returns -2 for a combination that is not built.
int launch_linear_gemm_parts(int parts, int y_dtype, const void* X, const void* W_b, const uint32_t* B_packed,
                             const uint16_t* v, void* Y, int64_t M, int64_t d_out, int64_t d_in,
                             hipStream_t stream);

// Integer tuning knobs from the environment variable PDELTA_TUNE ("key=value,key=value");
// returns `fallback` when the key is absent.  Every C-ABI entry point that launches opens a
// TuneScope, which reads the variable once for the whole call.
struct TuneScope {
    TuneScope();
    ~TuneScope();
    TuneScope(const TuneScope&) = delete;
    TuneScope& operator=(const TuneScope&) = delete;
};
int tune_value(const char* key, int fallback);

// Kernels that use more dynamic LDS than the default limit have to opt in once per device.
// `done_mask` is a static word of the call site (one bit per device): the attribute is set on
// the first launch on a device and never again.  Returns 0, or -1 when the runtime refuses.
int opt_in_dynamic_lds(const void* kernel, int bytes, unsigned* done_mask);

}  // namespace pdelta
