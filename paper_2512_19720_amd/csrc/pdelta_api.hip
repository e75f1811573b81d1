// C ABI of the pdelta library (see include/pdelta.h): argument validation on the host, then
// dispatch to the kernel families.  No allocation, no synchronisation, no state.
#include "pdelta.h"
#include "pdelta_probes.h"

#include <stdlib.h>
#include <string.h>

#include "pdelta_host.h"

namespace pdelta {

// PDELTA_TUNE is looked up in the environment once per C-ABI call (TuneScope, opened by every
// entry point that launches); inside the call the kernel selectors read the snapshot.  Without
// the variable a lookup costs one thread-local load.
namespace {
thread_local const char* t_tune_env = nullptr;
thread_local int t_tune_depth = 0;
}  // namespace

TuneScope::TuneScope()
{
    if (t_tune_depth++ == 0) t_tune_env = getenv("PDELTA_TUNE");
}
TuneScope::~TuneScope()
{
    if (--t_tune_depth == 0) t_tune_env = nullptr;
}

int tune_value(const char* key, int fallback)
{
    const char* env = t_tune_depth > 0 ? t_tune_env : getenv("PDELTA_TUNE");
    if (env == nullptr) return fallback;
    const size_t klen = strlen(key);
    for (const char* p = env; *p != '\0';) {
        if (strncmp(p, key, klen) == 0 && p[klen] == '=') return atoi(p + klen + 1);
        const char* comma = strchr(p, ',');
        if (comma == nullptr) break;
        p = comma + 1;
    }
    return fallback;
}

int opt_in_dynamic_lds(const void* kernel, int bytes, unsigned* done_mask)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return -1;
    const unsigned bit = 1u << (dev & 31);
    if (__atomic_load_n(done_mask, __ATOMIC_ACQUIRE) & bit) return 0;
    if (hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes) != hipSuccess) return -1;
    __atomic_fetch_or(done_mask, bit, __ATOMIC_RELEASE);
    return 0;
}

namespace {

constexpr int64_t kMaxDim = (int64_t)1 << 22;      // per-axis limit of pack's exact sums
constexpr int64_t kMaxTokens = (int64_t)1 << 23;

inline bool misaligned(const void* p) { return ((uintptr_t)p & 15u) != 0; }

// true when [a, a+na) and [b, b+nb) share a byte
inline bool overlaps(const void* a, size_t na, const void* b, size_t nb)
{
    const uintptr_t pa = (uintptr_t)a, pb = (uintptr_t)b;
    return pa < pb + nb && pb < pa + na;
}

inline bool is_w_dtype(int d) { return d == PDELTA_F16 || d == PDELTA_BF16; }
inline bool is_y_dtype(int d) { return d == PDELTA_F16 || d == PDELTA_BF16 || d == PDELTA_F32; }

int check_dims(int64_t d_out, int64_t d_in)
{
    if (d_out <= 0 || d_in <= 0) return PDELTA_EINVAL;
    if (d_in % 32 != 0 || d_out > kMaxDim || d_in > kMaxDim) return PDELTA_ESHAPE;
    return PDELTA_OK;
}

// Argument checks of one delta linear layer (no launch).
int linear_check(const void* X, const void* W_b, const uint32_t* B_packed, const uint16_t* v,
                 void* Y, int64_t M, int64_t d_out, int64_t d_in, int x_dtype, int y_dtype, int axis);

int linear_common(const void* X, const void* W_b, const uint32_t* B_packed, const uint16_t* v,
                  void* Y, int64_t M, int64_t d_out, int64_t d_in, int x_dtype, int y_dtype,
                  int axis, void* stream)
{
    const TuneScope tune_scope;
    if (const int rc = linear_check(X, W_b, B_packed, v, Y, M, d_out, d_in, x_dtype, y_dtype, axis))
        return rc;
    if (M == 0) return PDELTA_OK;
    hipStream_t s = (hipStream_t)stream;
    const int rc = M <= pdelta::kSkinnyMaxM
                       ? pdelta::launch_linear_skinny(x_dtype, y_dtype, axis, X, W_b, B_packed, v, Y, M,
                                                      d_out, d_in, s)
                       : pdelta::launch_linear_gemm(x_dtype, y_dtype, axis, X, W_b, B_packed, v, Y, M,
                                                    d_out, d_in, s);
    return rc == 0 ? PDELTA_OK : PDELTA_EHIP;
}

int linear_check(const void* X, const void* W_b, const uint32_t* B_packed, const uint16_t* v,
                 void* Y, int64_t M, int64_t d_out, int64_t d_in, int x_dtype, int y_dtype, int axis)
{
    if (W_b == nullptr || B_packed == nullptr || v == nullptr) return PDELTA_EINVAL;
    if (axis != PDELTA_ROW && axis != PDELTA_COL) return PDELTA_EINVAL;
    if (M < 0) return PDELTA_EINVAL;
    if (M > 0 && (X == nullptr || Y == nullptr)) return PDELTA_EINVAL;   // an empty batch has no X, Y
    if (const int rc = check_dims(d_out, d_in)) return rc;
    if (M > kMaxTokens) return PDELTA_ESHAPE;
    if (!is_w_dtype(x_dtype) || !is_y_dtype(y_dtype)) return PDELTA_EDTYPE;
    if (misaligned(X) || misaligned(W_b) || misaligned(B_packed) || misaligned(v) || misaligned(Y))
        return PDELTA_EALIGN;
    if (M == 0) return PDELTA_OK;
    const size_t y_bytes = (size_t)M * d_out * (y_dtype == PDELTA_F32 ? 4 : 2);
    const size_t v_bytes = (size_t)(axis == PDELTA_ROW ? d_out : d_in) * 2;
    if (overlaps(Y, y_bytes, X, (size_t)M * d_in * 2) ||
        overlaps(Y, y_bytes, W_b, (size_t)d_out * d_in * 2) ||
        overlaps(Y, y_bytes, B_packed, (size_t)d_out * d_in / 8) || overlaps(Y, y_bytes, v, v_bytes))
        return PDELTA_EINVAL;
    return PDELTA_OK;
}

}  // namespace
}  // namespace pdelta

extern "C" {
#pragma GCC visibility push(default)

int pdelta_probe_prefill_parts(int parts, const void* X, const void* W_b, const uint32_t* B_packed,
                               const uint16_t* v_row, void* Y, int64_t M, int64_t d_out, int64_t d_in,
                               int y_dtype, void* stream)
{
    using namespace pdelta;
    if (parts < 0 || parts > 15) return PDELTA_EINVAL;
    if (const int rc = linear_check(X, W_b, B_packed, v_row, Y, M, d_out, d_in, PDELTA_BF16, y_dtype, PDELTA_ROW))
        return rc;
    if (M <= 128) return PDELTA_ESHAPE;                 // the pipelined kernel is the one above 128 tokens
    const int rc = launch_linear_gemm_parts(parts, y_dtype, X, W_b, B_packed, v_row, Y, M, d_out, d_in,
                                            (hipStream_t)stream);
    return rc == 0 ? PDELTA_OK : (rc == -2 ? PDELTA_EINVAL : PDELTA_EHIP);
}

size_t pdelta_pack_workspace_bytes(int64_t d_out, int64_t d_in)
{
    if (d_out <= 0 || d_in <= 0) return 0;
    return pdelta::pack_workspace_bytes(d_out, d_in);
}

static int pack_check(const void* W_f, const void* W_b, int64_t d_out, int64_t d_in, int w_dtype,
                      uint32_t* B_packed, uint16_t* v_row, uint16_t* v_col, void* workspace,
                      size_t workspace_bytes, bool own_scratch = false)
{
    using namespace pdelta;
    if (W_f == nullptr || W_b == nullptr || B_packed == nullptr) return PDELTA_EINVAL;
    if (const int rc = check_dims(d_out, d_in)) return rc;
    if (!is_w_dtype(w_dtype)) return PDELTA_EDTYPE;
    // own_scratch: the partial sums go to the library's array, which no caller buffer can overlap
    const bool want_scales = (v_row != nullptr || v_col != nullptr) && !own_scratch;
    if (want_scales && (workspace == nullptr || workspace_bytes < pdelta_pack_workspace_bytes(d_out, d_in)))
        return PDELTA_EWORKSPACE;
    if (misaligned(W_f) || misaligned(W_b) || misaligned(B_packed) || misaligned(v_row) ||
        misaligned(v_col) || (want_scales && misaligned(workspace)))
        return PDELTA_EALIGN;
    // no output (signs, scale vectors, scratch) may share a byte with an input or another output
    const size_t w_bytes = (size_t)d_out * d_in * 2, b_bytes = (size_t)d_out * d_in / 8;
    struct Range { const void* p; size_t n; };
    const Range in[2] = {{W_f, w_bytes}, {W_b, w_bytes}};
    const Range out[4] = {{B_packed, b_bytes},
                          {v_row, v_row ? (size_t)d_out * 2 : 0},
                          {v_col, v_col ? (size_t)d_in * 2 : 0},
                          {want_scales ? workspace : nullptr, want_scales ? workspace_bytes : 0}};
    for (int a = 0; a < 4; ++a) {
        if (out[a].n == 0) continue;
        for (int b = 0; b < 2; ++b)
            if (overlaps(out[a].p, out[a].n, in[b].p, in[b].n)) return PDELTA_EINVAL;
        for (int b = a + 1; b < 4; ++b)
            if (out[b].n != 0 && overlaps(out[a].p, out[a].n, out[b].p, out[b].n)) return PDELTA_EINVAL;
    }
    return PDELTA_OK;
}

int pdelta_pack(const void* W_f, const void* W_b, int64_t d_out, int64_t d_in, int w_dtype,
                uint32_t* B_packed, uint16_t* v_row, uint16_t* v_col, void* workspace,
                size_t workspace_bytes, void* stream)
{
    using namespace pdelta;
    const TuneScope tune_scope;
    if (const int rc = pack_check(W_f, W_b, d_out, d_in, w_dtype, B_packed, v_row, v_col, workspace,
                                  workspace_bytes))
        return rc;
    const int rc = launch_pack_dispatch(w_dtype, W_f, W_b, d_out, d_in, B_packed, v_row, v_col,
                                        workspace, (hipStream_t)stream);
    return rc == 0 ? PDELTA_OK : PDELTA_EHIP;
}

size_t pdelta_pack_noalloc_max_bytes(void) { return pdelta::kPackScratchBytes; }

int pdelta_pack_noalloc(const void* W_f, const void* W_b, int64_t d_out, int64_t d_in, int w_dtype,
                        uint32_t* B_packed, uint16_t* v_row, uint16_t* v_col, void* stream)
{
    using namespace pdelta;
    const TuneScope tune_scope;
    // Everything that can be decided on the host comes first: the checks of pdelta_pack with a
    // stand-in scratch range that overlaps nothing, and the size limit of the library's array.
    if (const int rc = pack_check(W_f, W_b, d_out, d_in, w_dtype, B_packed, v_row, v_col, nullptr, 0,
                                  /*own_scratch=*/true))
        return rc;
    const bool want_scales = v_row != nullptr || v_col != nullptr;
    void* ws = nullptr;
    if (want_scales) {
        if (pack_workspace_bytes(d_out, d_in) > kPackScratchBytes) return PDELTA_EWORKSPACE;
        if (pack_static_scratch(&ws) != 0) return PDELTA_EHIP;
    }
    const int rc = launch_pack_dispatch(w_dtype, W_f, W_b, d_out, d_in, B_packed, v_row, v_col, ws,
                                        (hipStream_t)stream);
    return rc == 0 ? PDELTA_OK : PDELTA_EHIP;
}

int pdelta_pack_batch_plan(pdelta_pack_job* jobs_host, int32_t n_jobs)
{
    using namespace pdelta;
    if (n_jobs < 0 || (n_jobs > 0 && jobs_host == nullptr)) return PDELTA_EINVAL;
    int64_t tile = 0, fin = 0;
    for (int32_t j = 0; j < n_jobs; ++j) {
        pdelta_pack_job& J = jobs_host[j];
        if (const int rc = check_dims(J.d_out, J.d_in)) return rc;
        if (tile > 0x7FFFFFFF || fin > 0x7FFFFFFF) return PDELTA_ESHAPE;
        J.first_tile = (int32_t)tile;
        J.first_fin_block = (int32_t)fin;
        J.tile_blocks = pack_batch_tile_blocks(J.d_out);
        J.reserved = 0;
        tile += pack_batch_tiles(J.d_out, J.d_in, J.tile_blocks);
        fin += pack_batch_fin_blocks(J.d_out, J.d_in);
    }
    if (tile > 0x7FFFFFFF || fin > 0x7FFFFFFF) return PDELTA_ESHAPE;
    return PDELTA_OK;
}

int pdelta_pack_batch(const pdelta_pack_job* jobs_host, const pdelta_pack_job* jobs_device,
                      int32_t n_jobs, int w_dtype, void* stream)
{
    using namespace pdelta;
    const TuneScope tune_scope;
    if (n_jobs < 0) return PDELTA_EINVAL;
    if (n_jobs == 0) return PDELTA_OK;
    if (jobs_host == nullptr || jobs_device == nullptr) return PDELTA_EINVAL;
    if (misaligned(jobs_device)) return PDELTA_EALIGN;
    int64_t tile = 0, fin = 0;
    for (int32_t j = 0; j < n_jobs; ++j) {
        const pdelta_pack_job& J = jobs_host[j];
        if (const int rc = pack_check(J.W_f, J.W_b, J.d_out, J.d_in, w_dtype, J.B_packed, J.v_row, J.v_col,
                                      J.workspace, J.workspace_bytes))
            return rc;
        if (J.first_tile != (int32_t)tile || J.first_fin_block != (int32_t)fin ||
            J.tile_blocks != pack_batch_tile_blocks(J.d_out))
            return PDELTA_EINVAL;                                       // not planned, or edited
        tile += pack_batch_tiles(J.d_out, J.d_in, J.tile_blocks);
        fin += pack_batch_fin_blocks(J.d_out, J.d_in);
    }
    const int rc = launch_pack_batch(w_dtype, jobs_host, jobs_device, n_jobs, (hipStream_t)stream);
    return rc == 0 ? PDELTA_OK : PDELTA_EHIP;
}

int pdelta_linear_row(const void* X, const void* W_b, const uint32_t* B_packed,
                      const uint16_t* v_row, void* Y, int64_t M, int64_t d_out, int64_t d_in,
                      int x_dtype, int y_dtype, void* stream)
{
    return pdelta::linear_common(X, W_b, B_packed, v_row, Y, M, d_out, d_in, x_dtype, y_dtype,
                                 PDELTA_ROW, stream);
}

int pdelta_linear_col(const void* X, const void* W_b, const uint32_t* B_packed,
                      const uint16_t* v_col, void* Y, int64_t M, int64_t d_out, int64_t d_in,
                      int x_dtype, int y_dtype, void* stream)
{
    return pdelta::linear_common(X, W_b, B_packed, v_col, Y, M, d_out, d_in, x_dtype, y_dtype,
                                 PDELTA_COL, stream);
}

static int patch_check(const void* W_b, const uint32_t* B_packed, const uint16_t* v, int axis,
                       void* W_out, int64_t d_out, int64_t d_in, int w_dtype)
{
    using namespace pdelta;
    if (W_b == nullptr || B_packed == nullptr || v == nullptr || W_out == nullptr) return PDELTA_EINVAL;
    if (axis != PDELTA_ROW && axis != PDELTA_COL) return PDELTA_EINVAL;
    if (const int rc = check_dims(d_out, d_in)) return rc;
    if (!is_w_dtype(w_dtype)) return PDELTA_EDTYPE;
    if (misaligned(W_b) || misaligned(B_packed) || misaligned(v) || misaligned(W_out))
        return PDELTA_EALIGN;
    const size_t w_bytes = (size_t)d_out * d_in * 2;
    if (W_out != W_b && overlaps(W_out, w_bytes, W_b, w_bytes)) return PDELTA_EINVAL;
    if (overlaps(W_out, w_bytes, B_packed, w_bytes / 16) ||
        overlaps(W_out, w_bytes, v, (size_t)(axis == PDELTA_ROW ? d_out : d_in) * 2))
        return PDELTA_EINVAL;
    return PDELTA_OK;
}

int pdelta_patch(const void* W_b, const uint32_t* B_packed, const uint16_t* v, int axis,
                 void* W_out, int64_t d_out, int64_t d_in, int w_dtype, void* stream)
{
    using namespace pdelta;
    const TuneScope tune_scope;
    if (const int rc = patch_check(W_b, B_packed, v, axis, W_out, d_out, d_in, w_dtype)) return rc;
    const int rc = launch_patch_dispatch(w_dtype, axis, W_b, B_packed, v, W_out, d_out, d_in,
                                         (hipStream_t)stream);
    return rc == 0 ? PDELTA_OK : PDELTA_EHIP;
}

int pdelta_patch_batch(const pdelta_layer* layers_host, const pdelta_layer* layers_device,
                       int32_t n_layers, int w_dtype, void* stream)
{
    using namespace pdelta;
    const TuneScope tune_scope;
    if (n_layers < 0) return PDELTA_EINVAL;
    if (n_layers == 0) return PDELTA_OK;
    if (layers_host == nullptr || layers_device == nullptr) return PDELTA_EINVAL;
    if (misaligned(layers_device)) return PDELTA_EALIGN;
    int64_t first = 0;
    for (int32_t l = 0; l < n_layers; ++l) {
        const pdelta_layer& L = layers_host[l];
        if (const int rc = patch_check(L.W_b, L.B_packed, L.v, L.axis, L.Y, L.d_out, L.d_in, w_dtype))
            return rc;
        if (L.first_block != (int32_t)first) return PDELTA_EINVAL;     // not planned, or edited
        first += (L.d_out + 15) / 16;
    }
    int rc = launch_patch_batch(w_dtype, layers_host, layers_device, n_layers, (hipStream_t)stream);
    if (rc == 1) {                                                      // too many blocks for one grid
        rc = 0;
        for (int32_t l = 0; l < n_layers && rc == 0; ++l) {
            const pdelta_layer& L = layers_host[l];
            rc = launch_patch_dispatch(w_dtype, L.axis, L.W_b, L.B_packed, L.v, L.Y, L.d_out, L.d_in,
                                       (hipStream_t)stream);
        }
    }
    return rc == 0 ? PDELTA_OK : PDELTA_EHIP;
}

int pdelta_linear_batch_plan(pdelta_layer* layers_host, int32_t n_layers)
{
    if (n_layers < 0 || (n_layers > 0 && layers_host == nullptr)) return PDELTA_EINVAL;
    int64_t first = 0;
    for (int32_t l = 0; l < n_layers; ++l) {
        pdelta_layer& L = layers_host[l];
        if (L.axis != PDELTA_ROW && L.axis != PDELTA_COL) return PDELTA_EINVAL;
        if (const int rc = pdelta::check_dims(L.d_out, L.d_in)) return rc;
        if (first > 0x7FFFFFFF) return PDELTA_ESHAPE;
        L.first_block = (int32_t)first;
        first += (L.d_out + 15) / 16;
    }
    return PDELTA_OK;
}

int pdelta_linear_batch(const pdelta_layer* layers_host, const pdelta_layer* layers_device,
                        int32_t n_layers, int64_t M, int x_dtype, int y_dtype, void* stream)
{
    using namespace pdelta;
    const TuneScope tune_scope;
    if (n_layers < 0 || M < 0) return PDELTA_EINVAL;
    if (n_layers == 0) return PDELTA_OK;
    if (layers_host == nullptr || layers_device == nullptr) return PDELTA_EINVAL;
    if (misaligned(layers_device)) return PDELTA_EALIGN;
    int64_t first = 0;
    for (int32_t l = 0; l < n_layers; ++l) {
        const pdelta_layer& L = layers_host[l];
        if (const int rc = linear_check(L.X, L.W_b, L.B_packed, L.v, L.Y, M, L.d_out, L.d_in, x_dtype,
                                        y_dtype, L.axis))
            return rc;
        if (L.first_block != (int32_t)first) return PDELTA_EINVAL;     // not planned, or edited
        first += (L.d_out + 15) / 16;
    }
    if (M == 0) return PDELTA_OK;
    hipStream_t s = (hipStream_t)stream;
    int rc = M <= kSkinnyMaxM ? launch_linear_skinny_batch(x_dtype, y_dtype, layers_host, layers_device,
                                                           n_layers, M, s)
                              : 1;
    if (rc == 1) {                                                      // layer by layer
        rc = 0;
        for (int32_t l = 0; l < n_layers && rc == 0; ++l) {
            const pdelta_layer& L = layers_host[l];
            rc = M <= kSkinnyMaxM ? launch_linear_skinny(x_dtype, y_dtype, L.axis, L.X, L.W_b, L.B_packed,
                                                         L.v, L.Y, M, L.d_out, L.d_in, s)
                                  : launch_linear_gemm(x_dtype, y_dtype, L.axis, L.X, L.W_b, L.B_packed,
                                                       L.v, L.Y, M, L.d_out, L.d_in, s);
        }
    }
    return rc == 0 ? PDELTA_OK : PDELTA_EHIP;
}

int pdelta_linear_variants(const void* X, const void* W_b, const pdelta_variant* variants_host,
                           const pdelta_variant* variants_device, int32_t R, int axis, void* Y,
                           int64_t d_out, int64_t d_in, int x_dtype, int y_dtype, void* stream)
{
    using namespace pdelta;
    const TuneScope tune_scope;
    if (R < 0) return PDELTA_EINVAL;
    if (R > 0 && (variants_host == nullptr || variants_device == nullptr)) return PDELTA_EINVAL;
    if (misaligned(variants_device)) return PDELTA_EALIGN;
    if (axis != PDELTA_ROW && axis != PDELTA_COL && axis != PDELTA_PER_REQUEST) return PDELTA_EINVAL;
    if (R == 0) {
        if (const int rc = check_dims(d_out, d_in)) return rc;
        if (!is_w_dtype(x_dtype) || !is_y_dtype(y_dtype)) return PDELTA_EDTYPE;
        return PDELTA_OK;
    }
    // per-request axes: every record names its own mode; all equal -> the single-mode kernels
    int kernel_axis = axis;
    if (axis == PDELTA_PER_REQUEST) {
        kernel_axis = variants_host[0].axis;
        for (int32_t r = 0; r < R; ++r) {
            if (variants_host[r].axis != PDELTA_ROW && variants_host[r].axis != PDELTA_COL) return PDELTA_EINVAL;
            if (variants_host[r].axis != kernel_axis) kernel_axis = PDELTA_PER_REQUEST;
        }
    }
    for (int32_t r = 0; r < R; ++r)
        if (const int rc = linear_check(X, W_b, variants_host[r].B_packed, variants_host[r].v, Y, R, d_out, d_in,
                                        x_dtype, y_dtype, axis == PDELTA_PER_REQUEST ? variants_host[r].axis : axis))
            return rc;
    hipStream_t s = (hipStream_t)stream;
    int rc = launch_linear_variants(x_dtype, y_dtype, kernel_axis, X, W_b, variants_device, R, Y, d_out, d_in, s);
    if (rc == 1) {                                                      // request by request
        rc = 0;
        const size_t ysz = y_dtype == PDELTA_F32 ? 4 : 2;
        for (int32_t r = 0; r < R && rc == 0; ++r)
            rc = launch_linear_skinny(x_dtype, y_dtype, axis == PDELTA_PER_REQUEST ? variants_host[r].axis : axis,
                                      (const char*)X + (size_t)r * d_in * 2, W_b,
                                      variants_host[r].B_packed, variants_host[r].v,
                                      (char*)Y + (size_t)r * d_out * ysz, 1, d_out, d_in, s);
    }
    return rc == 0 ? PDELTA_OK : PDELTA_EHIP;
}

size_t pdelta_grad_v_workspace_bytes(int64_t M, int64_t d_out, int64_t d_in, int axis)
{
    if (M < 0 || d_out <= 0 || d_in <= 0 || (axis != PDELTA_ROW && axis != PDELTA_COL)) return 0;
    return pdelta::grad_v_workspace_bytes(M, d_out, d_in, axis);
}

int pdelta_grad_v(const void* X, const void* dY, const uint32_t* B_packed, int axis, float* grad_v,
                  int64_t M, int64_t d_out, int64_t d_in, int dtype, void* workspace,
                  size_t workspace_bytes, void* stream)
{
    using namespace pdelta;
    const TuneScope tune_scope;
    if (B_packed == nullptr || grad_v == nullptr) return PDELTA_EINVAL;
    if (axis != PDELTA_ROW && axis != PDELTA_COL) return PDELTA_EINVAL;
    if (M < 0) return PDELTA_EINVAL;
    if (M > 0 && (X == nullptr || dY == nullptr)) return PDELTA_EINVAL;
    if (const int rc = check_dims(d_out, d_in)) return rc;
    if (M > kMaxTokens) return PDELTA_ESHAPE;
    if (axis == PDELTA_COL && d_out % 32 != 0) return PDELTA_ESHAPE;
    if (!is_w_dtype(dtype)) return PDELTA_EDTYPE;
    if (workspace == nullptr || workspace_bytes < grad_v_workspace_bytes(M, d_out, d_in, axis))
        return PDELTA_EWORKSPACE;
    if (misaligned(X) || misaligned(dY) || misaligned(B_packed) || misaligned(grad_v) || misaligned(workspace))
        return PDELTA_EALIGN;
    const size_t g_bytes = (size_t)(axis == PDELTA_ROW ? d_out : d_in) * 4;
    if (overlaps(grad_v, g_bytes, X, (size_t)M * d_in * 2) || overlaps(grad_v, g_bytes, dY, (size_t)M * d_out * 2) ||
        overlaps(grad_v, g_bytes, B_packed, (size_t)d_out * d_in / 8) ||
        overlaps(grad_v, g_bytes, workspace, workspace_bytes))
        return PDELTA_EINVAL;
    const int rc = launch_grad_v(dtype, axis, X, dY, B_packed, grad_v, M, d_out, d_in, workspace, (hipStream_t)stream);
    return rc == 0 ? PDELTA_OK : PDELTA_EHIP;
}

// ---- blockwise ("per-group") and scalar scales -------------------------------------------------

// Layout of a blockwise scale array for these arguments, or an error code.
static int group_layout(int64_t d_out, int64_t d_in, int64_t group, int shared_rows, int* v_stride, int* g_shift,
                        size_t* v_bytes)
{
    if (const int rc = pdelta::check_dims(d_out, d_in)) return rc;
    if (group <= 0 || (shared_rows != 0 && shared_rows != 1)) return PDELTA_EINVAL;
    int64_t n_groups = 1;
    int shift = 31;                                     // one group spans the row: index 0 for every input
    if (group != d_in) {
        if (group < 32 || (group & (group - 1)) != 0 || d_in % group != 0) return PDELTA_ESHAPE;
        shift = __builtin_ctzll((unsigned long long)group);
        n_groups = d_in / group;
    }
    *v_stride = shared_rows ? 0 : (int)n_groups;
    *g_shift = shift;
    *v_bytes = (size_t)(shared_rows ? 1 : d_out) * (size_t)n_groups * 2;
    return PDELTA_OK;
}

size_t pdelta_pack_group_workspace_bytes(int64_t d_out, int64_t d_in, int64_t group, int shared_rows)
{
    int v_stride, g_shift;
    size_t v_bytes;
    if (group_layout(d_out, d_in, group, shared_rows, &v_stride, &g_shift, &v_bytes) != PDELTA_OK) return 0;
    return pdelta::pack_group_workspace_bytes(d_out, d_in, group, shared_rows);
}

int pdelta_pack_group(const void* W_f, const void* W_b, int64_t d_out, int64_t d_in, int w_dtype, int64_t group,
                      int shared_rows, uint32_t* B_packed, uint16_t* v, void* workspace, size_t workspace_bytes,
                      void* stream)
{
    using namespace pdelta;
    const TuneScope tune_scope;
    if (W_f == nullptr || W_b == nullptr || B_packed == nullptr || v == nullptr) return PDELTA_EINVAL;
    int v_stride, g_shift;
    size_t v_bytes;
    if (const int rc = group_layout(d_out, d_in, group, shared_rows, &v_stride, &g_shift, &v_bytes)) return rc;
    if (!is_w_dtype(w_dtype)) return PDELTA_EDTYPE;
    const size_t need = pack_group_workspace_bytes(d_out, d_in, group, shared_rows);
    if (need > 0 && (workspace == nullptr || workspace_bytes < need)) return PDELTA_EWORKSPACE;
    if (misaligned(W_f) || misaligned(W_b) || misaligned(B_packed) || misaligned(v) ||
        (need > 0 && misaligned(workspace)))
        return PDELTA_EALIGN;
    const size_t w_bytes = (size_t)d_out * d_in * 2, b_bytes = w_bytes / 16;
    struct Range { const void* p; size_t n; };
    const Range in[2] = {{W_f, w_bytes}, {W_b, w_bytes}};
    const Range out[3] = {{B_packed, b_bytes}, {v, v_bytes}, {need > 0 ? workspace : nullptr, need > 0 ? workspace_bytes : 0}};
    for (int a = 0; a < 3; ++a) {
        if (out[a].n == 0) continue;
        for (int b = 0; b < 2; ++b)
            if (overlaps(out[a].p, out[a].n, in[b].p, in[b].n)) return PDELTA_EINVAL;
        for (int b = a + 1; b < 3; ++b)
            if (out[b].n != 0 && overlaps(out[a].p, out[a].n, out[b].p, out[b].n)) return PDELTA_EINVAL;
    }
    const int rc = launch_pack_group(w_dtype, W_f, W_b, d_out, d_in, group, shared_rows, B_packed, v, workspace,
                                     (hipStream_t)stream);
    return rc == 0 ? PDELTA_OK : PDELTA_EHIP;
}

int pdelta_linear_group(const void* X, const void* W_b, const uint32_t* B_packed, const uint16_t* v, int64_t group,
                        int shared_rows, void* Y, int64_t M, int64_t d_out, int64_t d_in, int x_dtype, int y_dtype,
                        void* stream)
{
    using namespace pdelta;
    const TuneScope tune_scope;
    if (W_b == nullptr || B_packed == nullptr || v == nullptr || M < 0) return PDELTA_EINVAL;
    if (M > 0 && (X == nullptr || Y == nullptr)) return PDELTA_EINVAL;
    int v_stride, g_shift;
    size_t v_bytes;
    if (const int rc = group_layout(d_out, d_in, group, shared_rows, &v_stride, &g_shift, &v_bytes)) return rc;
    if (M > kMaxTokens) return PDELTA_ESHAPE;
    if (!is_w_dtype(x_dtype) || !is_y_dtype(y_dtype)) return PDELTA_EDTYPE;
    if (misaligned(X) || misaligned(W_b) || misaligned(B_packed) || misaligned(v) || misaligned(Y)) return PDELTA_EALIGN;
    if (M == 0) return PDELTA_OK;
    const size_t y_bytes = (size_t)M * d_out * (y_dtype == PDELTA_F32 ? 4 : 2);
    if (overlaps(Y, y_bytes, X, (size_t)M * d_in * 2) || overlaps(Y, y_bytes, W_b, (size_t)d_out * d_in * 2) ||
        overlaps(Y, y_bytes, B_packed, (size_t)d_out * d_in / 8) || overlaps(Y, y_bytes, v, v_bytes))
        return PDELTA_EINVAL;
    hipStream_t s = (hipStream_t)stream;
    const int rc = M <= kSkinnyMaxM ? launch_linear_skinny_group(x_dtype, y_dtype, X, W_b, B_packed, v, Y, M, d_out,
                                                                 d_in, v_stride, g_shift, s)
                                    : launch_linear_gemm_group(x_dtype, y_dtype, X, W_b, B_packed, v, Y, M, d_out,
                                                               d_in, v_stride, g_shift, s);
    return rc == 0 ? PDELTA_OK : PDELTA_EHIP;
}

int pdelta_patch_group(const void* W_b, const uint32_t* B_packed, const uint16_t* v, int64_t group, int shared_rows,
                       void* W_out, int64_t d_out, int64_t d_in, int w_dtype, void* stream)
{
    using namespace pdelta;
    const TuneScope tune_scope;
    if (W_b == nullptr || B_packed == nullptr || v == nullptr || W_out == nullptr) return PDELTA_EINVAL;
    int v_stride, g_shift;
    size_t v_bytes;
    if (const int rc = group_layout(d_out, d_in, group, shared_rows, &v_stride, &g_shift, &v_bytes)) return rc;
    if (!is_w_dtype(w_dtype)) return PDELTA_EDTYPE;
    if (misaligned(W_b) || misaligned(B_packed) || misaligned(v) || misaligned(W_out)) return PDELTA_EALIGN;
    const size_t w_bytes = (size_t)d_out * d_in * 2;
    if (W_out != W_b && overlaps(W_out, w_bytes, W_b, w_bytes)) return PDELTA_EINVAL;
    if (overlaps(W_out, w_bytes, B_packed, w_bytes / 16) || overlaps(W_out, w_bytes, v, v_bytes)) return PDELTA_EINVAL;
    const int rc = launch_patch_group(w_dtype, W_b, B_packed, v, W_out, d_out, d_in, v_stride, g_shift,
                                      (hipStream_t)stream);
    return rc == 0 ? PDELTA_OK : PDELTA_EHIP;
}

const char* pdelta_status_string(int status)
{
    switch (status) {
        case PDELTA_OK: return "PDELTA_OK";
        case PDELTA_EINVAL: return "PDELTA_EINVAL: null pointer, bad dimension or axis, or aliasing";
        case PDELTA_ESHAPE: return "PDELTA_ESHAPE: d_in not a multiple of 32 or dimension too large";
        case PDELTA_EALIGN: return "PDELTA_EALIGN: pointer not 16-byte aligned";
        case PDELTA_EDTYPE: return "PDELTA_EDTYPE: dtype not accepted here";
        case PDELTA_EWORKSPACE: return "PDELTA_EWORKSPACE: workspace missing or too small";
        case PDELTA_EHIP: return "PDELTA_EHIP: kernel launch failed";
        default: return "unknown pdelta status";
    }
}

#pragma GCC visibility pop
}  // extern "C"
