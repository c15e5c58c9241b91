// C ABI of the library: argument validation, kernel choice, launch.
// Everything here runs on the host; all checks precede any HIP call.
#include <stdint.h>
#include <string.h>

#include "sr_launch.h"

using namespace srd;

namespace {

size_t elem_size(sr_dtype d) { return (d == SR_F16 || d == SR_BF16) ? 2 : (d == SR_F8E4M3 ? 1 : 4); }
bool dtype_ok(int d) { return d == SR_F32 || d == SR_F16; }                    // images
bool coeff_dtype_ok(int d) { return dtype_ok(d) || d == SR_F8E4M3 || d == SR_BF16; }   // coefficients

size_t tensor_bytes(const sr_tensor* t) {
    return (size_t)t->n * t->c * t->h * t->w * elem_size(t->dtype);
}

bool overlaps(const sr_tensor* a, const sr_tensor* b) {
    const uintptr_t a0 = (uintptr_t)a->data, a1 = a0 + tensor_bytes(a);
    const uintptr_t b0 = (uintptr_t)b->data, b1 = b0 + tensor_bytes(b);
    return a0 < b1 && b0 < a1;
}

bool dims_ok(const sr_tensor* t) { return t->n >= 0 && t->c >= 0 && t->h >= 0 && t->w >= 0; }

bool aligned(const sr_tensor* t) { return ((uintptr_t)t->data % elem_size(t->dtype)) == 0; }

struct Plan {
    int status;      // SR_OK or an error
    int kernel;      // SR_KERNEL_GENERIC | SR_KERNEL_MFMA
    int tile;
    bool empty;      // nothing to do
    AssembleArgs args;
};

// Validate everything and build the kernel arguments.  No HIP calls.
void make_plan(Plan& p, const sr_tensor* lr, const sr_tensor* coeff, const sr_tensor* dict,
               int L, int k, int scale, int channels, const sr_tensor* out,
               const int* kept, int n_kept, const float* gamma, const sr_options* opts) {
    p.status = SR_OK;
    p.kernel = SR_KERNEL_GENERIC;
    p.tile = 0;
    p.empty = false;
    if (!lr || !coeff || !dict || !out) { p.status = SR_ERR_NULL; return; }
    if (!dtype_ok(lr->dtype) || !coeff_dtype_ok(coeff->dtype) || !dtype_ok(out->dtype) ||
        dict->dtype != SR_F32 || out->dtype != lr->dtype) { p.status = SR_ERR_UNSUPPORTED; return; }
    if (!dims_ok(lr) || !dims_ok(coeff) || !dims_ok(dict) || !dims_ok(out)) { p.status = SR_ERR_SHAPE; return; }
    if (k != 3 && k != 5 && k != 7) { p.status = SR_ERR_UNSUPPORTED; return; }
    if (scale < 2 || scale > 4) { p.status = SR_ERR_UNSUPPORTED; return; }
    if (L < 1 || L > SR_MAX_ATOMS || channels < 1 || channels > SR_MAX_CHANNELS) {
        p.status = SR_ERR_UNSUPPORTED; return;
    }
    if (opts && (opts->coeff_layout < SR_COEFF_PLANAR || opts->coeff_layout > SR_COEFF_BLOCKED ||
                 opts->coeff_kind < SR_COEFF_VALUES || opts->coeff_kind > SR_COEFF_LOGITS)) {
        p.status = SR_ERR_UNSUPPORTED; return;
    }
    // logits: the softmax runs over all L atoms, so there is no kept list; 8-bit logits are not taken
    const bool logits = opts && opts->coeff_kind == SR_COEFF_LOGITS;
    if (logits && (kept || gamma || coeff->dtype == SR_F8E4M3)) { p.status = SR_ERR_UNSUPPORTED; return; }
    if (lr->c != channels || out->c != channels ||
        dict->n != 1 || dict->c != L || dict->h != k || dict->w != k ||
        coeff->n != lr->n || out->n != lr->n ||
        (int64_t)lr->h * scale != out->h || (int64_t)lr->w * scale != out->w) { p.status = SR_ERR_SHAPE; return; }
    const bool pre_shuffle = opts && opts->coeff_layout == SR_COEFF_PRE_SHUFFLE;
    if (pre_shuffle ? (coeff->c != L * scale * scale || coeff->h != lr->h || coeff->w != lr->w)
                    : (coeff->c != L || coeff->h != out->h || coeff->w != out->w)) { p.status = SR_ERR_SHAPE; return; }
    // limits of the launch grids: the generic kernel takes four rows per workgroup in grid.y (<= 65535)
    if ((int64_t)lr->n > 65535 || (int64_t)out->h > 4 * 65535 || (int64_t)out->w > (1 << 20)) {
        p.status = SR_ERR_UNSUPPORTED; return;
    }
    if (opts) {
        for (int i = 0; i < 4; ++i)
            if (opts->reserved[i]) { p.status = SR_ERR_UNSUPPORTED; return; }
        if (opts->kernel < SR_KERNEL_AUTO || opts->kernel > SR_KERNEL_MFMA || opts->tile < 0) {
            p.status = SR_ERR_UNSUPPORTED; return;
        }
    }
    AssembleArgs& a = p.args;
    memset(&a, 0, sizeof(a));
    if (kept) {
        if (n_kept < 1 || n_kept > L) { p.status = SR_ERR_KEPT; return; }
        bool seen[SR_MAX_ATOMS] = {false};
        for (int i = 0; i < n_kept; ++i) {
            if (kept[i] < 0 || kept[i] >= L || seen[kept[i]]) { p.status = SR_ERR_KEPT; return; }
            seen[kept[i]] = true;
            a.kept[i] = kept[i];
            a.gamma[i] = gamma ? gamma[i] : 1.0f;
        }
        a.n_fold = n_kept;
    } else {
        if (gamma) { p.status = SR_ERR_KEPT; return; }
        for (int i = 0; i < L; ++i) { a.kept[i] = i; a.gamma[i] = 1.0f; }
        a.n_fold = L;
    }
    a.io_f16 = lr->dtype == SR_F16;
    a.coeff_dtype = coeff->dtype;
    p.empty = lr->n == 0 || lr->h == 0 || lr->w == 0;
    if (!p.empty) {
        if (!lr->data || !coeff->data || !dict->data || !out->data) { p.status = SR_ERR_NULL; return; }
        if (!aligned(lr) || !aligned(coeff) || !aligned(dict) || !aligned(out)) { p.status = SR_ERR_ALIGN; return; }
        if (overlaps(out, lr) || overlaps(out, coeff) || overlaps(out, dict)) { p.status = SR_ERR_ALIAS; return; }
    }
    a.lr = lr->data; a.coeff = coeff->data; a.dict = (const float*)dict->data; a.out = out->data;
    a.N = lr->n; a.C = channels; a.h = lr->h; a.w = lr->w;
    a.H = out->h; a.W = out->w; a.s = scale; a.L = L;
    a.pre_shuffle = pre_shuffle ? 1 : 0;
    a.pixel_major = opts && opts->coeff_layout == SR_COEFF_PIXEL_MAJOR ? 1 : 0;
    a.logits = logits ? 1 : 0;
    a.blocked = opts && opts->coeff_layout == SR_COEFF_BLOCKED ? 1 : 0;
    if (a.blocked && (L % 8 != 0 || out->w % 128 != 0)) { p.status = SR_ERR_UNSUPPORTED; return; }   // the order does not exist

    const int want = opts ? opts->kernel : SR_KERNEL_AUTO;
    const int tile = opts ? opts->tile : 0;
    const bool can_mfma = !p.empty && mfma_supported(a, k, coeff->dtype, tile);
    // a tile index other than 0 is an option of the matrix-core kernel: it never falls back silently
    if ((want == SR_KERNEL_MFMA || (tile != 0 && want != SR_KERNEL_GENERIC)) && !can_mfma) { p.status = SR_ERR_UNSUPPORTED; return; }
    p.kernel = (want == SR_KERNEL_GENERIC || !can_mfma) ? SR_KERNEL_GENERIC : SR_KERNEL_MFMA;
    p.tile = tile;
}

}  // namespace

extern "C" {

__attribute__((visibility("default"))) int sr_dict_assemble_ex(const sr_tensor* lr, const sr_tensor* coeff, const sr_tensor* dict,
                        int L, int k, int scale, int channels, sr_tensor* out, void* stream,
                        const int* kept, int n_kept, const float* gamma, const sr_options* opts) {
    Plan p;
    make_plan(p, lr, coeff, dict, L, k, scale, channels, out, kept, n_kept, gamma, opts);
    if (p.status != SR_OK) return p.status;
    if (p.empty) return SR_OK;
    const hipStream_t st = (hipStream_t)stream;
    const bool io_f16 = lr->dtype == SR_F16;
    hipError_t e = (p.kernel == SR_KERNEL_MFMA)
                       ? launch_mfma(p.args, k, io_f16, p.tile, st)
                       : launch_generic(p.args, k, io_f16, st);
    return e == hipSuccess ? SR_OK : SR_ERR_LAUNCH;
}

__attribute__((visibility("default"))) int sr_dict_assemble(const sr_tensor* lr, const sr_tensor* coeff, const sr_tensor* dict,
                     int L, int k, int scale, int channels, sr_tensor* out, void* stream) {
    return sr_dict_assemble_ex(lr, coeff, dict, L, k, scale, channels, out, stream,
                               nullptr, 0, nullptr, nullptr);
}

__attribute__((visibility("default"))) int sr_dict_assemble_selective(const sr_tensor* lr, const sr_tensor* coeff, const sr_tensor* dict,
                               int L, int k, int scale, int channels, sr_tensor* out, void* stream,
                               const int* kept, int n_kept, const float* gamma) {
    if (!kept) return SR_ERR_NULL;
    return sr_dict_assemble_ex(lr, coeff, dict, L, k, scale, channels, out, stream,
                               kept, n_kept, gamma, nullptr);
}

__attribute__((visibility("default"))) int sr_dict_assemble_plan(const sr_tensor* lr, const sr_tensor* coeff, const sr_tensor* dict,
                          int L, int k, int scale, int channels, const sr_tensor* out,
                          const int* kept, int n_kept, const sr_options* opts) {
    Plan p;
    make_plan(p, lr, coeff, dict, L, k, scale, channels, out, kept, n_kept, nullptr, opts);
    return p.status != SR_OK ? p.status : p.kernel;
}

__attribute__((visibility("default"))) int sr_dict_assemble_tile(const sr_tensor* lr, const sr_tensor* coeff, const sr_tensor* dict,
                          int L, int k, int scale, int channels, const sr_tensor* out,
                          const int* kept, int n_kept, const sr_options* opts, int* tile_w, int* tile_h) {
    if (!tile_w || !tile_h) return SR_ERR_NULL;
    Plan p;
    make_plan(p, lr, coeff, dict, L, k, scale, channels, out, kept, n_kept, nullptr, opts);
    if (p.status != SR_OK) return p.status;
    *tile_w = *tile_h = 0;
    if (p.kernel == SR_KERNEL_MFMA && !p.empty) mfma_tile_shape(p.args, k, coeff->dtype, p.tile, tile_w, tile_h);
    return p.kernel;
}

__attribute__((visibility("default"))) int sr_dict_assemble_launch_shape(const sr_tensor* lr, const sr_tensor* coeff, const sr_tensor* dict,
                          int L, int k, int scale, int channels, const sr_tensor* out,
                          const int* kept, int n_kept, const sr_options* opts, int shape[4]) {
    if (!shape) return SR_ERR_NULL;
    Plan p;
    make_plan(p, lr, coeff, dict, L, k, scale, channels, out, kept, n_kept, nullptr, opts);
    if (p.status != SR_OK) return p.status;
    shape[0] = shape[1] = shape[2] = shape[3] = 0;
    if (p.kernel == SR_KERNEL_MFMA && !p.empty)
        mfma_tile_shape(p.args, k, coeff->dtype, p.tile, &shape[0], &shape[1], &shape[2], &shape[3]);
    return p.kernel;
}

__attribute__((visibility("default"))) int sr_bicubic_upsample(const sr_tensor* lr, int scale, int channels, sr_tensor* out, void* stream) {
    if (!lr || !out) return SR_ERR_NULL;
    if (!dtype_ok(lr->dtype) || !dtype_ok(out->dtype)) return SR_ERR_UNSUPPORTED;
    if (out->dtype == SR_F16 && lr->dtype != SR_F16) return SR_ERR_UNSUPPORTED;
    if (!dims_ok(lr) || !dims_ok(out)) return SR_ERR_SHAPE;
    if (scale < 2 || scale > 4 || channels < 1 || channels > SR_MAX_CHANNELS) return SR_ERR_UNSUPPORTED;
    if (lr->c != channels || out->c != channels || out->n != lr->n ||
        (int64_t)lr->h * scale != out->h || (int64_t)lr->w * scale != out->w) return SR_ERR_SHAPE;
    if ((int64_t)lr->n * channels > 65535 || out->h > (1 << 18) || out->w > (1 << 20)) return SR_ERR_UNSUPPORTED;
    if (lr->n == 0 || lr->h == 0 || lr->w == 0) return SR_OK;
    if (!lr->data || !out->data) return SR_ERR_NULL;
    if (!aligned(lr) || !aligned(out)) return SR_ERR_ALIGN;
    if (overlaps(out, lr)) return SR_ERR_ALIAS;
    BicubicArgs a;
    a.lr = lr->data; a.out = out->data;
    a.NC = lr->n * channels; a.h = lr->h; a.w = lr->w; a.H = out->h; a.W = out->w; a.s = scale;
    hipError_t e = launch_bicubic(a, lr->dtype == SR_F16, out->dtype == SR_F16, (hipStream_t)stream);
    return e == hipSuccess ? SR_OK : SR_ERR_LAUNCH;
}

__attribute__((visibility("default"))) const char* sr_strerror(int status) {
    switch (status) {
    case SR_OK:              return "success";
    case SR_ERR_NULL:        return "a required pointer is NULL";
    case SR_ERR_SHAPE:       return "tensor sizes disagree with L, k, scale or channels";
    case SR_ERR_UNSUPPORTED: return "unsupported k, scale, L, channel count, dtype mix or option";
    case SR_ERR_ALIAS:       return "the output overlaps an input";
    case SR_ERR_KEPT:        return "bad kept-atom list";
    case SR_ERR_LAUNCH:      return "the HIP runtime refused the kernel launch";
    case SR_ERR_ALIGN:       return "a data pointer is not aligned to its element size";
    case SR_ERR_SCRATCH:     return "the call needs more scratch memory than the library's built-in buffer holds";
    default:                 return "unknown status";
    }
}

__attribute__((visibility("default"))) int sr_version(void) { return SR_VERSION; }

}  // extern "C"
