/*
 * sr_dict.h -- C ABI of the MI355X (gfx950) pixel-adaptive dictionary-assembly
 * library: the "dictionary query and filtering" path of a LAPAR-style
 * super-resolution model (paper section II-A, Eq. 2 and Eq. 3; stages 1, 3
 * and 4 of the inference flow in section II-B; compressed dictionaries per
 * section III-A).
 *
 * For every HR pixel i the path computes
 *
 *     F_i = Phi_i D          (stage 3, dictionary assembling, Eq. 2)
 *     y_i = F_i B_i^T        (stage 4, filtering, Eq. 2)
 *
 * where D is the L x k^2 dictionary, Phi_i the pixel's L coefficients and B_i
 * the k x k neighbourhood of the up-sampled LR image centred on pixel i
 * (stage 1).  The patch matrix B and the filter matrix F of Eq. 3 are never
 * written to memory: one fused kernel up-samples, folds and filters.
 *
 * Fixed semantics (the paper leaves them open; every workload uses these):
 *   - up-sampling is separable cubic convolution (Keys), a = -0.5, half-pixel
 *     centres (source coordinate (Y + 0.5)/scale - 0.5), LR indices clamped;
 *   - patch taps outside the HR image read the nearest pixel of the
 *     up-sampled image (replicate padding of the up-sampled image);
 *   - tap j = dy*k + dx of F_i multiplies U[Y + dy - r][X + dx - r],
 *     r = (k-1)/2: a correlation, no flip;
 *   - the same coefficients are applied to every image channel;
 *   - no clamping or rounding of intermediate values; arithmetic is fp32
 *     (fp16 and fp8 coefficients enter matrix-core products exactly,
 *     accumulation is fp32).
 *
 * All tensors are contiguous NCHW in DEVICE memory, allocated, owned and freed
 * by the caller.  The library allocates nothing, is re-entrant, and keeps nothing
 * between calls but what it has asked the device once (its number of compute
 * units and the rate of its constant clock, per host thread).  Work is enqueued on `stream` and the call returns without
 * synchronising: inputs and outputs must stay valid until the stream reaches
 * the end of the kernel.  `out` must not overlap any input.
 *
 * Every argument check happens on the host before anything is launched.  On
 * error nothing is launched, nothing is written, and a negative status is
 * returned; the library never aborts, throws or prints.
 */
#ifndef SR_DICT_H
#define SR_DICT_H

#ifdef __cplusplus
extern "C" {
#endif

#define SR_VERSION 300           /* major*10000 + minor*100 + patch */
#define SR_MAX_ATOMS 256         /* largest L (and n_kept) accepted   */
#define SR_MAX_CHANNELS 16       /* largest C accepted                */

/* SR_F8E4M3: one byte per value, 1 sign / 4 exponent (bias 7) / 3 mantissa bits,
 * subnormals, no infinities, largest finite 448, 0x7f and 0xff are NaN (the OCP
 * 8-bit "E4M3" format).  Accepted for the coefficient tensor only: a storage
 * format that halves the stream again; it is widened exactly before use.
 * SR_BF16: two bytes per value, the upper half of an IEEE binary32 (1 sign / 8 exponent /
 * 7 mantissa bits).  Accepted for the coefficient tensor only: what a network that runs in
 * bfloat16 produces, taken as it is (no conversion pass over the 1.2 GB of a 4K frame).
 * SR_U8: unsigned bytes; the atom indices of sr_dict_assemble_list only. */
typedef enum { SR_F32 = 0, SR_F16 = 1, SR_F8E4M3 = 2, SR_BF16 = 3, SR_U8 = 4 } sr_dtype;

/* Contiguous NCHW tensor in device memory. */
typedef struct {
    void*    data;
    sr_dtype dtype;
    int      n, c, h, w;
} sr_tensor;

typedef enum {
    SR_OK              =  0,
    SR_ERR_NULL        = -1,   /* a required pointer is NULL                      */
    SR_ERR_SHAPE       = -2,   /* descriptor sizes disagree with L/k/scale/channels */
    SR_ERR_UNSUPPORTED = -3,   /* even k, k not in {3,5,7}, scale not in {2,3,4},
                                  L or C over the maximum, dtype mix not built     */
    SR_ERR_ALIAS       = -4,   /* out overlaps an input                            */
    SR_ERR_KEPT        = -5,   /* kept list empty, too long, out of range or with
                                  a repeated index                                 */
    SR_ERR_LAUNCH      = -6,   /* the HIP runtime refused the launch               */
    SR_ERR_ALIGN       = -7,   /* a data pointer is not aligned to its element     */
    SR_ERR_SCRATCH     = -8    /* the call needs more scratch than the library's
                                  built-in buffer holds (sr_atom_gram_static)      */
} sr_status;

/* Kernel choice for sr_dict_assemble_ex. */
typedef enum {
    SR_KERNEL_AUTO    = 0,     /* the library picks                                */
    SR_KERNEL_GENERIC = 1,     /* fp32 vector-ALU kernel: every supported case      */
    SR_KERNEL_MFMA    = 2      /* matrix-core kernel (fp16 and fp8 coefficients on
                                  fp16 MFMA, fp32 coefficients on fp32 MFMA); the call
                                  fails with SR_ERR_UNSUPPORTED if the case does
                                  not qualify (see sr_dict_assemble_ex)            */
} sr_kernel;

/* How `coeff` is laid out (sr_options.coeff_layout). */
typedef enum {
    SR_COEFF_PLANAR      = 0,  /* [N][L][s*h][s*w]: one HR plane per atom          */
    SR_COEFF_PRE_SHUFFLE = 1,  /* [N][L*s*s][h][w]: what the coefficient network
                                  holds BEFORE its pixel-shuffle layer (section
                                  II-B, stage 2); channel l*s*s + i*s + j carries
                                  atom l at HR pixels (y*s + i, x*s + j)           */
    SR_COEFF_PIXEL_MAJOR = 2,  /* [N][s*h][s*w][L]: the L coefficients of a pixel
                                  side by side (what a producer that keeps its
                                  tensors channels-last writes); a storage order
                                  beyond the paper, same values, same result.  The
                                  descriptor keeps c = L, h = s*h, w = s*w.        */
    SR_COEFF_BLOCKED     = 3   /* the order in which the matrix-core kernel consumes
                                  the coefficients, for a producer willing to write
                                  it (beyond the paper; same values, same result):
                                  [N][s*h][s*w/128][4][piece][2][32][e].  A row is cut
                                  into units of 128 pixels; pixel 4 j + q of a unit is
                                  slot q, column j; a slot holds its 32 pixels' L
                                  atoms as pieces of 16 atoms, [half][j][8 atoms]:
                                  atom 16 piece + 8 half + e, and, if L % 16 == 8, a
                                  last piece [half][j][4 atoms]: atom 16 (L/16) +
                                  4 half + e.  Needs L % 8 == 0 and s*w % 128 == 0.
                                  The descriptor keeps c = L, h = s*h, w = s*w.     */
} sr_coeff_layout;

/* What the stored `coeff` values are (sr_options.coeff_kind). */
typedef enum {
    SR_COEFF_VALUES = 0,       /* the coefficients Phi themselves                  */
    SR_COEFF_LOGITS = 1        /* logits z: the coefficients are their per-pixel
                                  softmax over the L atoms, applied by the call.
                                  An extension beyond the paper (its coefficient
                                  network, section II-B stage 2, hands over Phi):
                                  for a producer whose last layer would be that
                                  normalisation, it saves a pass that reads and
                                  writes the whole tensor.                         */
} sr_coeff_kind;

typedef struct {
    int kernel;                /* sr_kernel                                        */
    int tile;                  /* matrix-core kernel tile shape index, 0 = the
                                  library's default for the frame; see
                                  sr_dict_assemble_tile                            */
    int coeff_layout;          /* sr_coeff_layout                                  */
    int coeff_kind;            /* sr_coeff_kind                                    */
    int reserved[4];           /* must be zero                                     */
} sr_options;

/*
 * Dense dictionary assembly (Eq. 2 / Eq. 3 with stage 1 fused in).
 *
 *   lr     [N][C][h][w]            f32 or f16   LR image x
 *   coeff  [N][L][s*h][s*w]        f32, f16, bf16 or f8e4m3   Phi, one plane per atom
 *   dict   [1][L][k][k]            f32          D, row-major taps
 *   out    [N][C][s*h][s*w]        same dtype as lr; written
 *   L, k, scale, channels          must equal coeff->c, dict->h (= dict->w),
 *                                  the HR/LR size ratio and lr->c
 *   stream hipStream_t, NULL = the default stream
 *
 * Supported: k in {3,5,7}; scale in {2,3,4}; 1 <= L <= SR_MAX_ATOMS;
 * 1 <= C <= SR_MAX_CHANNELS; N >= 0 (N = 0 or an empty image is a no-op
 * returning SR_OK).  With f16 or f8 coefficients the dictionary entries must
 * be finite in fp16 (|D| < 65504); f8 NaN codes give unspecified results.
 */
int sr_dict_assemble(const sr_tensor* lr, const sr_tensor* coeff, const sr_tensor* dict,
                     int L, int k, int scale, int channels,
                     sr_tensor* out, void* stream);

/*
 * Dictionary-selective assembly (section III-A: atoms whose selector beta_i is
 * zero are ignored; Eq. 9: kept atoms may carry a regression scale gamma).
 * Same nine leading arguments as sr_dict_assemble, `coeff` still holds all L
 * planes, but only the listed planes are read:
 *
 *     F_i = sum over j < n_kept of gamma[j] * Phi_i[kept[j]] * D[kept[j]]
 *
 *   kept   HOST array of n_kept distinct atom indices in [0, L), any order
 *   gamma  HOST array of n_kept scales, or NULL for all ones
 * Both arrays are copied before the call returns.
 */
int sr_dict_assemble_selective(const sr_tensor* lr, const sr_tensor* coeff, const sr_tensor* dict,
                               int L, int k, int scale, int channels,
                               sr_tensor* out, void* stream,
                               const int* kept, int n_kept, const float* gamma);

/*
 * As sr_dict_assemble_selective (kept == NULL means dense), with an explicit
 * kernel choice; `opts` == NULL means SR_KERNEL_AUTO.  The matrix-core kernel
 * qualifies when C is 1 or 3 (or 2 or 4 with f16 or bf16 coefficients and k = 5),
 * the tensors are small enough for 32-bit byte offsets (L*H*W*sizeof(coeff)
 * < 2^32, C*H*W < 2^30; with k = 5, C = 3 and f16 or bf16 coefficients an image of up
 * to 2^32 coefficients, e.g. an 8K frame with 72 planes, also qualifies: element
 * offsets), the HR width is a whole number of pixel groups (4
 * pixels; 2 for f32 coefficients and for f16 / bf16 coefficients with k = 7) or at
 * least 128, and
 *   f16 and bf16 coefficients: at most 128 folded atoms (k = 5, C = 2 or 4: 72);
 *   f32 coefficients: at most 128 folded atoms; k = 7: 17 to 128;
 *   f8  coefficients: as f32, and lr->data 4-byte aligned with an even number of
 *                     elements if the image is f16;
 *   images beyond 4 GB of coefficients (element offsets): at most 72 folded atoms.
 * Every other supported case runs on the generic kernel.
 *
 * opts->coeff_layout = SR_COEFF_PRE_SHUFFLE: `coeff` is the tensor the coefficient network
 * produces before its final pixel-shuffle, [N][L*s*s][h][w] (so coeff->c = L*scale*scale and
 * coeff->h, coeff->w are the LR sizes); the call gives exactly the result of shuffling it to
 * [N][L][s*h][s*w] first, without that 2 x (L * H * W) byte pass over memory.  Every kernel
 * takes it; the matrix-core kernel for k = 5, C = 3, f16 coefficients with up to 8 or 65 to 72
 * folded atoms, or bf16 coefficients with 65 to 72 and an LR width that is a multiple of 4 (byte
 * offsets), the generic kernel otherwise.
 *
 * opts->coeff_layout = SR_COEFF_PIXEL_MAJOR: `coeff` is stored [N][s*h][s*w][L] (described with
 * c = L, h = s*h, w = s*w as for the planar order).  A wavefront's row of 128 pixels is then one
 * contiguous piece of memory.  Every kernel takes it; the matrix-core kernel for k = 5, C = 3, all
 * of L = 72 f16 atoms (no kept list), an HR width that is a multiple of 128 and under 4 GB of
 * coefficients per image, the generic kernel otherwise.
 *
 * opts->coeff_layout = SR_COEFF_BLOCKED: see sr_coeff_layout; L % 8 != 0 or an HR width that is not a multiple of 128 is
 * SR_ERR_UNSUPPORTED.  A unit's 128 L coefficients are contiguous and every 16 bytes of it are a matrix-core operand of the
 * lane that loads them: no re-packing, no staging.  Every kernel takes it; the matrix-core kernel for k = 5, C = 3, all of
 * L = 72 f16, bf16 or f8 atoms, or f16 logits (no kept list), and under 4 GB of coefficients per image, the generic kernel otherwise.
 *
 * opts->coeff_kind = SR_COEFF_LOGITS: `coeff` holds logits z (f32, f16 or bf16; any layout above) and the call
 * computes, per pixel and over all L atoms,
 *     m = max_l z_l,   e_l = exp(z_l - m) rounded to the nearest binary16 value,   Phi_l = e_l / sum_l e_l
 * and then the assembly with these Phi: F_i = (sum_l e_l D_l) / (sum_l e_l).  The rounding is where the
 * exponentials become 16-bit operands of the fold, as stored f16 coefficients would be; the sum runs over the
 * rounded values, so a pixel's coefficients add up to one.  The exponential is evaluated in fp32 by the hardware
 * (about one unit in the last place), so a value that lies next to a rounding boundary may round the other way
 * than in exact arithmetic: one binary16 step in one coefficient.  A kept list or gamma is SR_ERR_UNSUPPORTED
 * (the normalisation needs every atom), and so are f8 logits.  Logits of -infinity give a zero coefficient;
 * NaN or +infinity logits give unspecified results.  The matrix-core kernel takes k = 5, C = 3, 49 to 72
 * f16 or bf16 atoms in the planar order or (LR width a multiple of 4) in the order before the pixel-shuffle, under 4 GB
 * per image; the generic kernel everything else.
 *
 * opts->tile (the launch-shape search of section III-B, Eq. 11-12, as a small set of compiled
 * tile shapes): index 0 is the library's default for the frame and is always accepted.  Other
 * indices exist only where alternative shapes are built - k = 5, C = 3, 65 to 72 folded f16
 * atoms, byte offsets: 1 = 64x8, 2 = 128x4, 3 = 64x16, 4 = 128x8, 5 = 64x32, 6 = 128x16,
 * 7 = 128x24 (scale 4 only) HR pixels per workgroup, i.e. 1, 1, 2, 2, 4, 4, 6 row groups per
 * wavefront of a four-wavefront workgroup, two workgroups per CU; 8 = 128x16 as one workgroup of
 * eight wavefronts per CU; 9 = 128x16 as two workgroups of two wavefronts, one wavefront per SIMD
 * (see sr_dict_assemble_launch_shape) - and are an option of the matrix-core kernel: with SR_KERNEL_AUTO or
 * SR_KERNEL_MFMA an index the case does not have is SR_ERR_UNSUPPORTED, never a silent
 * fall-back, so a sweep over the indices times each accepted one as a different kernel.
 */
int sr_dict_assemble_ex(const sr_tensor* lr, const sr_tensor* coeff, const sr_tensor* dict,
                        int L, int k, int scale, int channels,
                        sr_tensor* out, void* stream,
                        const int* kept, int n_kept, const float* gamma,
                        const sr_options* opts);

/*
 * Stage 1 alone (section II-B, stage 1): the up-sampled image U that the
 * patches B_i are cut from.
 *   lr [N][C][h][w] f32|f16  ->  out [N][C][scale*h][scale*w], dtype f32 or
 *   the dtype of lr.  The values are bit-identical to the ones the fused
 *   kernels use internally (before any narrowing to an f16 `out`).
 */
int sr_bicubic_upsample(const sr_tensor* lr, int scale, int channels,
                        sr_tensor* out, void* stream);

/*
 * Coefficients as per-pixel lists - AN EXTENSION, NOT IN THE PAPER.  The paper compresses the
 * dictionary once for the whole model (section III-A); its bandwidth argument (section II-A, Eq. 4:
 * what is skipped should not be loaded) also holds per pixel: a pixel's few dominant atoms carry
 * almost all of its coefficient mass.  Here every HR pixel brings `entries` pairs (atom index,
 * value), 3 bytes each with f16 values, instead of L dense coefficients:
 *
 *     F_i = sum over t < entries of value[t][i] * D[index[t][i]]           y_i = F_i B_i^T
 *
 *   index  [N][entries][s*h][s*w]  SR_U8        atom numbers, each below L and, within a pixel, all
 *                                               different (else: unspecified values at that pixel,
 *                                               never an access outside the dictionary)
 *   value  [N][entries][s*h][s*w]  f32 or f16   their coefficients; nothing is renormalised
 *   lr, dict, out, L, k, scale, channels, stream as for sr_dict_assemble; 1 <= entries <= SR_MAX_ATOMS.
 * Same statuses and rules as sr_dict_assemble (all checks on the host, one launch, no allocation).
 */
int sr_dict_assemble_list(const sr_tensor* lr, const sr_tensor* index, const sr_tensor* value,
                          const sr_tensor* dict, int L, int k, int scale, int channels, int entries,
                          sr_tensor* out, void* stream);

/* The same with an explicit kernel choice (sr_kernel).  The matrix-core kernel takes k = 5, C = 3,
 * f16 values, L <= 128, entries <= 16, an HR width that is a multiple of 4 and, for a pixel, atoms
 * that are all different (an atom listed twice, or an index >= L, gives unspecified values there;
 * the gather kernel, SR_KERNEL_GENERIC, adds repeated atoms as the definition above says). */
int sr_dict_assemble_list_ex(const sr_tensor* lr, const sr_tensor* index, const sr_tensor* value,
                             const sr_tensor* dict, int L, int k, int scale, int channels, int entries,
                             sr_tensor* out, void* stream, int kernel);

/* Which kernel sr_dict_assemble_ex would run for these arguments
 * (SR_KERNEL_GENERIC or SR_KERNEL_MFMA), or a negative sr_status.  Launches
 * nothing. */
int sr_dict_assemble_plan(const sr_tensor* lr, const sr_tensor* coeff, const sr_tensor* dict,
                          int L, int k, int scale, int channels,
                          const sr_tensor* out,
                          const int* kept, int n_kept, const sr_options* opts);

/* As sr_dict_assemble_plan, and also reports the tile (HR pixels per workgroup) of the
 * matrix-core instantiation that would run: *tile_w x *tile_h, or 0 x 0 where the library
 * does not report it (generic kernel; families with a single built shape).  Host only. */
int sr_dict_assemble_tile(const sr_tensor* lr, const sr_tensor* coeff, const sr_tensor* dict,
                          int L, int k, int scale, int channels,
                          const sr_tensor* out,
                          const int* kept, int n_kept, const sr_options* opts,
                          int* tile_w, int* tile_h);

/* The whole launch shape an index stands for (section III-B: the paper searches block size and
 * occupancy together, Eq. 11-12): shape[0] x shape[1] = the tile as above, shape[2] = wavefronts per
 * workgroup, shape[3] = workgroups resident per CU; zeros where the library does not report it.
 * Two indices never name the same four numbers.  Host only. */
int sr_dict_assemble_launch_shape(const sr_tensor* lr, const sr_tensor* coeff, const sr_tensor* dict,
                                  int L, int k, int scale, int channels,
                                  const sr_tensor* out,
                                  const int* kept, int n_kept, const sr_options* opts,
                                  int shape[4]);

/* Static, NUL-terminated description of a status code. */
const char* sr_strerror(int status);

/* SR_VERSION of the built library. */
int sr_version(void);

#ifdef __cplusplus
}
#endif
#endif /* SR_DICT_H */
