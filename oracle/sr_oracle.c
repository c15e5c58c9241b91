/*
 * sr_oracle.c -- TEST INFRASTRUCTURE, NOT THE PRODUCT.
 *
 * A plain, slow, double-precision CPU statement of what the pixel-adaptive
 * dictionary-assembly path computes.  Only the tests, the smoke check and the
 * benchmark's CPU-baseline leg may call it.  It shares no code, table or
 * constant with the HIP library and the HIP library never calls it.
 *
 * What is computed (paper section II-A, Eq. 2 and Eq. 3; stages 1, 3 and 4 of
 * the four-stage inference flow in section II-B):
 *
 *   stage 1   U = upsample(x)             the upsampled LR image; row i of the
 *                                         patch matrix B is the k x k window of
 *                                         U centred on HR pixel i
 *   stage 3   F_i = Phi_i D               per-pixel filter from L atoms
 *   stage 4   y_i = F_i B_i^T             dot product of filter and patch
 *
 * and the compressed-dictionary form of section III-A: atoms whose selector
 * beta is zero are ignored, kept atoms may carry a regression scale gamma
 * (Eq. 5, Eq. 9).
 *
 * Readings taken where the paper is silent (all are this build's choices):
 *   - the upsampler is the separable Keys cubic-convolution interpolator with
 *     parameter a (a = -0.5 in every workload), half-pixel centres
 *     (source coordinate (Y + 0.5)/s - 0.5) and replicated LR borders;
 *   - a patch tap that falls outside the HR image reads the nearest HR pixel
 *     of U (U is replicate-padded, the interpolator is not extrapolated);
 *   - the dot product is a correlation: tap j = dy*k + dx multiplies
 *     U[Y + dy - r][X + dx - r], r = (k-1)/2, no flip;
 *   - the same coefficients serve every image channel;
 *   - nothing is clamped or rounded on the way.
 *
 * Every function is the definition written out; there is no blocking, fusion
 * or reordering.  Rows may be split over OpenMP threads (each output element
 * is still computed by the same sequence of operations).
 *
 * Parity pins (tests/test_oracle_*.py): exact rational phase weights, quadratic
 * reproduction (fixes a = -0.5 and the coordinate convention), a library
 * bicubic at that library's own a, delta atoms, linearity, constant
 * preservation, an exact-rational apply-then-weight evaluator, a library
 * unfold + einsum for stages 3 + 4; the 8-bit E4M3 decoder by hand-computed
 * codes and a library decoder over all 256 codes (tests/test_oracle_fp8.py), the
 * bfloat16 decoder likewise over all 65536 codes (tests/test_oracle_bf16.py); the
 * pixel-shuffle by a hand-written example, by a library routine and by the index
 * identity it is defined by (tests/test_oracle_shuffle.py); the per-pixel list form
 * by the pinned dense form on the scattered list, hand-made lists, repeated entries
 * and linearity (tests/test_oracle_topk.py); the blocked storage order by hand-worked positions, a library's
 * reshape and axis move, and the whole path (tests/test_oracle_blocked.py); the logits form by a hand-made example with exact
 * values, a closed form (logarithms of integers), two libraries' softmax, the library's binary16
 * cast for the rounding, shift invariance and large logits (tests/test_oracle_logits.py).
 * No function here is unpinned.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORC_F32 = 0, ORC_F16 = 1, ORC_F64 = 2, ORC_F8E4M3 = 3, ORC_BF16 = 4 };

/* IEEE binary16 bit pattern -> double, exactly (subnormals, inf, nan). */
double orc_half_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int e = (h >> 10) & 0x1f;
    int m = h & 0x3ff;
    double v;
    if (e == 0)
        v = ldexp((double)m, -24);
    else if (e == 31)
        v = m ? NAN : INFINITY;
    else
        v = ldexp((double)(m + 1024), e - 25);
    return sign ? -v : v;
}

/*
 * 8-bit float "E4M3" (1 sign, 4 exponent bits with bias 7, 3 mantissa bits;
 * exponent field 0 holds subnormals m * 2^-9; there are no infinities, the
 * all-ones magnitude 0x7f is NaN, the largest finite value is 1.75 * 2^8 = 448)
 * -> double, exactly.  A storage format for coefficients only (an extension of
 * the paper's "do not move what you do not need", section III-A): the path
 * computes with the widened value.
 */
double orc_e4m3_to_double(uint8_t b)
{
    int sign = (b >> 7) & 1;
    int e = (b >> 3) & 0xf;
    int m = b & 0x7;
    double v;
    if (e == 15 && m == 7)
        v = NAN;
    else if (e == 0)
        v = ldexp((double)m, -9);
    else
        v = ldexp((double)(m + 8), e - 10);
    return sign ? -v : v;
}

/*
 * bfloat16 (1 sign, 8 exponent bits with bias 127, 7 mantissa bits: the upper
 * half of an IEEE binary32, so exponent field 0 holds subnormals m * 2^-133 and
 * 255 infinities and NaNs) -> double, exactly.  A storage format for
 * coefficients only: what a network that runs in bfloat16 produces.
 */
double orc_bf16_to_double(uint16_t b)
{
    int sign = (b >> 15) & 1;
    int e = (b >> 7) & 0xff;
    int m = b & 0x7f;
    double v;
    if (e == 0)
        v = ldexp((double)m, -133);
    else if (e == 255)
        v = m ? NAN : INFINITY;
    else
        v = ldexp((double)(m + 128), e - 134);
    return sign ? -v : v;
}

static double load_elem(const void *p, int dtype, size_t i)
{
    switch (dtype) {
    case ORC_F32: return (double)((const float *)p)[i];
    case ORC_F16: return orc_half_to_double(((const uint16_t *)p)[i]);
    case ORC_F8E4M3: return orc_e4m3_to_double(((const uint8_t *)p)[i]);
    case ORC_BF16: return orc_bf16_to_double(((const uint16_t *)p)[i]);
    default:      return ((const double *)p)[i];
    }
}

static long clampl(long v, long lo, long hi)
{
    return v < lo ? lo : (v > hi ? hi : v);
}

/* Keys cubic convolution kernel with free parameter a. */
double orc_keys(double t, double a)
{
    t = fabs(t);
    if (t <= 1.0)
        return (a + 2.0) * t * t * t - (a + 3.0) * t * t + 1.0;
    if (t < 2.0)
        return a * t * t * t - 5.0 * a * t * t + 8.0 * a * t - 4.0 * a;
    return 0.0;
}

/*
 * Source position of HR index Y at scale s: first tap index (floor - 1) and the
 * four weights for taps floor-1 .. floor+2.
 */
void orc_taps(long Y, int s, double a, long *first, double w[4])
{
    double src = ((double)Y + 0.5) / (double)s - 0.5;
    double fl = floor(src);
    double t = src - fl;
    *first = (long)fl - 1;
    w[0] = orc_keys(1.0 + t, a);
    w[1] = orc_keys(t, a);
    w[2] = orc_keys(1.0 - t, a);
    w[3] = orc_keys(2.0 - t, a);
}

/* One upsampled value U[n][c][Y][X] (stage 1). */
static double bicubic_at(const void *lr, int dtype, int c_total, int h, int w,
                         int s, double a, int n, int c, long Y, long X)
{
    long fy, fx;
    double wy[4], wx[4];
    orc_taps(Y, s, a, &fy, wy);
    orc_taps(X, s, a, &fx, wx);
    size_t plane = ((size_t)n * c_total + c) * (size_t)h * w;
    double acc = 0.0;
    for (int i = 0; i < 4; ++i) {
        long yy = clampl(fy + i, 0, h - 1);
        for (int j = 0; j < 4; ++j) {
            long xx = clampl(fx + j, 0, w - 1);
            acc += wy[i] * wx[j] * load_elem(lr, dtype, plane + (size_t)yy * w + xx);
        }
    }
    return acc;
}

/*
 * Stage 1 for a whole batch.  lr: [n][c][h][w] of lr_dtype; U: [n][c][s*h][s*w]
 * double, written.  Returns 0, or -1 on a bad argument.
 */
int orc_bicubic(const void *lr, int lr_dtype, int n, int c, int h, int w,
                int s, double a, double *U)
{
    if (!lr || !U || n < 0 || c < 1 || h < 1 || w < 1 || s < 1)
        return -1;
    long H = (long)s * h, W = (long)s * w;
#pragma omp parallel for collapse(2) schedule(static)
    for (long nc = 0; nc < (long)n * c; ++nc)
        for (long Y = 0; Y < H; ++Y)
            for (long X = 0; X < W; ++X)
                U[((size_t)nc * H + Y) * W + X] =
                    bicubic_at(lr, lr_dtype, c, h, w, s, a,
                               (int)(nc / c), (int)(nc % c), Y, X);
    return 0;
}

/* Stage 3 for one pixel: F[j] = sum over kept atoms of gamma * Phi * D. */
static void fold_pixel(const void *coeff, int cdtype, size_t pix_base,
                       size_t plane_stride, int L, const double *dict, int kk,
                       const int *kept, int n_kept, const double *gamma,
                       double *F)
{
    for (int j = 0; j < kk; ++j)
        F[j] = 0.0;
    int count = kept ? n_kept : L;
    for (int i = 0; i < count; ++i) {
        int l = kept ? kept[i] : i;
        double phi = load_elem(coeff, cdtype, pix_base + (size_t)l * plane_stride);
        if (gamma)
            phi *= gamma[i];
        for (int j = 0; j < kk; ++j)
            F[j] += phi * dict[(size_t)l * kk + j];
    }
}

/* Stage 4 for one pixel and one channel plane of U. */
static double apply_pixel(const double *Uplane, long H, long W, long Y, long X,
                          const double *F, int k)
{
    int r = (k - 1) / 2;
    double acc = 0.0;
    for (int dy = 0; dy < k; ++dy) {
        long yy = clampl(Y + dy - r, 0, H - 1);
        for (int dx = 0; dx < k; ++dx) {
            long xx = clampl(X + dx - r, 0, W - 1);
            acc += F[dy * k + dx] * Uplane[(size_t)yy * W + xx];
        }
    }
    return acc;
}

static int check_kept(const int *kept, int n_kept, int L)
{
    if (!kept)
        return 0;
    if (n_kept < 0)
        return -1;
    for (int i = 0; i < n_kept; ++i)
        if (kept[i] < 0 || kept[i] >= L)
            return -1;
    return 0;
}

/*
 * Stages 3 + 4 on HR rows [y0, y1) of every image of the batch.
 *   U      [n][c][H][W] double  (stage-1 result)
 *   coeff  [n][L][H][W] of coeff_dtype
 *   dict   [L][k][k] double
 *   kept   NULL (all L atoms, in order) or n_kept atom indices
 *   gamma  NULL (all 1) or one scale per listed atom
 *   out    [n][c][H][W] double; only rows [y0, y1) are written
 */
int orc_assemble_rows(const double *U, int n, int c, int H, int W,
                      const void *coeff, int coeff_dtype, int L,
                      const double *dict, int k,
                      const int *kept, int n_kept, const double *gamma,
                      int y0, int y1, double *out)
{
    if (!U || !coeff || !dict || !out || k < 1 || (k % 2) == 0 || k > 15 ||
        L < 1 || c < 1 || H < 1 || W < 1 || n < 0 || y0 < 0 || y1 > H ||
        check_kept(kept, n_kept, L))
        return -1;
    int kk = k * k;
    size_t plane = (size_t)H * W;
#pragma omp parallel for collapse(2) schedule(static)
    for (int b = 0; b < n; ++b)
        for (int Y = y0; Y < y1; ++Y) {
            double F[225];
            for (int X = 0; X < W; ++X) {
                size_t pix = (size_t)b * L * plane + (size_t)Y * W + X;
                fold_pixel(coeff, coeff_dtype, pix, plane, L, dict, kk,
                           kept, n_kept, gamma, F);
                for (int ch = 0; ch < c; ++ch)
                    out[(((size_t)b * c + ch) * H + Y) * W + X] =
                        apply_pixel(U + ((size_t)b * c + ch) * plane, H, W, Y, X, F, k);
            }
        }
    return 0;
}

/*
 * Stages 3 + 4 at listed HR pixels.  pts: n_pts triples (image, Y, X);
 * out: [n_pts][c] double.
 */
int orc_assemble_points(const double *U, int n, int c, int H, int W,
                        const void *coeff, int coeff_dtype, int L,
                        const double *dict, int k,
                        const int *kept, int n_kept, const double *gamma,
                        const int *pts, int n_pts, double *out)
{
    if (!U || !coeff || !dict || !out || !pts || k < 1 || (k % 2) == 0 ||
        k > 15 || L < 1 || check_kept(kept, n_kept, L))
        return -1;
    int kk = k * k;
    size_t plane = (size_t)H * W;
    for (int p = 0; p < n_pts; ++p) {
        int b = pts[3 * p], Y = pts[3 * p + 1], X = pts[3 * p + 2];
        if (b < 0 || b >= n || Y < 0 || Y >= H || X < 0 || X >= W)
            return -1;
        double F[225];
        size_t pix = (size_t)b * L * plane + (size_t)Y * W + X;
        fold_pixel(coeff, coeff_dtype, pix, plane, L, dict, kk, kept, n_kept, gamma, F);
        for (int ch = 0; ch < c; ++ch)
            out[(size_t)p * c + ch] =
                apply_pixel(U + ((size_t)b * c + ch) * plane, H, W, Y, X, F, k);
    }
    return 0;
}

/*
 * Stages 3 + 4 for coefficients stored as a per-pixel list of T (atom index, value) entries
 * instead of L dense planes.  AN EXTENSION, NOT IN THE PAPER: the paper selects atoms globally
 * (section III-A); this format carries a selection per pixel, following its argument that what
 * is skipped should not be loaded (section II-A, Eq. 4).  What is computed is Eq. 2 with the
 * listed terms only, nothing renormalised:
 *
 *     F_i = sum over t < T of value[t][i] * D[index[t][i]]          y_i = F_i B_i^T
 *
 * index: [n][T][H][W] bytes (each < L; an atom listed twice counts twice); value: [n][T][H][W] in
 * value_dtype; rows y0 <= Y < y1 of out [n][c][H][W] are written.
 */
int orc_assemble_topk_rows(const double *U, int n, int c, int H, int W,
                           const uint8_t *index, const void *value, int value_dtype, int T, int L,
                           const double *dict, int k, int y0, int y1, double *out)
{
    if (!U || !index || !value || !dict || !out || k < 1 || (k % 2) == 0 || k > 15 ||
        L < 1 || L > 256 || T < 1 || c < 1 || H < 1 || W < 1 || n < 0 || y0 < 0 || y1 > H)
        return -1;
    int kk = k * k;
    size_t plane = (size_t)H * W;
    int bad = 0;
#pragma omp parallel for collapse(2) schedule(static)
    for (int b = 0; b < n; ++b)
        for (int Y = y0; Y < y1; ++Y) {
            double F[225];
            for (int X = 0; X < W; ++X) {
                for (int j = 0; j < kk; ++j)
                    F[j] = 0.0;
                for (int t = 0; t < T; ++t) {
                    size_t at = ((size_t)b * T + t) * plane + (size_t)Y * W + X;
                    int l = index[at];
                    if (l >= L) {
                        bad = 1;
                        continue;
                    }
                    double v = load_elem(value, value_dtype, at);
                    for (int j = 0; j < kk; ++j)
                        F[j] += v * dict[(size_t)l * kk + j];
                }
                for (int ch = 0; ch < c; ++ch) {
                    const double *Uplane = U + ((size_t)b * c + ch) * plane;
                    out[(((size_t)b * c + ch) * H + Y) * W + X] = apply_pixel(Uplane, H, W, Y, X, F, k);
                }
            }
        }
    return bad ? -2 : 0;
}

/*
 * Pixel-shuffle of a coefficient tensor (paper section II-B, stage 2: the coefficient network
 * ends in a pixel-shuffle layer; what it holds before that layer is [n][L*s*s][h][w] at LR
 * resolution).  Moves stored elements, of `esize` bytes each, without looking at them:
 *
 *     out[b][l][y*s + i][x*s + j] = in[b][l*s*s + i*s + j][y][x]      0 <= i, j < s
 *
 * so channel l*s*s + i*s + j of the LR-resolution tensor holds the coefficients of atom l at
 * the HR pixels whose row is i and whose column is j modulo s.  `out` is [n][L][h*s][w*s].
 */
int orc_pixel_shuffle(const void *in, int esize, int n, int L, int h, int w, int s, void *out)
{
    if (!in || !out || esize < 1 || esize > 8 || n < 0 || L < 1 || h < 0 || w < 0 || s < 1)
        return -1;
    const unsigned char *src = (const unsigned char *)in;
    unsigned char *dst = (unsigned char *)out;
    size_t H = (size_t)h * s, W = (size_t)w * s;
    for (int b = 0; b < n; ++b)
        for (int l = 0; l < L; ++l)
            for (int i = 0; i < s; ++i)
                for (int j = 0; j < s; ++j)
                    for (int y = 0; y < h; ++y)
                        for (int x = 0; x < w; ++x) {
                            size_t from = ((((size_t)b * L + l) * s + i) * s + j) * ((size_t)h * w) + (size_t)y * w + x;
                            size_t to = ((size_t)b * L + l) * (H * W) + ((size_t)y * s + i) * W + ((size_t)x * s + j);
                            memcpy(dst + to * esize, src + from * esize, (size_t)esize);
                        }
    return 0;
}

/*
 * Coefficients stored pixel-major (an extension of the storage formats, not in the paper: what a producer
 * that keeps its tensors channels-last writes): in[b][y][x][l] holds the coefficient of atom l at HR pixel
 * (y, x), the L coefficients of a pixel side by side.  Moves the stored elements (esize bytes each) to the
 * planar order every other function here reads:
 *
 *     out[b][l][y][x] = in[b][y][x][l]
 */
int orc_pixel_major_to_planar(const void *in, int esize, int n, int L, int H, int W, void *out)
{
    if (!in || !out || esize < 1 || esize > 8 || n < 0 || L < 1 || H < 0 || W < 0)
        return -1;
    const unsigned char *src = (const unsigned char *)in;
    unsigned char *dst = (unsigned char *)out;
    for (int b = 0; b < n; ++b)
        for (int y = 0; y < H; ++y)
            for (int x = 0; x < W; ++x)
                for (int l = 0; l < L; ++l) {
                    size_t from = (((size_t)b * H + y) * W + x) * L + l;
                    size_t to = (((size_t)b * L + l) * H + y) * W + x;
                    memcpy(dst + to * esize, src + from * esize, (size_t)esize);
                }
    return 0;
}

/*
 * Coefficients stored BLOCKED (an extension of the storage formats, not in the paper: the order in which a
 * matrix-core kernel consumes them, for a producer that is willing to write it).  A row of the HR image is cut
 * into units of 128 pixels; pixel 4 j + q of a unit (0 <= j < 32, 0 <= q < 4) is "slot q, column j".  The stored
 * order is [b][y][unit][q][piece][half][j][e]:
 *   pieces 0 .. L/16 - 1   16 atoms each: atom 16 piece + 8 half + e, 0 <= e < 8
 *   one last piece if L % 16 == 8: atom 16 (L/16) + 4 half + e, 0 <= e < 4
 * so a unit holds 128 L elements and the whole tensor has the size of the planar one.  Needs L % 8 == 0 and
 * W % 128 == 0.  Moves the stored elements (esize bytes each) to the planar order every other function reads:
 *
 *     out[b][l][y][x] = in[b][y][x / 128][x % 4][piece(l)][half(l)][(x % 128) / 4][e(l)]
 */
int orc_blocked_to_planar(const void *in, int esize, int n, int L, int H, int W, void *out)
{
    if (!in || !out || esize < 1 || esize > 8 || n < 0 || L < 8 || L % 8 || H < 0 || W < 0 || W % 128)
        return -1;
    const unsigned char *src = (const unsigned char *)in;
    unsigned char *dst = (unsigned char *)out;
    int full = L / 16;                                     /* pieces of 16 atoms */
    size_t slot_elems = (size_t)32 * L;                    /* one slot: 32 pixels x L atoms */
    for (int b = 0; b < n; ++b)
        for (int y = 0; y < H; ++y)
            for (int x = 0; x < W; ++x)
                for (int l = 0; l < L; ++l) {
                    int unit = x / 128, j = (x % 128) / 4, q = x % 4;
                    size_t within;                         /* position inside the slot */
                    if (l < 16 * full) {
                        int piece = l / 16, half = (l % 16) / 8, e = l % 8;
                        within = (size_t)piece * 512 + (size_t)half * 256 + (size_t)j * 8 + e;
                    } else {
                        int half = (l - 16 * full) / 4, e = (l - 16 * full) % 4;
                        within = (size_t)full * 512 + (size_t)half * 128 + (size_t)j * 4 + e;
                    }
                    size_t from = ((((size_t)b * H + y) * (W / 128) + unit) * 4 + q) * slot_elems + within;
                    size_t to = (((size_t)b * L + l) * H + y) * W + x;
                    memcpy(dst + to * esize, src + from * esize, (size_t)esize);
                }
    return 0;
}

/*
 * A double rounded to the nearest IEEE binary16 value, ties to the even mantissa, as a double
 * (finite |v| < 65520; below 2^-14 the binary16 values are the multiples of 2^-24).
 */
double orc_round_to_half(double v)
{
    if (v == 0.0 || isnan(v) || isinf(v))
        return v;
    int e;
    (void)frexp(fabs(v), &e);                     /* |v| = f * 2^e, 0.5 <= f < 1 */
    int ulp_exp = e - 11;                         /* 11 significant bits */
    if (ulp_exp < -24)
        ulp_exp = -24;                            /* subnormal range: fixed spacing */
    /* v / ulp is exact (a power of two); nearbyint rounds halves to even in the default mode */
    return ldexp(nearbyint(ldexp(v, -ulp_exp)), ulp_exp);
}

/*
 * Coefficients handed over as LOGITS (an extension, not in the paper: the coefficient network of
 * section II-B, stage 2, stops before a normalising last layer and the assembly path applies it).
 * Per pixel, over the L atoms (z_l = stored logit of atom l, any stored type):
 *
 *     m     = max_l z_l
 *     e_l   = exp(z_l - m)          rounded to binary16 if round_half != 0
 *     Phi_l = e_l / sum_l e_l
 *
 * The rounding is the reading taken for this form: the exponentials enter the fold as 16-bit
 * operands, like stored fp16 coefficients would, and the sum is the sum of the rounded values, so
 * the Phi of a pixel still add up to one.  round_half == 0 gives the plain softmax (used to pin
 * this function against a library's).  in: [n][L][H][W] stored values; out: the same shape, double.
 */
int orc_softmax_planes(const void *in, int dtype, int n, int L, int H, int W, int round_half, double *out)
{
    if (!in || !out || n < 0 || L < 1 || H < 0 || W < 0)
        return -1;
    size_t plane = (size_t)H * W;
    for (int b = 0; b < n; ++b) {
#pragma omp parallel for schedule(static)
        for (long p = 0; p < (long)plane; ++p) {
            size_t base = (size_t)b * L * plane + (size_t)p;
            double m = load_elem(in, dtype, base);
            for (int l = 1; l < L; ++l) {
                double z = load_elem(in, dtype, base + (size_t)l * plane);
                if (z > m)
                    m = z;
            }
            double sum = 0.0;
            for (int l = 0; l < L; ++l) {
                double e = exp(load_elem(in, dtype, base + (size_t)l * plane) - m);
                if (round_half)
                    e = orc_round_to_half(e);
                out[base + (size_t)l * plane] = e;
                sum += e;
            }
            for (int l = 0; l < L; ++l)
                out[base + (size_t)l * plane] /= sum;
        }
    }
    return 0;
}

/* Threads the row loops above will use. */
int orc_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Set that number (n >= 1); returns the number now in force.  Timing only: the
 * results do not depend on it. */
int orc_set_threads(int n)
{
#ifdef _OPENMP
    if (n >= 1)
        omp_set_num_threads(n);
#else
    (void)n;
#endif
    return orc_threads();
}
