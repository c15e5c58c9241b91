// Matrix-core kernel (gfx950 / CDNA4).  Described for fp16 coefficients, the
// headline case; fp32 and 8-bit coefficients differ only in stage 3's operand
// handling (end of this comment).
//
// One fused, persistent kernel does stage 1 (up-sampling), stage 3
// (F_i = Phi_i D, paper Eq. 2) and stage 4 (y_i = F_i B_i^T) for tiles of HR
// pixels; neither F nor B of Eq. 3 ever reaches memory.  The only large stream
// is the coefficient tensor Phi (L planes, fp16), read exactly once.
//
// Stage 3 is a (taps x atoms) . (atoms x pixels) product per wavefront:
//
//     A = D^T, rows = filter taps (padded to 32), K = atoms  (constant per launch)
//     B = Phi, K = atoms, columns = 32 pixels                 (streamed from HBM)
//     v_mfma_f32_32x32x16_f16 (+ one v_mfma_f32_32x32x8_f16 when L % 16 == 8)
//
// The dictionary is fp32; it enters as hi + lo fp16 halves (two MFMAs per
// step), so the only rounding left is the one already in the stored fp16
// coefficients; accumulation is fp32.
//
// Lane roles.  Lane (j, hf) = (lane % 32, lane / 32):
//   * as B operand it supplies atoms 8*hf .. 8*hf+7 of a 16-atom step for pixel
//     j, so lanes j and j+32 load different coefficient planes of the SAME
//     pixels: each lane loads PX consecutive pixels of a plane with one vector
//     load and re-packs (atom pair, pixel) with v_perm_b32;
//   * the MFMA result leaves pixel j's taps split over lanes j and j+32
//     (rows 8*(v/4) + 4*hf + v%4).  Dictionary rows are ordered so that half 0
//     owns filter rows 0 .. RH0-1 and half 1 owns rows RH0 .. (one dummy row
//     with zero weights): both halves then use the same LDS offsets, shifted by
//     RH0 tile rows.  Each half filters its taps against the LDS patch tile
//     and the two partial sums are exchanged across the halves.
//
// Software pipeline.  The atom steps are the outer loop and the PX pixel slots
// the inner one, so the registers of a step are free as soon as its MFMAs are
// issued: the same step of the NEXT tile is loaded into them right away.  The
// coefficient loads of tile t+1 are therefore in flight during stage 4 of tile
// t and during the up-sampling of tile t+1; the LR footprint is prefetched one
// tile ahead as well.
//
// The up-sampled tile is stored in LDS column-swizzled, (x % PX) major, so the
// 32 pixels of one MFMA (stride PX in x) read consecutive banks.
//
// Other coefficient types (template argument CT):
//   * CT_F32: 2-atom steps of v_mfma_f32_32x32x2_f32; lane half hf loads plane
//     2*step + hf and the loaded words are the B operand as they are; the
//     dictionary stays fp32, products and sums are true fp32;
//   * CT_F8 (8-bit E4M3 storage): 4 pixels per 4-byte load; the bytes of two planes
//     are paired per pixel with a byte permute and each pair is widened exactly to
//     the fp16 operand word, then the fp16 steps above;
//   * CT_BF16: the fp16 flow with the bfloat16 matrix instructions and the
//     dictionary as two bfloat16 operands;
//   * CT_LIST8 / CT_LIST16 (an extension beyond the paper): no planes, but per-pixel
//     lists of (atom, value) entries, scattered into the B operand through LDS
//     (see the constants below);
//   * CT_LOGIT / CT_LOGIT_BF16 (an extension beyond the paper): the planes hold logits and the
//     softmax over the atoms is part of the operand path (see the constants below).
// Other coefficient layouts (template argument PSM): the planes as the coefficient
// network holds them before its pixel-shuffle layer, pixel-major storage and the blocked
// order that needs no re-packing at all (see the kernel's own comment).
//
// L2 write-back pacing.  The output leaves the CUs as ordinary stores and sits in the XCDs' L2s as dirty lines that
// the L2 writes to memory when it sees fit, interleaved with the read stream; reads and writes that alternate at the
// memory cost more than their bytes (the stores of the 4K frame, 7.6 % of the bytes, cost 22 % of the time).  One
// wavefront per XCD (wavefront 0 of workgroups 0 .. 7, which the dispatcher deals to the eight XCDs) therefore asks
// its L2 every 16 us - by a constant-rate clock, checked once per unit - to write its dirty lines back NOW (an
// agent-scope release fence, which the compiler turns into the L2 write-back instruction and a wait): the writes
// reach memory in bursts and the reads in between run undisturbed.  Measured: 4K frame 254 -> 241 us, the blocked
// order 240 -> 231 us, 1080p 68 -> 65.5 us, sixteen video frames 1.80 -> 1.72 ms, 58 kept atoms 224 -> 215 us; neutral
// at 43 kept atoms and for 720p fp32, 1-2 % slower with fewer atoms and with 8-bit coefficients, which are not bound
// by the stream: those instantiations are launched without it.  The period was swept from 4 to 48 us (8 us and
// less cost time, beyond 32 us the gain fades; sixteen video frames of 7x7 atoms: 1.72 ms at 16 us, 1.69 at 24 to 32,
// hence 28 us there); results are bit-identical.  -DSR_NO_L2_WRITEBACK builds without it.
//
// Measurement builds (python -m paper_2303_08999_amd.build -o other.so -DSR_ABLATE_...): the
// same launch with a part switched off, to see what that part costs.  SR_ABLATE_STORES keeps
// every instruction but never executes the output stores; SR_ABLATE_STAGE1 skips the two
// up-sampling passes (their barriers stay); results are then wrong by construction.
// SR_STORES_WRITE_THROUGH writes the fp32 output of the four-pixel instantiations through the L2
// (agent scope) instead of leaving dirty lines in it; results are unchanged.  The library built
// by default contains none of them.
#pragma once
#include <type_traits>

#include "sr_device.h"
#include "sr_launch.h"

namespace srd {

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x2 __attribute__((ext_vector_type(2)));

// how the coefficients are stored (template argument CT of the kernel)
constexpr int CT_F16 = 0, CT_F32 = 1, CT_F8 = 2, CT_BF16 = 3, CT_LIST8 = 4, CT_LIST16 = 5, CT_LOGIT = 6, CT_LOGIT_BF16 = 7;
// CT_LOGIT: the fp16 planes hold LOGITS (an extension beyond the paper, see sr_options.coeff_kind).  A unit's planes are
// loaded as in the fp16 form; once they are all there the lane takes the maximum of its pixels' logits (packed fp16
// maxima over its half of the planes, then one exchange with the other half), and where the fp16 form re-packs
// (atom pair, pixel) with a byte permute it forms exp2((z - max) log2 e) in fp32 - one mixed-precision
// multiply-add on the stored half and one exponential per value - and packs two of them, rounded to fp16, as the
// operand.  One padding row of the dictionary operand is all ones, so the matrix cores also return the sum of the
// exponentials of every pixel, in both lane halves; stage 4 multiplies its partial sums by the reciprocal.
// CT_LOGIT_BF16: bfloat16 logits.  The exponentials are fp16 operands all the same (11 significant bits, the range
// (0, 1]); a stored value is widened with a shift or a mask before the multiply-add.  The maxima are taken with the
// same packed fp16 instruction on the stored bits: sign, then magnitude bits, order bfloat16 values exactly as they
// order fp16 values, and the patterns that read as fp16 NaNs (bfloat16 magnitudes of 2^121 and up, the infinities
// among them) are passed over, which is what a logit of minus infinity, an atom switched off, asks for.
// CT_LIST8 / CT_LIST16: no dense planes; every pixel brings a list of up to 8 / 16 (atom index, fp16 value)
// entries (an extension beyond the paper, see sr_dict_assemble_list).  Each wavefront owns an LDS scratch
// [group of 8 atoms][32 pixels][8 atoms] fp16, all zero between uses.  Pixel slot by pixel slot it scatters
// the entries of 32 pixels into it (one 2-byte LDS write each; a lane writes only into its own pixel's 16-byte
// pieces, so few writes meet in a bank), reads its pieces back with 16-byte loads - the piece of group
// 2 c + hf is exactly the matrix cores' B operand of 16-atom step c in the dense form - and writes zeros where
// it wrote values.  The fold, the filtering and
// the store then run as for fp16 planes.
constexpr int LIST_MAX_ENTRIES = 16;

// SMIN: smallest scale the instantiation may be launched with.  The LR footprint
// of a tile shrinks with the scale, so an instantiation for scale 4 only needs half
// the LDS for the footprint and the vertical-pass buffer, and can afford a taller
// tile (fewer halo rows up-sampled per output row).
template <int K, int C, int NP8, int PX, int WR, int NW, int NU, int CT = CT_F16, int SMIN = 2, int NSUB = 1, int SWZ = 0>
struct Cfg {
    static constexpr bool F32 = CT == CT_F32, F8 = CT == CT_F8, BF = CT == CT_BF16, LIST = CT == CT_LIST8 || CT == CT_LIST16;
    static constexpr bool LG = CT == CT_LOGIT || CT == CT_LOGIT_BF16, LGB = CT == CT_LOGIT_BF16;
    static constexpr int LH = CT == CT_LIST8 ? 4 : 8;  // list form: entries a lane half loads
    static constexpr int LSW = 4 * NP8 * 32;           // list form: scratch words per wavefront
    static constexpr int KK = K * K, R = (K - 1) / 2;
    static constexpr int RH0 = (K + 1) / 2;            // filter rows owned by lane half 0
    static constexpr int NSLOT = RH0 * K;              // accumulator rows used per half
    static constexpr int NMB = (NSLOT + 15) / 16;      // 32-row MFMA blocks
    static constexpr int WC = 32 / WR;                 // lane columns per wavefront
    static constexpr int TW = WC * PX * NSUB;          // tile of HR pixels per workgroup: NU units per wavefront, each
    static constexpr int TH = WR * NW * NU / NSUB;     // WR rows of WC * PX pixels; NSUB units share a row (see PSM = 4)
    static_assert(NU % NSUB == 0, "whole rows per wavefront");
    static constexpr int NT = 64 * NW;
    static constexpr int UW = TW + K - 1;
    static constexpr int UH = TH + K;                  // + one dummy row for half 1
    // The tile is stored column-swizzled: column x at (x % SW) * NG + x / SW, so that lanes whose columns are SW
    // apart read consecutive words.  SW = PX, except in the scale-4 pre-shuffle form (NSUB = 2), whose lane pairs
    // are 16 columns apart: with eight classes they step by two words, and the odd NG puts a pair's second lane on
    // the odd banks.
    // SWZ = 1 (pixel-major coefficients): no swizzle, lane j's slots are pixels j, 32 + j, ... of the row.
    static constexpr int SW = SWZ ? SWZ : (NSUB == 2 ? 8 : PX);
    static constexpr int NG = ((UW + SW - 1) / SW) | (NSUB == 2 ? 1 : 0);   // stride between the classes
    static constexpr int P0 = SW * NG;
    // rows of one wavefront must land on disjoint banks: pitch == WC (mod 32)
    static constexpr int P = WR == 1 ? P0 : P0 + ((WC - P0 % 32) + 32) % 32;
    static constexpr int MAXLRY = (UH - 1) / SMIN + 5, MAXLRX = (UW - 1) / SMIN + 5;
    // fp16 coefficients: 16-atom MFMA steps and an optional 8-atom step;
    // fp32 coefficients: 2-atom steps of v_mfma_f32_32x32x2_f32, one load each
    static constexpr int N16 = F32 ? 0 : NP8 / 2, N8 = F32 ? 0 : NP8 % 2;
    static constexpr int N2 = F32 ? 4 * NP8 : 0;
    static constexpr int NLOAD = F32 ? N2 : (LIST ? 1 : 8 * N16 + 4 * N8);   // coefficient loads per lane and unit
    static constexpr int CB = F32 ? 4 : (F8 ? 1 : 2);  // bytes per stored coefficient
    static constexpr int NXC = (MAXLRX + 63) / 64;     // 64-column chunks of the LR footprint
    static constexpr int NLRP = (C * MAXLRY + NW - 1) / NW;   // (channel,row) pairs per wavefront
};

template <int BYTES> struct RawT;      // PX consecutive coefficients of one plane
template <> struct RawT<16> { typedef u32x4 type; };
template <> struct RawT<8> { typedef u32x2 type; };
template <> struct RawT<4> { typedef unsigned type; };

__device__ __forceinline__ unsigned raw_word(const u32x4& v, int m) { return v[m]; }
__device__ __forceinline__ unsigned raw_word(const u32x2& v, int m) { return v[m]; }
__device__ __forceinline__ unsigned raw_word(const unsigned& v, int) { return v; }

// Word m (fp16 pixels 2m, 2m+1) of one plane's raw load.  fp8 (e4m3) coefficients
// are widened here, two at a time; every e4m3 value is exact in fp16.
template <bool F8, int NWORD, typename RawV>
__device__ __forceinline__ void plane_words(const RawV& r, unsigned (&w)[NWORD]) {
    if constexpr (F8) {
        static_assert(NWORD == 2, "fp8 coefficients: four pixels per lane");
        typedef _Float16 h2 __attribute__((ext_vector_type(2)));
        const unsigned bits = raw_word(r, 0);           // four fp8 pixels
        w[0] = __builtin_bit_cast(unsigned, (h2)__builtin_amdgcn_cvt_scalef32_pk_f16_fp8(bits, 1.0f, false));
        w[1] = __builtin_bit_cast(unsigned, (h2)__builtin_amdgcn_cvt_scalef32_pk_f16_fp8(bits, 1.0f, true));
    } else {
#pragma unroll
        for (int m = 0; m < NWORD; ++m) w[m] = raw_word(r, m);
    }
}

// 16- and 8-atom steps of the fold on packed 16-bit operands: fp16, or (BF) bfloat16
template <bool BF>
__device__ __forceinline__ f32x16 mfma_16(const u32x4& a, const u32x4& b, const f32x16& c) {
    if constexpr (BF)
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
}
template <bool BF>
__device__ __forceinline__ f32x16 mfma_8(const u32x2& a, const u32x2& b, const f32x16& c) {
    if constexpr (BF)
        return __builtin_amdgcn_mfma_f32_32x32x8bf16_1k(__builtin_bit_cast(s16x4, a), __builtin_bit_cast(s16x4, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_32x32x8f16(__builtin_bit_cast(f16x4, a), __builtin_bit_cast(f16x4, b), c, 0, 0, 0);
}
// Dictionary values as two 16-bit operands, d ~ hi + lo: 22 significant bits in fp16,
// 16 in bfloat16 (whose coefficients carry 8).
template <bool BF, int N, typename V>
__device__ __forceinline__ void split_hi_lo(const float (&d)[N], V& hi, V& lo) {
    unsigned short h[N], l[N];
#pragma unroll
    for (int j = 0; j < N; ++j) {
        if constexpr (BF) {
            const __bf16 a = (__bf16)d[j];
            const __bf16 b = (__bf16)(d[j] - (float)a);
            h[j] = __builtin_bit_cast(unsigned short, a);
            l[j] = __builtin_bit_cast(unsigned short, b);
        } else {
            const _Float16 a = (_Float16)d[j];
            const _Float16 b = (_Float16)(d[j] - (float)a);
            h[j] = __builtin_bit_cast(unsigned short, a);
            l[j] = __builtin_bit_cast(unsigned short, b);
        }
    }
#pragma unroll
    for (int j = 0; j < N / 2; ++j) {
        hi[j] = (unsigned)h[2 * j] | ((unsigned)h[2 * j + 1] << 16);
        lo[j] = (unsigned)l[2 * j] | ((unsigned)l[2 * j + 1] << 16);
    }
}

// (atom pair, pixel q) from two planes' packed pixels
__device__ __forceinline__ unsigned pack_pair(unsigned plane_even, unsigned plane_odd, int q) {
    return __builtin_amdgcn_perm(plane_odd, plane_even, (q & 1) ? 0x07060302u : 0x05040100u);
}

// 8-bit coefficients: the four pixels of two planes as byte pairs (even plane, odd plane), pixels 0, 1 in w[0] and
// 2, 3 in w[1]; widen_pair then widens the pair of pixel q to the fp16 operand word (every E4M3 value is exact in fp16).
// Six instructions per plane pair where widening every plane first and pairing afterwards takes eight.
template <int NWORD>
__device__ __forceinline__ void pair_bytes(unsigned plane_even, unsigned plane_odd, unsigned (&w)[NWORD]) {
    static_assert(NWORD == 2, "8-bit coefficients: four pixels per lane");
    w[0] = __builtin_amdgcn_perm(plane_odd, plane_even, 0x05010400u);
    w[1] = __builtin_amdgcn_perm(plane_odd, plane_even, 0x07030602u);
}
__device__ __forceinline__ unsigned widen_pair(unsigned pairs, int q) {
    typedef _Float16 h2 __attribute__((ext_vector_type(2)));
    return (q & 1) ? __builtin_bit_cast(unsigned, (h2)__builtin_amdgcn_cvt_scalef32_pk_f16_fp8(pairs, 1.0f, true))
                   : __builtin_bit_cast(unsigned, (h2)__builtin_amdgcn_cvt_scalef32_pk_f16_fp8(pairs, 1.0f, false));
}

// logits form: (atom pair, pixel q) as the exponentials exp2(z * log2(e) + nm) of the two planes' logits, rounded to fp16
// (BF16: the stored logits are bfloat16, the upper half of a binary32)
template <bool BF16>
__device__ __forceinline__ unsigned exp_pair(unsigned plane_even, unsigned plane_odd, int q, float nm) {
    typedef _Float16 h2 __attribute__((ext_vector_type(2)));
    typedef float f2 __attribute__((ext_vector_type(2)));
    auto widen = [&](unsigned w) -> float {
        if constexpr (BF16) return __uint_as_float((q & 1) ? (w & 0xffff0000u) : (w << 16));
        else return (float)__builtin_bit_cast(h2, w)[q & 1];
    };
    const f2 e = {logit_exp(widen(plane_even), nm), logit_exp(widen(plane_odd), nm)};
    return __builtin_bit_cast(unsigned, __builtin_convertvector(e, h2));      // round to nearest even
}
// ... of one word's two logits (blocked order: two atoms of one pixel side by side)
__device__ __forceinline__ unsigned exp_word(unsigned pair, float nm) {
    typedef _Float16 h2 __attribute__((ext_vector_type(2)));
    typedef float f2 __attribute__((ext_vector_type(2)));
    const h2 z = __builtin_bit_cast(h2, pair);
    const f2 e = {logit_exp((float)z[0], nm), logit_exp((float)z[1], nm)};
    return __builtin_bit_cast(unsigned, __builtin_convertvector(e, h2));
}
// packed fp16 maximum of stored values (no canonicalising pass over the operands first)
__device__ __forceinline__ _Float16 __attribute__((ext_vector_type(2))) pk_max_f16(_Float16 __attribute__((ext_vector_type(2))) x,
                                                                                 _Float16 __attribute__((ext_vector_type(2))) y) {
    _Float16 __attribute__((ext_vector_type(2))) r;
    asm("v_pk_max_f16 %0, %1, %2" : "=v"(r) : "v"(x), "v"(y));
    return r;
}

// filter tap served by MFMA row i of block mb, or -1 (padding / dummy row)
template <int K>
__device__ __forceinline__ int tap_of_row(int i, int mb) {
    constexpr int RH0 = (K + 1) / 2, NSLOT = RH0 * K;
    const int half = (i >> 2) & 1;
    const int vv = 16 * mb + (((i >> 3) << 2) | (i & 3));
    if (vv >= NSLOT) return -1;
    const int dy = half * RH0 + vv / K, dx = vv % K;
    return dy < K ? dy * K + dx : -1;
}

// logits form: the MFMA row (one per lane half) that is all ones: the first padding row of the block that holds it
template <int K>
__device__ __forceinline__ bool sum_row(int i, int mb) {
    constexpr int NSLOT = ((K + 1) / 2) * K;
    return 16 * mb + (((i >> 3) << 2) | (i & 3)) == NSLOT;
}

struct TilePos { int n, ty, tx; };

// v = q * s + r, 0 <= r < s, for the scales the library takes (wave-uniform branch on s)
__device__ __forceinline__ void divmod_scale(int v, int s, int& q, int& r) {
    if (s == 4) { q = v >> 2; r = v & 3; }
    else if (s == 2) { q = v >> 1; r = v & 1; }
    else { q = v / 3; r = v - 3 * q; }
}

// PSM != 0: the coefficients are read in the layout the coefficient network holds before its
// pixel-shuffle layer, [L*s*s][h][w]: the s*s sub-pixels of an LR pixel lie in s*s LR planes.
//   PSM = 4 (scale 4) and PSM = 2 (scale 2): the fast forms.  Which HR pixel an MFMA column and
//     pixel slot stand for is free, as long as stage 4 and the store know it.  A lane still loads
//     8 bytes per plane, but from ONE sub-pixel plane: four consecutive LR pixels, i.e. four HR
//     pixels s apart, which become its four slots.  With n = lane % 32, j = n % 2, m = n / 2:
//       scale 2: the lane reads sub-pixel column j;  slot q is HR pixel X0 + 8 m + 2 q + j.
//         A unit is one row of 128 HR pixels = 64 LR pixels = one 128-byte line of each plane.
//       scale 4: 128 HR pixels of a row would be half a line of each plane, and a half-line
//         request occupies the L1 like a whole one (measured: the same bytes in 64-byte pieces
//         take 2.2 x the time unless the same wavefront asks for the other half right away).  So the
//         tile is 256 pixels wide and a row is TWO units, J = 0, 1: the lane reads sub-pixel column
//         2 J + j;  slot q is HR pixel X0 + 16 m + 4 q + 2 J + j.  Every load instruction still
//         covers whole lines (16 lanes x 8 bytes per plane).
//       scale 3: the tile is 384 pixels wide and a row is THREE units, J = 0, 1, 2: every lane reads
//         sub-pixel column J, lane n the LR columns 4 n .. 4 n + 3;  slot q is HR pixel X0 + 12 n + 3 q + J
//         (two whole lines of a plane per lane half).  No exchange before the store: after the third
//         unit a lane holds six adjacent pixels.
//     Loads are as many and as wide as in the HR-planar form.  Stage 4 reads the tile at those
//     pixels (per-lane LDS bases), and before the store lanes j = 0, 1 exchange results so that
//     each holds adjacent pixels again (scale 4: the results of unit J = 0 wait in registers for
//     J = 1, then a lane stores four adjacent pixels and a wavefront 1 KB per channel).
//   PSM = 1 (any scale): the PX consecutive HR pixels of a lane come from up to PX planes, one
//     16-bit load each, placed in the halves of the registers an HR-planar load would have
//     filled; everything after the loads is unchanged.  Four times the load instructions and a
//     register per element in flight: 2.6 x the time of the planar form at 4K.
// The result is the planar form's, bit for bit, in every case.
//
// PSM = 8: the coefficients are stored pixel-major, [H][W][L] (the L = 72 coefficients of a pixel side by
// side, 144 bytes; what a producer that keeps its tensors channels-last writes).  A unit's 128 pixels are
// then 18 432 CONTIGUOUS bytes: 18 loads of 16 bytes per lane, lane after lane (the friendliest request
// stream there is: the same bytes take 231 us where the planes take 249).  Sixteen bytes of a pixel are the
// eight atoms of half a 16-atom step, i.e. a B operand as it stands: pixel slot by pixel slot (slot q =
// pixels 32 q .. 32 q + 31 of the unit, 4 608 contiguous bytes) the loaded registers are copied to an LDS
// scratch as they are and lane (j, hf) reads its operand pieces back at pixel j, piece 2 c + hf.  No
// re-packing.  Lane j's slots are the pixels j, 32 + j, 64 + j, 96 + j: the tile is stored without a
// swizzle (consecutive lanes read consecutive words) and a lane stores single pixels (a wavefront half
// still writes 128 contiguous bytes).  The fold, stage 4 and the result are the planar form's, bit for bit.
//
// PSM = 9: the coefficients are stored BLOCKED (SR_COEFF_BLOCKED; a storage order beyond the paper, for a producer that
// is willing to write it): a unit's 128 x 72 coefficients are 18 432 contiguous bytes laid out as this kernel consumes
// them - slot q (pixel 4 j + q of the unit), then pieces of 16 atoms [lane half][column j][8 atoms] and a last piece
// [lane half][column j][4 atoms].  Lane (j, hf) = lane j + 32 hf loads 16 bytes at 16 * lane of a piece (a wavefront: 1 KB
// of contiguous memory per load) and holds the B operand of that 16-atom step and slot as it stands: no re-packing, no
// staging, and the slots are the planar form's four adjacent pixels, so stage 4 and the store are the planar form's too.
// (8-bit coefficients in the same order: 8 bytes per lane and piece, widened to the operand with four conversions.)
template <int K, int C, int NP8, int PX, int WR, int NW, int NU, int WPE, int CT, int SMIN, bool BIG, int PSM = 0>
__global__ __launch_bounds__(64 * NW, WPE)
void k_assemble_mfma(const AssembleArgs a, const int tiles_x, const int tiles_y, const int ntiles) {
    constexpr int NSUB = PSM == 4 ? 2 : (PSM == 3 ? 3 : 1);   // units per tile row
    constexpr bool PMAJ = PSM == 8;                // coefficients stored pixel-major, [H][W][L]
    constexpr bool BLK = PSM == 9;                 // coefficients stored blocked: the loaded registers are the operands
    using F = Cfg<K, C, NP8, PX, WR, NW, NU, CT, SMIN, NSUB, (PMAJ ? 1 : 0)>;
    constexpr bool F32 = F::F32, F8 = F::F8, BF = F::BF, LIST = F::LIST, LG = F::LG;
    static_assert(!LG || (PX == 4 && (PSM == 0 || PSM == 2 || PSM == 3 || PSM == 4 || PSM == 9) && !BIG && F::NSLOT < 16 * F::NMB),
                  "logits form: fp16 planes (or the permuted-slot forms of the layout before the pixel-shuffle), four pixels per lane, a free MFMA row");
    constexpr int LH = F::LH;                      // list entries a lane half loads
    static_assert(!LIST || (PX == 4 && WR == 1 && !BIG && PSM == 0 && NU % 2 == 0), "list form: four pixels per lane, one row per unit");
    constexpr bool PS = PSM == 1;                  // one 16-bit load per pixel
    constexpr bool PERM = PSM == 2 || PSM == 3 || PSM == 4;    // permuted pixel slots
    static_assert(PSM == 0 || ((CT == CT_F16 || (CT == CT_F8 && PSM == 9) ||
                                ((CT == CT_BF16 || CT == CT_LOGIT || CT == CT_LOGIT_BF16) && PSM != 1 && PSM != 8 &&
                                 (PSM != 9 || CT == CT_LOGIT || CT == CT_BF16))) && !BIG && PX == 4),
                  "pre-shuffle layout: 16-bit coefficients, four pixels per lane");
    static_assert(!PMAJ || (CT == CT_F16 && WR == 1 && NP8 == 9), "pixel-major coefficients: 72 fp16 atoms, one row per unit");
    static_assert(!BLK || ((CT == CT_F16 || CT == CT_BF16 || CT == CT_F8 || CT == CT_LOGIT) && WR == 1 && PX == 4),
                  "blocked coefficients: fp16 (values or logits), bfloat16 or 8-bit, one row of 128 pixels per unit");
    static_assert(!PERM || (WR == 1 && SMIN >= PSM), "permuted slots: one row per wavefront and unit");
    // row of the wavefront's unit within the tile, and which of the row's NSUB units it is
    auto unit_row = [](int unit, int wave_) { return (unit / NSUB) * NW + wave_; };
    constexpr int NPIX = PS ? PX : 1;              // pixel offsets a lane keeps per unit
    using Raw = typename RawT<PX * F::CB>::type;
    constexpr int NT = F::NT, P = F::P, NG = F::NG, UH = F::UH, UW = F::UW;
    constexpr int N16 = F::N16, N8 = F::N8, NMB = F::NMB;
    constexpr int MAXLRY = F::MAXLRY, MAXLRX = F::MAXLRX;

    __shared__ float U[C * UH * P];                 // up-sampled tile, column-swizzled
    __shared__ float V[C * UH * MAXLRX];            // after the vertical pass
    __shared__ float lrT[C * MAXLRY * MAXLRX];      // LR footprint (clamped reads)
    __shared__ float4 xw[UW], yw[UH];               // per-column / per-row tap weights
    __shared__ int xb[UW], yb[UH];                  // ... and first source index
    __shared__ float4 wk[8];                        // Keys weights by phase numerator m
    __shared__ u32x4 A16[(N16 ? N16 : 1) * NMB * 2 * 64];
    __shared__ u32x2 A8[(F32 ? 1 : NMB * 2) * 64];
    __shared__ float A32[(F32 ? F::N2 * NMB : 1) * 64];   // fp32 path: D[2*step + hf][tap of row]
    __shared__ unsigned ptab[2 * F::NLOAD];         // byte offset of the plane each lane half loads
    __shared__ u32x4 pmscr[PMAJ ? NW * 288 : 1];    // pixel-major: per wavefront, one slot's 32 pixels x 144 bytes
    __shared__ unsigned ltab[LIST ? 2 * LH : 1];    // list form: element offset of the entry plane each lane half loads
    __shared__ u32x4 lscr[LIST ? NW * F::LSW / 4 : 1];   // list form: per wavefront, [NP8 groups of 8 atoms][32 pixels][8 atoms] fp16

    const int tid0 = threadIdx.x;
    const int groups = (gridDim.x & 7) == 0 ? 8 : 1;
    const int G = gridDim.x / groups;                              // stride inside a share
    const int share = (ntiles + groups - 1) / groups;
    const int t_first = (int)(blockIdx.x % groups) * share + (int)(blockIdx.x / groups);
    const int t_end = min(ntiles, ((int)(blockIdx.x % groups) + 1) * share);
    if (t_first >= t_end) return;                                  // whole workgroup: no tile
    // First column of a tile.  When the image width is not a whole number of pixel
    // groups the last tile column is moved left to end at the image edge (a.xlast =
    // W - TW): it recomputes some pixels of its neighbour (same values, written twice)
    // and no lane ever holds a group that sticks out of its row.
    auto tile_x0 = [&](int tx) { return tx == tiles_x - 1 ? a.xlast : tx * F::TW; };

    // ---- once per workgroup: weight, plane-offset and dictionary operand tables ---
    // Where a coefficient lies within its image is a 32-bit offset: in bytes, or (BIG) in
    // elements, which reaches images of up to 2^32 coefficients (an 8K frame with 72 fp16
    // planes is 4.8 GB) at the price of a 64-bit address per load instead of a scalar base
    // plus a 32-bit offset.
    constexpr unsigned OU = BIG ? 1u : (unsigned)F::CB;                          // offset units per element
    const unsigned plane_b = (unsigned)a.H * (unsigned)a.W * OU;                 // offset units per coefficient plane
    auto caddr = [&](const char* img, unsigned off) -> const char* {
        if constexpr (BIG) return img + (size_t)off * (size_t)F::CB;
        else return img + off;
    };
    if (tid0 < 2 * a.s) {
        float wt[4];
        keys_weights(tid0, a.s, wt);
        wk[tid0] = make_float4(wt[0], wt[1], wt[2], wt[3]);
    }
    if constexpr (LIST) {
        for (int e = tid0; e < NW * F::LSW / 4; e += NT) lscr[e] = u32x4{0u, 0u, 0u, 0u};
        // half h takes entries h * ceil(T / 2) ...; a slot past the list repeats an entry the pixel has (the
        // half's first one, or entry 0): written twice to the same place with the same value
        const int per_half = (a.T + 1) / 2;
        for (int e = tid0; e < 2 * LH; e += NT) {
            const int h = e / LH, i = e - h * LH;
            int t = h * per_half + i;
            if (i >= per_half || t >= a.T) t = h * per_half < a.T ? h * per_half : 0;
            ltab[e] = (unsigned)t * ((unsigned)a.H * (unsigned)a.W);               // in elements
        }
    }
    for (int e = tid0; e < (LIST ? 0 : 2 * F::NLOAD); e += NT) {
        const int h = e / F::NLOAD, i = e - h * F::NLOAD;
        // load i of half h serves folded atom idx; padding atoms re-read the last plane
        const int idx = F32 ? 2 * i + h
                            : (i < 8 * N16 ? 16 * (i >> 3) + 8 * h + (i & 7) : 16 * N16 + 4 * h + (i - 8 * N16));
        ptab[e] = (unsigned)a.kept[idx < a.n_fold ? idx : a.n_fold - 1] * plane_b;
    }
    auto dval = [&](int idx, int tap) -> float {    // gamma * D[kept], zero for padding
        if (tap < 0 || idx >= a.n_fold) return 0.0f;
        return a.gamma[idx] * a.dict[(size_t)a.kept[idx] * F::KK + tap];
    };
    if (F32) {
        for (int e = tid0; e < F::N2 * NMB * 64; e += NT) {
            const int l = e & 63, blk = e >> 6, mb = blk % NMB, st = blk / NMB;
            A32[e] = dval(2 * st + (l >> 5), tap_of_row<K>(l & 31, mb));
        }
    }
    for (int e = tid0; e < N16 * NMB * 64; e += NT) {
        const int l = e & 63, blk = e >> 6, mb = blk % NMB, c16 = blk / NMB;
        const int tap = tap_of_row<K>(l & 31, mb);
        const bool ones = LG && sum_row<K>(l & 31, mb);       // logits form: this row sums the exponentials
        float dv[8];
#pragma unroll
        for (int jj = 0; jj < 8; ++jj) {
            const int idx = 16 * c16 + 8 * (l >> 5) + jj;
            dv[jj] = ones ? (idx < a.n_fold ? 1.0f : 0.0f) : dval(idx, tap);
        }
        u32x4 hi, lo;
        split_hi_lo<BF, 8>(dv, hi, lo);
        A16[(blk * 2 + 0) * 64 + l] = hi;
        A16[(blk * 2 + 1) * 64 + l] = lo;
    }
    if (N8) {
        for (int e = tid0; e < NMB * 64; e += NT) {
            const int l = e & 63, mb = e >> 6;
            const int tap = tap_of_row<K>(l & 31, mb);
            const bool ones = LG && sum_row<K>(l & 31, mb);
            float dv[4];
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) {
                const int idx = 16 * N16 + 4 * (l >> 5) + jj;
                dv[jj] = ones ? (idx < a.n_fold ? 1.0f : 0.0f) : dval(idx, tap);
            }
            u32x2 hi, lo;
            split_hi_lo<BF, 4>(dv, hi, lo);
            A8[(mb * 2 + 0) * 64 + l] = hi;
            A8[(mb * 2 + 1) * 64 + l] = lo;
        }
    }
    __syncthreads();

    // list form with up to 72 atoms, and pixel-major coefficients: the dictionary operands stay in registers (the
    // fold reads them once per pixel slot, four times as often as the dense form does)
    constexpr bool AREG = (LIST && NP8 <= 9) || PSM == 8;
    u32x4 areg[AREG ? 2 * N16 : 1];
    u32x2 areg8[AREG && N8 ? 2 : 1];
    if constexpr (AREG) {
#pragma unroll
        for (int i = 0; i < 2 * N16; ++i) {
            areg[i] = A16[i * 64 + (tid0 & 63)];
            asm volatile("" : "+v"(areg[i]));           // opaque: or the compiler reloads it from LDS at every use
        }
        if constexpr (N8 != 0) {
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                areg8[i] = A8[i * 64 + (tid0 & 63)];
                asm volatile("" : "+v"(areg8[i]));
            }
        }
    }

    // ---- tile walk.  Workgroups are dealt to the 8 XCDs round-robin by index, and
    //      each XCD has its own L2.  When the grid is a multiple of 8, XCD x (the
    //      workgroups with blockIdx.x % 8 == x) walks its own contiguous share of the
    //      tiles in raster order, so that tiles above one another, whose LR
    //      footprints overlap, meet in the same L2 at about the same time.  The
    //      step is pre-split into (image, tile row, tile column) so that no
    //      division is left in the loop.  All of it is scalar.
    const int per_img = tiles_x * tiles_y;
    const int step_n = G / per_img, step_r = G - step_n * per_img;
    const int step_y = step_r / tiles_x, step_x = step_r - step_y * tiles_x;
    auto advance = [&](TilePos p) -> TilePos {
        p.tx += step_x;
        if (p.tx >= tiles_x) { p.tx -= tiles_x; p.ty += 1; }
        p.ty += step_y;
        if (p.ty >= tiles_y) { p.ty -= tiles_y; p.n += 1; }
        p.n += step_n;
        return p;
    };
    TilePos cur;
    {
        const int t0 = t_first;
        cur.n = t0 / per_img;
        const int r2 = t0 - cur.n * per_img;
        cur.ty = r2 / tiles_x;
        cur.tx = r2 - cur.ty * tiles_x;
    }

    const int wave = __builtin_amdgcn_readfirstlane(tid0 >> 6);     // scalar, loop-invariant
    const char* lr_base = (const char*)a.lr;
    const unsigned lr_esz = a.io_f16 ? 2u : 4u;

    // LR footprint of a tile -> registers, as raw bits (fp16 is widened when it is
    // written to LDS).  Wavefront w takes (channel,row) pairs w, w+NW, ...; the lane
    // is the column.  Row addressing is scalar; one add per load on the vector side.
    //
    // Two forms.  LRBF (used where the coefficient stream is light enough for the
    // issue time of these loads to show, measured 4 % on the 8-bit 4K frame): every
    // slot is loaded unconditionally, as the aligned 32-bit word holding the
    // element (an fp16 image keeps which half in `par`, one bit per slot); slots
    // the tile does not need repeat the wavefront's first row / chunk, a line that
    // is already on its way.  No branch and one load type leave the compiler
    // nothing to merge at a join, so the loads go out back to back.  Otherwise:
    // only the needed slots are loaded (fewer requests, which is what counts when
    // the stream is the bound or the tile is small).
    constexpr bool LRBF = F8 && NP8 > 2;
    static_assert(!LRBF || F::NLRP * F::NXC <= 32, "one parity bit per footprint slot");
    const unsigned lr_sh = a.io_f16 ? 1u : 2u;          // log2 of the element size
    auto load_lr = [&](const TilePos tp, int lane, unsigned (&lrv)[F::NLRP][F::NXC], unsigned& par) {
        const TileOrigin o = tile_origin(tp.ty * F::TH, tile_x0(tp.tx), F::R, UH, UW, a.H, a.W, a.s);
        // the image's base is a 64-bit scalar; offsets within an image fit 32 bits
        const char* lr_img = lr_base + (size_t)tp.n * C * ((size_t)a.h * a.w * lr_esz);
        if constexpr (LRBF) {
            // aligned words: the image may start in the middle of one
            const unsigned mis = (unsigned)((uintptr_t)lr_img & 3u);
            const char* lr_al = lr_img - mis;
            unsigned xcol[F::NXC];
#pragma unroll
            for (int xc = 0; xc < F::NXC; ++xc) {
                xcol[xc] = (unsigned)clampi(o.lx0 + lane + 64 * xc, 0, a.w - 1);
                if (xc > 0 && 64 * xc >= o.nlx) xcol[xc] = xcol[0];
            }
            par = 0u;
            unsigned row0 = 0u;
#pragma unroll
            for (int u = 0; u < F::NLRP; ++u) {
                const int p = wave + NW * u, c = p / MAXLRY, ry = p - c * MAXLRY;
                const bool need = p < C * MAXLRY && ry < o.nly;
                unsigned row = ((unsigned)(need ? c : 0) * (unsigned)a.h +
                                (unsigned)clampi(o.ly0 + (need ? ry : 0), 0, a.h - 1)) * (unsigned)a.w;   // in elements
                if (u == 0) row0 = row;
                if (!need) row = row0;
#pragma unroll
                for (int xc = 0; xc < F::NXC; ++xc) {
                    const unsigned byte = ((row + xcol[xc]) << lr_sh) + mis;
                    par |= ((byte >> 1) & 1u) << (u * F::NXC + xc);
                    lrv[u][xc] = *(const unsigned*)(lr_al + (size_t)(byte & ~3u));
                }
            }
        } else {
            unsigned xo[F::NXC];
#pragma unroll
            for (int xc = 0; xc < F::NXC; ++xc) xo[xc] = (unsigned)clampi(o.lx0 + lane + 64 * xc, 0, a.w - 1) * lr_esz;
            auto rows = [&](auto f16) {
#pragma unroll
                for (int u = 0; u < F::NLRP; ++u) {
                    const int p = wave + NW * u, c = p / MAXLRY, ry = p - c * MAXLRY;
                    if (p < C * MAXLRY && ry < o.nly) {
                        const unsigned row = ((unsigned)c * (unsigned)a.h +
                                              (unsigned)clampi(o.ly0 + ry, 0, a.h - 1)) * (unsigned)a.w * lr_esz;
#pragma unroll
                        for (int xc = 0; xc < F::NXC; ++xc)
                            if (xc == 0 || 64 * xc < o.nlx) {     // whole 64-column chunks the tile never reads
                                const char* q = lr_img + (size_t)(row + xo[xc]);
                                lrv[u][xc] = decltype(f16)::value ? (unsigned)*(const unsigned short*)q : *(const unsigned*)q;
                            }
                    }
                }
            };
            if (a.io_f16) rows(std::true_type{});
            else rows(std::false_type{});
        }
    };

    // coefficient base of a tile for this lane: image base (scalar) + pixel offset
    auto phi_base = [&](const TilePos tp, int unit, int jr, int jc, unsigned (&pix_off)[NPIX]) -> const char* {
        const int y = tp.ty * F::TH + unit_row(unit, wave) * WR + jr, x = tile_x0(tp.tx) + PX * jc;
        const int yc = y < a.H ? y : a.H - 1, xc = x < a.W ? x : a.W - PX;   // out-of-image lanes re-read
        if constexpr (PERM) {
            // jc is the lane's column n: sub-pixel column (unit % NSUB) * 2 + n % 2, LR columns 4 m .. 4 m + 3, m = n / 2
            // (scale 3: every lane reads sub-pixel column unit % 3, lane n the LR columns 4 n .. 4 n + 3)
            const int jx = PSM == 3 ? unit % NSUB : (unit % NSUB) * 2 + jc % 2, m = PSM == 3 ? jc : jc / 2;
            const int ly = yc / PSM, iy = yc % PSM;
            int lx = tile_x0(tp.tx) / PSM + 4 * m;
            lx = lx + 4 <= a.w ? lx : a.w - 4;                                     // lanes past the image re-read
            pix_off[0] = ((unsigned)(iy * PSM + jx) * ((unsigned)a.h * (unsigned)a.w) +
                          (unsigned)ly * (unsigned)a.w + (unsigned)lx) * OU;
        } else if constexpr (PS) {
            int ly, iy;
            divmod_scale(yc, a.s, ly, iy);
            const unsigned hw = (unsigned)a.h * (unsigned)a.w;
#pragma unroll
            for (int q = 0; q < PX; ++q) {
                int lx, jx;
                divmod_scale(xc + q, a.s, lx, jx);
                pix_off[q] = ((unsigned)(iy * a.s + jx) * hw + (unsigned)ly * (unsigned)a.w + (unsigned)lx) * OU;
            }
        } else {
            pix_off[0] = ((unsigned)yc * (unsigned)a.W + (unsigned)xc) * OU;         // a valid address; never stored
        }
        return (const char*)a.coeff + (size_t)tp.n * a.L * ((size_t)a.H * a.W * F::CB);
    };
    // the PX coefficients of one plane (or plane group) that a lane owns
    auto load_raw = [&](const char* cimg, const unsigned (&pix_off)[NPIX], unsigned plane_off) -> Raw {
        if constexpr (PS) {
            typedef _Float16 h2 __attribute__((ext_vector_type(2)));
            Raw r;
#pragma unroll
            for (int m = 0; m < PX / 2; ++m) {
                h2 v;
                v[0] = __builtin_nontemporal_load((const _Float16*)(cimg + (pix_off[2 * m] + plane_off)));
                v[1] = __builtin_nontemporal_load((const _Float16*)(cimg + (pix_off[2 * m + 1] + plane_off)));
                r[m] = __builtin_bit_cast(unsigned, v);
            }
            return r;
        } else {
            return __builtin_nontemporal_load((const Raw*)caddr(cimg, pix_off[0] + plane_off));
        }
    };

    // list form: the entries of a unit, two register sets (the next unit's are loaded while this one is folded)
    u32x2 lval[2][LIST ? LH : 1];                   // four fp16 values (the lane's four pixels) per entry
    unsigned lidx[2][LIST ? LH : 1];                // their four atom numbers, one byte each
    auto load_list = [&](const TilePos tp, int unit, int jc, int hf, u32x2 (&val)[LIST ? LH : 1], unsigned (&idx)[LIST ? LH : 1]) {
        const int y = tp.ty * F::TH + unit_row(unit, wave), x = tile_x0(tp.tx) + PX * jc;
        const int yc = y < a.H ? y : a.H - 1, xc = x < a.W ? x : a.W - PX;
        const unsigned pix = (unsigned)yc * (unsigned)a.W + (unsigned)xc;           // elements within a plane
        const size_t img = (size_t)tp.n * a.T * ((size_t)a.H * a.W);
        const unsigned char* ibase = a.index + img;
        const char* vbase = (const char*)a.coeff + img * 2;
        const unsigned* lt = ltab + hf * LH;
#pragma unroll
        for (int e = 0; e < LH; ++e) {
            const unsigned at = lt[e] + pix;
            idx[e] = __builtin_nontemporal_load((const unsigned*)(ibase + at));
            val[e] = __builtin_nontemporal_load((const u32x2*)(vbase + (size_t)at * 2));
        }
    };
    // pixel-major: the unit's 18 432 bytes, 16 per lane and load; byte offset of the lane's first piece within the image
    constexpr int NPM = 18;
    u32x4 pm[PMAJ ? NPM : 1];
    auto pm_offset = [&](const TilePos tp, int unit, int lane_) -> unsigned {
        const int y = tp.ty * F::TH + unit * NW + wave;
        const unsigned yc = (unsigned)(y < a.H ? y : a.H - 1);                 // rows past the image re-read its last row
        return (yc * (unsigned)a.W + (unsigned)tile_x0(tp.tx)) * (unsigned)(16 * NP8) + 16u * (unsigned)lane_;
    };
    auto pm_image = [&](const TilePos tp) -> const char* {
        return (const char*)a.coeff + (size_t)tp.n * a.L * ((size_t)a.H * a.W * F::CB);
    };
    // blocked: byte offset of a unit within its image (a unit: 128 pixels x 8 NP8 atoms, contiguous), and its loads
    // (8-bit coefficients: the same order of elements, half the bytes: 8 bytes per lane and 16-atom piece, widened to the
    //  operand at its use)
    using B16 = typename std::conditional<F8, u32x2, u32x4>::type;
    using B8 = typename std::conditional<F8, unsigned, u32x2>::type;
    constexpr unsigned CBB = (unsigned)F::CB;
    B16 b16[BLK ? PX : 1][BLK && N16 ? N16 : 1];
    B8 b8[BLK ? PX : 1];
    constexpr unsigned SLOT_B = 32u * 8u * NP8 * CBB;   // bytes of a slot: 32 pixels x 8 NP8 atoms
    auto blk_offset = [&](const TilePos tp, int unit) -> unsigned {
        const int y = tp.ty * F::TH + unit * NW + wave;
        const unsigned yc = (unsigned)(y < a.H ? y : a.H - 1);                 // rows past the image re-read its last row
        return (yc * (unsigned)(a.W / 128) + (unsigned)tp.tx) * (4u * SLOT_B);
    };
    auto blk_load16 = [&](const char* img, unsigned unit_off, int lane_, int q, int c16) -> B16 {
        return __builtin_nontemporal_load((const B16*)(img + (unit_off + (unsigned)q * SLOT_B + 512u * CBB * c16 + 8u * CBB * lane_)));
    };
    auto blk_load8 = [&](const char* img, unsigned unit_off, int lane_, int q) -> B8 {
        return __builtin_nontemporal_load((const B8*)(img + (unit_off + (unsigned)q * SLOT_B + 512u * CBB * N16 + 4u * CBB * lane_)));
    };
    // an 8-atom run of 8-bit coefficients widened to the fp16 operand (exact), two values per conversion
    auto widen16 = [&](const u32x2& v) -> u32x4 {
        typedef _Float16 h2 __attribute__((ext_vector_type(2)));
        u32x4 r;
#pragma unroll
        for (int m = 0; m < 4; ++m)
            r[m] = (m & 1) ? __builtin_bit_cast(unsigned, (h2)__builtin_amdgcn_cvt_scalef32_pk_f16_fp8(v[m >> 1], 1.0f, true))
                           : __builtin_bit_cast(unsigned, (h2)__builtin_amdgcn_cvt_scalef32_pk_f16_fp8(v[m >> 1], 1.0f, false));
        return r;
    };
    auto widen8 = [&](unsigned v) -> u32x2 {
        typedef _Float16 h2 __attribute__((ext_vector_type(2)));
        u32x2 r;
        r[0] = __builtin_bit_cast(unsigned, (h2)__builtin_amdgcn_cvt_scalef32_pk_f16_fp8(v, 1.0f, false));
        r[1] = __builtin_bit_cast(unsigned, (h2)__builtin_amdgcn_cvt_scalef32_pk_f16_fp8(v, 1.0f, true));
        return r;
    };
    Raw raw[F::NLOAD];
    unsigned lrv[F::NLRP][F::NXC], lrpar = 0u;
#pragma unroll
    for (int u = 0; u < F::NLRP; ++u)
#pragma unroll
        for (int xc = 0; xc < F::NXC; ++xc) lrv[u][xc] = 0u;
    {
        const int lane = tid0 & 63, hf = lane >> 5, j = lane & 31;
        load_lr(cur, lane, lrv, lrpar);
        if constexpr (LIST) {
            load_list(cur, 0, j, hf, lval[0], lidx[0]);
        } else if constexpr (PMAJ) {
            const char* img = pm_image(cur);
            const unsigned off = pm_offset(cur, 0, lane);
#pragma unroll
            for (int i = 0; i < NPM; ++i) pm[i] = __builtin_nontemporal_load((const u32x4*)(img + (off + 1024u * i)));
        } else if constexpr (BLK) {
            const char* img = pm_image(cur);
            const unsigned off = blk_offset(cur, 0);
#pragma unroll
            for (int q = 0; q < PX; ++q) {
#pragma unroll
                for (int c16 = 0; c16 < N16; ++c16) b16[q][c16] = blk_load16(img, off, lane, q, c16);
                if constexpr (N8 != 0) b8[q] = blk_load8(img, off, lane, q);
            }
        } else {
            unsigned pix_off[NPIX];
            const char* cimg = phi_base(cur, 0, j / F::WC, j % F::WC, pix_off);
            const unsigned* pt = ptab + hf * F::NLOAD;
#pragma unroll
            for (int i = 0; i < F::NLOAD; ++i) raw[i] = load_raw(cimg, pix_off, pt[i]);
        }
    }

    // ---- stage 1 in three steps; a workgroup barrier separates each from the next.
    // (a) tap tables of a tile and its LR footprint, registers -> LDS
    // the first UW threads fill the column tables, UH of the last 64 the row tables
    static_assert(UH <= 64, "tile too tall for the table set-up");
    auto stage1_setup = [&](const TilePos tp, int tid) {
        const int lane = tid & 63;
        const int Y0 = tp.ty * F::TH, X0 = tile_x0(tp.tx);
        const TileOrigin o = tile_origin(Y0, X0, F::R, UH, UW, a.H, a.W, a.s);
        for (int xx = tid; xx < UW; xx += NT) {       // one pass unless the tile is wider than the workgroup
            int m;
            const int f = src_floor(clampi(X0 - F::R + xx, 0, a.W - 1), a.s, m);
            xw[xx] = wk[m];
            xb[xx] = clampi(f - 1 - o.lx0, 0, MAXLRX - 4);
        }
        if (tid >= NT - 64 && tid - (NT - 64) < UH) {
            const int i = tid - (NT - 64);
            int m;
            const int f = src_floor(clampi(Y0 - F::R + i, 0, a.H - 1), a.s, m);
            yw[i] = wk[m];
            yb[i] = clampi(f - 1 - o.ly0, 0, MAXLRY - 4);
        }
#pragma unroll
        for (int u = 0; u < F::NLRP; ++u) {
            const int p = wave + NW * u;
            if (p < C * MAXLRY) {
#pragma unroll
                for (int xc = 0; xc < F::NXC; ++xc)
                    if (lane + 64 * xc < MAXLRX) {
                        unsigned bits = lrv[u][xc];
                        if (LRBF && a.io_f16) bits = ((lrpar >> (u * F::NXC + xc)) & 1u) ? bits >> 16 : bits & 0xffffu;
                        lrT[p * MAXLRX + lane + 64 * xc] =
                            a.io_f16 ? __half2float(__ushort_as_half((unsigned short)bits)) : __uint_as_float(bits);
                    }
            }
        }
    };
    // (b) vertical pass on the narrow LR footprint: V[c][yy][rx].  Four elements per
    //     thread at a time, their table reads and then their 16 footprint reads
    //     issued together, so that LDS latency is paid once per batch and not twice
    //     per element.  Loads are clamped into range; only the store is guarded.
    auto stage1_vertical = [&](const TilePos tp, int tid) {
        const TileOrigin o = tile_origin(tp.ty * F::TH, tile_x0(tp.tx), F::R, UH, UW, a.H, a.W, a.s);
        // Items (row pr, footprint column rx), nlx columns to a row, dealt to the threads with
        // no idle lanes (rows padded to 32, 64 or 128 columns left 38 % of them idle at x4:
        // 8 atoms at 4K 90 -> 85 us, the E4M3 frame 160 -> 154 us).  idx / nlx by a multiply,
        // exact for idx < 2^22 / nlx and free of overflow for idx < 1024 nlx.
        static_assert(C * UH * MAXLRX * MAXLRX <= (1 << 22) && C * UH <= 1024, "item index beyond the exact range of the division");
        const int nlx = o.nlx < 4 ? 4 : o.nlx;
        const unsigned inv = ((1u << 22) + nlx - 1) / nlx;
        const int total = C * UH * nlx;
        for (int base = tid; base < total; base += 4 * NT) {
            float4 w4[4];
            int src[4], dst[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int idx = base + k * NT;
                const int idc = idx < total ? idx : total - 1;
                const int pr = (int)(((unsigned)idc * inv) >> 22), rx = idc - pr * nlx;
                const int c = pr / UH, yy = pr - c * UH;
                w4[k] = yw[yy];
                src[k] = (c * MAXLRY + yb[yy]) * MAXLRX + rx;
                dst[k] = idx < total ? pr * MAXLRX + rx : -1;
            }
            __builtin_amdgcn_sched_barrier(0);
            float v[4][4];
#pragma unroll
            for (int k = 0; k < 4; ++k)
#pragma unroll
                for (int i = 0; i < 4; ++i) v[k][i] = lrT[src[k] + i * MAXLRX];
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const float wt[4] = {w4[k].x, w4[k].y, w4[k].z, w4[k].w};
                if (dst[k] >= 0) V[dst[k]] = dot4(wt, v[k][0], v[k][1], v[k][2], v[k][3]);
            }
        }
    };
    // (c) horizontal pass into the swizzled tile: a thread owns one (channel,
    //     column), its weights stay in registers, rows are independent (no tables,
    //     immediate offsets).  Rows go in batches: all reads of a batch are issued
    //     before its arithmetic.
    auto stage1_horizontal = [&](int tid) {
        for (int col = tid; col < C * UW; col += NT) {
            const int c = col / UW, xx = col - c * UW;
            const float4 w4 = xw[xx];
            const float wt[4] = {w4.x, w4.y, w4.z, w4.w};
            const float* src = V + c * UH * MAXLRX + xb[xx];
            float* dst = U + c * UH * P + (xx % F::SW) * NG + xx / F::SW;
            constexpr int RB = 7;
#pragma unroll
            for (int y0 = 0; y0 < UH; y0 += RB) {
                float v[RB][4];
#pragma unroll
                for (int r = 0; r < RB; ++r)
                    if (y0 + r < UH) {
#pragma unroll
                        for (int i = 0; i < 4; ++i) v[r][i] = src[(y0 + r) * MAXLRX + i];
                    }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int r = 0; r < RB; ++r)
                    if (y0 + r < UH) dst[(y0 + r) * P] = dot4(wt, v[r][0], v[r][1], v[r][2], v[r][3]);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    };

    unsigned long long wb_last = a.wb_ticks > 0 ? __builtin_amdgcn_s_memrealtime() : 0ull;
    for (int t = t_first; t < t_end; t += G) {
        // Per-iteration copy of the thread id the optimiser cannot see through:
        // index arithmetic derived from it is recomputed each tile instead of
        // being hoisted out of the loop into dozens of long-lived registers.
        int tid = tid0;
        asm volatile("" : "+v"(tid));
        const int lane = tid & 63;
        const int hf = lane >> 5, j = lane & 31, jr = j / F::WC, jc = j % F::WC;
        const int Y0 = cur.ty * F::TH, X0 = tile_x0(cur.tx);
        const bool more_tiles = t + G < t_end;
        const TilePos nxt = more_tiles ? advance(cur) : cur;

        // (1) stage 1 of this tile.  (Spreading steps (a) and (b) of the next tile
        //     over the unit loop was measured slower: the extra mid-tile barrier and
        //     LDS traffic cost more than the shorter gap between tiles gains.)
        stage1_setup(cur, tid);
        __syncthreads();
#ifdef SR_ABLATE_STAGE1
        if (a.N < 0)
#endif
        stage1_vertical(cur, tid);
        __syncthreads();      // also: every wavefront is done with the previous tile's U
#ifdef SR_ABLATE_STAGE1
        if (a.N < 0)
#endif
        stage1_horizontal(tid);
        __syncthreads();
        const unsigned* pt = ptab + hf * F::NLOAD;
        float park[C][NSUB > 1 ? NSUB - 1 : 1][2];     // permuted slots, scales 3 and 4: the results of a row's earlier units wait for the last
        // The wavefront's NU units of this tile, one after the other; while a unit
        // is folded, the coefficients of the next one (same tile, or unit 0 of the
        // next tile) are loaded into the registers that fall free.
#pragma unroll
        for (int unit = 0; unit < NU; ++unit) {
        const bool last_unit = unit == NU - 1;
        const bool more = last_unit ? more_tiles : true;
        unsigned pix_next[NPIX];
        const char* cnext = nullptr;
        if constexpr (!LIST && !PMAJ && !BLK) cnext = last_unit ? phi_base(nxt, 0, jr, jc, pix_next) : phi_base(cur, unit + 1, jr, jc, pix_next);
        const char* bimg = nullptr;                    // blocked: the next unit's image and offset
        unsigned boff = 0u;
        if constexpr (BLK) {
            bimg = last_unit ? pm_image(nxt) : pm_image(cur);
            boff = last_unit ? blk_offset(nxt, 0) : blk_offset(cur, unit + 1);
        }

        // (3) stage 3 on the matrix cores: atom steps outer, pixel slots inner
        f32x16 acc[PX][NMB];
#pragma unroll
        for (int q = 0; q < PX; ++q)
#pragma unroll
            for (int mb = 0; mb < NMB; ++mb)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[q][mb][v] = 0.0f;
        if constexpr (LIST) {
            // the next unit's entries go into the other register set while this one is folded
            if (more) {
                if (last_unit) load_list(nxt, 0, jc, hf, lval[(unit + 1) & 1], lidx[(unit + 1) & 1]);
                else load_list(cur, unit + 1, jc, hf, lval[(unit + 1) & 1], lidx[(unit + 1) & 1]);
            }
            const u32x2 (&val)[LH] = lval[unit & 1];
            const unsigned (&idx)[LH] = lidx[unit & 1];
            static_assert(NMB == 1, "list form: one block of MFMA rows");
            // (16-bit writes and vector reads of the same words: the write goes through a type that may alias
            //  anything, or the compiler is free to move a read above the write it depends on)
            typedef unsigned short __attribute__((may_alias)) u16a;
            u32x4* const scrw = lscr + wave * (F::LSW / 4);
            char* const col = (char*)(scrw + jc);              // atom a of the lane's pixel: col + (a / 8) * 512 + (a % 8) * 2
            // Per pixel slot: scatter, read the operand pieces, write the zeros back - all three go out at once
            // (LDS serves a wavefront's requests in order) - and only the fold waits for the pieces.  The next
            // slot's requests are issued before this slot's fold, so that they travel while the matrix cores work.
            u32x4 bw16[2][N16 ? N16 : 1];
            u32x2 bw8[2];
            auto issue = [&](int q, int b) {
                // lanes j and j + 32 hold different entries of the same pixels.  An atom number the dictionary
                // does not have (a caller's error) is kept inside the pixel's own pieces.
                unsigned where[LH];
#pragma unroll
                for (int e = 0; e < LH; ++e) {
                    unsigned atom = (idx[e] >> (8 * q)) & 0xffu;
                    atom = atom < 8u * NP8 ? atom : 8u * NP8 - 1u;
                    where[e] = (atom >> 3) * 512u + (atom & 7u) * 2u;
                    *(u16a*)(col + where[e]) = (unsigned short)(val[e][q >> 1] >> (16 * (q & 1)));
                }
#pragma unroll
                for (int c16 = 0; c16 < N16; ++c16) bw16[b][c16] = scrw[(2 * c16 + hf) * 32 + jc];
                if constexpr (N8 != 0) bw8[b] = *(const u32x2*)(col + (2 * N16) * 512 + 8 * hf);
#pragma unroll
                for (int e = 0; e < LH; ++e) *(u16a*)(col + where[e]) = (unsigned short)0;
            };
            issue(0, 0);
#pragma unroll
            for (int q = 0; q < PX; ++q) {
                __builtin_amdgcn_sched_barrier(0);
                if (q + 1 < PX) issue(q + 1, (q + 1) & 1);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int c16 = 0; c16 < N16; ++c16)
#pragma unroll
                    for (int hl = 0; hl < 2; ++hl)
                        acc[q][0] = mfma_16<false>(AREG ? areg[c16 * 2 + hl] : A16[(c16 * 2 + hl) * 64 + lane], bw16[q & 1][c16], acc[q][0]);
                if constexpr (N8 != 0) {
#pragma unroll
                    for (int hl = 0; hl < 2; ++hl)
                        acc[q][0] = mfma_8<false>(AREG ? areg8[hl] : A8[hl * 64 + lane], bw8[q & 1], acc[q][0]);
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        if constexpr (PMAJ) {
            static_assert(NMB == 1 || !PMAJ, "pixel-major: one block of MFMA rows");
            const char* nimg = last_unit ? pm_image(nxt) : pm_image(cur);
            const unsigned noff = last_unit ? pm_offset(nxt, 0, lane) : pm_offset(cur, unit + 1, lane);
            char* const scr = (char*)(pmscr + wave * 288);
            const char* const mine = scr + jc * (16 * NP8);            // the lane's pixel of the slot
            auto reload = [&](int i) {
                if (more) pm[i] = __builtin_nontemporal_load((const u32x4*)(nimg + (noff + 1024u * i)));
            };
            // Slot q = stream bytes 4608 q .. 4608 q + 4607: four whole loads and half of the load that two slots
            // share.  stage(q): registers -> scratch (and the freed registers are re-loaded for the next unit), then
            // the lane's operand pieces back: sixteen bytes of a pixel are atoms 8 g .. 8 g + 7, piece 2 c + hf is
            // the operand of step c.  LDS serves a wavefront's requests in order, so the next slot is staged
            // before this slot's matrix instructions are issued and its pieces travel while they run.
            u32x4 bw16[2][N16 ? N16 : 1];
            u32x2 bw8[2];
            auto stage = [&](int q, int b) {
                const int first = (9 * q) / 2;                         // 0, 4, 9, 13
                if (q % 2 == 0) {
#pragma unroll
                    for (int i = 0; i < 4; ++i) *(u32x4*)(scr + 1024 * i + 16 * lane) = pm[first + i];
                    if (lane < 32) *(u32x4*)(scr + 4096 + 16 * lane) = pm[first + 4];
#pragma unroll
                    for (int i = 0; i < 4; ++i) reload(first + i);
                } else {
                    if (lane >= 32) *(u32x4*)(scr + 16 * (lane - 32)) = pm[first];
#pragma unroll
                    for (int i = 0; i < 4; ++i) *(u32x4*)(scr + 512 + 1024 * i + 16 * lane) = pm[first + 1 + i];
#pragma unroll
                    for (int i = 0; i < 5; ++i) reload(first + i);
                }
#pragma unroll
                for (int c16 = 0; c16 < N16; ++c16) bw16[b][c16] = *(const u32x4*)(mine + 32 * c16 + 16 * hf);
                if constexpr (N8 != 0) bw8[b] = *(const u32x2*)(mine + 32 * N16 + 8 * hf);
            };
            stage(0, 0);
#pragma unroll
            for (int q = 0; q < PX; ++q) {
                __builtin_amdgcn_sched_barrier(0);
                if (q + 1 < PX) stage(q + 1, (q + 1) & 1);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int c16 = 0; c16 < N16; ++c16)
#pragma unroll
                    for (int hl = 0; hl < 2; ++hl)
                        acc[q][0] = mfma_16<false>(AREG ? areg[c16 * 2 + hl] : A16[(c16 * 2 + hl) * 64 + lane], bw16[q & 1][c16], acc[q][0]);
                if constexpr (N8 != 0) {
#pragma unroll
                    for (int hl = 0; hl < 2; ++hl)
                        acc[q][0] = mfma_8<false>(AREG ? areg8[hl] : A8[hl * 64 + lane], bw8[q & 1], acc[q][0]);
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        if constexpr (F32) {
            // fp32 coefficients: the loaded words ARE the B operand (lane half hf holds
            // atom 2*step + hf of its pixels), no re-packing, exact fp32 products
#pragma unroll
            for (int st = 0; st < F::N2; ++st) {
                float av[NMB];
#pragma unroll
                for (int mb = 0; mb < NMB; ++mb) av[mb] = A32[(st * NMB + mb) * 64 + lane];
#pragma unroll
                for (int q = 0; q < PX; ++q)
#pragma unroll
                    for (int mb = 0; mb < NMB; ++mb)
                        acc[q][mb] = __builtin_amdgcn_mfma_f32_32x32x2f32(
                            av[mb], __uint_as_float(raw_word(raw[st], q)), acc[q][mb], 0, 0, 0);
                if ((st & 3) == 3) __builtin_amdgcn_sched_barrier(0);
                if (more)
                    raw[st] = load_raw(cnext, pix_next, pt[st]);
                if ((st & 3) == 3) __builtin_amdgcn_sched_barrier(0);
            }
        }
        // logits form: -max * log2(e) of the lane's four pixels, over all planes (both lane halves)
        float nm[PX];
        if constexpr (LG && BLK) {
            // blocked order: a word holds two atoms of ONE pixel (slot q); per slot the packed maximum over the lane's
            // words, the larger of its two halves, then the other lane half's
            typedef _Float16 h2 __attribute__((ext_vector_type(2)));
#pragma unroll
            for (int q = 0; q < PX; ++q) {
                const unsigned first = N16 ? b16[q][0][0] : b8[q][0];
                h2 mq = __builtin_bit_cast(h2, first);
#pragma unroll
                for (int c16 = 0; c16 < N16; ++c16)
#pragma unroll
                    for (int m = 0; m < 4; ++m) {
                        const unsigned word = b16[q][c16][m];       // (by value: a bit cast straight from the vector element read element 0)
                        mq = pk_max_f16(mq, __builtin_bit_cast(h2, word));
                    }
                if constexpr (N8 != 0) {
#pragma unroll
                    for (int m = 0; m < 2; ++m) {
                        const unsigned word = b8[q][m];
                        mq = pk_max_f16(mq, __builtin_bit_cast(h2, word));
                    }
                }
                const unsigned bits = __builtin_bit_cast(unsigned, mq);
                mq = pk_max_f16(mq, __builtin_bit_cast(h2, (bits >> 16) | (bits << 16)));       // both halves: the larger one
                const unsigned one = __builtin_bit_cast(unsigned, mq);
                const auto sw = __builtin_amdgcn_permlane32_swap(one, one, false, false);
                mq = pk_max_f16(__builtin_bit_cast(h2, (unsigned)sw[0]), __builtin_bit_cast(h2, (unsigned)sw[1]));
                nm[q] = logit_shift((float)mq[0]);
            }
        } else if constexpr (LG) {
            typedef _Float16 h2 __attribute__((ext_vector_type(2)));
            h2 mx[PX / 2];
#pragma unroll
            for (int m = 0; m < PX / 2; ++m) mx[m] = __builtin_bit_cast(h2, raw_word(raw[0], m));
#pragma unroll
            for (int i = 1; i < F::NLOAD; ++i)
#pragma unroll
                for (int m = 0; m < PX / 2; ++m) mx[m] = pk_max_f16(mx[m], __builtin_bit_cast(h2, raw_word(raw[i], m)));
#pragma unroll
            for (int m = 0; m < PX / 2; ++m) {
                const unsigned bits = __builtin_bit_cast(unsigned, mx[m]);
                const auto sw = __builtin_amdgcn_permlane32_swap(bits, bits, false, false);   // one of the two is the other half's
                mx[m] = pk_max_f16(__builtin_bit_cast(h2, (unsigned)sw[0]), __builtin_bit_cast(h2, (unsigned)sw[1]));
            }
#pragma unroll
            for (int q = 0; q < PX; ++q) {
                if constexpr (F::LGB) nm[q] = logit_shift(__uint_as_float((__builtin_bit_cast(unsigned, mx[q >> 1]) >> (16 * (q & 1))) << 16));
                else nm[q] = logit_shift((float)mx[q >> 1][q & 1]);
            }
        }
#pragma unroll
        for (int c16 = 0; c16 < (LIST || PMAJ ? 0 : N16); ++c16) {   // (the list and pixel-major forms have folded above)
            u32x4 av[NMB][2];
#pragma unroll
            for (int mb = 0; mb < NMB; ++mb)
#pragma unroll
                for (int hl = 0; hl < 2; ++hl) av[mb][hl] = A16[((c16 * NMB + mb) * 2 + hl) * 64 + lane];
            constexpr int NWORD = PX / 2 > 0 ? PX / 2 : 1;
            unsigned cw[8][NWORD];                  // the step's 8 planes as fp16 pixel pairs
            if constexpr (BLK) {
                // (blocked: the loaded registers are the operands)
            } else if constexpr (F8) {
                // 8-bit coefficients: pair the planes' BYTES first (two permutes per plane pair), widen afterwards
#pragma unroll
                for (int m = 0; m < 4; ++m) pair_bytes(raw_word(raw[8 * c16 + 2 * m], 0), raw_word(raw[8 * c16 + 2 * m + 1], 0), cw[2 * m]);
            } else {
#pragma unroll
                for (int i = 0; i < 8; ++i) plane_words<F8>(raw[8 * c16 + i], cw[i]);
            }
#pragma unroll
            for (int q = 0; q < PX; ++q) {
                u32x4 bw;
                if constexpr (BLK) {
                    if constexpr (F8) bw = widen16(b16[q][c16]);
                    else if constexpr (LG) {
#pragma unroll
                        for (int m = 0; m < 4; ++m) bw[m] = exp_word(b16[q][c16][m], nm[q]);
                    } else bw = b16[q][c16];
                }
#pragma unroll
                for (int m = 0; m < (BLK ? 0 : 4); ++m)
                    bw[m] = F8 ? widen_pair(cw[2 * m][q >> 1], q)
                          : LG ? exp_pair<F::LGB>(cw[2 * m][q >> 1], cw[2 * m + 1][q >> 1], q, nm[q])
                               : pack_pair(cw[2 * m][q >> 1], cw[2 * m + 1][q >> 1], q);
#pragma unroll
                for (int mb = 0; mb < NMB; ++mb)
#pragma unroll
                    for (int hl = 0; hl < 2; ++hl) acc[q][mb] = mfma_16<BF>(av[mb][hl], bw, acc[q][mb]);
            }
            __builtin_amdgcn_sched_barrier(0);
            if (more) {
                if constexpr (BLK) {
#pragma unroll
                    for (int q = 0; q < PX; ++q) b16[q][c16] = blk_load16(bimg, boff, lane, q, c16);
                } else {
#pragma unroll
                    for (int i = 0; i < 8; ++i)
                        raw[8 * c16 + i] = load_raw(cnext, pix_next, pt[8 * c16 + i]);
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        if constexpr (N8 != 0 && !LIST && !PMAJ) {
            u32x2 av[NMB][2];
#pragma unroll
            for (int mb = 0; mb < NMB; ++mb)
#pragma unroll
                for (int hl = 0; hl < 2; ++hl) av[mb][hl] = A8[(mb * 2 + hl) * 64 + lane];
            constexpr int NWORD = PX / 2 > 0 ? PX / 2 : 1;
            unsigned cw[4][NWORD];
            if constexpr (BLK) {
            } else if constexpr (F8) {
#pragma unroll
                for (int m = 0; m < 2; ++m) pair_bytes(raw_word(raw[8 * N16 + 2 * m], 0), raw_word(raw[8 * N16 + 2 * m + 1], 0), cw[2 * m]);
            } else {
#pragma unroll
                for (int i = 0; i < 4; ++i) plane_words<F8>(raw[8 * N16 + i], cw[i]);
            }
#pragma unroll
            for (int q = 0; q < PX; ++q) {
                u32x2 bw;
                if constexpr (BLK) {
                    if constexpr (F8) bw = widen8(b8[q]);
                    else if constexpr (LG) {
#pragma unroll
                        for (int m = 0; m < 2; ++m) bw[m] = exp_word(b8[q][m], nm[q]);
                    } else bw = b8[q];
                }
#pragma unroll
                for (int m = 0; m < (BLK ? 0 : 2); ++m)
                    bw[m] = F8 ? widen_pair(cw[2 * m][q >> 1], q)
                          : LG ? exp_pair<F::LGB>(cw[2 * m][q >> 1], cw[2 * m + 1][q >> 1], q, nm[q])
                               : pack_pair(cw[2 * m][q >> 1], cw[2 * m + 1][q >> 1], q);
#pragma unroll
                for (int mb = 0; mb < NMB; ++mb)
#pragma unroll
                    for (int hl = 0; hl < 2; ++hl) acc[q][mb] = mfma_8<BF>(av[mb][hl], bw, acc[q][mb]);
            }
            __builtin_amdgcn_sched_barrier(0);
            if (more) {
                if constexpr (BLK) {
#pragma unroll
                    for (int q = 0; q < PX; ++q) b8[q] = blk_load8(bimg, boff, lane, q);
                } else {
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        raw[8 * N16 + i] = load_raw(cnext, pix_next, pt[8 * N16 + i]);
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }

        // (4) stage 4: each half filters its taps against the LDS tile, channel by
        //     channel (a lane's PX slots share most of their patch values)
        const float* ub = U + (unit_row(unit, wave) * WR + jr + hf * F::RH0) * P + (PERM ? 0 : jc);
        // Permuted slots: slot q, tap dx reads tile column G m + e0 + j, with G = 8 or 16 (two groups of SW = 4 or 8
        // columns) and the compile-time e0 = 2 q + dx (scale 2) or 4 q + 2 J + dx (scale 4).  The swizzled index
        // of a column x is (x % SW) NG + x / SW.  The lane's j enters through two per-lane bases, so that every
        // read is base + immediate offset: e0 % SW < SW - 1: class e0 % SW + j of the same group; otherwise the
        // last class, or (j = 1) class 0 of the next group.
        unsigned ubo[2] = {0u, 0u};                    // as element offsets into U
        if constexpr (PMAJ) {
            // column 32 q + j + dx of an unswizzled tile: the lane enters as j
            ubo[0] = ubo[1] = (unsigned)((unit_row(unit, wave) * WR + jr + hf * F::RH0) * P + jc);
        }
        if constexpr (PERM) {
            const int jx = jc % 2, m = jc / 2;
            const int row0 = (unit_row(unit, wave) * WR + jr + hf * F::RH0) * P;
            if constexpr (PSM == 3) {
                // column 12 n + 3 q + J + dx: class and carry are compile-time, the lane enters as group 3 n
                ubo[0] = ubo[1] = (unsigned)(row0 + 3 * jc);
            } else {
                // (scale 2 and scale 4 alike: the pair's columns start 8 or 16 apart, two groups of SW columns)
                ubo[0] = (unsigned)(row0 + jx * NG + 2 * m);
                ubo[1] = (unsigned)(row0 + (jx ? 1 : (F::SW - 1) * NG) + 2 * m);
            }
        }
        float outp[C][PX];
        float rinv[PX];                                // logits form: one over the sum of the pixel's exponentials
        if constexpr (LG) {
#pragma unroll
            for (int q = 0; q < PX; ++q) rinv[q] = __builtin_amdgcn_rcpf(acc[q][F::NSLOT / 16][F::NSLOT % 16]);   // the sum is at least 1
        }
#pragma unroll
        for (int c = 0; c < C; ++c) {
            if constexpr (PERM || PMAJ) {
                // The slots share few patch values (they are s pixels apart): taken all at once a channel's
                // LDS reads would hold three times the registers of the planar form.  One filter row at a
                // time; the empty statement ties the next row's addresses to this row's sums.
                static_assert(F::NSLOT % K == 0 && PX == 4, "whole filter rows per lane half");
                float sq[PX];
#pragma unroll
                for (int q = 0; q < PX; ++q) sq[q] = 0.0f;
#pragma unroll
                for (int dyv = 0; dyv < F::NSLOT / K; ++dyv) {
#pragma unroll
                    for (int q = 0; q < PX; ++q)
#pragma unroll
                        for (int dxv = 0; dxv < K; ++dxv) {
                            const int vv = dyv * K + dxv;
                            if constexpr (PMAJ) {
                                sq[q] = fmaf(acc[q][vv / 16][vv % 16], U[ubo[0] + c * UH * P + dyv * P + 32 * q + dxv], sq[q]);
                            } else if constexpr (PSM == 3) {
                                const int e = 3 * q + (unit % NSUB) + dxv;
                                sq[q] = fmaf(acc[q][vv / 16][vv % 16], U[ubo[0] + c * UH * P + dyv * P + (e & 3) * NG + (e >> 2)], sq[q]);
                            } else {
                                // column within the pair's group, before the lane's j is added; classes of SW columns
                                constexpr int SW = F::SW;
                                const int e0 = PSM == 4 ? 4 * q + 2 * (unit % NSUB) + dxv : 2 * q + dxv;
                                const bool wrap = e0 % SW == SW - 1;
                                const int imm = c * UH * P + dyv * P + (wrap ? 0 : (e0 % SW) * NG) + e0 / SW;
                                sq[q] = fmaf(acc[q][vv / 16][vv % 16], U[ubo[wrap ? 1 : 0] + imm], sq[q]);
                            }
                        }
                    asm volatile("" : "+v"(ubo[0]), "+v"(ubo[1]), "+v"(sq[0]), "+v"(sq[1]), "+v"(sq[2]), "+v"(sq[3]));
                }
#pragma unroll
                for (int q = 0; q < PX; ++q) outp[c][q] = LG ? sq[q] * rinv[q] : sq[q];
            } else {
#pragma unroll
                for (int q = 0; q < PX; ++q) {
                    float s = 0.0f;
#pragma unroll
                    for (int vv = 0; vv < F::NSLOT; ++vv) {
                        const int dyv = vv / K, dxv = vv % K;
                        const int off = c * UH * P + dyv * P + ((q + dxv) % PX) * NG + (q + dxv) / PX;
                        s = fmaf(acc[q][vv / 16][vv % 16], ub[off], s);
                    }
                    outp[c][q] = LG ? s * rinv[q] : s;
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }

        // (5) add the two halves' partial sums: one cross-half swap per slot pair
        //     leaves half 0 with pixels 0..PX/2-1 of the lane's group and half 1
        //     with the rest; one vector store per channel
        // (permuted slots: the lane's own pixels start at X0 + 4 PSM m; after the exchange below it stores
        //  the two adjacent pixels that start at X0 + 4 PSM m + 2 PSM hf + 2 (n % PSM))
        // (permuted slots, scale 4: the lane pair's pixels start at X0 + 16 m; a lane stores the four adjacent ones at
        //  X0 + 16 m + 8 hf + 4 j, once both units of the row are done)
        const int y = Y0 + unit_row(unit, wave) * WR + jr;
        // (scale 3: a lane's pixels start at X0 + 12 n; it stores the six adjacent ones at X0 + 12 n + 6 hf)
        // (pixel-major: half hf holds the lane's pixels 64 hf + j and 64 hf + 32 + j)
        const int x = PMAJ ? X0 + jc : PSM == 3 ? X0 + 12 * jc : (PERM ? X0 + 4 * PSM * (jc / 2) : X0 + PX * jc);
        const bool valid = y < a.H && x < a.W;
        const unsigned plane_px = (unsigned)a.H * (unsigned)a.W;
        const unsigned o0 = PMAJ ? (unsigned)y * (unsigned)a.W + x + hf * 64
                          : PSM == 3 ? (unsigned)y * (unsigned)a.W + x + hf * 6
                          : PERM ? (unsigned)y * (unsigned)a.W + x + hf * (2 * PSM) + (PSM == 4 ? 4 : 2) * (jc % 2)
                                 : (unsigned)y * (unsigned)a.W + x + hf * (PX / 2);   // within the image
        char* const out_img = (char*)a.out + (size_t)cur.n * C * ((size_t)plane_px * (a.io_f16 ? 2 : 4));
#pragma unroll
        for (int c = 0; c < C; ++c) {
            float tot[PX / 2];
            float tot4[4] = {0.0f, 0.0f, 0.0f, 0.0f};  // scale-4 permuted slots: the four adjacent pixels a lane stores
            float tot6[6] = {0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f};   // scale 3: the six
#pragma unroll
            for (int q = 0; q < PX / 2; ++q) {
                const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(outp[c][q]),
                                                                 __float_as_uint(outp[c][q + PX / 2]), false, false);
                tot[q] = __uint_as_float(sw[0]) + __uint_as_float(sw[1]);
            }
            if constexpr (PSM == 4) {
                // The lane pair (j = 0, 1) holds, per unit J, the pixels 16 m + 8 hf + {4 t + 2 J + j}, t = slot.
                // Unit J = 0 parks its two results; after unit J = 1 lane j' takes slot t = j' of both lanes and
                // both units: the four adjacent pixels 4 j' + {0, 1 | 2, 3} = {J = 0: j = 0, 1 | J = 1: j = 0, 1}.
                if (unit % NSUB == 0) {
                    park[c][0][0] = tot[0];
                    park[c][0][1] = tot[1];
                    continue;
                }
                const bool odd = (jc & 1) != 0;
                const unsigned g0 = __float_as_uint(odd ? park[c][0][0] : park[c][0][1]);    // what the partner stores
                const unsigned g1 = __float_as_uint(odd ? tot[0] : tot[1]);
                const float r0 = __uint_as_float(__builtin_amdgcn_update_dpp(0u, g0, 0xB1, 0xf, 0xf, false));   // quad_perm [1,0,3,2]
                const float r1 = __uint_as_float(__builtin_amdgcn_update_dpp(0u, g1, 0xB1, 0xf, 0xf, false));
                tot4[0] = odd ? r0 : park[c][0][0];
                tot4[1] = odd ? park[c][0][1] : r0;
                tot4[2] = odd ? r1 : tot[0];
                tot4[3] = odd ? tot[1] : r1;
            } else if constexpr (PSM == 3) {
                // Slot t of unit J is pixel 6 hf + 3 t + J of the lane's twelve: after the third unit the lane holds
                // the six adjacent ones (t = 0: J = 0, 1, 2; t = 1: J = 0, 1, 2).
                if (unit % NSUB != NSUB - 1) {
                    park[c][unit % NSUB][0] = tot[0];
                    park[c][unit % NSUB][1] = tot[1];
                    continue;
                }
                tot6[0] = park[c][0][0]; tot6[1] = park[c][1][0]; tot6[2] = tot[0];
                tot6[3] = park[c][0][1]; tot6[4] = park[c][1][1]; tot6[5] = tot[1];
            } else if constexpr (PSM == 2) {
                // The lane pair (j = 0, 1) holds the 4 pixels 8 m + 4 hf + {2 t + j}: lane j' takes 2 j', 2 j' + 1,
                // i.e. slot j' of both lanes of the pair.
                const unsigned t0 = __float_as_uint(tot[0]), t1 = __float_as_uint(tot[1]);
                const unsigned a0 = __builtin_amdgcn_update_dpp(0u, t0, 0xA0, 0xf, 0xf, false);   // quad_perm [0,0,2,2]
                const unsigned a1 = __builtin_amdgcn_update_dpp(0u, t1, 0xA0, 0xf, 0xf, false);
                const unsigned b0 = __builtin_amdgcn_update_dpp(0u, t0, 0xF5, 0xf, 0xf, false);   // quad_perm [1,1,3,3]
                const unsigned b1 = __builtin_amdgcn_update_dpp(0u, t1, 0xF5, 0xf, 0xf, false);
                const bool hi_slot = (jc & 1) != 0;
                tot[0] = __uint_as_float(hi_slot ? a1 : a0);
                tot[1] = __uint_as_float(hi_slot ? b1 : b0);
            }
#ifdef SR_ABLATE_STORES
            if (valid && a.N < 0) {                       // never true: the stores stay in the code, unexecuted
#else
            if (valid) {
#endif
                const unsigned oe = o0 + c * plane_px;
                if constexpr (PMAJ) {
#pragma unroll
                    for (int t = 0; t < 2; ++t) {
                        if (a.io_f16) *(__half*)(out_img + (size_t)((oe + 32 * t) * 2u)) = narrow_f16(tot[t]);
                        else *(float*)(out_img + (size_t)((oe + 32 * t) * 4u)) = tot[t];
                    }
                } else if constexpr (PSM == 4) {
                    if (a.io_f16) {
                        __half2 lo2, hi2;
                        lo2.x = narrow_f16(tot4[0]); lo2.y = narrow_f16(tot4[1]);
                        hi2.x = narrow_f16(tot4[2]); hi2.y = narrow_f16(tot4[3]);
                        u32x2 w2;
                        w2[0] = __builtin_bit_cast(unsigned, lo2);
                        w2[1] = __builtin_bit_cast(unsigned, hi2);
                        *(u32x2*)(out_img + (size_t)(oe * 2u)) = w2;
                    } else {
                        *(float4*)(out_img + (size_t)(oe * 4u)) = make_float4(tot4[0], tot4[1], tot4[2], tot4[3]);
                    }
                } else if constexpr (PSM == 3) {
#pragma unroll
                    for (int i = 0; i < 3; ++i) {
                        if (a.io_f16) {
                            __half2 h2;
                            h2.x = narrow_f16(tot6[2 * i]);
                            h2.y = narrow_f16(tot6[2 * i + 1]);
                            *(__half2*)(out_img + (size_t)((oe + 2 * i) * 2u)) = h2;
                        } else {
                            *(float2*)(out_img + (size_t)((oe + 2 * i) * 4u)) = make_float2(tot6[2 * i], tot6[2 * i + 1]);
                        }
                    }
                } else if (a.io_f16) {
                    __half* op = (__half*)(out_img + (size_t)(oe * 2u));
                    if constexpr (PX >= 4) {
#pragma unroll
                        for (int q = 0; q < PX / 2; q += 2) {
                            __half2 h2;
                            h2.x = narrow_f16(tot[q]);
                            h2.y = narrow_f16(tot[q + 1]);
                            *(__half2*)(op + q) = h2;
                        }
                    } else {
                        op[0] = narrow_f16(tot[0]);
                    }
                } else {
                    float* op = (float*)(out_img + (size_t)(oe * 4u));
                    if constexpr (PX == 8) *(float4*)op = make_float4(tot[0], tot[1], tot[2], tot[3]);
#ifdef SR_STORES_WRITE_THROUGH
                    else if constexpr (PX == 4)
                        __hip_atomic_store((unsigned long long*)op, __builtin_bit_cast(unsigned long long, make_float2(tot[0], tot[1])),
                                           __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#else
                    else if constexpr (PX == 4) *(float2*)op = make_float2(tot[0], tot[1]);
#endif
                    else op[0] = tot[0];
                }
            }
        }
        // (6) L2 write-back pacing, see the note at the top of this file: workgroups 0 .. 7 run on the eight XCDs (fewer on a partition)
        if (a.wb_ticks > 0 && (int)blockIdx.x < a.wb_flushers && wave == 0) {
            const unsigned long long now = __builtin_amdgcn_s_memrealtime();
            if (now - wb_last >= (unsigned long long)a.wb_ticks) {
                wb_last = now;
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
            }
        }
        // (2) prefetch the next tile's LR footprint from inside the unit loop, where
        //     the wavefront waits on memory anyway, and not in the barrier-to-barrier
        //     up-sampling phase that every wavefront of the workgroup has to sit out
        if (unit == (NU > 1 ? 1 : 0) && more_tiles) load_lr(nxt, lane, lrv, lrpar);
        }   // unit
        cur = nxt;
    }
}

// ---------------------------------------------------------------------------
// Host side: launch of one instantiation on a persistent grid.
// ---------------------------------------------------------------------------
// CUs of the current device (asked once per device and thread)
inline int compute_units() {
    static thread_local int known[64];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
    if (known[dev] == 0) {
        int cus = 0;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1) cus = 256;
        known[dev] = cus;
    }
    return known[dev];
}

// rate of the constant clock s_memrealtime reads, in kHz (asked once per device and thread; 100 MHz if the runtime
// does not say)
inline long long wall_clock_khz() {
    static thread_local int known[64];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 100000;
    if (known[dev] == 0) {
        int khz = 0;
        if (hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, dev) != hipSuccess || khz < 1000) khz = 100000;
        known[dev] = khz;
    }
    return known[dev];
}

template <int K, int C, int NP8, int PX, int WR, int NW, int NU, int WPE, int CT = CT_F16, int SMIN = 2, bool BIG = false,
          int PSM = 0>
hipError_t launch_one(const AssembleArgs& a0, hipStream_t st) {
    using F = Cfg<K, C, NP8, PX, WR, NW, NU, CT, SMIN, (PSM == 4 ? 2 : (PSM == 3 ? 3 : 1)), (PSM == 8 ? 1 : 0)>;
    if (a0.s < SMIN) return hipErrorInvalidValue;       // its LDS footprint buffers would be too small
    if ((a0.pre_shuffle != 0) != (PSM >= 1 && PSM <= 4) || (a0.pixel_major != 0) != (PSM == 8)) return hipErrorInvalidValue;
    // logits: a softmax over every atom, so every plane is folded
    if ((a0.logits != 0) != (CT == CT_LOGIT || CT == CT_LOGIT_BF16) || (a0.logits && a0.n_fold != a0.L)) return hipErrorInvalidValue;
    if (a0.logits && (a0.coeff_dtype == SR_BF16) != (CT == CT_LOGIT_BF16)) return hipErrorInvalidValue;
    if (PSM == 8 && (a0.W % 128 != 0 || a0.L != 8 * NP8 || a0.n_fold != a0.L)) return hipErrorInvalidValue;
    if ((a0.blocked != 0) != (PSM == 9)) return hipErrorInvalidValue;
    if (PSM == 9 && (a0.W % 128 != 0 || a0.L != 8 * NP8 || a0.n_fold != a0.L)) return hipErrorInvalidValue;
    // permuted pixel slots: a lane owns four whole LR columns, the image must end on such a group
    if ((PSM == 2 || PSM == 3 || PSM == 4) && (a0.s != PSM || a0.w % 4 != 0)) return hipErrorInvalidValue;
    AssembleArgs a = a0;
#ifndef SR_NO_L2_WRITEBACK
    // L2 write-back pacing where the coefficient stream is the bound: 49 atoms and more, not the 8-bit and list forms
    // (measured neutral at 43 kept atoms, 1-2 % slower below and with 8-bit coefficients)
    if (NP8 >= 9 && CT != CT_F8 && !F::LIST) {
        // 16 us of the constant-rate clock the kernel reads (7x7 atoms: 28 us, measured); one asking workgroup per XCD
        // (32 CUs each: eight on the whole device, fewer on a partition of it)
        a.wb_ticks = (int)((K == 7 ? 28LL : 16LL) * wall_clock_khz() / 1000);
        const int xcds = compute_units() / 32;
        a.wb_flushers = xcds < 1 ? 1 : (xcds > 8 ? 8 : xcds);
    }
#endif
    const int tiles_x = (a.W + F::TW - 1) / F::TW, tiles_y = (a.H + F::TH - 1) / F::TH;
    a.xlast = (tiles_x - 1) * F::TW;
    if (a.W % PX != 0) {                                // ragged rows: the last tile column ends at the image edge
        if (a.W < F::TW) return hipErrorInvalidValue;
        a.xlast = a.W - F::TW;
    }
    const long long nt = (long long)tiles_x * tiles_y * a.N;
    if (nt > 0x7fffffffLL) return hipErrorInvalidValue;
    // as many workgroups as stay resident (WPE wavefronts per SIMD)
    const int cus = compute_units();
    const int cap = cus * (4 * WPE / NW > 0 ? 4 * WPE / NW : 1);
    const int blocks = nt < cap ? (int)nt : cap;
    hipLaunchKernelGGL((k_assemble_mfma<K, C, NP8, PX, WR, NW, NU, WPE, CT, SMIN, BIG, PSM>), dim3(blocks), dim3(F::NT), 0, st,
                       a, tiles_x, tiles_y, (int)nt);
    return hipGetLastError();
}

}  // namespace srd
