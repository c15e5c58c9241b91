// Matrix-core kernel for fp16 coefficients (gfx950 / CDNA4).
//
// One fused kernel does stage 1 (up-sampling), stage 3 (F_i = Phi_i D, paper
// Eq. 2) and stage 4 (y_i = F_i B_i^T) for a tile of HR pixels; neither F nor B
// of Eq. 3 ever reaches memory.  The only large stream is the coefficient
// tensor Phi (L planes, fp16), read exactly once with 16-byte (or 8-byte) loads.
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
//   * as B operand it supplies atoms 8*hf .. 8*hf+7 of the chunk for pixel j,
//     so lanes j and j+32 load different coefficient planes of the SAME pixels:
//     each lane loads PX consecutive pixels of a plane with one vector load and
//     re-packs (atom pair, pixel) with v_perm_b32;
//   * the MFMA result leaves pixel j's taps split over lanes j and j+32
//     (rows 8*(v/4) + 4*hf + v%4).  Dictionary rows are ordered so that half 0
//     owns filter rows 0 .. RH0-1 and half 1 owns rows RH0 .. (one dummy row
//     with zero weights): both halves then use the same LDS offsets, shifted by
//     RH0 tile rows.  Each half filters its taps against the LDS patch tile
//     and the two partial sums are exchanged across the halves.
//
// The up-sampled tile is stored in LDS column-swizzled, (x % PX) major, so the
// 32 pixels of one MFMA (stride PX in x) read consecutive banks.
#include "sr_device.h"
#include "sr_launch.h"

namespace srd {

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x2 __attribute__((ext_vector_type(2)));

template <int K, int C, int NP8, int PX, int WR, int NW>
struct Cfg {
    static constexpr int KK = K * K, R = (K - 1) / 2;
    static constexpr int RH0 = (K + 1) / 2;            // filter rows owned by lane half 0
    static constexpr int NSLOT = RH0 * K;              // accumulator rows used per half
    static constexpr int NMB = (NSLOT + 15) / 16;      // 32-row MFMA blocks
    static constexpr int WC = 32 / WR;                 // lane columns per wavefront
    static constexpr int TW = WC * PX, TH = WR * NW;   // tile of HR pixels per workgroup
    static constexpr int NT = 64 * NW;
    static constexpr int UW = TW + K - 1;
    static constexpr int UH = TH + K;                  // + one dummy row for half 1
    static constexpr int NG = (UW + PX - 1) / PX;      // stride between x % PX classes
    static constexpr int P0 = PX * NG;
    // rows of one wavefront must land on disjoint banks: pitch == WC (mod 32)
    static constexpr int P = WR == 1 ? P0 : P0 + ((WC - P0 % 32) + 32) % 32;
    static constexpr int MAXLRY = (UH - 1) / 2 + 5, MAXLRX = (UW - 1) / 2 + 5;
    static constexpr int N16 = NP8 / 2, N8 = NP8 % 2;  // 16-atom steps, optional 8-atom step
    static constexpr int NLOAD = 8 * N16 + 4 * N8;     // coefficient loads per lane and tile
    static constexpr int NLR = (C * MAXLRY * MAXLRX + NT - 1) / NT;
    static constexpr int AREGS = (N16 * 8 + N8 * 4) * NMB;
    static constexpr bool A_IN_REGS = false && AREGS <= 48;     // else the operand is re-read from LDS
};

template <int PX> struct RawT;
template <> struct RawT<8> { typedef u32x4 type; };
template <> struct RawT<4> { typedef u32x2 type; };

template <int PX>
__device__ __forceinline__ unsigned raw_word(const typename RawT<PX>::type& v, int m) { return v[m]; }

// (atom pair, pixel q) from two planes' packed pixels
__device__ __forceinline__ unsigned pack_pair(unsigned plane_even, unsigned plane_odd, int q) {
    return __builtin_amdgcn_perm(plane_odd, plane_even, (q & 1) ? 0x07060302u : 0x05040100u);
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

template <int K, int C, int NP8, int PX, int WR, int NW, int WPE>
__global__ __launch_bounds__(64 * NW, WPE)
void k_assemble_mfma(const AssembleArgs a, const int tiles_x, const int tiles_y, const int ntiles) {
    using F = Cfg<K, C, NP8, PX, WR, NW>;
    using Raw = typename RawT<PX>::type;
    constexpr int NT = F::NT, P = F::P, NG = F::NG, UH = F::UH, UW = F::UW;
    constexpr int N16 = F::N16, N8 = F::N8, NMB = F::NMB;
    constexpr int LRSZ = F::MAXLRY * F::MAXLRX;

    __shared__ float U[C * UH * P];
    __shared__ float hbuf[C * F::MAXLRY * UW];
    __shared__ float lrT[C * LRSZ];
    __shared__ float4 xw[UW], yw[UH];
    __shared__ int xb[UW], yb[UH];
    __shared__ u32x4 A16[(N16 ? N16 : 1) * NMB * 2 * 64];
    __shared__ u32x2 A8[NMB * 2 * 64];
    __shared__ unsigned ptab[2 * F::NLOAD];   // byte offset of the plane each lane half loads

    const int tid0 = threadIdx.x;

    // ---- dictionary operand tables: gamma * D[kept], hi + lo fp16 ---------------
    auto dval = [&](int idx, int tap) -> float {
        if (tap < 0 || idx >= a.n_fold) return 0.0f;
        return a.gamma[idx] * a.dict[(size_t)a.kept[idx] * F::KK + tap];
    };
    const unsigned plane_b = (unsigned)a.H * (unsigned)a.W * 2u;   // bytes per coefficient plane
    for (int e = tid0; e < 2 * F::NLOAD; e += NT) {
        const int h = e / F::NLOAD, i = e - h * F::NLOAD;
        // load i of half h serves folded atom idx; padding atoms re-read the last plane
        const int idx = i < 8 * N16 ? 16 * (i >> 3) + 8 * h + (i & 7) : 16 * N16 + 4 * h + (i - 8 * N16);
        ptab[e] = (unsigned)a.kept[idx < a.n_fold ? idx : a.n_fold - 1] * plane_b;
    }
    for (int e = tid0; e < N16 * NMB * 64; e += NT) {
        const int l = e & 63, blk = e >> 6, mb = blk % NMB, c16 = blk / NMB;
        const int tap = tap_of_row<K>(l & 31, mb);
        f16x8 hi, lo;
#pragma unroll
        for (int jj = 0; jj < 8; ++jj) {
            const float d = dval(16 * c16 + 8 * (l >> 5) + jj, tap);
            hi[jj] = (_Float16)d;
            lo[jj] = (_Float16)(d - (float)hi[jj]);
        }
        A16[(blk * 2 + 0) * 64 + l] = __builtin_bit_cast(u32x4, hi);
        A16[(blk * 2 + 1) * 64 + l] = __builtin_bit_cast(u32x4, lo);
    }
    if (N8) {
        for (int e = tid0; e < NMB * 64; e += NT) {
            const int l = e & 63, mb = e >> 6;
            const int tap = tap_of_row<K>(l & 31, mb);
            f16x4 hi, lo;
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) {
                const float d = dval(16 * N16 + 4 * (l >> 5) + jj, tap);
                hi[jj] = (_Float16)d;
                lo[jj] = (_Float16)(d - (float)hi[jj]);
            }
            A8[(mb * 2 + 0) * 64 + l] = __builtin_bit_cast(u32x2, hi);
            A8[(mb * 2 + 1) * 64 + l] = __builtin_bit_cast(u32x2, lo);
        }
    }
    __syncthreads();

    f16x8 a16r[F::A_IN_REGS ? (N16 ? N16 : 1) : 1][NMB][2];
    f16x4 a8r[NMB][2];
    if constexpr (F::A_IN_REGS) {
#pragma unroll
        for (int c16 = 0; c16 < N16; ++c16)
#pragma unroll
            for (int mb = 0; mb < NMB; ++mb)
#pragma unroll
                for (int hl = 0; hl < 2; ++hl)
                    a16r[c16][mb][hl] = __builtin_bit_cast(f16x8, A16[((c16 * NMB + mb) * 2 + hl) * 64 + (tid0 & 63)]);
    }
    if (N8) {
#pragma unroll
        for (int mb = 0; mb < NMB; ++mb)
#pragma unroll
            for (int hl = 0; hl < 2; ++hl)
                a8r[mb][hl] = __builtin_bit_cast(f16x4, A8[(mb * 2 + hl) * 64 + (tid0 & 63)]);
    }

    for (int t = blockIdx.x; t < ntiles; t += gridDim.x) {
        // Per-iteration copy of the thread id the optimiser cannot see through:
        // index arithmetic derived from it is recomputed each tile instead of
        // being hoisted out of the loop into dozens of long-lived registers.
        int tid = tid0;
        asm volatile("" : "+v"(tid));
        const int lane = tid & 63, wave = tid >> 6;
        const int hf = lane >> 5, j = lane & 31, jr = j / F::WC, jc = j % F::WC;
        const int per_img = tiles_x * tiles_y;
        const int n = t / per_img, r2 = t - n * per_img;
        const int tyi = r2 / tiles_x, txi = r2 - tyi * tiles_x;
        const int X0 = txi * F::TW, Y0 = tyi * F::TH;
        const TileOrigin o = tile_origin(Y0, X0, F::R, UH, a.H, a.W, a.s);

        // (1) LR footprint of the tile -> registers (issued first: loads return in order)
        float lrv[F::NLR];
#pragma unroll
        for (int u = 0; u < F::NLR; ++u) {
            const int idx = tid + u * NT;
            lrv[u] = 0.0f;
            if (idx < C * LRSZ) {
                const int c = idx / LRSZ, rem = idx - c * LRSZ;
                const int ry = rem / F::MAXLRX, rx = rem - ry * F::MAXLRX;
                const int yy = clampi(o.ly0 + ry, 0, a.h - 1), xx = clampi(o.lx0 + rx, 0, a.w - 1);
                const size_t off = (((size_t)n * C + c) * a.h + yy) * a.w + xx;
                lrv[u] = a.io_f16 ? __half2float(((const __half*)a.lr)[off]) : ((const float*)a.lr)[off];
            }
        }

        // (2) this lane's coefficients: PX pixels of NLOAD planes, all in flight at once.
        //     Out-of-image lanes and padding atoms re-read a valid address; their
        //     results are never stored / meet zero dictionary rows.
        const int y = Y0 + wave * WR + jr, x = X0 + PX * jc;
        const bool valid = y < a.H && x < a.W;
        const int yc = y < a.H ? y : a.H - 1, xc = x < a.W ? x : a.W - PX;
        const char* cimg = (const char*)a.coeff + (size_t)n * a.L * (size_t)plane_b;
        const unsigned pix_off = ((unsigned)yc * (unsigned)a.W + (unsigned)xc) * 2u;
        const unsigned* pt = ptab + hf * F::NLOAD;
        Raw raw[F::NLOAD];
#pragma unroll
        for (int c16 = 0; c16 < N16; ++c16)
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const unsigned voff = pix_off + pt[8 * c16 + i];
                raw[8 * c16 + i] = __builtin_nontemporal_load((const Raw*)(cimg + voff));
            }
        if (N8) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const unsigned voff = pix_off + pt[8 * N16 + i];
                raw[8 * N16 + i] = __builtin_nontemporal_load((const Raw*)(cimg + voff));
            }
        }

        // (3) stage 1: up-sampled patch tile -> LDS (coefficient loads stay in flight)
        build_taps<UW, F::MAXLRX, NT>(X0, F::R, a.W, a.s, o.lx0, xw, xb, tid);
        build_taps<UH, F::MAXLRY, NT>(Y0, F::R, a.H, a.s, o.ly0, yw, yb, tid);
#pragma unroll
        for (int u = 0; u < F::NLR; ++u) {
            const int idx = tid + u * NT;
            if (idx < C * LRSZ) lrT[idx] = lrv[u];
        }
        __syncthreads();
#pragma unroll
        for (int c = 0; c < C; ++c)
            hpass<F::MAXLRX, UW, NT>(lrT + c * LRSZ, hbuf + c * F::MAXLRY * UW, xw, xb, o.nly, tid);
        __syncthreads();
#pragma unroll
        for (int c = 0; c < C; ++c) {
            float* Uc = U + c * UH * P;
            vpass<UW, UH, NT>(hbuf + c * F::MAXLRY * UW, yw, yb, tid,
                              [&](int yy, int xx, float v) { Uc[yy * P + (xx % PX) * NG + xx / PX] = v; });
        }
        __syncthreads();

        // (4) per pixel slot: stage 3 on the matrix cores, stage 4 against the LDS tile
        const float* ub = U + (wave * WR + jr + hf * F::RH0) * P + jc;
        float outp[PX][C];
#pragma unroll
        for (int q = 0; q < PX; ++q) {
            f32x16 acc[NMB];
#pragma unroll
            for (int mb = 0; mb < NMB; ++mb)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[mb][v] = 0.0f;
#pragma unroll
            for (int c16 = 0; c16 < N16; ++c16) {
                u32x4 bw;
#pragma unroll
                for (int m = 0; m < 4; ++m)
                    bw[m] = pack_pair(raw_word<PX>(raw[8 * c16 + 2 * m], q >> 1),
                                      raw_word<PX>(raw[8 * c16 + 2 * m + 1], q >> 1), q);
                const f16x8 b = __builtin_bit_cast(f16x8, bw);
#pragma unroll
                for (int mb = 0; mb < NMB; ++mb)
#pragma unroll
                    for (int hl = 0; hl < 2; ++hl) {
                        f16x8 av;
                        if constexpr (F::A_IN_REGS) av = a16r[c16][mb][hl];
                        else av = __builtin_bit_cast(f16x8, A16[((c16 * NMB + mb) * 2 + hl) * 64 + lane]);
                        acc[mb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(av, b, acc[mb], 0, 0, 0);
                    }
            }
            if (N8) {
                u32x2 bw;
#pragma unroll
                for (int m = 0; m < 2; ++m)
                    bw[m] = pack_pair(raw_word<PX>(raw[8 * N16 + 2 * m], q >> 1),
                                      raw_word<PX>(raw[8 * N16 + 2 * m + 1], q >> 1), q);
                const f16x4 b = __builtin_bit_cast(f16x4, bw);
#pragma unroll
                for (int mb = 0; mb < NMB; ++mb)
#pragma unroll
                    for (int hl = 0; hl < 2; ++hl)
                        acc[mb] = __builtin_amdgcn_mfma_f32_32x32x8f16(a8r[mb][hl], b, acc[mb], 0, 0, 0);
            }
#pragma unroll
            for (int c = 0; c < C; ++c) {
                float s = 0.0f;
#pragma unroll
                for (int vv = 0; vv < F::NSLOT; ++vv) {
                    const int dyv = vv / K, dxv = vv % K;
                    const int off = c * UH * P + dyv * P + ((q + dxv) % PX) * NG + (q + dxv) / PX;
                    s = fmaf(acc[vv / 16][vv % 16], ub[off], s);
                }
                outp[q][c] = s;
                __builtin_amdgcn_sched_barrier(0);
            }
            // one slot at a time: keeps a single accumulator block live (other
            // wavefronts of the SIMD overlap their vector work with these MFMAs)
            __builtin_amdgcn_sched_barrier(0);
        }

        // (5) add the two halves' partial sums; half 0 keeps pixels 0..PX/2-1 of the
        //     lane's group, half 1 the rest; one vector store per channel
#pragma unroll
        for (int c = 0; c < C; ++c) {
            float tot[PX / 2];
#pragma unroll
            for (int q = 0; q < PX / 2; ++q) {
                const float mine = hf ? outp[q + PX / 2][c] : outp[q][c];
                const float send = hf ? outp[q][c] : outp[q + PX / 2][c];
                tot[q] = mine + __shfl_xor(send, 32, 64);
            }
            if (valid) {
                const size_t o0 = (((size_t)n * C + c) * a.H + y) * a.W + x + hf * (PX / 2);
                if (a.io_f16) {
                    __half* op = (__half*)a.out + o0;
#pragma unroll
                    for (int q = 0; q < PX / 2; q += 2) {
                        __half2 h2;
                        h2.x = narrow_f16(tot[q]);
                        h2.y = narrow_f16(tot[q + 1]);
                        *(__half2*)(op + q) = h2;
                    }
                } else {
                    float* op = (float*)a.out + o0;
                    if constexpr (PX == 8)
                        *(float4*)op = make_float4(tot[0], tot[1], tot[2], tot[3]);
                    else
                        *(float2*)op = make_float2(tot[0], tot[1]);
                }
            }
        }
    }
}

// ---------------------------------------------------------------------------
// Host side: which instantiation serves a call.
// ---------------------------------------------------------------------------
namespace {

struct Shape { int K, C, NP8, PX, WR, NW; };

template <int K, int C, int NP8, int PX, int WR, int NW, int WPE = 2>
hipError_t launch_one(const AssembleArgs& a, int persistent, hipStream_t st) {
    using F = Cfg<K, C, NP8, PX, WR, NW>;
    const int tiles_x = (a.W + F::TW - 1) / F::TW, tiles_y = (a.H + F::TH - 1) / F::TH;
    const long long nt = (long long)tiles_x * tiles_y * a.N;
    if (nt > 0x7fffffffLL) return hipErrorInvalidValue;
    int blocks = (int)nt;
    if (persistent) {
        int dev = 0, cus = 256;
        if (hipGetDevice(&dev) == hipSuccess)
            hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
        const int cap = cus * 2;
        if (blocks > cap) blocks = cap;
    }
    hipLaunchKernelGGL((k_assemble_mfma<K, C, NP8, PX, WR, NW, WPE>), dim3(blocks), dim3(F::NT), 0, st,
                       a, tiles_x, tiles_y, (int)nt);
    return hipGetLastError();
}

// atoms-per-launch capacity (in groups of 8) of the built instantiations
int np8_for(int k, int n_fold) {
    const int need = (n_fold + 7) / 8;
    if (k == 5) return need <= 9 ? 9 : (need <= 16 ? 16 : 0);
    if (k == 7) return need <= 16 ? 16 : 0;
    return 0;
}

}  // namespace

bool mfma_supported(const AssembleArgs& a, int k, bool coeff_f16, int tile) {
    if (!coeff_f16 || (k != 5 && k != 7) || (a.C != 1 && a.C != 3)) return false;
    if (a.W % 8 != 0 || a.W < 8 || a.H < 1) return false;
    if (((uintptr_t)a.coeff % 16) != 0 || ((uintptr_t)a.out % 16) != 0) return false;
    if ((unsigned long long)a.L * a.H * a.W * 2ull >= (1ull << 32)) return false;   // 32-bit plane offsets
    if (np8_for(k, a.n_fold) == 0) return false;
    if (tile < 0 || tile > 0) return false;
    return true;
}

hipError_t launch_mfma(const AssembleArgs& a, int k, bool io_f16, int tile, hipStream_t st) {
    (void)io_f16;
    const int np8 = np8_for(k, a.n_fold);
    const int persistent = 0;
    if (k == 5 && np8 == 9) {
        return a.C == 3 ? launch_one<5, 3, 9, 4, 2, 4, 2>(a, persistent, st)
                        : launch_one<5, 1, 9, 4, 1, 4>(a, persistent, st);
    }
    if (k == 5 && np8 == 16) {
        return a.C == 3 ? launch_one<5, 3, 16, 4, 2, 4>(a, persistent, st)
                        : launch_one<5, 1, 16, 4, 2, 4>(a, persistent, st);
    }
    if (k == 7 && np8 == 16) {
        return a.C == 3 ? launch_one<7, 3, 16, 4, 2, 4>(a, persistent, st)
                        : launch_one<7, 1, 16, 4, 2, 4>(a, persistent, st);
    }
    return hipErrorInvalidValue;
}

}  // namespace srd
