// Matrix-core kernel for fp16 coefficients (gfx950 / CDNA4).
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
    static constexpr int NXC = (MAXLRX + 63) / 64;     // 64-column chunks of the LR footprint
    static constexpr int NLRP = (C * MAXLRY + NW - 1) / NW;   // (channel,row) pairs per wavefront
};

template <int PX> struct RawT;
template <> struct RawT<8> { typedef u32x4 type; };
template <> struct RawT<4> { typedef u32x2 type; };
template <> struct RawT<2> { typedef unsigned type; };

__device__ __forceinline__ unsigned raw_word(const u32x4& v, int m) { return v[m]; }
__device__ __forceinline__ unsigned raw_word(const u32x2& v, int m) { return v[m]; }
__device__ __forceinline__ unsigned raw_word(const unsigned& v, int) { return v; }

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

struct TilePos { int n, Y0, X0; };

template <int K, int C, int NP8, int PX, int WR, int NW, int WPE>
__global__ __launch_bounds__(64 * NW, WPE)
void k_assemble_mfma(const AssembleArgs a, const int tiles_x, const int tiles_y, const int ntiles) {
    using F = Cfg<K, C, NP8, PX, WR, NW>;
    using Raw = typename RawT<PX>::type;
    constexpr int NT = F::NT, P = F::P, NG = F::NG, UH = F::UH, UW = F::UW;
    constexpr int N16 = F::N16, N8 = F::N8, NMB = F::NMB;
    constexpr int MAXLRY = F::MAXLRY, MAXLRX = F::MAXLRX;

    __shared__ float U[C * UH * P];
    __shared__ float hbuf[C * MAXLRY * UW];
    __shared__ float lrT[C * MAXLRY * MAXLRX];
    __shared__ float4 xw[UW], yw[UH];
    __shared__ int xb[UW], yb[UH];
    __shared__ u32x4 A16[(N16 ? N16 : 1) * NMB * 2 * 64];
    __shared__ u32x2 A8[NMB * 2 * 64];
    __shared__ unsigned ptab[2 * F::NLOAD];   // byte offset of the plane each lane half loads

    const int tid0 = threadIdx.x;
    if ((int)blockIdx.x >= ntiles) return;

    // ---- once per workgroup: plane offsets and dictionary operand tables ---------
    const unsigned plane_b = (unsigned)a.H * (unsigned)a.W * 2u;   // bytes per coefficient plane
    for (int e = tid0; e < 2 * F::NLOAD; e += NT) {
        const int h = e / F::NLOAD, i = e - h * F::NLOAD;
        // load i of half h serves folded atom idx; padding atoms re-read the last plane
        const int idx = i < 8 * N16 ? 16 * (i >> 3) + 8 * h + (i & 7) : 16 * N16 + 4 * h + (i - 8 * N16);
        ptab[e] = (unsigned)a.kept[idx < a.n_fold ? idx : a.n_fold - 1] * plane_b;
    }
    auto dval = [&](int idx, int tap) -> float {    // gamma * D[kept], zero for padding
        if (tap < 0 || idx >= a.n_fold) return 0.0f;
        return a.gamma[idx] * a.dict[(size_t)a.kept[idx] * F::KK + tap];
    };
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

    const int per_img = tiles_x * tiles_y;
    auto tile_pos = [&](int t) -> TilePos {
        TilePos p;
        p.n = t / per_img;
        const int r2 = t - p.n * per_img, tyi = r2 / tiles_x;
        p.Y0 = tyi * F::TH;
        p.X0 = (r2 - tyi * tiles_x) * F::TW;
        return p;
    };

    // LR footprint of a tile -> registers.  Wavefront w takes (channel,row) pairs
    // w, w+NW, ...; the lane is the column.  Everything but the column is scalar.
    auto load_lr = [&](const TilePos tp, int lane, int wave, float (&lrv)[F::NLRP][F::NXC]) {
        const TileOrigin o = tile_origin(tp.Y0, tp.X0, F::R, UH, a.H, a.W, a.s);
        int xo[F::NXC];
#pragma unroll
        for (int xc = 0; xc < F::NXC; ++xc) xo[xc] = clampi(o.lx0 + lane + 64 * xc, 0, a.w - 1);
#pragma unroll
        for (int u = 0; u < F::NLRP; ++u) {
            const int p = wave + NW * u, c = p / MAXLRY, ry = p - c * MAXLRY;
#pragma unroll
            for (int xc = 0; xc < F::NXC; ++xc) lrv[u][xc] = 0.0f;
            if (p < C * MAXLRY && ry < o.nly) {
                const size_t row = (((size_t)tp.n * C + c) * a.h + clampi(o.ly0 + ry, 0, a.h - 1)) * (size_t)a.w;
#pragma unroll
                for (int xc = 0; xc < F::NXC; ++xc)
                    lrv[u][xc] = a.io_f16 ? __half2float(((const __half*)a.lr + row)[xo[xc]])
                                          : ((const float*)a.lr + row)[xo[xc]];
            }
        }
    };

    // coefficient base of a tile for this lane: image base (scalar) + pixel offset
    auto phi_base = [&](const TilePos tp, int wave, int jr, int jc, unsigned& pix_off) -> const char* {
        const int y = tp.Y0 + wave * WR + jr, x = tp.X0 + PX * jc;
        const int yc = y < a.H ? y : a.H - 1, xc = x < a.W ? x : a.W - PX;   // out-of-image lanes re-read
        pix_off = ((unsigned)yc * (unsigned)a.W + (unsigned)xc) * 2u;         // a valid address; never stored
        return (const char*)a.coeff + (size_t)tp.n * a.L * (size_t)plane_b;
    };

    Raw raw[F::NLOAD];
    float lrv[F::NLRP][F::NXC];
    {
        const int lane = tid0 & 63, wave = tid0 >> 6, hf = lane >> 5, j = lane & 31;
        const TilePos tp = tile_pos(blockIdx.x);
        load_lr(tp, lane, wave, lrv);
        unsigned pix_off;
        const char* cimg = phi_base(tp, wave, j / F::WC, j % F::WC, pix_off);
        const unsigned* pt = ptab + hf * F::NLOAD;
#pragma unroll
        for (int i = 0; i < F::NLOAD; ++i)
            raw[i] = __builtin_nontemporal_load((const Raw*)(cimg + (pix_off + pt[i])));
    }

    for (int t = blockIdx.x; t < ntiles; t += gridDim.x) {
        // Per-iteration copy of the thread id the optimiser cannot see through:
        // index arithmetic derived from it is recomputed each tile instead of
        // being hoisted out of the loop into dozens of long-lived registers.
        int tid = tid0;
        asm volatile("" : "+v"(tid));
        const int lane = tid & 63, wave = tid >> 6;
        const int hf = lane >> 5, j = lane & 31, jr = j / F::WC, jc = j % F::WC;
        const TilePos tp = tile_pos(t);
        const TileOrigin o = tile_origin(tp.Y0, tp.X0, F::R, UH, a.H, a.W, a.s);

        // (1) stage 1: up-sampled patch tile -> LDS.  This tile's coefficient loads
        //     were issued one iteration ago and stay in flight meanwhile.
        build_taps<UW, MAXLRX, NT>(tp.X0, F::R, a.W, a.s, o.lx0, xw, xb, tid);
        build_taps<UH, MAXLRY, NT>(tp.Y0, F::R, a.H, a.s, o.ly0, yw, yb, tid);
#pragma unroll
        for (int u = 0; u < F::NLRP; ++u) {
            const int p = wave + NW * u;
            if (p < C * MAXLRY) {
#pragma unroll
                for (int xc = 0; xc < F::NXC; ++xc)
                    if (lane + 64 * xc < MAXLRX) lrT[p * MAXLRX + lane + 64 * xc] = lrv[u][xc];
            }
        }
        __syncthreads();
        hpass_cols<C, MAXLRY, MAXLRX, UW, NT>(lrT, hbuf, xw, xb, o.nly, tid);
        __syncthreads();
        vpass_cols<C, MAXLRY, UW, UH, NT>(hbuf, yw, yb, tid, [&](int c, int yy, int xx, float v) {
            U[c * UH * P + yy * P + (xx % PX) * NG + xx / PX] = v;
        });
        __syncthreads();

        // (2) prefetch for the next tile of this workgroup: LR footprint now, the
        //     coefficient steps as their registers fall free below
        const int tn = t + gridDim.x;
        const bool more = tn < ntiles;
        const TilePos tq = tile_pos(more ? tn : t);
        if (more) load_lr(tq, lane, wave, lrv);
        unsigned pix_next;
        const char* cnext = phi_base(tq, wave, jr, jc, pix_next);
        const unsigned* pt = ptab + hf * F::NLOAD;

        // (3) stage 3 on the matrix cores: atom steps outer, pixel slots inner
        f32x16 acc[PX][NMB];
#pragma unroll
        for (int q = 0; q < PX; ++q)
#pragma unroll
            for (int mb = 0; mb < NMB; ++mb)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[q][mb][v] = 0.0f;
#pragma unroll
        for (int c16 = 0; c16 < N16; ++c16) {
            f16x8 av[NMB][2];
#pragma unroll
            for (int mb = 0; mb < NMB; ++mb)
#pragma unroll
                for (int hl = 0; hl < 2; ++hl)
                    av[mb][hl] = __builtin_bit_cast(f16x8, A16[((c16 * NMB + mb) * 2 + hl) * 64 + lane]);
#pragma unroll
            for (int q = 0; q < PX; ++q) {
                u32x4 bw;
#pragma unroll
                for (int m = 0; m < 4; ++m)
                    bw[m] = pack_pair(raw_word(raw[8 * c16 + 2 * m], q >> 1),
                                      raw_word(raw[8 * c16 + 2 * m + 1], q >> 1), q);
                const f16x8 b = __builtin_bit_cast(f16x8, bw);
#pragma unroll
                for (int mb = 0; mb < NMB; ++mb)
#pragma unroll
                    for (int hl = 0; hl < 2; ++hl)
                        acc[q][mb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(av[mb][hl], b, acc[q][mb], 0, 0, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
            if (more) {
#pragma unroll
                for (int i = 0; i < 8; ++i)
                    raw[8 * c16 + i] = __builtin_nontemporal_load((const Raw*)(cnext + (pix_next + pt[8 * c16 + i])));
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        if (N8) {
            f16x4 av[NMB][2];
#pragma unroll
            for (int mb = 0; mb < NMB; ++mb)
#pragma unroll
                for (int hl = 0; hl < 2; ++hl)
                    av[mb][hl] = __builtin_bit_cast(f16x4, A8[(mb * 2 + hl) * 64 + lane]);
#pragma unroll
            for (int q = 0; q < PX; ++q) {
                u32x2 bw;
#pragma unroll
                for (int m = 0; m < 2; ++m)
                    bw[m] = pack_pair(raw_word(raw[8 * N16 + 2 * m], q >> 1),
                                      raw_word(raw[8 * N16 + 2 * m + 1], q >> 1), q);
                const f16x4 b = __builtin_bit_cast(f16x4, bw);
#pragma unroll
                for (int mb = 0; mb < NMB; ++mb)
#pragma unroll
                    for (int hl = 0; hl < 2; ++hl)
                        acc[q][mb] = __builtin_amdgcn_mfma_f32_32x32x8f16(av[mb][hl], b, acc[q][mb], 0, 0, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
            if (more) {
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    raw[8 * N16 + i] = __builtin_nontemporal_load((const Raw*)(cnext + (pix_next + pt[8 * N16 + i])));
            }
            __builtin_amdgcn_sched_barrier(0);
        }

        // (4) stage 4: each half filters its taps against the LDS tile, channel by
        //     channel (a lane's PX slots share most of their patch values)
        const float* ub = U + (wave * WR + jr + hf * F::RH0) * P + jc;
        float outp[C][PX];
#pragma unroll
        for (int c = 0; c < C; ++c) {
#pragma unroll
            for (int q = 0; q < PX; ++q) {
                float s = 0.0f;
#pragma unroll
                for (int vv = 0; vv < F::NSLOT; ++vv) {
                    const int dyv = vv / K, dxv = vv % K;
                    const int off = c * UH * P + dyv * P + ((q + dxv) % PX) * NG + (q + dxv) / PX;
                    s = fmaf(acc[q][vv / 16][vv % 16], ub[off], s);
                }
                outp[c][q] = s;
            }
            __builtin_amdgcn_sched_barrier(0);
        }

        // (5) add the two halves' partial sums; half 0 keeps pixels 0..PX/2-1 of the
        //     lane's group, half 1 the rest; one vector store per channel
        const int y = tp.Y0 + wave * WR + jr, x = tp.X0 + PX * jc;
        const bool valid = y < a.H && x < a.W;
        const int swap_addr = (lane ^ 32) << 2;
        const size_t plane_px = (size_t)a.H * a.W;
        const size_t o0 = ((size_t)tp.n * C * a.H + y) * (size_t)a.W + x + hf * (PX / 2);
#pragma unroll
        for (int c = 0; c < C; ++c) {
            float tot[PX / 2];
#pragma unroll
            for (int q = 0; q < PX / 2; ++q) {
                const float mine = hf ? outp[c][q + PX / 2] : outp[c][q];
                const float send = hf ? outp[c][q] : outp[c][q + PX / 2];
                tot[q] = mine + __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute(
                                    swap_addr, __builtin_bit_cast(int, send)));
            }
            if (valid) {
                if (a.io_f16) {
                    __half* op = (__half*)a.out + o0 + c * plane_px;
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
                    float* op = (float*)a.out + o0 + c * plane_px;
                    if constexpr (PX == 8) *(float4*)op = make_float4(tot[0], tot[1], tot[2], tot[3]);
                    else if constexpr (PX == 4) *(float2*)op = make_float2(tot[0], tot[1]);
                    else op[0] = tot[0];
                }
            }
        }
    }
}

// ---------------------------------------------------------------------------
// Host side: which instantiation serves a call.
// ---------------------------------------------------------------------------
namespace {

template <int K, int C, int NP8, int PX, int WR, int NW, int WPE = 2>
hipError_t launch_one(const AssembleArgs& a, hipStream_t st) {
    using F = Cfg<K, C, NP8, PX, WR, NW>;
    const int tiles_x = (a.W + F::TW - 1) / F::TW, tiles_y = (a.H + F::TH - 1) / F::TH;
    const long long nt = (long long)tiles_x * tiles_y * a.N;
    if (nt > 0x7fffffffLL) return hipErrorInvalidValue;
    // persistent grid: as many workgroups as stay resident (WPE wavefronts per SIMD)
    int dev = 0, cus = 256;
    if (hipGetDevice(&dev) == hipSuccess)
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    const int cap = cus * (4 * WPE / NW > 0 ? 4 * WPE / NW : 1);
    const int blocks = nt < cap ? (int)nt : cap;
    hipLaunchKernelGGL((k_assemble_mfma<K, C, NP8, PX, WR, NW, WPE>), dim3(blocks), dim3(F::NT), 0, st,
                       a, tiles_x, tiles_y, (int)nt);
    return hipGetLastError();
}

// atoms-per-launch capacity (in groups of 8) of the built instantiations, 0 = none
int np8_for(int k, int n_fold) {
    const int need = (n_fold + 7) / 8;
    if (k == 5) return need <= 9 ? 9 : 0;
    return 0;
}

constexpr int N_TILE_SHAPES = 4;

}  // namespace

bool mfma_supported(const AssembleArgs& a, int k, bool coeff_f16, int tile) {
    if (!coeff_f16 || (k != 5 && k != 7) || (a.C != 1 && a.C != 3)) return false;
    if (a.W % 8 != 0 || a.W < 8 || a.H < 1) return false;
    if (((uintptr_t)a.coeff % 16) != 0 || ((uintptr_t)a.out % 16) != 0) return false;
    if ((unsigned long long)a.L * a.H * a.W * 2ull >= (1ull << 32)) return false;   // 32-bit plane offsets
    if (np8_for(k, a.n_fold) == 0) return false;
    if (tile < 0 || tile >= N_TILE_SHAPES) return false;
    return true;
}

hipError_t launch_mfma(const AssembleArgs& a, int k, bool io_f16, int tile, hipStream_t st) {
    (void)io_f16;
    const int np8 = np8_for(k, a.n_fold);
    if (k == 5 && np8 == 9) {
        if (a.C == 3) {
            switch (tile) {
            case 1:  return launch_one<5, 3, 9, 4, 1, 4>(a, st);    // 128 x 4
            case 2:  return launch_one<5, 3, 9, 4, 2, 8>(a, st);    //  64 x 16, 8 wavefronts
            case 3:  return launch_one<5, 3, 9, 4, 1, 8>(a, st);    // 128 x 8,  8 wavefronts
            default: return launch_one<5, 3, 9, 4, 2, 4>(a, st);    //  64 x 8
            }
        }
        return launch_one<5, 1, 9, 4, 2, 4>(a, st);
    }
    return hipErrorInvalidValue;
}

}  // namespace srd
