// The wave-split members of the convolution kernel family for gfx950: for launches whose
// arithmetic is a few microseconds at most (single images, late layers of few pixels).
//
// Same GEMM view, same packed weights and same output code as the tiled members (wpk_igemm.h);
// the filter taps are followed by arithmetic instead of being read from the tap table.  What
// differs is who shares what.  A tiled workgroup stages its operands through
// LDS so that every wave reuses them, and it needs a long reduction per workgroup to repay the
// staging, the barriers and -- when the reduction has to be cut between workgroups to fill the
// device -- the meeting of the partial tiles in memory, several dependent memory round trips at
// the end of a launch that has little else to do.  Here a workgroup owns one tile of 32 pixels by
// BN channels and its WK waves cut the REDUCTION between them: every wave multiplies the whole tile
// over its own run of reduction rows, fetching both operands from global memory straight into
// the registers the MFMAs read (nothing in them is shared with another wave, so LDS would only add
// a store, a barrier and a load), and the waves' partial tiles meet in LDS: one barrier.  Where
// the tiled members need a reduction cut five ways across workgroups, these need none, or a
// shorter one.
//
// Operands.  Reduction rows are ordered (r, s, c) (the tap-major forms of the family: C a multiple
// of 32, see Problem::tapmajor and Problem::xquad), and the unit of work is an octet of eight
// rows: eight consecutive channels of one filter tap.  In the
// octet's four MFMAs (v_mfma_f32_32x32x2_f32) the low half-wave supplies rows 0..3 and the high
// half-wave rows 4..7, as in the tiled members.  So per octet a lane loads
//   weights: one 16-byte quad per 32-channel block -- packed [row/4][channel][4] is exactly that;
//   x [N][C][H][W]: four dwords, a channel stride apart (the stride rides in the scalar offset);
//   x [N][H][W][C]: one 16-byte quad (four consecutive channels of its pixel and tap).
// Out-of-image taps and pixels past the last one get a lane offset of all ones, which the buffer
// range check turns into a zero, as everywhere in the family.  PD octets are in flight per wave.
#ifndef WPK_WSPLIT_H
#define WPK_WSPLIT_H

#include "wpk_igemm.h"

namespace wpk {

// QUAD: x is channels-last and moves as channel quads (a.xl == 2); else [N][C][H][W] (a.xl == 3).
template <int BN, int WK, int PD, bool QUAD>
__global__ void __launch_bounds__(64 * WK) wsplit_kernel(const IgemmArgs a)
{
    constexpr int NNT = BN / 32;
    static_assert(BN % 32 == 0 && NNT >= 1 && NNT <= 2, "one or two 32-channel blocks per wave");
    static_assert(WK >= 1 && WK <= 8 && (WK & (WK - 1)) == 0, "1, 2, 4 or 8 waves");
    static_assert(PD >= 2 && PD <= 12, "octets in flight");
    // partial tiles of waves 1..WK-1: accumulator quad (block i, quad qd) of lane l at float
    // (((wk-1)*NNT + i)*4 + qd)*256 + 4*l -- 16-byte accesses, consecutive lanes, no conflicts
    __shared__ __attribute__((aligned(16))) float red[(WK > 1 ? WK - 1 : 1) * NNT * 16 * 64];

    touch_kernarg_lines();
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wk = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lrow = lane >> 5, lcol = lane & 31;

    // ---- which tile, which slice of the reduction -------------------------------------------------
    // (the arguments are used straight from the by-value kernel argument: this kernel has scalar
    // registers to spare, and every argument read at its place of use would be one more wait on the
    // scalar cache in a set-up that is a sixth of a short launch)
    const IgemmArgs *const c = &a;
    const int g = blockIdx.x;
    const int gr = a.remap ? xcd_remap(g, (int)gridDim.x) : g;
    const int slice = fdiv(gr, WPK_COLD_DIV(c, div_tiles));
    const int tile = gr - slice * c->tiles;
    int tile_m, tile_n;
    if (c->mfast) {
        tile_n = fdiv(tile, WPK_COLD_DIV(c, div_tiles_m));
        tile_m = tile - tile_n * c->tiles_m;
    } else {
        tile_m = fdiv(tile, WPK_COLD_DIV(c, div_tiles_n));
        tile_n = tile - tile_m * c->tiles_n;
    }
    const int m0 = tile_m * 32, n0 = tile_n * BN;
    // the slice's octets [s0, s1), cut evenly between the waves: this wave's are [obeg, oend)
    // (a wave with none contributes a tile of zeros)
    const int s0 = slice * c->steps_per_split, s1 = min(a.nsteps, s0 + c->steps_per_split);
    const int obeg = s0 + (s1 - s0) * wk / WK, oend = s0 + (s1 - s0) * (wk + 1) / WK;
    const int nr = oend - obeg;

    const __amdgpu_buffer_rsrc_t xrsrc = __builtin_amdgcn_make_buffer_rsrc(
        (void *)((const char *)a.x - a.x_bias), 0, (int)(a.x_bytes + a.x_bias), 0x00020000);
    const __amdgpu_buffer_rsrc_t wrsrc =
        __builtin_amdgcn_make_buffer_rsrc((void *)a.wp, 0, (int)a.w_bytes, 0x00020000);

    // ---- the loader's place in the reduction: the next octet to fetch, its first channel, and its
    //      filter tap (r, s) with the tap's byte offset in x.  Kept by arithmetic on the scalar unit
    //      (a step along the filter row, or to the start of the next one), not read from the tap table:
    //      a table entry costs a memory round trip before the first fetch can go out, which a launch
    //      of a few microseconds notices. ---------------------------------------------------------------
    const int px4 = QUAD ? a.C * 4 : 4;  // bytes between neighbouring pixels of x
    const int tap_step_s = c->dil_w * px4;
    const int tap_step_r = (c->dil_h * a.W - (a.S - 1) * c->dil_w) * px4;
    int ld_o = obeg;
    const int tap0 = fdiv(obeg * 8, WPK_COLD_DIV(c, div_tap));  // by C
    int ld_c0 = obeg * 8 - tap0 * a.C;
    int tap_r = fdiv(tap0, WPK_COLD_DIV(c, div_s));
    int tap_s = tap0 - tap_r * a.S;
    int tap_off = (tap_r * c->dil_h * a.W + tap_s * c->dil_w) * px4;
    // weights: the lane's quad of the octet's first block row, its channel
    const int wvoff = (lrow * a.Kpad + n0 + lcol) * 16;
    const int woct_bytes = 2 * a.Kpad * 16;  // one octet further
    // activations: the pixel's window, the half-wave's four channels
    int xvoff;
    unsigned xinv;
    pixel_window(c, m0 + lcol, xvoff, xinv);
    xvoff += lrow * 4 * (QUAD ? 4 : a.HW4);

    float xr[PD * 4];
    v4f wr[PD * NNT];
    // Loads of the loader's octet into register set SET; then the loader moves one octet on.
    // Every call issues the same instructions whether the octet is inside the run or past its end,
    // so that the count of loads in flight behind any register is the same on every path and the
    // waits the compiler places stay exact; an octet past the end gets lane offsets of all ones
    // (nothing is fetched, nobody reads the registers).
    auto issue = [&](auto SET) WPK_LAMBDA {
        constexpr int set = decltype(SET)::value;
        const int dead = ld_o < oend ? 0 : -1;
        const int xvb = xvoff | __builtin_amdgcn_sbfe((int)xinv, tap_r, 1) |
                        __builtin_amdgcn_sbfe((int)xinv, 16 + tap_s, 1) | dead;  // offset, or all ones
        if constexpr (QUAD) {
            v4f v = __builtin_bit_cast(
                v4f, __builtin_amdgcn_raw_buffer_load_b128(xrsrc, xvb, tap_off + ld_c0 * 4, 0));
            xr[set * 4] = v[0];
            xr[set * 4 + 1] = v[1];
            xr[set * 4 + 2] = v[2];
            xr[set * 4 + 3] = v[3];
        } else {
            static_for<4>([&](auto Q) WPK_LAMBDA {
                constexpr int q = decltype(Q)::value;
                xr[set * 4 + q] = __builtin_bit_cast(
                    float, __builtin_amdgcn_raw_buffer_load_b32(xrsrc, xvb, tap_off + (ld_c0 + q) * a.HW4, 0));
            });
        }
        const int wv = wvoff | dead;
        static_for<NNT>([&](auto I) WPK_LAMBDA {
            constexpr int i = decltype(I)::value;
            wr[set * NNT + i] = __builtin_bit_cast(
                v4f, __builtin_amdgcn_raw_buffer_load_b128(wrsrc, wv, ld_o * woct_bytes + i * 32 * 16, 0));
        });
        // (no branch at the change of tap: selects on the scalar unit; past the last tap the place keeps
        // moving, but nothing more is fetched)
        ld_o += 1;
        const bool next_tap = ld_c0 + 8 >= a.C;
        const bool next_row = next_tap && tap_s + 1 == a.S;
        ld_c0 = next_tap ? 0 : ld_c0 + 8;
        tap_off += next_row ? tap_step_r : next_tap ? tap_step_s : 0;
        tap_s = next_row ? 0 : next_tap ? tap_s + 1 : tap_s;
        tap_r += next_row ? 1 : 0;
    };

    v16f acc[NNT];
    static_for<NNT>([&](auto I) WPK_LAMBDA {
        static_for<16>([&](auto E) WPK_LAMBDA { acc[decltype(I)::value][decltype(E)::value] = 0.0f; });
    });
    auto multiply = [&](auto SET) WPK_LAMBDA {
        constexpr int set = decltype(SET)::value;
        static_for<4>([&](auto Q) WPK_LAMBDA {
            constexpr int q = decltype(Q)::value;
            static_for<NNT>([&](auto I) WPK_LAMBDA {
                constexpr int i = decltype(I)::value;
                acc[i] = __builtin_amdgcn_mfma_f32_32x32x2f32(wr[set * NNT + i][q], xr[set * 4 + q], acc[i], 0, 0, 0);
            });
        });
    };
    // Octet number r of the wave's run travels in register set r % PD.  The loop is left at the
    // first octet past the end of the run: no join inside it, so the accumulators stay where they
    // are and the fetched registers are not live after it.  Its body is kGroups groups of PD octets:
    // the compiler waits for every load in flight at the top of a loop body (not only for the set
    // the first step needs), which empties the pipeline once per pass through the body.
    constexpr int kGroups = 4;
    static_for<PD>([&](auto P) WPK_LAMBDA {
        issue(P);
        __builtin_amdgcn_sched_barrier(0);
    });
    int r = 0;
    auto step = [&](auto P) WPK_LAMBDA {
        constexpr int p = decltype(P)::value;
        if (r + p >= nr) return false;
        multiply(std::integral_constant<int, p % PD>{});
        issue(std::integral_constant<int, p % PD>{});
        __builtin_amdgcn_sched_barrier(0);
        return true;
    };
    while (static_all<kGroups * PD>(step)) r += kGroups * PD;

    // ---- the waves' partial tiles meet in wave 0 --------------------------------------------------
    if constexpr (WK > 1) {
        if (wk > 0) {
            static_for<NNT * 4>([&](auto Q) WPK_LAMBDA {
                constexpr int qd = decltype(Q)::value, i = qd / 4, e4 = qd % 4;
                v4f v = {acc[i][4 * e4], acc[i][4 * e4 + 1], acc[i][4 * e4 + 2], acc[i][4 * e4 + 3]};
                *reinterpret_cast<v4f *>(red + (((wk - 1) * NNT + i) * 4 + e4) * 256 + 4 * lane) = v;
            });
        }
        __syncthreads();
        if (wk > 0) return;
        static_for<WK - 1>([&](auto U) WPK_LAMBDA {
            static_for<NNT * 4>([&](auto Q) WPK_LAMBDA {
                constexpr int u = decltype(U)::value, qd = decltype(Q)::value, i = qd / 4, e4 = qd % 4;
                const v4f v = *reinterpret_cast<const v4f *>(red + ((u * NNT + i) * 4 + e4) * 256 + 4 * lane);
                acc[i][4 * e4] += v[0];
                acc[i][4 * e4 + 1] += v[1];
                acc[i][4 * e4 + 2] += v[2];
                acc[i][4 * e4 + 3] += v[3];
            });
        });
    }

    // ---- a reduction cut between workgroups: the slices of a tile meet through the workspace (each
    //      stores its partial tile to its slot and counts itself in; whoever comes last adds up the
    //      others and stores y), or, without one, through atomics into y, which the host zeroed ------
    const IgemmArgs *const ce = &a;
    bool atomic = false;
    if (ce->split_k > 1) {
        if (!ce->ws) {
            atomic = true;
        } else {
            constexpr int kCoherent = 17;  // sc0 | sc1: past the L2s, which do not snoop each other
            constexpr int SLOT = 32 * BN;  // floats; quad (i, e4) of lane l at (i*4 + e4)*256 + 4*l
            const __amdgpu_buffer_rsrc_t srsrc = __builtin_amdgcn_make_buffer_rsrc(
                (void *)(ce->ws + (size_t)tile * ce->ws_maxc * SLOT), 0, ce->ws_maxc * SLOT * 4, 0x00020000);
            static_for<NNT * 4>([&](auto Q) WPK_LAMBDA {
                constexpr int qd = decltype(Q)::value, i = qd / 4, e4 = qd % 4;
                v4f v = {acc[i][4 * e4], acc[i][4 * e4 + 1], acc[i][4 * e4 + 2], acc[i][4 * e4 + 3]};
                __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(v4u, v), srsrc,
                                                       (slice * SLOT + 4 * lane) * 4, qd * 1024, kCoherent);
            });
            // every store acknowledged before the arrival is counted
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
            __builtin_amdgcn_s_waitcnt(0);
            int before = 0;
            if (lane == 0) before = atomicAdd(ce->ws_cnt + tile, 1);
            before = __builtin_amdgcn_readfirstlane(before);
            if (before != ce->split_k - 1) return;      // not the last: done with this tile
            if (lane == 0) ce->ws_cnt[tile] = 0;          // leave the counter clean for the next launch
            // four slots at a time, all requested before the first is added (a slot number past the
            // last becomes an out-of-range offset, which loads 0)
            constexpr int kGang = 4;
            for (int t0 = 0; t0 < ce->split_k - 1; t0 += kGang) {
                v4f part[kGang][NNT * 4];
                static_for<kGang>([&](auto U) WPK_LAMBDA {
                    constexpr int u = decltype(U)::value;
                    const int t = t0 + u, sl = t + (t >= slice ? 1 : 0);  // t-th slot not mine
                    const unsigned off = t < ce->split_k - 1 ? (unsigned)((sl * SLOT + 4 * lane) * 4) : 0xffffffffu;
                    static_for<NNT * 4>([&](auto Q) WPK_LAMBDA {
                        constexpr int qd = decltype(Q)::value;
                        part[u][qd] = __builtin_bit_cast(
                            v4f, __builtin_amdgcn_raw_buffer_load_b128(srsrc, off, qd * 1024, kCoherent));
                    });
                });
                static_for<kGang * NNT * 4>([&](auto UQ) WPK_LAMBDA {
                    constexpr int u = decltype(UQ)::value / (NNT * 4), qd = decltype(UQ)::value % (NNT * 4);
                    constexpr int i = qd / 4, e4 = qd % 4;
                    acc[i][4 * e4] += part[u][qd][0];
                    acc[i][4 * e4 + 1] += part[u][qd][1];
                    acc[i][4 * e4 + 2] += part[u][qd][2];
                    acc[i][4 * e4 + 3] += part[u][qd][3];
                });
            }
        }
    }
    store_wave_tile<NNT, 1>(ce, acc, m0, n0, lrow, lcol, atomic);
}

template <int BN, int WK, int PD>
hipError_t launch_wsplit(const IgemmArgs &a, hipStream_t stream)
{
    dim3 grid((unsigned)(a.tiles_m * a.tiles_n * a.split_k));
    if (a.xl == 2)
        hipLaunchKernelGGL((wsplit_kernel<BN, WK, PD, true>), grid, dim3(64 * WK), 0, stream, a);
    else
        hipLaunchKernelGGL((wsplit_kernel<BN, WK, PD, false>), grid, dim3(64 * WK), 0, stream, a);
    return hipGetLastError();
}

}  // namespace wpk
#endif
