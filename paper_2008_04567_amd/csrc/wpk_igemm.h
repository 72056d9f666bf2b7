// The tiled implicit-GEMM forward convolution kernel family for gfx950 (CDNA4, wave64).
//
// GEMM view that matches NCHW memory: Y[kout][pixel] = sum_kk W[kout][kk] * Xcol[kk][pixel],
// pixel = (n,p,q) flattened, kk = (c,r,s) flattened in the weights' own KCRS order.  x and y are
// both contiguous along q, so activation loads and output stores coalesce along the pixel axis.
// The im2col matrix is never written to memory: per reduction step a workgroup gathers a
// BK x BM activation tile and a BK x BN weight tile into LDS.
//
// Gather.  A per-problem tap table gives, for every reduction row, the byte offset of its tap
// inside one image and the filter row r / column s it belongs to.  Each lane owns one output
// pixel: a constant byte offset of the pixel's window origin and a bit mask of the filter rows
// and columns that fall outside the image for that pixel.  A load is then one buffer load with
// the lane offset in the VGPR and the tap offset in the SGPR; out-of-image taps get an offset
// of all ones, which the buffer range check turns into a zero.
//
// LDS layout.  Both tiles are stored reduction-contiguous: tile[column][k] with a row pitch of
// BK+4 floats, so that a lane moves four consecutive k values of its column with one 16-byte LDS
// access and the 16 lanes served per clock hit 16 distinct groups of four banks.  The weights
// are pre-packed as [kk/4][kout][4] so that a 16-byte global load is exactly one such quad.
//
// Contraction.  v_mfma_f32_32x32x2_f32 multiplies A = 32 channels x 2 k by B = 2 k x 32 pixels.
// Lanes 0-31 supply k index 0 and lanes 32-63 k index 1 of both operands, and any pairing of k
// values is a valid contraction as long as A and B agree.  For eight consecutive k values the
// low half-wave holds k0..k0+3 and the high half-wave k0+4..k0+7 of its column (one 16-byte LDS
// read each); MFMA number q of four contracts the pair (k0+q, k0+4+q).  D = 32 x 32 has the pixel
// index on the lane axis, so each accumulator register of a half-wave stores 32 consecutive
// pixels (128 contiguous bytes of y).
#ifndef WPK_IGEMM_H
#define WPK_IGEMM_H

#include <hip/hip_runtime.h>

#include <type_traits>
#include <utility>

#include "wpk_internal.h"

namespace wpk {

typedef float v16f __attribute__((ext_vector_type(16)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef unsigned int v4u __attribute__((ext_vector_type(4)));

// Lambdas in the kernel must be inlined before the register arrays they capture are split up.
#define WPK_LAMBDA __attribute__((always_inline))

// Contiguous tile ranges per XCD: workgroup ids are dealt round-robin to the 8 XCDs, so id b runs
// on XCD b%8; this maps it to a tile index such that each XCD owns one contiguous range.
__device__ __forceinline__ int xcd_remap(int bid, int nblocks)
{
    int per = nblocks / kNumXcd, rem = nblocks % kNumXcd;
    int xcd = bid % kNumXcd, idx = bid / kNumXcd;
    return xcd * per + (xcd < rem ? xcd : rem) + idx;
}

// Compile-time loop: every array index in the kernel is a constant at the source level, so the
// register arrays below are split into scalars by the first optimisation passes and never end up
// in scratch or LDS.
template <class F, int... I>
__device__ __forceinline__ void static_for_impl(F &&f, std::integer_sequence<int, I...>)
{
    (f(std::integral_constant<int, I>{}), ...);
}
template <int N, class F>
__device__ __forceinline__ void static_for(F &&f)
{
    static_for_impl(f, std::make_integer_sequence<int, N>{});
}

// f(0) && f(1) && ... && f(N-1), left to right, stopping at the first false.
template <class F, int... I>
__device__ __forceinline__ bool static_all_impl(F &&f, std::integer_sequence<int, I...>)
{
    return (f(std::integral_constant<int, I>{}) && ...);
}
template <int N, class F>
__device__ __forceinline__ bool static_all(F &&f)
{
    return static_all_impl(f, std::make_integer_sequence<int, N>{});
}

__device__ __forceinline__ int fdiv(int n, const FastDiv &f)
{
    return (int)((__umulhi((unsigned)n, f.mul) + (unsigned)n) >> f.sh);
}

// Cache policy of the stores of y in [N][K][P][Q] layout (whole 128-byte runs per half-wave):
// sc0 | sc1, written through the per-XCD L2 as they are issued.
// With the default policy the outputs sit dirty in the L2s until the kernel ends and are written
// back then, before the next dispatch may start; nobody in this launch reads them again.  Measured:
// 0.8 us per launch on a layer that writes 12.8 MB, nothing on small outputs.
constexpr int kYStorePolicy = 17;

// Arguments that only a segment's set-up, its epilogue or the work iterator use are read from the
// kernel-argument segment at the place of use (scalar loads that hit the scalar cache) instead of
// being held in scalar registers from the kernel's entry on: together with everything the compiler
// derives from them ahead of the segment loop they overflowed the scalar register file, and every
// spilled value is a vector ALU instruction at the spill and at each reload, which the matrix pipe
// pays for.  The empty asm statement hides the pointer's origin, so the loads stay where they are.
typedef const IgemmArgs __attribute__((address_space(4))) *cold_ptr;
#define WPK_COLD_DIV(c, f) (FastDiv{(c)->f.mul, (c)->f.sh})
__device__ __forceinline__ cold_ptr cold_args()
{
    unsigned long long p = (unsigned long long)__builtin_amdgcn_kernarg_segment_ptr();
    asm volatile("" : "+s"(p));
    return (cold_ptr)p;
}

// The arguments span several 64-byte lines that no cache holds when a launch begins, and a kernel's
// set-up reads them in dependent batches (work iterator, then descriptors, then divisors): one
// memory round trip per batch.  Touching every line first puts all of them in flight at once; the
// loads after it hit the scalar cache.
__device__ __forceinline__ void touch_kernarg_lines()
{
    static_assert(sizeof(IgemmArgs) + 32 <= 6 * 64, "one more line to touch");
    const unsigned long long kp = (unsigned long long)__builtin_amdgcn_kernarg_segment_ptr();
    int l0, l1, l2, l3, l4, l5;  // (the sixth line also holds the launch dimensions the compiler appends)
    asm volatile("s_load_dword %0, %6, 0x0\n\ts_load_dword %1, %6, 0x40\n\ts_load_dword %2, %6, 0x80\n\t"
                 "s_load_dword %3, %6, 0xc0\n\ts_load_dword %4, %6, 0x100\n\ts_load_dword %5, %6, 0x140\n\t"
                 "s_waitcnt lgkmcnt(0)"
                 : "=&s"(l0), "=&s"(l1), "=&s"(l2), "=&s"(l3), "=&s"(l4), "=&s"(l5)
                 : "s"(kp)
                 : "memory");
}

// The tap table is read through the constant address space: wave-uniform scalar loads.
typedef const int __attribute__((address_space(4))) *tap_ptr;

// LDS row pitch (floats) of a reduction-contiguous tile with BK k values per column.
__host__ __device__ constexpr int lds_pitch(int bk) { return bk + 4; }

// Gather state of output pixel m: voff = byte offset of its window origin in x (before padding is
// subtracted; the padding shift is folded into the tap offsets and the buffer base, so it is never
// negative); inv: bit r set = filter row r is outside the image for this pixel, bit 16+s = column s;
// bit 31 is always set and is what the table's padding rows point at.  A pixel past the last one
// has every bit set.
// (ARGS: a pointer to the arguments -- cold_ptr where they are to be read at the place of use, a plain
// pointer to the by-value kernel argument where the compiler may keep them in scalar registers)
template <class ARGS>
__device__ __forceinline__ void pixel_window(const ARGS c, const int m, int &voff, unsigned &inv_out)
{
    voff = 0;
    inv_out = 0xffffffffu;
    if (m < c->M) {
        int n = fdiv(m, WPK_COLD_DIV(c, div_pq)), pq = m - n * c->PQ;
        int p = fdiv(pq, WPK_COLD_DIV(c, div_q)), q = pq - p * c->Q;
        int ih0 = p * c->stride_h - c->pad_h, iw0 = q * c->stride_w - c->pad_w;
        // channels-last x: c->xl 1 or 2; [N][C][H][W]: 0 or 3
        voff = (c->xl == 1 || c->xl == 2) ? ((n * c->H + p * c->stride_h) * c->W + q * c->stride_w) * c->C * 4
                                          : ((n * c->C * c->H + p * c->stride_h) * c->W + q * c->stride_w) * 4;
        unsigned inv = 0x80000000u;
        // rows below the image are r < -ih0, rows past it r >= H - ih0 when the dilation is 1:
        // two clamped shifts instead of a loop over the filter
        auto outside = [](int o0, int len, int taps) WPK_LAMBDA {
            const int lo = min(max(-o0, 0), taps), hi = min(max(len - o0, 0), taps);
            return ((1u << lo) - 1u) | (((1u << taps) - 1u) & ~((1u << hi) - 1u));
        };
        if (c->dil_h == 1) {
            inv |= outside(ih0, c->H, c->R);
        } else {
            for (int r = 0; r < c->R; ++r) {
                int ih = ih0 + r * c->dil_h;
                if (ih < 0 || ih >= c->H) inv |= 1u << r;
            }
        }
        if (c->dil_w == 1) {
            inv |= outside(iw0, c->W, c->S) << 16;
        } else {
            for (int sx = 0; sx < c->S; ++sx) {
                int iw = iw0 + sx * c->dil_w;
                if (iw < 0 || iw >= c->W) inv |= 1u << (16 + sx);
            }
        }
        inv_out = inv;
    }
}

// ---- what leaves a wave: its NNT x NMT accumulator blocks, whose first pixel is mbase and first
//      channel nbase, go to y -- plain stores with the fused epilogue applied, or fp32 atomics ----
template <int NNT, int NMT, class ARGS>
__device__ __forceinline__ void store_wave_tile(const ARGS ce, const v16f (&acc)[NNT * NMT], const int mbase,
                                                const int nbase, const int lrow, const int lcol, const bool atomic)
{
    // the host applies the epilogue itself after a launch that accumulates with atomics
    const bool fused = !atomic && (ce->bias || ce->res || ce->relu);

    // ---- epilogue: D[row = channel][col = pixel]; register e of lane l holds row
    //      8*(e/4) + 4*(l/32) + e%4 and column l%32 of its 32x32 block.  Buffer addressing: one
    //      32-bit lane offset per block plus a wave-uniform offset per register, instead of a
    //      64-bit address per output.  A NULL bias or residual becomes a buffer of zero records,
    //      whose loads return 0. ------------------------------------------------------------------
    const __amdgpu_buffer_rsrc_t yrsrc =
        __builtin_amdgcn_make_buffer_rsrc((void *)ce->y, 0, (int)ce->y_bytes, 0x00020000);
    // y[n][k][p][q]: consecutive channels are PQ elements apart; channels-last y[n][p][q][k]: 1
    const int PQ4 = ce->yl ? 4 : ce->PQ * 4;
    static_for<NMT>([&](auto J) WPK_LAMBDA {
        constexpr int j = decltype(J)::value;
        int m = mbase + j * 32 + lcol;
        if (m < ce->M) {
            int n = fdiv(m, WPK_COLD_DIV(ce, div_pq)), pq = m - n * ce->PQ;
            static_for<NNT>([&](auto I) WPK_LAMBDA {
                constexpr int i = decltype(I)::value;
                const int kbase = nbase + i * 32 + 4 * lrow;  // + 8*(e/4) + e%4
                // byte offset of (n, kbase, pq) in y; only used for channels below K, where it
                // is below y_bytes < 2^32
                const unsigned voff = ce->yl ? (unsigned)(((size_t)m * ce->K + kbase) * 4)
                                           : (unsigned)((((size_t)n * ce->K + kbase) * ce->PQ + pq) * 4);
                // A 32-channel block that lies wholly below K (the usual case) stores without a
                // bound check per register; the check costs an exec-mask round trip each.
                auto emit = [&](auto FULL, auto THROUGH) WPK_LAMBDA {
                    constexpr bool full = decltype(FULL)::value;
                    // channels-last outputs leave a lane in 16-byte pieces that only the L2 merges
                    // into whole lines: they keep the default write-back policy
                    constexpr int policy = decltype(THROUGH)::value ? kYStorePolicy : 0;
                    if (ce->yl == 2 && !atomic) {
                        // channels-last y with K a multiple of 4 and 16-byte aligned tensors: the four
                        // registers 4g..4g+3 of a lane are four consecutive channels of its pixel
                        const __amdgpu_buffer_rsrc_t brsrc = __builtin_amdgcn_make_buffer_rsrc(
                            (void *)(ce->bias ? ce->bias : ce->y), 0, ce->bias ? ce->K * 4 : 0, 0x00020000);
                        const __amdgpu_buffer_rsrc_t rrsrc = __builtin_amdgcn_make_buffer_rsrc(
                            (void *)(ce->res ? ce->res : ce->y), 0, ce->res ? (int)ce->y_bytes : 0, 0x00020000);
                        v4f add[4];
                        if (fused)
                            static_for<4>([&](auto G) WPK_LAMBDA {
                                constexpr int g = decltype(G)::value;
                                v4f t = __builtin_bit_cast(
                                    v4f, __builtin_amdgcn_raw_buffer_load_b128(brsrc, kbase * 4, 32 * g, 0));
                                if (full || kbase + 8 * g < ce->K)
                                    t += __builtin_bit_cast(
                                        v4f, __builtin_amdgcn_raw_buffer_load_b128(rrsrc, voff, 32 * g, 0));
                                add[g] = t;
                            });
                        static_for<4>([&](auto G) WPK_LAMBDA {
                            constexpr int g = decltype(G)::value;
                            if (full || kbase + 8 * g < ce->K) {
                                v4f v = {acc[i * NMT + j][4 * g], acc[i * NMT + j][4 * g + 1],
                                         acc[i * NMT + j][4 * g + 2], acc[i * NMT + j][4 * g + 3]};
                                if (fused) {
                                    v += add[g];
                                    if (ce->relu)
                                        v = (v4f){fmaxf(v[0], 0.0f), fmaxf(v[1], 0.0f), fmaxf(v[2], 0.0f),
                                                  fmaxf(v[3], 0.0f)};
                                }
                                __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(v4u, v), yrsrc, voff,
                                                                       32 * g, policy);
                            }
                        });
                    } else if (fused) {
                        const __amdgpu_buffer_rsrc_t brsrc = __builtin_amdgcn_make_buffer_rsrc(
                            (void *)(ce->bias ? ce->bias : ce->y), 0, ce->bias ? ce->K * 4 : 0, 0x00020000);
                        const __amdgpu_buffer_rsrc_t rrsrc = __builtin_amdgcn_make_buffer_rsrc(
                            (void *)(ce->res ? ce->res : ce->y), 0, ce->res ? (int)ce->y_bytes : 0, 0x00020000);
                        // everything the 16 outputs of this block add is fetched first, so the loads
                        // are all in flight together; then the stores
                        float add[16];
                        static_for<16>([&](auto E) WPK_LAMBDA {
                            constexpr int e = decltype(E)::value, de = 8 * (e / 4) + (e & 3);
                            float t = __builtin_bit_cast(
                                float, __builtin_amdgcn_raw_buffer_load_b32(brsrc, kbase * 4, de * 4, 0));
                            if (full || kbase + de < ce->K)
                                t += __builtin_bit_cast(
                                    float, __builtin_amdgcn_raw_buffer_load_b32(rrsrc, voff, de * PQ4, 0));
                            add[e] = t;
                        });
                        static_for<16>([&](auto E) WPK_LAMBDA {
                            constexpr int e = decltype(E)::value, de = 8 * (e / 4) + (e & 3);
                            if (full || kbase + de < ce->K) {
                                float v = acc[i * NMT + j][e] + add[e];
                                v = ce->relu ? fmaxf(v, 0.0f) : v;
                                __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned, v), yrsrc,
                                                                      voff, de * PQ4, policy);
                            }
                        });
                    } else if (atomic) {
                        // (no-return fp32 adds, addressed like the stores)
                        static_for<16>([&](auto E) WPK_LAMBDA {
                            constexpr int e = decltype(E)::value, de = 8 * (e / 4) + (e & 3);
                            if (full || kbase + de < ce->K) {
                                const float v = acc[i * NMT + j][e];
                                __builtin_amdgcn_raw_ptr_buffer_atomic_fadd_f32(v, yrsrc, voff, de * PQ4, 0);
                            }
                        });
                    } else {
                        static_for<16>([&](auto E) WPK_LAMBDA {
                            constexpr int e = decltype(E)::value, de = 8 * (e / 4) + (e & 3);
                            if (full || kbase + de < ce->K) {
                                // a copy first: a bit cast taken straight from a vector element
                                // reads element 0 with this compiler
                                const float v = acc[i * NMT + j][e];
                                __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned, v), yrsrc,
                                                                      voff, de * PQ4, policy);
                            }
                        });
                    }
                };
                const bool whole = nbase + i * 32 + 32 <= ce->K;
                if (ce->yl == 0) {
                    if (whole)
                        emit(std::true_type{}, std::true_type{});
                    else
                        emit(std::false_type{}, std::true_type{});
                } else {
                    if (whole)
                        emit(std::true_type{}, std::false_type{});
                    else
                        emit(std::false_type{}, std::false_type{});
                }
            });
        }
    });
}

// XL = 0: reduction rows ordered (c, r, s) and gathered one row at a time as described above, for
//   activations [N][C][H][W] or (a.xl = 1) channels-last ones: only the window origin and the
//   strides the host puts into the tap table differ.  This form takes any C.
// XL = 1 (a.xl = 2): activations channels-last, [N][H][W][C], reduction rows ordered (r, s, c)
//   and C a multiple of BK.  A lane still owns one output pixel; four consecutive reduction rows are four
//   consecutive channels of one tap, i.e. 16 contiguous bytes: one buffer_load_dwordx4 per quad.
//   A step lies inside a single tap (r, s), so one table entry per step gives the tap's byte
//   offset and mask bits, the channel offset is added on the scalar unit, and there are no
//   padding rows.  Everything downstream of the staging registers is shared.
// XL = 2 (a.xl = 3): activations [N][C][H][W] with C a multiple of every K-step, reduction rows
//   ordered (r, s, c) as well: a step is BK channels of ONE tap, so the lane's masked offset is
//   formed once per step instead of once per loaded element, and the channel stride H*W*4 goes
//   into the scalar offset of each one-dword load.  fp32 MFMAs issue through the same port as every
//   other vector ALU instruction (measured: each such instruction takes 4.4 cycles or more away from
//   the matrix rate, whichever wave it comes from), so the three address instructions per loaded
//   element of the XL = 0 form cost 10-15 % of the arithmetic time; this form has three per step.
//   A pointwise (1x1) layer is the single-tap case of it.
// The layout of y (and of a fused residual) is a run-time flag of the epilogue (a.yl).
template <int BM, int BN, int BK, int WM, int WN, int PD, int XL>
__global__ void __launch_bounds__(64 * WM * WN) igemm_kernel(const IgemmArgs a)
{
    constexpr int T = 64 * WM * WN;
    constexpr int TM = BM / WM, TN = BN / WN;    // wave tile
    constexpr int NMT = TM / 32, NNT = TN / 32;  // 32x32 MFMA blocks per wave tile
    constexpr int XP = BM > T ? BM / T : 1;      // pixels per thread in the gather
    constexpr int RG = T > BM ? T / BM : 1;      // row groups in the gather
    constexpr int XR = BK / RG;                  // consecutive reduction rows per thread and pixel
    constexpr int W4 = BK / 4 * BN;              // 16-byte quads in a weight tile
    constexpr int WL = (W4 + T - 1) / T;         // quads per thread
    constexpr int PX = lds_pitch(BK), PW = lds_pitch(BK);
    constexpr int XTILE = BM * PX, WTILE = BN * PW;
    static_assert(TM % 32 == 0 && TN % 32 == 0, "wave tile must be whole MFMA blocks");
    static_assert(BM % 64 == 0, "a wave gathers whole reduction rows");
    static_assert(BK % 8 == 0, "the MFMA pairing works on octets of k");
    static_assert(BK % RG == 0 && XR % 4 == 0, "a thread must own whole k quads");
    static_assert((T >= BM && T % BM == 0) || (T < BM && BM % T == 0), "gather mapping");
    static_assert(T % BN == 0, "weight quads: every thread keeps one channel");
    static_assert(PD >= 1 && PD <= 4, "one to four tiles in flight");

    __shared__ __attribute__((aligned(16))) float lds[2 * (XTILE + WTILE)];
    float *const Xs0 = lds, *const Ws0 = lds + 2 * XTILE;

    touch_kernarg_lines();
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wave_m = wave % WM, wave_n = wave / WM;
    const int lrow = lane >> 5, lcol = lane & 31;

    const __amdgpu_buffer_rsrc_t xrsrc = __builtin_amdgcn_make_buffer_rsrc(
        (void *)((const char *)a.x - a.x_bias), 0, (int)(a.x_bytes + a.x_bias), 0x00020000);
    const __amdgpu_buffer_rsrc_t wrsrc =
        __builtin_amdgcn_make_buffer_rsrc((void *)a.wp, 0, (int)a.w_bytes, 0x00020000);
    const tap_ptr taps = (tap_ptr)(unsigned long long)a.ktab;
    const int pm0 = tid % (T < BM ? T : BM);
    const int rg = __builtin_amdgcn_readfirstlane(tid / BM);  // 0 when T <= BM
    const int wkout = tid % BN, wkq = tid / BN;      // weight quads: this thread's channel, k quad
    const int wstep_bytes = (BK / 4) * a.Kpad * 16;  // one reduction step further
    const int wquad_bytes = (T / BN) * a.Kpad * 16;  // this thread's next quad in the same step

    // One segment of work: reduction steps [kbeg, kend) of output tile `tile`.  How the result
    // leaves the workgroup (mode):
    //   kStore  plain stores (the segment is the tile's whole reduction);
    //   kAtomic fp32 atomics into y, which the host zeroed (no workspace given);
    //   kFixup  the tile is shared by fix_n workgroups (reduction slices, or neighbouring runs
    //           of a persistent launch), this one being number fix_slot: each stores its partial
    //           tile to its slot of the workspace and bumps the tile's arrival counter; whoever
    //           arrives last adds up the other slots and stores y.  Nobody waits for anybody, y
    //           needs no zeroing, and the counter is back at zero when the kernel ends.
    enum { kStore = 0, kAtomic = 1, kFixup = 2 };
    __shared__ int arrival;
    auto run_segment = [&](const int tile, const int kbeg, const int kend, const int mode,
                           const int fix_j, const int fix_slot, const int fix_n) WPK_LAMBDA {
    if (kbeg >= kend) return;  // nothing to reduce: touch neither the tap table nor y
    int tile_m, tile_n;
    {
        const cold_ptr c = cold_args();
        if (c->mfast) {
            tile_n = fdiv(tile, WPK_COLD_DIV(c, div_tiles_m));
            tile_m = tile - tile_n * c->tiles_m;
        } else {
            tile_m = fdiv(tile, WPK_COLD_DIV(c, div_tiles_n));
            tile_n = tile - tile_m * c->tiles_n;
        }
    }
    const int m0 = tile_m * BM, n0 = tile_n * BN;

    // ---- per-thread gather state ---------------------------------------------------------------
    // xvoff: byte offset of the pixel's window origin (before padding is subtracted; the padding
    //        shift is folded into the tap offsets and the buffer base, so it is never negative);
    // xinv : bit r set = filter row r is outside the image for this pixel, bit 16+s = column s;
    //        bit 31 is always set and is what the table's padding rows point at.
    int xvoff[XP];
    unsigned xinv[XP];
    auto gather_state = [&]() WPK_LAMBDA {
    const cold_ptr c = cold_args();
    static_for<XP>([&](auto I) WPK_LAMBDA {
        constexpr int i = decltype(I)::value;
        pixel_window(c, m0 + pm0 + i * T, xvoff[i], xinv[i]);
    });
    };
    const int wvoff = (wkq * a.Kpad + n0 + wkout) * 16;

    // ---- staging registers: PD tiles (activations and weights) in flight between global memory
    //      and LDS.  Tile number r of the segment (r = step - kbeg) travels in set r % PD. ---------
    constexpr int NX = XP * XR;   // activation dwords per thread and tile
    constexpr int NXQ = NX / 4;   // ... stored to LDS as quads
    constexpr int NW = WL;        // weight quads per thread and tile
    constexpr bool TAPM = XL != 0;      // a step lies inside one filter tap (reduction order (r, s, c))
    constexpr bool QUAD = XL == 1;      // ... and a lane loads four channels at a time
    constexpr int NXL = QUAD ? NXQ : NX;  // activation load instructions per thread and tile
    float xr[PD * NX];
    v4f wr[PD * NW];
    int tap_off[XR], tap_rs[XR];  // wave-uniform: live in scalar registers

    // Tap lookup.  Reduction row kk = c*RS + rs.  A step starting at row k0 = c0*RS + phase sees
    // a pattern of (r, s, channel advance) that depends on phase alone, so a table of RS phases x
    // 32 rows -- a few KB, resident in the scalar cache -- serves every step; the step's channel
    // base c0*H*W*4 is added on the scalar unit.  (One table row per reduction row of the whole
    // problem would miss the scalar cache at every step and stall the wave on its first LDS wait.)
    // The last step of the reduction is the only one with padding rows past C*R*S; it reads a
    // separate 32-row table with exact entries.  Steps are visited in increasing order inside a
    // segment, so (c0, phase) advance incrementally.
    // Channels-last: tap_c0 is the tap index rs of the step and tap_phase its first channel; the
    // table has one entry per tap, {byte offset of the tap, mask bits}, and tap_cbase carries
    // the channel offset.
    int tap_cbase = 0;  // channel base of the tile whose taps are loaded, added at the use
    int tap_c0 = fdiv(kbeg * BK, WPK_COLD_DIV(cold_args(), div_tap));  // by C (tap-major forms) or R*S
    int tap_phase = TAPM ? kbeg * BK - tap_c0 * a.C : kbeg * BK - tap_c0 * a.RS;
    int xvb[XP];        // tap-major forms: the lane offset with the step's mask folded in
    auto fold_mask = [&]() WPK_LAMBDA {
        static_for<XP>([&](auto I) WPK_LAMBDA {
            constexpr int i = decltype(I)::value;
            xvb[i] = xvoff[i] | __builtin_amdgcn_sbfe((int)xinv[i], tap_rs[0] & 0xff, 1) |
                     __builtin_amdgcn_sbfe((int)xinv[i], tap_rs[0] >> 8, 1);  // offset, or all ones
        });
    };
    auto load_taps = [&](int step, bool fold = true) WPK_LAMBDA {
        if constexpr (TAPM) {
            tap_off[0] = taps[2 * tap_c0];
            tap_rs[0] = taps[2 * tap_c0 + 1];
            tap_cbase = (tap_phase + rg * XR) * (QUAD ? 4 : a.HW4);
            tap_phase += BK;
            if (tap_phase >= a.C) {
                tap_phase = 0;
                tap_c0 += 1;
            }
            if (fold) fold_mask();
            return;
        }
        const bool last = step == a.nsteps - 1;
        tap_ptr tp = last ? (tap_ptr)(unsigned long long)a.ttab + 2 * (rg * XR)
                          : taps + 2 * (tap_phase * 32 + rg * XR);
        tap_cbase = last ? 0 : tap_c0 * a.HW4;
        static_for<XR>([&](auto J) WPK_LAMBDA {
            constexpr int jj = decltype(J)::value;
            tap_off[jj] = tp[2 * jj];
            tap_rs[jj] = tp[2 * jj + 1];
        });
        tap_c0 += a.bk_div_rs;
        tap_phase += a.bk_mod_rs;
        if (tap_phase >= a.RS) {
            tap_phase -= a.RS;
            tap_c0 += 1;
        }
    };
    // global -> register set SET: activation dword E of the tile whose taps are loaded
    auto load_x = [&](auto SET, auto E) WPK_LAMBDA {
        if constexpr (QUAD) {  // E counts quads: pixel i, quad j4 of this thread's XR rows
            constexpr int set = decltype(SET)::value, e = decltype(E)::value;
            constexpr int i = e / (XR / 4), j4 = e % (XR / 4), b = set * NX + i * XR + 4 * j4;
            v4f v = __builtin_bit_cast(
                v4f, __builtin_amdgcn_raw_buffer_load_b128(xrsrc, xvb[i], tap_off[0] + tap_cbase + 16 * j4, 0));
            xr[b] = v[0];
            xr[b + 1] = v[1];
            xr[b + 2] = v[2];
            xr[b + 3] = v[3];
            return;
        }
        if constexpr (TAPM) {  // channel jj of this thread's XR, pixel i: the stride goes into the scalar offset
            constexpr int set = decltype(SET)::value, e = decltype(E)::value, i = e / XR, jj = e % XR;
            xr[set * NX + e] = __builtin_bit_cast(
                float, __builtin_amdgcn_raw_buffer_load_b32(xrsrc, xvb[i], tap_off[0] + tap_cbase + jj * a.HW4, 0));
            return;
        }
        constexpr int set = decltype(SET)::value, e = decltype(E)::value, i = e / XR, jj = e % XR;
        int bad = __builtin_amdgcn_sbfe((int)xinv[i], tap_rs[jj] & 0xff, 1) |
                  __builtin_amdgcn_sbfe((int)xinv[i], tap_rs[jj] >> 8, 1);  // 0 or all ones
        xr[set * NX + e] = __builtin_bit_cast(
            float, __builtin_amdgcn_raw_buffer_load_b32(xrsrc, xvoff[i] | bad, tap_off[jj] + tap_cbase, 0));
    };
    // global -> register set SET: weight quad E of the tile of `step`
    auto load_w = [&](auto SET, int step, auto E) WPK_LAMBDA {
        constexpr int set = decltype(SET)::value, i = decltype(E)::value;
        if (W4 % T == 0 || wkq + i * (T / BN) < BK / 4)
            wr[set * NW + i] = __builtin_bit_cast(
                v4f, __builtin_amdgcn_raw_buffer_load_b128(wrsrc, wvoff,
                                                           step * wstep_bytes + i * wquad_bytes, 0));
    };
    // register set SET -> LDS buffer `buf`
    auto store_x = [&](auto SET, int buf, auto E) WPK_LAMBDA {
        constexpr int set = decltype(SET)::value, e = decltype(E)::value;
        constexpr int i = e / (XR / 4), j4 = e % (XR / 4), b = set * NX + i * XR + 4 * j4;
        v4f v = {xr[b], xr[b + 1], xr[b + 2], xr[b + 3]};
        *reinterpret_cast<v4f *>(Xs0 + buf * XTILE + (pm0 + i * T) * PX + rg * XR + 4 * j4) = v;
    };
    auto store_w = [&](auto SET, int buf, auto E) WPK_LAMBDA {
        constexpr int set = decltype(SET)::value, i = decltype(E)::value;
        if (W4 % T == 0 || wkq + i * (T / BN) < BK / 4)
            *reinterpret_cast<v4f *>(Ws0 + buf * WTILE + wkout * PW + (wkq + i * (T / BN)) * 4) =
                wr[set * NW + i];
    };
    auto load_tile = [&](auto SET, int step) WPK_LAMBDA {
        load_taps(step);
        static_for<NXL>([&](auto E) WPK_LAMBDA { load_x(SET, E); });
        static_for<NW>([&](auto E) WPK_LAMBDA { load_w(SET, step, E); });
    };
    auto store_tile = [&](auto SET, int buf) WPK_LAMBDA {
        static_for<NXQ>([&](auto E) WPK_LAMBDA { store_x(SET, buf, E); });
        static_for<NW>([&](auto E) WPK_LAMBDA { store_w(SET, buf, E); });
    };

    v16f acc[NNT * NMT];
    static_for<NNT * NMT>([&](auto I) WPK_LAMBDA {
        static_for<16>([&](auto E) WPK_LAMBDA { acc[decltype(I)::value][decltype(E)::value] = 0.0f; });
    });

    // One reduction step, r-th of the segment.  The MFMAs read LDS buffer r&1.  Meanwhile tile
    // r+1, which has been in staging set (r+1)%PD since step r-PD, is stored to the other buffer
    // and tile r+1+PD is loaded from global memory into the set it frees, so a load has PD steps
    // to arrive.  In the main loop (INTERLEAVE) these stores and loads are dealt out one by one
    // behind the individual MFMAs, each of which keeps the matrix pipe busy for 64 cycles, so they
    // issue in its shadow; the LDS operands of octet o+1 are read before the MFMAs of octet o.
    // The last steps of a segment (no more tiles to load or store) run the plain form, with
    // whatever store and load is left done up front.  One barrier per step, at its end.
    constexpr int NM = (BK / 2) * NNT * NMT;       // MFMAs per step and wave
    constexpr int NIT = NXQ + NW + NXL + NW;       // stores (x, w) then loads (x, w)
    // the first load item must not come before the scalar tap loads it depends on
    static_assert(((NXQ + NW) * NM + NIT - 1) / NIT >= NNT * NMT, "taps are loaded too late");
    // Pipelined form (K-steps of two octets or more): the operands of a step's FIRST octet are read
    // during the step before it.  The step's only barrier sits in front of its last octet of
    // MFMAs: by then every LDS store of tile r+1 has been issued (they ride behind the MFMAs of
    // the octets before) and every wave holds the last operands of step r in registers, so right
    // after the barrier the first octet of step r+1 is read from the other buffer and arrives
    // while the last octet of step r is being multiplied.  A wave that has a SIMD to itself (the
    // end of every launch, every launch of few workgroups) then never waits for LDS at a step's
    // start; with one barrier-then-read per step that wait was a fifth of the step.
    constexpr int NO = BK / 8;                      // octets per step
    constexpr bool PIPE = NO >= 2;
    constexpr int NML = 4 * NNT * NMT;              // MFMAs per octet
    // every LDS store of the interleaved list rides behind an MFMA before the last octet
    static_assert(!PIPE || ((NXQ + NW) * NM + NIT - 1) / NIT <= NM - NML, "LDS stores reach the last octet");
    v4f av[2 * NNT], bv[2 * NMT];
    auto read_octet = [&](const int buf, auto HALF, const int oct) WPK_LAMBDA {
        constexpr int h = decltype(HALF)::value;
        const float *xs = Xs0 + buf * XTILE + (wave_m * TM + lcol) * PX + lrow * 4 + oct * 8;
        const float *ws = Ws0 + buf * WTILE + (wave_n * TN + lcol) * PW + lrow * 4 + oct * 8;
        static_for<NNT>([&](auto I) WPK_LAMBDA {
            av[h * NNT + decltype(I)::value] = *reinterpret_cast<const v4f *>(ws + decltype(I)::value * 32 * PW);
        });
        static_for<NMT>([&](auto J) WPK_LAMBDA {
            bv[h * NMT + decltype(J)::value] = *reinterpret_cast<const v4f *>(xs + decltype(J)::value * 32 * PX);
        });
    };
    auto step_body = [&](const int r, auto SET, auto INTERLEAVE) WPK_LAMBDA {
        constexpr bool inter = decltype(INTERLEAVE)::value;
        const int cur = r & 1;
        if constexpr (!PIPE) {
            read_octet(cur, std::integral_constant<int, 0>{}, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
        static_for<NO>([&](auto KO) WPK_LAMBDA {
            constexpr int ko = decltype(KO)::value;
            constexpr int c = ko & 1, nx = c ^ 1;
            if constexpr (ko + 1 < NO) {
                read_octet(cur, std::integral_constant<int, nx>{}, ko + 1);
                __builtin_amdgcn_sched_barrier(0);
            } else if constexpr (PIPE) {
                __syncthreads();
                // (after the last step of a segment this reads a tile nobody uses: in bounds, ignored)
                read_octet(cur ^ 1, std::integral_constant<int, nx>{}, 0);
                __builtin_amdgcn_sched_barrier(0);
            }
            static_for<NML>([&](auto QIJ) WPK_LAMBDA {
                constexpr int qij = decltype(QIJ)::value;
                constexpr int q = qij / (NNT * NMT), ij = qij % (NNT * NMT), i = ij / NMT, j = ij % NMT;
                constexpr int t = ko * NML + qij;  // number of this MFMA within the step
                acc[ij] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[c * NNT + i][q], bv[c * NMT + j][q],
                                                               acc[ij], 0, 0, 0);
                if constexpr (inter) {
                    // The scalar loads of the next tile's taps go behind the MFMA that is the last
                    // to wait for an operand of the first octet: scalar and LDS loads share one
                    // counter, so the next wait for LDS data also waits for them -- and from here
                    // that wait is most of an octet of MFMAs away.
                    if constexpr (t == NNT * NMT - 1) {
                        __builtin_amdgcn_sched_barrier(0);
                        load_taps(kbeg + r + 1 + PD);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                    // items [t*NIT/NM, (t+1)*NIT/NM) of the stores-then-loads list ride behind it
                    constexpr int lo = t * NIT / NM, hi = (t + 1) * NIT / NM;
                    static_for<hi - lo>([&](auto D) WPK_LAMBDA {
                        constexpr int it = lo + decltype(D)::value;
                        if constexpr (it < NXQ)
                            store_x(SET, cur ^ 1, std::integral_constant<int, it>{});
                        else if constexpr (it < NXQ + NW)
                            store_w(SET, cur ^ 1, std::integral_constant<int, it - NXQ>{});
                        else if constexpr (it < NXQ + NW + NXL)
                            load_x(SET, std::integral_constant<int, it - NXQ - NW>{});
                        else
                            load_w(SET, kbeg + r + 1 + PD, std::integral_constant<int, it - NXQ - NW - NXL>{});
                    });
                }
                __builtin_amdgcn_sched_barrier(0);
            });
        });
        if constexpr (!PIPE) __syncthreads();
    };
    using std::false_type;
    using std::true_type;

    // prologue: the loads of tiles 0..PD-1 are all issued before anything waits (one memory
    // latency, not two); then tile 0 goes to LDS buffer 0 and tile PD into the set it frees
    // (tile 0: the scalar tap loads and the weight loads, which depend on the tile alone, are
    // issued first; the per-pixel gather state is computed while they are in flight)
    const int nr = kend - kbeg;
    load_taps(kbeg, false);
    static_for<NW>([&](auto E) WPK_LAMBDA { load_w(std::integral_constant<int, 0>{}, kbeg, E); });
    gather_state();
    if constexpr (TAPM) fold_mask();
    static_for<NXL>([&](auto E) WPK_LAMBDA { load_x(std::integral_constant<int, 0>{}, E); });
    static_for<PD - 1>([&](auto P) WPK_LAMBDA {
        constexpr int t = decltype(P)::value + 1;
        if (t < nr) load_tile(std::integral_constant<int, t>{}, kbeg + t);
    });
    store_tile(std::integral_constant<int, 0>{}, 0);
    if (PD < nr) load_tile(std::integral_constant<int, 0>{}, kbeg + PD);
    __syncthreads();
    if constexpr (PIPE) read_octet(0, std::integral_constant<int, 0>{}, 0);
    int r = 0;
    // main loop: every step still has a tile to store (r+1) and one to load (r+1+PD)
    for (; r + 2 * PD < nr; r += PD)
        static_for<PD>([&](auto P) WPK_LAMBDA {
            constexpr int p = decltype(P)::value;
            step_body(r + p, std::integral_constant<int, (p + 1) % PD>{}, true_type{});
        });
    // tail: at most 2*PD steps
    for (; r < nr; ++r) {
        const int set = (r + 1) % PD;
        static_for<PD>([&](auto P) WPK_LAMBDA {
            if (set == decltype(P)::value) {
                if (r + 1 < nr) store_tile(P, (r & 1) ^ 1);
                if (r + 1 + PD < nr) load_tile(P, kbeg + r + 1 + PD);
            }
        });
        step_body(r, std::integral_constant<int, 0>{}, false_type{});
    }

    const cold_ptr ce = cold_args();  // (after the steps: what the meeting and the stores need)
    // ---- fix-up of a shared tile -----------------------------------------------------------------
    if (mode == kFixup) {
        // Slot layout: accumulator quad (ij, e4) of thread t at float (ij*4 + e4)*4*T + 4*t.
        // Partials travel between workgroups that may sit on different XCDs, whose L2 caches do
        // not snoop each other.  Instead of fences that write back and invalidate whole caches,
        // the partials alone are stored and loaded with the system-scope cache policy (write
        // through / read past the non-coherent levels); everything else stays cached.
        constexpr int kCoherent = 17;  // sc0 | sc1
        const __amdgpu_buffer_rsrc_t srsrc = __builtin_amdgcn_make_buffer_rsrc(
            (void *)(ce->ws + (size_t)fix_j * ce->ws_maxc * (BM * BN)), 0, ce->ws_maxc * (BM * BN) * 4,
            0x00020000);
        const int mine = (fix_slot * (BM * BN) + 4 * tid) * 4;
        static_for<NNT * NMT * 4>([&](auto Q) WPK_LAMBDA {
            constexpr int qd = decltype(Q)::value, ij = qd / 4, e4 = qd % 4;
            v4f v = {acc[ij][4 * e4], acc[ij][4 * e4 + 1], acc[ij][4 * e4 + 2], acc[ij][4 * e4 + 3]};
            __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(v4u, v), srsrc, mine,
                                                   qd * 16 * T, kCoherent);
        });
        // every store of this wave acknowledged, then every wave of the workgroup, before the
        // arrival is counted
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
        if (tid == 0) arrival = atomicAdd(ce->ws_cnt + fix_j, 1);
        __syncthreads();
        const int arrived_before = arrival;
        __syncthreads();  // everyone has read `arrival` before a later segment overwrites it
        if (arrived_before != fix_n - 1) return;  // not the last: done with this tile
        if (tid == 0) ce->ws_cnt[fix_j] = 0;        // leave the counter clean for the next launch
        // Add the other workgroups' slots to this one's accumulators.
        if constexpr (NNT * NMT == 1) {
            // a single 32x32 block per wave has little to load per slot: four slots at a time, all
            // requested before the first is added, so the sharers of a tile cost one memory round
            // trip per four of them (a slot number past the last becomes an out-of-range offset,
            // which loads 0)
            constexpr int kGang = 4;
            for (int t0 = 0; t0 < fix_n - 1; t0 += kGang) {
                v4f part[kGang][4];
                static_for<kGang>([&](auto U) WPK_LAMBDA {
                    constexpr int u = decltype(U)::value;
                    const int t = t0 + u, sl = t + (t >= fix_slot ? 1 : 0);  // t-th slot not mine
                    const unsigned off =
                        t < fix_n - 1 ? (unsigned)((sl * (BM * BN) + 4 * tid) * 4) : 0xffffffffu;
                    static_for<4>([&](auto Q) WPK_LAMBDA {
                        constexpr int qd = decltype(Q)::value;
                        part[u][qd] = __builtin_bit_cast(
                            v4f, __builtin_amdgcn_raw_buffer_load_b128(srsrc, off, qd * 16 * T, kCoherent));
                    });
                });
                static_for<4 * kGang>([&](auto UQ) WPK_LAMBDA {
                    constexpr int u = decltype(UQ)::value / 4, qd = decltype(UQ)::value % 4;
                    acc[0][4 * qd] += part[u][qd][0];
                    acc[0][4 * qd + 1] += part[u][qd][1];
                    acc[0][4 * qd + 2] += part[u][qd][2];
                    acc[0][4 * qd + 3] += part[u][qd][3];
                });
            }
        } else {
            for (int sl = 0; sl < fix_n; ++sl) {
                if (sl == fix_slot) continue;
                const int other = (sl * (BM * BN) + 4 * tid) * 4;
                static_for<NNT * NMT * 4>([&](auto Q) WPK_LAMBDA {
                    constexpr int qd = decltype(Q)::value, ij = qd / 4, e4 = qd % 4;
                    v4f v = __builtin_bit_cast(
                        v4f, __builtin_amdgcn_raw_buffer_load_b128(srsrc, other, qd * 16 * T, kCoherent));
                    acc[ij][4 * e4] += v[0];
                    acc[ij][4 * e4 + 1] += v[1];
                    acc[ij][4 * e4 + 2] += v[2];
                    acc[ij][4 * e4 + 3] += v[3];
                });
            }
        }
    }
    store_wave_tile<NNT, NMT>(ce, acc, m0 + wave_m * TM, n0 + wave_n * TN, lrow, lcol, mode == kAtomic);
    };  // run_segment

    // ---- which segments this workgroup runs ----------------------------------------------------
    // persist == 0: one workgroup per (tile, reduction slice): blockIdx -> tile, slice; the slices
    //   of a tile meet through the workspace if the host gave one, else through atomics.
    // persist  > 0: gridDim.x = G persistent workgroups.  Each takes whole tiles g, g+G, ...
    //   of the first tiles_dp = floor(tiles/G)*G tiles.  The reduction steps of the remaining
    //   tiles, laid end to end (`units` of them), are cut into runs of q or q+1 steps (the first
    //   `rem` get q+1), sk_groups of them: G, unless that would make the runs too short to be
    //   worth a prologue.  Either sk_groups further workgroups are appended to the grid and take
    //   one run each (a.runners: whenever all of them fit the device beside the G), or each of
    //   the first sk_groups workgroups does a run first, then its whole tiles.  A run that does
    //   not cover a tile's whole reduction shares the tile with its neighbours in g: fix-up
    //   through the workspace if the host gave one, else atomics into zeroed y.
    // (tiles_dp, sk_groups, q = sk_q, rem = sk_rem and the divisors come from the host: they
    // depend on the launch alone, and all of it fits 32 bits)
    const bool persistent = a.persist > 0;
    const int g = blockIdx.x;
    // With a.runners > 0 the grid is grid_persist + runners workgroups: the first grid_persist take
    // whole tiles only, the others one dealt-out run each and nothing else, so that a run and a
    // whole tile of the same compute unit proceed side by side instead of one after the other.
    const int G = a.runners ? a.grid_persist : (int)gridDim.x;
    const bool runner = a.runners && g >= G;
    int next_dp = g;
    // (remap: run number gr instead of g, so that consecutive runs -- neighbouring tiles, the
    // slices of one tile -- sit on one XCD and share its L2; G is a multiple of the number of XCDs,
    // so a runner's XCD is (g - G) % 8 as well)
    const int gl = runner ? g - G : g;
    const int gr = a.remap ? xcd_remap(gl, runner ? a.runners : G) : gl;
    int u0, u1;
    {
        const cold_ptr c = cold_args();
        const int q = c->sk_q, rem = c->sk_rem;
        const bool dealt = persistent && gr < c->sk_groups && (!a.runners || runner);
        u0 = dealt ? gr * q + min(gr, rem) : 0;
        u1 = dealt ? (gr + 1) * q + min(gr + 1, rem) : 0;
        if (runner) next_dp = c->tiles_dp;  // no whole tiles
    }
    bool once = !persistent;
    for (;;) {
        int tile, kbeg, kend, mode = kStore, fix_j = 0, fix_slot = 0, fix_n = 1;
        const cold_ptr c = cold_args();   // the iterator's constants, once per segment
        if (once) {
            once = false;
            const int slice = fdiv(gr, WPK_COLD_DIV(c, div_tiles));
            tile = gr - slice * c->tiles;
            kbeg = slice * c->steps_per_split;
            kend = min(a.nsteps, kbeg + c->steps_per_split);
            if (c->split_k > 1) {
                mode = c->ws ? kFixup : kAtomic;
                fix_j = tile;
                fix_slot = slice;
                fix_n = c->split_k;
            }
        } else if (persistent && u0 < u1) {
            // (the dealt-out run comes BEFORE the workgroup's whole tiles: the sharers of a tile then
            // meet while everybody else still has whole tiles to multiply, instead of after it, when
            // the chain of memory round trips of the meeting would be all the device has left to do)
            const int q = c->sk_q, rem = c->sk_rem;
            auto owner_of = [&](int u) {  // which workgroup's run holds unit u
                if (u < rem * (q + 1)) return fdiv(u, WPK_COLD_DIV(c, div_q1));
                return rem + fdiv(u - rem * (q + 1), WPK_COLD_DIV(c, div_q0));
            };
            fix_j = fdiv(u0, WPK_COLD_DIV(c, div_nsteps));
            tile = c->tiles_dp + fix_j;
            kbeg = u0 - fix_j * a.nsteps;
            kend = min(a.nsteps, kbeg + (u1 - u0));
            u0 += kend - kbeg;
            if (!(kbeg == 0 && kend == a.nsteps)) {
                const int first = owner_of(fix_j * a.nsteps);
                fix_n = owner_of((fix_j + 1) * a.nsteps - 1) - first + 1;
                fix_slot = gr - first;
                mode = c->ws ? kFixup : kAtomic;
            }
        } else if (persistent && next_dp < c->tiles_dp) {
            // (remap: within a round, each XCD takes a contiguous range of the round's G tiles, so
            // that tiles which share rows of x share an L2)
            tile = next_dp - g + gr;
            kbeg = 0;
            kend = a.nsteps;
            next_dp += G;
        } else {
            break;
        }
        run_segment(tile, kbeg, kend, mode, fix_j, fix_slot, fix_n);
    }
}

template <int BM, int BN, int BK, int WM, int WN, int PD, int XL>
hipError_t launch_gather_form(IgemmArgs a, hipStream_t stream)
{
    const auto kernel = igemm_kernel<BM, BN, BK, WM, WN, PD, XL>;
    if (a.persist > 0 && a.tiles_dp > 0 && a.sk_groups > 0) {
        // The tiles beyond the whole rounds go to workgroups of their own when every workgroup of
        // the larger grid is resident at once (how many a compute unit holds is asked once per
        // kernel); otherwise the first sk_groups workgroups do a run before their tiles.  (With no
        // whole round there is nothing to run beside: the grid stays as it is.)
        static std::atomic<int> resident{-1};  // workgroups per compute unit (every writer stores the same value)
        int n = resident.load(std::memory_order_relaxed);
        if (n < 0) {
            n = 0;
            if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, kernel, 64 * WM * WN, 0) != hipSuccess) {
                (void)hipGetLastError();
                n = 0;
            }
            resident.store(n, std::memory_order_relaxed);
        }
        const long long cus = a.grid_persist / a.persist;
        if ((long long)n * cus >= (long long)a.grid_persist + a.sk_groups) a.runners = a.sk_groups;
    }
    dim3 grid((unsigned)(a.persist > 0 ? a.grid_persist + a.runners : a.tiles_m * a.tiles_n * a.split_k));
    hipLaunchKernelGGL(kernel, grid, dim3(64 * WM * WN), 0, stream, a);
    return hipGetLastError();
}

// (wpk_wsplit.h)
template <int BN, int WK, int PD>
hipError_t launch_wsplit(const IgemmArgs &a, hipStream_t stream);

template <int BM, int BN, int BK, int WM, int WN, int PD>
hipError_t launch_igemm(const IgemmArgs &a, hipStream_t stream)
{
    if constexpr (BM == kWaveSplitBm) {
        static_assert(BK == 8, "the wave-split members work in octets");
        return launch_wsplit<BN, WM * WN, 4 * PD>(a, stream);
    } else {
        if (a.xl == 2) return launch_gather_form<BM, BN, BK, WM, WN, PD, 1>(a, stream);
        if (a.xl == 3) return launch_gather_form<BM, BN, BK, WM, WN, PD, 2>(a, stream);
        return launch_gather_form<BM, BN, BK, WM, WN, PD, 0>(a, stream);
    }
}

}  // namespace wpk
#endif
