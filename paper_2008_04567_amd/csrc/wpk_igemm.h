// The tiled implicit-GEMM forward convolution kernel family for gfx950 (CDNA4, wave64).
//
// GEMM view that matches NCHW memory: Y[kout][pixel] = sum_kk Wp[kk][kout] * Xcol[kk][pixel],
// pixel = (n,p,q) flattened, kk = (c,r,s) flattened in the weights' own KCRS order.  x and y are
// both contiguous along q, so activation loads and output stores coalesce along the pixel axis;
// the weights are re-packed once into reduction-major [CRSpad][Kpad] so a weight tile is a plain
// 16-byte-per-lane stream.  The im2col matrix is never written to memory: a workgroup gathers a
// BK x BM activation tile per step straight into LDS.  A per-problem tap table gives, for every
// reduction row, the element offset of its tap inside x and its tap number r*S+s; each lane keeps
// a 64-bit mask of the taps that fall inside the image for its pixel, and out-of-image taps are
// loaded through a buffer descriptor at an out-of-range offset, which returns zero.
//
// The contraction runs on v_mfma_f32_32x32x2_f32: A = 32 output channels x 2 reduction rows,
// B = 2 reduction rows x 32 pixels, D = 32 x 32 with the pixel index on the lane axis, so that
// each accumulator register of a half-wave stores 32 consecutive pixels (128 contiguous bytes).
#ifndef WPK_IGEMM_H
#define WPK_IGEMM_H

#include <hip/hip_runtime.h>

#include <type_traits>
#include <utility>

#include "wpk_internal.h"

namespace wpk {

typedef float v16f __attribute__((ext_vector_type(16)));
typedef float v4f __attribute__((ext_vector_type(4)));

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

// The tap table is read through the constant address space: wave-uniform scalar loads.
typedef const int __attribute__((address_space(4))) *tap_ptr;

template <int BM, int BN, int BK, int WM, int WN>
__global__ void __launch_bounds__(64 * WM * WN) igemm_kernel(const IgemmArgs a)
{
    constexpr int T = 64 * WM * WN;
    constexpr int TM = BM / WM, TN = BN / WN;   // wave tile
    constexpr int NMT = TM / 32, NNT = TN / 32; // 32x32 MFMA blocks per wave tile
    constexpr int XP = BM > T ? BM / T : 1;     // pixels per thread in the gather
    constexpr int RG = T > BM ? T / BM : 1;     // row groups in the gather
    constexpr int XR = BK / RG;                 // rows per thread per pixel
    constexpr int W4 = BK * BN / 4;             // float4s in a weight tile
    constexpr int WL = (W4 + T - 1) / T;
    static_assert(TM % 32 == 0 && TN % 32 == 0, "wave tile must be whole MFMA blocks");
    static_assert(BM % 64 == 0, "a wave gathers one reduction row at a time");
    static_assert(BK % RG == 0 && BK % 2 == 0, "row groups must divide the step");
    static_assert((T >= BM && T % BM == 0) || (T < BM && BM % T == 0), "gather mapping");

    __shared__ float Xs[2][BK * BM];
    __shared__ __attribute__((aligned(16))) float Ws[2][BK * BN];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wave_m = wave % WM, wave_n = wave / WM;

    int bid = blockIdx.x;
    if (a.remap) bid = xcd_remap(bid, gridDim.x);
    const int tile_n = bid % a.tiles_n;
    const int t2 = bid / a.tiles_n;
    const int tile_m = t2 % a.tiles_m;
    const int split = t2 / a.tiles_m;
    const int m0 = tile_m * BM, n0 = tile_n * BN;

    // ---- per-thread gather state: pixel offset inside x and the in-image tap mask ------------
    const int pm0 = tid % (T < BM ? T : BM);
    const int rg = __builtin_amdgcn_readfirstlane(tid / BM);  // 0 when T <= BM
    int xbase[XP];
    unsigned long long tapmask[XP];
    static_for<XP>([&](auto I) WPK_LAMBDA {
        constexpr int i = decltype(I)::value;
        int m = m0 + pm0 + i * T;
        xbase[i] = 0;
        tapmask[i] = 0;
        if (m < a.M) {
            int n = m / a.PQ, pq = m - n * a.PQ;
            int p = pq / a.Q, q = pq - p * a.Q;
            int ih0 = p * a.stride_h - a.pad_h, iw0 = q * a.stride_w - a.pad_w;
            xbase[i] = (n * a.C * a.H + ih0) * a.W + iw0;
            unsigned long long msk = 0;
            for (int r = 0; r < a.R; ++r) {
                int ih = ih0 + r * a.dil_h;
                bool hin = ih >= 0 && ih < a.H;
                for (int s = 0; s < a.S; ++s) {
                    int iw = iw0 + s * a.dil_w;
                    if (hin && iw >= 0 && iw < a.W) msk |= 1ull << (r * a.S + s);
                }
            }
            tapmask[i] = msk;
        }
    });
    const __amdgpu_buffer_rsrc_t xrsrc =
        __builtin_amdgcn_make_buffer_rsrc((void *)a.x, 0, (int)a.x_bytes, 0x00020000);
    const tap_ptr taps = (tap_ptr)(unsigned long long)a.ktab;
    const float *wsrc = a.wp + n0;

    float xr[XP * XR];
    v4f wr[WL];

    // A row group owns XR consecutive reduction rows of the step, so its tap-table entries are
    // one contiguous, wave-uniform block: fetched with scalar loads, all before the first use.
    auto gload = [&](int step) WPK_LAMBDA {
        const int k0 = step * BK;
        tap_ptr tp = taps + 2 * (k0 + rg * XR);
        int tap_off[XR], tap_idx[XR];
        static_for<XR>([&](auto J) WPK_LAMBDA {
            tap_off[decltype(J)::value] = tp[2 * decltype(J)::value];
            tap_idx[decltype(J)::value] = tp[2 * decltype(J)::value + 1];
        });
        static_for<XR>([&](auto J) WPK_LAMBDA {
            constexpr int jj = decltype(J)::value;
            static_for<XP>([&](auto I) WPK_LAMBDA {
                constexpr int i = decltype(I)::value;
                unsigned bit = (unsigned)(tapmask[i] >> tap_idx[jj]) & 1u;
                unsigned off = bit ? (unsigned)(xbase[i] + tap_off[jj]) * 4u : 0x80000000u;
                xr[i * XR + jj] = __builtin_bit_cast(
                    float, __builtin_amdgcn_raw_buffer_load_b32(xrsrc, (int)off, 0, 0));
            });
        });
        static_for<WL>([&](auto I) WPK_LAMBDA {
            constexpr int i = decltype(I)::value;
            int e = tid + i * T;
            if (W4 % T == 0 || e < W4) {
                int row = e / (BN / 4), c4 = e % (BN / 4);
                wr[i] = *reinterpret_cast<const v4f *>(wsrc + (size_t)(k0 + row) * a.Kpad + c4 * 4);
            }
        });
    };
    auto lstore = [&](int buf) WPK_LAMBDA {
        static_for<XR>([&](auto J) WPK_LAMBDA {
            constexpr int jj = decltype(J)::value;
            static_for<XP>([&](auto I) WPK_LAMBDA {
                constexpr int i = decltype(I)::value;
                Xs[buf][(rg * XR + jj) * BM + pm0 + i * T] = xr[i * XR + jj];
            });
        });
        static_for<WL>([&](auto I) WPK_LAMBDA {
            constexpr int i = decltype(I)::value;
            int e = tid + i * T;
            if (W4 % T == 0 || e < W4) *reinterpret_cast<v4f *>(&Ws[buf][e * 4]) = wr[i];
        });
    };

    v16f acc[NNT * NMT];
    static_for<NNT * NMT>([&](auto I) WPK_LAMBDA {
        static_for<16>([&](auto E) WPK_LAMBDA { acc[decltype(I)::value][decltype(E)::value] = 0.0f; });
    });

    const int kbeg = split * a.steps_per_split;
    const int kend = min(a.nsteps, kbeg + a.steps_per_split);
    const int lrow = lane >> 5, lcol = lane & 31;

    // Three-deep pipeline over two LDS buffers: while the MFMAs of step s read buffer s&1, the
    // tile of step s+1 (in registers since the previous step) is stored to the other buffer and
    // the global loads of step s+2 are issued.  One barrier per step, at its end.
    if (kbeg < kend) {
        gload(kbeg);
        lstore(0);
        if (kbeg + 1 < kend) gload(kbeg + 1);
    }
    __syncthreads();
    // LDS read instructions per row pair after the compiler pairs neighbouring 32-column blocks
    constexpr int DSR = (NNT + 1) / 2 + (NMT + 1) / 2;
    for (int step = kbeg; step < kend; ++step) {
        const int cur = (step - kbeg) & 1;
        const float *xs = Xs[cur] + wave_m * TM + lcol + lrow * BM;
        const float *ws = Ws[cur] + wave_n * TN + lcol + lrow * BN;
        // operands of row pair kk+2 are fetched from LDS before the MFMAs of row pair kk issue
        float av[2 * NNT], bv[2 * NMT];
        static_for<NNT>([&](auto I) WPK_LAMBDA { av[decltype(I)::value] = ws[decltype(I)::value * 32]; });
        static_for<NMT>([&](auto J) WPK_LAMBDA { bv[decltype(J)::value] = xs[decltype(J)::value * 32]; });
        asm volatile("" ::: "memory");
        __builtin_amdgcn_sched_barrier(0);
        if (step + 1 < kend) lstore(cur ^ 1);
        asm volatile("" ::: "memory");
        __builtin_amdgcn_sched_barrier(0);
        if (step + 2 < kend) gload(step + 2);
        asm volatile("" ::: "memory");
        __builtin_amdgcn_sched_barrier(0);
        static_for<BK / 2>([&](auto KK) WPK_LAMBDA {
            constexpr int kk = decltype(KK)::value * 2;
            constexpr int c = (kk >> 1) & 1, nx = c ^ 1;
            if constexpr (kk + 2 < BK) {
                static_for<NNT>([&](auto I) WPK_LAMBDA {
                    av[nx * NNT + decltype(I)::value] = ws[(kk + 2) * BN + decltype(I)::value * 32];
                });
                static_for<NMT>([&](auto J) WPK_LAMBDA {
                    bv[nx * NMT + decltype(J)::value] = xs[(kk + 2) * BM + decltype(J)::value * 32];
                });
                __builtin_amdgcn_sched_group_barrier(0x100, DSR, 0);
            }
            static_for<NNT>([&](auto I) WPK_LAMBDA {
                static_for<NMT>([&](auto J) WPK_LAMBDA {
                    constexpr int i = decltype(I)::value, j = decltype(J)::value;
                    acc[i * NMT + j] = __builtin_amdgcn_mfma_f32_32x32x2f32(
                        av[c * NNT + i], bv[c * NMT + j], acc[i * NMT + j], 0, 0, 0);
                });
            });
            __builtin_amdgcn_sched_group_barrier(0x008, NNT * NMT, 0);
        });
        __builtin_amdgcn_sched_barrier(0);
        __syncthreads();
    }

    // ---- epilogue: D[row = channel][col = pixel]; register e of lane l holds row
    //      8*(e/4) + 4*(l/32) + e%4 and column l%32 of its 32x32 block ---------------------------
    const bool atomic = a.split_k > 1;
    static_for<NMT>([&](auto J) WPK_LAMBDA {
        constexpr int j = decltype(J)::value;
        int m = m0 + wave_m * TM + j * 32 + lcol;
        if (m < a.M) {
            int n = m / a.PQ, pq = m - n * a.PQ;
            float *yp = a.y + (size_t)n * a.K * a.PQ + pq;
            static_for<NNT>([&](auto I) WPK_LAMBDA {
                constexpr int i = decltype(I)::value;
                static_for<16>([&](auto E) WPK_LAMBDA {
                    constexpr int e = decltype(E)::value;
                    int kout = n0 + wave_n * TN + i * 32 + 8 * (e / 4) + 4 * lrow + (e & 3);
                    if (kout < a.K) {
                        float *dst = yp + (size_t)kout * a.PQ;
                        if (atomic)
                            unsafeAtomicAdd(dst, acc[i * NMT + j][e]);
                        else
                            *dst = acc[i * NMT + j][e];
                    }
                });
            });
        }
    });
}

template <int BM, int BN, int BK, int WM, int WN>
hipError_t launch_igemm(const IgemmArgs &a, hipStream_t stream)
{
    dim3 grid((unsigned)(a.tiles_m * a.tiles_n * a.split_k));
    hipLaunchKernelGGL((igemm_kernel<BM, BN, BK, WM, WN>), grid, dim3(64 * WM * WN), 0, stream, a);
    return hipGetLastError();
}

}  // namespace wpk
#endif
