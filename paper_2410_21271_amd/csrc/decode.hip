// Small-M ("decode") kernels: y = x.What^T + t.B^T for up to 16 tokens per pass, and t = x.A^T.
//
// HBM-bound: every weight byte is read once, decoded in registers and fed to 16x16x32 fp16 MFMAs
// whose 16-row operand is the token block (rows beyond M are zero).  The weight tile supplies the
// other operand directly from the stored words of each lane (see tiles.hpp).  A workgroup of four
// wavefronts owns RB row blocks of 16 output rows; its wavefronts split the contraction dimension
// tile by tile (consecutive wavefronts read consecutive 1 KiB tiles), keep one fp32 accumulator per
// row block and combine them through LDS in a fixed order.  The low-rank up-projection is a
// continuation of the same contraction: after the backbone tiles the wavefronts run over the tiles
// of B with t as the activation operand and add into the SAME accumulators (Sec. 4.5 / App. A.6 of
// the paper fuse B's product into the quantised product's output; here nothing is written between
// the two), so y is converted and stored exactly once.
#include "kernels.hpp"
#include "tiles.hpp"

namespace eora {

struct Seg {
    const void* w;            // stored tiles
    const _Float16* scales;   // per (row block, group, row) fp16, or nullptr (F16)
    const uint32_t* zeros;    // asymmetric formats only
    const void* act;          // activation operand: fp16 (x) or fp32 (t), row-major
    int lda;                  // its row stride in elements
    int K;                    // contraction length
    int group;                // quantisation group (asymmetric formats)
};

template <int FMT>
struct FmtTraits;
template <> struct FmtTraits<S_Q4> { static constexpr int KT = 128; };
template <> struct FmtTraits<S_Q3> { static constexpr int KT = 128; };
template <> struct FmtTraits<S_Q4S128> { static constexpr int KT = 128; };
template <> struct FmtTraits<S_Q4S64> { static constexpr int KT = 64; };
template <> struct FmtTraits<S_F16> { static constexpr int KT = 32; };

// activation fragment of lane (token row m, column quarter j) for MFMA step t of k-tile g
template <bool ACT_F32, int KT>
__device__ __forceinline__ h8 load_act(const void* act, int lda, bool row_ok, int m, int col)
{
    Frag f;
    f.q = u4{0u, 0u, 0u, 0u};
    if (row_ok) {
        if constexpr (ACT_F32) {
            const float* p = (const float*)act + (size_t)m * lda + col;
            const f4 a = *(const f4*)p, b = *(const f4*)(p + 4);
            f.v = h8{(_Float16)a[0], (_Float16)a[1], (_Float16)a[2], (_Float16)a[3],
                     (_Float16)b[0], (_Float16)b[1], (_Float16)b[2], (_Float16)b[3]};
        } else {
            f.q = *(const u4*)((const _Float16*)act + (size_t)m * lda + col);
        }
    }
    return f.v;
}

template <int FMT, bool ACT_F32, int RB>
__device__ __forceinline__ void run_segment(f4 (&acc)[RB], const Seg& s, int wave, int lane, int m0, int M, int R0)
{
    constexpr int KT = FmtTraits<FMT>::KT;
    constexpr int NMF = KT / 32;                 // MFMAs (= stored words of a lane) per tile
    const int n = lane & 15, j = lane >> 4;
    const int ntk = s.K / KT;
    const int m = m0 + n;
    const bool row_ok = m < M;

    for (int g = wave; g < ntk; g += 4) {
        h8 xa[NMF];
#pragma unroll
        for (int t = 0; t < NMF; ++t)
            xa[t] = load_act<ACT_F32, KT>(s.act, s.lda, row_ok, m, g * KT + (KT / 4) * j + 8 * t);

#pragma unroll
        for (int rb = 0; rb < RB; ++rb) {
            const size_t tile = (size_t)(R0 + rb) * ntk + g;
            if constexpr (FMT == S_F16) {
                const h8 b = *((const h8*)s.w + tile * 64 + lane);
                acc[rb] = mfma16(xa[0], b, acc[rb]);
            } else {
                h8 b[NMF];
                float sc;
                if constexpr (FMT == S_Q4) {
                    const size_t rq = (size_t)(R0 + rb) * (s.K / s.group) + (size_t)g * KT / s.group;
                    const u4 w = *((const u4*)s.w + tile * 64 + lane);
                    const uint32_t z = load_zero(s.zeros, rq, n);
                    sc = (float)s.scales[rq * 16 + n];
                    const uint32_t c1024 = k1024(z), c64 = k64(z);
#pragma unroll
                    for (int t = 0; t < 4; ++t) b[t] = dq4_word(w[t], c1024, c64);
                } else if constexpr (FMT == S_Q3) {
                    const size_t rq = (size_t)(R0 + rb) * (s.K / s.group) + (size_t)g * KT / s.group;
                    const uint32_t* p = (const uint32_t*)s.w + (tile * 64 + lane) * 3;
                    const uint32_t d0 = p[0], d1 = p[1], d2 = p[2];
                    const uint32_t z = load_zero(s.zeros, rq, n);
                    sc = (float)s.scales[rq * 16 + n];
                    dq3_lane(d0, d1, d2, z, b);
                } else {   // symmetric 4-bit factor, zero-point 8, one group per k-tile
                    sc = (float)s.scales[tile * 16 + n];
                    const uint32_t c1024 = k1024(8u), c64 = k64(8u);
                    const uint32_t* p = (const uint32_t*)s.w + (tile * 64 + lane) * NMF;
#pragma unroll
                    for (int t = 0; t < NMF; ++t) b[t] = dq4_word(p[t], c1024, c64);
                }
                f4 part = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int t = 0; t < NMF; ++t) part = mfma16(xa[t], b[t], part);
                acc[rb] += sc * part;            // the lane's output column is row n of the tile
            }
        }
    }
}

// grid: x = row strips of 16*RB output rows, y = blocks of 16 tokens.  256 threads.
template <int FM, int FE, int RB, bool OUT_F32>
__global__ __launch_bounds__(256) void decode_kernel(DecodeArgs a)
{
    __shared__ f4 red[3][RB][64];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int R0 = blockIdx.x * RB;
    const int m0 = blockIdx.y * 16;

    f4 acc[RB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) acc[rb] = f4{0.f, 0.f, 0.f, 0.f};

    const Seg main{a.w, a.w_scales, a.w_zeros, a.x, a.d_in, a.d_in, a.group};
    run_segment<FM, false, RB>(acc, main, wave, lane, m0, a.M, R0);
    if constexpr (FE != S_NONE) {
        const Seg ext{a.B, a.B_scales, nullptr, a.t, a.r, a.r, 0};
        run_segment<FE, true, RB>(acc, ext, wave, lane, m0, a.M, R0);
    }

    if (wave > 0) {
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) red[wave - 1][rb][lane] = acc[rb];
    }
    __syncthreads();
    if (wave == 0) {
        const int n = lane & 15, j = lane >> 4;
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) {
            f4 v = acc[rb];
            v += red[0][rb][lane];
            v += red[1][rb][lane];
            v += red[2][rb][lane];
            const int o = (R0 + rb) * 16 + n;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int m = m0 + 4 * j + i;          // accumulator register i holds token row 4*j+i
                if (m < a.M) {
                    if constexpr (OUT_F32) ((float*)a.y)[(size_t)m * a.d_out + o] = v[i];
                    else ((_Float16*)a.y)[(size_t)m * a.d_out + o] = (_Float16)v[i];
                }
            }
        }
    }
}

template <int FM, int FE, bool OUT_F32>
static hipError_t launch_rb(const DecodeArgs& a, hipStream_t stream)
{
    const int nblk = a.d_out / 16;
    const int mblocks = (a.M + 15) / 16;
    // Larger strips reuse the activation fragments over more weight tiles, smaller ones give
    // more workgroups; keep at least ~2 workgroups per compute unit when the shape allows.
    int rb = 1;
    if (a.M > 4) {
        if (nblk % 4 == 0 && nblk / 4 >= 512) rb = 4;
        else if (nblk % 2 == 0 && nblk / 2 >= 512) rb = 2;
    }
    const dim3 block(256);
    if (rb == 4) hipLaunchKernelGGL((decode_kernel<FM, FE, 4, OUT_F32>), dim3(nblk / 4, mblocks), block, 0, stream, a);
    else if (rb == 2) hipLaunchKernelGGL((decode_kernel<FM, FE, 2, OUT_F32>), dim3(nblk / 2, mblocks), block, 0, stream, a);
    else hipLaunchKernelGGL((decode_kernel<FM, FE, 1, OUT_F32>), dim3(nblk, mblocks), block, 0, stream, a);
    return hipGetLastError();
}

template <int FM>
static hipError_t launch_ext(const DecodeArgs& a, int fe, hipStream_t stream)
{
    switch (fe) {
        case S_NONE: return launch_rb<FM, S_NONE, false>(a, stream);
        case S_F16: return launch_rb<FM, S_F16, false>(a, stream);
        case S_Q4S128: return launch_rb<FM, S_Q4S128, false>(a, stream);
        case S_Q4S64: return launch_rb<FM, S_Q4S64, false>(a, stream);
        default: return hipErrorInvalidValue;
    }
}

hipError_t launch_decode(const DecodeArgs& a, int fm, int fe, hipStream_t stream)
{
    switch (fm) {
        case S_Q4: return launch_ext<S_Q4>(a, fe, stream);
        case S_Q3: return launch_ext<S_Q3>(a, fe, stream);
        default: return hipErrorInvalidValue;
    }
}

// t = x.A^T as fp32 M x r: the same kernel with A as the weight operand and no extension.
hipError_t launch_downproj(const DecodeArgs& a, int fa, hipStream_t stream)
{
    switch (fa) {
        case S_F16: return launch_rb<S_F16, S_NONE, true>(a, stream);
        case S_Q4S128: return launch_rb<S_Q4S128, S_NONE, true>(a, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace eora
