// Prefill (many tokens): y = x.What^T + t.B^T as ONE MFMA-bound GEMM whose contraction runs over
// d_in (backbone, dequantised on the way) and then over r (B's tiles with t = x.A^T as the
// activation) into the same fp32 accumulators (Sec. 3 forward equation, Alg. 1 step 7; the fusion of
// B's product into the backbone's output follows Sec. 4.5 / App. A.6).  t itself is a first, small
// launch of the same kernel with A as the weight operand (fp16 M x r into scratch): recomputing it
// per output tile would cost r / 128 times the backbone's MFMA work.
//
// Workgroup: 4 wavefronts (2 x 2), tile = 128 tokens x 128 output rows, contraction in steps of 128
// (one quantisation group).  At 4096 flop/clk per compute unit this tile needs about 40 bytes/clk of
// L2 -> compute-unit traffic at MFMA peak (x as fp16, weights as 4-bit codes), inside the 64 bytes/clk
// a compute unit can take; a 256 x 64 tile would need 68.  Per step
//   - x: the 128 x 128 slab is read with coalesced 16-byte loads (256 bytes per token row) into
//     registers one step ahead and written to LDS as MFMA operand fragments (16 tokens x 32 columns =
//     1 KiB, one conflict-free ds_read_b128 each; a swizzle keeps the scattered writes conflict-free);
//   - weights: each wavefront takes two stored tiles (their words ARE the lane's fragments,
//     tiles.hpp), one step ahead, decodes them to the exact integers code - zero, multiplies by the
//     fp16 group scale and writes the four fragments to LDS; fp16 tiles (A, B) are copied as they are.
//     The scale is folded in here (one fp16 rounding of scale*(code-zero), relative error <= 2^-11 per
//     weight) instead of on the accumulators as in decode: scaling 16 accumulator blocks per group
//     would cost as many VALU cycles as the group's MFMAs;
//   - each wavefront owns 64 tokens x 64 rows: 4 x 4 accumulator blocks, 8 fragment reads per 16 MFMAs.
// LDS is single-buffered (64 KiB, so two workgroups share a compute unit and one computes while the
// other refills): barrier, refill from the prefetch registers, barrier, issue the next prefetch,
// contract.  The epilogue transposes through LDS so that y is written in 128-byte rows.
#include "segments.hpp"

namespace eora {

constexpr int PF_BM = 128, PF_BN = 128;
constexpr int PF_XS = 32 * 1024;                      // x slab: 8 token blocks x 4 slices x 1 KiB
constexpr int PF_WS = 32 * 1024;                      // weights: 8 row blocks x 4 slices x 1 KiB
constexpr int PF_LDS = PF_XS + PF_WS;

struct WReg {
    uint32_t w[4];
    uint32_t zw;
    _Float16 sc;
};

// quantised tile of row block R, k-tile g of the first segment
template <int FMT>
__device__ __forceinline__ void load_wtile(WReg& r, const PrefillArgs& a, int R, int g, int lane)
{
    const int n = lane & 15;
    const int G = a.K1 / 128;
    const size_t tile = (size_t)R * G + g;
    load_words<Fmt<FMT>::WORDS>(*(uint32_t(*)[Fmt<FMT>::WORDS])r.w, (const uint32_t*)a.w + (tile * 64 + lane) * Fmt<FMT>::WORDS);
    const size_t row = (size_t)R * 16 + n;
    if constexpr (Fmt<FMT>::ASYM) {
        const int NG = a.K1 / a.group, grp = (g * 128) / a.group;
        r.sc = a.w_scales[row * NG + grp];
        r.zw = (a.w_zeros[row * ((NG + 7) / 8) + (grp >> 3)] >> (4 * (grp & 7))) & 0xFu;
    } else {
        r.sc = a.w_scales[row * G + g];
        r.zw = 8u;
    }
}

// decode, scale in fp16, write the four fragments of row block slot `rbs` (0..7)
template <int FMT>
__device__ __forceinline__ void store_wtile(const WReg& r, int rbs, int lane)
{
    h8 b[4];
    decode_tile<FMT>(*(const uint32_t(*)[Fmt<FMT>::WORDS])r.w, r.zw, b);
    const h8 s = {r.sc, r.sc, r.sc, r.sc, r.sc, r.sc, r.sc, r.sc};
#pragma unroll
    for (int t = 0; t < 4; ++t) *(h8*)(eora_smem + PF_XS + (rbs * 4 + t) * 1024 + lane * 16) = b[t] * s;
}

// fp16 tiles (KT = 32): the four tiles of a 128-wide step of row block R are the four fragments
__device__ __forceinline__ void load_f16_tiles(u4 (&v)[4], const void* __restrict__ tiles, int K, int R, int step, int lane)
{
    const u4* p = (const u4*)tiles + ((size_t)R * (K / 32) + 4 * step) * 64 + lane;
#pragma unroll
    for (int t = 0; t < 4; ++t) v[t] = p[t * 64];
}

__device__ __forceinline__ void store_f16_tiles(const u4 (&v)[4], int rbs, int lane)
{
#pragma unroll
    for (int t = 0; t < 4; ++t) *(u4*)(eora_smem + PF_XS + (rbs * 4 + t) * 1024 + lane * 16) = v[t];
}

// x slab of one step: thread tid owns the 16-byte chunks c = tid + 256*i, i = 0..7; chunk c is token row
// c / 16 of the tile and columns 8*(c % 16) .. +7 of the step (coalesced: 256 bytes per row).
__device__ __forceinline__ void load_x(u4 (&v)[8], const _Float16* __restrict__ act, int ld, int M, int m0, int col0, int tid)
{
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int c = tid + 256 * i;
        int row = m0 + (c >> 4);
        row = row < M ? row : M - 1;                  // rows beyond M re-read the last row; never stored
        v[i] = *(const u4*)(act + (size_t)row * ld + col0 + 8 * (c & 15));
    }
}

// The fragment (token block mb, slice t) holds for lane (n, j) the columns that the weight fragment of
// that slice holds: 32j + 8t + i for a quantised tile (quarter_major: a lane owns a contiguous quarter
// of the 128 columns), 32t + 8j + i for four fp16 tiles of 32 columns.  Slot n is XOR-ed with 4t so
// that the 64 lanes of a store (4 rows x 16 chunks) spread over all LDS banks.
__device__ __forceinline__ void store_x(const u4 (&v)[8], bool quarter_major, int tid)
{
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int c = tid + 256 * i;
        const int row = c >> 4, kc = c & 15;
        const int j = quarter_major ? kc >> 2 : kc & 3, t = quarter_major ? kc & 3 : kc >> 2;
        const int mb = row >> 4, n = row & 15;
        *(u4*)(eora_smem + ((mb * 4 + t) * 64 + 16 * j + (n ^ (4 * t))) * 16) = v[i];
    }
}

__device__ __forceinline__ void contract_step(f4 (&acc)[4][4], int wm, int wn, int lane)
{
    const int n = lane & 15, j = lane >> 4;
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        h8 af[4], bf[4];
#pragma unroll
        for (int mb = 0; mb < 4; ++mb)
            af[mb] = *(const h8*)(eora_smem + (((4 * wm + mb) * 4 + t) * 64 + 16 * j + (n ^ (4 * t))) * 16);
#pragma unroll
        for (int rb = 0; rb < 4; ++rb)
            bf[rb] = *(const h8*)(eora_smem + PF_XS + (((4 * wn + rb) * 4 + t) * 64 + lane) * 16);
#pragma unroll
        for (int mb = 0; mb < 4; ++mb)
#pragma unroll
            for (int rb = 0; rb < 4; ++rb) acc[mb][rb] = mfma16(af[mb], bf[rb], acc[mb][rb]);
    }
}

// FM: format of the first segment's weights (S_Q4, S_Q3 asymmetric; S_Q4S128; S_F16).  EXT: continue over a
// second segment of fp16 tiles (B) with its own activations (t).
template <int FM, bool EXT>
__global__ __launch_bounds__(256) void prefill_kernel(PrefillArgs a)
{
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int wm = wave >> 1, wn = wave & 1;                      // this wavefront's 64 x 64 quadrant
    const int ntn = (a.N + PF_BN - 1) / PF_BN;
    const int m0 = (blockIdx.x / ntn) * PF_BM;
    const int R0 = (blockIdx.x % ntn) * 8;
    const int nblk = a.N / 16;
    // the two row blocks (slots 2*wave, 2*wave+1) this wavefront decodes, clamped to valid ones
    const int Ra = R0 + 2 * wave < nblk ? R0 + 2 * wave : nblk - 1;
    const int Rb = R0 + 2 * wave + 1 < nblk ? R0 + 2 * wave + 1 : nblk - 1;
    const int G1 = a.K1 / 128, G2 = EXT ? a.K2 / 128 : 0, GT = G1 + G2;
    constexpr bool W16 = FM == S_F16;                             // first segment's weights are fp16 tiles

    f4 acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int k = 0; k < 4; ++k) acc[i][k] = f4{0.f, 0.f, 0.f, 0.f};

    u4 xr[8];                                                     // prefetched x slab of the next step
    WReg wa, wb;                                                  // prefetched quantised tiles
    u4 fa[4], fb[4];                                              // prefetched fp16 tiles
    load_x(xr, a.x, a.ldx, a.M, m0, 0, tid);
    if constexpr (W16) {
        load_f16_tiles(fa, a.w, a.K1, Ra, 0, lane);
        load_f16_tiles(fb, a.w, a.K1, Rb, 0, lane);
    } else {
        load_wtile<FM>(wa, a, Ra, 0, lane);
        load_wtile<FM>(wb, a, Rb, 0, lane);
    }

    for (int s = 0; s < GT; ++s) {
        const bool seg2 = EXT && s >= G1;
        const bool cur16 = W16 || seg2;
        __syncthreads();                                          // everyone has finished reading the previous step
        store_x(xr, !cur16, tid);
        if (cur16) {
            store_f16_tiles(fa, 2 * wave, lane);
            store_f16_tiles(fb, 2 * wave + 1, lane);
        } else {
            if constexpr (!W16) {
                store_wtile<FM>(wa, 2 * wave, lane);
                store_wtile<FM>(wb, 2 * wave + 1, lane);
            }
        }
        __syncthreads();                                          // the step's operands are in LDS
        if (s + 1 < GT) {
            const bool n2 = EXT && s + 1 >= G1;
            if (n2) {
                load_x(xr, a.x2, a.ldx2, a.M, m0, (s + 1 - G1) * 128, tid);
                load_f16_tiles(fa, a.w2, a.K2, Ra, s + 1 - G1, lane);
                load_f16_tiles(fb, a.w2, a.K2, Rb, s + 1 - G1, lane);
            } else {
                load_x(xr, a.x, a.ldx, a.M, m0, (s + 1) * 128, tid);
                if constexpr (W16) {
                    load_f16_tiles(fa, a.w, a.K1, Ra, s + 1, lane);
                    load_f16_tiles(fb, a.w, a.K1, Rb, s + 1, lane);
                } else {
                    load_wtile<FM>(wa, a, Ra, s + 1, lane);
                    load_wtile<FM>(wb, a, Rb, s + 1, lane);
                }
            }
        }
        contract_step(acc, wm, wn, lane);
    }

    // ---- epilogue: fp32 -> fp16, transpose through LDS, 128-byte row stores ----------------------------
    __syncthreads();                                              // all fragment reads done: LDS is free
    constexpr int TS = 72;                                        // halves per token row in the staging tile (64 + pad)
    _Float16* tile = (_Float16*)eora_smem + wave * 64 * TS;
    const int n = lane & 15, j = lane >> 4;
#pragma unroll
    for (int mb = 0; mb < 4; ++mb)
#pragma unroll
        for (int rb = 0; rb < 4; ++rb)
#pragma unroll
            for (int i = 0; i < 4; ++i) tile[(16 * mb + 4 * j + i) * TS + 16 * rb + n] = (_Float16)acc[mb][rb][i];
    __syncthreads();
#pragma unroll
    for (int it = 0; it < 8; ++it) {
        const int tok = 8 * it + (lane >> 3), chunk = lane & 7;
        const int m = m0 + 64 * wm + tok, o = (R0 + 4 * wn) * 16 + chunk * 8;
        const u4 v = *(const u4*)(tile + tok * TS + chunk * 8);
        if (m < a.M && o < a.N) *(u4*)((_Float16*)a.y + (size_t)m * a.ldy + o) = v;
    }
}

template <int FM, bool EXT>
static hipError_t launch_pf(const PrefillArgs& a, hipStream_t stream)
{
    auto kern = prefill_kernel<FM, EXT>;
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, PF_LDS);
    if (e != hipSuccess) return e;
    const int ntn = (a.N + PF_BN - 1) / PF_BN, ntm = (a.M + PF_BM - 1) / PF_BM;
    hipLaunchKernelGGL(kern, dim3(ntn * ntm), dim3(256), PF_LDS, stream, a);
    return hipGetLastError();
}

hipError_t launch_prefill(const PrefillArgs& a, int fm, bool ext, hipStream_t stream)
{
    switch (fm) {
        case S_Q4: return ext ? launch_pf<S_Q4, true>(a, stream) : launch_pf<S_Q4, false>(a, stream);
        case S_Q3: return ext ? launch_pf<S_Q3, true>(a, stream) : launch_pf<S_Q3, false>(a, stream);
        case S_Q4S128: return ext ? hipErrorInvalidValue : launch_pf<S_Q4S128, false>(a, stream);
        case S_F16: return ext ? hipErrorInvalidValue : launch_pf<S_F16, false>(a, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace eora
