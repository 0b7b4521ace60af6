// The compensated compressed linear layer for up to 16 tokens per token block, in ONE launch:
//
//      y = x.What^T + (x.A^T).B^T          (Sec. 3 forward equation, Alg. 1 step 7)
//
// HBM-bound: every stored byte is read once, decoded in registers (tiles.hpp) and fed to
// 16x16x32 fp16 MFMAs whose 16-row operand is the token block (rows beyond M are zero).
//
// A workgroup of NW wavefronts owns a strip of RB row blocks (16 output rows each).  Its wavefronts
// split the contraction dimension tile by tile (consecutive wavefronts read consecutive tiles, so
// the workgroup streams one contiguous range), each keeps fp32 accumulators and the workgroup
// combines them through LDS in a fixed order; y is converted and stored once.
//
// The low-rank path is folded into the same launch and the same accumulators (the paper, Sec. 4.5
// and App. A.6, fuses only B's product and leaves x.A^T to a separate launch):
//   phase A  t = x.A^T is cut into units (16 rows of A) x (a range of k-tiles).  Workgroups draw
//            units from a ticket counter before they touch their strip, so every unit is owned by
//            a workgroup that is already running and never waits: no co-residency assumption.
//            The unit's partial goes to scratch; the last unit of a row block (arrival counter)
//            adds the partials in a fixed order, publishes its 16 columns of t and bumps `ready`.
//   phase W  backbone tiles of the strip (independent of t; hides phase A's latency).
//   phase B  wavefronts that own tiles of B wait (bounded spin) for `ready`, then continue the
//            contraction over B's tiles with t as the activation operand.  t stays fp32 in scratch
//            and is split into a high and a low fp16 part for the MFMA, so no precision is lost.
// The last workgroup to finish resets the counters, which therefore stay zero between launches.
#include "kernels.hpp"
#include "tiles.hpp"

namespace eora {

template <int FMT> struct Fmt;
template <> struct Fmt<S_Q4> { static constexpr int KT = 128, WORDS = 4; static constexpr bool ASYM = true; };
template <> struct Fmt<S_Q3> { static constexpr int KT = 128, WORDS = 3; static constexpr bool ASYM = true; };
template <> struct Fmt<S_Q4S128> { static constexpr int KT = 128, WORDS = 4; static constexpr bool ASYM = false; };
template <> struct Fmt<S_Q4S64> { static constexpr int KT = 64, WORDS = 2; static constexpr bool ASYM = false; };
template <> struct Fmt<S_F16> { static constexpr int KT = 32, WORDS = 4; static constexpr bool ASYM = false; };

struct Seg {
    const uint32_t* w;        // stored tiles
    const _Float16* scales;   // nullptr for F16
    const uint32_t* zeros;    // asymmetric formats only
    int ntk;                  // k-tiles per row block
    int NG;                   // quantisation groups per row (asymmetric formats)
    int gdiv;                 // k-tiles per quantisation group
};

struct __attribute__((packed, aligned(4))) Words3 { uint32_t a, b, c; };

// Registers of one pipeline step: the stored words of RB tiles (same k-tile, RB row blocks).
template <int FMT, int RB>
struct Step {
    uint32_t w[RB][Fmt<FMT>::WORDS];
    uint32_t zw[RB];
    _Float16 sc[RB];
};

template <int FMT, int RB>
__device__ __forceinline__ void load_step(Step<FMT, RB>& s, const Seg& seg, int R0, int g, int lane)
{
    constexpr int WORDS = Fmt<FMT>::WORDS;
    const int n = lane & 15;
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        const size_t tile = (size_t)(R0 + rb) * seg.ntk + g;
        const uint32_t* p = seg.w + (tile * 64 + lane) * WORDS;
        if constexpr (WORDS == 4) {
            const u4 v = *(const u4*)p;
            s.w[rb][0] = v[0]; s.w[rb][1] = v[1]; s.w[rb][2] = v[2]; s.w[rb][3] = v[3];
        } else if constexpr (WORDS == 3) {
            const Words3 v = *(const Words3*)p;
            s.w[rb][0] = v.a; s.w[rb][1] = v.b; s.w[rb][2] = v.c;
        } else {
            const uint2 v = *(const uint2*)p;
            s.w[rb][0] = v.x; s.w[rb][1] = v.y;
        }
        if constexpr (Fmt<FMT>::ASYM) {
            const size_t rq = (size_t)(R0 + rb) * seg.NG + (seg.gdiv == 1 ? g : g / seg.gdiv);
            s.zw[rb] = seg.zeros[2 * rq + (n >> 3)];
            s.sc[rb] = seg.scales[rq * 16 + n];
        } else if constexpr (FMT != S_F16) {
            s.sc[rb] = seg.scales[tile * 16 + n];
        }
    }
}

// fp16 activation fragments of k-tile g for the lane's token row (zero for rows beyond M)
template <int FMT>
__device__ __forceinline__ void load_act(h8 (&xa)[Fmt<FMT>::KT / 32], int g, int lane,
                                         const _Float16* __restrict__ x, int ldx, int m, bool row_ok)
{
    constexpr int KT = Fmt<FMT>::KT, NMF = KT / 32;
    const int j = lane >> 4;
#pragma unroll
    for (int t = 0; t < NMF; ++t) {
        Frag f;
        f.q = u4{0u, 0u, 0u, 0u};
        xa[t] = f.v;
    }
    if (row_ok) {
        const _Float16* px = x + (size_t)m * ldx + g * KT + (KT / 4) * j;
#pragma unroll
        for (int t = 0; t < NMF; ++t) xa[t] = *(const h8*)(px + 8 * t);
    }
}

// decode one tile's words into MFMA fragments and its scale
template <int FMT>
__device__ __forceinline__ float decode_tile(const uint32_t (&w)[Fmt<FMT>::WORDS], uint32_t zw, _Float16 sc, int n,
                                             h8 (&b)[Fmt<FMT>::KT / 32])
{
    constexpr int NMF = Fmt<FMT>::KT / 32;
    if constexpr (FMT == S_F16) {
        Frag f;
        f.u[0] = w[0]; f.u[1] = w[1]; f.u[2] = w[2]; f.u[3] = w[3];
        b[0] = f.v;
        return 1.0f;
    } else if constexpr (FMT == S_Q3) {
        const uint32_t z = (zw >> (4 * (n & 7))) & 0xFu;
        dq3_lane(w[0], w[1], w[2], z, b);
        return (float)sc;
    } else {
        uint32_t z = 8u;
        if constexpr (FMT == S_Q4) z = (zw >> (4 * (n & 7))) & 0xFu;
        const uint32_t c1024 = k1024(z), c64 = k64(z);
#pragma unroll
        for (int t = 0; t < NMF; ++t) b[t] = dq4_word(w[t], c1024, c64);
        return (float)sc;
    }
}

template <int FMT, int RB>
__device__ __forceinline__ void compute_step(const Step<FMT, RB>& s, const h8 (&xa)[Fmt<FMT>::KT / 32], f4 (&acc)[RB],
                                             int lane)
{
    constexpr int NMF = Fmt<FMT>::KT / 32;
    const int n = lane & 15;
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        h8 b[NMF];
        const float sc = decode_tile<FMT>(s.w[rb], s.zw[rb], s.sc[rb], n, b);
        if constexpr (FMT == S_F16) {
            acc[rb] = mfma16(xa[0], b[0], acc[rb]);
        } else {
            f4 part = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int t = 0; t < NMF; ++t) part = mfma16(xa[t], b[t], part);
            acc[rb] += sc * part;        // exact integers times x, scaled once per group in fp32
        }
    }
}

// Contraction over k-tiles g_begin + wave, + NW, ... < g_end.  PD (even) steps of weight loads are
// kept in flight (they come from HBM); the activation fragments (L1 / L2 hits) run one step ahead.
template <int FMT, int RB, int NW, int PD>
__device__ __forceinline__ void run_tiles(f4 (&acc)[RB], const Seg& seg, int R0, int g_begin, int g_end, int wave,
                                          int lane, const _Float16* __restrict__ x, int ldx, int m, bool row_ok)
{
    static_assert(PD % 2 == 0, "pipeline depth must be even (activation fragments ping-pong)");
    constexpr int NMF = Fmt<FMT>::KT / 32;
    Step<FMT, RB> buf[PD];
    h8 xa[2][NMF];
    const int first = g_begin + wave;
    const int nsteps = first < g_end ? (g_end - first + NW - 1) / NW : 0;
#pragma unroll
    for (int u = 0; u < PD; ++u)
        if (u < nsteps) load_step<FMT, RB>(buf[u], seg, R0, first + u * NW, lane);
    if (nsteps > 0) load_act<FMT>(xa[0], first, lane, x, ldx, m, row_ok);
    for (int base = 0; base < nsteps; base += PD) {
#pragma unroll
        for (int u = 0; u < PD; ++u) {
            const int s = base + u;
            if (s < nsteps) {
                const Step<FMT, RB> cur = buf[u];
                if (s + 1 < nsteps) load_act<FMT>(xa[(u + 1) & 1], first + (s + 1) * NW, lane, x, ldx, m, row_ok);
                if (s + PD < nsteps) load_step<FMT, RB>(buf[u], seg, R0, first + (s + PD) * NW, lane);
                compute_step<FMT, RB>(cur, xa[u & 1], acc, lane);
            }
        }
    }
}

// Extension over B's tiles with the fp32 activation t split into high and low fp16 parts.
template <int FMT, int RB, int NW>
__device__ __forceinline__ void run_ext(f4 (&acc)[RB], const Seg& seg, int R0, int wave, int lane,
                                        const float* __restrict__ t, int ldt, int m, bool row_ok)
{
    constexpr int KT = Fmt<FMT>::KT, WORDS = Fmt<FMT>::WORDS, NMF = KT / 32;
    const int n = lane & 15, j = lane >> 4;
    for (int g = wave; g < seg.ntk; g += NW) {
        h8 hi[NMF], lo[NMF];
#pragma unroll
        for (int q = 0; q < NMF; ++q) {
            float v[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) v[i] = 0.f;
            if (row_ok) {
                const float* p = t + (size_t)m * ldt + g * KT + (KT / 4) * j + 8 * q;
                const f4 a = *(const f4*)p, b = *(const f4*)(p + 4);
#pragma unroll
                for (int i = 0; i < 4; ++i) { v[i] = a[i]; v[4 + i] = b[i]; }
            }
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const _Float16 h = (_Float16)v[i];
                hi[q][i] = h;
                lo[q][i] = (_Float16)(v[i] - (float)h);
            }
        }
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) {
            const size_t tile = (size_t)(R0 + rb) * seg.ntk + g;
            const uint32_t* p = seg.w + (tile * 64 + lane) * WORDS;
            uint32_t w[WORDS];
#pragma unroll
            for (int i = 0; i < WORDS; ++i) w[i] = p[i];
            _Float16 sc = (_Float16)1.0f;
            if constexpr (FMT != S_F16) sc = seg.scales[tile * 16 + n];
            h8 b[NMF];
            const float scf = decode_tile<FMT>(w, 0u, sc, n, b);
            f4 part = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int q = 0; q < NMF; ++q) {
                part = mfma16(hi[q], b[q], part);
                part = mfma16(lo[q], b[q], part);
            }
            acc[rb] += scf * part;
        }
    }
}

__device__ __forceinline__ uint32_t ld_relaxed(const uint32_t* p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// grid: x = strips of 16*RB output rows, y = token blocks of 16.  NW*64 threads.
template <int FM, int FA, int FE, int RB, int NW>
__global__ __launch_bounds__(NW * 64) void fused_kernel(FusedArgs a)
{
    __shared__ f4 red[NW - 1][RB][64];
    __shared__ uint32_t s_word;

    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int n = lane & 15, j = lane >> 4;
    const int yb = blockIdx.y;
    const int m = 16 * yb + n;              // token row this lane feeds as the activation operand
    const bool row_ok = m < a.M;
    uint32_t* ctr = a.hdr + HDR_BLOCK0 + HDR_PER_BLOCK * yb;   // [0] ticket, [1] ready, [2..] arrivals

    // ---------------------------------------------------------------- phase A: t = x.A^T
    if constexpr (FA != S_NONE) {
        constexpr int KTA = Fmt<FA>::KT;
        const int NRB = a.r / 16;
        const int units = NRB * a.kcn;
        const Seg sa{(const uint32_t*)a.A, a.A_scales, nullptr, a.d_in / KTA, 0, 1};
        const int tiles_per_chunk = sa.ntk / a.kcn;
        for (;;) {
            if (threadIdx.x == 0) s_word = atomicAdd(&ctr[0], 1u);
            __syncthreads();
            const uint32_t u = s_word;
            __syncthreads();
            if (u >= (uint32_t)units) break;
            const int rho = u % NRB, kc = u / NRB;
            f4 part[1] = {f4{0.f, 0.f, 0.f, 0.f}};
            run_tiles<FA, 1, NW, 4>(part, sa, rho, kc * tiles_per_chunk, (kc + 1) * tiles_per_chunk, wave, lane,
                                    a.x, a.d_in, m, row_ok);
            if (wave > 0) red[wave - 1][0][lane] = part[0];
            __syncthreads();
            float* slot = a.tpart + (((size_t)kc * NRB + rho) * gridDim.y + yb) * 256;
            if (wave == 0) {
                f4 v = part[0];
#pragma unroll
                for (int w2 = 0; w2 < NW - 1; ++w2) v += red[w2][0][lane];
                *(f4*)(slot + 4 * lane) = v;
                __threadfence();                                   // release the partial
            }
            __syncthreads();
            if (threadIdx.x == 0) s_word = atomicAdd(&ctr[2 + rho], 1u);
            __syncthreads();
            const bool last = s_word == (uint32_t)(a.kcn - 1);
            __syncthreads();
            if (last) {
                if (wave == 0) {
                    __threadfence();                               // acquire the other units' partials
                    f4 v = {0.f, 0.f, 0.f, 0.f};
                    for (int k2 = 0; k2 < a.kcn; ++k2)
                        v += *(const f4*)(a.tpart + (((size_t)k2 * NRB + rho) * gridDim.y + yb) * 256 + 4 * lane);
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const int mm = 16 * yb + 4 * j + i;        // accumulator register i is token row 4*j+i
                        if (mm < a.M) a.t[(size_t)mm * a.r + 16 * rho + n] = v[i];
                    }
                    __threadfence();                               // release t
                    if (lane == 0) atomicAdd(&ctr[1], 1u);
                }
            }
        }
    }

    // ---------------------------------------------------------------- phase W: backbone
    const int R0 = blockIdx.x * RB;
    f4 acc[RB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) acc[rb] = f4{0.f, 0.f, 0.f, 0.f};
    {
        const int NG = a.d_in / a.group;
        const Seg sw{(const uint32_t*)a.w, a.w_scales, a.w_zeros, a.d_in / 128, NG, a.group / 128};
        run_tiles<FM, RB, NW, (RB == 1 ? 4 : 2)>(acc, sw, R0, 0, sw.ntk, wave, lane, a.x, a.d_in, m, row_ok);
    }

    // ---------------------------------------------------------------- phase B: += t.B^T
    if constexpr (FE != S_NONE) {
        const Seg sb{(const uint32_t*)a.B, a.B_scales, nullptr, a.r / Fmt<FE>::KT, 0, 1};
        if (wave < sb.ntk) {
            const uint32_t need = a.r / 16;
            int spins = 0;
            bool ok = true;
            while (ld_relaxed(&ctr[1]) < need) {
                __builtin_amdgcn_s_sleep(8);
                if (++spins > a.spin_limit) { ok = false; break; }
            }
            if (ok) {
                __threadfence();                                   // acquire t
                run_ext<FE, RB, NW>(acc, sb, R0, wave, lane, a.t, a.r, m, row_ok);
            } else if (lane == 0) {
                atomicOr(&a.hdr[HDR_ERROR], 1u);                   // never expected: owners of units do not wait
            }
        }
    }

    // ---------------------------------------------------------------- combine, convert, store
    if (wave > 0) {
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) red[wave - 1][rb][lane] = acc[rb];
    }
    __syncthreads();
    if (wave == 0) {
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) {
            f4 v = acc[rb];
#pragma unroll
            for (int w2 = 0; w2 < NW - 1; ++w2) v += red[w2][rb][lane];
            const int o = (R0 + rb) * 16 + n;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int mm = 16 * yb + 4 * j + i;
                if (mm < a.M) a.y[(size_t)mm * a.d_out + o] = (_Float16)v[i];
            }
        }
    }

    // ---------------------------------------------------------------- last workgroup clears the counters
    if constexpr (FA != S_NONE) {
        __syncthreads();
        if (threadIdx.x == 0) s_word = atomicAdd(&a.hdr[HDR_EXIT], 1u);
        __syncthreads();
        if (s_word == gridDim.x * gridDim.y - 1) {
            for (int i = threadIdx.x; i < (int)(HDR_PER_BLOCK * gridDim.y); i += NW * 64) a.hdr[HDR_BLOCK0 + i] = 0u;
            if (threadIdx.x == 0) a.hdr[HDR_EXIT] = 0u;
        }
    }
}

// ------------------------------------------------------------------------------------------------
template <int FM, int FA, int FE, int RB, int NW>
static hipError_t launch_one(const FusedArgs& a, dim3 grid, hipStream_t stream)
{
    hipLaunchKernelGGL((fused_kernel<FM, FA, FE, RB, NW>), grid, dim3(NW * 64), 0, stream, a);
    return hipGetLastError();
}

template <int FM, int FA, int FE>
static hipError_t launch_cfg(const FusedArgs& a, hipStream_t stream)
{
    const int nblk = a.d_out / 16;
    const int G = a.d_in / 128;
    const int yblocks = (a.M + 15) / 16;
    // Few tokens: one row block per workgroup, most workgroups.  More tokens: strips of 4 (or 2) row
    // blocks so the activation fragments are reused, as long as enough workgroups remain.
    int rb = 1;
    if (a.M > 4) {
        if (nblk % 4 == 0 && nblk / 4 >= 256) rb = 4;
        else if (nblk % 2 == 0 && nblk / 2 >= 256) rb = 2;
    }
    // Wavefronts per workgroup: enough k-tiles per wavefront to pipeline, enough wavefronts to fill the chip.
    const int nw = (rb == 1 && G >= 64 && nblk <= 512) ? 16 : 8;
    const dim3 grid(nblk / rb, yblocks);
    if (rb == 4) return launch_one<FM, FA, FE, 4, 8>(a, grid, stream);
    if (rb == 2) return launch_one<FM, FA, FE, 2, 8>(a, grid, stream);
    if (nw == 16) return launch_one<FM, FA, FE, 1, 16>(a, grid, stream);
    return launch_one<FM, FA, FE, 1, 8>(a, grid, stream);
}

template <int FM>
static hipError_t launch_ab(const FusedArgs& a, int fa, int fe, hipStream_t stream)
{
    if (fe == S_NONE) return launch_cfg<FM, S_NONE, S_NONE>(a, stream);
    if (fa == S_F16 && fe == S_F16) return launch_cfg<FM, S_F16, S_F16>(a, stream);
    if (fa == S_Q4S128 && fe == S_Q4S128) return launch_cfg<FM, S_Q4S128, S_Q4S128>(a, stream);
    if (fa == S_Q4S128 && fe == S_Q4S64) return launch_cfg<FM, S_Q4S128, S_Q4S64>(a, stream);
    return hipErrorInvalidValue;
}

hipError_t launch_fused(const FusedArgs& a, int fm, int fa, int fe, hipStream_t stream)
{
    switch (fm) {
        case S_Q4: return launch_ab<S_Q4>(a, fa, fe, stream);
        case S_Q3: return launch_ab<S_Q3>(a, fa, fe, stream);
        default: return hipErrorInvalidValue;
    }
}

__global__ void clear_words_kernel(uint32_t* p, int nwords)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < nwords) p[i] = 0u;
}

hipError_t launch_clear_words(uint32_t* p, int nwords, hipStream_t stream)
{
    hipLaunchKernelGGL(clear_words_kernel, dim3((nwords + 255) / 256), dim3(256), 0, stream, p, nwords);
    return hipGetLastError();
}

}  // namespace eora
