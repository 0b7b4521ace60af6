// The compensated compressed linear layer for up to 16 tokens per token block, in ONE launch:
//
//      y = x.What^T + (x.A^T).B^T          (Sec. 3 forward equation, Alg. 1 step 7)
//
// HBM-bound: every stored byte is read once, decoded in registers (tiles.hpp) and fed to
// 16x16x32 fp16 MFMAs whose 16-row operand is the token block (rows beyond M are zero).
//
// A workgroup of NW wavefronts owns a strip of RB row blocks (16 output rows each).  Its wavefronts
// split the contraction dimension in quads of four consecutive 128-wide k-tiles (one 8-byte load
// brings the four group scales of a row, one word its four zero-points), keep fp32 accumulators
// and combine them through LDS in a fixed order; y is converted and stored once.  Everything a
// wavefront will need is requested up front, small operands first (x, scales, zero-points), then
// the weight tiles, so that the tiles can be consumed in arrival order.  For few tokens x is staged
// once per workgroup in LDS; the activation fragments of a tile are then LDS reads instead of
// global loads that would queue behind the weight stream.
//
// The low-rank path is folded into the same launch and the same accumulators (the paper, Sec. 4.5
// and App. A.6, fuses only B's product and leaves x.A^T to a separate launch):
//   phase A  t = x.A^T is cut into units (16 rows of A) x (one of kcn ranges of k-tiles).  Unit u
//            belongs to workgroup u (workgroups are dispatched in index order, and an owner runs its
//            units before anything else and never waits, so no owner can be starved by a waiter).
//            The owner writes its fp32 partial to scratch and then publishes flag[u] = epoch + 1.
//   phase W  backbone tiles of the strip (independent of t; hides phase A's latency).
//   phase B  one wavefront polls the flags (bounded), then the wavefronts that own tiles of B add
//            the kcn partials in a fixed order to get their slice of t (fp32), split it into a high
//            and a low fp16 part and continue the contraction over B's tiles.
// Nothing is reset between launches: flags are compared with epoch + 1 and the epoch word is
// advanced once per launch, by the last workgroup to check in on a spread-out arrival counter
// (every workgroup reads the epoch before it checks in).
#include "kernels.hpp"
#include "tiles.hpp"

namespace eora {

template <int FMT> struct Fmt;
template <> struct Fmt<S_Q4> { static constexpr int KT = 128, WORDS = 4; static constexpr bool ASYM = true; };
template <> struct Fmt<S_Q3> { static constexpr int KT = 128, WORDS = 3; static constexpr bool ASYM = true; };
template <> struct Fmt<S_Q4S128> { static constexpr int KT = 128, WORDS = 4; static constexpr bool ASYM = false; };
template <> struct Fmt<S_Q4S64> { static constexpr int KT = 64, WORDS = 2; static constexpr bool ASYM = false; };
template <> struct Fmt<S_F16> { static constexpr int KT = 32, WORDS = 4; static constexpr bool ASYM = false; };

struct __attribute__((packed, aligned(4))) Words3 { uint32_t a, b, c; };

template <int WORDS>
__device__ __forceinline__ void load_words(uint32_t (&w)[WORDS], const uint32_t* __restrict__ p)
{
    if constexpr (WORDS == 4) {
        const u4 v = *(const u4*)p;
        w[0] = v[0]; w[1] = v[1]; w[2] = v[2]; w[3] = v[3];
    } else if constexpr (WORDS == 3) {
        const Words3 v = *(const Words3*)p;
        w[0] = v.a; w[1] = v.b; w[2] = v.c;
    } else {
        const uint2 v = *(const uint2*)p;
        w[0] = v.x; w[1] = v.y;
    }
}

// Where the activation fragments come from: LDS (x staged by the workgroup) or global memory.
// Both pointers are kept with their own address space so that the loads are ds_read / global_load
// and never flat.
template <bool XLDS>
struct ActSrc {
    const _Float16* g;        // global: token block's first row
    int ldg;
    int lds_off;              // LDS: byte offset of the staged block inside the dynamic LDS
    int lds_ld;               // LDS row stride in halves
};

extern __shared__ __attribute__((aligned(16))) unsigned char eora_smem[];

template <int NMF, bool XLDS>
__device__ __forceinline__ void load_act(h8 (&xa)[NMF], const ActSrc<XLDS>& src, int col, int m, bool row_ok)
{
#pragma unroll
    for (int t = 0; t < NMF; ++t) {
        Frag f;
        f.q = u4{0u, 0u, 0u, 0u};
        xa[t] = f.v;
    }
    if (row_ok) {
        if constexpr (XLDS) {
            const _Float16* px = (const _Float16*)(eora_smem + src.lds_off) + m * src.lds_ld + col;
#pragma unroll
            for (int t = 0; t < NMF; ++t) xa[t] = *(const h8*)(px + 8 * t);
        } else {
            const _Float16* px = src.g + (size_t)m * src.ldg + col;
#pragma unroll
            for (int t = 0; t < NMF; ++t) xa[t] = *(const h8*)(px + 8 * t);
        }
    }
}

// decode one tile's words into MFMA fragments
template <int FMT>
__device__ __forceinline__ void decode_tile(const uint32_t (&w)[Fmt<FMT>::WORDS], uint32_t z, h8 (&b)[Fmt<FMT>::KT / 32])
{
    constexpr int NMF = Fmt<FMT>::KT / 32;
    if constexpr (FMT == S_F16) {
        Frag f;
        f.u[0] = w[0]; f.u[1] = w[1]; f.u[2] = w[2]; f.u[3] = w[3];
        b[0] = f.v;
    } else if constexpr (FMT == S_Q3) {
        dq3_lane(w[0], w[1], w[2], z, b);
    } else {
        const uint32_t c1024 = k1024(z), c64 = k64(z);
#pragma unroll
        for (int t = 0; t < NMF; ++t) b[t] = dq4_word(w[t], c1024, c64);
    }
}

// ------------------------------------------------------------------------------------------------
// Backbone: quads of four consecutive k-tiles, RB row blocks each.
template <int FMT, int RB>
struct Quad {
    uint32_t w[RB][4][Fmt<FMT>::WORDS];
    uint2 sc[RB];       // four fp16 scales (tiles 4q .. 4q+3) of the lane's row
    uint32_t zq[RB];    // their four zero-points, one nibble each
};

struct Backbone {
    const uint32_t* w;
    const _Float16* scales;   // row-major d_out x NG
    const uint32_t* zeros;    // row-major d_out x NGW words, nibble g%8 of word g/8
    int G, NG, NGW, gdiv;
};

template <int FMT, int RB>
__device__ __forceinline__ void load_quad_meta(Quad<FMT, RB>& s, const Backbone& bb, int R0, int q, int lane)
{
    const int n = lane & 15, g0 = 4 * q;
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        const size_t row = (size_t)(R0 + rb) * 16 + n;
        if (bb.gdiv == 1 && (bb.NG & 3) == 0 && g0 + 3 < bb.G) {      // 8-byte aligned: NG and g0 are multiples of 4
            s.sc[rb] = *(const uint2*)(bb.scales + row * bb.NG + g0);
            s.zq[rb] = (bb.zeros[row * bb.NGW + (g0 >> 3)] >> (4 * (g0 & 7))) & 0xFFFFu;
        } else {                                  // coarser groups or a ragged last quad: element by element
            uint32_t sw[4] = {0u, 0u, 0u, 0u}, zq = 0u;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int g = g0 + i;
                if (g < bb.G) {
                    const int grp = g / bb.gdiv;
                    sw[i] = __builtin_bit_cast(uint16_t, bb.scales[row * bb.NG + grp]);
                    zq |= ((bb.zeros[row * bb.NGW + (grp >> 3)] >> (4 * (grp & 7))) & 0xFu) << (4 * i);
                }
            }
            s.sc[rb] = uint2{sw[0] | (sw[1] << 16), sw[2] | (sw[3] << 16)};
            s.zq[rb] = zq;
        }
    }
}

template <int FMT, int RB>
__device__ __forceinline__ void load_quad_words(Quad<FMT, RB>& s, const Backbone& bb, int R0, int q, int lane)
{
    constexpr int WORDS = Fmt<FMT>::WORDS;
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int g = 4 * q + i;
            if (g < bb.G) {
                const size_t tile = (size_t)(R0 + rb) * bb.G + g;
                load_words<WORDS>(s.w[rb][i], bb.w + (tile * 64 + lane) * WORDS);
            } else {
#pragma unroll
                for (int k = 0; k < WORDS; ++k) s.w[rb][i][k] = 0u;
            }
        }
    }
}

template <int FMT, int RB, bool XLDS>
__device__ __forceinline__ void compute_quad(const Quad<FMT, RB>& s, const Backbone& bb, int q, f4 (&acc)[RB],
                                             const ActSrc<XLDS>& act, int lane, int m, bool row_ok)
{
    const int j = lane >> 4;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int g = 4 * q + i;
        if (g < bb.G) {
            h8 xa[4];
            load_act<4, XLDS>(xa, act, g * 128 + 32 * j, m, row_ok);
#pragma unroll
            for (int rb = 0; rb < RB; ++rb) {
                h8 b[4];
                decode_tile<FMT>(s.w[rb][i], (s.zq[rb] >> (4 * i)) & 0xFu, b);
                f4 part = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int t = 0; t < 4; ++t) part = mfma16(xa[t], b[t], part);
                const uint32_t sw = (i < 2) ? s.sc[rb].x : s.sc[rb].y;
                const _Float16 sc = __builtin_bit_cast(_Float16, (uint16_t)((i & 1) ? (sw >> 16) : (sw & 0xFFFFu)));
                acc[rb] += (float)sc * part;     // exact integers times x, scaled once per group in fp32
            }
        }
    }
}

// ------------------------------------------------------------------------------------------------
// Factor tiles (A in phase A with x, B in phase B with t): plain per-tile steps.
struct Factor {
    const uint32_t* w;
    const _Float16* scales;   // row-major rows x ntk (4-bit factors), nullptr for fp16
    int ntk;                  // k-tiles per row block
};

template <int FMT>
struct FTile {
    uint32_t w[Fmt<FMT>::WORDS];
    _Float16 sc;
};

template <int FMT>
__device__ __forceinline__ void load_ftile(FTile<FMT>& s, const Factor& f, int R, int g, int lane)
{
    constexpr int WORDS = Fmt<FMT>::WORDS;
    if constexpr (FMT != S_F16) s.sc = f.scales[((size_t)R * 16 + (lane & 15)) * f.ntk + g];
    else s.sc = (_Float16)1.0f;
    const size_t tile = (size_t)R * f.ntk + g;
    load_words<WORDS>(s.w, f.w + (tile * 64 + lane) * WORDS);
}

// phase A: partial of t over k-tiles g_begin + wave, + NW, ... < g_end of row block R of A
template <int FMT, int NW, bool XLDS>
__device__ __forceinline__ f4 run_factor_a(const Factor& f, int R, int g_begin, int g_end, int wave, int lane,
                                           const ActSrc<XLDS>& act, int m, bool row_ok)
{
    constexpr int KT = Fmt<FMT>::KT, NMF = KT / 32, PD = 4;
    const int j = lane >> 4;
    FTile<FMT> buf[PD];
    const int first = g_begin + wave;
    const int nsteps = first < g_end ? (g_end - first + NW - 1) / NW : 0;
#pragma unroll
    for (int u = 0; u < PD; ++u)
        if (u < nsteps) load_ftile<FMT>(buf[u], f, R, first + u * NW, lane);
    f4 acc = {0.f, 0.f, 0.f, 0.f};
    for (int base = 0; base < nsteps; base += PD) {
#pragma unroll
        for (int u = 0; u < PD; ++u) {
            const int s = base + u;
            if (s < nsteps) {
                const FTile<FMT> cur = buf[u];
                const int g = first + s * NW;
                if (s + PD < nsteps) load_ftile<FMT>(buf[u], f, R, first + (s + PD) * NW, lane);
                h8 xa[NMF], b[NMF];
                load_act<NMF, XLDS>(xa, act, g * KT + (KT / 4) * j, m, row_ok);
                decode_tile<FMT>(cur.w, 8u, b);
                if constexpr (FMT == S_F16) {
                    acc = mfma16(xa[0], b[0], acc);
                } else {
                    f4 part = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int t = 0; t < NMF; ++t) part = mfma16(xa[t], b[t], part);
                    acc += (float)cur.sc * part;
                }
            }
        }
    }
    return acc;
}

__device__ __forceinline__ uint32_t ld_relaxed(const uint32_t* p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// grid: x = strips of 16*RB output rows, y = token blocks of 16.  NW*64 threads.
// XLDS: x of this token block is staged in dynamic LDS (row stride d_in + 32 halves).
template <int FM, int FA, int FE, int RB, int NW, bool XLDS>
__global__ __launch_bounds__(NW * 64) void fused_kernel(FusedArgs a)
{
    __shared__ f4 red[NW - 1][RB][64];
    __shared__ uint32_t s_epoch, s_ok;

    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int n = lane & 15, j = lane >> 4;
    const int yb = blockIdx.y;
    const int m_blk = 16 * yb;               // first token of this block
    const int mt = a.M - m_blk < 16 ? a.M - m_blk : 16;      // tokens in this block
    const bool row_ok = n < mt;              // lane feeds token row n of the block as the activation operand
    const int R0 = blockIdx.x * RB;
    constexpr bool LOWRANK = FA != S_NONE;

    // ---- requests, small operands first ------------------------------------------------------
    const int ldxs = a.d_in + 32;            // LDS row stride (halves): 64 bytes of padding against bank conflicts
    _Float16* xs = (_Float16*)eora_smem;
    u4 xstage[XLDS ? 4 : 1];
    const int xchunks = (a.d_in / 8);        // 16-byte chunks per token row
    if constexpr (XLDS) {
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int c = threadIdx.x + k * NW * 64;
            if (c < mt * xchunks) xstage[k] = *((const u4*)(a.x + (size_t)(m_blk + c / xchunks) * a.d_in) + c % xchunks);
        }
    }
    uint32_t epoch = 0;
    if constexpr (LOWRANK) {
        if (threadIdx.x == 0) {
            epoch = __hip_atomic_load(&a.hdr[HDR_EPOCH], __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_AGENT);
            s_epoch = epoch;
        }
    }

    const Backbone bb{(const uint32_t*)a.w, a.w_scales, a.w_zeros, a.d_in / 128, a.d_in / a.group,
                      (a.d_in / a.group + 7) / 8, a.group / 128};
    const int Q = (bb.G + 3) / 4;
    constexpr int PDQ = RB == 1 ? 2 : 1;     // quads of weight loads in flight per wavefront
    Quad<FM, RB> qbuf[PDQ];
    const int nq = wave < Q ? (Q - wave + NW - 1) / NW : 0;
#pragma unroll
    for (int u = 0; u < PDQ; ++u)
        if (u < nq) load_quad_meta<FM, RB>(qbuf[u], bb, R0, wave + u * NW, lane);

    // first tile of B for this wavefront (its words do not depend on t)
    const Factor fb{(const uint32_t*)a.B, a.B_scales, LOWRANK ? a.r / Fmt<LOWRANK ? FE : S_F16>::KT : 0};
    FTile<LOWRANK ? FE : S_F16> bpre[RB];
    if constexpr (LOWRANK) {
        if (wave < fb.ntk) {
#pragma unroll
            for (int rb = 0; rb < RB; ++rb) load_ftile<FE>(bpre[rb], fb, R0 + rb, wave, lane);
        }
    }
#pragma unroll
    for (int u = 0; u < PDQ; ++u)
        if (u < nq) load_quad_words<FM, RB>(qbuf[u], bb, R0, wave + u * NW, lane);

    // ---- check in (the last workgroup to do so advances the epoch) --------------------------------
    if constexpr (LOWRANK) {
        if (threadIdx.x == 0) {
            const uint32_t total = gridDim.x * gridDim.y;
            const uint32_t lin = blockIdx.y * gridDim.x + blockIdx.x;
            const uint32_t k = lin % HDR_NSUB;
            const uint32_t quota = (total - k + HDR_NSUB - 1) / HDR_NSUB;
            if (atomicAdd(&a.hdr[HDR_SUB0 + HDR_SUB_STRIDE * k], 1u) == quota - 1) {
                a.hdr[HDR_SUB0 + HDR_SUB_STRIDE * k] = 0u;
                const uint32_t nsub = total < HDR_NSUB ? total : HDR_NSUB;
                if (atomicAdd(&a.hdr[HDR_TOP], 1u) == nsub - 1) {
                    a.hdr[HDR_TOP] = 0u;
                    a.hdr[HDR_EPOCH] = epoch + 1;       // every workgroup has read the epoch by now
                }
            }
        }
    }

    // ---- stage x ----------------------------------------------------------------------------------
    const ActSrc<XLDS> act{a.x + (size_t)m_blk * a.d_in, a.d_in, 0, ldxs};
    if constexpr (XLDS) {
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int c = threadIdx.x + k * NW * 64;
            if (c < mt * xchunks) *(u4*)(xs + (size_t)(c / xchunks) * ldxs + (c % xchunks) * 8) = xstage[k];
        }
    }
    __syncthreads();
    if constexpr (LOWRANK) epoch = s_epoch;

    // ---- phase A: this workgroup's units of t = x.A^T ---------------------------------------------
    if constexpr (LOWRANK) {
        constexpr int KTA = Fmt<FA>::KT;
        const int NRB = a.r / 16;
        const int units = NRB * a.kcn;
        const Factor fa{(const uint32_t*)a.A, a.A_scales, a.d_in / KTA};
        const int tiles_per_chunk = fa.ntk / a.kcn;
        uint32_t* flags = a.hdr + HDR_FLAGS0 + HDR_FLAGS_PER_BLOCK * yb;
        for (int u = blockIdx.x; u < units; u += gridDim.x) {
            const int rho = u % NRB, kc = u / NRB;
            const f4 part = run_factor_a<FA, NW, XLDS>(fa, rho, kc * tiles_per_chunk, (kc + 1) * tiles_per_chunk, wave, lane,
                                                 act, n, row_ok);
            if (wave > 0) red[wave - 1][0][lane] = part;
            __syncthreads();
            if (wave == 0) {
                f4 v = part;
#pragma unroll
                for (int w2 = 0; w2 < NW - 1; ++w2) v += red[w2][0][lane];
                // partial layout: [token block][kc][token row][r]; register i is token row 4*j+i, column n
                float* dst = a.tpart + ((size_t)(yb * a.kcn + kc) * 16) * a.r + 16 * rho + n;
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    if (4 * j + i < mt) dst[(size_t)(4 * j + i) * a.r] = v[i];
                __threadfence();                                   // release the partial
                if (lane == 0) __hip_atomic_store(&flags[u], epoch + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
            __syncthreads();
        }
    }

    // ---- phase W: backbone -----------------------------------------------------------------------
    f4 acc[RB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) acc[rb] = f4{0.f, 0.f, 0.f, 0.f};
    for (int base = 0; base < nq; base += PDQ) {
#pragma unroll
        for (int u = 0; u < PDQ; ++u) {
            const int s = base + u;
            if (s < nq) {
                const Quad<FM, RB> cur = qbuf[u];
                const int q = wave + s * NW;
                if (s + PDQ < nq) {
                    load_quad_meta<FM, RB>(qbuf[u], bb, R0, wave + (s + PDQ) * NW, lane);
                    load_quad_words<FM, RB>(qbuf[u], bb, R0, wave + (s + PDQ) * NW, lane);
                }
                compute_quad<FM, RB, XLDS>(cur, bb, q, acc, act, lane, n, row_ok);
            }
        }
    }

    // ---- phase B: += t.B^T -----------------------------------------------------------------------
    if constexpr (LOWRANK) {
        const int units = (a.r / 16) * a.kcn;
        const uint32_t* flags = a.hdr + HDR_FLAGS0 + HDR_FLAGS_PER_BLOCK * yb;
        if (wave == 0) {
            bool ok = false;
            for (int spins = 0; spins <= a.spin_limit; ++spins) {
                bool all = true;
                for (int f = lane; f < units; f += 64) all = all && (ld_relaxed(&flags[f]) == epoch + 1);
                if (__all(all)) { ok = true; break; }
                __builtin_amdgcn_s_sleep(4);
            }
            if (lane == 0) {
                s_ok = ok ? 1u : 0u;
                if (!ok) atomicOr(&a.hdr[HDR_ERROR], 1u);          // never expected: owners of units do not wait
            }
        }
        __syncthreads();
        if (s_ok && wave < fb.ntk) {
            __threadfence();                                       // acquire the partials
            constexpr int KTB = Fmt<FE>::KT, NMF = KTB / 32;
            for (int g = wave; g < fb.ntk; g += NW) {
                h8 hi[NMF], lo[NMF];
#pragma unroll
                for (int q = 0; q < NMF; ++q) {
                    f4 v0 = {0.f, 0.f, 0.f, 0.f}, v1 = {0.f, 0.f, 0.f, 0.f};
                    if (row_ok) {
                        const float* p = a.tpart + ((size_t)(yb * a.kcn) * 16 + n) * a.r + g * KTB + (KTB / 4) * j + 8 * q;
                        for (int kc = 0; kc < a.kcn; ++kc) {       // fixed order: the result does not depend on timing
                            v0 += *(const f4*)(p + (size_t)kc * 16 * a.r);
                            v1 += *(const f4*)(p + (size_t)kc * 16 * a.r + 4);
                        }
                    }
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const _Float16 h0 = (_Float16)v0[i], h1 = (_Float16)v1[i];
                        hi[q][i] = h0;
                        hi[q][4 + i] = h1;
                        lo[q][i] = (_Float16)(v0[i] - (float)h0);
                        lo[q][4 + i] = (_Float16)(v1[i] - (float)h1);
                    }
                }
#pragma unroll
                for (int rb = 0; rb < RB; ++rb) {
                    FTile<FE> cur;
                    if (g == wave) cur = bpre[rb];
                    else load_ftile<FE>(cur, fb, R0 + rb, g, lane);
                    h8 b[NMF];
                    decode_tile<FE>(cur.w, 8u, b);
                    f4 part = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int q = 0; q < NMF; ++q) {
                        part = mfma16(hi[q], b[q], part);
                        part = mfma16(lo[q], b[q], part);
                    }
                    acc[rb] += (float)cur.sc * part;
                }
            }
        }
    }

    // ---- combine, convert, store -------------------------------------------------------------------
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
            for (int i = 0; i < 4; ++i)
                if (4 * j + i < mt) a.y[(size_t)(m_blk + 4 * j + i) * a.d_out + o] = (_Float16)v[i];
        }
    }
}

// ------------------------------------------------------------------------------------------------
template <int FM, int FA, int FE, int RB, int NW, bool XLDS>
static hipError_t launch_one(const FusedArgs& a, dim3 grid, size_t lds, hipStream_t stream)
{
    auto kern = fused_kernel<FM, FA, FE, RB, NW, XLDS>;
    if (lds > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(kern, grid, dim3(NW * 64), lds, stream, a);
    return hipGetLastError();
}

template <int FM, int FA, int FE>
static hipError_t launch_cfg(const FusedArgs& a, hipStream_t stream)
{
    const int nblk = a.d_out / 16;
    const int yblocks = (a.M + 15) / 16;
    // x is staged in LDS when one token block of it is small (decode); otherwise fragments come from
    // global memory and strips of 4 (or 2) row blocks reuse them.
    const int mt = a.M < 16 ? a.M : 16;
    const size_t xbytes = (size_t)mt * (a.d_in + 32) * 2;
    if (mt <= 4 && (size_t)mt * a.d_in * 2 <= 4 * 8 * 64 * 16)
        return launch_one<FM, FA, FE, 1, 8, true>(a, dim3(nblk, yblocks), xbytes, stream);
    int rb = 1;
    if (nblk % 4 == 0 && nblk / 4 >= 256) rb = 4;
    else if (nblk % 2 == 0 && nblk / 2 >= 256) rb = 2;
    const dim3 grid(nblk / rb, yblocks);
    if (rb == 4) return launch_one<FM, FA, FE, 4, 8, false>(a, grid, 0, stream);
    if (rb == 2) return launch_one<FM, FA, FE, 2, 8, false>(a, grid, 0, stream);
    return launch_one<FM, FA, FE, 1, 8, false>(a, grid, 0, stream);
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
