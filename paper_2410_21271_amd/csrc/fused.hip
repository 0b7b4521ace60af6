// The compensated compressed linear layer for up to 16 tokens per token block, in ONE launch:
//
//      y = x.What^T + (x.A^T).B^T          (Sec. 3 forward equation, Alg. 1 step 7)
//
// HBM-bound: every stored byte is read once, decoded in registers (tiles.hpp) and fed to
// 16x16x32 fp16 MFMAs whose 16-row operand is the token block (rows beyond M repeat row 0; never stored).
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
//            belongs to workgroup u of the token block, a producer that owns no output rows
//            (workgroups are dispatched in index order and a producer never waits, so no producer
//            can be starved by a waiter).  It writes its fp32 partial to scratch and then publishes
//            flag[u] = epoch + 1.
//   phase W  backbone tiles of the strip (independent of t; hides phase A's latency).
//   phase B  one wavefront polls the flags (bounded), then the wavefronts that own tiles of B add
//            the kcn partials in a fixed order to get their slice of t (fp32), split it into a high
//            and a low fp16 part and continue the contraction over B's tiles.
// Nothing is reset between launches: flags are compared with epoch + 1 and the epoch word is
// advanced once per launch, by the last workgroup to check in on a spread-out arrival counter
// (every workgroup reads the epoch before it checks in).
#include "segments.hpp"

namespace eora {

#ifdef EORA_TIMELINE
// debug build only: per-workgroup time stamps (100 MHz counter) behind the partials of t
#define FTL_STAMP(slot) do { if (threadIdx.x == 0) ((unsigned long long*)(a.tpart + (1 << 20)))[(blockIdx.y * gridDim.x + blockIdx.x) * 8 + (slot)] = wall_clock64(); } while (0)
#else
#define FTL_STAMP(slot) do { } while (0)
#endif

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
    constexpr bool LOWRANK = FA != S_NONE;
    // The first `units` workgroups of a token block are PRODUCERS: one unit of t = x.A^T each, no output
    // rows, so nothing but the consumers waits on them; the others own a strip of RB row blocks.
    const int units = LOWRANK ? (a.r / 16) * a.kcn : 0;
    const bool producer = (int)blockIdx.x < units;
    const int R0 = producer ? 0 : ((int)blockIdx.x - units) * RB;

    if constexpr (LOWRANK) {
        if (producer) {
            // ===================================================================== producer
            __builtin_amdgcn_s_setprio(3);                 // everyone's critical path
            FTL_STAMP(0);
            constexpr int KTA = Fmt<FA>::KT;
            CheckIn pci{0u, 0u, 0u};
            if (threadIdx.x == 0) check_in_load(pci, a.hdr);
            const int NRB = a.r / 16;
            const int u = blockIdx.x, rho = u % NRB, kc = u / NRB;
            const Factor fa{(const uint32_t*)a.A, a.A_scales, a.d_in / KTA};
            const int tpc = fa.ntk / a.kcn;
            const f4 part = run_factor_a_eager<FA, NW>(fa, rho, kc * tpc, (kc + 1) * tpc, wave, lane,
                                                       a.x + (size_t)m_blk * a.d_in, a.d_in, n, row_ok);
            if (threadIdx.x == 0) {
                check_in_issue(pci, a.hdr, blockIdx.y * gridDim.x + blockIdx.x);
                s_epoch = pci.epoch;
            }
            FTL_STAMP(1);
            if (wave > 0) red[wave - 1][0][lane] = part;
            __syncthreads();
            if (wave == 0) {
                f4 v = part;
#pragma unroll
                for (int w2 = 0; w2 < NW - 1; ++w2) v += red[w2][0][lane];
                // partial layout: [token block][kc][token row][r], every element an 8-byte (value, epoch + 1)
                // pair written by ONE write-through store: a reader that finds this launch's tag has this
                // launch's value, so the flag (same wavefront, later instruction) need not wait for these
                // stores to be acknowledged.  Register i is token row 4*j+i, column n.
                unsigned long long* dst = a.tpair + ((size_t)(yb * a.kcn + kc) * 16) * a.r + 16 * rho + n;
                const float vs[4] = {v.x, v.y, v.z, v.w};
                const unsigned long long tag = (unsigned long long)(s_epoch + 1) << 32;
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    if (4 * j + i < mt)
                        __hip_atomic_store(&dst[(size_t)(4 * j + i) * a.r], tag | __builtin_bit_cast(uint32_t, vs[i]),
                                           __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                FTL_STAMP(2);
                if (lane == 0) {
                    __hip_atomic_store(&a.hdr[HDR_FLAGS0 + HDR_FLAGS_PER_BLOCK * yb + u], pci.epoch + 1, __ATOMIC_RELAXED,
                                       __HIP_MEMORY_SCOPE_AGENT);
                    check_in_finish(pci, a.hdr, gridDim.x * gridDim.y);
                }
            }
            return;
        }
    }

    FTL_STAMP(0);
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

    const Backbone bb{(const uint32_t*)a.w, a.w_scales, a.w_zeros, a.d_in / 128, a.d_in / a.group,
                      (a.d_in / a.group + 7) / 8, a.group / 128};
    const int Q = (bb.G + 3) / 4;
    constexpr int PDQ = RB == 1 ? 2 : 1;     // quads of weight loads in flight per wavefront
    Quad<FM, RB> qbuf[PDQ];
    const int nq = (!producer && wave < Q) ? (Q - wave + NW - 1) / NW : 0;
#pragma unroll
    for (int u = 0; u < PDQ; ++u)
        if (u < nq) load_quad_meta<FM, RB>(qbuf[u], bb, R0, wave + u * NW, lane);

    // first tile of B for this wavefront (its words do not depend on t)
    const Factor fb{(const uint32_t*)a.B, a.B_scales, LOWRANK ? a.r / Fmt<LOWRANK ? FE : S_F16>::KT : 0};
    FTile<LOWRANK ? FE : S_F16> bpre[RB];
    if constexpr (LOWRANK) {
        if (!producer && wave < fb.ntk) {
#pragma unroll
            for (int rb = 0; rb < RB; ++rb) load_ftile<FE>(bpre[rb], fb, R0 + rb, wave, lane);
        }
    }
#pragma unroll
    for (int u = 0; u < PDQ; ++u)
        if (u < nq) load_quad_words<FM, RB>(qbuf[u], bb, R0, wave + u * NW, lane);

    // ---- check in (the last workgroup to do so advances the epoch) --------------------------------
    CheckIn ci{0u, 0u, 0u};
    if constexpr (LOWRANK) {
        if (threadIdx.x == 0) {
            check_in_load(ci, a.hdr);
            check_in_issue(ci, a.hdr, blockIdx.y * gridDim.x + blockIdx.x);
            s_epoch = ci.epoch;
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

    FTL_STAMP(1);
    // a first look at the flags, requested now and examined after the backbone
    uint32_t early = 0;
    if constexpr (LOWRANK) {
        if (wave == 0) early = ld_relaxed(a.hdr + HDR_FLAGS0 + HDR_FLAGS_PER_BLOCK * yb + (lane < units ? lane : units - 1));
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

    FTL_STAMP(2);
    // ---- phase B: += t.B^T -----------------------------------------------------------------------
    if constexpr (LOWRANK) {
        const uint32_t* flags = a.hdr + HDR_FLAGS0 + HDR_FLAGS_PER_BLOCK * yb;
        if (wave == 0) {
            bool ok = a.spin_limit >= 0 && units <= 64 && __all(early == epoch + 1);      // a negative limit: every wait counts as expired (test hook)
            for (int spins = 0; !ok && spins <= a.spin_limit; ++spins) {
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
        FTL_STAMP(3);
        __syncthreads();
        float* ts = (float*)(eora_smem + (XLDS ? (size_t)mt * ldxs * 2 : 0));      // t of this token block: mt x r fp32
        if (s_ok) {
            // Every thread adds the kcn partials of four elements of t, in a fixed order, into LDS.  Ordinary
            // cached loads first: the flags are up, so the stores were issued long ago and have all but
            // certainly landed; the tags say whether that held, and a thread that finds an old tag reads
            // again past the caches until it does (bounded).
            const int T = mt * a.r;
            bool good_all = true;
            for (int e = 4 * (int)threadIdx.x; e < T; e += 4 * NW * 64) {
                const unsigned long long* p = a.tpair + ((size_t)(yb * a.kcn) * 16) * a.r + e;     // row e / r, column e % r
                uint2 pr[MAX_KCN][4];
#pragma unroll
                for (int kc = 0; kc < MAX_KCN; ++kc) {                 // all k-ranges requested at once
                    const uint2* pk = (const uint2*)(p + (size_t)(kc < a.kcn ? kc : a.kcn - 1) * 16 * a.r);
#pragma unroll
                    for (int c = 0; c < 4; ++c) pr[kc][c] = pk[c];
                }
                float v[4] = {0.f, 0.f, 0.f, 0.f};
                uint32_t bad = 0;
#pragma unroll
                for (int kc = 0; kc < MAX_KCN; ++kc) {                 // fixed order
                    if (kc < a.kcn) {
#pragma unroll
                        for (int c = 0; c < 4; ++c) {
                            bad |= pr[kc][c].y ^ (epoch + 1);
                            v[c] += __builtin_bit_cast(float, pr[kc][c].x);
                        }
                    }
                }
                bool good = bad == 0;
                for (int spins = 0; !good && spins <= a.spin_limit; ++spins) {
                    bad = 0;
                    float w[4] = {0.f, 0.f, 0.f, 0.f};
                    for (int kc = 0; kc < a.kcn; ++kc) {
#pragma unroll
                        for (int c = 0; c < 4; ++c) {
                            const unsigned long long q = __hip_atomic_load(p + (size_t)kc * 16 * a.r + c, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                            bad |= (uint32_t)(q >> 32) ^ (epoch + 1);
                            w[c] += __builtin_bit_cast(float, (uint32_t)q);
                        }
                    }
                    good = bad == 0;
                    v[0] = w[0]; v[1] = w[1]; v[2] = w[2]; v[3] = w[3];
                }
                good_all = good_all && good;
                if (a.adapter) {       // the four columns e % r .. + 3 belong to one adapter (r_per is a multiple of 4)
                    if (a.adapter[m_blk + e / a.r] != (e % a.r) / a.r_per) v[0] = v[1] = v[2] = v[3] = 0.f;
                }
                *(f4*)(ts + e) = f4{v[0], v[1], v[2], v[3]};
            }
            if (!good_all) atomicOr(&a.hdr[HDR_ERROR], 1u);            // never expected
        }
        __syncthreads();
        if (s_ok && wave < fb.ntk) {
            constexpr int KTB = Fmt<FE>::KT, NMF = KTB / 32;
            for (int g = wave; g < fb.ntk; g += NW) {
                h8 hi[NMF], lo[NMF];
#pragma unroll
                for (int q = 0; q < NMF; ++q) {
                    // (token rows beyond the block read row 0: their results are never stored)
                    const float* p = ts + (row_ok ? n : 0) * a.r + g * KTB + (KTB / 4) * j + 8 * q;
                    const f4 v0 = *(const f4*)p, v1 = *(const f4*)(p + 4);
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

    FTL_STAMP(4);
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
    FTL_STAMP(5);
    if constexpr (LOWRANK) {
        if (threadIdx.x == 0) check_in_finish(ci, a.hdr, gridDim.x * gridDim.y);
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
    note_launch("fused FM=%d FA=%d RB=%d NW=%d XLDS=%d", FM, FA, RB, NW, (int)XLDS);
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
    const int units = (FA != S_NONE) ? (a.r / 16) * a.kcn : 0;      // producer workgroups per token block, first in x
    const size_t tbytes = (FA != S_NONE) ? (size_t)mt * a.r * 4 : 0;   // t of a token block, fp32, in LDS
    if (mt <= 4 && (size_t)mt * a.d_in * 2 <= 4 * 8 * 64 * 16)
        return launch_one<FM, FA, FE, 1, 8, true>(a, dim3(nblk + units, yblocks), xbytes + tbytes, stream);
    int rb = 1;
    if (nblk % 4 == 0 && nblk / 4 >= 256) rb = 4;
    else if (nblk % 2 == 0 && nblk / 2 >= 256) rb = 2;
    const dim3 grid(nblk / rb + units, yblocks);
    if (rb == 4) return launch_one<FM, FA, FE, 4, 8, false>(a, grid, tbytes, stream);
    if (rb == 2) return launch_one<FM, FA, FE, 2, 8, false>(a, grid, tbytes, stream);
    return launch_one<FM, FA, FE, 1, 8, false>(a, grid, tbytes, stream);
}

template <int FM>
static hipError_t launch_ab(const FusedArgs& a, int fa, int fe, hipStream_t stream)
{
    if (fe == S_NONE) return launch_cfg<FM, S_NONE, S_NONE>(a, stream);
    if (fa == S_F16 && fe == S_F16) return launch_cfg<FM, S_F16, S_F16>(a, stream);
    if (fa == S_Q4S128 && fe == S_Q4S128) return launch_cfg<FM, S_Q4S128, S_Q4S128>(a, stream);
    if (fa == S_Q4S128 && fe == S_Q4S64) return launch_cfg<FM, S_Q4S128, S_Q4S64>(a, stream);
    if (fa == S_Q3S128 && fe == S_Q3S128) return launch_cfg<FM, S_Q3S128, S_Q3S128>(a, stream);
    return hipErrorInvalidValue;
}

hipError_t launch_fused(const FusedArgs& a, int fm, int fa, int fe, hipStream_t stream)
{
    switch (fm) {
        case S_Q4: return launch_ab<S_Q4>(a, fa, fe, stream);
        case S_Q3: return launch_ab<S_Q3>(a, fa, fe, stream);
        case S_Q2: return launch_ab<S_Q2>(a, fa, fe, stream);
        default: return hipErrorInvalidValue;
    }
}

// every word 0, except the epoch word, which starts at `epoch0`
__global__ void clear_words_kernel(uint32_t* p, int nwords, uint32_t epoch0)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < nwords) p[i] = i == HDR_EPOCH ? epoch0 : 0u;
}

hipError_t launch_clear_words(uint32_t* p, int nwords, uint32_t epoch0, hipStream_t stream)
{
    hipLaunchKernelGGL(clear_words_kernel, dim3((nwords + 255) / 256), dim3(256), 0, stream, p, nwords, epoch0);
    return hipGetLastError();
}

}  // namespace eora
