// Decode kernel for one to four tokens: the same layer as fused.hip,
//
//      y = x.What^T + (x.A^T).B^T          (Sec. 3 forward equation, Alg. 1 step 7)
//
// written as straight-line code for the shapes where the contraction dimension is an exact number
// of quads per wavefront (d_in / 512 == NW * NQ).  Nothing a load depends on is behind a divergent
// branch: out-of-range lanes read clamped (valid) addresses and their results are never stored, so
// the compiler can keep every request of a wavefront in flight and consume tiles as they arrive.
//
// Roles are split by workgroup index.  The first `units` workgroups are PRODUCERS: each computes one
// unit of t = x.A^T ((16 rows of A) x (one of kcn ranges of k-tiles)), writes its fp32 partial
// through to memory and raises flag[u] = epoch + 1; it owns no output rows, so nothing waits on its
// critical path but the consumers.  The other workgroups are CONSUMERS: one strip of 16 output rows
// each; backbone first, then one wavefront polls the flags, adds the kcn partials in a fixed order
// into t (fp32, in LDS), and the wavefronts that own tiles of B continue the same accumulators with
// t split into a high and a low fp16 part.  Producers come first in dispatch order and never wait.
#include "segments.hpp"

namespace eora {

constexpr int XSTAGE = 4;   // 16-byte chunks of x a thread may stage
constexpr int TWO_BLOCKS_FROM = 1024;   // row blocks of a launch from which a workgroup takes two

#ifdef EORA_TIMELINE
// debug build only: per-workgroup time stamps (100 MHz counter) behind the partials of t
#define TL_STAMP(slot) do { if (tid == 0) (a.tpair + (1 << 20))[blockIdx.x * 8 + (slot)] = wall_clock64(); } while (0)
#else
#define TL_STAMP(slot) do { } while (0)
#endif

// Member m's entry of a per-member argument array, chosen with scalar selects among the four entries (all at
// fixed places of the argument block, requested with the first batch of scalar loads) instead of a load at a
// computed offset, which could only be issued once m is known: one dependent round trip less at the start of
// every workgroup.
template <typename T>
__device__ __forceinline__ T pick_member(const T (&arr)[MAX_GROUP], int m)
{
    T v = arr[0];
    v = m == 1 ? arr[1] : v;
    v = m == 2 ? arr[2] : v;
    v = m == 3 ? arr[3] : v;
    return v;
}

template <int FM, int FA, int FE, int NW, int NQ, bool M1, int RB>
__global__ __launch_bounds__(NW * 64, (16 + NW - 1) / NW) void small_kernel(GroupArgs a)   // second bound: wavefronts per SIMD, i.e. at most 128 registers for four-wavefront workgroups
{
    constexpr bool LOWRANK = FA != S_NONE;
    constexpr int NT = NW * 64;
    constexpr int WORDS = Fmt<FM>::WORDS;
    __shared__ float red[NW][RB][4][16];
    __shared__ uint32_t s_epoch, s_ok;

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int n = lane & 15, j = lane >> 4;
    const int mt = M1 ? 1 : a.M;                         // 1..4 tokens, one token block (M1: exactly one)
    const int mrow = n < mt ? n : 0;                     // lanes beyond the tokens re-read row 0; their results are dropped
    const int upl = LOWRANK ? (a.r / 16) * a.kcn : 0;    // units of t (= producer workgroups) per member
    const int nprod = upl * a.n;                         // producer workgroups
    const int ldxs = a.d_in + 32;                        // LDS row stride of x in halves (64 bytes of padding)
    _Float16* xs = (_Float16*)eora_smem;
    float* ts = (float*)(eora_smem + (size_t)mt * ldxs * 2);     // t, fp32 mt x r (consumers)

    CheckIn ci{0u, 0u, 0u};
    TL_STAMP(0);
    if constexpr (LOWRANK) {
        if (tid == 0) check_in_load(ci, a.hdr);          // first request of the kernel: it returns first
    }

    // ---- x: requested first, by everyone ---------------------------------------------------------
    // A row of x is d_in / 8 = NQ * NT chunks of 16 bytes, so chunk (tid + k * NT) of the staged block is
    // chunk tid + (k % NQ) * NT of token row k / NQ: no division.  Rows beyond the tokens repeat row 0.
    constexpr int XS = M1 ? NQ : XSTAGE;
    u4 xstage[XS];
#pragma unroll
    for (int k = 0; k < XS; ++k) {
        const int xrow = (k / NQ) < mt ? (k / NQ) : 0;
        xstage[k] = *((const u4*)(a.x + (size_t)xrow * a.d_in) + tid + (k % NQ) * NT);
    }

    if constexpr (LOWRANK) {
    if ((int)blockIdx.x < nprod) {
        // ======================================================================= producer
        __builtin_amdgcn_s_setprio(3);                   // everyone's critical path: issue ahead of the consumers' dequant
        constexpr int KTA = Fmt<FA>::KT, NMF = KTA / 32;
        const int NRB = a.r / 16;
        const int u = blockIdx.x, mem = u / upl, ul = u % upl, rho = ul % NRB, kc = ul / NRB;
        const Factor fa{(const uint32_t*)pick_member(a.A, mem), pick_member(a.A_scales, mem), a.d_in / KTA};
        const int tpc = fa.ntk / a.kcn;                  // k-tiles of this unit
        const int first = kc * tpc + wave;
        const int nsteps = wave < tpc ? (tpc - wave + NW - 1) / NW : 0;
        constexpr int PD = 4;
        FTile<FA> buf[PD];
#pragma unroll
        for (int s = 0; s < PD; ++s) {
            const int ss = s < nsteps ? s : (nsteps > 0 ? nsteps - 1 : 0);
            load_ftile<FA>(buf[s], fa, rho, (nsteps > 0 ? first : kc * tpc) + ss * NW, lane);
        }
        __builtin_amdgcn_sched_barrier(0);               // all requests are out before the first result is used
        if (tid == 0) s_epoch = ci.epoch;
#pragma unroll
        for (int k = 0; k < XS; ++k) *(u4*)(xs + ((k / NQ) < mt ? (k / NQ) : 0) * ldxs + (tid + (k % NQ) * NT) * 8) = xstage[k];
        __syncthreads();
        if (tid == 0) check_in_issue(ci, a.hdr, blockIdx.x);
        TL_STAMP(1);
        const uint32_t epoch = s_epoch;
        f4 acc = {0.f, 0.f, 0.f, 0.f};
        for (int base = 0; base < nsteps; base += PD) {
#pragma unroll
            for (int s = 0; s < PD; ++s) {
                if (base + s < nsteps) {
                    const FTile<FA> cur = buf[s];
                    const int g = first + (base + s) * NW;
                    if (base + s + PD < nsteps) load_ftile<FA>(buf[s], fa, rho, first + (base + s + PD) * NW, lane);
                    h8 xa[NMF], b[NMF];
                    const _Float16* px = xs + mrow * ldxs + g * KTA + (KTA / 4) * j;
#pragma unroll
                    for (int t = 0; t < NMF; ++t) xa[t] = *(const h8*)(px + 8 * t);
                    decode_tile<FA>(cur.w, 8u, b);
                    if constexpr (FA == S_F16) {
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
        // token rows 0..3 live in lanes j == 0, register i = row
        if (j == 0) {
#pragma unroll
            for (int i = 0; i < 4; ++i) red[wave][0][i][n] = acc[i];
        }
        __syncthreads();
        TL_STAMP(2);
        if (tid < 16 * mt) {
            const int i = tid >> 4, col = tid & 15;
            float v = 0.f;
#pragma unroll
            for (int w2 = 0; w2 < NW; ++w2) v += red[w2][0][i][col];
            // partial layout: [kc][token row (16)][r], every element an 8-byte (value, epoch + 1) pair
            // written by ONE write-through store: a reader that finds this launch's tag has this
            // launch's value, so the flag below need not wait for these stores to be acknowledged
            const unsigned long long pr = ((unsigned long long)(epoch + 1) << 32) | __builtin_bit_cast(uint32_t, v);
            __hip_atomic_store(&a.tpair[(((size_t)mem * a.kcn + kc) * 16 + i) * a.r + 16 * rho + col], pr, __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_AGENT);
        }
        // (tid < 16 * mt) is within wavefront 0, whose lane 0 raises the flag: same wavefront, later instruction
        TL_STAMP(3);
        if (tid == 0) {
            for (int rep = 0; rep < HDR_FLAG_REPLICAS; ++rep)      // one copy per group of pollers
                __hip_atomic_store(&a.hdr[HDR_FLAGS0 + HDR_FLAGS_REPLICA_STRIDE * rep + u], epoch + 1, __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_AGENT);
            check_in_finish(ci, a.hdr, gridDim.x);
        }
        return;
    }
    }

    // =========================================================================== consumer
    int R = blockIdx.x - nprod, mem = 0;                 // strip of RB row blocks within its member
    {
        const int s0 = a.d_out[0] / (16 * RB), s1 = a.d_out[1] / (16 * RB), s2 = a.d_out[2] / (16 * RB);
        if (a.n > 1 && R >= s0) {
            R -= s0;
            mem = 1;
            if (a.n > 2 && R >= s1) {
                R -= s1;
                mem = 2;
                if (a.n > 3 && R >= s2) {
                    R -= s2;
                    mem = 3;
                }
            }
        }
    }
    const int d_out_m = pick_member(a.d_out, mem);
    _Float16* const y_m = pick_member(a.y, mem);
    const _Float16* const w_scales = pick_member(a.w_scales, mem);
    const uint32_t* const w_zeros = pick_member(a.w_zeros, mem);
    const uint32_t* const w_tiles = (const uint32_t*)pick_member(a.w, mem);
    const int G = a.d_in / 128;                          // == 4 * NW * NQ, one quantisation group per k-tile
    uint2 sc[RB][NQ];
    uint32_t zq[RB][NQ];
    uint32_t wd[RB][NQ][4][WORDS];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        const size_t row = (size_t)(R * RB + rb) * 16 + n;
#pragma unroll
        for (int q = 0; q < NQ; ++q) {
            const int g0 = 4 * (wave + q * NW);
            sc[rb][q] = *(const uint2*)(w_scales + row * G + g0);
            zq[rb][q] = w_zeros[row * (G / 8) + (g0 >> 3)];
        }
    }
    const Factor fb{(const uint32_t*)pick_member(a.B, mem), pick_member(a.B_scales, mem), LOWRANK ? a.r / Fmt<LOWRANK ? FE : S_F16>::KT : 0};
    FTile<LOWRANK ? FE : S_F16> bpre[RB];
    if constexpr (LOWRANK) {
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) load_ftile<FE>(bpre[rb], fb, R * RB + rb, wave < fb.ntk ? wave : 0, lane);
    }
    // the first row block's tiles now; a further row block's quad q is requested when quad q of the
    // row block before it has been consumed (same registers, no second buffer)
    // this lane's words of tile (R * RB) * G + 4 * wave; every other tile it reads is a compile-time
    // number of tiles further on (32-bit word index: a matrix of this format stays far below 16 GiB)
    const uint32_t* const wp = w_tiles + (uint32_t)((((uint32_t)(R * RB) * G + 4 * wave) * 64 + lane) * WORDS);
#pragma unroll
    for (int q = 0; q < NQ; ++q) {
#pragma unroll
        for (int i = 0; i < 4; ++i) load_words<WORDS>(wd[0][q][i], wp + (4 * q * NW + i) * 64 * WORDS);
    }
    // Every request above is in flight before anything below consumes one: without this fence the
    // scheduler moves uses of the first results (zero-point constants, x to LDS) in between the
    // requests, and the tiles requested after such a use wait a whole round trip longer.
    __builtin_amdgcn_sched_barrier(0);
    if constexpr (LOWRANK) {
        if (tid == 0) s_epoch = ci.epoch;
    }
#pragma unroll
    for (int k = 0; k < XS; ++k) *(u4*)(xs + ((k / NQ) < mt ? (k / NQ) : 0) * ldxs + (tid + (k % NQ) * NT) * 8) = xstage[k];
    __syncthreads();

    TL_STAMP(1);
    uint32_t early = 0;
    // ---- backbone ------------------------------------------------------------------------------------
    f4 acc[RB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) acc[rb] = f4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        // a first look at the flags, requested before the last row block and examined after it: when
        // the producers are done by the time this request reaches memory, the poll below costs no
        // round trip
        if constexpr (LOWRANK) {
            if (rb == RB - 1 && wave == 0)
                early = ld_relaxed(a.hdr + HDR_FLAGS0 + HDR_FLAGS_REPLICA_STRIDE * (blockIdx.x % HDR_FLAG_REPLICAS) + mem * upl +
                                   (lane < upl ? lane : upl - 1));
        }
#pragma unroll
        for (int q = 0; q < NQ; ++q) {
            const int g0 = 4 * (wave + q * NW);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                h8 xa[4], b[4];
                const _Float16* px = xs + mrow * ldxs + (g0 + i) * 128 + 32 * j;
#pragma unroll
                for (int t = 0; t < 4; ++t) xa[t] = *(const h8*)(px + 8 * t);
                decode_tile<FM>(wd[rb][q][i], (zq[rb][q] >> (4 * ((g0 & 7) + i))) & 0xFu, b);
                f4 part = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int t = 0; t < 4; ++t) part = mfma16(xa[t], b[t], part);
                const uint32_t sw = (i < 2) ? sc[rb][q].x : sc[rb][q].y;
                const _Float16 s16 = __builtin_bit_cast(_Float16, (uint16_t)((i & 1) ? (sw >> 16) : (sw & 0xFFFFu)));
                // exact integers times x, scaled once per group in fp32 (one token: only register 0 is ever stored)
                if constexpr (M1) acc[rb][0] += (float)s16 * part[0];
                else acc[rb] += (float)s16 * part;
            }
            if constexpr (RB > 1) {
                if (rb + 1 < RB) {
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        load_words<WORDS>(wd[rb + 1][q][i], wp + ((size_t)(rb + 1) * G + 4 * q * NW + i) * 64 * WORDS);
                }
            }
        }
    }

    TL_STAMP(2);
    // ---- low-rank continuation ---------------------------------------------------------------------
    if constexpr (LOWRANK) {
        // checks in now, with every tile consumed: the atomic's answer is needed at the very end only
        if (tid == 0) check_in_issue(ci, a.hdr, blockIdx.x);
        const uint32_t epoch = s_epoch;
        if (wave == 0) {
            // the units of this workgroup's own member only
            const uint32_t* flags = a.hdr + HDR_FLAGS0 + HDR_FLAGS_REPLICA_STRIDE * (blockIdx.x % HDR_FLAG_REPLICAS) + mem * upl;
            bool ok = a.spin_limit >= 0 && upl <= 64 && __all(early == epoch + 1);      // a negative limit: every wait counts as expired (test hook)
            for (int spins = 0; !ok && spins <= a.spin_limit; ++spins) {
                bool all = true;
                for (int f = lane; f < upl; f += 64) all = all && (ld_relaxed(&flags[f]) == epoch + 1);
                if (__all(all)) { ok = true; break; }
                __builtin_amdgcn_s_sleep(2);
            }
            TL_STAMP(4);
            if (ok) {
                // The partials are read with ordinary (cached) loads first: the flags are up, so their
                // stores were issued long ago and have all but certainly landed, and caches hold
                // nothing of them from before the launch.  The tags say whether that held; a lane
                // that finds an old tag reads again past the caches until it does (bounded).
                const int T = mt * a.r;                  // elements of t; a.r is a multiple of 32
                for (int e = 4 * lane; e < T; e += 256) {
                    const int i = e / a.r, col = e % a.r;
                    const unsigned long long* p = a.tpair + ((size_t)mem * a.kcn * 16 + i) * a.r + col;
                    float v0 = 0.f, v1 = 0.f, v2 = 0.f, v3 = 0.f;
                    uint32_t bad = 0;
#pragma unroll 4
                    for (int kc = 0; kc < a.kcn; ++kc) {                       // fixed order
                        const uint2* pk = (const uint2*)(p + (size_t)kc * 16 * a.r);
                        const uint2 p0 = pk[0], p1 = pk[1], p2 = pk[2], p3 = pk[3];      // .x value, .y tag
                        bad |= (p0.y ^ (epoch + 1)) | (p1.y ^ (epoch + 1)) | (p2.y ^ (epoch + 1)) | (p3.y ^ (epoch + 1));
                        v0 += __builtin_bit_cast(float, p0.x);
                        v1 += __builtin_bit_cast(float, p1.x);
                        v2 += __builtin_bit_cast(float, p2.x);
                        v3 += __builtin_bit_cast(float, p3.x);
                    }
                    bool good = bad == 0;
                    for (int spins = 0; !good && spins <= a.spin_limit; ++spins) {
                        bad = 0;
                        float w[4] = {0.f, 0.f, 0.f, 0.f};
                        for (int kc = 0; kc < a.kcn; ++kc) {
#pragma unroll
                            for (int c = 0; c < 4; ++c) {
                                const unsigned long long pr = __hip_atomic_load(p + (size_t)kc * 16 * a.r + c, __ATOMIC_RELAXED,
                                                                                __HIP_MEMORY_SCOPE_AGENT);
                                bad |= (uint32_t)(pr >> 32) ^ (epoch + 1);
                                w[c] += __builtin_bit_cast(float, (uint32_t)pr);
                            }
                        }
                        good = bad == 0;
                        v0 = w[0]; v1 = w[1]; v2 = w[2]; v3 = w[3];
                    }
                    const f4 v = {v0, v1, v2, v3};
                    ok = ok && good;
                    *(f4*)(ts + e) = v;
                }
                ok = __all(ok);
            }
            TL_STAMP(5);
            if (lane == 0) {
                s_ok = ok ? 1u : 0u;
                if (!ok) atomicOr(&a.hdr[HDR_ERROR], 1u);          // never expected: producers do not wait
            }
        }
        __syncthreads();
        if (s_ok) {
            constexpr int KTB = Fmt<FE>::KT, NMF = KTB / 32;
            for (int g = wave; g < fb.ntk; g += NW) {
                h8 hi[NMF], lo[NMF];                     // t split once, used for the RB row blocks
#pragma unroll
                for (int q = 0; q < NMF; ++q) {
                    const float* p = ts + mrow * a.r + g * KTB + (KTB / 4) * j + 8 * q;
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
                    else load_ftile<FE>(cur, fb, R * RB + rb, g, lane);
                    h8 b[NMF];
                    decode_tile<FE>(cur.w, 8u, b);
                    f4 part = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int q = 0; q < NMF; ++q) {
                        part = mfma16(hi[q], b[q], part);
                        part = mfma16(lo[q], b[q], part);
                    }
                    if constexpr (M1) acc[rb][0] += (float)cur.sc * part[0];
                    else acc[rb] += (float)cur.sc * part;
                }
            }
        }
    }

    // ---- combine, convert, store -------------------------------------------------------------------
    if (j == 0) {
#pragma unroll
        for (int rb = 0; rb < RB; ++rb)
#pragma unroll
            for (int i = 0; i < (M1 ? 1 : 4); ++i) red[wave][rb][i][n] = acc[rb][i];
    }
    __syncthreads();
    if (tid < 16 * mt) {
        const int i = tid >> 4, col = tid & 15;
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) {
            float v = 0.f;
#pragma unroll
            for (int w2 = 0; w2 < NW; ++w2) v += red[w2][rb][i][col];
            y_m[(size_t)i * d_out_m + (R * RB + rb) * 16 + col] = (_Float16)v;
        }
    }
    TL_STAMP(6);
    if constexpr (LOWRANK) {
        if (tid == 0) check_in_finish(ci, a.hdr, gridDim.x);
    }
}

// ------------------------------------------------------------------------------------------------
template <int FM, int FA, int FE, int NW, int NQ, bool M1, int RB>
static hipError_t launch_small_m(const GroupArgs& a, hipStream_t stream)
{
    auto kern = small_kernel<FM, FA, FE, NW, NQ, M1, RB>;
    const size_t lds = (size_t)a.M * (a.d_in + 32) * 2 + (size_t)a.M * a.r * 4;
    if (lds > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    int blocks = (FA != S_NONE) ? (a.r / 16) * a.kcn * a.n : 0;     // producers first
    for (int m = 0; m < a.n; ++m) blocks += a.d_out[m] / (16 * RB);
    note_launch("small FM=%d FA=%d NW=%d NQ=%d RB=%d n=%d", FM, FA, NW, NQ, RB, a.n);
    hipLaunchKernelGGL(kern, dim3(blocks), dim3(NW * 64), lds, stream, a);
    return hipGetLastError();
}

template <int FM, int FA, int FE, int NW, int NQ>
static hipError_t launch_small_one(const GroupArgs& a, hipStream_t stream)
{
    if (a.M == 1) {
        // Launches of more row blocks than can be resident at once give every workgroup two of them:
        // then all workgroups start together and each pays the wait for t once, at its very end.
        if constexpr (NQ <= 2 && FA != S_NONE) {           // (the bare layer has no such wait: one row block each streams best)
            int blocks = 0;
            bool even = true;
            for (int m = 0; m < a.n; ++m) {
                blocks += a.d_out[m] / 16;
                even = even && a.d_out[m] % 32 == 0;
            }
            if (even && blocks > TWO_BLOCKS_FROM) return launch_small_m<FM, FA, FE, NW, NQ, true, 2>(a, stream);
        }
        return launch_small_m<FM, FA, FE, NW, NQ, true, 1>(a, stream);
    }
    if constexpr (NQ <= XSTAGE / 2) return launch_small_m<FM, FA, FE, NW, NQ, false, 1>(a, stream);   // M * NQ <= XSTAGE
    return hipErrorInvalidValue;
}

template <int FM, int FA, int FE>
static hipError_t launch_small_shape(const GroupArgs& a, int nw, int nq, hipStream_t stream)
{
    if (nw == 8 && nq == 1) return launch_small_one<FM, FA, FE, 8, 1>(a, stream);
    if (nw == 8 && nq == 2) return launch_small_one<FM, FA, FE, 8, 2>(a, stream);
    if (nw == 14 && nq == 2) return launch_small_one<FM, FA, FE, 14, 2>(a, stream);
    if (nw == 14 && nq == 4) return launch_small_one<FM, FA, FE, 14, 4>(a, stream);
    if (nw == 4 && nq == 1) return launch_small_one<FM, FA, FE, 4, 1>(a, stream);
    if (nw == 4 && nq == 2) return launch_small_one<FM, FA, FE, 4, 2>(a, stream);
    if (nw == 7 && nq == 4) return launch_small_one<FM, FA, FE, 7, 4>(a, stream);
    if (nw == 16 && nq == 1) return launch_small_one<FM, FA, FE, 16, 1>(a, stream);
    return hipErrorInvalidValue;
}

template <int FM>
static hipError_t launch_small_ab(const GroupArgs& a, int fa, int fe, int nw, int nq, hipStream_t stream)
{
    if (fe == S_NONE) return launch_small_shape<FM, S_NONE, S_NONE>(a, nw, nq, stream);
    if (fa == S_F16 && fe == S_F16) return launch_small_shape<FM, S_F16, S_F16>(a, nw, nq, stream);
    if (fa == S_Q4S128 && fe == S_Q4S128) return launch_small_shape<FM, S_Q4S128, S_Q4S128>(a, nw, nq, stream);
    if (fa == S_Q4S128 && fe == S_Q4S64) return launch_small_shape<FM, S_Q4S128, S_Q4S64>(a, nw, nq, stream);
    if (fa == S_Q3S128 && fe == S_Q3S128) return launch_small_shape<FM, S_Q3S128, S_Q3S128>(a, nw, nq, stream);
    return hipErrorInvalidValue;
}

// Shapes this kernel takes: 1..4 tokens, one quantisation group per k-tile, d_in / 512 an exact
// number of quads per wavefront from the table below, x small enough to stage.
bool small_kernel_fits(int M, int d_in, int group, int* nw, int* nq)
{
    if (M < 1 || M > 4 || group != 128 || d_in % 512) return false;
    const int Q = d_in / 512;
    static const int table[][2] = {{4, 2}, {7, 4}, {8, 2}, {14, 4}, {4, 1}, {8, 1}, {14, 2}, {16, 1}};   // first match wins
    for (const auto& t : table) {
        if (t[0] * t[1] == Q && (size_t)M * (d_in / 8) <= (size_t)XSTAGE * t[0] * 64) {
            *nw = t[0];
            *nq = t[1];
            return true;
        }
    }
    return false;
}

hipError_t launch_small(const GroupArgs& a, int fm, int fa, int fe, int nw, int nq, hipStream_t stream)
{
    switch (fm) {
        case S_Q4: return launch_small_ab<S_Q4>(a, fa, fe, nw, nq, stream);
        case S_Q3: return launch_small_ab<S_Q3>(a, fa, fe, nw, nq, stream);
        case S_Q2: return launch_small_ab<S_Q2>(a, fa, fe, nw, nq, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace eora
