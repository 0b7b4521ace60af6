// The compensated quantised layer for 5 .. 127 tokens, in ONE launch:
//
//      y = x.What^T + (x.A^T).B^T          (Sec. 3 forward equation, Alg. 1 step 7)
//
// HBM-bound like the decode kernel, but a token block's x (16 tokens) is now as many bytes as four row blocks
// of 4-bit weights, so it must not be fetched per stored tile by every wavefront that needs it.  A workgroup
// is NWR row blocks x NWK ranges of the contraction length, one wavefront each, and up to TB token blocks.
// Per step every range advances by one 128-column chunk: x[16 TB tokens][128] of the range goes global ->
// registers (requested 2 or 4 steps before its LDS write) -> one of the range's two LDS slots and is read from
// there by the range's NWR wavefronts; a stored tile, decoded once, serves all TB token blocks.  Stored tiles
// come in quads (one 8-byte load brings a row's four group scales, one word its four zero-points): one quad is
// in flight while the other is consumed, and it is refilled into the registers just used.  All requests are
// plain loads and every step issues the same ones (past the end: the last chunk again, never used), so the
// compiler's wait counts stay exact.  One barrier per step: after it chunk c is visible to the range's readers
// and everyone has left the other slot, which is rewritten at once.
//
// LDS slot layout: 16-byte piece q of token row t (columns 8q .. 8q+7 of the chunk) sits at piece index
// 16 t + (q ^ (t & 15)): the 16 lanes that read one q for 16 tokens hit 16 different bank groups.
//
// Arithmetic is the decode kernel's: integer codes minus zero-point exact in fp16, fp32 accumulation per
// 128-group, scaled once per group in fp32; t in fp32, split into a high and a low fp16 part for B's product.
// Low-rank path: producer workgroups first (one unit of t = x.A^T each, per token block), partials as tagged
// (value, epoch + 1) pairs, flags, fixed-order sums.  After the backbone the wavefronts of a row block share
// B's tiles, then the ranges' accumulators are added in a fixed order through LDS.
#include "segments.hpp"

namespace eora {

#ifdef EORA_TIMELINE
// debug build only: per-workgroup time stamps (100 MHz counter) behind the partials of t
#define WTL_STAMP(slot) do { if (threadIdx.x == 0) ((unsigned long long*)(a.tpart + (1 << 20)))[blockIdx.x * 8 + (slot)] = wall_clock64(); } while (0)
#else
#define WTL_STAMP(slot) do { } while (0)
#endif


// gbid: index of the workgroup in the launch; bid: its index among its member's workgroups; flag0: the member's
// first flag inside a token block's flags
template <int FM, int FA, int FE, int NWR, int NWK, int TB>
__device__ __forceinline__ void wide_q_body(const FusedArgs& a, const int gbid, const int bid, const int flag0)
{
    constexpr int NW = NWR * NWK;
    constexpr bool LOWRANK = FA != S_NONE;
    constexpr int SLOT = TB * 4096;                       // bytes: 16 TB tokens x 128 columns
    static_assert((4 * TB) % NWR == 0, "the 1 KiB pieces of a chunk divide evenly over a range's wavefronts");
    constexpr int XN = 4 * TB / NWR;                      // pieces per wavefront
    constexpr int WQ_D = XN > 2 ? 2 : 4;                  // steps between a request for x and its LDS write (registers: WQ_D x XN x 4)
    __shared__ f4 pred[NW > 1 ? NW - 1 : 1][64];          // a producer's cross-wavefront sum
    __shared__ uint32_t s_epoch, s_ok;

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int n = lane & 15, j = lane >> 4;
    const int wr = wave % NWR, wk = wave / NWR;
    const int yblocks = (a.M + 15) / 16;
    const int units = LOWRANK ? (a.r / 16) * a.kcn : 0;
    const int nprod = units * yblocks;

    CheckIn ci{0u, 0u, 0u};
    if constexpr (LOWRANK) {
        if (tid == 0) check_in_load(ci, a.hdr);
        if (bid < nprod) {
            // ===================================================================== producer
            __builtin_amdgcn_s_setprio(3);                 // everyone's critical path
            WTL_STAMP(0);
            constexpr int KTA = Fmt<FA>::KT;
            const int yb = bid / units, u = bid % units;
            const int m_blk = 16 * yb;
            const int mt = a.M - m_blk < 16 ? a.M - m_blk : 16;
            const int NRB = a.r / 16;
            const int rho = u % NRB, kc = u / NRB;
            const Factor fa{(const uint32_t*)a.A, a.A_scales, a.d_in / KTA};
            const int tpc = fa.ntk / a.kcn;
            const f4 part = run_factor_a_eager<FA, NW>(fa, rho, kc * tpc, (kc + 1) * tpc, wave, lane,
                                                       a.x + (size_t)m_blk * a.d_in, a.d_in, n, n < mt);
            if (tid == 0) {
                check_in_issue(ci, a.hdr, gbid);
                s_epoch = ci.epoch;
            }
            WTL_STAMP(1);
            if (wave > 0) pred[wave - 1][lane] = part;
            __syncthreads();
            if (wave == 0) {
                f4 v = part;
#pragma unroll
                for (int w2 = 0; w2 < NW - 1; ++w2) v += pred[w2][lane];
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
                WTL_STAMP(2);
                if (lane == 0) {
                    __hip_atomic_store(&a.hdr[HDR_FLAGS0 + HDR_FLAGS_PER_BLOCK * yb + flag0 + u], s_epoch + 1, __ATOMIC_RELAXED,
                                       __HIP_MEMORY_SCOPE_AGENT);
                    check_in_finish(ci, a.hdr, gridDim.x);
                }
            }
            return;
        }
    }

    // ========================================================================= consumer
    WTL_STAMP(0);
    const int RBs = a.d_out / 16;
    const int NTG = (yblocks + TB - 1) / TB;              // groups of TB token blocks
    const int cidx = bid - nprod;
    const int tg = cidx % NTG, rg = cidx / NTG;
    const int m0 = tg * TB * 16;                          // first token of the group
    const int Rw = rg * NWR + wr;
    const bool active = Rw < RBs;                         // a ragged last row group: the wavefront only helps staging
    const int R = active ? Rw : RBs - 1;
    const Backbone bb{(const uint32_t*)a.w, a.w_scales, a.w_zeros, a.d_in / 128, a.d_in / a.group,
                      (a.d_in / a.group + 7) / 8, a.group / 128};
    const int GK = bb.G / NWK;                            // chunks = stored tiles per range; a multiple of 4
    const int NQ = GK / 4;                                // quads per range
    const int q0 = wk * NQ;                               // the range's first quad
    unsigned char* xk = eora_smem + wk * 2 * SLOT;        // the range's two slots
    // piece q of a chunk: token rows 4 q .. 4 q + 3, lane -> row 4 q + lane / 16, 16-byte piece lane % 16
    const _Float16* xsrc[XN];
    int xdst[XN];
#pragma unroll
    for (int i = 0; i < XN; ++i) {
        const int trow = 4 * (wr + i * NWR) + (lane >> 4);
        // rows beyond the tokens: all their lanes read one and the same valid piece (one cache line per request
        // instead of sixteen; no divergent branch); their results are dropped
        const bool live = m0 + trow < a.M;
        xsrc[i] = a.x + (size_t)(live ? m0 + trow : m0) * a.d_in + (size_t)wk * GK * 128 + (live ? 8 * (lane & 15) : 0);
        xdst[i] = (trow * 16 + ((lane & 15) ^ (trow & 15))) * 16;
    }
    // Workgroups walk their ranges from different starting chunks (quads rotated by rq, the tiles inside a quad
    // by ri): the rows of x are a multiple of 4 KiB apart, so workgroups in step would all ask the same L2
    // channel for the same chunk at the same time.
    const int rot = cidx % GK, rq = rot >> 2, ri = rot & 3;
    auto quad_at = [&](int qq) {                          // qq < 2 NQ
        const int v = qq + rq;
        return v >= NQ ? v - NQ : v;
    };
    auto chunk_at = [&](int step) {                       // steps past the end: the last one again
        const int st = step < GK ? step : GK - 1;
        return 4 * quad_at(st >> 2) + ((st + ri) & 3);
    };
    auto load_quad = [&](Quad<FM, 1>& qd, int qq) {       // register slot i holds tile (i + ri) % 4 of the quad
        const int q = q0 + quad_at(qq < NQ ? qq : NQ - 1);
        load_quad_meta<FM, 1>(qd, bb, R, q, lane);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const size_t tile = (size_t)R * bb.G + 4 * q + ((i + ri) & 3);
            load_words<Fmt<FM>::WORDS>(qd.w[0][i], bb.w + (tile * 64 + lane) * Fmt<FM>::WORDS);
        }
    };
    Quad<FM, 1> qb[2];
    u4 xr[WQ_D][XN];
#pragma unroll
    for (int s = 0; s < WQ_D; ++s) {
#pragma unroll
        for (int i = 0; i < XN; ++i) xr[s][i] = *(const u4*)(xsrc[i] + chunk_at(s) * 128);
    }
#pragma unroll
    for (int h = 0; h < 2; ++h) load_quad(qb[h], h);
    // B's first tile of this wavefront (its words do not depend on t)
    constexpr int FEB = LOWRANK ? FE : S_F16;
    const Factor fb{(const uint32_t*)a.B, a.B_scales, LOWRANK ? a.r / Fmt<FEB>::KT : 0};
    FTile<FEB> bpre;
    if constexpr (LOWRANK) load_ftile<FE>(bpre, fb, R, wk < fb.ntk ? wk : 0, lane);
    if constexpr (LOWRANK) {
        if (tid == 0) {
            check_in_issue(ci, a.hdr, gbid);
            s_epoch = ci.epoch;
        }
    }
    // chunk 0 -> slot 0; its registers take chunk WQ_D
#pragma unroll
    for (int i = 0; i < XN; ++i) {
        *(u4*)(xk + xdst[i]) = xr[0][i];
        xr[0][i] = *(const u4*)(xsrc[i] + chunk_at(WQ_D) * 128);
    }

    WTL_STAMP(1);
    f4 acc[TB];
#pragma unroll
    for (int tb = 0; tb < TB; ++tb) acc[tb] = f4{0.f, 0.f, 0.f, 0.f};
    // this lane's activation fragments of a tile: 32 consecutive columns from 32 j, pieces 4 j .. 4 j + 3
    int poff[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) poff[t] = (n * 16 + ((4 * j + t) ^ n)) * 16;

    // a first look at the flags, requested before the last quads and examined after them: when the producers
    // are done by then, the wait below costs no round trip
    uint32_t early = 0;
    for (int qi = 0; qi < NQ; qi += 2) {
        if constexpr (LOWRANK && TB == 1) {
            if (wave == 0 && qi + 2 >= NQ)
                early = ld_relaxed(a.hdr + HDR_FLAGS0 + HDR_FLAGS_PER_BLOCK * tg + flag0 + (lane < units ? lane : units - 1));
        }
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int qq = qi + h;
            if (qq < NQ) {                                // uniform over the workgroup
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int c = 4 * qq + i;             // step = chunk of the range
                    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");       // own LDS writes of chunk c done
                    __builtin_amdgcn_s_barrier();
                    // chunk c + 1 -> the slot everyone has just left; its registers take the chunk WQ_D further on
                    const int s1 = (i + 1) % WQ_D;
                    const int cx = chunk_at(c + 1 + WQ_D);
#pragma unroll
                    for (int k = 0; k < XN; ++k) {
                        *(u4*)(xk + ((c + 1) & 1) * SLOT + xdst[k]) = xr[s1][k];
                        xr[s1][k] = *(const u4*)(xsrc[k] + cx * 128);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                    h8 b[4];
                    const int ti = (i + ri) & 3;          // the tile's place in its quad: its zero-point nibble and scale
                    decode_tile<FM>(qb[h].w[0][i], (qb[h].zq[0] >> (4 * ti)) & 0xFu, b);
                    const unsigned long long s64 = qb[h].sc[0].x | ((unsigned long long)qb[h].sc[0].y << 32);
                    const float sc = (float)__builtin_bit_cast(_Float16, (uint16_t)(s64 >> (16 * ti)));
                    const unsigned char* xs = xk + (c & 1) * SLOT;
#pragma unroll
                    for (int tb = 0; tb < TB; ++tb) {
                        const unsigned char* px = xs + tb * 4096;
                        f4 part = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                        for (int t = 0; t < 4; ++t) part = mfma16(*(const h8*)(px + poff[t]), b[t], part);
                        acc[tb] += sc * part;             // exact integers times x, scaled once per group in fp32
                    }
                }
                // the quad's registers are free again: the request for the quad two on goes out last
                __builtin_amdgcn_sched_barrier(0);
                load_quad(qb[h], qq + 2);
            }
        }
    }
    __syncthreads();                                      // nobody reads x any more: the slots are reused below
    WTL_STAMP(2);

    // ---- low-rank continuation: acc[token][row] += t[token][:] . B[row][:] ----------------------------------
    if constexpr (LOWRANK) {
        // t (16 x r fp32 per token block) goes over the x slots, as many token blocks at a time as fit
        float* ts = (float*)eora_smem;
        const int tsz = 16 * a.r;                         // floats per token block
        const int lds_floats = NWK * 2 * SLOT / 4 > tsz ? NWK * 2 * SLOT / 4 : tsz;
        const int nb = lds_floats / tsz;                  // >= 1
        const uint32_t epoch = s_epoch;
        if (wave == 0) {
            bool ok = true;
            const bool seen = a.spin_limit >= 0 && TB == 1 && units <= 64 && __all(early == epoch + 1);   // a negative limit: every wait counts as expired (test hook)
#pragma unroll
            for (int tb = 0; tb < TB; ++tb) {
                const int yb = tg * TB + tb;
                if (yb >= yblocks || !ok || seen) continue;
                const uint32_t* flags = a.hdr + HDR_FLAGS0 + HDR_FLAGS_PER_BLOCK * yb + flag0;
                bool up = false;
                for (int spins = 0; spins <= a.spin_limit; ++spins) {
                    bool all = true;
                    for (int f = lane; f < units; f += 64) all = all && (ld_relaxed(&flags[f]) == epoch + 1);
                    if (__all(all)) { up = true; break; }
                    __builtin_amdgcn_s_sleep(2);
                }
                ok = up;
            }
            if (lane == 0) {
                s_ok = ok ? 1u : 0u;
                if (!ok) atomicOr(&a.hdr[HDR_ERROR], 1u);  // never expected: producers do not wait
            }
        }
        __syncthreads();
        WTL_STAMP(3);
        if (s_ok) {
            constexpr int KTB = Fmt<FE>::KT, NMF = KTB / 32;
            bool good_all = true;
#pragma unroll
            for (int tb = 0; tb < TB; ++tb) {
                if (tb % nb == 0) {                       // uniform over the workgroup: the next nb token blocks' t
                    if (tb > 0) __syncthreads();          // the previous ones have been used
                    for (int q = 0; q < nb && tb + q < TB; ++q) {
                        const int yq = tg * TB + tb + q;
                        if (yq >= yblocks) break;
                        const int mq = a.M - 16 * yq < 16 ? a.M - 16 * yq : 16;
                        // Every thread adds the kcn partials of four elements of t, in a fixed order.  Ordinary
                        // cached loads first: the flags are up, so the stores were issued long ago and have all
                        // but certainly landed; the tags say whether that held, and a thread that finds an old
                        // tag reads again past the caches until it does (bounded).
                        const int T = mq * a.r;
                        for (int e = 4 * tid; e < T; e += 4 * NW * 64) {
                            const unsigned long long* p = a.tpair + ((size_t)(yq * a.kcn) * 16) * a.r + e;     // row e / r, column e % r
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
                            good_all = good_all && good;
                            if (a.adapter) {   // several adapters side by side: a token row keeps its own adapter's columns
                                if (a.adapter[16 * yq + e / a.r] != (e % a.r) / a.r_per) v0 = v1 = v2 = v3 = 0.f;
                            }
                            *(f4*)(ts + q * tsz + e) = f4{v0, v1, v2, v3};
                        }
                    }
                    __syncthreads();
                }
                const int yb = tg * TB + tb;
                if (yb < yblocks) {
                    const int mt = a.M - 16 * yb < 16 ? a.M - 16 * yb : 16;
                    const float* trow = ts + (tb % nb) * tsz + (n < mt ? n : 0) * a.r + (KTB / 4) * j;
                    for (int g = wk; g < fb.ntk; g += NWK) {      // the row block's wavefronts share B's tiles
                        FTile<FE> cur;
                        if (g == wk) cur = bpre;
                        else load_ftile<FE>(cur, fb, R, g, lane);
                        h8 b[NMF];
                        decode_tile<FE>(cur.w, 8u, b);
                        f4 part = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                        for (int q = 0; q < NMF; ++q) {
                            const float* p = trow + g * KTB + 8 * q;
                            const f4 v0 = *(const f4*)p, v1 = *(const f4*)(p + 4);
                            const float e0[4] = {v0.x, v0.y, v0.z, v0.w}, e1[4] = {v1.x, v1.y, v1.z, v1.w};
                            h8 hi, lo;
#pragma unroll
                            for (int i = 0; i < 4; ++i) {
                                const _Float16 h0 = (_Float16)e0[i], h1 = (_Float16)e1[i];
                                hi[i] = h0;
                                hi[4 + i] = h1;
                                lo[i] = (_Float16)(e0[i] - (float)h0);
                                lo[4 + i] = (_Float16)(e1[i] - (float)h1);
                            }
                            part = mfma16(hi, b[q], part);
                            part = mfma16(lo, b[q], part);
                        }
                        acc[tb] += (float)cur.sc * part;
                    }
                }
            }
            if (!good_all) atomicOr(&a.hdr[HDR_ERROR], 1u);            // never expected
        }
        if constexpr (NWK > 1) __syncthreads();           // t has been used: the LDS is reused below
    }

    WTL_STAMP(4);
    // ---- add the ranges' accumulators in a fixed order, convert, store ---------------------------------------
    if constexpr (NWK > 1) {
        f4* red = (f4*)eora_smem;                         // [range - 1][row block][token block][lane]
        if (wk > 0) {
#pragma unroll
            for (int tb = 0; tb < TB; ++tb) red[(((wk - 1) * NWR + wr) * TB + tb) * 64 + lane] = acc[tb];
        }
        __syncthreads();
        if (wk == 0) {
#pragma unroll
            for (int tb = 0; tb < TB; ++tb) {
#pragma unroll
                for (int k2 = 1; k2 < NWK; ++k2) acc[tb] += red[(((k2 - 1) * NWR + wr) * TB + tb) * 64 + lane];
            }
        }
    }
    if (wk == 0 && active) {
        // register i is token row 4*j+i of the token block, output column n of the row block
#pragma unroll
        for (int tb = 0; tb < TB; ++tb) {
            const f4 v = acc[tb];
            const float vs[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int m = m0 + 16 * tb + 4 * j + i;
                if (m < a.M) a.y[(size_t)m * a.d_out + R * 16 + n] = (_Float16)vs[i];
            }
        }
    }
    WTL_STAMP(5);
    if constexpr (LOWRANK) {
        if (tid == 0) check_in_finish(ci, a.hdr, gridDim.x);
    }
}

// one linear: the arguments sit at fixed places of the kernel's argument block
template <int FM, int FA, int FE, int NWR, int NWK, int TB>
__global__ __launch_bounds__(NWR * NWK * 64, TB == 1 ? 4 : 2) void wide_q_kernel(FusedArgs a)
{
    wide_q_body<FM, FA, FE, NWR, NWK, TB>(a, blockIdx.x, blockIdx.x, 0);
}

// several linears that share x: each workgroup first finds the member it works for (uniform; one more dependent
// scalar load at the start than the kernel above, which is why that one is kept).  The members' workgroups
// follow one another, each member's producers before its consumers, so a waiting workgroup's producers always
// have lower indices.
template <int FM, int FA, int FE, int NWR, int NWK, int TB>
__global__ __launch_bounds__(NWR * NWK * 64, TB == 1 ? 4 : 2) void wide_q_group_kernel(WideGroupArgs grp)
{
    int mem = 0;
#pragma unroll
    for (int i = 1; i < 4; ++i)
        if (i < grp.n && (int)blockIdx.x >= grp.first[i]) mem = i;
    wide_q_body<FM, FA, FE, NWR, NWK, TB>(grp.m[mem], blockIdx.x, (int)blockIdx.x - grp.first[mem], grp.flag0[mem]);
}

// ------------------------------------------------------------------------------------------------
struct WideCfg { int nwr, nwk, tb; };

// the split of a workgroup into row blocks and ranges, and the token blocks per workgroup, for a shape
static bool pick_wide(int M, int d_in, int d_out, int r, WideCfg* out)
{
    if (M <= 4 || d_in % 512 != 0) return false;
    const int yblocks = (M + 15) / 16, rbs = d_out / 16;
    // More row blocks per workgroup first: x is fetched once per workgroup, and that traffic (workgroups x 16
    // tokens x d_in) is what bounds these launches.  Measured on the 8B shapes: with the low-rank term half as
    // many workgroups as compute units still win; the bare layer wants the chip filled.
    static const int cand[4][2] = {{4, 2}, {2, 4}, {1, 8}, {1, 4}};
    for (int c = 0; c < 4; ++c) {
        const int nwr = cand[c][0], nwk = cand[c][1];
        if (d_in % (512 * nwk) != 0) continue;
        const int need = r > 0 ? 128 : (c == 0 ? 192 : 256);
        const int groups = (rbs + nwr - 1) / nwr;
        if (groups * yblocks >= need) {
            // several token blocks per workgroup (a stored tile is decoded once for all of them, and the weights
            // cross from L2 once per workgroup instead of once per token block) as long as the chip stays filled
            // (192 workgroups, one per compute unit at their register count; measured at 64 tokens on the 8B
            // shapes: the gate projection 39.8 -> 31.9 us with four token blocks per workgroup and 224 workgroups,
            // the 4096-row linears lose with 128)
            int tb = 1;
            if (c == 0) {
                if (yblocks >= 4 && groups * ((yblocks + 3) / 4) >= 192) tb = 4;
                else if (yblocks >= 2 && groups * ((yblocks + 1) / 2) >= 192) tb = 2;
            }
            *out = {nwr, nwk, tb};
            return true;
        }
    }
    return false;                                         // too few rows to fill the chip this way
}

bool wide_q_fits(int M, int d_in, int d_out, int r)
{
    WideCfg c;
    return r <= 512 && pick_wide(M, d_in, d_out, r, &c);
}

template <int NWR, int TB>
static int wide_blocks(const FusedArgs& a, bool lowrank)
{
    const int yblocks = (a.M + 15) / 16;
    const int nprod = lowrank ? (a.r / 16) * a.kcn * yblocks : 0;
    const int nrg = (a.d_out / 16 + NWR - 1) / NWR;
    return nrg * ((yblocks + TB - 1) / TB) + nprod;
}

template <int FM, int FA, int FE, int NWR, int NWK, int TB>
static hipError_t launch_wide_one(const FusedArgs* members, int n, hipStream_t stream)
{
    const FusedArgs& a = members[0];
    const size_t xb = (size_t)NWK * 2 * TB * 4096, tb = (size_t)16 * a.r * 4;
    const size_t lds = xb > tb ? xb : tb;
    note_launch("wide_q FM=%d FA=%d NWR=%d NWK=%d TB=%d n=%d", FM, FA, NWR, NWK, TB, n);
    if (n == 1) {
        auto kern1 = wide_q_kernel<FM, FA, FE, NWR, NWK, TB>;
        if (lds > 48 * 1024) {
            hipError_t e = hipFuncSetAttribute((const void*)kern1, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) return e;
        }
        hipLaunchKernelGGL(kern1, dim3(wide_blocks<NWR, TB>(a, FA != S_NONE)), dim3(NWR * NWK * 64), lds, stream, a);
        return hipGetLastError();
    }
    auto kern = wide_q_group_kernel<FM, FA, FE, NWR, NWK, TB>;
    if (lds > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    WideGroupArgs g{};
    g.n = n;
    int total = 0;
    const int units = (FA != S_NONE) ? (a.r / 16) * a.kcn : 0;
    for (int i = 0; i < 4; ++i) {
        g.m[i] = members[i < n ? i : 0];
        g.first[i] = total;
        g.flag0[i] = (i < n ? i : 0) * units;
        if (i < n) total += wide_blocks<NWR, TB>(members[i], FA != S_NONE);
    }
    hipLaunchKernelGGL(kern, dim3(total), dim3(NWR * NWK * 64), lds, stream, g);
    return hipGetLastError();
}

// one configuration for all members: chosen for the rows of all of them together
static bool pick_wide_group(const FusedArgs* members, int n, WideCfg* c)
{
    int rows = 0;
    for (int i = 0; i < n; ++i) rows += members[i].d_out;
    return pick_wide(members[0].M, members[0].d_in, rows, members[0].r, c);
}

template <int FM, int FA, int FE>
static hipError_t launch_wide_cfg(const FusedArgs* members, int n, hipStream_t stream)
{
    WideCfg c;
    if (!pick_wide_group(members, n, &c)) return hipErrorInvalidValue;
    if (c.nwr == 4 && c.tb == 4) return launch_wide_one<FM, FA, FE, 4, 2, 4>(members, n, stream);
    if (c.nwr == 4 && c.tb == 2) return launch_wide_one<FM, FA, FE, 4, 2, 2>(members, n, stream);
    if (c.nwr == 4) return launch_wide_one<FM, FA, FE, 4, 2, 1>(members, n, stream);
    if (c.nwr == 2) return launch_wide_one<FM, FA, FE, 2, 4, 1>(members, n, stream);
    if (c.nwk == 8) return launch_wide_one<FM, FA, FE, 1, 8, 1>(members, n, stream);
    return launch_wide_one<FM, FA, FE, 1, 4, 1>(members, n, stream);
}

template <int FM>
static hipError_t launch_wide_ab(const FusedArgs* members, int n, int fa, int fe, hipStream_t stream)
{
    if (fe == S_NONE) return launch_wide_cfg<FM, S_NONE, S_NONE>(members, n, stream);
    if (fa == S_F16 && fe == S_F16) return launch_wide_cfg<FM, S_F16, S_F16>(members, n, stream);
    if (fa == S_Q4S128 && fe == S_Q4S128) return launch_wide_cfg<FM, S_Q4S128, S_Q4S128>(members, n, stream);
    if (fa == S_Q4S128 && fe == S_Q4S64) return launch_wide_cfg<FM, S_Q4S128, S_Q4S64>(members, n, stream);
    if (fa == S_Q3S128 && fe == S_Q3S128) return launch_wide_cfg<FM, S_Q3S128, S_Q3S128>(members, n, stream);
    return hipErrorInvalidValue;
}

hipError_t launch_wide_q_group(const FusedArgs* members, int n, int fm, int fa, int fe, hipStream_t stream)
{
    if (n < 1 || n > 4) return hipErrorInvalidValue;
    switch (fm) {
        case S_Q4: return launch_wide_ab<S_Q4>(members, n, fa, fe, stream);
        case S_Q3: return launch_wide_ab<S_Q3>(members, n, fa, fe, stream);
        case S_Q2: return launch_wide_ab<S_Q2>(members, n, fa, fe, stream);
        default: return hipErrorInvalidValue;
    }
}

hipError_t launch_wide_q(const FusedArgs& a, int fm, int fa, int fe, hipStream_t stream)
{
    return launch_wide_q_group(&a, 1, fm, fa, fe, stream);
}

bool wide_q_group_fits(int M, int d_in, const int* d_out, int n, int r)
{
    int rows = 0;
    for (int i = 0; i < n; ++i) rows += d_out[i];
    WideCfg c;
    return n >= 1 && n <= 4 && r <= 512 && pick_wide(M, d_in, rows, r, &c);
}

}  // namespace eora
