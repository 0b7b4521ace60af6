// The compensated layer with a 2:4 structured-sparse fp16 backbone (Sec. 1 and Sec. 4.2 of the
// paper use 2:4 as the pruning format that hardware accelerates):
//
//      y = x.What^T + (x.A^T).B^T          (Sec. 3 forward equation, Alg. 1 step 7)
//
// HBM-bound: 1.125 bytes per dense weight position are read once.  The stored tile of a wavefront
// (16 rows x 128 dense columns: per lane two 16-byte groups of kept values and one word of 2-bit
// positions) is exactly the sparse operand of two v_smfmac_f32_16x16x64_f16, so nothing is expanded
// or decoded: the matrix core skips the pruned positions.  The instruction wants the sparse matrix
// as its row operand, hence the accumulator is D[output row][token] here (lane l: rows 4*(l/16)+i,
// token l%16), the transpose of the quantised kernels' orientation.  Per lane the dense operand of
// block s is x[64s + 8j .. +7] and x[64s + 32 + 8j .. +7] (j = l/16).
//
// Launch structure, flag protocol and the low-rank continuation are those of the decode kernel:
// producer workgroups first (one unit of t = x.A^T each, per token block), then one consumer
// workgroup per (16 output rows, token block of 16).  For 1..4 tokens x is staged in LDS through registers
// (plain loads only); otherwise the fragments come from global memory.
#include "segments.hpp"

namespace eora {

// one stored tile of a wavefront.  VQ: the kept values are 4-bit codes (Sec. 4.2: pruned, then quantised)
template <bool VQ> struct SpT;
template <> struct SpT<false> {
    u4 v0, v1;        // kept values of the two 64-column blocks
    uint32_t idx;     // positions: low 16 bits block 0, high 16 bits block 1
};
template <> struct SpT<true> {
    uint32_t w[3];    // eight codes per block (element e = 2q + v in nibble 4(e%2) + e/2), then the positions
    uint32_t meta;    // fp16 scale | zero-point << 16 of (tile, row n)
};

typedef _Float16 h16 __attribute__((ext_vector_type(16)));

// tile g of row block R (G tiles per row block).  Nothing loaded is touched here.
// ONCE: no other workgroup of the launch reads this tile (non-temporal requests, see load_words).
template <bool VQ, bool ONCE>
__device__ __forceinline__ void load_sptile(SpT<VQ>& t, const SparseArgs& a, int R, int g, int G, int lane)
{
    const size_t tile = (size_t)R * G + g;
    if constexpr (!VQ) {
        const u4* p = (const u4*)(a.values + tile * 1024) + lane;
        if constexpr (ONCE) {
            t.idx = __builtin_nontemporal_load(a.indices + tile * 64 + lane);
            t.v0 = __builtin_nontemporal_load(p);
            t.v1 = __builtin_nontemporal_load(p + 64);
        } else {
            t.idx = a.indices[tile * 64 + lane];
            t.v0 = p[0];
            t.v1 = p[64];
        }
    } else {
        load_words<3, ONCE>(t.w, a.qtiles + (tile * 64 + lane) * 3);       // one 12-byte request
        t.meta = a.qmeta[tile * 16 + (lane & 15)];
    }
}

__device__ __forceinline__ h8 as_h8(u4 v) { return __builtin_bit_cast(h8, v); }

__device__ __forceinline__ int sp_idx(const SpT<false>& t) { return (int)t.idx; }
__device__ __forceinline__ int sp_idx(const SpT<true>& t) { return (int)t.w[2]; }

// the sparse operands of the tile's two blocks.  Quantised: code - zero exact, times the fp16 group scale
// (one fp16 rounding of scale*(code - zero), relative error <= 2^-11 per weight: the accumulator holds four
// rows per lane, so scaling it per group instead would need four row scales per lane and tile).
template <bool VQ>
__device__ __forceinline__ void sp_operands(const SpT<VQ>& t, h8& a0, h8& a1)
{
    if constexpr (!VQ) {
        a0 = as_h8(t.v0);
        a1 = as_h8(t.v1);
    } else {
        const uint32_t z = (t.meta >> 16) & 0xFu;
        const uint32_t c1024 = k1024(z), c64 = k64(z);
        const _Float16 sc = __builtin_bit_cast(_Float16, (uint16_t)(t.meta & 0xFFFFu));
        const h8 sv = {sc, sc, sc, sc, sc, sc, sc, sc};
        a0 = dq4_word(t.w[0], c1024, c64) * sv;
        a1 = dq4_word(t.w[1], c1024, c64) * sv;
    }
}

// the token block's x (mt <= 4 rows of d_in fp16) -> LDS, rows padded by 64 bytes, through registers: all
// requests of the kernel stay plain loads (with global -> LDS copies among them the compiler no longer counts
// on in-order answers and drains every request before each use)
template <int NW>
__device__ __forceinline__ void stage_x(const _Float16* __restrict__ x, int mt, int d_in, int tid)
{
    constexpr int T = NW * 64;
    const int ppr = d_in / 8;                             // 16-byte pieces per row
    for (int row = 0; row < mt; ++row) {                  // one row at a time: few registers
        const _Float16* src = x + (size_t)row * d_in;
        unsigned char* d = eora_smem + (size_t)row * (d_in + 32) * 2;
        for (int p0 = tid; p0 < ppr; p0 += 2 * T) {
            const int p1 = p0 + T < ppr ? p0 + T : p0;
            const u4 v0 = *(const u4*)(src + p0 * 8);
            const u4 v1 = *(const u4*)(src + p1 * 8);
            *(u4*)(d + p0 * 16) = v0;
            if (p0 + T < ppr) *(u4*)(d + p1 * 16) = v1;
        }
    }
}

// gbid: index of the workgroup in the launch; bid: its index among its member's workgroups; flag0: the member's
// first flag inside a token block's flags (one linear: gbid == bid, flag0 == 0)
template <int FA, int FE, int NW, bool XLDS, bool VQ>
__device__ __forceinline__ void sparse_body(const SparseArgs& a, const int gbid, const int bid, const int flag0)
{
    constexpr bool LOWRANK = FA != S_NONE;
    constexpr int PD = 4;                                 // tiles of loads in flight per wavefront
    // one buffer for the cross-wavefront sums: producers and consumers are different workgroups
    __shared__ f4 red_raw[NW][64];
    f4 (*red)[64] = red_raw;
    float (*redp)[16][16] = (float (*)[16][16])red_raw;
    __shared__ uint32_t s_epoch, s_ok;

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int n = lane & 15, j = lane >> 4;
    const int yblocks = (a.M + 15) / 16;
    const int units = LOWRANK ? (a.r / 16) * a.kcn : 0;
    const int nprod = units * yblocks;
    const bool producer = bid < nprod;
    // Consumers: workgroups are handed to the 8 XCDs round-robin, each with an L2 of its own.  With several
    // token blocks the blocks of one row block are therefore given indices 8 apart: they land on the same
    // XCD one after the other and the row block's weights come from HBM once, not once per token block.
    const int cidx = bid - nprod;
    const bool xcd_map = yblocks > 1 && (a.d_out / 16) % 8 == 0;
    const int c_yb = xcd_map ? (cidx / 8) % yblocks : cidx % yblocks;
    const int c_R = xcd_map ? (cidx / (8 * yblocks)) * 8 + cidx % 8 : cidx / yblocks;
    const int yb = producer ? bid / (units > 0 ? units : 1) : c_yb;
    const int m_blk = 16 * yb;
    const int mt = a.M - m_blk < 16 ? a.M - m_blk : 16;
    const int mrow = n < mt ? n : 0;                      // lanes beyond the tokens re-read row 0; results dropped
    const int ldxs = a.d_in + 32;
    const _Float16* xg = a.x + (size_t)m_blk * a.d_in;
    const ActSrc<XLDS> act{xg, a.d_in, 0, ldxs};
    float* ts = (float*)(eora_smem + (XLDS ? (size_t)mt * ldxs * 2 : 0));      // t of this token block: 16 x r fp32

    CheckIn ci{0u, 0u, 0u};
    if constexpr (LOWRANK) {
        if (tid == 0) check_in_load(ci, a.hdr);           // first request: it returns first
    }
    if constexpr (LOWRANK) {
        if (producer) {
            // ===================================================================== producer
            constexpr int KTA = Fmt<FA>::KT;
            const int NRB = a.r / 16;
            const int u = bid % units, rho = u % NRB, kc = u / NRB;
            const Factor fa{(const uint32_t*)a.A, nullptr, a.d_in / KTA};
            const int tpc = fa.ntk / a.kcn;
            if (tid == 0) {
                check_in_issue(ci, a.hdr, gbid);
                s_epoch = ci.epoch;
            }
            if constexpr (XLDS) stage_x<NW>(xg, mt, a.d_in, tid);
            __syncthreads();
            const f4 part = run_factor_a<FA, NW, XLDS>(fa, rho, kc * tpc, (kc + 1) * tpc, wave, lane, act, mrow, true);
#pragma unroll
            for (int i = 0; i < 4; ++i) redp[wave][4 * j + i][n] = part[i];       // register i is token row 4*j+i, column n
            __syncthreads();
            if (tid < 256) {
                const int i = tid >> 4, col = tid & 15;
                if (i < mt) {
                    float v = 0.f;
#pragma unroll
                    for (int w2 = 0; w2 < NW; ++w2) v += redp[w2][i][col];
                    // partial layout: [token block][kc][token row (16)][r], every element an 8-byte
                    // (value, epoch + 1) pair written by ONE write-through store: a reader that finds this
                    // launch's tag has this launch's value, so the flag need not wait for acknowledgements
                    const unsigned long long pr = ((unsigned long long)(s_epoch + 1) << 32) | __builtin_bit_cast(uint32_t, v);
                    __hip_atomic_store(&a.tpair[((size_t)(yb * a.kcn + kc) * 16 + i) * a.r + 16 * rho + col], pr,
                                       __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
            }
            __syncthreads();                                      // all pairs are on their way
            if (tid == 0) {
                for (int rep = 0; rep < HDR_FLAG_REPLICAS; ++rep)  // one copy per group of pollers
                    __hip_atomic_store(&a.hdr[HDR_FLAGS0 + HDR_FLAGS_REPLICA_STRIDE * rep + HDR_FLAGS_PER_BLOCK * yb + flag0 + u],
                                       s_epoch + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                check_in_finish(ci, a.hdr, gridDim.x);
            }
            return;
        }
    }

    // ========================================================================= consumer
    const int R = c_R;
    const int G = a.d_in / 128;
    const int nsteps = wave < G ? (G - wave + NW - 1) / NW : 0;
    // step s of this wavefront is stored tile wave + s NW of the row block; requests past the end fetch the
    // last one again (never used): every step issues the same requests, refilled into the registers just used
    const int last = nsteps > 0 ? nsteps - 1 : 0;
    const int g_first = nsteps > 0 ? wave : 0;
    SpT<VQ> buf[PD];
#pragma unroll
    for (int s = 0; s < PD; ++s) load_sptile<VQ, XLDS>(buf[s], a, R, g_first + (s < nsteps ? s : last) * NW, G, lane);
    const Factor fb{(const uint32_t*)a.B, nullptr, LOWRANK ? a.r / 32 : 0};
    FTile<S_F16> bpre;
    if constexpr (LOWRANK) load_ftile<S_F16, XLDS>(bpre, fb, R, wave < fb.ntk ? wave : 0, lane);
    if constexpr (LOWRANK) {
        if (tid == 0) {
            check_in_issue(ci, a.hdr, gbid);
            s_epoch = ci.epoch;
        }
    }
    // a first look at the flags, examined after the backbone: for all but the first workgroups on a CU the
    // producers are done by now and the wait below costs no round trip
    uint32_t early = 0;
    if constexpr (LOWRANK) {
        if (wave == 0)
            early = ld_relaxed(a.hdr + HDR_FLAGS0 + HDR_FLAGS_REPLICA_STRIDE * (blockIdx.x % HDR_FLAG_REPLICAS) +
                               HDR_FLAGS_PER_BLOCK * yb + flag0 + (lane < units ? lane : units - 1));
    }
    if constexpr (XLDS) {
        stage_x<NW>(xg, mt, a.d_in, tid);
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");           // own LDS writes done; tile requests stay in flight
        __builtin_amdgcn_s_barrier();
    } else {
        __syncthreads();
    }

    f4 acc = {0.f, 0.f, 0.f, 0.f};
    for (int base = 0; base < nsteps; base += PD) {
#pragma unroll
        for (int s = 0; s < PD; ++s) {
            if (base + s < nsteps) {
                const int g = wave + (base + s) * NW;
                h8 sa[2];
                sp_operands<VQ>(buf[s], sa[0], sa[1]);
#pragma unroll
                for (int blk = 0; blk < 2; ++blk) {
                    h8 x0, x1;
                    const int col = g * 128 + 64 * blk + 8 * j;
                    if constexpr (XLDS) {
                        const _Float16* px = (const _Float16*)eora_smem + mrow * ldxs + col;
                        x0 = *(const h8*)px;
                        x1 = *(const h8*)(px + 32);
                    } else {
                        const _Float16* px = xg + (size_t)mrow * a.d_in + col;
                        x0 = *(const h8*)px;
                        x1 = *(const h8*)(px + 32);
                    }
                    const h16 xb = __builtin_shufflevector(x0, x1, 0, 1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11, 12, 13, 14, 15);
                    if (blk == 0) acc = __builtin_amdgcn_smfmac_f32_16x16x64_f16(sa[0], xb, acc, sp_idx(buf[s]), 0, 0);
                    else acc = __builtin_amdgcn_smfmac_f32_16x16x64_f16(sa[1], xb, acc, sp_idx(buf[s]), 0, 1);
                }
            }
            __builtin_amdgcn_sched_barrier(0);
            const int sn = base + s + PD;
            load_sptile<VQ, XLDS>(buf[s], a, R, g_first + (sn < nsteps ? sn : last) * NW, G, lane);
        }
    }

    // ---- low-rank continuation: acc[row][token] += B[row][:] . t[token][:] -------------------------
    if constexpr (LOWRANK) {
        const uint32_t epoch = s_epoch;
        if (wave == 0) {
            const uint32_t* flags = a.hdr + HDR_FLAGS0 + HDR_FLAGS_REPLICA_STRIDE * (blockIdx.x % HDR_FLAG_REPLICAS) + HDR_FLAGS_PER_BLOCK * yb + flag0;
            bool ok = a.spin_limit >= 0 && units <= 64 && __all(early == epoch + 1);      // a negative limit: every wait counts as expired (test hook)
            for (int spins = 0; !ok && spins <= a.spin_limit; ++spins) {
                bool all = true;
                for (int f = lane; f < units; f += 64) all = all && (ld_relaxed(&flags[f]) == epoch + 1);
                if (__all(all)) { ok = true; break; }
                __builtin_amdgcn_s_sleep(2);
            }
            if (ok) {
                // The partials are read with ordinary (cached) loads first: the flags are up, so their stores
                // were issued long ago and have all but certainly landed, and caches hold nothing of them from
                // before the launch.  The tags say whether that held; a lane that finds an old tag reads again
                // past the caches until it does (bounded).
                const int T = mt * a.r;                  // a.r is a multiple of 32
                for (int e = 4 * lane; e < T; e += 256) {
                    const unsigned long long* p = a.tpair + ((size_t)(yb * a.kcn) * 16) * a.r + e;     // row e / r, column e % r
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
            if (lane == 0) {
                s_ok = ok ? 1u : 0u;
                if (!ok) atomicOr(&a.hdr[HDR_ERROR], 1u);
            }
        }
        __syncthreads();
        if (s_ok) {
            for (int g = wave; g < fb.ntk; g += NW) {
                FTile<S_F16> cur;
                if (g == wave) cur = bpre;
                else load_ftile<S_F16, XLDS>(cur, fb, R, g, lane);
                h8 b[1];
                decode_tile<S_F16>(cur.w, 0u, b);
                const float* p = ts + mrow * a.r + g * 32 + 8 * j;
                const f4 v0 = *(const f4*)p, v1 = *(const f4*)(p + 4);
                h8 hi, lo;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const _Float16 h0 = (_Float16)v0[i], h1 = (_Float16)v1[i];
                    hi[i] = h0;
                    hi[4 + i] = h1;
                    lo[i] = (_Float16)(v0[i] - (float)h0);
                    lo[4 + i] = (_Float16)(v1[i] - (float)h1);
                }
                acc = mfma16(b[0], hi, acc);             // B's rows are the row operand, t the column operand
                acc = mfma16(b[0], lo, acc);
            }
        }
    }

    // ---- combine, convert, store: lane holds rows 4*j+i of the strip for token n ----------------------
    red[wave][lane] = acc;
    __syncthreads();
    if (wave == 0) {
        f4 v = red[0][lane];
#pragma unroll
        for (int w2 = 1; w2 < NW; ++w2) v += red[w2][lane];
        if (n < mt) {
            typedef _Float16 h4 __attribute__((ext_vector_type(4)));
            const h4 o = {(_Float16)v[0], (_Float16)v[1], (_Float16)v[2], (_Float16)v[3]};
            *(h4*)(a.y + (size_t)(m_blk + n) * a.d_out + R * 16 + 4 * j) = o;
        }
    }
    if constexpr (LOWRANK) {
        if (tid == 0) check_in_finish(ci, a.hdr, gridDim.x);
    }
}


// ---------------------------------------------------------------------------------------------------
// More than 4 tokens and many output rows: one wavefront per row block (whole contraction length), NW row
// blocks and up to TB token blocks of 16 per workgroup.  A token block's x is 1.8x the bytes of a row
// block's weights, so x is shared through LDS by the NW wavefronts, and a stored tile, once in registers,
// serves all TB token blocks.  Per step one 128-column chunk: x[16 TB tokens][128] goes global ->
// registers (requested XW_D steps before its LDS write) -> one of two LDS slots, and the wavefront's stored
// tile of the same columns is requested XW_D steps ahead as well.  All requests are plain loads: with
// global -> LDS copies among them the compiler would no longer count on in-order answers and would drain
// every request before each use.  One barrier per step: after it chunk c is visible to everyone and
// everyone has left the other slot, which is rewritten at once.
//
// LDS slot layout: 16-byte piece q of token row t (columns 8q .. 8q+7 of the chunk) sits at piece index
// 16 t + (q ^ (t & 15)): the 16 lanes that read one q for 16 tokens hit 16 different bank groups.
// Producers, flags, partials and the continuation are those of the kernel above.
template <int FA, int NW, int TB, int XW_D, bool VQ, bool ONCE>      // XW_D: steps between a request and its use; divides d_in / 128; ONCE: one group of token blocks, so every stored tile is read by one workgroup
__device__ __forceinline__ void sparse_wide_body(const SparseArgs& a, const int gbid, const int bid, const int flag0)
{
    constexpr bool LOWRANK = FA != S_NONE;
    constexpr int SLOT = TB * 16 * 256;                   // bytes per slot
    constexpr int NCP = TB * 4;                           // 1 KiB pieces of a chunk of x (4 token rows each)
    static_assert(NCP % NW == 0, "the pieces divide evenly over the wavefronts");
    constexpr int XN = NCP / NW;                          // per wavefront
    __shared__ float redp[NW][16][16];
    __shared__ uint32_t s_epoch, s_ok;

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int n = lane & 15, j = lane >> 4;
    const int yblocks = (a.M + 15) / 16;
    const int units = LOWRANK ? (a.r / 16) * a.kcn : 0;
    const int nprod = units * yblocks;
    const bool producer = bid < nprod;

    CheckIn ci{0u, 0u, 0u};
    if constexpr (LOWRANK) {
        if (tid == 0) check_in_load(ci, a.hdr);
        if (producer) {
            // ===================================================================== producer
            constexpr int KTA = Fmt<FA>::KT;
            const int yb = bid / units;
            const int m_blk = 16 * yb;
            const int mt = a.M - m_blk < 16 ? a.M - m_blk : 16;
            const int mrow = n < mt ? n : 0;
            const ActSrc<false> act{a.x + (size_t)m_blk * a.d_in, a.d_in, 0, 0};
            const int NRB = a.r / 16;
            const int u = bid % units, rho = u % NRB, kc = u / NRB;
            const Factor fa{(const uint32_t*)a.A, nullptr, a.d_in / KTA};
            const int tpc = fa.ntk / a.kcn;
            if (tid == 0) {
                check_in_issue(ci, a.hdr, gbid);
                s_epoch = ci.epoch;
            }
            __syncthreads();
            const f4 part = run_factor_a<FA, NW, false>(fa, rho, kc * tpc, (kc + 1) * tpc, wave, lane, act, mrow, true);
#pragma unroll
            for (int i = 0; i < 4; ++i) redp[wave][4 * j + i][n] = part[i];
            __syncthreads();
            for (int e = tid; e < 256; e += NW * 64) {
                const int i = e >> 4, col = e & 15;
                if (i < mt) {
                    float v = 0.f;
#pragma unroll
                    for (int w2 = 0; w2 < NW; ++w2) v += redp[w2][i][col];
                    *(volatile float*)&a.tpart[((size_t)(yb * a.kcn + kc) * 16 + i) * a.r + 16 * rho + col] = v;
                }
            }
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");      // write-through stores acknowledged
            __syncthreads();
            if (tid == 0) {
                for (int rep = 0; rep < HDR_FLAG_REPLICAS; ++rep)
                    __hip_atomic_store(&a.hdr[HDR_FLAGS0 + HDR_FLAGS_REPLICA_STRIDE * rep + HDR_FLAGS_PER_BLOCK * yb + flag0 + u],
                                       s_epoch + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                check_in_finish(ci, a.hdr, gridDim.x);
            }
            return;
        }
    }

    // ========================================================================= consumer
    const int RBs = a.d_out / 16;
    const int NTG = (yblocks + TB - 1) / TB;              // groups of TB token blocks
    // ranges of the contraction (a.ksplit > 1: a long contraction with few rows): range ks of KS covers chunks
    // [c0, c0 + Gs); every range writes its fp32 partial output, the launcher's second kernel adds them in order
    const int KS = a.ksplit, ks = (bid - nprod) % KS;
    const int cidx = (bid - nprod) / KS;
    const int tg = cidx % NTG, rg = cidx / NTG;
    const int m0 = tg * TB * 16;                          // first token of the group
    const int Rw = rg * NW + wave;
    const bool active = Rw < RBs;                         // a ragged last row group: the wavefront only helps staging
    const int R = active ? Rw : RBs - 1;
    const int G = a.d_in / 128;                           // chunks = stored tiles per row block
    const int Gs = G / KS, c0 = ks * Gs;                  // this range's chunks
    // piece q of a chunk: token rows 4 q .. 4 q + 3, lane -> row 4 q + lane / 16, 16-byte piece lane % 16
    const _Float16* xsrc[XN];
    int xdst[XN];
#pragma unroll
    for (int i = 0; i < XN; ++i) {
        const int trow = 4 * (wave + i * NW) + (lane >> 4);
        const int grow = m0 + trow < a.M ? m0 + trow : a.M - 1;      // rows beyond the tokens: a valid row, results dropped
        xsrc[i] = a.x + (size_t)grow * a.d_in + (size_t)c0 * 128 + 8 * (lane & 15);      // (chunk s of the range at + s * 128)
        xdst[i] = (trow * 16 + ((lane & 15) ^ (trow & 15))) * 16;
    }
    auto load_tile = [&](SpT<VQ>& t, int c) { load_sptile<VQ, ONCE>(t, a, R, c0 + c, G, lane); };      // c: chunk within the range
    SpT<VQ> buf[XW_D];
    u4 xr[XW_D][XN];
#pragma unroll
    for (int s = 0; s < XW_D; ++s) {                      // Gs is a multiple of XW_D
#pragma unroll
        for (int i = 0; i < XN; ++i) xr[s][i] = *(const u4*)(xsrc[i] + s * 128);
        load_tile(buf[s], s);
    }
    if constexpr (LOWRANK) {
        if (tid == 0) {
            check_in_issue(ci, a.hdr, gbid);
            s_epoch = ci.epoch;
        }
    }
    // chunk 0 -> slot 0; its registers take chunk XW_D
#pragma unroll
    for (int i = 0; i < XN; ++i) {
        *(u4*)(eora_smem + xdst[i]) = xr[0][i];
        xr[0][i] = *(const u4*)(xsrc[i] + (XW_D < Gs ? XW_D : Gs - 1) * 128);
    }

    f4 acc[TB];
#pragma unroll
    for (int tb = 0; tb < TB; ++tb) acc[tb] = f4{0.f, 0.f, 0.f, 0.f};
    // piece offsets of this lane's four dense-operand reads of a token block: (blk, half) -> piece 8 blk + 4 half + j
    int poff[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) poff[q] = (n * 16 + ((8 * (q >> 1) + 4 * (q & 1) + j) ^ n)) * 16;

    for (int base = 0; base < Gs; base += XW_D) {
#pragma unroll
        for (int s = 0; s < XW_D; ++s) {
            const int c = base + s;
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");       // own LDS writes of chunk c done
            __builtin_amdgcn_s_barrier();
            // chunk c + 1 -> the slot everyone has just left; its registers take the chunk XW_D further on
            // (past the end: the last chunk again, never used)
            const int s1 = (s + 1) % XW_D;
            const int cx = c + 1 + XW_D < Gs ? c + 1 + XW_D : Gs - 1;
#pragma unroll
            for (int i = 0; i < XN; ++i) {
                *(u4*)(eora_smem + ((c + 1) & 1) * SLOT + xdst[i]) = xr[s1][i];
                xr[s1][i] = *(const u4*)(xsrc[i] + cx * 128);
            }
            __builtin_amdgcn_sched_barrier(0);
            const unsigned char* xs = eora_smem + (c & 1) * SLOT;
            h8 sa0, sa1;
            sp_operands<VQ>(buf[s], sa0, sa1);
#pragma unroll
            for (int tb = 0; tb < TB; ++tb) {
                const unsigned char* px = xs + tb * 4096;
                const h8 x00 = *(const h8*)(px + poff[0]), x01 = *(const h8*)(px + poff[1]);
                const h8 x10 = *(const h8*)(px + poff[2]), x11 = *(const h8*)(px + poff[3]);
                const h16 xa = __builtin_shufflevector(x00, x01, 0, 1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11, 12, 13, 14, 15);
                const h16 xb = __builtin_shufflevector(x10, x11, 0, 1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11, 12, 13, 14, 15);
                acc[tb] = __builtin_amdgcn_smfmac_f32_16x16x64_f16(sa0, xa, acc[tb], sp_idx(buf[s]), 0, 0);
                acc[tb] = __builtin_amdgcn_smfmac_f32_16x16x64_f16(sa1, xb, acc[tb], sp_idx(buf[s]), 0, 1);
            }
            // the tile's registers are free again: the request for the tile XW_D chunks on goes out last
            __builtin_amdgcn_sched_barrier(0);
            load_tile(buf[s], c + XW_D < Gs ? c + XW_D : Gs - 1);
        }
    }

    // ---- low-rank continuation: acc[row][token] += B[row][:] . t[token][:] (range 0 adds it) ----------------
    if constexpr (LOWRANK) {
      if (ks == 0) {
        // t (16 x r fp32 per token block) goes over the x slots, as many token blocks at a time as fit
        float* ts = (float*)eora_smem;
        const int tsz = 16 * a.r;                         // floats per token block
        const int lds_floats = 2 * SLOT / 4 > tsz ? 2 * SLOT / 4 : tsz;
        const int nb = lds_floats / tsz;                  // >= 1
        const Factor fb{(const uint32_t*)a.B, nullptr, a.r / 32};
        constexpr int BPRE = 4;                           // B's first tiles are requested before the wait for t
        FTile<S_F16> bt[BPRE];
#pragma unroll
        for (int g = 0; g < BPRE; ++g) load_ftile<S_F16, ONCE>(bt[g], fb, R, g < fb.ntk ? g : 0, lane);
        __syncthreads();                                  // nobody reads x any more
        const uint32_t epoch = s_epoch;
        if (wave == 0) {
            bool ok = true;
#pragma unroll
            for (int tb = 0; tb < TB; ++tb) {
                const int yb = tg * TB + tb;
                if (yb >= yblocks || !ok) continue;
                const uint32_t* flags = a.hdr + HDR_FLAGS0 + HDR_FLAGS_REPLICA_STRIDE * (blockIdx.x % HDR_FLAG_REPLICAS) + HDR_FLAGS_PER_BLOCK * yb + flag0;
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
                if (!ok) atomicOr(&a.hdr[HDR_ERROR], 1u);
            }
        }
        __syncthreads();
        if (s_ok) {
            // ordinary cached loads: the partials were written through before their flags, none of their
            // lines is read in this launch before all flags are up, caches hold nothing older
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
#pragma unroll
            for (int tb = 0; tb < TB; ++tb) {
                if (tb % nb == 0) {                       // uniform over the workgroup: the next nb token blocks' t
                    if (tb > 0) __syncthreads();          // the previous ones have been used
                    for (int q = 0; q < nb && tb + q < TB; ++q) {
                        const int yq = tg * TB + tb + q;
                        if (yq >= yblocks) break;
                        const int mq = a.M - 16 * yq < 16 ? a.M - 16 * yq : 16;
                        const int T = mq * a.r;
                        for (int e = 4 * tid; e < T; e += NW * 256) {
                            const float* p = a.tpart + ((size_t)(yq * a.kcn) * 16) * a.r + e;
                            f4 v = {0.f, 0.f, 0.f, 0.f};
#pragma unroll 4
                            for (int kc = 0; kc < a.kcn; ++kc) v += *(const f4*)(p + (size_t)kc * 16 * a.r);   // fixed order
                            *(f4*)(ts + q * tsz + e) = v;
                        }
                    }
                    __syncthreads();
                }
                const int yb = tg * TB + tb;
                if (yb < yblocks) {
                    const int mt = a.M - 16 * yb < 16 ? a.M - 16 * yb : 16;
                    const int mrow = n < mt ? n : 0;
                    const float* tq = ts + (tb % nb) * tsz + mrow * a.r + 8 * j;
                    auto contract = [&](const FTile<S_F16>& cur, int g) {
                        h8 b[1];
                        decode_tile<S_F16>(cur.w, 0u, b);
                        const float* p = tq + g * 32;
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
                        acc[tb] = mfma16(b[0], hi, acc[tb]);
                        acc[tb] = mfma16(b[0], lo, acc[tb]);
                    };
#pragma unroll
                    for (int g = 0; g < BPRE; ++g)
                        if (g < fb.ntk) contract(bt[g], g);
                    for (int g = BPRE; g < fb.ntk; ++g) {
                        FTile<S_F16> cur;
                        load_ftile<S_F16, ONCE>(cur, fb, R, g, lane);
                        contract(cur, g);
                    }
                }
            }
        }
      }
    }

    // ---- convert, store: lane holds rows 4*j+i of its row block for token n of each token block ----------
#pragma unroll
    for (int tb = 0; tb < TB; ++tb) {
        const int m = m0 + 16 * tb + n;
        if (active && m < a.M) {
            const f4 v = acc[tb];
            if (KS > 1) {                                 // this range's fp32 partial output
                *(f4*)(a.ypart + ((size_t)ks * a.M + m) * a.d_out + R * 16 + 4 * j) = v;
            } else {
                typedef _Float16 h4 __attribute__((ext_vector_type(4)));
                const h4 o = {(_Float16)v.x, (_Float16)v.y, (_Float16)v.z, (_Float16)v.w};
                *(h4*)(a.y + (size_t)m * a.d_out + R * 16 + 4 * j) = o;
            }
        }
    }
    if constexpr (LOWRANK) {
        if (tid == 0) check_in_finish(ci, a.hdr, gridDim.x);
    }
}

// One linear: the arguments sit at fixed places of the kernel's argument block.  Several linears that share x
// (SparseGroupArgs): each workgroup first finds its member (uniform; one more dependent scalar load at the
// start, which is why single linears keep kernels of their own); the members' workgroups follow one another,
// each member's producers before its consumers, so a waiting workgroup's producers always have lower indices.
__device__ __forceinline__ int sparse_member(const SparseGroupArgs& grp)
{
    int mem = 0;
#pragma unroll
    for (int i = 1; i < 4; ++i)
        if (i < grp.n && (int)blockIdx.x >= grp.first[i]) mem = i;
    return mem;
}

template <int FA, int FE, int NW, bool XLDS, bool VQ>
__global__ __launch_bounds__(NW * 64, 6) void sparse_kernel(SparseArgs a)
{
    sparse_body<FA, FE, NW, XLDS, VQ>(a, blockIdx.x, blockIdx.x, 0);
}

template <int FA, int FE, int NW, bool XLDS, bool VQ>
__global__ __launch_bounds__(NW * 64, 6) void sparse_group_kernel(SparseGroupArgs grp)
{
    const int mem = sparse_member(grp);
    sparse_body<FA, FE, NW, XLDS, VQ>(grp.m[mem], blockIdx.x, (int)blockIdx.x - grp.first[mem], grp.flag0[mem]);
}

template <int FA, int NW, int TB, int XW_D, bool VQ, bool ONCE>
__global__ __launch_bounds__(NW * 64) void sparse_wide_kernel(SparseArgs a)
{
    sparse_wide_body<FA, NW, TB, XW_D, VQ, ONCE>(a, blockIdx.x, blockIdx.x, 0);
}

template <int FA, int NW, int TB, int XW_D, bool VQ, bool ONCE>
__global__ __launch_bounds__(NW * 64) void sparse_wide_group_kernel(SparseGroupArgs grp)
{
    const int mem = sparse_member(grp);
    sparse_wide_body<FA, NW, TB, XW_D, VQ, ONCE>(grp.m[mem], blockIdx.x, (int)blockIdx.x - grp.first[mem], grp.flag0[mem]);
}

// fills the member table; blocks(i) = workgroups of member i
template <typename F>
static int fill_group(SparseGroupArgs& g, const SparseArgs* members, int n, int units, F blocks)
{
    g.n = n;
    int total = 0;
    for (int i = 0; i < 4; ++i) {
        g.m[i] = members[i < n ? i : 0];
        g.first[i] = total;
        g.flag0[i] = (i < n ? i : 0) * units;
        if (i < n) total += blocks(members[i]);
    }
    return total;
}

template <int FA, int NW, int TB, int XW_D, bool VQ, bool ONCE = false>
static hipError_t launch_sparse_wide(const SparseArgs* members, int n, hipStream_t stream)
{
    const SparseArgs& a = members[0];
    const size_t xb = (size_t)2 * TB * 4096, tb = (size_t)16 * a.r * 4;
    const size_t lds = xb > tb ? xb : tb;
    const int yblocks = (a.M + 15) / 16;
    const int units = (FA != S_NONE) ? (a.r / 16) * a.kcn : 0;
    auto blocks = [&](const SparseArgs& m) { return ((m.d_out / 16 + NW - 1) / NW) * ((yblocks + TB - 1) / TB) * m.ksplit + units * yblocks; };
    note_launch("sparse_wide FA=%d NW=%d TB=%d VQ=%d n=%d ksplit=%d", FA, NW, TB, (int)VQ, n, a.ksplit);
    if (n == 1) {
        auto kern = sparse_wide_kernel<FA, NW, TB, XW_D, VQ, ONCE>;
        if (lds > 48 * 1024) {
            hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) return e;
        }
        hipLaunchKernelGGL(kern, dim3(blocks(a)), dim3(NW * 64), lds, stream, a);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess || a.ksplit == 1) return e;
        // y = fp16(sum of the ranges' partial outputs, in the order of the ranges)
        return launch_reduce_parts(a.ypart, a.y, (size_t)a.M * a.d_out, a.ksplit, stream);
    }
    auto kern = sparse_wide_group_kernel<FA, NW, TB, XW_D, VQ, ONCE>;
    if (lds > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    SparseGroupArgs g{};
    const int total = fill_group(g, members, n, units, blocks);
    hipLaunchKernelGGL(kern, dim3(total), dim3(NW * 64), lds, stream, g);
    return hipGetLastError();
}

size_t sparse_split_bytes(int M, int d_in, int d_out)
{
    if (M <= 4 || M >= 128 || d_in < SP_SPLIT_MIN_D_IN) return 0;
    return (size_t)SP_MAX_SPLIT * M * d_out * sizeof(float);
}

template <int FA, bool VQ>
static hipError_t launch_sparse_wide_cfg(const SparseArgs* members, int n, int nw, int tb, hipStream_t stream)
{
    // up to 64 tokens in workgroups of four token blocks: every stored tile is read by one workgroup, once
    // (70B 2:4 layer at 64 tokens: gate+up 120.7 -> 110.2 us with non-temporal requests; the launches in which two
    // groups of token blocks read the same tiles lose 6-10 % with them and keep ordinary loads)
    const bool once = members[0].M <= 16 * tb;
    if (nw == 16) return once ? launch_sparse_wide<FA, 16, 4, 4, VQ, true>(members, n, stream)       // sixteen row blocks: four token blocks (one 1 KiB piece per wavefront)
                              : launch_sparse_wide<FA, 16, 4, 4, VQ>(members, n, stream);
    if (nw == 8) {                                        // eight row blocks: two or four token blocks (whole 1 KiB pieces per wavefront)
        if (tb == 2) return launch_sparse_wide<FA, 8, 2, 4, VQ>(members, n, stream);
        return once ? launch_sparse_wide<FA, 8, 4, 4, VQ, true>(members, n, stream) : launch_sparse_wide<FA, 8, 4, 4, VQ>(members, n, stream);
    }
    // four row blocks: one or two token blocks (with three or four of them the eight-row-block split above
    // always has its 192 workgroups too, and comes first)
    if (tb == 2) return launch_sparse_wide<FA, 4, 2, 4, VQ>(members, n, stream);
    if (tb == 1) return launch_sparse_wide<FA, 4, 1, 4, VQ>(members, n, stream);
    return hipErrorInvalidValue;
}

template <int FA, int FE, int NW, bool XLDS, bool VQ>
static hipError_t launch_sparse_one(const SparseArgs* members, int n, hipStream_t stream)
{
    const SparseArgs& a = members[0];
    const int mt = a.M < 16 ? a.M : 16;
    const size_t lds = (XLDS ? (size_t)mt * (a.d_in + 32) * 2 : 0) + (size_t)mt * a.r * 4;      // x, then t
    const int yblocks = (a.M + 15) / 16;
    const int units = (FA != S_NONE) ? (a.r / 16) * a.kcn : 0;
    auto blocks = [&](const SparseArgs& m) { return (m.d_out / 16) * yblocks + units * yblocks; };
    note_launch("sparse FA=%d NW=%d XLDS=%d VQ=%d n=%d", FA, NW, (int)XLDS, (int)VQ, n);
    if (n == 1) {
        auto kern = sparse_kernel<FA, FE, NW, XLDS, VQ>;
        if (lds > 48 * 1024) {
            hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) return e;
        }
        hipLaunchKernelGGL(kern, dim3(blocks(a)), dim3(NW * 64), lds, stream, a);
        return hipGetLastError();
    }
    auto kern = sparse_group_kernel<FA, FE, NW, XLDS, VQ>;
    if (lds > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    SparseGroupArgs g{};
    const int total = fill_group(g, members, n, units, blocks);
    hipLaunchKernelGGL(kern, dim3(total), dim3(NW * 64), lds, stream, g);
    return hipGetLastError();
}

template <bool VQ>
static hipError_t launch_sparse_vq(const SparseArgs* members, int n, hipStream_t stream)
{
    const SparseArgs& a = members[0];
    // x in LDS for 1..4 tokens when it fits next to t (d_in a multiple of 512 for the 1 KiB copy chunks)
    const bool xlds = a.M <= 4 && a.d_in % 512 == 0 && (size_t)a.M * (a.d_in + 32) * 2 + a.M * (size_t)a.r * 4 <= 140 * 1024;
    // Several tokens and enough row groups: x shared through LDS.  A workgroup fetches all of its token
    // blocks' x, so more row blocks (8, then 4) and more token blocks (4, 2, 1) per workgroup come first, as
    // long as 192 (eight row blocks) or 256 workgroups remain (measured on the 70B shapes at 64 tokens: the gate
    // projection gains 15 % from eight row blocks with 224 workgroups, the 8192-row linears lose with 128).
    // The members of a group are counted together.
    const int yblocks = (a.M + 15) / 16;
    if (a.M > 4 && a.d_in % 512 == 0 && a.r <= 512) {
        for (int nw = 16; nw >= 4; nw = nw > 8 ? 8 : nw - 4) {
            for (int tb = yblocks < 4 ? yblocks : 4; tb >= 1; tb = tb > 2 ? (tb + 1) / 2 : tb - 1) {
                if (nw == 16 && tb != 4) continue;
                if (nw == 8 && tb != 2 && tb != 4) continue;
                int groups = 0;
                for (int i = 0; i < n; ++i) groups += (members[i].d_out / 16 + nw - 1) / nw;
                // a long contraction with few rows (one linear, room for the partial outputs): 2 or 4 ranges of it in
                // different workgroups before the workgroup gets smaller (the down projection of the 70B layer at 64
                // tokens: 256 workgroups of four wavefronts over 224 steps each, or 256 of eight over 56)
                const int smax = (n == 1 && a.ypart && a.d_in >= SP_SPLIT_MIN_D_IN && nw >= 8) ? SP_MAX_SPLIT : 1;
                for (int ks = 1; ks <= smax; ks *= 2) {
                    if ((a.d_in / 128) % (ks * 4) != 0) break;
                    if (groups * ((yblocks + tb - 1) / tb) * ks >= (nw >= 8 ? 192 : 256)) {
                        SparseArgs m[4] = {members[0], members[n > 1 ? 1 : 0], members[n > 2 ? 2 : 0], members[n > 3 ? 3 : 0]};
                        for (int i = 0; i < 4; ++i) m[i].ksplit = ks;
                        return a.r == 0 ? launch_sparse_wide_cfg<S_NONE, VQ>(m, n, nw, tb, stream)
                                        : launch_sparse_wide_cfg<S_F16, VQ>(m, n, nw, tb, stream);
                    }
                }
            }
        }
    }
    if (a.r == 0) return xlds ? launch_sparse_one<S_NONE, S_NONE, 8, true, VQ>(members, n, stream)
                              : launch_sparse_one<S_NONE, S_NONE, 8, false, VQ>(members, n, stream);
    return xlds ? launch_sparse_one<S_F16, S_F16, 8, true, VQ>(members, n, stream)
                : launch_sparse_one<S_F16, S_F16, 8, false, VQ>(members, n, stream);
}

hipError_t launch_sparse_group(const SparseArgs* members, int n, hipStream_t stream)
{
    if (n < 1 || n > 4) return hipErrorInvalidValue;
    return members[0].qtiles ? launch_sparse_vq<true>(members, n, stream) : launch_sparse_vq<false>(members, n, stream);
}

hipError_t launch_sparse(const SparseArgs& a, hipStream_t stream) { return launch_sparse_group(&a, 1, stream); }

}  // namespace eora
