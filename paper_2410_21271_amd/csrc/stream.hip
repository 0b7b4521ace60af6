// The compensated quantised layer for 5 .. 16 tokens with x resident in LDS:
//
//      y = x.What^T + (x.A^T).B^T          (Sec. 3 forward equation, Alg. 1 step 7)
//
// HBM-bound: every stored byte is read once.  With 16 tokens a token block's x is as many bytes as four row blocks
// of 4-bit weights, so x must stay put while the weights stream past it.  For d_in <= 4096 the whole x (16 tokens x
// d_in halves, 128 KiB at 4096) fits the LDS of a compute unit: ONE workgroup of 16 wavefronts per compute unit keeps
// it there for its whole life, and every output tile is finished inside the workgroup that started it: no partial
// tile ever goes through memory.
//
// A workgroup owns a contiguous run of 16-row blocks of the launch's members.  Its wavefronts are KS ranges of the
// contraction length x SLOTS row blocks at a time (KS * SLOTS = 16); a wavefront's work is a fixed sequence of
// units (up to four stored tiles, with one load for their scales and one for their zero-points), requested three
// units ahead into the registers just consumed, the first ones before x is staged.  The accumulators stay in
// registers until the workgroup's last tile is consumed; then x is dead, and its LDS takes the KS partial tiles of
// every row block and t.  One wavefront per row block adds the partial tiles in the order of the ranges, continues
// with t.B^T and stores y.  Two barriers per workgroup after the staging of x.
//
// Low-rank path: the launch's first workgroups each begin with one 16-row block of A: all sixteen wavefronts take a
// sixteenth of the contraction, the partial tiles are added through LDS in a fixed order, and that 16 x 16 tile of
// t = x.A^T is published as (value, launch tag) pairs, one 8-byte write-through store each.  These workgroups own
// fewer output row blocks, by about the bytes of their block of A.  After the first barrier every thread reads its
// few pairs of t: a pair with this launch's tag is this launch's value; a stale one is read again, past the caches
// (bounded).  Nobody waits for an acknowledgement.  (Asking for the pairs earlier, while stored tiles are still in
// flight, was measured slower: the registers it holds cost more than the round trip it hides.)
//
// Arithmetic is the decode kernel's: codes as fp16 subnormals, position factors in the staged x, zero-points as
// -z sum(x) per (token, group), fp32 accumulation per group scaled once (tiles.hpp); t in fp32, split into a high
// and a low fp16 part for B's product.
// A wavefront that waits for t relies on the workgroups that hold A's blocks running: they are the launch's first,
// and the grid never exceeds one workgroup per compute unit.
#include "segments.hpp"

namespace eora {

#ifdef EORA_TIMELINE
// debug build only (never part of libeora.so): per-workgroup time stamps (100 MHz counter) kept in LDS and written 32 MiB behind t at the end
#define RTL_DECL __shared__ unsigned long long s_tl[16]; __shared__ unsigned long long s_tlw[64]; if (threadIdx.x < 16) s_tl[threadIdx.x] = 0ull; \
    if (threadIdx.x == 0) { s_tl[12] = __builtin_amdgcn_s_getreg(63492); s_tl[13] = __builtin_amdgcn_s_getreg(63508); }
#define RTL_STAMP(slot) do { if (threadIdx.x == 0) s_tl[slot] = wall_clock64(); } while (0)
#define RTL_WSTAMP(i) do { if ((threadIdx.x & 63) == 0) s_tlw[(threadIdx.x >> 6) * 4 + (i)] = wall_clock64(); } while (0)
#define RTL_FLUSH() do { __syncthreads(); if (threadIdx.x < 16) (a.tpair + (1 << 22))[blockIdx.x * 16 + threadIdx.x] = s_tl[threadIdx.x]; \
    if (threadIdx.x < 64) (a.tpair + (1 << 22) + (1 << 16))[blockIdx.x * 64 + threadIdx.x] = s_tlw[threadIdx.x]; } while (0)
#else
#define RTL_DECL do { } while (0)
#define RTL_STAMP(slot) do { } while (0)
#define RTL_WSTAMP(i) do { } while (0)
#define RTL_FLUSH() do { } while (0)
#endif

constexpr int RX_NW = 16, RX_NT = RX_NW * 64;
constexpr int RX_RMAX = 4;                       // rounds of SLOTS row blocks a workgroup takes at most
constexpr int RX_TP = 4;                         // pairs of t a thread requests together

template <typename T>
__device__ __forceinline__ T sk_pick(const T (&arr)[MAX_GROUP], int m)
{
    T v = arr[0];
    v = m == 1 ? arr[1] : v;
    v = m == 2 ? arr[2] : v;
    v = m == 3 ? arr[3] : v;
    return v;
}

template <int K>
__device__ __forceinline__ float sk_row_shr(float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x110 + K, 0xF, 0xF, true));
}

// 1 / xscale_chunk: brings a staged fragment back to x itself (A's product needs x, not x times the position factors)
template <int WORDS>
__device__ __forceinline__ h8 sk_unscale(int c)
{
    const _Float16 o = (_Float16)1.0f, e = (_Float16)8.0f, q = (_Float16)4.0f, s = (_Float16)16.0f, x = (_Float16)64.0f;
    if constexpr (WORDS == 4) {
        return h8{o, o, s, s, o, o, s, s};
    } else if constexpr (WORDS == 2) {
        return h8{o, o, q, q, s, s, x, x};
    } else {
        const h8 c0 = {o, o, e, e, x, x, o, o}, c1 = {e, e, o, o, e, e, x, x}, c2 = {o, o, e, e, o, o, e, e}, c3 = {x, x, o, o, e, e, o, o};
        h8 r = c0;
        r = c == 1 ? c1 : r;
        r = c == 2 ? c2 : r;
        r = c == 3 ? c3 : r;
        return r;
    }
}


// A partial tile handed from one range's workgroup to another's: 256 (value, launch tag) pairs, pair (i, lane) =
// register i of the lane at i * 64 + lane, so that one store instruction of a wavefront fills four whole
// 128-byte lines (write-through stores of parts of a line are read-modify-writes at the memory).
__device__ __forceinline__ void rx_store_tile(unsigned long long* dst, const f4& v, uint32_t tag)
{
    const unsigned long long t = (unsigned long long)tag << 32;
    const float vs[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 4; ++i)
        __hip_atomic_store(dst + i * 64, t | __builtin_bit_cast(uint32_t, vs[i]), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// The owner's sum over the S ranges in ascending order: its own tile `mine` at position `own`, the others' from
// slots[(k < own ? k : k - 1) * stride] (this lane's pairs), up to three ranges requested together; a tile whose
// tags are stale is read again (bounded).  Returns false if a wait expired.
__device__ __forceinline__ bool rx_cross_sum(const unsigned long long* slots, size_t stride, int S, int own, const f4& mine,
                                             uint32_t tag, int spin_limit, f4& out)
{
    constexpr int KB = 3;
    const int lim = spin_limit < 0 ? (1 << 22) : spin_limit;         // (a negative limit expires the waits for t only)
    f4 sum = {0.f, 0.f, 0.f, 0.f};
    bool fine = true;
    bool mine_added = false;
    for (int i0 = 0; i0 < S - 1; i0 += KB) {              // i: slot index of the other ranges, range k = i < own ? i : i + 1
        unsigned long long pr[KB][4] = {};
        bool good = false;
        for (int sp = 0; !good && sp <= lim; ++sp) {
            if (sp > 0) __builtin_amdgcn_s_sleep(2);
            uint32_t bad = 0;
#pragma unroll
            for (int kk = 0; kk < KB; ++kk) {
                const int i = i0 + kk < S - 1 ? i0 + kk : S - 2;      // past the last: that one again (not added)
#pragma unroll
                for (int e = 0; e < 4; ++e) pr[kk][e] = __hip_atomic_load(slots + (size_t)i * stride + e * 64, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
#pragma unroll
            for (int kk = 0; kk < KB; ++kk)
#pragma unroll
                for (int e = 0; e < 4; ++e) bad |= (uint32_t)(pr[kk][e] >> 32) ^ tag;
            good = bad == 0;
        }
        fine = fine && good;
#pragma unroll
        for (int kk = 0; kk < KB; ++kk) {
            const int i = i0 + kk;
            if (i < S - 1) {
                if (i == own) {                           // range `own` comes before range i + 1
                    sum += mine;
                    mine_added = true;
                }
                sum += f4{__builtin_bit_cast(float, (uint32_t)pr[kk][0]), __builtin_bit_cast(float, (uint32_t)pr[kk][1]),
                          __builtin_bit_cast(float, (uint32_t)pr[kk][2]), __builtin_bit_cast(float, (uint32_t)pr[kk][3])};
            }
        }
    }
    if (!mine_added) sum += mine;                         // the owner is the last range
    out = sum;
    return fine;
}

template <int FM, int FA, int FE, int NTW>       // NTW: stored tiles of a row block per wavefront
__global__ __launch_bounds__(RX_NT) void resident_kernel(StreamArgs a)
{
    constexpr bool LOWRANK = FA != S_NONE;
    constexpr int WORDS = Fmt<FM>::WORDS;
    constexpr int FAB = LOWRANK ? FA : S_F16, FEB = LOWRANK ? FE : S_F16;     // (valid formats also where the low-rank code is compiled out)
    constexpr int UT = NTW < 4 ? NTW : 4, UPR = NTW / UT;                       // tiles per unit, units per round
    constexpr int NL = RX_RMAX * UPR;                                           // units of a wavefront at most
    constexpr int WQ = FA == S_F16 ? 2 : 3;                                     // units in flight (with fp16 factors there are no registers for a third: eight tiles of A are held across the staging of x)
    __shared__ uint32_t s_epoch, s_err;
    RTL_DECL;
    RTL_STAMP(0);
    RTL_WSTAMP(3);

    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;    // (wave: uniform, in a scalar register)
    const int n = lane & 15, j = lane >> 4;
    // d_in beyond 4096: S ranges of KC = d_in / S columns; a workgroup belongs to range s and keeps that range's x
    const int S = a.S, KC = a.d_in / S;
    const int bid = (int)blockIdx.x, s = bid % S, wi = bid / S;       // range, index among the range's workgroups
    const int G = a.d_in / 128, GL = KC / 128, ldx = KC + 8;          // halves per staged row of x (16 bytes of padding: conflict-free fragment reads)
    const int KS = GL / NTW, SLOTS = RX_NW / KS;                      // (KS * SLOTS wavefronts stream; with 28 groups in a range 14 of the 16)
    const int ks = wave % KS, slot = wave / KS;
    _Float16* xs = (_Float16*)eora_smem;                              // [16][ldx]
    float* gs = (float*)(eora_smem + (size_t)16 * ldx * 2);           // [GL][16]: -z's factor of (group, token)
    f4* pa = (f4*)(gs + GL * 16);                                     // [16][64]: partial tiles of a block of A
    // after the backbone, over x: the row blocks' partial tiles [round][wavefront][64], then t [member][16][r + 4]
    f4* p2 = (f4*)eora_smem;
    float* ts = (float*)(eora_smem + (size_t)RX_RMAX * RX_NW * 64 * 16);
    const int ldt = a.r + 4;

    const int NAm = LOWRANK ? a.r / 16 : 0, nprod = NAm * a.n;        // A's row blocks: per member, in all (one per workgroup, the first ones)
    const int nb0 = a.d_out[0] / 16, nb1 = a.n > 1 ? a.d_out[1] / 16 : 0, nb2 = a.n > 2 ? a.d_out[2] / 16 : 0,
              nb3 = a.n > 3 ? a.d_out[3] / 16 : 0;
    const int NO = nb0 + nb1 + nb2 + nb3;
    const bool producer = wi < nprod;
    const bool tagged = LOWRANK || S > 1;                             // the launch uses (and advances) the workspace's launch counter
    // output row blocks [b0, b1) of this workgroup (every range's workgroups cut the blocks alike)
    int b0 = producer ? wi * a.qp : nprod * a.qp + (wi - nprod) * a.q;
    int b1 = b0 + (producer ? a.qp : a.q);
    b0 = b0 < NO ? b0 : NO;
    b1 = b1 < NO ? b1 : NO;
    const int nblk = b1 - b0;
    const int rounds_w = (slot < SLOTS && slot < nblk) ? (nblk - slot + SLOTS - 1) / SLOTS : 0;
    const int nunits = rounds_w * UPR;

    uint32_t epoch_v = 0;
    if (tagged && tid == 0) epoch_v = ld_relaxed(&a.hdr[HDR_EPOCH]);

    // output block o of the launch -> its member and row block there
    auto locate = [&](int o, int& mem, int& rb) __attribute__((always_inline)) {      // (selects, no branches: a request must not sit behind a merge of paths)
        const int c1 = nb0, c2 = nb0 + nb1, c3 = nb0 + nb1 + nb2;
        const bool m1 = a.n > 1 && o >= c1, m2 = a.n > 2 && o >= c2, m3 = a.n > 3 && o >= c3;
        mem = (m1 ? 1 : 0) + (m2 ? 1 : 0) + (m3 ? 1 : 0);
        rb = o - (m3 ? c3 : (m2 ? c2 : (m1 ? c1 : 0)));
    };

    // ---- stored tiles: unit L = round L / UPR, tiles ks * NTW + (L % UPR) * UT .. + UT - 1 of its row block ---------
    uint2 sc[WQ];
    uint32_t zq[WQ];
    uint32_t wq[WQ][UT][WORDS];
    // (le: the unit whose tiles are fetched into the registers of unit L; le == L except for the first requests of a
    // wavefront with fewer units than it has in flight, which fetch a valid unit again instead of branching)
    auto request_at = [&](auto Lc, int le) __attribute__((always_inline)) {
        constexpr int L = decltype(Lc)::value, Q = L % WQ;
        int mem, rb;
        const int o = b0 + (le / UPR) * SLOTS + slot;
        locate(o < NO ? o : NO - 1, mem, rb);
        const int g0 = s * GL + ks * NTW + (le % UPR) * UT;           // (group of the whole contraction)
        const size_t row = (size_t)rb * 16 + n;
        if constexpr (UT == 4) sc[Q] = *(const uint2*)(sk_pick(a.w_scales, mem) + row * G + g0);
        else sc[Q] = uint2{*(const uint32_t*)(sk_pick(a.w_scales, mem) + row * G + g0), 0u};
        zq[Q] = sk_pick(a.w_zeros, mem)[row * (G / 8) + (g0 >> 3)] >> (4 * (g0 & 7));
        const uint32_t* wp = (const uint32_t*)sk_pick(a.w, mem) + (((size_t)rb * G + g0) * 64 + lane) * WORDS;
#pragma unroll
        for (int i = 0; i < UT; ++i) load_words<WORDS, true>(wq[Q][i], wp + (size_t)i * 64 * WORDS);
    };
    auto request = [&](auto Lc) __attribute__((always_inline)) { request_at(Lc, decltype(Lc)::value); };
    // The first requests go out before x is staged.  A workgroup that begins with a block of A asks for ALL of that
    // block's tiles instead (its critical path: every workgroup of the launch ends up waiting for t), and for its first
    // stored tiles of the backbone once those are consumed.
    constexpr int KTA = Fmt<FAB>::KT, NMFA = KTA / 32, ATW = 256 / KTA;     // ATW: tiles of A per wavefront at most (a range has <= 4096 columns: 256 each)
    const Factor fa{(const uint32_t*)sk_pick(a.A, producer ? wi / (NAm > 0 ? NAm : 1) : 0),
                    sk_pick(a.A_scales, producer ? wi / (NAm > 0 ? NAm : 1) : 0), a.d_in / KTA};
    const int ntkl = KC / KTA;                                        // A's tiles of a row block inside the range
    int nwa = RX_NW;                                                  // wavefronts that take part in a block of A: the largest divisor of ntkl up to 16
    while (ntkl % nwa != 0) --nwa;
    const int tpw = ntkl / nwa;                                       // tiles of each
    FTile<FAB> abuf[ATW];
    auto first_requests = [&]() __attribute__((always_inline)) {
        if (0 < nunits) request(std::integral_constant<int, 0>{});
        if (1 < nunits) request(std::integral_constant<int, 1>{});
        if constexpr (WQ > 2) {
            if (2 < nunits) request(std::integral_constant<int, 2>{});
        }
    };
    // ---- x of the range first: 16 x KC halves, KC / 512 <= 8 16-byte chunks per thread, ALL requested before any stored
    // tile.  Loads return to a wavefront in the order it issued them: x asked for after the first stored tiles waited
    // behind 12 KiB of them per wavefront (192 KiB per compute unit, 9 of a launch's 20 us) although it comes from the
    // L2 cache.  Every load below is unconditional (a chunk past the range's last, or a row beyond the tokens, reads
    // chunk 0 / row 0 again and is not staged), so the compiler's wait counts for x stay exact while the stored tiles
    // requested after it are still in flight.
    const int cpr_ = KC / 8;
    const int nkm = ((a.M < 16 ? a.M : 16) * cpr_ + RX_NT - 1) / RX_NT;      // chunks per thread that reach a token row (<= KC / 512 <= 8)
    bool a_first = false;
    if constexpr (LOWRANK) a_first = producer;
    // (XB: chunks a thread requests, 4 while that covers the tokens, e.g. up to eight tokens at d_in 4096: half the requests)
    auto front = [&](auto XBc) __attribute__((always_inline)) {
        constexpr int XB = decltype(XBc)::value;
        const int cpr = cpr_;                                             // chunks per row (a multiple of 16: a group's chunks stay in one DPP row)
        // (the bare layer keeps its stored tiles ahead of x: it has three units in flight and launches with a single
        // unit per wavefront would fetch that unit three times below; measured slower there, faster with factors)
        if constexpr (!LOWRANK) {
            first_requests();
            __builtin_amdgcn_sched_barrier(0);
        }
        u4 xv[XB];
        {
            const _Float16* const xsrc = a.x + (size_t)s * KC;
#pragma unroll
            for (int k = 0; k < XB; ++k) {
                const int c = tid + (k < nkm ? k : 0) * RX_NT;
                // a wavefront's 64 chunks lie in one row (cpr is a multiple of 64): the row is a scalar
                const int row = __builtin_amdgcn_readfirstlane((int)__umulhi((uint32_t)c, a.cpr_magic)), cc = c - row * cpr;
                xv[k] = *(const u4*)(xsrc + (size_t)(row < a.M ? row : 0) * a.d_in + cc * 8);
            }
        }
        RTL_STAMP(9);
        RTL_WSTAMP(0);
        // rows beyond the tokens are not staged: what LDS holds there reaches only accumulator rows that are never
        // stored (the rows of a matrix product are independent)
        auto stage_x = [&]() __attribute__((always_inline)) {
            const h8 pat = xscale_chunk<WORDS>(tid & 3);                  // RX_NT is a multiple of 4: the chunk's place in its lane's 32 columns
            const h2 ones = {(_Float16)1.0f, (_Float16)1.0f};
#pragma unroll
            for (int k = 0; k < XB; ++k) {
                const int c = tid + k * RX_NT;
                const int row = __builtin_amdgcn_readfirstlane((int)__umulhi((uint32_t)c, a.cpr_magic)), cc = c - row * cpr;
                if (k < nkm && row < a.M) {
                    Frag f;
                    f.q = xv[k];
                    float sum = 0.f;
#pragma unroll
                    for (int e = 0; e < 4; ++e) sum = __builtin_amdgcn_fdot2(f.p[e], ones, sum, false);
                    // the 16 chunks of a group sit in the 16 lanes of one DPP row: inclusive scan, the last lane ends with the sum
                    sum += sk_row_shr<1>(sum);
                    sum += sk_row_shr<2>(sum);
                    sum += sk_row_shr<4>(sum);
                    sum += sk_row_shr<8>(sum);
                    if ((tid & 15) == 15) gs[(cc >> 4) * 16 + row] = sum * 0x1p-24f;
                    f.v = f.v * pat;
                    *(u4*)(xs + (size_t)row * ldx + cc * 8) = f.q;
                }
            }
        };
        // The first stored tiles (for a workgroup that begins with a block of A: that block's tiles) go out behind x and
        // before x is staged, as a fixed number of unconditional loads on either path (a wavefront with fewer units, or
        // with no part in the block of A, fetches a valid tile again and never uses it).  More paths, one per number
        // of units, were tried: where paths with different numbers of loads in flight meet, the compiler waits for all
        // of them, and the barrier behind the staging then waited for every stored tile requested so far.
        if (a_first) {
            const int rho = wi % (NAm > 0 ? NAm : 1), wv = wave < nwa ? wave : 0;
#pragma unroll
            for (int u = 0; u < ATW; ++u) load_ftile<FAB, true>(abuf[u], fa, rho, s * ntkl + wv * tpw + (u < tpw ? u : tpw - 1), lane);
            __builtin_amdgcn_sched_barrier(0);                            // (all of them out before anything below waits)
            RTL_WSTAMP(1);
            stage_x();
        } else {
            if constexpr (LOWRANK) {
                const int last = nunits > 0 ? nunits - 1 : 0;
                request_at(std::integral_constant<int, 0>{}, 0);
                request_at(std::integral_constant<int, 1>{}, 1 < nunits ? 1 : last);
                if constexpr (WQ > 2) request_at(std::integral_constant<int, 2>{}, 2 < nunits ? 2 : last);
                __builtin_amdgcn_sched_barrier(0);
            }
            RTL_WSTAMP(1);
            stage_x();
        }
    };
    if (nkm <= 4) front(std::integral_constant<int, 4>{});
    else front(std::integral_constant<int, 8>{});
    RTL_STAMP(11);
    RTL_WSTAMP(2);
    if (tid == 0) {
        s_epoch = epoch_v;
        s_err = 0u;
    }
    __syncthreads();
    RTL_STAMP(1);
    const uint32_t tag = s_epoch + 1;
    bool fine = true;
    if (tagged && tid == 0) arrive(epoch_v, a.hdr, bid);              // (an atomic nobody waits for; the epoch has been read)
    // partial tiles that cross ranges (S > 1): for t [S - 1][A blocks][256] pairs, then for y [S - 1][output blocks][256];
    // the owner of block b is range b mod S and keeps its own tile in registers
    unsigned long long* const part_t = a.part;
    unsigned long long* const part_y = a.part + (size_t)(S - 1) * nprod * 256;

    // ---- a block of A: t's 16 x 16 tile (member, rows 16 rho ..) over the whole contraction --------------------------
    if constexpr (LOWRANK) {
        if (producer) {
            const int mem = wi / NAm, rho = wi - mem * NAm;
            f4 acc_a = {0.f, 0.f, 0.f, 0.f};
            if (wave < nwa) {
                const int t0 = wave * tpw;
#pragma unroll
                for (int u = 0; u < ATW; ++u) {
                    if (u < tpw) {
                        h8 b[NMFA];
                        decode_tile<FAB>(abuf[u].w, 8u, b);
                        const _Float16* px = xs + (size_t)n * ldx + (t0 + u) * KTA + (KTA / 4) * j;
                        f4 part = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                        for (int q = 0; q < NMFA; ++q) {
                            // chunk number of these eight columns modulo 4: the fragment's position factors
                            const h8 xa = *(const h8*)(px + 8 * q) * sk_unscale<WORDS>(NMFA == 1 ? j : q);
                            part = mfma16(xa, b[q], part);
                        }
                        if constexpr (FAB == S_F16) acc_a += part;
                        else acc_a += (float)abuf[u].sc * part;
                    }
                }
            }
            // (the block's first stored tiles are requested behind the publication of t: issuing requests can take
            // a wavefront more than a microsecond while the memory pipeline is full, and every workgroup of the
            // launch ends up waiting for t)
            pa[wave * 64 + lane] = acc_a;
            __syncthreads();
            if (wave != 0) first_requests();
            if (wave == 0) {
                f4 v = pa[lane];
                for (int k = 1; k < nwa; ++k) v += pa[k * 64 + lane];
                const int own = wi % S;                               // the range that adds this block's S partial tiles and publishes t
                if (s != own) {
                    rx_store_tile(part_t + ((size_t)(s < own ? s : s - 1) * nprod + wi) * 256 + lane, v, tag);
                } else {
                    if (S > 1) {
                        f4 all;
                        fine = rx_cross_sum(part_t + (size_t)wi * 256 + lane, (size_t)nprod * 256, S, own, v, tag, a.spin_limit, all) && fine;
                        v = all;
                    }
                    // register v of lane (n, j): token 4j + v, row 16 rho + n of t
                    const float tv[4] = {v.x, v.y, v.z, v.w};
                    unsigned long long* const dst = a.tpair + ((size_t)mem * 16) * a.r + 16 * rho + n;
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        __hip_atomic_store(dst + (size_t)(4 * j + i) * a.r, ((unsigned long long)tag << 32) | __builtin_bit_cast(uint32_t, tv[i]),
                                           __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
            }
            if (wave == 0) first_requests();
            RTL_STAMP(8);
        }
    }

    // ---- the backbone --------------------------------------------------------------------------------------------
    // this thread's pairs of t: elements tid, tid + 1024, ... of [member][16][r], read after the backbone
    const int T = LOWRANK ? a.n * 16 * a.r : 0;
    unsigned long long tp[RX_TP];
    // the wavefront that finishes local row block `wave` asks for B's first tiles of it when its last stored tile is consumed
    constexpr int KTB = Fmt<FEB>::KT, NMFB = KTB / 32, BPRE = NMFB == 1 ? 4 : 1;
    const bool reducer = wave < nblk;
    int rmem = 0, rrb = 0;
    if (reducer) locate(b0 + wave, rmem, rrb);
    const int yown = (b0 + wave) % S;                                 // the range that finishes this row block (adds t.B^T, the other ranges' tiles, stores y)
    const bool finisher = reducer && s == yown;
    const Factor fb{(const uint32_t*)sk_pick(a.B, rmem), sk_pick(a.B_scales, rmem), LOWRANK ? a.r / KTB : 0};
    FTile<FEB> bt[BPRE];
    f4 acc[RX_RMAX];
#pragma unroll
    for (int r2 = 0; r2 < RX_RMAX; ++r2) acc[r2] = f4{0.f, 0.f, 0.f, 0.f};
    auto consume = [&](auto Lc) __attribute__((always_inline)) {
        constexpr int L = decltype(Lc)::value, Q = L % WQ;
        const int g0 = ks * NTW + (L % UPR) * UT;
#pragma unroll
        for (int i = 0; i < UT; ++i) {
            h8 b[4];
            raw_tile<WORDS>(wq[Q][i], b);
            const float zf = -(float)((zq[Q] >> (4 * i)) & 0xFu);
            f4 part = zf * *(const f4*)(gs + (g0 + i) * 16 + 4 * j);  // tokens 4j .. 4j+3: the registers of this lane
            const _Float16* px = xs + (size_t)n * ldx + (g0 + i) * 128 + 32 * j;
#pragma unroll
            for (int t = 0; t < 4; ++t) part = mfma16(*(const h8*)(px + 8 * t), b[t], part);
            const uint32_t sw = (i < 2) ? sc[Q].x : sc[Q].y;
            const _Float16 s16 = __builtin_bit_cast(_Float16, (uint16_t)((i & 1) ? (sw >> 16) : (sw & 0xFFFFu)));
            acc[L / UPR] += (float)s16 * part;
        }
        if constexpr (L + WQ < NL) {
            if (L + WQ < nunits) request(std::integral_constant<int, L + WQ>{});
        }
    };
    static_assert(NL <= 8, "more units than the unrolled sequence below");
    if (0 < nunits) consume(std::integral_constant<int, 0>{});
    RTL_STAMP(2);
    if (1 < nunits) consume(std::integral_constant<int, 1>{});
    if (2 < nunits) consume(std::integral_constant<int, 2>{});
    if (3 < nunits) consume(std::integral_constant<int, 3>{});
    if constexpr (NL > 4) {
        if (4 < nunits) consume(std::integral_constant<int, 4>{});
        if (5 < nunits) consume(std::integral_constant<int, 5>{});
        if (6 < nunits) consume(std::integral_constant<int, 6>{});
        if (7 < nunits) consume(std::integral_constant<int, 7>{});
    }

    if constexpr (LOWRANK) {
        if (finisher) {
#pragma unroll
            for (int u = 0; u < BPRE; ++u) load_ftile<FEB, true>(bt[u], fb, rrb, u < fb.ntk ? u : 0, lane);
        }
    }

    // ---- x is dead: its LDS takes the partial tiles and t -----------------------------------------------------------
    RTL_STAMP(3);
    __syncthreads();
    RTL_STAMP(4);
#pragma unroll
    for (int r2 = 0; r2 < RX_RMAX; ++r2)
        if (r2 < rounds_w) p2[(r2 * RX_NW + wave) * 64 + lane] = acc[r2] * 0x1p24f;      // (the subnormal codes' common factor)
    if constexpr (LOWRANK) {
        for (int e0 = 0; e0 < T; e0 += RX_TP * RX_NT) {
            // first an ordinary, cached load: the workgroups of an XCD share its L2's copy (a stale copy shows by its tag)
#pragma unroll
            for (int u = 0; u < RX_TP; ++u) {
                const int e = e0 + tid + u * RX_NT;
                tp[u] = a.tpair[e < T ? e : 0];
            }
            // a pair with this launch's tag is this launch's value; stale ones: all of the thread's pairs again, together
            bool good = a.spin_limit >= 0;                            // (a negative limit: every wait counts as expired)
            for (int sp = 0;; ++sp) {
                uint32_t bad = 0;
#pragma unroll
                for (int u = 0; u < RX_TP; ++u)
                    if (e0 + tid + u * RX_NT < T) bad |= (uint32_t)(tp[u] >> 32) ^ tag;
                good = good && bad == 0;
                if (good || sp >= a.spin_limit) break;
                good = true;
                __builtin_amdgcn_s_sleep(2);
#pragma unroll
                for (int u = 0; u < RX_TP; ++u) {
                    const int e = e0 + tid + u * RX_NT;
                    tp[u] = __hip_atomic_load(a.tpair + (e < T ? e : 0), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
            }
            fine = fine && good;
#pragma unroll
            for (int u = 0; u < RX_TP; ++u) {
                const int e = e0 + tid + u * RX_NT;
                if (e < T) {
                    const int row = e / a.r, col = e - row * a.r;     // row: member * 16 + token
                    float v = __builtin_bit_cast(float, (uint32_t)tp[u]);
                    // several adapters side by side (one member): a token row keeps its own adapter's columns of t
                    if (a.adapter && a.adapter[row < a.M ? row : 0] != col / a.r_per) v = 0.f;
                    ts[row * ldt + col] = v;
                }
            }
        }
        if (!__all(fine)) s_err = 1u;
    }
    RTL_STAMP(5);
    __syncthreads();
    RTL_STAMP(6);

    // ---- one wavefront per row block: the ranges' partial tiles in their order, t.B^T, y -----------------------------
    if (reducer) {
        const int rnd = wave / SLOTS, sl = wave % SLOTS;
        const f4* src = p2 + ((size_t)rnd * RX_NW + sl * KS) * 64 + lane;
        f4 ysum = src[0];
        for (int k = 1; k < KS; ++k) ysum += src[k * 64];
        if constexpr (LOWRANK) {
            if (finisher && s_err == 0u) {                            // (t never came: y lacks the low-rank term, the launch reports it)
                const float* trow = ts + (size_t)(rmem * 16 + n) * ldt + (KTB / 4) * j;
                auto ext_tile = [&](const FTile<FEB>& cw, int g) __attribute__((always_inline)) {
                    h8 b[NMFB];
                    decode_tile<FEB>(cw.w, 8u, b);
                    f4 part = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int q = 0; q < NMFB; ++q) {
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
                    if constexpr (FEB == S_F16) ysum += part;
                    else ysum += (float)cw.sc * part;
                };
                for (int g0 = 0; g0 < fb.ntk; g0 += BPRE) {
#pragma unroll
                    for (int u = 0; u < BPRE; ++u) {
                        if (g0 + u < fb.ntk) {
                            const FTile<FEB> cw = bt[u];
                            if (g0 + u + BPRE < fb.ntk) load_ftile<FEB, true>(bt[u], fb, rrb, g0 + u + BPRE, lane);
                            ext_tile(cw, g0 + u);
                        }
                    }
                }
            }
        }
        const int o = b0 + wave;
        if (!finisher) {
            rx_store_tile(part_y + ((size_t)(s < yown ? s : s - 1) * NO + o) * 256 + lane, ysum, tag);
        } else {
            if (S > 1) {
                f4 all;
                if (!rx_cross_sum(part_y + (size_t)o * 256 + lane, (size_t)NO * 256, S, yown, ysum, tag, a.spin_limit, all) && lane == 0)
                    atomicOr(&a.hdr[HDR_ERROR], 1u);
                ysum = all;
            }
            const float yv[4] = {ysum.x, ysum.y, ysum.z, ysum.w};
            _Float16* const y = sk_pick(a.y, rmem);
            const int d_out = sk_pick(a.d_out, rmem);
#pragma unroll
            for (int v = 0; v < 4; ++v)
                if (4 * j + v < a.M) y[(size_t)(4 * j + v) * d_out + rrb * 16 + n] = (_Float16)yv[v];
        }
    }

    RTL_STAMP(7);
    RTL_FLUSH();
    // ---- the launch's last workgroup (by index) advances the launch counter once every workgroup has arrived ---------
    if (tagged) {
        if (tid == 0 && s_err) atomicOr(&a.hdr[HDR_ERROR], 1u);
        if (bid == (int)gridDim.x - 1 && wave == RX_NW - 1) {
            if (!advance_epoch(s_epoch, a.hdr, gridDim.x, lane, a.spin_limit) && lane == 0) atomicOr(&a.hdr[HDR_ERROR], 1u);
        }
    }
}

// ------------------------------------------------------------------------------------------------------------------
constexpr size_t RX_LDS_MAX = 159 * 1024;       // dynamic LDS of a workgroup at most (a compute unit has 160 KiB; a few static bytes beside)

// ranges of the contraction: one while x fits a compute unit's LDS, else the fewest of at most 4096 columns each
static int resident_ranges(int d_in) { return (d_in + 4095) / 4096; }

static size_t resident_lds(int d_in, int r, int n)
{
    const int KC = d_in / resident_ranges(d_in);
    const size_t front = (size_t)16 * (KC + 8) * 2 + (size_t)(KC / 128) * 16 * 4 + (size_t)RX_NW * 64 * 16;
    const size_t back = (size_t)RX_RMAX * RX_NW * 64 * 16 + (size_t)n * 16 * (r + 4) * 4;
    return front > back ? front : back;
}

// how a launch is cut: S ranges, NTW tiles per wavefront, q row blocks per workgroup (qp for one that begins with a
// block of A), wgs workgroups (a multiple of S)
struct ResidentPlan {
    int S, ntw, q, qp, wgs;
};

static int device_cus()
{
    static int cus = 0;
    if (cus == 0) {
        int dev = 0;
        hipDeviceProp_t prop;
        if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) return 0;
        cus = prop.multiProcessorCount;
    }
    return cus;
}

// Below this many row blocks in a launch the kernel for 5 .. 127 tokens is the faster one when x is one range
// (measured: every workgroup here stages the whole x, which a launch of few rows does not earn back).
constexpr int RX_MIN_BLOCKS = 256;
static int g_min_blocks = RX_MIN_BLOCKS;
void set_resident_min_blocks(int blocks) { g_min_blocks = blocks < 0 ? RX_MIN_BLOCKS : blocks; }

static bool resident_plan(int d_in, int r, int fm, int fa, const int* d_out, int n, ResidentPlan& p)
{
    const int cus = device_cus();
    if (cus <= 0) return false;
    p.S = resident_ranges(d_in);
    if (d_in % (p.S * 512) != 0) return false;
    const int per_range = cus / p.S;                                  // workgroups of a range: one workgroup per compute unit in all
    int NO = 0;
    for (int m = 0; m < n; ++m) NO += d_out[m] / 16;
    const int nprod = r > 0 ? n * (r / 16) : 0;
    if (nprod > per_range / 2) return false;
    // a block of A in output row blocks, by stored bytes
    const int wbits = fm == S_Q4 ? 4 : fm == S_Q3 ? 3 : 2, abits = fa == S_F16 ? 16 : 4;
    const int acost = r > 0 ? (abits + wbits - 1) / wbits : 0;
    p.q = (NO + nprod * acost + per_range - 1) / per_range;
    p.q = p.q < 1 ? 1 : p.q;
    p.qp = p.q > acost ? p.q - acost : 0;
    const int rest = NO - nprod * p.qp;
    const int w = nprod + (rest > 0 ? (rest + p.q - 1) / p.q : 0);
    if (w > per_range) return false;
    p.wgs = w * p.S;
    // the smallest NTW whose row-block slots reach min(q, 4); failing that, the admissible one with the most slots
    const int GL = d_in / p.S / 128;
    int best = 0, best_slots = 0;
    for (int ntw = 2; ntw <= 8; ntw *= 2) {
        if (GL % ntw != 0) continue;
        const int KS = GL / ntw;
        if (KS < 1 || KS > RX_NW) continue;
        const int slots = RX_NW / KS, rounds = (p.q + slots - 1) / slots;
        if (rounds > RX_RMAX || p.q > RX_NW) continue;
        if (slots >= (p.q < 4 ? p.q : 4)) {
            p.ntw = ntw;
            return true;
        }
        if (slots > best_slots) {
            best = ntw;
            best_slots = slots;
        }
    }
    p.ntw = best;
    return best != 0;
}

// pairs of the workspace's region of tagged values: t itself first, the partial tiles that cross ranges behind it
constexpr size_t RX_T_PAIRS = 8192;                                   // n * 16 * r <= 16 * 512
constexpr size_t RX_REGION_PAIRS = 32 * 16 * 512;                     // (the region's size, api.hip: MAX_PART_ELEMS)

bool stream_fits(int M, int d_in, int group, int r, int fm, int fa, const int* d_out, int n)
{
    if (M < 5 || M > 16 || group != 128) return false;
    const int S = resident_ranges(d_in);
    if (S == 1 && d_in != 1024 && d_in != 2048 && d_in != 4096) return false;
    if (r > 0 && fa != S_F16 && fa != S_Q4S128) return false;
    if (r > 0 && fa == S_Q4S128 && r % 128 != 0) return false;        // (B's 64-column tiles of a rank-64 pair: not instantiated here)
    if (r % 32 != 0 || n * r > 512 || resident_lds(d_in, r, n) > RX_LDS_MAX) return false;
    int NO = 0;
    for (int m = 0; m < n; ++m) NO += d_out[m] / 16;
    if (S == 1 && NO < g_min_blocks) return false;
    if (S > 1 && RX_T_PAIRS + (size_t)(S - 1) * (NO + n * (r / 16)) * 256 > RX_REGION_PAIRS) return false;
    ResidentPlan p;
    return resident_plan(d_in, r, fm, fa, d_out, n, p);
}

template <int FM, int FA, int FE, int NTW>
static hipError_t launch_resident_one(StreamArgs a, const ResidentPlan& p, hipStream_t stream)
{
    auto kern = resident_kernel<FM, FA, FE, NTW>;
    const size_t lds = resident_lds(a.d_in, FA != S_NONE ? a.r : 0, a.n);
    static bool prepared = false;
    if (!prepared) {
        const hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)RX_LDS_MAX);
        if (e != hipSuccess) return e;
        prepared = true;
    }
    a.q = p.q;
    a.qp = p.qp;
    a.S = p.S;
    a.cpr_magic = (uint32_t)((0x100000000ull + (uint64_t)(a.d_in / p.S / 8) - 1) / (uint64_t)(a.d_in / p.S / 8));     // exact for c * cpr < 2^32
    a.part = a.tpair + RX_T_PAIRS;
    if (p.S > 1) note_launch("resident FM=%d FA=%d NTW=%d S=%d n=%d wgs=%d q=%d", FM, FA, NTW, p.S, a.n, p.wgs, p.q);
    else note_launch("resident FM=%d FA=%d NTW=%d n=%d wgs=%d q=%d", FM, FA, NTW, a.n, p.wgs, p.q);
    hipLaunchKernelGGL(kern, dim3(p.wgs), dim3(RX_NT), lds, stream, a);
    return hipGetLastError();
}

template <int FM, int FA, int FE>
static hipError_t launch_resident_ntw(const StreamArgs& a, const ResidentPlan& p, hipStream_t stream)
{
    switch (p.ntw) {
        case 2: return launch_resident_one<FM, FA, FE, 2>(a, p, stream);
        case 4: return launch_resident_one<FM, FA, FE, 4>(a, p, stream);
        case 8: return launch_resident_one<FM, FA, FE, 8>(a, p, stream);
        default: return hipErrorInvalidValue;
    }
}

template <int FM>
static hipError_t launch_stream_ab(const StreamArgs& a, const ResidentPlan& p, int fa, int fe, hipStream_t stream)
{
    if (fe == S_NONE) return launch_resident_ntw<FM, S_NONE, S_NONE>(a, p, stream);
    if (fa == S_F16 && fe == S_F16) return launch_resident_ntw<FM, S_F16, S_F16>(a, p, stream);
    if (fa == S_Q4S128 && fe == S_Q4S128) return launch_resident_ntw<FM, S_Q4S128, S_Q4S128>(a, p, stream);
    return hipErrorInvalidValue;
}

hipError_t launch_stream(const StreamArgs& a, int fm, int fa, int fe, hipStream_t stream)
{
    ResidentPlan p;
    if (!resident_plan(a.d_in, fe == S_NONE ? 0 : a.r, fm, fa, a.d_out, a.n, p)) return hipErrorInvalidValue;
    switch (fm) {
        case S_Q4: return launch_stream_ab<S_Q4>(a, p, fa, fe, stream);
        case S_Q3: return launch_stream_ab<S_Q3>(a, p, fa, fe, stream);
        case S_Q2: return launch_stream_ab<S_Q2>(a, p, fa, fe, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace eora
