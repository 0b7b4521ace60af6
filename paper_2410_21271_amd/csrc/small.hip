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
// unit of t = x.A^T ((16 rows of A) x (one of kcn ranges of k-tiles)) and writes it as (value, launch tag)
// pairs, one 8-byte write-through store each; it owns no output rows and signals nothing else.  The other
// workgroups are CONSUMERS: a strip of one or two 16-row blocks each, its stored tiles requested quad by quad
// into the registers just consumed; after the backbone every thread reads its elements of t (the pairs of the
// kcn ranges, added as two partial sums in a fixed order into LDS; a pair with an older tag is read again,
// bounded), and the wavefronts share B's product in 32-column slices, continuing the same accumulators with
// t split into a high and a low fp16 part.  Producers come first in dispatch order and never wait.
//
// The stored codes enter the MFMA as they are: masked in place they are fp16 subnormals (tiles.hpp), the
// position factors sit in the staged x, the zero-points in one term per (token, group), the scale and the
// common 2^24 in fp32 on the accumulator.  Nobody waits on a returning atomic: a workgroup announces that it
// has read the launch counter with an atomic whose answer it ignores, and the launch's last workgroup
// advances the counter at its very end.
#include "segments.hpp"

#include <type_traits>

namespace eora {

constexpr int XSTAGE = 4;   // 16-byte chunks of x a thread may stage

#ifdef EORA_TIMELINE
// debug build only (never part of libeora.so): per-workgroup time stamps (100 MHz counter) kept in LDS and written 32 MiB behind the partials of t at the end
#define STL_DECL __shared__ unsigned long long s_tl[16]; if (threadIdx.x < 16) s_tl[threadIdx.x] = 0ull; \
    if (threadIdx.x == 0) { s_tl[12] = __builtin_amdgcn_s_getreg(63492); s_tl[13] = __builtin_amdgcn_s_getreg(63508); }
#define STL_STAMP(slot) do { if (threadIdx.x == 0) s_tl[slot] = wall_clock64(); } while (0)
#define STL_COUNT(slot, v) atomicAdd(&s_tl[slot], (unsigned long long)(v))
#define STL_FLUSH() do { __syncthreads(); if (threadIdx.x < 16) (a.tpair + (1 << 22))[blockIdx.x * 16 + threadIdx.x] = s_tl[threadIdx.x]; } while (0)
#else
#define STL_DECL do { } while (0)
#define STL_STAMP(slot) do { } while (0)
#define STL_COUNT(slot, v) do { } while (0)
#define STL_FLUSH() do { } while (0)
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

template <int K>
__device__ __forceinline__ float dpp_row_shr(float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x110 + K, 0xF, 0xF, true));
}

// One 32-column slice of a row block of B: the unit the wavefronts of a workgroup share B's product in.  fp16 tiles are
// one slice each; a 4-bit tile of KT columns is KT / 32 slices, one stored word per lane each (word q of the lane
// holds its columns 8q .. 8q+7 of the tile's quarter); 3-bit tiles cannot be cut by words and stay whole.
template <int FMT> struct BSlice {
    static constexpr bool SLICED = FMT == S_Q4S128 || FMT == S_Q4S64;
    static constexpr int NMF = SLICED ? 1 : Fmt<FMT>::KT / 32;       // MFMA steps per unit
    static constexpr int UNITS_PER_TILE = SLICED ? Fmt<FMT>::KT / 32 : 1;
    uint32_t w[SLICED ? 1 : Fmt<FMT>::WORDS];
    _Float16 sc;
};

template <int FMT>
__device__ __forceinline__ void load_bslice(BSlice<FMT>& s, const Factor& f, int R, int unit, int lane)
{
    constexpr int WORDS = Fmt<FMT>::WORDS, UPT = BSlice<FMT>::UNITS_PER_TILE;
    const int g = unit / UPT, q = unit % UPT;
    if constexpr (FMT != S_F16) s.sc = f.scales[((size_t)R * 16 + (lane & 15)) * f.ntk + g];
    else s.sc = (_Float16)1.0f;
    const uint32_t* p = f.w + (((size_t)R * f.ntk + g) * 64 + lane) * WORDS;
    if constexpr (BSlice<FMT>::SLICED) s.w[0] = p[q];
    else load_words<WORDS, true>(s.w, p);
}

template <int FMT>
__device__ __forceinline__ void decode_bslice(const BSlice<FMT>& s, h8 (&b)[BSlice<FMT>::NMF])
{
    if constexpr (BSlice<FMT>::SLICED) b[0] = dq4_word(s.w[0], k1024(8u), k64(8u));
    else decode_tile<FMT>(s.w, 8u, b);
}

// x of the token block -> LDS.  PLAIN: as it is (producers: A's product needs x itself).  Otherwise multiplied
// column by column with the position factors of the backbone format (tiles.hpp, xscale_chunk), and the sum of
// each group of 128 columns of the UNSCALED x, times 2^-24, goes to gs[row * G + group] (fp32): the zero-point
// term of the group.  Chunk (tid + k * NT) of the staged block is chunk tid + (k % NQ) * NT of token row k / NQ.
template <int WORDS, int NT, int NQ, int XS, bool PLAIN>
__device__ __forceinline__ void stage_x_small(const u4 (&xstage)[XS], _Float16* xs, float* gs, int mt, int ldxs, int G, int tid)
{
    const h8 pat = PLAIN ? h8{} : xscale_chunk<WORDS>(tid & 3);       // NT is a multiple of 4: the chunk's place in its lane's 32 columns
#pragma unroll
    for (int k = 0; k < XS; ++k) {
        const int row = k / NQ, chunk = tid + (k % NQ) * NT;
        const bool live = row < mt;
        Frag f;
        f.q = xstage[k];
        if constexpr (!PLAIN) {
            const h2 ones = {(_Float16)1.0f, (_Float16)1.0f};
            float sum = 0.f;
#pragma unroll
            for (int e = 0; e < 4; ++e) sum = __builtin_amdgcn_fdot2(f.p[e], ones, sum, false);     // fp32 sum of the pair, one instruction
            // the 16 chunks of a group sit in the 16 lanes of one DPP row: inclusive scan by row shifts (lanes
            // shifted in from outside the row read 0), fixed order; the row's last lane ends with the group's sum
            sum += dpp_row_shr<1>(sum);
            sum += dpp_row_shr<2>(sum);
            sum += dpp_row_shr<4>(sum);
            sum += dpp_row_shr<8>(sum);
            if (live && (tid & 15) == 15) gs[row * G + (chunk >> 4)] = sum * 0x1p-24f;
            f.v = f.v * pat;
        }
        if (live) *(u4*)(xs + row * ldxs + chunk * 8) = f.q;
    }
}

template <int FM, int FA, int FE, int NW, int NQ, bool M1, int RBK, bool MIX>          // RBK: row blocks of the launch's longest strips; MIX: the later strips are single row blocks
__global__ __launch_bounds__(NW * 64, 4) void small_kernel(GroupArgs a)   // second bound: wavefronts per SIMD, i.e. at most 128 registers (two 7- or 8-wavefront workgroups per compute unit)
{
    constexpr bool LOWRANK = FA != S_NONE;
    constexpr int NT = NW * 64;
    constexpr int WORDS = Fmt<FM>::WORDS;
    __shared__ float red[NW][RBK][4][16];
    __shared__ uint32_t s_epoch, s_bad;
    STL_DECL;
    STL_STAMP(0);

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int n = lane & 15, j = lane >> 4;
    const int mt = M1 ? 1 : a.M;                         // 1..4 tokens, one token block (M1: exactly one)
    const int mrow = n < mt ? n : 0;                     // lanes beyond the tokens re-read row 0; their results are dropped
    const int upl = LOWRANK ? (a.r / 16) * a.kcn : 0;    // units of t (= producer workgroups) per member
    const int nprod = upl * a.n;                         // producer workgroups
    const int ldxs = a.d_in + 32;                        // LDS row stride of x in halves (64 bytes of padding)
    const int G = a.d_in / 128;                          // == 4 * NW * NQ, one quantisation group per k-tile
    _Float16* xs = (_Float16*)eora_smem;
    float* gs = (float*)(eora_smem + (size_t)mt * ldxs * 2);      // zero-point terms: (M1 ? 1 : 4) x G, rows beyond the tokens zero
    float* ts = gs + (M1 ? 1 : 4) * G;                            // t as two partial sums, fp32 2 x mt x r (consumers)

    CheckIn ci{0u, 0u, 0u};
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
            load_ftile<FA, true>(buf[s], fa, rho, (nsteps > 0 ? first : kc * tpc) + ss * NW, lane);
        }
        __builtin_amdgcn_sched_barrier(0);               // all requests are out before the first result is used
        if (tid == 0) s_epoch = ci.epoch;
        stage_x_small<WORDS, NT, NQ, XS, true>(xstage, xs, gs, mt, ldxs, G, tid);
        __syncthreads();
        if (tid == 0) arrive(ci.epoch, a.hdr, blockIdx.x);
        STL_STAMP(1);
        const uint32_t epoch = s_epoch;
        f4 acc = {0.f, 0.f, 0.f, 0.f};
        for (int base = 0; base < nsteps; base += PD) {
#pragma unroll
            for (int s = 0; s < PD; ++s) {
                if (base + s < nsteps) {
                    const FTile<FA> cur = buf[s];
                    const int g = first + (base + s) * NW;
                    if (base + s + PD < nsteps) load_ftile<FA, true>(buf[s], fa, rho, first + (base + s + PD) * NW, lane);
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
        if (tid < 16 * mt) {
            const int i = tid >> 4, col = tid & 15;
            float v = 0.f;
#pragma unroll
            for (int w2 = 0; w2 < NW; ++w2) v += red[w2][0][i][col];
            // partial layout: [kc][token row (16)][r], every element an 8-byte (value, epoch + 1) pair
            // written by ONE write-through store: a reader that finds this launch's tag has this
            // launch's value; nothing else is signalled
            const unsigned long long pr = ((unsigned long long)(epoch + 1) << 32) | __builtin_bit_cast(uint32_t, v);
            __hip_atomic_store(&a.tpair[(((size_t)mem * a.kcn + kc) * 16 + i) * a.r + 16 * rho + col], pr, __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_AGENT);
        }
        STL_STAMP(7);
        STL_FLUSH();
        return;
    }
    }

    // =========================================================================== consumer
    // The strip: its first row block g0 counted over all members, then the member and the row block within it.  Uniform
    // launches give every workgroup RBK row blocks.  A mixed launch (MIX) gives the first a.c2n consumers RBK == 2
    // and all later ones a single row block (the kernel then holds both straight-line bodies and a workgroup takes one of
    // them under a uniform branch), which lets the launcher even out the row blocks per compute unit.
    int rbn = RBK, mem = 0, rb0;                         // row blocks of this strip, its member, its first row block within the member
    if constexpr (MIX) {
        const int c = blockIdx.x - nprod;
        int g0 = c * RBK;                                // first row block counted over all members
        if (c >= a.c2n) {
            g0 = a.c2n + c;
            rbn = 1;
        }
        const int s0 = a.d_out[0] / 16, s1 = a.d_out[1] / 16, s2 = a.d_out[2] / 16;
        if (a.n > 1 && g0 >= s0) {
            g0 -= s0;
            mem = 1;
            if (a.n > 2 && g0 >= s1) {
                g0 -= s1;
                mem = 2;
                if (a.n > 3 && g0 >= s2) {
                    g0 -= s2;
                    mem = 3;
                }
            }
        }
        rb0 = g0;
    } else {
        int R = blockIdx.x - nprod;                      // strip of RBK row blocks within its member
        const int s0 = a.d_out[0] / (16 * RBK), s1 = a.d_out[1] / (16 * RBK), s2 = a.d_out[2] / (16 * RBK);
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
        rb0 = R * RBK;
    }
    if constexpr (MIX) {
        // both straight-line bodies; a workgroup takes one of them under a uniform branch
        auto strip = [&](auto RBc) __attribute__((always_inline)) {
            constexpr int RB = decltype(RBc)::value;
#include "small_strip.inc"
        };
        if (rbn == 1) strip(std::integral_constant<int, 1>{});
        else strip(std::integral_constant<int, RBK>{});
    } else {
        constexpr int RB = RBK;
#include "small_strip.inc"
    }
    STL_FLUSH();
}

// ------------------------------------------------------------------------------------------------
// Instantiations whose kernel with both strip lengths stays within 128 registers without scratch (the build refuses
// scratch in this file, so a wrong entry here fails the build).
template <int FM, int FA, int FE, int NW, int NQ>
constexpr bool mixed_fits()
{
    return NW == 4 && NQ == 2 && FA != S_Q3S128 && !(FM == S_Q3 && FE == S_Q4S64) && !(FM == S_Q4 && FA == S_F16);
}

template <int FM, int FA, int FE, int NW, int NQ, bool M1, int RB, bool MIX = false>
static hipError_t launch_small_m(const GroupArgs& a, hipStream_t stream)
{
    auto kern = small_kernel<FM, FA, FE, NW, NQ, M1, RB, MIX>;
    const size_t lds = (size_t)a.M * (a.d_in + 32) * 2 + (size_t)(M1 ? 1 : 4) * (a.d_in / 128) * 4 + (size_t)2 * a.M * a.r * 4;   // x, zero-point terms, the two halves of t
    if (lds > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    int blocks = (FA != S_NONE) ? (a.r / 16) * a.kcn * a.n : 0;     // producers first
    if (MIX) {
        int nb = 0;
        for (int m = 0; m < a.n; ++m) nb += a.d_out[m] / 16;
        blocks += nb - a.c2n;                                       // c2n strips of two, the other row blocks one by one
    } else {
        for (int m = 0; m < a.n; ++m) blocks += a.d_out[m] / (16 * RB);
    }
    note_launch("small FM=%d FA=%d NW=%d NQ=%d RB=%d n=%d c2=%d", FM, FA, NW, NQ, RB, a.n, MIX ? a.c2n : -1);
    hipLaunchKernelGGL(kern, dim3(blocks), dim3(NW * 64), lds, stream, a);
    return hipGetLastError();
}

template <int FM, int FA, int FE, int NW, int NQ>
static hipError_t launch_small_one(const GroupArgs& a, hipStream_t stream)
{
    if (a.M == 1) {
        // A low-rank launch wants ALL its workgroups resident from the start: a consumer that only gets a slot when
        // the producers have left starts microseconds late and then still needs the whole streaming time, and a
        // consumer that waits for t at its end holds its slot.  So a workgroup takes 2 or 4 row blocks (a strip)
        // when one each would not fit next to the producers (the dispatcher deals workgroups to the compute units
        // round-robin, so a launch fits exactly when it has no more workgroups than slots; an eighth of slack, kept
        // at first, sent a single 14336-row linear to strips of two on a half-empty chip: 9.65 -> 9.25 us without).
        // 128 registers: 16 wavefronts, i.e. 16 / NW workgroups, per compute unit.
        // (The bare layer has no such wait: one row block each streams best; with 3-bit factors, and with 4-bit
        // factors on a 4-bit backbone, the strip instantiations do not fit 128 registers.)
        if constexpr (NQ <= 2 && FA != S_NONE && FA != S_Q3S128) {
            int blocks = 0;
            bool even2 = true, even4 = true;
            for (int m = 0; m < a.n; ++m) {
                blocks += a.d_out[m] / 16;
                even2 = even2 && a.d_out[m] % 32 == 0;
                even4 = even4 && a.d_out[m] % 64 == 0;
            }
            const int nprod = (a.r / 16) * a.kcn * a.n, room = 256 * (16 / NW);
            if (blocks + nprod > room) {
                // (a four-block strip as straight-line code does not fit 128 registers)
                if (even2) {
                    // Workgroups go to the compute units round-robin by index, 16 / NW to each.  With strips of two
                    // everywhere, the units whose first workgroup is a producer stream two row blocks less than the
                    // others and the launch ends with the others.  Mixed strips even that out: every slot but a unit's
                    // last takes a strip of two (or a producer), the last slot of the units without a producer and the
                    // slots the producers leave behind take the remaining row blocks one by one.
                    if constexpr (mixed_fits<FM, FA, FE, NW, NQ>()) {
                        GroupArgs b = a;
                        const int cus = 256, slots = cus * (16 / NW);
                        b.c2n = slots - cus;
                        const int c1n = blocks - 2 * b.c2n;
                        if (nprod <= cus && c1n >= cus - nprod && c1n <= 2 * cus) return launch_small_m<FM, FA, FE, NW, NQ, true, 2, true>(b, stream);
                    }
                    return launch_small_m<FM, FA, FE, NW, NQ, true, 2>(a, stream);
                }
            }
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
