// Pieces shared by the layer kernels: stored-format traits, tile loads and decoding, the factor
// (A / B) tile steps, activation-fragment sources and the launch check-in.
#pragma once
#include "kernels.hpp"
#include "tiles.hpp"

namespace eora {

template <int FMT> struct Fmt;
template <> struct Fmt<S_Q4> { static constexpr int KT = 128, WORDS = 4; static constexpr bool ASYM = true; };
template <> struct Fmt<S_Q3> { static constexpr int KT = 128, WORDS = 3; static constexpr bool ASYM = true; };
template <> struct Fmt<S_Q2> { static constexpr int KT = 128, WORDS = 2; static constexpr bool ASYM = true; };
template <> struct Fmt<S_Q4S128> { static constexpr int KT = 128, WORDS = 4; static constexpr bool ASYM = false; };
template <> struct Fmt<S_Q3S128> { static constexpr int KT = 128, WORDS = 3; static constexpr bool ASYM = false; };
template <> struct Fmt<S_Q4S64> { static constexpr int KT = 64, WORDS = 2; static constexpr bool ASYM = false; };
template <> struct Fmt<S_F16> { static constexpr int KT = 32, WORDS = 4; static constexpr bool ASYM = false; };

struct __attribute__((packed, aligned(4))) Words3 { uint32_t a, b, c; };

__device__ __forceinline__ uint32_t ld_relaxed(const uint32_t* p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// ONCE: the launch reads these bytes exactly once (every token of the call is in the workgroup that streams
// them): the request carries the non-temporal hint, so the line is not kept in the caches at the cost of lines
// that are read again (x, t, scales).  Kernels in which several workgroups read the same stored tile (one
// per group of token blocks) leave it off: there the second reader would miss.
template <int WORDS, bool ONCE = false>
__device__ __forceinline__ void load_words(uint32_t (&w)[WORDS], const uint32_t* __restrict__ p)
{
    if constexpr (ONCE) {
        typedef uint32_t u3a __attribute__((ext_vector_type(3), aligned(4)));
        typedef uint32_t u2v __attribute__((ext_vector_type(2)));
        if constexpr (WORDS == 4) {
            const u4 v = __builtin_nontemporal_load((const u4*)p);
            w[0] = v[0]; w[1] = v[1]; w[2] = v[2]; w[3] = v[3];
        } else if constexpr (WORDS == 3) {
            const u3a v = __builtin_nontemporal_load((const u3a*)p);
            w[0] = v[0]; w[1] = v[1]; w[2] = v[2];
        } else {
            const u2v v = __builtin_nontemporal_load((const u2v*)p);
            w[0] = v[0]; w[1] = v[1];
        }
    } else if constexpr (WORDS == 4) {
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

// Activation fragments of token row m.  Lanes beyond the token block (row_ok false) read row 0 instead:
// rows of a matmul are independent and their results are never stored, and a load that every lane
// executes keeps the requests of a wavefront free of divergent branches (which would make the
// compiler wait for all outstanding requests at each of them).
template <int NMF, bool XLDS>
__device__ __forceinline__ void load_act(h8 (&xa)[NMF], const ActSrc<XLDS>& src, int col, int m, bool row_ok)
{
    const int mr = row_ok ? m : 0;
    if constexpr (XLDS) {
        const _Float16* px = (const _Float16*)(eora_smem + src.lds_off) + mr * src.lds_ld + col;
#pragma unroll
        for (int t = 0; t < NMF; ++t) xa[t] = *(const h8*)(px + 8 * t);
    } else {
        const _Float16* px = src.g + (size_t)mr * src.ldg + col;
#pragma unroll
        for (int t = 0; t < NMF; ++t) xa[t] = *(const h8*)(px + 8 * t);
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
    } else if constexpr (FMT == S_Q3S128) {
        dq3_lane(w[0], w[1], w[2], 4u, b);           // symmetric 3-bit factor: the zero-point is the constant 4
    } else if constexpr (FMT == S_Q2) {
        dq2_word(w[0], z, b[0], b[1]);
        dq2_word(w[1], z, b[2], b[3]);
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

template <int FMT, bool ONCE = false>
__device__ __forceinline__ void load_ftile(FTile<FMT>& s, const Factor& f, int R, int g, int lane)
{
    constexpr int WORDS = Fmt<FMT>::WORDS;
    if constexpr (FMT != S_F16) s.sc = f.scales[((size_t)R * 16 + (lane & 15)) * f.ntk + g];
    else s.sc = (_Float16)1.0f;
    const size_t tile = (size_t)R * f.ntk + g;
    load_words<WORDS, ONCE>(s.w, f.w + (tile * 64 + lane) * WORDS);
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


// The same partial for a PRODUCER workgroup, which has nothing else to do: the tiles of A and the
// activation fragments of up to PD steps are all requested before the first one is used (one memory
// round trip for the whole unit when it has at most PD steps per wavefront).
template <int FMT, int NW>
__device__ __forceinline__ f4 run_factor_a_eager(const Factor& f, int R, int g_begin, int g_end, int wave, int lane,
                                                 const _Float16* __restrict__ xg, int ldg, int m, bool row_ok)
{
    constexpr int KT = Fmt<FMT>::KT, NMF = KT / 32, PD = NMF == 1 ? 8 : 2;
    const int j = lane >> 4;
    const int first = g_begin + wave;
    const int nsteps = first < g_end ? (g_end - first + NW - 1) / NW : 0;
    const _Float16* xrow = xg + (size_t)(row_ok ? m : 0) * ldg + (KT / 4) * j;
    f4 acc = {0.f, 0.f, 0.f, 0.f};
    for (int base = 0; base < nsteps; base += PD) {
        FTile<FMT> buf[PD];
        h8 xa[PD][NMF];
#pragma unroll
        for (int u = 0; u < PD; ++u) {
            const int s = base + u < nsteps ? base + u : nsteps - 1;         // clamped: always a valid tile
            const int g = first + s * NW;
            load_ftile<FMT>(buf[u], f, R, g, lane);
#pragma unroll
            for (int t = 0; t < NMF; ++t) xa[u][t] = *(const h8*)(xrow + (size_t)g * KT + 8 * t);
        }
#pragma unroll
        for (int u = 0; u < PD; ++u) {
            if (base + u < nsteps) {
                h8 b[NMF];
                decode_tile<FMT>(buf[u].w, 8u, b);
                if constexpr (FMT == S_F16) {
                    acc = mfma16(xa[u][0], b[0], acc);
                } else {
                    f4 part = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int t = 0; t < NMF; ++t) part = mfma16(xa[u][t], b[t], part);
                    acc += (float)buf[u].sc * part;
                }
            }
        }
    }
    return acc;
}

// Every workgroup of a low-rank launch reads the epoch and then checks in on one of HDR_NSUB
// spread-out counters; the last one to check in advances the epoch for the next launch.  One thread
// per workgroup runs the three steps; they are separate so that neither the epoch load nor the
// returning atomic stalls it: load at the top of the kernel, issue once the value is there, look at
// the returned count at the very end.
struct CheckIn {
    uint32_t epoch, count, k;
};

__device__ __forceinline__ void check_in_load(CheckIn& c, const uint32_t* hdr) { c.epoch = ld_relaxed(&hdr[HDR_EPOCH]); }

__device__ __forceinline__ void check_in_issue(CheckIn& c, uint32_t* hdr, uint32_t lin)
{
    // the epoch must have been READ before this workgroup checks in (the last one to check in
    // overwrites it): make the value live here and keep the atomic below this point
    asm volatile("" : "+v"(c.epoch) : : "memory");
    c.k = lin % HDR_NSUB;
    c.count = atomicAdd(&hdr[HDR_SUB0 + HDR_SUB_STRIDE * c.k], 1u);
}

__device__ __forceinline__ void check_in_finish(const CheckIn& c, uint32_t* hdr, uint32_t total)
{
    const uint32_t quota = (total - c.k + HDR_NSUB - 1) / HDR_NSUB;
    if (c.count == quota - 1) {
        hdr[HDR_SUB0 + HDR_SUB_STRIDE * c.k] = 0u;
        const uint32_t nsub = total < HDR_NSUB ? total : HDR_NSUB;
        if (atomicAdd(&hdr[HDR_TOP], 1u) == nsub - 1) {
            hdr[HDR_TOP] = 0u;
            hdr[HDR_EPOCH] = c.epoch + 1;           // every workgroup has read the epoch by now
        }
    }
}

// The same bookkeeping without a returning atomic on anybody's path (decode kernel): every workgroup reads the
// epoch and, once it has the value, ARRIVES on one of the HDR_NSUB counters with an atomic whose answer nobody
// waits for; the launch's last workgroup (by index), at its very end, waits until all have arrived (they all
// have long since: arriving is the first thing a workgroup does), clears the counters and advances the epoch.
// Compatible with check_in_* on the same workspace: both leave the counters at zero.
__device__ __forceinline__ void arrive(uint32_t epoch, uint32_t* hdr, uint32_t lin)
{
    asm volatile("" : "+v"(epoch) : : "memory");          // the epoch has been READ before this workgroup counts as arrived
    __hip_atomic_fetch_add(&hdr[HDR_SUB0 + HDR_SUB_STRIDE * (lin % HDR_NSUB)], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// one wavefront of the launch's last workgroup; lane k < HDR_NSUB looks after counter k.  Returns false when the
// bounded wait expired (the counters are then left as they are and the epoch does not advance).
__device__ __forceinline__ bool advance_epoch(uint32_t epoch, uint32_t* hdr, uint32_t total, int lane, int spin_limit)
{
    const uint32_t quota = lane < HDR_NSUB ? (total - lane + HDR_NSUB - 1) / HDR_NSUB : 0u;      // workgroups with lin % HDR_NSUB == lane
    bool all = false;
    for (int spins = 0; spins <= (spin_limit < 0 ? 0 : spin_limit); ++spins) {
        const uint32_t c = lane < HDR_NSUB ? ld_relaxed(&hdr[HDR_SUB0 + HDR_SUB_STRIDE * lane]) : 0u;
        if (__all(c == quota)) { all = true; break; }
        __builtin_amdgcn_s_sleep(8);
    }
    if (!all) return false;
    if (lane < HDR_NSUB) __hip_atomic_store(&hdr[HDR_SUB0 + HDR_SUB_STRIDE * lane], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (lane == 0) __hip_atomic_store(&hdr[HDR_EPOCH], epoch + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return true;
}

}  // namespace eora
