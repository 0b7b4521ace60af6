// Prefill (many tokens): y = x.What^T + t.B^T as ONE MFMA-bound GEMM whose contraction runs over
// d_in (backbone, dequantised on the way) and then over r (B's tiles with t = x.A^T as the
// activation) into the same fp32 accumulators (Sec. 3 forward equation, Alg. 1 step 7; the fusion of
// B's product into the backbone's output follows Sec. 4.5 / App. A.6).  t itself is a first, small
// launch of the same kernel with A as the weight operand (fp16 M x r into scratch): recomputing it
// per output tile would cost r / 128 times the backbone's MFMA work.
//
// Workgroup: 8 wavefronts, tile = 128 tokens x 256 output rows, contraction in steps of 128 (one
// quantisation group); each wavefront owns all 128 tokens x 32 rows = 4 accumulator blocks of
// v_mfma_f32_32x32x16_f16, the instruction with the highest sustained rate here (measured with
// register-only loops: 2.2 PFLOP/s against 1.9 for the 16x16x32 form).  Its operand layout is:
// lane l holds 8 consecutive k (8*(l/32) ..) of token / output row l%32; result register v of lane l
// is token 8*(v/4) + 4*(l/32) + v%4, output row l%32 (checked on the device against a host matmul).
//   - Weights never touch LDS.  The stored tiles (16 rows x 128 columns, lane (n, j) = row n, columns
//     32j .. 32j+31, tiles.hpp) feed this MFMA as well: lane l = n + 16*h + 32*kg of the wavefront loads,
//     for jp = 0, 1, the 16 bytes of stored lane (n, 2*jp + kg) of the tile of its row block h; word
//     t of that load decodes to the operand of the k-slice (jp, t): columns 32*(2jp+kg) + 8t .. +7 of
//     output row 16*h + n of the wavefront's 32.  Every wavefront loads its own two tiles one step
//     ahead, decodes them to the exact integers code - zero and multiplies by the fp16 group scale
//     (one fp16 rounding of scale*(code-zero), relative error <= 2^-11 per weight; scaling the
//     accumulators per group instead would cost as many VALU cycles as the group's MFMAs).  Every
//     weight is decoded exactly once per workgroup, and LDS carries only x.
//   - x: the 128 x 128 slab is read with coalesced 16-byte loads (256 bytes per token row) into
//     registers two steps ahead and written one step ahead to the other of two LDS buffers as MFMA
//     operand fragments (32 tokens x 16 columns = 1 KiB, one ds_read_b128 each; an XOR of the token
//     slot with the slice number keeps both the scattered writes and the reads free of bank
//     conflicts): one barrier per step.
//   - The two wavefronts of a SIMD (w and w + 4) run the two halves of a step, decode (VALU) and
//     contraction (MFMA), in opposite order, so that the two pipes are busy at the same time.
// One workgroup per compute unit (two wavefronts per SIMD, at most 256 registers).  The epilogue
// transposes through LDS so that y is written in 128-byte rows.
#include "segments.hpp"

namespace eora {

typedef float f16v __attribute__((ext_vector_type(16)));

// one member of a launch, as the helpers below see it
struct PfView {
    const _Float16* x;
    int ldx;
    const void* w;
    const _Float16* w_scales;
    const uint32_t* w_zeros;
    int group;
    const _Float16* x2;
    int ldx2;
    const void* w2;
    const _Float16* w2_scales;
    void* y;
    int ldy;
    int M, N, K1, K2;
    int ksplit;
    float* part;
    int ldp, pcol;
};

constexpr int PF_BM = 128, PF_BN = 256;
constexpr int PF_NW = 8, PF_NT = PF_NW * 64;         // wavefronts: 2 (tokens) x 4 (rows)
constexpr int PF_XS = 32 * 1024;                      // one x slab: 4 token blocks x 8 slices x 1 KiB
constexpr int PF_LDS = 2 * PF_XS;                     // the two x slabs; the epilogue's staging tiles (40 KiB) reuse them

__device__ __forceinline__ f16v mfma32(h8 a, h8 b, f16v c) { return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0); }

// weights of one 128-wide step for the wavefront's two pairs of row blocks, exactly as loaded: nothing
// here is touched before decode_wpre(), a whole step later (any arithmetic on a loaded value at load
// time would make the wavefront wait for the request it has just issued)
template <int FMT>
struct WPre {
    uint32_t w[2][Fmt<FMT>::WORDS];                   // [jp]
    uint32_t zraw;                                    // the word that holds the group's zero-point nibble
    uint32_t sraw;                                    // fp16 scale bits, zero-extended
    int zshift;                                       // 4 * (group index % 8)
};
template <>
struct WPre<S_F16> {
    u4 v[8];                                          // [slice]: four tiles of 32 columns = eight slices of 16
};

// Rl: the row block (2*wn + h, clamped) whose row n this lane supplies.  tiles / scales / zeros / K / group: the
// segment's stored operand (first segment: the backbone, or A for the down-projection launch; second: B).
template <int FMT>
__device__ __forceinline__ void load_wpre_from(WPre<FMT>& r, const void* tiles, const _Float16* scales, const uint32_t* zeros,
                                               int K, int group, int Rl, int g, int lane)
{
    const int n = lane & 15, kg = lane >> 5;
    constexpr int WORDS = Fmt<FMT>::WORDS;
    const int G = K / 128;
    const int NG = Fmt<FMT>::ASYM ? K / group : G, grp = Fmt<FMT>::ASYM ? (g * 128) / group : g;
    r.zshift = 4 * (grp & 7);
    const uint32_t* tile = (const uint32_t*)tiles + ((size_t)Rl * G + g) * 64 * WORDS;
#pragma unroll
    for (int jp = 0; jp < 2; ++jp) load_words<WORDS>(r.w[jp], tile + (16 * (2 * jp + kg) + n) * WORDS);
    const size_t row = (size_t)Rl * 16 + n;
    r.sraw = ((const uint16_t*)scales)[row * NG + grp];
    if constexpr (Fmt<FMT>::ASYM) r.zraw = zeros[row * ((NG + 7) / 8) + (grp >> 3)];
}

template <int FMT>
__device__ __forceinline__ void load_wpre(WPre<FMT>& r, const PfView& a, int Rl, int g, int lane)
{
    load_wpre_from<FMT>(r, a.w, a.w_scales, a.w_zeros, a.K1, a.group, Rl, g, lane);
}

// decode to operands bf[slice], slice = 4*jp + t, scale folded in fp16
template <int FMT>
__device__ __forceinline__ void decode_wpre(const WPre<FMT>& r, h8 (&bf)[8])
{
    const uint32_t z = Fmt<FMT>::ASYM ? (r.zraw >> r.zshift) & 0xFu : 8u;       // (symmetric formats carry their constant themselves)
    const _Float16 sc = __builtin_bit_cast(_Float16, (uint16_t)r.sraw);
    const h8 s = {sc, sc, sc, sc, sc, sc, sc, sc};
#pragma unroll
    for (int jp = 0; jp < 2; ++jp) {
        h8 b[4];
        decode_tile<FMT>(r.w[jp], z, b);
#pragma unroll
        for (int t = 0; t < 4; ++t) bf[4 * jp + t] = b[t] * s;
    }
}

// fp16 tiles (A for the down-projection launch, B in the second segment) straight into operands
__device__ __forceinline__ void load_b_frags(h8 (&bf)[8], const void* __restrict__ tiles, int K, int Rl, int step, int lane)
{
    const int n = lane & 15, kg = lane >> 5;
    const u4* p = (const u4*)tiles + ((size_t)Rl * (K / 32) + 4 * step) * 64 + n;
#pragma unroll
    for (int f = 0; f < 8; ++f) bf[f] = __builtin_bit_cast(h8, p[(f >> 1) * 64 + 16 * (2 * (f & 1) + kg)]);
}

// x slab of one step: thread tid owns the 16-byte chunks c = tid + 256*i, i = 0..7; chunk c is token row
// c / 16 of the tile and columns 8*(c % 16) .. +7 of the step (coalesced: 256 bytes per row).
constexpr int PF_XC = 2048 / PF_NT;                   // 16-byte chunks of the slab per thread
__device__ __forceinline__ void load_x(u4 (&v)[PF_XC], const _Float16* __restrict__ act, int ld, int M, int m0, int col0, int tid)
{
#pragma unroll
    for (int i = 0; i < PF_XC; ++i) {
        const int c = tid + PF_NT * i;
        int row = m0 + (c >> 4);
        row = row < M ? row : M - 1;                  // rows beyond M re-read the last row; never stored
        v[i] = *(const u4*)(act + (size_t)row * ld + col0 + 8 * (c & 15));
    }
}

// The operand (token block tb of 32, slice f) holds for lane (token slot, kg) the eight columns that the
// weight operand of slice f holds for kg: chunk kc = 4*(2*jp + kg) + t, f = 4*jp + t, for a quantised
// tile (quarter_major); chunk kc = 4*tile + 2*s + kg, f = 2*tile + s, for four fp16 tiles.  The token slot
// is XOR-ed with 2*f + kg: the 16 lanes that write one token row's chunks, and the 16 lanes of a read
// that differ in token, then hit 16 different bank groups.
__device__ __forceinline__ int x_slot(int tb, int f, int kg, int tr) { return ((tb * 8 + f) * 64 + 32 * kg + (tr ^ (2 * f + kg))) * 16; }

__device__ __forceinline__ void store_x(const u4 (&v)[PF_XC], unsigned char* buf, bool quarter_major, int tid)
{
#pragma unroll
    for (int i = 0; i < PF_XC; ++i) {
        const int c = tid + PF_NT * i;
        const int row = c >> 4, kc = c & 15;
        const int f = quarter_major ? ((kc >> 3) << 2) | (kc & 3) : kc >> 1;
        const int kg = quarter_major ? (kc >> 2) & 1 : kc & 1;
        *(u4*)(buf + x_slot(row >> 5, f, kg, row & 31)) = v[i];
    }
}

// The activation fragments of slice f + 2 are requested from LDS right after the MFMAs of slice f have been
// issued (two register sets): left to itself the compiler keeps two fragments and waits for each pair of
// LDS reads right before the two MFMAs that use them, and the LDS latency, not the MFMA pipe, then sets the
// pace of this phase.
__device__ __forceinline__ void contract_step(f16v (&acc)[4], const h8 (&bf)[8], const unsigned char* buf, int lane)
{
    const int tr = lane & 31, kg = lane >> 5;
    h8 af[2][4];
#pragma unroll
    for (int f = 0; f < 2; ++f)
#pragma unroll
        for (int mb = 0; mb < 4; ++mb) af[f][mb] = *(const h8*)(buf + x_slot(mb, f, kg, tr));
#pragma unroll
    for (int f = 0; f < 8; ++f) {
#pragma unroll
        for (int mb = 0; mb < 4; ++mb) acc[mb] = mfma32(af[f & 1][mb], bf[f], acc[mb]);
        if (f + 2 < 8) {
#pragma unroll
            for (int mb = 0; mb < 4; ++mb) af[f & 1][mb] = *(const h8*)(buf + x_slot(mb, f + 2, kg, tr));
        }
    }
    __builtin_amdgcn_sched_group_barrier(0x100, 8, 0);            // LDS reads of slices 0 and 1
#pragma unroll
    for (int f = 0; f < 6; ++f) {
        __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);        // the MFMAs of slice f
        __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);        // the LDS reads of slice f + 2
    }
    __builtin_amdgcn_sched_group_barrier(0x008, 8, 0);
}

template <bool V> struct PfFlag { static constexpr bool value = V; };

// FM: format of the first segment's weights (S_Q4, S_Q3, S_Q2 asymmetric; S_Q4S128, S_Q3S128, S_F16 for the
// down-projection launch).  FE2: S_NONE, or the format of a second segment's tiles (B: S_F16, S_Q4S128, S_Q3S128):
// the kernel then continues over a
// second segment of fp16 tiles (B) with its own activations (t).
template <int FM, int FE2>
__global__ __launch_bounds__(PF_NT, 2) void prefill_kernel(PrefillArgs ga)
{
    constexpr bool EXT = FE2 != S_NONE;
    constexpr bool E16 = FE2 == S_F16 || FE2 == S_NONE;           // second segment's tiles are fp16 (or there is none)
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int wn = wave;                                          // this wavefront's 128 tokens x 32 rows of the 128 x 256 tile
    int ntn = 0;                                                  // column tiles of all members
    for (int m = 0; m < ga.n; ++m) ntn += (ga.N[m] + PF_BN - 1) / PF_BN;
    const int ntm = (ga.M + PF_BM - 1) / PF_BM;
    const int tile_id = blockIdx.x % (ntn * ntm), ks = blockIdx.x / (ntn * ntm);     // ks > 0 only with ksplit > 1
    const int m0 = (tile_id / ntn) * PF_BM;
    int nt = tile_id % ntn, mem = 0;                              // column tile within its member
    while (mem + 1 < ga.n && nt >= (ga.N[mem] + PF_BN - 1) / PF_BN) {
        nt -= (ga.N[mem] + PF_BN - 1) / PF_BN;
        ++mem;
    }
    const PfView a{ga.x, ga.ldx, ga.w[mem], ga.w_scales[mem], ga.w_zeros[mem], ga.group, ga.x2[mem], ga.ldx2, ga.w2[mem], ga.w2_scales[mem],
                   ga.y[mem], ga.ldy[mem], ga.M, ga.N[mem], ga.K1, ga.K2, ga.ksplit, ga.part, ga.ldp, ga.pcol[mem]};
    const int R0 = nt * (PF_BN / 16);
    const int nblk = a.N / 16;
    const int h = (lane >> 4) & 1;
    const int Rl = R0 + 2 * wn + h < nblk ? R0 + 2 * wn + h : nblk - 1;   // the row block this lane supplies a row of, clamped to a valid one
    const int G1 = a.K1 / 128, G2 = EXT ? a.K2 / 128 : 0;
    const int sb = EXT ? 0 : ks * (G1 / a.ksplit);               // this workgroup's steps: [sb, GT)
    const int GT = EXT ? G1 + G2 : sb + G1 / a.ksplit;
    constexpr bool W16 = FM == S_F16;                             // first segment's weights are fp16 tiles
    unsigned char* const buf0 = eora_smem;
    unsigned char* const buf1 = eora_smem + PF_XS;

    f16v acc[4];                                                  // token blocks of 32
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int q = 0; q < 16; ++q) acc[i][q] = 0.f;

    // x slab of step s into registers (steps past the end re-read the last one; never stored)
    auto fetch_x = [&](u4 (&v)[PF_XC], int s) {
        s = s < GT ? s : GT - 1;
        if (EXT && s >= G1) load_x(v, a.x2, a.ldx2, a.M, m0, (s - G1) * 128, tid);
        else load_x(v, a.x, a.ldx, a.M, m0, s * 128, tid);
    };
    u4 xr[PF_XC];
    // the stored tiles of two steps are in flight: one step (about 2 us) is less than a memory round trip
    // under load.  Step sb + i uses set i & 1 (the loops below are unrolled in pairs: no run-time index).
    WPre<W16 ? S_Q4 : FM> wp[2];                                  // (unused for fp16 tiles)
    fetch_x(xr, sb);
    if constexpr (!W16) {
        const int lastw = (EXT ? G1 : GT) - 1;
        load_wpre<FM>(wp[0], a, Rl, sb, lane);
        load_wpre<FM>(wp[1], a, Rl, sb + 1 < lastw ? sb + 1 : lastw, lane);
    }
    store_x(xr, buf0, !W16, tid);
    fetch_x(xr, sb + 1);                                          // xr always holds the slab of the step after the one in LDS
    __syncthreads();

#ifdef EORA_TIMELINE
    long long tl[5] = {0, 0, 0, 0, 0}, tl0 = clock64(), tlstart = tl0;
#define PF_STAMP(i) do { const long long now = clock64(); tl[i] += now - tl0; tl0 = now; } while (0)
#else
#define PF_STAMP(i) do { } while (0)
#endif
    // Operands of step s into bf.  First segment: decode of the prefetched tiles and the request for the
    // following step's (fp16 tiles are operands as they are: no prefetch copy).  Second segment: B's tiles.
    h8 bf[8];
    const int last1 = (EXT ? G1 : GT) - 1;                        // last step of the first segment
    auto prep_main = [&](auto par_tag, int s) {                   // par_tag: (s - sb) & 1
        constexpr int PAR = decltype(par_tag)::value ? 1 : 0;
        s = s < last1 ? s : last1;                                // past the end: the last one again, never used
        if constexpr (W16) {
            load_b_frags(bf, a.w, a.K1, Rl, s, lane);
        } else {
            decode_wpre<FM>(wp[PAR], bf);
            load_wpre<FM>(wp[PAR], a, Rl, s + 2 < last1 ? s + 2 : last1, lane);
        }
    };
    auto prep_ext = [&](int s) {
        s = s < GT ? s : GT - 1;
        if constexpr (E16) {
            load_b_frags(bf, a.w2, a.K2, Rl, s - G1, lane);
        } else {                                                  // quantised B: a handful of steps, loaded and decoded in place
            WPre<E16 ? S_Q4S128 : FE2> wb;
            load_wpre_from<E16 ? S_Q4S128 : FE2>(wb, a.w2, a.w2_scales, nullptr, a.K2, 128, Rl, s - G1, lane);
            decode_wpre<E16 ? S_Q4S128 : FE2>(wb, bf);
        }
    };
    // The two wavefronts that share a SIMD (w and w + 4) run the two halves of a step in opposite order,
    // so that one decodes (VALU) while the other contracts (MFMA): wavefronts 0..3 decode step s at the
    // top of iteration s, wavefronts 4..7 decoded it at the bottom of iteration s - 1.  Measured with
    // both in the same order: the second decoder waits for the first, and its MFMAs then run alone.
    // Each order, and each kind of operand preparation, gets a loop of its own under wavefront-uniform
    // branches: with "if (late)" or "if (second segment)" inside one loop the compiler no longer knows how
    // many requests follow the one it needs and waits for all of them, i.e. for the x slab requested a
    // moment ago, at every decode.
    auto step = [&](auto late_tag, auto ext_tag, auto par_tag, int s) {     // par_tag: (s - sb) & 1
        constexpr bool LATE = decltype(late_tag)::value, EXTP = decltype(ext_tag)::value, PAR = decltype(par_tag)::value;
        PF_STAMP(4);
        unsigned char* const cur = ((s - sb) & 1) ? buf1 : buf0;
        unsigned char* const nxt = ((s - sb) & 1) ? buf0 : buf1;
        if constexpr (!LATE) {
            if constexpr (EXTP) prep_ext(s);
            else prep_main(PfFlag<PAR>{}, s);
            // nothing crosses this point: left alone, the scheduler sinks the requests for the next step's
            // weights below the MFMAs, and the next step then starts by waiting for them
            __builtin_amdgcn_sched_barrier(0);
        }
        PF_STAMP(0);
        contract_step(acc, bf, cur, lane);
#ifdef EORA_TIMELINE
        __builtin_amdgcn_sched_barrier(0);
        PF_STAMP(1);
#endif
        // the next step's slab goes to the other buffer (free since the barrier of the step before)
        store_x(xr, nxt, !((EXT && s + 1 >= G1) ? E16 : W16), tid);      // the fragment order follows the weight operand's
        fetch_x(xr, s + 2);
        if constexpr (LATE) {
            __builtin_amdgcn_sched_barrier(0);
            if constexpr (EXTP) prep_ext(s + 1);
            else prep_main(PfFlag<!PAR>{}, s + 1);
        }
#ifdef EORA_TIMELINE
        __builtin_amdgcn_sched_barrier(0);
        PF_STAMP(2);
#endif
        __syncthreads();
        PF_STAMP(3);
    };
    const int s1 = last1 + 1;                                     // first step of the second segment (= GT without one)
    // steps [from, to) in pairs, so that the parity of a step is known at compile time
    auto run = [&](auto late_tag, auto ext_tag, int from, int to) {
        int s = from;
        if ((s - sb) & 1) {
            if (s < to) step(late_tag, ext_tag, PfFlag<true>{}, s);
            ++s;
        }
        for (; s + 1 < to; s += 2) {
            step(late_tag, ext_tag, PfFlag<false>{}, s);
            step(late_tag, ext_tag, PfFlag<true>{}, s + 1);
        }
        if (s < to) step(late_tag, ext_tag, PfFlag<false>{}, s);
    };
    if (__builtin_amdgcn_readfirstlane(wave) >= PF_NW / 2) {
        prep_main(PfFlag<false>{}, sb);
        if constexpr (EXT) {
            run(PfFlag<true>{}, PfFlag<false>{}, sb, s1 - 1);
            run(PfFlag<true>{}, PfFlag<true>{}, s1 - 1, GT);
        } else {
            run(PfFlag<true>{}, PfFlag<false>{}, sb, GT);
        }
    } else {
        run(PfFlag<false>{}, PfFlag<false>{}, sb, s1);
        if constexpr (EXT) run(PfFlag<false>{}, PfFlag<true>{}, s1, GT);
    }
#ifdef EORA_TIMELINE
    if ((blockIdx.x == 0 || blockIdx.x == 700) && lane == 0)
        printf("wg %d wave %d: decode+wload %lld  contract %lld  storex+fetch %lld  barrier %lld  loop-top %lld  total %lld (clock64 ticks, %d steps)\n",
               (int)blockIdx.x, wave, tl[0], tl[1], tl[2], tl[3], tl[4], clock64() - tlstart, GT - sb);
#endif

    // ---- split contraction: this part's fp32 tile, 128-byte rows straight from the accumulators ------
    if (!EXT && a.ksplit > 1) {
#pragma unroll
        for (int mb = 0; mb < 4; ++mb)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int m = m0 + 32 * mb + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
                const int o = (R0 + 2 * wn) * 16 + (lane & 31);
                if (m < a.M && o < a.N) a.part[((size_t)ks * a.M + m) * a.ldp + a.pcol + o] = acc[mb][v];
            }
        return;
    }
    // ---- epilogue: fp32 -> fp16, transpose through LDS, 128-byte row stores ----------------------------
    // (wavefront-private staging tiles of 64 tokens, two passes: 40 KiB, so that the kernel's LDS stays at the
    // two x slabs and two workgroups fit a compute unit)
    constexpr int TS = 40;                                        // halves per token row in the staging tile (32 + pad)
    _Float16* tile = (_Float16*)eora_smem + wave * 64 * TS;
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
        if (pass) __syncthreads();                                // (keeps the two passes of a wavefront apart in program order)
#pragma unroll
        for (int mb2 = 0; mb2 < 2; ++mb2)
#pragma unroll
            for (int v = 0; v < 16; ++v)
                tile[(32 * mb2 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3)) * TS + (lane & 31)] = (_Float16)acc[2 * pass + mb2][v];
        __syncthreads();
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            const int tok = 16 * it + (lane >> 2), chunk = lane & 3;  // 64-byte rows: four 16-byte chunks
            const int m = m0 + 64 * pass + tok, o = (R0 + 2 * wn) * 16 + chunk * 8;
            const u4 v = *(const u4*)(tile + tok * TS + chunk * 8);
            if (m < a.M && o < a.N) *(u4*)((_Float16*)a.y + (size_t)m * a.ldy + o) = v;
        }
    }
}

template <int FM, int FE2>
static hipError_t launch_pf(const PrefillArgs& a, hipStream_t stream)
{
    constexpr bool EXT = FE2 != S_NONE;
    auto kern = prefill_kernel<FM, FE2>;
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, PF_LDS);
    if (e != hipSuccess) return e;
    int ntn = 0;
    for (int m = 0; m < a.n; ++m) ntn += (a.N[m] + PF_BN - 1) / PF_BN;
    const int ntm = (a.M + PF_BM - 1) / PF_BM;
    note_launch("prefill FM=%d EXT=%d ksplit=%d n=%d FE=%d", FM, (int)EXT, a.ksplit, a.n, FE2);
    hipLaunchKernelGGL(kern, dim3(ntn * ntm * (EXT ? 1 : a.ksplit)), dim3(PF_NT), PF_LDS, stream, a);
    return hipGetLastError();
}

__global__ __launch_bounds__(256) void reduce_parts_kernel(const float* __restrict__ part, _Float16* __restrict__ T, size_t count, int ksplit)
{
    const size_t i = 4 * ((size_t)blockIdx.x * 256 + threadIdx.x);
    if (i >= count) return;
    f4 v = *(const f4*)(part + i);
    for (int ks = 1; ks < ksplit; ++ks) v += *(const f4*)(part + ks * count + i);      // fixed order
    typedef _Float16 h4 __attribute__((ext_vector_type(4)));
    *(h4*)(T + i) = h4{(_Float16)v[0], (_Float16)v[1], (_Float16)v[2], (_Float16)v[3]};
}

hipError_t launch_reduce_parts(const float* part, void* T, size_t count, int ksplit, hipStream_t stream)
{
    hipLaunchKernelGGL(reduce_parts_kernel, dim3((unsigned)((count / 4 + 255) / 256)), dim3(256), 0, stream, part, (_Float16*)T, count, ksplit);
    return hipGetLastError();
}

template <int FM>
static hipError_t launch_pf_ext(const PrefillArgs& a, int fe2, hipStream_t stream)
{
    switch (fe2) {
        case S_NONE: return launch_pf<FM, S_NONE>(a, stream);
        case S_F16: return launch_pf<FM, S_F16>(a, stream);
        case S_Q4S128: return launch_pf<FM, S_Q4S128>(a, stream);
        case S_Q3S128: return launch_pf<FM, S_Q3S128>(a, stream);
        default: return hipErrorInvalidValue;
    }
}

// fe2: S_NONE, or the format of the second segment's tiles
hipError_t launch_prefill(const PrefillArgs& a, int fm, int fe2, hipStream_t stream)
{
    switch (fm) {
        case S_Q4: return launch_pf_ext<S_Q4>(a, fe2, stream);
        case S_Q3: return launch_pf_ext<S_Q3>(a, fe2, stream);
        case S_Q2: return launch_pf_ext<S_Q2>(a, fe2, stream);
        case S_Q4S128: return fe2 != S_NONE ? hipErrorInvalidValue : launch_pf<S_Q4S128, S_NONE>(a, stream);
        case S_Q3S128: return fe2 != S_NONE ? hipErrorInvalidValue : launch_pf<S_Q3S128, S_NONE>(a, stream);
        case S_F16: return fe2 != S_NONE ? hipErrorInvalidValue : launch_pf<S_F16, S_NONE>(a, stream);
        default: return hipErrorInvalidValue;
    }
}

// T[m][c] = 0 wherever column c does not belong to the adapter of token row m (several adapters side by side)
__global__ __launch_bounds__(256) void mask_t_kernel(_Float16* __restrict__ T, const int* __restrict__ adapter, int M, int R, int r_per)
{
    const size_t i = 8 * ((size_t)blockIdx.x * 256 + threadIdx.x);       // eight columns of one row (R and r_per are multiples of 8)
    if (i >= (size_t)M * R) return;
    const int m = (int)(i / R), c = (int)(i % R);
    if (adapter[m] != c / r_per) *(u4*)(T + i) = u4{0u, 0u, 0u, 0u};
}

hipError_t launch_mask_t(void* T, const int* adapter, int M, int R, int r_per, hipStream_t stream)
{
    const size_t chunks = (size_t)M * R / 8;
    hipLaunchKernelGGL(mask_t_kernel, dim3((unsigned)((chunks + 255) / 256)), dim3(256), 0, stream, (_Float16*)T, adapter, M, R, r_per);
    return hipGetLastError();
}

}  // namespace eora
