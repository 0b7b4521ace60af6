// Internal launch interface between the C-ABI entry points (api.hip) and the kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace eora {

// stored formats a contraction segment can read
enum SegFmt { S_NONE = 0, S_Q4 = 1, S_Q3 = 2, S_Q4S128 = 3, S_Q4S64 = 4, S_F16 = 5, S_Q2 = 6, S_Q3S128 = 7 };

// backbone format of a bit width (2, 3 or 4)
inline int backbone_format(int w_bits) { return w_bits == 4 ? S_Q4 : (w_bits == 3 ? S_Q3 : S_Q2); }

// Workspace header (32-bit words).  Counters that different workgroups hit at the same time sit in
// different 128-byte lines.
constexpr int HDR_EPOCH = 0;                    // advanced once per low-rank launch
constexpr int HDR_ERROR = 1;                    // sticky: a bounded wait expired
constexpr int HDR_TOP = 32;                     // arrival counter of the sub-counters
constexpr int HDR_SUB0 = 64;                    // HDR_NSUB arrival sub-counters, HDR_SUB_STRIDE words apart
constexpr int HDR_SUB_STRIDE = 32;
constexpr int HDR_NSUB = 32;
constexpr int HDR_FLAGS0 = 2048;                // per token block: one flag per unit of t
constexpr int HDR_FLAGS_PER_BLOCK = 512;        // (r/16) * kcn <= 32 * 16
constexpr int MAX_YBLOCKS = 16;                 // token blocks per launch (256 tokens)
constexpr int HDR_FLAG_REPLICAS = 8;             // the decode kernels keep 8 copies of the flags, one per group of pollers
constexpr int HDR_FLAGS_REPLICA_STRIDE = HDR_FLAGS_PER_BLOCK * MAX_YBLOCKS;
constexpr int HDR_WORDS = HDR_FLAGS0 + HDR_FLAGS_REPLICA_STRIDE * HDR_FLAG_REPLICAS;
constexpr int MAX_KCN = 8;                      // k-ranges of the down-projection (quantised backbones; the 2:4 decode kernel takes up to 16)

// Host-side record of the kernel instantiation the most recent layer launch of this process chose, read
// back through eora_debug_last_launch() (tests assert that a shape reaches the instantiation it is meant to
// cover).  `fmt` is a printf format for up to six ints and must be a string literal.  Not synchronised.
void note_launch(const char* fmt, int a = 0, int b = 0, int c = 0, int d = 0, int e = 0, int f = 0, int g = 0);

struct FusedArgs {
    const _Float16* x;        // M x d_in fp16 row-major
    const void* w;            // backbone tiles
    const _Float16* w_scales;
    const uint32_t* w_zeros;
    const void* A;            // r x d_in tiles
    const _Float16* A_scales;
    const void* B;            // d_out x r tiles
    const _Float16* B_scales;
    _Float16* y;              // M x d_out fp16 row-major
    uint32_t* hdr;            // workspace header
    float* tpart;             // (timeline builds: stamps)
    unsigned long long* tpair;   // token blocks x kcn x 16 x r (value, tag) pairs: partials of t
    int M, d_in, d_out, r, group, kcn, spin_limit;
    // several adapters side by side in A and B (r = their ranks together): token row m keeps only the
    // r_per columns of t that belong to adapter[m] (-1: none).  nullptr: one adapter, nothing masked.
    // Read by fused.hip and wideq.hip.
    const int* adapter;
    int r_per;
};

hipError_t launch_fused(const FusedArgs& a, int fm, int fa, int fe, hipStream_t stream);

// Kernel for 5 .. 127 tokens (wideq.hip): x shared through LDS by the wavefronts of a workgroup.
bool wide_q_fits(int M, int d_in, int d_out, int r);
hipError_t launch_wide_q(const FusedArgs& a, int fm, int fa, int fe, hipStream_t stream);
// The same kernel for up to four linears that read the same x (same M, d_in, r, kcn, formats; own weights,
// factors, y, d_out, tpair region): the members' workgroups follow one another in one launch.
struct WideGroupArgs {
    FusedArgs m[4];
    int first[4];             // first workgroup of member i
    int flag0[4];             // first flag of member i inside a token block's flags
    int n;
};
bool wide_q_group_fits(int M, int d_in, const int* d_out, int n, int r);
hipError_t launch_wide_q_group(const FusedArgs* members, int n, int fm, int fa, int fe, hipStream_t stream);

// Kernel for 5 .. 16 tokens with x resident in LDS (stream.hip): one workgroup of 16 wavefronts per compute unit keeps
// the whole x (d_in <= 4096) and finishes every output tile it starts; t is handed over as tagged pairs.
struct StreamArgs {
    const _Float16* x;                  // M x d_in fp16 row-major, shared
    const void* w[4];                   // backbone tiles
    const _Float16* w_scales[4];
    const uint32_t* w_zeros[4];
    const void* A[4];                   // r x d_in tiles
    const _Float16* A_scales[4];
    const void* B[4];                   // d_out x r tiles
    const _Float16* B_scales[4];
    _Float16* y[4];                     // M x d_out fp16 row-major
    int d_out[4];
    int n;                              // members, 1..4
    uint32_t* hdr;                      // workspace header
    unsigned long long* tpair;          // [member][16 tokens][r] tagged t
    int M, d_in, r, spin_limit;
    int q, qp;                          // output row blocks per workgroup; per workgroup that begins with a block of A (set by the launcher)
    const int* adapter;                 // null, or one adapter index per token row (several adapters side by side in A and B)
    int r_per;                          // rank of one adapter (adapter != null)
    uint32_t cpr_magic;                 // ceil(2^32 / (16-byte chunks of x per row of a range)): division by multiply-high (set by the launcher)
    int S;                              // ranges of the contraction, one workgroup each per run of row blocks (set by the launcher)
    unsigned long long* part;           // tagged partial tiles that cross ranges, behind t in the same region (set by the launcher)
};
// d_out: the members' rows (n of them)
bool stream_fits(int M, int d_in, int group, int r, int fm, int fa, const int* d_out, int n);
hipError_t launch_stream(const StreamArgs& a, int fm, int fa, int fe, hipStream_t stream);
void set_resident_min_blocks(int blocks);      // test hook: stream_fits' lower limit of row blocks (negative: the default)

// Decode kernel for 1..4 tokens (small.hip).  One launch serves up to MAX_GROUP linears that read the
// same x (the q/k/v or the gate/up projections of a decoder layer): same d_in, rank and formats,
// own weights, factors, output and d_out.
constexpr int MAX_GROUP = 4;
struct GroupArgs {
    const _Float16* x;                  // M x d_in fp16 row-major, shared
    const void* w[MAX_GROUP];           // backbone tiles
    const _Float16* w_scales[MAX_GROUP];
    const uint32_t* w_zeros[MAX_GROUP];
    const void* A[MAX_GROUP];           // r x d_in tiles
    const _Float16* A_scales[MAX_GROUP];
    const void* B[MAX_GROUP];           // d_out x r tiles
    const _Float16* B_scales[MAX_GROUP];
    _Float16* y[MAX_GROUP];             // M x d_out fp16 row-major
    int d_out[MAX_GROUP];
    int n;                              // members, 1..MAX_GROUP
    uint32_t* hdr;                      // workspace header
    unsigned long long* tpair;          // members x kcn x 16 x r (value, tag) pairs: partials of t
    int M, d_in, r, group, kcn, spin_limit;
    // several adapters side by side in A and B (one member; r = their ranks together): token row m keeps only the
    // r_per columns of t that belong to adapter[m] (anything else: none).  nullptr: nothing masked.
    const int* adapter;
    int r_per;
    int c2n;                            // set by the launcher: -1, or the number of leading consumer strips of two row blocks in a launch whose later strips are single row blocks
};
// whether the shape fits the decode kernel, with its wavefront / quad split
bool small_kernel_fits(int M, int d_in, int group, int* nw, int* nq);
hipError_t launch_small(const GroupArgs& a, int fm, int fa, int fe, int nw, int nq, hipStream_t stream);
hipError_t launch_clear_words(uint32_t* p, int nwords, uint32_t epoch0, hipStream_t stream);

struct SparseArgs {
    const _Float16* x;        // M x d_in fp16 row-major
    const _Float16* values;   // SP24 kept values (fp16 backbone), or
    const uint32_t* indices;  // SP24 positions, or
    const uint32_t* qtiles;   // SP24Q4: three words per (tile, lane): codes of both halves, positions
    const uint32_t* qmeta;    // SP24Q4: one word per (tile, row): fp16 scale | zero-point << 16
    const void* A;            // r x d_in F16 tiles
    const void* B;            // d_out x r F16 tiles
    _Float16* y;              // M x d_out fp16 row-major
    uint32_t* hdr;            // workspace header
    float* tpart;             // token blocks x kcn x 16 x r fp32 partials of t (kernel for many tokens and rows)
    unsigned long long* tpair;   // the same as (value, tag) pairs (decode kernel)
    int M, d_in, d_out, r, kcn, spin_limit;
    // long contractions at 5 .. 127 tokens (kernel for many tokens, one linear): room for the fp32 partial outputs of
    // up to SP_MAX_SPLIT ranges of the contraction, [range][M][d_out] (null: the contraction is never split); the
    // launcher sets ksplit
    float* ypart;
    int ksplit;
};
constexpr int SP_MAX_SPLIT = 4;
constexpr int SP_SPLIT_MIN_D_IN = 16384;        // contractions from this length on may be split
// bytes of SparseArgs::ypart a call of this shape needs (0: no split is ever chosen for it)
size_t sparse_split_bytes(int M, int d_in, int d_out);

hipError_t launch_sparse(const SparseArgs& a, hipStream_t stream);
// up to four 2:4 linears that read the same x in one launch (same M, d_in, r, kcn, backbone kind; own weights,
// factors, y, d_out and regions of the partials)
struct SparseGroupArgs {
    SparseArgs m[4];
    int first[4];             // first workgroup of member i
    int flag0[4];             // first flag of member i inside a token block's flags
    int n;
};
hipError_t launch_sparse_group(const SparseArgs* members, int n, hipStream_t stream);

// Prefill GEMM (prefill.hip): y[M x N] = act[M x K1] . W1^T (+ act2[M x K2] . W2^T), fp16 output, for up to
// MAX_GROUP members that read the same act (own weights, second-segment operands, output and N).
struct PrefillArgs {
    const _Float16* x;        // first segment's activations, row stride ldx (shared)
    int ldx;
    int group;
    int ldx2;                 // row stride of the second segment's activations
    int M, K1, K2;
    int ksplit;               // > 1: workgroup (tile, ks) contracts the ks-th part of K1 only and writes its
    float* part;              //      fp32 tile to part[ks][M][ldp] (columns pcol ..) instead of y; no second segment then
    int ldp;
    int n;                    // members
    const void* w[MAX_GROUP];            // first segment's weight tiles (N rows, K1 columns)
    const _Float16* w_scales[MAX_GROUP];
    const uint32_t* w_zeros[MAX_GROUP];
    const _Float16* x2[MAX_GROUP];       // second segment's activations (t)
    const void* w2[MAX_GROUP];           // second segment's tiles (N rows, K2 columns)
    const _Float16* w2_scales[MAX_GROUP];   // their scales (quantised B)
    void* y[MAX_GROUP];                  // fp16, row stride ldy
    int ldy[MAX_GROUP];
    int N[MAX_GROUP];
    int pcol[MAX_GROUP];
};

// fm: format of the first segment's weights; fe2: S_NONE, or the format of the second segment's tiles
hipError_t launch_prefill(const PrefillArgs& a, int fm, int fe2, hipStream_t stream);
// T (fp16 M x R, R adapters' ranks together): zero wherever a column does not belong to adapter[m]'s r_per columns
hipError_t launch_mask_t(void* T, const int* adapter, int M, int R, int r_per, hipStream_t stream);

// T[i] = fp16(sum over ks, in order, of part[ks][i]), i < count (count % 4 == 0)
hipError_t launch_reduce_parts(const float* part, void* T, size_t count, int ksplit, hipStream_t stream);

hipError_t launch_unpack_q(const uint32_t* qweight, const uint32_t* qzeros, uint8_t* codes, uint8_t* zeros,
                           int d_in, int d_out, int w_bits, int group, hipStream_t stream);
hipError_t launch_dequant_q(const uint32_t* qweight, const _Float16* scales, const uint32_t* qzeros, float* W,
                            int d_in, int d_out, int w_bits, int group, hipStream_t stream);
hipError_t launch_expand_sp24(const _Float16* values, const uint32_t* indices, _Float16* W,
                              int d_in, int d_out, hipStream_t stream);
hipError_t launch_expand_sp24q4(const uint32_t* qtiles, const uint32_t* qmeta, float* W, int d_in, int d_out, hipStream_t stream);

// measurement probes (debug.hip): an empty launch, and a pure streaming read of `bytes` (a multiple of 32 KiB)
hipError_t launch_probe_empty(uint32_t* sink, hipStream_t stream);
hipError_t launch_probe_stream(const void* src, size_t bytes, uint32_t* sink, hipStream_t stream);

}  // namespace eora
