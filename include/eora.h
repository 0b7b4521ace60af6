/*
 * eora.h - C ABI of the MI355X (gfx950) library for the EoRA compensated compressed linear layer
 *
 *      y = x . What^T + (x . A^T) . B^T
 *
 * (arXiv 2410.21271, Sec. 3: forward equation "What X + B' A X", Algorithm 1 step 7; the paper
 * writes the column convention, this library the row convention: x is M x d_in, What is
 * d_out x d_in, A is r x d_in, B is d_out x r, y is M x d_out.)  What is the unmodified compressed
 * backbone weight (Sec. 2), A and B the rank-r
 * compensation factors produced offline by Algorithm 1 steps 1-6.
 *
 * General rules
 *  - Plain C.  Every pointer is a DEVICE pointer unless the comment says HOST.
 *  - The caller owns all memory.  The library allocates nothing on the device and keeps no state.
 *  - Device work is enqueued on `stream` (a hipStream_t passed as void*, NULL = default stream);
 *    no call synchronises with the host.  Results are valid once the caller has synchronised.
 *  - Every function returns an eora_status.  Arguments are validated before anything is enqueued:
 *    on an error nothing is launched and no output is touched.
 *  - Inputs are never modified.  y is OVERWRITTEN (the caller need not clear it).
 *  - All device pointers must be 16-byte aligned.
 *  - Determinism: no floating-point atomics are used; the reduction order is fixed by the launch
 *    configuration, so equal inputs give bit-equal outputs from run to run.
 *
 * Stored formats (all weight-like operands are TILE-MAJOR; rows = output rows, K = contraction
 * length).  A tile is 16 rows x KT columns and maps onto one 64-lane wavefront: lane
 * l = 16*j + n owns row n of the tile and the j-th quarter of its columns.  Tiles are ordered
 * row-block first: tile = (row/16) * (K/KT) + col/KT.
 *
 *  Q4 (4-bit codes; KT = 128 for the backbone, min(128,K) for a factor): lane l owns columns
 *      c = (KT/4)*j + 8*t + kk of the tile, t = 0..KT/32-1, kk = 0..7.  32-bit word
 *      tile*(2*KT) + l*(KT/32) + t  holds the eight codes of (l, t); column kk sits in nibble
 *      e = 4*(kk%2) + kk/2 (bits 4e..4e+3): even columns in the low 16 bits, odd ones in the
 *      high 16 bits, so that one AND extracts two adjacent columns as a pair of 16-bit lanes.
 *  Q3 (3-bit codes, KT = 128, exactly 3.0 bits per weight): lane l owns three consecutive words
 *      tile*192 + 3*l + d.  Its 32 columns cc form pairs p = cc/2 (h = cc%2: 0 low / 1 high
 *      16-bit half).  Pairs 0..14 sit in word p/5 at bits 16h + 3*(p%5) .. +2.  Bit 15 of each
 *      half carries the last pair: bit b of the code of column 30+h is bit 16h+15 of word b.
 *  Q2 (2-bit codes, KT = 128, backbone only; the 2-bit setting of App. A.14): lane l owns two
 *      consecutive words tile*128 + 2*l + u; column cc = 0..31 of its quarter sits in word u = cc/16
 *      at bits 16h + 2p .. +1, h = cc%2, p = (cc%16)/2: eight pairs of adjacent columns per word.
 *      Zero-points (0..3) use the common nibble array below.
 *  zero-points: 4-bit, one per (row, group), row-major, eight groups per 32-bit word: word
 *      row*NGW + q/8, nibble q%8, with NG = K/group, q = col/group, NGW = ceil(NG/8) (so a lane
 *      finds the zero-points of four consecutive k-tiles of its row in one word).
 *  scales: fp16, row-major, element row*NG + q.
 *  F16 (fp16 factor, KT = 32): element (tile*64 + l)*8 + i is column 32*(col/32) + 8*j + i.
 *  SP24 (2:4 sparse fp16, tile = 16 rows x 128 dense columns): lane l owns dense columns
 *      64*s + 16*j + 4*q + p (s = 0,1; q = 0..3 group of four; p = 0..3 position); each group
 *      keeps two values v = 0,1 at positions p_0 < p_1.  values: fp16 element
 *      tile*1024 + s*512 + l*8 + 2*q + v.  indices: one 32-bit word per (tile, lane), bits
 *      16*s + 4*q + 2*v .. +1 hold p_v.
 *  SP24Q4 (2:4 sparse, kept values as 4-bit codes: pruned, then quantised, Sec. 4.2): tiles as SP24.
 *      qtiles: three 32-bit words per (tile, lane), words (tile*64 + l)*3 + 0, 1, 2: word s = 0, 1 holds
 *      the lane's eight kept values of half s, element e = 2*q + v in nibble 4*(e%2) + e/2; word 2 is
 *      the SP24 index word.  qmeta: one word per (tile, row n), word tile*16 + n: bits 0..15 the fp16
 *      scale, bits 16..19 the zero-point of the quantisation group that holds the tile's columns (a
 *      group of `group` DENSE columns, a multiple of 128, spans group/128 tiles, which repeat them).
 *      A kept value at dense column c of row o is scale * (code - zero).  0.41 bytes per dense weight.
 *
 * Dequantisation (asymmetric group-wise quantisation, Sec. 4.1 and App. A.11):
 *      What[o][i] = scale[o][i/group] * (code[o][i] - zero[o][i/group])
 * Quantised factors (Sec. 4.5, "quantised EoRA") are symmetric 4-bit: the zero-point is the
 * constant 8, scales are fp16, one per row and per group of min(128,K) columns of the
 * contraction dimension (d_in for A, r for B).
 */
#ifndef EORA_H
#define EORA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    EORA_OK = 0,
    EORA_ERR_NULL = -1,        /* a required pointer is NULL */
    EORA_ERR_SHAPE = -2,       /* a size violates the constraints listed at the function */
    EORA_ERR_UNSUPPORTED = -3, /* w_bits / ab_bits / group value not implemented */
    EORA_ERR_ALIGN = -4,       /* a device pointer is not 16-byte aligned */
    EORA_ERR_WORKSPACE = -5,   /* workspace missing or smaller than eora_workspace_bytes() */
    EORA_ERR_LAUNCH = -6,      /* the HIP runtime refused a launch (hipGetLastError) */
    EORA_ERR_VALUE = -7,       /* host packer: a code / zero-point / position is out of range */
    EORA_ERR_TIMEOUT = -8,     /* eora_workspace_error: a bounded in-kernel wait expired (results invalid) */
    EORA_ERR_NOT_CONVERGED = -9 /* eora_factors: the Jacobi sweeps did not settle within their limit */
} eora_status;

/* HOST.  Static string for a status code. */
const char* eora_status_string(int status);

/* ---------------------------------------------------------------------------------------------
 * Sizes (HOST, pure functions).  Return 0 for invalid arguments.
 * ------------------------------------------------------------------------------------------ */
size_t eora_qweight_bytes(int d_in, int d_out, int w_bits);          /* d_out*d_in*w_bits/8 */
size_t eora_qzeros_bytes(int d_in, int d_out, int group);            /* d_out*ceil(d_in/group/8)*4 */
size_t eora_scales_bytes(int d_in, int d_out, int group);            /* d_out*(d_in/group)*2 */
size_t eora_sp24_values_bytes(int d_in, int d_out);                  /* d_out*d_in          */
size_t eora_sp24_indices_bytes(int d_in, int d_out);                 /* d_out*d_in/8        */
size_t eora_sp24q4_tiles_bytes(int d_in, int d_out);                 /* d_out*d_in*3/8      */
size_t eora_sp24q4_meta_bytes(int d_in, int d_out);                  /* d_out*(d_in/128)*4  */
/* Scratch the forward calls need: a header of counters, the down-projection t = x.A^T (M x r)
 * and its partial sums.  The workspace must be cleared ONCE with eora_workspace_init() before the
 * first forward call on it; every forward call leaves it usable for the next, so no per-call
 * clearing (and nothing a HIP graph could not replay) is needed.  Calls that may overlap in time
 * (different streams) need different workspaces.  r == 0 still needs a workspace.  A workspace of
 * the size of the largest (M, r) serves smaller calls too.  For 5 .. 127 tokens and d_in >= 16384 the
 * size also holds 4 * M * d_out floats: a 2:4 call of such a shape may cut its contraction into ranges
 * whose partial outputs are added, in a fixed order, by a second kernel of the same call. */
size_t eora_workspace_bytes(int M, int d_in, int d_out, int r);
/* Size that lets eora_linear_q_group() serve n_members members in one pass also for M >= 128 (the
 * down-projections of all members then sit side by side in the scratch).  With a workspace of only
 * eora_workspace_bytes() such a call still works, member by member. */
size_t eora_workspace_bytes_group(int M, int d_in, int r, int n_members);
/* Enqueues the clearing of all `workspace_bytes` bytes on `stream` (and the start of the workspace's launch
 * counter at a value no other initialisation in this process uses, so that memory which held a workspace
 * before can never be mistaken for this one's). */
int eora_workspace_init(void* workspace, size_t workspace_bytes, void* stream);
/* Diagnostic.  SYNCHRONISES `stream`, then reports EORA_ERR_TIMEOUT if a kernel that used this
 * workspace gave up its bounded wait for the down-projection (its y is then invalid; re-initialise
 * the workspace), else EORA_OK.  The wait cannot expire in a healthy run: the workgroups it waits
 * for are running and never wait themselves. */
int eora_workspace_error(const void* workspace, void* stream);
/* HOST, test hook: iterations of that bounded wait (process-wide; default 1 << 22, about a second).
 * 0 makes a wait give up at once if t is not ready when it first looks.  A negative value makes every such
 * wait count as expired without looking, so that the error path (EORA_ERR_TIMEOUT from eora_workspace_error,
 * y without the low-rank term) can be exercised deterministically with every kernel still terminating
 * normally. */
void eora_debug_set_spin_limit(int iterations);
/* HOST, test hook: the fewest 16-row blocks (all members of a launch together) for which a call with 5 .. 16 tokens
 * and d_in of 1024, 2048 or 4096 takes the kernel that keeps x resident in LDS (process-wide; default 256, the
 * measured crossover: launches with fewer rows are faster in the kernel that serves 5 .. 127 tokens).  Tests lower
 * it to reach that kernel with small shapes; a negative value restores the default. */
void eora_debug_set_resident_min_blocks(int blocks);
/* HOST, test hook: route != 0 makes eora_factors() always take the eigendecomposition of the Gram matrix (the
 * route of a nearly singular one), so that tests reach it with well-conditioned inputs too; 0 restores the choice
 * by the pivots (process-wide). */
void eora_debug_set_factors_route(int route);
/* HOST, test hook: writes into out (capacity bytes, NUL-terminated) the name and template parameters of the
 * layer kernel the most recent forward launch of this process chose, e.g. "sparse_wide FA=5 NW=8 TB=4 VQ=0 n=1"
 * (empty before the first launch), so that a test can assert that its shape reaches the instantiation it is
 * meant to cover.  Process-wide, not synchronised with concurrent callers.  Errors: EORA_ERR_NULL. */
int eora_debug_last_launch(char* out, size_t capacity);
/* Measurement probes, enqueued on `stream` like a forward call, for quoting a layer kernel's time against what
 * the device does with no arithmetic at all.  kind 0: an empty kernel of 256 workgroups (the launch floor; src
 * and bytes ignored).  kind 1: a kernel that only reads `bytes` bytes from src (DEVICE, 16-byte aligned;
 * 32 KiB per workgroup, every request of a workgroup in flight at once) and stores nothing: the streaming-read
 * rate a launch of that size can reach.  sink: DEVICE, at least 256 bytes, 16-byte aligned (never written in
 * practice).  Constraints: bytes > 0 and a multiple of 32768.  Errors: EORA_ERR_NULL / ALIGN / SHAPE /
 * UNSUPPORTED (kind) / LAUNCH. */
int eora_debug_probe(int kind, const void* src, size_t bytes, void* sink, void* stream);

/* ---------------------------------------------------------------------------------------------
 * Host-side packers: logical arrays (HOST pointers, row-major) -> stored bytes (HOST pointers).
 * They define the stored formats above in code; outputs may then be copied to the device.
 * Constraints: d_out % 16 == 0, d_in % 128 == 0, group % 128 == 0, d_in % group == 0.
 * ------------------------------------------------------------------------------------------ */
/* codes: d_out x d_in, values < 2^w_bits; zeros: d_out x d_in/group, same range;
 * scales: d_out x d_in/group fp16 bit patterns.  w_bits is 2, 3 or 4. */
int eora_pack_q(const uint8_t* codes, const uint8_t* zeros, const uint16_t* scales,
                int d_in, int d_out, int w_bits, int group,
                void* qweight_out, void* qzeros_out, void* scales_out);
/* fp16 factor, rows x cols (A: r x d_in; B: d_out x r).  rows % 16 == 0, cols % 32 == 0. */
int eora_pack_factor_f16(const uint16_t* mat, int rows, int cols, void* out);
/* 4-bit symmetric factor: codes rows x cols in 0..15 (zero-point 8), scales rows x cols/KT fp16,
 * KT = min(128, cols).  rows % 16 == 0, cols == 64 or cols % 128 == 0. */
int eora_pack_factor_q4(const uint8_t* codes, const uint16_t* scales, int rows, int cols,
                        void* q_out, void* scales_out);
/* 3-bit symmetric factor (App. A.9 quantises the factors to 3 and 4 bits): codes rows x cols in 0..7
 * (zero-point 4) in the Q3 tile layout, scales rows x cols/128 fp16.  rows % 16 == 0, cols % 128 == 0. */
int eora_pack_factor_q3(const uint8_t* codes, const uint16_t* scales, int rows, int cols,
                        void* q_out, void* scales_out);
/* 2:4 sparse backbone: vals d_out x d_in/2 fp16 bit patterns (the kept values in column order),
 * pos d_out x d_in/2 their positions 0..3 inside the group of four, strictly ascending per pair. */
int eora_pack_sp24(const uint16_t* vals, const uint8_t* pos, int d_in, int d_out,
                   void* values_out, void* indices_out);
/* 2:4 sparse backbone with 4-bit kept values: codes d_out x d_in/2 in 0..15 (the kept values in column
 * order), pos as above, zeros / scales d_out x d_in/group as for eora_pack_q (the group of a kept value
 * is that of its dense column).  qtiles_out takes eora_sp24q4_tiles_bytes, qmeta_out eora_sp24q4_meta_bytes. */
int eora_pack_sp24q4(const uint8_t* codes, const uint8_t* pos, const uint8_t* zeros, const uint16_t* scales,
                     int d_in, int d_out, int group, void* qtiles_out, void* qmeta_out);

/* ---------------------------------------------------------------------------------------------
 * The layer.  Sec. 3 forward equation / Alg. 1 step 7; the fused low-rank path follows Sec. 4.5
 * and App. A.6 (B's product accumulates into the same output as the quantised product) and goes
 * further: x.A^T is folded in as well, so y is written exactly once.
 *
 * x        fp16 row-major M x d_in
 * qweight  Q4 or Q3 tiles (w_bits), scales / qzeros as described above
 * A, B     F16 tiles (ab_bits == 16; A_scales = B_scales = NULL), Q4 symmetric tiles with fp16
 *          scales (ab_bits == 4) or Q3 symmetric tiles with fp16 scales (ab_bits == 3).  r == 0 (then A, B may be NULL) is the bare compressed layer,
 *          i.e. the adapter switched off.
 * y        fp16 row-major M x d_out, overwritten; fp32 accumulation, one round-to-nearest-even
 *          conversion at the end.
 * Constraints: M >= 0 (M == 0 is a no-op), d_out % 16 == 0, d_in % 128 == 0, group % 128 == 0,
 *          d_in % group == 0 (group == d_in is channel-wise quantisation), w_bits in {2,3,4},
 *          ab_bits in {16,4,3}, r <= 512 and r % 32 == 0 (ab_bits 16), r == 64 or r % 128 == 0
 *          (ab_bits 4), r % 128 == 0 (ab_bits 3).
 * ------------------------------------------------------------------------------------------ */
int eora_linear_q(const void* x, const void* qweight, const void* scales, const void* qzeros,
                  const void* A, const void* B, const void* A_scales, const void* B_scales,
                  void* y, int M, int d_in, int d_out, int r, int w_bits, int group, int ab_bits,
                  void* workspace, size_t workspace_bytes, void* stream);

/* eora_linear_q for callers that cannot allocate device memory or pass a workspace (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): same arguments without the workspace, same
 * kernels, bit-identical results.  The workspace is an array inside the library's device code (3.3 MiB on every
 * GPU the library runs on, held until the process ends), found once per device with hipGetSymbolAddress and
 * cleared once, on the first call's stream; the call allocates nothing.
 * Limit: M <= 127 (EORA_ERR_WORKSPACE beyond: the many-token path needs scratch that grows with M); all other
 * constraints and errors as eora_linear_q.  Every call on a GPU shares that GPU's array: calls that may overlap
 * in time on one GPU (different streams without ordering between them) race and must use eora_linear_q with
 * workspaces of their own; so must a second call whose stream is not ordered after the first call's stream
 * (which carries the one-time clearing). */
int eora_linear_q_static(const void* x, const void* qweight, const void* scales, const void* qzeros,
                         const void* A, const void* B, const void* A_scales, const void* B_scales,
                         void* y, int M, int d_in, int d_out, int r, int w_bits, int group, int ab_bits,
                         void* stream);

/* Several layers that read the SAME x in one launch: the query / key / value projections, or the
 * gate / up projections, of a decoder layer (the paper compensates every linear of the model the
 * same way, Sec. 3; which of them share an input is the transformer's structure).  Member m is an
 * eora_linear_q layer of its own (own weights, factors, output and d_out); M, d_in, r, w_bits,
 * group and ab_bits are common.  For one to four tokens and group == 128 this is one launch, which
 * pays the launch and the hand-over of x.A^T once, with results bit-identical to n_members separate
 * eora_linear_q calls.  For 5 .. 127 tokens it is one launch too when the members together have enough
 * rows to fill the chip, and for M >= 128 (fp16 factors, r % 128 == 0, or r == 0) the members' rows
 * form one GEMM, which keeps narrow members (d_out = 1024) from leaving most of the chip idle; in
 * these two cases sums may be split differently than in a separate call (results agree to rounding,
 * and are the same from run to run).  Other shapes run the members one after the other.
 * members: HOST array (read during the call only) of 1..4 entries; pointers inside are DEVICE
 * pointers with the meaning and constraints of the eora_linear_q arguments of the same name.
 * workspace: at least the largest eora_workspace_bytes(M, d_in, d_out_m, r); see
 * eora_workspace_bytes_group(). */
typedef struct {
    const void* qweight;
    const void* scales;
    const void* qzeros;
    const void* A;
    const void* B;
    const void* A_scales;
    const void* B_scales;
    void* y;
    int d_out;
} eora_q_member;
int eora_linear_q_group(const void* x, const eora_q_member* members, int n_members,
                        int M, int d_in, int r, int w_bits, int group, int ab_bits,
                        void* workspace, size_t workspace_bytes, void* stream);

/* Several adapters over one backbone in one batch: token row m is compensated with the pair
 * (A_a, B_a), a = adapter_of_row[m] in [0, n_adapters), or not at all for a = -1:
 *      y[m] = x[m].What^T + (x[m].A_a^T).B_a^T
 * (Sec. 1, Sec. 3: the compensation is a separate residual path that leaves What untouched, so pairs
 * fitted for different tasks can be loaded next to one backbone and chosen per request.)
 * A_all: the adapters' A stacked by rows, (n_adapters*r) x d_in, packed as ONE factor (eora_pack_factor_*);
 * B_all: their B side by side, d_out x (n_adapters*r), packed as one factor; A_scales / B_scales likewise
 * for ab_bits 4 and 3.  adapter_of_row: DEVICE, M int32, read by the kernel (values outside [-1, n_adapters)
 * behave as -1).  All adapters are streamed whatever the rows select; the backbone is streamed once.
 * Constraints: as eora_linear_q with rank n_adapters*r (<= 512); r % 32 == 0 (r % 128 == 0 for
 * ab_bits 4 and 3, so that no scale group spans two adapters); workspace of
 * eora_workspace_bytes(M, d_in, d_out, n_adapters*r).  Errors as eora_linear_q. */
int eora_linear_q_multi(const void* x, const void* qweight, const void* scales, const void* qzeros,
                        const void* A_all, const void* B_all, const void* A_scales, const void* B_scales,
                        const void* adapter_of_row, void* y,
                        int M, int d_in, int d_out, int r, int n_adapters, int w_bits, int group, int ab_bits,
                        void* workspace, size_t workspace_bytes, void* stream);

/* Same layer with a 2:4 structured-sparse fp16 backbone (Sec. 1, Sec. 4.2); A, B are F16 tiles.
 * Constraints as above with r % 32 == 0. */
int eora_linear_sp24(const void* x, const void* values, const void* indices,
                     const void* A, const void* B, void* y,
                     int M, int d_in, int d_out, int r,
                     void* workspace, size_t workspace_bytes, void* stream);

/* Same layer with a backbone that is 2:4 pruned and then quantised to 4 bits (Sec. 4.2 evaluates the
 * combination; stored format SP24Q4 above); A, B are F16 tiles.  All pointers DEVICE.  The kept values
 * enter the sparse MFMA as fp16(scale * (code - zero)): one fp16 rounding per weight.
 * Constraints and errors as for eora_linear_sp24 (the quantisation groups are part of the stored bytes). */
int eora_linear_sp24q4(const void* x, const void* qtiles, const void* qmeta,
                       const void* A, const void* B, void* y,
                       int M, int d_in, int d_out, int r,
                       void* workspace, size_t workspace_bytes, void* stream);

/* Several 2:4 layers that read the SAME x in one launch (query / key / value, gate / up), as
 * eora_linear_q_group does for quantised backbones: member m is an eora_linear_sp24 layer (values and
 * indices given, qtiles = qmeta = NULL) or an eora_linear_sp24q4 layer (qtiles and qmeta given, values =
 * indices = NULL) of its own; all members are of the same kind and share M, d_in and r.  One launch for
 * M <= 256 (results equal those of separate calls to rounding; bit-identical for M <= 4); larger M runs
 * the members one after the other.  members: HOST array of 1..4 entries, read during the call only.
 * workspace: at least the largest eora_workspace_bytes(M, d_in, d_out_m, r).  Errors as eora_linear_sp24. */
typedef struct {
    const void* values;
    const void* indices;
    const void* qtiles;
    const void* qmeta;
    const void* A;
    const void* B;
    void* y;
    int d_out;
} eora_sp_member;
int eora_linear_sp24_group(const void* x, const eora_sp_member* members, int n_members,
                           int M, int d_in, int r, void* workspace, size_t workspace_bytes, void* stream);

/* ---------------------------------------------------------------------------------------------
 * Parity exports (integer / exact work, compared bit for bit against the CPU oracle).
 * ------------------------------------------------------------------------------------------ */
/* codes_u8: d_out x d_in row-major; zeros_u8: d_out x d_in/group row-major. */
int eora_unpack_q(const void* qweight, const void* qzeros, void* codes_u8, void* zeros_u8,
                  int d_in, int d_out, int w_bits, int group, void* stream);
/* W_f32: d_out x d_in row-major fp32; scale*(code-zero) is exact in fp32. */
int eora_dequant_q(const void* qweight, const void* scales, const void* qzeros, void* W_f32,
                   int d_in, int d_out, int w_bits, int group, void* stream);
/* W_f16: d_out x d_in row-major fp16 with the pruned positions written as +0. */
int eora_expand_sp24(const void* values, const void* indices, void* W_f16,
                     int d_in, int d_out, void* stream);
/* W_f32: d_out x d_in row-major fp32: scale*(code-zero) at the kept positions (exact in fp32), +0 elsewhere. */
int eora_expand_sp24q4(const void* qtiles, const void* qmeta, void* W_f32, int d_in, int d_out, void* stream);

/* ---------------------------------------------------------------------------------------------
 * Calibration: the factors themselves (Sec. 3, Algorithm 1, steps 1-6), in fp64 on the device.
 * ------------------------------------------------------------------------------------------ */
/* HOST.  Scratch eora_factors() needs (five matrices of the size of the weight or of the Gram matrix
 * in fp64); 0 for invalid arguments. */
size_t eora_factors_workspace_bytes(int d_in, int d_out, int r);
/* All pointers DEVICE, 16-byte aligned, row-major.  W_f32, W_hat_f32: d_out x d_in fp32, the weight and
 * its compressed version (e.g. from eora_dequant_q).  Xt_f32: d_in x n_tokens fp32, the calibration
 * activations X~ with one column per token.  Outputs: B_f64 = B' = U' Sigma' (d_out x r), A_f64 = A
 * (r x d_in), sigma_f64 (r singular values of dW Q', descending; may be NULL), so that What + B'A
 * minimises || (W - What - B'A) X~ ||_F over rank-r corrections (Theorem 1).  Signs of the r components
 * are arbitrary (B'A is not).  eig_floor in [0, 1): eigenvalues of X~ X~^T below eig_floor times the
 * largest are raised to it before the inverse square root of step 6 (the paper assumes an invertible Q').
 * How steps 2-4 and 6 are computed: with X~ X~^T = L L^T (Cholesky), dW L is dW Q sqrt(Lambda) times an orthogonal
 * matrix on the right, so step 5 finds the same U' and Sigma' and step 6's A is Sigma'^-1 U'^T dW: the same B' and A
 * as the eigendecomposition gives whenever no eigenvalue is clamped.  That route is taken when every pivot of the
 * factorisation stays above 1e4 * eig_floor * max diag(X~ X~^T); otherwise (a Gram matrix that close to singular,
 * e.g. fewer tokens than channels) the eigendecomposition with the clamp is computed, by a one-sided (block)
 * Jacobi iteration.  The SVD of step 5 is such an iteration in both cases.  The call SYNCHRONISES `stream` once
 * after the factorisation, once per sweep and before returning, and allocates nothing on the device.
 * stats: HOST pointer to eight doubles or NULL: for steps 2-3, then for the SVD, the number of sweeps, the
 * milliseconds its rounds took (events on `stream`), the workgroups that rotated their rows, and the rows a
 * workgroup handles per round (16: block rounds, taken when the row count is a multiple of 16 and the row
 * lengths are multiples of 128; 2: pair rounds).  The Cholesky route reports, in place of the first four, 0 sweeps,
 * its milliseconds, the length of the rows the SVD's sweeps rotated, and 0.  That length is min(d_in, d_out) when the
 * matrix of step 5, at least twice as long as it has rows, was first reduced to a square factor with the same singular
 * values and left singular vectors (T T^T = C C^T by a second Cholesky factorisation; not possible for an error of
 * rank below min(d_in, d_out)), else max(d_in, d_out).
 * Constraints: d_in, d_out even and <= 16384, 1 <= r <= min(d_in, d_out), n_tokens >= 1.
 * Errors: EORA_ERR_NULL / SHAPE / VALUE (eig_floor) / WORKSPACE / ALIGN / LAUNCH, and
 * EORA_ERR_NOT_CONVERGED (outputs then undefined). */
int eora_factors(const void* W_f32, const void* W_hat_f32, const void* Xt_f32,
                 int n_tokens, int d_in, int d_out, int r, double eig_floor,
                 void* B_f64, void* A_f64, void* sigma_f64,
                 void* workspace, size_t workspace_bytes, void* stream, double* stats);

/* All pointers DEVICE, 16-byte aligned.  The factors of eora_factors() as the forward entry points read
 * them (ab_bits == 16): rounded once to fp16 and written in the F16 tile layout, A_tiles r x d_in
 * (2*r*d_in bytes), B_tiles d_out x r.  balance != 0 first rescales component i by
 * s_i = sqrt(|B'_i| / |A_i|) (column i of B' divided by s_i, row i of A multiplied by it): B'A is
 * unchanged and both factors of a component get the norm sqrt(|B'_i| |A_i|), which keeps them inside
 * fp16's range whatever the singular values are (B' = U' Sigma' carries them, A the inverse square roots
 * of Lambda; Alg. 1 steps 5 and 6).  scratch: r doubles (balance != 0 only).  Asynchronous on `stream`.
 * Constraints: d_in % 32 == 0, d_out % 16 == 0, r % 32 == 0.
 * Errors: EORA_ERR_NULL / SHAPE / ALIGN / WORKSPACE (scratch) / LAUNCH. */
int eora_factors_store_f16(const void* B_f64, const void* A_f64, int d_in, int d_out, int r, int balance,
                           void* A_tiles, void* B_tiles, void* scratch, size_t scratch_bytes, void* stream);

/* The same hand-over with QUANTISED factors (Sec. 4.5, App. A.9), ab_bits in {4, 3}: symmetric
 * round-to-nearest per row and group of min(128, K) columns of the contraction dimension,
 * scale = fp16(max |v| / qpos), qpos = 7 (4-bit) or 3 (3-bit), 1 for an all-zero group;
 * code = clip(rint(v / scale) + zp, 1, 2 zp - 1) with the implicit zero-point zp = 8 or 4.  Outputs in the
 * Q4 / Q3 symmetric factor formats the forward entry points read with the same ab_bits: A_q r x d_in,
 * A_scales r x d_in/128 fp16, B_q d_out x r, B_scales d_out x r/min(128, r) fp16.  balance, scratch as
 * for eora_factors_store_f16.  Constraints: d_in % 128 == 0, d_out % 16 == 0, r % 128 == 0 (or r == 64
 * with ab_bits 4).  Errors: EORA_ERR_NULL / UNSUPPORTED / SHAPE / ALIGN / WORKSPACE / LAUNCH. */
int eora_factors_store_q(const void* B_f64, const void* A_f64, int d_in, int d_out, int r, int ab_bits, int balance,
                         void* A_q, void* A_scales, void* B_q, void* B_scales,
                         void* scratch, size_t scratch_bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* EORA_H */
