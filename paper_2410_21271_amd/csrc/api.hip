// C-ABI entry points: argument validation and the static choice of kernel.  No device memory is
// allocated here and nothing is kept between calls.
#include "eora.h"
#include "kernels.hpp"

#include <atomic>
#include <cstdio>
#include <cstdlib>
#include <mutex>

namespace eora {

namespace {
struct LaunchNote { const char* fmt; int v[7]; };
LaunchNote g_last_launch = {nullptr, {0, 0, 0, 0, 0, 0, 0}};
}  // namespace

void note_launch(const char* fmt, int a, int b, int c, int d, int e, int f, int g) { g_last_launch = {fmt, {a, b, c, d, e, f, g}}; }

}  // namespace eora

namespace {

using namespace eora;

constexpr size_t WS_HEADER = 270336;       // counters and flags (HDR_WORDS 32-bit words)
constexpr int MAX_RANK = 512;
constexpr int CHUNK_TOKENS = 16 * MAX_YBLOCKS;      // tokens per launch of the small-M kernels
constexpr int PREFILL_MIN_TOKENS = 128;             // from here on the GEMM kernel takes over
static_assert(HDR_WORDS * 4 <= WS_HEADER, "header too small");

int g_spin_limit = 1 << 22;                // bounded wait of the up-projection (about a second)

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline size_t round256(size_t v) { return (v + 255) & ~(size_t)255; }

int check_backbone_shape(int M, int d_in, int d_out, int r)
{
    if (M < 0 || d_in <= 0 || d_out <= 0 || r < 0) return EORA_ERR_SHAPE;
    if (d_out % 16 || d_in % 128 || r > MAX_RANK) return EORA_ERR_SHAPE;
    return EORA_OK;
}

// Set EORA_VERBOSE=1 to have a refused launch explain itself on stderr.
bool failed(hipError_t e, const char* what)
{
    if (e == hipSuccess) return false;
    static const bool verbose = getenv("EORA_VERBOSE") != nullptr;      // read once per process
    if (verbose) fprintf(stderr, "eora: %s: %s\n", what, hipGetErrorString(e));
    return true;
}

int check_group(int d_in, int group)
{
    if (group <= 0 || group % 128 || d_in % group) return EORA_ERR_SHAPE;
    return EORA_OK;
}

// workspace = header | tagged partials (decode kernel) | fp32 partials (fused.hip, sparse.hip) | t (fp16, prefill).
// The regions sit at fixed offsets whatever (M, r) a call has, so that calls of different shapes on one
// workspace never read one region's bytes as another's.  (token blocks) x kcn <= 32 and r <= 512.
constexpr size_t MAX_PART_ELEMS = 32 * 16 * 512;
constexpr size_t WS_PAIRS = WS_HEADER;
constexpr size_t WS_PARTS = WS_PAIRS + MAX_PART_ELEMS * 8;
constexpr size_t WS_T = WS_PARTS + MAX_PART_ELEMS * 4;

// one launch of the kernel for 5 .. 16 tokens (x resident in LDS) for validated members that share x; the caller has
// checked stream_fits
int launch_stream_group(const void* x, const eora_q_member* members, int n, int M, int d_in, int r, int w_bits,
                        int fa, int fe, void* workspace, hipStream_t stream, const int* adapter = nullptr, int r_per = 0)
{
    StreamArgs a{};
    a.x = (const _Float16*)x;
    for (int m = 0; m < 4; ++m) {
        const eora_q_member& e = members[m < n ? m : 0];
        a.w[m] = e.qweight;
        a.w_scales[m] = (const _Float16*)e.scales;
        a.w_zeros[m] = (const uint32_t*)e.qzeros;
        a.A[m] = e.A;
        a.A_scales[m] = (const _Float16*)e.A_scales;
        a.B[m] = e.B;
        a.B_scales[m] = (const _Float16*)e.B_scales;
        a.y[m] = (_Float16*)e.y;
        a.d_out[m] = m < n ? e.d_out : 0;
    }
    a.n = n;
    a.hdr = (uint32_t*)workspace;
    a.tpair = (unsigned long long*)((char*)workspace + WS_PAIRS);
    a.M = M;
    a.d_in = d_in;
    a.r = r;
    a.spin_limit = g_spin_limit;
    a.adapter = adapter;
    a.r_per = r_per;
    if (failed(launch_stream(a, backbone_format(w_bits), fa, fe, stream), "linear_q (stream)")) return EORA_ERR_LAUNCH;
    return EORA_OK;
}

// factor formats of the (r, ab_bits) a call names
int factor_formats(int r, int ab_bits, int* fa, int* fe)
{
    *fa = *fe = S_NONE;
    if (r == 0) return EORA_OK;
    if (ab_bits == 16) {
        if (r % 32) return EORA_ERR_SHAPE;
        *fa = *fe = S_F16;
    } else if (ab_bits == 4) {
        if (r != 64 && r % 128) return EORA_ERR_SHAPE;
        *fe = (r == 64) ? S_Q4S64 : S_Q4S128;
        *fa = S_Q4S128;
    } else if (ab_bits == 3) {
        if (r % 128) return EORA_ERR_SHAPE;
        *fa = *fe = S_Q3S128;
    } else {
        return EORA_ERR_UNSUPPORTED;
    }
    return EORA_OK;
}

// k-ranges of the down-projection: many for few tokens (every consumer adds the partials itself),
// a divisor of the number of 128-wide k-tiles
int pick_kcn(int M, int d_in)
{
    // (token blocks) x kcn <= 32: the partials' region is sized for that
    const int yblocks = ((M < CHUNK_TOKENS ? M : CHUNK_TOKENS) + 15) / 16;
    int cap = 32 / yblocks < MAX_KCN ? 32 / yblocks : MAX_KCN;
    // with more than 4 tokens every consumer reads (tokens x r x kcn) partials: few ranges
    // (a long contraction at many tokens keeps eight: its producers would otherwise take longer than the launch
    // streams; measured on the 28672- and 14336-long down projections at 64 tokens, 73.4 -> 69.3 and 40.5 -> 39.1 us)
    if (M > 4 && cap > 4 && !(M > 16 && d_in > 8192)) cap = 4;
    int kcn = 1;
    for (int c = 2; c <= cap; ++c)
        if ((d_in / 128) % c == 0) kcn = c;
    return kcn;
}

// Parts the prefill down-projection t = x.A^T (few output tiles: r / 128 per 128 tokens) splits its
// contraction into so that the launch fills the chip; their fp32 tiles are added in a fixed order.
int pick_ksplit(int M, int d_in, int r)
{
    if (r == 0) return 1;
    const int tiles = ((M + 127) / 128) * ((r + 255) / 256), G = d_in / 128;       // the GEMM kernel's tile is 128 x 256
    int want = (256 + tiles - 1) / tiles;
    want = want > 8 ? 8 : want;
    int ks = 1;
    for (int c = 2; c <= want; ++c)
        if (G % c == 0) ks = c;
    return ks;
}

// Many tokens: MFMA-bound GEMM (t = x.A^T first, then one GEMM over d_in and r)
// (fp16, 4-bit or 3-bit factors; the rank in whole steps of 128)
bool prefill_fits(int M, int r, int ab_bits) { return M >= PREFILL_MIN_TOKENS && (r == 0 || r % 128 == 0) && (ab_bits == 16 || ab_bits == 4 || ab_bits == 3 || r == 0); }

// scratch of the prefill path for n members: t (fp16, M x n*r) and the fp32 parts of its split contraction
size_t prefill_scratch_bytes(int M, int d_in, int r, int n)
{
    const int ks = pick_ksplit(M, d_in, n * r);
    return round256((size_t)M * n * r * 2) + (ks > 1 ? (size_t)ks * M * n * r * sizeof(float) : 0);
}

// validated members that share x, as GEMMs: one launch for every member's t (the members' A side by side), one
// for every member's y
int launch_prefill_group(const void* x, const eora_q_member* members, int n, int M, int d_in, int r, int w_bits, int group,
                         int fa, int fe, const int* adapter, int r_per, void* workspace, hipStream_t stream)
{
    _Float16* T = (_Float16*)((char*)workspace + WS_T);           // M x (n * r): member m owns columns m*r ..
    if (r > 0) {
        PrefillArgs p{};
        p.x = (const _Float16*)x; p.ldx = d_in;
        p.group = 128;
        p.M = M; p.K1 = d_in;
        p.n = n;
        p.ksplit = pick_ksplit(M, d_in, n * r);
        p.part = (float*)((char*)workspace + WS_T + round256((size_t)M * n * r * 2));
        p.ldp = n * r;
        for (int m = 0; m < n; ++m) {
            p.w[m] = members[m].A;
            p.w_scales[m] = (const _Float16*)members[m].A_scales;
            p.y[m] = T + (size_t)m * r; p.ldy[m] = n * r;
            p.N[m] = r; p.pcol[m] = m * r;
        }
        if (failed(launch_prefill(p, fa, S_NONE, stream), "prefill down-projection")) return EORA_ERR_LAUNCH;
        if (p.ksplit > 1 && failed(launch_reduce_parts(p.part, T, (size_t)M * n * r, p.ksplit, stream), "prefill down-projection sum"))
            return EORA_ERR_LAUNCH;
        // several adapters side by side (one member): a token row keeps its own adapter's columns of t
        if (adapter && failed(launch_mask_t(T, adapter, M, n * r, r_per, stream), "prefill adapter mask")) return EORA_ERR_LAUNCH;
    }
    PrefillArgs p{};
    p.x = (const _Float16*)x; p.ldx = d_in;
    p.group = group;
    p.M = M; p.K1 = d_in; p.K2 = r;
    p.ldx2 = n * r;
    p.n = n;
    p.ksplit = 1;
    for (int m = 0; m < n; ++m) {
        p.w[m] = members[m].qweight;
        p.w_scales[m] = (const _Float16*)members[m].scales;
        p.w_zeros[m] = (const uint32_t*)members[m].qzeros;
        p.x2[m] = T + (size_t)m * r;
        p.w2[m] = members[m].B;
        p.w2_scales[m] = (const _Float16*)members[m].B_scales;
        p.y[m] = members[m].y; p.ldy[m] = members[m].d_out;
        p.N[m] = members[m].d_out;
    }
    if (failed(launch_prefill(p, backbone_format(w_bits), r > 0 ? fe : S_NONE, stream), "prefill")) return EORA_ERR_LAUNCH;
    return EORA_OK;
}

// one launch of the decode kernel for validated members that share x
int launch_group(const void* x, const eora_q_member* members, int n, int M, int d_in, int r, int w_bits, int group,
                 int fa, int fe, int nw, int nq, void* workspace, hipStream_t stream, const int* adapter = nullptr, int r_per = 0)
{
    if (M == 0) return EORA_OK;
    GroupArgs a{};
    a.x = (const _Float16*)x;
    for (int m = 0; m < n; ++m) {
        a.w[m] = members[m].qweight;
        a.w_scales[m] = (const _Float16*)members[m].scales;
        a.w_zeros[m] = (const uint32_t*)members[m].qzeros;
        a.A[m] = members[m].A;
        a.A_scales[m] = (const _Float16*)members[m].A_scales;
        a.B[m] = members[m].B;
        a.B_scales[m] = (const _Float16*)members[m].B_scales;
        a.y[m] = (_Float16*)members[m].y;
        a.d_out[m] = members[m].d_out;
    }
    a.n = n;
    a.hdr = (uint32_t*)workspace;
    a.tpair = (unsigned long long*)((char*)workspace + WS_PAIRS);
    a.M = M;
    a.d_in = d_in;
    a.r = r;
    a.group = group;
    a.kcn = pick_kcn(M, d_in);
    if (r > 128) {
        // Large ranks: fewer k-ranges.  Every consumer reads r x kcn pairs of t and there are (r / 16) x kcn producers:
        // at most 1024 pairs per consumer, but no range longer than 4096 columns (measured on the 8B layer with 4-bit
        // factors, 7 launches: rank 512 90.9 -> 73.1 us, rank 256 67.1 -> 61.5 us; rank 128 is faster with eight).
        int cap = 1024 / r < 2 ? 2 : 1024 / r;
        while (cap * 4096 < d_in) cap *= 2;
        while (a.kcn > cap && a.kcn % 2 == 0) a.kcn /= 2;
    }
    a.spin_limit = g_spin_limit;
    a.adapter = adapter;
    a.r_per = r_per;
    a.c2n = -1;
    if (failed(launch_small(a, backbone_format(w_bits), fa, fe, nw, nq, stream), "linear_q (decode)")) return EORA_ERR_LAUNCH;
    return EORA_OK;
}

}  // namespace

extern "C" {

size_t eora_workspace_bytes(int M, int d_in, int d_out, int r)
{
    if (check_backbone_shape(M, d_in, d_out, r) != EORA_OK) return 0;
    // partials of t for the small-M kernels, and t itself as fp16 M x r for the prefill GEMM
    // (and, for a 2:4 call with a long contraction at 5 .. 127 tokens, the partial outputs of its ranges)
    return WS_T + (M >= PREFILL_MIN_TOKENS ? prefill_scratch_bytes(M, d_in, r, 1) : sparse_split_bytes(M, d_in, d_out));
}

size_t eora_workspace_bytes_group(int M, int d_in, int r, int n_members)
{
    if (n_members < 1 || n_members > MAX_GROUP || check_backbone_shape(M, d_in, 16, r) != EORA_OK) return 0;
    return WS_T + (M >= PREFILL_MIN_TOKENS ? prefill_scratch_bytes(M, d_in, r, n_members) : 0);
}

int eora_workspace_init(void* workspace, size_t workspace_bytes, void* stream)
{
    if (!workspace) return EORA_ERR_NULL;
    if (!aligned16(workspace)) return EORA_ERR_ALIGN;
    if (workspace_bytes < WS_HEADER) return EORA_ERR_WORKSPACE;
    // everything is cleared, not only the header: the tagged partials must not hold a leftover word
    // that reads as the tag of a coming launch
    if (workspace_bytes / 4 > 0x7fffffffull) return EORA_ERR_WORKSPACE;
    // The epoch does not start at 0: tags and flags are compared with epoch + 1, and memory that held a workspace
    // before (freed and handed out again) may still sit in a cache with that incarnation's tags.  Every
    // initialisation in this process starts from its own range of 2^20 epochs, so a tag never means two things.
    static std::atomic<uint32_t> incarnation{0};
    const uint32_t epoch0 = ((incarnation.fetch_add(1) + 1u) & 0xFFFu) << 20;
    if (failed(launch_clear_words((uint32_t*)workspace, (int)(workspace_bytes / 4), epoch0, (hipStream_t)stream), "workspace_init"))
        return EORA_ERR_LAUNCH;
    return EORA_OK;
}

int eora_workspace_error(const void* workspace, void* stream)
{
    if (!workspace) return EORA_ERR_NULL;
    uint32_t flag = 0;
    if (hipMemcpyAsync(&flag, (const uint32_t*)workspace + HDR_ERROR, sizeof(flag), hipMemcpyDeviceToHost,
                       (hipStream_t)stream) != hipSuccess)
        return EORA_ERR_LAUNCH;
    if (hipStreamSynchronize((hipStream_t)stream) != hipSuccess) return EORA_ERR_LAUNCH;
    return flag ? EORA_ERR_TIMEOUT : EORA_OK;
}

void eora_debug_set_spin_limit(int iterations) { g_spin_limit = iterations < 0 ? -1 : iterations; }

void eora_debug_set_resident_min_blocks(int blocks) { set_resident_min_blocks(blocks); }

int eora_debug_probe(int kind, const void* src, size_t bytes, void* sink, void* stream)
{
    if (!sink) return EORA_ERR_NULL;
    if (!aligned16(sink)) return EORA_ERR_ALIGN;
    if (kind == 0) {
        if (failed(launch_probe_empty((uint32_t*)sink, (hipStream_t)stream), "probe (empty)")) return EORA_ERR_LAUNCH;
        return EORA_OK;
    }
    if (kind != 1) return EORA_ERR_UNSUPPORTED;
    if (!src) return EORA_ERR_NULL;
    if (!aligned16(src)) return EORA_ERR_ALIGN;
    if (bytes == 0 || bytes % 32768 || bytes / 32768 > 0x7fffffffull) return EORA_ERR_SHAPE;
    if (failed(launch_probe_stream(src, bytes, (uint32_t*)sink, (hipStream_t)stream), "probe (stream)")) return EORA_ERR_LAUNCH;
    return EORA_OK;
}

int eora_debug_last_launch(char* out, size_t capacity)
{
    if (!out || capacity == 0) return EORA_ERR_NULL;
    const LaunchNote n = g_last_launch;
    if (!n.fmt) {
        out[0] = 0;
        return EORA_OK;
    }
    snprintf(out, capacity, n.fmt, n.v[0], n.v[1], n.v[2], n.v[3], n.v[4], n.v[5], n.v[6]);
    return EORA_OK;
}

// every check of one quantised layer; nothing is enqueued
static int validate_linear_q(const void* x, const eora_q_member& e, int M, int d_in, int r, int w_bits, int group,
                             int ab_bits, const void* workspace, size_t workspace_bytes, int* fa, int* fe)
{
    if (!x || !e.qweight || !e.scales || !e.qzeros || !e.y) return EORA_ERR_NULL;
    if (w_bits < 2 || w_bits > 4) return EORA_ERR_UNSUPPORTED;
    int rc = check_backbone_shape(M, d_in, e.d_out, r);
    if (rc != EORA_OK) return rc;
    rc = check_group(d_in, group);
    if (rc != EORA_OK) return rc;
    *fe = *fa = S_NONE;
    if (r > 0) {
        if (!e.A || !e.B) return EORA_ERR_NULL;
        if (ab_bits != 16 && ab_bits != 4 && ab_bits != 3) return EORA_ERR_UNSUPPORTED;
        if (ab_bits != 16 && (!e.A_scales || !e.B_scales)) return EORA_ERR_NULL;
        rc = factor_formats(r, ab_bits, fa, fe);
        if (rc != EORA_OK) return rc;
        if (!aligned16(e.A) || !aligned16(e.B) || !aligned16(e.A_scales) || !aligned16(e.B_scales)) return EORA_ERR_ALIGN;
    }
    if (!aligned16(x) || !aligned16(e.qweight) || !aligned16(e.scales) || !aligned16(e.qzeros) || !aligned16(e.y))
        return EORA_ERR_ALIGN;
    if (!workspace) return EORA_ERR_WORKSPACE;
    if (!aligned16(workspace)) return EORA_ERR_ALIGN;
    if (workspace_bytes < eora_workspace_bytes(M, d_in, e.d_out, r)) return EORA_ERR_WORKSPACE;
    return EORA_OK;
}

// one validated quantised layer
static int run_linear_q(const void* x, const eora_q_member& e, int M, int d_in, int r, int w_bits, int group, int ab_bits,
                        int fa, int fe, void* workspace, void* stream)
{
    const void *qweight = e.qweight, *scales = e.scales, *qzeros = e.qzeros, *A = e.A, *B = e.B;
    const void *A_scales = e.A_scales, *B_scales = e.B_scales;
    void* y = e.y;
    const int d_out = e.d_out;
    if (M == 0) return EORA_OK;

    if (prefill_fits(M, r, ab_bits)) return launch_prefill_group(x, &e, 1, M, d_in, r, w_bits, group, fa, fe, nullptr, 0, workspace, (hipStream_t)stream);

    int nw = 0, nq = 0;
    if (small_kernel_fits(M, d_in, group, &nw, &nq))
        return launch_group(x, &e, 1, M, d_in, r, w_bits, group, fa, fe, nw, nq, workspace, (hipStream_t)stream);

    if (stream_fits(M, d_in, group, r, backbone_format(w_bits), fa, &d_out, 1))
        return launch_stream_group(x, &e, 1, M, d_in, r, w_bits, fa, fe, workspace, (hipStream_t)stream);

    // k-ranges of the down-projection: a divisor of the number of 128-wide k-tiles
    const int kcn = pick_kcn(M, d_in);
    for (int m0 = 0; m0 < M; m0 += CHUNK_TOKENS) {
        FusedArgs a{};
        a.x = (const _Float16*)x + (size_t)m0 * d_in;
        a.w = qweight;
        a.w_scales = (const _Float16*)scales;
        a.w_zeros = (const uint32_t*)qzeros;
        a.A = A;
        a.A_scales = (const _Float16*)A_scales;
        a.B = B;
        a.B_scales = (const _Float16*)B_scales;
        a.y = (_Float16*)y + (size_t)m0 * d_out;
        a.hdr = (uint32_t*)workspace;
        a.tpart = (float*)((char*)workspace + WS_PARTS);
        a.tpair = (unsigned long long*)((char*)workspace + WS_PAIRS);
        a.M = M - m0 < CHUNK_TOKENS ? M - m0 : CHUNK_TOKENS;
        a.d_in = d_in;
        a.d_out = d_out;
        a.r = r;
        a.group = group;
        a.kcn = kcn;
        a.spin_limit = g_spin_limit;
        const int fm = backbone_format(w_bits);
        const hipError_t e = wide_q_fits(a.M, d_in, d_out, r) ? launch_wide_q(a, fm, fa, fe, (hipStream_t)stream)
                                                               : launch_fused(a, fm, fa, fe, (hipStream_t)stream);
        if (failed(e, "linear_q")) return EORA_ERR_LAUNCH;
    }
    return EORA_OK;
}

int eora_linear_q(const void* x, const void* qweight, const void* scales, const void* qzeros,
                  const void* A, const void* B, const void* A_scales, const void* B_scales,
                  void* y, int M, int d_in, int d_out, int r, int w_bits, int group, int ab_bits,
                  void* workspace, size_t workspace_bytes, void* stream)
{
    const eora_q_member e{qweight, scales, qzeros, A, B, A_scales, B_scales, y, d_out};
    int fa, fe;
    const int rc = validate_linear_q(x, e, M, d_in, r, w_bits, group, ab_bits, workspace, workspace_bytes, &fa, &fe);
    if (rc != EORA_OK) return rc;
    return run_linear_q(x, e, M, d_in, r, w_bits, group, ab_bits, fa, fe, workspace, stream);
}

// ---- the same layer for callers that cannot allocate ---------------------------------------------------------
namespace {
// Workspace of eora_linear_q_static: one array per GPU the library's code is loaded on, held until the process
// ends.  Its size is that of eora_workspace_bytes() for any call below PREFILL_MIN_TOKENS tokens (header, tagged
// partials, fp32 partials).  In host code the array's name is only a handle for hipGetSymbolAddress: the device
// address it yields (per device) is what kernels and the clearing launch are given.
constexpr size_t STATIC_SCRATCH_BYTES = WS_T;
__device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];
constexpr int MAX_DEVICES = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[MAX_DEVICES] = {};
bool g_scratch_cleared[MAX_DEVICES] = {};

// the current device's array, cleared (enqueued on `stream`) the first time it is handed out
int static_scratch(void** out, hipStream_t stream)
{
    int device = -1;
    if (hipGetDevice(&device) != hipSuccess || device < 0 || device >= MAX_DEVICES) return EORA_ERR_LAUNCH;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[device]) {
        void* p = nullptr;
        if (failed(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)), "static scratch address") || !p) return EORA_ERR_LAUNCH;
        g_scratch_ptr[device] = p;
    }
    if (!g_scratch_cleared[device]) {
        const int rc = eora_workspace_init(g_scratch_ptr[device], STATIC_SCRATCH_BYTES, stream);
        if (rc != EORA_OK) return rc;
        g_scratch_cleared[device] = true;
    }
    *out = g_scratch_ptr[device];
    return EORA_OK;
}
}  // namespace

int eora_linear_q_static(const void* x, const void* qweight, const void* scales, const void* qzeros,
                         const void* A, const void* B, const void* A_scales, const void* B_scales,
                         void* y, int M, int d_in, int d_out, int r, int w_bits, int group, int ab_bits, void* stream)
{
    if (M >= PREFILL_MIN_TOKENS) return EORA_ERR_WORKSPACE;       // the many-token path needs scratch that grows with M
    const eora_q_member e{qweight, scales, qzeros, A, B, A_scales, B_scales, y, d_out};
    int fa, fe;
    // every check before the array is touched (a placeholder stands in for the workspace pointer)
    int rc = validate_linear_q(x, e, M, d_in, r, w_bits, group, ab_bits, x, STATIC_SCRATCH_BYTES, &fa, &fe);
    if (rc != EORA_OK) return rc;
    if (M == 0) return EORA_OK;
    void* ws = nullptr;
    rc = static_scratch(&ws, (hipStream_t)stream);
    if (rc != EORA_OK) return rc;
    return run_linear_q(x, e, M, d_in, r, w_bits, group, ab_bits, fa, fe, ws, stream);
}

int eora_linear_q_multi(const void* x, const void* qweight, const void* scales, const void* qzeros,
                        const void* A_all, const void* B_all, const void* A_scales, const void* B_scales,
                        const void* adapter_of_row, void* y, int M, int d_in, int d_out, int r, int n_adapters,
                        int w_bits, int group, int ab_bits, void* workspace, size_t workspace_bytes, void* stream)
{
    if (n_adapters < 1 || r < 1 || r % 32 || (ab_bits != 16 && r % 128)) return EORA_ERR_SHAPE;
    if ((long long)n_adapters * r > MAX_RANK) return EORA_ERR_SHAPE;
    if (!adapter_of_row) return EORA_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(adapter_of_row) & 3u) return EORA_ERR_ALIGN;
    const int R = n_adapters * r;
    const eora_q_member e{qweight, scales, qzeros, A_all, B_all, A_scales, B_scales, y, d_out};
    int fa, fe;
    const int rc = validate_linear_q(x, e, M, d_in, R, w_bits, group, ab_bits, workspace, workspace_bytes, &fa, &fe);
    if (rc != EORA_OK) return rc;
    if (M == 0) return EORA_OK;
    // many tokens: the GEMM path, with t masked per row between its two launches
    if (prefill_fits(M, R, ab_bits))
        return launch_prefill_group(x, &e, 1, M, d_in, R, w_bits, group, fa, fe, (const int*)adapter_of_row, r, workspace, (hipStream_t)stream);
    // one to four tokens: the decode kernel, with t masked where it is gathered
    int nw = 0, nq = 0;
    if (small_kernel_fits(M, d_in, group, &nw, &nq))
        return launch_group(x, &e, 1, M, d_in, R, w_bits, group, fa, fe, nw, nq, workspace, (hipStream_t)stream, (const int*)adapter_of_row, r);
    // 5 .. 16 tokens and enough rows: the kernel with x resident in LDS, with t masked where it goes to LDS
    if (stream_fits(M, d_in, group, R, backbone_format(w_bits), fa, &d_out, 1))
        return launch_stream_group(x, &e, 1, M, d_in, R, w_bits, fa, fe, workspace, (hipStream_t)stream, (const int*)adapter_of_row, r);
    const int kcn = pick_kcn(M, d_in);
    for (int m0 = 0; m0 < M; m0 += CHUNK_TOKENS) {
        FusedArgs a{};
        a.x = (const _Float16*)x + (size_t)m0 * d_in;
        a.w = qweight;
        a.w_scales = (const _Float16*)scales;
        a.w_zeros = (const uint32_t*)qzeros;
        a.A = A_all;
        a.A_scales = (const _Float16*)A_scales;
        a.B = B_all;
        a.B_scales = (const _Float16*)B_scales;
        a.y = (_Float16*)y + (size_t)m0 * d_out;
        a.hdr = (uint32_t*)workspace;
        a.tpart = (float*)((char*)workspace + WS_PARTS);
        a.tpair = (unsigned long long*)((char*)workspace + WS_PAIRS);
        a.M = M - m0 < CHUNK_TOKENS ? M - m0 : CHUNK_TOKENS;
        a.d_in = d_in;
        a.d_out = d_out;
        a.r = R;
        a.group = group;
        a.kcn = kcn;
        a.spin_limit = g_spin_limit;
        a.adapter = (const int*)adapter_of_row + m0;
        a.r_per = r;
        const int fm = backbone_format(w_bits);
        const hipError_t err = wide_q_fits(a.M, d_in, d_out, R) ? launch_wide_q(a, fm, fa, fe, (hipStream_t)stream)
                                                                 : launch_fused(a, fm, fa, fe, (hipStream_t)stream);
        if (failed(err, "linear_q_multi")) return EORA_ERR_LAUNCH;
    }
    return EORA_OK;
}

int eora_linear_q_group(const void* x, const eora_q_member* members, int n_members,
                        int M, int d_in, int r, int w_bits, int group, int ab_bits,
                        void* workspace, size_t workspace_bytes, void* stream)
{
    if (!x || !members) return EORA_ERR_NULL;
    if (n_members < 1 || n_members > MAX_GROUP) return EORA_ERR_SHAPE;
    int fa = S_NONE, fe = S_NONE;
    for (int m = 0; m < n_members; ++m) {               // every member is validated before anything is enqueued
        const int rc = validate_linear_q(x, members[m], M, d_in, r, w_bits, group, ab_bits, workspace, workspace_bytes, &fa, &fe);
        if (rc != EORA_OK) return rc;
    }
    int nw = 0, nq = 0;
    if (small_kernel_fits(M, d_in, group, &nw, &nq) &&
        (r == 0 || (r / 16) * pick_kcn(M, d_in) * n_members <= HDR_FLAGS_PER_BLOCK))
        return launch_group(x, members, n_members, M, d_in, r, w_bits, group, fa, fe, nw, nq, workspace, (hipStream_t)stream);
    if (prefill_fits(M, r, ab_bits) && workspace_bytes >= eora_workspace_bytes_group(M, d_in, r, n_members))
        return launch_prefill_group(x, members, n_members, M, d_in, r, w_bits, group, fa, fe, nullptr, 0, workspace, (hipStream_t)stream);
    if (n_members >= 1) {
        int rows[MAX_GROUP] = {0, 0, 0, 0};
        for (int m = 0; m < n_members; ++m) rows[m] = members[m].d_out;
        if (stream_fits(M, d_in, group, r, backbone_format(w_bits), fa, rows, n_members))
            return launch_stream_group(x, members, n_members, M, d_in, r, w_bits, fa, fe, workspace, (hipStream_t)stream);
    }
    if (n_members > 1 && M > 4 && M < PREFILL_MIN_TOKENS) {
        // 5 .. 127 tokens: the members' workgroups in one launch of the kernel that shares x through LDS, if together
        // they have the rows it wants.  k-ranges: the members' partials and flags share the regions of one call.
        int d_outs[MAX_GROUP];
        for (int m = 0; m < n_members; ++m) d_outs[m] = members[m].d_out;
        const int yblocks = (M + 15) / 16;
        int kcn = 1;
        for (int c = 2; c <= 4; ++c)
            if ((d_in / 128) % c == 0 && n_members * yblocks * c <= 32) kcn = c;
        const bool regions_ok = n_members * yblocks * kcn <= 32 && (r / 16) * kcn * n_members <= HDR_FLAGS_PER_BLOCK;
        if (regions_ok && wide_q_group_fits(M, d_in, d_outs, n_members, r)) {
            FusedArgs as[MAX_GROUP];
            for (int m = 0; m < n_members; ++m) {
                const eora_q_member& e = members[m];
                FusedArgs a{};
                a.x = (const _Float16*)x;
                a.w = e.qweight;
                a.w_scales = (const _Float16*)e.scales;
                a.w_zeros = (const uint32_t*)e.qzeros;
                a.A = e.A;
                a.A_scales = (const _Float16*)e.A_scales;
                a.B = e.B;
                a.B_scales = (const _Float16*)e.B_scales;
                a.y = (_Float16*)e.y;
                a.hdr = (uint32_t*)workspace;
                a.tpart = (float*)((char*)workspace + WS_PARTS);
                a.tpair = (unsigned long long*)((char*)workspace + WS_PAIRS) + (size_t)m * yblocks * kcn * 16 * r;
                a.M = M;
                a.d_in = d_in;
                a.d_out = e.d_out;
                a.r = r;
                a.group = group;
                a.kcn = kcn;
                a.spin_limit = g_spin_limit;
                as[m] = a;
            }
            if (failed(launch_wide_q_group(as, n_members, backbone_format(w_bits), fa, fe, (hipStream_t)stream), "linear_q_group"))
                return EORA_ERR_LAUNCH;
            return EORA_OK;
        }
    }
    for (int m = 0; m < n_members; ++m) {               // other shapes (or a workspace sized for one member): one after the other
        const int rc = run_linear_q(x, members[m], M, d_in, r, w_bits, group, ab_bits, fa, fe, workspace, stream);
        if (rc != EORA_OK) return rc;
    }
    return EORA_OK;
}

namespace {
// both 2:4 entry points: exactly one of values / qvalues is given
int run_linear_sparse(const void* x, const void* values, const void* indices, const void* qtiles, const void* qmeta,
                      const void* A, const void* B, void* y,
                      int M, int d_in, int d_out, int r, void* workspace, size_t workspace_bytes, void* stream)
{
    int rc = check_backbone_shape(M, d_in, d_out, r);
    if (rc != EORA_OK) return rc;
    if (r > 0) {
        if (!A || !B) return EORA_ERR_NULL;
        if (r % 32) return EORA_ERR_SHAPE;
        if (!aligned16(A) || !aligned16(B)) return EORA_ERR_ALIGN;
    }
    if (!aligned16(x) || !aligned16(values) || !aligned16(qtiles) || !aligned16(qmeta) || !aligned16(indices) || !aligned16(y)) return EORA_ERR_ALIGN;
    if (!workspace) return EORA_ERR_WORKSPACE;
    if (!aligned16(workspace)) return EORA_ERR_ALIGN;
    if (workspace_bytes < eora_workspace_bytes(M, d_in, d_out, r)) return EORA_ERR_WORKSPACE;
    if (M == 0) return EORA_OK;
    int kcn = pick_kcn(M, d_in);
    // (the longest contractions at 1..4 tokens: sixteen ranges, so that the producers are done before the first
    // consumers reach their tails; 70B down projection 51.1 -> 50.4 us, with 4-bit kept values 29.5 -> 27.7 us)
    if (M <= 4 && d_in > 16384 && (d_in / 128) % 16 == 0 && (r / 16) * 16 <= HDR_FLAGS_PER_BLOCK) kcn = 16;
    for (int m0 = 0; m0 < M; m0 += CHUNK_TOKENS) {
        SparseArgs a{};
        a.x = (const _Float16*)x + (size_t)m0 * d_in;
        a.values = (const _Float16*)values;
        a.indices = (const uint32_t*)indices;
        a.qtiles = (const uint32_t*)qtiles;
        a.qmeta = (const uint32_t*)qmeta;
        a.A = A;
        a.B = B;
        a.y = (_Float16*)y + (size_t)m0 * d_out;
        a.hdr = (uint32_t*)workspace;
        a.tpart = (float*)((char*)workspace + WS_PARTS);
        a.tpair = (unsigned long long*)((char*)workspace + WS_PAIRS);
        a.M = M - m0 < CHUNK_TOKENS ? M - m0 : CHUNK_TOKENS;
        a.d_in = d_in;
        a.d_out = d_out;
        a.r = r;
        a.kcn = kcn;
        a.spin_limit = g_spin_limit;
        a.ksplit = 1;
        a.ypart = sparse_split_bytes(M, d_in, d_out) ? (float*)((char*)workspace + WS_T) : nullptr;
        if (failed(launch_sparse(a, (hipStream_t)stream), "linear_sp24")) return EORA_ERR_LAUNCH;
    }
    return EORA_OK;
}
}  // namespace

int eora_linear_sp24_group(const void* x, const eora_sp_member* members, int n_members,
                           int M, int d_in, int r, void* workspace, size_t workspace_bytes, void* stream)
{
    if (!x || !members) return EORA_ERR_NULL;
    if (n_members < 1 || n_members > MAX_GROUP) return EORA_ERR_SHAPE;
    const bool vq = members[0].qtiles != nullptr;
    for (int m = 0; m < n_members; ++m) {               // every member is validated before anything is enqueued
        const eora_sp_member& e = members[m];
        if (!e.y) return EORA_ERR_NULL;
        if (vq ? (!e.qtiles || !e.qmeta || e.values || e.indices) : (!e.values || !e.indices || e.qtiles || e.qmeta)) return EORA_ERR_NULL;
        int rc = check_backbone_shape(M, d_in, e.d_out, r);
        if (rc != EORA_OK) return rc;
        if (r > 0) {
            if (!e.A || !e.B) return EORA_ERR_NULL;
            if (r % 32) return EORA_ERR_SHAPE;
            if (!aligned16(e.A) || !aligned16(e.B)) return EORA_ERR_ALIGN;
        }
        if (!aligned16(x) || !aligned16(e.values) || !aligned16(e.qtiles) || !aligned16(e.qmeta) || !aligned16(e.indices) || !aligned16(e.y))
            return EORA_ERR_ALIGN;
        if (!workspace) return EORA_ERR_WORKSPACE;
        if (!aligned16(workspace)) return EORA_ERR_ALIGN;
        if (workspace_bytes < eora_workspace_bytes(M, d_in, e.d_out, r)) return EORA_ERR_WORKSPACE;
    }
    if (M == 0) return EORA_OK;
    // one launch when the members' partials and flags fit the regions of one call; else one after the other
    const int yblocks = (M + 15) / 16;
    int kcn = pick_kcn(M, d_in);
    // (the longest contractions at 1..4 tokens: sixteen ranges, so that the producers are done before the first
    // consumers reach their tails; 70B down projection 51.1 -> 50.4 us, with 4-bit kept values 29.5 -> 27.7 us)
    if (M <= 4 && d_in > 16384 && (d_in / 128) % 16 == 0 && (r / 16) * 16 <= HDR_FLAGS_PER_BLOCK) kcn = 16;
    while (kcn > 1 && (n_members * yblocks * kcn > 32 || (d_in / 128) % kcn)) --kcn;
    const bool one_launch = n_members > 1 && M <= CHUNK_TOKENS && n_members * yblocks * kcn <= 32 &&
                            (r / 16) * kcn * n_members <= HDR_FLAGS_PER_BLOCK;
    if (!one_launch) {
        for (int m = 0; m < n_members; ++m) {
            const eora_sp_member& e = members[m];
            const int rc = run_linear_sparse(x, e.values, e.indices, e.qtiles, e.qmeta, e.A, e.B, e.y, M, d_in, e.d_out, r,
                                             workspace, workspace_bytes, stream);
            if (rc != EORA_OK) return rc;
        }
        return EORA_OK;
    }
    SparseArgs as[MAX_GROUP];
    for (int m = 0; m < n_members; ++m) {
        const eora_sp_member& e = members[m];
        SparseArgs a{};
        a.x = (const _Float16*)x;
        a.values = (const _Float16*)e.values;
        a.indices = (const uint32_t*)e.indices;
        a.qtiles = (const uint32_t*)e.qtiles;
        a.qmeta = (const uint32_t*)e.qmeta;
        a.A = e.A;
        a.B = e.B;
        a.y = (_Float16*)e.y;
        a.hdr = (uint32_t*)workspace;
        const size_t region = (size_t)m * yblocks * kcn * 16 * r;        // this member's partials of t
        a.tpart = (float*)((char*)workspace + WS_PARTS) + region;
        a.tpair = (unsigned long long*)((char*)workspace + WS_PAIRS) + region;
        a.M = M;
        a.d_in = d_in;
        a.d_out = e.d_out;
        a.r = r;
        a.kcn = kcn;
        a.spin_limit = g_spin_limit;
        a.ksplit = 1;                                                    // (grouped launches never split the contraction)
        as[m] = a;
    }
    if (failed(launch_sparse_group(as, n_members, (hipStream_t)stream), "linear_sp24_group")) return EORA_ERR_LAUNCH;
    return EORA_OK;
}

int eora_linear_sp24(const void* x, const void* values, const void* indices,
                     const void* A, const void* B, void* y,
                     int M, int d_in, int d_out, int r,
                     void* workspace, size_t workspace_bytes, void* stream)
{
    if (!x || !values || !indices || !y) return EORA_ERR_NULL;
    return run_linear_sparse(x, values, indices, nullptr, nullptr, A, B, y, M, d_in, d_out, r,
                             workspace, workspace_bytes, stream);
}

int eora_linear_sp24q4(const void* x, const void* qtiles, const void* qmeta,
                       const void* A, const void* B, void* y,
                       int M, int d_in, int d_out, int r,
                       void* workspace, size_t workspace_bytes, void* stream)
{
    if (!x || !qtiles || !qmeta || !y) return EORA_ERR_NULL;
    return run_linear_sparse(x, nullptr, nullptr, qtiles, qmeta, A, B, y, M, d_in, d_out, r,
                             workspace, workspace_bytes, stream);
}

int eora_unpack_q(const void* qweight, const void* qzeros, void* codes_u8, void* zeros_u8,
                  int d_in, int d_out, int w_bits, int group, void* stream)
{
    if (!qweight || !qzeros || !codes_u8 || !zeros_u8) return EORA_ERR_NULL;
    if (w_bits < 2 || w_bits > 4) return EORA_ERR_UNSUPPORTED;
    int rc = check_backbone_shape(1, d_in, d_out, 0);
    if (rc != EORA_OK) return rc;
    rc = check_group(d_in, group);
    if (rc != EORA_OK) return rc;
    if (!aligned16(qweight) || !aligned16(qzeros)) return EORA_ERR_ALIGN;
    if (failed(launch_unpack_q((const uint32_t*)qweight, (const uint32_t*)qzeros, (uint8_t*)codes_u8,
                               (uint8_t*)zeros_u8, d_in, d_out, w_bits, group, (hipStream_t)stream), "unpack_q"))
        return EORA_ERR_LAUNCH;
    return EORA_OK;
}

int eora_dequant_q(const void* qweight, const void* scales, const void* qzeros, void* W_f32,
                   int d_in, int d_out, int w_bits, int group, void* stream)
{
    if (!qweight || !scales || !qzeros || !W_f32) return EORA_ERR_NULL;
    if (w_bits < 2 || w_bits > 4) return EORA_ERR_UNSUPPORTED;
    int rc = check_backbone_shape(1, d_in, d_out, 0);
    if (rc != EORA_OK) return rc;
    rc = check_group(d_in, group);
    if (rc != EORA_OK) return rc;
    if (!aligned16(qweight) || !aligned16(scales) || !aligned16(qzeros) || !aligned16(W_f32)) return EORA_ERR_ALIGN;
    if (failed(launch_dequant_q((const uint32_t*)qweight, (const _Float16*)scales, (const uint32_t*)qzeros,
                                (float*)W_f32, d_in, d_out, w_bits, group, (hipStream_t)stream), "dequant_q"))
        return EORA_ERR_LAUNCH;
    return EORA_OK;
}

int eora_expand_sp24(const void* values, const void* indices, void* W_f16, int d_in, int d_out, void* stream)
{
    if (!values || !indices || !W_f16) return EORA_ERR_NULL;
    int rc = check_backbone_shape(1, d_in, d_out, 0);
    if (rc != EORA_OK) return rc;
    if (!aligned16(values) || !aligned16(indices) || !aligned16(W_f16)) return EORA_ERR_ALIGN;
    if (failed(launch_expand_sp24((const _Float16*)values, (const uint32_t*)indices, (_Float16*)W_f16, d_in, d_out,
                                  (hipStream_t)stream), "expand_sp24"))
        return EORA_ERR_LAUNCH;
    return EORA_OK;
}

int eora_expand_sp24q4(const void* qtiles, const void* qmeta, void* W_f32, int d_in, int d_out, void* stream)
{
    if (!qtiles || !qmeta || !W_f32) return EORA_ERR_NULL;
    int rc = check_backbone_shape(1, d_in, d_out, 0);
    if (rc != EORA_OK) return rc;
    if (!aligned16(qtiles) || !aligned16(qmeta) || !aligned16(W_f32)) return EORA_ERR_ALIGN;
    if (failed(launch_expand_sp24q4((const uint32_t*)qtiles, (const uint32_t*)qmeta, (float*)W_f32, d_in, d_out,
                                    (hipStream_t)stream), "expand_sp24q4"))
        return EORA_ERR_LAUNCH;
    return EORA_OK;
}

}  // extern "C"
