// Algorithm 1 (Sec. 3), steps 1-6, in fp64 on the device: the factors B' (d_out x r) and A (r x d_in) that
// compensate a compressed weight, from the weight, its compressed version and calibration activations.
//
//   1  dW = W - What
//   2  X~ X~^T = Q Lambda Q^T          one-sided Jacobi on the rows of the Gram matrix (rotations accumulated)
//   3  Q' = Q sqrt(Lambda)
//   4  dW' = dW Q'
//   5  rank-r SVD of dW'               one-sided Jacobi on the rows of dW' (or of its transpose, whichever
//                                      has fewer rows), top r rows by norm
//   6  A = A' sqrt(Lambda)^-1 Q^T
//
// One-sided (Hestenes) Jacobi: plane rotations of row pairs until all rows are mutually orthogonal.  For a
// symmetric positive semi-definite G, R G with orthogonal rows means R G^2 R^T is diagonal, so the rows of the
// accumulated rotation R are eigenvectors of G and r_p . (R G)_p its eigenvalues.  For a general matrix T,
// R T with orthogonal rows is Sigma V^T (row norms = singular values, R = U^T).  A round of the round-robin
// schedule rotates m/2 disjoint pairs, one workgroup per pair, rows held in registers; m-1 rounds visit every
// pair once (a sweep); sweeps repeat until one passes without a rotation.
#include "eora.h"

#include <hip/hip_runtime.h>
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>

namespace eora {
namespace {

constexpr int JPT = 8;                 // double2 items per thread and row
constexpr int MAX_DIM = 16384;         // 2 * JPT * 1024
constexpr int MAX_SWEEPS = 60;

__device__ inline double wave_sum(double v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

// One round: workgroup i rotates the row pair (p, q) of the round-robin schedule.  H: m x L row-major;
// V: m x m row-major or nullptr.  rows with squared norm <= abs_floor count as zero.
template <int NT>
__global__ __launch_bounds__(NT) void jacobi_round_kernel(double* __restrict__ H, int L, double* __restrict__ V,
                                                          int m, int round, double tol, double abs_floor,
                                                          unsigned* __restrict__ rotations)
{
    const int i = blockIdx.x, mm = m - 1, tid = threadIdx.x;
    int p, q;
    if (i == 0) {
        p = round;
        q = mm;
    } else {
        p = (round + i) % mm;
        q = (round + mm - i) % mm;
    }
    const int L2 = L >> 1;
    double2* rp = reinterpret_cast<double2*>(H + (size_t)p * L);
    double2* rq = reinterpret_cast<double2*>(H + (size_t)q * L);
    double2 hp[JPT], hq[JPT];
    double app = 0, aqq = 0, apq = 0;
#pragma unroll
    for (int k = 0; k < JPT; ++k) {
        const int idx = tid + k * NT;
        hp[k] = hq[k] = make_double2(0.0, 0.0);
        if (idx < L2) {
            hp[k] = rp[idx];
            hq[k] = rq[idx];
        }
        app += hp[k].x * hp[k].x + hp[k].y * hp[k].y;
        aqq += hq[k].x * hq[k].x + hq[k].y * hq[k].y;
        apq += hp[k].x * hq[k].x + hp[k].y * hq[k].y;
    }
    __shared__ double red[3][16];
    __shared__ double cs[2];
    __shared__ int go;
    app = wave_sum(app);
    aqq = wave_sum(aqq);
    apq = wave_sum(apq);
    constexpr int NWV = NT / 64;
    if ((tid & 63) == 0) {
        red[0][tid >> 6] = app;
        red[1][tid >> 6] = aqq;
        red[2][tid >> 6] = apq;
    }
    __syncthreads();
    if (tid == 0) {
        double a = 0, b = 0, c = 0;
        for (int w = 0; w < NWV; ++w) {
            a += red[0][w];
            b += red[1][w];
            c += red[2][w];
        }
        int rotate = 0;
        if (a > abs_floor && b > abs_floor && fabs(c) > tol * sqrt(a) * sqrt(b)) {
            const double zeta = (b - a) / (2.0 * c);
            const double t = copysign(1.0, zeta) / (fabs(zeta) + sqrt(1.0 + zeta * zeta));
            const double co = 1.0 / sqrt(1.0 + t * t);
            cs[0] = co;
            cs[1] = co * t;
            rotate = 1;
            atomicAdd(rotations, 1u);
        }
        go = rotate;
    }
    __syncthreads();
    if (!go) return;
    const double co = cs[0], si = cs[1];
#pragma unroll
    for (int k = 0; k < JPT; ++k) {
        const int idx = tid + k * NT;
        if (idx < L2) {
            rp[idx] = make_double2(co * hp[k].x - si * hq[k].x, co * hp[k].y - si * hq[k].y);
            rq[idx] = make_double2(si * hp[k].x + co * hq[k].x, si * hp[k].y + co * hq[k].y);
        }
    }
    if (V) {
        double2* vp = reinterpret_cast<double2*>(V + (size_t)p * m);
        double2* vq = reinterpret_cast<double2*>(V + (size_t)q * m);
        for (int idx = tid; idx < (m >> 1); idx += NT) {
            const double2 a = vp[idx], b = vq[idx];
            vp[idx] = make_double2(co * a.x - si * b.x, co * a.y - si * b.y);
            vq[idx] = make_double2(si * a.x + co * b.x, si * a.y + co * b.y);
        }
    }
}

// ------------------------------------------------------------------------------------------------------------
// Block version of a round, for m % 16 == 0 and row lengths that are multiples of 128: a workgroup takes two
// blocks of eight rows (16 x L), forms their 16 x 16 Gram matrix S with fp64 MFMAs, diagonalises S in LDS with a
// small two-sided Jacobi iteration (S = J D J^T, J orthogonal), and replaces the rows by J^T times the rows
// (MFMAs again), which makes all 16 mutually orthogonal at once: 120 row pairs for three passes over the rows
// instead of one pair for two.  The eigenvector rows get the same J^T.
//
// v_mfma_f64_16x16x4_f64 operand layout (lane l, n = l % 16, g = l / 16): A[i = n][k = g], B[k = g][j = n],
// result register v holds D[i = 4 v + g][j = n].
typedef double d4 __attribute__((ext_vector_type(4)));
constexpr int BJ_NT = 512, BJ_NW = BJ_NT / 64;
constexpr int BJ_INNER_SWEEPS = 30;

__device__ __forceinline__ d4 mfma64(double a, double b, d4 c) { return __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, c, 0, 0, 0); }

// rows <- J^T rows for the 16 rows (block P, block Q) of X (row length len, a multiple of 128)
__device__ __forceinline__ void apply_rotation(double* __restrict__ X, int len, int P, int Q, const double (*J)[17], int wave,
                                               int lane)
{
    const int n = lane & 15, g = lane >> 4;
    double aJ[4];                       // A operand of step kk: (J^T)[i = n][k = 4 kk + g] = J[4 kk + g][n]
    size_t rowoff[4];                   // rows 4 kk + g (loads) = rows 4 v + g (stores)
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
        const int j = 4 * kk + g;
        aJ[kk] = J[j][n];
        rowoff[kk] = (size_t)(j < 8 ? 8 * P + j : 8 * Q + j - 8) * len;
    }
    const int ngroups = len / 128;      // a group: 128 columns = four chunks of 32 (two columns per lane)
    for (int gi = wave; gi < ngroups; gi += BJ_NW) {
        double2 ld[4][4];
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int kk = 0; kk < 4; ++kk)
                ld[u][kk] = *reinterpret_cast<const double2*>(X + rowoff[kk] + 128 * gi + 32 * u + 2 * n);
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            d4 d0 = {0, 0, 0, 0}, d1 = {0, 0, 0, 0};
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) {
                d0 = mfma64(aJ[kk], ld[u][kk].x, d0);
                d1 = mfma64(aJ[kk], ld[u][kk].y, d1);
            }
#pragma unroll
            for (int v = 0; v < 4; ++v)
                *reinterpret_cast<double2*>(X + rowoff[v] + 128 * gi + 32 * u + 2 * n) = make_double2(d0[v], d1[v]);
        }
    }
}

__global__ __launch_bounds__(BJ_NT) void jacobi_block_round_kernel(double* __restrict__ H, int L, double* __restrict__ V, int m,
                                                                    int round, double tol, double abs_floor,
                                                                    unsigned* __restrict__ rotations)
{
    __shared__ double Sw[BJ_NW][16][17];
    __shared__ double S[16][17], J[16][17];
    __shared__ double rco[8], rsi[8];
    __shared__ int rp[8], rq[8];
    __shared__ int s_any[BJ_INNER_SWEEPS];      // one flag per sweep, so that none is ever cleared while in use
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int n = lane & 15, g = lane >> 4;
    const int nb = m / 8, mm = nb - 1, i = blockIdx.x;
    int P, Q;
    if (i == 0) {
        P = round;
        Q = mm;
    } else {
        P = (round + i) % mm;
        Q = (round + mm - i) % mm;
    }
    // ---- Gram matrix of the 16 rows: lane (n, g) feeds row n, both operands of the MFMA are the same register
    {
        const double* row = H + (size_t)(n < 8 ? 8 * P + n : 8 * Q + n - 8) * L;
        d4 acc = {0, 0, 0, 0};
        const int ngroups = L / 128;
        for (int gi = wave; gi < ngroups; gi += BJ_NW) {
            double2 ld[16];             // columns 128 gi + 8 e + 2 g + {0, 1}, e = 0 .. 15
#pragma unroll
            for (int e = 0; e < 16; ++e) ld[e] = *reinterpret_cast<const double2*>(row + 128 * gi + 8 * e + 2 * g);
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                acc = mfma64(ld[e].x, ld[e].x, acc);
                acc = mfma64(ld[e].y, ld[e].y, acc);
            }
        }
#pragma unroll
        for (int v = 0; v < 4; ++v) Sw[wave][4 * v + g][n] = acc[v];
    }
    __syncthreads();
    if (tid < 256) {
        const int r = tid >> 4, c = tid & 15;
        double t = 0;
#pragma unroll
        for (int w = 0; w < BJ_NW; ++w) t += Sw[w][r][c];
        S[r][c] = t;
        J[r][c] = r == c ? 1.0 : 0.0;
    }
    if (tid < BJ_INNER_SWEEPS) s_any[tid] = 0;
    __syncthreads();
    // ---- S = J D J^T by two-sided Jacobi: eight disjoint pairs per step, fifteen steps per sweep
    bool rotated = false;
    for (int sweep = 0; sweep < BJ_INNER_SWEEPS; ++sweep) {
        for (int step = 0; step < 15; ++step) {
            if (tid < 8) {
                int p, q;
                if (tid == 0) {
                    p = step;
                    q = 15;
                } else {
                    p = (step + tid) % 15;
                    q = (step + 15 - tid) % 15;
                }
                const double a = S[p][p], b = S[q][q], c = S[p][q];
                double co = 1.0, si = 0.0;
                if (a > abs_floor && b > abs_floor && fabs(c) > tol * sqrt(a) * sqrt(b)) {
                    const double zeta = (b - a) / (2.0 * c);
                    const double t = copysign(1.0, zeta) / (fabs(zeta) + sqrt(1.0 + zeta * zeta));
                    co = 1.0 / sqrt(1.0 + t * t);
                    si = co * t;
                    s_any[sweep] = 1;
                }
                rp[tid] = p;
                rq[tid] = q;
                rco[tid] = co;
                rsi[tid] = si;
            }
            __syncthreads();
            if (tid < 256) {            // rows of S (threads 0 .. 127), columns of J (128 .. 255)
                const int k = (tid & 127) >> 4, c = tid & 15;
                const int p = rp[k], q = rq[k];
                const double co = rco[k], si = rsi[k];
                if (tid < 128) {
                    const double a = S[p][c], b = S[q][c];
                    S[p][c] = co * a - si * b;
                    S[q][c] = si * a + co * b;
                } else {
                    const double a = J[c][p], b = J[c][q];
                    J[c][p] = co * a - si * b;
                    J[c][q] = si * a + co * b;
                }
            }
            __syncthreads();
            if (tid < 128) {            // columns of S
                const int k = tid >> 4, r = tid & 15;
                const int p = rp[k], q = rq[k];
                const double co = rco[k], si = rsi[k];
                const double a = S[r][p], b = S[r][q];
                S[r][p] = co * a - si * b;
                S[r][q] = si * a + co * b;
            }
            __syncthreads();
        }
        if (s_any[sweep] == 0) break;       // written before the last barrier of the sweep: uniform
        rotated = true;
    }
    if (!rotated) return;               // the 16 rows were orthogonal already (uniform over the workgroup)
    if (tid == 0) atomicAdd(rotations, 1u);
    apply_rotation(H, L, P, Q, J, wave, lane);
    if (V) apply_rotation(V, m, P, Q, J, wave, lane);
}

// C[i][j] = beta * C[i][j] + alpha * sum_k A[i*ai + k*ak] * B[j*bj + k*bk], i < M, j < N, k < K (beta == 0: C is
// not read).  64 x 64 outputs per workgroup of 256 threads, 4 x 4 per thread, operands staged through LDS sixteen k
// at a time.  lower != 0: only the tiles that touch the lower triangle (j0 <= i0) are computed (symmetric updates).
template <typename TA, typename TB>
__global__ __launch_bounds__(256) void gemm_kernel(const TA* __restrict__ A, long ai, long ak, const TB* __restrict__ B,
                                                   long bj, long bk, double* C, long ldc, int M, int N, int K,
                                                   double alpha, double beta, int lower)
{
    __shared__ double As[16][65], Bs[16][65];
    const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
    const int i0 = blockIdx.y * 64, j0 = blockIdx.x * 64;
    if (lower && j0 > i0) return;
    double acc[4][4] = {};
    for (int k0 = 0; k0 < K; k0 += 16) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            int ii, kk;
            if (ak == 1) {
                kk = tid & 15;
                ii = (tid >> 4) + 16 * e;
            } else {
                ii = tid & 63;
                kk = (tid >> 6) + 4 * e;
            }
            const int gi = i0 + ii, gk = k0 + kk;
            As[kk][ii] = (gi < M && gk < K) ? (double)A[(size_t)gi * ai + (size_t)gk * ak] : 0.0;
            int jj, kb;
            if (bk == 1) {
                kb = tid & 15;
                jj = (tid >> 4) + 16 * e;
            } else {
                jj = tid & 63;
                kb = (tid >> 6) + 4 * e;
            }
            const int gj = j0 + jj, gkb = k0 + kb;
            Bs[kb][jj] = (gj < N && gkb < K) ? (double)B[(size_t)gj * bj + (size_t)gkb * bk] : 0.0;
        }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < 16; ++k) {
            double a[4], b[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                a[e] = As[k][ty + 16 * e];
                b[e] = Bs[k][tx + 16 * e];
            }
#pragma unroll
            for (int e = 0; e < 4; ++e)
#pragma unroll
                for (int f = 0; f < 4; ++f) acc[e][f] += a[e] * b[f];
        }
        __syncthreads();
    }
#pragma unroll
    for (int e = 0; e < 4; ++e)
#pragma unroll
        for (int f = 0; f < 4; ++f) {
            const int gi = i0 + ty + 16 * e, gj = j0 + tx + 16 * f;
            if (gi < M && gj < N) {
                double v = alpha * acc[e][f];
                if (beta != 0.0) v += beta * C[(size_t)gi * ldc + gj];
                C[(size_t)gi * ldc + gj] = v;
            }
        }
}

// ------------------------------------------------------------------------------------------------------------
// Cholesky factor of the Gram matrix, G = L L^T, in place in the lower triangle (right-looking, blocks of 64):
// any S with S S^T = X~ X~^T serves Algorithm 1 as the eigenvectors times the roots of the eigenvalues do (the
// two differ by an orthogonal factor on the right, which the SVD of step 5 absorbs), and L costs n^3 / 3 flops.
constexpr int CH_NB = 64;

// thr[0] = rel * max_i G[i][i]: pivots at or below it make the factorisation give up (flag)
__global__ __launch_bounds__(1024) void pivot_floor_kernel(const double* __restrict__ G, int n, double rel, double* __restrict__ thr)
{
    __shared__ double red[1024];
    double m = 0.0;
    for (int i = threadIdx.x; i < n; i += 1024) m = fmax(m, G[(size_t)i * n + i]);
    red[threadIdx.x] = m;
    __syncthreads();
    for (int s2 = 512; s2 > 0; s2 >>= 1) {
        if ((int)threadIdx.x < s2) red[threadIdx.x] = fmax(red[threadIdx.x], red[threadIdx.x + s2]);
        __syncthreads();
    }
    if (threadIdx.x == 0) thr[0] = rel * red[0];
}

// the nb x nb diagonal block at (j0, j0): unblocked factorisation in LDS; the block's strict upper part is zeroed
__global__ __launch_bounds__(256) void potrf_block_kernel(double* __restrict__ A, long lda, int j0, int nb,
                                                          const double* __restrict__ thr, unsigned* __restrict__ flag)
{
    __shared__ double S[CH_NB][CH_NB + 1];
    const int tid = threadIdx.x;
    double* const blk = A + (size_t)j0 * lda + j0;
    for (int e = tid; e < CH_NB * CH_NB; e += 256) {
        const int i = e >> 6, c = e & 63;
        S[i][c] = (i < nb && c <= i) ? blk[(size_t)i * lda + c] : 0.0;
    }
    __syncthreads();
    const double floor_abs = thr[0];
    for (int j = 0; j < nb; ++j) {
        if (tid == 0) {
            double d = S[j][j];
            if (!(d > floor_abs)) {                       // not (numerically) positive definite: give up, stay finite
                atomicOr(flag, 1u);
                d = floor_abs > 0.0 ? floor_abs : 1.0;
            }
            S[j][j] = sqrt(d);
        }
        __syncthreads();
        if (tid > j && tid < nb) S[tid][j] /= S[j][j];
        __syncthreads();
        for (int e = tid; e < CH_NB * CH_NB; e += 256) {
            const int i = e >> 6, c = e & 63;
            if (c > j && i >= c && i < nb) S[i][c] -= S[i][j] * S[c][j];
        }
        __syncthreads();
    }
    for (int e = tid; e < CH_NB * CH_NB; e += 256) {
        const int i = e >> 6, c = e & 63;
        if (i < nb && c < nb) blk[(size_t)i * lda + c] = c <= i ? S[i][c] : 0.0;
    }
}

// rows j0 + nb .. n - 1 of the block column at j0: x L11^T = a, one thread per row, L11 (the factored diagonal
// block) in LDS, every thread reading the same entry at the same time
__global__ __launch_bounds__(256) void panel_solve_kernel(double* __restrict__ A, long lda, int j0, int nb, int n)
{
    __shared__ double L[CH_NB][CH_NB + 1];
    const int tid = threadIdx.x;
    for (int e = tid; e < CH_NB * CH_NB; e += 256) {
        const int i = e >> 6, c = e & 63;
        L[i][c] = (i < nb && c <= i) ? A[(size_t)(j0 + i) * lda + j0 + c] : (i == c ? 1.0 : 0.0);
    }
    __syncthreads();
    const int row = j0 + nb + blockIdx.x * 256 + tid;
    if (row >= n) return;
    double* const a = A + (size_t)row * lda + j0;
    double x[CH_NB];
#pragma unroll
    for (int c = 0; c < CH_NB; ++c) x[c] = c < nb ? a[c] : 0.0;
#pragma unroll
    for (int c = 0; c < CH_NB; ++c) {
        double v = x[c];
#pragma unroll
        for (int e = 0; e < c; ++e) v -= x[e] * L[c][e];
        x[c] = v / L[c][c];
    }
#pragma unroll
    for (int c = 0; c < CH_NB; ++c)
        if (c < nb) a[c] = x[c];
}

__global__ void zero_upper_kernel(double* __restrict__ A, int n)
{
    const size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= (size_t)n * n) return;
    const int i = (int)(e / n), c = (int)(e - (size_t)i * n);
    if (c > i) A[e] = 0.0;
}

// dst[c][i] = src[i][c] for an n x n matrix
__global__ void transpose_kernel(const double* __restrict__ src, double* __restrict__ dst, int n)
{
    __shared__ double tile[32][33];
    const int bx = blockIdx.x * 32, by = blockIdx.y * 32, tx = threadIdx.x & 31, ty = threadIdx.x >> 5;      // 256 threads: 32 x 8
    for (int e = ty; e < 32; e += 8)
        tile[e][tx] = (by + e < n && bx + tx < n) ? src[(size_t)(by + e) * n + bx + tx] : 0.0;
    __syncthreads();
    for (int e = ty; e < 32; e += 8)
        if (bx + e < n && by + tx < n) dst[(size_t)(bx + e) * n + by + tx] = tile[tx][e];
}

__global__ void iota_kernel(int* __restrict__ idx, int r)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < r) idx[i] = i;
}

// Bn[i][o] = B[o][i] / sigma[i]^2 (B: d_out x r)
__global__ void scaled_transpose_kernel(const double* __restrict__ B, const double* __restrict__ sigma, int d_out, int r,
                                        double* __restrict__ Bn)
{
    const size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= (size_t)d_out * r) return;
    const int i = (int)(e / d_out), o = (int)(e - (size_t)i * d_out);
    const double sg = sigma[i];
    Bn[e] = sg > 0.0 ? B[(size_t)o * r + i] / (sg * sg) : 0.0;
}

__global__ void sub_kernel(const float* __restrict__ W, const float* __restrict__ What, double* __restrict__ dW, size_t n)
{
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dW[i] = (double)W[i] - (double)What[i];
}

__global__ void identity_kernel(double* __restrict__ V, int m)
{
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < (size_t)m * m) V[i] = (i / m == i % m) ? 1.0 : 0.0;
}

__global__ void copy_kernel(const double* __restrict__ src, double* __restrict__ dst, size_t n)
{
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] = src[i];
}

__global__ void clear_counter_kernel(unsigned* c) { *c = 0; }

// out[p] = sum_k X[p][k] * Y[p][k]; one workgroup of 256 per row
__global__ __launch_bounds__(256) void row_dot_kernel(const double* __restrict__ X, const double* __restrict__ Y, int L,
                                                      double* __restrict__ out)
{
    const int p = blockIdx.x;
    double s = 0;
    for (int k = threadIdx.x; k < L; k += 256) s += X[(size_t)p * L + k] * Y[(size_t)p * L + k];
    __shared__ double red[4];
    s = wave_sum(s);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = s;
    __syncthreads();
    if (threadIdx.x == 0) out[p] = red[0] + red[1] + red[2] + red[3];
}

// root[p] = sqrt(max(lam[p], floor * max lam)), inv[p] = 1 / root[p]; one workgroup
__global__ __launch_bounds__(1024) void eig_roots_kernel(const double* __restrict__ lam, int m, double floor_rel,
                                                         double* __restrict__ root, double* __restrict__ inv)
{
    __shared__ double red[16];
    __shared__ double top;
    double mx = -INFINITY;
    for (int k = threadIdx.x; k < m; k += 1024) mx = fmax(mx, lam[k]);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) mx = fmax(mx, __shfl_xor(mx, o, 64));
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = mx;
    __syncthreads();
    if (threadIdx.x == 0) {
        double t = red[0];
        for (int w = 1; w < 16; ++w) t = fmax(t, red[w]);
        top = t;
    }
    __syncthreads();
    for (int k = threadIdx.x; k < m; k += 1024) {
        const double r = sqrt(fmax(lam[k], floor_rel * top));
        root[k] = r;
        inv[k] = 1.0 / r;
    }
}

// X[p][k] *= (by_row ? s[p] : s[k])
__global__ void scale_kernel(double* __restrict__ X, int rows, int L, const double* __restrict__ s, int by_row)
{
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < (size_t)rows * L) X[i] *= by_row ? s[i / L] : s[i % L];
}

// idx[rank] = p for the r rows of largest sq (ties: lower row first); sigma[rank] = sqrt(sq[p])
__global__ void top_rows_kernel(const double* __restrict__ sq, int m, int r, int* __restrict__ idx, double* __restrict__ sigma)
{
    const int p = blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= m) return;
    const double v = sq[p];
    int rank = 0;
    for (int q = 0; q < m; ++q) {
        const double u = sq[q];
        rank += (u > v) || (u == v && q < p);
    }
    if (rank < r) {
        idx[rank] = p;
        sigma[rank] = sqrt(v);
    }
}

// dst[i][k] = src[idx[i]][k] * sigma[i]^power   (power = -1: unit rows; 0: copy; -2: divided by the square)
__global__ void gather_rows_kernel(const double* __restrict__ src, int L, const int* __restrict__ idx,
                                   const double* __restrict__ sigma, int power, double* __restrict__ dst, int r)
{
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (size_t)r * L) return;
    const int row = (int)(i / L), k = (int)(i % L);
    const double s = sigma[row];
    // a vanishing singular value (error of rank below r, or no error at all) gives a zero component, not 0/0
    const double f = power == 0 ? 1.0 : (s > 0.0 ? (power == -1 ? 1.0 / s : 1.0 / (s * s)) : 0.0);
    dst[i] = src[(size_t)idx[row] * L + k] * f;
}

// dst[o][i] = src[idx[i]][o]   (dst: L x r)
__global__ void gather_rows_transposed_kernel(const double* __restrict__ src, int L, const int* __restrict__ idx,
                                              double* __restrict__ dst, int r)
{
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (size_t)r * L) return;
    const int o = (int)(i / r), c = (int)(i % r);
    dst[i] = src[(size_t)idx[c] * L + o];
}

// s[i] = sqrt(|B'_i| / |A_i|) for component i (column i of B: d_out x r, row i of A: r x d_in), 1 if either
// vanishes; one workgroup of 256 per component
__global__ __launch_bounds__(256) void balance_kernel(const double* __restrict__ B, const double* __restrict__ A, int d_in,
                                                      int d_out, int r, double* __restrict__ s)
{
    const int i = blockIdx.x;
    double nb = 0, na = 0;
    for (int o = threadIdx.x; o < d_out; o += 256) nb += B[(size_t)o * r + i] * B[(size_t)o * r + i];
    for (int k = threadIdx.x; k < d_in; k += 256) na += A[(size_t)i * d_in + k] * A[(size_t)i * d_in + k];
    __shared__ double red[2][4];
    nb = wave_sum(nb);
    na = wave_sum(na);
    if ((threadIdx.x & 63) == 0) {
        red[0][threadIdx.x >> 6] = nb;
        red[1][threadIdx.x >> 6] = na;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        nb = sqrt(red[0][0] + red[0][1] + red[0][2] + red[0][3]);
        na = sqrt(red[1][0] + red[1][1] + red[1][2] + red[1][3]);
        s[i] = (nb > 0.0 && na > 0.0) ? sqrt(nb / na) : 1.0;
    }
}

// One thread per (tile, lane) of the F16 tile layout (tile = 16 rows x 32 columns, lane l = 16 j + n owns row n,
// columns 8 j .. 8 j + 7): eight values of X (rows x K fp64 row-major), scaled, rounded once to fp16.
// by_row: the scale of a value is s[row] (A: times s) or 1 / s[column] (B: divided by s); s == nullptr: 1.
__global__ void store_f16_tiles_kernel(const double* __restrict__ X, int rows, int K, const double* __restrict__ s, int by_row,
                                       _Float16* __restrict__ out)
{
    const size_t L = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (L >= (size_t)rows * K / 8) return;
    const int ntk = K / 32;
    const size_t tile = L / 64;
    const int lane = (int)(L % 64);
    const int R = (int)(tile / ntk), g = (int)(tile % ntk);
    const int j = lane >> 4, n = lane & 15;
    const int row = 16 * R + n, col0 = 32 * g + 8 * j;
    for (int i = 0; i < 8; ++i) {
        double v = X[(size_t)row * K + col0 + i];
        if (s) v = by_row ? v * s[row] : v / s[col0 + i];
        out[L * 8 + i] = (_Float16)v;
    }
}

// Symmetric quantisation of a factor X (rows x K fp64) into the Q4 (BITS = 4, KT = 128 or 64) or Q3 (BITS = 3,
// KT = 128) tile layout with one fp16 scale per row and group of KT columns (Sec. 4.5, App. A.9: quantised
// factors).  One wavefront per tile: lane l = 16 j + n owns row n and columns (KT/4) j .. of the tile; the four
// lanes of a row find the group's largest magnitude with two shuffles.  scale = fp16(max |v| / qpos)
// (1 for an all-zero group), code = clip(rint(v / scale) + zp, 1, 2 zp - 1), zp = 2^(BITS-1), qpos = zp - 1.
// s / by_row: the balancing scale of store_f16_tiles_kernel.
template <int BITS, int KT>
__global__ __launch_bounds__(64) void store_q_tiles_kernel(const double* __restrict__ X, int rows, int K, const double* __restrict__ s,
                                                           int by_row, uint32_t* __restrict__ out, _Float16* __restrict__ scales)
{
    constexpr int CPL = KT / 4, ZP = 1 << (BITS - 1), QPOS = ZP - 1;
    const int tile = blockIdx.x, lane = threadIdx.x;
    const int ntk = K / KT;
    const int R = tile / ntk, g = tile % ntk;
    const int j = lane >> 4, n = lane & 15;
    const int row = 16 * R + n, col0 = KT * g + CPL * j;
    double v[CPL];
    double amax = 0.0;
#pragma unroll
    for (int c = 0; c < CPL; ++c) {
        double x = X[(size_t)row * K + col0 + c];
        if (s) x = by_row ? x * s[row] : x / s[col0 + c];
        v[c] = x;
        amax = fmax(amax, fabs(x));
    }
    amax = fmax(amax, __shfl_xor(amax, 16, 64));
    amax = fmax(amax, __shfl_xor(amax, 32, 64));
    _Float16 sc = (_Float16)(amax / (double)QPOS);
    if (sc == (_Float16)0.0f) sc = (_Float16)1.0f;
    const double scd = (double)sc;
    uint32_t code[CPL];
#pragma unroll
    for (int c = 0; c < CPL; ++c) {
        double q = rint(v[c] / scd) + (double)ZP;
        q = fmin(fmax(q, 1.0), (double)(2 * ZP - 1));
        code[c] = (uint32_t)q;
    }
    if (j == 0) scales[(size_t)row * ntk + g] = sc;
    if constexpr (BITS == 4) {
        constexpr int WPL = KT / 32;
#pragma unroll
        for (int t = 0; t < WPL; ++t) {
            uint32_t w = 0;
#pragma unroll
            for (int kk = 0; kk < 8; ++kk) w |= code[8 * t + kk] << (4 * (4 * (kk % 2) + kk / 2));
            out[((size_t)tile * 64 + lane) * WPL + t] = w;
        }
    } else {
        uint32_t d[3] = {0u, 0u, 0u};
#pragma unroll
        for (int cc = 0; cc < 30; ++cc) d[(cc / 2) / 5] |= code[cc] << (16 * (cc % 2) + 3 * ((cc / 2) % 5));
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int b = 0; b < 3; ++b) d[b] |= ((code[30 + h] >> b) & 1u) << (16 * h + 15);
#pragma unroll
        for (int b = 0; b < 3; ++b) out[((size_t)tile * 64 + lane) * 3 + b] = d[b];
    }
}

inline unsigned blocks(size_t n, int per = 256) { return (unsigned)((n + per - 1) / per); }

template <typename TA, typename TB>
void gemm(const TA* A, long ai, long ak, const TB* B, long bj, long bk, double* C, long ldc, int M, int N, int K,
          hipStream_t st, double alpha = 1.0, double beta = 0.0, int lower = 0)
{
    hipLaunchKernelGGL((gemm_kernel<TA, TB>), dim3((N + 63) / 64, (M + 63) / 64), dim3(256), 0, st, A, ai, ak, B, bj, bk, C,
                       ldc, M, N, K, alpha, beta, lower);
}

// G (n x n, row-major, symmetric) -> L in its lower triangle, zeros above.  Enqueues only; *flag (device, cleared
// here) is raised if a pivot is not above rel * max diag(G): the factor is then unusable.
void cholesky(double* G, int n, double rel, double* thr, unsigned* flag, hipStream_t st)
{
    hipLaunchKernelGGL(clear_counter_kernel, dim3(1), dim3(1), 0, st, flag);
    hipLaunchKernelGGL(pivot_floor_kernel, dim3(1), dim3(1024), 0, st, G, n, rel, thr);
    for (int j0 = 0; j0 < n; j0 += CH_NB) {
        const int nb = n - j0 < CH_NB ? n - j0 : CH_NB, rest = n - j0 - nb;
        hipLaunchKernelGGL(potrf_block_kernel, dim3(1), dim3(256), 0, st, G, (long)n, j0, nb, thr, flag);
        if (rest <= 0) break;
        hipLaunchKernelGGL(panel_solve_kernel, dim3((rest + 255) / 256), dim3(256), 0, st, G, (long)n, j0, nb, n);
        // trailing matrix -= panel . panel^T (the tiles of its lower triangle)
        double* const P = G + (size_t)(j0 + nb) * n + j0;
        gemm(P, (long)n, 1L, P, (long)n, 1L, G + (size_t)(j0 + nb) * n + (j0 + nb), (long)n, rest, rest, nb, st, -1.0, 1.0, 1);
    }
    hipLaunchKernelGGL(zero_upper_kernel, dim3(blocks((size_t)n * n)), dim3(256), 0, st, G, n);
}

bool block_rounds_fit(int L, bool with_v, int m) { return m % 16 == 0 && m >= 32 && L % 128 == 0 && (!with_v || m % 128 == 0); }

void jacobi_round(double* H, int L, double* V, int m, int round, double tol, double abs_floor, unsigned* rot, hipStream_t st)
{
    const dim3 g(m / 2);
    const int need = (L / 2 + JPT - 1) / JPT;          // threads that cover a row
    if (need <= 64)
        hipLaunchKernelGGL(jacobi_round_kernel<64>, g, dim3(64), 0, st, H, L, V, m, round, tol, abs_floor, rot);
    else if (need <= 128)
        hipLaunchKernelGGL(jacobi_round_kernel<128>, g, dim3(128), 0, st, H, L, V, m, round, tol, abs_floor, rot);
    else if (need <= 256)
        hipLaunchKernelGGL(jacobi_round_kernel<256>, g, dim3(256), 0, st, H, L, V, m, round, tol, abs_floor, rot);
    else if (need <= 512)
        hipLaunchKernelGGL(jacobi_round_kernel<512>, g, dim3(512), 0, st, H, L, V, m, round, tol, abs_floor, rot);
    else
        hipLaunchKernelGGL(jacobi_round_kernel<1024>, g, dim3(1024), 0, st, H, L, V, m, round, tol, abs_floor, rot);
}

// Sweeps until one passes without a rotation.  Synchronises the stream once per sweep.  sq: m doubles of
// scratch.  Returns the number of sweeps, or -1 if MAX_SWEEPS did not suffice, or -2 on a runtime error.
// stats (may be null): sweeps, milliseconds between two events around the sweeps, workgroups that rotated
// their rows, rows per workgroup (2: pair rounds, 16: block rounds).
int jacobi_sweeps(double* H, int L, double* V, int m, double* sq, unsigned* rot, hipStream_t st, double* rotations);

int jacobi(double* H, int L, double* V, int m, double* sq, unsigned* rot, hipStream_t st, double* stats)
{
    hipEvent_t e0 = nullptr, e1 = nullptr;
    const bool timed = stats && hipEventCreate(&e0) == hipSuccess && hipEventCreate(&e1) == hipSuccess;
    if (timed) hipEventRecord(e0, st);
    double rotations = 0;
    const int sweeps = jacobi_sweeps(H, L, V, m, sq, rot, st, &rotations);
    if (timed) {
        float ms = 0;
        hipEventRecord(e1, st);
        hipEventSynchronize(e1);
        hipEventElapsedTime(&ms, e0, e1);
        stats[0] = sweeps;
        stats[1] = ms;
        stats[2] = rotations;
        stats[3] = (block_rounds_fit(L, V != nullptr, m)) ? 16 : 2;
    }
    if (e0) hipEventDestroy(e0);
    if (e1) hipEventDestroy(e1);
    return sweeps;
}

int jacobi_sweeps(double* H, int L, double* V, int m, double* sq, unsigned* rot, hipStream_t st, double* rotations)
{
    // rows far below the largest are zero for every purpose here, and rotating them would never settle
    hipLaunchKernelGGL(row_dot_kernel, dim3(m), dim3(256), 0, st, H, H, L, sq);
    double* host = (double*)malloc(sizeof(double) * m);
    if (!host) return -2;
    if (hipMemcpyAsync(host, sq, sizeof(double) * m, hipMemcpyDeviceToHost, st) != hipSuccess ||
        hipStreamSynchronize(st) != hipSuccess) {
        free(host);
        return -2;
    }
    double top = 0;
    for (int p = 0; p < m; ++p) top = host[p] > top ? host[p] : top;
    free(host);
    const double abs_floor = top * 1e-30;
    const double tol = sqrt((double)L) * 1.1102230246251565e-16;
    for (int sweep = 1; sweep <= MAX_SWEEPS; ++sweep) {
        hipLaunchKernelGGL(clear_counter_kernel, dim3(1), dim3(1), 0, st, rot);
        if (block_rounds_fit(L, V != nullptr, m)) {
            for (int round = 0; round < m / 8 - 1; ++round)
                hipLaunchKernelGGL(jacobi_block_round_kernel, dim3(m / 16), dim3(BJ_NT), 0, st, H, L, V, m, round, tol, abs_floor, rot);
        } else {
            for (int round = 0; round < m - 1; ++round) jacobi_round(H, L, V, m, round, tol, abs_floor, rot, st);
        }
        unsigned n = 0;
        if (hipMemcpyAsync(&n, rot, sizeof(n), hipMemcpyDeviceToHost, st) != hipSuccess ||
            hipStreamSynchronize(st) != hipSuccess)
            return -2;
        if (getenv("EORA_VERBOSE")) fprintf(stderr, "eora: jacobi m=%d L=%d sweep %d: %u rotations\n", m, L, sweep, n);
        *rotations += n;
        if (n == 0) return sweep;
    }
    return -1;
}

inline size_t r256(size_t v) { return (v + 255) & ~(size_t)255; }

struct Layout {
    size_t dW, H, V, T, T0, lam, root, inv, sq, sigma, idx, Ap, Bn, rot, total;
};

Layout layout(int d_in, int d_out, int r)
{
    Layout l;
    size_t o = 0;
    auto take = [&](size_t bytes) {
        const size_t at = o;
        o += r256(bytes);
        return at;
    };
    const size_t big = (size_t)(d_in > d_out ? d_in : d_out);
    l.dW = take(8 * (size_t)d_out * d_in);
    l.H = take(8 * (size_t)d_in * d_in);
    l.V = take(8 * (size_t)d_in * d_in);
    l.T = take(8 * (size_t)d_out * d_in);
    l.T0 = take(8 * (size_t)d_out * d_in);
    l.lam = take(8 * (size_t)d_in);
    l.root = take(8 * (size_t)d_in);
    l.inv = take(8 * (size_t)d_in);
    l.sq = take(8 * big);
    l.sigma = take(8 * (size_t)r);
    l.idx = take(4 * (size_t)r);
    l.Ap = take(8 * (size_t)r * d_in);
    l.Bn = take(8 * (size_t)r * d_out);
    l.rot = take(256);
    l.total = o;
    return l;
}

int g_factors_route = 0;                    // test hook: 0 = Cholesky factor when the Gram matrix allows it, 1 = always the eigendecomposition

int check_shape(int n_tokens, int d_in, int d_out, int r)
{
    if (n_tokens < 1 || d_in < 2 || d_out < 2 || r < 1) return EORA_ERR_SHAPE;
    if (d_in % 2 || d_out % 2 || d_in > MAX_DIM || d_out > MAX_DIM) return EORA_ERR_SHAPE;
    if (r > d_in || r > d_out) return EORA_ERR_SHAPE;
    return EORA_OK;
}

}  // namespace
}  // namespace eora

using namespace eora;

extern "C" void eora_debug_set_factors_route(int route) { g_factors_route = route == 1 ? 1 : 0; }

extern "C" size_t eora_factors_workspace_bytes(int d_in, int d_out, int r)
{
    if (check_shape(1, d_in, d_out, r) != EORA_OK) return 0;
    return layout(d_in, d_out, r).total;
}

extern "C" int eora_factors(const void* W_f32, const void* W_hat_f32, const void* Xt_f32, int n_tokens, int d_in, int d_out,
                            int r, double eig_floor, void* B_f64, void* A_f64, void* sigma_f64, void* workspace,
                            size_t workspace_bytes, void* stream, double* stats)
{
    if (!W_f32 || !W_hat_f32 || !Xt_f32 || !B_f64 || !A_f64) return EORA_ERR_NULL;
    const int rc = check_shape(n_tokens, d_in, d_out, r);
    if (rc != EORA_OK) return rc;
    if (!(eig_floor >= 0.0) || eig_floor >= 1.0) return EORA_ERR_VALUE;
    const Layout l = layout(d_in, d_out, r);
    if (!workspace || workspace_bytes < l.total) return EORA_ERR_WORKSPACE;
    if (reinterpret_cast<uintptr_t>(workspace) & 15u) return EORA_ERR_ALIGN;
    hipStream_t st = (hipStream_t)stream;
    char* ws = (char*)workspace;
    double* dW = (double*)(ws + l.dW);
    double* H = (double*)(ws + l.H);
    double* V = (double*)(ws + l.V);
    double* T = (double*)(ws + l.T);
    double* T0 = (double*)(ws + l.T0);
    double* lam = (double*)(ws + l.lam);
    double* root = (double*)(ws + l.root);
    double* inv = (double*)(ws + l.inv);
    double* sq = (double*)(ws + l.sq);
    double* sigma = (double*)(ws + l.sigma);
    int* idx = (int*)(ws + l.idx);
    double* Ap = (double*)(ws + l.Ap);
    double* Bn = (double*)(ws + l.Bn);
    unsigned* rot = (unsigned*)(ws + l.rot);
    const float* W = (const float*)W_f32;
    const float* What = (const float*)W_hat_f32;
    const float* Xt = (const float*)Xt_f32;
    const size_t nw = (size_t)d_out * d_in;
    const int k = d_in;

    // steps 1, 2: error and Gram matrix
    hipLaunchKernelGGL(sub_kernel, dim3(blocks(nw)), dim3(256), 0, st, W, What, dW, nw);
    gemm(Xt, (long)n_tokens, 1L, Xt, (long)n_tokens, 1L, H, (long)k, k, k, n_tokens, st);

    // Steps 2-4 and 6 by a Cholesky factor.  With X~ X~^T = L L^T, dW L equals dW Q sqrt(Lambda) times an orthogonal
    // matrix on the right, so step 5 finds the same U' and Sigma', and step 6's A = Sigma'^-1 U'^T (dW L) L^-1 is
    // Sigma'^-1 U'^T dW: no inverse at all.  Identical B' and A (up to the signs of the components) whenever no
    // eigenvalue is clamped; taken when every pivot stays above 1e4 * eig_floor * max diag (a Gram matrix that
    // close to singular may have clamped eigenvalues: then the eigendecomposition below decides, as it does when
    // the test hook asks for it).
    bool chol = false;
    if (g_factors_route == 0) {
        unsigned* flag = rot + 16;
        double* thr = (double*)(rot + 32);
        hipEvent_t e0 = nullptr, e1 = nullptr;
        const bool timed = stats && hipEventCreate(&e0) == hipSuccess && hipEventCreate(&e1) == hipSuccess;
        if (timed) hipEventRecord(e0, st);
        cholesky(H, k, 1e4 * eig_floor, thr, flag, st);
        if (timed) hipEventRecord(e1, st);
        unsigned bad = 1;
        const bool copied = hipMemcpyAsync(&bad, flag, sizeof(bad), hipMemcpyDeviceToHost, st) == hipSuccess &&
                            hipStreamSynchronize(st) == hipSuccess;
        if (timed) {
            float ms = 0;
            hipEventElapsedTime(&ms, e0, e1);
            stats[0] = 0;                        // no sweeps, no rotations, no rows: the Cholesky route
            stats[1] = ms;
            stats[2] = 0;
            stats[3] = 0;
        }
        if (e0) hipEventDestroy(e0);
        if (e1) hipEventDestroy(e1);
        if (!copied) return EORA_ERR_LAUNCH;
        chol = bad == 0;
        if (!chol) gemm(Xt, (long)n_tokens, 1L, Xt, (long)n_tokens, 1L, H, (long)k, k, k, n_tokens, st);      // the Gram matrix again
    }
    int sweeps = 0;
    if (!chol) {
        // step 2: eigenvectors as the rows of V
        hipLaunchKernelGGL(identity_kernel, dim3(blocks((size_t)k * k)), dim3(256), 0, st, V, k);
        sweeps = jacobi(H, k, V, k, sq, rot, st, stats);
        if (sweeps < 0) return sweeps == -1 ? EORA_ERR_NOT_CONVERGED : EORA_ERR_LAUNCH;
        hipLaunchKernelGGL(row_dot_kernel, dim3(k), dim3(256), 0, st, H, V, k, lam);
        // step 3: sqrt(Lambda), with eigenvalues below eig_floor * max raised to it
        hipLaunchKernelGGL(eig_roots_kernel, dim3(1), dim3(1024), 0, st, lam, k, eig_floor, root, inv);
    }

    const bool by_rows = d_out <= d_in;         // which side of dW' has fewer rows to rotate
    const int m = by_rows ? d_out : k, n = by_rows ? k : d_out;       // T: m rows of length n, m <= n
    // step 4: T = dW' (by_rows) or its transpose
    if (by_rows) {
        if (chol) {
            // T = dW L (d_out x k): T[o][j] = sum_i dW[o][i] L[i][j]
            gemm(dW, (long)k, 1L, H, 1L, (long)k, T, (long)k, d_out, k, k, st);
        } else {
            // T[o][j] = root[j] * sum_i dW[o][i] V[j][i]
            gemm(dW, (long)k, 1L, V, (long)k, 1L, T, (long)k, d_out, k, k, st);
            hipLaunchKernelGGL(scale_kernel, dim3(blocks(nw)), dim3(256), 0, st, T, d_out, k, root, 0);
        }
    } else {
        if (chol) {
            // T = (dW L)^T (k x d_out): T[j][o] = sum_i L[i][j] dW[o][i]
            gemm(H, 1L, (long)k, dW, (long)k, 1L, T, (long)d_out, k, d_out, k, st);
        } else {
            // T[j][o] = root[j] * sum_i V[j][i] dW[o][i]
            gemm(V, (long)k, 1L, dW, (long)k, 1L, T, (long)d_out, k, d_out, k, st);
            hipLaunchKernelGGL(scale_kernel, dim3(blocks(nw)), dim3(256), 0, st, T, k, d_out, root, 1);
        }
    }

    // Step 5 on a square factor when T is at least twice as long as it has rows (Cholesky route only; H and V are
    // free by now): with T T^T = C C^T (Cholesky, C lower), T = C F^T for an F with orthonormal columns, so T and C
    // have the same singular values and left singular vectors w_i; the sweeps rotate the m rows of C^T (length m
    // instead of n) to sigma_i w_i^T, and w_i^T T is the row sigma_i z_i^T the sweeps over T itself would have
    // ended with.  The r largest components are accurate to the rounding of T T^T relative to sigma_1^2; a T of
    // rank below m (an error of low rank) has no such factor: then, as before, the rows of T are rotated.
    bool square = false;
    if (chol && n >= 2 * m) {
        unsigned* flag = rot + 16;
        double* thr = (double*)(rot + 32);
        gemm(T, (long)n, 1L, T, (long)n, 1L, H, (long)m, m, m, n, st);
        cholesky(H, m, 1e-14, thr, flag, st);
        unsigned bad = 1;
        if (hipMemcpyAsync(&bad, flag, sizeof(bad), hipMemcpyDeviceToHost, st) != hipSuccess || hipStreamSynchronize(st) != hipSuccess)
            return EORA_ERR_LAUNCH;
        square = bad == 0;
    }
    const double* Tkeep = T;                    // T as step 4 left it
    if (square) {
        double* Y = V;                          // C^T
        hipLaunchKernelGGL(transpose_kernel, dim3((m + 31) / 32, (m + 31) / 32), dim3(256), 0, st, (const double*)H, Y, m);
        sweeps = jacobi(Y, m, nullptr, m, sq, rot, st, stats ? stats + 4 : nullptr);
        if (sweeps < 0) return sweeps == -1 ? EORA_ERR_NOT_CONVERGED : EORA_ERR_LAUNCH;
        hipLaunchKernelGGL(row_dot_kernel, dim3(m), dim3(256), 0, st, Y, Y, m, sq);
        hipLaunchKernelGGL(top_rows_kernel, dim3(blocks(m)), dim3(256), 0, st, sq, m, r, idx, sigma);
        // the r rows sigma_i z_i^T = w_i^T T, into T0 (r x n)
        double* Wr = by_rows ? Bn : Ap;         // r x m unit rows w_i^T (Bn: r x d_out, Ap: r x k)
        hipLaunchKernelGGL(gather_rows_kernel, dim3(blocks((size_t)r * m)), dim3(256), 0, st, Y, m, idx, sigma, -1, Wr, r);
        gemm(Wr, (long)m, 1L, T, 1L, (long)n, T0, (long)n, r, n, m, st);
        hipLaunchKernelGGL(iota_kernel, dim3(blocks(r)), dim3(256), 0, st, idx, r);
        if (stats) stats[2] = m;                // (Cholesky route: the length of the rows the SVD's sweeps rotated)
    } else {
        hipLaunchKernelGGL(copy_kernel, dim3(blocks(nw)), dim3(256), 0, st, T, T0, nw);
        Tkeep = T0;
        // step 5: rows of T -> sigma_i z_i^T
        sweeps = jacobi(T, n, nullptr, m, sq, rot, st, stats ? stats + 4 : nullptr);
        if (sweeps < 0) return sweeps == -1 ? EORA_ERR_NOT_CONVERGED : EORA_ERR_LAUNCH;
        hipLaunchKernelGGL(row_dot_kernel, dim3(m), dim3(256), 0, st, T, T, n, sq);
        hipLaunchKernelGGL(top_rows_kernel, dim3(blocks(m)), dim3(256), 0, st, sq, m, r, idx, sigma);
        if (stats && chol) stats[2] = n;
    }
    const double* Tc = square ? T0 : T;         // rows idx[i]: sigma_i z_i^T
    if (by_rows) {
        // z_i = v_i: A' = rows of V'^T; B' = U' Sigma' = dW' A'^T
        hipLaunchKernelGGL(gather_rows_kernel, dim3(blocks((size_t)r * k)), dim3(256), 0, st, Tc, k, idx, sigma, -1, Ap, r);
        gemm(Tkeep, (long)k, 1L, Ap, (long)k, 1L, (double*)B_f64, (long)r, d_out, r, k, st);
        // Cholesky route, step 6: A = Sigma'^-2 B'^T dW
        if (chol) hipLaunchKernelGGL(scaled_transpose_kernel, dim3(blocks((size_t)r * d_out)), dim3(256), 0, st, (const double*)B_f64, sigma, d_out, r, Bn);
    } else {
        // z_i = u_i: the columns of B' are sigma_i u_i
        hipLaunchKernelGGL(gather_rows_transposed_kernel, dim3(blocks((size_t)r * d_out)), dim3(256), 0, st, Tc, d_out, idx,
                           (double*)B_f64, r);
        // A' = Sigma'^-1 U'^T dW' : A'[i][j] = sum_o (sigma_i u_i[o] / sigma_i^2) dW'[o][j]
        hipLaunchKernelGGL(gather_rows_kernel, dim3(blocks((size_t)r * d_out)), dim3(256), 0, st, Tc, d_out, idx, sigma, -2, Bn,
                           r);
        if (!chol) gemm(Bn, (long)d_out, 1L, Tkeep, (long)d_out, 1L, Ap, (long)k, r, k, d_out, st);
    }
    if (chol) {
        // step 6 without an inverse: A[i][j] = sum_o (sigma_i u_i[o] / sigma_i^2) dW[o][j]
        gemm(Bn, (long)d_out, 1L, dW, 1L, (long)k, (double*)A_f64, (long)k, r, k, d_out, st);
    } else {
        // step 6: A = A' sqrt(Lambda)^-1 Q^T : A[i][j] = sum_e A'[i][e] inv[e] V[e][j]
        hipLaunchKernelGGL(scale_kernel, dim3(blocks((size_t)r * k)), dim3(256), 0, st, Ap, r, k, inv, 0);
        gemm(Ap, (long)k, 1L, V, 1L, (long)k, (double*)A_f64, (long)k, r, k, k, st);
    }
    if (sigma_f64) hipLaunchKernelGGL(copy_kernel, dim3(blocks(r)), dim3(256), 0, st, sigma, (double*)sigma_f64, (size_t)r);
    if (hipGetLastError() != hipSuccess) return EORA_ERR_LAUNCH;
    if (hipStreamSynchronize(st) != hipSuccess) return EORA_ERR_LAUNCH;
    return EORA_OK;
}

extern "C" int eora_factors_store_f16(const void* B_f64, const void* A_f64, int d_in, int d_out, int r, int balance,
                                      void* A_tiles, void* B_tiles, void* scratch, size_t scratch_bytes, void* stream)
{
    if (!B_f64 || !A_f64 || !A_tiles || !B_tiles) return EORA_ERR_NULL;
    if (d_in <= 0 || d_out <= 0 || r <= 0 || d_in % 32 || d_out % 16 || r % 32) return EORA_ERR_SHAPE;
    if ((reinterpret_cast<uintptr_t>(A_tiles) | reinterpret_cast<uintptr_t>(B_tiles) | reinterpret_cast<uintptr_t>(B_f64) |
         reinterpret_cast<uintptr_t>(A_f64)) & 15u)
        return EORA_ERR_ALIGN;
    double* s = nullptr;
    if (balance) {
        if (!scratch || scratch_bytes < sizeof(double) * (size_t)r) return EORA_ERR_WORKSPACE;
        if (reinterpret_cast<uintptr_t>(scratch) & 15u) return EORA_ERR_ALIGN;
        s = (double*)scratch;
    }
    hipStream_t st = (hipStream_t)stream;
    if (s) hipLaunchKernelGGL(balance_kernel, dim3(r), dim3(256), 0, st, (const double*)B_f64, (const double*)A_f64, d_in, d_out, r, s);
    hipLaunchKernelGGL(store_f16_tiles_kernel, dim3(blocks((size_t)r * d_in / 8)), dim3(256), 0, st, (const double*)A_f64, r, d_in,
                       (const double*)s, 1, (_Float16*)A_tiles);
    hipLaunchKernelGGL(store_f16_tiles_kernel, dim3(blocks((size_t)d_out * r / 8)), dim3(256), 0, st, (const double*)B_f64, d_out, r,
                       (const double*)s, 0, (_Float16*)B_tiles);
    if (hipGetLastError() != hipSuccess) return EORA_ERR_LAUNCH;
    return EORA_OK;
}

extern "C" int eora_factors_store_q(const void* B_f64, const void* A_f64, int d_in, int d_out, int r, int ab_bits, int balance,
                                    void* A_q, void* A_scales, void* B_q, void* B_scales, void* scratch, size_t scratch_bytes,
                                    void* stream)
{
    if (!B_f64 || !A_f64 || !A_q || !A_scales || !B_q || !B_scales) return EORA_ERR_NULL;
    if (ab_bits != 4 && ab_bits != 3) return EORA_ERR_UNSUPPORTED;
    if (d_in <= 0 || d_out <= 0 || r <= 0 || d_in % 128 || d_out % 16) return EORA_ERR_SHAPE;
    if (!(r % 128 == 0 || (ab_bits == 4 && r == 64))) return EORA_ERR_SHAPE;
    if ((reinterpret_cast<uintptr_t>(A_q) | reinterpret_cast<uintptr_t>(B_q) | reinterpret_cast<uintptr_t>(A_scales) |
         reinterpret_cast<uintptr_t>(B_scales) | reinterpret_cast<uintptr_t>(B_f64) | reinterpret_cast<uintptr_t>(A_f64)) & 15u)
        return EORA_ERR_ALIGN;
    double* s = nullptr;
    if (balance) {
        if (!scratch || scratch_bytes < sizeof(double) * (size_t)r) return EORA_ERR_WORKSPACE;
        if (reinterpret_cast<uintptr_t>(scratch) & 15u) return EORA_ERR_ALIGN;
        s = (double*)scratch;
    }
    hipStream_t st = (hipStream_t)stream;
    const double* A = (const double*)A_f64;
    const double* B = (const double*)B_f64;
    if (s) hipLaunchKernelGGL(balance_kernel, dim3(r), dim3(256), 0, st, B, A, d_in, d_out, r, s);
    const dim3 ga((r / 16) * (d_in / 128)), gb((d_out / 16) * (r / (r == 64 ? 64 : 128)));
    if (ab_bits == 4) {
        hipLaunchKernelGGL((store_q_tiles_kernel<4, 128>), ga, dim3(64), 0, st, A, r, d_in, (const double*)s, 1, (uint32_t*)A_q, (_Float16*)A_scales);
        if (r == 64)
            hipLaunchKernelGGL((store_q_tiles_kernel<4, 64>), gb, dim3(64), 0, st, B, d_out, r, (const double*)s, 0, (uint32_t*)B_q, (_Float16*)B_scales);
        else
            hipLaunchKernelGGL((store_q_tiles_kernel<4, 128>), gb, dim3(64), 0, st, B, d_out, r, (const double*)s, 0, (uint32_t*)B_q, (_Float16*)B_scales);
    } else {
        hipLaunchKernelGGL((store_q_tiles_kernel<3, 128>), ga, dim3(64), 0, st, A, r, d_in, (const double*)s, 1, (uint32_t*)A_q, (_Float16*)A_scales);
        hipLaunchKernelGGL((store_q_tiles_kernel<3, 128>), gb, dim3(64), 0, st, B, d_out, r, (const double*)s, 0, (uint32_t*)B_q, (_Float16*)B_scales);
    }
    if (hipGetLastError() != hipSuccess) return EORA_ERR_LAUNCH;
    return EORA_OK;
}
