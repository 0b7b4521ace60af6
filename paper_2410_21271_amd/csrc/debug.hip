// Parity exports: stored bytes -> row-major logical arrays (integer / exact work).
// One thread per (tile, lane): it decodes the words it owns with plain shifts and masks and
// scatters the results; these kernels are meant to be obviously right, not fast.
#include "kernels.hpp"

namespace eora {

__device__ __forceinline__ uint32_t code_q4(const uint32_t* w, int cc)
{
    const int t = cc >> 3, kk = cc & 7;
    const int e = 4 * (kk & 1) + (kk >> 1);
    return (w[t] >> (4 * e)) & 0xFu;
}

__device__ __forceinline__ uint32_t code_q3(const uint32_t* w, int cc)
{
    if (cc < 30) {
        const int p = cc >> 1, h = cc & 1;
        return (w[p / 5] >> (16 * h + 3 * (p % 5))) & 7u;
    }
    const int s = 16 * (cc - 30) + 15;
    return ((w[0] >> s) & 1u) | (((w[1] >> s) & 1u) << 1) | (((w[2] >> s) & 1u) << 2);
}

__device__ __forceinline__ uint32_t code_q2(const uint32_t* w, int cc)
{
    return (w[cc >> 4] >> (16 * (cc & 1) + 2 * ((cc & 15) >> 1))) & 3u;
}

template <bool DEQUANT>
__global__ void unpack_q_kernel(const uint32_t* __restrict__ qweight, const _Float16* __restrict__ scales,
                                const uint32_t* __restrict__ qzeros, uint8_t* __restrict__ codes,
                                uint8_t* __restrict__ zeros_out, float* __restrict__ W,
                                int d_in, int d_out, int w_bits, int group)
{
    const size_t L = (size_t)blockIdx.x * blockDim.x + threadIdx.x;     // global (tile, lane)
    const size_t nlanes = (size_t)d_out * d_in / 32;
    if (L >= nlanes) return;
    const int ntk = d_in / 128, NG = d_in / group;
    const size_t tile = L / 64;
    const int lane = (int)(L % 64);
    const int R = (int)(tile / ntk), g = (int)(tile % ntk);
    const int j = lane >> 4, n = lane & 15;
    const int row = 16 * R + n, col0 = 128 * g + 32 * j;
    const int q = col0 / group;
    const int NGW = (NG + 7) / 8;
    const uint32_t z = (qzeros[(size_t)row * NGW + (q >> 3)] >> (4 * (q & 7))) & 0xFu;
    uint32_t w[4];
    const int wpl = w_bits;                    // words per lane: 32 codes of w_bits bits
    for (int t = 0; t < wpl; ++t) w[t] = qweight[L * wpl + t];
    float s = 0.f;
    if (DEQUANT) s = (float)scales[(size_t)row * NG + q];
    for (int cc = 0; cc < 32; ++cc) {
        const uint32_t c = w_bits == 4 ? code_q4(w, cc) : (w_bits == 3 ? code_q3(w, cc) : code_q2(w, cc));
        const size_t idx = (size_t)row * d_in + col0 + cc;
        if (DEQUANT) W[idx] = s * (float)((int)c - (int)z);      // 11-bit x 5-bit product: exact in fp32
        else codes[idx] = (uint8_t)c;
    }
    if (!DEQUANT && col0 % group == 0) zeros_out[(size_t)row * NG + q] = (uint8_t)z;
}

__global__ void expand_sp24_kernel(const _Float16* __restrict__ values, const uint32_t* __restrict__ indices,
                                   _Float16* __restrict__ W, int d_in, int d_out)
{
    const size_t L = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t nlanes = (size_t)d_out * d_in / 32;
    if (L >= nlanes) return;
    const int ntk = d_in / 128;
    const size_t tile = L / 64;
    const int lane = (int)(L % 64);
    const int R = (int)(tile / ntk), g = (int)(tile % ntk);
    const int j = lane >> 4, n = lane & 15;
    const uint32_t word = indices[L];
    for (int s = 0; s < 2; ++s)
        for (int q = 0; q < 4; ++q) {
            _Float16 out[4] = {(_Float16)0.f, (_Float16)0.f, (_Float16)0.f, (_Float16)0.f};
            for (int v = 0; v < 2; ++v) {
                const int p = (word >> (16 * s + 4 * q + 2 * v)) & 3;
                out[p] = values[tile * 1024 + s * 512 + lane * 8 + 2 * q + v];
            }
            _Float16* dst = W + (size_t)(16 * R + n) * d_in + 128 * g + 64 * s + 16 * j + 4 * q;
            for (int p = 0; p < 4; ++p) dst[p] = out[p];
        }
}

// 2:4 sparse with 4-bit kept values -> dense fp32: scale*(code - zero) at the kept positions (exact in
// fp32), +0 elsewhere.  One thread per (tile, lane), plain shifts and masks.
__global__ void expand_sp24q4_kernel(const uint32_t* __restrict__ qtiles, const uint32_t* __restrict__ qmeta,
                                     float* __restrict__ W, int d_in, int d_out)
{
    const size_t L = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t nlanes = (size_t)d_out * d_in / 32;
    if (L >= nlanes) return;
    const int ntk = d_in / 128;
    const size_t tile = L / 64;
    const int lane = (int)(L % 64);
    const int R = (int)(tile / ntk), g = (int)(tile % ntk);
    const int j = lane >> 4, n = lane & 15;
    const size_t row = (size_t)16 * R + n;
    const uint32_t m = qmeta[tile * 16 + n];
    const float sc = (float)__builtin_bit_cast(_Float16, (uint16_t)(m & 0xFFFFu));
    const int z = (int)((m >> 16) & 0xFu);
    const uint32_t word = qtiles[3 * L + 2];
    for (int s = 0; s < 2; ++s) {
        const uint32_t cw = qtiles[3 * L + s];
        for (int q = 0; q < 4; ++q) {
            float out[4] = {0.f, 0.f, 0.f, 0.f};
            for (int v = 0; v < 2; ++v) {
                const int p = (word >> (16 * s + 4 * q + 2 * v)) & 3;
                const int e = 2 * q + v;
                const int code = (int)((cw >> (4 * (4 * (e % 2) + e / 2))) & 0xFu);
                out[p] = sc * (float)(code - z);
            }
            float* dst = W + row * d_in + 128 * g + 64 * s + 16 * j + 4 * q;
            for (int p = 0; p < 4; ++p) dst[p] = out[p];
        }
    }
}

static dim3 grid_for(size_t nlanes) { return dim3((unsigned)((nlanes + 255) / 256)); }

hipError_t launch_unpack_q(const uint32_t* qweight, const uint32_t* qzeros, uint8_t* codes, uint8_t* zeros,
                           int d_in, int d_out, int w_bits, int group, hipStream_t stream)
{
    const size_t nlanes = (size_t)d_out * d_in / 32;
    hipLaunchKernelGGL((unpack_q_kernel<false>), grid_for(nlanes), dim3(256), 0, stream, qweight,
                       (const _Float16*)nullptr, qzeros, codes, zeros, (float*)nullptr, d_in, d_out, w_bits, group);
    return hipGetLastError();
}

hipError_t launch_dequant_q(const uint32_t* qweight, const _Float16* scales, const uint32_t* qzeros, float* W,
                            int d_in, int d_out, int w_bits, int group, hipStream_t stream)
{
    const size_t nlanes = (size_t)d_out * d_in / 32;
    hipLaunchKernelGGL((unpack_q_kernel<true>), grid_for(nlanes), dim3(256), 0, stream, qweight, scales, qzeros,
                       (uint8_t*)nullptr, (uint8_t*)nullptr, W, d_in, d_out, w_bits, group);
    return hipGetLastError();
}

hipError_t launch_expand_sp24(const _Float16* values, const uint32_t* indices, _Float16* W,
                              int d_in, int d_out, hipStream_t stream)
{
    const size_t nlanes = (size_t)d_out * d_in / 32;
    hipLaunchKernelGGL(expand_sp24_kernel, grid_for(nlanes), dim3(256), 0, stream, values, indices, W, d_in, d_out);
    return hipGetLastError();
}

hipError_t launch_expand_sp24q4(const uint32_t* qtiles, const uint32_t* qmeta, float* W, int d_in, int d_out, hipStream_t stream)
{
    const size_t nlanes = (size_t)d_out * d_in / 32;
    hipLaunchKernelGGL(expand_sp24q4_kernel, grid_for(nlanes), dim3(256), 0, stream, qtiles, qmeta, W, d_in, d_out);
    return hipGetLastError();
}

// ---- measurement probes: what a launch costs and what a pure read of n bytes reaches on this device ----------
typedef uint32_t u4 __attribute__((ext_vector_type(4)));

__global__ void probe_empty_kernel(uint32_t* sink)
{
    if (sink == nullptr && threadIdx.x == 4096) sink[0] = 1u;      // never true: the kernel does nothing
}

// every workgroup of 256 threads reads 32 KiB: eight 16-byte loads per lane, all in flight at once; the result
// is consumed without being stored (the store's condition never holds for data that is not all-ones patterns).
// The requests carry the non-temporal hint, as the layer kernels' requests for stored tiles do: a pure read of
// 56 MB reaches 6.15 TB/s with it and 5.7 TB/s without, of 241 MB 6.85 against 6.3.
__global__ __launch_bounds__(256) void probe_stream_kernel(const u4* __restrict__ src, uint32_t* sink)
{
    const u4* p = src + (size_t)blockIdx.x * 2048 + threadIdx.x;
    u4 v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = __builtin_nontemporal_load(p + u * 256);
    u4 acc = v[0];
#pragma unroll
    for (int u = 1; u < 8; ++u) acc ^= v[u];
    if ((acc[0] ^ acc[1] ^ acc[2] ^ acc[3]) == 0x9E3779B9u && acc[0] == 0x7F4A7C15u) sink[blockIdx.x & 63] = 1u;
}

hipError_t launch_probe_empty(uint32_t* sink, hipStream_t stream)
{
    hipLaunchKernelGGL(probe_empty_kernel, dim3(256), dim3(256), 0, stream, sink);
    return hipGetLastError();
}

hipError_t launch_probe_stream(const void* src, size_t bytes, uint32_t* sink, hipStream_t stream)
{
    hipLaunchKernelGGL(probe_stream_kernel, dim3((unsigned)(bytes / 32768)), dim3(256), 0, stream, (const u4*)src, sink);
    return hipGetLastError();
}

}  // namespace eora
