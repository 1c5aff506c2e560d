// naut_probe.hip -- a register-only MFMA loop: what the matrix pipes of this chip sustain when nothing else
// runs (no LDS, no global memory, no vector arithmetic), on operands of a chosen kind.  Not part of the
// attention path: it exists so that the benchmark can print, beside the published peak, the rate the same
// instruction (v_mfma_f32_32x32x16_bf16) reaches on the box at hand -- the chip lowers its clock under
// sustained matrix load, and by how much depends on the operand data.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "naut_attn.h"
#include "naut_common.h"

namespace {

using namespace naut;

constexpr int PROBE_WAVES = 8;   // two wavefronts per SIMD, as in the pipelined attention kernel
constexpr int PROBE_UNROLL = 16; // MFMAs per loop trip
constexpr int PROBE_NA = 8, PROBE_NB = 4, PROBE_NC = 4;

// 64-bit mix (splitmix64 finaliser) for the operand bit patterns
__device__ __forceinline__ unsigned long long mix64(unsigned long long z)
{
    z = (z ^ (z >> 30)) * 0xbf58476d1ce4e5b9ull;
    z = (z ^ (z >> 27)) * 0x94d049bb133111ebull;
    return z ^ (z >> 31);
}

// One bf16 bit pattern: kind 0 -> +0; kind 1 -> a value with a random sign, a random 7-bit fraction and an
// exponent spread over a few binades around 1 (what normally distributed data looks like to the multipliers).
__device__ __forceinline__ unsigned bf16_pattern(unsigned long long r, int kind)
{
    if (kind == 0)
        return 0u;
    const unsigned sign = (unsigned)(r & 1) << 15;
    const unsigned frac = (unsigned)(r >> 1) & 0x7f;
    const unsigned expo = 124u + ((unsigned)(r >> 8) & 3u) + ((unsigned)(r >> 10) & 1u);  // 2^-3 .. 2^1
    return sign | (expo << 7) | frac;
}

__global__ __launch_bounds__(PROBE_WAVES * 64, 1) void naut_probe_mfma_kernel(float* out, int trips, int kind)
{
    const unsigned gid = blockIdx.x * blockDim.x + threadIdx.x;
    i32x4_t a[PROBE_NA], b[PROBE_NB];
    unsigned long long r = mix64(0x2604'14825ull + gid);
    auto frag = [&]() {
        i32x4_t f;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            r = mix64(r + 0x9e3779b97f4a7c15ull);
            f[w] = (int)(bf16_pattern(r, kind) | (bf16_pattern(r >> 20, kind) << 16));
        }
        return f;
    };
#pragma unroll
    for (int i = 0; i < PROBE_NA; ++i)
        a[i] = frag();
#pragma unroll
    for (int i = 0; i < PROBE_NB; ++i)
        b[i] = frag();
    f32x16_t c[PROBE_NC];
#pragma unroll
    for (int i = 0; i < PROBE_NC; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e)
            c[i][e] = 0.f;
    for (int t = 0; t < trips; ++t) {
#pragma unroll
        for (int u = 0; u < PROBE_UNROLL; ++u)  // a fresh A operand every MFMA, as with K and V fragments from LDS
            c[u % PROBE_NC] = In<NAUT_BF16>::mfma(a[u % PROBE_NA], b[(u / PROBE_NC) % PROBE_NB], c[u % PROBE_NC]);
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < PROBE_NC; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e)
            s += c[i][e];
    out[gid] = s;
}

}  // namespace

extern "C" {

int naut_probe_mfma(float* out, size_t out_floats, int work_groups, int trips, int kind, void* stream)
{
    if (!out)
        return fail(NAUT_ERR_NULL, "out must be a non-NULL device pointer");
    if (work_groups <= 0 || trips <= 0 || (kind != 0 && kind != 1))
        return fail(NAUT_ERR_SHAPE, "work_groups and trips must be positive, kind 0 or 1");
    if (out_floats < (size_t)work_groups * PROBE_WAVES * 64)
        return fail(NAUT_ERR_SHAPE, "out must hold work_groups * 512 floats");
    hipLaunchKernelGGL(naut_probe_mfma_kernel, dim3((unsigned)work_groups), dim3(PROBE_WAVES * 64), 0, (hipStream_t)stream,
                       out, trips, kind);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess)
        return fail_launch(e);
    return NAUT_OK;
}

}  // extern "C"
