// MFMA-only ceiling probe for bench.py: what the bf16 matrix cores of this chip deliver, at the clock the chip
// grants, to a kernel that does nothing but v_mfma_f32_32x32x16_bf16 on operands held in registers.
// Not part of libvfa.so; bench.py loads it to put a measured ceiling beside the published peak.
//
// Launch shape as the attention kernel's: 512-thread workgroups (two waves per SIMD), one or more per CU.
// Each wave loads 8 A and 8 B fragments (32 x 16 bf16 each) from `data` once and then runs `iters` rounds of
// 16 independent MFMAs on them (4 accumulators x 4 operand pairs), so the matrix pipe never waits for a
// dependent result.  The operand VALUES matter for the clock (power follows how many bits toggle), so the
// caller passes both normally distributed data (what attention sees) and zeros.
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

__global__ __launch_bounds__(512, 2) void mfma_probe_kernel(const uint16_t* data, float* out, int iters) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    bf16x8 a[8], b[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        a[i] = *reinterpret_cast<const bf16x8*>(data + ((size_t)(wave * 16 + i) * 64 + lane) * 8);
        b[i] = *reinterpret_cast<const bf16x8*>(data + ((size_t)(wave * 16 + 8 + i) * 64 + lane) * 8);
    }
    f32x16 acc[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) acc[i] = f32x16{0};
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < 16; ++u)
            acc[u & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[(u + (u >> 2)) & 7], b[u & 7], acc[u & 3], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) s += acc[i][r];
    out[(size_t)blockIdx.x * 512 + threadIdx.x] = s;
}

extern "C" {

// bytes of `data` (bf16) a launch reads: 8 waves x 16 fragments x 64 lanes x 8 elements
size_t mfma_probe_data_elems(void) { return (size_t)8 * 16 * 64 * 8; }

// FLOP of one launch
double mfma_probe_flop(int blocks, int iters) { return (double)blocks * 8.0 * (double)iters * 16.0 * 2.0 * 32.0 * 32.0 * 16.0; }

// data: device, mfma_probe_data_elems() bf16 values; out: device, blocks * 512 floats.  Returns 0 or -1.
int mfma_probe_launch(const void* data, void* out, int blocks, int iters, void* stream) {
    if (!data || !out || blocks <= 0 || iters <= 0) return -1;
    (void)hipGetLastError();
    mfma_probe_kernel<<<dim3((unsigned)blocks), 512, 0, (hipStream_t)stream>>>((const uint16_t*)data, (float*)out, iters);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

}  // extern "C"
