// Ceiling probes for bench.py.  Not part of libvfa.so; bench.py loads this library to put measured ceilings beside
// the published peaks: what the matrix cores of this chip deliver, at the clock the chip grants, to a kernel that does
// nothing but MFMAs on operands held in registers (bf16: v_mfma_f32_32x32x16_bf16; 8-bit: v_mfma_scale_f32_32x32x64_f8f6f4
// on E4M3 operands), and what HBM delivers to a kernel that only reads.
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

// 8-bit form: 32x32x64 E4M3 products (unit block scales), 8 A and 8 B fragments of 32 bytes per lane
typedef __attribute__((ext_vector_type(8))) int i32x8;
__global__ __launch_bounds__(512, 2) void mfma_fp8_probe_kernel(const uint8_t* data, float* out, int iters) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    i32x8 a[4], b[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        a[i] = *reinterpret_cast<const i32x8*>(data + ((size_t)(wave * 8 + i) * 64 + lane) * 32);
        b[i] = *reinterpret_cast<const i32x8*>(data + ((size_t)(wave * 8 + 4 + i) * 64 + lane) * 32);
    }
    f32x16 acc[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) acc[i] = f32x16{0};
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < 16; ++u)
            acc[u & 3] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a[(u + (u >> 2)) & 3], b[u & 3], acc[u & 3], 0, 0, 0, 0x7f7f7f7f, 0,
                                                                         0x7f7f7f7f);
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) s += acc[i][r];
    out[(size_t)blockIdx.x * 512 + threadIdx.x] = s;
}

// streaming read: every lane reads 16 bytes per step, a workgroup 4 KiB, the grid walks the buffer once
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
template <int U>
__global__ __launch_bounds__(256) void hbm_read_probe_kernel(const u32x4* data, uint32_t* out, size_t n16) {
    const size_t stride = (size_t)gridDim.x * 256;
    u32x4 acc = {0, 0, 0, 0};
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    for (; i + (U - 1) * stride < n16; i += U * stride) {  // U loads in flight per lane
        u32x4 x[U];
#pragma unroll
        for (int u = 0; u < U; ++u) x[u] = __builtin_nontemporal_load(data + i + u * stride);
#pragma unroll
        for (int u = 0; u < U; ++u) acc ^= x[u];
    }
    for (; i < n16; i += stride) acc ^= data[i];
    out[(size_t)blockIdx.x * 256 + threadIdx.x] = acc[0] ^ acc[1] ^ acc[2] ^ acc[3];
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

// E4M3 form: data = 8 waves x 8 fragments x 64 lanes x 32 bytes; FLOP per launch = mfma_probe_flop(blocks, iters) * 4
size_t mfma_fp8_probe_data_bytes(void) { return (size_t)8 * 8 * 64 * 32; }
int mfma_fp8_probe_launch(const void* data, void* out, int blocks, int iters, void* stream) {
    if (!data || !out || blocks <= 0 || iters <= 0) return -1;
    (void)hipGetLastError();
    mfma_fp8_probe_kernel<<<dim3((unsigned)blocks), 512, 0, (hipStream_t)stream>>>((const uint8_t*)data, (float*)out, iters);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

// reads `bytes` (a multiple of 16) from data once with 4, 8 or 16 loads in flight per lane; out: blocks * 256 dwords
int hbm_read_probe_launch(const void* data, void* out, size_t bytes, int blocks, int loads_in_flight, void* stream) {
    if (!data || !out || blocks <= 0 || (bytes & 15)) return -1;
    (void)hipGetLastError();
    const dim3 grid((unsigned)blocks);
    hipStream_t s = (hipStream_t)stream;
    if (loads_in_flight >= 16) hbm_read_probe_kernel<16><<<grid, 256, 0, s>>>((const u32x4*)data, (uint32_t*)out, bytes / 16);
    else if (loads_in_flight >= 8) hbm_read_probe_kernel<8><<<grid, 256, 0, s>>>((const u32x4*)data, (uint32_t*)out, bytes / 16);
    else hbm_read_probe_kernel<4><<<grid, 256, 0, s>>>((const u32x4*)data, (uint32_t*)out, bytes / 16);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

}  // extern "C"
