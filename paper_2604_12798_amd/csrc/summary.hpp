// Key-block summary pre-passes (sabsmax and the ablated representations).
#pragma once
#include "common.hpp"

namespace {

// ---------------------------------------------------------------------------------------------
// Key-block summary: one workgroup per (b*Hkv + h, j); signed element of largest magnitude per
// dimension over the block's keys, ties to the positive value.  Works on bf16 bit patterns:
// magnitude order = order of (bits & 0x7fff); on equal magnitude the smaller pattern is the
// positive one.
__device__ inline uint32_t sabs_pick(uint32_t a, uint32_t b) {  // one bf16 in the low 16 bits
    const uint32_t ma = a & 0x7fffu, mb = b & 0x7fffu;
    return ma > mb ? a : (mb > ma ? b : min(a, b));
}
__device__ inline uint32_t sabs_pick2(uint32_t a, uint32_t b) {  // two packed bf16
    return sabs_pick(a & 0xffffu, b & 0xffffu) | (sabs_pick(a >> 16, b >> 16) << 16);
}

// N = row stride of one head's key array (its capacity), n_valid = keys present, Tc = block stride of
// one head's summary array, j0 = first block to (re)compute: a growing cache recomputes only the
// blocks that received keys.
// With per-sequence lengths (old_len / new_len device arrays indexed by batch entry, Hkv heads per entry) the
// grid covers every block of the capacity and a workgroup whose block received no key returns at once.
template <int D>
__global__ __launch_bounds__(256) void kblock_summary_kernel(const uint16_t* __restrict__ K, uint16_t* __restrict__ R,
                                                             int N, int n_valid, int Tc, int block_n, int j0,
                                                             const int* __restrict__ old_len = nullptr,
                                                             const int* __restrict__ new_len = nullptr, int Hkv = 1) {
    constexpr int CH = D / 8;        // 16-byte chunks per row
    constexpr int RG = 256 / CH;     // row groups
    __shared__ u32x4 part[RG][CH];
    const int j = j0 + blockIdx.x, bh = blockIdx.y;
    if (new_len) {
        const int b = bh / Hkv;
        const int n_new = min(max(new_len[b], 0), N), n_old = min(max(old_len[b], 0), n_new);
        if (j < n_old / block_n || j * block_n >= n_new) return;  // (uniform over the workgroup)
        n_valid = n_new;
    }
    const int ch = threadIdx.x % CH, rg = threadIdx.x / CH;
    const int c0 = j * block_n, c1 = min(n_valid, c0 + block_n);
    const uint16_t* base = K + (size_t)bh * N * D;
    u32x4 acc = {0, 0, 0, 0};
    for (int r = c0 + rg; r < c1; r += RG) {
        const u32x4 x = *reinterpret_cast<const u32x4*>(base + (size_t)r * D + ch * 8);
#pragma unroll
        for (int e = 0; e < 4; ++e) acc[e] = sabs_pick2(acc[e], x[e]);
    }
    part[rg][ch] = acc;
    __syncthreads();
    if (rg == 0) {
        for (int q = 1; q < RG; ++q) {
            const u32x4 x = part[q][ch];
#pragma unroll
            for (int e = 0; e < 4; ++e) acc[e] = sabs_pick2(acc[e], x[e]);
        }
        *reinterpret_cast<u32x4*>(R + ((size_t)bh * Tc + j) * D + ch * 8) = acc;
    }
}

// The three ablated block representations (ablation of the k_repr construction): per dimension the
// maximum (mode 1), the mean (mode 2: fp32 sum in a fixed order, rounded to bf16) or the largest
// magnitude without its sign (mode 3).  Not on the hot path: one thread per (row group, 8 dims).
template <int D>
__global__ __launch_bounds__(256) void kblock_summary_alt_kernel(const uint16_t* __restrict__ K, uint16_t* __restrict__ R,
                                                                 int N, int Tc, int block_n, int mode) {
    constexpr int CH = D / 8;
    constexpr int RG = 256 / CH;
    __shared__ float part[RG][D];
    const int j = blockIdx.x, bh = blockIdx.y;
    const int ch = threadIdx.x % CH, rg = threadIdx.x / CH;
    const int c0 = j * block_n, c1 = min(N, c0 + block_n);
    const uint16_t* base = K + (size_t)bh * N * D;
    float acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = mode == 1 ? -INFINITY : 0.f;
    for (int r = c0 + rg; r < c1; r += RG) {
        const u32x4 x = *reinterpret_cast<const u32x4*>(base + (size_t)r * D + ch * 8);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float v = __uint_as_float(((x[e >> 1] >> (16 * (e & 1))) & 0xffffu) << 16);
            acc[e] = mode == 1 ? fmaxf(acc[e], v) : (mode == 2 ? acc[e] + v : fmaxf(acc[e], fabsf(v)));
        }
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) part[rg][ch * 8 + e] = acc[e];
    __syncthreads();
    if (rg == 0) {
        const int nrg = min(RG, c1 - c0);  // row groups that saw at least one row
        uint32_t out[4];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float a = acc[e];
            for (int q = 1; q < nrg; ++q) {
                const float v = part[q][ch * 8 + e];
                a = mode == 2 ? a + v : fmaxf(a, v);
            }
            if (mode == 2) a /= (float)(c1 - c0);
            const uint32_t bits = pack_bf16(a, 0.f) & 0xffffu;
            out[e >> 1] = (e & 1) ? (out[e >> 1] | (bits << 16)) : bits;
        }
        *reinterpret_cast<u32x4*>(R + ((size_t)bh * Tc + j) * D + ch * 8) = u32x4{out[0], out[1], out[2], out[3]};
    }
}

}  // namespace
