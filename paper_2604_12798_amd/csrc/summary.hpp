// Key-block summary pre-passes (sabsmax and the ablated representations).
#pragma once
#include "common.hpp"

namespace {

// ---------------------------------------------------------------------------------------------
// Key-block summary (Alg. 1, first loop): per dimension the element of largest magnitude of the block's keys with its
// sign, ties to the positive value.  HBM bound: K is read once.  One WAVE per key block, four blocks per workgroup:
// a lane owns one 16-byte chunk of every RG-th row, issues its loads eight at a time (no loop-carried dependence
// between them), reduces in registers, and the RG lanes of a chunk combine through lane exchanges: no LDS, no
// barrier, 128 bytes per lane in flight.
// Works on bf16 bit patterns, two to a dword: the key (magnitude << 1) | (sign ? 0 : 1) orders elements by magnitude
// and, at equal magnitude, puts the positive one on top, so the pick is an unsigned 16-bit maximum of keys.
typedef __attribute__((ext_vector_type(2))) unsigned short u16x2;
__device__ inline uint32_t sabs_key(uint32_t x) { return ((x << 1) & 0xfffefffeu) | ((~x >> 15) & 0x00010001u); }
__device__ inline uint32_t sabs_unkey(uint32_t k) { return ((k >> 1) & 0x7fff7fffu) | ((~k & 0x00010001u) << 15); }
__device__ inline uint32_t key_max(uint32_t a, uint32_t b) {
    return __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(u16x2, a), __builtin_bit_cast(u16x2, b)));
}

// N = row stride of one head's key array (its capacity), n_valid = keys present, Tc = block stride of
// one head's summary array, j0 = first block to (re)compute and n_blocks their number: a growing cache
// recomputes only the blocks that received keys.
// With per-sequence lengths (old_len / new_len device arrays indexed by batch entry, Hkv heads per entry) the
// grid covers every block of the capacity and a wave whose block received no key returns at once.
template <int D>
__global__ __launch_bounds__(256) void kblock_summary_kernel(const uint16_t* __restrict__ K, uint16_t* __restrict__ R,
                                                             int N, int n_valid, int Tc, int block_n, int j0, int n_blocks,
                                                             const int* __restrict__ old_len = nullptr,
                                                             const int* __restrict__ new_len = nullptr, int Hkv = 1) {
    constexpr int CH = D / 8;        // 16-byte chunks per row
    constexpr int RG = 64 / CH;      // rows a wave reads at once
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int jb = blockIdx.x * 4 + wave, bh = blockIdx.y;
    if (jb >= n_blocks) return;
    const int j = j0 + jb;
    if (new_len) {
        const int b = bh / Hkv;
        const int n_new = min(max(new_len[b], 0), N), n_old = min(max(old_len[b], 0), n_new);
        if (j < n_old / block_n || j * block_n >= n_new) return;  // (uniform over the wave)
        n_valid = n_new;
    }
    const int ch = lane % CH, rg = lane / CH;
    const int c0 = j * block_n, c1 = min(n_valid, c0 + block_n);
    const uint16_t* base = K + (size_t)bh * N * D + ch * 8;
    const uint32_t zero_key = sabs_key(0u);  // +0: the smallest magnitude, already the positive one
    u32x4 acc = {zero_key, zero_key, zero_key, zero_key};
    for (int r0 = c0 + rg; r0 < c1; r0 += 8 * RG) {
        u32x4 x[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int r = r0 + u * RG;
            // (non-temporal: a streaming read; 10 % faster at 64 MiB of keys, no change to the attention kernel behind it)
            x[u] = r < c1 ? __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(base + (size_t)r * D)) : u32x4{0, 0, 0, 0};
        }
#pragma unroll
        for (int u = 0; u < 8; ++u)
#pragma unroll
            for (int e = 0; e < 4; ++e) acc[e] = key_max(acc[e], sabs_key(x[u][e]));
    }
#pragma unroll
    for (int m = CH; m < 64; m <<= 1)
#pragma unroll
        for (int e = 0; e < 4; ++e) acc[e] = key_max(acc[e], (uint32_t)__shfl_xor((int)acc[e], m));
    if (rg == 0) {
        const u32x4 out = {sabs_unkey(acc[0]), sabs_unkey(acc[1]), sabs_unkey(acc[2]), sabs_unkey(acc[3])};
        *reinterpret_cast<u32x4*>(R + ((size_t)bh * Tc + j) * D + ch * 8) = out;
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
