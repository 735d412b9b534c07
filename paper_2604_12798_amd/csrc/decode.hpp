// Decode kernels: one query token per head against a growing key/value cache.
#pragma once
#include "common.hpp"

namespace {

// ---------------------------------------------------------------------------------------------
// Decode: one query token per head against a key/value cache, the keys split over workgroups.
// A wave carries the Hq / Hkv (<= 32) query heads of one KV head as the columns of its score tile
// (unused columns repeat the last head).  Three small kernels:
//   decode_max_kernel    per (KV head, split): max of q . summary over the split's share of the cache's
//                        block summaries, and the exact max over its share of the sink / local tiles
//   decode_split_kernel  per (KV head, split): with m = the max of all those partial maxima, fixed,
//                        sum exp(s - m) and sum exp(s - m) v over the split's key range
//   decode_merge_kernel  per query head: ADD the partial sums (no max in the merge, because no split
//                        ever rescales), divide, write O and LSE
// The work is HBM bound (K and V are read once), so single-wave workgroups with a small tile ring (64 KiB of LDS, two
// per CU) and the same tile helpers as the prefill kernels are enough.
struct DecodeParams {
    const uint16_t* Q;      // [B, Hq, d]
    const uint16_t* K;      // [B, Hkv, n_cap, d]
    const uint16_t* V;
    const uint16_t* Krepr;  // [B, Hkv, tc_cap, d]
    float* pm;              // [B * Hq, n_splits]     partial maxima, log2 units
    float* lpart;           // [B * Hq, n_splits]     partial sums of exp
    float* opart;           // [B * Hq, n_splits, d]  partial sums of exp * v
    uint16_t* O;            // [B, Hq, d]
    float* LSE;             // [B, Hq] or null
    int B, Hq, Hkv, n_cap, n_keys, tc_cap, n_splits, n_sink, n_local, use_minit;
    const int* seq_lens;    // null, or [B] device array: valid keys per batch entry (clamped to [1, n_cap]) instead of n_keys
    float c;
};

template <int D>
__device__ __forceinline__ void decode_rows(const DecodeParams& p, int bh, int lane, int& b, int& h, bf16x8* qf) {
    const int g = p.Hq / p.Hkv, hkv = bh % p.Hkv;
    b = bh / p.Hkv;
    h = hkv * g + min(lane & 31, g - 1);
#pragma unroll
    for (int kk = 0; kk < D / 16; ++kk)
        qf[kk] = *reinterpret_cast<const bf16x8*>(p.Q + ((size_t)b * p.Hq + h) * D + 16 * kk + 8 * (lane >> 5));
}

template <int D>
__global__ __launch_bounds__(64) void decode_max_kernel(const DecodeParams p) {
    using T = Tile<D>;
    __shared__ __attribute__((aligned(16))) uint8_t buf[T::BYTES];
    const int lane = threadIdx.x, ql = lane & 31, hh = lane >> 5;
    const int split = blockIdx.x, bh = blockIdx.y;
    int b, h;
    bf16x8 qf[D / 16];
    decode_rows<D>(p, bh, lane, b, h, qf);
    const int n_keys = p.seq_lens ? min(max(p.seq_lens[b], 1), p.n_cap) : p.n_keys;
    const int Tc = (n_keys + BN - 1) / BN;
    float mx = -INFINITY;
    f32x16 st[2];
    if (p.use_minit) {
        const uint16_t* Rg = p.Krepr + (size_t)bh * p.tc_cap * D;
        for (int ts = split; ts * BN < Tc; ts += p.n_splits) {
            load_tile<D, 1>(Rg, ts * BN, Tc, buf, false, 0, lane);
            wait_vm0_and_sync();
            qk_tile_pipe<D>(buf, qf, st, ql, hh);
            mx = fmaxf(mx, tile_rowmax<true>(st, ts * BN, Tc - 1, hh));
            __syncthreads();
        }
    }
    // sink tiles [0, n1) and local tiles [lo2, Tc): dealt round-robin over the splits
    const int n1 = min(p.n_sink, Tc), lo2 = max(n1, Tc - p.n_local);
    const uint16_t* Kg = p.K + (size_t)bh * p.n_cap * D;
    for (int u = split; u < n1 + (Tc - lo2); u += p.n_splits) {
        const int j = u < n1 ? u : lo2 + (u - n1);
        load_tile<D, 1>(Kg, j * BN, n_keys, buf, false, 0, lane);
        wait_vm0_and_sync();
        qk_tile_pipe<D>(buf, qf, st, ql, hh);
        mx = fmaxf(mx, tile_rowmax<true>(st, j * BN, n_keys - 1, hh));
        __syncthreads();
    }
    const float m2 = xhalf_max(mx) * p.c;
    if (ql < p.Hq / p.Hkv && hh == 0) p.pm[((size_t)b * p.Hq + h) * p.n_splits + split] = m2;
}

template <int D>
__global__ __launch_bounds__(64) void decode_split_kernel(const DecodeParams p) {
    using T = Tile<D>;
    constexpr int DB = D / 32;
    // K ring of three tiles filled two tiles ahead, V single buffered: 4 tiles = 64 KiB at d = 128, two workgroups per
    // CU; no wait in the loop drains the load queue: each waits only for the tile it is about to read
    __shared__ __attribute__((aligned(16))) uint8_t smem[4 * T::BYTES];
    uint8_t* const Ks = smem;
    uint8_t* const Vs = smem + 3 * T::BYTES;
    constexpr int NI = BN / (1024 / T::ROWB);  // load instructions per tile (one wave)
    constexpr int WAIT_BUT_1 = 0x0F70 | (NI & 15) | ((NI >> 4) << 14);              // s_waitcnt vmcnt(NI)
    constexpr int WAIT_BUT_2 = 0x0F70 | ((2 * NI) & 15) | (((2 * NI) >> 4) << 14);  // s_waitcnt vmcnt(2 NI)
    const int lane = threadIdx.x, ql = lane & 31, hh = lane >> 5;
    const int split = blockIdx.x, bh = blockIdx.y;
    int b, h;
    bf16x8 qf[D / 16];
    decode_rows<D>(p, bh, lane, b, h, qf);
    const size_t row = (size_t)b * p.Hq + h;
    float m2 = -INFINITY;
    for (int s = 0; s < p.n_splits; ++s) m2 = fmaxf(m2, p.pm[row * p.n_splits + s]);

    const int n_keys = p.seq_lens ? min(max(p.seq_lens[b], 1), p.n_cap) : p.n_keys;
    const int Tc = (n_keys + BN - 1) / BN;
    const int per = (Tc + p.n_splits - 1) / p.n_splits;
    const int t_lo = split * per, t_hi = min(Tc, t_lo + per);
    const uint16_t* Kg = p.K + (size_t)bh * p.n_cap * D;
    const uint16_t* Vg = p.V + (size_t)bh * p.n_cap * D;
    f32x16 ot[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db) ot[db] = f32x16{0};
    float lsum = 0.f;
    // requests in flight, oldest first, at the top of iteration t: K(t) [first iteration only], K(t + 1)
    if (t_lo < t_hi) load_tile<D, 1>(Kg, t_lo * BN, n_keys, Ks, false, 0, lane);
    if (t_lo + 1 < t_hi) load_tile<D, 1>(Kg, (t_lo + 1) * BN, n_keys, Ks + T::BYTES, false, 0, lane);
    int slot = 0;
    for (int t = t_lo; t < t_hi; ++t) {
        // the V buffer's last readers (the P.V MFMAs of the previous tile) have all issued
        load_tile<D, 1>(Vg, t * BN, n_keys, Vs, true, 0, lane);
        const int s2 = slot >= 1 ? slot - 1 : 2;  // slot of K(t + 2) = (slot + 2) % 3
        const bool more2 = t + 2 < t_hi, more1 = t + 1 < t_hi;
        if (more2) load_tile<D, 1>(Kg, (t + 2) * BN, n_keys, Ks + s2 * T::BYTES, false, 0, lane);
        // K(t) has landed when at most [K(t + 1)], V(t), [K(t + 2)] are still out
        const int later = (more1 ? 1 : 0) + 1 + (more2 ? 1 : 0);
        if (later == 3) __builtin_amdgcn_s_waitcnt(0x0F70 | ((3 * NI) & 15) | (((3 * NI) >> 4) << 14));
        else if (later == 2) __builtin_amdgcn_s_waitcnt(WAIT_BUT_2);
        else __builtin_amdgcn_s_waitcnt(WAIT_BUT_1);
        __syncthreads();
        f32x16 st[2];
        uint32_t pk[16];
        qk_tile_pipe<D>(Ks + slot * T::BYTES, qf, st, ql, hh);
        softmax_tile<false, true, DB>(st, pk, ot, m2, lsum, p.c, t * BN, n_keys - 1, hh);  // frozen max, ragged tail masked
        // V(t) has landed when at most K(t + 2) is still out (K(t + 1) was requested before V(t))
        if (more2) __builtin_amdgcn_s_waitcnt(WAIT_BUT_1);
        else __builtin_amdgcn_s_waitcnt(0x0F70);
        __syncthreads();
        pv_tile_pipe<D>(Vs, pk, ot, lane, hh);
        __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0): this tile's LDS reads are done before its buffers are refilled
        slot = slot == 2 ? 0 : slot + 1;
    }
    const float l = xhalf_sum(lsum);
    if (ql < p.Hq / p.Hkv) {
        if (hh == 0) p.lpart[row * p.n_splits + split] = l;
        float* og = p.opart + (row * p.n_splits + split) * D;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4)
                *reinterpret_cast<f32x4*>(og + 32 * db + 8 * q4 + 4 * hh) =
                    f32x4{ot[db][4 * q4], ot[db][4 * q4 + 1], ot[db][4 * q4 + 2], ot[db][4 * q4 + 3]};
    }
}

template <int D>
__global__ __launch_bounds__(D) void decode_merge_kernel(const DecodeParams p) {
    const size_t row = blockIdx.x;
    const int t = threadIdx.x;
    float m2 = -INFINITY, l = 0.f, o = 0.f;
    for (int s = 0; s < p.n_splits; ++s) {  // fixed order: the result does not depend on scheduling
        m2 = fmaxf(m2, p.pm[row * p.n_splits + s]);
        l += p.lpart[row * p.n_splits + s];
        o += p.opart[(row * p.n_splits + s) * D + t];
    }
    p.O[row * D + t] = (uint16_t)(pack_bf16(l > 0.f ? o / l : 0.f, 0.f) & 0xffffu);
    if (p.LSE && t == 0) p.LSE[row] = l > 0.f ? (m2 + __builtin_amdgcn_logf(l)) * kLn2 : -INFINITY;
}

}  // namespace
