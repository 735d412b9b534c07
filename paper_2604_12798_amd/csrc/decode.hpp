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
// The work is HBM bound (K and V are read once), so single-wave workgroups with the score and P.V helpers of the prefill
// kernels are enough; what matters is how the tiles are fetched: into registers, with non-temporal loads, one tile ahead,
// and from there into the two LDS tiles a workgroup owns (see decode_split_kernel).
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

// One 64-row tile, global -> registers with the tile mover's lane mapping (every instruction covers whole rows, 1 KiB
// contiguous; the swizzle is applied on the global side), and registers -> LDS at the positions the LDS-direct mover
// writes.  The loads are non-temporal: the cache is streamed through once per step and is larger than L2 and the
// memory-side cache, and plain loads, which allocate there, cost 12 % of the stream's rate (LDS-direct loads another 7 %).
// A whole tile (FULL) is addressed as a wave-uniform tile base plus a per-lane 32-bit offset that repeats every 16 rows
// (offs[u & 3]: four values for K at d = 128, one otherwise); a ragged last tile clamps its rows.
template <int D>
__device__ __forceinline__ void tile_lane_offsets(bool is_v, int lane, uint32_t* offs) {
    using T = Tile<D>;
    constexpr int RPI = 1024 / T::ROWB;
    const int cp = lane % T::CH;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int rr = RPI * u + lane / T::CH;
        const int ch = is_v ? (cp ^ ((rr & (T::CH / 4 - 1)) << 2)) : (cp ^ (rr & (T::CH - 1)));
        offs[u] = (uint32_t)((lane / T::CH) * T::ROWB + ch * 16);
    }
}
template <int D, bool FULL>
__device__ __forceinline__ void tile_to_regs(const uint16_t* base, int first_row, int row_limit, bool is_v, int lane,
                                             const uint32_t* offs, u32x4* r) {
    using T = Tile<D>;
    constexpr int RPI = 1024 / T::ROWB, NI = BN / RPI;
    if (FULL) {
        const uint8_t* tb = reinterpret_cast<const uint8_t*>(base) + (size_t)first_row * T::ROWB;
#pragma unroll
        for (int u = 0; u < NI; ++u) r[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(tb + (u * 1024 + offs[u & 3])));
    } else {
        const int cp = lane % T::CH;
#pragma unroll
        for (int u = 0; u < NI; ++u) {
            const int rr = RPI * u + lane / T::CH;
            const int ch = is_v ? (cp ^ ((rr & (T::CH / 4 - 1)) << 2)) : (cp ^ (rr & (T::CH - 1)));
            const int gr = min(first_row + rr, row_limit - 1);
            r[u] = __builtin_nontemporal_load(
                reinterpret_cast<const u32x4*>(reinterpret_cast<const uint8_t*>(base) + (size_t)gr * T::ROWB + ch * 16));
        }
    }
}
template <int D>
__device__ __forceinline__ void regs_to_tile(uint8_t* dst, int lane, const u32x4* r) {
    using T = Tile<D>;
    constexpr int NI = BN / (1024 / T::ROWB);
#pragma unroll
    for (int u = 0; u < NI; ++u) *reinterpret_cast<u32x4*>(dst + u * 1024 + lane * 16) = r[u];
}

// The tiles are staged through registers: while tile t is worked on, V(t + 1) and K(t + 1), then K(t + 2), are in flight
// in registers (the accumulation registers: loads and LDS writes take them directly), each requested one tile ahead of
// its use, and LDS holds only the two tiles being read (32 KiB at d = 128; one wave per SIMD, four workgroups per CU).  The LDS executes a wave's instructions in
// order: a tile is written over its predecessor behind the last read of that one, without a wait.  The steady loop runs
// over whole tiles and has no branch between a load and its use, so that the compiler's wait counts stay exact (a load
// that sits behind a branch makes it wait for everything at the join); the last one to three tiles, among them a
// ragged one, take the same body with the missing requests compiled out.
template <int D>
__global__ __launch_bounds__(64) void decode_split_kernel(const DecodeParams p) {
    using T = Tile<D>;
    constexpr int DB = D / 32;
    constexpr int NI = BN / (1024 / T::ROWB);
    __shared__ __attribute__((aligned(16))) uint8_t smem[2 * T::BYTES];
    uint8_t* const Ks = smem;
    uint8_t* const Vs = smem + T::BYTES;
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
    const int t_whole = min(t_hi, n_keys / BN);  // tiles below this index are whole
    const uint16_t* Kg = p.K + (size_t)bh * p.n_cap * D;
    const uint16_t* Vg = p.V + (size_t)bh * p.n_cap * D;
    uint32_t offk[4], offv[4];
    tile_lane_offsets<D>(false, lane, offk);
    tile_lane_offsets<D>(true, lane, offv);
    f32x16 ot[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db) ot[db] = f32x16{0};
    float lsum = 0.f;
    u32x4 rk[NI], rv[NI];
    // tile t.  On entry K(t) is in LDS, rv holds V(t) and, requested after it, rk holds K(t + 1) (HASK1).
    // HASV1 / HASK2: tiles t + 1 / t + 2 exist; FULL: the tiles requested here are whole
    auto body = [&](int t, auto hasv1_c, auto hask1_c, auto hask2_c, auto full_c) __attribute__((always_inline)) {
        constexpr bool HASV1 = decltype(hasv1_c)::value, HASK1 = decltype(hask1_c)::value, HASK2 = decltype(hask2_c)::value;
        constexpr bool FULL = decltype(full_c)::value;
        f32x16 st[2];
        uint32_t pk[16];
        qk_tile_pipe<D>(Ks, qf, st, ql, hh);
        softmax_tile<false, !FULL, DB>(st, pk, ot, m2, lsum, p.c, t * BN, n_keys - 1, hh);  // frozen max; a ragged tail is masked
        __builtin_amdgcn_sched_barrier(0);  // (requests and LDS writes go out where they are written, not where the scheduler likes them)
        regs_to_tile<D>(Vs, lane, rv);  // V(t) has landed when only K(t + 1) is still out
        if (HASV1) tile_to_regs<D, FULL>(Vg, (t + 1) * BN, n_keys, true, lane, offv, rv);
        __builtin_amdgcn_sched_barrier(0);
        pv_tile_pipe<D>(Vs, pk, ot, lane, hh);
        __builtin_amdgcn_sched_barrier(0);
        if (HASK1) regs_to_tile<D>(Ks, lane, rk);  // K(t + 1) has landed when only V(t + 1) is still out
        if (HASK2) tile_to_regs<D, FULL>(Kg, (t + 2) * BN, n_keys, false, lane, offk, rk);
        __builtin_amdgcn_sched_barrier(0);
    };
    using Y = std::true_type;
    using N_ = std::false_type;
    if (t_lo < t_hi) {
        tile_to_regs<D, false>(Kg, t_lo * BN, n_keys, false, lane, offk, rk);
        tile_to_regs<D, false>(Vg, t_lo * BN, n_keys, true, lane, offv, rv);
        __builtin_amdgcn_sched_barrier(0);
        regs_to_tile<D>(Ks, lane, rk);
        __builtin_amdgcn_sched_barrier(0);
        int t = t_lo;
        if (t + 2 < t_whole) {  // (the request for K(t + 1) is not behind a branch of its own: see above)
            tile_to_regs<D, true>(Kg, (t + 1) * BN, n_keys, false, lane, offk, rk);
            do {  // tiles t + 1 and t + 2 are whole and inside the range
                body(t, Y{}, Y{}, Y{}, Y{});
                ++t;
            } while (t + 2 < t_whole);
        } else if (t + 1 < t_hi) {
            tile_to_regs<D, false>(Kg, (t + 1) * BN, n_keys, false, lane, offk, rk);
        }
        const int left = t_hi - t;  // 1 .. 3 (t_hi <= t_whole + 1)
        if (left == 3) {
            body(t, Y{}, Y{}, Y{}, N_{});
            body(t + 1, Y{}, Y{}, N_{}, N_{});
            body(t + 2, N_{}, N_{}, N_{}, N_{});
        } else if (left == 2) {
            body(t, Y{}, Y{}, N_{}, N_{});
            body(t + 1, N_{}, N_{}, N_{}, N_{});
        } else {
            body(t, N_{}, N_{}, N_{}, N_{});
        }
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
