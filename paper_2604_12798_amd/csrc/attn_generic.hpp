// Generic bf16 attention kernel: any supported (d, block_m), all modes and ablation switches.
#pragma once
#include "common.hpp"

namespace {

// ---------------------------------------------------------------------------------------------
// Generic kernel: any supported (d, block_m); NW waves, one query block per workgroup, two
// workgroups per CU.  Tile k+1 streams into the other LDS buffer while tile k computes.
template <int D, int NW, int MODE>
__global__ __launch_bounds__(64 * NW, 2) void attn_fwd_kernel(const Params p) {
    using T = Tile<D>;
    constexpr int BM = 32 * NW;
    constexpr int NT = 64 * NW;
    constexpr int KK = D / 16;  // k-steps of Q K^T
    constexpr int DB = D / 32;  // 32-row blocks of O^T

    __shared__ __attribute__((aligned(16))) uint8_t smem[4 * T::BYTES];  // K[2], V[2]
    __shared__ int votes[2][NW];
    uint8_t* const Ks = smem;
    uint8_t* const Vs = smem + 2 * T::BYTES;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform: keep it in an SGPR
    const int ql = lane & 31;  // query column inside the wave
    const int hh = lane >> 5;  // which half of the k / row split this lane holds

    // ---- workgroup -> (b, h, i): heavy (late) query blocks first; all query heads of one KV
    // head, and the KV heads congruent mod 8, stay on one XCD (workgroup ids go round-robin
    // over the 8 XCDs) so their K/V tiles share that XCD's L2.
    const int g = p.Hq / p.Hkv;
    const int G = p.B * p.Hkv;
    int b, h, i;
    {
        const int id = blockIdx.x;
        if ((G & 7) == 0) {
            const int x = id & 7, y = id >> 3;
            const int per = p.Tr * g;
            const int kvl = y / per, rem = y - kvl * per;
            i = p.Tr - 1 - rem / g;
            const int kv = kvl * 8 + x;
            b = kv / p.Hkv;
            h = (kv - b * p.Hkv) * g + rem % g;
        } else {
            const int bh = id % (p.B * p.Hq);
            i = p.Tr - 1 - id / (p.B * p.Hq);
            b = bh / p.Hq;
            h = bh - b * p.Hq;
        }
    }
    const int hkv = h / g;
    const int N = p.N;
    const int row0 = i * BM;
    const int last_row = min(N, row0 + BM) - 1;
    const int a_lo = row0 / BN, a_hi = last_row / BN;
    const int j_hi = p.causal ? a_hi : p.Tc - 1;

    const uint16_t* Qg = p.Q + ((size_t)(b * p.Hq + h) * N) * D;
    const uint16_t* Kg = p.K + ((size_t)(b * p.Hkv + hkv) * N) * D;
    const uint16_t* Vg = p.V + ((size_t)(b * p.Hkv + hkv) * N) * D;

    // ---- Q fragments: B operand of S^T = K Q^T; lane holds Q[row0 + 32*wave + ql][16*kk + 8*hh .. +7]
    const int qrow = row0 + 32 * wave + ql;
    const int qrow_c = min(qrow, N - 1);
    const int limit = p.causal ? qrow_c : N - 1;  // last visible key of this lane's query
    bf16x8 qf[KK];
#pragma unroll
    for (int kk = 0; kk < KK; ++kk)
        qf[kk] = *reinterpret_cast<const bf16x8*>(Qg + (size_t)qrow_c * D + 16 * kk + 8 * hh);

    // ---- m-initialisation: m2 = c * max_j Q_i . Krepr_j over visible key blocks (raw scores here)
    float m2 = -INFINITY;
    if (!is_fa(MODE) && p.use_minit) {
        const uint16_t* Rg = p.Krepr + ((size_t)(b * p.Hkv + hkv) * p.Tc) * D;
        float mx = -INFINITY;
        const int n_sum_tiles = (j_hi + BN) / BN;
        // left operand: this lane's query row, or (block-wise ablation) the block's summary in every column,
        // which gives all rows of the block the same seed
        bf16x8 qm[KK];
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) qm[kk] = qf[kk];
        if (p.Qrepr) {
            const uint16_t* Qr = p.Qrepr + ((size_t)(b * p.Hq + h) * p.Tr + i) * D;
#pragma unroll
            for (int kk = 0; kk < KK; ++kk) qm[kk] = *reinterpret_cast<const bf16x8*>(Qr + 16 * kk + 8 * hh);
        }
        for (int ts = 0; ts < n_sum_tiles; ++ts) {
            __syncthreads();  // previous tile's readers are done
            load_tile<D, NW>(Rg, ts * BN, p.Tc, Ks, false, wave, lane);
            wait_vm0_and_sync();
            f32x16 st[2];
            qk_tile<D>(Ks, qm, st, ql, hh);
            mx = fmaxf(mx, tile_rowmax<true>(st, ts * BN, j_hi, hh));
        }
        m2 = xhalf_max(mx) * p.c;
        __syncthreads();
    }

    const Visit vis = make_visit<MODE>(p, a_lo, a_hi, j_hi);

    if (MODE == MODE_VSA && p.mask) {  // tiles this query block never visits
        uint8_t* mrow = p.mask + ((size_t)(b * p.Hq + h) * p.Tr + i) * p.Tc;
        for (int j = j_hi + 1 + tid; j < p.Tc; j += NT) mrow[j] = 2;
    }

    f32x16 ot[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db) ot[db] = f32x16{0};
    float lsum = 0.f;  // this lane's share of l (its 32 of the 64 keys of every tile)

    {
        const int j0 = vis.tile(0);
        load_tile<D, NW>(Kg, j0 * BN, N, Ks, false, wave, lane);
        load_tile<D, NW>(Vg, j0 * BN, N, Vs, true, wave, lane);
        wait_vm0_and_sync();
    }
    for (int k = 0; k < vis.total; ++k) {
        const int j = vis.tile(k);
        const int buf = k & 1;
        if (k + 1 < vis.total) {
            const int jn = vis.tile(k + 1);
            load_tile<D, NW>(Kg, jn * BN, N, Ks + (buf ^ 1) * T::BYTES, false, wave, lane);
            load_tile<D, NW>(Vg, jn * BN, N, Vs + (buf ^ 1) * T::BYTES, true, wave, lane);
        }
        const bool special = vis.special(k);
        const bool masked = (p.causal && j * BN + BN - 1 > row0) || (j + 1) * BN > N;
        f32x16 st[2];
        // the wave that issues MFMAs gets the issue slots first; a wave of the other workgroup on this
        // SIMD fills the gaps with its softmax
        __builtin_amdgcn_s_setprio(1);
        qk_tile_pipe<D>(Ks + buf * T::BYTES, qf, st, ql, hh);
        __builtin_amdgcn_s_setprio(0);
        bool keep = true;
        if (MODE == MODE_VSA) {
            // block vote: skip iff every row of the query block has m~ < m - threshold
            const float mx = masked ? tile_rowmax<true>(st, j * BN, limit, hh) : tile_rowmax<false>(st, 0, 0, hh);
            const float mt2 = xhalf_max(mx) * p.c;
            const bool row_keeps = (qrow < N) && (mt2 != -INFINITY) && !(mt2 < m2 - p.thr2);
            const bool wave_keeps = __builtin_amdgcn_ballot_w64(row_keeps) != 0;
            if (lane == 0) votes[buf][wave] = wave_keeps ? 1 : 0;
            __syncthreads();
            int any = 0;
#pragma unroll
            for (int w = 0; w < NW; ++w) any |= votes[buf][w];
            keep = any != 0;
            if (p.mask && tid == 0) p.mask[((size_t)(b * p.Hq + h) * p.Tr + i) * p.Tc + j] = keep ? 0 : 1;
            if (p.rowskip && keep) {  // row-level variant: a row that failed the test contributes nothing to a kept tile
#pragma unroll
                for (int t = 0; t < 2; ++t)
#pragma unroll
                    for (int r = 0; r < 16; ++r) st[t][r] = row_keeps ? st[t][r] : -INFINITY;
            }
        }
        if (keep) {
            uint32_t pk[16];
            if (special) {
                // (VSA takes the conditional-rescale form too; its tau2 is negative unless the variant asks for it,
                // and then only the branch over an all-ones rescale is left of it)
                constexpr bool LAZY = is_lazy(MODE) || MODE == MODE_VSA;
                constexpr int SE = softexp_every(MODE);
                if (masked) softmax_tile<true, true, DB, true, LAZY, SE>(st, pk, ot, m2, lsum, p.c, j * BN, limit, hh, p.tau2);
                else softmax_tile<true, false, DB, true, LAZY, SE>(st, pk, ot, m2, lsum, p.c, j * BN, limit, hh, p.tau2);
            } else {
                if (masked) softmax_tile<false, true, DB>(st, pk, ot, m2, lsum, p.c, j * BN, limit, hh);
                else softmax_tile<false, false, DB>(st, pk, ot, m2, lsum, p.c, j * BN, limit, hh);
            }
            __builtin_amdgcn_s_setprio(1);
            pv_tile_pipe<D>(Vs + buf * T::BYTES, pk, ot, lane, hh);
            __builtin_amdgcn_s_setprio(0);
        }
        wait_vm0_and_sync();
    }
    store_output<D>(p, ot, m2, lsum, b, h, qrow, hh);
}

}  // namespace
