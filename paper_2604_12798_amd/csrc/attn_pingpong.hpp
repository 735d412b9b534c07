// Ping-pong bf16 attention kernel for d = 128, block_m = 128: the kernel the headline workloads run on
// (Alg. 1 and the online-softmax baselines; Alg. 2 has a kernel of its own in attn_vsa.hpp).
#pragma once
#include "common.hpp"

namespace {

// ---------------------------------------------------------------------------------------------
// Ping-pong kernel for d = 128, block_m = 128, an even number of query heads per KV head.
// One workgroup = 8 waves = two groups of 4; group G handles query head 2*hp + G of the same KV
// head at the same query block, so both groups walk the same K/V tile sequence and every tile is
// fetched once for 256 query rows.  The two waves that share a SIMD belong to different groups
// and run half an interval apart: while one issues MFMAs (P.V of the previous tile, then Q.K^T of
// the current one) the other runs its softmax on the vector ALU.  One workgroup barrier per tile
// re-establishes the stagger and hands LDS ring slots over.  K/V tiles sit in a 4-deep LDS ring
// filled two tiles ahead.
constexpr int PP_STAGES = 4;
constexpr int PP_LDS_BYTES = 2 * PP_STAGES * Tile<128>::BYTES;

template <int MODE>
__global__ __launch_bounds__(512, 2) void attn_fwd_pp_kernel(const Params p) {
    constexpr int D = 128;
    using T = Tile<D>;
    constexpr int BM = 128, KK = D / 16, DB = D / 32, NWV = 8;
    extern __shared__ __attribute__((aligned(16))) uint8_t pp_smem[];
    uint8_t* const Ks = pp_smem;
    uint8_t* const Vs = pp_smem + PP_STAGES * T::BYTES;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform: keep it in an SGPR
    const int grp = wave >> 2;  // which query head of the pair
    const int w4 = wave & 3;    // 32-row slice of the query block
    const int ql = lane & 31;
    const int hh = lane >> 5;

    // Two ways to pair the groups (p.pair_blocks): 0 = two query heads of one KV head at the same query
    // block (needs an even number of heads per KV head); 1 = the same head at two adjacent query blocks,
    // a 256-row super-block.  In the second form the workgroup-level geometry below spans both blocks,
    // so the visit list is the union of what the two blocks need: the local set covers both diagonals,
    // and under a causal mask the first group finds the second group's diagonal tiles fully masked
    // (exp gives 0; two wasted tiles per workgroup).  Only h, the rows and the m-init range are per group.
    const int pb = p.pair_blocks;
    const int g = p.Hq / p.Hkv, gp = pb ? g : g >> 1;  // units (heads or head pairs) per KV head
    const int Ti = pb ? (p.Tr + 1) >> 1 : p.Tr;        // query blocks or super-blocks
    const int G = p.B * p.Hkv;
    // Work items (one query block or super-block of one head or head pair).  persist = 0: one item per
    // workgroup, item = workgroup id.  persist = P > 0: P workgroups (one per CU) each take every P-th item of
    // the list, in boustrophedon order so that the early (long) and late (short) items even out.
    const int n_items = G * gp * Ti;
    for (int round = 0;; ++round) {
    int b, hkv, hp, i;
    {
        int id = blockIdx.x;
        if (p.persist) {
            const int xs = (G & 7) == 0 ? 8 : 1;            // lists: one per XCD, or one for the whole chip
            const int pw = p.persist / xs, len = n_items / xs;
            const int c = blockIdx.x / xs;
            const int y = round * pw + ((round & 1) ? pw - 1 - c : c);
            if (y >= len) break;
            id = (blockIdx.x % xs) + xs * y;
        }
        if ((G & 7) == 0) {
            const int x = id & 7, y = id >> 3;
            const int per = Ti * gp;
            const int kvl = y / per, rem = y - kvl * per;
            i = Ti - 1 - rem / gp;
            hp = rem % gp;
            const int kv = kvl * 8 + x;
            b = kv / p.Hkv;
            hkv = kv - b * p.Hkv;
        } else {
            const int per = G * gp;
            i = Ti - 1 - id / per;
            const int rem = id % per;
            hp = rem % gp;
            const int kv = rem / gp;
            b = kv / p.Hkv;
            hkv = kv - b * p.Hkv;
        }
    }
    const int h = pb ? hkv * g + hp : hkv * g + 2 * hp + grp;
    const int N = p.N;
    const int row0 = (pb ? 2 * i : i) * BM;                      // first row of the workgroup
    const int last_row = min(N, row0 + (pb ? 2 * BM : BM)) - 1;  // last row of the workgroup
    const int a_lo = row0 / BN, a_hi = last_row / BN;
    const int j_hi = p.causal ? a_hi : p.Tc - 1;
    const int row0_g = row0 + (pb ? grp * BM : 0);               // first row of this group
    // last key block this group's rows can see (a group past the end of the sequence mirrors row N - 1)
    const int j_hi_g = p.causal ? (min(N, row0_g + BM) - 1) / BN : p.Tc - 1;

    const uint16_t* Qg = p.Q + ((size_t)(b * p.Hq + h) * N) * D;
    const uint16_t* Kg = p.K + ((size_t)(b * p.Hkv + hkv) * N) * D;
    const uint16_t* Vg = p.V + ((size_t)(b * p.Hkv + hkv) * N) * D;

    const int qrow = row0_g + 32 * w4 + ql;
    const int qrow_c = min(qrow, N - 1);
    const int limit = p.causal ? qrow_c : N - 1;
    bf16x8 qf[KK];
#pragma unroll
    for (int kk = 0; kk < KK; ++kk)
        qf[kk] = *reinterpret_cast<const bf16x8*>(Qg + (size_t)qrow_c * D + 16 * kk + 8 * hh);

    float m2 = -INFINITY;

    Visit vis = make_visit<MODE>(p, a_lo, a_hi, j_hi);
    const int nv = vis.total;

    f32x16 ot[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db) ot[db] = f32x16{0};
    float lsum = 0.f;
    f32x16 st[2];
    uint32_t pk[16];
    bool pv_pending = false;  // pk holds a tile whose P.V has not been accumulated yet

    // ---- LDS-direct tile loads.  Per-lane byte offsets inside a tile are fixed for the whole kernel
    // (rows 4*(8u + wave) + lane/16, swizzled chunk), so a full tile costs one scalar base per matrix
    // and four load instructions per wave.  A ragged last tile clamps its rows and takes the slow path.
    uint32_t offK[2], offV[2];
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        const int r = 4 * (u * NWV + wave) + (lane >> 4), cp = lane & 15;
        offK[u] = r * T::ROWB + ((cp ^ (r & 15)) << 4);
        offV[u] = r * T::ROWB + ((cp ^ ((r & 3) << 2)) << 4);
    }
    // LDS byte address of this wave's first 1 KiB piece of ring slot 0 (K ring; the V ring sits
    // PP_STAGES tiles further), as an integer: address arithmetic below stays on the scalar unit
    const uint32_t lds_k0 = __builtin_amdgcn_readfirstlane(
        (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint8_t*)(Ks + wave * 1024));
    auto uniform64 = [&](const uint16_t* ptr) __attribute__((always_inline)) {  // tell the compiler the pointer is wave-uniform
        const uint64_t b64 = (uint64_t)(uintptr_t)ptr;
        // (readfirstlane returns a signed int: go through uint32_t so the low half is not sign-extended)
        const uint32_t b_lo = (uint32_t)__builtin_amdgcn_readfirstlane((uint32_t)b64);
        const uint32_t b_hi = (uint32_t)__builtin_amdgcn_readfirstlane((uint32_t)(b64 >> 32));
        return ((uint64_t)b_hi << 32) | (uint64_t)b_lo;
    };
    auto issue = [&](int k) __attribute__((always_inline)) {  // tile of visit k -> ring slot k & 3 (this wave's 2 + 2 instructions)
        const int j = vis.tile(k);
        if (j * BN + BN <= N) {
            // one asm block for the four loads: M0 (the LDS base of an LDS-direct load) is saved once and
            // restored at the end; pieces u = 0, 1 of a tile are 8 KiB apart in LDS
            const uint64_t kb = uniform64(Kg + (size_t)j * BN * D), vb = uniform64(Vg + (size_t)j * BN * D);
            const uint32_t lk0 = lds_k0 + (k & 3) * T::BYTES, lk1 = lk0 + NWV * 1024;
            const uint32_t lv0 = lk0 + PP_STAGES * T::BYTES, lv1 = lv0 + NWV * 1024;
            uint32_t m0_save;
            asm volatile(
                "s_mov_b32 %0, m0\n\t"
                "s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %5, %9\n\t"
                "s_mov_b32 m0, %3\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %7, %10\n\t"
                "s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %6, %9\n\t"
                "s_mov_b32 m0, %4\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %8, %10\n\t"
                "s_mov_b32 m0, %0"
                : "=&s"(m0_save)
                : "s"(lk0), "s"(lk1), "s"(lv0), "s"(lv1), "v"(offK[0]), "v"(offK[1]), "v"(offV[0]), "v"(offV[1]), "s"(kb),
                  "s"(vb)
                : "memory");
        } else {
            load_tile<D, NWV>(Kg, j * BN, N, Ks + (k & 3) * T::BYTES, false, wave, lane);
            load_tile<D, NWV>(Vg, j * BN, N, Vs + (k & 3) * T::BYTES, true, wave, lane);
        }
    };
    auto tile_masked = [&](int j) __attribute__((always_inline)) { return (p.causal && j * BN + BN - 1 > row0) || (j + 1) * BN > N; };

    // ---- fragment loaders.  ld_v: the 4 V^T fragments (db = 0..3) of key chunk c; ld_k: the 4 K
    // fragments (kk, t) = (2*kk2, 0), (2*kk2, 1), (2*kk2+1, 0), (2*kk2+1, 1).
    const int kbase = T::k_base(ql, hh), vbase = T::v_base(lane, hh);
    auto ld_v = [&](bf16x8* f, const uint8_t* vt, int c) __attribute__((always_inline)) {
#pragma unroll
        for (int db = 0; db < DB; ++db) {
            const uint8_t* a = vt + (vbase ^ (db << 6)) + 16 * c * T::ROWB;
            const s16x4 v0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(a));
            const s16x4 v1 =
                __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(a + 8 * T::ROWB));
            const u32x2 a0 = __builtin_bit_cast(u32x2, v0), a1 = __builtin_bit_cast(u32x2, v1);
            const u32x4 aw = {a0[0], a0[1], a1[0], a1[1]};
            f[db] = __builtin_bit_cast(bf16x8, aw);
        }
    };
    auto ld_k = [&](bf16x8* f, const uint8_t* kt, int kk2) __attribute__((always_inline)) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int kk = 2 * kk2 + (e >> 1), t = e & 1;
            f[e] = *reinterpret_cast<const bf16x8*>(kt + (kbase ^ (kk << 5)) + t * 32 * T::ROWB);
        }
    };
    auto pv4 = [&](const bf16x8* f, int c) __attribute__((always_inline)) {
        const u32x4 pw = {pk[4 * c], pk[4 * c + 1], pk[4 * c + 2], pk[4 * c + 3]};
        const bf16x8 pf = __builtin_bit_cast(bf16x8, pw);
#pragma unroll
        for (int db = 0; db < DB; ++db) ot[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f[db], pf, ot[db], 0, 0, 0);
    };
    auto qk4 = [&](const bf16x8* f, int kk2) __attribute__((always_inline)) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int kk = 2 * kk2 + (e >> 1), t = e & 1;
            st[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f[e], qf[kk], st[t], 0, 0, 0);
        }
    };
    bf16x8 fa[4], fb[4];  // fragment double buffer of the matrix phase

    // Matrix phase of visit k in the steady state: P.V of visit k-1 (its chunk-0 fragments are already
    // in fa, fetched at the end of the vector phase), then Q.K^T of visit k.  Fragments for the next
    // four MFMAs are read from LDS while the current four issue.  Nothing else is on this path.
    auto matrix_phase_full = [&](int k) __attribute__((always_inline)) {
        const uint8_t* vt = Vs + ((k - 1) & 3) * T::BYTES;
        const uint8_t* kt = Ks + (k & 3) * T::BYTES;
        if (!is_fa(MODE)) __builtin_amdgcn_s_setprio(1);
        else __builtin_amdgcn_s_setprio(0);  // (also keeps the phase a scheduling region of its own)
        st[0] = f32x16{0};
        st[1] = f32x16{0};
        ld_v(fb, vt, 1); pv4(fa, 0);
        ld_v(fa, vt, 2); pv4(fb, 1);
        ld_v(fb, vt, 3); pv4(fa, 2);
        ld_k(fa, kt, 0); pv4(fb, 3);
        ld_k(fb, kt, 1); qk4(fa, 0);
        ld_k(fa, kt, 2); qk4(fb, 1);
        ld_k(fb, kt, 3); qk4(fa, 2);
        qk4(fb, 3);
#pragma unroll
        for (int gq = 0; gq < 3; ++gq)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);  // 2 LDS reads
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // 1 MFMA
            }
#pragma unroll
        for (int gq = 0; gq < 4; ++gq)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            }
        __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);
        __builtin_amdgcn_s_setprio(0);
    };
    // Matrix phase without a pending P.V (first visit, or the previous tile was skipped): Q.K^T only.
    auto matrix_phase_qk = [&](int k) __attribute__((always_inline)) {
        if (!is_fa(MODE)) __builtin_amdgcn_s_setprio(1);
        else __builtin_amdgcn_s_setprio(0);  // (also keeps the phase a scheduling region of its own)
        qk_tile<D>(Ks + (k & 3) * T::BYTES, qf, st, ql, hh);
        __builtin_amdgcn_s_setprio(0);
    };
    // Start of every vector phase: this wave's share of the tile that matrix phases will reach two
    // intervals from now goes into the ring slot whose last readers finished before the previous
    // barrier, and the share issued one interval earlier is waited for, so that the barrier ending this
    // interval publishes it one full interval before its first use.  Group 1's vector phase kv sits
    // in the same interval as group 0's kv + 1, hence the "+ grp".
    auto fetch_ahead = [&](int k) __attribute__((always_inline)) {
        const int ki = k + 2 + grp;
        if (ki < nv) {
            issue(ki);
            __builtin_amdgcn_s_waitcnt(0x0F74);  // vmcnt(4): all but the 4 loads just issued have landed
        } else {
            __builtin_amdgcn_s_waitcnt(0x0F70);
        }
    };
    // vector phase of visit k: softmax (or the skip decision) on the scores the matrix phase left in st.
    // SPECIAL / FAST / FIRST are compile-time so that every loop below has exactly one softmax body:
    // FAST = the tile needs no masking; FIRST = nothing accumulated yet (no rescale).
    auto vector_phase = [&](int k, auto special_c, auto fast_c, auto first_c) __attribute__((always_inline)) {
        constexpr bool SPECIAL = decltype(special_c)::value, FAST = decltype(fast_c)::value,
                       FIRST = decltype(first_c)::value;
        const int j = vis.tile(k);
        // Which wave of a SIMD gets the issue slots first decides how well MFMA and vector work overlap:
        // measured, the frozen-max modes do best with the matrix phase on top (its one issue per 32 cycles
        // is never delayed), the exact-max baseline, whose vector phase is the longer one, with the
        // vector phase on top.
        if (is_fa(MODE)) __builtin_amdgcn_s_setprio(2);
        fetch_ahead(k);
        pv_pending = true;
        {
            if (FAST)
                softmax_tile<SPECIAL, false, DB, !FIRST, is_lazy(MODE), softexp_every(MODE)>(st, pk, ot, m2, lsum, p.c, j * BN,
                                                                                             limit, hh, p.tau2);
            else
                softmax_tile<SPECIAL, true, DB, !FIRST, is_lazy(MODE), softexp_every(MODE)>(
                    st, pk, ot, m2, lsum, p.c, j * BN, tile_masked(j) ? limit : 0x3fffffff, hh, p.tau2);
            ld_v(fa, Vs + (k & 3) * T::BYTES, 0);  // first fragments of the coming P.V, in flight over the barrier
        }
        if (is_fa(MODE)) __builtin_amdgcn_s_setprio(0);
    };
    using std::false_type;
    using std::true_type;

    // ---- prologue: the first two tiles are requested before the m-initialisation, which stages its summary
    // tiles in the other half of the ring (slots 2 and 3 of the K and of the V ring: four tiles = 256 key
    // blocks per batch), so that their latency is not paid again after it
    issue(0);
    if (nv > 1) issue(1);
    if (!is_fa(MODE) && p.use_minit) {
        const uint16_t* Rg = p.Krepr + ((size_t)(b * p.Hkv + hkv) * p.Tc) * D;
        float mx = -INFINITY;
        const int n_sum_tiles = (j_hi + BN) / BN;
        auto stage = [&](int u) __attribute__((always_inline)) { return pp_smem + ((u & 1) + 2 + (u >> 1) * PP_STAGES) * T::BYTES; };
        for (int t0 = 0; t0 < n_sum_tiles; t0 += 4) {
            const int nb = min(4, n_sum_tiles - t0);
            if (t0) __syncthreads();  // the previous batch's readers are done
            for (int u = 0; u < nb; ++u) load_tile<D, NWV>(Rg, (t0 + u) * BN, p.Tc, stage(u), false, wave, lane);
            wait_vm0_and_sync();
            for (int u = 0; u < nb; ++u) {
                qk_tile<D>(stage(u), qf, st, ql, hh);
                mx = fmaxf(mx, tile_rowmax<true>(st, (t0 + u) * BN, j_hi_g, hh));
            }
        }
        m2 = xhalf_max(mx) * p.c;
        __syncthreads();
    }
    // visits 0 and 1 resident, group 1's share of visit 2 in flight
    if (grp == 1 && nv > 2) {
        issue(2);
        __builtin_amdgcn_s_waitcnt(0x0F74);
    } else {
        __builtin_amdgcn_s_waitcnt(0x0F70);
    }
    __syncthreads();

    // Visits split into: visit 0 (no P.V pending, nothing to rescale); the remaining sink/local visits
    // of VFA (exact-max update); a run of unmasked visits that all take one path (frozen max for
    // VFA, exact-max for FA); and the trailing
    // visits that may need masking (tiles on the diagonal or past the end of a ragged sequence).
    constexpr bool TAIL_SPECIAL = is_fa(MODE);
    const int n_lead = is_fa(MODE) ? 0 : vis.n_special;  // visits [0, n_lead) are sink/local
    int k_fast_end = max(n_lead, 1);
    {
        int j_masked = p.causal ? a_lo : p.Tc;  // first tile index that needs masking
        if (N % BN) j_masked = min(j_masked, p.Tc - 1);
        int cnt = max(0, j_masked - vis.n1);  // visits of the ascending tail with tile index < j_masked
        if (vis.n2 > 0) cnt -= max(0, min(j_masked, vis.s2 + vis.n2) - vis.s2);
        k_fast_end = max(k_fast_end, min(nv, n_lead + cnt));
    }
    auto drain = [&]() __attribute__((always_inline)) {  // the P.V of the last visit
        if (pv_pending) {
            const uint8_t* vt = Vs + ((nv - 1) & 3) * T::BYTES;
            pv4(fa, 0);
#pragma unroll
            for (int c = 1; c < 4; ++c) {
                ld_v(fb, vt, c);
                pv4(fb, c);
            }
        }
    };
    // k may equal nv for group 1 (the matrix phase that follows its last vector phase): the Q.K^T half
    // then runs on whatever the ring slot holds and its scores are never used; only the P.V counts.
    auto matrix_any = [&](int k) __attribute__((always_inline)) {
        if (pv_pending) matrix_phase_full(k);
        else matrix_phase_qk(k);
    };
    // One interval = the stretch between two workgroup barriers.  Group 0 runs matrix phase kv and then
    // vector phase kv; group 1 runs vector phase kv and then matrix phase kv + 1.  So each interval
    // starts with one group on the matrix cores and the other on the vector ALU, but neither waits for
    // the other inside the interval: whichever group has MFMAs ready keeps the matrix pipe fed.
    // The whole loop nest is instantiated once per group (GRP is a compile-time constant) so that each
    // copy is straight-line code for the register allocator.
    auto run_group = [&](auto grp_c) __attribute__((always_inline)) {
        constexpr int GRP = decltype(grp_c)::value;
        auto interval = [&](int kv, auto special_c, auto fast_c, auto first_c, auto steady_c) __attribute__((always_inline)) {
            constexpr bool STEADY = decltype(steady_c)::value;
            if (GRP == 0) {
                if (STEADY) matrix_phase_full(kv);
                else matrix_any(kv);
            }
            __builtin_amdgcn_sched_barrier(0);  // keep the two phases apart in the instruction stream
            vector_phase(kv, special_c, fast_c, first_c);
            __builtin_amdgcn_sched_barrier(0);
            if (GRP == 1) {
                if (STEADY) matrix_phase_full(kv + 1);
                else matrix_any(kv + 1);
            }
            __builtin_amdgcn_s_barrier();
        };
        if (GRP == 1) {  // group 1 starts half an interval late
            matrix_phase_qk(0);
            __builtin_amdgcn_s_barrier();
        }
        if (is_fa(MODE) || n_lead > 0) interval(0, true_type{}, false_type{}, true_type{}, false_type{});
        else interval(0, false_type{}, false_type{}, true_type{}, false_type{});
        int k = 1;
        for (; k < min(n_lead, nv); ++k) interval(k, true_type{}, false_type{}, false_type{}, false_type{});
        for (; k < k_fast_end; ++k)
            interval(k, std::integral_constant<bool, TAIL_SPECIAL>{}, true_type{}, false_type{}, true_type{});
        for (; k < nv; ++k)
            interval(k, std::integral_constant<bool, TAIL_SPECIAL>{}, false_type{}, false_type{}, false_type{});
        if (GRP == 0) {
            drain();
            __builtin_amdgcn_s_barrier();
        }
        store_output<D>(p, ot, m2, lsum, b, h, qrow, hh);  // inside the per-group copy: nothing merges after it
    };
    {
        if (grp == 0) run_group(std::integral_constant<int, 0>{});
        else run_group(std::integral_constant<int, 1>{});
    }
    if (!p.persist) break;
    __syncthreads();  // the next item's prologue overwrites the ring
    }
}

}  // namespace
