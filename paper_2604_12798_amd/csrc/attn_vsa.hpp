// VSA (Alg. 2) on the ping-pong structure for d = 128, block_m = 128: the kernel vsa_attn_fwd runs on.
#pragma once
#include "common.hpp"

namespace {

// ---------------------------------------------------------------------------------------------
// Same workgroup shape as attn_fwd_pp_kernel: 8 waves = two groups of 4, group G on query head 2 hp + G of one KV
// head (or on the second of two adjacent query blocks of one head), the two waves of a SIMD in different groups and
// half an interval apart, one workgroup barrier per tile.  What differs is what Alg. 2 needs: a tile's fate is one
// decision of all four waves of a group, and a skipped tile must cost neither a V tile nor an exponential.  So a tile
// passes through three stages, one interval apart, and nothing waits for a vote:
//   interval y      Q.K^T of visit y into one of TWO score buffers, row max, this wave's vote into LDS
//   (barrier: the votes of visit y are visible)
//   interval y + 1  the four votes are read: the tile is dropped, or its softmax runs (from the other score buffer,
//                   while Q.K^T of visit y + 1 fills the first) and its V tile is requested
//   interval y + 2  P.V of visit y
// A skipped tile is a K tile, 16 MFMAs and about 50 vector instructions per wave; it never touches V.  The exact-max
// update of a sink / local tile is split: the new max (the row max is known from the vote) is adopted as soon as the
// decision is read, before the next vote is cast with it, as Alg. 2 orders it; the rescale of l and O by
// exp(m_old - m_new) follows with the tile's softmax.
//
// LDS: K ring of 6 tiles filled five visits ahead (a skipped tile takes half the time of a kept one, so K has to run
// further ahead of the matrix phases than in the dense kernels), V ring of 2.  Group 0's waves fetch the K tiles,
// group 1's the V tiles (only of tiles that either group keeps), so each wave has one kind of load in flight and its
// own count to wait on.
//
// A step (one interval of one group) exists in two forms.  The general one decides per visit whether it is an
// exact-max one, whether its tile needs a mask or is a ragged last tile, and whether it lies inside the visit list at
// all.  The fast one is for steps whose visits (y - 2 .. y + 5) are all "plain" - frozen max, no mask, whole tile -
// which is nearly every step of a long sequence: those questions are answered at compile time and the scalar
// bookkeeping per step halves.  A wave issues about one instruction per five cycles whatever its kind, so scalar
// instructions cost as much as the others here.
// The kernel needs 233 of the 256 vector registers in its steady loops, and whether the register allocator finds that
// fit depends on details of the formulation and on the scheduler's pressure tracking: this file is compiled in a
// translation unit of its own (vsa_pp.hip) with the option that makes the fast loops free of scratch accesses.  A
// scratch reload waits for vmcnt(0), which also drains the tile prefetches, so a spill inside a steady loop costs a
// factor, not a few percent; check the generated code after touching the step body.
constexpr int VSA_DK = 6, VSA_DV = 2, VSA_AHEAD = 5;
constexpr int VSA_LDS_BYTES = (VSA_DK + VSA_DV) * Tile<128>::BYTES;

__global__ __launch_bounds__(512, 2) void attn_vsa_pp_kernel(const Params p) {
    constexpr int D = 128;
    using T = Tile<D>;
    constexpr int BM = 128, KK = D / 16, DB = D / 32, NWV = 8;
    extern __shared__ __attribute__((aligned(16))) uint8_t vsa_smem[];
    __shared__ int votes[2][2][4];  // [visit parity][group][wave of the group]
    uint8_t* const Ks = vsa_smem;
    uint8_t* const Vs = vsa_smem + VSA_DK * T::BYTES;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int grp = wave >> 2;
    const int w4 = wave & 3;
    const int ql = lane & 31;
    const int hh = lane >> 5;

    // work items as in attn_fwd_pp_kernel: head pairs (pb = 0) or pairs of adjacent query blocks (pb = 1), longest
    // first, one list per XCD when the KV heads divide evenly; persistent workgroups take fixed boustrophedon shares
    const int pb = p.pair_blocks;
    const int g = p.Hq / p.Hkv, gp = pb ? g : g >> 1;
    const int Ti = pb ? (p.Tr + 1) >> 1 : p.Tr;
    const int G = p.B * p.Hkv;
    const int n_items = G * gp * Ti;
    for (int round = 0;; ++round) {
    int b, hkv, hp, i;
    {
        int id = blockIdx.x;
        if (p.persist) {
            const int xs = (G & 7) == 0 ? 8 : 1;
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
    const int row0 = (pb ? 2 * i : i) * BM;
    const int last_row = min(N, row0 + (pb ? 2 * BM : BM)) - 1;
    const int a_lo = row0 / BN, a_hi = last_row / BN;
    const int j_hi = p.causal ? a_hi : p.Tc - 1;
    const int row0_g = row0 + (pb ? grp * BM : 0);
    const int j_hi_g = p.causal ? (min(N, row0_g + BM) - 1) / BN : p.Tc - 1;  // last key block this group's rows can see

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

    Visit vis = make_visit<MODE_VSA>(p, a_lo, a_hi, j_hi);
    if (pb) {
        // block pairs (causal, at most one local block per query block): the second block's local tiles come first
        // (exact-max for group 1, invisible to group 0), then the first block's (exact-max for group 0, ordinary frozen
        // tiles for group 1, whose max is final by then): each group meets its own tiles in Alg. 2's order
        const int lo_b = (row0 + BM) / BN;
        vis.n2b = vis.n2 > 0 ? max(0, vis.s2 + vis.n2 - max(vis.s2, lo_b)) : 0;
    }
    const int nv = vis.total;
    const int n_lead = vis.n_special;
    uint8_t* mrow = nullptr;
    const int i_blk = pb ? 2 * i + grp : i;
    if (p.mask && i_blk < p.Tr) {
        mrow = p.mask + ((size_t)(b * p.Hq + h) * p.Tr + i_blk) * p.Tc;
        for (int j = j_hi_g + 1 + (tid & 255); j < p.Tc; j += 256) mrow[j] = 2;
    }
    // is visit k an exact-max one for this group?  (block pairs: a local tile is, only for the group whose block it belongs to)
    auto own_special = [&](int k) __attribute__((always_inline)) {
        return k < n_lead && (!pb || k < vis.n1 || ((k - vis.n1 < vis.n2b) == (grp == 1)));
    };
    // first key block that needs a mask: the one holding column row0 + 1 under a causal mask, else a ragged last one
    const int j_mask = min(p.causal ? (row0 + 1) / BN : p.Tc, N / BN);
    auto tile_masked = [&](int j) __attribute__((always_inline)) { return j >= j_mask; };
    // "plain" visits [n_lead, k_plain): frozen max, no mask, whole tile.  The visits behind the sink / local ones walk
    // the remaining tiles in ascending order, so the plain ones are those of them with a tile index below j_mask
    int k_plain;
    {
        int cnt = max(0, j_mask - vis.n1);                                                      // such tiles below j_mask ...
        if (vis.n2 > 0) cnt -= max(0, min(j_mask, vis.s2 + vis.n2) - max(vis.s2, vis.n1));     // ... that are not local ones
        k_plain = min(vis.total, n_lead + max(cnt, 0));
    }

    // vis.tile(k) for a visit behind the sink / local ones (k >= n_lead): the remaining tiles in ascending order
    auto tile_plain = [&](int k) __attribute__((always_inline)) {
        const int t = k - vis.n2;
        return (vis.n2 > 0 && t >= vis.s2) ? t + vis.n2 : t;
    };
    // ---- tile loads: a wave of a group moves pieces 4 u + w4 (u = 0..3; a piece = 4 rows = 1 KiB) of its group's kind
    // of tile.  The row swizzles repeat every 16 rows, so the four pieces share one per-lane offset and differ by
    // 4 KiB in the global base and in the LDS base.
    const uint32_t lds0 = __builtin_amdgcn_readfirstlane(
        (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint8_t*)(vsa_smem + w4 * 1024));
    auto uniform64 = [&](const uint16_t* ptr) __attribute__((always_inline)) {
        const uint64_t b64 = (uint64_t)(uintptr_t)ptr;
        const uint32_t b_lo = (uint32_t)__builtin_amdgcn_readfirstlane((uint32_t)b64);
        const uint32_t b_hi = (uint32_t)__builtin_amdgcn_readfirstlane((uint32_t)(b64 >> 32));
        return ((uint64_t)b_hi << 32) | (uint64_t)b_lo;
    };
    // tile j of K (group 0) or V (group 1) into ring slot `slot` of that ring: this wave's four pieces
    auto issue_tile = [&](int j, int slot, auto fast_c) __attribute__((always_inline)) {
        constexpr bool FAST = decltype(fast_c)::value;
        const uint16_t* src = (grp == 0 ? Kg : Vg) + (size_t)j * BN * D;
        if (FAST || __builtin_expect(j * BN + BN <= N, 1)) {
            // the per-lane offset (row 4 w4 + lane / 16 of a piece, swizzled chunk) is recomputed from the lane number
            // at every request: eight vector instructions, against a register held for the whole kernel
            const int ln = __builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
            const int r0l = 4 * w4 + (ln >> 4), cp = ln & 15;
            const uint32_t off_ld = grp == 0 ? (uint32_t)(r0l * T::ROWB + ((cp ^ (r0l & 15)) << 4))
                                             : (uint32_t)(r0l * T::ROWB + ((cp ^ ((r0l & 3) << 2)) << 4));
            const uint64_t g0 = uniform64(src), g1 = g0 + 4096, g2 = g0 + 8192, g3 = g0 + 12288;
            const uint32_t l0 = lds0 + ((grp == 0 ? 0 : VSA_DK) + slot) * T::BYTES, l1 = l0 + 4096, l2 = l0 + 8192, l3 = l0 + 12288;
            uint32_t m0_save;  // M0 carries the LDS base of an LDS-direct load; the compiler's own value is put back at the end
            asm volatile(
                "s_mov_b32 %0, m0\n\t"
                "s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %5, %6\n\t"
                "s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %5, %7\n\t"
                "s_mov_b32 m0, %3\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %5, %8\n\t"
                "s_mov_b32 m0, %4\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %5, %9\n\t"
                "s_mov_b32 m0, %0"
                : "=&s"(m0_save)
                : "s"(l0), "s"(l1), "s"(l2), "s"(l3), "v"(off_ld), "s"(g0), "s"(g1), "s"(g2), "s"(g3)
                : "memory");
        } else {  // ragged last tile: rows clamped, the generic mover (same four load instructions per wave)
            load_tile<D, 4>(grp == 0 ? Kg : Vg, j * BN, N, (grp == 0 ? Ks : Vs) + slot * T::BYTES, grp != 0, w4, lane);
        }
    };

    // ---- fragments (as in the dense kernel: four in flight, fragment i + 4 requested behind the MFMA that used i)
    int kb = T::k_base(ql, hh), vb = T::v_base(lane, hh);
    bf16x8 fr[4];
    f32x16 ot[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db) ot[db] = f32x16{0};
    f32x16 sa[2], sb[2];  // the two score buffers: visit y computes into buffer y & 1
    uint32_t pk[16];      // exp(S - m) of the last kept visit, bf16 pairs
    float m2 = -INFINITY, lsum = 0.f;
    float mt = -INFINITY;     // row max (log2 units) of the tile last voted on
    float m_bef = -INFINITY;  // the max before the last adopted exact-max tile (for its rescale)

    auto qk = [&](f32x16* st, int slot) __attribute__((always_inline)) {
        const uint8_t* kt = Ks + slot * T::BYTES;
        asm volatile("" : "+v"(kb));
        auto ldk1 = [&](int f) __attribute__((always_inline)) {  // fragment f = (k-step f / 2, key half f % 2)
            return *reinterpret_cast<const bf16x8*>(kt + (kb ^ ((f >> 1) << 5)) + (f & 1) * 32 * T::ROWB);
        };
#pragma unroll
        for (int f = 0; f < 4; ++f) fr[f] = ldk1(f);
#pragma unroll
        for (int f = 0; f < 16; ++f) {
            st[f & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[f & 3], qf[f >> 1], f < 2 ? f32x16{0} : st[f & 1], 0, 0, 0);
            if (f + 4 < 16) fr[f & 3] = ldk1(f + 4);
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    auto pv = [&](int slot) __attribute__((always_inline)) {  // O^T += V^T P^T with the tile in V ring slot `slot`
        const uint8_t* vt = Vs + slot * T::BYTES;
        asm volatile("" : "+v"(vb));
        auto ldv1 = [&](int c, int db) __attribute__((always_inline)) {
            const uint8_t* a = vt + (vb ^ (db << 6)) + 16 * c * T::ROWB;
            const s16x4 v0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(a));
            const s16x4 v1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(a + 8 * T::ROWB));
            const u32x2 a0 = __builtin_bit_cast(u32x2, v0), a1 = __builtin_bit_cast(u32x2, v1);
            const u32x4 aw = {a0[0], a0[1], a1[0], a1[1]};
            return __builtin_bit_cast(bf16x8, aw);
        };
#pragma unroll
        for (int db = 0; db < DB; ++db) fr[db] = ldv1(0, db);
#pragma unroll
        for (int f = 0; f < 16; ++f) {
            const int c = f >> 2, db = f & 3;
            const u32x4 pw = {pk[4 * c], pk[4 * c + 1], pk[4 * c + 2], pk[4 * c + 3]};
            ot[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[db], __builtin_bit_cast(bf16x8, pw), ot[db], 0, 0, 0);
            if (c < 3) fr[db] = ldv1(c + 1, db);
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    // this wave's say on "skip the tile of visit k" (scores in st), with the max as it stands after visit k - 1
    auto vote = [&](const f32x16* st, int k, auto fast_c) __attribute__((always_inline)) {
        constexpr bool FAST = decltype(fast_c)::value;
        const int j = FAST ? 0 : vis.tile(k);
        const float mx = !FAST && __builtin_expect(tile_masked(j), 0) ? tile_rowmax<true>(st, j * BN, limit, hh) : tile_rowmax<false>(st, 0, 0, hh);
        mt = xhalf_max(mx) * p.c;
        const bool row_keeps = (qrow < N) && (mt != -INFINITY) && !(mt < m2 - p.thr2);
        const bool wave_keeps = __builtin_amdgcn_ballot_w64(row_keeps) != 0;
        if (lane == 0) votes[k & 1][grp][w4] = wave_keeps ? 1 : 0;
        __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0): the vote is in LDS before this wave reaches the next barrier
    };
    // the votes of visit k, a barrier old: bit 0 = this group keeps the tile, bit 1 = either group does (V is needed)
    auto read_votes = [&](int k) __attribute__((always_inline)) {
        const int* v = &votes[k & 1][0][0];
        const int mine = v[4 * grp] | v[4 * grp + 1] | v[4 * grp + 2] | v[4 * grp + 3];
        const int other = v[4 * (grp ^ 1)] | v[4 * (grp ^ 1) + 1] | v[4 * (grp ^ 1) + 2] | v[4 * (grp ^ 1) + 3];
        return __builtin_amdgcn_readfirstlane((mine ? 1 : 0) | ((mine | other) ? 2 : 0));
    };
    // visit k has been decided: write its mask byte, and for a kept exact-max tile adopt the new max
    auto adopt = [&](int k, bool keep, auto fast_c) __attribute__((always_inline)) {
        constexpr bool FAST = decltype(fast_c)::value;
        const int j = FAST ? tile_plain(k) : vis.tile(k);
        if (mrow && j <= j_hi_g && (tid & 255) == 0) mrow[j] = keep ? 0 : 1;  // (a tile past j_hi_g is the other block's)
        if (!FAST && __builtin_expect(keep && own_special(k), 0)) {
            m_bef = m2;
            m2 = fmaxf(m2, mt);
        }
    };
    // softmax of kept visit k from its score buffer into pk; l and (for an exact-max tile) the rescale of l and O
    auto softmax = [&](f32x16* st, int k, auto fast_c) __attribute__((always_inline)) {
        constexpr bool FAST = decltype(fast_c)::value;
        const int j = FAST ? 0 : vis.tile(k);
        if (!FAST && __builtin_expect(own_special(k), 0)) {
            const float alpha = __builtin_amdgcn_exp2f(m_bef - (m2 == -INFINITY ? 0.f : m2));
            lsum *= alpha;
#pragma unroll
            for (int db = 0; db < DB; ++db) ot[db] *= alpha;
        }
        float mfix = m2 == -INFINITY ? 0.f : m2;
        if (!FAST && __builtin_expect(tile_masked(j), 0)) softmax_tile<false, true, DB>(st, pk, ot, mfix, lsum, p.c, j * BN, limit, hh);
        else softmax_tile<false, false, DB>(st, pk, ot, mfix, lsum, p.c, j * BN, limit, hh);
    };

    // ---- prologue: K tiles 0 and 1 are requested before the m-initialisation, which stages its summary tiles in
    // the four tiles behind them (K ring slots 2 .. 4 and the first V slot; four tiles = 256 key blocks per batch)
    if (grp == 0) {
        issue_tile(vis.tile(0), 0, std::false_type{});
        if (nv > 1) issue_tile(vis.tile(1), 1, std::false_type{});
    }
    if (p.use_minit) {
        const uint16_t* Rg = p.Krepr + ((size_t)(b * p.Hkv + hkv) * p.Tc) * D;
        float mx = -INFINITY;
        const int n_sum_tiles = (j_hi + BN) / BN;
        for (int t0 = 0; t0 < n_sum_tiles; t0 += 4) {
            const int nb = min(4, n_sum_tiles - t0);
            if (t0) __syncthreads();
            for (int u = 0; u < nb; ++u) load_tile<D, NWV>(Rg, (t0 + u) * BN, p.Tc, Ks + (2 + u) * T::BYTES, false, wave, lane);
            wait_vm0_and_sync();
            for (int u = 0; u < nb; ++u) {
                qk_tile<D>(Ks + (2 + u) * T::BYTES, qf, sa, ql, hh);
                mx = fmaxf(mx, tile_rowmax<true>(sa, (t0 + u) * BN, j_hi_g, hh));
            }
        }
        m2 = xhalf_max(mx) * p.c;
        __syncthreads();
    }
    if (grp == 0)
        for (int k = 2; k < min(nv, VSA_AHEAD); ++k) issue_tile(vis.tile(k), k, std::false_type{});

    if (!p.use_minit) wait_vm0_and_sync();  // nothing has waited for K tiles 0 and 1 yet

    // ---- the pipeline: step y = matrix phase y, then vector phase y
    int kslot = 0;                         // K ring slot of visit y
    bool keep1 = false, keep2 = false;     // this group keeps visit y - 1 / y - 2
    auto step = [&](int y, auto buf_c, auto grp_c, auto fast_c) __attribute__((always_inline)) {
        constexpr int BUF = decltype(buf_c)::value, GRP = decltype(grp_c)::value;
        constexpr bool FAST = decltype(fast_c)::value;  // visits y - 2 .. y + AHEAD are all plain and inside the list
        f32x16* const st_new = BUF ? sb : sa;   // Q.K^T of visit y goes here
        f32x16* const st_old = BUF ? sa : sb;   // scores of visit y - 1
        // -- matrix phase
        if (GRP == 0) {  // interval y starts: the votes of visit y - 1 are in
            keep1 = false;
            if (FAST || (y >= 1 && y <= nv)) {
                keep1 = (read_votes(y - 1) & 1) != 0;
                adopt(y - 1, keep1, fast_c);
            }
        }
        __builtin_amdgcn_sched_barrier(0);  // (the decision's bookkeeping stays in front of the matrix phase)
        __builtin_amdgcn_s_setprio(1);
        if ((FAST || y >= 2) && keep2) pv(BUF);  // V of visit y - 2 sits in slot (y - 2) & 1 = BUF
        if (FAST || y < nv) {
            qk(st_new, kslot);
            vote(st_new, y, fast_c);
        }
        __builtin_amdgcn_s_setprio(0);
        __builtin_amdgcn_sched_barrier(0);
        if (GRP == 1) {
            __builtin_amdgcn_s_waitcnt(0x0F70);  // this wave's pieces of the V tile requested half an interval ago
            __builtin_amdgcn_s_barrier();
        }
        // -- vector phase
        bool keep0 = false;
        if (GRP == 1 && (FAST || y < nv)) {  // interval y + 1 starts: the votes of visit y are in
            const int v = read_votes(y);
            keep0 = (v & 1) != 0;
            if (v & 2) issue_tile(FAST ? tile_plain(y) : vis.tile(y), BUF, fast_c);
        }
        if (GRP == 0) {  // K tile of visit y + AHEAD; the tile of visit y + 1 has landed before this interval ends
            if (FAST || y + VSA_AHEAD < nv) {
                issue_tile(FAST ? tile_plain(y + VSA_AHEAD) : vis.tile(y + VSA_AHEAD), kslot == 0 ? VSA_DK - 1 : kslot - 1, fast_c);
                __builtin_amdgcn_s_waitcnt(0x4F70);  // vmcnt(16): all but the last four tiles' pieces
            } else {
                __builtin_amdgcn_s_waitcnt(0x0F70);
            }
            // V of visit y - 1, if anyone keeps it, is fetched by group 1 at the start of this interval
        }
        if ((FAST || (y >= 1 && y <= nv)) && keep1) softmax(st_old, y - 1, fast_c);
        if (GRP == 1 && (FAST || y < nv)) adopt(y, keep0, fast_c);  // (after the softmax of visit y - 1, which still needs the max as it was)
        __builtin_amdgcn_sched_barrier(0);
        if (GRP == 0) __builtin_amdgcn_s_barrier();
        keep2 = keep1;
        if (GRP == 1) keep1 = keep0;
        kslot = kslot + 1 == VSA_DK ? 0 : kslot + 1;
    };
    auto run = [&](auto grp_c) __attribute__((always_inline)) {
        // steps 0 .. nv + 1 (the last two drain the pipeline), rounded up to an even count so that a step's score
        // buffer is a compile-time choice; the extra step only passes its barrier.  General steps up to the first step
        // whose visits are all plain, fast steps (in pairs) while they stay plain, general steps for the rest
        int y = 0;
        const int y_f0 = (n_lead + 2 + 1) & ~1;  // y - 2 >= n_lead, rounded up to even
        const int y_f1 = k_plain - VSA_AHEAD;    // y + AHEAD < k_plain; fast steps are y_f0 <= y < y_f1
        if (y_f0 + 2 <= y_f1) {
            for (; y < y_f0; y += 2) {
                step(y, std::integral_constant<int, 0>{}, grp_c, std::false_type{});
                step(y + 1, std::integral_constant<int, 1>{}, grp_c, std::false_type{});
            }
            for (; y + 2 <= y_f1; y += 2) {
                step(y, std::integral_constant<int, 0>{}, grp_c, std::true_type{});
                step(y + 1, std::integral_constant<int, 1>{}, grp_c, std::true_type{});
            }
        }
        for (; y < nv + 2; y += 2) {
            step(y, std::integral_constant<int, 0>{}, grp_c, std::false_type{});
            step(y + 1, std::integral_constant<int, 1>{}, grp_c, std::false_type{});
        }
        store_output<D>(p, ot, m2, lsum, b, h, qrow, hh);
    };
    if (grp == 0) run(std::integral_constant<int, 0>{});
    else run(std::integral_constant<int, 1>{});
    if (!p.persist) break;
    __syncthreads();  // the next item's prologue overwrites the rings
    }
}

}  // namespace
