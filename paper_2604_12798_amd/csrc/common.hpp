// VFA / VSA / online-softmax attention forward for gfx950 (MI355X), and the C ABI around it.
//
// One workgroup owns one query block (block_m rows of one head); each of its NW = block_m / 32
// waves owns 32 query rows.  Key/value tiles of 64 keys stream through LDS.  Scores are
// computed TRANSPOSED, S^T = K_j Q_i^T, with v_mfma_f32_32x32x16_bf16: in the accumulator
// layout every lane then holds 32 scores of ONE query (lane & 31), so the softmax row
// statistics are in-lane plus one exchange with lane ^ 32, the rescale factor is a per-lane
// scalar, and exp(S^T) converted to bf16 is already laid out as the B operand of
// O^T += V_j^T P^T.  V_j^T fragments come from the row-major V tile in LDS through the
// transposing read ds_read_b64_tr_b16.
//
// Softmax runs in the log2 domain: p = exp2(s * c - m2) with c = scale * log2(e) and m2 = c * (row
// max of the raw scores); LSE = (m2 + log2 l) * ln 2.
//
// This header: vector types, modes, kernel parameters, LDS tile layout, visit order, tile movers and the
// score / softmax / P.V building blocks shared by the bf16 kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <math.h>
#include <type_traits>

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

constexpr int BN = 64;  // keys per tile (= block_n)
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

enum Mode { MODE_FA = 0, MODE_VFA = 1, MODE_VSA = 2, MODE_FA_LAZY = 3, MODE_FA_SOFTEXP = 4 };
// the two online-softmax baselines: ascending order, row max on every tile, no summaries
constexpr bool is_fa(int mode) { return mode == MODE_FA || mode == MODE_FA_LAZY || mode == MODE_FA_SOFTEXP; }
constexpr bool is_lazy(int mode) { return mode == MODE_FA_LAZY || mode == MODE_FA_SOFTEXP; }
// MODE_FA_SOFTEXP: every SOFTEXP_EVERY-th exponential of a tile is computed with ordinary vector instructions
#ifndef VFA_SOFTEXP_EVERY
#define VFA_SOFTEXP_EVERY 2
#endif
constexpr int SOFTEXP_EVERY = VFA_SOFTEXP_EVERY;
constexpr int softexp_every(int mode) { return mode == MODE_FA_SOFTEXP ? SOFTEXP_EVERY : 0; }

struct Params {
    const uint16_t* Q;
    const uint16_t* K;
    const uint16_t* V;
    const uint16_t* Krepr;
    uint16_t* O;
    float* LSE;
    uint8_t* mask;
    int B, Hq, Hkv, N, Tr, Tc;
    int causal, n_sink, n_local, use_minit;
    const uint16_t* Qrepr;  // ablation: [B,Hq,Tr,D] one summary per query block replaces the rows of Q_i in the
                            // approximate score (null = the row-wise method); generic kernel only
    int pair_blocks;  // ping-pong kernel: the two wave groups take two adjacent query blocks of one head (else two heads)
    int persist;      // ping-pong kernel: number of persistent workgroups (0 = one work item per workgroup)
    int order_asc;    // ablation: visit key blocks in ascending order (sink / local blocks keep the exact-max update)
    int all_special;  // ablation: exact-max update on every visited block
    int rowskip;      // skip variant: in a kept tile, rows that fail the threshold test are suppressed (generic kernel)
    float c;     // softmax scale * log2(e)
    float thr2;  // skip threshold in log2 units
    float tau2;  // MODE_FA_LAZY: a row keeps its old max while the new one exceeds it by at most tau2 (log2 units)
};

// ---------------------------------------------------------------------------------------------
// LDS tile layout.  A tile is 64 rows of D bf16 (ROWB = 2*D bytes, CH = ROWB/16 16-byte chunks).
// K tiles are read with ds_read_b128, 32 consecutive rows at one chunk column per half wave:
// chunk' = chunk ^ (row & (CH-1)) spreads 16 consecutive rows over all 64 banks.
// V tiles are read with ds_read_b64_tr_b16, 4 consecutive rows x 64 contiguous bytes per half
// wave: the 64-byte window index is XORed with (row & 3) so the 4 rows use distinct banks.
template <int D>
struct Tile {
    static constexpr int ROWB = 2 * D;
    static constexpr int CH = ROWB / 16;
    static constexpr int BYTES = BN * ROWB;
    __device__ static int k_off(int row, int chunk) { return row * ROWB + ((chunk ^ (row & (CH - 1))) << 4); }
    __device__ static int v_off(int row, int chunk) { return row * ROWB + ((chunk ^ ((row & (CH / 4 - 1)) << 2)) << 4); }
    // Per-lane bases from which every fragment address of a tile follows by XOR with a constant
    // (the swizzles are XORs, so the varying index bits commute with them):
    //   K fragment (t, kk) of lane (ql, hh):  (k_base(ql, hh) ^ (kk << 5)) + t * 32 * ROWB
    //   V fragment (c, u, db) of a lane:      (v_base(lane, hh) ^ (db << 6)) + (16 c + 8 u) * ROWB
    __device__ static int k_base(int ql, int hh) { return ql * ROWB + ((hh ^ (ql & (CH - 1))) << 4); }
    __device__ static int v_base(int lane, int hh) {
        const int s = lane & 15, dsel = (lane >> 4) & 1, row = 4 * hh + (s >> 2);
        return row * ROWB + (((2 * dsel + ((s & 3) >> 1)) ^ ((row & (CH / 4 - 1)) << 2)) << 4) + ((s & 1) << 3);
    }
};

__device__ inline float xhalf_max(float x) {
    // max of x over the lane pair (l, l ^ 32)
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ inline float xhalf_sum(float x) {
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

__device__ inline uint32_t pack_bf16(float a, float b) {
    f32x2 v = {a, b};
    bf16x2 r = __builtin_convertvector(v, bf16x2);  // v_cvt_pk_bf16_f32, round to nearest even
    return __builtin_bit_cast(uint32_t, r);
}

// ---------------------------------------------------------------------------------------------
// Visit order of one query block: [0, n1) sink tiles, [s2, s2 + n2) local tiles, then the
// remaining visible tiles ascending.  The first n_special visits take the exact-max update.
struct Visit {
    int n1, s2, n2, total, n_special;
    int n2b;  // block-pair VSA: the last n2b local tiles belong to the second query block and are visited first
    int m1, ms2, mn2;  // ascending-order ablation: tiles [0, m1) and [ms2, ms2 + mn2) are the sink / local ones
    __device__ int tile(int k) const {  // branch-free: this sits on the scalar unit in front of every tile fetch
        const int r = k - n1;
        const int lead = k < n1 ? k : (r < n2b ? s2 + (n2 - n2b) + r : s2 + (r - n2b));
        int tail = k - n2;                                  // = n1 + (k - n1 - n2)
        tail += (n2 > 0 && tail >= s2) ? n2 : 0;
        return k < n1 + n2 ? lead : tail;
    }
    __device__ bool special(int k) const { return k < n_special || k < m1 || (k >= ms2 && k < ms2 + mn2); }
};

template <int MODE>
__device__ inline Visit make_visit(const Params& p, int a_lo, int a_hi, int j_hi) {
    Visit vis;
    vis.n1 = 0; vis.s2 = 0; vis.n2 = 0; vis.n2b = 0;
    vis.m1 = 0; vis.ms2 = 0; vis.mn2 = 0;
    vis.total = j_hi + 1;
    if (is_fa(MODE)) {
        vis.n_special = vis.total;
    } else {
        vis.n1 = min(p.n_sink, j_hi + 1);
        if (p.n_local > 0) {
            const int lo = max(max(0, a_lo - (p.n_local - 1)), vis.n1), hi = min(a_hi, j_hi);
            if (hi >= lo) { vis.s2 = lo; vis.n2 = hi - lo + 1; }
        }
        vis.n_special = vis.n1 + vis.n2;
        if (p.order_asc) {  // same sink / local sets, but no block is moved to the front
            vis.m1 = vis.n1; vis.ms2 = vis.s2; vis.mn2 = vis.n2;
            vis.n1 = 0; vis.s2 = 0; vis.n2 = 0; vis.n_special = 0;
        }
        if (p.all_special) vis.n_special = vis.total;
    }
    return vis;
}

// ---------------------------------------------------------------------------------------------
// Tile mover: global -> LDS directly (global_load_lds_dwordx4: lane l of a wave writes 16 bytes
// at the wave-uniform LDS address + 16*l, so one instruction fills RPI whole rows).  The swizzle
// is applied on the global side: the lane that owns LDS chunk position cp of row r fetches
// global chunk cp ^ f(r).  NWAVES waves share the tile's instructions round-robin.
template <int D, int NWAVES>
__device__ __forceinline__ void load_tile(const uint16_t* base, int first_row, int row_limit, uint8_t* dst,
                                          bool is_v, int wave, int lane) {
    using T = Tile<D>;
    constexpr int RPI = 1024 / T::ROWB;  // rows per wave instruction
    constexpr int NI = BN / RPI / NWAVES;  // instructions per wave per tile
    static_assert(NI >= 1, "too many waves for this tile");
    const bool full = first_row + BN <= row_limit;
#pragma unroll
    for (int u = 0; u < NI; ++u) {
        const int q = u * NWAVES + wave;
        const int r = RPI * q + lane / T::CH;
        const int cp = lane % T::CH;
        const int ch = is_v ? (cp ^ ((r & (T::CH / 4 - 1)) << 2)) : (cp ^ (r & (T::CH - 1)));
        const int gr = full ? first_row + r : min(first_row + r, row_limit - 1);
        // Written as inline asm on purpose: the compiler's wait-count pass treats every LDS read as
        // dependent on every outstanding LDS-direct load and would drain them all (vmcnt(0)) before the
        // first ds_read of a phase, which defeats the prefetch.  The callers wait explicitly instead.
        const uint32_t lds_addr = __builtin_amdgcn_readfirstlane(
            (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint8_t*)(dst + q * 1024));
        const uint16_t* src = base + (size_t)gr * D + ch * 8;
        uint32_t m0_save;  // M0 carries the LDS base of the load; put back what the compiler had there
        asm volatile(
            "s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %2, off\n\ts_mov_b32 m0, %0"
            : "=&s"(m0_save)
            : "s"(lds_addr), "v"(src)
            : "memory");
    }
}

// S^T tile: st[t][i] = raw score of query ql against key 32*t + 8*(i/4) + 4*hh + (i%4)
template <int D>
__device__ __forceinline__ void qk_tile(const uint8_t* kt, const bf16x8* qf, f32x16* st, int ql, int hh) {
    using T = Tile<D>;
    st[0] = f32x16{0};
    st[1] = f32x16{0};
#pragma unroll
    for (int kk = 0; kk < D / 16; ++kk)
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const bf16x8 kf = *reinterpret_cast<const bf16x8*>(kt + T::k_off(32 * t + ql, 2 * kk + hh));
            st[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[kk], st[t], 0, 0, 0);
        }
}

// in-lane max of a score tile, entries with key index > limit excluded when MASKED.  The test is
// written against rel = limit - key0 - 4*hh so that the per-entry side is a compile-time constant.
template <bool MASKED>
__device__ __forceinline__ float tile_rowmax(const f32x16* st, int key0, int limit, int hh) {
    float mx = -INFINITY;
    const int rel = limit - key0 - 4 * hh;
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r)
            mx = fmaxf(mx, (!MASKED || 32 * t + 8 * (r >> 2) + (r & 3) <= rel) ? st[t][r] : -INFINITY);
    return mx;
}

// 2^x without the transcendental unit (related work: FlashAttention-4's software exponential): split x into
// integer and fraction, a cubic for 2^fraction on [0, 1) (p(0) = 1 exactly, relative error <= 2.1e-4, far below
// the bf16 rounding of P), and the integer added into the exponent field.  x <= about 2^7; -inf gives 2^-126.
__device__ __forceinline__ float exp2_soft(float x) {
    const float xc = fmaxf(x, -126.f);
    const float n = __builtin_floorf(xc);
    const float f = xc - n;  // in [0, 1]; exactly 1 only for a tiny negative xc, where q(1) 2^-1 is still right
                             // (the fraction instruction would return 1 there too, but then n must not be derived from it)
    const float q = __builtin_fmaf(__builtin_fmaf(__builtin_fmaf(0.07764090f, f, 0.22760449f), f, 0.69466668f), f, 1.0f);
    return __uint_as_float(__float_as_uint(q) + ((uint32_t)(int)n << 23));
}

// Softmax step of one tile for this lane's query: st (raw scores) -> pk (exp, bf16 pairs),
// lsum += row sum.  SPECIAL: exact online-softmax update of m2 with rescale of lsum and ot;
// otherwise m2 is frozen: no row max, no rescale (Alg. 1 / Table 1).
// RESCALE = false is for the first visited tile, whose accumulators are still zero.  With MASKED the
// caller may pass limit = INT_MAX for a tile that needs no masking (one code path, no branch).
// LAZY (conditional rescale, with SPECIAL): a row adopts the new max only when it exceeds the old one by
// more than tau2; otherwise it keeps the old max and its scale factor is exactly 1, and when that
// holds for every row of the wave the whole rescale (lsum and the 16 * DB accumulator registers) is
// branched over.  exp(S - m) may then reach 2^tau2, which bf16 / fp32 hold without trouble.
// SOFT_EVERY > 0: of every SOFT_EVERY consecutive exponentials one is computed by exp2_soft.
template <bool SPECIAL, bool MASKED, int DB, bool RESCALE = true, bool LAZY = false, int SOFT_EVERY = 0>
__device__ __forceinline__ void softmax_tile(f32x16* st, uint32_t* pk, f32x16* ot, float& m2, float& lsum, float c,
                                             int key0, int limit, int hh, float tau2 = 0.f) {
    if (MASKED) {
        const int rel = limit - key0 - 4 * hh;
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int r = 0; r < 16; ++r) st[t][r] = (32 * t + 8 * (r >> 2) + (r & 3) <= rel) ? st[t][r] : -INFINITY;
    }
    float msub = m2;
    if (SPECIAL) {
        const float mx = tile_rowmax<false>(st, 0, 0, hh);
        float m_new = fmaxf(m2, xhalf_max(mx) * c);
        bool rescale = true;
        if (LAZY) {
            if (m2 != -INFINITY && m_new - m2 <= tau2) m_new = m2;
            rescale = __builtin_amdgcn_ballot_w64(m_new != m2) != 0;  // wave-uniform
        }
        msub = (m_new == -INFINITY) ? 0.f : m_new;
        if (RESCALE && rescale) {
            const float alpha = __builtin_amdgcn_exp2f(m2 - msub);
            lsum *= alpha;
#pragma unroll
            for (int db = 0; db < DB; ++db) ot[db] *= alpha;
        }
        m2 = m_new;
    }
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int r = 0; r < 16; r += 2) {
            const float x0 = __builtin_fmaf(st[t][r], c, -msub), x1 = __builtin_fmaf(st[t][r + 1], c, -msub);
            const float p0 = (SOFT_EVERY > 0 && (16 * t + r) % SOFT_EVERY == 0) ? exp2_soft(x0) : __builtin_amdgcn_exp2f(x0);
            const float p1 = (SOFT_EVERY > 0 && (16 * t + r + 1) % SOFT_EVERY == 0) ? exp2_soft(x1) : __builtin_amdgcn_exp2f(x1);
            lsum += p0;
            lsum += p1;
            pk[8 * t + (r >> 1)] = pack_bf16(p0, p1);
        }
}

// O^T += V^T P^T for one tile.  P^T fragment of key chunk c (16 keys) = registers 8*(c&1)..+7 of
// st[c >> 1] in order, i.e. pk[4c..4c+3]; the matching V^T fragment: lane gets
// V[16c + 8u + 4hh + e][32db + (lane & 31)], e = 0..3, u = 0, 1, via two transposing reads.
template <int D>
__device__ __forceinline__ void pv_tile(const uint8_t* vt, const uint32_t* pk, f32x16* ot, int lane, int hh) {
    using T = Tile<D>;
    const int s = lane & 15, dsel = (lane >> 4) & 1;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        const u32x4 pw = {pk[4 * c], pk[4 * c + 1], pk[4 * c + 2], pk[4 * c + 3]};
        const bf16x8 pf = __builtin_bit_cast(bf16x8, pw);
#pragma unroll
        for (int db = 0; db < D / 32; ++db) {
            const int chunk = 4 * db + 2 * dsel + ((s & 3) >> 1);
            const int key0 = 16 * c + 4 * hh + (s >> 2);
            const s16x4 v0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                (__attribute__((address_space(3))) s16x4*)(vt + T::v_off(key0, chunk) + ((s & 1) << 3)));
            const s16x4 v1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                (__attribute__((address_space(3))) s16x4*)(vt + T::v_off(key0 + 8, chunk) + ((s & 1) << 3)));
            const u32x2 a0 = __builtin_bit_cast(u32x2, v0), a1 = __builtin_bit_cast(u32x2, v1);
            const u32x4 aw = {a0[0], a0[1], a1[0], a1[1]};
            ot[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, aw), pf, ot[db], 0, 0, 0);
        }
    }
}

// Software-pipelined forms of qk_tile / pv_tile: the LDS reads for the next group of MFMAs are issued
// before the current group, and the scheduler is told to keep that order (one read per MFMA slot).
template <int D>
__device__ __forceinline__ void qk_tile_pipe(const uint8_t* kt, const bf16x8* qf, f32x16* st, int ql, int hh) {
    using T = Tile<D>;
    constexpr int NG = D / 32;  // groups of 4 MFMAs: k-steps (2g, 2g+1) x key halves (0, 1)
    const int kbase = T::k_base(ql, hh);
    bf16x8 f[2][4];
    auto ld = [&](bf16x8* dst, int g) __attribute__((always_inline)) {
#pragma unroll
        for (int e = 0; e < 4; ++e)
            dst[e] = *reinterpret_cast<const bf16x8*>(kt + (kbase ^ ((2 * g + (e >> 1)) << 5)) + (e & 1) * 32 * T::ROWB);
    };
    st[0] = f32x16{0};
    st[1] = f32x16{0};
    ld(f[0], 0);
#pragma unroll
    for (int g = 0; g < NG; ++g) {
        if (g + 1 < NG) ld(f[(g + 1) & 1], g + 1);
#pragma unroll
        for (int e = 0; e < 4; ++e)
            st[e & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f[g & 1][e], qf[2 * g + (e >> 1)], st[e & 1], 0, 0, 0);
    }
    __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
#pragma unroll
    for (int g = 0; g + 1 < NG; ++g)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        }
    __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);
}

template <int D>
__device__ __forceinline__ void pv_tile_pipe(const uint8_t* vt, const uint32_t* pk, f32x16* ot, int lane, int hh) {
    using T = Tile<D>;
    constexpr int DB = D / 32;
    const int vbase = T::v_base(lane, hh);
    bf16x8 f[2][DB];
    auto ld = [&](bf16x8* dst, int c) __attribute__((always_inline)) {
#pragma unroll
        for (int db = 0; db < DB; ++db) {
            const uint8_t* a = vt + (vbase ^ (db << 6)) + 16 * c * T::ROWB;
            const s16x4 v0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(a));
            const s16x4 v1 =
                __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(a + 8 * T::ROWB));
            const u32x2 a0 = __builtin_bit_cast(u32x2, v0), a1 = __builtin_bit_cast(u32x2, v1);
            const u32x4 aw = {a0[0], a0[1], a1[0], a1[1]};
            dst[db] = __builtin_bit_cast(bf16x8, aw);
        }
    };
    ld(f[0], 0);
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        if (c < 3) ld(f[(c + 1) & 1], c + 1);
        const u32x4 pw = {pk[4 * c], pk[4 * c + 1], pk[4 * c + 2], pk[4 * c + 3]};
        const bf16x8 pf = __builtin_bit_cast(bf16x8, pw);
#pragma unroll
        for (int db = 0; db < DB; ++db) ot[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f[c & 1][db], pf, ot[db], 0, 0, 0);
    }
    __builtin_amdgcn_sched_group_barrier(0x100, 2 * DB, 0);
#pragma unroll
    for (int c = 0; c < 3; ++c)
#pragma unroll
        for (int db = 0; db < DB; ++db) {
            __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        }
    __builtin_amdgcn_sched_group_barrier(0x008, DB, 0);
}

// O = O^T / l (bf16, round to nearest even), LSE = (m2 + log2 l) ln 2.
// A lane holds, per 32-wide block of d, four runs of four consecutive elements (d = 8 q + 4 hh + 0..3) of its
// query's row, and the lane 32 further holds the runs in between.  The two trade every second run
// (`v_permlane32_swap`), after which each owns runs of eight: 16-byte stores, half as many store instructions
// (the output phase of a workgroup is bound by how fast the memory pipeline takes these scattered stores).
template <int D>
__device__ __forceinline__ void store_output(const Params& p, const f32x16* ot, float m2, float lsum, int b, int h,
                                             int qrow, int hh) {
    const float l = xhalf_sum(lsum);
    const float inv = l > 0.f ? 1.f / l : 0.f;
    u32x4 w[D / 32][2];
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int e = 8 * u;  // first accumulator register of run 2u; run 2u + 1 starts four registers on
            const uint32_t a0 = pack_bf16(ot[db][e] * inv, ot[db][e + 1] * inv), a1 = pack_bf16(ot[db][e + 2] * inv, ot[db][e + 3] * inv);
            const uint32_t b0 = pack_bf16(ot[db][e + 4] * inv, ot[db][e + 5] * inv), b1 = pack_bf16(ot[db][e + 6] * inv, ot[db][e + 7] * inv);
            // lower half lanes keep run 2u and receive the partner's run 2u (elements 16u .. 16u+7);
            // upper half lanes receive the partner's run 2u + 1 and keep their own (elements 16u+8 .. 16u+15)
            const auto r0 = __builtin_amdgcn_permlane32_swap(a0, b0, false, false);
            const auto r1 = __builtin_amdgcn_permlane32_swap(a1, b1, false, false);
            w[db][u] = u32x4{r0[0], r1[0], r0[1], r1[1]};
        }
    if (qrow < p.N) {
        uint16_t* Og = p.O + ((size_t)(b * p.Hq + h) * p.N + qrow) * D;
#pragma unroll
        for (int db = 0; db < D / 32; ++db)
#pragma unroll
            for (int u = 0; u < 2; ++u) *reinterpret_cast<u32x4*>(Og + 32 * db + 16 * u + 8 * hh) = w[db][u];
        if (p.LSE && hh == 0)
            p.LSE[(size_t)(b * p.Hq + h) * p.N + qrow] = l > 0.f ? (m2 + __builtin_amdgcn_logf(l)) * kLn2 : -INFINITY;
    }
}

__device__ __forceinline__ void wait_vm0_and_sync() {
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): this wave's LDS-direct loads have landed
    __syncthreads();
}

}  // namespace
