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
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <math.h>
#include <type_traits>

#include "vfa.h"

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
    __shared__ int votes[2][2][4];
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
    if (MODE == MODE_VSA && pb) {
        // Block pairs under Alg. 2 (causal, at most one local block per query block): the second block's
        // local tiles come first (exact-max for group 1, invisible to group 0), then the first block's
        // (exact-max for group 0, ordinary frozen tiles for group 1, whose max is final by then), so each
        // group meets its own tiles in the order Alg. 2 gives them and takes the same skip decisions.
        const int lo_b = (row0 + BM) / BN;  // first tile of the second block's diagonal
        vis.n2b = vis.n2 > 0 ? max(0, vis.s2 + vis.n2 - max(vis.s2, lo_b)) : 0;
    }
    const int nv = vis.total;
    uint8_t* mrow = nullptr;
    const int i_blk = pb ? 2 * i + grp : i;  // this group's query block
    if (MODE == MODE_VSA && p.mask && i_blk < p.Tr) {
        mrow = p.mask + ((size_t)(b * p.Hq + h) * p.Tr + i_blk) * p.Tc;
        for (int j = j_hi_g + 1 + (tid & 255); j < p.Tc; j += 256) mrow[j] = 2;
    }

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

    auto vote = [&](int k) __attribute__((always_inline)) {  // VSA: this wave's say on "skip the tile of visit k"
        const int j = vis.tile(k);
        const float mx = tile_masked(j) ? tile_rowmax<true>(st, j * BN, limit, hh) : tile_rowmax<false>(st, 0, 0, hh);
        const float mt2 = xhalf_max(mx) * p.c;
        const bool row_keeps = (qrow < N) && (mt2 != -INFINITY) && !(mt2 < m2 - p.thr2);
        const bool wave_keeps = __builtin_amdgcn_ballot_w64(row_keeps) != 0;
        if (lane == 0) votes[k & 1][grp][w4] = wave_keeps ? 1 : 0;
        __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0): the vote is in LDS before this wave reaches the next barrier
    };

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
        const bool keep = true;
        pv_pending = keep;
        if (keep) {
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
    // of VFA / VSA (exact-max update); a run of unmasked visits that all take one path (frozen max for
    // VFA, exact-max for FA; VSA does not use it because its tiles may be skipped); and the trailing
    // visits that may need masking (tiles on the diagonal or past the end of a ragged sequence).
    constexpr bool TAIL_SPECIAL = is_fa(MODE);
    const int n_lead = is_fa(MODE) ? 0 : vis.n_special;  // visits [0, n_lead) are sink/local
    int k_fast_end = MODE == MODE_VSA ? n_lead : max(n_lead, 1);
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
    if constexpr (MODE == MODE_VSA) {
        // VSA keeps the ping-pong schedule and its one barrier per tile by DEFERRING the block's decision: the
        // matrix phase of visit k computes Q.K^T and casts this wave's vote; the vector phase runs the softmax
        // of visit k speculatively into pk and three scalars (its row sum, and for an exact-max tile the new max
        // and the rescale factor) without touching m, l or O; the NEXT matrix phase, one barrier later, reads the
        // four votes, and only then commits (rescale, l, m, P.V) or drops the tile.  A skipped tile costs its
        // Q.K^T, the row max and a wasted softmax on the vector ALU, which runs under the other group's MFMAs;
        // it saves the P.V and, above all, needs no synchronisation of its own.
        float lk = 0.f, alpha_k = 1.f, mnew_k = m2;  // what visit k - 1 left to commit
        bool have_prev = false, prev_special = false;
        int j_prev = 0;
        int kb = kbase, vb = vbase;
        // (fragments: four in flight, fragment i + 4 requested right behind the MFMA that consumed fragment i;
        // the addresses are rebuilt per phase from a copy of the lane's base the compiler cannot see through)
        auto pv_prev = [&](int k) __attribute__((always_inline)) {  // P.V of visit k
            const uint8_t* vt = Vs + (k & 3) * T::BYTES;
            asm volatile("" : "+v"(vb));
            auto ldv1 = [&](int c, int db) __attribute__((always_inline)) {
                const uint8_t* a = vt + (vb ^ (db << 6)) + 16 * c * T::ROWB;
                const s16x4 v0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(a));
                const s16x4 v1 =
                    __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(a + 8 * T::ROWB));
                const u32x2 a0 = __builtin_bit_cast(u32x2, v0), a1 = __builtin_bit_cast(u32x2, v1);
                const u32x4 aw = {a0[0], a0[1], a1[0], a1[1]};
                return __builtin_bit_cast(bf16x8, aw);
            };
#pragma unroll
            for (int db = 0; db < DB; ++db) fa[db] = ldv1(0, db);
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int c = i >> 2, db = i & 3;
                const u32x4 pw = {pk[4 * c], pk[4 * c + 1], pk[4 * c + 2], pk[4 * c + 3]};
                ot[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[db], __builtin_bit_cast(bf16x8, pw), ot[db], 0, 0, 0);
                if (c < 3) fa[db] = ldv1(c + 1, db);
                __builtin_amdgcn_sched_barrier(0);
            }
        };
        // softmax of the tile in st into pk, lk (and mnew_k, alpha_k for an exact-max tile); m2, lsum, ot are left alone
        auto spec_softmax = [&](int j, auto special_c, auto fast_c) __attribute__((always_inline)) {
            constexpr bool SPECIAL = decltype(special_c)::value, FAST = decltype(fast_c)::value;
            float mt = m2;
            lk = 0.f;
            if (FAST) softmax_tile<SPECIAL, false, DB, false>(st, pk, ot, mt, lk, p.c, j * BN, limit, hh);
            else softmax_tile<SPECIAL, true, DB, false>(st, pk, ot, mt, lk, p.c, j * BN, tile_masked(j) ? limit : 0x3fffffff, hh);
            mnew_k = mt;
            alpha_k = SPECIAL ? __builtin_amdgcn_exp2f(m2 - (mt == -INFINITY ? 0.f : mt)) : 1.f;
        };
        // decision on the previous visit (its votes were cast a barrier ago), then commit or drop
        // PS: was the previous visit an exact-max one?  0 = no, 1 = yes, 2 = look at prev_special (the steady loops
        // know the answer at compile time and so carry no rescale of the 64 accumulator registers at all)
        auto resolve = [&](auto ps_c) __attribute__((always_inline)) {
            constexpr int PS = decltype(ps_c)::value;
            bool keep = false;
            if (have_prev) {
                const int kp = (j_prev >> 16) & 1;  // parity of the previous visit
                keep = __builtin_amdgcn_readfirstlane(votes[kp][grp][0] | votes[kp][grp][1] | votes[kp][grp][2] |
                                                      votes[kp][grp][3]) != 0;
                const int j = j_prev & 0xffff;
                if (mrow && j <= j_hi_g && (tid & 255) == 0) mrow[j] = keep ? 0 : 1;  // (a tile past j_hi_g is the other block's)
                if (keep) {
                    if (PS == 1 || (PS == 2 && prev_special)) {
                        lsum = lsum * alpha_k + lk;
#pragma unroll
                        for (int db = 0; db < DB; ++db) ot[db] *= alpha_k;
                        m2 = mnew_k;
                    } else {
                        lsum += lk;
                    }
                }
            }
            return keep;
        };
        auto matrix_vsa = [&](int k, auto ps_c) __attribute__((always_inline)) {
            const uint8_t* kt = Ks + (k & 3) * T::BYTES;
            asm volatile("" : "+v"(kb));
            auto ldk1 = [&](int i) __attribute__((always_inline)) {  // fragment i = (k-step i / 2, key half i % 2)
                return *reinterpret_cast<const bf16x8*>(kt + (kb ^ ((i >> 1) << 5)) + (i & 1) * 32 * T::ROWB);
            };
            __builtin_amdgcn_s_setprio(1);
#pragma unroll
            for (int i = 0; i < 4; ++i) fa[i] = ldk1(i);  // in flight while the decision is read
            const bool keep = resolve(ps_c);
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                st[i & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i & 3], qf[i >> 1], i < 2 ? f32x16{0} : st[i & 1], 0, 0, 0);
                if (i + 4 < 16) fa[i & 3] = ldk1(i + 4);
                __builtin_amdgcn_sched_barrier(0);
            }
            vote(k);
            __builtin_amdgcn_sched_barrier(0);
            if (keep) pv_prev(k - 1);
            __builtin_amdgcn_s_setprio(0);
        };
        // speculative softmax of visit k: st -> pk, lk (and mnew_k, alpha_k); m2, lsum, ot are left alone
        auto vector_vsa = [&](int k, auto special_c, auto fast_c) __attribute__((always_inline)) {
            constexpr bool SPECIAL = decltype(special_c)::value, FAST = decltype(fast_c)::value;
            const int j = vis.tile(k);
            fetch_ahead(k);
            spec_softmax(j, special_c, fast_c);
            prev_special = SPECIAL;
            have_prev = true;
            j_prev = j | ((k & 1) << 16);
        };
        // block pairs: a local tile is exact-max only for the group whose block it belongs to
        auto own_special = [&](int k) __attribute__((always_inline)) {
            return !pb || k < vis.n1 || ((k - vis.n1 < vis.n2b) == (grp == 1));
        };
        // Both groups run M(0) V(0) M(1) V(1) ...; group 0 passes the barrier after each vector phase, group 1
        // after each matrix phase, which puts group 1 half an interval behind as in the other modes.
        using PS0 = std::integral_constant<int, 0>;
        using PS2 = std::integral_constant<int, 2>;
        // (one copy of the loop nest per group, as in the other modes: straight-line code for the register allocator)
        auto run_vsa = [&](auto grp_c) __attribute__((always_inline)) {
            constexpr int GRP = decltype(grp_c)::value;
            auto step = [&](int k, auto ps_c, auto special_c, auto fast_c) __attribute__((always_inline)) {
                matrix_vsa(k, ps_c);
                if (GRP == 1) __builtin_amdgcn_s_barrier();
                __builtin_amdgcn_sched_barrier(0);
                vector_vsa(k, special_c, fast_c);
                if (GRP == 0) __builtin_amdgcn_s_barrier();
                __builtin_amdgcn_sched_barrier(0);
            };
            int k = 0;
            for (; k < min(n_lead, nv); ++k) {
                if (own_special(k)) step(k, PS2{}, true_type{}, false_type{});
                else step(k, PS2{}, false_type{}, false_type{});
            }
            if (k < nv) {  // the first frozen visit still has an exact-max visit to resolve
                step(k, PS2{}, false_type{}, false_type{});
                ++k;
            }
            for (; k < k_fast_end; ++k) step(k, PS0{}, false_type{}, true_type{});
            for (; k < nv; ++k) step(k, PS0{}, false_type{}, false_type{});
            if (resolve(PS2{})) pv_prev(nv - 1);  // the last visit's decision (its votes are a barrier old for both groups)
            store_output<D>(p, ot, m2, lsum, b, h, qrow, hh);
        };
        if (grp == 0) run_vsa(std::integral_constant<int, 0>{});
        else run_vsa(std::integral_constant<int, 1>{});
    } else {
        if (grp == 0) run_group(std::integral_constant<int, 0>{});
        else run_group(std::integral_constant<int, 1>{});
    }
    if (!p.persist) break;
    __syncthreads();  // the next item's prologue overwrites the ring
    }
}

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
// The work is HBM bound (K and V are read once), so single-wave workgroups with a two-deep tile ring
// (64 KiB of LDS, two per CU) and the same tile helpers as the prefill kernels are enough.
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
    // K is double buffered, V single buffered: 3 tiles = 48 KiB at d = 128, so three workgroups share a CU
    // and keep three times (next K tile + this V tile) in flight, which is what an HBM-bound loop needs
    __shared__ __attribute__((aligned(16))) uint8_t smem[3 * T::BYTES];
    uint8_t* const Ks = smem;
    uint8_t* const Vs = smem + 2 * T::BYTES;
    constexpr int NI = BN / (1024 / T::ROWB);  // load instructions per tile (one wave)
    constexpr int WAIT_ALL_BUT_ONE_TILE = 0x0F70 | (NI & 15) | ((NI >> 4) << 14);  // s_waitcnt vmcnt(NI)
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
    if (t_lo < t_hi) {
        load_tile<D, 1>(Kg, t_lo * BN, n_keys, Ks, false, 0, lane);
        wait_vm0_and_sync();
    }
    for (int t = t_lo; t < t_hi; ++t) {
        const int cur = (t - t_lo) & 1;
        // the V buffer's last readers (the P.V MFMAs of the previous tile) have all issued
        load_tile<D, 1>(Vg, t * BN, n_keys, Vs, true, 0, lane);
        const bool more = t + 1 < t_hi;
        if (more) load_tile<D, 1>(Kg, (t + 1) * BN, n_keys, Ks + (cur ^ 1) * T::BYTES, false, 0, lane);
        f32x16 st[2];
        uint32_t pk[16];
        qk_tile_pipe<D>(Ks + cur * T::BYTES, qf, st, ql, hh);
        softmax_tile<false, true, DB>(st, pk, ot, m2, lsum, p.c, t * BN, n_keys - 1, hh);  // frozen max, ragged tail masked
        if (more) __builtin_amdgcn_s_waitcnt(WAIT_ALL_BUT_ONE_TILE);  // V(t) has landed; K(t + 1) may still be on its way
        else __builtin_amdgcn_s_waitcnt(0x0F70);
        __syncthreads();
        pv_tile_pipe<D>(Vs, pk, ot, lane, hh);
        wait_vm0_and_sync();
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

// ---------------------------------------------------------------------------------------------
// FP8 (E4M3) path: the 8-bit tensor regime of the paper's performance discussion ("C8V32": matrix
// products in 8 bit, softmax in fp32).  v_mfma_f32_32x32x64_f8f6f4 does a 32 x 32 x 64 product in
// 64 cycles, twice the bf16 rate, so a 64-key tile is 4 + 4 MFMAs per wave instead of 16 + 16 and the
// softmax arithmetic, unchanged, weighs twice as much.  Measured pairing of the operands: byte j of
// lane (row, half) of A meets byte j of lane (col, same half) of B, so any assignment of the 64
// k-indices to (half, byte) works as long as both operands use the same one:
//   Q.K^T  k-step kh (0, 1): byte j of half hh = feature 64 kh + 32 hh + j, for K rows and Q rows alike
//   P.V    byte j of half hh = key 32 (j / 16) + 8 ((j % 16) / 4) + 4 hh + j % 4 of the tile: the order in
//          which the score accumulators of a lane, packed four to a dword, already sit; V is stored
//          transposed and permuted to that order by the packing pre-pass, so one 32-byte read per
//          lane is the whole A operand and no transposing read is needed.
// exp(S - m) goes to E4M3 scaled by 2^(8 - H): the conversion instruction does not saturate (beyond
// 448 it writes NaN), so the value is capped by the clamp modifier of the exponential itself:
// q = min(exp2(s c - m - H), 1), stored as q 2^8, and l sums the same q.  H = 0 for the exact-max
// baseline (exp <= 1 by construction); the frozen-max mode takes H = 4: exact while the frozen max
// is at most 4 log2-units (2.8 nats) below the true one, capped (never NaN) beyond.
typedef __attribute__((ext_vector_type(8))) int i32x8;
typedef __attribute__((ext_vector_type(2))) short s16x2;

struct Tile8 {
    static constexpr int KBYTES = BN * 128;   // K tile: 64 rows of 128 bytes
    static constexpr int VBYTES = 128 * BN;   // V^T tile: 128 rows (features) of 64 bytes (keys, permuted)
    // 16-byte chunk c of row r is stored at chunk position c ^ key(r); chosen so that 16 consecutive
    // rows reading the same logical chunk cover all 64 banks
    __device__ static int k_off(int r, int c) { return r * 128 + ((c ^ ((r >> 1) & 7)) << 4); }
    __device__ static int v_off(int r, int c) { return r * 64 + ((c ^ ((r >> 2) & 3)) << 4); }
};

// E4M3 x E4M3; scale_a = four copies of an E8M0 exponent byte that multiplies the A operand's 32-element
// blocks by 2^(byte - 127) inside the instruction (0x7f7f7f7f = 2^0); the B operand is not scaled
__device__ __forceinline__ f32x16 mfma_f8(const i32x8& a, const i32x8& b, const f32x16& c, int scale_a = 0x7f7f7f7f) {
    return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, c, 0, 0, 0, scale_a, 0, 0x7f7f7f7f);
}

// K tile (IS_V = false: rows of 128 bytes from a row-major [*, 128] array, rows clamped to row_limit - 1)
// or V^T tile (IS_V = true: a contiguous 8 KiB block) -> LDS, 8 one-KiB pieces shared by NWAVES waves
template <bool IS_V, int NWAVES>
__device__ __forceinline__ void load_tile8(const uint8_t* base, int first_row, int row_limit, uint8_t* dst, int wave,
                                           int lane) {
    constexpr int NI = 8 / NWAVES;
#pragma unroll
    for (int u = 0; u < NI; ++u) {
        const int q = u * NWAVES + wave;
        int r, c;
        const uint8_t* src;
        if (IS_V) {
            r = 16 * q + (lane >> 2);
            c = (lane & 3) ^ ((r >> 2) & 3);
            src = base + r * 64 + c * 16;
        } else {
            r = 8 * q + (lane >> 3);
            c = (lane & 7) ^ ((r >> 1) & 7);
            src = base + (size_t)min(first_row + r, row_limit - 1) * 128 + c * 16;
        }
        const uint32_t lds_addr = __builtin_amdgcn_readfirstlane(
            (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint8_t*)(dst + q * 1024));
        uint32_t m0_save;
        asm volatile(
            "s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %2, off\n\ts_mov_b32 m0, %0"
            : "=&s"(m0_save)
            : "s"(lds_addr), "v"(src)
            : "memory");
    }
}

__device__ __forceinline__ i32x8 lds_frag8(const uint8_t* a0, const uint8_t* a1) {
    const u32x4 lo = *reinterpret_cast<const u32x4*>(a0), hi = *reinterpret_cast<const u32x4*>(a1);
    return i32x8{(int)lo[0], (int)lo[1], (int)lo[2], (int)lo[3], (int)hi[0], (int)hi[1], (int)hi[2], (int)hi[3]};
}

// S^T tile from an E4M3 K tile: st[t][i] as in qk_tile: products of the codes' values times the power of
// two in scale_a, plus *start (a value per lane, i.e. per query, already spread over 16 registers) if given
__device__ __forceinline__ void qk_tile8(const uint8_t* kt, const i32x8* qf, f32x16* st, int ql, int hh,
                                         int scale_a = 0x7f7f7f7f, const f32x16* start = nullptr) {
    i32x8 f[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {  // e = 2 t + kh
        const int row = 32 * (e >> 1) + ql, c0 = 4 * (e & 1) + 2 * hh;
        f[e] = lds_frag8(kt + Tile8::k_off(row, c0), kt + Tile8::k_off(row, c0 + 1));
    }
#pragma unroll
    for (int e = 0; e < 4; ++e)
        st[e >> 1] = mfma_f8(f[e], qf[e & 1], (e & 1) ? st[e >> 1] : (start ? *start : f32x16{0}), scale_a);
}

// P_BF8: the P operand holds E5M2 codes (V stays E4M3)
template <bool P_BF8 = false>
__device__ __forceinline__ void pv_tile8(const uint8_t* vt, const uint32_t* pk, f32x16* ot, int lane, int hh) {
    const i32x8 pf = {(int)pk[0], (int)pk[1], (int)pk[2], (int)pk[3], (int)pk[4], (int)pk[5], (int)pk[6], (int)pk[7]};
    i32x8 f[4];
#pragma unroll
    for (int db = 0; db < 4; ++db) {
        const int row = 32 * db + (lane & 31);
        f[db] = lds_frag8(vt + Tile8::v_off(row, 2 * hh), vt + Tile8::v_off(row, 2 * hh + 1));
    }
#pragma unroll
    for (int db = 0; db < 4; ++db)
        ot[db] = P_BF8 ? __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(f[db], pf, ot[db], 0, 1, 0, 0x7f7f7f7f, 0, 0x7f7f7f7f)
                       : mfma_f8(f[db], pf, ot[db]);
}

// four values in [0, 1] -> one dword of 8-bit codes: E4M3 of q * 2^8, or (P_BF8) E5M2 of q * 2^15, which trades one
// mantissa bit for 14 more binades below 1: for a frozen max that may sit far above the scores
template <bool P_BF8>
__device__ __forceinline__ uint32_t pack_p8(const float* q) {
    s16x2 w = {0, 0};
    if (P_BF8) {
        w = __builtin_amdgcn_cvt_scalef32_pk_bf8_f32(w, q[0], q[1], 0x1p-15f, false);
        w = __builtin_amdgcn_cvt_scalef32_pk_bf8_f32(w, q[2], q[3], 0x1p-15f, true);
    } else {
        w = __builtin_amdgcn_cvt_scalef32_pk_fp8_f32(w, q[0], q[1], 0.00390625f, false);  // / 2^-8
        w = __builtin_amdgcn_cvt_scalef32_pk_fp8_f32(w, q[2], q[3], 0.00390625f, true);
    }
    return __builtin_bit_cast(uint32_t, w);
}

// softmax step with E4M3 output: as softmax_tile, but q = min(exp2(s c - m - H), 1) (clamp modifier of the
// exponential), lsum += q, and four q's go to one dword as q * 2^8 (pk[0..7] = the B operand of P.V)
template <bool SPECIAL, bool MASKED, bool P_BF8 = false>
__device__ __forceinline__ void softmax_tile8(f32x16* st, uint32_t* pk, f32x16* ot, float& m2, float& lsum, float c,
                                              float headroom, int key0, int limit, int hh) {
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
        const float m_new = fmaxf(m2, xhalf_max(mx) * c);
        msub = (m_new == -INFINITY) ? 0.f : m_new;
        const float alpha = __builtin_amdgcn_exp2f(m2 - msub);
        lsum *= alpha;
#pragma unroll
        for (int db = 0; db < 4; ++db) ot[db] *= alpha;
        m2 = m_new;
    }
    const float sub = msub + headroom;
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int r = 0; r < 16; r += 4) {
            float q[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                q[e] = __builtin_amdgcn_fmed3f(__builtin_amdgcn_exp2f(__builtin_fmaf(st[t][r + e], c, -sub)), 0.f, 1.f);
                lsum += q[e];
            }
            pk[4 * t + (r >> 2)] = pack_p8<P_BF8>(q);
        }
}

// The same for a frozen tile when the scores arrive as s c - m - H already (scale folded into the MFMA, the
// rest into its accumulator start): exp, sum, convert.  Nothing per score is left of the scaling and the
// subtraction, which the exact-max path cannot avoid because its m depends on the very tile.
template <bool MASKED, bool P_BF8 = false>
__device__ __forceinline__ void softmax_tile8_folded(f32x16* st, uint32_t* pk, float& lsum, int key0, int limit, int hh) {
    if (MASKED) {
        const int rel = limit - key0 - 4 * hh;
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int r = 0; r < 16; ++r) st[t][r] = (32 * t + 8 * (r >> 2) + (r & 3) <= rel) ? st[t][r] : -INFINITY;
    }
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int r = 0; r < 16; r += 4) {
            float q[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                q[e] = __builtin_amdgcn_fmed3f(__builtin_amdgcn_exp2f(st[t][r + e]), 0.f, 1.f);
                lsum += q[e];
            }
            pk[4 * t + (r >> 2)] = pack_p8<P_BF8>(q);
        }
}

struct Fp8Params {
    const uint8_t* Q;      // [B, Hq, N, 128] E4M3
    const uint8_t* K;      // [B, Hkv, N, 128]
    const uint8_t* Vt;     // [B, Hkv, Tc, 128, 64]: per key tile, features x permuted keys
    const uint8_t* Krepr;  // [B, Hkv, Tc, 128]
    uint16_t* O;           // [B, Hq, N, 128] bf16
    float* LSE;
    int B, Hq, Hkv, N, Tr, Tc;
    int causal, n_sink, n_local, use_minit;
    float c;          // softmax scale * descale_q * descale_k * log2(e): multiplies the raw code products
    int scale_a;      // FOLD: that factor is a power of two and sits here as four E8M0 bytes (then c = 1)
    float descale_v;  // multiplies O
    float headroom;   // H above
};

// One workgroup = 4 waves x 32 query rows = one 128-row query block of one head; two-deep K / V^T ring
// (32 KiB), several workgroups per CU.  MODE_FA or MODE_VFA.
// FOLD (Alg. 1 only, when the factor between code products and log2-domain scores is a power of two): the
// K operand's block scale applies it inside every Q.K^T MFMA, and on frozen tiles the accumulators start at
// -(m + H), so the scores come out of the matrix unit ready for exp2.
template <int MODE, bool FOLD>
__global__ __launch_bounds__(256, FOLD ? 3 : 2) void attn_fp8_kernel(const Fp8Params p) {
    static_assert(!FOLD || MODE == MODE_VFA, "folding needs a max that is known before the tile");
    const int sa = FOLD ? p.scale_a : 0x7f7f7f7f;
    constexpr int D = 128, BM = 128, DB = 4;
    __shared__ __attribute__((aligned(16))) uint8_t smem[2 * (Tile8::KBYTES + Tile8::VBYTES)];
    uint8_t* const Ks = smem;
    uint8_t* const Vs = smem + 2 * Tile8::KBYTES;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int ql = lane & 31, hh = lane >> 5;
    const int g = p.Hq / p.Hkv;
    int b, h, i;
    {
        const int id = blockIdx.x, G = p.B * p.Hkv;
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
    const int hkv = h / g, N = p.N;
    const int row0 = i * BM, last_row = min(N, row0 + BM) - 1;
    const int a_lo = row0 / BN, a_hi = last_row / BN;
    const int j_hi = p.causal ? a_hi : p.Tc - 1;
    const uint8_t* Kg = p.K + ((size_t)(b * p.Hkv + hkv) * N) * D;
    const uint8_t* Vg = p.Vt + ((size_t)(b * p.Hkv + hkv) * p.Tc) * Tile8::VBYTES;
    const int qrow = row0 + 32 * wave + ql, qrow_c = min(qrow, N - 1);
    const int limit = p.causal ? qrow_c : N - 1;
    i32x8 qf[2];
    {
        const uint8_t* qp = p.Q + ((size_t)(b * p.Hq + h) * N + qrow_c) * D + 32 * hh;
#pragma unroll
        for (int kh = 0; kh < 2; ++kh) {
            const u32x4 lo = *reinterpret_cast<const u32x4*>(qp + 64 * kh), hi = *reinterpret_cast<const u32x4*>(qp + 64 * kh + 16);
            qf[kh] = i32x8{(int)lo[0], (int)lo[1], (int)lo[2], (int)lo[3], (int)hi[0], (int)hi[1], (int)hi[2], (int)hi[3]};
        }
    }
    float m2 = -INFINITY;
    if (MODE == MODE_VFA && p.use_minit) {
        const uint8_t* Rg = p.Krepr + ((size_t)(b * p.Hkv + hkv) * p.Tc) * D;
        float mx = -INFINITY;
        for (int ts = 0; ts * BN <= j_hi; ++ts) {
            __syncthreads();
            load_tile8<false, 4>(Rg, ts * BN, p.Tc, Ks, wave, lane);
            wait_vm0_and_sync();
            f32x16 st[2];
            qk_tile8(Ks, qf, st, ql, hh, sa);
            mx = fmaxf(mx, tile_rowmax<true>(st, ts * BN, j_hi, hh));
        }
        m2 = xhalf_max(mx) * p.c;
        __syncthreads();
    }
    Params vp{};
    vp.n_sink = p.n_sink; vp.n_local = p.n_local;
    const Visit vis = make_visit<MODE>(vp, a_lo, a_hi, j_hi);
    f32x16 ot[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db) ot[db] = f32x16{0};
    float lsum = 0.f;
    {
        const int j0 = vis.tile(0);
        load_tile8<false, 4>(Kg, j0 * BN, N, Ks, wave, lane);
        load_tile8<true, 4>(Vg + (size_t)j0 * Tile8::VBYTES, 0, 0, Vs, wave, lane);
        wait_vm0_and_sync();
    }
    f32x16 start;  // FOLD: -(m + H) of this lane's query in all 16 registers, set once the max is frozen
    // One visit; SPECIAL and MASKED are compile-time so that each of the three loops below has one softmax body.
    auto visit = [&](int k, auto special_c, auto masked_c) __attribute__((always_inline)) {
        constexpr bool SPECIAL = decltype(special_c)::value, MASKED = decltype(masked_c)::value;
        const int j = vis.tile(k), buf = k & 1;
        if (k + 1 < vis.total) {
            const int jn = vis.tile(k + 1);
            load_tile8<false, 4>(Kg, jn * BN, N, Ks + (buf ^ 1) * Tile8::KBYTES, wave, lane);
            load_tile8<true, 4>(Vg + (size_t)jn * Tile8::VBYTES, 0, 0, Vs + (buf ^ 1) * Tile8::VBYTES, wave, lane);
        }
        f32x16 st[2];
        uint32_t pk[8];
        __builtin_amdgcn_s_setprio(1);
        if (FOLD && !SPECIAL) qk_tile8(Ks + buf * Tile8::KBYTES, qf, st, ql, hh, sa, &start);
        else qk_tile8(Ks + buf * Tile8::KBYTES, qf, st, ql, hh, sa);
        __builtin_amdgcn_s_setprio(0);
        const bool needs_mask = (p.causal && j * BN + BN - 1 > row0) || (j + 1) * BN > N;
        if (FOLD && !SPECIAL) softmax_tile8_folded<MASKED>(st, pk, lsum, j * BN, needs_mask ? limit : 0x3fffffff, hh);
        else softmax_tile8<SPECIAL, MASKED>(st, pk, ot, m2, lsum, p.c, p.headroom, j * BN, needs_mask ? limit : 0x3fffffff, hh);
        __builtin_amdgcn_s_setprio(1);
        pv_tile8(Vs + buf * Tile8::VBYTES, pk, ot, lane, hh);
        __builtin_amdgcn_s_setprio(0);
        wait_vm0_and_sync();
    };
    using std::false_type;
    using std::true_type;
    // visits [0, n_lead): sink / local (exact-max, may need masking); [n_lead, k_fast_end): a run of unmasked
    // tiles that all take one path (frozen for Alg. 1, exact-max for the baseline); the rest: the same with masking
    constexpr bool TAIL_SPECIAL = is_fa(MODE);
    const int n_lead = TAIL_SPECIAL ? 0 : min(vis.n_special, vis.total);
    int k_fast_end;
    {
        int j_masked = p.causal ? a_lo : p.Tc;
        if (N % BN) j_masked = min(j_masked, p.Tc - 1);
        int cnt = max(0, j_masked - vis.n1);
        if (vis.n2 > 0) cnt -= max(0, min(j_masked, vis.s2 + vis.n2) - vis.s2);
        k_fast_end = max(n_lead, min(vis.total, n_lead + cnt));
    }
    int k = 0;
    for (; k < n_lead; ++k) visit(k, true_type{}, true_type{});
    if (FOLD) {
        const float v = -(m2 + p.headroom);
#pragma unroll
        for (int r = 0; r < 16; ++r) start[r] = v;
    }
    for (; k < k_fast_end; ++k) visit(k, std::integral_constant<bool, TAIL_SPECIAL>{}, false_type{});
    for (; k < vis.total; ++k) visit(k, std::integral_constant<bool, TAIL_SPECIAL>{}, true_type{});
    // O = descale_v * 2^-8 * O^T / l (the codes of P carry 2^8); LSE = (m2 + H + log2 l) ln 2  (l sums exp2(s c - m2 - H))
    const float l = xhalf_sum(lsum);
    const float inv = l > 0.f ? p.descale_v * 0.00390625f / l : 0.f;
    if (qrow < N) {
        uint16_t* Og = p.O + ((size_t)(b * p.Hq + h) * N + qrow) * D;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                const u32x2 w = {pack_bf16(ot[db][4 * q4] * inv, ot[db][4 * q4 + 1] * inv),
                                 pack_bf16(ot[db][4 * q4 + 2] * inv, ot[db][4 * q4 + 3] * inv)};
                *reinterpret_cast<u32x2*>(Og + 32 * db + 8 * q4 + 4 * hh) = w;
            }
        if (p.LSE && hh == 0)
            p.LSE[(size_t)(b * p.Hq + h) * N + qrow] =
                l > 0.f ? (m2 + p.headroom + __builtin_amdgcn_logf(l)) * kLn2 : -INFINITY;
    }
}

// bf16 -> E4M3 codes of x * inv_scale (saturated at +-448), same layout.  8 elements per thread.
__global__ __launch_bounds__(256) void fp8_quantize_kernel(const uint16_t* __restrict__ X, uint8_t* __restrict__ Y,
                                                           long long n8, float inv_scale) {
    const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
    if (i >= n8) return;
    const u32x4 x = *reinterpret_cast<const u32x4*>(X + i * 8);
    float v[8];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        v[2 * e] = fminf(fmaxf(__uint_as_float(x[e] << 16) * inv_scale, -448.f), 448.f);
        v[2 * e + 1] = fminf(fmaxf(__uint_as_float(x[e] & 0xffff0000u) * inv_scale, -448.f), 448.f);
    }
    int w0 = __builtin_amdgcn_cvt_pk_fp8_f32(v[0], v[1], 0, false);
    w0 = __builtin_amdgcn_cvt_pk_fp8_f32(v[2], v[3], w0, true);
    int w1 = __builtin_amdgcn_cvt_pk_fp8_f32(v[4], v[5], 0, false);
    w1 = __builtin_amdgcn_cvt_pk_fp8_f32(v[6], v[7], w1, true);
    *reinterpret_cast<u32x2*>(Y + i * 8) = u32x2{(uint32_t)w0, (uint32_t)w1};
}

// V [BH, N, 128] bf16 -> per 64-key tile a [128 features][64 keys] E4M3 block with the keys in the order the
// P.V operand wants them (byte 32 hh + j of a row = key 32 (j / 16) + 8 ((j % 16) / 4) + 4 hh + j % 4);
// keys beyond N are written as 0.  One workgroup per (tile, head); transposition through LDS.
__global__ __launch_bounds__(256) void fp8_pack_v_kernel(const uint16_t* __restrict__ V, uint8_t* __restrict__ Vt, int N,
                                                         int Tc, float inv_scale) {
    __shared__ uint8_t codes[BN][128 + 4];
    const int j = blockIdx.x, bh = blockIdx.y, tid = threadIdx.x;
    const uint16_t* src = V + ((size_t)bh * N + (size_t)j * BN) * 128;
    for (int idx = tid; idx < BN * 64; idx += 256) {  // pairs of features
        const int key = idx >> 6, f2 = idx & 63;
        uint32_t w = 0;
        if (j * BN + key < N) w = *reinterpret_cast<const uint32_t*>(src + (size_t)key * 128 + 2 * f2);
        const float a = fminf(fmaxf(__uint_as_float(w << 16) * inv_scale, -448.f), 448.f);
        const float b = fminf(fmaxf(__uint_as_float(w & 0xffff0000u) * inv_scale, -448.f), 448.f);
        const uint32_t c2 = (uint32_t)__builtin_amdgcn_cvt_pk_fp8_f32(a, b, 0, false);
        codes[key][2 * f2] = (uint8_t)(c2 & 0xff);
        codes[key][2 * f2 + 1] = (uint8_t)((c2 >> 8) & 0xff);
    }
    __syncthreads();
    uint8_t* dst = Vt + ((size_t)bh * Tc + j) * Tile8::VBYTES;
    for (int idx = tid; idx < 128 * 16; idx += 256) {  // (feature, group of 4 output bytes)
        const int f = idx >> 4, q = idx & 15;          // output bytes 4 q .. 4 q + 3 of row f
        const int hh = q >> 3, jj = 4 * (q & 7);       // byte 32 hh + jj + e
        uint32_t w = 0;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int jb = jj + e;
            const int key = 32 * (jb >> 4) + 8 * ((jb & 15) >> 2) + 4 * hh + (jb & 3);
            w |= (uint32_t)codes[key][f] << (8 * e);
        }
        *reinterpret_cast<uint32_t*>(dst + f * 64 + 4 * q) = w;
    }
}

// sabsmax over E4M3 codes (sign-magnitude: the 7 low bits order the magnitudes; tie -> the positive code)
__global__ __launch_bounds__(128) void fp8_kblock_summary_kernel(const uint8_t* __restrict__ K, uint8_t* __restrict__ R, int N,
                                                                 int Tc) {
    const int j = blockIdx.x, bh = blockIdx.y, t = threadIdx.x;
    const uint8_t* base = K + ((size_t)bh * N + (size_t)j * BN) * 128 + t;
    const int rows = min(BN, N - j * BN);
    uint32_t best = base[0];
    for (int r = 1; r < rows; ++r) {
        const uint32_t x = base[(size_t)r * 128];
        const uint32_t mb = best & 0x7f, mx = x & 0x7f;
        best = mx > mb ? x : (mb > mx ? best : min(best, x));
    }
    R[((size_t)bh * Tc + j) * 128 + t] = (uint8_t)best;
}

// ---------------------------------------------------------------------------------------------
// MXFP4 scores: the 4-bit tensor regime (Q.K^T on E2M1 elements with one E8M0 scale per 32 features, the
// published MX block format; P.V stays on E4M3 as above, since exp(S - m) in [0, 1] needs more than the one
// mantissa bit of E2M1).  v_mfma_scale_f32_32x32x64_f8f6f4 with both operands E2M1 runs a 64-deep step in
// 32 cycles, twice the E4M3 rate, and takes the block scales as operands: lane (row, half hh) supplies the
// scale byte of its own 32 elements, k = 32 hh .. 32 hh + 31 of the step, which are features
// 64 kh + 32 hh .. + 31: exactly one MX block.  The scale byte is replicated into all four bytes of its
// register, so the byte select of the instruction does not matter.
// Key-block summaries of MXFP4 keys are not MXFP4 vectors (their entries come from keys with different
// scales): they are kept as MX blocks of E5M2 elements (two mantissa bits cover the one of E2M1, and the 29
// binades below the block maximum cover the spread of the keys' scales), and the m-initialisation multiplies
// them with the E2M1 queries in the same instruction (A = E5M2, B = E2M1).  Measured for that mixed form: the
// k index of an element is 32 hh + j for nibble j of a 4-bit operand, but 16 hh + j (j < 16) or
// 32 + 16 hh + (j - 16) for byte j of an 8-bit operand, and the scale of lane half b covers k = 32 b .. 32 b + 31
// in both (for 8-bit data: bytes 16 b .. 16 b + 15 of BOTH halves).  Two operands of equal width pair up whatever
// the order, which is all the paths above need; here the summary's 16-byte chunks are picked to match.
struct Tile4 {
    static constexpr int KBYTES = BN * 64;  // K tile: 64 rows of 64 bytes (128 nibbles)
    // 16-byte chunk c (0..3) of row r sits at chunk position c ^ ((r >> 2) & 3): 16 consecutive rows reading one
    // logical chunk cover all 64 banks
    __device__ static int k_off(int r, int c) { return r * 64 + ((c ^ ((r >> 2) & 3)) << 4); }
};

// E2M1 magnitudes by code (sign in bit 3)
__device__ __forceinline__ float e2m1_value(uint32_t code) {
    const uint32_t mag = code & 7u;
    const float v = mag < 2u ? 0.5f * (float)mag : __builtin_ldexpf(1.0f + 0.5f * (float)(mag & 1u), (int)(mag >> 1) - 1);
    return (code & 8u) ? -v : v;
}

// X bf16 -> MXFP4: thread = 8 consecutive elements, 4 threads = one block of 32.  y = x * pre_scale (fp32);
// scale byte = exponent field of max|y| - 2, at least 0; element = y / 2^(byte - 127) rounded to the nearest
// of 0, 0.5, 1, 1.5, 2, 3, 4, 6, ties to the even mantissa (the comparisons below), saturated at 6.
__global__ __launch_bounds__(256) void mx4_quantize_kernel(const uint16_t* __restrict__ X, uint8_t* __restrict__ Y,
                                                           uint8_t* __restrict__ S, long long n8, float pre_scale) {
    const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
    const bool live = i < n8;  // (n8 is a multiple of 4, so the four threads of a block are live together)
    u32x4 x = {0, 0, 0, 0};
    if (live) x = *reinterpret_cast<const u32x4*>(X + i * 8);
    float v[8];
    float amax = 0.f;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        v[2 * e] = __uint_as_float(x[e] << 16) * pre_scale;
        v[2 * e + 1] = __uint_as_float(x[e] & 0xffff0000u) * pre_scale;
        amax = fmaxf(amax, fmaxf(fabsf(v[2 * e]), fabsf(v[2 * e + 1])));
    }
    amax = fmaxf(amax, __shfl_xor(amax, 1));
    amax = fmaxf(amax, __shfl_xor(amax, 2));
    const int ef = (int)((__float_as_uint(amax) >> 23) & 0xffu);
    const int sb = max(ef - 2, 0);
    const float mult = __uint_as_float((uint32_t)(254 - sb) << 23);  // 2^(127 - sb)
    uint32_t w = 0;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const float y = fabsf(v[e]) * mult;
        uint32_t c = (uint32_t)(y > 0.25f) + (uint32_t)(y >= 0.75f) + (uint32_t)(y > 1.25f) + (uint32_t)(y >= 1.75f) +
                     (uint32_t)(y > 2.5f) + (uint32_t)(y >= 3.5f) + (uint32_t)(y > 5.0f);
        c |= (__float_as_uint(v[e]) >> 28) & 8u;
        w |= c << (4 * e);
    }
    if (live) {
        *reinterpret_cast<uint32_t*>(Y + i * 4) = w;
        if ((threadIdx.x & 3) == 0) S[i >> 2] = (uint8_t)sb;
    }
}

// sabsmax of a block of MXFP4 keys, per feature over the dequantised values (tie -> the positive one), stored
// as MX blocks of E5M2: scale byte = exponent field of the block maximum - 15; codes [B*Hkv, Tc, 128],
// scales [B*Hkv, Tc, 4].  One thread per feature.
__global__ __launch_bounds__(128) void mx4_kblock_summary_kernel(const uint8_t* __restrict__ K4, const uint8_t* __restrict__ KS,
                                                                 uint8_t* __restrict__ R, uint8_t* __restrict__ RS, int N,
                                                                 int Tc) {
    const int j = blockIdx.x, bh = blockIdx.y, t = threadIdx.x;
    const int rows = min(BN, N - j * BN);
    const uint8_t* kc = K4 + ((size_t)bh * N + (size_t)j * BN) * 64 + (t >> 1);
    const uint8_t* ks = KS + ((size_t)bh * N + (size_t)j * BN) * 4 + (t >> 5);
    float best = 0.f;
    for (int r = 0; r < rows; ++r) {
        const uint32_t code = ((uint32_t)kc[(size_t)r * 64] >> (4 * (t & 1))) & 0xfu;
        const float v = __builtin_ldexpf(e2m1_value(code), (int)ks[(size_t)r * 4] - 127);
        const float av = fabsf(v), ab = fabsf(best);
        best = (r == 0 || av > ab || (av == ab && v > best)) ? v : best;
    }
    best = best == 0.f ? 0.f : best;  // a column of zeros of either sign: +0
    float amax = fabsf(best);
#pragma unroll
    for (int o = 16; o >= 1; o >>= 1) amax = fmaxf(amax, __shfl_xor(amax, o));  // the 32 features of one MX block
    const int ef = (int)((__float_as_uint(amax) >> 23) & 0xffu);
    const int sb = max(ef - 15, 0);
    const float y = __builtin_ldexpf(best, 127 - sb);  // at most 1.5 * 2^15: inside E5M2's finite range
    R[((size_t)bh * Tc + j) * 128 + t] = (uint8_t)(__builtin_amdgcn_cvt_pk_bf8_f32(y, 0.f, 0, false) & 0xff);
    if ((t & 31) == 0) RS[((size_t)bh * Tc + j) * 4 + (t >> 5)] = (uint8_t)sb;
}

__device__ __forceinline__ f32x16 mfma_f4(const u32x4& a, const u32x4& b, const f32x16& c, int scale_a, int scale_b) {
    const i32x8 av = {(int)a[0], (int)a[1], (int)a[2], (int)a[3], 0, 0, 0, 0};
    const i32x8 bv = {(int)b[0], (int)b[1], (int)b[2], (int)b[3], 0, 0, 0, 0};
    return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(av, bv, c, 4, 4, 0, scale_a, 0, scale_b);
}
__device__ __forceinline__ f32x16 mfma_bf8_f4(const i32x8& a, const u32x4& b, const f32x16& c, int scale_a, int scale_b) {
    const i32x8 bv = {(int)b[0], (int)b[1], (int)b[2], (int)b[3], 0, 0, 0, 0};
    return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, bv, c, 1, 4, 0, scale_a, 0, scale_b);
}

// byte n (0..3, per lane) of x in all four bytes
__device__ __forceinline__ int spread_byte(uint32_t x, uint32_t n) {
    return (int)__builtin_amdgcn_perm(x, x, n * 0x01010101u);
}

// 64 dwords (the four scale bytes of rows first_row .. first_row + 63 of a row-major [*, 4] array, rows clamped
// to row_limit - 1) -> LDS, by one wave
__device__ __forceinline__ void load_scales64(const uint8_t* base, int first_row, int row_limit, uint32_t* dst, int lane) {
    const uint8_t* src = base + (size_t)min(first_row + lane, row_limit - 1) * 4;
    const uint32_t lds_addr =
        __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint32_t*)dst);
    uint32_t m0_save;
    asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dword %2, off\n\ts_mov_b32 m0, %0"
                 : "=&s"(m0_save)
                 : "s"(lds_addr), "v"(src)
                 : "memory");
}

// MXFP4 K tile (64 rows of 64 bytes from a row-major [*, 64] array, rows clamped) -> LDS: four one-KiB pieces,
// one per wave
__device__ __forceinline__ void load_tile4(const uint8_t* base, int first_row, int row_limit, uint8_t* dst, int wave,
                                           int lane) {
    const int r = 16 * wave + (lane >> 2);
    const int c = (lane & 3) ^ ((r >> 2) & 3);
    const uint8_t* src = base + (size_t)min(first_row + r, row_limit - 1) * 64 + c * 16;
    const uint32_t lds_addr = __builtin_amdgcn_readfirstlane(
        (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint8_t*)(dst + wave * 1024));
    uint32_t m0_save;
    asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %2, off\n\ts_mov_b32 m0, %0"
                 : "=&s"(m0_save)
                 : "s"(lds_addr), "v"(src)
                 : "memory");
}

// S^T tile from an MXFP4 K tile and its scales: st[t][i] as in qk_tile, in units of the dequantised products
// (the block scales are applied inside the instruction), plus *start if given
__device__ __forceinline__ void qk_tile4(const uint8_t* kt, const uint32_t* ksc, const u32x4* qf, const int* qs, f32x16* st,
                                         int ql, int hh, const f32x16* start = nullptr) {
    u32x4 f[4];
    uint32_t sc[2];
#pragma unroll
    for (int t = 0; t < 2; ++t) sc[t] = ksc[32 * t + ql];
#pragma unroll
    for (int e = 0; e < 4; ++e)  // e = 2 t + kh
        f[e] = *reinterpret_cast<const u32x4*>(kt + Tile4::k_off(32 * (e >> 1) + ql, 2 * (e & 1) + hh));
#pragma unroll
    for (int e = 0; e < 4; ++e)
        st[e >> 1] = mfma_f4(f[e], qf[e & 1], (e & 1) ? st[e >> 1] : (start ? *start : f32x16{0}),
                             spread_byte(sc[e >> 1], 2 * (e & 1) + hh), qs[e & 1]);
}

struct Mx4Params {
    const uint8_t* Q;       // [B, Hq, N, 64] E2M1 pairs
    const uint8_t* Qs;      // [B, Hq, N, 4] E8M0
    const uint8_t* K;       // [B, Hkv, N, 64]
    const uint8_t* Ks;      // [B, Hkv, N, 4]
    const uint8_t* Vt;      // [B, Hkv, Tc, 128, 64] E4M3, as in the FP8 path
    const uint8_t* Krepr;   // [B, Hkv, Tc, 128] E5M2
    const uint8_t* KreprS;  // [B, Hkv, Tc, 4] E8M0
    uint16_t* O;
    float* LSE;
    int B, Hq, Hkv, N, Tr, Tc;
    int causal, n_sink, n_local, use_minit;
    float c;          // softmax scale * log2(e) (1 when FOLD)
    float descale_v;
    float headroom;
};

// As attn_fp8_kernel with the score product on MXFP4 operands.  FOLD (Alg. 1 only, softmax scale * log2(e) = 1,
// i.e. the caller folded that factor into Q before quantising): frozen tiles start their accumulators at
// -(m + H) and go to exp2 untouched.
template <int MODE, bool FOLD>
__global__ __launch_bounds__(256, 3) void attn_mx4_kernel(const Mx4Params p) {
    static_assert(!FOLD || MODE == MODE_VFA, "folding needs a max that is known before the tile");
    constexpr int D = 128, BM = 128, DB = 4;
    // Alg. 1 keeps exp(S - m) in E5M2: the summaries of MXFP4 keys collect the upward rounding errors of 64 keys per
    // feature, so the seeded max can sit ten binades above the scores, more than E4M3 has to spare
    constexpr bool P_BF8 = MODE == MODE_VFA;
    // two K stages of 4 KiB (together: the 8 KiB summary tile of the m-initialisation), two V^T stages of 8 KiB
    __shared__ __attribute__((aligned(16))) uint8_t smem[2 * Tile4::KBYTES + 2 * Tile8::VBYTES];
    __shared__ uint32_t kscale[2][BN];
    uint8_t* const Ksm = smem;
    uint8_t* const Vsm = smem + 2 * Tile4::KBYTES;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int ql = lane & 31, hh = lane >> 5;
    const int g = p.Hq / p.Hkv;
    int b, h, i;
    {
        const int id = blockIdx.x, G = p.B * p.Hkv;
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
    const int hkv = h / g, N = p.N;
    const int row0 = i * BM, last_row = min(N, row0 + BM) - 1;
    const int a_lo = row0 / BN, a_hi = last_row / BN;
    const int j_hi = p.causal ? a_hi : p.Tc - 1;
    const uint8_t* Kg = p.K + ((size_t)(b * p.Hkv + hkv) * N) * 64;
    const uint8_t* Ksg = p.Ks + ((size_t)(b * p.Hkv + hkv) * N) * 4;
    const uint8_t* Vg = p.Vt + ((size_t)(b * p.Hkv + hkv) * p.Tc) * Tile8::VBYTES;
    const int qrow = row0 + 32 * wave + ql, qrow_c = min(qrow, N - 1);
    const int limit = p.causal ? qrow_c : N - 1;
    u32x4 qf[2];
    int qs[2];
    {
        const size_t qr = (size_t)(b * p.Hq + h) * N + qrow_c;
        const uint32_t sw = *reinterpret_cast<const uint32_t*>(p.Qs + qr * 4);
#pragma unroll
        for (int kh = 0; kh < 2; ++kh) {
            qf[kh] = *reinterpret_cast<const u32x4*>(p.Q + qr * 64 + 32 * kh + 16 * hh);
            qs[kh] = spread_byte(sw, 2 * kh + hh);
        }
    }
    auto load_k = [&](int j, int buf) __attribute__((always_inline)) {
        load_tile4(Kg, j * BN, N, Ksm + buf * Tile4::KBYTES, wave, lane);
        if (wave == 0) load_scales64(Ksg, j * BN, N, kscale[buf], lane);
    };
    float m2 = -INFINITY;
    if (MODE == MODE_VFA && p.use_minit) {
        const uint8_t* Rg = p.Krepr + ((size_t)(b * p.Hkv + hkv) * p.Tc) * D;
        const uint8_t* RSg = p.KreprS + ((size_t)(b * p.Hkv + hkv) * p.Tc) * 4;
        float mx = -INFINITY;
        for (int ts = 0; ts * BN <= j_hi; ++ts) {
            __syncthreads();
            load_tile8<false, 4>(Rg, ts * BN, p.Tc, Ksm, wave, lane);
            if (wave == 0) load_scales64(RSg, ts * BN, p.Tc, kscale[0], lane);
            wait_vm0_and_sync();
            f32x16 st[2];
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                const int row = 32 * t + ql;
                const uint32_t sc = kscale[0][row];
#pragma unroll
                for (int kh = 0; kh < 2; ++kh) {
                    // 8-bit operand: bytes 0..15 of half hh are k = 16 hh + j, bytes 16..31 are k = 32 + 16 hh + j
                    const int c0 = 4 * kh + hh;
                    const i32x8 f = lds_frag8(Ksm + Tile8::k_off(row, c0), Ksm + Tile8::k_off(row, c0 + 2));
                    st[t] = mfma_bf8_f4(f, qf[kh], kh ? st[t] : f32x16{0}, spread_byte(sc, 2 * kh + hh), qs[kh]);
                }
            }
            mx = fmaxf(mx, tile_rowmax<true>(st, ts * BN, j_hi, hh));
        }
        m2 = xhalf_max(mx) * p.c;
        __syncthreads();
    }
    Params vp{};
    vp.n_sink = p.n_sink; vp.n_local = p.n_local;
    const Visit vis = make_visit<MODE>(vp, a_lo, a_hi, j_hi);
    f32x16 ot[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db) ot[db] = f32x16{0};
    float lsum = 0.f;
    {
        const int j0 = vis.tile(0);
        load_k(j0, 0);
        load_tile8<true, 4>(Vg + (size_t)j0 * Tile8::VBYTES, 0, 0, Vsm, wave, lane);
        wait_vm0_and_sync();
    }
    f32x16 start;  // FOLD: -(m + H) of this lane's query in all 16 registers, set once the max is frozen
    auto visit = [&](int k, auto special_c, auto masked_c) __attribute__((always_inline)) {
        constexpr bool SPECIAL = decltype(special_c)::value, MASKED = decltype(masked_c)::value;
        const int j = vis.tile(k), buf = k & 1;
        if (k + 1 < vis.total) {
            const int jn = vis.tile(k + 1);
            load_k(jn, buf ^ 1);
            load_tile8<true, 4>(Vg + (size_t)jn * Tile8::VBYTES, 0, 0, Vsm + (buf ^ 1) * Tile8::VBYTES, wave, lane);
        }
        f32x16 st[2];
        uint32_t pk[8];
        __builtin_amdgcn_s_setprio(1);
        if (FOLD && !SPECIAL) qk_tile4(Ksm + buf * Tile4::KBYTES, kscale[buf], qf, qs, st, ql, hh, &start);
        else qk_tile4(Ksm + buf * Tile4::KBYTES, kscale[buf], qf, qs, st, ql, hh);
        __builtin_amdgcn_s_setprio(0);
        const bool needs_mask = (p.causal && j * BN + BN - 1 > row0) || (j + 1) * BN > N;
        if (FOLD && !SPECIAL) softmax_tile8_folded<MASKED, P_BF8>(st, pk, lsum, j * BN, needs_mask ? limit : 0x3fffffff, hh);
        else softmax_tile8<SPECIAL, MASKED, P_BF8>(st, pk, ot, m2, lsum, p.c, p.headroom, j * BN, needs_mask ? limit : 0x3fffffff, hh);
        __builtin_amdgcn_s_setprio(1);
        pv_tile8<P_BF8>(Vsm + buf * Tile8::VBYTES, pk, ot, lane, hh);
        __builtin_amdgcn_s_setprio(0);
        wait_vm0_and_sync();
    };
    using std::false_type;
    using std::true_type;
    constexpr bool TAIL_SPECIAL = is_fa(MODE);
    const int n_lead = TAIL_SPECIAL ? 0 : min(vis.n_special, vis.total);
    int k_fast_end;
    {
        int j_masked = p.causal ? a_lo : p.Tc;
        if (N % BN) j_masked = min(j_masked, p.Tc - 1);
        int cnt = max(0, j_masked - vis.n1);
        if (vis.n2 > 0) cnt -= max(0, min(j_masked, vis.s2 + vis.n2) - vis.s2);
        k_fast_end = max(n_lead, min(vis.total, n_lead + cnt));
    }
    int k = 0;
    for (; k < n_lead; ++k) visit(k, true_type{}, true_type{});
    if (FOLD) {
        const float v = -(m2 + p.headroom);
#pragma unroll
        for (int r = 0; r < 16; ++r) start[r] = v;
    }
    for (; k < k_fast_end; ++k) visit(k, std::integral_constant<bool, TAIL_SPECIAL>{}, false_type{});
    for (; k < vis.total; ++k) visit(k, std::integral_constant<bool, TAIL_SPECIAL>{}, true_type{});
    const float l = xhalf_sum(lsum);
    const float inv = l > 0.f ? p.descale_v * (P_BF8 ? 0x1p-15f : 0x1p-8f) / l : 0.f;
    if (qrow < N) {
        uint16_t* Og = p.O + ((size_t)(b * p.Hq + h) * N + qrow) * D;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                const u32x2 w = {pack_bf16(ot[db][4 * q4] * inv, ot[db][4 * q4 + 1] * inv),
                                 pack_bf16(ot[db][4 * q4 + 2] * inv, ot[db][4 * q4 + 3] * inv)};
                *reinterpret_cast<u32x2*>(Og + 32 * db + 8 * q4 + 4 * hh) = w;
            }
        if (p.LSE && hh == 0)
            p.LSE[(size_t)(b * p.Hq + h) * N + qrow] =
                l > 0.f ? (m2 + p.headroom + __builtin_amdgcn_logf(l)) * kLn2 : -INFINITY;
    }
}

// ---------------------------------------------------------------------------------------------
// host side
inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline int ceil_div(int a, int b) { return (a + b - 1) / b; }

int check_common(const void* Q, const void* K, const void* V, void* O, const float* LSE, int B, int Hq, int Hkv,
                 int N, int d, int block_m, int block_n) {
    if (B < 0 || N < 0 || Hq <= 0 || Hkv <= 0 || d <= 0 || block_m <= 0 || block_n <= 0) return VFA_ERR_INVALID_ARG;
    if (Hq % Hkv != 0) return VFA_ERR_INVALID_ARG;
    if (d != 64 && d != 128) return VFA_ERR_UNSUPPORTED;
    if (!(block_n == 64 && (block_m == 64 || block_m == 128))) return VFA_ERR_UNSUPPORTED;
    if (B == 0 || N == 0) return VFA_OK;
    if (!Q || !K || !V || !O) return VFA_ERR_INVALID_ARG;
    if (!aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned16(O)) return VFA_ERR_INVALID_ARG;
    if (LSE && (reinterpret_cast<uintptr_t>(LSE) & 3u)) return VFA_ERR_INVALID_ARG;
    const long long wgs = (long long)B * Hq * ceil_div(N, block_m);
    if (wgs > 0x7fffffffLL || (long long)B * Hq * N > 0x7fffffffLL) return VFA_ERR_UNSUPPORTED;
    return VFA_OK;
}

// number of compute units of the current device (0 if the query fails), looked up once per device
int cu_count() {
    static int cached[64];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 0;
    if (cached[dev] == 0) {
        int n = 0;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = -1;
        cached[dev] = n;
    }
    return cached[dev] > 0 ? cached[dev] : 0;
}

template <int MODE>
int launch_fwd(const Params& p, int d, int block_m, hipStream_t s) {
    (void)hipGetLastError();
    const int g = p.Hq / p.Hkv;
    // ping-pong kernel: head pairs when the heads per KV head are even; otherwise (MHA, odd groups) pairs of
    // adjacent query blocks; for VSA only where each block still meets its tiles in Alg. 2's order
    // (causal, at most one local block), since the skip decisions depend on the max at the time of the visit
    const bool head_pairs = (g & 1) == 0;
    if (d == 128 && block_m == 128 && !p.order_asc && !p.all_special && !p.rowskip && !p.Qrepr &&
        !(MODE == MODE_VSA && p.tau2 >= 0.f) &&
        (head_pairs || MODE != MODE_VSA || (p.causal && p.n_local <= 1))) {
        static bool attr_set = false;  // opt in to more than 64 KB of LDS once per instantiation
        if (!attr_set) {
            if (hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_fwd_pp_kernel<MODE>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, PP_LDS_BYTES) != hipSuccess)
                return VFA_ERR_HIP;
            attr_set = true;
        }
        Params q = p;
        q.pair_blocks = head_pairs ? 0 : 1;
        unsigned n_wg = (unsigned)(head_pairs ? p.B * (p.Hq / 2) * p.Tr : p.B * p.Hq * ((p.Tr + 1) / 2));
        // One workgroup fills a CU (128 KiB of LDS), so with more work items than CUs the kernel runs one
        // persistent workgroup per CU over a static share of the items: the next item starts without a
        // workgroup launch (worth about 1 % at N = 16K and 30 % at N = 4K, measured).
        const int n_cu = cu_count();
        if (n_cu > 0 && (n_cu & 7) == 0 && n_wg > (unsigned)n_cu) {
            q.persist = n_cu;
            n_wg = (unsigned)n_cu;
        }
        const dim3 grid_pp(n_wg);
        attn_fwd_pp_kernel<MODE><<<grid_pp, 512, PP_LDS_BYTES, s>>>(q);
        return hipGetLastError() == hipSuccess ? VFA_OK : VFA_ERR_HIP;
    }
    const dim3 grid((unsigned)(p.B * p.Hq * p.Tr));
    if (d == 128 && block_m == 128) attn_fwd_kernel<128, 4, MODE><<<grid, 256, 0, s>>>(p);
    else if (d == 128 && block_m == 64) attn_fwd_kernel<128, 2, MODE><<<grid, 128, 0, s>>>(p);
    else if (d == 64 && block_m == 128) attn_fwd_kernel<64, 4, MODE><<<grid, 256, 0, s>>>(p);
    else if (d == 64 && block_m == 64) attn_fwd_kernel<64, 2, MODE><<<grid, 128, 0, s>>>(p);
    else return VFA_ERR_UNSUPPORTED;
    return hipGetLastError() == hipSuccess ? VFA_OK : VFA_ERR_HIP;
}

int summary_launch(const void* K, void* Krepr, int B, int Hkv, int N, int d, int block_n, int repr_mode, hipStream_t s) {
    const int Tc = ceil_div(N, block_n);
    const dim3 grid((unsigned)Tc, (unsigned)(B * Hkv));
    const uint16_t* k = (const uint16_t*)K;
    uint16_t* r = (uint16_t*)Krepr;
    (void)hipGetLastError();
    if (repr_mode == 0) {
        if (d == 128) kblock_summary_kernel<128><<<grid, 256, 0, s>>>(k, r, N, N, Tc, block_n, 0);
        else kblock_summary_kernel<64><<<grid, 256, 0, s>>>(k, r, N, N, Tc, block_n, 0);
    } else {
        if (d == 128) kblock_summary_alt_kernel<128><<<grid, 256, 0, s>>>(k, r, N, Tc, block_n, repr_mode);
        else kblock_summary_alt_kernel<64><<<grid, 256, 0, s>>>(k, r, N, Tc, block_n, repr_mode);
    }
    return hipGetLastError() == hipSuccess ? VFA_OK : VFA_ERR_HIP;
}

int vfa_vsa_common(int mode, const void* Q, const void* K, const void* V, void* O, float* LSE, int B, int Hq, int Hkv,
                   int N, int d, int block_m, int block_n, int causal, int n_sink, int n_local, int use_minit,
                   float softmax_scale, float thr_nats, unsigned char* skip_mask, void* workspace,
                   size_t workspace_bytes, void* stream, int repr_mode = 0, int reorder = 1, int freeze = 1,
                   int rowskip = 0, float lazy_tau = -1.f, int q_repr_mode = 0) {
    int rc = check_common(Q, K, V, O, LSE, B, Hq, Hkv, N, d, block_m, block_n);
    if (rc != VFA_OK) return rc;
    if (n_sink < 0 || n_local < 0) return VFA_ERR_INVALID_ARG;
    if (!use_minit && n_sink + n_local == 0 && freeze) return VFA_ERR_INVALID_ARG;
    if (repr_mode < 0 || repr_mode > 3) return VFA_ERR_INVALID_ARG;
    if (q_repr_mode < 0 || q_repr_mode > 3 || (q_repr_mode && use_minit != 1)) return VFA_ERR_INVALID_ARG;
    if (!(lazy_tau < 0.f) && !isfinite(lazy_tau)) return VFA_ERR_INVALID_ARG;   // negative = off; NaN / inf rejected
    if (lazy_tau != lazy_tau) return VFA_ERR_INVALID_ARG;
    if ((rowskip || lazy_tau >= 0.f) && (mode != MODE_VSA || freeze)) return VFA_ERR_INVALID_ARG;
    if (mode == MODE_VSA && !(thr_nats > 0.f && isfinite(thr_nats))) return VFA_ERR_INVALID_ARG;
    if (!isfinite(softmax_scale)) return VFA_ERR_INVALID_ARG;
    if (use_minit < 0 || use_minit > 2) return VFA_ERR_INVALID_ARG;
    if (B == 0 || N == 0) return VFA_OK;
    const size_t krepr_bytes = vfa_workspace_bytes(B, Hkv, N, d, block_n);
    if (use_minit) {
        const size_t need = krepr_bytes + (q_repr_mode ? vfa_workspace_bytes(B, Hq, N, d, block_m) : 0);
        if (!workspace || !aligned16(workspace) || workspace_bytes < need) return VFA_ERR_INVALID_ARG;
        if ((long long)B * (q_repr_mode ? Hq : Hkv) > 65535) return VFA_ERR_UNSUPPORTED;
    }
    hipStream_t s = (hipStream_t)stream;
    void* qrepr = nullptr;
    if (use_minit == 1) {
        rc = summary_launch(K, workspace, B, Hkv, N, d, block_n, repr_mode, s);
        if (rc != VFA_OK) return rc;
        if (q_repr_mode) {  // the same reductions over the query blocks: 1 = unsigned absmax, 2 = sabsmax, 3 = mean
            static const int kSummaryMode[4] = {0, 3, 0, 2};
            qrepr = (char*)workspace + krepr_bytes;
            rc = summary_launch(Q, qrepr, B, Hq, N, d, block_m, kSummaryMode[q_repr_mode], s);
            if (rc != VFA_OK) return rc;
        }
    }
    Params p{};
    p.Q = (const uint16_t*)Q; p.K = (const uint16_t*)K; p.V = (const uint16_t*)V;
    p.Krepr = (const uint16_t*)workspace; p.O = (uint16_t*)O; p.LSE = LSE; p.mask = skip_mask;
    p.Qrepr = (const uint16_t*)qrepr;
    p.B = B; p.Hq = Hq; p.Hkv = Hkv; p.N = N; p.Tr = ceil_div(N, block_m); p.Tc = ceil_div(N, block_n);
    p.causal = causal ? 1 : 0; p.n_sink = n_sink; p.n_local = n_local; p.use_minit = use_minit ? 1 : 0;
    p.order_asc = reorder ? 0 : 1; p.all_special = freeze ? 0 : 1;
    p.rowskip = rowskip ? 1 : 0; p.tau2 = lazy_tau >= 0.f ? lazy_tau : -1.f;
    const float scale = softmax_scale > 0.f ? softmax_scale : 1.0f / sqrtf((float)d);
    p.c = scale * kLog2e;
    p.thr2 = thr_nats * kLog2e;
    return mode == MODE_VSA ? launch_fwd<MODE_VSA>(p, d, block_m, s) : launch_fwd<MODE_VFA>(p, d, block_m, s);
}

int fa_common(int mode, const void* Q, const void* K, const void* V, void* O, float* LSE, int B, int Hq, int Hkv,
              int N, int d, int block_m, int block_n, int causal, float softmax_scale, float tau, void* stream) {
    int rc = check_common(Q, K, V, O, LSE, B, Hq, Hkv, N, d, block_m, block_n);
    if (rc != VFA_OK) return rc;
    if (!isfinite(softmax_scale)) return VFA_ERR_INVALID_ARG;
    if (B == 0 || N == 0) return VFA_OK;
    Params p{};
    p.Q = (const uint16_t*)Q; p.K = (const uint16_t*)K; p.V = (const uint16_t*)V;
    p.O = (uint16_t*)O; p.LSE = LSE;
    p.B = B; p.Hq = Hq; p.Hkv = Hkv; p.N = N; p.Tr = ceil_div(N, block_m); p.Tc = ceil_div(N, block_n);
    p.causal = causal ? 1 : 0;
    const float scale = softmax_scale > 0.f ? softmax_scale : 1.0f / sqrtf((float)d);
    p.c = scale * kLog2e;
    p.tau2 = tau;  // tau is already a count of factors of two: tau * ln 2 nats = tau in the log2 domain
    if (mode == MODE_FA_SOFTEXP) return launch_fwd<MODE_FA_SOFTEXP>(p, d, block_m, (hipStream_t)stream);
    if (mode == MODE_FA_LAZY) return launch_fwd<MODE_FA_LAZY>(p, d, block_m, (hipStream_t)stream);
    return launch_fwd<MODE_FA>(p, d, block_m, (hipStream_t)stream);
}

int decode_common(const void* Q, const void* K, const void* V, const void* Krepr, void* O, float* LSE, int B, int Hq,
                  int Hkv, int n_cap, int n_keys, const int* seq_lens, int d, int block_n, int n_sink, int n_local,
                  int use_minit, int n_splits, float softmax_scale, void* workspace, size_t workspace_bytes, void* stream);

}  // namespace

extern "C" {

size_t vfa_workspace_bytes(int B, int Hkv, int N, int d, int block_n) {
    if (B <= 0 || Hkv <= 0 || N <= 0 || d <= 0 || block_n <= 0) return 0;
    const size_t bytes = (size_t)B * Hkv * ceil_div(N, block_n) * d * 2;
    return (bytes + 255) & ~(size_t)255;
}

int vfa_kblock_summary(const void* K, void* Krepr, int B, int Hkv, int N, int d, int block_n, void* stream) {
    return vfa_kblock_summary_mode(K, Krepr, B, Hkv, N, d, block_n, 0, stream);
}

int vfa_kblock_summary_mode(const void* K, void* Krepr, int B, int Hkv, int N, int d, int block_n, int repr_mode,
                            void* stream) {
    if (B < 0 || N < 0 || Hkv <= 0 || block_n <= 0) return VFA_ERR_INVALID_ARG;
    if (repr_mode < 0 || repr_mode > 3) return VFA_ERR_INVALID_ARG;
    if (d != 64 && d != 128) return VFA_ERR_UNSUPPORTED;
    if (B == 0 || N == 0) return VFA_OK;
    if (!K || !Krepr || !aligned16(K) || !aligned16(Krepr)) return VFA_ERR_INVALID_ARG;
    if ((long long)B * Hkv > 65535) return VFA_ERR_UNSUPPORTED;
    return summary_launch(K, Krepr, B, Hkv, N, d, block_n, repr_mode, (hipStream_t)stream);
}

int fa_baseline_fwd(const void* Q, const void* K, const void* V, void* O, float* LSE, int B, int Hq, int Hkv, int N,
                    int d, int block_m, int block_n, int causal, float softmax_scale, void* stream) {
    return fa_common(MODE_FA, Q, K, V, O, LSE, B, Hq, Hkv, N, d, block_m, block_n, causal, softmax_scale, 0.f, stream);
}

int fa_lazy_rescale_fwd(const void* Q, const void* K, const void* V, void* O, float* LSE, int B, int Hq, int Hkv,
                        int N, int d, int block_m, int block_n, int causal, float softmax_scale, float rescale_tau,
                        void* stream) {
    if (!(rescale_tau >= 0.f && isfinite(rescale_tau))) return VFA_ERR_INVALID_ARG;
    return fa_common(MODE_FA_LAZY, Q, K, V, O, LSE, B, Hq, Hkv, N, d, block_m, block_n, causal, softmax_scale, rescale_tau,
                     stream);
}

int fa_lazy_rescale_softexp_fwd(const void* Q, const void* K, const void* V, void* O, float* LSE, int B, int Hq, int Hkv,
                                int N, int d, int block_m, int block_n, int causal, float softmax_scale,
                                float rescale_tau, void* stream) {
    if (!(rescale_tau >= 0.f && isfinite(rescale_tau))) return VFA_ERR_INVALID_ARG;
    return fa_common(MODE_FA_SOFTEXP, Q, K, V, O, LSE, B, Hq, Hkv, N, d, block_m, block_n, causal, softmax_scale,
                     rescale_tau, stream);
}

int vfa_attn_fwd(const void* Q, const void* K, const void* V, void* O, float* LSE, int B, int Hq, int Hkv, int N,
                 int d, int block_m, int block_n, int causal, int n_sink, int n_local, int use_minit,
                 float softmax_scale, void* workspace, size_t workspace_bytes, void* stream) {
    return vfa_vsa_common(MODE_VFA, Q, K, V, O, LSE, B, Hq, Hkv, N, d, block_m, block_n, causal, n_sink, n_local,
                          use_minit, softmax_scale, 0.f, nullptr, workspace, workspace_bytes, stream);
}

int vsa_attn_fwd(const void* Q, const void* K, const void* V, void* O, float* LSE, int B, int Hq, int Hkv, int N,
                 int d, int block_m, int block_n, int causal, int n_sink, int n_local, int use_minit,
                 float softmax_scale, float skip_threshold_nats, unsigned char* skip_mask, void* workspace,
                 size_t workspace_bytes, void* stream) {
    return vfa_vsa_common(MODE_VSA, Q, K, V, O, LSE, B, Hq, Hkv, N, d, block_m, block_n, causal, n_sink, n_local,
                          use_minit, softmax_scale, skip_threshold_nats, skip_mask, workspace, workspace_bytes, stream);
}

int vfa_variant_fwd(const void* Q, const void* K, const void* V, void* O, float* LSE, int B, int Hq, int Hkv, int N,
                    int d, int block_m, int block_n, int causal, int n_sink, int n_local, int use_minit, int repr_mode,
                    int q_repr_mode, int reorder, int freeze, int rowskip, float lazy_rescale_tau, float softmax_scale,
                    float skip_threshold_nats, unsigned char* skip_mask, void* workspace, size_t workspace_bytes,
                    void* stream) {
    const bool skipping = skip_threshold_nats != 0.f;
    return vfa_vsa_common(skipping ? MODE_VSA : MODE_VFA, Q, K, V, O, LSE, B, Hq, Hkv, N, d, block_m, block_n, causal,
                          n_sink, n_local, use_minit, softmax_scale, skip_threshold_nats, skipping ? skip_mask : nullptr,
                          workspace, workspace_bytes, stream, repr_mode, reorder, freeze, rowskip, lazy_rescale_tau,
                          q_repr_mode);
}

int vfa_kblock_summary_append(const void* K, void* Krepr, int B, int Hkv, int n_cap, int n_old, int n_new, int d,
                              int block_n, void* stream) {
    if (B < 0 || Hkv <= 0 || n_cap < 0 || block_n <= 0) return VFA_ERR_INVALID_ARG;
    if (n_old < 0 || n_new < n_old || n_new > n_cap) return VFA_ERR_INVALID_ARG;
    if (d != 64 && d != 128) return VFA_ERR_UNSUPPORTED;
    if (B == 0 || n_new == n_old) return VFA_OK;
    if (!K || !Krepr || !aligned16(K) || !aligned16(Krepr)) return VFA_ERR_INVALID_ARG;
    if ((long long)B * Hkv > 65535) return VFA_ERR_UNSUPPORTED;
    const int j0 = n_old / block_n, j1 = ceil_div(n_new, block_n);  // blocks [j0, j1) received keys
    const int tc_cap = ceil_div(n_cap, block_n);
    const dim3 grid((unsigned)(j1 - j0), (unsigned)(B * Hkv));
    hipStream_t s = (hipStream_t)stream;
    (void)hipGetLastError();
    if (d == 128)
        kblock_summary_kernel<128><<<grid, 256, 0, s>>>((const uint16_t*)K, (uint16_t*)Krepr, n_cap, n_new, tc_cap, block_n, j0);
    else
        kblock_summary_kernel<64><<<grid, 256, 0, s>>>((const uint16_t*)K, (uint16_t*)Krepr, n_cap, n_new, tc_cap, block_n, j0);
    return hipGetLastError() == hipSuccess ? VFA_OK : VFA_ERR_HIP;
}

size_t vfa_decode_workspace_bytes(int B, int Hq, int d, int n_splits) {
    if (B <= 0 || Hq <= 0 || d <= 0 || n_splits <= 0) return 0;
    const size_t bytes = (size_t)B * Hq * n_splits * (2 + (size_t)d) * sizeof(float);
    return (bytes + 255) & ~(size_t)255;
}

int vfa_decode_fwd(const void* Q, const void* K, const void* V, const void* Krepr, void* O, float* LSE, int B, int Hq,
                   int Hkv, int n_cap, int n_keys, int d, int block_n, int n_sink, int n_local, int use_minit,
                   int n_splits, float softmax_scale, void* workspace, size_t workspace_bytes, void* stream) {
    if (n_keys < 1 || n_keys > n_cap) return VFA_ERR_INVALID_ARG;
    return decode_common(Q, K, V, Krepr, O, LSE, B, Hq, Hkv, n_cap, n_keys, nullptr, d, block_n, n_sink, n_local, use_minit,
                         n_splits, softmax_scale, workspace, workspace_bytes, stream);
}

int vfa_decode_varlen_fwd(const void* Q, const void* K, const void* V, const void* Krepr, void* O, float* LSE, int B,
                          int Hq, int Hkv, int n_cap, const int* seq_lens, int d, int block_n, int n_sink, int n_local,
                          int use_minit, int n_splits, float softmax_scale, void* workspace, size_t workspace_bytes,
                          void* stream) {
    if (B > 0 && (!seq_lens || (reinterpret_cast<uintptr_t>(seq_lens) & 3u))) return VFA_ERR_INVALID_ARG;
    return decode_common(Q, K, V, Krepr, O, LSE, B, Hq, Hkv, n_cap, n_cap, seq_lens, d, block_n, n_sink, n_local, use_minit,
                         n_splits, softmax_scale, workspace, workspace_bytes, stream);
}

int vfa_kblock_summary_append_varlen(const void* K, void* Krepr, int B, int Hkv, int n_cap, const int* old_lens,
                                     const int* new_lens, int d, int block_n, void* stream) {
    if (B < 0 || Hkv <= 0 || n_cap < 0 || block_n <= 0) return VFA_ERR_INVALID_ARG;
    if (d != 64 && d != 128) return VFA_ERR_UNSUPPORTED;
    if (B == 0 || n_cap == 0) return VFA_OK;
    if (!K || !Krepr || !old_lens || !new_lens || !aligned16(K) || !aligned16(Krepr)) return VFA_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(old_lens) | reinterpret_cast<uintptr_t>(new_lens)) & 3u) return VFA_ERR_INVALID_ARG;
    if ((long long)B * Hkv > 65535) return VFA_ERR_UNSUPPORTED;
    const int tc_cap = ceil_div(n_cap, block_n);
    const dim3 grid((unsigned)tc_cap, (unsigned)(B * Hkv));
    hipStream_t s = (hipStream_t)stream;
    (void)hipGetLastError();
    if (d == 128)
        kblock_summary_kernel<128><<<grid, 256, 0, s>>>((const uint16_t*)K, (uint16_t*)Krepr, n_cap, 0, tc_cap, block_n, 0, old_lens, new_lens, Hkv);
    else
        kblock_summary_kernel<64><<<grid, 256, 0, s>>>((const uint16_t*)K, (uint16_t*)Krepr, n_cap, 0, tc_cap, block_n, 0, old_lens, new_lens, Hkv);
    return hipGetLastError() == hipSuccess ? VFA_OK : VFA_ERR_HIP;
}

}  // extern "C"

namespace {
int decode_common(const void* Q, const void* K, const void* V, const void* Krepr, void* O, float* LSE, int B, int Hq,
                  int Hkv, int n_cap, int n_keys, const int* seq_lens, int d, int block_n, int n_sink, int n_local,
                  int use_minit, int n_splits, float softmax_scale, void* workspace, size_t workspace_bytes, void* stream) {
    if (B < 0 || Hq <= 0 || Hkv <= 0 || n_cap <= 0 || d <= 0 || block_n <= 0) return VFA_ERR_INVALID_ARG;
    if (Hq % Hkv != 0 || n_sink < 0 || n_local < 0 || n_splits < 1 || n_splits > 4096) return VFA_ERR_INVALID_ARG;
    if (use_minit != 0 && use_minit != 1) return VFA_ERR_INVALID_ARG;
    if (!use_minit && n_sink + n_local == 0) return VFA_ERR_INVALID_ARG;
    if (!isfinite(softmax_scale)) return VFA_ERR_INVALID_ARG;
    if ((d != 64 && d != 128) || block_n != BN || Hq / Hkv > 32) return VFA_ERR_UNSUPPORTED;
    if (B == 0) return VFA_OK;
    if (!Q || !K || !V || !O || !workspace || (use_minit && !Krepr)) return VFA_ERR_INVALID_ARG;
    if (!aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned16(O) || !aligned16(workspace) ||
        (use_minit && !aligned16(Krepr)))
        return VFA_ERR_INVALID_ARG;
    if (LSE && (reinterpret_cast<uintptr_t>(LSE) & 3u)) return VFA_ERR_INVALID_ARG;
    if (workspace_bytes < vfa_decode_workspace_bytes(B, Hq, d, n_splits)) return VFA_ERR_INVALID_ARG;
    if ((long long)B * Hkv > 65535 || (long long)B * Hq > 0x7fffffffLL) return VFA_ERR_UNSUPPORTED;
    DecodeParams p{};
    p.Q = (const uint16_t*)Q; p.K = (const uint16_t*)K; p.V = (const uint16_t*)V; p.Krepr = (const uint16_t*)Krepr;
    p.O = (uint16_t*)O; p.LSE = LSE;
    p.B = B; p.Hq = Hq; p.Hkv = Hkv; p.n_cap = n_cap; p.n_keys = n_keys; p.seq_lens = seq_lens; p.tc_cap = ceil_div(n_cap, block_n);
    p.n_splits = n_splits; p.n_sink = n_sink; p.n_local = n_local; p.use_minit = use_minit;
    const float scale = softmax_scale > 0.f ? softmax_scale : 1.0f / sqrtf((float)d);
    p.c = scale * kLog2e;
    const size_t rows = (size_t)B * Hq * n_splits;
    p.opart = (float*)workspace; p.pm = p.opart + rows * d; p.lpart = p.pm + rows;  // the 16-byte stores go first
    hipStream_t s = (hipStream_t)stream;
    const dim3 grid((unsigned)n_splits, (unsigned)(B * Hkv));
    (void)hipGetLastError();
    if (d == 128) {
        decode_max_kernel<128><<<grid, 64, 0, s>>>(p);
        decode_split_kernel<128><<<grid, 64, 0, s>>>(p);
        decode_merge_kernel<128><<<(unsigned)(B * Hq), 128, 0, s>>>(p);
    } else {
        decode_max_kernel<64><<<grid, 64, 0, s>>>(p);
        decode_split_kernel<64><<<grid, 64, 0, s>>>(p);
        decode_merge_kernel<64><<<(unsigned)(B * Hq), 64, 0, s>>>(p);
    }
    return hipGetLastError() == hipSuccess ? VFA_OK : VFA_ERR_HIP;
}
}  // namespace

extern "C" {

size_t vfa_fp8_v_bytes(int B, int Hkv, int N) {
    if (B <= 0 || Hkv <= 0 || N <= 0) return 0;
    return (size_t)B * Hkv * ceil_div(N, BN) * Tile8::VBYTES;
}

int vfa_fp8_quantize(const void* X, void* X8, long long n, float inv_scale, void* stream) {
    if (n < 0 || (n & 7) || !(inv_scale > 0.f) || !isfinite(inv_scale)) return VFA_ERR_INVALID_ARG;
    if (n == 0) return VFA_OK;
    if (!X || !X8 || !aligned16(X) || (reinterpret_cast<uintptr_t>(X8) & 7u)) return VFA_ERR_INVALID_ARG;
    const long long n8 = n / 8, blocks = (n8 + 255) / 256;
    if (blocks > 0x7fffffffLL) return VFA_ERR_UNSUPPORTED;
    (void)hipGetLastError();
    fp8_quantize_kernel<<<(unsigned)blocks, 256, 0, (hipStream_t)stream>>>((const uint16_t*)X, (uint8_t*)X8, n8, inv_scale);
    return hipGetLastError() == hipSuccess ? VFA_OK : VFA_ERR_HIP;
}

int vfa_fp8_pack_v(const void* V, void* Vt, int B, int Hkv, int N, int d, float inv_scale, void* stream) {
    if (B < 0 || Hkv <= 0 || N < 0 || !(inv_scale > 0.f) || !isfinite(inv_scale)) return VFA_ERR_INVALID_ARG;
    if (d != 128) return VFA_ERR_UNSUPPORTED;
    if (B == 0 || N == 0) return VFA_OK;
    if (!V || !Vt || !aligned16(V) || !aligned16(Vt)) return VFA_ERR_INVALID_ARG;
    if ((long long)B * Hkv > 65535) return VFA_ERR_UNSUPPORTED;
    const int Tc = ceil_div(N, BN);
    (void)hipGetLastError();
    fp8_pack_v_kernel<<<dim3((unsigned)Tc, (unsigned)(B * Hkv)), 256, 0, (hipStream_t)stream>>>((const uint16_t*)V, (uint8_t*)Vt,
                                                                                              N, Tc, inv_scale);
    return hipGetLastError() == hipSuccess ? VFA_OK : VFA_ERR_HIP;
}

int vfa_fp8_attn_fwd(int frozen, const void* Q8, const void* K8, const void* Vt8, void* O, float* LSE, int B, int Hq, int Hkv,
                     int N, int d, int block_m, int block_n, int causal, int n_sink, int n_local, int use_minit,
                     float softmax_scale, float descale_q, float descale_k, float descale_v, void* workspace,
                     size_t workspace_bytes, void* stream) {
    if (B < 0 || N < 0 || Hq <= 0 || Hkv <= 0 || d <= 0 || block_m <= 0 || block_n <= 0) return VFA_ERR_INVALID_ARG;
    if (Hq % Hkv != 0 || (frozen != 0 && frozen != 1)) return VFA_ERR_INVALID_ARG;
    if (!(descale_q > 0.f && descale_k > 0.f && descale_v > 0.f) || !isfinite(descale_q * descale_k) || !isfinite(descale_v) ||
        !isfinite(softmax_scale))
        return VFA_ERR_INVALID_ARG;
    if (frozen) {
        if (n_sink < 0 || n_local < 0 || use_minit < 0 || use_minit > 2) return VFA_ERR_INVALID_ARG;
        if (!use_minit && n_sink + n_local == 0) return VFA_ERR_INVALID_ARG;
    }
    if (d != 128 || block_m != 128 || block_n != BN) return VFA_ERR_UNSUPPORTED;
    if (B == 0 || N == 0) return VFA_OK;
    if (!Q8 || !K8 || !Vt8 || !O || !aligned16(Q8) || !aligned16(K8) || !aligned16(Vt8) || !aligned16(O)) return VFA_ERR_INVALID_ARG;
    if (LSE && (reinterpret_cast<uintptr_t>(LSE) & 3u)) return VFA_ERR_INVALID_ARG;
    const int Tc = ceil_div(N, BN), Tr = ceil_div(N, block_m);
    if ((long long)B * Hq * Tr > 0x7fffffffLL || (long long)B * Hq * N > 0x7fffffffLL || (long long)B * Hkv > 65535)
        return VFA_ERR_UNSUPPORTED;
    const bool minit = frozen && use_minit;
    if (minit && (!workspace || !aligned16(workspace) || workspace_bytes < (size_t)B * Hkv * Tc * 128)) return VFA_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)stream;
    (void)hipGetLastError();
    if (minit && use_minit == 1) {
        fp8_kblock_summary_kernel<<<dim3((unsigned)Tc, (unsigned)(B * Hkv)), 128, 0, s>>>((const uint8_t*)K8, (uint8_t*)workspace, N, Tc);
        if (hipGetLastError() != hipSuccess) return VFA_ERR_HIP;
    }
    Fp8Params p{};
    p.Q = (const uint8_t*)Q8; p.K = (const uint8_t*)K8; p.Vt = (const uint8_t*)Vt8; p.Krepr = (const uint8_t*)workspace;
    p.O = (uint16_t*)O; p.LSE = LSE;
    p.B = B; p.Hq = Hq; p.Hkv = Hkv; p.N = N; p.Tr = Tr; p.Tc = Tc;
    p.causal = causal ? 1 : 0; p.n_sink = n_sink; p.n_local = n_local; p.use_minit = minit ? 1 : 0;
    const float scale = softmax_scale > 0.f ? softmax_scale : 1.0f / sqrtf((float)d);
    p.c = scale * descale_q * descale_k * kLog2e;
    p.descale_v = descale_v;
    p.headroom = frozen ? 4.f : 0.f;
    // Alg. 1 with the factor between code products and log2-domain scores a power of two (the caller's choice
    // of descale_q decides): that factor moves into the MFMA's block scale and the frozen max into its
    // accumulator start
    bool fold = false;
    if (frozen) {
        int ex = 0;
        const float mant = frexpf(p.c, &ex);  // p.c = mant * 2^ex, mant in [0.5, 1)
        if (fabsf(mant - 0.5f) <= 0x1p-18f && ex - 1 >= -100 && ex - 1 <= 100) {
            fold = true;
            p.scale_a = (127 + ex - 1) * 0x01010101;
            p.c = 1.f;
        }
    }
    const dim3 grid((unsigned)(B * Hq * Tr));
    if (fold) attn_fp8_kernel<MODE_VFA, true><<<grid, 256, 0, s>>>(p);
    else if (frozen) attn_fp8_kernel<MODE_VFA, false><<<grid, 256, 0, s>>>(p);
    else attn_fp8_kernel<MODE_FA, false><<<grid, 256, 0, s>>>(p);
    return hipGetLastError() == hipSuccess ? VFA_OK : VFA_ERR_HIP;
}

size_t vfa_mxfp4_workspace_bytes(int B, int Hkv, int N) {
    if (B <= 0 || Hkv <= 0 || N <= 0) return 0;
    const size_t bytes = (size_t)B * Hkv * ceil_div(N, BN) * (128 + 4);
    return (bytes + 255) & ~(size_t)255;
}

int vfa_mxfp4_quantize(const void* X, void* X4, void* XS, long long n, float pre_scale, void* stream) {
    if (n < 0 || (n & 31) || !(pre_scale > 0.f) || !isfinite(pre_scale)) return VFA_ERR_INVALID_ARG;
    if (n == 0) return VFA_OK;
    if (!X || !X4 || !XS || !aligned16(X) || (reinterpret_cast<uintptr_t>(X4) & 3u)) return VFA_ERR_INVALID_ARG;
    const long long n8 = n / 8, blocks = (n8 + 255) / 256;
    if (blocks > 0x7fffffffLL) return VFA_ERR_UNSUPPORTED;
    (void)hipGetLastError();
    mx4_quantize_kernel<<<(unsigned)blocks, 256, 0, (hipStream_t)stream>>>((const uint16_t*)X, (uint8_t*)X4, (uint8_t*)XS, n8,
                                                                          pre_scale);
    return hipGetLastError() == hipSuccess ? VFA_OK : VFA_ERR_HIP;
}

int vfa_mxfp4_attn_fwd(int frozen, const void* Q4, const void* QS, const void* K4, const void* KS, const void* Vt8, void* O,
                       float* LSE, int B, int Hq, int Hkv, int N, int d, int block_m, int block_n, int causal, int n_sink,
                       int n_local, int use_minit, float softmax_scale, float descale_v, void* workspace,
                       size_t workspace_bytes, void* stream) {
    if (B < 0 || N < 0 || Hq <= 0 || Hkv <= 0 || d <= 0 || block_m <= 0 || block_n <= 0) return VFA_ERR_INVALID_ARG;
    if (Hq % Hkv != 0 || (frozen != 0 && frozen != 1)) return VFA_ERR_INVALID_ARG;
    if (!(descale_v > 0.f) || !isfinite(descale_v) || !isfinite(softmax_scale)) return VFA_ERR_INVALID_ARG;
    if (frozen) {
        if (n_sink < 0 || n_local < 0 || use_minit < 0 || use_minit > 2) return VFA_ERR_INVALID_ARG;
        if (!use_minit && n_sink + n_local == 0) return VFA_ERR_INVALID_ARG;
    }
    if (d != 128 || block_m != 128 || block_n != BN) return VFA_ERR_UNSUPPORTED;
    if (B == 0 || N == 0) return VFA_OK;
    if (!Q4 || !QS || !K4 || !KS || !Vt8 || !O) return VFA_ERR_INVALID_ARG;
    if (!aligned16(Q4) || !aligned16(K4) || !aligned16(Vt8) || !aligned16(O)) return VFA_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(QS) & 3u) || (reinterpret_cast<uintptr_t>(KS) & 3u)) return VFA_ERR_INVALID_ARG;
    if (LSE && (reinterpret_cast<uintptr_t>(LSE) & 3u)) return VFA_ERR_INVALID_ARG;
    const int Tc = ceil_div(N, BN), Tr = ceil_div(N, block_m);
    if ((long long)B * Hq * Tr > 0x7fffffffLL || (long long)B * Hq * N > 0x7fffffffLL || (long long)B * Hkv > 65535)
        return VFA_ERR_UNSUPPORTED;
    const bool minit = frozen && use_minit;
    if (minit && (!workspace || !aligned16(workspace) || workspace_bytes < vfa_mxfp4_workspace_bytes(B, Hkv, N)))
        return VFA_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)stream;
    uint8_t* const repr = (uint8_t*)workspace;
    uint8_t* const repr_s = repr ? repr + (size_t)B * Hkv * Tc * 128 : nullptr;  // (a multiple of 128: dword aligned)
    (void)hipGetLastError();
    if (minit && use_minit == 1) {
        mx4_kblock_summary_kernel<<<dim3((unsigned)Tc, (unsigned)(B * Hkv)), 128, 0, s>>>((const uint8_t*)K4, (const uint8_t*)KS,
                                                                                         repr, repr_s, N, Tc);
        if (hipGetLastError() != hipSuccess) return VFA_ERR_HIP;
    }
    Mx4Params p{};
    p.Q = (const uint8_t*)Q4; p.Qs = (const uint8_t*)QS; p.K = (const uint8_t*)K4; p.Ks = (const uint8_t*)KS;
    p.Vt = (const uint8_t*)Vt8; p.Krepr = repr; p.KreprS = repr_s;
    p.O = (uint16_t*)O; p.LSE = LSE;
    p.B = B; p.Hq = Hq; p.Hkv = Hkv; p.N = N; p.Tr = Tr; p.Tc = Tc;
    p.causal = causal ? 1 : 0; p.n_sink = n_sink; p.n_local = n_local; p.use_minit = minit ? 1 : 0;
    const float scale = softmax_scale > 0.f ? softmax_scale : 1.0f / sqrtf((float)d);
    p.c = scale * kLog2e;
    p.descale_v = descale_v;
    p.headroom = frozen ? 4.f : 0.f;
    // Alg. 1 with the scores already in log2 units (the caller multiplied Q by scale * log2(e) before quantising
    // and passes softmax_scale = ln 2): nothing is left to multiply, and the frozen max becomes the accumulators' start
    const bool fold = frozen && fabsf(p.c - 1.f) <= 0x1p-18f;
    if (fold) p.c = 1.f;
    const dim3 grid((unsigned)(B * Hq * Tr));
    if (fold) attn_mx4_kernel<MODE_VFA, true><<<grid, 256, 0, s>>>(p);
    else if (frozen) attn_mx4_kernel<MODE_VFA, false><<<grid, 256, 0, s>>>(p);
    else attn_mx4_kernel<MODE_FA, false><<<grid, 256, 0, s>>>(p);
    return hipGetLastError() == hipSuccess ? VFA_OK : VFA_ERR_HIP;
}

const char* vfa_strerror(int code) {
    switch (code) {
        case VFA_OK: return "ok";
        case VFA_ERR_INVALID_ARG: return "invalid argument";
        case VFA_ERR_UNSUPPORTED: return "unsupported shape (d must be 64 or 128; blocks 64x64 or 128x64)";
        case VFA_ERR_HIP: return "HIP launch error";
        default: return "unknown error code";
    }
}

}  // extern "C"
