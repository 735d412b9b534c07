// FP8 (E4M3) attention kernel and its pre-passes.
#pragma once
#include "common.hpp"

namespace {

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

// a wave-uniform pointer as two scalar registers (the compiler cannot always see that it is uniform)
__device__ __forceinline__ uint64_t uniform_ptr(const void* ptr) {
    const uint64_t b64 = (uint64_t)(uintptr_t)ptr;
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((uint32_t)b64);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((uint32_t)(b64 >> 32));
    return ((uint64_t)hi << 32) | (uint64_t)lo;
}

// one LDS-direct load: lane l's 16 (BYTES = 16) or 4 bytes at base + off go to LDS address lds_addr + BYTES * l.
// Scalar base plus a 32-bit lane offset: one address register per lane instead of a 64-bit pointer.
template <int BYTES>
__device__ __forceinline__ void lds_dma(uint64_t base, uint32_t off, uint32_t lds_addr) {
    uint32_t m0_save;
    if (BYTES == 16)
        asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %2, %3\n\ts_mov_b32 m0, %0"
                     : "=&s"(m0_save)
                     : "s"(lds_addr), "v"(off), "s"(base)
                     : "memory");
    else
        asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dword %2, %3\n\ts_mov_b32 m0, %0"
                     : "=&s"(m0_save)
                     : "s"(lds_addr), "v"(off), "s"(base)
                     : "memory");
}

// K tile (IS_V = false: rows of 128 bytes from a row-major [*, 128] array, rows clamped to row_limit - 1)
// or V^T tile (IS_V = true: a contiguous 8 KiB block) -> LDS, 8 one-KiB pieces shared by NWAVES waves.
// base is the same for all lanes of the wave.
template <bool IS_V, int NWAVES>
__device__ __forceinline__ void load_tile8(const uint8_t* base, int first_row, int row_limit, uint8_t* dst, int wave,
                                           int lane) {
    constexpr int NI = 8 / NWAVES;
    const uint64_t sb = uniform_ptr(base);
#pragma unroll
    for (int u = 0; u < NI; ++u) {
        const int q = u * NWAVES + wave;
        int r, c;
        uint32_t off;
        if (IS_V) {
            r = 16 * q + (lane >> 2);
            c = (lane & 3) ^ ((r >> 2) & 3);
            off = (uint32_t)(r * 64 + c * 16);
        } else {
            r = 8 * q + (lane >> 3);
            c = (lane & 7) ^ ((r >> 1) & 7);
            off = (uint32_t)min(first_row + r, row_limit - 1) * 128u + (uint32_t)(c * 16);
        }
        const uint32_t lds_addr = __builtin_amdgcn_readfirstlane(
            (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint8_t*)(dst + q * 1024));
        lds_dma<16>(sb, off, lds_addr);
    }
}

__device__ __forceinline__ i32x8 lds_frag8(const uint8_t* a0, const uint8_t* a1) {
    const u32x4 lo = *reinterpret_cast<const u32x4*>(a0), hi = *reinterpret_cast<const u32x4*>(a1);
    return i32x8{(int)lo[0], (int)lo[1], (int)lo[2], (int)lo[3], (int)hi[0], (int)hi[1], (int)hi[2], (int)hi[3]};
}

// S^T tile from an E4M3 K tile: st[t][i] as in qk_tile: products of the codes' values times the power of
// two in scale_a, plus *start (a value per lane, i.e. per query, already spread over 16 registers) if given
// (NARROW: two fragments in flight instead of four, for a kernel that is short of registers)
template <bool NARROW = false>
__device__ __forceinline__ void qk_tile8(const uint8_t* kt, const i32x8* qf, f32x16* st, int ql, int hh,
                                         int scale_a = 0x7f7f7f7f, const f32x16* start = nullptr) {
    if (NARROW) {
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            i32x8 g[2];
#pragma unroll
            for (int kh = 0; kh < 2; ++kh) {
                const int row = 32 * t + ql, c0 = 4 * kh + 2 * hh;
                g[kh] = lds_frag8(kt + Tile8::k_off(row, c0), kt + Tile8::k_off(row, c0 + 1));
            }
            st[t] = mfma_f8(g[0], qf[0], start ? *start : f32x16{0}, scale_a);
            st[t] = mfma_f8(g[1], qf[1], st[t], scale_a);
        }
        return;
    }
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
template <bool P_BF8 = false, bool NARROW = false>
__device__ __forceinline__ void pv_tile8(const uint8_t* vt, const uint32_t* pk, f32x16* ot, int lane, int hh) {
    const i32x8 pf = {(int)pk[0], (int)pk[1], (int)pk[2], (int)pk[3], (int)pk[4], (int)pk[5], (int)pk[6], (int)pk[7]};
    if (NARROW) {  // two fragments in flight instead of four
#pragma unroll
        for (int d2 = 0; d2 < 2; ++d2) {
            i32x8 g[2];
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const int row = 32 * (2 * d2 + u) + (lane & 31);
                g[u] = lds_frag8(vt + Tile8::v_off(row, 2 * hh), vt + Tile8::v_off(row, 2 * hh + 1));
            }
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const int db = 2 * d2 + u;
                ot[db] = P_BF8 ? __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(g[u], pf, ot[db], 0, 1, 0, 0x7f7f7f7f, 0, 0x7f7f7f7f)
                               : mfma_f8(g[u], pf, ot[db]);
            }
        }
        return;
    }
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
    // each conversion writes one half of w and keeps the other: start from whatever the register holds (an empty
    // asm "defines" it) instead of spending a move per dword on a zero that the second conversion overwrites
    uint32_t w0;
    asm volatile("" : "=v"(w0));
    s16x2 w = __builtin_bit_cast(s16x2, w0);
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

// ---- Alg. 1 without exponentials (NOEXP).  The code of a small float read as an integer is a piecewise-linear
// logarithm: an E5M2 code c = 4 E + m stands for 2^(E - 15) (1 + m / 4), the chord approximation of
// 2^(c / 4 - 15), never more than 6.15 % above it.  So when a score arrives as x = s - m - H in log2 units, the
// code of exp2(x) 2^15 is, up to that chord error and the rounding to a quarter of a binade, just
// round(4 x + 120): a multiply-add and a float-to-byte conversion.  The multiply (4 = 2^2) goes into the MFMA's
// block scale and the add into its accumulator start (the frozen max is known before the tile), so a frozen
// tile's scores leave the matrix unit AS CODES: what is left per score is a clamp to the largest finite code and
// v_cvt_pk_u8_f32 (round to nearest even, saturating at 0: measured).  The offset is lowered by
// 4 log2(1.0303) = 0.1723 to centre the chord error: weight / exact weight lies in [0.89, 1.12] (the format's
// own rounding would give +-12.5 %).  E5M2 rather than E4M3 because the window has to hold, below the frozen max,
// the headroom, the overshoot of the seed and the spread of the row, and E4M3's subnormal codes, which the
// rounded-exponential path leans on for its last three binades, are not logarithmic.  The row sum comes from
// the same rounded weights through one more MFMA (a block of ones times P), so O = sum(w v) / sum(w) is a properly
// normalised average under weights that are each within 12 % of the exact ones; LSE inherits that error.
constexpr float kCodeOffset = 119.8277f;  // 4 * (15 + 15) - 0.1723
constexpr float kMaxCode = 123.f;          // 0x7B = 57344, the largest finite E5M2 value
constexpr float kCodesPerBinade = 4.f;

template <bool MASKED>
__device__ __forceinline__ void codes_tile8(f32x16* st, uint32_t* pk, int key0, int limit, int hh, float add = 0.f) {
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int r = 0; r < 16; r += 4) {
            uint32_t w = 0;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                float c = __builtin_amdgcn_fmed3f(st[t][r + e] + add, 0.f, kMaxCode);  // (fminf would first quiet a NaN)
                if (MASKED) c = (32 * t + 8 * ((r + e) >> 2) + ((r + e) & 3) <= limit - key0 - 4 * hh) ? c : 0.f;
                w = __builtin_amdgcn_cvt_pk_u8_f32(c, e, w);
            }
            pk[4 * t + (r >> 2)] = w;
        }
}

// exact-max tile of the NOEXP form: st holds 4 * (log2-domain scores); row max, rescale of ot and of the row-sum
// block lt, then codes relative to the new max
template <bool MASKED>
__device__ __forceinline__ void special_tile8_noexp(f32x16* st, uint32_t* pk, f32x16* ot, f32x16& lt, float& m2, float headroom,
                                                    int key0, int limit, int hh) {
    if (MASKED) {
        const int rel = limit - key0 - 4 * hh;
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int r = 0; r < 16; ++r) st[t][r] = (32 * t + 8 * (r >> 2) + (r & 3) <= rel) ? st[t][r] : -INFINITY;
    }
    const float mx = tile_rowmax<false>(st, 0, 0, hh);
    const float m_new = fmaxf(m2, xhalf_max(mx) * (1.f / kCodesPerBinade));
    const float msub = (m_new == -INFINITY) ? 0.f : m_new;
    const float alpha = __builtin_amdgcn_exp2f(m2 - msub);
    lt *= alpha;
#pragma unroll
    for (int db = 0; db < 4; ++db) ot[db] *= alpha;
    m2 = m_new;
    const float sub = kCodesPerBinade * (msub + headroom) - kCodeOffset;
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) st[t][r] -= sub;   // (-inf stays -inf: code 0)
    codes_tile8<false>(st, pk, 0, 0, hh);
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
template <int MODE, bool FOLD, bool NOEXP = false>
__global__ __launch_bounds__(256, FOLD ? 3 : 2) void attn_fp8_kernel(const Fp8Params p) {
    static_assert(!FOLD || MODE == MODE_VFA, "folding needs a max that is known before the tile");
    static_assert(!NOEXP || FOLD, "codes straight from the matrix unit need the scale and the max folded into it");
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
    float code0 = 0.f;  // NOEXP: code offset - 4 (m + H), added on the vector side (16 registers matter more than 32 adds)
    f32x16 lt = {0};  // NOEXP: 32 copies of this lane's row sum of the rounded weights (times 2^15)
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
        if (NOEXP) qk_tile8<true>(Ks + buf * Tile8::KBYTES, qf, st, ql, hh, sa);
        else if (FOLD && !SPECIAL) qk_tile8(Ks + buf * Tile8::KBYTES, qf, st, ql, hh, sa, &start);
        else qk_tile8(Ks + buf * Tile8::KBYTES, qf, st, ql, hh, sa);
        __builtin_amdgcn_s_setprio(0);
        const bool needs_mask = (p.causal && j * BN + BN - 1 > row0) || (j + 1) * BN > N;
        if (NOEXP && !SPECIAL) codes_tile8<MASKED>(st, pk, j * BN, needs_mask ? limit : 0x3fffffff, hh, code0);
        else if (NOEXP) special_tile8_noexp<MASKED>(st, pk, ot, lt, m2, p.headroom, j * BN, needs_mask ? limit : 0x3fffffff, hh);
        else if (FOLD && !SPECIAL) softmax_tile8_folded<MASKED>(st, pk, lsum, j * BN, needs_mask ? limit : 0x3fffffff, hh);
        else softmax_tile8<SPECIAL, MASKED>(st, pk, ot, m2, lsum, p.c, p.headroom, j * BN, needs_mask ? limit : 0x3fffffff, hh);
        __builtin_amdgcn_s_setprio(1);
        pv_tile8<NOEXP, NOEXP>(Vs + buf * Tile8::VBYTES, pk, ot, lane, hh);
        if (NOEXP) {
            // row sums of the rounded weights: a block of ones times P (E5M2).  The ones are E2M1 (1.0 = code 2): a
            // 4-bit operand takes four registers instead of eight, and with all elements equal the different order of
            // the k index in 4-bit and 8-bit operands does not matter
            const i32x8 ones = {0x22222222, 0x22222222, 0x22222222, 0x22222222, 0, 0, 0, 0};
            const i32x8 pf = {(int)pk[0], (int)pk[1], (int)pk[2], (int)pk[3], (int)pk[4], (int)pk[5], (int)pk[6], (int)pk[7]};
            lt = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(ones, pf, lt, 4, 1, 0, 0x7f7f7f7f, 0, 0x7f7f7f7f);
        }
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
        if (NOEXP) code0 = kCodeOffset + kCodesPerBinade * v;
#pragma unroll
        for (int r = 0; r < 16; ++r) start[r] = v;
    }
    for (; k < k_fast_end; ++k) visit(k, std::integral_constant<bool, TAIL_SPECIAL>{}, false_type{});
    for (; k < vis.total; ++k) visit(k, std::integral_constant<bool, TAIL_SPECIAL>{}, true_type{});
    // O = descale_v * 2^-8 * O^T / l (the codes of P carry 2^8); LSE = (m2 + H + log2 l) ln 2  (l sums exp2(s c - m2 - H))
    // (NOEXP: every register of lt holds the whole row sum, with the same 2^15 as the numerator)
    const float l = NOEXP ? lt[0] * 0x1p-15f : xhalf_sum(lsum);
    const float inv = l > 0.f ? p.descale_v * (NOEXP ? 0x1p-15f : 0x1p-8f) / l : 0.f;
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

// sabsmax over E4M3 codes (sign-magnitude: the 7 low bits order the magnitudes; tie -> the positive code, the
// smaller one; the rule is commutative and associative, so any reduction order gives the same bytes).
// 256 threads: thread (rg, ch) takes the 16-byte chunk ch of rows rg and rg + 32 (rows past the end of a ragged
// block repeat its last row, which changes nothing), then 128 threads fold the 32 partial rows of one feature each.
__device__ __forceinline__ uint32_t fp8_sabs_pick(uint32_t a, uint32_t b) {
    const uint32_t ma = a & 0x7f, mb = b & 0x7f;
    return mb > ma ? b : (ma > mb ? a : min(a, b));
}
__global__ __launch_bounds__(256) void fp8_kblock_summary_kernel(const uint8_t* __restrict__ K, uint8_t* __restrict__ R, int N,
                                                                 int Tc) {
    __shared__ u32x4 part[32][8];
    const int j = blockIdx.x, bh = blockIdx.y, tid = threadIdx.x;
    const int rg = tid >> 3, ch = tid & 7;
    const int rows = min(BN, N - j * BN);
    const uint8_t* base = K + ((size_t)bh * N + (size_t)j * BN) * 128 + ch * 16;
    const u32x4 a = *reinterpret_cast<const u32x4*>(base + (size_t)min(rg, rows - 1) * 128);
    const u32x4 b = *reinterpret_cast<const u32x4*>(base + (size_t)min(rg + 32, rows - 1) * 128);
    u32x4 best;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        uint32_t w = 0;
#pragma unroll
        for (int q = 0; q < 4; ++q) w |= fp8_sabs_pick((a[e] >> (8 * q)) & 0xffu, (b[e] >> (8 * q)) & 0xffu) << (8 * q);
        best[e] = w;
    }
    part[rg][ch] = best;
    __syncthreads();
    if (tid < 128) {
        const uint8_t* col = reinterpret_cast<const uint8_t*>(&part[0][0]) + tid;
        uint32_t v = col[0];
        for (int r = 1; r < 32; ++r) v = fp8_sabs_pick(v, col[r * 128]);
        R[((size_t)bh * Tc + j) * 128 + tid] = (uint8_t)v;
    }
}

}  // namespace
