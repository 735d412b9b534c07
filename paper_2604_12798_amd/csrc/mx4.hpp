// Attention with MXFP4 scores (E2M1 elements, E8M0 block scales) and its pre-passes.
#pragma once
#include "common.hpp"
#include "fp8.hpp"

namespace {

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
// scales [B*Hkv, Tc, 4].  256 threads: thread (row, blk) dequantises the 32 elements of MX block blk of key row
// into LDS (rows past the end of a ragged block repeat its last row), then one thread per feature folds the 64
// rows; the pick is commutative and associative up to the sign of a zero, which is set to + at the end.
__global__ __launch_bounds__(256) void mx4_kblock_summary_kernel(const uint8_t* __restrict__ K4, const uint8_t* __restrict__ KS,
                                                                 uint8_t* __restrict__ R, uint8_t* __restrict__ RS, int N,
                                                                 int Tc) {
    __shared__ float val[BN][128 + 1];
    const int j = blockIdx.x, bh = blockIdx.y, tid = threadIdx.x;
    const int rows = min(BN, N - j * BN);
    {
        const int row = tid >> 2, blk = tid & 3;
        const size_t r = (size_t)bh * N + (size_t)j * BN + min(row, rows - 1);
        const u32x4 c = *reinterpret_cast<const u32x4*>(K4 + r * 64 + blk * 16);
        const int e = (int)KS[r * 4 + blk] - 127;
#pragma unroll
        for (int q = 0; q < 32; ++q) val[row][32 * blk + q] = __builtin_ldexpf(e2m1_value((c[q >> 3] >> (4 * (q & 7))) & 0xfu), e);
    }
    __syncthreads();
    if (tid < 128) {
        const int t = tid;
        float best = val[0][t];
        for (int r = 1; r < BN; ++r) {
            const float v = val[r][t];
            const float av = fabsf(v), ab = fabsf(best);
            best = (av > ab || (av == ab && v > best)) ? v : best;
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
// to row_limit - 1) -> LDS, by one wave; base is the same for all lanes
__device__ __forceinline__ void load_scales64(const uint8_t* base, int first_row, int row_limit, uint32_t* dst, int lane) {
    const uint32_t lds_addr =
        __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint32_t*)dst);
    lds_dma<4>(uniform_ptr(base), (uint32_t)min(first_row + lane, row_limit - 1) * 4u, lds_addr);
}

// MXFP4 K tile (64 rows of 64 bytes from a row-major [*, 64] array, rows clamped) -> LDS: four one-KiB pieces,
// one per wave; base is the same for all lanes
__device__ __forceinline__ void load_tile4(const uint8_t* base, int first_row, int row_limit, uint8_t* dst, int wave,
                                           int lane) {
    const int r = 16 * wave + (lane >> 2);
    const int c = (lane & 3) ^ ((r >> 2) & 3);
    const uint32_t lds_addr = __builtin_amdgcn_readfirstlane(
        (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint8_t*)(dst + wave * 1024));
    lds_dma<16>(uniform_ptr(base), (uint32_t)min(first_row + r, row_limit - 1) * 64u + (uint32_t)(c * 16), lds_addr);
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
// NOEXP (with FOLD): the weights' E5M2 codes are taken from the scores as in attn_fp8_kernel's form without
// exponentials; the factor 4 of the code scale is added to the queries' block-scale bytes (two binades).
template <int MODE, bool FOLD, bool NOEXP = false>
__global__ __launch_bounds__(256, 3) void attn_mx4_kernel(const Mx4Params p) {
    static_assert(!FOLD || MODE == MODE_VFA, "folding needs a max that is known before the tile");
    static_assert(!NOEXP || FOLD, "codes straight from the matrix unit need the scores in log2 units");
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
            qs[kh] = spread_byte(sw, 2 * kh + hh) + (NOEXP ? 0x02020202 : 0);  // (scale bytes of real data are far from 253)
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
    f32x16 lt = {0};   // NOEXP: 32 copies of this lane's row sum of the rounded weights (times 2^15)
    float code0 = 0.f;  // NOEXP: code offset - 4 (m + H)
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
        if (FOLD && !SPECIAL && !NOEXP) qk_tile4(Ksm + buf * Tile4::KBYTES, kscale[buf], qf, qs, st, ql, hh, &start);
        else qk_tile4(Ksm + buf * Tile4::KBYTES, kscale[buf], qf, qs, st, ql, hh);
        __builtin_amdgcn_s_setprio(0);
        const bool needs_mask = (p.causal && j * BN + BN - 1 > row0) || (j + 1) * BN > N;
        if (NOEXP && !SPECIAL) codes_tile8<MASKED>(st, pk, j * BN, needs_mask ? limit : 0x3fffffff, hh, code0);
        else if (NOEXP) special_tile8_noexp<MASKED>(st, pk, ot, lt, m2, p.headroom, j * BN, needs_mask ? limit : 0x3fffffff, hh);
        else if (FOLD && !SPECIAL) softmax_tile8_folded<MASKED, P_BF8>(st, pk, lsum, j * BN, needs_mask ? limit : 0x3fffffff, hh);
        else softmax_tile8<SPECIAL, MASKED, P_BF8>(st, pk, ot, m2, lsum, p.c, p.headroom, j * BN, needs_mask ? limit : 0x3fffffff, hh);
        __builtin_amdgcn_s_setprio(1);
        pv_tile8<P_BF8>(Vsm + buf * Tile8::VBYTES, pk, ot, lane, hh);
        if (NOEXP) {  // row sums of the rounded weights: a block of E2M1 ones times P (E5M2)
            const i32x8 ones = {0x22222222, 0x22222222, 0x22222222, 0x22222222, 0, 0, 0, 0};
            const i32x8 pf = {(int)pk[0], (int)pk[1], (int)pk[2], (int)pk[3], (int)pk[4], (int)pk[5], (int)pk[6], (int)pk[7]};
            lt = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(ones, pf, lt, 4, 1, 0, 0x7f7f7f7f, 0, 0x7f7f7f7f);
        }
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
        if (NOEXP) code0 = kCodeOffset + kCodesPerBinade * v;
#pragma unroll
        for (int r = 0; r < 16; ++r) start[r] = v;
    }
    for (; k < k_fast_end; ++k) visit(k, std::integral_constant<bool, TAIL_SPECIAL>{}, false_type{});
    for (; k < vis.total; ++k) visit(k, std::integral_constant<bool, TAIL_SPECIAL>{}, true_type{});
    // (NOEXP: every register of lt holds the whole row sum, with the same 2^15 as the numerator)
    const float l = NOEXP ? lt[0] * 0x1p-15f : xhalf_sum(lsum);
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

}  // namespace
