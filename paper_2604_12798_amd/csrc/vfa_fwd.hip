// C ABI of libvfa.so (declared in vfa.h): argument checks, kernel selection and launches.  The kernels live in the
// headers included below and are compiled for gfx950 in this translation unit, except attn_vsa_pp_kernel (vsa_pp.hip).
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <math.h>
#include <atomic>

#include "vfa.h"

#include "common.hpp"
#include "attn_generic.hpp"
#include "attn_pingpong.hpp"
#include "vsa_pp.hpp"
#include "summary.hpp"
#include "decode.hpp"
#include "fp8.hpp"
#include "mx4.hpp"

namespace {

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

// Host-side caches.  Everything the library remembers between calls is a per-device fact that any thread would
// compute to the same value (a CU count, "this kernel's LDS limit has been raised", the address of the device
// array below), held in atomics: two threads that race on a first call both do the lookup and store the same thing.
constexpr int kMaxDevices = 64;

int current_device() {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return -1;
    return dev;
}

// number of compute units of the current device (0 if the query fails), looked up once per device
int cu_count() {
    static std::atomic<int> cached[kMaxDevices];
    const int dev = current_device();
    if (dev < 0) return 0;
    int n = cached[dev].load(std::memory_order_relaxed);
    if (n == 0) {
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = -1;
        cached[dev].store(n, std::memory_order_relaxed);
    }
    return n > 0 ? n : 0;
}

// opt a kernel in to more than 64 KiB of LDS, once per kernel and device (idempotent, so a race only repeats it)
template <typename KernelT>
bool raise_lds_limit(KernelT kernel, int bytes, std::atomic<unsigned char>* done) {
    const int dev = current_device();
    if (dev < 0) return false;
    if (done[dev].load(std::memory_order_acquire)) return true;
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, bytes) != hipSuccess)
        return false;
    done[dev].store(1, std::memory_order_release);
    return true;
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
        static std::atomic<unsigned char> lds_raised[kMaxDevices];  // one set of flags per instantiation
        if constexpr (MODE == MODE_VSA) {
            const int dev = current_device();
            if (dev < 0) return VFA_ERR_HIP;
            if (!lds_raised[dev].load(std::memory_order_acquire)) {
                if (vfa_detail_vsa_pp_raise_lds() != 0) return VFA_ERR_HIP;
                lds_raised[dev].store(1, std::memory_order_release);
            }
        } else {
            if (!raise_lds_limit(&attn_fwd_pp_kernel<MODE>, PP_LDS_BYTES, lds_raised)) return VFA_ERR_HIP;
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
        if constexpr (MODE == MODE_VSA) return vfa_detail_vsa_pp_launch(&q, sizeof(q), n_wg, s) == 0 ? VFA_OK : VFA_ERR_HIP;
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
    const dim3 grid4((unsigned)ceil_div(Tc, 4), (unsigned)(B * Hkv));  // sabsmax: one wave per block, four to a workgroup
    const uint16_t* k = (const uint16_t*)K;
    uint16_t* r = (uint16_t*)Krepr;
    (void)hipGetLastError();
    if (repr_mode == 0) {
        if (d == 128) kblock_summary_kernel<128><<<grid4, 256, 0, s>>>(k, r, N, N, Tc, block_n, 0, Tc);
        else kblock_summary_kernel<64><<<grid4, 256, 0, s>>>(k, r, N, N, Tc, block_n, 0, Tc);
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
    // ascending order, no seed, no sink block: a query block whose first key block is not one of its local ones would
    // meet a frozen tile with the max still at -inf
    if (!use_minit && !reorder && n_sink == 0 && freeze) return VFA_ERR_INVALID_ARG;
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

// The one device array of the library: the partial sums of vfa_decode_noalloc_fwd's key ranges (what the
// workspace argument carries in vfa_decode_fwd).  Every device the library is used on holds its own copy, at
// its own address, until the process ends.  In host code the name below is only a handle for
// hipGetSymbolAddress: the kernels receive the address that call returns, never the name.
static __device__ __align__(256) unsigned char scratch[VFA_DECODE_NOALLOC_MAX_BYTES];

namespace {

// device address of `scratch` on the calling thread's current device; looked up on the first call per device
void* scratch_address() {
    static std::atomic<void*> addr[kMaxDevices];
    const int dev = current_device();
    if (dev < 0) return nullptr;
    void* ptr = addr[dev].load(std::memory_order_acquire);
    if (!ptr) {
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) {
            (void)hipGetLastError();
            return nullptr;
        }
        addr[dev].store(ptr, std::memory_order_release);
    }
    return ptr;
}

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
    const dim3 grid((unsigned)ceil_div(j1 - j0, 4), (unsigned)(B * Hkv));
    hipStream_t s = (hipStream_t)stream;
    (void)hipGetLastError();
    if (d == 128)
        kblock_summary_kernel<128><<<grid, 256, 0, s>>>((const uint16_t*)K, (uint16_t*)Krepr, n_cap, n_new, tc_cap, block_n, j0, j1 - j0);
    else
        kblock_summary_kernel<64><<<grid, 256, 0, s>>>((const uint16_t*)K, (uint16_t*)Krepr, n_cap, n_new, tc_cap, block_n, j0, j1 - j0);
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

int vfa_decode_noalloc_fwd(const void* Q, const void* K, const void* V, const void* Krepr, void* O, float* LSE, int B,
                           int Hq, int Hkv, int n_cap, int n_keys, int d, int block_n, int n_sink, int n_local,
                           int use_minit, int n_splits, float softmax_scale, void* stream) {
    if (n_keys < 1 || n_keys > n_cap) return VFA_ERR_INVALID_ARG;
    if (B < 0 || Hq <= 0 || d <= 0 || n_splits < 1) return VFA_ERR_INVALID_ARG;
    if (B == 0) return VFA_OK;
    // (rows * (2 + d) floats, in 64-bit arithmetic: the size check must not itself overflow)
    if ((unsigned long long)B * (unsigned long long)Hq * (unsigned long long)n_splits * (2ull + (unsigned long long)d) * 4ull >
        (unsigned long long)VFA_DECODE_NOALLOC_MAX_BYTES)
        return VFA_ERR_TOO_LARGE;
    void* const ws = scratch_address();
    if (!ws) return VFA_ERR_HIP;
    return decode_common(Q, K, V, Krepr, O, LSE, B, Hq, Hkv, n_cap, n_keys, nullptr, d, block_n, n_sink, n_local, use_minit,
                         n_splits, softmax_scale, ws, VFA_DECODE_NOALLOC_MAX_BYTES, stream);
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
    const dim3 grid((unsigned)ceil_div(tc_cap, 4), (unsigned)(B * Hkv));
    hipStream_t s = (hipStream_t)stream;
    (void)hipGetLastError();
    if (d == 128)
        kblock_summary_kernel<128><<<grid, 256, 0, s>>>((const uint16_t*)K, (uint16_t*)Krepr, n_cap, 0, tc_cap, block_n, 0, tc_cap, old_lens, new_lens, Hkv);
    else
        kblock_summary_kernel<64><<<grid, 256, 0, s>>>((const uint16_t*)K, (uint16_t*)Krepr, n_cap, 0, tc_cap, block_n, 0, tc_cap, old_lens, new_lens, Hkv);
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

}  // extern "C"

namespace {

int fp8_common(int frozen, bool noexp, const void* Q8, const void* K8, const void* Vt8, void* O, float* LSE, int B, int Hq,
               int Hkv, int N, int d, int block_m, int block_n, int causal, int n_sink, int n_local, int use_minit,
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
            // (the form without exponentials takes its scores times 4: two more in the exponent byte, and the
            // factor that turns a raw row max into log2 units becomes 1/4)
            p.scale_a = (127 + ex - 1 + (noexp ? 2 : 0)) * 0x01010101;
            p.c = noexp ? 0.25f : 1.f;
        }
    }
    if (noexp && !fold) return VFA_ERR_INVALID_ARG;  // (before anything is launched)
    (void)hipGetLastError();
    if (minit && use_minit == 1) {
        fp8_kblock_summary_kernel<<<dim3((unsigned)Tc, (unsigned)(B * Hkv)), 256, 0, s>>>((const uint8_t*)K8, (uint8_t*)workspace, N, Tc);
        if (hipGetLastError() != hipSuccess) return VFA_ERR_HIP;
    }
    const dim3 grid((unsigned)(B * Hq * Tr));
    if (noexp) attn_fp8_kernel<MODE_VFA, true, true><<<grid, 256, 0, s>>>(p);
    else if (fold) attn_fp8_kernel<MODE_VFA, true><<<grid, 256, 0, s>>>(p);
    else if (frozen) attn_fp8_kernel<MODE_VFA, false><<<grid, 256, 0, s>>>(p);
    else attn_fp8_kernel<MODE_FA, false><<<grid, 256, 0, s>>>(p);
    return hipGetLastError() == hipSuccess ? VFA_OK : VFA_ERR_HIP;
}

}  // namespace

extern "C" {

int vfa_fp8_attn_fwd(int frozen, const void* Q8, const void* K8, const void* Vt8, void* O, float* LSE, int B, int Hq, int Hkv,
                     int N, int d, int block_m, int block_n, int causal, int n_sink, int n_local, int use_minit,
                     float softmax_scale, float descale_q, float descale_k, float descale_v, void* workspace,
                     size_t workspace_bytes, void* stream) {
    return fp8_common(frozen, false, Q8, K8, Vt8, O, LSE, B, Hq, Hkv, N, d, block_m, block_n, causal, n_sink, n_local, use_minit,
                      softmax_scale, descale_q, descale_k, descale_v, workspace, workspace_bytes, stream);
}

int vfa_fp8_attn_noexp_fwd(const void* Q8, const void* K8, const void* Vt8, void* O, float* LSE, int B, int Hq, int Hkv, int N,
                           int d, int block_m, int block_n, int causal, int n_sink, int n_local, int use_minit,
                           float softmax_scale, float descale_q, float descale_k, float descale_v, void* workspace,
                           size_t workspace_bytes, void* stream) {
    return fp8_common(1, true, Q8, K8, Vt8, O, LSE, B, Hq, Hkv, N, d, block_m, block_n, causal, n_sink, n_local, use_minit,
                      softmax_scale, descale_q, descale_k, descale_v, workspace, workspace_bytes, stream);
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

}  // extern "C"

namespace {

int mx4_common(int frozen, bool noexp, const void* Q4, const void* QS, const void* K4, const void* KS, const void* Vt8, void* O,
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
    {
        const float sc = softmax_scale > 0.f ? softmax_scale : 1.0f / sqrtf((float)d);
        if (noexp && !(fabsf(sc * kLog2e - 1.f) <= 0x1p-18f)) return VFA_ERR_INVALID_ARG;  // (before anything is launched)
    }
    (void)hipGetLastError();
    if (minit && use_minit == 1) {
        mx4_kblock_summary_kernel<<<dim3((unsigned)Tc, (unsigned)(B * Hkv)), 256, 0, s>>>((const uint8_t*)K4, (const uint8_t*)KS,
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
    if (fold) p.c = noexp ? 0.25f : 1.f;  // (without exponentials the scores come out times 4)
    const dim3 grid((unsigned)(B * Hq * Tr));
    if (noexp) attn_mx4_kernel<MODE_VFA, true, true><<<grid, 256, 0, s>>>(p);
    else if (fold) attn_mx4_kernel<MODE_VFA, true><<<grid, 256, 0, s>>>(p);
    else if (frozen) attn_mx4_kernel<MODE_VFA, false><<<grid, 256, 0, s>>>(p);
    else attn_mx4_kernel<MODE_FA, false><<<grid, 256, 0, s>>>(p);
    return hipGetLastError() == hipSuccess ? VFA_OK : VFA_ERR_HIP;
}

}  // namespace

extern "C" {

int vfa_mxfp4_attn_fwd(int frozen, const void* Q4, const void* QS, const void* K4, const void* KS, const void* Vt8, void* O,
                       float* LSE, int B, int Hq, int Hkv, int N, int d, int block_m, int block_n, int causal, int n_sink,
                       int n_local, int use_minit, float softmax_scale, float descale_v, void* workspace,
                       size_t workspace_bytes, void* stream) {
    return mx4_common(frozen, false, Q4, QS, K4, KS, Vt8, O, LSE, B, Hq, Hkv, N, d, block_m, block_n, causal, n_sink, n_local,
                      use_minit, softmax_scale, descale_v, workspace, workspace_bytes, stream);
}

int vfa_mxfp4_attn_noexp_fwd(const void* Q4, const void* QS, const void* K4, const void* KS, const void* Vt8, void* O,
                             float* LSE, int B, int Hq, int Hkv, int N, int d, int block_m, int block_n, int causal,
                             int n_sink, int n_local, int use_minit, float softmax_scale, float descale_v, void* workspace,
                             size_t workspace_bytes, void* stream) {
    return mx4_common(1, true, Q4, QS, K4, KS, Vt8, O, LSE, B, Hq, Hkv, N, d, block_m, block_n, causal, n_sink, n_local,
                      use_minit, softmax_scale, descale_v, workspace, workspace_bytes, stream);
}

const char* vfa_strerror(int code) {
    switch (code) {
        case VFA_OK: return "ok";
        case VFA_ERR_INVALID_ARG: return "invalid argument";
        case VFA_ERR_UNSUPPORTED: return "unsupported shape (d must be 64 or 128; blocks 64x64 or 128x64)";
        case VFA_ERR_HIP: return "HIP launch error";
        case VFA_ERR_TOO_LARGE: return "problem needs more scratch than the library's fixed device array holds (use the entry point that takes a workspace)";
        default: return "unknown error code";
    }
}

}  // extern "C"
