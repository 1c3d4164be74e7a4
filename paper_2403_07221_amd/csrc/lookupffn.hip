// C ABI of the LookupFFN forward pass (declared in include/lookupffn.h): argument
// validation, launch-shape planning and kernel launches.  All arithmetic of the
// method is in hash_kernel.hpp and gather_kernel.hpp.
#include "lookupffn.h"

#include <hip/hip_runtime.h>

#include <cmath>
#include <cstring>
#include <map>
#include <mutex>
#include <string>
#include <vector>

#include "bh_hash_kernel.hpp"
#include "gather_kernel.hpp"
#include "gather_lds_kernel.hpp"
#include "hash_kernel.hpp"

// Build parts.  This file compiles whole (LFFN_PART undefined) or as parts that are linked together, so
// that the kernel families compile side by side: part 0 holds the C ABI, the host logic and the hash and
// re-pack kernels; parts 1 .. 11 hold one family of kernel launchers each (declared just below).  No
// kernel is instantiated in two parts.
#ifdef LFFN_PART
#define LFFN_HAS(p) (LFFN_PART == (p))
#else
#define LFFN_HAS(p) 1
#endif

namespace lffn_host {
using namespace lffn;
int hip_fail(hipError_t e, const char *what);  // part 0
int allow_lds(const void *kern, size_t lds);   // part 0
// part 1: the direct gather kernel
int gather_direct_part(bool bf16, int lpt, const GatherArgs &a, bool probes, dim3 grid, hipStream_t s);
// parts 2, 3: the LDS-staged gather kernel (plain sum; weighted and multi-probe)
int gather_lds_plain_part(int tok, const GatherLdsArgs &a, int fr, int sw, dim3 grid, size_t lds, hipStream_t s);
int gather_lds_weighted_part(int tok, const GatherLdsArgs &a, int fr, int sw, dim3 grid, size_t lds, hipStream_t s);
int gather_lds_probes_part(int tok, const GatherLdsArgs &a, int fr, int sw, dim3 grid, size_t lds, hipStream_t s);
// parts 4 .. 11: the BH hash kernel.  Plain: d_pad = 64 .. 256, 512, 1024; weighted: d_pad = 64 .. 256, then
// 512 and 1024 each split by the way the rows are read (four coordinates at a time or one by one): the
// wide weighted kernels are the slowest to compile by far
int bh_plain_lo_part(int L, const BhArgs &a, int block, dim3 grid, size_t lds, hipStream_t s);
int bh_plain_512_part(const BhArgs &a, int block, dim3 grid, size_t lds, hipStream_t s);
int bh_plain_1024_part(const BhArgs &a, int block, dim3 grid, size_t lds, hipStream_t s);
int bh_weighted_lo_part(int L, const BhArgs &a, int block, dim3 grid, size_t lds, hipStream_t s);
int bh_weighted_512_vec4_part(const BhArgs &a, int block, dim3 grid, size_t lds, hipStream_t s);
int bh_weighted_512_scalar_part(const BhArgs &a, int block, dim3 grid, size_t lds, hipStream_t s);
int bh_weighted_1024_vec4_part(const BhArgs &a, int block, dim3 grid, size_t lds, hipStream_t s);
int bh_weighted_1024_scalar_part(const BhArgs &a, int block, dim3 grid, size_t lds, hipStream_t s);
}  // namespace lffn_host

namespace {

using namespace lffn;
using lffn_host::allow_lds;
using lffn_host::hip_fail;

#define LFFN_HIP(call)                                       \
    do {                                                     \
        hipError_t e_ = (call);                              \
        if (e_ != hipSuccess) return hip_fail(e_, #call);    \
    } while (0)

#if LFFN_HAS(0)
constexpr int kVersion = 100;  // 0.1.0
constexpr int kMaxLog2N = 12;  // d_pad <= 4096
thread_local std::string g_hip_error;
const char *g_last_gather = "";  // name of the gather kernel the most recent launch used
#endif

// ---------------------------------------------------------------- kernel launchers (templates: every part may use them)
template <bool BF16, int LPT>
void launch_gather_t(const GatherArgs &a, bool probes, dim3 grid, hipStream_t s)
{
    if (probes)
        hipLaunchKernelGGL((gather_kernel<BF16, LPT, 2>), grid, dim3(kGatherThreads), 0, s, a);
    else if (a.weights)
        hipLaunchKernelGGL((gather_kernel<BF16, LPT, 1>), grid, dim3(kGatherThreads), 0, s, a);
    else
        hipLaunchKernelGGL((gather_kernel<BF16, LPT, 0>), grid, dim3(kGatherThreads), 0, s, a);
}

template <bool BF16>
int launch_gather_lpt(int lpt, const GatherArgs &a, bool probes, dim3 grid, hipStream_t s)
{
    switch (lpt) {
        case 1: launch_gather_t<BF16, 1>(a, probes, grid, s); break;
        case 2: launch_gather_t<BF16, 2>(a, probes, grid, s); break;
        case 4: launch_gather_t<BF16, 4>(a, probes, grid, s); break;
        case 8: launch_gather_t<BF16, 8>(a, probes, grid, s); break;
        case 16: launch_gather_t<BF16, 16>(a, probes, grid, s); break;
        case 32: launch_gather_t<BF16, 32>(a, probes, grid, s); break;
        case 64: launch_gather_t<BF16, 64>(a, probes, grid, s); break;
        default: return LFFN_E_UNSUPPORTED;
    }
    return LFFN_OK;
}

template <int TOK, int FR, bool WEIGHTED, int SW, bool PROBES = false>
int launch_gather_lds_fr(const GatherLdsArgs &a, dim3 grid, size_t lds, hipStream_t s)
{
    auto kern = gather_lds_kernel<TOK, FR, WEIGHTED, SW, PROBES>;
    int rc = allow_lds(reinterpret_cast<const void *>(kern), lds);
    if (rc != LFFN_OK) return rc;
    hipLaunchKernelGGL(kern, grid, dim3(kLdsThreads), lds, s, a);
    return LFFN_OK;
}

// fr = 16 KB copy rounds per table slice, sw = lanes per token (both fixed by the plan)
template <int TOK, bool WEIGHTED = false>
int launch_gather_lds_t(const GatherLdsArgs &a, int fr, int sw, dim3 grid, size_t lds, hipStream_t s)
{
    if constexpr (TOK <= 13) {
        if (sw == 8)
            return fr == 4   ? launch_gather_lds_fr<TOK, 4, WEIGHTED, 8>(a, grid, lds, s)
                   : fr == 2 ? launch_gather_lds_fr<TOK, 2, WEIGHTED, 8>(a, grid, lds, s)
                             : launch_gather_lds_fr<TOK, 1, WEIGHTED, 8>(a, grid, lds, s);
    }
    if (sw != 4) return LFFN_E_UNSUPPORTED;
    if constexpr (TOK == 8 || TOK == 13 || TOK == 16) {  // 64-byte slices
        return fr == 4   ? launch_gather_lds_fr<TOK, 4, WEIGHTED, 4>(a, grid, lds, s)
               : fr == 2 ? launch_gather_lds_fr<TOK, 2, WEIGHTED, 4>(a, grid, lds, s)
                         : launch_gather_lds_fr<TOK, 1, WEIGHTED, 4>(a, grid, lds, s);
    }
    return LFFN_E_UNSUPPORTED;
}

// multi-probe form: fp32 tables; 128-byte slices for tau 7, 8, 64-byte slices for tau 9, 10
template <int TOK>
int launch_gather_lds_probes(const GatherLdsArgs &a, int fr, int sw, dim3 grid, size_t lds, hipStream_t s)
{
    if constexpr (TOK <= 13 && TOK != 12) {
        if (sw == 8 && fr == 2) return launch_gather_lds_fr<TOK, 2, true, 8, true>(a, grid, lds, s);
        if (sw == 8 && fr == 1) return launch_gather_lds_fr<TOK, 1, true, 8, true>(a, grid, lds, s);
    }
    if constexpr (TOK == 8 || TOK == 13 || TOK == 16) {
        if (sw == 4 && fr == 4) return launch_gather_lds_fr<TOK, 4, true, 4, true>(a, grid, lds, s);
        if (sw == 4 && fr == 2) return launch_gather_lds_fr<TOK, 2, true, 4, true>(a, grid, lds, s);
    }
    return LFFN_E_UNSUPPORTED;
}

template <int L, int TB, bool VEC4, bool WEIGHTED>
int launch_bh_k(const BhArgs &a, dim3 grid, size_t lds, hipStream_t s)
{
    auto kern = bh_hash_kernel<L, TB, VEC4, WEIGHTED>;
    int rc = allow_lds(reinterpret_cast<const void *>(kern), lds);
    if (rc != LFFN_OK) return rc;
    hipLaunchKernelGGL(kern, grid, dim3(kBhThreads), lds, s, a);
    return LFFN_OK;
}

template <int L, bool VEC4, bool WEIGHTED>
int launch_bh_v(const BhArgs &a, int block, dim3 grid, size_t lds, hipStream_t s)
{
    switch (block) {
        case 16: return launch_bh_k<L, 1, VEC4, WEIGHTED>(a, grid, lds, s);
        case 32: return launch_bh_k<L, 2, VEC4, WEIGHTED>(a, grid, lds, s);
        case 64: return launch_bh_k<L, 4, VEC4, WEIGHTED>(a, grid, lds, s);
    }
    return LFFN_E_UNSUPPORTED;
}

template <int L, bool WEIGHTED>
int launch_bh_w(const BhArgs &a, int block, dim3 grid, size_t lds, hipStream_t s)
{
    return a.x_vec4 ? launch_bh_v<L, true, WEIGHTED>(a, block, grid, lds, s)
                    : launch_bh_v<L, false, WEIGHTED>(a, block, grid, lds, s);
}

}  // namespace

// ---------------------------------------------------------------- the parts' launch functions
namespace lffn_host {

#if LFFN_HAS(1)
int gather_direct_part(bool bf16, int lpt, const GatherArgs &a, bool probes, dim3 grid, hipStream_t s)
{
    return bf16 ? launch_gather_lpt<true>(lpt, a, probes, grid, s) : launch_gather_lpt<false>(lpt, a, probes, grid, s);
}
#endif

#if LFFN_HAS(2)
int gather_lds_plain_part(int tok, const GatherLdsArgs &a, int fr, int sw, dim3 grid, size_t lds, hipStream_t s)
{
    if (tok <= 4) return launch_gather_lds_t<4>(a, fr, sw, grid, lds, s);
    if (tok <= 8) return launch_gather_lds_t<8>(a, fr, sw, grid, lds, s);
    if (tok <= 12) return launch_gather_lds_t<12>(a, fr, sw, grid, lds, s);
    if (tok <= 13) return launch_gather_lds_t<13>(a, fr, sw, grid, lds, s);
    if (tok <= 16 && sw == 4) return launch_gather_lds_t<16>(a, fr, sw, grid, lds, s);
    return LFFN_E_UNSUPPORTED;
}
#endif

#if LFFN_HAS(3)
int gather_lds_weighted_part(int tok, const GatherLdsArgs &a, int fr, int sw, dim3 grid, size_t lds, hipStream_t s)
{
    if (tok <= 4) return launch_gather_lds_t<4, true>(a, fr, sw, grid, lds, s);
    if (tok <= 8) return launch_gather_lds_t<8, true>(a, fr, sw, grid, lds, s);
    if (tok <= 12) return launch_gather_lds_t<12, true>(a, fr, sw, grid, lds, s);
    if (tok <= 13) return launch_gather_lds_t<13, true>(a, fr, sw, grid, lds, s);
    if (tok <= 16 && sw == 4) return launch_gather_lds_t<16, true>(a, fr, sw, grid, lds, s);
    return LFFN_E_UNSUPPORTED;
}

int gather_lds_probes_part(int tok, const GatherLdsArgs &a, int fr, int sw, dim3 grid, size_t lds, hipStream_t s)
{
    if (tok <= 4) return launch_gather_lds_probes<4>(a, fr, sw, grid, lds, s);
    if (tok <= 8) return launch_gather_lds_probes<8>(a, fr, sw, grid, lds, s);
    if (tok <= 13) return launch_gather_lds_probes<13>(a, fr, sw, grid, lds, s);
    if (tok <= 16) return launch_gather_lds_probes<16>(a, fr, sw, grid, lds, s);
    return LFFN_E_UNSUPPORTED;
}
#endif

#if LFFN_HAS(4)
int bh_plain_lo_part(int L, const BhArgs &a, int block, dim3 grid, size_t lds, hipStream_t s)
{
    switch (L) {
        case 6: return launch_bh_w<6, false>(a, block, grid, lds, s);
        case 7: return launch_bh_w<7, false>(a, block, grid, lds, s);
        case 8: return launch_bh_w<8, false>(a, block, grid, lds, s);
    }
    return LFFN_E_UNSUPPORTED;
}
#endif

#if LFFN_HAS(5)
int bh_plain_512_part(const BhArgs &a, int block, dim3 grid, size_t lds, hipStream_t s)
{
    return launch_bh_w<9, false>(a, block, grid, lds, s);
}
#endif

#if LFFN_HAS(6)
int bh_plain_1024_part(const BhArgs &a, int block, dim3 grid, size_t lds, hipStream_t s)
{
    return launch_bh_w<10, false>(a, block, grid, lds, s);
}
#endif

#if LFFN_HAS(7)
int bh_weighted_lo_part(int L, const BhArgs &a, int block, dim3 grid, size_t lds, hipStream_t s)
{
    switch (L) {
        case 6: return launch_bh_w<6, true>(a, block, grid, lds, s);
        case 7: return launch_bh_w<7, true>(a, block, grid, lds, s);
        case 8: return launch_bh_w<8, true>(a, block, grid, lds, s);
    }
    return LFFN_E_UNSUPPORTED;
}
#endif

#if LFFN_HAS(8)
int bh_weighted_512_vec4_part(const BhArgs &a, int block, dim3 grid, size_t lds, hipStream_t s)
{
    return launch_bh_v<9, true, true>(a, block, grid, lds, s);
}
#endif

#if LFFN_HAS(9)
int bh_weighted_512_scalar_part(const BhArgs &a, int block, dim3 grid, size_t lds, hipStream_t s)
{
    return launch_bh_v<9, false, true>(a, block, grid, lds, s);
}
#endif

#if LFFN_HAS(10)
int bh_weighted_1024_vec4_part(const BhArgs &a, int block, dim3 grid, size_t lds, hipStream_t s)
{
    return launch_bh_v<10, true, true>(a, block, grid, lds, s);
}
#endif

#if LFFN_HAS(11)
int bh_weighted_1024_scalar_part(const BhArgs &a, int block, dim3 grid, size_t lds, hipStream_t s)
{
    return launch_bh_v<10, false, true>(a, block, grid, lds, s);
}
#endif

#if LFFN_HAS(0)
int hip_fail(hipError_t e, const char *what)
{
    g_hip_error = std::string(what) + ": " + hipGetErrorString(e);
    return LFFN_E_HIP;
}

// kernels that use more than 64 KB of dynamic LDS must be told so, once per device and kernel
int allow_lds(const void *kern, size_t lds)
{
    static std::mutex mu;
    static std::map<std::pair<int, const void *>, size_t> configured;  // (device, kernel) -> LDS bytes set up
    int dev = 0;
    LFFN_HIP(hipGetDevice(&dev));
    std::lock_guard<std::mutex> lk(mu);
    size_t &have = configured[std::make_pair(dev, kern)];
    if (have < lds) {
        LFFN_HIP(hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        have = lds;
    }
    return LFFN_OK;
}
#endif

}  // namespace lffn_host

#if LFFN_HAS(0)  // ================ everything below: host logic and the C ABI ================
namespace {


int log2_pad(int d)
{
    int l = 0;
    while ((1 << l) < d) ++l;
    return l;
}

bool dtype_ok(int t) { return t == LFFN_F32 || t == LFFN_BF16; }
bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

// ---------------------------------------------------------------- options
struct Options {
    int lanes_per_token = 0;  // 0 = default
    int xcd_order = 0;        // 0 = default, 1 = on, -1 = off
    int gather_path = 0;      // 0 = choose, 1 = direct kernel, 2 = LDS-staged kernel (if the shape allows)
    int hash_path = 0;        // 0 = choose, 1 = generic kernel only
    int hash_blocks = 0;      // 0 = default grid cap of the d_pad = 1024 hash kernel
    int slice_lanes = 0;      // 0 = choose, 4 = 64-byte column slices in the staged gather where possible
    int token_slots = 0;      // 0 = choose, else the most token slots per lane of the staged gather
} g_opt;

// ---------------------------------------------------------------- timing
struct Timing {
    int on = 0;  // bit 0: time hash launches, bit 1: time gather launches
    std::vector<std::pair<hipEvent_t, hipEvent_t>> ev[2];
    std::vector<std::pair<hipEvent_t, hipEvent_t>> pool;
} g_tm;

struct TimedLaunch {
    int which;
    hipStream_t s;
    hipEvent_t a = nullptr, b = nullptr;
    bool ok = true;
    bool active() const { return (g_tm.on >> which) & 1; }
    TimedLaunch(int which_, hipStream_t s_) : which(which_), s(s_)
    {
        if (!active()) return;
        if (!g_tm.pool.empty()) {
            a = g_tm.pool.back().first;
            b = g_tm.pool.back().second;
            g_tm.pool.pop_back();
        } else if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess) {
            ok = false;
            return;
        }
        ok = hipEventRecord(a, s) == hipSuccess;
    }
    void done()
    {
        if (!active() || !a || !b) return;
        (void)hipEventRecord(b, s);
        g_tm.ev[which].emplace_back(a, b);
    }
};

// ---------------------------------------------------------------- library-owned workspace
struct Workspace {
    void *ptr = nullptr;
    size_t bytes = 0;
};
std::mutex g_ws_mu;
std::map<int, Workspace> g_ws;

int own_workspace(size_t need, void **out)
{
    int dev = 0;
    LFFN_HIP(hipGetDevice(&dev));
    std::lock_guard<std::mutex> lk(g_ws_mu);
    Workspace &w = g_ws[dev];
    if (w.bytes < need) {
        if (w.ptr) {
            LFFN_HIP(hipDeviceSynchronize());
            LFFN_HIP(hipFree(w.ptr));
            w.ptr = nullptr;
            w.bytes = 0;
        }
        size_t sz = (need + (size_t(1) << 20) - 1) & ~((size_t(1) << 20) - 1);
        LFFN_HIP(hipMalloc(&w.ptr, sz));
        w.bytes = sz;
    }
    *out = w.ptr;
    return LFFN_OK;
}

// ---------------------------------------------------------------- validation
int check_hash(const void *x, const int8_t *signs, const uint16_t *codes, int64_t n, int d, int k,
               int tau, int n_rounds, int x_dtype, bool weighted = false)
{
    if (!x || !signs || !codes) return LFFN_E_NULL;
    if (n < 0 || d < 1 || k < 1 || n_rounds < 1) return LFFN_E_SIZE;
    if (tau < 1 || tau > 16) return LFFN_E_TAU;
    if (!dtype_ok(x_dtype)) return LFFN_E_DTYPE;
    if (k > (1 << 20) || n > (int64_t(1) << 40) || n_rounds > 64) return LFFN_E_SIZE;
    if (log2_pad(d) > kMaxLog2N || d > (1 << kMaxLog2N)) return LFFN_E_UNSUPPORTED;
    const int N = 1 << log2_pad(d);
    const int64_t P = ((int64_t)k * tau + N - 1) / N;
    if (P > 4096) return LFFN_E_SIZE;
    if (hash_lds_bytes((int)P, n_rounds, N, weighted) > 64 * 1024) return LFFN_E_UNSUPPORTED;
    if (!aligned(x, x_dtype == LFFN_F32 ? 4 : 2) || !aligned(codes, 2)) return LFFN_E_ALIGN;
    return LFFN_OK;
}

int check_weights(const float *weights)
{
    if (!weights) return LFFN_E_NULL;
    if (!aligned(weights, 4)) return LFFN_E_ALIGN;
    return LFFN_OK;
}

int check_gather(const uint16_t *codes, const void *tables, const float *y, int64_t n, int k, int tau,
                 int d_out, int table_dtype)
{
    if (!codes || !tables || !y) return LFFN_E_NULL;
    if (n < 0 || k < 1 || d_out < 1) return LFFN_E_SIZE;
    if (tau < 1 || tau > 16) return LFFN_E_TAU;
    if (!dtype_ok(table_dtype)) return LFFN_E_DTYPE;
    if (k > (1 << 20) || n > (int64_t(1) << 40) || d_out > (1 << 24)) return LFFN_E_SIZE;
    const int w = table_dtype == LFFN_F32 ? 4 : 8;
    if (d_out % w != 0) return LFFN_E_ALIGN;
    if (!aligned(tables, 16) || !aligned(y, 16) || !aligned(codes, 2)) return LFFN_E_ALIGN;
    // row index (j << tau) + code must fit 32 bits
    if (((int64_t)k << tau) > (int64_t(1) << 31)) return LFFN_E_SIZE;
    return LFFN_OK;
}

// ---------------------------------------------------------------- launches
template <int L>
void launch_hash_t(const HashArgs &a, bool probes, dim3 grid, size_t lds, hipStream_t s)
{
    if (probes)
        hipLaunchKernelGGL((hash_kernel<L, 2>), grid, dim3(kHashThreads), lds, s, a);
    else if (a.weights || a.wpk)
        hipLaunchKernelGGL((hash_kernel<L, 1>), grid, dim3(kHashThreads), lds, s, a);
    else
        hipLaunchKernelGGL((hash_kernel<L, 0>), grid, dim3(kHashThreads), lds, s, a);
}

template <int R>
void launch_hash1024_t(const HashArgs &a, bool probes, dim3 grid, size_t lds, hipStream_t s)
{
    if (probes)
        hipLaunchKernelGGL((hash1024_kernel<R, 2>), grid, dim3(kHashThreads), lds, s, a);
    else if (a.weights || a.wpk)
        hipLaunchKernelGGL((hash1024_kernel<R, 1>), grid, dim3(kHashThreads), lds, s, a);
    else
        hipLaunchKernelGGL((hash1024_kernel<R, 0>), grid, dim3(kHashThreads), lds, s, a);
}

// Writes codes[n][k] when `codes` is given, else the packed layout of the LDS-staged gather;
// with `weights` also the gather weights of the weighted variant ([n][k] beside `codes`,
// table-major [k][n_pad] beside `packed`).
int launch_hash(const void *x, const int8_t *signs, uint16_t *codes, uint32_t *packed, float *weights, int64_t n,
                int d, int k, int tau, int n_rounds, int x_dtype, hipStream_t s, bool probes = false)
{
    const int L = log2_pad(d);
    const int N = 1 << L;
    HashArgs a;
    a.x = x;
    a.signs = signs;
    a.codes = codes;
    a.packed = codes ? nullptr : packed;
    a.weights = codes ? weights : nullptr;
    a.wpk = codes ? nullptr : weights;
    a.n_pad = packed_n_pad(n);
    a.n = n;
    a.d = d;
    a.k = k;
    a.tau = tau;
    a.n_rounds = n_rounds;
    a.P = (int)(((int64_t)k * tau + N - 1) / N);
    a.x_bf16 = x_dtype == LFFN_BF16;
    a.scale = (float)(1.0 / std::sqrt((double)N));
    TimedLaunch tl(0, s);
    // d_pad = 1024 with up to four rounds: the two-layout kernel (needs 16-byte aligned signs, and
    // rows that start on 16-byte boundaries when it loads them as vectors)
    const size_t xrow = (size_t)d * (a.x_bf16 ? 2 : 4);
    const bool weighted = weights != nullptr;
    if (g_opt.hash_path != 1 && L == 10 && n_rounds <= 4 && aligned(signs, 16) &&
        h1024_lds_bytes(a.P, weighted) <= 64 * 1024 &&
        (d % 4 != 0 || (aligned(x, 16) && xrow % (a.x_bf16 ? 8 : 16) == 0))) {
        int64_t blocks = (n + kHashWaves - 1) / kHashWaves;
        const int64_t cap = g_opt.hash_blocks ? g_opt.hash_blocks : 4096;
        if (blocks > cap) blocks = cap;
        const dim3 grid((unsigned)blocks);
        const size_t lds = h1024_lds_bytes(a.P, weighted);
        switch (n_rounds) {
            case 1: launch_hash1024_t<1>(a, probes, grid, lds, s); break;
            case 2: launch_hash1024_t<2>(a, probes, grid, lds, s); break;
            case 3: launch_hash1024_t<3>(a, probes, grid, lds, s); break;
            default: launch_hash1024_t<4>(a, probes, grid, lds, s); break;
        }
        LFFN_HIP(hipGetLastError());
        tl.done();
        return LFFN_OK;
    }
    const size_t lds = hash_lds_bytes(a.P, n_rounds, N, weighted);
    int64_t blocks = (n + kHashWaves - 1) / kHashWaves;
    if (blocks > 2048) blocks = 2048;
    const dim3 grid((unsigned)blocks);
    switch (L) {
#define LFFN_CASE(l) case l: launch_hash_t<l>(a, probes, grid, lds, s); break;
        LFFN_CASE(0) LFFN_CASE(1) LFFN_CASE(2) LFFN_CASE(3) LFFN_CASE(4) LFFN_CASE(5) LFFN_CASE(6)
        LFFN_CASE(7) LFFN_CASE(8) LFFN_CASE(9) LFFN_CASE(10) LFFN_CASE(11) LFFN_CASE(12)
#undef LFFN_CASE
        default: return LFFN_E_UNSUPPORTED;
    }
    LFFN_HIP(hipGetLastError());
    tl.done();
    return LFFN_OK;
}

int gcd(int a, int b) { return b ? gcd(b, a % b) : a; }
int64_t round256(int64_t b) { return (b + 255) & ~int64_t(255); }

constexpr int kLdsMinBytes = 84 * 1024;  // more than half of the 160 KB LDS: one workgroup per CU

int device_cus(int *cus)
{
    static std::mutex mu;
    static std::map<int, int> cache;
    int dev = 0;
    LFFN_HIP(hipGetDevice(&dev));
    std::lock_guard<std::mutex> lk(mu);
    auto it = cache.find(dev);
    if (it == cache.end()) {
        int n = 0;
        LFFN_HIP(hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev));
        it = cache.emplace(dev, n).first;
    }
    *cus = it->second;
    return LFFN_OK;
}

// Largest number of tokens a workgroup gets in one piece, mirroring the kernel's split.
int64_t lds_tokens_per_block(int64_t n, int n_units, int token_splits, int Bx)
{
    const int m = (n_units + kXcds - 1) / kXcds;  // units of the fullest XCD
    const int64_t unit_tokens = (n + token_splits - 1) / token_splits;
    if (m >= Bx) return unit_tokens;
    const int blocks = Bx / m;  // the unit with the fewest workgroups
    return (unit_tokens + blocks - 1) / blocks;
}

// Launch shape of the LDS-staged gather for one problem size (no pointers involved).
struct LdsPlan {
    bool use = false;
    GatherLdsArgs a;
    int tok = 0;
    int sw = 8;     // lanes per token: 8 = 128-byte column slices, 4 = 64-byte ones
    int fr = 1;     // 16 KB copy rounds per table slice
    int shift = 7;  // log2 of the row-piece bytes: what the packed codes are scaled by.  The hash kernels
                    // write shift 7; a plan with shift 6 takes its codes through the re-pack kernel.
    unsigned grid = 0;
    size_t lds = 0;
    bool widen = false;        // bf16 tables: the kernel reads an fp32 copy made first in `widened`
    int64_t widen_bytes = 0;   // size of that copy
    void *widened = nullptr;   // set by the entry point once it has the scratch memory
};

// `can_widen`: the caller can provide scratch memory for an fp32 copy of bf16 tables (the staged kernel
// reads fp32 rows only).
int plan_gather_lds(int64_t n, int k, int tau, int d_out, bool bf16, LdsPlan *p, bool weighted = false,
                    bool probes = false, bool can_widen = false)
{
    (void)weighted;
    p->use = false;
    p->widen = false;
    p->widen_bytes = 0;
    p->widened = nullptr;
    if (g_opt.gather_path == 1) return LFFN_OK;
    if (bf16 && !can_widen) return LFFN_OK;
    const int rows = 1 << tau;
    if (tau < 7 || tau > 10 || k % 2 != 0) return LFFN_OK;
    // column slices: 128 bytes (8 lanes per token) up to tau = 8; 64 bytes from tau = 9 on (two 512-row
    // tables per stage and half the copy volume per token measured faster than one per stage; tau = 10
    // fits a 64 KB buffer only this way).  The 64-byte form exists for fp32 tables and tau >= 8.
    int sw = tau <= 8 ? 8 : 4;
    if (g_opt.slice_lanes == 4 && tau >= 8) sw = 4;
    if (g_opt.slice_lanes == 8 && tau <= 9) sw = 8;
    if (probes) sw = tau <= 8 ? 8 : 4;  // the multi-probe form is built for these pairings only
    const int groups = kLdsThreads / sw;
    // the kernel indexes tokens and bytes inside one table with 32 bits
    if (n >= (int64_t(1) << 31) - 4096 || (int64_t)rows * d_out * 4 >= (int64_t(1) << 32)) return LFFN_OK;
    int cus = 0;
    int rc = device_cus(&cus);
    if (rc != LFFN_OK) return rc;
    if (cus < kXcds || cus % kXcds != 0) return LFFN_OK;
    GatherLdsArgs &a = p->a;
    a.n = n;
    a.n_pad = packed_n_pad(n);
    a.k = k;
    a.tau = tau;
    a.d_out = d_out;
    a.row_bytes = (uint32_t)d_out * 4;  // of the fp32 rows the kernel reads
    a.nvec = (int)(a.row_bytes / 16);
    a.n_slices = (a.nvec + sw - 1) / sw;
    a.token_splits = kXcds / gcd(a.n_slices, kXcds);
    a.n_units = a.n_slices * a.token_splits;
    a.blocks_per_xcd = cus / kXcds;
    const int64_t tpb = lds_tokens_per_block(n, a.n_units, a.token_splits, a.blocks_per_xcd);
    int tok_max = sw == 4 ? 16 : 13;
    // the multi-probe form holds a share per probe beside the accumulators: 13 slots spill in its
    // hot loop, 8 measured faster up to tau = 9 (tau = 10 has 16 copy rounds per table to amortise)
    if (probes && tau <= 9) tok_max = 8;
    if (g_opt.token_slots && g_opt.token_slots < tok_max) tok_max = g_opt.token_slots;
    const int64_t nchunks = (tpb + (int64_t)groups * tok_max - 1) / ((int64_t)groups * tok_max);
    const int64_t chunk = (tpb + nchunks - 1) / nchunks;
    // Staging pays only when a chunk re-uses each staged row a few times; with bf16 tables the whole
    // table set is widened first (6 bytes moved per element), which a batch of 64 tokens per row repays
    // (configuration 3's shape at 16384 tokens: 108 us against 124 us direct; at 8192 the direct kernel wins).
    if (g_opt.gather_path != 2 && (chunk < 2 * (int64_t)rows || (bf16 && n < 64 * (int64_t)rows))) return LFFN_OK;
    p->tok = (int)((chunk + groups - 1) / groups);
    if (probes && sw == 8 && p->tok > 8) p->tok = 13;  // multi-probe form: 4, 8 or 13 slots
    if (sw == 4) p->tok = p->tok > 13 ? 16 : p->tok > 8 ? 13 : 8;  // the 64-byte form is built for 8, 13 and 16 token slots
    p->sw = sw;
    p->fr = rows / groups;
    p->shift = sw == 8 ? 7 : 6;
    p->lds = gather_lds_bytes(tau, sw);
    if (p->lds < (size_t)kLdsMinBytes) p->lds = kLdsMinBytes;
    p->grid = (unsigned)cus;
    p->widen = bf16;
    p->widen_bytes = bf16 ? round256((int64_t)k * rows * d_out * 4) : 0;
    p->use = true;
    return LFFN_OK;
}

// After the plan: does the scratch memory at hand have room for the widened tables?  `base` bytes are
// taken by the call itself.  A caller workspace that is too small for the copy turns the staged kernel
// off (the direct kernel reads bf16 rows); returns the bytes to add to `base`.
int64_t widen_room(LdsPlan *p, const void *workspace, int64_t workspace_bytes, int64_t base)
{
    if (!p->use || !p->widen) return 0;
    if (workspace && workspace_bytes < base + p->widen_bytes) {
        p->use = false;
        return 0;
    }
    return p->widen_bytes;
}

int launch_gather_lds(const LdsPlan &p, const uint32_t *packed, const float *wpk, const void *tables, float *y,
                      bool bf16, hipStream_t s, bool probes = false)
{
    GatherLdsArgs a = p.a;
    a.packed = packed;
    a.wpk = wpk;
    a.tables = static_cast<const char *>(tables);
    a.y = y;
    const dim3 grid(p.grid);
    int rc = LFFN_E_UNSUPPORTED;
    TimedLaunch tl(1, s);
    if (p.widen) {
        if (!bf16 || !p.widened) return LFFN_E_UNSUPPORTED;
        const long long n8 = (long long)a.k * (1ll << a.tau) * a.d_out / 8;
        long long wb = (n8 + 255) / 256;
        if (wb > 8192) wb = 8192;
        hipLaunchKernelGGL(widen_tables_kernel, dim3((unsigned)wb), dim3(256), 0, s,
                           static_cast<const uint4 *>(tables), static_cast<uint4 *>(p.widened), n8);
        LFFN_HIP(hipGetLastError());
        a.tables = static_cast<const char *>(p.widened);
    }
    if (probes)
        rc = lffn_host::gather_lds_probes_part(p.tok, a, p.fr, p.sw, grid, p.lds, s);
    else if (wpk)
        rc = lffn_host::gather_lds_weighted_part(p.tok, a, p.fr, p.sw, grid, p.lds, s);
    else
        rc = lffn_host::gather_lds_plain_part(p.tok, a, p.fr, p.sw, grid, p.lds, s);
    if (rc != LFFN_OK) return rc;
    LFFN_HIP(hipGetLastError());
    tl.done();
    g_last_gather = "gather_lds_kernel";
    return LFFN_OK;
}

int64_t packed_bytes(int64_t n, int k) { return ((int64_t)(k + 1) / 2) * packed_n_pad(n) * 4; }
int64_t probes_spk_bytes(int64_t n, int k, int tau) { return round256((int64_t)k * (tau + 1) * packed_n_pad(n) * 4); }

int launch_gather_direct(const uint16_t *codes, const float *weights, const void *tables, float *y, int64_t n,
                         int k, int tau, int d_out, int table_dtype, hipStream_t s, bool probes = false)
{
    const bool bf16 = table_dtype == LFFN_BF16;
    const int esz = bf16 ? 2 : 4;
    GatherArgs a;
    a.codes = codes;
    a.weights = weights;
    a.tables = static_cast<const char *>(tables);
    a.y = y;
    a.n = n;
    a.k = k;
    a.tau = tau;
    a.d_out = d_out;
    a.row_bytes = (uint32_t)d_out * esz;
    a.nvec = (int)(a.row_bytes / 16);
    a.codes_vec8 = (k % 8 == 0) && aligned(codes, 16) && (!weights || aligned(weights, 16));

    int lpt = g_opt.lanes_per_token;
    if (lpt == 0) {
        lpt = 8;  // 128-byte slices: one L2 line per (token, table)
        while (lpt > 1 && lpt / 2 >= a.nvec) lpt /= 2;
    }
    const int tpw = 64 / lpt;
    a.n_slices = (a.nvec + lpt - 1) / lpt;
    const int64_t ntb = (n + (int64_t)kGatherWaves * tpw - 1) / ((int64_t)kGatherWaves * tpw);
    if (ntb > (int64_t(1) << 30)) return LFFN_E_SIZE;
    a.ntb = (int)ntb;

    const double table_bytes = (double)k * (double)(1u << tau) * a.row_bytes;
    bool xcd = table_bytes > 4.0 * 1024 * 1024 && ntb >= 64;
    if (g_opt.xcd_order == 1) xcd = true;
    if (g_opt.xcd_order == -1) xcd = false;
    a.xcd_mode = xcd;
    int64_t blocks;
    if (xcd) {
        // split the token range so that the number of units is a multiple of the XCD count
        const int splits = kXcds / gcd(a.n_slices, kXcds);
        a.tb_per_unit = (int)((ntb + splits - 1) / splits);
        a.n_units = a.n_slices * splits;
        blocks = (int64_t)(a.n_units / kXcds) * kXcds * a.tb_per_unit;
    } else {
        a.tb_per_unit = (int)ntb;
        a.n_units = a.n_slices;
        blocks = (int64_t)a.n_units * ntb;
    }
    if (blocks > 0x7FFFFFFFLL) return LFFN_E_SIZE;
    const dim3 grid((unsigned)blocks);
    TimedLaunch tl(1, s);
    int rc = lffn_host::gather_direct_part(bf16, lpt, a, probes, grid, s);
    if (rc != LFFN_OK) return rc;
    LFFN_HIP(hipGetLastError());
    tl.done();
    g_last_gather = "gather_kernel";
    return LFFN_OK;
}

// ---- BH{m} hash --------------------------------------------------------------------------------
int check_bh(const void *x, const float *bmats, int64_t n, int d, int k, int tau, int block, int n_factors,
             int x_dtype, bool weighted = false)
{
    if (!x || !bmats) return LFFN_E_NULL;
    if (n < 0 || d < 1 || k < 1 || n_factors < 1) return LFFN_E_SIZE;
    if (tau < 1 || tau > 16) return LFFN_E_TAU;
    // the weights are reduced inside one 16-coordinate tile: a table must not straddle tiles
    if (weighted && tau != 4 && tau != 8 && tau != 16) return LFFN_E_UNSUPPORTED;
    if (!dtype_ok(x_dtype)) return LFFN_E_DTYPE;
    if (k > (1 << 20) || n > (int64_t(1) << 40) || n_factors > 64) return LFFN_E_SIZE;
    const int L = log2_pad(d);
    if (L > 10 || d > 1024) return LFFN_E_UNSUPPORTED;
    const int N = L < 6 ? 64 : 1 << L;  // widths below 64 are not built
    if (L < 6) return LFFN_E_UNSUPPORTED;
    if (block != 16 && block != 32 && block != 64) return LFFN_E_UNSUPPORTED;
    if (block > N) return LFFN_E_SIZE;
    const int64_t P = ((int64_t)k * tau + N - 1) / N;
    if (P > 64 || bh_lds_bytes((int)P, N) > 150 * 1024) return LFFN_E_UNSUPPORTED;
    if (!aligned(x, x_dtype == LFFN_F32 ? 4 : 2) || !aligned(bmats, 4)) return LFFN_E_ALIGN;
    return LFFN_OK;
}

int64_t bh_pack_bytes(int d, int k, int tau, int block, int n_factors)
{
    const int N = 1 << log2_pad(d);
    const int64_t P = ((int64_t)k * tau + N - 1) / N;
    return round256(P * n_factors * (int64_t)N * block * 4);
}

// Packs the factors into `apack` (bh_pack_bytes) and hashes; writes codes[n][k] (and weights[n][k] if
// given) or the packed layout (and wpk[k][n_pad] if given).
int launch_hash_bh(const void *x, const float *bmats, float *apack, uint16_t *codes, uint32_t *packed, int64_t n,
                   int d, int k, int tau, int block, int n_factors, int x_dtype, hipStream_t s,
                   float *weights = nullptr, float *wpk = nullptr)
{
    const int L = log2_pad(d);
    const int N = 1 << L;
    BhArgs a;
    a.x = x;
    a.apack = apack;
    a.codes = codes;
    a.packed = codes ? nullptr : packed;
    a.weights = codes ? weights : nullptr;
    a.wpk = codes ? nullptr : wpk;
    a.n_pad = packed_n_pad(n);
    a.n = n;
    a.d = d;
    a.k = k;
    a.tau = tau;
    a.n_factors = n_factors;
    a.P = (int)(((int64_t)k * tau + N - 1) / N);
    a.x_bf16 = x_dtype == LFFN_BF16;
    a.x_vec4 = d % 4 == 0 && aligned(x, a.x_bf16 ? 8 : 16);
    a.scale = (float)(1.0 / std::sqrt((double)N));
    const long long total = (long long)a.P * n_factors * N * block;
    long long pb = (total + 255) / 256;
    if (pb > 2048) pb = 2048;
    TimedLaunch tl(0, s);
    hipLaunchKernelGGL(bh_pack_kernel, dim3((unsigned)pb), dim3(256), 0, s, bmats, apack, N, block, total);
    LFFN_HIP(hipGetLastError());
    int64_t blocks = ((n + kBhTok - 1) / kBhTok + kBhWaves - 1) / kBhWaves;
    if (blocks > 4096) blocks = 4096;
    const dim3 grid((unsigned)blocks);
    const size_t lds = bh_lds_bytes(a.P, N);
    const bool weighted = a.weights || a.wpk;
    int rc;
    if (L <= 8)
        rc = weighted ? lffn_host::bh_weighted_lo_part(L, a, block, grid, lds, s)
                      : lffn_host::bh_plain_lo_part(L, a, block, grid, lds, s);
    else if (!weighted)
        rc = L == 9 ? lffn_host::bh_plain_512_part(a, block, grid, lds, s)
                    : lffn_host::bh_plain_1024_part(a, block, grid, lds, s);
    else if (L == 9)
        rc = a.x_vec4 ? lffn_host::bh_weighted_512_vec4_part(a, block, grid, lds, s)
                      : lffn_host::bh_weighted_512_scalar_part(a, block, grid, lds, s);
    else
        rc = a.x_vec4 ? lffn_host::bh_weighted_1024_vec4_part(a, block, grid, lds, s)
                      : lffn_host::bh_weighted_1024_scalar_part(a, block, grid, lds, s);
    if (rc != LFFN_OK) return rc;
    LFFN_HIP(hipGetLastError());
    tl.done();
    return LFFN_OK;
}

// workspace of the weighted forward pass: codes [n][k] uint16 then weights [n][k] fp32, or (staged
// gather) packed codes then table-major weights [k][n_pad]
int64_t weighted_codes_bytes(int64_t n, int k) { return ((int64_t)n * k * 2 + 255) & ~int64_t(255); }

// grid of the tiled re-pack kernels: one workgroup per 64 x 64 tile, capped (they stride over the rest)
unsigned repack_grid(int64_t n_rows, int64_t m)
{
    int64_t blocks = ((m + 63) / 64) * ((n_rows + 63) / 64);
    if (blocks > 16384) blocks = 16384;
    return (unsigned)(blocks < 1 ? 1 : blocks);
}

int launch_repack_codes(const uint16_t *codes, uint32_t *packed, int64_t n, int64_t n_pad, int k, int tau,
                        int shift, hipStream_t s)
{
    hipLaunchKernelGGL(repack_codes_kernel, dim3(repack_grid(n_pad, k / 2)), dim3(256), 0, s, codes, packed,
                       (long long)n, (long long)n_pad, k, tau, shift);
    LFFN_HIP(hipGetLastError());
    return LFFN_OK;
}

int launch_repack_shares(const float *shares, float *spk, int64_t n, int64_t n_pad, int k, int tau, hipStream_t s)
{
    const int64_t m = (int64_t)k * (tau + 1);
    hipLaunchKernelGGL(repack_shares_kernel, dim3(repack_grid(n, m)), dim3(256), 0, s, shares, spk, (long long)n,
                       (long long)n_pad, (long long)m);
    LFFN_HIP(hipGetLastError());
    return LFFN_OK;
}

int launch_repack_weights(const float *weights, float *wpk, int64_t n, int64_t n_pad, int k, hipStream_t s)
{
    hipLaunchKernelGGL(repack_shares_kernel, dim3(repack_grid(n, k)), dim3(256), 0, s, weights, wpk, (long long)n,
                       (long long)n_pad, (long long)k);
    LFFN_HIP(hipGetLastError());
    return LFFN_OK;
}

}  // namespace

extern "C" {

int lookupffn_hash(const void *x, const int8_t *signs, uint16_t *codes, int64_t n_tokens, int d, int k,
                   int tau, int n_rounds, int x_dtype, void *hip_stream)
{
    int rc = check_hash(x, signs, codes, n_tokens, d, k, tau, n_rounds, x_dtype);
    if (rc != LFFN_OK || n_tokens == 0) return rc;
    return launch_hash(x, signs, codes, nullptr, nullptr, n_tokens, d, k, tau, n_rounds, x_dtype,
                       static_cast<hipStream_t>(hip_stream));
}

int lookupffn_hash_weighted(const void *x, const int8_t *signs, uint16_t *codes, float *weights, int64_t n_tokens,
                            int d, int k, int tau, int n_rounds, int x_dtype, void *hip_stream)
{
    int rc = check_hash(x, signs, codes, n_tokens, d, k, tau, n_rounds, x_dtype, true);
    if (rc == LFFN_OK) rc = check_weights(weights);
    if (rc != LFFN_OK || n_tokens == 0) return rc;
    return launch_hash(x, signs, codes, nullptr, weights, n_tokens, d, k, tau, n_rounds, x_dtype,
                       static_cast<hipStream_t>(hip_stream));
}

int lookupffn_gather_weighted(const uint16_t *codes, const float *weights, const void *tables, float *y,
                              int64_t n_tokens, int k, int tau, int d_out, int table_dtype, void *hip_stream)
{
    int rc = check_gather(codes, tables, y, n_tokens, k, tau, d_out, table_dtype);
    if (rc == LFFN_OK) rc = check_weights(weights);
    if (rc != LFFN_OK || n_tokens == 0) return rc;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    LdsPlan plan;
    const bool bf16 = table_dtype == LFFN_BF16;
    rc = plan_gather_lds(n_tokens, k, tau, d_out, bf16, &plan, true, false, true);
    if (rc != LFFN_OK) return rc;
    if (plan.use && aligned(codes, 4)) {
        // the staged kernel reads packed codes and table-major weights: repack into the library's buffer
        const int64_t pb = round256(packed_bytes(n_tokens, k));
        void *ws = nullptr;
        const int64_t wb = round256((int64_t)k * plan.a.n_pad * 4);
        rc = own_workspace((size_t)(pb + wb + plan.widen_bytes), &ws);
        if (rc != LFFN_OK) return rc;
        plan.widened = plan.widen ? static_cast<char *>(ws) + pb + wb : nullptr;
        uint32_t *packed = static_cast<uint32_t *>(ws);
        float *wpk = reinterpret_cast<float *>(static_cast<char *>(ws) + pb);
        rc = launch_repack_codes(codes, packed, n_tokens, plan.a.n_pad, k, tau, plan.shift, s);
        if (rc != LFFN_OK) return rc;
        rc = launch_repack_weights(weights, wpk, n_tokens, plan.a.n_pad, k, s);
        if (rc != LFFN_OK) return rc;
        return launch_gather_lds(plan, packed, wpk, tables, y, bf16, s);
    }
    return launch_gather_direct(codes, weights, tables, y, n_tokens, k, tau, d_out, table_dtype, s);
}

int lookupffn_hash_probes(const void *x, const int8_t *signs, uint16_t *codes, float *shares, int64_t n_tokens,
                          int d, int k, int tau, int n_rounds, int x_dtype, void *hip_stream)
{
    int rc = check_hash(x, signs, codes, n_tokens, d, k, tau, n_rounds, x_dtype, true);
    if (rc == LFFN_OK) rc = check_weights(shares);
    if (rc != LFFN_OK || n_tokens == 0) return rc;
    return launch_hash(x, signs, codes, nullptr, shares, n_tokens, d, k, tau, n_rounds, x_dtype,
                       static_cast<hipStream_t>(hip_stream), true);
}

int lookupffn_gather_probes(const uint16_t *codes, const float *shares, const void *tables, float *y,
                            int64_t n_tokens, int k, int tau, int d_out, int table_dtype, void *hip_stream)
{
    int rc = check_gather(codes, tables, y, n_tokens, k, tau, d_out, table_dtype);
    if (rc == LFFN_OK) rc = check_weights(shares);
    if (rc != LFFN_OK || n_tokens == 0) return rc;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    LdsPlan plan;
    rc = plan_gather_lds(n_tokens, k, tau, d_out, table_dtype == LFFN_BF16, &plan, true, true);
    if (rc != LFFN_OK) return rc;
    if (plan.use && aligned(codes, 4)) {
        // staged form: packed codes and table-major shares in the library's buffer
        const int64_t pb = round256(packed_bytes(n_tokens, k));
        void *ws = nullptr;
        rc = own_workspace((size_t)(pb + probes_spk_bytes(n_tokens, k, tau)), &ws);
        if (rc != LFFN_OK) return rc;
        uint32_t *packed = static_cast<uint32_t *>(ws);
        float *spk = reinterpret_cast<float *>(static_cast<char *>(ws) + pb);
        rc = launch_repack_codes(codes, packed, n_tokens, plan.a.n_pad, k, tau, plan.shift, s);
        if (rc != LFFN_OK) return rc;
        rc = launch_repack_shares(shares, spk, n_tokens, plan.a.n_pad, k, tau, s);
        if (rc != LFFN_OK) return rc;
        return launch_gather_lds(plan, packed, spk, tables, y, false, s, true);
    }
    return launch_gather_direct(codes, shares, tables, y, n_tokens, k, tau, d_out, table_dtype, s, true);
}

int64_t lookupffn_workspace_bytes_probes(int64_t n_tokens, int k, int tau)
{
    if (n_tokens <= 0 || k < 1 || tau < 1 || tau > 16) return 0;
    // ABI codes and shares, and beside them the staged gather's packed codes and table-major shares
    return weighted_codes_bytes(n_tokens, k) + round256((int64_t)n_tokens * k * (tau + 1) * 4) +
           round256(packed_bytes(n_tokens, k)) + probes_spk_bytes(n_tokens, k, tau);
}

int lookupffn_forward_probes(const void *x, const int8_t *signs, const void *tables, float *y, int64_t n_tokens,
                             int d, int k, int tau, int d_out, int n_rounds, int x_dtype, int table_dtype,
                             void *workspace, int64_t workspace_bytes, void *hip_stream)
{
    const uint16_t *stand_in = reinterpret_cast<const uint16_t *>(uintptr_t(256));
    int rc = check_hash(x, signs, stand_in, n_tokens, d, k, tau, n_rounds, x_dtype, true);
    if (rc != LFFN_OK) return rc;
    rc = check_gather(stand_in, tables, y, n_tokens, k, tau, d_out, table_dtype);
    if (rc != LFFN_OK) return rc;
    const int64_t need = lookupffn_workspace_bytes_probes(n_tokens, k, tau);
    if (workspace) {
        if (workspace_bytes < need) return LFFN_E_WORKSPACE;
        if (!aligned(workspace, 256)) return LFFN_E_ALIGN;
    }
    if (n_tokens == 0) return LFFN_OK;
    void *ws = workspace;
    if (!ws) {
        rc = own_workspace((size_t)need, &ws);
        if (rc != LFFN_OK) return rc;
    }
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    uint16_t *codes = static_cast<uint16_t *>(ws);
    float *shares = reinterpret_cast<float *>(static_cast<char *>(ws) + weighted_codes_bytes(n_tokens, k));
    rc = launch_hash(x, signs, codes, nullptr, shares, n_tokens, d, k, tau, n_rounds, x_dtype, s, true);
    if (rc != LFFN_OK) return rc;
    LdsPlan plan;
    rc = plan_gather_lds(n_tokens, k, tau, d_out, table_dtype == LFFN_BF16, &plan, true, true);
    if (rc != LFFN_OK) return rc;
    if (plan.use) {
        char *staged = static_cast<char *>(ws) + weighted_codes_bytes(n_tokens, k) +
                       round256((int64_t)n_tokens * k * (tau + 1) * 4);
        uint32_t *packed = reinterpret_cast<uint32_t *>(staged);
        float *spk = reinterpret_cast<float *>(staged + round256(packed_bytes(n_tokens, k)));
        rc = launch_repack_codes(codes, packed, n_tokens, plan.a.n_pad, k, tau, plan.shift, s);
        if (rc != LFFN_OK) return rc;
        rc = launch_repack_shares(shares, spk, n_tokens, plan.a.n_pad, k, tau, s);
        if (rc != LFFN_OK) return rc;
        return launch_gather_lds(plan, packed, spk, tables, y, false, s, true);
    }
    return launch_gather_direct(codes, shares, tables, y, n_tokens, k, tau, d_out, table_dtype, s, true);
}

int64_t lookupffn_workspace_bytes_weighted(int64_t n_tokens, int k)
{
    if (n_tokens <= 0 || k < 1) return 0;
    const int64_t direct = weighted_codes_bytes(n_tokens, k) + round256((int64_t)n_tokens * k * 4);
    const int64_t staged = round256(packed_bytes(n_tokens, k)) + round256((int64_t)k * packed_n_pad(n_tokens) * 4);
    return direct + staged;  // both: the 64-byte-slice form re-packs from the ABI layout
}

int lookupffn_forward_weighted(const void *x, const int8_t *signs, const void *tables, float *y, int64_t n_tokens,
                               int d, int k, int tau, int d_out, int n_rounds, int x_dtype, int table_dtype,
                               void *workspace, int64_t workspace_bytes, void *hip_stream)
{
    const uint16_t *stand_in = reinterpret_cast<const uint16_t *>(uintptr_t(256));
    int rc = check_hash(x, signs, stand_in, n_tokens, d, k, tau, n_rounds, x_dtype, true);
    if (rc != LFFN_OK) return rc;
    rc = check_gather(stand_in, tables, y, n_tokens, k, tau, d_out, table_dtype);
    if (rc != LFFN_OK) return rc;
    const int64_t need = lookupffn_workspace_bytes_weighted(n_tokens, k);
    if (workspace) {
        if (workspace_bytes < need) return LFFN_E_WORKSPACE;
        if (!aligned(workspace, 256)) return LFFN_E_ALIGN;
    }
    if (n_tokens == 0) return LFFN_OK;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    const bool bf16 = table_dtype == LFFN_BF16;
    LdsPlan plan;
    rc = plan_gather_lds(n_tokens, k, tau, d_out, bf16, &plan, true, false, true);
    if (rc != LFFN_OK) return rc;
    const int64_t extra = widen_room(&plan, workspace, workspace_bytes, need);
    void *ws = workspace;
    if (!ws) {
        rc = own_workspace((size_t)(need + extra), &ws);
        if (rc != LFFN_OK) return rc;
    }
    plan.widened = extra ? static_cast<char *>(ws) + need : nullptr;
    if (plan.use && plan.shift != 7) {
        // 64-byte slices: ABI codes and weights, then the two re-pack kernels
        char *base = static_cast<char *>(ws);
        uint32_t *packed = reinterpret_cast<uint32_t *>(base);
        float *wpk = reinterpret_cast<float *>(base + round256(packed_bytes(n_tokens, k)));
        char *abi = base + round256(packed_bytes(n_tokens, k)) + round256((int64_t)k * packed_n_pad(n_tokens) * 4);
        uint16_t *codes = reinterpret_cast<uint16_t *>(abi);
        float *weights = reinterpret_cast<float *>(abi + weighted_codes_bytes(n_tokens, k));
        rc = launch_hash(x, signs, codes, nullptr, weights, n_tokens, d, k, tau, n_rounds, x_dtype, s);
        if (rc != LFFN_OK) return rc;
        rc = launch_repack_codes(codes, packed, n_tokens, plan.a.n_pad, k, tau, plan.shift, s);
        if (rc != LFFN_OK) return rc;
        rc = launch_repack_weights(weights, wpk, n_tokens, plan.a.n_pad, k, s);
        if (rc != LFFN_OK) return rc;
        return launch_gather_lds(plan, packed, wpk, tables, y, bf16, s);
    }
    if (plan.use) {
        uint32_t *packed = static_cast<uint32_t *>(ws);
        float *wpk = reinterpret_cast<float *>(static_cast<char *>(ws) + round256(packed_bytes(n_tokens, k)));
        rc = launch_hash(x, signs, nullptr, packed, wpk, n_tokens, d, k, tau, n_rounds, x_dtype, s);
        if (rc != LFFN_OK) return rc;
        return launch_gather_lds(plan, packed, wpk, tables, y, bf16, s);
    }
    uint16_t *codes = static_cast<uint16_t *>(ws);
    float *weights = reinterpret_cast<float *>(static_cast<char *>(ws) + weighted_codes_bytes(n_tokens, k));
    rc = launch_hash(x, signs, codes, nullptr, weights, n_tokens, d, k, tau, n_rounds, x_dtype, s);
    if (rc != LFFN_OK) return rc;
    return launch_gather_direct(codes, weights, tables, y, n_tokens, k, tau, d_out, table_dtype, s);
}

int lookupffn_gather(const uint16_t *codes, const void *tables, float *y, int64_t n_tokens, int k, int tau,
                     int d_out, int table_dtype, void *hip_stream)
{
    int rc = check_gather(codes, tables, y, n_tokens, k, tau, d_out, table_dtype);
    if (rc != LFFN_OK || n_tokens == 0) return rc;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    const bool bf16 = table_dtype == LFFN_BF16;
    LdsPlan plan;
    rc = plan_gather_lds(n_tokens, k, tau, d_out, bf16, &plan, false, false, true);
    if (rc != LFFN_OK) return rc;
    if (plan.use && aligned(codes, 4)) {
        // the staged kernel reads codes in its packed layout: repack into the library's buffer
        // (bf16 tables: their fp32 copy goes behind it)
        void *ws = nullptr;
        const int64_t pb = round256(packed_bytes(n_tokens, k));
        rc = own_workspace((size_t)(pb + plan.widen_bytes), &ws);
        if (rc != LFFN_OK) return rc;
        plan.widened = plan.widen ? static_cast<char *>(ws) + pb : nullptr;
        uint32_t *packed = static_cast<uint32_t *>(ws);
        rc = launch_repack_codes(codes, packed, n_tokens, plan.a.n_pad, k, tau, plan.shift, s);
        if (rc != LFFN_OK) return rc;
        return launch_gather_lds(plan, packed, nullptr, tables, y, bf16, s);
    }
    return launch_gather_direct(codes, nullptr, tables, y, n_tokens, k, tau, d_out, table_dtype, s);
}

int64_t lookupffn_workspace_bytes_tables(int k, int tau, int d_out, int table_dtype)
{
    if (table_dtype != LFFN_BF16 || k < 1 || tau < 1 || tau > 16 || d_out < 1) return 0;
    return round256((int64_t)k * (int64_t(1) << tau) * d_out * 4);
}

int64_t lookupffn_workspace_bytes(int64_t n_tokens, int k)
{
    if (n_tokens <= 0 || k < 1) return 0;
    // the packed layout with its token padding, and [n][k] uint16 beside it (the 64-byte-slice form of the
    // staged gather takes its codes through the re-pack kernel; otherwise only one of the two is used)
    return round256(packed_bytes(n_tokens, k)) + round256(n_tokens * (int64_t)k * 2);
}

int lookupffn_forward(const void *x, const int8_t *signs, const void *tables, float *y, int64_t n_tokens,
                      int d, int k, int tau, int d_out, int n_rounds, int x_dtype, int table_dtype,
                      void *workspace, int64_t workspace_bytes, void *hip_stream)
{
    // the codes pointer is checked for NULL by the two step checks; give them a stand-in
    // until the real buffer is known
    const uint16_t *stand_in = reinterpret_cast<const uint16_t *>(uintptr_t(256));
    int rc = check_hash(x, signs, stand_in, n_tokens, d, k, tau, n_rounds, x_dtype);
    if (rc != LFFN_OK) return rc;
    rc = check_gather(stand_in, tables, y, n_tokens, k, tau, d_out, table_dtype);
    if (rc != LFFN_OK) return rc;
    const int64_t need = lookupffn_workspace_bytes(n_tokens, k);
    if (workspace) {
        if (workspace_bytes < need) return LFFN_E_WORKSPACE;
        if (!aligned(workspace, 256)) return LFFN_E_ALIGN;
    }
    if (n_tokens == 0) return LFFN_OK;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    const bool bf16 = table_dtype == LFFN_BF16;
    LdsPlan plan;
    rc = plan_gather_lds(n_tokens, k, tau, d_out, bf16, &plan, false, false, true);
    if (rc != LFFN_OK) return rc;
    const int64_t extra = widen_room(&plan, workspace, workspace_bytes, need);
    void *ws = workspace;
    if (!ws) {
        rc = own_workspace((size_t)(need + extra), &ws);
        if (rc != LFFN_OK) return rc;
    }
    plan.widened = extra ? static_cast<char *>(ws) + need : nullptr;
    if (plan.use && plan.shift != 7) {
        // 64-byte slices: ABI codes, then the re-pack kernel scales them for 64-byte row pieces
        uint32_t *packed = static_cast<uint32_t *>(ws);
        uint16_t *codes = reinterpret_cast<uint16_t *>(static_cast<char *>(ws) + round256(packed_bytes(n_tokens, k)));
        rc = launch_hash(x, signs, codes, nullptr, nullptr, n_tokens, d, k, tau, n_rounds, x_dtype, s);
        if (rc != LFFN_OK) return rc;
        rc = launch_repack_codes(codes, packed, n_tokens, plan.a.n_pad, k, tau, plan.shift, s);
        if (rc != LFFN_OK) return rc;
        return launch_gather_lds(plan, packed, nullptr, tables, y, bf16, s);
    }
    if (plan.use) {
        uint32_t *packed = static_cast<uint32_t *>(ws);
        rc = launch_hash(x, signs, nullptr, packed, nullptr, n_tokens, d, k, tau, n_rounds, x_dtype, s);
        if (rc != LFFN_OK) return rc;
        return launch_gather_lds(plan, packed, nullptr, tables, y, bf16, s);
    }
    uint16_t *codes = static_cast<uint16_t *>(ws);
    rc = launch_hash(x, signs, codes, nullptr, nullptr, n_tokens, d, k, tau, n_rounds, x_dtype, s);
    if (rc != LFFN_OK) return rc;
    return launch_gather_direct(codes, nullptr, tables, y, n_tokens, k, tau, d_out, table_dtype, s);
}

int64_t lookupffn_workspace_bytes_bh(int64_t n_tokens, int d, int k, int tau, int block, int n_factors)
{
    if (d < 1 || d > 1024 || k < 1 || tau < 1 || tau > 16 || block < 1 || n_factors < 1 || n_factors > 64) return 0;
    return bh_pack_bytes(d, k, tau, block, n_factors) + lookupffn_workspace_bytes(n_tokens, k);
}

int lookupffn_hash_bh(const void *x, const float *bmats, uint16_t *codes, int64_t n_tokens, int d, int k, int tau,
                      int block, int n_factors, int x_dtype, void *workspace, int64_t workspace_bytes,
                      void *hip_stream)
{
    int rc = check_bh(x, bmats, n_tokens, d, k, tau, block, n_factors, x_dtype);
    if (rc != LFFN_OK) return rc;
    if (!codes) return LFFN_E_NULL;
    if (!aligned(codes, 2)) return LFFN_E_ALIGN;
    const int64_t need = bh_pack_bytes(d, k, tau, block, n_factors);
    if (workspace) {
        if (workspace_bytes < need) return LFFN_E_WORKSPACE;
        if (!aligned(workspace, 256)) return LFFN_E_ALIGN;
    }
    if (n_tokens == 0) return LFFN_OK;
    void *ws = workspace;
    if (!ws) {
        rc = own_workspace((size_t)need, &ws);
        if (rc != LFFN_OK) return rc;
    }
    return launch_hash_bh(x, bmats, static_cast<float *>(ws), codes, nullptr, n_tokens, d, k, tau, block, n_factors,
                          x_dtype, static_cast<hipStream_t>(hip_stream));
}

int lookupffn_forward_bh(const void *x, const float *bmats, const void *tables, float *y, int64_t n_tokens, int d,
                         int k, int tau, int d_out, int block, int n_factors, int x_dtype, int table_dtype,
                         void *workspace, int64_t workspace_bytes, void *hip_stream)
{
    int rc = check_bh(x, bmats, n_tokens, d, k, tau, block, n_factors, x_dtype);
    if (rc != LFFN_OK) return rc;
    const uint16_t *stand_in = reinterpret_cast<const uint16_t *>(uintptr_t(256));
    rc = check_gather(stand_in, tables, y, n_tokens, k, tau, d_out, table_dtype);
    if (rc != LFFN_OK) return rc;
    const int64_t pack = bh_pack_bytes(d, k, tau, block, n_factors);
    const int64_t need = pack + lookupffn_workspace_bytes(n_tokens, k);
    if (workspace) {
        if (workspace_bytes < need) return LFFN_E_WORKSPACE;
        if (!aligned(workspace, 256)) return LFFN_E_ALIGN;
    }
    if (n_tokens == 0) return LFFN_OK;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    const bool bf16 = table_dtype == LFFN_BF16;
    LdsPlan plan;
    rc = plan_gather_lds(n_tokens, k, tau, d_out, bf16, &plan, false, false, true);
    if (rc != LFFN_OK) return rc;
    if (plan.shift != 7) plan.use = false;  // the BH hash writes codes scaled for 128-byte row pieces only
    const int64_t extra = widen_room(&plan, workspace, workspace_bytes, need);
    void *ws = workspace;
    if (!ws) {
        rc = own_workspace((size_t)(need + extra), &ws);
        if (rc != LFFN_OK) return rc;
    }
    plan.widened = extra ? static_cast<char *>(ws) + need : nullptr;
    float *apack = static_cast<float *>(ws);
    void *scratch = static_cast<char *>(ws) + pack;
    if (plan.use) {
        uint32_t *packed = static_cast<uint32_t *>(scratch);
        rc = launch_hash_bh(x, bmats, apack, nullptr, packed, n_tokens, d, k, tau, block, n_factors, x_dtype, s);
        if (rc != LFFN_OK) return rc;
        return launch_gather_lds(plan, packed, nullptr, tables, y, bf16, s);
    }
    uint16_t *codes = static_cast<uint16_t *>(scratch);
    rc = launch_hash_bh(x, bmats, apack, codes, nullptr, n_tokens, d, k, tau, block, n_factors, x_dtype, s);
    if (rc != LFFN_OK) return rc;
    return launch_gather_direct(codes, nullptr, tables, y, n_tokens, k, tau, d_out, table_dtype, s);
}

int64_t lookupffn_workspace_bytes_bh_weighted(int64_t n_tokens, int d, int k, int tau, int block, int n_factors)
{
    if (d < 1 || d > 1024 || k < 1 || tau < 1 || tau > 16 || block < 1 || n_factors < 1 || n_factors > 64) return 0;
    return bh_pack_bytes(d, k, tau, block, n_factors) + lookupffn_workspace_bytes_weighted(n_tokens, k);
}

int lookupffn_hash_bh_weighted(const void *x, const float *bmats, uint16_t *codes, float *weights, int64_t n_tokens,
                               int d, int k, int tau, int block, int n_factors, int x_dtype, void *workspace,
                               int64_t workspace_bytes, void *hip_stream)
{
    int rc = check_bh(x, bmats, n_tokens, d, k, tau, block, n_factors, x_dtype, true);
    if (rc != LFFN_OK) return rc;
    if (!codes || !weights) return LFFN_E_NULL;
    if (!aligned(codes, 2) || !aligned(weights, 4)) return LFFN_E_ALIGN;
    const int64_t need = bh_pack_bytes(d, k, tau, block, n_factors);
    if (workspace) {
        if (workspace_bytes < need) return LFFN_E_WORKSPACE;
        if (!aligned(workspace, 256)) return LFFN_E_ALIGN;
    }
    if (n_tokens == 0) return LFFN_OK;
    void *ws = workspace;
    if (!ws) {
        rc = own_workspace((size_t)need, &ws);
        if (rc != LFFN_OK) return rc;
    }
    return launch_hash_bh(x, bmats, static_cast<float *>(ws), codes, nullptr, n_tokens, d, k, tau, block, n_factors,
                          x_dtype, static_cast<hipStream_t>(hip_stream), weights, nullptr);
}

int lookupffn_forward_bh_weighted(const void *x, const float *bmats, const void *tables, float *y, int64_t n_tokens,
                                  int d, int k, int tau, int d_out, int block, int n_factors, int x_dtype,
                                  int table_dtype, void *workspace, int64_t workspace_bytes, void *hip_stream)
{
    int rc = check_bh(x, bmats, n_tokens, d, k, tau, block, n_factors, x_dtype, true);
    if (rc != LFFN_OK) return rc;
    const uint16_t *stand_in = reinterpret_cast<const uint16_t *>(uintptr_t(256));
    rc = check_gather(stand_in, tables, y, n_tokens, k, tau, d_out, table_dtype);
    if (rc != LFFN_OK) return rc;
    const int64_t pack = bh_pack_bytes(d, k, tau, block, n_factors);
    const int64_t need = pack + lookupffn_workspace_bytes_weighted(n_tokens, k);
    if (workspace) {
        if (workspace_bytes < need) return LFFN_E_WORKSPACE;
        if (!aligned(workspace, 256)) return LFFN_E_ALIGN;
    }
    if (n_tokens == 0) return LFFN_OK;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    const bool bf16 = table_dtype == LFFN_BF16;
    LdsPlan plan;
    rc = plan_gather_lds(n_tokens, k, tau, d_out, bf16, &plan, true, false, true);
    if (rc != LFFN_OK) return rc;
    if (plan.shift != 7) plan.use = false;  // the BH hash writes codes scaled for 128-byte row pieces only
    const int64_t extra = widen_room(&plan, workspace, workspace_bytes, need);
    void *ws = workspace;
    if (!ws) {
        rc = own_workspace((size_t)(need + extra), &ws);
        if (rc != LFFN_OK) return rc;
    }
    plan.widened = extra ? static_cast<char *>(ws) + need : nullptr;
    float *apack = static_cast<float *>(ws);
    char *scratch = static_cast<char *>(ws) + pack;
    if (plan.use) {
        uint32_t *packed = reinterpret_cast<uint32_t *>(scratch);
        float *wpk = reinterpret_cast<float *>(scratch + round256(packed_bytes(n_tokens, k)));
        rc = launch_hash_bh(x, bmats, apack, nullptr, packed, n_tokens, d, k, tau, block, n_factors, x_dtype, s,
                            nullptr, wpk);
        if (rc != LFFN_OK) return rc;
        return launch_gather_lds(plan, packed, wpk, tables, y, bf16, s);
    }
    uint16_t *codes = reinterpret_cast<uint16_t *>(scratch);
    float *weights = reinterpret_cast<float *>(scratch + weighted_codes_bytes(n_tokens, k));
    rc = launch_hash_bh(x, bmats, apack, codes, nullptr, n_tokens, d, k, tau, block, n_factors, x_dtype, s, weights,
                        nullptr);
    if (rc != LFFN_OK) return rc;
    return launch_gather_direct(codes, weights, tables, y, n_tokens, k, tau, d_out, table_dtype, s);
}

int lookupffn_release_workspace(void)
{
    std::lock_guard<std::mutex> lk(g_ws_mu);
    int rc = LFFN_OK;
    for (auto &kv : g_ws) {
        if (!kv.second.ptr) continue;
        int cur = 0;
        if (hipGetDevice(&cur) != hipSuccess || hipSetDevice(kv.first) != hipSuccess ||
            hipDeviceSynchronize() != hipSuccess || hipFree(kv.second.ptr) != hipSuccess)
            rc = LFFN_E_HIP;
        (void)hipSetDevice(cur);
        kv.second = Workspace();
    }
    g_ws.clear();
    return rc;
}

int lookupffn_timing_enable(int mask)
{
    if (mask < 0 || mask > 3) return LFFN_E_SIZE;
    g_tm.on = mask;
    return LFFN_OK;
}

int lookupffn_timing_reset(void)
{
    for (auto &v : g_tm.ev) {
        for (auto &p : v) {
            (void)hipEventSynchronize(p.second);
            g_tm.pool.push_back(p);
        }
        v.clear();
    }
    return LFFN_OK;
}

int lookupffn_timing_read(int which, double *total_ms, int64_t *launches)
{
    if (which < 0 || which > 1) return LFFN_E_SIZE;
    if (!total_ms || !launches) return LFFN_E_NULL;
    double sum = 0.0;
    for (auto &p : g_tm.ev[which]) {
        LFFN_HIP(hipEventSynchronize(p.second));
        float ms = 0.0f;
        LFFN_HIP(hipEventElapsedTime(&ms, p.first, p.second));
        sum += ms;
    }
    *total_ms = sum;
    *launches = (int64_t)g_tm.ev[which].size();
    return LFFN_OK;
}

int lookupffn_set_option(const char *key, int value)
{
    if (!key) return LFFN_E_NULL;
    if (!std::strcmp(key, "lanes_per_token")) {
        if (value != 0 && (value < 1 || value > 64 || (value & (value - 1)))) return LFFN_E_SIZE;
        g_opt.lanes_per_token = value;
        return LFFN_OK;
    }
    if (!std::strcmp(key, "hash_path")) {
        if (value < 0 || value > 1) return LFFN_E_SIZE;
        g_opt.hash_path = value;
        return LFFN_OK;
    }
    if (!std::strcmp(key, "hash_blocks")) {
        if (value < 0 || value > 65536) return LFFN_E_SIZE;
        g_opt.hash_blocks = value;
        return LFFN_OK;
    }
    if (!std::strcmp(key, "slice_lanes")) {
        if (value != 0 && value != 4 && value != 8) return LFFN_E_SIZE;
        g_opt.slice_lanes = value;
        return LFFN_OK;
    }
    if (!std::strcmp(key, "token_slots")) {
        if (value != 0 && value != 4 && value != 8 && value != 13 && value != 16) return LFFN_E_SIZE;
        g_opt.token_slots = value;
        return LFFN_OK;
    }
    if (!std::strcmp(key, "gather_path")) {
        if (value < 0 || value > 2) return LFFN_E_SIZE;
        g_opt.gather_path = value;
        return LFFN_OK;
    }
    if (!std::strcmp(key, "xcd_order")) {
        if (value < -1 || value > 1) return LFFN_E_SIZE;
        g_opt.xcd_order = value;
        return LFFN_OK;
    }
    return LFFN_E_SIZE;
}

const char *lookupffn_strerror(int status)
{
    switch (status) {
        case LFFN_OK: return "success";
        case LFFN_E_NULL: return "a required pointer is NULL";
        case LFFN_E_SIZE: return "a size argument is out of range";
        case LFFN_E_TAU: return "tau must be in [1, 16]";
        case LFFN_E_DTYPE: return "unknown dtype";
        case LFFN_E_ALIGN: return "pointer alignment or d_out granularity not met";
        case LFFN_E_UNSUPPORTED: return "shape not supported (d_pad above 4096)";
        case LFFN_E_WORKSPACE: return "workspace too small";
        case LFFN_E_HIP: return "a HIP call failed";
        default: return "unknown status";
    }
}

const char *lookupffn_last_hip_error(void) { return g_hip_error.c_str(); }

const char *lookupffn_last_gather_kernel(void) { return g_last_gather; }

int lookupffn_version(void) { return kVersion; }

}  // extern "C"

#endif  // LFFN_HAS(0)
