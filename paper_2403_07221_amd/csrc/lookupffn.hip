// C ABI of the LookupFFN forward pass (declared in include/lookupffn.h): argument
// validation, launch-shape planning and kernel launches.  All arithmetic of the
// method is in hash_kernel.hpp and gather_kernel.hpp.
#include "lookupffn.h"

#include <hip/hip_runtime.h>

#include <atomic>
#include <cmath>
#include <cstring>
#include <map>
#include <mutex>
#include <string>
#include <vector>

#include "bh_hash_kernel.hpp"
#include "forward_stack_kernel.hpp"
#include "gather_kernel.hpp"
#include "gather_lds_kernel.hpp"
#include "gather_ring_kernel.hpp"
#include "hash_kernel.hpp"
#include "hash_row_kernel.hpp"

// Build parts.  This file compiles whole (LFFN_PART undefined) or as parts that are linked together, so
// that the kernel families compile side by side: part 0 holds the C ABI, the host logic and the hash and
// re-pack kernels; parts 1 .. 16 hold one family of kernel launchers each (declared just below).  No
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
// While an AttrOnly object lives on this thread, the launchers of kernels that need more than 64 KB of LDS
// only register that need with the runtime and launch nothing (lookupffn_init).
bool attr_only();                              // part 0
struct AttrOnly {
    AttrOnly();
    ~AttrOnly();
};
// part 1: the direct gather kernel
int gather_direct_part(int kind, int lpt, const GatherArgs &a, bool probes, dim3 grid, hipStream_t s);
int gather_direct_load();  // makes the runtime load part 1's code object now (lookupffn_init)
// parts 2, 3: the LDS-staged gather kernel (plain sum; weighted and multi-probe)
int gather_lds_plain_part(int tok, const GatherLdsArgs &a, int fr, int sw, dim3 grid, size_t lds, hipStream_t s);
int gather_lds_plain13_part(const GatherLdsArgs &a, int fr, dim3 grid, size_t lds, hipStream_t s);  // part 16
int gather_lds_weighted_part(int tok, const GatherLdsArgs &a, int fr, int sw, dim3 grid, size_t lds, hipStream_t s);
int gather_lds_probes_part(int tok, const GatherLdsArgs &a, int fr, int sw, dim3 grid, size_t lds, hipStream_t s);
// part 12: the lagged, bank-interleaved staged gather (prepared tables, tau <= 8)
int gather_ring_part(int threads, int tok, const GatherRingArgs &a, dim3 grid, hipStream_t s);
// part 13: hash and gather of a few tokens, one or several chained layers, in one launch
int forward_stack_part(int n_rounds, int kind, const StackArgs &a, dim3 grid, int threads, size_t lds, hipStream_t s);
int forward_stack_load();
// parts 14, 15: the hash with a token per row of lanes, d_pad = 1024 (four tokens per wavefront) and 512 (eight)
int hash_row16_part(int n_rounds, const HashArgs &a, dim3 grid, size_t lds, hipStream_t s);
int hash_row8_part(int n_rounds, const HashArgs &a, dim3 grid, size_t lds, hipStream_t s);
int hash_row16_load();
int hash_row8_load();
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
thread_local const char *t_last_gather = "";  // name of the gather kernel this thread's most recent launch used
thread_local const char *t_last_hash = "";    // the same for the hash kernel
thread_local int t_attr_only = 0;
#endif

// ---------------------------------------------------------------- kernel launchers (templates: every part may use them)
template <int KIND, int LPT>
void launch_gather_t(const GatherArgs &a, bool probes, dim3 grid, hipStream_t s)
{
    if (probes)
        hipLaunchKernelGGL((gather_kernel<KIND, LPT, 2>), grid, dim3(kGatherThreads), 0, s, a);
    else if (a.weights)
        hipLaunchKernelGGL((gather_kernel<KIND, LPT, 1>), grid, dim3(kGatherThreads), 0, s, a);
    else
        hipLaunchKernelGGL((gather_kernel<KIND, LPT, 0>), grid, dim3(kGatherThreads), 0, s, a);
}

template <int KIND>
int launch_gather_lpt(int lpt, const GatherArgs &a, bool probes, dim3 grid, hipStream_t s)
{
    switch (lpt) {
        case 1: launch_gather_t<KIND, 1>(a, probes, grid, s); break;
        case 2: launch_gather_t<KIND, 2>(a, probes, grid, s); break;
        case 4: launch_gather_t<KIND, 4>(a, probes, grid, s); break;
        case 8: launch_gather_t<KIND, 8>(a, probes, grid, s); break;
        case 16: launch_gather_t<KIND, 16>(a, probes, grid, s); break;
        case 32: launch_gather_t<KIND, 32>(a, probes, grid, s); break;
        case 64: launch_gather_t<KIND, 64>(a, probes, grid, s); break;
        default: return LFFN_E_UNSUPPORTED;
    }
    return LFFN_OK;
}

template <int TOK, int FR, bool WEIGHTED, int SW, bool PROBES = false>
int launch_gather_lds_fr(const GatherLdsArgs &a, dim3 grid, size_t lds, hipStream_t s)
{
    auto kern = gather_lds_kernel<TOK, FR, WEIGHTED, SW, PROBES>;
    int rc = allow_lds(reinterpret_cast<const void *>(kern), lds);
    if (rc != LFFN_OK || lffn_host::attr_only()) return rc;
    hipLaunchKernelGGL(kern, grid, dim3(kLdsThreads), lds, s, a);
    return LFFN_OK;
}

// fr = 16 KB copy rounds per table slice, sw = lanes per token (both fixed by the plan)
// SW8: this part also holds the 128-byte-slice form of TOK (part 16 holds the plain one with 13 slots)
template <int TOK, bool WEIGHTED = false, bool SW8 = true>
int launch_gather_lds_t(const GatherLdsArgs &a, int fr, int sw, dim3 grid, size_t lds, hipStream_t s)
{
    if constexpr (TOK <= 13 && SW8) {
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
    if (rc != LFFN_OK || lffn_host::attr_only()) return rc;
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
int gather_direct_part(int kind, int lpt, const GatherArgs &a, bool probes, dim3 grid, hipStream_t s)
{
    switch (kind) {
        case kElemF32: return launch_gather_lpt<kElemF32>(lpt, a, probes, grid, s);
        case kElemBF16: return launch_gather_lpt<kElemBF16>(lpt, a, probes, grid, s);
        case kElemF16: return launch_gather_lpt<kElemF16>(lpt, a, probes, grid, s);
    }
    return LFFN_E_DTYPE;
}

int gather_direct_load()
{
    hipFuncAttributes attr;
    hipError_t e = hipFuncGetAttributes(&attr, reinterpret_cast<const void *>(gather_kernel<kElemF32, 8, 0>));
    return e == hipSuccess ? LFFN_OK : hip_fail(e, "hipFuncGetAttributes(gather_kernel)");
}
#endif

#if LFFN_HAS(2)
int gather_lds_plain_part(int tok, const GatherLdsArgs &a, int fr, int sw, dim3 grid, size_t lds, hipStream_t s)
{
    if (tok <= 4) return launch_gather_lds_t<4>(a, fr, sw, grid, lds, s);
    if (tok <= 8) return launch_gather_lds_t<8>(a, fr, sw, grid, lds, s);
    if (tok <= 12) return launch_gather_lds_t<12>(a, fr, sw, grid, lds, s);
    if (tok <= 13 && sw == 8) return gather_lds_plain13_part(a, fr, grid, lds, s);
    if (tok <= 13) return launch_gather_lds_t<13, false, false>(a, fr, sw, grid, lds, s);
    if (tok <= 16 && sw == 4) return launch_gather_lds_t<16>(a, fr, sw, grid, lds, s);
    return LFFN_E_UNSUPPORTED;
}
#endif

#if LFFN_HAS(16)
// The plain sum with 13 token slots and 128-byte slices -- the kernel of the 16384-token benchmark layer -- is
// compiled on its own so that it can take the scheduler setting that suits it (see build.py).
int gather_lds_plain13_part(const GatherLdsArgs &a, int fr, dim3 grid, size_t lds, hipStream_t s)
{
    return fr == 4   ? launch_gather_lds_fr<13, 4, false, 8>(a, grid, lds, s)
           : fr == 2 ? launch_gather_lds_fr<13, 2, false, 8>(a, grid, lds, s)
                     : launch_gather_lds_fr<13, 1, false, 8>(a, grid, lds, s);
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

#if LFFN_HAS(12)
template <int THREADS, int TOK>
int launch_gather_ring_t(const GatherRingArgs &a, dim3 grid, hipStream_t s)
{
    auto kern = gather_ring_kernel<THREADS, TOK>;
    int rc = allow_lds(reinterpret_cast<const void *>(kern), kRingLdsBytes);
    if (rc != LFFN_OK || attr_only()) return rc;
    hipLaunchKernelGGL(kern, grid, dim3(THREADS), kRingLdsBytes, s, a);
    return LFFN_OK;
}

int gather_ring_part(int threads, int tok, const GatherRingArgs &a, dim3 grid, hipStream_t s)
{
    if (threads == 1024) {
        switch (tok) {
            case 4: return launch_gather_ring_t<1024, 4>(a, grid, s);
            case 8: return launch_gather_ring_t<1024, 8>(a, grid, s);
            case 12: return launch_gather_ring_t<1024, 12>(a, grid, s);
            case 13: return launch_gather_ring_t<1024, 13>(a, grid, s);
            case 14: return launch_gather_ring_t<1024, 14>(a, grid, s);
        }
    } else if (threads == 512) {
        switch (tok) {
            case 8: return launch_gather_ring_t<512, 8>(a, grid, s);
            case 16: return launch_gather_ring_t<512, 16>(a, grid, s);
            case 20: return launch_gather_ring_t<512, 20>(a, grid, s);
            case 24: return launch_gather_ring_t<512, 24>(a, grid, s);
            case 28: return launch_gather_ring_t<512, 28>(a, grid, s);
            case 32: return launch_gather_ring_t<512, 32>(a, grid, s);
        }
    }
    return LFFN_E_UNSUPPORTED;
}
#endif

#if LFFN_HAS(13)
template <int R>
int launch_forward_stack_r(int kind, const StackArgs &a, dim3 grid, int threads, size_t lds, hipStream_t s)
{
    switch (kind) {
        case kElemF32: hipLaunchKernelGGL((forward_stack_kernel<R, kElemF32>), grid, dim3(threads), lds, s, a); break;
        case kElemBF16: hipLaunchKernelGGL((forward_stack_kernel<R, kElemBF16>), grid, dim3(threads), lds, s, a); break;
        case kElemF16: hipLaunchKernelGGL((forward_stack_kernel<R, kElemF16>), grid, dim3(threads), lds, s, a); break;
        default: return LFFN_E_DTYPE;
    }
    return LFFN_OK;
}

int forward_stack_part(int n_rounds, int kind, const StackArgs &a, dim3 grid, int threads, size_t lds, hipStream_t s)
{
    if (threads < 64 || threads > 1024 || threads % 64) return LFFN_E_UNSUPPORTED;
    switch (n_rounds) {
        case 1: return launch_forward_stack_r<1>(kind, a, grid, threads, lds, s);
        case 2: return launch_forward_stack_r<2>(kind, a, grid, threads, lds, s);
        case 3: return launch_forward_stack_r<3>(kind, a, grid, threads, lds, s);
        case 4: return launch_forward_stack_r<4>(kind, a, grid, threads, lds, s);
    }
    return LFFN_E_UNSUPPORTED;
}

int forward_stack_load()
{
    hipFuncAttributes attr;
    hipError_t e = hipFuncGetAttributes(&attr, reinterpret_cast<const void *>(forward_stack_kernel<3, kElemF32>));
    return e == hipSuccess ? LFFN_OK : hip_fail(e, "hipFuncGetAttributes(forward_stack_kernel)");
}
#endif

#if LFFN_HAS(14) || LFFN_HAS(15)
// WMODE of the lane-row kernel: 0 codes only, 1 weights reduced in registers (tau divides the lanes of a token),
// 2 weights of any tau through the z window
inline int row_wmode(const HashArgs &a, int lpt) { return !(a.weights || a.wpk) ? 0 : lpt % a.tau == 0 ? 1 : 2; }

template <int MFULL, int WMODE, int LPT>
int launch_hash_row_r(int n_rounds, const HashArgs &a, dim3 grid, size_t lds, hipStream_t s)
{
    switch (n_rounds) {
        case 1: hipLaunchKernelGGL((hash_row_kernel<1, MFULL, WMODE, LPT>), grid, dim3(kRowThreads), lds, s, a); break;
        case 2: hipLaunchKernelGGL((hash_row_kernel<2, MFULL, WMODE, LPT>), grid, dim3(kRowThreads), lds, s, a); break;
        case 3: hipLaunchKernelGGL((hash_row_kernel<3, MFULL, WMODE, LPT>), grid, dim3(kRowThreads), lds, s, a); break;
        case 4: hipLaunchKernelGGL((hash_row_kernel<4, MFULL, WMODE, LPT>), grid, dim3(kRowThreads), lds, s, a); break;
        default: return LFFN_E_UNSUPPORTED;
    }
    return LFFN_OK;
}

// MFULL: the kernel built for one row length, three rounds; else the form with run-time bounds
template <int MFULL, int LPT>
int launch_hash_row_m(int n_rounds, const HashArgs &a, dim3 grid, size_t lds, hipStream_t s)
{
    const int wmode = row_wmode(a, LPT);
    if (MFULL != 0) {
        if (wmode == 0) hipLaunchKernelGGL((hash_row_kernel<3, MFULL, 0, LPT>), grid, dim3(kRowThreads), lds, s, a);
        else if (wmode == 1) hipLaunchKernelGGL((hash_row_kernel<3, MFULL, 1, LPT>), grid, dim3(kRowThreads), lds, s, a);
        else hipLaunchKernelGGL((hash_row_kernel<3, MFULL, 2, LPT>), grid, dim3(kRowThreads), lds, s, a);
        return LFFN_OK;
    }
    return wmode == 0   ? launch_hash_row_r<0, 0, LPT>(n_rounds, a, grid, lds, s)
           : wmode == 1 ? launch_hash_row_r<0, 1, LPT>(n_rounds, a, grid, lds, s)
                        : launch_hash_row_r<0, 2, LPT>(n_rounds, a, grid, lds, s);
}
#endif

#if LFFN_HAS(14)
int hash_row16_part(int n_rounds, const HashArgs &a, dim3 grid, size_t lds, hipStream_t s)
{
    // built for the row lengths of the paper's models (d = 768 and 1024, three rounds); any other multiple of
    // 16 in range takes the form with run-time bounds
    if (n_rounds == 3 && a.d == 768) return launch_hash_row_m<48, 16>(3, a, grid, lds, s);
    if (n_rounds == 3 && a.d == 1024) return launch_hash_row_m<64, 16>(3, a, grid, lds, s);
    return launch_hash_row_m<0, 16>(n_rounds, a, grid, lds, s);
}

int hash_row16_load()
{
    hipFuncAttributes attr;
    hipError_t e = hipFuncGetAttributes(&attr, reinterpret_cast<const void *>(hash_row_kernel<3, 0, 0, 16>));
    return e == hipSuccess ? LFFN_OK : hip_fail(e, "hipFuncGetAttributes(hash_row_kernel, 16 lanes per token)");
}
#endif

#if LFFN_HAS(15)
int hash_row8_part(int n_rounds, const HashArgs &a, dim3 grid, size_t lds, hipStream_t s)
{
    if (n_rounds == 3 && a.d == 512) return launch_hash_row_m<64, 8>(3, a, grid, lds, s);  // the paper's small models
    return launch_hash_row_m<0, 8>(n_rounds, a, grid, lds, s);
}

int hash_row8_load()
{
    hipFuncAttributes attr;
    hipError_t e = hipFuncGetAttributes(&attr, reinterpret_cast<const void *>(hash_row_kernel<3, 0, 0, 8>));
    return e == hipSuccess ? LFFN_OK : hip_fail(e, "hipFuncGetAttributes(hash_row_kernel, 8 lanes per token)");
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

bool attr_only() { return t_attr_only > 0; }
AttrOnly::AttrOnly() { ++t_attr_only; }
AttrOnly::~AttrOnly() { --t_attr_only; }

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

bool dtype_ok(int t) { return t == LFFN_F32 || t == LFFN_BF16 || t == LFFN_F16; }
static_assert((int)LFFN_F32 == (int)kElemF32 && (int)LFFN_BF16 == (int)kElemBF16 && (int)LFFN_F16 == (int)kElemF16, "the ABI's dtype codes are the kernels' element kinds");
bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }
int gcd(int a, int b) { return b ? gcd(b, a % b) : a; }
int64_t round256(int64_t b) { return (b + 255) & ~int64_t(255); }

// ---------------------------------------------------------------- options
// Tuning knobs (lookupffn_set_option).  Every entry point takes one snapshot at its start, so a
// concurrent lookupffn_set_option can change which kernel the NEXT call runs, never a call in flight.
struct Options {
    int lanes_per_token = 0;  // 0 = default
    int xcd_order = 0;        // 0 = default, 1 = on, -1 = off
    int gather_path = 0;      // 0 = choose, 1 = direct kernel, 2 = the staged kernel whenever the shape allows,
                              // 4 = the ring kernel whenever the shape allows (else as 2)
    int hash_path = 0;        // 0 = choose, 1 = generic kernel only, 2 = no token-per-lane-row kernel, 3 = that kernel for every batch size
    int hash_blocks = 0;      // 0 = default grid cap of the d_pad = 1024 hash kernel
    int slice_lanes = 0;      // 0 = choose, 4 = 64-byte column slices in the staged gather where possible
    int token_slots = 0;      // 0 = choose, else the most token slots per lane of the staged gather
    int ring_threads = 0;     // 0 = choose, 512 / 1024 = workgroup size of the ring gather
    int small_tokens = 0;     // 0 = default, -1 = never: up to this many tokens lookupffn_forward runs as one
                              // hash-and-gather launch (when the shape is that kernel's)
};
constexpr int kSmallTokensDefault = 512;  // k = 96, d_out = 768: 23 us against 33 us at 512 tokens, even at about 900
std::mutex g_opt_mu;
Options g_opt;
Options options_snapshot()
{
    std::lock_guard<std::mutex> lk(g_opt_mu);
    return g_opt;
}

// ---------------------------------------------------------------- timing
struct Timing {
    std::mutex mu;
    std::atomic<int> on{0};  // bit 0: time hash launches, bit 1: time gather launches
    std::vector<std::pair<hipEvent_t, hipEvent_t>> ev[2];
    std::vector<std::pair<hipEvent_t, hipEvent_t>> pool;
} g_tm;

struct TimedLaunch {
    int which;
    hipStream_t s;
    hipEvent_t a = nullptr, b = nullptr;
    bool on;
    TimedLaunch(int which_, hipStream_t s_) : which(which_), s(s_), on((g_tm.on.load() >> which_) & 1)
    {
        if (!on) return;
        {
            std::lock_guard<std::mutex> lk(g_tm.mu);
            if (!g_tm.pool.empty()) {
                a = g_tm.pool.back().first;
                b = g_tm.pool.back().second;
                g_tm.pool.pop_back();
            }
        }
        if (!a && (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess)) {
            on = false;
            return;
        }
        on = hipEventRecord(a, s) == hipSuccess;
    }
    void done()
    {
        if (!on || !a || !b) return;
        (void)hipEventRecord(b, s);
        std::lock_guard<std::mutex> lk(g_tm.mu);
        g_tm.ev[which].emplace_back(a, b);
    }
};

// ---------------------------------------------------------------- library-owned workspace (workspace == NULL)
// Grow-only: a larger request allocates a new buffer and keeps the old ones until
// lookupffn_release_workspace(), so work already enqueued (or captured) with an old buffer stays valid and
// nothing synchronises.
struct Workspace {
    void *ptr = nullptr;
    size_t bytes = 0;
    std::vector<void *> retired;
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
        const size_t sz = (need + (size_t(1) << 20) - 1) & ~((size_t(1) << 20) - 1);
        void *p = nullptr;
        LFFN_HIP(hipMalloc(&p, sz));
        if (w.ptr) w.retired.push_back(w.ptr);
        w.ptr = p;
        w.bytes = sz;
    }
    *out = w.ptr;
    return LFFN_OK;
}

// A call's scratch memory, handed out front to back in 256-byte aligned pieces.
struct Scratch {
    char *base = nullptr;
    int64_t bytes = 0, used = 0;
    template <class T>
    T *take(int64_t n)
    {
        n = round256(n);
        if (!base || used + n > bytes) return nullptr;
        T *p = reinterpret_cast<T *>(base + used);
        used += n;
        return p;
    }
};

// Resolves the (workspace, workspace_bytes) pair of an entry point: the caller's buffer, or the library's.
int get_scratch(void *workspace, int64_t workspace_bytes, int64_t need, Scratch *sc)
{
    if (workspace) {
        if (workspace_bytes < need) return LFFN_E_WORKSPACE;
        if (!aligned(workspace, 256)) return LFFN_E_ALIGN;
        sc->base = static_cast<char *>(workspace);
        sc->bytes = workspace_bytes;
        return LFFN_OK;
    }
    if (need == 0) return LFFN_OK;
    void *p = nullptr;
    int rc = own_workspace((size_t)need, &p);
    if (rc != LFFN_OK) return rc;
    sc->base = static_cast<char *>(p);
    sc->bytes = need;
    return LFFN_OK;
}

// ---------------------------------------------------------------- static scratch (lookupffn_forward_static)
// Device memory that exists from the moment the code object is loaded: the workspace of the entry point
// for callers that cannot allocate.  Every GPU the library runs on holds its own copy until the process
// ends.  The name is a host-side stand-in, not a device address: host code uses the address
// hipGetSymbolAddress returns for the current device (kept per device below), never the name.
constexpr int64_t kStaticScratchBytes = int64_t(16) << 20;
static __device__ __align__(256) __attribute__((used)) unsigned char scratch[kStaticScratchBytes];

std::mutex g_static_mu;
std::map<int, void *> g_static_ptr;  // device -> address of that device's copy of `scratch`

int static_scratch(void **out)
{
    int dev = 0;
    LFFN_HIP(hipGetDevice(&dev));
    std::lock_guard<std::mutex> lk(g_static_mu);
    auto it = g_static_ptr.find(dev);
    if (it == g_static_ptr.end()) {
        void *p = nullptr;
        LFFN_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p || !aligned(p, 256)) return hip_fail(hipErrorInvalidSymbol, "hipGetSymbolAddress(scratch)");
        it = g_static_ptr.emplace(dev, p).first;
    }
    *out = it->second;
    return LFFN_OK;
}

// ---------------------------------------------------------------- tables: row-major or prepared
// Bytes per row piece of the prepared (slice-major) layout: 128 up to tau = 8 (the staged gather's
// 128-byte column slices; its 64-byte form reads half pieces), 64 from tau = 9 on.
int prepared_piece_bytes(int tau) { return tau <= 8 ? 128 : 64; }

struct TableRef {
    const char *p = nullptr;
    int kind = kElemF32;    // element type of the buffer the kernels read (prepared tables are always fp32)
    bool prepared = false;
    int pw = 0;             // prepared: bytes per row piece
    int y_kind = kElemF32;  // storage type of the output rows (LFFN_Y_BF16 / LFFN_Y_F16 in table_dtype)
};

TableRef table_ref(const void *tables, int table_dtype, int tau)
{
    TableRef t;
    t.p = static_cast<const char *>(tables);
    t.prepared = (table_dtype & LFFN_PREPARED) != 0;
    t.kind = t.prepared ? kElemF32 : (table_dtype & 0xFF);  // LFFN_F32 / BF16 / F16 are the kernels' kinds 0 / 1 / 2
    t.pw = t.prepared ? prepared_piece_bytes(tau) : 0;
    t.y_kind = (table_dtype & LFFN_Y_BF16) ? kElemBF16 : (table_dtype & LFFN_Y_F16) ? kElemF16 : kElemF32;
    return t;
}

int64_t prepared_tables_bytes(int k, int tau, int d_out)
{
    const int64_t pw = prepared_piece_bytes(tau);
    const int64_t n_ps = ((int64_t)d_out * 4 + pw - 1) / pw;
    return round256(n_ps * k * (int64_t(1) << tau) * pw);
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

int check_gather(const uint16_t *codes, const void *tables, const void *y, int64_t n, int k, int tau,
                 int d_out, int table_dtype)
{
    if (!codes || !tables || !y) return LFFN_E_NULL;
    if (n < 0 || k < 1 || d_out < 1) return LFFN_E_SIZE;
    if (tau < 1 || tau > 16) return LFFN_E_TAU;
    if ((table_dtype & ~(0xFF | LFFN_PREPARED | LFFN_Y_BF16 | LFFN_Y_F16)) != 0 || !dtype_ok(table_dtype & 0xFF))
        return LFFN_E_DTYPE;
    if ((table_dtype & LFFN_Y_BF16) && (table_dtype & LFFN_Y_F16)) return LFFN_E_DTYPE;
    if (k > (1 << 20) || n > (int64_t(1) << 40) || d_out > (1 << 24)) return LFFN_E_SIZE;
    const int w = (table_dtype & 0xFF) == LFFN_F32 ? 4 : 8;
    if (d_out % w != 0) return LFFN_E_ALIGN;
    const size_t ta = (table_dtype & LFFN_PREPARED) ? 256 : 16;
    const size_t ya = (table_dtype & (LFFN_Y_BF16 | LFFN_Y_F16)) ? 8 : 16;  // four outputs are stored at a time
    if (!aligned(tables, ta) || !aligned(y, ya) || !aligned(codes, 2)) return LFFN_E_ALIGN;
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

// What a hash launch writes: codes[n][k] (and weights[n][k], or shares[n][k][1+tau] with `probes`), or --
// when `codes` is NULL -- the staged gather's packed codes (and table-major weights wpk[k][n_pad]).
struct HashOut {
    uint16_t *codes = nullptr;
    uint32_t *packed = nullptr;
    float *weights = nullptr;  // beside `codes`: [n][k] or [n][k][1+tau]; beside `packed`: wpk[k][n_pad]
    bool probes = false;
    int shift = kPackedShift;  // what the packed codes are scaled by: log2 of the staged gather's row-piece bytes
};

// Host-side extent check of one hash launch: every index the kernels form from (n, k, tau, n_pad)
// stays inside the buffers the caller of launch_hash carved out.  `cap_*` are the byte sizes of the
// regions behind out.codes / out.packed / out.weights (0 = unknown: a caller-owned ABI output).
bool hash_extents_ok(const HashOut &o, int64_t n, int k, int tau, int64_t n_pad, int64_t cap_codes,
                     int64_t cap_packed, int64_t cap_weights)
{
    if (o.codes) {
        if (cap_codes && n * k * 2 > cap_codes) return false;
        const int64_t per = o.probes ? (int64_t)k * (tau + 1) : k;
        if (o.weights && cap_weights && n * per * 4 > cap_weights) return false;
        return true;
    }
    // packed[s * n_pad + t], s < k/2, t < n_pad;  wpk[j * n_pad + t], j < k, t < n
    if (n_pad < n) return false;
    if (cap_packed && (int64_t)(k / 2) * n_pad * 4 > cap_packed) return false;
    if (o.weights && cap_weights && ((int64_t)(k - 1) * n_pad + n) * 4 > cap_weights) return false;
    return true;
}

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

int launch_hash(const void *x, const int8_t *signs, const HashOut &out, int64_t n, int d, int k, int tau,
                int n_rounds, int x_dtype, hipStream_t s, const Options &opt)
{
    const int L = log2_pad(d);
    const int N = 1 << L;
    HashArgs a{};
    a.x = x;
    a.signs = signs;
    a.codes = out.codes;
    a.packed = out.codes ? nullptr : out.packed;
    a.weights = out.codes ? out.weights : nullptr;
    a.wpk = out.codes ? nullptr : out.weights;
    a.n_pad = packed_n_pad(n);
    a.packed_shift = out.shift;
    a.n = n;
    a.d = d;
    a.k = k;
    a.tau = tau;
    a.n_rounds = n_rounds;
    a.P = (int)(((int64_t)k * tau + N - 1) / N);
    a.x_kind = x_dtype;  // LFFN_F32 / BF16 / F16 are the kernels' kinds 0 / 1 / 2
    a.scale = (float)(1.0 / std::sqrt((double)N));
    if (!a.codes && !a.packed) return LFFN_E_NULL;
    if (out.probes && (!a.codes || !a.weights)) return LFFN_E_UNSUPPORTED;  // shares exist in the ABI layout only
    TimedLaunch tl(0, s);
    // d_pad = 1024 or 512, up to four rounds, codes alone or with the gather weights (reduced in registers when
    // tau divides the lanes of a token: a table is then a run of lanes of one register; else through a z window
    // in LDS): a token per row of 16 (8) lanes, four (eight) tokens per wavefront, no LDS transposes.  A lane holds every 16th (8th) coordinate: d a multiple
    // of 16 makes "in range" a per-register question.
    // It needs a batch that gives most SIMDs two waves of tokens to pull ahead; below that one group's latency
    // decides and the one-token kernels are faster.  Measured crossovers: d_pad = 1024 about 2048 tokens (4096
    // with weights), d_pad = 512 (twice the tokens per wave) about 6000 (10000 with weights).
    const int lpt = L == 10 ? 16 : 8;
    const bool row_weights_ok = !out.weights || !out.probes;
    const bool row_window = out.weights && lpt % tau != 0;  // weights through the z window in LDS
    const int64_t row_from = lpt == 16 ? (out.weights ? 4096 : 2048) : (out.weights ? 12288 : 6144);
    const bool row_wanted = opt.hash_path == 3 || (opt.hash_path == 0 && n >= row_from);
    if (row_wanted && (L == 10 || L == 9) && d % 16 == 0 && n_rounds >= 1 && n_rounds <= 4 && row_weights_ok &&
        aligned(signs, 16) && hrow_lds_bytes(a.P, n_rounds, lpt, row_window) <= 64 * 1024) {
        // two workgroups per compute unit fill it (two waves per SIMD); a larger batch is worked through in
        // several groups of tokens per wave, the next group's rows in flight during a transform
        int cus = 0;
        int rc = device_cus(&cus);
        if (rc != LFFN_OK) return rc;
        const int64_t groups = (n + 64 / lpt - 1) / (64 / lpt);
        int64_t blocks = (groups + kRowWaves - 1) / kRowWaves;
        const int64_t cap = opt.hash_blocks ? opt.hash_blocks : 2 * (int64_t)cus;
        if (blocks > cap) blocks = cap;
        const size_t lds = hrow_lds_bytes(a.P, n_rounds, lpt, row_window);
        rc = lpt == 16 ? lffn_host::hash_row16_part(n_rounds, a, dim3((unsigned)blocks), lds, s)
                       : lffn_host::hash_row8_part(n_rounds, a, dim3((unsigned)blocks), lds, s);
        if (rc != LFFN_OK) return rc;
        LFFN_HIP(hipGetLastError());
        tl.done();
        t_last_hash = "hash_row_kernel";
        return LFFN_OK;
    }
    // d_pad = 1024 with up to four rounds: the two-layout kernel (needs 16-byte aligned signs, and
    // rows that start on 16-byte boundaries when it loads them as vectors)
    const size_t xrow = (size_t)d * (a.x_kind ? 2 : 4);
    const bool weighted = out.weights != nullptr;
    if (opt.hash_path != 1 && L == 10 && n_rounds <= 4 && aligned(signs, 16) &&
        h1024_lds_bytes(a.P, weighted) <= 64 * 1024 &&
        (d % 4 != 0 || (aligned(x, 16) && xrow % (a.x_kind ? 8 : 16) == 0))) {
        int64_t blocks = (n + kHashWaves - 1) / kHashWaves;
        const int64_t cap = opt.hash_blocks ? opt.hash_blocks : 4096;
        if (blocks > cap) blocks = cap;
        const dim3 grid((unsigned)blocks);
        const size_t lds = h1024_lds_bytes(a.P, weighted);
        switch (n_rounds) {
            case 1: launch_hash1024_t<1>(a, out.probes, grid, lds, s); break;
            case 2: launch_hash1024_t<2>(a, out.probes, grid, lds, s); break;
            case 3: launch_hash1024_t<3>(a, out.probes, grid, lds, s); break;
            default: launch_hash1024_t<4>(a, out.probes, grid, lds, s); break;
        }
        LFFN_HIP(hipGetLastError());
        tl.done();
        t_last_hash = "hash1024_kernel";
        return LFFN_OK;
    }
    const size_t lds = hash_lds_bytes(a.P, n_rounds, N, weighted);
    int64_t blocks = (n + kHashWaves - 1) / kHashWaves;
    if (blocks > 2048) blocks = 2048;
    const dim3 grid((unsigned)blocks);
    switch (L) {
#define LFFN_CASE(l) case l: launch_hash_t<l>(a, out.probes, grid, lds, s); break;
        LFFN_CASE(0) LFFN_CASE(1) LFFN_CASE(2) LFFN_CASE(3) LFFN_CASE(4) LFFN_CASE(5) LFFN_CASE(6)
        LFFN_CASE(7) LFFN_CASE(8) LFFN_CASE(9) LFFN_CASE(10) LFFN_CASE(11) LFFN_CASE(12)
#undef LFFN_CASE
        default: return LFFN_E_UNSUPPORTED;
    }
    LFFN_HIP(hipGetLastError());
    tl.done();
    t_last_hash = "hash_kernel";
    return LFFN_OK;
}

constexpr int kLdsMinBytes = 84 * 1024;  // more than half of the 160 KB LDS: one workgroup per CU

// Largest number of tokens a workgroup gets in one piece, mirroring the kernel's split.
int64_t lds_tokens_per_block(int64_t n, int n_units, int token_splits, int Bx)
{
    const int m = (n_units + kXcds - 1) / kXcds;  // units of the fullest XCD
    const int64_t unit_tokens = (n + token_splits - 1) / token_splits;
    if (m >= Bx) return unit_tokens;
    const int blocks = Bx / m;  // the unit with the fewest workgroups
    return (unit_tokens + blocks - 1) / blocks;
}

enum Mode { kPlain = 0, kWeighted = 1, kProbes = 2 };

// Launch shape of the LDS-staged gather for one problem size (no pointers involved).
struct LdsPlan {
    bool use = false;
    GatherLdsArgs a{};
    int tok = 0;
    int sw = 8;     // lanes per token: 8 = 128-byte column slices, 4 = 64-byte ones
    int fr = 1;     // 16 KB copy rounds per table slice
    int shift = 7;  // log2 of the row-piece bytes: what the packed codes are scaled by (the hash kernels and the
                    // re-pack kernel scale by whatever the plan says)
    unsigned grid = 0;
    size_t lds = 0;
    int tail = 0;   // tables left to the direct kernel, which adds them onto the staged kernel's y: 1 when
                    // k is odd (the staged kernel takes its tables in pairs), else 0
};

int plan_gather_lds(int64_t n, int k, int tau, int d_out, const TableRef &T, Mode mode, const Options &opt,
                    LdsPlan *p)
{
    p->use = false;
    if (opt.gather_path == 1) return LFFN_OK;
    if (T.kind) return LFFN_OK;  // the staged kernel reads fp32 rows: 16-bit tables take it once prepared
    const int rows = 1 << tau;
    if (tau < 7 || tau > 10) return LFFN_OK;
    // an odd k: the first k - 1 tables staged, the last one added by the direct kernel, which re-reads the
    // fp32 sums (so not with 16-bit outputs, which are rounded once from the complete sum)
    const int tail = k & 1;
    if (tail && (k < 3 || T.y_kind != 0)) return LFFN_OK;
    // column slices: 128 bytes (8 lanes per token) up to tau = 8; 64 bytes from tau = 9 on (two 512-row
    // tables per stage and half the copy volume per token measured faster than one per stage; tau = 10
    // fits a 64 KB buffer only this way).  The 64-byte form exists for tau >= 8.
    int sw = tau <= 8 ? 8 : 4;
    if (opt.slice_lanes == 4 && tau >= 8) sw = 4;
    if (opt.slice_lanes == 8 && tau <= 9) sw = 8;
    if (mode == kProbes) sw = tau <= 8 ? 8 : 4;  // the multi-probe form is built for these pairings only
    if (T.prepared && sw * 16 > T.pw) sw = T.pw / 16;  // a token's row piece must lie inside one prepared piece
    if (sw == 4 && tau < 8) return LFFN_OK;
    const int groups = kLdsThreads / sw;
    // the kernel indexes tokens and bytes inside one table with 32 bits
    if (n >= (int64_t(1) << 31) - 4096 || (int64_t)rows * d_out * 4 >= (int64_t(1) << 32)) return LFFN_OK;
    int cus = 0;
    int rc = device_cus(&cus);
    if (rc != LFFN_OK) return rc;
    if (cus < kXcds || cus % kXcds != 0) return LFFN_OK;
    GatherLdsArgs &a = p->a;
    a = GatherLdsArgs{};
    a.n = n;
    a.n_pad = packed_n_pad(n);
    a.k = k - tail;
    a.tau = tau;
    a.d_out = d_out;
    const uint32_t row_bytes = (uint32_t)d_out * 4;  // of the fp32 rows the kernel reads
    a.nvec = (int)(row_bytes / 16);
    a.n_slices = (a.nvec + sw - 1) / sw;
    a.token_splits = kXcds / gcd(a.n_slices, kXcds);
    a.n_units = a.n_slices * a.token_splits;
    a.blocks_per_xcd = cus / kXcds;
    if (T.prepared) {
        a.spp = (uint32_t)(T.pw / (sw * 16));
        a.row_stride = (uint32_t)T.pw;
        a.table_stride = (unsigned long long)rows * T.pw;
        a.slice_stride = (unsigned long long)k * rows * T.pw;
    } else {
        a.spp = 1;
        a.row_stride = row_bytes;
        a.table_stride = (unsigned long long)rows * row_bytes;
        a.slice_stride = (unsigned long long)sw * 16;
    }
    const int64_t tpb = lds_tokens_per_block(n, a.n_units, a.token_splits, a.blocks_per_xcd);
    int tok_max = sw == 4 ? 16 : 13;
    // the multi-probe form holds a share per probe beside the accumulators: 13 slots spill in its
    // hot loop, 8 measured faster up to tau = 9 (tau = 10 has 16 copy rounds per table to amortise)
    if (mode == kProbes && tau <= 9) tok_max = 8;
    if (opt.token_slots && opt.token_slots < tok_max) tok_max = opt.token_slots;
    const int64_t nchunks = (tpb + (int64_t)groups * tok_max - 1) / ((int64_t)groups * tok_max);
    const int64_t chunk = (tpb + nchunks - 1) / nchunks;
    // Staging pays only when a chunk re-uses each staged row a few times.
    if (opt.gather_path < 2 && chunk < 2 * (int64_t)rows) return LFFN_OK;
    p->tok = (int)((chunk + groups - 1) / groups);
    if (mode == kProbes && sw == 8 && p->tok > 8) p->tok = 13;  // multi-probe form: 4, 8 or 13 slots
    if (sw == 4) p->tok = p->tok > 13 ? 16 : p->tok > 8 ? 13 : 8;  // the 64-byte form is built for 8, 13 and 16 token slots
    p->sw = sw;
    p->fr = rows / groups;
    p->shift = sw == 8 ? 7 : 6;
    p->lds = gather_lds_bytes(tau, sw);
    if (p->lds < (size_t)kLdsMinBytes) p->lds = kLdsMinBytes;
    p->grid = (unsigned)cus;
    p->tail = tail;
    p->use = true;
    return LFFN_OK;
}

// Byte counts of the scratch regions.  The arguments may be anything a caller passes to a size query, so
// the products are formed in 128 bits and a count that no buffer can have saturates at kBytesMax (every
// workspace is then too small, and nothing overflows).
constexpr int64_t kBytesMax = INT64_MAX & ~int64_t(255);
typedef unsigned __int128 u128;
int64_t sat_bytes(u128 b)
{
    b = (b + 255) & ~u128(255);
    return b > (u128)kBytesMax ? kBytesMax : (int64_t)b;
}
int64_t sat_add(int64_t a, int64_t b) { return a > kBytesMax - b ? kBytesMax : a + b; }
u128 n_pad_of(int64_t n) { return n > (int64_t(1) << 60) ? (u128)1 << 61 : (u128)packed_n_pad(n); }
// packed codes of either staged kernel: [k/2][n_pad] words, or the ring kernel's lagged [k/2 + 3][n_pad]
int64_t packed_bytes(int64_t n, int k) { return sat_bytes((u128)ring_code_words(k) * n_pad_of(n) * 4); }
int64_t wpk_bytes(int64_t n, int k) { return sat_bytes((u128)k * n_pad_of(n) * 4); }
int64_t spk_bytes(int64_t n, int k, int tau) { return sat_bytes((u128)k * (u128)(tau + 1) * n_pad_of(n) * 4); }
int64_t abi_codes_bytes(int64_t n, int k) { return sat_bytes((u128)n * (u128)k * 2); }
int64_t abi_weights_bytes(int64_t n, int k, int tau, Mode m)
{
    return m == kPlain ? 0 : sat_bytes((u128)n * (u128)k * (u128)(m == kProbes ? tau + 1 : 1) * 4);
}
// scratch of a stand-alone gather: the staged kernel's packed codes and table-major weights / shares
int64_t gather_ws_bytes(int64_t n, int k, int tau, Mode m)
{
    if (n <= 0 || k < 1) return 0;
    return sat_add(packed_bytes(n, k), m == kWeighted ? wpk_bytes(n, k) : m == kProbes ? spk_bytes(n, k, tau) : 0);
}
// scratch of a forward pass: the hash's ABI-layout outputs and the gather's scratch
int64_t forward_ws_bytes(int64_t n, int k, int tau, Mode m)
{
    if (n <= 0 || k < 1) return 0;
    return sat_add(sat_add(abi_codes_bytes(n, k), abi_weights_bytes(n, k, tau, m)), gather_ws_bytes(n, k, tau, m));
}

int launch_gather_lds(const LdsPlan &p, const uint32_t *packed, const float *wpk, const TableRef &T, void *y,
                      Mode mode, hipStream_t s)
{
    GatherLdsArgs a = p.a;
    a.packed = packed;
    a.wpk = wpk;
    a.tables = T.p;
    a.y = y;
    a.y_kind = T.y_kind;
    // extents the kernel assumes: rows * copy rounds cover a table exactly, the stage fits its buffer,
    // token windows of 16 x 256 tokens past any token stay inside the padded code arrays
    if ((kLdsThreads / p.sw) * p.fr != (1 << a.tau) || a.n_pad < a.n + 16 * 256 || (a.k & 1) || T.kind ||
        (mode != kPlain) != (wpk != nullptr) || !packed)
        return LFFN_E_UNSUPPORTED;
    const dim3 grid(p.grid);
    int rc = LFFN_E_UNSUPPORTED;
    TimedLaunch tl(1, s);
    if (mode == kProbes)
        rc = lffn_host::gather_lds_probes_part(p.tok, a, p.fr, p.sw, grid, p.lds, s);
    else if (mode == kWeighted)
        rc = lffn_host::gather_lds_weighted_part(p.tok, a, p.fr, p.sw, grid, p.lds, s);
    else
        rc = lffn_host::gather_lds_plain_part(p.tok, a, p.fr, p.sw, grid, p.lds, s);
    if (rc != LFFN_OK) return rc;
    LFFN_HIP(hipGetLastError());
    tl.done();
    t_last_gather = "gather_lds_kernel";
    return LFFN_OK;
}

// j_first > 0: only the tables [j_first, k) are summed, onto what y already holds (fp32 y and fp32 rows).
int launch_gather_direct(const uint16_t *codes, const float *weights, const TableRef &T, void *y, int64_t n,
                         int k, int tau, int d_out, Mode mode, hipStream_t s, const Options &opt, int j_first = 0)
{
    const int esz = T.kind ? 2 : 4;
    if (j_first < 0 || j_first >= k || (j_first && (T.kind || T.y_kind))) return LFFN_E_UNSUPPORTED;
    if ((mode != kPlain) != (weights != nullptr)) return LFFN_E_NULL;
    GatherArgs a{};
    a.codes = codes + j_first;
    a.weights = weights ? weights + (size_t)j_first * (mode == kProbes ? tau + 1 : 1) : nullptr;
    a.y = y;
    a.y_kind = T.y_kind;
    a.n = n;
    a.k = k - j_first;
    a.code_stride = k;
    a.accumulate = j_first > 0;
    a.tau = tau;
    a.d_out = d_out;
    const uint32_t row_bytes = (uint32_t)d_out * esz;
    a.nvec = (int)(row_bytes / 16);
    a.codes_vec8 = j_first == 0 && (k % 8 == 0) && aligned(codes, 16) && (!weights || aligned(weights, 16));

    int lpt = opt.lanes_per_token;
    if (lpt == 0) {
        lpt = 8;  // 128-byte slices: one L2 line per (token, table)
        while (lpt > 1 && lpt / 2 >= a.nvec) lpt /= 2;
    }
    if (T.prepared && lpt * 16 > T.pw) lpt = T.pw / 16;  // a token's piece lies inside one prepared piece
    const int tpw = 64 / lpt;
    a.n_slices = (a.nvec + lpt - 1) / lpt;
    if (T.prepared) {
        a.spp = (uint32_t)(T.pw / (lpt * 16));
        a.row_stride = (uint32_t)T.pw;
        a.slice_stride = ((unsigned long long)k << tau) * T.pw;
    } else {
        a.spp = 1;
        a.row_stride = row_bytes;
        a.slice_stride = (unsigned long long)lpt * 16;
    }
    a.tables = T.p + ((size_t)j_first << tau) * a.row_stride;  // row (j << tau) + code of either layout
    const int64_t ntb = (n + (int64_t)kGatherWaves * tpw - 1) / ((int64_t)kGatherWaves * tpw);
    if (ntb > (int64_t(1) << 30)) return LFFN_E_SIZE;
    a.ntb = (int)ntb;

    const double table_bytes = (double)k * (double)(1u << tau) * row_bytes;
    bool xcd = table_bytes > 4.0 * 1024 * 1024 && ntb >= 64;
    if (opt.xcd_order == 1) xcd = true;
    if (opt.xcd_order == -1) xcd = false;
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
    int rc = lffn_host::gather_direct_part(T.kind, lpt, a, mode == kProbes, grid, s);
    if (rc != LFFN_OK) return rc;
    LFFN_HIP(hipGetLastError());
    tl.done();
    t_last_gather = "gather_kernel";
    return LFFN_OK;
}

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

// ABI weights [n][m] -> table-major [m][n_pad]  (m = k, or k * (1 + tau) for the multi-probe shares)
int launch_repack_weights(const float *weights, float *wpk, int64_t n, int64_t n_pad, int64_t m, hipStream_t s)
{
    hipLaunchKernelGGL(repack_shares_kernel, dim3(repack_grid(n, m)), dim3(256), 0, s, weights, wpk, (long long)n,
                       (long long)n_pad, (long long)m);
    LFFN_HIP(hipGetLastError());
    return LFFN_OK;
}

// Launch shape of the lagged, bank-interleaved staged gather (gather_ring_kernel): prepared tables of up
// to 256 rows, plain sum.
struct RingPlan {
    bool use = false;
    GatherRingArgs a{};
    int threads = 0, tok = 0;
    unsigned grid = 0;
};

int plan_gather_ring(int64_t n, int k, int tau, int d_out, const TableRef &T, Mode mode, const Options &opt,
                     RingPlan *p)
{
    p->use = false;
    // On request only (gather_path 4).  Measured on the RoBERTa-base shape it does not beat the double-buffered
    // staged kernel: its reads are conflict-free, but both kernels are bound by the four vector adds per 16 bytes
    // read, and this one pays a barrier and an LDS write per table.
    if (opt.gather_path != 4 || mode != kPlain || !T.prepared || T.pw < 64) return LFFN_OK;
    if (tau < 7 || tau > 8 || k > 480) return LFFN_OK;   // 256-row slices; the re-pack kernel's 64 x k tile fits LDS
    if (n >= (int64_t(1) << 31) - 4096) return LFFN_OK;
    int cus = 0;
    int rc = device_cus(&cus);
    if (rc != LFFN_OK) return rc;
    if (cus < kXcds || cus % kXcds != 0) return LFFN_OK;
    const int rows = 1 << tau;
    GatherRingArgs &a = p->a;
    a = GatherRingArgs{};
    a.n = n;
    a.n_pad = packed_n_pad(n);
    a.k = k;
    a.tau = tau;
    a.d_out = d_out;
    a.nvec = d_out / 4;
    a.n_slices = (a.nvec + 3) / 4;
    a.token_splits = kXcds / gcd(a.n_slices, kXcds);
    a.n_units = a.n_slices * a.token_splits;
    a.blocks_per_xcd = cus / kXcds;
    a.row_stride = (uint32_t)T.pw;
    a.spp = (uint32_t)(T.pw / 64);
    a.table_stride = (uint32_t)(rows * T.pw);
    a.slice_stride = (unsigned long long)k * rows * T.pw;
    // tokens of the fullest workgroup, as the kernel splits them (in units of 16 tokens)
    const int64_t tpb = 16 * lds_tokens_per_block((n + 15) / 16, a.n_units, a.token_splits, a.blocks_per_xcd);
    // workgroup shapes that are built: (threads, token slots), a chunk holds threads / 4 * slots tokens
    static const int shapes[][2] = {{1024, 4}, {1024, 8}, {1024, 12}, {1024, 13}, {1024, 14}, {512, 8}, {512, 16}, {512, 20}, {512, 24}, {512, 28}, {512, 32}};
    int64_t cap_max = 0;
    for (auto &sh : shapes) {
        if (opt.ring_threads && sh[0] != opt.ring_threads) continue;
        if (opt.token_slots && sh[1] > opt.token_slots) continue;
        const int64_t cap = (int64_t)sh[0] / 4 * sh[1];
        if (cap > cap_max) cap_max = cap;
    }
    if (cap_max == 0) return LFFN_OK;
    const int64_t nchunks = (tpb + cap_max - 1) / cap_max;
    const int64_t chunk = ((tpb / 16 + nchunks - 1) / nchunks) * 16;  // tokens of the longest chunk
    // the shape with the fewest slots that holds a chunk; 1024 threads first (more waves to hide latency)
    int best = -1;
    for (int i = 0; i < (int)(sizeof(shapes) / sizeof(shapes[0])); ++i) {
        if (opt.ring_threads && shapes[i][0] != opt.ring_threads) continue;
        if (opt.token_slots && shapes[i][1] > opt.token_slots) continue;
        const int64_t cap = (int64_t)shapes[i][0] / 4 * shapes[i][1];
        if (cap < chunk) continue;
        if (best < 0 || cap < (int64_t)shapes[best][0] / 4 * shapes[best][1]) best = i;
    }
    if (best < 0) return LFFN_OK;
    p->threads = shapes[best][0];
    p->tok = shapes[best][1];
    p->grid = (unsigned)cus;
    p->use = true;
    return LFFN_OK;
}

int launch_gather_ring(const RingPlan &p, const uint16_t *codes, uint32_t *packed, const TableRef &T, void *y,
                       hipStream_t s)
{
    GatherRingArgs a = p.a;
    if (!packed || !T.prepared || a.n_pad < a.n + 16 * 256) return LFFN_E_UNSUPPORTED;
    // codes in the ABI layout -> lagged packed layout (scaled by the 256-byte LDS row stride)
    int64_t blocks = (a.n_pad + 63) / 64;
    if (blocks > 8192) blocks = 8192;
    const size_t tile = (size_t)64 * (a.k | 1) * sizeof(uint16_t);
    TimedLaunch tl(1, s);
    hipLaunchKernelGGL(repack_codes_lag_kernel, dim3((unsigned)blocks), dim3(256), tile, s, codes, packed,
                       (long long)a.n, (long long)a.n_pad, a.k, a.tau, kRingShift);
    LFFN_HIP(hipGetLastError());
    a.packed = packed;
    a.tables = T.p;
    a.y = y;
    a.y_kind = T.y_kind;
    int rc = lffn_host::gather_ring_part(p.threads, p.tok, a, dim3(p.grid), s);
    if (rc != LFFN_OK) return rc;
    LFFN_HIP(hipGetLastError());
    tl.done();
    t_last_gather = "gather_ring_kernel";
    return LFFN_OK;
}

// Gather from ABI-layout codes (and weights / shares): the staged kernel through the re-pack kernels when
// the plan says so and the scratch has room, else the direct kernel.
int gather_from_abi(Mode mode, const uint16_t *codes, const float *weights, const TableRef &T, void *y, int64_t n,
                    int k, int tau, int d_out, const LdsPlan &plan, Scratch *sc, hipStream_t s, const Options &opt)
{
    RingPlan ring;
    int rrc = plan_gather_ring(n, k, tau, d_out, T, mode, opt, &ring);
    if (rrc != LFFN_OK) return rrc;
    if (ring.use) {
        uint32_t *packed = sc->take<uint32_t>(packed_bytes(n, k));
        if (packed) return launch_gather_ring(ring, codes, packed, T, y, s);
    }
    if (plan.use && aligned(codes, 4)) {
        uint32_t *packed = sc->take<uint32_t>(packed_bytes(n, k));
        float *wpk = mode == kWeighted ? sc->take<float>(wpk_bytes(n, k))
                     : mode == kProbes ? sc->take<float>(spk_bytes(n, k, tau)) : nullptr;
        if (packed && (mode == kPlain || wpk)) {
            int rc = launch_repack_codes(codes, packed, n, plan.a.n_pad, k, tau, plan.shift, s);
            if (rc != LFFN_OK) return rc;
            if (mode != kPlain) {
                rc = launch_repack_weights(weights, wpk, n, plan.a.n_pad, (int64_t)k * (mode == kProbes ? tau + 1 : 1), s);
                if (rc != LFFN_OK) return rc;
            }
            rc = launch_gather_lds(plan, packed, wpk, T, y, mode, s);
            if (rc != LFFN_OK || !plan.tail) return rc;
            rc = launch_gather_direct(codes, weights, T, y, n, k, tau, d_out, mode, s, opt, k - plan.tail);
            t_last_gather = "gather_lds_kernel";  // the one that did all tables but the last
            return rc;
        }
    }
    return launch_gather_direct(codes, weights, T, y, n, k, tau, d_out, mode, s, opt);
}

// ---- BH{m} hash --------------------------------------------------------------------------------
int check_bh(const void *x, const float *bmats, int64_t n, int d, int k, int tau, int block, int n_factors,
             int x_dtype, bool weighted = false)
{
    if (!x || !bmats) return LFFN_E_NULL;
    if (n < 0 || d < 1 || k < 1 || n_factors < 1) return LFFN_E_SIZE;
    if (tau < 1 || tau > 16) return LFFN_E_TAU;
    if (!dtype_ok(x_dtype)) return LFFN_E_DTYPE;
    if (k > (1 << 20) || n > (int64_t(1) << 40) || n_factors > 64) return LFFN_E_SIZE;
    const int L = log2_pad(d);
    if (L > 10 || d > 1024) return LFFN_E_UNSUPPORTED;
    const int N = L < 6 ? 64 : 1 << L;  // widths below 64 are not built
    if (L < 6) return LFFN_E_UNSUPPORTED;
    const int b = block & ~LFFN_PREPARED;
    if (b != 16 && b != 32 && b != 64) return LFFN_E_UNSUPPORTED;
    if (b > N) return LFFN_E_SIZE;
    const int64_t P = ((int64_t)k * tau + N - 1) / N;
    if (P > 64 || bh_lds_bytes((int)P, N, weighted && !(tau == 4 || tau == 8 || tau == 16)) > 150 * 1024) return LFFN_E_UNSUPPORTED;
    if (!aligned(x, x_dtype == LFFN_F32 ? 4 : 2) || !aligned(bmats, (block & LFFN_PREPARED) ? 256 : 4)) return LFFN_E_ALIGN;
    return LFFN_OK;
}

// The BH kernel reduces a table's weight inside one 16-coordinate tile of z (tau = 4, 8, 16: the weighted
// instantiations).  For any other tau the plain instantiation forms the weights from z through a window in LDS.
bool bh_weights_in_kernel(int tau) { return tau == 4 || tau == 8 || tau == 16; }

int64_t bh_pack_bytes(int d, int k, int tau, int block, int n_factors)
{
    const int N = 1 << log2_pad(d);
    const int64_t P = ((int64_t)k * tau + N - 1) / N;
    return round256(P * n_factors * (int64_t)N * block * 4);
}

// The factors in MFMA-operand order (one-time: lookupffn_prepare_bh, or per call into scratch)
int launch_bh_pack(const float *bmats, float *apack, int d, int k, int tau, int block, int n_factors, hipStream_t s)
{
    const int N = 1 << log2_pad(d);
    const int64_t P = ((int64_t)k * tau + N - 1) / N;
    const long long total = (long long)P * n_factors * N * block;
    long long pb = (total + 255) / 256;
    if (pb > 2048) pb = 2048;
    hipLaunchKernelGGL(bh_pack_kernel, dim3((unsigned)pb), dim3(256), 0, s, bmats, apack, N, block, total);
    LFFN_HIP(hipGetLastError());
    return LFFN_OK;
}

// Hashes with the packed factors `apack`; `pack_from` != NULL: re-order them from there first.
int launch_hash_bh(const void *x, const float *pack_from, const float *apack_in, float *apack_scratch,
                   const HashOut &out, int64_t n, int d, int k, int tau, int block, int n_factors, int x_dtype,
                   hipStream_t s)
{
    const int L = log2_pad(d);
    const int N = 1 << L;
    BhArgs a{};
    a.x = x;
    a.apack = pack_from ? apack_scratch : apack_in;
    a.codes = out.codes;
    a.packed = out.codes ? nullptr : out.packed;
    a.weights = out.codes ? out.weights : nullptr;
    a.wpk = out.codes ? nullptr : out.weights;
    a.n_pad = packed_n_pad(n);
    a.packed_shift = out.shift;
    a.n = n;
    a.d = d;
    a.k = k;
    a.tau = tau;
    a.n_factors = n_factors;
    a.P = (int)(((int64_t)k * tau + N - 1) / N);
    a.x_kind = x_dtype;  // LFFN_F32 / BF16 / F16 are the kernels' kinds 0 / 1 / 2
    a.x_vec4 = d % 4 == 0 && aligned(x, a.x_kind ? 8 : 16);
    a.scale = (float)(1.0 / std::sqrt((double)N));
    if (!a.apack || (!a.codes && !a.packed) || out.probes) return LFFN_E_NULL;
    a.window = out.weights && !bh_weights_in_kernel(tau);  // weights through the z window of the plain kernels
    TimedLaunch tl(0, s);
    if (pack_from) {
        int rc = launch_bh_pack(pack_from, apack_scratch, d, k, tau, block, n_factors, s);
        if (rc != LFFN_OK) return rc;
    }
    int64_t blocks = ((n + kBhTok - 1) / kBhTok + kBhWaves - 1) / kBhWaves;
    if (blocks > 4096) blocks = 4096;
    const dim3 grid((unsigned)blocks);
    const size_t lds = bh_lds_bytes(a.P, N, a.window != 0);
    const bool weighted = (a.weights || a.wpk) && !a.window;  // the instantiations that reduce weights in registers
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

// ---------------------------------------------------------------- the forward pass, all variants
// ---------------------------------------------------------------- the one-launch path for a few tokens
// Whether forward_stack_kernel takes this shape (checked without a HIP call).
bool stack_shape_ok(const void *x, const int8_t *const *signs, const void *const *tables, int n_layers, int64_t n,
                    int d, int k, int tau, int d_out, int n_rounds, int x_dtype, int table_dtype)
{
    if (log2_pad(d) != 10 || n_rounds > 4 || n_layers < 1 || n_layers > kStackMaxLayers) return false;
    if (n_layers > 1 && d_out != d) return false;
    if (n > 0x7FFFFFFF) return false;
    const bool xb = x_dtype != LFFN_F32;
    const size_t xrow = (size_t)d * (xb ? 2 : 4);
    if (d % 4 == 0 && !(aligned(x, 16) && xrow % (xb ? 8 : 16) == 0)) return false;
    for (int l = 0; l < n_layers; ++l)
        if (!aligned(signs[l], 16)) return false;
    const int P = (int)(((int64_t)k * tau + 1023) / 1024);
    if (stack_lds_bytes(P, k) > 64 * 1024) return false;
    const TableRef T = table_ref(tables[0], table_dtype, tau);
    const int64_t bytes = T.prepared ? prepared_tables_bytes(k, tau, d_out)
                                     : ((int64_t)k << tau) * d_out * (T.kind ? 2 : 4);
    return bytes < (int64_t(1) << 31);
}

// Call only with stack_shape_ok(...) true and every argument validated.
int launch_forward_stack(const void *x, const int8_t *const *signs, const void *const *tables, void *y, int64_t n,
                         int d, int k, int tau, int d_out, int n_rounds, int n_layers, int x_dtype, int table_dtype,
                         hipStream_t s)
{
    const TableRef T = table_ref(tables[0], table_dtype, tau);
    StackArgs a{};
    a.x = x;
    a.y = y;
    a.y_kind = T.y_kind;
    for (int l = 0; l < n_layers; ++l) {
        a.signs[l] = signs[l];
        a.tables[l] = static_cast<const char *>(tables[l]);
    }
    a.n = n;
    a.d = d;
    a.d_out = d_out;
    a.k = k;
    a.tau = tau;
    a.P = (int)(((int64_t)k * tau + 1023) / 1024);
    a.n_layers = n_layers;
    a.x_kind = x_dtype;  // LFFN_F32 / BF16 / F16 are the kernels' kinds 0 / 1 / 2
    a.scale = (float)(1.0 / std::sqrt(1024.0));
    const int64_t rows = int64_t(1) << tau;
    if (T.prepared) {
        a.row_dwords = (uint32_t)d_out;
        a.piece_shift = T.pw == 128 ? 7 : 6;
        a.row_stride = (uint32_t)T.pw;
        a.slice_stride = (uint32_t)((int64_t)k * rows * T.pw);
        a.table_bytes = (uint32_t)prepared_tables_bytes(k, tau, d_out);
    } else {
        const int64_t row_bytes = (int64_t)d_out * (T.kind ? 2 : 4);
        a.row_dwords = (uint32_t)(row_bytes / 4);
        a.piece_shift = 31;
        a.row_stride = (uint32_t)row_bytes;
        a.slice_stride = 0;
        a.table_bytes = (uint32_t)((int64_t)k * rows * row_bytes);
    }
    int threads = (int)((a.row_dwords + 63) / 64 * 64);
    if (threads > 1024) threads = 1024;
    TimedLaunch tl(1, s);
    int rc = lffn_host::forward_stack_part(n_rounds, T.kind, a, dim3((unsigned)n), threads, stack_lds_bytes(a.P, k), s);
    if (rc != LFFN_OK) return rc;
    LFFN_HIP(hipGetLastError());
    tl.done();
    t_last_gather = "forward_stack_kernel";
    t_last_hash = "forward_stack_kernel";
    return LFFN_OK;
}

// Hash: the sign-diagonal rounds (`signs`, n_rounds) or the BH factors (`bmats`, block, n_factors).
struct HashSpec {
    const int8_t *signs = nullptr;
    int n_rounds = 0;
    const float *bmats = nullptr;  // row-major factors, or the prepared copy when `bh_prepared`
    int block = 0, n_factors = 0;
    bool bh_prepared = false;
    bool bh() const { return bmats != nullptr; }
};

int64_t forward_need(const HashSpec &h, Mode mode, int64_t n, int d, int k, int tau)
{
    if (n <= 0) return 0;
    const int64_t pack = (h.bh() && !h.bh_prepared) ? bh_pack_bytes(d, k, tau, h.block, h.n_factors) : 0;
    return sat_add(pack, forward_ws_bytes(n, k, tau, mode));
}

int forward_core(const HashSpec &h, Mode mode, const void *x, const void *tables, void *y, int64_t n, int d,
                 int k, int tau, int d_out, int x_dtype, int table_dtype, void *workspace,
                 int64_t workspace_bytes, hipStream_t s)
{
    const uint16_t *stand_in = reinterpret_cast<const uint16_t *>(uintptr_t(256));  // the codes live in scratch
    int rc = h.bh() ? check_bh(x, h.bmats, n, d, k, tau, h.block | (h.bh_prepared ? LFFN_PREPARED : 0), h.n_factors,
                               x_dtype, mode == kWeighted)
                    : check_hash(x, h.signs, stand_in, n, d, k, tau, h.n_rounds, x_dtype, mode != kPlain);
    if (rc != LFFN_OK) return rc;
    if (h.bh() && mode == kProbes) return LFFN_E_UNSUPPORTED;
    rc = check_gather(stand_in, tables, y, n, k, tau, d_out, table_dtype);
    if (rc != LFFN_OK) return rc;
    const int64_t need = forward_need(h, mode, n, d, k, tau);
    Scratch sc;
    if (workspace) {  // a caller's buffer is checked even for an empty batch
        if (workspace_bytes < need) return LFFN_E_WORKSPACE;
        if (!aligned(workspace, 256)) return LFFN_E_ALIGN;
    }
    if (n == 0) return LFFN_OK;
    const Options opt = options_snapshot();
    if (!h.bh() && mode == kPlain && opt.gather_path == 0 && opt.hash_path == 0 && opt.small_tokens >= 0 &&
        n <= (opt.small_tokens ? opt.small_tokens : kSmallTokensDefault) &&
        stack_shape_ok(x, &h.signs, &tables, 1, n, d, k, tau, d_out, h.n_rounds, x_dtype, table_dtype))
        return launch_forward_stack(x, &h.signs, &tables, y, n, d, k, tau, d_out, h.n_rounds, 1, x_dtype, table_dtype, s);
    rc = get_scratch(workspace, workspace_bytes, need, &sc);
    if (rc != LFFN_OK) return rc;
    const TableRef T = table_ref(tables, table_dtype, tau);
    LdsPlan plan;
    rc = plan_gather_lds(n, k, tau, d_out, T, mode, opt, &plan);
    if (rc != LFFN_OK) return rc;
    float *apack = (h.bh() && !h.bh_prepared) ? sc.take<float>(bh_pack_bytes(d, k, tau, h.block, h.n_factors)) : nullptr;
    if (h.bh() && !h.bh_prepared && !apack) return LFFN_E_WORKSPACE;
    auto run_hash = [&](const HashOut &out) -> int {
        if (h.bh())
            return launch_hash_bh(x, h.bh_prepared ? nullptr : h.bmats, h.bh_prepared ? h.bmats : nullptr, apack, out, n,
                                  d, k, tau, h.block, h.n_factors, x_dtype, s);
        return launch_hash(x, h.signs, out, n, d, k, tau, h.n_rounds, x_dtype, s, opt);
    };
    // the hash kernels write the staged gather's layout themselves, scaled for its row pieces (unless the
    // variant is the multi-probe one, whose shares exist in the ABI layout only)
    RingPlan ring;
    rc = plan_gather_ring(n, k, tau, d_out, T, mode, opt, &ring);
    if (rc != LFFN_OK) return rc;
    if (!ring.use && plan.use && !plan.tail && mode != kProbes) {
        HashOut out;
        out.shift = plan.shift;
        const int64_t pb = packed_bytes(n, k), wb = mode == kWeighted ? wpk_bytes(n, k) : 0;
        out.packed = sc.take<uint32_t>(pb);
        out.weights = mode == kWeighted ? sc.take<float>(wb) : nullptr;
        if (!out.packed || (mode == kWeighted && !out.weights)) return LFFN_E_WORKSPACE;
        if (!hash_extents_ok(out, n, k, tau, plan.a.n_pad, 0, pb, wb)) return LFFN_E_WORKSPACE;
        rc = run_hash(out);
        if (rc != LFFN_OK) return rc;
        return launch_gather_lds(plan, out.packed, out.weights, T, y, mode, s);
    }
    HashOut out;
    const int64_t cb = abi_codes_bytes(n, k), wb = abi_weights_bytes(n, k, tau, mode);
    out.codes = sc.take<uint16_t>(cb);
    out.weights = mode != kPlain ? sc.take<float>(wb) : nullptr;
    out.probes = mode == kProbes;
    if (!out.codes || (mode != kPlain && !out.weights)) return LFFN_E_WORKSPACE;
    if (!hash_extents_ok(out, n, k, tau, plan.a.n_pad, cb, 0, wb)) return LFFN_E_WORKSPACE;
    rc = run_hash(out);
    if (rc != LFFN_OK) return rc;
    return gather_from_abi(mode, out.codes, out.weights, T, y, n, k, tau, d_out, plan, &sc, s, opt);
}

int gather_core(Mode mode, const uint16_t *codes, const float *weights, const void *tables, void *y, int64_t n,
                int k, int tau, int d_out, int table_dtype, void *workspace, int64_t workspace_bytes, hipStream_t s)
{
    int rc = check_gather(codes, tables, y, n, k, tau, d_out, table_dtype);
    if (rc == LFFN_OK && mode != kPlain) rc = check_weights(weights);
    if (rc != LFFN_OK) return rc;
    const int64_t need = gather_ws_bytes(n, k, tau, mode);
    if (workspace) {
        if (workspace_bytes < need) return LFFN_E_WORKSPACE;
        if (!aligned(workspace, 256)) return LFFN_E_ALIGN;
    }
    if (n == 0) return LFFN_OK;
    const Options opt = options_snapshot();
    const TableRef T = table_ref(tables, table_dtype, tau);
    LdsPlan plan;
    rc = plan_gather_lds(n, k, tau, d_out, T, mode, opt, &plan);
    if (rc != LFFN_OK) return rc;
    RingPlan ring;
    rc = plan_gather_ring(n, k, tau, d_out, T, mode, opt, &ring);
    if (rc != LFFN_OK) return rc;
    Scratch sc;
    if (ring.use || (plan.use && aligned(codes, 4))) {  // only the staged kernels need scratch
        rc = get_scratch(workspace, workspace_bytes, need, &sc);
        if (rc != LFFN_OK) return rc;
    }
    return gather_from_abi(mode, codes, weights, T, y, n, k, tau, d_out, plan, &sc, s, opt);
}

HashSpec sign_hash(const int8_t *signs, int n_rounds)
{
    HashSpec h;
    h.signs = signs;
    h.n_rounds = n_rounds;
    return h;
}
HashSpec bh_hash(const float *bmats, int block, int n_factors)
{
    HashSpec h;
    h.bmats = bmats;
    h.block = block & ~LFFN_PREPARED;
    h.n_factors = n_factors;
    h.bh_prepared = (block & LFFN_PREPARED) != 0;
    return h;
}

// stand-alone BH hash (codes, and weights for the weighted variant) into caller buffers
int hash_bh_core(const void *x, const float *bmats, uint16_t *codes, float *weights, bool weighted, int64_t n, int d,
                 int k, int tau, int block, int n_factors, int x_dtype, void *workspace, int64_t workspace_bytes,
                 hipStream_t s)
{
    int rc = check_bh(x, bmats, n, d, k, tau, block, n_factors, x_dtype, weighted);
    if (rc != LFFN_OK) return rc;
    if (!codes || (weighted && !weights)) return LFFN_E_NULL;
    if (!aligned(codes, 2) || (weighted && !aligned(weights, 4))) return LFFN_E_ALIGN;
    const HashSpec h = bh_hash(bmats, block, n_factors);
    const int64_t pb = h.bh_prepared ? 0 : bh_pack_bytes(d, k, tau, h.block, n_factors);
    const int64_t need = pb;
    if (workspace) {
        if (workspace_bytes < need) return LFFN_E_WORKSPACE;
        if (!aligned(workspace, 256)) return LFFN_E_ALIGN;
    }
    if (n == 0) return LFFN_OK;
    Scratch sc;
    rc = get_scratch(workspace, workspace_bytes, need, &sc);
    if (rc != LFFN_OK) return rc;
    float *apack = h.bh_prepared ? nullptr : sc.take<float>(pb);
    if (!h.bh_prepared && !apack) return LFFN_E_WORKSPACE;
    HashOut out;
    out.codes = codes;
    out.weights = weighted ? weights : nullptr;
    return launch_hash_bh(x, h.bh_prepared ? nullptr : bmats, h.bh_prepared ? bmats : nullptr, apack, out, n, d, k,
                          tau, h.block, n_factors, x_dtype, s);
}

bool bh_shape_ok(int d, int k, int tau, int block, int n_factors)
{
    return !(d < 1 || d > 1024 || k < 1 || tau < 1 || tau > 16 || block < 1 || n_factors < 1 || n_factors > 64);
}

}  // namespace

extern "C" {

int lookupffn_init(void)
{
    int cus = 0;
    int rc = device_cus(&cus);
    if (rc != LFFN_OK) return rc;
    {
        void *p = nullptr;  // the static scratch array's address on this device
        rc = static_scratch(&p);
        if (rc != LFFN_OK) return rc;
    }
    // code objects are loaded on first use: do that now for the two parts no attribute call below touches
    // (this one: hash, re-pack and prepare kernels; and the direct gather's)
    {
        hipFuncAttributes attr;
        LFFN_HIP(hipFuncGetAttributes(&attr, reinterpret_cast<const void *>(repack_codes_kernel)));
        rc = lffn_host::gather_direct_load();
        if (rc != LFFN_OK) return rc;
    }
    // every kernel that asks for more than 64 KB of dynamic LDS is told so now, so that no later launch
    // has to (the attribute call is not a stream operation and has no place inside a graph capture)
    lffn_host::AttrOnly scope;
    const size_t lds = 160 * 1024;
    GatherLdsArgs ga{};
    BhArgs ba{};
    for (int tok : {4, 8, 12, 13, 16})
        for (int fr : {1, 2, 4})
            for (int sw : {4, 8}) {
                for (int part = 0; part < 3; ++part) {
                    rc = part == 0   ? lffn_host::gather_lds_plain_part(tok, ga, fr, sw, dim3(1), lds, nullptr)
                         : part == 1 ? lffn_host::gather_lds_weighted_part(tok, ga, fr, sw, dim3(1), lds, nullptr)
                                     : lffn_host::gather_lds_probes_part(tok, ga, fr, sw, dim3(1), lds, nullptr);
                    if (rc != LFFN_OK && rc != LFFN_E_UNSUPPORTED) return rc;
                }
            }
    rc = lffn_host::hash_row16_load();
    if (rc != LFFN_OK) return rc;
    rc = lffn_host::hash_row8_load();
    if (rc != LFFN_OK) return rc;
    rc = lffn_host::forward_stack_load();
    if (rc != LFFN_OK) return rc;
    {
        GatherRingArgs ra{};
        for (int threads : {512, 1024})
            for (int tok = 1; tok <= 32; ++tok) {
                rc = lffn_host::gather_ring_part(threads, tok, ra, dim3(1), nullptr);
                if (rc != LFFN_OK && rc != LFFN_E_UNSUPPORTED) return rc;
            }
    }
    for (int L = 6; L <= 10; ++L)
        for (int block : {16, 32, 64})
            for (int vec4 = 0; vec4 < 2; ++vec4)
                for (int weighted = 0; weighted < 2; ++weighted) {
                    ba.x_vec4 = vec4;
                    if (L <= 8)
                        rc = weighted ? lffn_host::bh_weighted_lo_part(L, ba, block, dim3(1), lds, nullptr)
                                      : lffn_host::bh_plain_lo_part(L, ba, block, dim3(1), lds, nullptr);
                    else if (!weighted)
                        rc = L == 9 ? lffn_host::bh_plain_512_part(ba, block, dim3(1), lds, nullptr)
                                    : lffn_host::bh_plain_1024_part(ba, block, dim3(1), lds, nullptr);
                    else if (L == 9)
                        rc = vec4 ? lffn_host::bh_weighted_512_vec4_part(ba, block, dim3(1), lds, nullptr)
                                  : lffn_host::bh_weighted_512_scalar_part(ba, block, dim3(1), lds, nullptr);
                    else
                        rc = vec4 ? lffn_host::bh_weighted_1024_vec4_part(ba, block, dim3(1), lds, nullptr)
                                  : lffn_host::bh_weighted_1024_scalar_part(ba, block, dim3(1), lds, nullptr);
                    if (rc != LFFN_OK && rc != LFFN_E_UNSUPPORTED) return rc;
                }
    return LFFN_OK;
}

int lookupffn_hash(const void *x, const int8_t *signs, uint16_t *codes, int64_t n_tokens, int d, int k,
                   int tau, int n_rounds, int x_dtype, void *hip_stream)
{
    int rc = check_hash(x, signs, codes, n_tokens, d, k, tau, n_rounds, x_dtype);
    if (rc != LFFN_OK || n_tokens == 0) return rc;
    HashOut out;
    out.codes = codes;
    return launch_hash(x, signs, out, n_tokens, d, k, tau, n_rounds, x_dtype, static_cast<hipStream_t>(hip_stream),
                       options_snapshot());
}

int lookupffn_hash_weighted(const void *x, const int8_t *signs, uint16_t *codes, float *weights, int64_t n_tokens,
                            int d, int k, int tau, int n_rounds, int x_dtype, void *hip_stream)
{
    int rc = check_hash(x, signs, codes, n_tokens, d, k, tau, n_rounds, x_dtype, true);
    if (rc == LFFN_OK) rc = check_weights(weights);
    if (rc != LFFN_OK || n_tokens == 0) return rc;
    HashOut out;
    out.codes = codes;
    out.weights = weights;
    return launch_hash(x, signs, out, n_tokens, d, k, tau, n_rounds, x_dtype, static_cast<hipStream_t>(hip_stream),
                       options_snapshot());
}

int lookupffn_hash_probes(const void *x, const int8_t *signs, uint16_t *codes, float *shares, int64_t n_tokens,
                          int d, int k, int tau, int n_rounds, int x_dtype, void *hip_stream)
{
    int rc = check_hash(x, signs, codes, n_tokens, d, k, tau, n_rounds, x_dtype, true);
    if (rc == LFFN_OK) rc = check_weights(shares);
    if (rc != LFFN_OK || n_tokens == 0) return rc;
    HashOut out;
    out.codes = codes;
    out.weights = shares;
    out.probes = true;
    return launch_hash(x, signs, out, n_tokens, d, k, tau, n_rounds, x_dtype, static_cast<hipStream_t>(hip_stream),
                       options_snapshot());
}

int lookupffn_gather(const uint16_t *codes, const void *tables, void *y, int64_t n_tokens, int k, int tau,
                     int d_out, int table_dtype, void *workspace, int64_t workspace_bytes, void *hip_stream)
{
    return gather_core(kPlain, codes, nullptr, tables, y, n_tokens, k, tau, d_out, table_dtype, workspace,
                       workspace_bytes, static_cast<hipStream_t>(hip_stream));
}

int lookupffn_gather_weighted(const uint16_t *codes, const float *weights, const void *tables, void *y,
                              int64_t n_tokens, int k, int tau, int d_out, int table_dtype, void *workspace,
                              int64_t workspace_bytes, void *hip_stream)
{
    return gather_core(kWeighted, codes, weights, tables, y, n_tokens, k, tau, d_out, table_dtype, workspace,
                       workspace_bytes, static_cast<hipStream_t>(hip_stream));
}

int lookupffn_gather_probes(const uint16_t *codes, const float *shares, const void *tables, void *y,
                            int64_t n_tokens, int k, int tau, int d_out, int table_dtype, void *workspace,
                            int64_t workspace_bytes, void *hip_stream)
{
    return gather_core(kProbes, codes, shares, tables, y, n_tokens, k, tau, d_out, table_dtype, workspace,
                       workspace_bytes, static_cast<hipStream_t>(hip_stream));
}

int64_t lookupffn_workspace_bytes_gather(int64_t n_tokens, int k)
{
    return (n_tokens <= 0 || k < 1) ? 0 : gather_ws_bytes(n_tokens, k, 1, kPlain);
}
int64_t lookupffn_workspace_bytes_gather_weighted(int64_t n_tokens, int k)
{
    return (n_tokens <= 0 || k < 1) ? 0 : gather_ws_bytes(n_tokens, k, 1, kWeighted);
}
int64_t lookupffn_workspace_bytes_gather_probes(int64_t n_tokens, int k, int tau)
{
    return (n_tokens <= 0 || k < 1 || tau < 1 || tau > 16) ? 0 : gather_ws_bytes(n_tokens, k, tau, kProbes);
}

int64_t lookupffn_workspace_bytes(int64_t n_tokens, int k)
{
    return (n_tokens <= 0 || k < 1) ? 0 : forward_ws_bytes(n_tokens, k, 1, kPlain);
}
int64_t lookupffn_workspace_bytes_weighted(int64_t n_tokens, int k)
{
    return (n_tokens <= 0 || k < 1) ? 0 : forward_ws_bytes(n_tokens, k, 1, kWeighted);
}
int64_t lookupffn_workspace_bytes_probes(int64_t n_tokens, int k, int tau)
{
    return (n_tokens <= 0 || k < 1 || tau < 1 || tau > 16) ? 0 : forward_ws_bytes(n_tokens, k, tau, kProbes);
}
int64_t lookupffn_workspace_bytes_bh(int64_t n_tokens, int d, int k, int tau, int block, int n_factors)
{
    if (!bh_shape_ok(d, k, tau, block & ~LFFN_PREPARED, n_factors)) return 0;
    const int64_t pack = (block & LFFN_PREPARED) ? 0 : bh_pack_bytes(d, k, tau, block, n_factors);
    return sat_add(pack, n_tokens > 0 ? forward_ws_bytes(n_tokens, k, tau, kPlain) : 0);
}
int64_t lookupffn_workspace_bytes_bh_weighted(int64_t n_tokens, int d, int k, int tau, int block, int n_factors)
{
    if (!bh_shape_ok(d, k, tau, block & ~LFFN_PREPARED, n_factors)) return 0;
    const int64_t pack = (block & LFFN_PREPARED) ? 0 : bh_pack_bytes(d, k, tau, block, n_factors);
    return sat_add(pack, n_tokens > 0 ? forward_ws_bytes(n_tokens, k, tau, kWeighted) : 0);
}

int lookupffn_forward(const void *x, const int8_t *signs, const void *tables, void *y, int64_t n_tokens,
                      int d, int k, int tau, int d_out, int n_rounds, int x_dtype, int table_dtype,
                      void *workspace, int64_t workspace_bytes, void *hip_stream)
{
    return forward_core(sign_hash(signs, n_rounds), kPlain, x, tables, y, n_tokens, d, k, tau, d_out, x_dtype,
                        table_dtype, workspace, workspace_bytes, static_cast<hipStream_t>(hip_stream));
}

int lookupffn_forward_stack(const void *x, const int8_t *const *signs, const void *const *tables, void *y,
                            int64_t n_tokens, int d, int k, int tau, int d_out, int n_rounds, int n_layers,
                            int x_dtype, int table_dtype, void *hip_stream)
{
    if (!signs || !tables) return LFFN_E_NULL;
    if (n_layers < 1 || n_layers > kStackMaxLayers) return LFFN_E_SIZE;
    const uint16_t *stand_in = reinterpret_cast<const uint16_t *>(uintptr_t(256));  // no codes leave the kernel
    for (int l = 0; l < n_layers; ++l) {
        int rc = check_hash(x, signs[l], stand_in, n_tokens, d, k, tau, n_rounds, x_dtype);
        if (rc == LFFN_OK) rc = check_gather(stand_in, tables[l], y, n_tokens, k, tau, d_out, table_dtype);
        if (rc != LFFN_OK) return rc;
    }
    if (n_layers > 1 && d_out != d) return LFFN_E_SIZE;
    if (!stack_shape_ok(x, signs, tables, n_layers, n_tokens, d, k, tau, d_out, n_rounds, x_dtype, table_dtype))
        return LFFN_E_UNSUPPORTED;
    if (n_tokens == 0) return LFFN_OK;
    return launch_forward_stack(x, signs, tables, y, n_tokens, d, k, tau, d_out, n_rounds, n_layers, x_dtype,
                                table_dtype, static_cast<hipStream_t>(hip_stream));
}

int64_t lookupffn_static_scratch_bytes(void) { return kStaticScratchBytes; }

int lookupffn_forward_static(const void *x, const int8_t *signs, const void *tables, void *y, int64_t n_tokens,
                             int d, int k, int tau, int d_out, int n_rounds, int x_dtype, int table_dtype,
                             void *hip_stream)
{
    // sizes first (no HIP call yet): a batch whose intermediates do not fit the static array is refused
    if (n_tokens > 0 && k >= 1 && tau >= 1 && tau <= 16 && n_tokens <= (int64_t(1) << 40) && k <= (1 << 20) &&
        forward_ws_bytes(n_tokens, k, tau, kPlain) > kStaticScratchBytes)
        return LFFN_E_WORKSPACE;
    void *ws = reinterpret_cast<void *>(uintptr_t(256));  // stand-in until the arguments have been checked
    if (n_tokens > 0 && x && signs && tables && y) {
        int rc = static_scratch(&ws);
        if (rc != LFFN_OK) return rc;
    }
    return forward_core(sign_hash(signs, n_rounds), kPlain, x, tables, y, n_tokens, d, k, tau, d_out, x_dtype,
                        table_dtype, ws, kStaticScratchBytes, static_cast<hipStream_t>(hip_stream));
}

int lookupffn_forward_weighted(const void *x, const int8_t *signs, const void *tables, void *y, int64_t n_tokens,
                               int d, int k, int tau, int d_out, int n_rounds, int x_dtype, int table_dtype,
                               void *workspace, int64_t workspace_bytes, void *hip_stream)
{
    return forward_core(sign_hash(signs, n_rounds), kWeighted, x, tables, y, n_tokens, d, k, tau, d_out, x_dtype,
                        table_dtype, workspace, workspace_bytes, static_cast<hipStream_t>(hip_stream));
}

int lookupffn_forward_probes(const void *x, const int8_t *signs, const void *tables, void *y, int64_t n_tokens,
                             int d, int k, int tau, int d_out, int n_rounds, int x_dtype, int table_dtype,
                             void *workspace, int64_t workspace_bytes, void *hip_stream)
{
    return forward_core(sign_hash(signs, n_rounds), kProbes, x, tables, y, n_tokens, d, k, tau, d_out, x_dtype,
                        table_dtype, workspace, workspace_bytes, static_cast<hipStream_t>(hip_stream));
}

int lookupffn_hash_bh(const void *x, const float *bmats, uint16_t *codes, int64_t n_tokens, int d, int k, int tau,
                      int block, int n_factors, int x_dtype, void *workspace, int64_t workspace_bytes,
                      void *hip_stream)
{
    return hash_bh_core(x, bmats, codes, nullptr, false, n_tokens, d, k, tau, block, n_factors, x_dtype, workspace,
                        workspace_bytes, static_cast<hipStream_t>(hip_stream));
}

int lookupffn_hash_bh_weighted(const void *x, const float *bmats, uint16_t *codes, float *weights, int64_t n_tokens,
                               int d, int k, int tau, int block, int n_factors, int x_dtype, void *workspace,
                               int64_t workspace_bytes, void *hip_stream)
{
    if (!weights) return (x && bmats && codes) ? LFFN_E_NULL : LFFN_E_NULL;
    return hash_bh_core(x, bmats, codes, weights, true, n_tokens, d, k, tau, block, n_factors, x_dtype, workspace,
                        workspace_bytes, static_cast<hipStream_t>(hip_stream));
}

int lookupffn_forward_bh(const void *x, const float *bmats, const void *tables, void *y, int64_t n_tokens, int d,
                         int k, int tau, int d_out, int block, int n_factors, int x_dtype, int table_dtype,
                         void *workspace, int64_t workspace_bytes, void *hip_stream)
{
    return forward_core(bh_hash(bmats, block, n_factors), kPlain, x, tables, y, n_tokens, d, k, tau, d_out, x_dtype,
                        table_dtype, workspace, workspace_bytes, static_cast<hipStream_t>(hip_stream));
}

int lookupffn_forward_bh_weighted(const void *x, const float *bmats, const void *tables, void *y, int64_t n_tokens,
                                  int d, int k, int tau, int d_out, int block, int n_factors, int x_dtype,
                                  int table_dtype, void *workspace, int64_t workspace_bytes, void *hip_stream)
{
    return forward_core(bh_hash(bmats, block, n_factors), kWeighted, x, tables, y, n_tokens, d, k, tau, d_out,
                        x_dtype, table_dtype, workspace, workspace_bytes, static_cast<hipStream_t>(hip_stream));
}

// ---- one-time preparation of the learned constants ------------------------------------------------
int64_t lookupffn_prepared_tables_bytes(int k, int tau, int d_out, int table_dtype)
{
    if (k < 1 || tau < 1 || tau > 16 || d_out < 1 || !dtype_ok(table_dtype)) return 0;
    if (d_out % (table_dtype == LFFN_F32 ? 4 : 8) != 0 || ((int64_t)k << tau) > (int64_t(1) << 31)) return 0;
    return prepared_tables_bytes(k, tau, d_out);
}

int lookupffn_prepare_tables(const void *tables, int k, int tau, int d_out, int table_dtype, void *prepared,
                             int64_t prepared_bytes, void *hip_stream)
{
    if (!tables || !prepared) return LFFN_E_NULL;
    if (k < 1 || d_out < 1 || k > (1 << 20) || d_out > (1 << 24)) return LFFN_E_SIZE;
    if (tau < 1 || tau > 16) return LFFN_E_TAU;
    if (!dtype_ok(table_dtype)) return LFFN_E_DTYPE;
    if (d_out % (table_dtype == LFFN_F32 ? 4 : 8) != 0) return LFFN_E_ALIGN;
    if (((int64_t)k << tau) > (int64_t(1) << 31)) return LFFN_E_SIZE;
    if (!aligned(tables, 16) || !aligned(prepared, 256)) return LFFN_E_ALIGN;
    const int64_t need = prepared_tables_bytes(k, tau, d_out);
    if (prepared_bytes < need) return LFFN_E_WORKSPACE;
    const int pw = prepared_piece_bytes(tau), ppw = pw / 16;
    const int rows = 1 << tau, nvec = d_out / 4;
    const long long n_ps = (nvec + ppw - 1) / ppw;
    const long long n_out = n_ps * k * rows * ppw;
    long long blocks = (n_out + 255) / 256;
    if (blocks > 16384) blocks = 16384;
    hipLaunchKernelGGL(prepare_tables_kernel, dim3((unsigned)blocks), dim3(256), 0, static_cast<hipStream_t>(hip_stream),
                       tables, static_cast<uint4 *>(prepared), k, rows, nvec, ppw, table_dtype, n_out);
    LFFN_HIP(hipGetLastError());
    return LFFN_OK;
}

int64_t lookupffn_prepared_bh_bytes(int d, int k, int tau, int block, int n_factors)
{
    if (!bh_shape_ok(d, k, tau, block, n_factors) || (block != 16 && block != 32 && block != 64)) return 0;
    return bh_pack_bytes(d, k, tau, block, n_factors);
}

int lookupffn_prepare_bh(const float *bmats, int d, int k, int tau, int block, int n_factors, void *prepared,
                         int64_t prepared_bytes, void *hip_stream)
{
    if (!prepared) return LFFN_E_NULL;
    const float *stand_in_x = reinterpret_cast<const float *>(uintptr_t(256));
    int rc = check_bh(stand_in_x, bmats, 0, d, k, tau, block, n_factors, LFFN_F32);
    if (rc != LFFN_OK) return rc;
    if (!aligned(prepared, 256)) return LFFN_E_ALIGN;
    if (prepared_bytes < bh_pack_bytes(d, k, tau, block, n_factors)) return LFFN_E_WORKSPACE;
    return launch_bh_pack(bmats, static_cast<float *>(prepared), d, k, tau, block, n_factors,
                          static_cast<hipStream_t>(hip_stream));
}

int lookupffn_release_workspace(void)
{
    std::lock_guard<std::mutex> lk(g_ws_mu);
    int rc = LFFN_OK;
    int cur = 0;
    const bool have_cur = hipGetDevice(&cur) == hipSuccess;
    for (auto &kv : g_ws) {
        if (!kv.second.ptr && kv.second.retired.empty()) continue;
        if (hipSetDevice(kv.first) != hipSuccess || hipDeviceSynchronize() != hipSuccess) rc = LFFN_E_HIP;
        if (kv.second.ptr && hipFree(kv.second.ptr) != hipSuccess) rc = LFFN_E_HIP;
        for (void *p : kv.second.retired)
            if (hipFree(p) != hipSuccess) rc = LFFN_E_HIP;
        kv.second = Workspace();
    }
    if (have_cur) (void)hipSetDevice(cur);
    g_ws.clear();
    return rc;
}

int lookupffn_timing_enable(int mask)
{
    if (mask < 0 || mask > 3) return LFFN_E_SIZE;
    g_tm.on.store(mask);
    return LFFN_OK;
}

int lookupffn_timing_reset(void)
{
    std::lock_guard<std::mutex> lk(g_tm.mu);
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
    std::lock_guard<std::mutex> lk(g_tm.mu);
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

int lookupffn_timing_read_each(int which, double *ms_out, int64_t capacity, int64_t *launches)
{
    if (which < 0 || which > 1 || capacity < 0) return LFFN_E_SIZE;
    if (!launches || (capacity > 0 && !ms_out)) return LFFN_E_NULL;
    std::lock_guard<std::mutex> lk(g_tm.mu);
    int64_t i = 0;
    for (auto &p : g_tm.ev[which]) {
        if (i >= capacity) break;
        LFFN_HIP(hipEventSynchronize(p.second));
        float ms = 0.0f;
        LFFN_HIP(hipEventElapsedTime(&ms, p.first, p.second));
        ms_out[i++] = ms;
    }
    *launches = (int64_t)g_tm.ev[which].size();
    return LFFN_OK;
}

int lookupffn_set_option(const char *key, int value)
{
    if (!key) return LFFN_E_NULL;
    std::lock_guard<std::mutex> lk(g_opt_mu);
    if (!std::strcmp(key, "lanes_per_token")) {
        if (value != 0 && (value < 1 || value > 64 || (value & (value - 1)))) return LFFN_E_SIZE;
        g_opt.lanes_per_token = value;
        return LFFN_OK;
    }
    if (!std::strcmp(key, "hash_path")) {
        if (value < 0 || value > 3) return LFFN_E_SIZE;
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
    if (!std::strcmp(key, "ring_threads")) {
        if (value != 0 && value != 512 && value != 1024) return LFFN_E_SIZE;
        g_opt.ring_threads = value;
        return LFFN_OK;
    }
    if (!std::strcmp(key, "small_tokens")) {
        if (value < -1 || value > (1 << 20)) return LFFN_E_SIZE;
        g_opt.small_tokens = value;
        return LFFN_OK;
    }
    if (!std::strcmp(key, "token_slots")) {
        if (value < 0 || value > 32) return LFFN_E_SIZE;
        g_opt.token_slots = value;
        return LFFN_OK;
    }
    if (!std::strcmp(key, "gather_path")) {
        if (value < 0 || value > 4) return LFFN_E_SIZE;
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
        case LFFN_E_UNSUPPORTED: return "shape not supported by this entry point";
        case LFFN_E_WORKSPACE: return "workspace or output buffer too small";
        case LFFN_E_HIP: return "a HIP call failed";
        default: return "unknown status";
    }
}

const char *lookupffn_last_hip_error(void) { return g_hip_error.c_str(); }

const char *lookupffn_last_gather_kernel(void) { return t_last_gather; }
const char *lookupffn_last_hash_kernel(void) { return t_last_hash; }

int lookupffn_version(void) { return kVersion; }

}  // extern "C"

#endif  // LFFN_HAS(0)
