// Gather step of the LookupFFN forward pass for gfx950:
//   y[t][:] = sum_{j<k} tables[j][code[t][j]][:]        (Sec. 3.1, eq. "lookup")
// and its weighted form y[t][:] = sum_j w[t][j] * tables[j][code[t][j]][:] (Sec. 4; one fused
// multiply-add per element and table, in table order), and the multi-probe form
//   y[t][:] = sum_j sum_{probe <= tau} p[t][j][probe] * tables[j][code ^ flip(probe)][:]
// (Sec. 3.1, eq. "partial_softmax": the selected row, then the rows one bit away, bit 0 first).
//
// Work decomposition.  A table row is cut into column slices of LPT lanes x 16
// bytes (LPT = "lanes per token"); a wavefront handles 64/LPT tokens of one
// slice: lane = (token within the wave, 16-byte piece within the slice).  Each
// lane walks the k tables in order, fetches its 16 bytes of the selected row
// with one dwordx4 load and adds them into fp32 accumulators -- the same
// sequential fp32 sum per output element as a plain loop over j.
//
// Why slices: one slice of all k tables (k * 2^tau * LPT*16 bytes, 3 MiB for
// k = 96, tau = 8, LPT = 8) fits the 4 MiB L2 of one XCD while a whole table
// set (72 MiB) does not.  Blocks are numbered so that the eight XCDs (block b
// runs on XCD b % 8) each sweep all their tokens for one slice before moving
// to the next one, so after first touch the row fetches are L2 hits instead of
// trips to the Infinity Cache / HBM.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "elem16.hpp"

namespace lffn {

constexpr int kGatherThreads = 256;
constexpr int kGatherWaves = kGatherThreads / 64;
constexpr int kXcds = 8;

struct GatherArgs {
    const uint16_t *codes;  // [n][k]
    const float *weights;   // [n][k] for the weighted form, [n][k][1+tau] for the multi-probe form, else NULL
    const char *tables;     // [k][rows][d_out] fp32, bf16 or IEEE half
    void *y;                // [n][d_out] fp32, or bf16 / IEEE half when y_kind says so
    int y_kind;             // 0 fp32, 1 bf16, 2 IEEE half
    long long n;
    int k, tau, d_out;
    int nvec;          // 16-byte pieces per row
    int n_slices;      // ceil(nvec / LPT)
    int n_units;       // n_slices * token_splits; a unit = (slice, contiguous range of token blocks)
    int tb_per_unit;   // token blocks in one unit
    int ntb;           // token blocks in total; a token block = kGatherWaves * (64/LPT) tokens
    int xcd_mode;      // 1: block order is XCD-sliced (see above); 0: plain
    int codes_vec8;    // 1: k % 8 == 0 and codes (and weights) 16-byte aligned -> read 8 at a time
    int code_stride;   // codes (and weights, and groups of 1 + tau shares) per token in the arrays; k unless
                       // the launch covers only some of the tables
    int accumulate;    // 1: the sums start from what y holds (fp32 y, fp32 rows) instead of zero
    // The 16-byte piece q of row r = (j << tau) + code in slice s sits at
    //   tables + (s / spp) * slice_stride + (s % spp) * LPT*16 + r * row_stride + q*16
    // row-major tables: spp = 1, slice_stride = LPT*16, row_stride = bytes of a row; prepared tables
    // (slice-major, PW bytes per row piece): spp = PW / (LPT*16), slice_stride = k * rows * PW, row_stride = PW.
    uint32_t row_stride;
    uint32_t spp;
    unsigned long long slice_stride;
};

// KIND: element type of the rows (0 fp32, 1 bf16, 2 IEEE half)
template <int KIND>
struct Acc {
    static constexpr int W = KIND ? 8 : 4;  // elements in 16 bytes
    float f[W];
    __device__ __forceinline__ void zero()
    {
#pragma unroll
        for (int i = 0; i < W; ++i) f[i] = 0.0f;
    }
    // Empty asm that "touches" the accumulators: keeps the compiler from sinking the additions
    // past this point (it otherwise defers them to the loop latch, stretching the live ranges
    // of every fetched row).
    __device__ __forceinline__ void pin()
    {
        asm volatile("" : "+v"(f[0]), "+v"(f[1]), "+v"(f[2]), "+v"(f[3]));
        if constexpr (KIND != 0) asm volatile("" : "+v"(f[4]), "+v"(f[5]), "+v"(f[6]), "+v"(f[7]));
    }
    // the W elements of 16 bytes of a row, widened exactly
    __device__ __forceinline__ void unpack(const uint4 &r, float (&e)[W]) const
    {
        if constexpr (KIND != 0) {
            const float2 a = widen16x2<KIND == 0 ? 1 : KIND>(r.x), b = widen16x2<KIND == 0 ? 1 : KIND>(r.y),
                         c = widen16x2<KIND == 0 ? 1 : KIND>(r.z), d = widen16x2<KIND == 0 ? 1 : KIND>(r.w);
            e[0] = a.x;
            e[1] = a.y;
            e[2] = b.x;
            e[3] = b.y;
            e[4] = c.x;
            e[5] = c.y;
            e[6] = d.x;
            e[7] = d.y;
        } else {
            e[0] = __uint_as_float(r.x);
            e[1] = __uint_as_float(r.y);
            e[2] = __uint_as_float(r.z);
            e[3] = __uint_as_float(r.w);
        }
    }
    __device__ __forceinline__ void add(const uint4 &r)
    {
        float e[W];
        unpack(r, e);
#pragma unroll
        for (int i = 0; i < W; ++i) f[i] += e[i];
    }
    // acc += w * row, one rounding per element
    __device__ __forceinline__ void fma(const uint4 &r, float w)
    {
        float e[W];
        unpack(r, e);
#pragma unroll
        for (int i = 0; i < W; ++i) f[i] = __builtin_fmaf(w, e[i], f[i]);
    }
};

__device__ __forceinline__ uint32_t code_of(const uint4 &c, int u)
{
    const uint32_t w = u < 2 ? c.x : u < 4 ? c.y : u < 6 ? c.z : c.w;
    return (u & 1) ? (w >> 16) : (w & 0xFFFFu);
}

// WMODE: 0 = plain sum, 1 = weighted form, 2 = multi-probe form
template <int KIND, int LPT, int WMODE>
__global__ __launch_bounds__(kGatherThreads) void gather_kernel(GatherArgs a)
{
    constexpr int TPW = 64 / LPT;  // tokens per wave
    const unsigned lane = threadIdx.x & 63u;
    const unsigned wave = threadIdx.x >> 6;

    // ---- block -> (slice, token block) -------------------------------------------------
    int unit, tbl;
    if (a.xcd_mode) {
        const int xcd = (int)(blockIdx.x % kXcds);
        const int q = (int)(blockIdx.x / kXcds);
        unit = (q / a.tb_per_unit) * kXcds + xcd;
        tbl = q % a.tb_per_unit;
    } else {
        unit = (int)(blockIdx.x % (unsigned)a.n_units);
        tbl = (int)(blockIdx.x / (unsigned)a.n_units);
    }
    if (unit >= a.n_units) return;
    const int slice = unit % a.n_slices;
    const int tb = (unit / a.n_slices) * a.tb_per_unit + tbl;
    if (tb >= a.ntb) return;

    const long long t = ((long long)tb * kGatherWaves + wave) * TPW + lane / LPT;
    const int vec = slice * LPT + (int)(lane % LPT);
    if (t >= a.n || vec >= a.nvec) return;  // no barrier below: early exit is safe

    const uint16_t *crow = a.codes + t * a.code_stride;
    const char *tcol = a.tables + (size_t)((unsigned)slice / a.spp) * (size_t)a.slice_stride +
                       (size_t)((unsigned)slice % a.spp) * (LPT * 16u) + (size_t)(lane % LPT) * 16u;
    const uint32_t rmask = (1u << a.tau) - 1u;
    const uint32_t row_bytes = a.row_stride;
    const int k = a.k, tau = a.tau;

    auto row = [&](int j, uint32_t code) -> uint4 {
        const uint32_t r = ((uint32_t)j << tau) + (code & rmask);
        return *reinterpret_cast<const uint4 *>(tcol + (unsigned long long)r * row_bytes);
    };

    Acc<KIND> acc;
    acc.zero();
    if constexpr (KIND == 0) {
        if (a.accumulate) {
            const float4 y0 = *reinterpret_cast<const float4 *>(static_cast<const float *>(a.y) +
                                                                 (size_t)t * a.d_out + (size_t)vec * 4);
            acc.f[0] = y0.x, acc.f[1] = y0.y, acc.f[2] = y0.z, acc.f[3] = y0.w;
        }
    }

    int j0 = 0;
    if constexpr (WMODE == 2) {
        const float *wp = a.weights + t * a.code_stride * (tau + 1);
        const int np = tau + 1;
        for (int j = 0; j < k; ++j, wp += np) {
            const uint32_t g = crow[j] & rmask;
            int pr = 0;
            for (; pr + 3 <= np; pr += 3) {  // three probes at a time: rows and shares first, then the adds
                uint4 r[3];
                float w[3];
#pragma unroll
                for (int u = 0; u < 3; ++u) {
                    const int q = pr + u;
                    r[u] = row(j, q == 0 ? g : g ^ (1u << (q - 1)));
                    w[u] = wp[q];
                }
#pragma unroll
                for (int u = 0; u < 3; ++u) acc.fma(r[u], w[u]);
            }
            for (; pr < np; ++pr) acc.fma(row(j, pr == 0 ? g : g ^ (1u << (pr - 1))), wp[pr]);
        }
        j0 = k;
    } else if constexpr (WMODE == 1) {
        const float *wrow = a.weights + t * a.code_stride;
        if (a.codes_vec8) {
            const uint4 *c8 = reinterpret_cast<const uint4 *>(crow);
            const float4 *w4 = reinterpret_cast<const float4 *>(wrow);
            const int nch = k >> 3;
            uint4 cn = c8[0];
            float4 wan = w4[0], wbn = w4[1];
            for (int ch = 0; ch < nch; ++ch) {
                const uint4 c = cn;
                const float4 wa = wan, wb = wbn;
                const int nx = ch + 1 < nch ? ch + 1 : ch;  // next chunk's codes and weights go out first
                cn = c8[nx];
                wan = w4[2 * nx];
                wbn = w4[2 * nx + 1];
                uint4 r[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) r[u] = row(ch * 8 + u, code_of(c, u));
                acc.fma(r[0], wa.x);
                acc.fma(r[1], wa.y);
                acc.fma(r[2], wa.z);
                acc.fma(r[3], wa.w);
                acc.fma(r[4], wb.x);
                acc.fma(r[5], wb.y);
                acc.fma(r[6], wb.z);
                acc.fma(r[7], wb.w);
            }
            j0 = nch * 8;
        }
        for (; j0 < k; ++j0) acc.fma(row(j0, crow[j0]), wrow[j0]);
    } else if (a.codes_vec8) {
        const uint4 *c8 = reinterpret_cast<const uint4 *>(crow);
        const int nch = k >> 3;  // chunks of 8 codes
        int ch = 0;
        if (nch >= 2) {
            uint4 c0 = c8[0], c1 = c8[1];
            for (; ch + 2 <= nch; ch += 2) {
                const uint4 u0 = c0, u1 = c1;
                // fetch the next two code chunks before the row loads of this pair go out
                const int nx = ch + 2 <= nch - 2 ? ch + 2 : nch - 2;
                c0 = c8[nx];
                c1 = c8[nx + 1];
                uint4 r[16];
#pragma unroll
                for (int u = 0; u < 8; ++u) r[u] = row(ch * 8 + u, code_of(u0, u));
#pragma unroll
                for (int u = 0; u < 8; ++u) r[8 + u] = row(ch * 8 + 8 + u, code_of(u1, u));
#pragma unroll
                for (int u = 0; u < 16; ++u) acc.add(r[u]);
            }
        }
        if (ch < nch) {
            const uint4 u0 = c8[ch];
            uint4 r[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) r[u] = row(ch * 8 + u, code_of(u0, u));
#pragma unroll
            for (int u = 0; u < 8; ++u) acc.add(r[u]);
            ++ch;
        }
        j0 = nch * 8;
    }
    for (; j0 + 4 <= k; j0 += 4) {
        uint4 r[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) r[u] = row(j0 + u, crow[j0 + u]);
#pragma unroll
        for (int u = 0; u < 4; ++u) acc.add(r[u]);
    }
    for (; j0 < k; ++j0) acc.add(row(j0, crow[j0]));

    // ---- a6: store, streaming (y is written once and not read again here) -------------
    const size_t e = (size_t)t * a.d_out + (size_t)vec * Acc<KIND>::W;
    store_y4(a.y, e, acc.f[0], acc.f[1], acc.f[2], acc.f[3], a.y_kind);
    if constexpr (KIND != 0) store_y4(a.y, e + 4, acc.f[4], acc.f[5], acc.f[6], acc.f[7], a.y_kind);
}

}  // namespace lffn
