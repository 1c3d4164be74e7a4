// LDS-staged gather for small tables (2^tau * 128 bytes * 2 buffers must fit the 160 KB LDS):
//   y[t][:] = sum_{j<k} tables[j][code[t][j]][:]        (Sec. 3.1, eq. "lookup")
//
// With tau = 8 a table has only 256 rows, so a batch of thousands of tokens
// picks every row many times.  A 1024-thread workgroup owns one 128-byte
// column slice and a chunk of up to 128*TOK tokens.  For each table j in turn
// it copies the slice of all 2^tau rows (32 KB at tau = 8) into LDS once --
// double-buffered, table j+1 is in flight while table j is consumed -- and
// every (token, 16-byte piece) lane then reads its selected row from LDS with
// one ds_read_b128 (eight consecutive lanes read one contiguous 128-byte row
// piece: conflict-free) and adds it to its fp32 accumulators.  Each output
// element is still the sequential fp32 sum over j = 0..k-1, so results equal
// the direct kernel's bit for bit, while the L2 -> CU traffic drops from one
// row per (token, table) to one row per (chunk, table, row).
//
// Work distribution is static and XCD-aware: slice-units are dealt to the
// eight XCDs round-robin (block b runs on XCD b % 8), and the workgroups of
// one XCD split its units' token ranges evenly, so every CU gets one chunk of
// near-equal size and the slice a CU streams stays in its XCD's L2.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "gather_kernel.hpp"

namespace lffn {

constexpr int kLdsThreads = 1024;
constexpr int kLdsGroups = kLdsThreads / 8;  // token groups per workgroup (8 lanes per token)

struct GatherLdsArgs {
    const uint16_t *codes;  // [n][k], k % 2 == 0, 4-byte aligned
    const char *tables;
    float *y;
    long long n;
    int k, tau, d_out;
    int nvec;           // 16-byte pieces per row
    int n_slices;       // ceil(nvec / 8)
    int token_splits;   // a unit = (slice, one of token_splits equal token ranges)
    int n_units;        // n_slices * token_splits
    int blocks_per_xcd; // gridDim.x / kXcds
    uint32_t row_bytes;
};

// balanced split of [0, len) into `parts` pieces: start of piece i (32-bit arithmetic only)
__device__ __forceinline__ uint32_t split_at(uint32_t len, uint32_t parts, uint32_t i)
{
    const uint32_t base = len / parts, rem = len - base * parts;
    return base * i + (i < rem ? i : rem);
}

template <bool BF16, int TOK, int FILL>
__global__ __launch_bounds__(kLdsThreads) void gather_lds_kernel(GatherLdsArgs a)
{
    extern __shared__ uint4 sbuf[];
    const uint32_t tid = threadIdx.x;
    const uint32_t g = tid >> 3, q = tid & 7u;
    const uint32_t rows = 1u << a.tau;
    const uint32_t bufsz = rows * 8u;  // uint4 elements per buffer
    const uint32_t rmask = rows - 1u;
    const uint32_t k = (uint32_t)a.k;
    const uint32_t n = (uint32_t)a.n;  // the host uses this kernel only for n < 2^31

    // ---- which (unit, token range) pairs does this workgroup own? ---------------------
    const uint32_t xcd = blockIdx.x % kXcds;
    const uint32_t c = blockIdx.x / kXcds;
    const uint32_t Bx = (uint32_t)a.blocks_per_xcd;
    if ((uint32_t)a.n_units <= xcd) return;
    const uint32_t m = ((uint32_t)a.n_units - xcd + kXcds - 1) / kXcds;  // units dealt to this XCD
    uint32_t u_first, u_step, u_end, part, parts;
    if (m >= Bx) {  // at least one unit per workgroup: take whole units c, c+Bx, ...
        u_first = c;
        u_step = Bx;
        u_end = m;
        part = 0;
        parts = 1;
    } else {        // several workgroups share a unit: split its token range evenly
        u_first = c * m / Bx;
        u_step = 1;
        u_end = u_first + 1;
        const uint32_t first_blk = (u_first * Bx + m - 1) / m;
        const uint32_t next_blk = ((u_first + 1) * Bx + m - 1) / m;
        part = c - first_blk;
        parts = next_blk - first_blk;
    }

    for (uint32_t ui = u_first; ui < u_end; ui += u_step) {
        const uint32_t unit = ui * kXcds + xcd;
        const uint32_t slice = unit % (uint32_t)a.n_slices;
        const uint32_t split = unit / (uint32_t)a.n_slices;
        const uint32_t s0 = split_at(n, (uint32_t)a.token_splits, split);
        const uint32_t s1 = split_at(n, (uint32_t)a.token_splits, split + 1);
        const uint32_t r0 = s0 + split_at(s1 - s0, parts, part), r1 = s0 + split_at(s1 - s0, parts, part + 1);
        if (r1 <= r0) continue;  // uniform over the workgroup

        const uint32_t vec = slice * 8u + q;
        const bool vec_ok = vec < (uint32_t)a.nvec;

        // fill role of this thread: pieces tid, tid + 1024, ... of the [rows][8] slice;
        // byte offsets inside one table fit 32 bits (checked by the host)
        uint32_t foff[FILL];
        bool fok[FILL];
#pragma unroll
        for (int f = 0; f < FILL; ++f) {
            const uint32_t p = tid + (uint32_t)f * kLdsThreads;
            const uint32_t prow = p >> 3, pvec = slice * 8u + (p & 7u);
            fok[f] = p < bufsz && pvec < (uint32_t)a.nvec;
            foff[f] = fok[f] ? prow * a.row_bytes + pvec * 16u : 0u;
        }
        const size_t table_stride = (size_t)rows * a.row_bytes;

        const uint32_t len = r1 - r0;
        const uint32_t nchunks = (len + kLdsGroups * TOK - 1) / (kLdsGroups * TOK);
        for (uint32_t ch = 0; ch < nchunks; ++ch) {
            const uint32_t c0 = r0 + split_at(len, nchunks, ch), c1 = r0 + split_at(len, nchunks, ch + 1);
            // Accumulator i belongs to token c0 + i*128 + g.  Tokens past the chunk end are clamped
            // to its last token for the loads and skipped at the store.
            const uint32_t kbytes = k * 2u;
            const uint32_t last_off = (c1 - 1u - c0) * kbytes;
            const char *cchunk = reinterpret_cast<const char *>(a.codes) + (size_t)c0 * kbytes;  // uniform
            const uint32_t goff = g * kbytes;
            auto load_codes = [&](int i, uint32_t j) -> uint32_t {
                uint32_t off = goff + (uint32_t)i * (kLdsGroups * kbytes);
                off = off < last_off ? off : last_off;
                return *reinterpret_cast<const uint32_t *>(cchunk + (off + j * 2u));
            };

            Acc<BF16> acc[TOK];
#pragma unroll
            for (int i = 0; i < TOK; ++i) acc[i].zero();

            // prologue: table 0 into buffer 0, first two codes of every token
            uint4 fill[FILL];
#pragma unroll
            for (int f = 0; f < FILL; ++f)
                fill[f] = fok[f] ? *reinterpret_cast<const uint4 *>(a.tables + foff[f]) : make_uint4(0, 0, 0, 0);
            uint32_t cr[TOK];  // codes of tables j, j+1 (low, high half)
#pragma unroll
            for (int i = 0; i < TOK; ++i) cr[i] = load_codes(i, 0);
#pragma unroll
            for (int f = 0; f < FILL; ++f)
                if (tid + f * kLdsThreads < bufsz) sbuf[tid + f * kLdsThreads] = fill[f];
            __syncthreads();

            for (uint32_t j = 0; j < k; j += 2) {
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    const uint32_t jj = j + u;
                    const bool more = jj + 1 < k;
                    if (more) {
                        const char *tnext = a.tables + (size_t)(jj + 1) * table_stride;  // uniform
#pragma unroll
                        for (int f = 0; f < FILL; ++f)
                            fill[f] = fok[f] ? *reinterpret_cast<const uint4 *>(tnext + foff[f])
                                             : make_uint4(0, 0, 0, 0);
                    }
                    const uint4 *buf = sbuf + u * bufsz + q;
                    // LDS reads in batches of RB tokens: bounds the registers held by rows in flight
                    constexpr int RB = 4;
#pragma unroll
                    for (int b0 = 0; b0 < TOK; b0 += RB) {
                        uint4 r[RB];
#pragma unroll
                        for (int i = 0; i < RB; ++i)
                            if (b0 + i < TOK) {
                                const uint32_t code = (u ? (cr[b0 + i] >> 16) : (cr[b0 + i] & 0xFFFFu)) & rmask;
                                r[i] = buf[code * 8u];
                            }
#pragma unroll
                        for (int i = 0; i < RB; ++i)
                            if (b0 + i < TOK) {
                                acc[b0 + i].add(r[i]);
                                acc[b0 + i].pin();
                            }
                    }
                    if (u == 1 && j + 2 < k) {
#pragma unroll
                        for (int i = 0; i < TOK; ++i) cr[i] = load_codes(i, j + 2);
                    }
                    if (more) {
                        uint4 *dst = sbuf + (u ^ 1) * bufsz;
#pragma unroll
                        for (int f = 0; f < FILL; ++f)
                            if (tid + f * kLdsThreads < bufsz) dst[tid + f * kLdsThreads] = fill[f];
                    }
                    __syncthreads();
                }
            }

            if (vec_ok) {
                typedef float f4 __attribute__((ext_vector_type(4)));
#pragma unroll
                for (int i = 0; i < TOK; ++i) {
                    const uint32_t t = c0 + (uint32_t)i * kLdsGroups + g;
                    if (t >= c1) continue;
                    float *yp = a.y + (size_t)t * a.d_out + (size_t)vec * Acc<BF16>::W;
                    f4 o0 = {acc[i].f[0], acc[i].f[1], acc[i].f[2], acc[i].f[3]};
                    __builtin_nontemporal_store(o0, reinterpret_cast<f4 *>(yp));
                    if constexpr (BF16) {
                        f4 o1 = {acc[i].f[4], acc[i].f[5], acc[i].f[6], acc[i].f[7]};
                        __builtin_nontemporal_store(o1, reinterpret_cast<f4 *>(yp) + 1);
                    }
                }
            }
        }
    }
}

}  // namespace lffn
