// Small-batch forward pass of LookupFFN for gfx950: hash and gather of one or several chained layers in a
// single launch (Sec. 3.1: z = x (D1 H)(D2 H)(D3 H) -- eq. "hadamard" --, tau-bit sign codes, then
// y = sum_j T_j[code_j] -- eq. "lookup"; layer l+1 takes layer l's y as its x).
//
// With a handful of tokens the two-kernel path spends its time in launches and in a chip that is almost
// empty; here one workgroup owns one token for the whole stack, so nothing leaves the compute unit between
// the hash and the gather, nor between layers:
//   * wave 0 transforms the row (the same round function as hash1024_kernel, so the same bits), forms the
//     sign-bit string and turns each code into the byte offset of the selected row, in LDS;
//   * every lane then owns one dword of the output row (one fp32 column, or two 16-bit columns) and walks the
//     k tables IN ORDER: the row offset is wave-uniform, so the fetch is a buffer load with the lane's
//     column offset in a VGPR and the row offset in an SGPR; 32 fetches are issued back to back into one
//     register set while the previous 32 are added;
//   * the sum goes to LDS as the next layer's input (two buffers, swapped per layer: one barrier separates
//     a layer's writes from the next layer's reads) and, after the last layer, to y.
// The additions are the same sequential fp32 sum per output element as the large-batch gather kernels
// make, so a stack run equals the layer-by-layer loop bit for bit.
//
// What bounds it: one compute unit takes in rows from beyond its L2 at about 27 bytes per clock (64 GB/s),
// whatever the load width (1, 2, 4 dwords per lane) or the number of loads in flight (16 to 96 per wave
// were tried, all at once or as a queue); k rows of d_out fp32 values are 288 KiB for k = 96, d_out = 768,
// i.e. 4.5 us, and the three rounds of a 1024-point transform in one wave take about 1.7 us (spread over
// four waves that exchange through LDS they take as long: the butterflies of a round depend on one
// another).
//
// Shapes: d_pad = 1024 (512 < d <= 1024); table set below 2 GiB (32-bit buffer offsets); row-major fp32, bf16
// or IEEE half tables, or the prepared (slice-major, fp32) layout.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "hash_kernel.hpp"

namespace lffn {

constexpr int kStackMaxLayers = 32;
constexpr int kStackChunk = 32;  // fetches issued back to back into one register set

struct StackArgs {
    const void *x;  // [n][d], input of the first layer
    void *y;        // [n][d_out], output of the last layer: fp32, or bf16 / IEEE half when y_kind says so
    int y_kind;
    const int8_t *signs[kStackMaxLayers];  // per layer [P][R][1024]
    const char *tables[kStackMaxLayers];   // per layer, all in the same layout
    long long n;
    int d, d_out, k, tau, P, n_layers;
    int x_kind;  // element type of x: 0 fp32, 1 bf16, 2 IEEE half
    float scale;
    uint32_t row_dwords;  // dwords of one table row
    // byte offset of dword q of row r (r = (j << tau) + code), with b = 4q:
    //   (b >> piece_shift) * slice_stride + (b & ((1 << piece_shift) - 1)) + r * row_stride
    // row-major tables: piece_shift = 31 (the quotient is 0), row_stride = bytes of a row;
    // prepared tables: pieces of 1 << piece_shift bytes, row_stride = the piece, slice_stride = k * rows * piece
    uint32_t piece_shift, row_stride;
    uint32_t slice_stride;
    uint32_t table_bytes;  // extent of one layer's tables
};

__host__ __device__ inline int stack_code_words(int k) { return (k + kStackChunk - 1) / kStackChunk * kStackChunk; }
__host__ __device__ inline int stack_bit_words(int P) { return (hash_bit_words(P, 1024) + 3) & ~3; }
// LDS: wave 0's transpose area and bit string, the row offsets, two row buffers of 1024 floats
__host__ __device__ inline size_t stack_lds_bytes(int P, int k)
{
    return ((size_t)kH1024TransposeWords + stack_bit_words(P) + stack_code_words(k) + 2 * 1024) * 4;
}

template <int R, int KIND>
__global__ __launch_bounds__(1024) void forward_stack_kernel(StackArgs a)
{
    constexpr int N = 1024, NREG = 16;
    constexpr bool HALF16 = KIND != 0;  // two 16-bit columns per dword
    constexpr int CH = HALF16 ? kStackChunk / 2 : kStackChunk;  // two accumulators and the unpacking need registers too
    extern __shared__ uint32_t lds[];
    const unsigned tid = threadIdx.x;
    const unsigned lane = tid & 63u;
    const unsigned wave = tid >> 6;
    const int P = a.P;
    uint32_t *tp = lds;
    uint32_t *bitw = tp + kH1024TransposeWords;
    const int n_bitw = stack_bit_words(P);
    uint32_t *rowoff = bitw + n_bitw;
    const int n_off = stack_code_words(a.k);
    float *rowbuf = reinterpret_cast<float *>(rowoff + n_off);  // [2][1024]
    const long long t = blockIdx.x;

    // bit string, row offsets (those past k stay 0, a valid row), row buffers (the padding d .. 1023 stays 0)
    for (unsigned i = tid; i < (unsigned)(n_bitw + n_off) + 2u * N; i += blockDim.x) bitw[i] = 0;
    H1024Lane L;
    h1024_lane_setup((uint32_t)(uintptr_t)tp, lane, L);
    const bool vec_ok = (a.d % 4) == 0;
    __syncthreads();

    for (int l = 0; l < a.n_layers; ++l) {
        float *cur = rowbuf + (l & 1) * N, *nxt = rowbuf + ((l + 1) & 1) * N;
        if (wave == 0) {
            // ---- a1: the row in layout A (lane = i[9:4], register = i[3:0]) -------------------------
            float xv[NREG];
            if (l == 0) {
                h1024_load_row(a.x, t, a.d, a.x_kind, vec_ok, lane, xv);
            } else {
#pragma unroll
                for (int m = 0; m < 4; ++m) {
                    const float4 f = *reinterpret_cast<const float4 *>(cur + lane * 16 + 4 * m);
                    xv[4 * m] = f.x;
                    xv[4 * m + 1] = f.y;
                    xv[4 * m + 2] = f.z;
                    xv[4 * m + 3] = f.w;
                }
            }
            const int8_t *sg = a.signs[l];
            for (int p = 0; p < P; ++p) {
                uint32_t sw[R][4];
#pragma unroll
                for (int rd = 0; rd < R; ++rd) {
                    const uint4 w = *reinterpret_cast<const uint4 *>(sg + ((size_t)p * R + rd) * N + lane * 16);
                    sw[rd][0] = w.x;
                    sw[rd][1] = w.y;
                    sw[rd][2] = w.z;
                    sw[rd][3] = w.w;
                }
                float v[NREG];
#pragma unroll
                for (int e = 0; e < NREG; ++e) v[e] = xv[e];
#pragma unroll
                for (int rd = 0; rd < R; ++rd) {
                    if (rd + 1 < R)
                        h1024_round<false>(v, sw[rd], L, lane, a.scale);
                    else
                        h1024_round<true>(v, sw[rd], L, lane, a.scale);
                }
                h1024_sign_bits(v, lane, bitw, p);
            }
            wave_lds_fence();
            // ---- a4: code j -> byte offset of row (j << tau) + code ---------------------------------
            for (int j = (int)lane; j < a.k; j += 64)
                rowoff[j] = (((uint32_t)j << a.tau) + hash_code_at(bitw, (unsigned)j, a.tau)) * a.row_stride;
        }
        __syncthreads();

        // ---- a5: every lane sums its dword of the k selected rows, in table order -----------------------
        const __amdgpu_buffer_rsrc_t rsrc =
            __builtin_amdgcn_make_buffer_rsrc(const_cast<char *>(a.tables[l]), 0, (int)a.table_bytes, 0x00020000);
        const bool last = l + 1 == a.n_layers;
        for (uint32_t q = tid; q < a.row_dwords; q += blockDim.x) {
            const uint32_t b = q * 4u;
            const uint32_t voff = (b >> a.piece_shift) * a.slice_stride + (b & ((1u << a.piece_shift) - 1u));
            float acc0 = 0.0f, acc1 = 0.0f;
            uint32_t ra[CH], rb[CH];
            auto issue = [&](uint32_t (&r)[CH], int j0) {
#pragma unroll
                for (int u = 0; u < CH; u += 4) {
                    const uint4 o = *reinterpret_cast<const uint4 *>(rowoff + j0 + u);  // same for all lanes
                    r[u] = __builtin_amdgcn_raw_buffer_load_b32(rsrc, voff, __builtin_amdgcn_readfirstlane(o.x), 0);
                    r[u + 1] = __builtin_amdgcn_raw_buffer_load_b32(rsrc, voff, __builtin_amdgcn_readfirstlane(o.y), 0);
                    r[u + 2] = __builtin_amdgcn_raw_buffer_load_b32(rsrc, voff, __builtin_amdgcn_readfirstlane(o.z), 0);
                    r[u + 3] = __builtin_amdgcn_raw_buffer_load_b32(rsrc, voff, __builtin_amdgcn_readfirstlane(o.w), 0);
                }
            };
            // tables past k in the last chunk were fetched from offset 0 (a valid row) and are not added
            auto add_n = [&](const uint32_t (&r)[CH], int n_add) {
#pragma unroll
                for (int u = 0; u < CH; ++u) {
                    if (u < n_add) {
                        if constexpr (HALF16) {
                            const float2 e = widen16x2<KIND == 0 ? 1 : KIND>(r[u]);
                            acc0 += e.x;
                            acc1 += e.y;
                        } else {
                            acc0 += __uint_as_float(r[u]);
                        }
                    }
                }
            };
            auto add = [&](const uint32_t (&r)[CH], int j0) {
                if (j0 + CH <= a.k)
                    add_n(r, CH);
                else
                    add_n(r, a.k - j0);
            };
            const int n_ch = n_off / CH;
            issue(ra, 0);
            for (int c = 0; c < n_ch; c += 2) {
                if (c + 1 < n_ch) issue(rb, (c + 1) * CH);
                add(ra, c * CH);
                if (c + 2 < n_ch) issue(ra, (c + 2) * CH);
                if (c + 1 < n_ch) add(rb, (c + 1) * CH);
            }
            const uint32_t col = q * (HALF16 ? 2 : 1);
            if (!last) {
                nxt[col] = acc0;
                if constexpr (HALF16) nxt[col + 1] = acc1;
            } else {
                const size_t e = (size_t)t * a.d_out + col;
                if (a.y_kind == kElemF32) {
                    static_cast<float *>(a.y)[e] = acc0;
                    if constexpr (HALF16) static_cast<float *>(a.y)[e + 1] = acc1;
                } else {
                    static_cast<uint16_t *>(a.y)[e] = (uint16_t)narrow16(acc0, a.y_kind);
                    if constexpr (HALF16) static_cast<uint16_t *>(a.y)[e + 1] = (uint16_t)narrow16(acc1, a.y_kind);
                }
            }
        }
        __syncthreads();
    }
}

}  // namespace lffn
