// BH{m} hash of the LookupFFN forward pass for gfx950 (Sec. 3.2, eq. "block_acdc"):
//   z = x R,  R = prod_{i=1..m} B_i H,  B_i block-diagonal (blocks of 16, 32 or 64), H the
//   Walsh-Hadamard transform scaled by d_pad^(-1/2);  code_j = decimal(sign(z_j)) (Sec. 3.1).
//
// The block-diagonal step is a batch of small dense products over tokens -- the one part of the
// path that is a contraction -- and runs on the matrix cores: a wavefront owns 16 tokens and
// computes, per 16-coordinate output tile, (B^T x^T) with v_mfma_f32_16x16x4f32, tokens along the
// N dimension.  fp32 MFMA accumulates its four products as a chain of fused multiply-adds in
// ascending k, and chains of MFMAs extend that chain, so every output is the same
// "acc = fma(v_c, B[c][j], acc), c ascending from +0" sequence as a plain loop.
//
// Register layout (no data movement between the product and the transform).  A tile is 16
// coordinates x 16 tokens in 4 VGPRs: lane l = (token t = l % 16, group g = l / 16), register r
// holds coordinate 16*tile + g + 4*r.  This is the MFMA result layout with the output rows
// permuted (row 4g + r of the result carries coordinate g + 4r), and register kk of a tile is
// directly the B-operand of k-step kk (k-slot g = coordinate 4*kk + g): the result of one round
// feeds the next without a shuffle.  The matrices are pre-packed into that operand order.
// The transform's butterflies are (a + c, a - c) with a the lower coordinate, strides ascending:
// stride 1, 2 pair lanes l ^ 16, l ^ 32 (v_permlane16/32_swap), strides 4, 8 pair registers of a
// tile, strides >= 16 pair tiles.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "hash_kernel.hpp"

namespace lffn {

constexpr int kBhThreads = 256;
constexpr int kBhWaves = kBhThreads / 64;
constexpr int kBhTok = 16;  // tokens per wavefront

struct BhArgs {
    const void *x;        // [n][d] fp32 or bf16
    const float *apack;   // packed factors, see bh_pack_kernel
    uint16_t *codes;      // [n][k], or NULL when `packed` is written
    uint32_t *packed;     // packed codes of the staged gather, or NULL
    long long n_pad;
    long long n;
    int d, k, tau, n_factors, P;
    int x_bf16;
    float scale;
};

// words of LDS per wave: one bit string of P*N bits per token
__host__ __device__ inline int bh_bit_words(int P, int N) { return hash_bit_words(P, N); }
__host__ inline size_t bh_lds_bytes(int P, int N) { return sizeof(uint32_t) * (size_t)kBhWaves * kBhTok * bh_bit_words(P, N); }

// Packed factor layout: apack[p][f][o][ii][l][kk], o < N/16 output tiles, ii < b/16 input tiles of
// o's block, l < 64 lanes, kk < 4 k-steps; the element is
//   B_{p,f}[c][j],  c = 16*(first tile of the block + ii) + l/16 + 4*kk,
//                   j = 16*o + (l%16)/4 + 4*((l%16)%4)
// i.e. exactly the A-operand (row m = l%16, k-slot l/16) of the MFMA that adds input tile ii's
// k-step kk into output tile o.
__global__ __launch_bounds__(256) void bh_pack_kernel(const float *bmats, float *apack, int N, int b, long long total)
{
    const int tb = b / 16, nt = N / 16;
    for (long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x; idx < total;
         idx += (long long)gridDim.x * blockDim.x) {
        const int kk = (int)(idx & 3), l = (int)((idx >> 2) & 63);
        long long rest = idx >> 8;
        const int ii = (int)(rest % tb);
        rest /= tb;
        const int o = (int)(rest % nt);
        const long long pf = rest / nt;  // p * n_factors + f
        const int blk = (16 * o) / b;
        const int c = 16 * (blk * tb + ii) + l / 16 + 4 * kk;
        const int m = l % 16;
        const int j = 16 * o + (m >> 2) + 4 * (m & 3);
        apack[idx] = bmats[((pf * (N / b) + blk) * b + (c - blk * b)) * b + (j - blk * b)];
    }
}

typedef float mfma_f4 __attribute__((ext_vector_type(4)));

// LOG2N: d_pad = 2^LOG2N (64 .. 1024); TB = block / 16 (1, 2, 4)
template <int LOG2N, int TB>
__global__ __launch_bounds__(kBhThreads) void bh_hash_kernel(BhArgs a)
{
    constexpr int N = 1 << LOG2N;
    constexpr int NT = N / 16;  // tiles
    static_assert(NT >= TB && NT >= 4, "d_pad of at least 64 and at least one block");
    extern __shared__ uint32_t lds[];
    const unsigned lane = threadIdx.x & 63u;
    const unsigned wave = threadIdx.x >> 6;
    const unsigned tl = lane & 15u, g = lane >> 4;
    const int P = a.P;
    const int n_bitw = bh_bit_words(P, N);
    uint32_t *bits = lds + wave * (kBhTok * n_bitw);  // [16 tokens][n_bitw]

    const long long n_groups = (a.n + kBhTok - 1) / kBhTok;
    const long long gw = (long long)blockIdx.x * kBhWaves + wave;
    const long long n_waves = (long long)gridDim.x * kBhWaves;
    const float scale = a.scale;

    for (long long grp = gw; grp < n_groups; grp += n_waves) {
        const long long t = grp * kBhTok + tl;  // this lane's token
        const bool t_ok = t < a.n;
        for (int i = (int)lane; i < kBhTok * n_bitw; i += 64) bits[i] = 0;
        wave_lds_fence();

        for (int p = 0; p < P; ++p) {
            // ---- a1: this lane's coordinates of its token: tile beta, register r <-> 16*beta + g + 4r
            float v[NT][4];
#pragma unroll
            for (int beta = 0; beta < NT; ++beta)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int c = 16 * beta + (int)g + 4 * r;
                    float f = 0.0f;
                    if (t_ok && c < a.d) {
                        if (a.x_bf16)
                            f = __uint_as_float((uint32_t)((const uint16_t *)a.x)[t * a.d + c] << 16);
                        else
                            f = ((const float *)a.x)[t * a.d + c];
                    }
                    v[beta][r] = f;
                }

            for (int f = 0; f < a.n_factors; ++f) {
                // ---- block-diagonal factor on the matrix cores ---------------------------------
                const mfma_f4 *ap = reinterpret_cast<const mfma_f4 *>(a.apack) +
                                    ((size_t)(p * a.n_factors + f) * NT * TB) * 64 + lane;
#pragma unroll
                for (int blk = 0; blk < NT / TB; ++blk) {
                    mfma_f4 acc[TB];
#pragma unroll
                    for (int o = 0; o < TB; ++o) {
                        acc[o] = mfma_f4{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
                        for (int ii = 0; ii < TB; ++ii) {
                            const mfma_f4 am = ap[((blk * TB + o) * TB + ii) * 64];
#pragma unroll
                            for (int kk = 0; kk < 4; ++kk)
                                acc[o] = __builtin_amdgcn_mfma_f32_16x16x4f32(am[kk], v[blk * TB + ii][kk], acc[o], 0, 0, 0);
                        }
                    }
#pragma unroll
                    for (int o = 0; o < TB; ++o)
#pragma unroll
                        for (int r = 0; r < 4; ++r) v[blk * TB + o][r] = acc[o][r];
                }

                // ---- Walsh-Hadamard transform, ascending stride, then the scale -----------------
#pragma unroll
                for (int beta = 0; beta < NT; ++beta) {  // strides 1, 2: lanes l^16, l^32
                    swap_butterfly<16>(v[beta][0], v[beta][1]);
                    swap_butterfly<16>(v[beta][2], v[beta][3]);
                    swap_butterfly<32>(v[beta][0], v[beta][1]);
                    swap_butterfly<32>(v[beta][2], v[beta][3]);
                }
#pragma unroll
                for (int beta = 0; beta < NT; ++beta) {  // strides 4, 8: registers of a tile
#pragma unroll
                    for (int r = 0; r < 4; r += 2) {
                        const float x0 = v[beta][r], x1 = v[beta][r + 1];
                        v[beta][r] = x0 + x1;
                        v[beta][r + 1] = x0 - x1;
                    }
#pragma unroll
                    for (int r = 0; r < 2; ++r) {
                        const float x0 = v[beta][r], x1 = v[beta][r + 2];
                        v[beta][r] = x0 + x1;
                        v[beta][r + 2] = x0 - x1;
                    }
                }
#pragma unroll
                for (int h = 1; h < NT; h <<= 1)  // strides 16 and up: tiles
#pragma unroll
                    for (int beta = 0; beta < NT; ++beta)
                        if ((beta & h) == 0) {
#pragma unroll
                            for (int r = 0; r < 4; ++r) {
                                const float x0 = v[beta][r], x1 = v[beta + h][r];
                                v[beta][r] = x0 + x1;
                                v[beta + h][r] = x0 - x1;
                            }
                        }
#pragma unroll
                for (int beta = 0; beta < NT; ++beta)
#pragma unroll
                    for (int r = 0; r < 4; ++r) v[beta][r] = v[beta][r] * scale;
            }

            // ---- a4: sign bits into the tokens' bit strings: word w covers tiles 2w, 2w+1 --------
            uint32_t *row = bits + tl * n_bitw + p * (N / 32);
#pragma unroll
            for (int w = 0; w < NT / 2; ++w) {
                uint32_t m = 0;
#pragma unroll
                for (int hb = 0; hb < 2; ++hb)
#pragma unroll
                    for (int r = 0; r < 4; ++r) m |= (v[2 * w + hb][r] >= 0.0f ? 1u : 0u) << (16 * hb + 4 * r);
                atomicOr(&row[w], m << g);
            }
        }
        wave_lds_fence();

        // ---- codes: code j = bits [j*tau, (j+1)*tau) of the token's string, little-endian ------
        const uint32_t cmask = (1u << a.tau) - 1u;
        for (int tt = 0; tt < kBhTok; ++tt) {
            const long long tok = grp * kBhTok + tt;
            if (tok >= a.n) break;  // uniform
            const uint32_t *bw = bits + tt * n_bitw;
            auto code_at = [&](unsigned j) -> uint32_t {
                const unsigned bit = j * (unsigned)a.tau;
                const unsigned wi = bit >> 5, sh = bit & 31u;
                const unsigned long long both = ((unsigned long long)bw[wi + 1] << 32) | bw[wi];
                return (uint32_t)(both >> sh) & cmask;
            };
            if (a.packed) {
                for (int s = (int)lane; s < a.k / 2; s += 64)
                    a.packed[(long long)s * a.n_pad + tok] =
                        (code_at(2u * s) << kPackedShift) | (code_at(2u * s + 1u) << (16 + kPackedShift));
            } else {
                for (int j = (int)lane; j < a.k; j += 64) a.codes[tok * a.k + j] = (uint16_t)code_at((unsigned)j);
            }
        }
        wave_lds_fence();
    }

    // zero the token padding of the packed layout
    if (a.packed) {
        for (long long t = a.n + gw; t < a.n_pad; t += n_waves)
            for (int s = (int)lane; s < a.k / 2; s += 64) a.packed[(long long)s * a.n_pad + t] = 0u;
    }
}

}  // namespace lffn
