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

#include "gather_lds_kernel.hpp"
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
    float *weights;       // weighted variant: gather weights [n][k] (beside `codes`), or NULL
    float *wpk;           // weighted variant: the same table-major, [k][n_pad] (beside `packed`), or NULL
    int window;           // plain instantiation with `weights` / `wpk` set: the weights of a tau whose tables
                          // straddle tiles, formed from z through a window in LDS (see the kernel)
    long long n_pad;
    int packed_shift;     // log2 of the row-piece bytes the packed codes are scaled by
    long long n;
    int d, k, tau, n_factors, P;
    int x_kind;  // element type of x: 0 fp32, 1 bf16, 2 IEEE half
    int x_vec4;           // rows may be read four coordinates at a time (alignment checked by the host)
    float scale;
};

// The packed factors stream through LDS in chunks of up to 16 KB (16 tile products) shared by the
// four waves of a workgroup, through a ring of four buffers: a chunk is requested three chunks
// ahead of its use (a chunk of block-16 products is consumed in about 0.2 us, far less than a trip
// to L2), and the requests for the next factor travel while the transform runs.
constexpr int kBhChunkBytes = 16 * 1024;
constexpr int kBhRing = 4;
__host__ __device__ constexpr int bh_chunk_tiles(int N, int TB)
{
    // output tiles per chunk: 16 tile products = 16 / TB output tiles, at most the whole vector
    return 16 / TB < N / 16 ? 16 / TB : N / 16;
}
// words of LDS per wave: one bit string of P*N bits per token
__host__ __device__ inline int bh_bit_words(int P, int N) { return hash_bit_words(P, N); }
// z window of the weights of a tau other than 4, 8, 16: per wave, for each of its 16 tokens, kBhWinTail
// coordinates before the current run of kBhWin(N) coordinates and the run itself; an odd number of words per
// token spreads the tokens over the banks
constexpr int kBhWinTail = 16;
__host__ __device__ constexpr int kBhWin(int N) { return N < 128 ? N : 128; }
__host__ __device__ constexpr int bh_win_stride(int N) { return kBhWin(N) + kBhWinTail + 1; }
__host__ inline size_t bh_lds_bytes(int P, int N, bool window = false)
{
    return kBhRing * (size_t)kBhChunkBytes + sizeof(uint32_t) * (size_t)kBhWaves * kBhTok * bh_bit_words(P, N) +
           (window ? sizeof(float) * (size_t)kBhWaves * kBhTok * bh_win_stride(N) : 0);
}

// Packed factor layout: apack[p][f][o][ii][l][kk], o < N/16 output tiles, ii < b/16 input tiles of
// o's block, l < 64 lanes, kk < 4 k-steps; the element is
//   B_{p,f}[c][j],  c = 16*(first tile of the block + ii) + l/16 + 4*kk,
//                   j = 16*o + (l%16)/4 + 4*((l%16)%4)
// i.e. exactly the A-operand (row m = l%16, k-slot l/16) of the MFMA that adds input tile ii's
// k-step kk into output tile o.
#if !defined(LFFN_PART) || LFFN_PART == 0  // a plain function: defined by part 0 only of a build in parts
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
#endif

typedef float mfma_f4 __attribute__((ext_vector_type(4)));

// Transform stages inside one tile (strides 1, 2: lanes l ^ 16, l ^ 32; strides 4, 8: registers),
// ascending, each butterfly (a + c, a - c) with a the lower coordinate.
__device__ __forceinline__ void tile_stages(float (&t)[4])
{
    swap_butterfly<16>(t[0], t[1]);
    swap_butterfly<16>(t[2], t[3]);
    swap_butterfly<32>(t[0], t[1]);
    swap_butterfly<32>(t[2], t[3]);
#pragma unroll
    for (int r = 0; r < 4; r += 2) {
        const float x0 = t[r], x1 = t[r + 1];
        t[r] = x0 + x1;
        t[r + 1] = x0 - x1;
    }
#pragma unroll
    for (int r = 0; r < 2; ++r) {
        const float x0 = t[r], x1 = t[r + 2];
        t[r] = x0 + x1;
        t[r + 2] = x0 - x1;
    }
}

// Reduction over the four lane groups (rows of 16 lanes) of two registers at once: returns a register
// whose even rows hold op over all rows of x and whose odd rows hold op over all rows of y.
template <bool MUL>
__device__ __forceinline__ float reduce_rows(float x, float y)
{
    auto s = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(y), false, false);
    // s[0] = (x.r0, y.r0, x.r2, y.r2), s[1] = (x.r1, y.r1, x.r3, y.r3)
    const float c = MUL ? __uint_as_float(s[0]) * __uint_as_float(s[1]) : __uint_as_float(s[0]) + __uint_as_float(s[1]);
    auto t = __builtin_amdgcn_permlane32_swap(__float_as_uint(c), __float_as_uint(c), false, false);
    // t[0] = (c.r0, c.r1, c.r0, c.r1), t[1] = (c.r2, c.r3, c.r2, c.r3)
    return MUL ? __uint_as_float(t[0]) * __uint_as_float(t[1]) : __uint_as_float(t[0]) + __uint_as_float(t[1]);
}

// LOG2N: d_pad = 2^LOG2N (64 .. 1024); TB = block / 16 (1, 2, 4); VEC4: rows are read four coordinates
// at a time (d % 4 == 0, aligned rows), else one by one; WEIGHTED: also the gather weights of the
// weighted variant (Sec. 4), for tau = 4, 8 or 16 (a table then lies inside one tile).
template <int LOG2N, int TB, bool VEC4, bool WEIGHTED = false>
__global__ __launch_bounds__(kBhThreads) void bh_hash_kernel(BhArgs a)
{
    constexpr int N = 1 << LOG2N;
    constexpr int NT = N / 16;                  // tiles
    constexpr int CT = bh_chunk_tiles(N, TB);   // output tiles per chunk
    constexpr int NCH = NT / CT;                // chunks per factor
    constexpr int CQ = CT * TB;                 // tile products (1 KB of operands each) per chunk
    static_assert(NT >= TB && NT >= 4 && NT % CT == 0 && CT % TB == 0, "chunks hold whole blocks");
    static_assert(CQ * 1024 <= kBhChunkBytes, "a chunk fits its buffer");
    extern __shared__ uint32_t lds[];
    const unsigned lane = threadIdx.x & 63u;
    const unsigned wave = threadIdx.x >> 6;
    const unsigned tl = lane & 15u, g = lane >> 4;
    const int P = a.P;
    const int n_bitw = bh_bit_words(P, N);
    const uint32_t lds0 = (uint32_t)(uintptr_t)lds;            // the two operand buffers
    uint32_t *bits = lds + kBhRing * (kBhChunkBytes / 4) + wave * (kBhTok * n_bitw);  // [16 tokens][n_bitw]

    const long long n_groups = (a.n + kBhTok - 1) / kBhTok;
    const long long gw = (long long)blockIdx.x * kBhWaves + wave;
    const long long n_waves = (long long)gridDim.x * kBhWaves;
    const long long iters = (n_groups + n_waves - 1) / n_waves;  // the same for every wave: the loop has barriers
    const float scale = a.scale;

    // Operand stream: chunk id (p * n_factors + f) * NCH + c is CQ KB at apack + id * CQ KB; every
    // thread copies 16 bytes per 4 KB.  The stream is cyclic (the next token group starts over); the
    // chunk with sequence number `seq` sits in ring buffer seq % kBhRing.
    const uint32_t n_chunks = (uint32_t)(P * a.n_factors * NCH);
    constexpr int kCopies = CQ / 4;  // copy instructions per thread and chunk
    auto copy_chunk = [&](uint32_t id, uint32_t buf) {
        const char *src = reinterpret_cast<const char *>(a.apack) + (size_t)id * (CQ * 1024);  // uniform
#pragma unroll
        for (int i = 0; i < kCopies; ++i)
            lds_dma16(src + i * 4096, threadIdx.x * 16u, lds0 + buf * kBhChunkBytes + i * 4096 + wave * 1024u);
    };
    uint32_t seq = 0;      // sequence number of the chunk consumed next
    uint32_t next_id = 0;  // id of the chunk requested next (sequence number seq + kBhRing - 1 once primed)
#pragma unroll
    for (int i = 0; i < kBhRing - 1; ++i) {
        copy_chunk(next_id, (uint32_t)i);
        next_id = next_id + 1 < n_chunks ? next_id + 1 : 0u;
    }

    for (long long it = 0; it < iters; ++it) {
        const long long grp = gw + it * n_waves;
        const long long t = grp * kBhTok + tl;  // this lane's token
        const bool t_ok = t < a.n;
        for (int i = (int)lane; i < kBhTok * n_bitw; i += 64) bits[i] = 0;
        wave_lds_fence();

        for (int p = 0; p < P; ++p) {
            // ---- a1: this lane's coordinates of its token: tile beta, register r <-> 16*beta + g + 4r
            float v[NT][4];
            const long long tc = t_ok ? t : a.n - 1;  // idle token lanes read the last token and zero it
            if constexpr (VEC4) {
                // rows start on 16-byte (fp32) / 8-byte (bf16) boundaries and d % 4 == 0: the lane loads
                // coordinates 16*beta + 4g .. + 3 in one piece (one base address per lane, the tile is an
                // immediate offset; tiles wholly inside or outside the row are told apart by uniform
                // branches), then a 4 x 4 transpose between lane groups and registers (two rounds of
                // lane-row swaps) gives the layout above
                const char *xrow = reinterpret_cast<const char *>(a.x) + (tc * a.d + 4 * (long long)g) * (a.x_kind ? 2 : 4);
                auto piece = [&](int beta) -> float4 {
                    if (a.x_kind) {
                        const uint2 w = *reinterpret_cast<const uint2 *>(xrow + beta * 32);
                        const float2 lo = widen16x2(w.x, a.x_kind), hi = widen16x2(w.y, a.x_kind);
                        return make_float4(lo.x, lo.y, hi.x, hi.y);
                    }
                    return *reinterpret_cast<const float4 *>(xrow + beta * 64);
                };
#pragma unroll
                for (int beta = 0; beta < NT; ++beta) {
                    float4 f = make_float4(0.f, 0.f, 0.f, 0.f);
                    if (16 * beta + 16 <= a.d) {
                        f = piece(beta);
                    } else if (16 * beta < a.d) {
                        if (16 * beta + 4 * (int)g < a.d) f = piece(beta);
                    }
                    uint32_t e0 = t_ok ? __float_as_uint(f.x) : 0u, e1 = t_ok ? __float_as_uint(f.y) : 0u,
                             e2 = t_ok ? __float_as_uint(f.z) : 0u, e3 = t_ok ? __float_as_uint(f.w) : 0u;
                    // rows of 16 lanes = lane groups; swap16 exchanges (first, odd rows) with (second, even rows)
                    auto s01 = __builtin_amdgcn_permlane16_swap(e0, e1, false, false);
                    auto s23 = __builtin_amdgcn_permlane16_swap(e2, e3, false, false);
                    // swap32 exchanges (first, upper half) with (second, lower half)
                    auto s02 = __builtin_amdgcn_permlane32_swap(s01[0], s23[0], false, false);
                    auto s13 = __builtin_amdgcn_permlane32_swap(s01[1], s23[1], false, false);
                    v[beta][0] = __uint_as_float(s02[0]);
                    v[beta][1] = __uint_as_float(s13[0]);
                    v[beta][2] = __uint_as_float(s02[1]);
                    v[beta][3] = __uint_as_float(s13[1]);
                }
            } else {
#pragma unroll
                for (int beta = 0; beta < NT; ++beta)
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const int c = 16 * beta + (int)g + 4 * r;
                        float f = 0.0f;
                        if (t_ok && c < a.d) {
                            if (a.x_kind)
                                f = widen16(((const uint16_t *)a.x)[t * a.d + c], a.x_kind);
                            else
                                f = ((const float *)a.x)[t * a.d + c];
                        }
                        v[beta][r] = f;
                    }
            }

            for (int f = 0; f < a.n_factors; ++f) {
                // ---- block-diagonal factor on the matrix cores ---------------------------------
#pragma unroll
                for (int c = 0; c < NCH; ++c) {
                    // This chunk is complete once every wave's copies of it have landed: vector-memory
                    // operations retire in order, so all but the newest 2 * kCopies (the two chunks
                    // requested after it) must be done.  The barrier also frees the buffer of the
                    // previous chunk for the next request.
                    static_assert(kBhRing == 4 && 2 * kCopies <= 8, "wait count below");
                    if constexpr (kCopies == 4) __builtin_amdgcn_s_waitcnt(0x0F70 | 8);       // vmcnt(8)
                    else if constexpr (kCopies == 2) __builtin_amdgcn_s_waitcnt(0x0F70 | 4);  // vmcnt(4)
                    else __builtin_amdgcn_s_waitcnt(0x0F70 | 2);                               // vmcnt(2)
                    __syncthreads();
                    const uint32_t buf = seq % kBhRing;
                    copy_chunk(next_id, (seq + kBhRing - 1) % kBhRing);
                    next_id = next_id + 1 < n_chunks ? next_id + 1 : 0u;
                    const uint32_t abase = lds0 + buf * kBhChunkBytes + lane * 16u;
                    // operand quads of the chunk in order ((block, output tile, input tile)); the read of
                    // quad i+1 is issued before the four MFMAs of quad i so that it overlaps them
                    auto ld_quad = [&](int qi) -> u32x4 {
                        return *reinterpret_cast<const __attribute__((address_space(3))) u32x4 *>(
                            (uintptr_t)(abase + (uint32_t)(qi * 1024)));
                    };
                    u32x4 aw = ld_quad(0);
#pragma unroll
                    for (int blk = 0; blk < CT / TB; ++blk) {
                        mfma_f4 acc[TB];
#pragma unroll
                        for (int o = 0; o < TB; ++o) {
                            acc[o] = mfma_f4{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
                            for (int ii = 0; ii < TB; ++ii) {
                                const int qi = (blk * TB + o) * TB + ii;
                                const u32x4 cur = aw;
                                if (qi + 1 < CQ) aw = ld_quad(qi + 1);
                                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                                for (int kk = 0; kk < 4; ++kk)
                                    acc[o] = __builtin_amdgcn_mfma_f32_16x16x4f32(
                                        __uint_as_float(cur[kk]), v[c * CT + blk * TB + ii][kk], acc[o], 0, 0, 0);
                                // In the shadow of these MFMAs: the tile-local transform stages (strides
                                // 1 .. 8) of one tile of the previous chunk, whose products are complete.
                                if (c > 0 && qi % TB == 0) {
                                    tile_stages(v[(c - 1) * CT + qi / TB]);
#pragma unroll
                                    for (int kk = 0; kk < 4; ++kk) {
                                        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // one MFMA
                                        __builtin_amdgcn_sched_group_barrier(0x002, 6, 0);  // six vector-ALU ops
                                    }
                                }
                                __builtin_amdgcn_sched_barrier(0);
                            }
                        }
#pragma unroll
                        for (int o = 0; o < TB; ++o)
#pragma unroll
                            for (int r = 0; r < 4; ++r) v[c * CT + blk * TB + o][r] = acc[o][r];
                    }
                    ++seq;
                }

                // ---- Walsh-Hadamard transform, ascending stride, then the scale -----------------
                // strides 1 .. 8 of the last chunk's tiles (the other tiles had theirs during the products)
#pragma unroll
                for (int beta = (NCH - 1) * CT; beta < NT; ++beta) tile_stages(v[beta]);
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

            // ---- weighted variant: w_j = |z_j|_1 / prod_b (1 + exp(-2|z_jb|)) (Sec. 4) --------------
            // A tile holds coordinate g + 4r of its 16 in (lane group g, register r): a table of
            // tau = 4 is one register over the four lane groups, tau = 8 two registers, tau = 16 the
            // whole tile.  Four consecutive tables 4q .. 4q+3 of the projection are reduced together
            // (two pair reductions, one per half of the lane groups) so that lane group g ends with
            // the weight of table 4q + g: one store per lane for four tables.  All weights of a chunk
            // of tables are computed first (straight-line code), then stored.
            if constexpr (WEIGHTED) {
                auto emit = [&](auto tau_c) {
                    constexpr int TAU = decltype(tau_c)::value;
                    constexpr int TPQ = TAU / 4;           // tiles per group of four tables (1, 2, 4)
                    constexpr int NQ = NT / TPQ;           // groups of four tables in the projection
                    constexpr int QC = NQ < 32 ? NQ : 32;  // groups computed before their stores
                    const int jb = p * (N / TAU) + (int)g;  // this lane's table in group 0
                    auto az = [&](int beta, int r) { return __builtin_fabsf(v[beta][r]); };
                    auto ez = [&](int beta, int r) {        // 1 + exp(-2|z|)
                        return 1.0f + __builtin_amdgcn_exp2f(__builtin_fabsf(v[beta][r]) * -2.885390082f);
                    };
#pragma unroll
                    for (int q0 = 0; q0 < NQ; q0 += QC) {
                        float res[QC];
#pragma unroll
                        for (int qi = 0; qi < QC; ++qi) {
                            const int q = q0 + qi;
                            float sx[2], sy[2], px[2], py[2];  // [half]: tables 4q + 2*half (x) and + 1 (y)
#pragma unroll
                            for (int h = 0; h < 2; ++h) {
                                if constexpr (TAU == 4) {
                                    sx[h] = az(q, 2 * h);
                                    px[h] = ez(q, 2 * h);
                                    sy[h] = az(q, 2 * h + 1);
                                    py[h] = ez(q, 2 * h + 1);
                                } else if constexpr (TAU == 8) {
                                    const int beta = 2 * q + h;
                                    sx[h] = az(beta, 0) + az(beta, 1);
                                    px[h] = ez(beta, 0) * ez(beta, 1);
                                    sy[h] = az(beta, 2) + az(beta, 3);
                                    py[h] = ez(beta, 2) * ez(beta, 3);
                                } else {
                                    const int bx = 4 * q + 2 * h, by = bx + 1;
                                    sx[h] = (az(bx, 0) + az(bx, 1)) + (az(bx, 2) + az(bx, 3));
                                    px[h] = (ez(bx, 0) * ez(bx, 1)) * (ez(bx, 2) * ez(bx, 3));
                                    sy[h] = (az(by, 0) + az(by, 1)) + (az(by, 2) + az(by, 3));
                                    py[h] = (ez(by, 0) * ez(by, 1)) * (ez(by, 2) * ez(by, 3));
                                }
                            }
                            // even lane groups get x's total, odd ones y's; groups 0, 1 keep half 0
                            const float s0 = reduce_rows<false>(sx[0], sy[0]), s1 = reduce_rows<false>(sx[1], sy[1]);
                            const float p0 = reduce_rows<true>(px[0], py[0]), p1 = reduce_rows<true>(px[1], py[1]);
                            res[qi] = (g < 2 ? s0 : s1) * __builtin_amdgcn_rcpf(g < 2 ? p0 : p1);
                        }
                        if (a.wpk) {
                            // table-major: the 16 tokens of a lane group are consecutive
                            float *wp = a.wpk + wpk_index(jb + 4 * q0, t, a.n_pad);
#pragma unroll
                            for (int qi = 0; qi < QC; ++qi) {
                                if (t_ok && jb + 4 * (q0 + qi) < a.k) *wp = res[qi];
                                wp += 4 * a.n_pad;
                            }
                        } else {
                            float *wq = a.weights + t * a.k + jb + 4 * q0;
#pragma unroll
                            for (int qi = 0; qi < QC; ++qi)
                                if (t_ok && jb + 4 * (q0 + qi) < a.k) wq[4 * qi] = res[qi];
                        }
                    }
                };
                if (a.tau == 8)
                    emit(std::integral_constant<int, 8>{});
                else if (a.tau == 16)
                    emit(std::integral_constant<int, 16>{});
                else
                    emit(std::integral_constant<int, 4>{});
            }

            // ---- weighted variant for any other tau: a table then straddles tiles (and may run from one
            // projection into the next), so z goes through a window in LDS, kBhWin coordinates of all 16 tokens at
            // a time; the lanes take a (token, table) pair each and form the same sum and product coordinate
            // by coordinate.  A table is handled in the run that holds its last coordinate; the 16 coordinates
            // before a run are kept (across projections too).  Register r of tile beta is coordinate
            // 16*beta + g + 4r.
            if constexpr (!WEIGHTED) {
                if (a.window) {
                    constexpr int QW = kBhWin(N), QT = QW / 16, ZS = bh_win_stride(N);
                    float *zw = reinterpret_cast<float *>(lds + kBhRing * (kBhChunkBytes / 4) + kBhWaves * (kBhTok * n_bitw)) +
                                wave * (kBhTok * ZS);
                    const int tau = a.tau;
#pragma unroll
                    for (int q0 = 0; q0 < NT; q0 += QT) {
                        wave_lds_fence();
                        {
                            float *zt = zw + tl * ZS + kBhWinTail + g;
#pragma unroll
                            for (int b = 0; b < QT; ++b)
#pragma unroll
                                for (int r = 0; r < 4; ++r) zt[16 * b + 4 * r] = v[q0 + b][r];
                        }
                        wave_lds_fence();
                        const long long lo = (long long)p * N + 16 * q0;  // first coordinate of the run in the bit string
                        const int jlo = (int)(lo / tau);
                        long long jhi = (lo + QW) / tau;
                        if (jhi > a.k) jhi = a.k;
                        const int ntab = (int)jhi - jlo;
                        for (int idx = (int)lane; idx < kBhTok * ntab; idx += 64) {
                            // table-major output: the 16 tokens of a table are neighbours; else a token's tables are
                            const int tt = a.wpk ? (idx & 15) : idx / ntab;
                            const int j = jlo + (a.wpk ? (idx >> 4) : idx - tt * ntab);
                            const long long tok = grp * kBhTok + tt;
                            const float *zz = zw + tt * ZS + kBhWinTail + (int)((long long)j * tau - lo);  // may start in the tail
                            float sum = 0.0f, q = 1.0f;
                            for (int b = 0; b < tau; ++b) {
                                const float az = __builtin_fabsf(zz[b]);
                                sum += az;
                                q *= 1.0f + __builtin_amdgcn_exp2f(az * -2.885390082f);  // exp(-2 az) = 2^(-2 az log2 e)
                            }
                            const float w = sum * __builtin_amdgcn_rcpf(q);  // q >= 1
                            if (tok < a.n) {
                                if (a.wpk) a.wpk[wpk_index(j, tok, a.n_pad)] = w;
                                else a.weights[tok * a.k + j] = w;
                            }
                        }
                        // the run's last 16 coordinates become the tail of the next run: 16 tokens x 16 words
                        wave_lds_fence();
                        float keep[4];
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            const int e = (int)lane + 64 * i;  // token e / 16, word e % 16
                            keep[i] = zw[(e >> 4) * ZS + kBhWinTail + QW - kBhWinTail + (e & 15)];
                        }
                        wave_lds_fence();
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            const int e = (int)lane + 64 * i;
                            zw[(e >> 4) * ZS + (e & 15)] = keep[i];
                        }
                    }
                    wave_lds_fence();
                }
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
                        (code_at(2u * s) << a.packed_shift) | (code_at(2u * s + 1u) << (16 + a.packed_shift));
            } else {
                for (int j = (int)lane; j < a.k; j += 64) a.codes[tok * a.k + j] = (uint16_t)code_at((unsigned)j);
            }
        }
        wave_lds_fence();
    }

    __builtin_amdgcn_s_waitcnt(0x0F70);  // the last requested chunks are never used: let them land before the wave ends

    // zero the token padding of the packed layout
    if (a.packed) {
        for (long long t = a.n + gw; t < a.n_pad; t += n_waves)
            for (int s = (int)lane; s < a.k / 2; s += 64) a.packed[(long long)s * a.n_pad + t] = 0u;
    }
}

}  // namespace lffn
