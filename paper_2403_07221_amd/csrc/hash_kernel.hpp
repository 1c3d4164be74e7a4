// Hash step of the LookupFFN forward pass for gfx950 (wave64):
//   z = x R,  R = D_1 H D_2 H ... (Sec. 3.2, eq. "hadamard"), code_j = decimal(sign(z_j)) (Sec. 3.1).
//
// One wavefront owns one token at a time.  Coordinate i of the padded vector
// lives in lane (i % 64), register (i / 64), so the Walsh-Hadamard butterflies
// of stride 1..32 are cross-lane exchanges (DPP for 1, 2, 4, 8; the gfx950
// v_permlane16_swap / v_permlane32_swap for 16, 32) and those of stride >= 64
// are plain register pairs.  Stages run in ascending stride and every
// butterfly is (a + c, a - c) with a the lower index, in fp32 without
// contraction, so each coordinate goes through the same sequence of roundings
// as the textbook in-place loop and the sign bits come out identical.
//
// Sign bits: `v >= 0` per register is a 64-bit lane mask, i.e. 64 consecutive
// bits of the token's bit string; the masks go to a small per-wave LDS array
// and lane j then cuts code j = bits [j*tau, (j+1)*tau) out of it.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "elem16.hpp"

namespace lffn {

// Layout of the gather kernels' internal "packed" codes (the scratch buffer of the forward
// pass when the LDS-staged gather is used): packed[s][t], s < k/2, t < n_pad, one 32-bit word
// holding the LDS byte offsets (code << 7, i.e. code * 128-byte row pieces) of tables 2s (low
// half) and 2s+1 (high half).  The token axis is padded so that a workgroup may read a full
// 16 x 256 token window past any token without leaving the buffer; padding entries are zero.
__host__ __device__ inline long long packed_n_pad(long long n) { return ((n + 127) / 128) * 128 + 16 * 256; }
constexpr int kPackedShift = 7;
// index of (table j, token t) in the staged gather's weight array: table-major, token-contiguous
__host__ __device__ inline long long wpk_index(long long j, long long t, long long n_pad)
{
    return j * n_pad + t;  // [k][n_pad]
}

struct HashArgs {
    const void *x;        // [n][d] fp32 or bf16
    const int8_t *signs;  // [P][R][N]
    uint16_t *codes;      // [n][k], or NULL when `packed` is written instead
    uint32_t *packed;     // packed codes (see above), or NULL
    float *weights;       // [n][k] gather weights of the weighted variant (Sec. 4), or NULL
    float *wpk;           // the same weights table-major, [k][n_pad], for the LDS-staged gather, or NULL
    long long n_pad;      // token stride of `packed`
    int packed_shift;     // log2 of the row-piece bytes the packed codes are scaled by (7: 128-byte pieces, 6: 64-byte)
    long long n;
    int d, k, tau, n_rounds, P;
    int x_kind;           // element type of x: 0 fp32, 1 bf16, 2 IEEE half
    float scale;          // (float)(1 / sqrt(N))
};

constexpr int kHashThreads = 256;
constexpr int kHashWaves = kHashThreads / 64;

// words of LDS one wave needs for a token's bit string (P*N bits, one spare word, even count)
__host__ __device__ inline int hash_bit_words(int P, int N)
{
    int w = (P * N + 31) / 32 + 1;
    return (w + 1) & ~1;
}
// 32-bit flip words per (projection, round, lane): bit r = "negate register r"
__host__ __device__ inline int hash_flip_words(int N) { return N > 2048 ? 2 : 1; }

// Weighted variant: a wave keeps the soft codes z of the current projection (N words) behind a
// 16-word tail holding the last 16 coordinates of the projections before it, so that a table
// whose tau <= 16 coordinates straddle a projection boundary is read from one window.
constexpr int kZTail = 16;
__host__ __device__ inline int hash_z_words(int N, bool weighted) { return weighted ? N + kZTail : 0; }

__host__ inline size_t hash_lds_bytes(int P, int R, int N, bool weighted = false)
{
    return sizeof(uint32_t) * ((size_t)P * R * hash_flip_words(N) * 64 +
                               (size_t)kHashWaves * (hash_bit_words(P, N) + hash_z_words(N, weighted)));
}

__device__ __forceinline__ float fxor(float v, uint32_t m) { return __uint_as_float(__float_as_uint(v) ^ m); }

// value of `v` in lane (lane ^ H), H in {1, 2, 4, 8}, by DPP
template <int H>
__device__ __forceinline__ float dpp_xor(float v)
{
    int i = __float_as_int(v);
    if constexpr (H == 1) i = __builtin_amdgcn_update_dpp(0, i, 0xB1, 0xF, 0xF, true);        // quad_perm [1,0,3,2]
    else if constexpr (H == 2) i = __builtin_amdgcn_update_dpp(0, i, 0x4E, 0xF, 0xF, true);   // quad_perm [2,3,0,1]
    else if constexpr (H == 4) {
        i = __builtin_amdgcn_update_dpp(0, i, 0x141, 0xF, 0xF, true);                         // row_half_mirror: l -> l^7
        i = __builtin_amdgcn_update_dpp(0, i, 0x1B, 0xF, 0xF, true);                          // quad_perm [3,2,1,0]: l -> l^3
    } else {
        static_assert(H == 8, "DPP exchange covers strides 1, 2, 4, 8");
        i = __builtin_amdgcn_update_dpp(0, i, 0x128, 0xF, 0xF, true);                         // row_ror:8: l -> l^8
    }
    return __int_as_float(i);
}

// butterfly of stride H (16 or 32 lanes) on two registers at once:
// swap halves, add/sub, swap back -- no per-lane sign fix-up needed.
template <int H>
__device__ __forceinline__ void swap_butterfly(float &a, float &b)
{
    uint32_t ua = __float_as_uint(a), ub = __float_as_uint(b);
    float lo, hi;
    if constexpr (H == 16) {
        auto s = __builtin_amdgcn_permlane16_swap(ua, ub, false, false);
        lo = __uint_as_float(s[0]);
        hi = __uint_as_float(s[1]);
    } else {
        auto s = __builtin_amdgcn_permlane32_swap(ua, ub, false, false);
        lo = __uint_as_float(s[0]);
        hi = __uint_as_float(s[1]);
    }
    const float sum = lo + hi, dif = lo - hi;
    if constexpr (H == 16) {
        auto s = __builtin_amdgcn_permlane16_swap(__float_as_uint(sum), __float_as_uint(dif), false, false);
        a = __uint_as_float(s[0]);
        b = __uint_as_float(s[1]);
    } else {
        auto s = __builtin_amdgcn_permlane32_swap(__float_as_uint(sum), __float_as_uint(dif), false, false);
        a = __uint_as_float(s[0]);
        b = __uint_as_float(s[1]);
    }
}

// one cross-lane stage (stride H < 64) on every register
template <int H, int NREG>
__device__ __forceinline__ void lane_stage(float (&v)[NREG], unsigned lane)
{
    if constexpr ((H == 16 || H == 32) && NREG >= 2) {
#pragma unroll
        for (int r = 0; r < NREG; r += 2) swap_butterfly<H>(v[r], v[r + 1]);
    } else if constexpr (H == 16 || H == 32) {
        const uint32_t m = (lane & H) ? 0x80000000u : 0u;
        const int src = (int)((lane ^ H) << 2);
#pragma unroll
        for (int r = 0; r < NREG; ++r) {
            const float p = __int_as_float(__builtin_amdgcn_ds_bpermute(src, __float_as_int(v[r])));
            v[r] = p + fxor(v[r], m);
        }
    } else {
        // lower lane: self + partner; upper lane: partner - self  (= a - c with a the lower index)
        const uint32_t m = (lane & H) ? 0x80000000u : 0u;
#pragma unroll
        for (int r = 0; r < NREG; ++r) v[r] = dpp_xor<H>(v[r]) + fxor(v[r], m);
    }
}

// one in-register stage: register stride HH = stride / 64
template <int HH, int NREG>
__device__ __forceinline__ void reg_stage(float (&v)[NREG])
{
#pragma unroll
    for (int r = 0; r < NREG; ++r) {
        if ((r & HH) == 0) {
            const float a = v[r], c = v[r + HH];
            v[r] = a + c;
            v[r + HH] = a - c;
        }
    }
}

// unnormalised transform of N = 2^LOG2N coordinates, ascending stride
template <int LOG2N, int NREG>
__device__ __forceinline__ void fwht_wave(float (&v)[NREG], unsigned lane)
{
    if constexpr (LOG2N > 0) lane_stage<1, NREG>(v, lane);
    if constexpr (LOG2N > 1) lane_stage<2, NREG>(v, lane);
    if constexpr (LOG2N > 2) lane_stage<4, NREG>(v, lane);
    if constexpr (LOG2N > 3) lane_stage<8, NREG>(v, lane);
    if constexpr (LOG2N > 4) lane_stage<16, NREG>(v, lane);
    if constexpr (LOG2N > 5) lane_stage<32, NREG>(v, lane);
    if constexpr (LOG2N > 6) reg_stage<1, NREG>(v);
    if constexpr (LOG2N > 7) reg_stage<2, NREG>(v);
    if constexpr (LOG2N > 8) reg_stage<4, NREG>(v);
    if constexpr (LOG2N > 9) reg_stage<8, NREG>(v);
    if constexpr (LOG2N > 10) reg_stage<16, NREG>(v);
    if constexpr (LOG2N > 11) reg_stage<32, NREG>(v);
}

__device__ __forceinline__ void wave_lds_fence()
{
    // LDS operations of one wave complete in issue order; this only stops the compiler
    // from moving LDS accesses across the point.
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Gather weights of the tables whose last coordinate lies in projection p (Sec. 4, the weighted
// variant used in the paper's experiments): with S_g the sign row that the code selects,
//   w_j = <z_j, S_g> exp(<z_j, S_g>) / prod_b (exp(z_jb) + exp(-z_jb))
//       = |z_j|_1 / prod_b (1 + exp(-2 |z_jb|)),
// the second form being the first with numerator and denominator divided by exp(|z_j|_1); it
// cannot overflow.  `z_at(c)` returns coordinate c of projection p for 0 <= c < N and coordinate
// N + c of the concatenation before it for -16 < c < 0.  One lane per table.
// WMODE 1: the weight above; WMODE 2: the multi-probe shares (below), written to `weights` as
// [n][k][1+tau].  The mode is a template parameter of the kernels, so each variant is its own binary.
template <int WMODE, class ZAt>
__device__ __forceinline__ void emit_weights(const HashArgs &a, long long t, int p, int N, unsigned lane, ZAt z_at)
{
    const int tau = a.tau;
    const long long lo = (long long)p * N;
    const int jlo = (int)(lo / tau);
    long long jhi = (lo + N) / tau;
    if (jhi > a.k) jhi = a.k;
    if constexpr (WMODE == 2) {
        // Multi-probe shares (Sec. 3.1, eq. "partial_softmax", rows within one sign flip of sign(z_j)):
        // the selected row's soft-max share is prod_b sigmoid(2|z_jb|) = 1 / prod_b (1 + e_b) with
        // e_b = exp(-2|z_jb|), and flipping bit b multiplies it by e_b.
        for (int j = jlo + (int)lane; j < (int)jhi; j += 64) {
            const int c0 = (int)((long long)j * tau - lo);
            float q = 1.0f;
            for (int b = 0; b < tau; ++b)
                q *= 1.0f + __builtin_amdgcn_exp2f(__builtin_fabsf(z_at(c0 + b)) * -2.885390082f);
            const float p0 = __fdividef(1.0f, q);
            float *out = a.weights + (t * a.k + j) * (tau + 1);
            out[0] = p0;
            for (int b = 0; b < tau; ++b)
                out[1 + b] = p0 * __builtin_amdgcn_exp2f(__builtin_fabsf(z_at(c0 + b)) * -2.885390082f);
        }
        return;
    }
    for (int j = jlo + (int)lane; j < (int)jhi; j += 64) {
        const int c0 = (int)((long long)j * tau - lo);
        float s = 0.0f, q = 1.0f;
        for (int b = 0; b < tau; ++b) {
            const float az = __builtin_fabsf(z_at(c0 + b));
            s += az;
            q *= 1.0f + __builtin_amdgcn_exp2f(az * -2.885390082f);  // exp(-2 az) = 2^(-2 az log2 e)
        }
        const float w = __fdividef(s, q);
        if (a.wpk)
            a.wpk[wpk_index(j, t, a.n_pad)] = w;
        else
            a.weights[t * a.k + j] = w;
    }
}

// WMODE: 0 = codes only, 1 = codes and gather weights (Sec. 4), 2 = codes and multi-probe shares
template <int LOG2N, int WMODE>
__global__ __launch_bounds__(kHashThreads) void hash_kernel(HashArgs a)
{
    constexpr bool WEIGHTED = WMODE != 0;
    constexpr int N = 1 << LOG2N;
    constexpr int NREG = N >= 64 ? N / 64 : 1;
    constexpr int FW = N > 2048 ? 2 : 1;
    extern __shared__ uint32_t lds[];

    const unsigned tid = threadIdx.x;
    const unsigned lane = tid & 63u;
    const unsigned wave = tid >> 6;
    const int P = a.P, R = a.n_rounds;

    // ---- block prologue: pack the sign diagonals into per-lane flip words ----------------
    // flip[(p*R + r)*FW + w][lane] bit b  <->  signs[p][r][lane + 64*(32*w + b)] < 0
    uint32_t *flip = lds;
    const int n_flip = P * R * FW * 64;
    for (int idx = (int)tid; idx < n_flip; idx += kHashThreads) {
        const int l = idx & 63;
        const int w = (idx >> 6) % FW;
        const int pr = (idx >> 6) / FW;
        const int8_t *D = a.signs + (size_t)pr * N;
        uint32_t bits = 0;
#pragma unroll 4
        for (int b = 0; b < 32; ++b) {
            const int i = l + 64 * (32 * w + b);
            if (i < N && D[i] < 0) bits |= 1u << b;
        }
        flip[idx] = bits;
    }
    const int n_bitw = hash_bit_words(P, N);
    uint32_t *bitw = lds + n_flip + wave * (n_bitw + hash_z_words(N, WEIGHTED));
    float *zwin = reinterpret_cast<float *>(bitw + n_bitw);  // [kZTail tail][N current projection]
    for (int i = (int)lane; i < n_bitw; i += 64) bitw[i] = 0;
    __syncthreads();

    const long long wave0 = (long long)blockIdx.x * kHashWaves + wave;
    const long long n_waves = (long long)gridDim.x * kHashWaves;
    const float scale = a.scale;

    for (long long t = wave0; t < a.n; t += n_waves) {
        // ---- a1: load the token's row, widen, zero-pad ----------------------------------
        float xv[NREG];
#pragma unroll
        for (int r = 0; r < NREG; ++r) {
            const int i = (int)lane + 64 * r;
            float f = 0.0f;
            if (i < a.d) {
                if (a.x_kind)
                    f = widen16(((const uint16_t *)a.x)[t * a.d + i], a.x_kind);
                else
                    f = ((const float *)a.x)[t * a.d + i];
            }
            xv[r] = f;
        }

        if constexpr (N < 64) {
            wave_lds_fence();
            for (int i = (int)lane; i < n_bitw; i += 64) bitw[i] = 0;
        }

        for (int p = 0; p < P; ++p) {
            float v[NREG];
#pragma unroll
            for (int r = 0; r < NREG; ++r) v[r] = xv[r];

            for (int rd = 0; rd < R; ++rd) {
                // ---- a2: sign diagonal ---------------------------------------------------
                const uint32_t *fw = flip + ((p * R + rd) * FW) * 64 + lane;
                const uint32_t w0 = fw[0];
                uint32_t w1 = 0;
                if constexpr (FW == 2) w1 = fw[64];
#pragma unroll
                for (int r = 0; r < NREG; ++r) {
                    const uint32_t w = r < 32 ? w0 : w1;
                    v[r] = fxor(v[r], ((w >> (r & 31)) & 1u) << 31);
                }
                // ---- a3: Walsh-Hadamard transform, then the d_pad^(-1/2) scale -----------
                fwht_wave<LOG2N, NREG>(v, lane);
#pragma unroll
                for (int r = 0; r < NREG; ++r) v[r] = v[r] * scale;
            }

            // ---- a4: sign bits of this projection into the wave's bit string ------------
            if constexpr (N >= 64) {
                // the mask of register r is bits [64r, 64r+64) of this projection; lane 0 stores them
                unsigned long long m[NREG];
#pragma unroll
                for (int r = 0; r < NREG; ++r) m[r] = __builtin_amdgcn_ballot_w64(v[r] >= 0.0f);
                if (lane == 0) {
                    unsigned long long *dst = reinterpret_cast<unsigned long long *>(bitw) + p * (N / 64);
#pragma unroll
                    for (int r = 0; r < NREG; ++r) dst[r] = m[r];
                }
            } else {
                const unsigned long long m = __builtin_amdgcn_ballot_w64(v[0] >= 0.0f);
                if (lane == 0) {
                    const uint32_t keep = (uint32_t)m & (N == 32 ? 0xFFFFFFFFu : ((1u << (N & 31)) - 1u));
                    const int bit = p * N;
                    bitw[bit >> 5] |= keep << (bit & 31);
                }
            }

            // ---- weighted variant: weights of the tables that end in this projection ----
            if constexpr (WEIGHTED) {
#pragma unroll
                for (int r = 0; r < NREG; ++r)
                    if ((int)lane + 64 * r < N) zwin[kZTail + (int)lane + 64 * r] = v[r];
                wave_lds_fence();
                emit_weights<WMODE>(a, t, p, N, lane, [&](int c) { return zwin[kZTail + c]; });
                if (p + 1 < P) {
                    // slide the tail: it becomes the last 16 coordinates up to the end of projection p
                    wave_lds_fence();
                    float keep = 0.0f;
                    if (lane < kZTail) keep = zwin[(int)lane + N];
                    wave_lds_fence();
                    if (lane < kZTail) zwin[lane] = keep;
                }
                wave_lds_fence();
            }
        }
        wave_lds_fence();

        // ---- a4: code j = bits [j*tau, (j+1)*tau), little-endian ---------------------------
        const uint32_t cmask = (1u << a.tau) - 1u;
        auto code_at = [&](unsigned j) -> uint32_t {
            const unsigned bit = j * (unsigned)a.tau;
            const unsigned wi = bit >> 5, sh = bit & 31u;
            const unsigned long long both = ((unsigned long long)bitw[wi + 1] << 32) | bitw[wi];
            return (uint32_t)(both >> sh) & cmask;
        };
        if (a.packed) {
            for (int s = (int)lane; s < a.k / 2; s += 64)
                a.packed[(long long)s * a.n_pad + t] =
                    (code_at(2u * s) << a.packed_shift) | (code_at(2u * s + 1u) << (16 + a.packed_shift));
        } else {
            for (int j = (int)lane; j < a.k; j += 64) a.codes[t * a.k + j] = (uint16_t)code_at((unsigned)j);
        }
        wave_lds_fence();
    }

    // zero the token padding of the packed layout
    if (a.packed) {
        for (long long t = a.n + wave0; t < a.n_pad; t += n_waves)
            for (int s = (int)lane; s < a.k / 2; s += 64) a.packed[(long long)s * a.n_pad + t] = 0u;
    }
}

// ---------------------------------------------------------------------------------------
// d_pad = 1024 variant (RoBERTa-base / -large widths): same butterflies, fewer cross-lane steps.
//
// The generic kernel keeps coordinate i in (lane i%64, register i/64) for the whole transform, so
// six of the ten stages of a round are lane exchanges costing 2-3 instructions per register.
// Here a round runs in two register layouts and changes between them through LDS:
//   layout A: lane = i[9:4], register = i[3:0]   strides 1, 2, 4, 8       are register pairs
//   layout B: lane = (i[9:8], i[3:0]), register = i[7:4]
//                                                strides 16, 32, 64, 128 are register pairs,
//                                                strides 256, 512 are the permlane16/32 swaps
// i.e. eight of ten stages cost one instruction per register.  The per-wave 4 KB transpose
// area holds coordinate i at word sigma(i) = i ^ ((i >> 4) & 0x3C); with that swizzle the
// 16-byte accesses of layout A and the 4-byte accesses of layout B are both bank-conflict free.
// Every butterfly is still (a + c, a - c), a the lower index, strides ascending, fp32, no
// contraction: the rounding sequence of each coordinate is the textbook loop's.
// The sign diagonals sit in registers in layout A (16 consecutive int8 per lane and round =
// one 16-byte load); the token's row is one contiguous 64-byte run per lane.
constexpr int kH1024TransposeWords = 1024;

__host__ __device__ inline int h1024_wave_words(int P, bool weighted)
{
    return kH1024TransposeWords + hash_bit_words(P, 1024) + (weighted ? kZTail : 0);
}
__host__ inline size_t h1024_lds_bytes(int P, bool weighted = false)
{
    return sizeof(uint32_t) * (size_t)kHashWaves * h1024_wave_words(P, weighted);
}

typedef __attribute__((address_space(3))) uint32_t lds_u32;
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) u32x4_t lds_u32x4;
typedef __attribute__((address_space(3))) uint16_t lds_u16;

// ---- pieces of the d_pad = 1024 transform, shared by hash1024_kernel and the small-batch forward kernel ----

// LDS byte addresses of a lane's pieces of the per-wave transpose area (at LDS byte address tp0) in both layouts
struct H1024Lane {
    uint32_t adrA[4];   // quarter m of the lane's 16 consecutive coordinates (16 bytes)
    uint32_t adrB[16];  // register r of layout B
};

__device__ __forceinline__ void h1024_lane_setup(uint32_t tp0, unsigned lane, H1024Lane &L)
{
#pragma unroll
    for (int m = 0; m < 4; ++m)
        L.adrA[m] = tp0 + 4u * ((((lane & 0x3Cu) | ((lane ^ (lane >> 4)) & 3u)) << 4) | ((m ^ ((lane >> 2) & 3u)) << 2));
    const uint32_t c = lane >> 4, l = lane & 15u;
    const uint32_t base = (c << 8) | (c << 4) | l;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const uint32_t K = ((uint32_t)(r >> 2) << 6) | ((uint32_t)(r & 3) << 4) | ((uint32_t)(r >> 2) << 2);
        L.adrB[r] = tp0 + 4u * (base ^ K);
    }
}

// a1: coordinates lane*16 .. lane*16+15 of row t (d elements of kind x_kind), widened, zero-padded.
// vec_ok: d % 4 == 0 and the rows start 16-byte (fp32) / 8-byte (16-bit kinds) aligned.
__device__ __forceinline__ void h1024_load_row(const void *x, long long t, int d, int x_kind, bool vec_ok, unsigned lane,
                                               float (&xv)[16])
{
    const int i0 = (int)lane * 16;
    if (vec_ok) {
#pragma unroll
        for (int m = 0; m < 4; ++m) {
            float4 f = make_float4(0.f, 0.f, 0.f, 0.f);
            if (i0 + 4 * m < d) {
                if (x_kind) {
                    const uint2 w = *reinterpret_cast<const uint2 *>((const uint16_t *)x + t * d + i0 + 4 * m);
                    const float2 lo = widen16x2(w.x, x_kind), hi = widen16x2(w.y, x_kind);
                    f = make_float4(lo.x, lo.y, hi.x, hi.y);
                } else {
                    f = *reinterpret_cast<const float4 *>((const float *)x + t * d + i0 + 4 * m);
                }
            }
            xv[4 * m] = f.x;
            xv[4 * m + 1] = f.y;
            xv[4 * m + 2] = f.z;
            xv[4 * m + 3] = f.w;
        }
    } else {
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            float f = 0.0f;
            if (i0 + e < d) {
                if (x_kind)
                    f = widen16(((const uint16_t *)x)[t * d + i0 + e], x_kind);
                else
                    f = ((const float *)x)[t * d + i0 + e];
            }
            xv[e] = f;
        }
    }
}

// One round on v in layout A (lane = i[9:4], register = i[3:0]): sign diagonal (sw: the lane's 16 int8 as four
// words), strides 1 .. 8, A -> B through LDS, strides 16 .. 128 in registers, 256 / 512 across lanes, scale;
// unless LAST, back to layout A for the next round.  After a LAST round v is in layout B.
template <bool LAST>
__device__ __forceinline__ void h1024_round(float (&v)[16], const uint32_t (&sw)[4], const H1024Lane &L, unsigned lane,
                                            float scale)
{
    constexpr int NREG = 16;
#pragma unroll
    for (int e = 0; e < NREG; ++e) v[e] = fxor(v[e], (sw[e >> 2] << (24 - 8 * (e & 3))) & 0x80000000u);
    reg_stage<1, NREG>(v);
    reg_stage<2, NREG>(v);
    reg_stage<4, NREG>(v);
    reg_stage<8, NREG>(v);
    wave_lds_fence();
#pragma unroll
    for (int m = 0; m < 4; ++m) {
        u32x4_t q = {__float_as_uint(v[4 * m]), __float_as_uint(v[4 * m + 1]), __float_as_uint(v[4 * m + 2]),
                     __float_as_uint(v[4 * m + 3])};
        *reinterpret_cast<lds_u32x4 *>((uintptr_t)L.adrA[m]) = q;
    }
    wave_lds_fence();
#pragma unroll
    for (int r = 0; r < NREG; ++r) v[r] = __uint_as_float(*reinterpret_cast<lds_u32 *>((uintptr_t)L.adrB[r]));
    reg_stage<1, NREG>(v);
    reg_stage<2, NREG>(v);
    reg_stage<4, NREG>(v);
    reg_stage<8, NREG>(v);
    lane_stage<16, NREG>(v, lane);
    lane_stage<32, NREG>(v, lane);
#pragma unroll
    for (int r = 0; r < NREG; ++r) v[r] = v[r] * scale;
    if constexpr (!LAST) {
        wave_lds_fence();
#pragma unroll
        for (int r = 0; r < NREG; ++r) *reinterpret_cast<lds_u32 *>((uintptr_t)L.adrB[r]) = __float_as_uint(v[r]);
        wave_lds_fence();
#pragma unroll
        for (int m = 0; m < 4; ++m) {
            const u32x4_t q = *reinterpret_cast<lds_u32x4 *>((uintptr_t)L.adrA[m]);
            v[4 * m] = __uint_as_float(q.x);
            v[4 * m + 1] = __uint_as_float(q.y);
            v[4 * m + 2] = __uint_as_float(q.z);
            v[4 * m + 3] = __uint_as_float(q.w);
        }
    }
}

// a4: sign bits of projection p (v in layout B) into the wave's bit string.  Bit l of register r's lane mask is
// coordinate i = (l[5:4] << 8) | (r << 4) | l[3:0]: each 16-bit quarter c of the mask is the run of bits
// [c*256 + r*16, +16) of this projection; lane c stores quarter c of every register.
__device__ __forceinline__ void h1024_sign_bits(const float (&v)[16], unsigned lane, uint32_t *bitw, int p)
{
    unsigned long long msk[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) msk[r] = __builtin_amdgcn_ballot_w64(v[r] >= 0.0f);
    if (lane < 4) {
        lds_u16 *dst = reinterpret_cast<lds_u16 *>((uintptr_t)((uint32_t)(uintptr_t)bitw + 2u * (p * 64 + lane * 16)));
#pragma unroll
        for (int r = 0; r < 16; ++r) dst[r] = (uint16_t)(msk[r] >> (16 * lane));
    }
}

// code j = bits [j*tau, (j+1)*tau) of the bit string, little-endian
__device__ __forceinline__ uint32_t hash_code_at(const uint32_t *bitw, unsigned j, int tau)
{
    const unsigned bit = j * (unsigned)tau;
    const unsigned wi = bit >> 5, sh = bit & 31u;
    const unsigned long long both = ((unsigned long long)bitw[wi + 1] << 32) | bitw[wi];
    return (uint32_t)(both >> sh) & ((1u << tau) - 1u);
}

template <int R, int WMODE>
__global__ __launch_bounds__(kHashThreads) __attribute__((amdgpu_waves_per_eu(4, 4))) void hash1024_kernel(HashArgs a)
{
    constexpr bool WEIGHTED = WMODE != 0;
    constexpr int N = 1024, NREG = 16;
    extern __shared__ uint32_t lds[];
    const unsigned lane = threadIdx.x & 63u;
    const unsigned wave = threadIdx.x >> 6;
    const int P = a.P;
    uint32_t *tp = lds + wave * h1024_wave_words(P, WEIGHTED);  // transpose area, the bit string, the z tail
    uint32_t *bitw = tp + kH1024TransposeWords;
    const int n_bitw = hash_bit_words(P, N);
    float *ztail = reinterpret_cast<float *>(bitw + n_bitw);
    for (int i = (int)lane; i < n_bitw; i += 64) bitw[i] = 0;

    H1024Lane L;
    h1024_lane_setup((uint32_t)(uintptr_t)tp, lane, L);

    const long long gw = (long long)blockIdx.x * kHashWaves + wave;
    const long long n_waves = (long long)gridDim.x * kHashWaves;
    const float scale = a.scale;
    const bool vec_ok = (a.d % 4) == 0;  // rows start 16-byte (fp32) / 8-byte (bf16) aligned: checked by the host

    // a2: projection p's diagonals in layout A: 16 consecutive int8 per lane and round, kept as
    // four words; the XOR mask of coordinate e is the sign bit of byte e moved to bit 31
    // (signs are 16-byte aligned: host-checked)
    uint32_t sw[R][4];
    auto load_masks = [&](int p) {
#pragma unroll
        for (int rd = 0; rd < R; ++rd) {
            const uint4 w = *reinterpret_cast<const uint4 *>(a.signs + ((size_t)p * R + rd) * N + lane * 16);
            sw[rd][0] = w.x;
            sw[rd][1] = w.y;
            sw[rd][2] = w.z;
            sw[rd][3] = w.w;
        }
    };
    if (P == 1 && gw < a.n) load_masks(0);

    float xn[NREG];
    if (gw < a.n) h1024_load_row(a.x, gw, a.d, a.x_kind, vec_ok, lane, xn);
    for (long long t = gw; t < a.n; t += n_waves) {
        float xv[NREG];
#pragma unroll
        for (int e = 0; e < NREG; ++e) xv[e] = xn[e];
        if (t + n_waves < a.n) h1024_load_row(a.x, t + n_waves, a.d, a.x_kind, vec_ok, lane, xn);

        for (int p = 0; p < P; ++p) {
            if (P > 1) load_masks(p);
            float v[NREG];
#pragma unroll
            for (int e = 0; e < NREG; ++e) v[e] = xv[e];
#pragma unroll
            for (int rd = 0; rd < R; ++rd) {
                if (rd + 1 < R)
                    h1024_round<false>(v, sw[rd], L, lane, scale);
                else
                    h1024_round<true>(v, sw[rd], L, lane, scale);
            }
            h1024_sign_bits(v, lane, bitw, p);

            // ---- weighted variant: z of this projection into the transpose area (coordinate i at
            // word sigma(i)), then the weights of the tables that end in this projection.
            if constexpr (WEIGHTED) {
                wave_lds_fence();
#pragma unroll
                for (int r = 0; r < NREG; ++r) *reinterpret_cast<lds_u32 *>((uintptr_t)L.adrB[r]) = __float_as_uint(v[r]);
                wave_lds_fence();
                auto z_at = [&](int c) -> float {
                    if (c < 0) return ztail[kZTail + c];
                    return __uint_as_float(tp[c ^ ((c >> 4) & 0x3C)]);
                };
                emit_weights<WMODE>(a, t, p, N, lane, z_at);
                if (p + 1 < P) {
                    wave_lds_fence();
                    float keep = 0.0f;
                    if (lane < kZTail) keep = z_at(N - kZTail + (int)lane);
                    wave_lds_fence();
                    if (lane < kZTail) ztail[lane] = keep;
                }
                wave_lds_fence();
            }
        }
        wave_lds_fence();

        // ---- a4: code j = bits [j*tau, (j+1)*tau), little-endian ---------------------------
        if (a.packed) {
            for (int s = (int)lane; s < a.k / 2; s += 64)
                a.packed[(long long)s * a.n_pad + t] = (hash_code_at(bitw, 2u * s, a.tau) << a.packed_shift) |
                                                       (hash_code_at(bitw, 2u * s + 1u, a.tau) << (16 + a.packed_shift));
        } else {
            for (int j = (int)lane; j < a.k; j += 64) a.codes[t * a.k + j] = (uint16_t)hash_code_at(bitw, (unsigned)j, a.tau);
        }
        wave_lds_fence();
    }

    // zero the token padding of the packed layout
    if (a.packed) {
        for (long long t = a.n + gw; t < a.n_pad; t += n_waves)
            for (int s = (int)lane; s < a.k / 2; s += 64) a.packed[(long long)s * a.n_pad + t] = 0u;
    }
}

// The re-pack kernels are plain functions: when the library is built in parts only part 0 defines them.
#if !defined(LFFN_PART) || LFFN_PART == 0
// The re-pack kernels transpose a token-major matrix src[n][m] into the table-major dst[m][n_pad] the
// staged gather reads, through 64 x 64 LDS tiles so that both the reads (along m) and the writes (along
// n) are contiguous; grid-stride over tiles.
//   ZERO_PAD: also write zeros to the token padding [n, n_pad) (the packed codes need valid rows there).
template <bool ZERO_PAD, class F>
__device__ __forceinline__ void transpose_tiles(uint32_t *dst, long long n, long long n_pad, long long m, F word)
{
    __shared__ uint32_t tile[64][65];
    const long long n_out = ZERO_PAD ? n_pad : n;
    const long long tiles_m = (m + 63) / 64, tiles_n = (n_out + 63) / 64;
    const int c = threadIdx.x & 63, r0 = threadIdx.x >> 6;  // column within the tile, first of the thread's rows
    for (long long tl = blockIdx.x; tl < tiles_m * tiles_n; tl += gridDim.x) {
        const long long t0 = (tl / tiles_m) * 64, j0 = (tl % tiles_m) * 64;
        __syncthreads();
#pragma unroll
        for (int r = r0; r < 64; r += 4) tile[r][c] = (t0 + r < n && j0 + c < m) ? word(t0 + r, j0 + c) : 0u;
        __syncthreads();
#pragma unroll
        for (int r = r0; r < 64; r += 4)
            if (j0 + r < m && t0 + c < n_out) dst[(j0 + r) * n_pad + t0 + c] = tile[c][r];
    }
}

// ABI weights [n][k] -> wpk[k][n_pad]; ABI shares [n][k][1+tau] -> spk[k][1+tau][n_pad]  (m = k or k * (1 + tau);
// token padding left as it is: those slots are never stored)
__global__ __launch_bounds__(256) void repack_shares_kernel(const float *shares, float *spk, long long n,
                                                            long long n_pad, long long m)
{
    const uint32_t *src = reinterpret_cast<const uint32_t *>(shares);
    transpose_tiles<false>(reinterpret_cast<uint32_t *>(spk), n, n_pad, m,
                           [=](long long t, long long c) { return src[t * m + c]; });
}

// ABI codes [n][k] -> packed[k/2][n_pad]: two codes per word, reduced modulo 2^tau and scaled by 2^shift (for
// a stand-alone gather call that takes the LDS-staged kernel, and for the staged kernel's 64-byte-slice
// form, which needs shift 6); zeros in the token padding.  Even k with 4-byte aligned codes is read a pair
// at a time; an odd k is read code by code and its last table is left out (the caller adds it otherwise).
__global__ __launch_bounds__(256) void repack_codes_kernel(const uint16_t *codes, uint32_t *packed, long long n,
                                                           long long n_pad, int k, int tau, int shift)
{
    const uint32_t cmask = (1u << tau) - 1u;
    auto scale = [=](uint32_t lo, uint32_t hi) { return ((lo & cmask) << shift) | ((hi & cmask) << (16 + shift)); };
    const long long m = k / 2;
    if (k & 1) {
        transpose_tiles<true>(packed, n, n_pad, m, [=](long long t, long long c) {
            const uint16_t *p = codes + t * k + 2 * c;
            return scale(p[0], p[1]);
        });
    } else {
        const uint32_t *src = reinterpret_cast<const uint32_t *>(codes);
        transpose_tiles<true>(packed, n, n_pad, m, [=](long long t, long long c) {
            const uint32_t pair = src[t * m + c];
            return scale(pair, pair >> 16);
        });
    }
}
#endif

}  // namespace lffn
