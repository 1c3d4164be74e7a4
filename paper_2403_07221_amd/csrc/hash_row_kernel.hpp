// Hash step for d_pad = 1024 and 512 with a token per row of lanes (gfx950, wave64):
//   z = x R,  R = D_1 H D_2 H ... (Sec. 3.2, eq. "hadamard"), code_j = decimal(sign(z_j)) (Sec. 3.1).
//
// A token occupies LPT lanes of one DPP row (LPT = 16 for d_pad = 1024: four tokens per wavefront; LPT = 8 for
// d_pad = 512: eight tokens) and 64 registers: coordinate i lives in register i / LPT of the lane that stands
// for c = i % LPT.  No stage of the transform leaves the token's lanes, so there is no LDS transpose and no
// lane swap between rows:
//   * strides LPT .. d_pad / 2 are register pairs (a, c) -> (a + c, a - c);
//   * strides 1, 2, 4 (, 8) exchange with the lane whose c differs in one bit.  DPP reaches lane ^ 1, ^ 2, ^ 7
//     (row_half_mirror) and ^ 8 in one step but not ^ 4, so c is mapped to lanes linearly over GF(2),
//       lane = c0 * 1  ^  c1 * 2  ^  c2 * 7  ^  c3 * 8      (c = lane with its two low bits inverted when bit 2 is set)
//     and the exchanges are those DPP controls.  A butterfly is one instruction per coordinate:
//       v <- v + s * v[partner],  s = +1 where the lane holds the lower index, -1 where it holds the upper,
//     as a fused multiply-add with the DPP operand (s * partner is exact, so the one rounding is that of the
//     add / subtract).  The lower lane gets a + c; the upper lane gets c_own - a_partner = -(a - c): it keeps
//     the negated value.  Negation is exact and commutes with every later add, subtract and rounding, and the
//     partner lanes of the later exchange stages and all registers of a lane carry the same number of
//     negations, so it is undone once per round, in the multiplier below.
//   * the round's scale, the undoing of the negations (parity of c) and the NEXT round's sign diagonal are one
//     multiplier per coordinate, +-scale, read from LDS (built once per workgroup); the first round's
//     diagonal is an XOR word per coordinate from the same table.
// Each coordinate therefore goes through the additions of the textbook in-place loop, in ascending stride,
// with the same roundings, and the sign bits come out identical to the one-token-per-wave kernels'.
//
// Sign bits: `v >= 0` per register is a lane mask = LPT consecutive bits of the bit string for each of the
// wave's tokens, in lane order; v_writelane collects the 64 masks into two registers (lane m holds mask m), the
// lane order is turned into c order there (the four bits of every odd nibble reversed), and the pieces go
// to the tokens' bit strings in LDS, from which the lanes of a token cut the codes.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "hash_kernel.hpp"

namespace lffn {

constexpr int kRowThreads = 256;
constexpr int kRowWaves = kRowThreads / 64;
constexpr int kRowRegs = 64;         // coordinates per lane
constexpr int kRowLaneWords = 68;    // words between the constants of two lanes: 64 + 4, so that the 16-byte reads
                                     // of an instruction (one address per c, shared by the tokens) fall on all banks

// constants: [P][1 + R][LPT lanes][kRowLaneWords]; slot 0 the first round's XOR words, slot 1 + r the
// multipliers at the end of round r
__host__ __device__ inline size_t hrow_const_words(int P, int R, int lpt) { return (size_t)P * (R + 1) * lpt * kRowLaneWords; }
// z window of the weights of a tau that does not divide LPT: per wave one token's z of the current projection
// and, per token of the wave, the last kZTail coordinates of the projections before it
__host__ __device__ inline size_t hrow_window_words(int lpt, bool window)
{
    return window ? (size_t)kRowWaves * (64 * lpt + (64 / lpt) * kZTail) : 0;
}
__host__ __device__ inline size_t hrow_lds_bytes(int P, int R, int lpt, bool window = false)
{
    return 4 * (hrow_const_words(P, R, lpt) + (size_t)kRowWaves * (64 / lpt) * hash_bit_words(P, 64 * lpt) +
                hrow_window_words(lpt, window));
}

typedef __attribute__((address_space(3))) uint8_t lds_u8;

// sixteen butterflies of one exchange stage: v[m] += s * v[m] of the partner lane.  The leading s_nop covers
// the two wait states a DPP read needs after a vector write of the same register, which the compiler cannot
// see into an asm statement to insert.
#define LFFN_ROW_FMAC(i, ctrl) "v_fmac_f32_dpp %" #i ", %" #i ", %16 " ctrl " row_mask:0xf bank_mask:0xf\n\t"
#define LFFN_ROW_STAGE16(ctrl)                                                                                      \
    "s_nop 1\n\t" LFFN_ROW_FMAC(0, ctrl) LFFN_ROW_FMAC(1, ctrl) LFFN_ROW_FMAC(2, ctrl) LFFN_ROW_FMAC(3, ctrl)          \
        LFFN_ROW_FMAC(4, ctrl) LFFN_ROW_FMAC(5, ctrl) LFFN_ROW_FMAC(6, ctrl) LFFN_ROW_FMAC(7, ctrl)                    \
            LFFN_ROW_FMAC(8, ctrl) LFFN_ROW_FMAC(9, ctrl) LFFN_ROW_FMAC(10, ctrl) LFFN_ROW_FMAC(11, ctrl)              \
                LFFN_ROW_FMAC(12, ctrl) LFFN_ROW_FMAC(13, ctrl) LFFN_ROW_FMAC(14, ctrl) LFFN_ROW_FMAC(15, ctrl)

// BIT = index bit 0 .. 3 of the exchange; s = +-1 of this lane for that bit
template <int BIT>
__device__ __forceinline__ void row_exchange16(float *v, float s)
{
#define LFFN_ROW_OPS                                                                                                \
    "+v"(v[0]), "+v"(v[1]), "+v"(v[2]), "+v"(v[3]), "+v"(v[4]), "+v"(v[5]), "+v"(v[6]), "+v"(v[7]), "+v"(v[8]),    \
        "+v"(v[9]), "+v"(v[10]), "+v"(v[11]), "+v"(v[12]), "+v"(v[13]), "+v"(v[14]), "+v"(v[15])
    if constexpr (BIT == 0) asm volatile(LFFN_ROW_STAGE16("quad_perm:[1,0,3,2]") : LFFN_ROW_OPS : "v"(s));
    else if constexpr (BIT == 1) asm volatile(LFFN_ROW_STAGE16("quad_perm:[2,3,0,1]") : LFFN_ROW_OPS : "v"(s));
    else if constexpr (BIT == 2) asm volatile(LFFN_ROW_STAGE16("row_half_mirror") : LFFN_ROW_OPS : "v"(s));
    else asm volatile(LFFN_ROW_STAGE16("row_ror:8") : LFFN_ROW_OPS : "v"(s));
#undef LFFN_ROW_OPS
}

template <int BIT, int LIVE>
__device__ __forceinline__ void row_exchange(float (&v)[kRowRegs], float s)
{
#pragma unroll
    for (int g = 0; g < LIVE; g += 16) row_exchange16<BIT>(&v[g], s);
}

// value of x in the lane whose c differs in bit BIT
template <int BIT>
__device__ __forceinline__ float row_partner(float x)
{
    constexpr int ctrl = BIT == 0 ? 0xB1 : BIT == 1 ? 0x4E : BIT == 2 ? 0x141 : 0x128;  // the exchanges' controls
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), ctrl, 0xF, 0xF, true));
}

// Gather weights of the tables in projection p for tau = 2^SH <= LPT (see the call).  Register m holds LPT >> SH
// tables per token; table j's weight goes to weights[t][j] or, table-major, to wpk[j][t].  After the all-reduce
// every lane of a table's run holds its weight, so for tau >= 4 lane x of the run picks the weight of register
// m0 + x of a block of S = min(8, tau) registers: one store per block, every lane a different (table, token),
// instead of one store per register from one lane in tau.
template <int SH, int LPT>
__device__ __forceinline__ void row_weights(const HashArgs &a, const float (&v)[kRowRegs], int p, int n_reg, unsigned c,
                                            long long t, bool t_ok)
{
    constexpr int PER_REG = LPT >> SH;                      // tables per register
    constexpr int TAU = 1 << SH;
    constexpr int S = TAU >= 8 ? 8 : TAU >= 4 ? 4 : 1;      // registers per store
    static_assert(TAU <= LPT, "a table's coordinates lie in one register");
    const unsigned x = c & (unsigned)(TAU - 1);             // position in the table's run of lanes
    const int jl = p * ((64 * LPT) >> SH) + (int)(c >> SH) + (S > 1 ? (int)x * PER_REG : 0);  // this lane's table in block 0
    const bool writer = t_ok && x < (unsigned)S;
    float *dst = a.wpk ? a.wpk + wpk_index(jl, t, a.n_pad) : a.weights + t * a.k + jl;
    const long long step = a.wpk ? (long long)PER_REG * a.n_pad : PER_REG;   // elements from one register's table to the next's
    // eight registers at a time: their reduction chains are independent and interleave
#pragma unroll
    for (int m0 = 0; m0 < kRowRegs; m0 += 8) {
        if (m0 < n_reg) {
            float sum[8], q[8], w[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                sum[u] = __builtin_fabsf(v[m0 + u]);
                q[u] = 1.0f + __builtin_amdgcn_exp2f(sum[u] * -2.885390082f);  // exp(-2 |z|) = 2^(-2 |z| log2 e)
            }
            if constexpr (SH > 0) {
#pragma unroll
                for (int u = 0; u < 8; ++u) { sum[u] += row_partner<0>(sum[u]); q[u] *= row_partner<0>(q[u]); }
            }
            if constexpr (SH > 1) {
#pragma unroll
                for (int u = 0; u < 8; ++u) { sum[u] += row_partner<1>(sum[u]); q[u] *= row_partner<1>(q[u]); }
            }
            if constexpr (SH > 2) {
#pragma unroll
                for (int u = 0; u < 8; ++u) { sum[u] += row_partner<2>(sum[u]); q[u] *= row_partner<2>(q[u]); }
            }
            if constexpr (SH > 3) {
#pragma unroll
                for (int u = 0; u < 8; ++u) { sum[u] += row_partner<3>(sum[u]); q[u] *= row_partner<3>(q[u]); }
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) w[u] = sum[u] * __builtin_amdgcn_rcpf(q[u]);  // q >= 1: no overflow; reciprocal good to 1 ulp
#pragma unroll
            for (int b0 = 0; b0 < 8; b0 += S) {
                float ws = w[b0];
#pragma unroll
                for (int u = 1; u < S; ++u) ws = x == (unsigned)u ? w[b0 + u] : ws;
                const int mb = m0 + b0;                                      // first register of the block
                if (writer && jl + mb * PER_REG < a.k) dst[mb * step] = ws;
            }
        }
    }
}

// lane order -> c order inside every 16-bit group of w: the four bits of the odd nibbles reversed
__device__ __forceinline__ uint32_t row_c_order(uint32_t w)
{
    const uint32_t r = __builtin_bswap32(__builtin_bitreverse32(w));  // nibble k reversed, now at nibble k ^ 1
    return (w & 0x0F0F0F0Fu) | ((r & 0x0F0F0F0Fu) << 4);
}

// lane M of (lo, hi) <- the two halves of the lane mask of `v[M] >= 0`, for M = 0 .. 63, four masks per asm
// statement.  The s_nop covers the two wait states gfx950 needs between a vector compare writing a scalar
// register and a vector instruction reading it, which the compiler cannot insert for an asm statement.
template <int M>
__device__ __forceinline__ void row_collect_masks(const float (&v)[kRowRegs], uint32_t &lo, uint32_t &hi)
{
    if constexpr (M < kRowRegs) {
        const unsigned long long b0 = __builtin_amdgcn_ballot_w64(v[M] >= 0.0f);
        const unsigned long long b1 = __builtin_amdgcn_ballot_w64(v[M + 1] >= 0.0f);
        const unsigned long long b2 = __builtin_amdgcn_ballot_w64(v[M + 2] >= 0.0f);
        const unsigned long long b3 = __builtin_amdgcn_ballot_w64(v[M + 3] >= 0.0f);
        asm volatile(
            "s_nop 1\n\t"
            "v_writelane_b32 %0, %2, %10\n\tv_writelane_b32 %1, %3, %10\n\t"
            "v_writelane_b32 %0, %4, %11\n\tv_writelane_b32 %1, %5, %11\n\t"
            "v_writelane_b32 %0, %6, %12\n\tv_writelane_b32 %1, %7, %12\n\t"
            "v_writelane_b32 %0, %8, %13\n\tv_writelane_b32 %1, %9, %13"
            : "+v"(lo), "+v"(hi)
            : "s"((uint32_t)b0), "s"((uint32_t)(b0 >> 32)), "s"((uint32_t)b1), "s"((uint32_t)(b1 >> 32)),
              "s"((uint32_t)b2), "s"((uint32_t)(b2 >> 32)), "s"((uint32_t)b3), "s"((uint32_t)(b3 >> 32)),
              "n"(M), "n"(M + 1), "n"(M + 2), "n"(M + 3));
        row_collect_masks<M + 4>(v, lo, hi);
    }
}

// in-register butterflies of stride HH over the registers below LIVE (a multiple of 2 * HH)
template <int HH, int LIVE>
__device__ __forceinline__ void row_reg_stage(float (&v)[kRowRegs])
{
#pragma unroll
    for (int r = 0; r < LIVE; ++r) {
        if ((r & HH) == 0) {
            const float a = v[r], c = v[r + HH];
            v[r] = a + c;
            v[r + HH] = a - c;
        }
    }
}

// R rounds; LPT lanes per token (16: d_pad = 1024, 8: d_pad = 512); MFULL = d / LPT when the kernel is built for
// one row length (registers MFULL .. 63 are padding: their first-round work up to the stride of 8 registers is
// left out, zeros staying zeros), 0 = any d that is a multiple of 16.
// The kernel keeps two sets of rows in registers (the one being transformed and the next one, in flight), about
// 230 registers per lane: two waves per SIMD, which is enough because a wave's instructions are independent
// for 64 registers at a stretch; the grid is sized so that a wave works through several groups of tokens.
// WMODE: 0 codes only; 1 codes and gather weights, tau divides LPT (reduced in registers); 2 codes and gather
// weights of any tau <= 16, through a z window in LDS (one token at a time, a lane per table)
template <int R, int MFULL, int WMODE, int LPT>
__global__ __launch_bounds__(kRowThreads) void hash_row_kernel(HashArgs a)
{
    static_assert(LPT == 16 || LPT == 8, "a token is a row of 16 lanes or half of one");
    constexpr int N = 64 * LPT;
    constexpr int LB = LPT == 16 ? 4 : 3;   // index bits held by the lanes
    constexpr int TOK = 64 / LPT;           // tokens per wave
    constexpr int LIVE = MFULL ? ((MFULL + 15) / 16) * 16 : kRowRegs;  // registers that can be non-zero at the start
    extern __shared__ uint32_t lds[];
    const unsigned tid = threadIdx.x;
    const unsigned lane = tid & 63u, wave = tid >> 6;
    const unsigned row = lane / LPT;                                     // which of the wave's tokens
    const unsigned c = (lane & (LPT - 1u)) ^ ((lane & 4u) ? 3u : 0u);    // i % LPT of this lane's coordinates
    const int P = a.P;
    const int W = hash_bit_words(P, N);
    uint32_t *consts = lds;
    uint32_t *bits_wave = lds + hrow_const_words(P, R, LPT) + (size_t)wave * TOK * W;
    // window mode: [N] z of one token, then [TOK][kZTail] tails (see hrow_window_words)
    float *zwin = reinterpret_cast<float *>(lds + hrow_const_words(P, R, LPT) + (size_t)kRowWaves * TOK * W) +
                  (size_t)wave * (N + TOK * kZTail);
    float *ztail = zwin + N;

    const int m_full = MFULL ? MFULL : __builtin_amdgcn_readfirstlane(a.d / LPT);
    const long long n_groups = (a.n + TOK - 1) / TOK;
    const long long gw = (long long)blockIdx.x * kRowWaves + wave;
    const long long n_waves = (long long)gridDim.x * kRowWaves;

    // ---- a1: a token's row, zero-padded to N.  d is a multiple of 16 (host-checked): register m is in
    // range for every lane or for none.  A row past the end of the batch reads the last token's.
    // xn holds the rows in flight as they come from memory: fp32 values, or the 16 bits of a bf16 / half element
    // (widened where the rows are taken over, in one place, by a wave-uniform choice of the element type)
    float xn[kRowRegs];
    auto load_rows = [&](long long g, int m0 = 0, int m1 = kRowRegs) {  // registers m0 .. m1 - 1
        const long long t = g * TOK + row;
        const long long t_ld = t < a.n ? t : a.n - 1;
        if (a.x_kind == kElemF32) {
            const float *xr = static_cast<const float *>(a.x) + t_ld * a.d + c;
#pragma unroll
            for (int m = 0; m < kRowRegs; ++m) {
                if (m < m0 || m >= m1) continue;
                if constexpr (MFULL != 0) xn[m] = m < MFULL ? xr[LPT * m] : 0.0f;
                else xn[m] = m < m_full ? xr[LPT * m] : 0.0f;
            }
        } else {
            const uint16_t *xr = static_cast<const uint16_t *>(a.x) + t_ld * a.d + c;
#pragma unroll
            for (int m = 0; m < kRowRegs; ++m) {
                if (m < m0 || m >= m1) continue;
                uint32_t bits = 0u;
                if constexpr (MFULL != 0) { if (m < MFULL) bits = xr[LPT * m]; }
                else { if (m < m_full) bits = xr[LPT * m]; }
                xn[m] = __uint_as_float(bits);
            }
        }
    };
    auto take_rows = [&](float (&v)[kRowRegs]) {
        if (a.x_kind == kElemF32) {
#pragma unroll
            for (int m = 0; m < kRowRegs; ++m) v[m] = xn[m];
        } else if (a.x_kind == kElemBF16) {
#pragma unroll
            for (int m = 0; m < kRowRegs; ++m) v[m] = __uint_as_float(__float_as_uint(xn[m]) << 16);
        } else {
#pragma unroll
            for (int m = 0; m < kRowRegs; ++m) v[m] = half_bits_to_float((uint16_t)__float_as_uint(xn[m]));
        }
    };
    if (gw < n_groups) load_rows(gw);  // in flight while the constants are built

    // ---- a2: the constants, once per workgroup.  A unit = 16 consecutive diagonal entries of one
    // (projection, round), read as one 16-byte word (signs are 16-byte aligned: host-checked)
    {
        const uint32_t sc = __float_as_uint(a.scale);
        constexpr int UNITS = N / 16;  // per (projection, round)
        for (int u = (int)tid; u < P * R * UNITS; u += kRowThreads) {
            const int mu = u % UNITS, pr = u / UNITS, p = pr / R, rd = pr - p * R;
            const uint4 w16 = reinterpret_cast<const uint4 *>(a.signs)[u];
            const uint32_t wd[4] = {w16.x, w16.y, w16.z, w16.w};
            uint32_t *dst = consts + (size_t)(p * (R + 1) + rd) * LPT * kRowLaneWords;
#pragma unroll
            for (int b = 0; b < 16; ++b) {
                const int i = 16 * mu + b, ci = i & (LPT - 1), m = i >> LB;
                const uint32_t neg = (wd[b >> 2] << (24 - 8 * (b & 3))) & 0x80000000u;  // sign bit of byte b
                // slot 0: the first diagonal as an XOR word; slot rd >= 1: the multiplier at the end of round
                // rd - 1 = scale, parity of c, diagonal rd
                const uint32_t odd = (__builtin_popcount(ci) & 1) ? 0x80000000u : 0u;
                dst[ci * kRowLaneWords + m] = rd == 0 ? neg : (sc ^ neg ^ odd);
            }
        }
        for (int u = (int)tid; u < P * kRowRegs; u += kRowThreads) {  // end of the last round: no diagonal
            const int m = u & 63, p = u >> 6;
            uint32_t *dst = consts + (size_t)(p * (R + 1) + R) * LPT * kRowLaneWords + m;
#pragma unroll
            for (int ci = 0; ci < LPT; ++ci) dst[ci * kRowLaneWords] = sc ^ ((__builtin_popcount(ci) & 1) ? 0x80000000u : 0u);
        }
        for (int i = (int)lane; i < TOK * W; i += 64) bits_wave[i] = 0;
    }
    __syncthreads();

    // +1 where this lane holds the lower index of the exchange of bit b of c, -1 where the upper
    const float s0 = (c & 1u) ? -1.0f : 1.0f, s1 = (c & 2u) ? -1.0f : 1.0f;
    const float s2 = (c & 4u) ? -1.0f : 1.0f, s3 = (c & 8u) ? -1.0f : 1.0f;
    const uint32_t cbase = (uint32_t)(uintptr_t)consts + c * (kRowLaneWords * 4u);  // LDS byte address of this lane's constants
    const uint32_t *bits_row = bits_wave + row * W;
    constexpr int SLOT = LPT * kRowLaneWords / 4;  // 16-byte words between two slots of the constants

    for (long long g = gw; g < n_groups; g += n_waves) {
        const long long t = g * TOK + row;
        const bool t_ok = t < a.n;
        for (int p = 0; p < P; ++p) {
            float v[kRowRegs];
            take_rows(v);
            // xn keeps this group's rows for its next projection; during the last projection's transform the next
            // group's rows are fetched into it, a share of the registers after each round's butterflies: all at
            // once, the requests fill the memory pipeline and the wave waits at their issue (26.7 against 27.9 us
            // for 16384 rows of 768)
            const bool fetch_next = p + 1 == P && g + n_waves < n_groups;
            const lds_u32x4 *cp = reinterpret_cast<const lds_u32x4 *>((uintptr_t)cbase) + p * (R + 1) * SLOT;
            // ---- a2: first diagonal ----
#pragma unroll
            for (int q = 0; q < LIVE / 4; ++q) {
                const u32x4_t w = cp[q];
                v[4 * q] = fxor(v[4 * q], w.x);
                v[4 * q + 1] = fxor(v[4 * q + 1], w.y);
                v[4 * q + 2] = fxor(v[4 * q + 2], w.z);
                v[4 * q + 3] = fxor(v[4 * q + 3], w.w);
            }
#pragma unroll
            for (int rd = 0; rd < R; ++rd) {
                // ---- a3: strides 1 .. LPT / 2 across the lanes of the token, LPT .. N / 2 in registers ----
                if (rd == 0) {
                    row_exchange<0, LIVE>(v, s0);
                    row_exchange<1, LIVE>(v, s1);
                    row_exchange<2, LIVE>(v, s2);
                    if constexpr (LPT == 16) row_exchange<3, LIVE>(v, s3);
                    row_reg_stage<1, LIVE>(v);
                    row_reg_stage<2, LIVE>(v);
                    row_reg_stage<4, LIVE>(v);
                    row_reg_stage<8, LIVE>(v);
                } else {
                    row_exchange<0, kRowRegs>(v, s0);
                    row_exchange<1, kRowRegs>(v, s1);
                    row_exchange<2, kRowRegs>(v, s2);
                    if constexpr (LPT == 16) row_exchange<3, kRowRegs>(v, s3);
                    row_reg_stage<1, kRowRegs>(v);
                    row_reg_stage<2, kRowRegs>(v);
                    row_reg_stage<4, kRowRegs>(v);
                    row_reg_stage<8, kRowRegs>(v);
                }
                row_reg_stage<16, kRowRegs>(v);
                row_reg_stage<32, kRowRegs>(v);
                __builtin_amdgcn_sched_barrier(0);
                if (fetch_next) {
                    constexpr int SHARE = (kRowRegs + R - 1) / R;
                    load_rows(g + n_waves, rd * SHARE, rd + 1 < R ? (rd + 1) * SHARE : kRowRegs);
                }
                __builtin_amdgcn_sched_barrier(0);
                // scale, negations undone, next diagonal
                const lds_u32x4 *cm = cp + (rd + 1) * SLOT;
#pragma unroll
                for (int q = 0; q < kRowRegs / 4; ++q) {
                    const u32x4_t w = cm[q];
                    v[4 * q] = v[4 * q] * __uint_as_float(w.x);
                    v[4 * q + 1] = v[4 * q + 1] * __uint_as_float(w.y);
                    v[4 * q + 2] = v[4 * q + 2] * __uint_as_float(w.z);
                    v[4 * q + 3] = v[4 * q + 3] * __uint_as_float(w.w);
                }
            }
            // ---- a4: sign bits.  Mask m = bits [LPT m, LPT m + LPT) of each token's string, lane order ----
            uint32_t lo = 0, hi = 0;
            row_collect_masks<0>(v, lo, hi);
            // ---- weighted variant (Sec. 4): w_j = |z_j|_1 / prod_b (1 + exp(-2 |z_jb|)).  tau divides LPT
            // (host-checked), so a table's coordinates are tau neighbouring c of one register: sum and product
            // are all-reduced over those lanes with the exchanges' DPP controls, and the weight is
            // sum * (1 / product).
            if constexpr (WMODE == 1) {
                const long long bits_left = (long long)a.k * a.tau - (long long)p * N;
                const int n_reg = bits_left >= N ? kRowRegs : (int)((bits_left + LPT - 1) / LPT);  // registers that hold table coordinates
                switch (a.tau) {
                    case 1: row_weights<0, LPT>(a, v, p, n_reg, c, t, t_ok); break;
                    case 2: row_weights<1, LPT>(a, v, p, n_reg, c, t, t_ok); break;
                    case 4: row_weights<2, LPT>(a, v, p, n_reg, c, t, t_ok); break;
                    case 8: row_weights<3, LPT>(a, v, p, n_reg, c, t, t_ok); break;
                    default:
                        if constexpr (LPT == 16) row_weights<4, LPT>(a, v, p, n_reg, c, t, t_ok);
                        break;
                }
            }
            // Any other tau (a table then crosses registers, and may cross from one projection into the next): z
            // goes through LDS, one token at a time; the wave's lanes take a table each and form the same sum and
            // product coordinate by coordinate.  Tables are handled in the projection that holds their last
            // coordinate; the 16 coordinates before a projection's start are kept per token.
            if constexpr (WMODE == 2) {
                const int tau = a.tau;
                const long long lo_bit = (long long)p * N;
                const int jlo = (int)(lo_bit / tau);
                long long jhi = (lo_bit + N) / tau;
                if (jhi > a.k) jhi = a.k;
#pragma unroll 1
                for (int tr = 0; tr < TOK; ++tr) {  // the wave's tokens in turn
                    wave_lds_fence();
                    if (row == (unsigned)tr) {
#pragma unroll
                        for (int m = 0; m < kRowRegs; ++m) zwin[LPT * m + (int)c] = v[m];
                    }
                    wave_lds_fence();
                    const long long tw = g * TOK + tr;
                    const float *tail = ztail + tr * kZTail;
                    if (tw < a.n) {
                        for (int j = jlo + (int)lane; j < (int)jhi; j += 64) {
                            const int c0 = (int)((long long)j * tau - lo_bit);  // may be negative: the table began before
                            float sum = 0.0f, q = 1.0f;
                            for (int b = 0; b < tau; ++b) {
                                const int cc = c0 + b;
                                const float az = __builtin_fabsf(cc < 0 ? tail[kZTail + cc] : zwin[cc]);
                                sum += az;
                                q *= 1.0f + __builtin_amdgcn_exp2f(az * -2.885390082f);  // exp(-2 az) = 2^(-2 az log2 e)
                            }
                            const float w = sum * __builtin_amdgcn_rcpf(q);  // q >= 1
                            if (a.wpk) a.wpk[wpk_index(j, tw, a.n_pad)] = w;
                            else a.weights[tw * a.k + j] = w;
                        }
                    }
                    if (p + 1 < P) {  // the last 16 coordinates of this projection become the token's tail
                        wave_lds_fence();
                        float keep = 0.0f;
                        if (lane < (unsigned)kZTail) keep = zwin[N - kZTail + (int)lane];
                        wave_lds_fence();
                        if (lane < (unsigned)kZTail) ztail[tr * kZTail + (int)lane] = keep;
                    }
                }
                wave_lds_fence();
            }
            lo = row_c_order(lo);
            hi = row_c_order(hi);
            // lane m: piece m (LPT bits) of projection p of the first half of the wave's tokens (lo) and of the
            // second half (hi)
            if constexpr (LPT == 16) {
                const uint32_t hb = (uint32_t)(uintptr_t)bits_wave + 2u * (uint32_t)(p * 64 + (int)lane);
                *reinterpret_cast<lds_u16 *>((uintptr_t)hb) = (uint16_t)lo;
                *reinterpret_cast<lds_u16 *>((uintptr_t)(hb + 4u * W)) = (uint16_t)(lo >> 16);
                *reinterpret_cast<lds_u16 *>((uintptr_t)(hb + 8u * W)) = (uint16_t)hi;
                *reinterpret_cast<lds_u16 *>((uintptr_t)(hb + 12u * W)) = (uint16_t)(hi >> 16);
            } else {
                const uint32_t hb = (uint32_t)(uintptr_t)bits_wave + (uint32_t)(p * 64 + (int)lane);
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    *reinterpret_cast<lds_u8 *>((uintptr_t)(hb + 4u * W * r)) = (uint8_t)(lo >> (8 * r));
                    *reinterpret_cast<lds_u8 *>((uintptr_t)(hb + 4u * W * (4 + r))) = (uint8_t)(hi >> (8 * r));
                }
            }
        }
        wave_lds_fence();

        // ---- a4: code j = bits [j*tau, (j+1)*tau), little-endian; the lanes of a token share its codes ----
        if (t_ok) {
            const unsigned q = lane & (LPT - 1u);
            if (a.packed) {
                for (int s = (int)q; s < a.k / 2; s += LPT)
                    a.packed[(long long)s * a.n_pad + t] = (hash_code_at(bits_row, 2u * s, a.tau) << a.packed_shift) |
                                                           (hash_code_at(bits_row, 2u * s + 1u, a.tau) << (16 + a.packed_shift));
            } else {
                for (int j = (int)q; j < a.k; j += LPT)
                    a.codes[t * a.k + j] = (uint16_t)hash_code_at(bits_row, (unsigned)j, a.tau);
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
