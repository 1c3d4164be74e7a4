// Hash step for d_pad = 1024, four tokens per wavefront (gfx950, wave64):
//   z = x R,  R = D_1 H D_2 H ... (Sec. 3.2, eq. "hadamard"), code_j = decimal(sign(z_j)) (Sec. 3.1).
//
// A token occupies one DPP row of 16 lanes and 64 registers: coordinate i lives in register i[9:4] of the
// lane that stands for c = i[3:0].  No stage of the transform leaves the lane row, so there is no LDS
// transpose and no lane swap between rows:
//   * strides 16 .. 512 are register pairs (a, c) -> (a + c, a - c);
//   * strides 1, 2, 4, 8 exchange with the lane whose c differs in one bit.  DPP reaches lane ^ 1, ^ 2, ^ 7
//     (row_half_mirror) and ^ 8 in one step but not ^ 4, so c is mapped to lanes linearly over GF(2),
//       lane = c0 * 1  ^  c1 * 2  ^  c2 * 7  ^  c3 * 8      (c = lane with its two low bits inverted when bit 2 is set)
//     and the four exchanges are those four DPP controls.  A butterfly is one instruction per coordinate:
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
// Sign bits: `v >= 0` per register is a lane mask = 16 consecutive bits of the bit string for each of the
// four tokens, in lane order; v_writelane collects the 64 masks into two registers (lane m holds mask m), the
// lane order is turned into c order there (the four bits of every odd nibble reversed), and the halfwords go
// to the tokens' bit strings in LDS, from which the lanes of a row cut the codes.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "hash_kernel.hpp"

namespace lffn {

constexpr int kX4Threads = 256;
constexpr int kX4Waves = kX4Threads / 64;
constexpr int kX4Tokens = 4;        // tokens per wave: one per DPP row
constexpr int kX4Regs = 64;         // coordinates per lane
constexpr int kX4LaneWords = 68;    // words between the constants of two lanes: 64 + 4, so that the sixteen
                                    // 16-byte reads of an instruction fall on all 64 banks

// constants: [P][1 + R][16 lanes][kX4LaneWords]; slot 0 the first round's XOR words, slot 1 + r the
// multipliers at the end of round r
__host__ __device__ inline size_t hx4_const_words(int P, int R) { return (size_t)P * (R + 1) * 16 * kX4LaneWords; }
__host__ __device__ inline size_t hx4_lds_bytes(int P, int R)
{
    return 4 * (hx4_const_words(P, R) + (size_t)kX4Waves * kX4Tokens * hash_bit_words(P, 1024));
}

// c (= i[3:0]) of a lane and back
__host__ __device__ inline unsigned hx4_c_of_lane(unsigned l) { return (l & 15u) ^ ((l & 4u) ? 3u : 0u); }

// sixteen butterflies of one exchange stage: v[m] += s * v[m] of the partner lane.  The leading s_nop covers
// the two wait states a DPP read needs after a vector write of the same register, which the compiler cannot
// see into an asm statement to insert.
#define LFFN_X4_FMAC(i, ctrl) "v_fmac_f32_dpp %" #i ", %" #i ", %16 " ctrl " row_mask:0xf bank_mask:0xf\n\t"
#define LFFN_X4_STAGE16(ctrl)                                                                                      \
    "s_nop 1\n\t" LFFN_X4_FMAC(0, ctrl) LFFN_X4_FMAC(1, ctrl) LFFN_X4_FMAC(2, ctrl) LFFN_X4_FMAC(3, ctrl)          \
        LFFN_X4_FMAC(4, ctrl) LFFN_X4_FMAC(5, ctrl) LFFN_X4_FMAC(6, ctrl) LFFN_X4_FMAC(7, ctrl)                    \
            LFFN_X4_FMAC(8, ctrl) LFFN_X4_FMAC(9, ctrl) LFFN_X4_FMAC(10, ctrl) LFFN_X4_FMAC(11, ctrl)              \
                LFFN_X4_FMAC(12, ctrl) LFFN_X4_FMAC(13, ctrl) LFFN_X4_FMAC(14, ctrl) LFFN_X4_FMAC(15, ctrl)

// BIT = index bit 0 .. 3 of the exchange; s = +-1 of this lane for that bit
template <int BIT>
__device__ __forceinline__ void x4_exchange16(float *v, float s)
{
#define LFFN_X4_OPS                                                                                                \
    "+v"(v[0]), "+v"(v[1]), "+v"(v[2]), "+v"(v[3]), "+v"(v[4]), "+v"(v[5]), "+v"(v[6]), "+v"(v[7]), "+v"(v[8]),    \
        "+v"(v[9]), "+v"(v[10]), "+v"(v[11]), "+v"(v[12]), "+v"(v[13]), "+v"(v[14]), "+v"(v[15])
    if constexpr (BIT == 0) asm volatile(LFFN_X4_STAGE16("quad_perm:[1,0,3,2]") : LFFN_X4_OPS : "v"(s));
    else if constexpr (BIT == 1) asm volatile(LFFN_X4_STAGE16("quad_perm:[2,3,0,1]") : LFFN_X4_OPS : "v"(s));
    else if constexpr (BIT == 2) asm volatile(LFFN_X4_STAGE16("row_half_mirror") : LFFN_X4_OPS : "v"(s));
    else asm volatile(LFFN_X4_STAGE16("row_ror:8") : LFFN_X4_OPS : "v"(s));
#undef LFFN_X4_OPS
}

template <int BIT, int LIVE>
__device__ __forceinline__ void x4_exchange(float (&v)[kX4Regs], float s)
{
#pragma unroll
    for (int g = 0; g < LIVE; g += 16) x4_exchange16<BIT>(&v[g], s);
}

// value of x in the lane whose c differs in bit BIT
template <int BIT>
__device__ __forceinline__ float x4_partner(float x)
{
    constexpr int ctrl = BIT == 0 ? 0xB1 : BIT == 1 ? 0x4E : BIT == 2 ? 0x141 : 0x128;  // the exchanges' controls
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), ctrl, 0xF, 0xF, true));
}

// Gather weights of the tables in projection p for tau = 2^SH (see the call).  Register m holds 16 >> SH tables
// per token; table j's weight goes to weights[t][j] or, table-major, to wpk[j][t].  After the all-reduce every
// lane of a table's run holds its weight, so for tau >= 4 lane x of the run picks the weight of register
// m0 + x of a block of S = min(8, tau) registers: one store per block, every lane a different (table, token),
// instead of one store per register from one lane in tau.
template <int SH>
__device__ __forceinline__ void x4_weights(const HashArgs &a, const float (&v)[kX4Regs], int p, int n_reg, unsigned c,
                                           long long t, bool t_ok)
{
    constexpr int PER_REG = 16 >> SH;                       // tables per register
    constexpr int TAU = 1 << SH;
    constexpr int S = TAU >= 8 ? 8 : TAU >= 4 ? 4 : 1;      // registers per store
    const unsigned x = c & (unsigned)(TAU - 1);             // position in the table's run of lanes
    const int jl = p * (1024 >> SH) + (int)(c >> SH) + (S > 1 ? (int)x * PER_REG : 0);  // this lane's table in block 0
    const bool writer = t_ok && x < (unsigned)S;
    float *dst = a.wpk ? a.wpk + wpk_index(jl, t, a.n_pad) : a.weights + t * a.k + jl;
    const long long step = a.wpk ? (long long)PER_REG * a.n_pad : PER_REG;   // elements from one register's table to the next's
    // eight registers at a time: their reduction chains are independent and interleave
#pragma unroll
    for (int m0 = 0; m0 < kX4Regs; m0 += 8) {
        if (m0 < n_reg) {
            float sum[8], q[8], w[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                sum[u] = __builtin_fabsf(v[m0 + u]);
                q[u] = 1.0f + __builtin_amdgcn_exp2f(sum[u] * -2.885390082f);  // exp(-2 |z|) = 2^(-2 |z| log2 e)
            }
            if constexpr (SH > 0) {
#pragma unroll
                for (int u = 0; u < 8; ++u) { sum[u] += x4_partner<0>(sum[u]); q[u] *= x4_partner<0>(q[u]); }
            }
            if constexpr (SH > 1) {
#pragma unroll
                for (int u = 0; u < 8; ++u) { sum[u] += x4_partner<1>(sum[u]); q[u] *= x4_partner<1>(q[u]); }
            }
            if constexpr (SH > 2) {
#pragma unroll
                for (int u = 0; u < 8; ++u) { sum[u] += x4_partner<2>(sum[u]); q[u] *= x4_partner<2>(q[u]); }
            }
            if constexpr (SH > 3) {
#pragma unroll
                for (int u = 0; u < 8; ++u) { sum[u] += x4_partner<3>(sum[u]); q[u] *= x4_partner<3>(q[u]); }
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
__device__ __forceinline__ uint32_t x4_c_order(uint32_t w)
{
    const uint32_t r = __builtin_bswap32(__builtin_bitreverse32(w));  // nibble k reversed, now at nibble k ^ 1
    return (w & 0x0F0F0F0Fu) | ((r & 0x0F0F0F0Fu) << 4);
}

// lane M of (lo, hi) <- the two halves of the lane mask of `v[M] >= 0`, for M = 0 .. 63, four masks per asm
// statement.  The s_nop covers the two wait states gfx950 needs between a vector compare writing a scalar
// register and a vector instruction reading it, which the compiler cannot insert for an asm statement.
template <int M>
__device__ __forceinline__ void x4_collect_masks(const float (&v)[kX4Regs], uint32_t &lo, uint32_t &hi)
{
    if constexpr (M < kX4Regs) {
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
        x4_collect_masks<M + 4>(v, lo, hi);
    }
}

// in-register butterflies of stride HH over the registers below LIVE (a multiple of 2 * HH)
template <int HH, int LIVE>
__device__ __forceinline__ void x4_reg_stage(float (&v)[kX4Regs])
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

// R rounds; MFULL = d / 16 when the kernel is built for one row length (registers MFULL .. 63 are padding:
// their first-round work up to stride 128 is left out, zeros staying zeros), 0 = any d that is a multiple of 16.
// The kernel keeps two sets of rows in registers (the one being transformed and the next one, in flight), about
// 230 registers per lane: two waves per SIMD, which is enough because a wave's instructions are independent
// for 64 registers at a stretch; the grid is sized so that a wave works through several groups of tokens.
template <int R, int MFULL, bool WEIGHTED>
__global__ __launch_bounds__(kX4Threads) void hash1024x4_kernel(HashArgs a)
{
    constexpr int N = 1024;
    constexpr int LIVE = MFULL ? ((MFULL + 15) / 16) * 16 : kX4Regs;  // registers that can be non-zero at the start
    extern __shared__ uint32_t lds[];
    const unsigned tid = threadIdx.x;
    const unsigned lane = tid & 63u, wave = tid >> 6;
    const unsigned row = lane >> 4;              // which of the wave's four tokens
    const unsigned c = hx4_c_of_lane(lane);      // i[3:0] of this lane's coordinates
    const int P = a.P;
    const int W = hash_bit_words(P, N);
    uint32_t *consts = lds;
    uint32_t *bits_wave = lds + hx4_const_words(P, R) + (size_t)wave * kX4Tokens * W;

    const int m_full = MFULL ? MFULL : __builtin_amdgcn_readfirstlane(a.d >> 4);
    const long long n_groups = (a.n + kX4Tokens - 1) / kX4Tokens;
    const long long gw = (long long)blockIdx.x * kX4Waves + wave;
    const long long n_waves = (long long)gridDim.x * kX4Waves;

    // ---- a1: a token's row, zero-padded to 1024.  d is a multiple of 16 (host-checked): register m is in
    // range for every lane or for none.  A row past the end of the batch reads the last token's.
    float xn[kX4Regs];  // the rows in flight
    auto load_rows = [&](long long g, int m0 = 0, int m1 = kX4Regs) {  // registers m0 .. m1 - 1
        float (&v)[kX4Regs] = xn;
        const long long t = g * kX4Tokens + row;
        const long long t_ld = t < a.n ? t : a.n - 1;
        if (a.x_kind == kElemF32) {
            const float *xr = static_cast<const float *>(a.x) + t_ld * a.d + c;
#pragma unroll
            for (int m = 0; m < kX4Regs; ++m) {
                if (m < m0 || m >= m1) continue;
                if constexpr (MFULL != 0) v[m] = m < MFULL ? xr[16 * m] : 0.0f;
                else v[m] = m < m_full ? xr[16 * m] : 0.0f;
            }
        } else {
            const uint16_t *xr = static_cast<const uint16_t *>(a.x) + t_ld * a.d + c;
#pragma unroll
            for (int m = 0; m < kX4Regs; ++m) {
                if (m < m0 || m >= m1) continue;
                if constexpr (MFULL != 0) v[m] = m < MFULL ? widen16(xr[16 * m], a.x_kind) : 0.0f;
                else v[m] = m < m_full ? widen16(xr[16 * m], a.x_kind) : 0.0f;
            }
        }
    };
    if (gw < n_groups) load_rows(gw);  // in flight while the constants are built

    // ---- a2: the constants, once per workgroup.  A unit = the 16 diagonal entries 16 m .. 16 m + 15 of one
    // (projection, round), read as one 16-byte word (signs are 16-byte aligned: host-checked)
    {
        const uint32_t sc = __float_as_uint(a.scale);
        for (int u = (int)tid; u < P * R * 64; u += kX4Threads) {
            const int m = u & 63, pr = u >> 6, p = pr / R, rd = pr - p * R;
            const uint4 w16 = reinterpret_cast<const uint4 *>(a.signs)[u];
            const uint32_t wd[4] = {w16.x, w16.y, w16.z, w16.w};
            uint32_t *dst = consts + (size_t)(p * (R + 1) + rd) * 16 * kX4LaneWords + m;
#pragma unroll
            for (int ci = 0; ci < 16; ++ci) {
                const uint32_t neg = (wd[ci >> 2] << (24 - 8 * (ci & 3))) & 0x80000000u;  // sign bit of byte ci
                // slot 0: the first diagonal as an XOR word; slot rd >= 1: the multiplier at the end of round
                // rd - 1 = scale, parity of c, diagonal rd
                const uint32_t odd = (__builtin_popcount(ci) & 1) ? 0x80000000u : 0u;
                dst[ci * kX4LaneWords] = rd == 0 ? neg : (sc ^ neg ^ odd);
            }
        }
        for (int u = (int)tid; u < P * 64; u += kX4Threads) {  // end of the last round: no diagonal
            const int m = u & 63, p = u >> 6;
            uint32_t *dst = consts + (size_t)(p * (R + 1) + R) * 16 * kX4LaneWords + m;
#pragma unroll
            for (int ci = 0; ci < 16; ++ci) dst[ci * kX4LaneWords] = sc ^ ((__builtin_popcount(ci) & 1) ? 0x80000000u : 0u);
        }
        for (int i = (int)lane; i < kX4Tokens * W; i += 64) bits_wave[i] = 0;
    }
    __syncthreads();

    // +1 where this lane holds the lower index of the exchange of bit b of c, -1 where the upper
    const float s0 = (c & 1u) ? -1.0f : 1.0f, s1 = (c & 2u) ? -1.0f : 1.0f;
    const float s2 = (c & 4u) ? -1.0f : 1.0f, s3 = (c & 8u) ? -1.0f : 1.0f;
    const uint32_t cbase = (uint32_t)(uintptr_t)consts + c * (kX4LaneWords * 4u);  // LDS byte address of this lane's constants
    const uint32_t *bits_row = bits_wave + row * W;

    for (long long g = gw; g < n_groups; g += n_waves) {
        const long long t = g * kX4Tokens + row;
        const bool t_ok = t < a.n;
        for (int p = 0; p < P; ++p) {
            float v[kX4Regs];
#pragma unroll
            for (int m = 0; m < kX4Regs; ++m) v[m] = xn[m];
            // the next rows (this group's again, for its next projection) are fetched during this transform, a
            // share of the registers after each round's butterflies: all at once, the requests fill the memory
            // pipeline and the wave waits at their issue (26.7 against 27.9 us for configuration 2's batch)
            const long long gn = p + 1 < P ? g : g + n_waves;
            const lds_u32x4 *cp = reinterpret_cast<const lds_u32x4 *>((uintptr_t)cbase) + p * (R + 1) * (4 * kX4LaneWords);
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
                // ---- a3: strides 1 .. 8 across the lanes of the row, 16 .. 512 in registers ----
                if (rd == 0) {
                    x4_exchange<0, LIVE>(v, s0);
                    x4_exchange<1, LIVE>(v, s1);
                    x4_exchange<2, LIVE>(v, s2);
                    x4_exchange<3, LIVE>(v, s3);
                    x4_reg_stage<1, LIVE>(v);
                    x4_reg_stage<2, LIVE>(v);
                    x4_reg_stage<4, LIVE>(v);
                    x4_reg_stage<8, LIVE>(v);
                } else {
                    x4_exchange<0, kX4Regs>(v, s0);
                    x4_exchange<1, kX4Regs>(v, s1);
                    x4_exchange<2, kX4Regs>(v, s2);
                    x4_exchange<3, kX4Regs>(v, s3);
                    x4_reg_stage<1, kX4Regs>(v);
                    x4_reg_stage<2, kX4Regs>(v);
                    x4_reg_stage<4, kX4Regs>(v);
                    x4_reg_stage<8, kX4Regs>(v);
                }
                x4_reg_stage<16, kX4Regs>(v);
                x4_reg_stage<32, kX4Regs>(v);
                __builtin_amdgcn_sched_barrier(0);
                if (gn < n_groups) {
                    constexpr int SHARE = (kX4Regs + R - 1) / R;
                    load_rows(gn, rd * SHARE, rd + 1 < R ? (rd + 1) * SHARE : kX4Regs);
                }
                __builtin_amdgcn_sched_barrier(0);
                // scale, negations undone, next diagonal
                const lds_u32x4 *cm = cp + (rd + 1) * (4 * kX4LaneWords);
#pragma unroll
                for (int q = 0; q < kX4Regs / 4; ++q) {
                    const u32x4_t w = cm[q];
                    v[4 * q] = v[4 * q] * __uint_as_float(w.x);
                    v[4 * q + 1] = v[4 * q + 1] * __uint_as_float(w.y);
                    v[4 * q + 2] = v[4 * q + 2] * __uint_as_float(w.z);
                    v[4 * q + 3] = v[4 * q + 3] * __uint_as_float(w.w);
                }
            }
            // ---- a4: sign bits.  Mask m = bits [16 m, 16 m + 16) of each token's string, lane order ----
            uint32_t lo = 0, hi = 0;
            x4_collect_masks<0>(v, lo, hi);
            // ---- weighted variant (Sec. 4): w_j = |z_j|_1 / prod_b (1 + exp(-2 |z_jb|)).  tau divides 16
            // (host-checked), so a table's coordinates are tau neighbouring c of one register: sum and product
            // are all-reduced over those lanes with the exchanges' DPP controls, and the lane with the
            // table's first coordinate stores sum * (1 / product).
            if constexpr (WEIGHTED) {
                const long long bits_left = (long long)a.k * a.tau - (long long)p * N;
                const int n_reg = bits_left >= N ? kX4Regs : (int)((bits_left + 15) >> 4);  // registers that hold table coordinates
                switch (a.tau) {
                    case 1: x4_weights<0>(a, v, p, n_reg, c, t, t_ok); break;
                    case 2: x4_weights<1>(a, v, p, n_reg, c, t, t_ok); break;
                    case 4: x4_weights<2>(a, v, p, n_reg, c, t, t_ok); break;
                    case 8: x4_weights<3>(a, v, p, n_reg, c, t, t_ok); break;
                    default: x4_weights<4>(a, v, p, n_reg, c, t, t_ok); break;
                }
            }
            lo = x4_c_order(lo);
            hi = x4_c_order(hi);
            // lane m: halfword m of projection p of tokens 0, 1 (lo) and 2, 3 (hi)
            const uint32_t hb = (uint32_t)(uintptr_t)bits_wave + 2u * (uint32_t)(p * 64 + (int)lane);
            *reinterpret_cast<lds_u16 *>((uintptr_t)hb) = (uint16_t)lo;
            *reinterpret_cast<lds_u16 *>((uintptr_t)(hb + 4u * W)) = (uint16_t)(lo >> 16);
            *reinterpret_cast<lds_u16 *>((uintptr_t)(hb + 8u * W)) = (uint16_t)hi;
            *reinterpret_cast<lds_u16 *>((uintptr_t)(hb + 12u * W)) = (uint16_t)(hi >> 16);
        }
        wave_lds_fence();

        // ---- a4: code j = bits [j*tau, (j+1)*tau), little-endian; the 16 lanes of a row share its codes ----
        if (t_ok) {
            const unsigned q = lane & 15u;
            if (a.packed) {
                for (int s = (int)q; s < a.k / 2; s += 16)
                    a.packed[(long long)s * a.n_pad + t] = (hash_code_at(bits_row, 2u * s, a.tau) << kPackedShift) |
                                                           (hash_code_at(bits_row, 2u * s + 1u, a.tau) << (16 + kPackedShift));
            } else {
                for (int j = (int)q; j < a.k; j += 16)
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
