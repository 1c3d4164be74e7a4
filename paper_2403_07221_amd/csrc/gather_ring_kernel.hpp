// LDS-staged gather with bank-conflict-free row reads, for prepared (slice-major) tables of up to 256 rows
// (tau <= 8), plain sum:
//   y[t][:] = sum_{j<k} tables[j][code[t][j]][:]        (Sec. 3.1, eq. "lookup")
// Runs on request only (option gather_path = 4): measured on the RoBERTa-base shape (16384 tokens, k = 96,
// d_out = 768) it takes 99 us + 11 us for its code re-pack against 90 us for gather_lds_kernel.  Its row reads
// are conflict-free (measured alone: 135-140 TB/s over the chip against 69-80 TB/s for rows picked at random),
// but both kernels turn out to be bound by the four vector adds per 16 bytes read (a stand-alone read-and-add
// loop of this kernel's pattern sits at the vector-ALU issue rate: 0.43 us per table for 12 token slots), and
// this one pays a barrier, an LDS write and two buffer loads per table on top, and a burst of output stores at
// the end of its single pass.  Kept because it is the measured answer to "take the bank conflicts out".
//
// How the reads are made conflict-free:
//
//   * A workgroup (1024 threads, or 512 with twice the registers) owns one 64-byte column slice and a chunk of
//     up to THREADS/4 * TOK tokens.  A token group is 4 lanes (one quad); the 4 groups of a 16-lane pass have
//     lags 0, 1, 2, 3: at step h
//     a group of lag p adds table h - p.  In LDS the slices of four consecutive tables are interleaved
//     at a row stride of 256 bytes -- table j's row r sits at
//         ((j >> 2) & 1) * 64 KB + r * 256 + (j & 3) * 64
//     -- so the four groups of a pass read four different 64-byte bank quarters whatever rows they pick.
//     Each accumulator still adds its tables in the order j = 0, 1, .., k-1 in fp32, so y is bit-equal to
//     the plain sequential sum; lagging groups start up to 3 steps late and finish up to 3 steps late.
//   * The LDS holds a ring of 8 table slices (2 x 64 KB).  During step h the tables h-3 .. h are being
//     read and the tables h+1 .. h+4 are being written: a table's 16 KB arrive in four pieces per lane
//     over the four steps before its first use.  The pieces travel memory -> registers -> LDS (a
//     buffer load two steps ahead of its ds_write_b128), not through the LDS-DMA path: a DMA
//     instruction writes 1 KB of consecutive LDS, which in this layout belongs to four different tables
//     and would have to be issued with three quarters of its lanes masked off -- measured at the
//     full per-instruction cost (17 clocks per wave instruction whatever the mask).  The lanes of class
//     c = (lane / 4) % 4 fill the tables j = c (mod 4), so the 16 lanes of a write pass also cover four bank
//     quarters.
//   * One barrier per step (LDS-only fence: the global loads in flight are not waited for).  The last
//     read batch of a step is consumed after the barrier, overlapping the first reads of the next step.
//
// Codes come pre-shifted by the lag ("lagged packed" layout, written by repack_codes_lag_kernel): word
// w of token t holds the LDS row offsets (code << 8) of tables 2w - p(t) and 2w + 1 - p(t), p(t) = (t / 4) % 4,
// zero where that table does not exist, so at step h every lane uses half h % 2 of word h / 2.  Chunks
// start at multiples of 16 tokens, which makes a token's lag a function of its index alone.  As in the
// other staged kernel the words are quad-shared: a lane keeps those of the token slots 4m + (lane % 4).
//
// Before a lagging group's first table and after its last one it still reads rows of whatever the ring holds
// (always inside the staging area) but does not add them.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "elem16.hpp"

#include "gather_kernel.hpp"
#include "gather_lds_kernel.hpp"
#include "hash_kernel.hpp"

namespace lffn {

constexpr int kRingLdsBytes = 128 * 1024;       // 8 table slices of 256 rows x 64 bytes
constexpr int kRingShift = 8;                   // packed codes are scaled by the 256-byte LDS row stride
constexpr int kRingAhead = 2;                   // a table piece is loaded this many steps before it is written (2 or 4;
                                                // 4 measured no faster and costs 8 more registers)

// words per token of the lagged packed layout: tables -3 .. k+2 in pairs, and two more (zero) words so that
// the kernel's look-ahead of two pairs needs no bound check
__host__ __device__ inline long long ring_code_words(int k) { return ((long long)(k + 2) >> 1) + 3; }

struct GatherRingArgs {
    const uint32_t *packed;  // lagged packed codes [ring_code_words(k)][n_pad]
    long long n_pad;
    const char *tables;      // prepared tables: [slice of pw bytes][k][rows][pw], fp32
    void *y;   // [n][d_out] fp32, or bf16 / IEEE half when y_kind says so
    int y_kind;
    long long n;
    int k, tau, d_out;
    int nvec;            // 16-byte pieces per row
    int n_slices;        // 64-byte column slices: ceil(nvec / 4)
    int token_splits;    // a unit = (slice, one of token_splits token ranges)
    int n_units;
    int blocks_per_xcd;
    uint32_t row_stride;             // pw
    uint32_t spp;                    // 64-byte slices per prepared piece: pw / 64
    uint32_t table_stride;           // rows * pw
    unsigned long long slice_stride; // k * rows * pw
};

// word 3 of a raw buffer resource: 32-bit data format, offsets checked against the byte count
constexpr int kBufferRsrcFlags = 0x00020000;

// THREADS = 1024 (4 waves per SIMD, 128 registers per lane: up to 12 token slots) or 512 (2 waves per SIMD, 256
// registers: up to 32 slots); a chunk holds THREADS / 4 * TOK tokens either way.
template <int THREADS, int TOK>
__global__ __launch_bounds__(THREADS) void gather_ring_kernel(GatherRingArgs a)
{
    static_assert(THREADS == 1024 || THREADS == 512, "one workgroup per CU, 16 or 8 waves");
    static_assert(TOK >= 1 && TOK <= 32, "token slots per lane");
    constexpr int G = THREADS / 4;      // token groups (quads) per workgroup
    // Token slots.  The first 4 * NQ slots come in quads: slot i of group g is token c0 + 4G * (i / 4) + 4g + i % 4,
    // and the code words of a quad of slots are shared by the group's four lanes (lane r keeps slot 4m + r in
    // register m; a use is a DPP quad broadcast).  The last NT = TOK % 4 slots are single: slot 4 * NQ + j of group
    // g is token c0 + 4G * NQ + G * j + o(g), o(g) = 16 * (g / 16) + 4 * (g % 4) + (g / 4) % 4 -- a permutation of
    // 0 .. G-1 under which the token's lag class (token / 4) % 4 is still g % 4 -- and every lane of the group
    // holds that slot's word.  A chunk is therefore any G * TOK consecutive tokens.
    constexpr int NQ = TOK / 4, NT = TOK % 4;
    constexpr int WQ = NQ + NT;         // code registers per pair of tables
    constexpr int RB = THREADS == 1024 ? 2 : 4;  // row reads per batch
    constexpr int NB = (TOK + RB - 1) / RB;  // batches per step; batch b of step s uses read buffer (s * NB + b) % 2
    constexpr int D = kRingAhead;
    constexpr int FROWS = THREADS / 16;      // rows one fill instruction of the workgroup covers
    constexpr int PPS = 64 / FROWS;          // fill pieces per lane and step (a step fills 64 rows of 4 tables)
    static_assert(D == 4 || D == 2, "the fill registers rotate with the 4-step unrolled loop");
    extern __shared__ uint4 sbuf[];
    // LDS addresses below are formed with XOR on bit 16 (the two halves of the ring), relative to the start of
    // the dynamic LDS; this kernel has no static LDS, so that start is address 0
    if ((uint32_t)(uintptr_t)sbuf != 0u) return;
    const uint32_t tid = threadIdx.x;
    const uint32_t q = tid & 3u, g = tid >> 2;
    const uint32_t p = g & 3u;   // lag of this lane's token group = class of the tables this lane fills
    const uint32_t n = (uint32_t)a.n;  // the host uses this kernel only for n < 2^31
    const int k = a.k;

    // ---- which (unit, token range) pairs does this workgroup own?  (as in gather_lds_kernel) ----
    const uint32_t xcd = blockIdx.x % kXcds;
    const uint32_t cb = blockIdx.x / kXcds;
    const uint32_t Bx = (uint32_t)a.blocks_per_xcd;
    if ((uint32_t)a.n_units <= xcd) return;
    const uint32_t m = ((uint32_t)a.n_units - xcd + kXcds - 1) / kXcds;
    uint32_t u_first, u_step, u_end, part, parts;
    if (m >= Bx) {
        u_first = cb;
        u_step = Bx;
        u_end = m;
        part = 0;
        parts = 1;
    } else {
        u_first = cb * m / Bx;
        u_step = 1;
        u_end = u_first + 1;
        const uint32_t first_blk = (u_first * Bx + m - 1) / m;
        const uint32_t next_blk = ((u_first + 1) * Bx + m - 1) / m;
        part = cb - first_blk;
        parts = next_blk - first_blk;
    }
    const uint32_t n16 = (n + 15u) / 16u;  // token ranges are split in units of 16 tokens

    // ---- fill role: element e of this lane's class is piece e % 4 of table p + 4 * (e / 4): the rows
    // frow + r * FROWS + 64 * (e % 4), r < PPS, 16 bytes at column q of the 64-byte slice.  Element e is loaded at step
    // e + p - 4 - D and written to LDS at step e + p - 4.  The loads are buffer loads on the slice (all k
    // tables of it, contiguous): an element past the last table is out of range and reads as zero, and
    // writing it is harmless -- its ring slot is free by the same rule as for a real table and nothing that
    // is stored ever reads it.  So no fill needs a check (nor do 128-row tables, whose pieces 2 and 3 land in
    // rows that no code selects).
    const uint32_t frow = tid >> 4;
    const uint32_t fill_dst0 = (frow << 8) + (p << 6) + (q << 4);                    // + ((e & 7) << 14)
    const uint32_t fill_src0 = p * a.table_stride + frow * a.row_stride + (q << 4);  // + (e / 4) * src_quad + (e % 4) * src_piece
    const uint32_t src_piece = 64u * a.row_stride, src_quad = 4u * a.table_stride;
    // per-lane constants of the 4-step unrolled loop, step s = h % 4 of the quad h = 4m .. 4m + 3:
    //   (the LDS address the lane writes at step h, fill_dst0 + ((h + 4 - p) % 8 << 14), is formed in the step from
    //   the step number: one register instead of four)
    //   tb0[s]  LDS address of the lane's piece of row 0 of the table it adds at step 4m + s, m even
    //   (the source offset of the element the lane loads at step h is formed in the step as well)
    uint32_t tb0[4];
#pragma unroll
    for (int s4 = 0; s4 < 4; ++s4) {
        const uint32_t jr = (uint32_t)(s4 - (int)p);       // table added at step s4 (m = 0), modulo 8
        tb0[s4] = (q << 4) + ((jr & 3u) << 6) + ((jr & 4u) << 14);
    }
    // source offset of element e: fill_src0 + (e / 4) * src_quad + (e % 4) * src_piece, both strides powers of two
    const uint32_t lg_piece = 31u - (uint32_t)__builtin_clz(src_piece), lg_quad = 31u - (uint32_t)__builtin_clz(src_quad);
    auto fill_src = [&](uint32_t e) -> uint32_t { return fill_src0 + ((e >> 2) << lg_quad) + ((e & 3u) << lg_piece); };
    auto lds_u4 = [](uint32_t addr) { return reinterpret_cast<__attribute__((address_space(3))) u32x4 *>((uintptr_t)addr); };

    for (uint32_t ui = u_first; ui < u_end; ui += u_step) {
        const uint32_t unit = ui * kXcds + xcd;
        uint32_t slice = unit % (uint32_t)a.n_slices;
        const uint32_t split = unit / (uint32_t)a.n_slices;
        // the two 64-byte halves of a 128-byte line go to units that run side by side on one XCD
        if ((uint32_t)a.n_slices % 16u == 0u) {
            const uint32_t i = slice / kXcds;
            slice = ((i >> 1) * kXcds + slice % kXcds) * 2u + (i & 1u);
        }
        const uint32_t s0 = split_at(n16, (uint32_t)a.token_splits, split);
        const uint32_t s1 = split_at(n16, (uint32_t)a.token_splits, split + 1);
        const uint32_t r0 = (s0 + split_at(s1 - s0, parts, part)) * 16u;
        uint32_t r1 = (s0 + split_at(s1 - s0, parts, part + 1)) * 16u;
        if (r1 > n) r1 = n;
        if (r1 <= r0) continue;  // uniform over the workgroup

        const uint32_t half_off = (slice % a.spp) * 64u;
        const char *slice_base = a.tables + (size_t)(slice / a.spp) * (size_t)a.slice_stride + half_off;  // uniform
        const __amdgpu_buffer_rsrc_t trs = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<char *>(slice_base), 0, (int)((uint32_t)a.slice_stride - half_off), kBufferRsrcFlags);

        const uint32_t len = r1 - r0;
        const uint32_t nchunks = (len + G * TOK - 1) / (G * TOK);
        const uint32_t len16 = (len + 15u) / 16u;
        for (uint32_t ch = 0; ch < nchunks; ++ch) {
            const uint32_t c0 = r0 + split_at(len16, nchunks, ch) * 16u;
            uint32_t c1 = r0 + split_at(len16, nchunks, ch + 1) * 16u;
            if (c1 > r1) c1 = r1;
            const uint32_t lane_tok = (4u * g + q) * 4u;  // byte offset of the lane's token in a quad register's row
            const uint32_t tail_tok = (16u * (g >> 4) + 4u * (g & 3u) + ((g >> 2) & 3u)) * 4u;  // same for a single slot: o(g)
            auto load_codes = [&](uint32_t w, uint32_t(&cr)[WQ]) {
                // word row w, tokens c0 .. c0 + G * TOK (inside the padded row): a buffer of its own
                const char *base = reinterpret_cast<const char *>(a.packed) + ((size_t)w * a.n_pad + c0) * 4u;  // uniform
                const __amdgpu_buffer_rsrc_t crs =
                    __builtin_amdgcn_make_buffer_rsrc(const_cast<char *>(base), 0, 4 * G * TOK, kBufferRsrcFlags);
#pragma unroll
                for (int mm = 0; mm < NQ; ++mm) cr[mm] = __builtin_amdgcn_raw_buffer_load_b32(crs, lane_tok, mm * (16 * G), 0);
#pragma unroll
                for (int j = 0; j < NT; ++j)
                    cr[NQ + j] = __builtin_amdgcn_raw_buffer_load_b32(crs, tail_tok, NQ * (16 * G) + j * (4 * G), 0);
            };

            Acc<false> acc[TOK];
#pragma unroll
            for (int i = 0; i < TOK; ++i) acc[i].zero();
            u32x4 fr[D][PPS];           // table pieces in flight: fr[h % D] is written to LDS at step h
            uint32_t crA[WQ], crB[WQ];  // code words of the steps 4m, 4m + 1 / 4m + 2, 4m + 3
            uint32_t half[WQ];          // the current step's 16-bit halves of the code words
            uint4 rd[2][RB];            // row reads in flight

            auto issue = [&](int b, uint32_t tb, uint4(&dst)[RB]) {
#pragma unroll
                for (int i = 0; i < RB; ++i) {
                    const int slot = b * RB + i;
                    if (slot < TOK) {
                        const uint32_t off = slot < 4 * NQ ? quad_bcast(half[slot >> 2], slot & 3) : half[NQ + slot - 4 * NQ];
                        const u32x4 v = *lds_u4(tb + off);
                        dst[i] = make_uint4(v.x, v.y, v.z, v.w);
                    }
                }
            };
            auto consume = [&](int b, const uint4(&src)[RB]) {
#pragma unroll
                for (int i = 0; i < RB; ++i) {
                    if (b * RB + i < TOK) {
                        acc[b * RB + i].add(src[i]);
                        acc[b * RB + i].pin();
                    }
                }
            };
            auto fill_load = [&](u32x4(&dst)[PPS], uint32_t voff, uint32_t soff) {
#pragma unroll
                for (int r = 0; r < PPS; ++r)
                    dst[r] = __builtin_amdgcn_raw_buffer_load_b128(trs, voff + (uint32_t)r * (FROWS * a.row_stride), soff, 0);
            };
            auto fill_store = [&](uint32_t addr, const u32x4(&src)[PPS]) {
#pragma unroll
                for (int r = 0; r < PPS; ++r) *lds_u4(addr + (uint32_t)r * (FROWS * 256u)) = src[r];
            };
            auto barrier = [&]() {
                // LDS operations only: the global loads in flight stay in flight
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
                __builtin_amdgcn_s_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
            };
            auto store_y = [&]() {
                // the output addresses are formed here, from a lane index the compiler cannot see through: left
                // alone it computes all of them before the main loop and keeps them in registers across it
                uint32_t lt = tid;
                asm volatile("" : "+v"(lt));
                const uint32_t sg = lt >> 2, sq = lt & 3u, svec = slice * 4u + sq;
                const uint32_t so = 16u * (sg >> 4) + 4u * (sg & 3u) + ((sg >> 2) & 3u);
                if (svec < (uint32_t)a.nvec) {
#pragma unroll
                    for (int i = 0; i < TOK; ++i) {
                        const uint32_t t = i < 4 * NQ ? c0 + (4u * G) * (uint32_t)(i >> 2) + 4u * sg + (uint32_t)(i & 3)
                                                      : c0 + (4u * G) * NQ + (uint32_t)G * (uint32_t)(i - 4 * NQ) + so;
                        if (t >= c1) continue;
                        store_y4(a.y, (size_t)t * a.d_out + (size_t)svec * 4u, acc[i].f[0], acc[i].f[1], acc[i].f[2],
                                 acc[i].f[3], a.y_kind);
                    }
                }
            };

            // ---- prologue: the fills of the steps before step 0 (no reads yet) --------------------------
            barrier();  // the previous chunk's last reads are done before its slices are overwritten
            {
                // (per-lane values of the prologue are formed from an opaque copy of the lane index, or the
                // compiler keeps them all in registers across the main loop of every chunk)
                uint32_t lt = tid;
                asm volatile("" : "+v"(lt));
                const uint32_t pq = (lt >> 2) & 3u, pfrow = lt >> 4;
                const uint32_t pdst0 = (pfrow << 8) + (pq << 6) + ((lt & 3u) << 4);
                const uint32_t psrc0 = pq * a.table_stride + pfrow * a.row_stride + ((lt & 3u) << 4);
                load_codes(0, crA);
                load_codes(1, crB);
                // steps -4 - D .. -5 load only, steps -4 .. -1 write what was loaded D steps before and load
#pragma unroll
                for (int hh = -4 - D; hh < 0; ++hh) {
                    const int ew = hh + 4 - (int)pq, el = ew + D;  // elements written / loaded at step hh
                    u32x4(&reg)[PPS] = fr[(hh + 8) % D];
                    if (hh >= -4 && ew >= 0) fill_store(pdst0 + ((uint32_t)ew << 14), reg);
                    if (el >= 0) fill_load(reg, psrc0 + (uint32_t)(el >> 2) * src_quad + ((uint32_t)el & 3u) * src_piece, 0);
                }
            }
            const int h_last = k + 2;  // the step in which the groups of lag 3 add table k - 1
            bool pending = false;       // is the last read batch of the step before still to be added?

            // One step h = 4 * quad + S.  EDGE: one of the first or last steps, in which some groups have not
            // started yet (lag > h) or have finished (h - lag > k - 1): every lane reads (whatever rows the ring
            // holds), only the groups in range add, and nothing stays pending.  Otherwise the last batch stays
            // pending and is added behind the next step's first reads.
            auto step = [&](auto s_tag, auto edge_tag, int h, bool pend) {
                constexpr int S = decltype(s_tag)::value;
                constexpr bool EDGE = decltype(edge_tag)::value;
                uint32_t(&cr)[WQ] = (S & 2) ? crB : crA;
                const uint32_t tog = ((uint32_t)h & 4u) << 14;       // odd quads use the other half of the ring
                barrier();
                fill_store(fill_dst0 + ((((uint32_t)(h + 4) - p) & 7u) << 14), fr[S % D]);  // element h + 4 - p
                fill_load(fr[S % D], fill_src((uint32_t)(h + 4 + D) - p), 0);  // element h + 4 - p + D
#pragma unroll
                for (int mm = 0; mm < WQ; ++mm) half[mm] = (S & 1) ? (cr[mm] >> 16) : (cr[mm] & 0xFFFFu);
                const uint32_t tb = tb0[S] ^ tog;
                constexpr int B0 = (S * NB) & 1;  // read buffer of this step's first batch
                issue(0, tb, rd[B0]);
                if (pend) consume(NB - 1, rd[B0 ^ 1]);  // the step before ended on the other buffer
                if constexpr (!EDGE) {
#pragma unroll
                    for (int b = 1; b < NB; ++b) {
                        issue(b, tb, rd[(B0 + b) & 1]);
                        consume(b - 1, rd[(B0 + b - 1) & 1]);
                    }
                } else {
                    const int j = h - (int)p;  // the table this lane's group is at
                    const bool in_range = j >= 0 && j < k;
#pragma unroll
                    for (int b = 1; b < NB; ++b) {
                        issue(b, tb, rd[(B0 + b) & 1]);
                        if (in_range) consume(b - 1, rd[(B0 + b - 1) & 1]);
                    }
                    if (in_range) consume(NB - 1, rd[(B0 + NB - 1) & 1]);
                }
                if constexpr (S & 1) load_codes((uint32_t)(h >> 1) + 2u, cr);  // the pair of steps h + 3, h + 4
            };
            using yes = std::integral_constant<bool, true>;
            using no = std::integral_constant<bool, false>;
            using i0 = std::integral_constant<int, 0>;
            using i1 = std::integral_constant<int, 1>;
            using i2 = std::integral_constant<int, 2>;
            using i3 = std::integral_constant<int, 3>;

            step(i0{}, yes{}, 0, false);
            step(i1{}, yes{}, 1, false);
            step(i2{}, yes{}, 2, false);
            step(i3{}, yes{}, 3, false);
            int h = 4;
            for (; h + 3 < k - 1; h += 4) {
                step(i0{}, no{}, h, pending);
                step(i1{}, no{}, h + 1, true);
                step(i2{}, no{}, h + 2, true);
                step(i3{}, no{}, h + 3, true);
                pending = true;
            }
            for (; h <= h_last; h += 4) {
                step(i0{}, yes{}, h, pending);
                pending = false;
                if (h + 1 > h_last) break;
                step(i1{}, yes{}, h + 1, false);
                if (h + 2 > h_last) break;
                step(i2{}, yes{}, h + 2, false);
                if (h + 3 > h_last) break;
                step(i3{}, yes{}, h + 3, false);
            }
            store_y();
        }
    }
}

#if !defined(LFFN_PART) || LFFN_PART == 0  // a plain function: defined by part 0 only of a build in parts
// ABI codes [n][k] -> lagged packed codes [ring_code_words(k)][n_pad] for gather_ring_kernel: word w of
// token t = the codes of tables 2w - p and 2w + 1 - p (p = (t / 4) % 4), reduced modulo 2^tau and scaled by
// 2^shift, in the low / high half; zero for tables outside [0, k) and for the token padding [n, n_pad).
// One workgroup per 64 tokens: their code rows are one contiguous run, read into LDS as it lies.
__global__ __launch_bounds__(256) void repack_codes_lag_kernel(const uint16_t *codes, uint32_t *packed, long long n,
                                                               long long n_pad, int k, int tau, int shift)
{
    extern __shared__ uint16_t tile[];  // [64][k + 1]  (odd word stride for k even: no bank conflicts on the column reads)
    const int ks = k | 1;
    const uint32_t cmask = (1u << tau) - 1u;
    const long long W = ring_code_words(k);
    const long long blocks = (n_pad + 63) / 64;
    for (long long blk = blockIdx.x; blk < blocks; blk += gridDim.x) {
        const long long t0 = blk * 64;
        __syncthreads();
        const long long cnt = (t0 < n ? (n - t0 < 64 ? n - t0 : 64) : 0) * k;  // codes of this block's tokens
        for (long long i = threadIdx.x; i < cnt; i += blockDim.x) tile[(i / k) * ks + (i % k)] = codes[t0 * k + i];
        __syncthreads();
        const int tt = threadIdx.x & 63;
        const long long t = t0 + tt;
        const int p = (int)((t >> 2) & 3);
        for (long long w = threadIdx.x >> 6; w < W; w += blockDim.x >> 6) {
            uint32_t word = 0;
            if (t < n) {
                const int j0 = (int)(2 * w) - p;
                if (j0 >= 0 && j0 < k) word |= ((uint32_t)tile[tt * ks + j0] & cmask) << shift;
                if (j0 + 1 >= 0 && j0 + 1 < k) word |= ((uint32_t)tile[tt * ks + j0 + 1] & cmask) << (16 + shift);
            }
            if (t < n_pad) packed[w * n_pad + t] = word;
        }
    }
}
#endif

}  // namespace lffn
