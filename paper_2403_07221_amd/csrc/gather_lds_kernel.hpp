// LDS-staged gather for tables of 2^7 .. 2^10 rows (k even, fp32 rows; for an odd k the host gives this
// kernel the first k - 1 tables and lets the direct kernel add the last one onto its sums):
//   y[t][:] = sum_{j<k} tables[j][code[t][j]][:]        (Sec. 3.1, eq. "lookup")
//
// With tau = 8 a table has only 256 rows, so a batch of thousands of tokens
// picks every row many times.  A 1024-thread workgroup owns one column slice
// (128 bytes of every row up to tau = 8 or 9, 64 bytes from tau = 8 or 9 on)
// and a chunk of tokens.  Tables are taken one stage at a time: the slice of
// all 2^tau rows of two tables (one table when it fills a 64 KB buffer) is copied
// into LDS once by global_load_lds (memory -> LDS without a
// trip through registers), double-buffered so that stage s+1 streams in while
// stage s is consumed.  Every (token, 16-byte piece) lane then reads its
// selected row from LDS with one ds_read_b128 (the lanes of a token read one
// contiguous row piece) and adds it to its fp32 accumulators.  Each
// output element is still the sequential fp32 sum over j = 0..k-1, so results
// equal the direct kernel's bit for bit, while the L2 -> CU traffic drops from
// one row per (token, table) to one row per (chunk, table, row).
//
// Codes come in the packed layout written by the hash kernel (one 32-bit word
// per token and stage holding both tables' LDS row offsets, token-contiguous).
// The eight lanes of a token would all hold the same word, so the words are
// quad-shared: each lane keeps only those of the token slots i with i % 4 ==
// its position in its quad, and a use takes the word through a DPP quad
// broadcast -- a quarter of the registers and load instructions, one cache
// line per load.  The vector-memory instructions of a stage (next
// stage's row copies and codes) are issued a few at a time between the LDS
// read batches: a wave issues in order, so a burst of them at the top of the
// stage would hold every wave at the texture-address queue while LDS and the
// vector ALU sit idle.
//
// Weighted form (Sec. 4: y = sum_j w_j T_j[code_j]): the fp32 weights come table-major and
// token-contiguous (wpk[j][n_pad]) and are quad-shared like the code words; each row is
// accumulated with one fused multiply-add per element.
//
// bf16 tables: the staged copy is fp32.  Widening inside this kernel (per stage and workgroup, through
// registers and LDS writes) measured no faster than the direct kernel, and the tables are learned
// constants, so the widening happens once, outside the forward pass: prepare_tables_kernel (below) writes an
// fp32, slice-major copy that this kernel and the direct kernel read.
//
// Work distribution is static and XCD-aware: slice-units are dealt to the
// eight XCDs round-robin (block b runs on XCD b % 8), and the workgroups of
// one XCD split its units' token ranges evenly, so every CU gets one chunk of
// near-equal size and the slice a CU streams stays in its XCD's L2.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "elem16.hpp"

#include <type_traits>

#include "gather_kernel.hpp"
#include "hash_kernel.hpp"

namespace lffn {

constexpr int kLdsThreads = 1024;
// Lanes per token SW (8 or 4): a token group reads one SW*16-byte row piece, the workgroup owns a
// column slice of that width and kLdsThreads / SW token groups.
constexpr int kLdsBufBytes = 64 * 1024;      // one staging buffer (two of them are in use)
constexpr int kLdsMaxTok = 16;               // token slots per lane the packed padding allows for
#ifndef LFFN_LDS_RB
#define LFFN_LDS_RB 3
#endif
#ifndef LFFN_LDS_CO
#define LFFN_LDS_CO 0   // read batch in which the first code load of the next stage is issued
#endif
#ifndef LFFN_LDS_WO
#define LFFN_LDS_WO 4   // same for its first weight load
#endif

struct GatherLdsArgs {
    const uint32_t *packed;  // [k/2][n_pad] packed codes (see hash_kernel.hpp)
    const float *wpk;        // weighted form: [k][n_pad] weights, table-major (wpk_index); multi-probe form:
                             // [k][1+tau][n_pad] shares.  The token padding [n, n_pad) is never initialised:
                             // slots past a chunk's end multiply it into accumulators that are never stored.
    long long n_pad;
    const char *tables;      // fp32 rows, row-major [k][rows][d_out] or the slice-major prepared layout
    void *y;            // [n][d_out] fp32, or bf16 / IEEE half when y_kind says so
    int y_kind;         // 0 fp32, 1 bf16, 2 IEEE half
    long long n;
    int k, tau, d_out;
    int nvec;           // 16-byte pieces per row
    int n_slices;       // ceil(nvec / lanes per token)
    int token_splits;   // a unit = (slice, one of token_splits equal token ranges)
    int n_units;        // n_slices * token_splits
    int blocks_per_xcd; // gridDim.x / kXcds
    // Where the piece (slice, table j, row r, 16-byte piece q) lives:
    //   tables + (slice / spp) * slice_stride + (slice % spp) * SW*16 + j * table_stride + r * row_stride + q*16
    // row-major tables: spp = 1, slice_stride = SW*16, row_stride = d_out*4, table_stride = rows * row_stride;
    // prepared tables (one slice of all tables contiguous, PW bytes per row piece): spp = PW / (SW*16),
    // slice_stride = k * rows * PW, row_stride = PW, table_stride = rows * PW.
    uint32_t row_stride;
    uint32_t spp;
    unsigned long long table_stride;
    unsigned long long slice_stride;
};

// bytes of LDS the kernel needs: two buffers (sw = lanes per token)
__host__ __device__ inline size_t gather_lds_bytes(int tau, int sw)
{
    const size_t tbl = ((size_t)16 * sw) << tau;
    return 2 * (2 * tbl <= (size_t)kLdsBufBytes ? 2 * tbl : tbl);
}

// balanced split of [0, len) into `parts` pieces: start of piece i (32-bit arithmetic only)
__device__ __forceinline__ uint32_t split_at(uint32_t len, uint32_t parts, uint32_t i)
{
    const uint32_t base = len / parts, rem = len - base * parts;
    return base * i + (i < rem ? i : rem);
}

// One global_load_lds_dwordx4: every active lane copies 16 bytes from gbase + voff to LDS byte
// address lds_base + 16 * lane (lds_base and gbase wave-uniform).  Issued through inline asm so
// that the compiler does not serialise later LDS reads of the *other* buffer behind it; the
// caller waits with s_waitcnt vmcnt(0) before the barrier that publishes the buffer.
__device__ __forceinline__ void lds_dma16(const char *gbase, uint32_t voff, uint32_t lds_base)
{
    const uint32_t m = __builtin_amdgcn_readfirstlane(lds_base);
    // M0 is written here, so it is named as clobbered: the compiler then keeps none of its own M0
    // values live across the statement (it warns that M0 is a reserved register; that is the point).
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 1\n\tglobal_load_lds_dwordx4 %1, %2"
                 :
                 : "s"(m), "v"(voff), "s"(gbase)
                 : "memory", "m0");
#pragma clang diagnostic pop
}

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// batch that issues the i-th deferred load of a stage with nbt batches: i itself, wrapped
__host__ __device__ constexpr int vm_slot(int i, int nbt) { return i % nbt; }

// value of `v` in lane Q of the caller's quad (DPP quad_perm [Q,Q,Q,Q])
template <int Q>
__device__ __forceinline__ float quad_bcast(float v)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), Q * 0x55, 0xF, 0xF, true));
}
__device__ __forceinline__ float quad_bcast(float v, int q)
{
    return q == 0 ? quad_bcast<0>(v) : q == 1 ? quad_bcast<1>(v) : q == 2 ? quad_bcast<2>(v) : quad_bcast<3>(v);
}
__device__ __forceinline__ uint32_t quad_bcast(uint32_t v, int q)
{
    return __float_as_uint(quad_bcast(__uint_as_float(v), q));
}

// FR = 16 KB copy rounds per table slice (one round = every thread copies 16 bytes = G rows): 1, 2, 4.
// Tables per stage TPS: two (FR <= 2: both halves of a code word are consumed in one stage) or one
// (FR = 4: a 64 KB slice fills a buffer; even stages take the low half of the code word, odd stages
// the high half).  SW = lanes per token: 8 (128-byte column slices; tau = 7, 8, 9 <-> FR = 1, 2, 4)
// or 4 (64-byte slices; tau = 8, 9, 10 <-> FR = 1, 2, 4).  The packed codes must be scaled by the
// row-piece bytes: code << 7 for SW = 8 (what the hash kernels write), code << 6 for SW = 4 (written
// by the re-pack kernel from ABI codes; 1023 << 7 would not fit the 16-bit half of a code word).
// PROBES (with WEIGHTED): the multi-probe form (Sec. 3.1, eq. "partial_softmax"): every stage is swept
// 1 + tau times, sweep p reading the rows code ^ flip(p) with the shares of probe p
// (wpk[(j * (1 + tau) + p) * n_pad + t]); the staged slice is copied once per stage.
template <int TOK, int FR, bool WEIGHTED, int SW = 8, bool PROBES = false>
__global__ __launch_bounds__(kLdsThreads) void gather_lds_kernel(GatherLdsArgs a)
{
    static_assert(!PROBES || WEIGHTED, "the multi-probe form carries weights");
    static_assert(TOK <= kLdsMaxTok, "packed-code padding covers 16 token slots");
    static_assert(FR == 1 || FR == 2 || FR == 4, "table slices of 16, 32 or 64 KB");
    static_assert(SW == 8 || SW == 4, "128- or 64-byte column slices");
    constexpr int TPS = FR <= 2 ? 2 : 1;
    constexpr int G = kLdsThreads / SW;   // token groups per workgroup = rows per copy round
    constexpr uint32_t PIECE = SW * 16u;  // bytes of a row inside the slice
    static_assert(TPS * FR * 16 * 1024 <= kLdsBufBytes, "a stage fits one buffer");
    extern __shared__ uint4 sbuf[];
    const uint32_t tid = threadIdx.x;
    const uint32_t wave = tid >> 6;
    const uint32_t g = tid / SW, q = tid % SW;
    const uint32_t rows = (uint32_t)G * FR;          // == 1 << a.tau (checked by the host)
    const uint32_t tbl_bytes = rows * PIECE;         // one table slice in LDS
    const uint32_t buf_bytes = tbl_bytes * TPS;  // one buffer (one stage)
    const uint32_t n = (uint32_t)a.n;                // the host uses this kernel only for n < 2^31
    const uint32_t nstages = (uint32_t)a.k / TPS;
    const uint32_t lds0 = (uint32_t)(uintptr_t)sbuf;  // LDS byte address of the staging area

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
        uint32_t slice = unit % (uint32_t)a.n_slices;
        const uint32_t split = unit / (uint32_t)a.n_slices;
        if constexpr (SW == 4) {
            // A 64-byte slice is half of a 128-byte cache line.  Dealt round-robin, the two halves of
            // every line would go to different XCDs and each L2 would fetch the whole line.  With the
            // slice count a multiple of 16 (then slice % 8 is the XCD) the XCD's units 2i and 2i + 1,
            // which run side by side, take the two halves of the same lines instead.
            if ((uint32_t)a.n_slices % 16u == 0u) {
                const uint32_t i = slice / kXcds;
                slice = ((i >> 1) * kXcds + slice % kXcds) * 2u + (i & 1u);
            }
        }
        const uint32_t s0 = split_at(n, (uint32_t)a.token_splits, split);
        const uint32_t s1 = split_at(n, (uint32_t)a.token_splits, split + 1);
        const uint32_t r0 = s0 + split_at(s1 - s0, parts, part), r1 = s0 + split_at(s1 - s0, parts, part + 1);
        if (r1 <= r0) continue;  // uniform over the workgroup

        const uint32_t vec = slice * (uint32_t)SW + q;
        const bool vec_ok = vec < (uint32_t)a.nvec;

        // Fill role of this thread: piece (row g, column piece q) of each group of 128 rows.
        // Lanes whose piece lies outside the row (ragged last slice) copy piece 0 instead: they
        // never store a result, and this keeps the copy free of divergent control flow.
        // Offsets inside one table fit 32 bits.
        const uint32_t foff = g * a.row_stride + (vec_ok ? q : 0u) * 16u;
        const size_t table_stride = (size_t)a.table_stride;
        const char *slice_base = a.tables + (size_t)(slice / a.spp) * (size_t)a.slice_stride +
                                 (size_t)(slice % a.spp) * PIECE;  // uniform
        // piece idx = table-in-stage * FR + round, of stage s, into buffer b
        auto fill_piece = [&](uint32_t s, uint32_t b, int idx) {
            const uint32_t tb = (uint32_t)idx / FR, f = (uint32_t)idx % FR;
            const char *tsrc = slice_base + (size_t)(s * TPS + tb) * table_stride +
                               (size_t)f * G * a.row_stride;  // uniform
            lds_dma16(tsrc, foff, lds0 + b * buf_bytes + tb * tbl_bytes + (f * kLdsThreads + wave * 64u) * 16u);
        };

        const uint32_t len = r1 - r0;
        const uint32_t nchunks = (len + G * TOK - 1) / (G * TOK);
        for (uint32_t ch = 0; ch < nchunks; ++ch) {
            const uint32_t c0 = r0 + split_at(len, nchunks, ch), c1 = r0 + split_at(len, nchunks, ch + 1);
            // Token slots.  The eight lanes of a token group would all hold the same code word and
            // weights, so these are quad-shared: a lane keeps those of the slots 4m + r, r = its
            // position in its quad, in register m, and a use fetches them with a DPP quad broadcast
            // (a quarter of the registers and load instructions).  Slot i of group g is token
            //   c0 + 4G*(i/4) + 4g + i%4   for the full quads of slots (i < 4*(TOK/4)),
            //   c0 + G*i + g               for the remaining TOK % 4 slots,
            // so that register m of a wave's lanes covers consecutive tokens: one or two cache lines
            // per load instruction.  Slots past the chunk end read the codes of later tokens or of the
            // zero padding (always a valid row), add them, and store nothing.
            constexpr int WQ = (TOK + 3) / 4, FQ = TOK / 4;
            const uint32_t r4 = q & 3u;
            auto slot_token = [&](int i) -> uint32_t {
                return i < 4 * FQ ? c0 + (4u * G) * (uint32_t)(i >> 2) + 4u * g + (uint32_t)(i & 3)
                                  : c0 + (uint32_t)G * (uint32_t)i + g;
            };
            const uint32_t lq_full = (4u * g + r4) * 4u;          // byte offset of the lane's token in a full quad register
            const uint32_t lq_tail = (r4 * G + g) * 4u;            // same for the tail register
            auto reg_offset = [&](int m) -> uint32_t {
                return m < FQ ? (uint32_t)m * (16u * G) + lq_full : (uint32_t)m * (16u * G) + lq_tail;
            };
            constexpr int NCR = WQ;  // code registers and code loads per stage
            auto load_code = [&](uint32_t s, int m, uint32_t(&cr)[NCR]) {
                const char *base = reinterpret_cast<const char *>(a.packed) + ((size_t)s * a.n_pad + c0) * 4u;  // uniform
                cr[m] = *reinterpret_cast<const uint32_t *>(base + reg_offset(m));
            };
            // LDS row offset of slot i in table u of the stage: the low / high half of its code word.
            // Both halves are split off the word before the broadcast (once per register and stage),
            // so a use is one DPP add and the two tables' broadcasts are distinct values.
            auto row_offset = [&](const uint32_t(&cr)[NCR], int u, int i) -> uint32_t {
                return u ? quad_bcast(cr[i >> 2] >> 16, i & 3) : quad_bcast(cr[i >> 2] & 0xFFFFu, i & 3);
            };
            // weights: table u of stage s, register m
            constexpr int NWL = TPS * WQ;
            auto load_weight = [&](uint32_t s, int i, float(&wr)[TPS][WQ]) {
                const int u = i / WQ, m = i % WQ;
                const char *base = reinterpret_cast<const char *>(a.wpk) +
                                   ((size_t)(s * TPS + (uint32_t)u) * a.n_pad + c0) * 4u;  // uniform
                wr[u][m] = *reinterpret_cast<const float *>(base + reg_offset(m));
            };

            // codes of a stage's two tables per token slot; two sets so that the next stage's codes
            // load while the current stage is consumed
            uint32_t crA[NCR], crB[NCR];
            float wA[TPS][WQ], wB[TPS][WQ];
            Acc<false> acc[TOK];
#pragma unroll
            for (int i = 0; i < TOK; ++i) acc[i].zero();

            // LDS byte address of this lane's piece of row 0, per (buffer, table-in-stage)
            const uint32_t qb = lds0 + q * 16u;

            // One stage: consume buffer b with codes `cr`; meanwhile start stage s+1 (rows -> buffer
            // b^1, codes -> cr_next), its vector-memory instructions spread over the read batches.
            // `mode_tag`: TPS == 2: ignored.  TPS == 1: 0 = this stage's table is the low half of `cr`,
            // 1 = the high half, and the next stage needs the next code word (loaded into cr_next).
            auto run_stage = [&](auto more_tag, auto mode_tag, uint32_t s, uint32_t b, const uint32_t(&cr)[NCR],
                                 uint32_t(&cr_next)[NCR], const float(&w)[TPS][WQ],
                                 float(&w_next)[TPS][WQ]) {
                constexpr bool MORE = decltype(more_tag)::value;
                constexpr int HALF = decltype(mode_tag)::value;
                constexpr bool LOADC = TPS == 2 || HALF == 1;  // does the next stage start a new code word?
                constexpr int RB = LFFN_LDS_RB;              // row reads per batch
                constexpr int NB = (TOK + RB - 1) / RB;      // batches per table
                constexpr int NBT = TPS * NB;            // batches per stage
                uint4 r[2][RB];
                auto issue = [&](int bi, uint4(&dst)[RB]) {  // bi = u * NB + batch within table u
                    const int u = bi / NB, b0 = (bi % NB) * RB;
                    const uint32_t base = qb + b * buf_bytes + (uint32_t)u * tbl_bytes;
#pragma unroll
                    for (int i = 0; i < RB; ++i)
                        if (b0 + i < TOK) {
                            const uint32_t off = row_offset(cr, TPS == 2 ? u : HALF, b0 + i);
                            const u32x4 v = *reinterpret_cast<const __attribute__((address_space(3))) u32x4 *>(
                                (uintptr_t)(base + off));
                            dst[i] = make_uint4(v.x, v.y, v.z, v.w);
                        }
                };
                auto consume = [&](int bi, const uint4(&src)[RB]) {
                    const int u = bi / NB, b0 = (bi % NB) * RB;
#pragma unroll
                    for (int i = 0; i < RB; ++i)
                        if (b0 + i < TOK) {
                            if constexpr (WEIGHTED)
                                acc[b0 + i].fma(src[i], quad_bcast(w[u][(b0 + i) >> 2], (b0 + i) & 3));
                            else
                                acc[b0 + i].add(src[i]);
                            acc[b0 + i].pin();
                        }
                };
                issue(0, r[0]);
#pragma unroll
                for (int bi = 0; bi < NBT; ++bi) {
                    if (bi + 1 < NBT) issue(bi + 1, r[(bi + 1) & 1]);
                    if constexpr (MORE) {
                        // vector-memory work of the next stage, a little per batch: row copies first
                        // (they take longest), then its codes, then its weights
                        // short stages (up to 8 token slots) of the plain sum with 128-byte slices issue the
                        // copies together in the first batch (P6, P7: 4 % faster); with 12 or 13 slots, and in
                        // the weighted form, whose batches also carry weight loads, spreading them measured
                        // as fast or faster; a 64 KB stage of one 1024-row table (64-byte slices) gains 5 % from the
                        // early issue (the same form with two 512-row tables per stage loses 6 %)
                        constexpr bool COPY_FIRST = !WEIGHTED && ((SW == 8 && TOK <= 8) || (SW == 4 && FR == 4));
#pragma unroll
                        for (int idx = 0; idx < TPS * FR; ++idx)
                            if ((COPY_FIRST ? 0 : vm_slot(idx, NBT)) == bi) fill_piece(s + 1, b ^ 1u, idx);
                        if constexpr (LOADC) {
#pragma unroll
                            for (int m = 0; m < NCR; ++m)
                                if (vm_slot(LFFN_LDS_CO + m, NBT) == bi) load_code((s + 1) * TPS / 2, m, cr_next);
                        }
                        if constexpr (WEIGHTED) {
#pragma unroll
                            for (int m = 0; m < NWL; ++m)
                                if (vm_slot(LFFN_LDS_WO + m, NBT) == bi) load_weight(s + 1, m, w_next);
                        }
                    }
                    consume(bi, r[bi & 1]);
                }
                __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): next stage's rows and codes have landed
                __syncthreads();
            };
            // ---- multi-probe form: one sweep of the stage per probe --------------------------------
            // shares of probe pr for table u of stage s, register m
            auto load_share = [&](uint32_t s, int i, uint32_t pr, float(&wr)[TPS][WQ]) {
                const int u = i / WQ, m = i % WQ;
                const char *base = reinterpret_cast<const char *>(a.wpk) +
                                   ((size_t)((s * TPS + (uint32_t)u) * ((uint32_t)a.tau + 1u) + pr) * a.n_pad + c0) * 4u;  // uniform
                wr[u][m] = *reinterpret_cast<const float *>(base + reg_offset(m));
            };
            // One sweep: rows code ^ flip with shares `w`; meanwhile the shares of (ns, npr) travel into
            // w_next and, in a stage's last sweep (FILL), the next stage's row copies and codes.
            auto sweep = [&](auto fill_tag, auto mode_tag, uint32_t s, uint32_t b, const uint32_t(&cr)[NCR],
                             uint32_t(&cr_next)[NCR], const float(&w)[TPS][WQ], float(&w_next)[TPS][WQ],
                             uint32_t flip, bool more_shares, uint32_t ns, uint32_t npr) {
                constexpr bool FILL = decltype(fill_tag)::value;
                constexpr int HALF = decltype(mode_tag)::value;
                constexpr bool LOADC = TPS == 2 || HALF == 1;
                constexpr int RB = LFFN_LDS_RB;
                constexpr int NB = (TOK + RB - 1) / RB;
                constexpr int NBT = TPS * NB;
                uint4 r[2][RB];
                auto issue = [&](int bi, uint4(&dst)[RB]) {
                    const int u = bi / NB, b0 = (bi % NB) * RB;
                    const uint32_t base = qb + b * buf_bytes + (uint32_t)u * tbl_bytes;
#pragma unroll
                    for (int i = 0; i < RB; ++i)
                        if (b0 + i < TOK) {
                            const uint32_t off = row_offset(cr, TPS == 2 ? u : HALF, b0 + i) ^ flip;
                            const u32x4 v = *reinterpret_cast<const __attribute__((address_space(3))) u32x4 *>(
                                (uintptr_t)(base + off));
                            dst[i] = make_uint4(v.x, v.y, v.z, v.w);
                        }
                };
                auto consume = [&](int bi, const uint4(&src)[RB]) {
                    const int u = bi / NB, b0 = (bi % NB) * RB;
#pragma unroll
                    for (int i = 0; i < RB; ++i)
                        if (b0 + i < TOK) {
                            acc[b0 + i].fma(src[i], quad_bcast(w[u][(b0 + i) >> 2], (b0 + i) & 3));
                            acc[b0 + i].pin();
                        }
                };
                issue(0, r[0]);
#pragma unroll
                for (int bi = 0; bi < NBT; ++bi) {
                    if (bi + 1 < NBT) issue(bi + 1, r[(bi + 1) & 1]);
                    // the next sweep's shares first: they are needed soonest
                    if (more_shares) {
#pragma unroll
                        for (int m = 0; m < NWL; ++m)
                            if (vm_slot(m / 2, NBT) == bi) load_share(ns, m, npr, w_next);  // two per batch, early
                    }
                    if constexpr (FILL) {
#pragma unroll
                        for (int idx = 0; idx < TPS * FR; ++idx)
                            if (vm_slot(idx, NBT) == bi) fill_piece(s + 1, b ^ 1u, idx);
                        if constexpr (LOADC) {
#pragma unroll
                            for (int m = 0; m < NCR; ++m)
                                if (vm_slot(LFFN_LDS_CO + m, NBT) == bi) load_code((s + 1) * TPS / 2, m, cr_next);
                        }
                    }
                    consume(bi, r[bi & 1]);
                }
            };
            // a whole stage: 1 + tau sweeps, then the barrier that publishes the next stage's buffer
            auto run_stage_probes = [&](auto more_tag, auto mode_tag, uint32_t s, uint32_t b, const uint32_t(&cr)[NCR],
                                        uint32_t(&cr_next)[NCR], float(&w)[TPS][WQ], float(&w_next)[TPS][WQ]) {
                constexpr bool MORE = decltype(more_tag)::value;
                const uint32_t tau = (uint32_t)a.tau;
                for (uint32_t pr = 0; pr < tau; ++pr) {
                    sweep(std::integral_constant<bool, false>{}, mode_tag, s, b, cr, cr_next, w, w_next,
                          pr ? (PIECE << (pr - 1u)) : 0u, true, s, pr + 1u);
#pragma unroll
                    for (int u = 0; u < TPS; ++u)
#pragma unroll
                        for (int m = 0; m < WQ; ++m) w[u][m] = w_next[u][m];
                }
                sweep(more_tag, mode_tag, s, b, cr, cr_next, w, w_next, PIECE << (tau - 1u), MORE, s + 1u, 0u);
#pragma unroll
                for (int u = 0; u < TPS; ++u)
#pragma unroll
                    for (int m = 0; m < WQ; ++m) w[u][m] = w_next[u][m];
                __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): next stage's rows, codes and first shares have landed
                __syncthreads();
            };

            using yes = std::integral_constant<bool, true>;
            using no = std::integral_constant<bool, false>;

            // prologue: stage 0 into buffer 0, its codes
#pragma unroll
            for (int idx = 0; idx < TPS * FR; ++idx) fill_piece(0, 0, idx);
#pragma unroll
            for (int i = 0; i < NCR; ++i) load_code(0, i, crA);
            if constexpr (PROBES) {
#pragma unroll
                for (int i = 0; i < NWL; ++i) load_share(0, i, 0u, wA);
            } else if constexpr (WEIGHTED) {
#pragma unroll
                for (int i = 0; i < NWL; ++i) load_weight(0, i, wA);
            }
            __builtin_amdgcn_s_waitcnt(0x0F70);
            __syncthreads();

            // all stages but the last start their successor; buffers, code sets and weight sets alternate
            using t0 = std::integral_constant<int, 0>;
            using t1 = std::integral_constant<int, 1>;
            uint32_t s = 0;
            if constexpr (PROBES) {
                // the shares of the sweep in progress stay in wA, those in flight in wB
                if constexpr (TPS == 2) {
                    for (; s + 2 < nstages; s += 2) {
                        run_stage_probes(yes{}, t0{}, s, 0u, crA, crB, wA, wB);
                        run_stage_probes(yes{}, t0{}, s + 1, 1u, crB, crA, wA, wB);
                    }
                    if (s + 1 < nstages) {
                        run_stage_probes(yes{}, t0{}, s, 0u, crA, crB, wA, wB);
                        run_stage_probes(no{}, t0{}, s + 1, 1u, crB, crA, wA, wB);
                    } else {
                        run_stage_probes(no{}, t0{}, s, 0u, crA, crB, wA, wB);
                    }
                } else {
                    for (; s + 4 < nstages; s += 4) {
                        run_stage_probes(yes{}, t0{}, s, 0u, crA, crB, wA, wB);
                        run_stage_probes(yes{}, t1{}, s + 1, 1u, crA, crB, wA, wB);
                        run_stage_probes(yes{}, t0{}, s + 2, 0u, crB, crA, wA, wB);
                        run_stage_probes(yes{}, t1{}, s + 3, 1u, crB, crA, wA, wB);
                    }
                    if (s + 2 < nstages) {
                        run_stage_probes(yes{}, t0{}, s, 0u, crA, crB, wA, wB);
                        run_stage_probes(yes{}, t1{}, s + 1, 1u, crA, crB, wA, wB);
                        run_stage_probes(yes{}, t0{}, s + 2, 0u, crB, crA, wA, wB);
                        run_stage_probes(no{}, t1{}, s + 3, 1u, crB, crA, wA, wB);
                    } else {
                        run_stage_probes(yes{}, t0{}, s, 0u, crA, crB, wA, wB);
                        run_stage_probes(no{}, t1{}, s + 1, 1u, crA, crB, wA, wB);
                    }
                }
            } else if constexpr (TPS == 2) {
                for (; s + 2 < nstages; s += 2) {
                    run_stage(yes{}, t0{}, s, 0u, crA, crB, wA, wB);
                    run_stage(yes{}, t0{}, s + 1, 1u, crB, crA, wB, wA);
                }
                if (s + 1 < nstages) {
                    run_stage(yes{}, t0{}, s, 0u, crA, crB, wA, wB);
                    run_stage(no{}, t0{}, s + 1, 1u, crB, crA, wB, wA);
                } else {
                    run_stage(no{}, t0{}, s, 0u, crA, crB, wA, wB);
                }
            } else {
                // one table per stage, two stages per code word (k is even): word p = s/2 sits in crA for
                // even p, crB for odd p
                for (; s + 4 < nstages; s += 4) {
                    run_stage(yes{}, t0{}, s, 0u, crA, crB, wA, wB);
                    run_stage(yes{}, t1{}, s + 1, 1u, crA, crB, wB, wA);
                    run_stage(yes{}, t0{}, s + 2, 0u, crB, crA, wA, wB);
                    run_stage(yes{}, t1{}, s + 3, 1u, crB, crA, wB, wA);
                }
                if (s + 2 < nstages) {
                    run_stage(yes{}, t0{}, s, 0u, crA, crB, wA, wB);
                    run_stage(yes{}, t1{}, s + 1, 1u, crA, crB, wB, wA);
                    run_stage(yes{}, t0{}, s + 2, 0u, crB, crA, wA, wB);
                    run_stage(no{}, t1{}, s + 3, 1u, crB, crA, wB, wA);
                } else {
                    run_stage(yes{}, t0{}, s, 0u, crA, crB, wA, wB);
                    run_stage(no{}, t1{}, s + 1, 1u, crA, crB, wB, wA);
                }
            }

            {
                // The output addresses are formed here, from a lane index the compiler cannot see through: left
                // alone it computes all TOK of them before the stage loop and keeps them in registers across it
                // (the 12-, 13- and 16-slot forms then spill in their hot loop).
                uint32_t lt = tid;
                asm volatile("" : "+v"(lt));
                const uint32_t sg = lt / SW, svec = slice * (uint32_t)SW + lt % SW;
#pragma unroll
                for (int i = 0; i < TOK; ++i) {
                    const uint32_t t = i < 4 * FQ ? c0 + (4u * G) * (uint32_t)(i >> 2) + 4u * sg + (uint32_t)(i & 3)
                                                  : c0 + (uint32_t)G * (uint32_t)i + sg;
                    if (t >= c1 || svec >= (uint32_t)a.nvec) continue;
                    store_y4(a.y, (size_t)t * a.d_out + (size_t)svec * 4u, acc[i].f[0], acc[i].f[1], acc[i].f[2],
                             acc[i].f[3], a.y_kind);
                }
            }
        }
    }
}

#if !defined(LFFN_PART) || LFFN_PART == 0  // a plain function: defined by part 0 only of a build in parts
// One-time re-layout of the learned tables T_j (Sec. 3.1, eq. "lookup") for the gather kernels: fp32
// elements (bf16 and IEEE half rows widened exactly), slice-major,
//   dst[ps][j][row][PW bytes],  ps < ceil(d_out*4 / PW),
// so that the column slice of ALL tables a workgroup streams is one contiguous run.  Pieces past the end
// of a row (ragged last slice) are zero.  One 16-byte output piece per thread and step.
//   nvec = d_out / 4 (pieces per fp32 row), ppw = PW / 16, n_out = output pieces in total
__global__ __launch_bounds__(256) void prepare_tables_kernel(const void *src, uint4 *dst, int k, int rows, int nvec,
                                                             int ppw, int kind, long long n_out)
{
    for (long long o = (long long)blockIdx.x * blockDim.x + threadIdx.x; o < n_out;
         o += (long long)gridDim.x * blockDim.x) {
        const int p = (int)(o % ppw);
        long long rest = o / ppw;
        const int row = (int)(rest % rows);
        rest /= rows;
        const int j = (int)(rest % k);
        const long long ps = rest / k;
        const long long vec = ps * ppw + p;
        uint4 v = make_uint4(0u, 0u, 0u, 0u);
        if (vec < nvec) {
            const long long piece = ((long long)j * rows + row) * nvec + vec;
            if (kind) {
                const uint2 w = static_cast<const uint2 *>(src)[piece];
                const float2 lo = widen16x2(w.x, kind), hi = widen16x2(w.y, kind);
                v = make_uint4(__float_as_uint(lo.x), __float_as_uint(lo.y), __float_as_uint(hi.x), __float_as_uint(hi.y));
            } else {
                v = static_cast<const uint4 *>(src)[piece];
            }
        }
        dst[o] = v;
    }
}
#endif

}  // namespace lffn
