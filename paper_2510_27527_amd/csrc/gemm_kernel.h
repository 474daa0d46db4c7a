// NT GEMM on two packed NVFP4 operands for gfx950 (the three products of TetraJet-v2 Sec. 2.3
// all reduce to Out[M x N] = A[M x K] * B[N x K]^T once each operand is grouped along K).
//
// CDNA4's block-scaled MFMA takes E8M0 scales per 32 elements, NVFP4 has E4M3 scales per 16, so
// the exact route is: stage the packed tiles (codes + scale bytes) in LDS, expand
// code * S_block to FP16 in registers (6 significant bits, 2^-14 <= |v| <= 168 after a 2^-4
// pre-scale: exact and normal in FP16), feed v_mfma_f32_32x32x16_f16 with FP32 accumulation and
// multiply by the two FP32 outer scales (and 2^8) in the epilogue.
//
// Work split: 256 threads = 2 x 2 waves; each wave owns TM x TN tiles of 32 x 32.  Within one
// 64-wide K chunk a lane (row r = lane % 32, kg = lane / 32) holds the 32 codes k = 32 kg .. 32 kg + 31
// of its row (one 128-bit LDS read) and uses 8 of them per MFMA; A and B use the same assignment,
// so the order of k inside a chunk does not matter.  Small outputs with a long reduction (the
// weight gradient) are split along K into FP32 partials that a second kernel sums in a fixed order.
#pragma once
#include "gemm_args.h"

namespace tj {

namespace {

constexpr int kThreads = kGemmThreads;
constexpr int kNC = 2;        // 64-k chunks per pipeline stage
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));

__device__ __forceinline__ half2_t scale_pair(uint32_t sc)
{
    // E4M3 byte << 7 is the FP16 pattern of S_block * 2^-8 (same field layout, bias 15 vs 7; E4M3 subnormals become
    // FP16 subnormals of the same value)
    return __builtin_bit_cast(half2_t, sc * 0x00800080u);
}

// eight codes (one dword) times the block scale -> eight FP16 holding P * S_block * 2^-4.  The conversion's scale
// operand contributes a power of two only (it uses the exponent of its argument): 2^4 here, so that the product
// with S_block * 2^-8 is a normal FP16 for every scale code; both factors and the product are exact.
__device__ __forceinline__ half8_t expand8(uint32_t q, half2_t f)
{
    const half2_t p0 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(q, 16.0f, 0) * f;
    const half2_t p1 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(q, 16.0f, 1) * f;
    const half2_t p2 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(q, 16.0f, 2) * f;
    const half2_t p3 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(q, 16.0f, 3) * f;
    half8_t r;
    r[0] = p0.x; r[1] = p0.y; r[2] = p1.x; r[3] = p1.y;
    r[4] = p2.x; r[5] = p2.y; r[6] = p3.x; r[7] = p3.y;
    return r;
}

// Global -> LDS copies that bypass registers: every lane supplies a global address, the wave's data
// lands at lds_addr + lane * 16 (or * 4).  Written as inline assembly so that completion is tracked only
// by the explicit s_waitcnt vmcnt(n) of the pipeline (the compiler would otherwise wait for every
// outstanding copy before each LDS read).  lds_addr must be wave-uniform; the s_nop covers the wait state
// between a scalar write of M0 and the copy that uses it.
// The global address is a wave-uniform 64-bit base plus a 32-bit unsigned byte offset per lane.
__device__ __forceinline__ void lds_dma16(const void *base, uint32_t off, uint32_t lds_addr)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" : : "s"(lds_addr), "v"(off), "s"(base) : "memory", "m0");
}
__device__ __forceinline__ void lds_dma4(const void *base, uint32_t off, uint32_t lds_addr)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, %2" : : "s"(lds_addr), "v"(off), "s"(base) : "memory", "m0");
}

// a wave-uniform pointer the compiler computed in vector registers, moved to scalar registers
__device__ __forceinline__ const void *to_scalar(const void *p)
{
    const uint64_t v = reinterpret_cast<uint64_t>(p);
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v), hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return reinterpret_cast<const void *>(((uint64_t)hi << 32) | lo);
}

__device__ __forceinline__ uint32_t pick(uint4 v, int i) { return i == 0 ? v.x : i == 1 ? v.y : i == 2 ? v.z : v.w; }

// Epilogue of both product kernels: outer scales, conversion, stores.
// SWAP (bf16 output): a lane holds one output row (m = lane % 32) and, per 32 x 32 block, four runs of four consecutive
// columns; otherwise lanes run along the columns and accumulator element e sits in row 8 * (e / 4) + 4 * (lane / 32) + e % 4.
template <int TM, int TN, int OUT, bool SWAP, int OUTER>
__device__ __forceinline__ void store_tile(float16_t (&acc)[TM][TN], const GemmArgs &g, int64_t m0, int64_t n0, int wm, int wn,
                                           int lr, int kg, uint8_t *stage)
{
    constexpr bool SPLIT = OUT == 2;
    float alpha = 1.0f;
    // tensor mode: both outer scales and the 2^8 of the FP16 pre-scale; block mode: the outer scales are already in
    if (!SPLIT) alpha = OUTER == 0 ? g.a_gscale[0] * g.b_gscale[0] * 256.0f : 256.0f;
    if (SWAP && (g.N & 7) == 0 && m0 + 64 * TM <= g.M && n0 + 64 * TN <= g.N) {
        // Whole tile, rows 16-byte aligned: a wave's 32 x (32 TN) block of outputs goes through the wave's own corner of
        // LDS (the pipeline buffers are free by now) and leaves as whole rows - sixteen lanes write one row's 64 TN
        // contiguous bytes, a store instruction four rows - instead of 16-byte pieces of 32 different rows, which cost
        // the memory pipeline eight times as many cache-line accesses.  Row pitch 64 TN + 8 bytes: the 8-byte writes
        // of 32 rows and the 8-byte reads of 2 x 16 pieces both spread over all banks.  Two buffers alternate; the
        // LDS executes one wave's instructions in order, so neither a barrier nor a wait is needed between a block's
        // reads and the writes of the block after next.
        constexpr int PITCH = 64 * TN + 8;
        uint8_t *outb = reinterpret_cast<uint8_t *>(g.out);
        const int lane = lr + 32 * kg, wave = wm * 2 + wn;
        const int piece = lane & 15, rsub = lane >> 4;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            uint8_t *buf = stage + (wave * 2 + (i & 1)) * 32 * PITCH;
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const bf16x2_t lo = __builtin_convertvector((float2_t){acc[i][j][4 * q] * alpha, acc[i][j][4 * q + 1] * alpha}, bf16x2_t);
                    const bf16x2_t hi = __builtin_convertvector((float2_t){acc[i][j][4 * q + 2] * alpha, acc[i][j][4 * q + 3] * alpha}, bf16x2_t);
                    *reinterpret_cast<uint2 *>(buf + lr * PITCH + (j * 32 + 8 * q + 4 * kg) * 2) =
                        make_uint2(__builtin_bit_cast(uint32_t, lo), __builtin_bit_cast(uint32_t, hi));
                }
            const int64_t mrow = m0 + (wm * TM + i) * 32, ncol = n0 + wn * TN * 32;
            if (piece < 4 * TN) {
#pragma unroll
                for (int it = 0; it < 8; ++it) {
                    const int row = 4 * it + rsub;
                    const uint2 a = *reinterpret_cast<const uint2 *>(buf + row * PITCH + piece * 16);
                    const uint2 b = *reinterpret_cast<const uint2 *>(buf + row * PITCH + piece * 16 + 8);
                    *reinterpret_cast<uint4 *>(outb + ((mrow + row) * g.N + ncol) * 2 + piece * 16) = make_uint4(a.x, a.y, b.x, b.y);
                }
            }
        }
    } else if (SWAP) {
        // a lane holds one output row (m = lane % 32) and, per 32 x 32 block, four runs of four consecutive columns
        // (n = 8 * (e / 4) + 4 * (lane / 32) + e % 4): each run leaves as one 8-byte store
        uint16_t *outh = reinterpret_cast<uint16_t *>(g.out);
        const bool vec = (g.N & 3) == 0;             // then every run is aligned and entirely inside or outside
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int64_t m = m0 + (wm * TM + i) * 32 + lr;
            if (m >= g.M) continue;
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int64_t n = n0 + (wn * TN + j) * 32 + 8 * q + 4 * kg;
                    const float v0 = acc[i][j][4 * q] * alpha, v1 = acc[i][j][4 * q + 1] * alpha;
                    const float v2 = acc[i][j][4 * q + 2] * alpha, v3 = acc[i][j][4 * q + 3] * alpha;
                    if (vec) {
                        if (n < g.N) {
                            const bf16x2_t lo = __builtin_convertvector((float2_t){v0, v1}, bf16x2_t);
                            const bf16x2_t hi = __builtin_convertvector((float2_t){v2, v3}, bf16x2_t);
                            *reinterpret_cast<uint2 *>(outh + m * g.N + n) =
                                make_uint2(__builtin_bit_cast(uint32_t, lo), __builtin_bit_cast(uint32_t, hi));
                        }
                    } else {
                        const float v[4] = {v0, v1, v2, v3};
#pragma unroll
                        for (int t = 0; t < 4; ++t)
                            if (n + t < g.N) outh[m * g.N + n + t] = (uint16_t)f32_to_bf16_bits(v[t]);
                    }
                }
        }
    } else {
        // acc element e of a lane: row 8 * (e / 4) + 4 * (lane / 32) + e % 4, column lane % 32
        float *outf = reinterpret_cast<float *>(g.out);
        if (SPLIT) outf += (int64_t)blockIdx.z * g.M * g.N;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int64_t n = n0 + (wn * TN + j) * 32 + lr;
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int64_t m = m0 + (wm * TM + i) * 32 + 8 * (e >> 2) + 4 * kg + (e & 3);
                    if (m < g.M && n < g.N) outf[m * g.N + n] = acc[i][j][e] * alpha;
                }
            }
    }
}

// Tile TM*64 x TN*64 per workgroup (2 x 2 waves, TM x TN MFMA tiles of 32 x 32 each), NC chunks of
// 64 k per pipeline stage, three stage buffers in LDS.  Codes and scale bytes go global -> LDS
// directly (a wave instruction fills 64 consecutive 16-byte / 4-byte slots), two stages ahead.
//   codes : slot of (row, 16-byte piece p of the stage's row segment) = row * SLOTS + (p ^ swz(row)), swz(row) =
//           (row >> 2) % SLOTS: 16 consecutive rows then cover 16 different 16-byte columns of the 256-byte bank row
//   scales: dword of (chunk c, row) = c * ROWS + row   (A rows first, then B rows); when K is a multiple of 256
//           (PS = true) scale bytes are instead fetched 16 per row (four chunks = two stages) into a ring of
//           three [ROWS][16] buffers, half of the rows per stage, four stages ahead: one 16-byte request per
//           row and 256 k instead of four 4-byte requests
// The reduction is a software pipeline over 16-wide k steps: while the MFMAs of step g run, the
// FP4 -> FP16 expansion of step g + 1 is issued (about four VALU instructions per MFMA), and the
// raw codes of the next chunk are fetched from LDS one step earlier.  One barrier per stage, placed
// two steps before its end so that the first step of the next stage is expanded under the last
// MFMAs of this one.  Rows past M / N read clamped (valid) addresses and are never stored; chunks
// past the end of K get zero scales.
template <int TM, int TN>
struct RawFrags {
    uint4 qa[TM], qb[TN];       // 32 codes per fragment
};
template <int TM, int TN>
struct OpFrags {
    half8_t a[TM], b[TN];
};

// OUTER = 1: operands with one FP32 outer scale per row and 128 k (the paper's 1 x 128 outer block, Sec. 2.2).  A
// pipeline stage is exactly one outer block, so each stage accumulates into a fresh set of accumulators (its first
// MFMA takes zero as addend) and at its end  total += stage_sum * S_A[m, kb] * S_B[n, kb]  in FP32 (two vector
// instructions per accumulator element and stage, which is why this mode keeps at most 2 x 4 tiles per wave).  The
// outer scales of a stage travel global -> LDS with the same direct copies, one float per row, into a ring of four.
template <int TM, int TN, int NC, int OUT, bool PS, int OUTER>   // OUT: 0 bf16, 1 f32, 2 raw f32 split-K partial
__global__ __launch_bounds__(kThreads, (TM * TN * (OUTER + 1) >= 8 ? 1 : 2)) void gemm_nt_kernel(GemmArgs g)
{
    constexpr int BM = 64 * TM, BN = 64 * TN, ROWS = BM + BN;
    constexpr int SLOTS = 2 * NC;                       // 16-byte pieces per row per stage
    constexpr int A_SLOTS = BM * SLOTS, B_SLOTS = BN * SLOTS;
    constexpr int LA = A_SLOTS / kThreads, LB = B_SLOTS / kThreads, LS = PS ? 0 : ROWS * NC / kThreads;
    constexpr int LG = OUTER ? (ROWS / 64 + 3) / 4 : 0;  // outer-scale copies per thread per stage (64 rows each)
    constexpr int NSTAGE = LA + LB + LG + (PS ? 0 : LS); // copies per thread that issue_loads() makes for one stage
    constexpr int NLOAD = NSTAGE + (PS ? 1 : 0);         // direct-to-LDS loads per thread per stage
    constexpr int CODE_BYTES = (A_SLOTS + B_SLOTS) * 16; // one stage of codes; three of them, then the scales
    constexpr int SC_BYTES = PS ? ROWS * 16 : ROWS * NC * 4;   // one scale buffer (a pair of stages / one stage)
    constexpr int SC_BASE = 3 * CODE_BYTES;
    constexpr int GS_BASE = SC_BASE + 3 * SC_BYTES;      // OUTER: ring of four [ROWS] float buffers
    static_assert(!OUTER || NC == 2, "a stage must be one 128-k outer block");
    static_assert(!OUTER || TM * TN <= 8, "two accumulator sets must fit the register file");
    constexpr int STEPS = NC * 4;
    // bf16 output: the MFMA takes the B fragment as its row operand, so that a lane ends up with runs of four
    // consecutive output columns (8-byte stores); FP32 output keeps lanes along the columns (128 contiguous bytes
    // per row and store instruction)
    constexpr bool SWAP = OUT == 0;
    static_assert(!PS || NC == 2, "paired scale fetch assumes two chunks per stage");
    static_assert(NC % 2 == 0, "chunk parity must repeat per stage");
    static_assert(LA >= 1 && LB >= 1 && A_SLOTS % kThreads == 0 && B_SLOTS % kThreads == 0, "tile too small");
    static_assert(PS || (LS >= 1 && (ROWS * NC) % kThreads == 0), "per-chunk scale fetch needs whole instructions");
    static_assert(NLOAD <= 15, "vmcnt immediate below assumes at most 15 loads per stage");
    static_assert(OUT != 0 || 4 * 2 * 32 * (64 * TN + 8) <= 3 * CODE_BYTES, "the bf16 epilogue stages its rows in the code buffers");

    extern __shared__ __attribute__((aligned(16))) uint8_t smem_raw[];

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 1, wn = wave & 1;
    const int lr = lane & 31, kg = lane >> 5;
    const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void *)smem_raw;

    // workgroup -> tile: consecutive ids of one XCD (ids are dealt round-robin over 8 XCDs) walk
    // down a column of tiles, in groups of 8 tile rows
    const int total = g.tiles_m * g.tiles_n;
    int pid = blockIdx.x;
    {
        const int per_xcd = total / 8;
        if (pid < per_xcd * 8) pid = (pid & 7) * per_xcd + (pid >> 3);
    }
    constexpr int GROUP = 8;
    const int group_sz = GROUP * g.tiles_n;
    const int gid = pid / group_sz;
    const int first_m = gid * GROUP;
    const int gm = (g.tiles_m - first_m) < GROUP ? (g.tiles_m - first_m) : GROUP;
    const int tile_m = first_m + (pid % group_sz) % gm;
    const int tile_n = (pid % group_sz) / gm;

    const int64_t m0 = (int64_t)tile_m * BM, n0 = (int64_t)tile_n * BN;
    const int64_t chunks_total = g.K / 64;
    const int64_t cbeg = (int64_t)blockIdx.z * g.chunks_per_split;
    int64_t cend = cbeg + g.chunks_per_split;
    if (cend > chunks_total) cend = chunks_total;
    const int nchunks = (int)(cend - cbeg);
    const int nk = (nchunks + NC - 1) / NC;
    const int64_t cstride = g.K / 2, sstride = g.K / 16;

    float16_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

    float16_t part[OUTER ? TM : 1][OUTER ? TN : 1];      // OUTER: the running sum of the current 128-k block
    float16_t zero16;
#pragma unroll
    for (int e = 0; e < 16; ++e) zero16[e] = 0.0f;

    if (nchunks > 0) {
        // Per-lane constants of the loads: 32-bit byte offsets from the tile's (uniform) base pointers, the
        // piece / chunk index each load covers, and a bit mask of the loads whose row exists.
        uint32_t coff[LA + LB], soff[PS ? 2 : LS];
        uint32_t cpieces = 0, schunks = 0, rowmask = 0;      // 4 bits per load / 1 bit per load
#pragma unroll
        for (int u = 0; u < LA + LB; ++u) {
            const bool isA = u < LA;
            const int slot = ((isA ? u : u - LA) * 4 + wave) * 64 + lane, row = slot / SLOTS, pos = slot % SLOTS;
            const int piece = pos ^ ((row >> 2) & (SLOTS - 1));
            coff[u] = (uint32_t)row * (uint32_t)cstride + (uint32_t)piece * 16u;
            cpieces |= (uint32_t)piece << (4 * u);
            if ((isA ? m0 : n0) + row < (isA ? g.M : g.N)) rowmask |= 1u << u;
        }
        if (!PS) {
#pragma unroll
            for (int u = 0; u < LS; ++u) {
                const int q = u * 4 + wave, c = q / (ROWS / 64), row = (q % (ROWS / 64)) * 64 + lane;
                const bool isA = row < BM;
                soff[u] = (uint32_t)(isA ? row : row - BM) * (uint32_t)sstride + (uint32_t)c * 4u;
                schunks |= (uint32_t)c << (4 * u);
                if ((isA ? m0 + row : n0 + row - BM) < (isA ? g.M : g.N)) rowmask |= 1u << (LA + LB + u);
            }
        } else {
            // half h of a pair: wave-instruction q = 4 h + wave covers rows (q % (ROWS/64)) * 64 .. + 63
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int row = ((h * 4 + wave) % (ROWS / 64)) * 64 + lane;
                const bool isA = row < BM;
                const bool ok = (isA ? m0 + row : n0 + row - BM) < (isA ? g.M : g.N);
                soff[h] = ok ? (uint32_t)(isA ? row : row - BM) * (uint32_t)sstride : 0u;
            }
        }
        // OUTER: copy u of a stage brings the outer scales of rows (q % (ROWS/64)) * 64 .. + 63, q = 4 u + wave (when
        // ROWS/64 is no multiple of four the surplus copies repeat a block: same values to the same place)
        uint32_t goff[OUTER ? LG : 1];
        const int64_t nkb = g.K >> 7;
        if (OUTER) {
#pragma unroll
            for (int u = 0; u < LG; ++u) {
                const int row = ((u * 4 + wave) % (ROWS / 64)) * 64 + lane;
                const bool isA = row < BM;
                const bool ok = (isA ? m0 + row : n0 + row - BM) < (isA ? g.M : g.N);
                goff[u] = ok ? (uint32_t)(isA ? row : row - BM) * (uint32_t)nkb * 4u : 0u;
            }
        }
        const bool tile_full = m0 + BM <= g.M && n0 + BN <= g.N;
        const uint8_t *a_cbase = g.a_codes + m0 * cstride + cbeg * 32, *b_cbase = g.b_codes + n0 * cstride + cbeg * 32;
        const uint8_t *a_sbase = g.a_scales + m0 * sstride + cbeg * 4, *b_sbase = g.b_scales + n0 * sstride + cbeg * 4;
        // OUTER: outer scales of the tile's rows for the split's first 128-k block (a split starts on a block boundary)
        const float *a_gbase = OUTER ? g.a_gscale + m0 * nkb + (cbeg >> 1) : nullptr;
        const float *b_gbase = OUTER ? g.b_gscale + n0 * nkb + (cbeg >> 1) : nullptr;
        auto issue_outer = [&](int kt) {
            // stage kt = block kt of the split, into ring slot kt % 4; stages past the end re-fetch block 0 (never used)
            const int kb = (int64_t)kt * NC < nchunks ? kt : 0;
#pragma unroll
            for (int u = 0; u < LG; ++u) {
                const int rb = (u * 4 + wave) % (ROWS / 64);
                lds_dma4(to_scalar((rb * 64 < BM ? a_gbase : b_gbase) + kb), goff[u], lds_base + GS_BASE + ((kt & 3) * ROWS + rb * 64) * 4);
            }
        };

        // All loads of stage kt.  Interior tiles and stages fully inside the split take the straight path;
        // otherwise loads of missing rows or of chunks past the end are skipped (their LDS slots keep stale
        // bytes: missing rows are never stored, late chunks get zero scales when they are read).
        auto issue_loads = [&](int kt, int buf) {
            const int64_t c0 = (int64_t)kt * NC;                  // first chunk of the stage, relative to cbeg
            const uint32_t dst = lds_base + buf * CODE_BYTES;
            const uint32_t sdst = lds_base + SC_BASE + buf * SC_BYTES;
            const uint8_t *ac = a_cbase + c0 * 32, *bc = b_cbase + c0 * 32;
            const uint8_t *as = a_sbase + c0 * 4, *bs = b_sbase + c0 * 4;
            if (tile_full && c0 + NC <= nchunks) {
#pragma unroll
                for (int u = 0; u < LA + LB; ++u) {
                    const int lds_slot = (u < LA ? 0 : A_SLOTS) + ((u < LA ? u : u - LA) * 4 + wave) * 64;
                    lds_dma16(u < LA ? ac : bc, coff[u], dst + lds_slot * 16);
                }
#pragma unroll
                for (int u = 0; u < LS; ++u) {
                    const int q = u * 4 + wave;
                    lds_dma4((q % (ROWS / 64)) * 64 < BM ? as : bs, soff[u], sdst + q * 256);
                }
            } else {
                // Same number of instructions (the pipeline counts them with vmcnt); loads that have nothing
                // to fetch are pointed at the first bytes of the tile instead.
                const bool stage_ok = c0 < nchunks;
#pragma unroll
                for (int u = 0; u < LA + LB; ++u) {
                    const int lds_slot = (u < LA ? 0 : A_SLOTS) + ((u < LA ? u : u - LA) * 4 + wave) * 64;
                    const int64_t piece = c0 * 2 + ((cpieces >> (4 * u)) & 15);
                    const bool ok = ((rowmask >> u) & 1u) && piece < (int64_t)nchunks * 2;
                    lds_dma16(stage_ok ? (u < LA ? ac : bc) : (u < LA ? a_cbase : b_cbase), ok ? coff[u] : 0u,
                              dst + lds_slot * 16);
                }
#pragma unroll
                for (int u = 0; u < LS; ++u) {
                    const int q = u * 4 + wave;
                    const bool isA = (q % (ROWS / 64)) * 64 < BM;
                    const int64_t c = c0 + ((schunks >> (4 * u)) & 15);
                    const bool ok = ((rowmask >> (LA + LB + u)) & 1u) && c < nchunks;
                    lds_dma4(stage_ok ? (isA ? as : bs) : (isA ? a_sbase : b_sbase), ok ? soff[u] : 0u,
                             sdst + q * 256);
                }
            }
            if (OUTER) issue_outer(kt);
        };
        // PS: half h of scale pair P (16 scale bytes = 256 k per row) into pair buffer P % 3; pairs past the end
        // re-fetch pair 0 (valid memory, never consumed)
        const int npairs = nchunks / 4;
        auto issue_scale_half = [&](int P, int h) {
            const int rb = (h * 4 + wave) % (ROWS / 64);
            const bool isA = rb * 64 < BM;
            const int Pl = P < npairs ? P : 0;
            const uint8_t *base = (isA ? a_sbase : b_sbase) + (int64_t)Pl * 16;
            lds_dma16(base, soff[h], lds_base + SC_BASE + (P % 3) * SC_BYTES + rb * 64 * 16);
        };

        uint32_t scA[NC][TM], scB[NC][TN];   // four scale bytes per chunk and fragment row
        uint32_t live[NC];                    // 0xFF, or 0 for a chunk past the end of K (its scales count as zero)
        auto read_raw = [&](RawFrags<TM, TN> &r, int buf, int c, bool is_live) {
            const uint4 *codes = reinterpret_cast<const uint4 *>(smem_raw + buf * CODE_BYTES);
            const uint32_t *scales = reinterpret_cast<const uint32_t *>(smem_raw + SC_BASE + buf * SC_BYTES) + c * ROWS;
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                const int row = (wm * TM + i) * 32 + lr;
                r.qa[i] = codes[row * SLOTS + ((2 * c + kg) ^ ((row >> 2) & (SLOTS - 1)))];
                if (!PS) scA[c][i] = scales[row];
            }
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int row = (wn * TN + j) * 32 + lr;
                r.qb[j] = codes[A_SLOTS + row * SLOTS + ((2 * c + kg) ^ ((row >> 2) & (SLOTS - 1)))];
                if (!PS) scB[c][j] = scales[BM + row];
            }
            if (!PS) live[c] = is_live ? 0xFFu : 0u;
        };
        // PS: the two chunk dwords of stage kt for every fragment row (second half of the pair for odd stages)
        auto read_stage_scales = [&](int kt) {
            const uint2 *sp = reinterpret_cast<const uint2 *>(smem_raw + SC_BASE + ((kt >> 1) % 3) * SC_BYTES) + (kt & 1);
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                const uint2 v = sp[((wm * TM + i) * 32 + lr) * 2];
                scA[0][i] = v.x; scA[1][i] = v.y;
            }
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const uint2 v = sp[(BM + (wn * TN + j) * 32 + lr) * 2];
                scB[0][j] = v.x; scB[1][j] = v.y;
            }
        };

        half2_t fA[TM], fB[TN];
        auto expand = [&](OpFrags<TM, TN> &o, const RawFrags<TM, TN> &r, int c, int ks) {
            if ((ks & 1) == 0) {
                const uint32_t mask = PS ? 0xFFu : live[c];
#pragma unroll
                for (int i = 0; i < TM; ++i) fA[i] = scale_pair((scA[c][i] >> (16 * kg + 4 * ks)) & mask);
#pragma unroll
                for (int j = 0; j < TN; ++j) fB[j] = scale_pair((scB[c][j] >> (16 * kg + 4 * ks)) & mask);
            }
#pragma unroll
            for (int i = 0; i < TM; ++i) o.a[i] = expand8(pick(r.qa[i], ks), fA[i]);
#pragma unroll
            for (int j = 0; j < TN; ++j) o.b[j] = expand8(pick(r.qb[j], ks), fB[j]);
        };

        RawFrags<TM, TN> raw[2];
        OpFrags<TM, TN> op[2];

        issue_loads(0, 0);
        if (PS) {
            issue_scale_half(0, 0); issue_scale_half(0, 1);
            issue_scale_half(1, 0); issue_scale_half(1, 1);
            issue_loads(1, 1);
            __builtin_amdgcn_s_waitcnt(0x0F70 | NSTAGE);      // everything but stage 1's own copies has landed
        } else {
            issue_loads(1, 1);
            __builtin_amdgcn_s_waitcnt(0x0F70 | NLOAD);       // vmcnt(NLOAD): stage 0 has landed
        }
        __syncthreads();
        if (PS) read_stage_scales(0);
        read_raw(raw[0], 0, 0, true);
        expand(op[0], raw[0], 0, 0);

        int buf = 0;
        for (int kt = 0; kt < nk; ++kt) {
            const int nbuf = buf == 2 ? 0 : buf + 1;
            issue_loads(kt + 2, nbuf == 2 ? 0 : nbuf + 1);
            if (PS) issue_scale_half((kt >> 1) + 2, kt & 1);
#pragma unroll
            for (int gs = 0; gs < STEPS; ++gs) {
                const int c = gs / 4, ks = gs % 4;
                if (ks == 1 && c + 1 < NC) read_raw(raw[(c + 1) & 1], buf, c + 1, kt * NC + c + 1 < nchunks);
                if (gs == STEPS - 2) {
                    __builtin_amdgcn_s_waitcnt(0x0F70 | NLOAD);   // all but the newest stage's loads: stage kt+1 has landed
                    __syncthreads();
                    if (PS) read_stage_scales(kt + 1);
                    read_raw(raw[0], nbuf, 0, (kt + 1) * NC < nchunks);
                }
                if (gs + 1 < STEPS) expand(op[(gs + 1) & 1], raw[((gs + 1) / 4) & 1], (gs + 1) / 4, (gs + 1) % 4);
                else expand(op[0], raw[0], 0, 0);
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j) {
                        float16_t &dst = OUTER ? part[i][j] : acc[i][j];
                        const float16_t addend = (OUTER && gs == 0) ? zero16 : dst;
                        dst = SWAP ? __builtin_amdgcn_mfma_f32_32x32x16_f16(op[gs & 1].b[j], op[gs & 1].a[i], addend, 0, 0, 0)
                                   : __builtin_amdgcn_mfma_f32_32x32x16_f16(op[gs & 1].a[i], op[gs & 1].b[j], addend, 0, 0, 0);
                    }
                // issue order: one MFMA, then (in the steps that fetch raw fragments) two LDS reads, then its
                // share of the expansion's VALU instructions
                const bool fetch = (ks == 1 && c + 1 < NC) || gs == STEPS - 2;
#pragma unroll
                for (int q = 0; q < TM * TN; ++q) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                    if (fetch && q < TM + TN) {
                        if (PS && gs != STEPS - 2) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                        else __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
                    }
                    __builtin_amdgcn_sched_group_barrier(0x002, (8 * (TM + TN) + TM * TN - 1) / (TM * TN) + 1, 0);
                }
            }
            if (OUTER) {
                // end of the stage = end of outer block kt: total += stage_sum * S_A[m] * S_B[n].  The block's scales
                // landed before the previous stage's barrier; ring slot kt % 4 is next written by the copies of stage
                // kt + 4, which are issued after the NEXT stage's barrier, so every wave is done reading by then.
                // The side that varies with the accumulator element (columns when SWAP, rows otherwise) is read as four
                // runs of four consecutive floats, the other side is one float per lane and tile.
                const float *gsr = reinterpret_cast<const float *>(smem_raw + GS_BASE) + (kt & 3) * ROWS;
                float s_lane[SWAP ? TM : TN];
                if (SWAP) {
#pragma unroll
                    for (int i = 0; i < TM; ++i) s_lane[i] = gsr[(wm * TM + i) * 32 + lr];
                } else {
#pragma unroll
                    for (int j = 0; j < TN; ++j) s_lane[j] = gsr[BM + (wn * TN + j) * 32 + lr];
                }
#pragma unroll
                for (int v = 0; v < (SWAP ? TN : TM); ++v) {
                    const float *base = SWAP ? gsr + BM + (wn * TN + v) * 32 + 4 * kg : gsr + (wm * TM + v) * 32 + 4 * kg;
                    float4 sv[4];
#pragma unroll
                    for (int q = 0; q < 4; ++q) sv[q] = *reinterpret_cast<const float4 *>(base + 8 * q);
#pragma unroll
                    for (int w = 0; w < (SWAP ? TM : TN); ++w) {
                        const int i = SWAP ? w : v, j = SWAP ? v : w;
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            acc[i][j][4 * q + 0] = __builtin_fmaf(part[i][j][4 * q + 0], sv[q].x * s_lane[w], acc[i][j][4 * q + 0]);
                            acc[i][j][4 * q + 1] = __builtin_fmaf(part[i][j][4 * q + 1], sv[q].y * s_lane[w], acc[i][j][4 * q + 1]);
                            acc[i][j][4 * q + 2] = __builtin_fmaf(part[i][j][4 * q + 2], sv[q].z * s_lane[w], acc[i][j][4 * q + 2]);
                            acc[i][j][4 * q + 3] = __builtin_fmaf(part[i][j][4 * q + 3], sv[q].w * s_lane[w], acc[i][j][4 * q + 3]);
                        }
                    }
                }
            }
            buf = nbuf;
        }
        __builtin_amdgcn_s_waitcnt(0x0F70);                // drain the look-ahead loads before the LDS is reused / released
    }
    // the epilogue stages its output in the pipeline's LDS: every wave's copies have landed and every wave is done
    // reading fragments
    if (SWAP) __syncthreads();

    store_tile<TM, TN, OUT, SWAP, OUTER>(acc, g, m0, n0, wm, wn, lr, kg, smem_raw);
}

template <int TM, int TN, int OUT, bool PS, int OUTER>
hipError_t launch_cfg(const GemmArgs &g, dim3 grid, hipStream_t st)
{
    constexpr int BM = 64 * TM, BN = 64 * TN;
    constexpr int lds = 3 * ((BM + BN) * 2 * kNC * 16 + (BM + BN) * (PS ? 16 : kNC * 4)) + (OUTER ? 4 * (BM + BN) * 4 : 0);
    auto kern = gemm_nt_kernel<TM, TN, kNC, OUT, PS, OUTER>;
    // once per instantiation; the initialisation of a function-local static is thread-safe
    static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                                       hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (attr != hipSuccess) return attr;
    hipLaunchKernelGGL(kern, grid, dim3(kThreads), lds, st, g);
    return hipGetLastError();
}

// tile: 0 256x256 (tensor mode only: block mode needs two accumulator sets), 1 256x128, 2 128x256, 3 128x128,
// 4 128x192 (paired scale fetch only)
template <int OUT, bool PS, int OUTER>
hipError_t launch_tile(int tile, const GemmArgs &g, dim3 grid, hipStream_t st)
{
    switch (tile) {
        case 0:
            if constexpr (OUTER == 0) return launch_cfg<4, 4, OUT, PS, 0>(g, grid, st);
            else return hipErrorInvalidValue;
        case 1: return launch_cfg<4, 2, OUT, PS, OUTER>(g, grid, st);
        case 2: return launch_cfg<2, 4, OUT, PS, OUTER>(g, grid, st);
        case 4:
            if constexpr (PS) return launch_cfg<2, 3, OUT, true, OUTER>(g, grid, st);
            else return hipErrorInvalidValue;
        default: return launch_cfg<2, 2, OUT, PS, OUTER>(g, grid, st);
    }
}

}  // namespace

}  // namespace tj
