// bf16 MFMA kernels of the mixed-batch LoRA linear layer for gfx950 (MI355X, wave64).
//
// Three kernels, all built from the same LDS tile format and bf16 MFMA inner product:
//   gemm_lora   y  = x W  + (s h) B_a        (forward;  W and B_a are [K][N])
//               dx = dy W^T + dh A_a^T       (backward; W and A_a are read [N][K])
//               One dense GEMM whose K loop is extended by 16-wide steps that multiply the
//               low-rank activations of the tile's rows with their adapter's table.
//   skinny      h  = x A_a, dh = s dy B_a^T  rank-wide outputs, HBM-bound; split over K with
//               fixed-order partial sums (no float atomics).
//   grad        dB_a = s h^T dy, dA_a = x^T dh   contraction over the adapter's training
//               tokens, rank x d outputs in fp32, split over tokens with ordered partials.
//
// LDS tile format: a tile holds R rows of 64 bf16 (128 bytes) along the contraction index.
// The row is cut into eight 16-byte chunks and chunk c of row r is stored at chunk position
// c ^ ((r ^ (r >> 3)) & 7).  A wave reading one chunk column of 32 consecutive rows, and a
// wave writing eight consecutive rows of one chunk column, both touch every bank once.
//
// MFMA operand layout (v_mfma_f32_32x32x16_bf16): lane l supplies 8 consecutive K values
// (one chunk) of row/column l % 32, K offset 8 * (l / 32); the result register j of lane l
// is element [8 * (j / 4) + 4 * (l / 32) + j % 4][l % 32].  (16x16x32: row/column l % 16,
// K offset 8 * (l / 16); result [4 * (l / 16) + j][l % 16].)  The GEMM tiles use the 16x16x32
// form: with real operand values it costs less power per flop, and the GEMMs are limited by
// power; the 32x32x16 form remains for the rank-wide tile pass (PARTIAL), which is bound by memory.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <algorithm>
#include <type_traits>

#include "kernels.h"

namespace collm {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi)
{
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    typedef float floatx2 __attribute__((ext_vector_type(2)));
    floatx2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

// Chunk swizzle of a K-major tile (rows of 128 bytes = 8 chunks of 16).  Measured on the device with the two
// fragment-read patterns (16 rows x 4 chunks per ds_read_b128 for the 16x16x32 MFMA, 32 rows x 2 chunks for the
// 32x32x16 one), four waves reading at once: this choice reads 1 KiB per wave in 28-29 cycles in both patterns;
// (row ^ (row >> 3)) & 7 takes 32 in the first and row & 7 takes 35 in the second (no swizzle: 64 and 128).
__device__ __forceinline__ int swz(int row) { return (row >> 1) & 7; }

// byte offset of chunk c of row r inside a tile
__device__ __forceinline__ int tile_off(int row, int c) { return row * 128 + ((c ^ swz(row)) << 4); }

__device__ __forceinline__ bf16x8 lds_frag(const uint8_t *tile, int row, int c)
{
    return *reinterpret_cast<const bf16x8 *>(tile + tile_off(row, c));
}

typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
// ds_read_b64_tr_b16: within each group of 16 lanes, lane s supplies the address of 4
// consecutive 16-bit values (row s / 4, columns 4 (s % 4) ..) of a 4 x 16 block and lane i
// receives column i of that block (checked on the device)
__device__ __forceinline__ bf16x4 lds_tr(const uint8_t *p)
{
    typedef short short4v __attribute__((ext_vector_type(4)));
    const short4v v = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (short4v __attribute__((address_space(3))) *)(p));
    return __builtin_bit_cast(bf16x4, v);
}

__device__ __forceinline__ uint4 ldg16(const void *p) { return *reinterpret_cast<const uint4 *>(p); }

// XCD-aware tile order: consecutive workgroup ids go round-robin to the 8 XCDs, each with
// its own L2.  Give every XCD one contiguous run of the logical tile order, and make that
// order walk groups of GM row tiles column by column so that concurrently running tiles of
// one XCD share rows of the first operand and columns of the second.
// band (a multiple of 8, or 0): the grid is walked in bands of that many row tiles, one band after the other, each
// in the order above.  What the chip works on at a time is then the band's rows of the first operand and the column
// tiles the XCDs are at; when all rows of the first operand together exceed the last-level cache (256 MB) but a band's
// fit, every column step after a band's first finds them there instead of in memory.
__host__ __device__ __forceinline__ void tile_coords(int pid, int tiles_m, int tiles_n, int band, int &tm, int &tn)
{
    int row0 = 0;
    if (band > 0 && band < tiles_m) {
        const int band_tiles = band * tiles_n;  // a multiple of 8: a band starts with XCD 0
        const int b = pid / band_tiles;
        pid -= b * band_tiles;
        row0 = b * band;
        tiles_m = tiles_m - row0 < band ? tiles_m - row0 : band;
    }
    const int total = tiles_m * tiles_n;
    const int per = total >> 3, rem = total & 7;
    const int xcd = pid & 7, local = pid >> 3;
    const int logical = xcd * per + (xcd < rem ? xcd : rem) + local;
    constexpr int GM = 8;
    const int group = logical / (GM * tiles_n);
    const int first = group * GM;
    const int gsz = (tiles_m - first) < GM ? (tiles_m - first) : GM;
    const int in_group = logical - group * GM * tiles_n;
    tm = row0 + first + in_group % gsz;
    tn = in_group / gsz;
}

// =========================================================================================
// gemm_lora
//
// Block tile BM x BN, K step 64, WGM x WGN waves of (BM/WGM) x (BN/WGN) each.  Software
// pipeline, two LDS stages filled by direct global -> LDS loads; operand fragments of the next
// MFMA phase are read from LDS while this one multiplies.
// Global loads are buffer loads: rows that do not exist (padding rows, columns beyond N,
// K tail) get an offset beyond the buffer and read as zero, so the loop has no branches.
// =========================================================================================
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
constexpr uint32_t kOob = 0x80000000u;  // beyond any buffer (tensors are limited to 2 GiB)

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void *base, uint32_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, bytes, 0x00020000);
}
__device__ __forceinline__ uint4 buf16(__amdgpu_buffer_rsrc_t r, uint32_t off)
{
    const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(r, off, 0, 0);
    return make_uint4(v.x, v.y, v.z, v.w);
}

// Direct global -> LDS load of 16 bytes per lane (buffer_load_dwordx4 ... lds): the 64 lanes
// of a wave fill 1 KiB of LDS starting at the wave-uniform address `lds_base`, lane l at
// lds_base + 16 l; which 16 bytes a lane fetches is up to its own offset, so any permutation
// inside that KiB is free.  Out-of-range offsets deliver zeros.  The load is tracked by vmcnt
// only; the compiler does not know it writes LDS, so the code that issues it also waits
// (s_waitcnt vmcnt(0)) before the barrier that publishes the data.
typedef int i32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ i32x4 make_rsrc_words(const void *base, uint32_t bytes)
{
    const uint64_t b = reinterpret_cast<uint64_t>(base);
    i32x4 r;
    r.x = (int)(uint32_t)b;
    r.y = (int)((uint32_t)(b >> 32) & 0xffffu);
    r.z = (int)bytes;
    r.w = 0x00020000;
    return r;
}
__device__ __forceinline__ void dma16(i32x4 rsrc, uint32_t voff, uint32_t lds_base)
{
    asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds" ::"s"(lds_base), "v"(voff), "s"(rsrc) : "m0", "memory");
}
// the same with a wave-uniform byte offset added to every lane's address (not part of the range check)
__device__ __forceinline__ void dma16s(i32x4 rsrc, uint32_t voff, uint32_t soff, uint32_t lds_base)
{
    asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds" ::"s"(lds_base), "v"(voff), "s"(rsrc), "s"(soff) : "m0", "memory");
}
// the same from a 64-bit address per lane (no range check)
__device__ __forceinline__ void dma16g(uint64_t addr, uint32_t lds_base)
{
    asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_base), "v"(addr) : "m0", "memory");
}
// One v_mfma_f32_16x16x32_bf16, accumulator in place.  Written out because the compiler's register allocation of
// the builtin breaks down with 64 four-register accumulators per lane (it copies them between the two register
// files around the MFMAs).  The waits for operands that LDS reads deliver are still placed by the compiler; the
// wait states between the last MFMA and the first ordinary read of an accumulator are the caller's (mfma16_settle).
__device__ __forceinline__ void mfma16(floatx4 &c, const bf16x8 &a, const bf16x8 &b)
{
    asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(c) : "v"(a), "v"(b));
}
__device__ __forceinline__ void mfma16_settle() { asm volatile("s_nop 7\n\ts_nop 7" ::: "memory"); }
__device__ __forceinline__ void wait_dma() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }
template <int N> __device__ __forceinline__ void wait_dma_but() { asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory"); }
// every load and LDS read of this wave has completed, then meet the other waves
__device__ __forceinline__ void drain_and_barrier() { asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// Four consecutive extension steps of a row tile, unpacked into wave-uniform registers.
struct ExtBatch {
    uint32_t kr[kExtBatch];    // koff | rank << 16   (0: no step)
    uint32_t rows[kExtBatch];  // row_lo | row_hi << 16
    uint64_t tab[kExtBatch];
};

// Which direct load rides behind which MFMA.  A K tile of the direct-load pipeline has three phases
// in which loads may be issued: the MFMAs of step 3 that follow the barrier (phase 0), step 0 (phase 1)
// and step 1 (phase 2).  Measured on the 256 x 256 tile: bunching loads (one per MFMA) stalls the wave
// on the CU's load path, issuing them late leaves the last ones too little time to land; 3/8 of the
// loads in phase 0, 1/2 in phase 1 and the rest at the start of phase 2, evenly spaced inside a phase,
// was the best split.  slot[phase][m] is the load issued behind MFMA m, or -1.
template <int NM, int PRE, int ND, int N0 = ND * 3 / 8, int N1 = ND / 2>
struct DmaSlots {
    int slot[3][NM];
    int n[3];
    constexpr DmaSlots() : slot{}, n{N0, N1, ND - N0 - N1}
    {
        int d = 0;
        for (int ph = 0; ph < 3; ++ph) {
            const int lo = ph == 0 ? PRE : 0, width = NM - lo;
            // more loads than slots cannot happen for the tile shapes in use (checked by the caller)
            for (int m = 0; m < NM; ++m) slot[ph][m] = -1;
            for (int i = 0; i < n[ph]; ++i) {
                int m = lo + (ph == 2 ? i : i * width / n[ph]);  // phase 2: as early as possible
                while (m < NM && slot[ph][m] >= 0) ++m;
                if (m < NM) slot[ph][m] = d++;
            }
        }
    }
    constexpr int placed() const
    {
        int c = 0;
        for (int ph = 0; ph < 3; ++ph)
            for (int m = 0; m < NM; ++m) c += slot[ph][m] >= 0;
        return c;
    }
};

// Block `blk` of `n_blk` reads its contiguous share of `bytes` bytes at `base` (16-byte aligned), sixteen 16-byte loads
// per thread in flight (the share of a block is mostly one such round: what counts is that everything is asked for
// at once), and drops them.  The values are folded into a word that is stored only if it takes a value the data
// cannot be relied on never to produce and the size is one that never occurs, so that the loads stay.
__device__ __forceinline__ void warm_cache(const void *base, uint64_t bytes, int blk, int n_blk, int tid, int n_thr)
{
    constexpr int U = 16;
    const uint64_t per = ((bytes / 16 + n_blk - 1) / n_blk) * 16;
    const uint64_t lo = (uint64_t)blk * per, hi = lo + per < bytes ? lo + per : bytes;
    const uint8_t *src = reinterpret_cast<const uint8_t *>(base);
    uint32_t fold = 0;
    for (uint64_t off = lo + (uint64_t)tid * 16; off < hi; off += (uint64_t)n_thr * 16 * U) {
        uint4 v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint64_t o = off + (uint64_t)u * n_thr * 16;
            v[u] = o + 16 <= hi ? ldg16(src + o) : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) fold ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
    }
    if (fold == 0x9e3779b9u && bytes == 1) *reinterpret_cast<volatile uint32_t *>(const_cast<void *>(base)) = fold;
}

// PARTIAL: the same tile machinery as a rank-wide pass over long runs of one adapter's rows.  A
// block takes one item (up to BM rows of one adapter, blockIdx.x), BN of the adapter's rank
// columns (blockIdx.y) and one slice of K (blockIdx.z); the second operand is the adapter's own
// table; there are no extension steps, and the fp32 sums go to the workspace of partial sums that
// skinny_finish_kernel adds up.
// SWIGLU (N-major second operand, WGN = 2): a column tile holds BN / 2 gate columns j0 .. and the BN / 2 up
// columns act_col + j0 .. of the same outputs; the waves of the left half hold the gate values, those
// of the right half the up values of the same rows.  The extension steps run over both siblings' ranks
// (rank r each, multiples of 16): a step of the first r multiplies into the gate half only, one of the
// second r into the up half only.  In the epilogue the two waves that hold the gate and the up values of the
// same rows swap halves through LDS, each finishes half of the rows: silu(gate) * up, rounded once, stored as
// [rows][N = d_ff]; training rows also keep both pre-activations.
// SIBS: sibling projections side by side in the columns; the low-rank extension then loads the rows' operand per
// batch at the sibling's offset inside each adapter's ranks (see the extension below).
// SPLITK: the GEMM itself with K cut into gridDim.y slices (few rows against a long contraction: too few tiles to
// fill the GPU).  A block takes one tile and one slice; slice 0 also runs the tile's extension steps; the fp32
// sums go to the workspace and gemm_finish_kernel adds the slices, rounds once and scatters the rows.
// LDS stages of the PARTIAL loop (128x128 tiles: 32 KiB each).  The loop is bound by what a wave has to issue per
// tile (its direct loads, then its fragment reads and MFMAs, one wave per SIMD), not by the latency of the loads
// (about 800 cycles from L2 or beyond): with tables as they lie in memory ([K][rank], transposing reads) two
// blocks per CU whose phases interleave, two stages each, beat one block with four; with K-major tables
// (fewer, cheaper fragment reads) the four stages do.
constexpr int kWideStages = 4;
constexpr int wide_stages(bool t_kmajor) { return t_kmajor ? kWideStages : 2; }
template <int BM, int BN, int WGM, int WGN, bool B_KMAJOR, bool PARTIAL = false, bool SWIGLU = false, bool SPLITK = false,
          bool SIBS = false>
__global__ void __launch_bounds__(WGM *WGN * 64, (!PARTIAL && BM * BN == 128 * 128) ? 2 : 1) gemm_lora_kernel(GemmArgs p)
{
    // the GEMM tiles run the 16x16x32 MFMA form, the rank-wide pass the 32x32x16 one
    constexpr bool M16 = !PARTIAL;
    static_assert(!SWIGLU || (!B_KMAJOR && !PARTIAL && WGN == 2), "SwiGLU epilogue: N-major, two wave columns");
    static_assert(!SPLITK || (!PARTIAL && !SWIGLU), "K slices: plain tiles only");
    constexpr int NT = WGM * WGN * 64;
    constexpr int WM = BM / WGM, WN = BN / WGN;
    constexpr int MI = WM / 32, NI = WN / 32;
    // second operand in LDS: K-major -> BN rows of 64 K values (swizzled chunks); N-major ->
    // 64 rows (K) of BN values as they lie in memory, chunk c of row k stored at chunk position
    // c ^ ((k & 3) << 2) so that the four rows a transposing read touches use different banks (16x16x32 form:
    // also ^ 2 for rows 8-15 of every 16, see bcl_of)
    constexpr int BPITCH = BN * 2;
    constexpr int BTILE = B_KMAJOR ? BN * 128 : 64 * BPITCH;
    constexpr int ATILE = BM * 128;
    constexpr int STAGE = ATILE + BTILE;
    // LDS map [A0 A1 B0 B1], so that the fragment reads of both stages lie within the immediate-offset range of
    // one per-lane base.
    constexpr int A_ST1 = ATILE;
    constexpr int B_ST0 = 2 * ATILE;
    constexpr int B_ST1 = 2 * ATILE + BTILE;
    constexpr int ACH = BM * 8 / NT;   // 16-byte chunks of the row tile per thread
    constexpr int BCH = BN * 8 / NT;   // chunks of the second operand's tile per thread
    constexpr int NG = BN / 8;         // chunks per N-major row
    static_assert((BM * 8) % NT == 0 && (BN * 8) % NT == 0 && NT % NG == 0 && (NT / NG) % 4 == 0, "tile/thread mismatch");
    static_assert(ACH % 4 == 0 || ACH == 2, "row chunks are moved in four (or two) parts per K step");
    extern __shared__ __align__(16) uint8_t smem[];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave % WGM, wn = wave / WGM;
    int tile_m, tile_n;
    int m0, K, N, rows_in = BM;
    const void *a_base = p.a, *b_base = p.b;
    uint32_t a_bytes = p.a_bytes, b_bytes = p.b_bytes, ldb = (uint32_t)p.ldb;
    if constexpr (PARTIAL) {
        if (blockIdx.x >= (unsigned)p.n_items) {
            // a warm-up block: its share of the next GEMM's weight, read once and dropped
            if (blockIdx.y == 0 && blockIdx.z == 0) warm_cache(p.warm_base, p.warm_bytes, blockIdx.x - p.n_items, p.warm_blocks, tid, NT);
            return;
        }
        // consecutive items mostly belong to one adapter; blocks go round-robin to the 8 XCDs, so give every XCD a
        // contiguous run of the items: an adapter's table then comes through one L2 instead of eight
        const int n_it = p.n_items, per = n_it >> 3, rem = n_it & 7, xc = blockIdx.x & 7;
        tile_m = xc * per + (xc < rem ? xc : rem) + (blockIdx.x >> 3);
        const SkinnyItem it = p.items[tile_m];
        tile_n = blockIdx.y;
        m0 = it.row_lo;
        rows_in = it.n_rows;
        N = p.part_n_sib > 1 ? it.rank / p.part_n_sib : it.rank;
        // the block's slice of K: both operands start at its first K index, and the second one ends
        // with the slice (its rows beyond it must read as zeros)
        const int k_begin = blockIdx.z * p.k_per_split;
        K = p.K - k_begin < p.k_per_split ? p.K - k_begin : p.k_per_split;
        ldb = B_KMAJOR ? (uint32_t)(p.tab_ld ? p.tab_ld : p.K) : (uint32_t)N;
        const uint32_t a_skip = (uint32_t)k_begin * 2u;
        const uint32_t b_skip = B_KMAJOR ? (uint32_t)(k_begin + p.tab_off) * 2u : (uint32_t)k_begin * ldb * 2u;
        a_base = reinterpret_cast<const uint8_t *>(p.a) + a_skip;
        a_bytes = p.a_bytes - a_skip;
        b_base = reinterpret_cast<const uint8_t *>(p.tab[it.adapter]) + b_skip;
        b_bytes = B_KMAJOR ? (uint32_t)N * ldb * 2u - b_skip : (uint32_t)K * ldb * 2u;
    } else {
        tile_coords(blockIdx.x, p.tiles_m, p.tiles_n, p.band_m, tile_m, tile_n);
        tile_m += p.tile_m_base;
        m0 = tile_m * BM;
        K = p.K;
        N = p.N;
        if constexpr (SPLITK) {
            // the block's slice of K, as above
            const int k_begin = blockIdx.y * p.k_per_split;
            K = p.K - k_begin < p.k_per_split ? p.K - k_begin : p.k_per_split;
            const uint32_t a_skip = (uint32_t)k_begin * 2u;
            const uint32_t b_skip = B_KMAJOR ? (uint32_t)k_begin * 2u : (uint32_t)k_begin * ldb * 2u;
            a_base = reinterpret_cast<const uint8_t *>(p.a) + a_skip;
            a_bytes = p.a_bytes - a_skip;
            b_base = reinterpret_cast<const uint8_t *>(p.b) + b_skip;
            b_bytes = B_KMAJOR ? p.b_bytes - b_skip : (uint32_t)K * ldb * 2u;
        }
    }
    const int n0 = SWIGLU ? tile_n * (BN / 2) : (PARTIAL ? 0 : p.n_base) + tile_n * BN;
    // tile column c (a multiple of 8) -> column of the second operand and of the expand tables
    auto src_col = [&](int c) -> int {
        if constexpr (SWIGLU) return c < BN / 2 ? n0 + c : p.act_col + n0 + c - BN / 2;
        return n0 + c;
    };
    // ... and whether that column exists (N: columns of the output)
    auto col_on = [&](int c) -> bool {
        if constexpr (SWIGLU) return n0 + (c < BN / 2 ? c : c - BN / 2) < N;
        return n0 + c < N;
    };
    const int32_t *__restrict__ row_tok = p.row_tok;
    int sib = 0;  // which of the sibling projections this column tile belongs to
    if constexpr (!PARTIAL) {
#pragma unroll
        for (int j = 0; j < 3; ++j)
            if (j + 1 < p.n_sib && n0 >= p.sib_col[j]) sib = j + 1;
    }


    // The block's first loads form chains (row order -> rows of the first operand; step offsets -> step records),
    // and nothing else runs on the CU meanwhile (256x256) or little (128x128): the chains are started side by
    // side, the tokens of this thread's rows first.
    const int c8 = tid & 7, r8 = tid >> 3;
    int tok_of[BM * 8 / NT];
#pragma unroll
    for (int i = 0; i < BM * 8 / NT; ++i) {
        const int r = r8 + i * (NT / 8);
        tok_of[i] = (!PARTIAL || r < rows_in) ? row_tok[m0 + r] : -1;
    }

    // extension steps of this row tile; the first batch is fetched now, long before it is needed
    const int e0 = PARTIAL ? 0 : __builtin_amdgcn_readfirstlane(p.ext_off[tile_m]);
    const int e1 = PARTIAL ? 0 : ((SPLITK && blockIdx.y != 0) ? e0 : __builtin_amdgcn_readfirstlane(p.ext_off[tile_m + 1]));
    // The records of a batch come through the scalar cache (their own counter, so waiting for them
    // does not wait for the direct loads in flight).  Load and wait are one statement: registers
    // that a load is still writing must never be visible to the compiler, which may move or spill
    // them.  The step array is padded by a batch, and the index is clamped to the tile's last step,
    // so the 64 bytes read always lie inside it.
    typedef uint32_t u32x16 __attribute__((ext_vector_type(16)));
    auto fetch_batch = [&](int eb) {
        const int last = e1 > 0 ? e1 - 1 : 0;
        const int idx = eb < last ? eb : last;
        const uint64_t addr = reinterpret_cast<uint64_t>(p.ext) + (uint64_t)idx * sizeof(ExtStep);
        u32x16 raw;
        asm volatile("s_load_dwordx16 %0, %1, 0x0\n\ts_waitcnt lgkmcnt(0)" : "=&s"(raw) : "s"(addr));
        ExtBatch bt;
#pragma unroll
        for (int j = 0; j < kExtBatch; ++j) {
            const bool on = eb + j < e1;
            bt.kr[j] = on ? raw[4 * j] : 0u;
            bt.rows[j] = on ? raw[4 * j + 1] : 0u;
            bt.tab[j] = ((uint64_t)raw[4 * j + 3] << 32) | raw[4 * j + 2];
        }
        return bt;
    };
    // The first 64 step records of the tile are fetched once, one per lane (the load completes before any direct
    // load is in flight, see below); a batch then comes out of the lanes with readlane.  (Tiles with more steps fetch the later
    // batches through the scalar cache.)
    uint4 rec = make_uint4(0u, 0u, 0u, 0u);
    if constexpr (!PARTIAL) {
        if (e0 + lane < e1) rec = *reinterpret_cast<const uint4 *>(p.ext + e0 + lane);
    }
    auto get_batch = [&](int eb) {
        const int rel = eb - e0;
        if (rel + kExtBatch > 64) return fetch_batch(eb);
        ExtBatch bt;
#pragma unroll
        for (int j = 0; j < kExtBatch; ++j) {
            const bool on = eb + j < e1;
            const uint32_t kr = (uint32_t)__builtin_amdgcn_readlane((int)rec.x, rel + j);
            const uint32_t rows = (uint32_t)__builtin_amdgcn_readlane((int)rec.y, rel + j);
            const uint32_t tlo = (uint32_t)__builtin_amdgcn_readlane((int)rec.z, rel + j);
            const uint32_t thi = (uint32_t)__builtin_amdgcn_readlane((int)rec.w, rel + j);
            bt.kr[j] = on ? kr : 0u;
            bt.rows[j] = on ? rows : 0u;
            bt.tab[j] = ((uint64_t)thi << 32) | tlo;
        }
        return bt;
    };

    // ---- per-thread source offsets (bytes) ------------------------------------------------
    // A thread owns fixed LDS positions: in K-major tiles row r8 + i NT/8, chunk position c8;
    // in the N-major tile row bk0 + i NT/NG, chunk position bng.  The 64 lanes of a wave own
    // one contiguous KiB per i, which is what a direct-to-LDS load fills.  The swizzle decides
    // which chunk of the source belongs at that position.
    // rows r8 + i NT/8 (NT/8 = 32 or 64) all have the swizzle of row r8
    static_assert((NT / 8) % 16 == 0, "the swizzle repeats every 16 rows");
    const int cl0 = c8 ^ swz(r8);  // source chunk of this thread, for every i
    uint32_t aoff[ACH];
#pragma unroll
    for (int i = 0; i < ACH; ++i) {
        const int tok = tok_of[i];
        const int cl = cl0;
        aoff[i] = tok >= 0 ? (uint32_t)tok * (uint32_t)p.lda * 2u + cl * 16u : kOob;
    }
    constexpr int NB = BCH;
    uint32_t boff[NB];
    uint32_t bstep = 0;  // N-major: advance of one K step, zero for columns beyond N
    const uint32_t bstep_u = 64u * ldb * 2u;  // the same as a wave-uniform value
    const int bng = tid % NG, bk0 = tid / NG;
    const int bcl = bng ^ ((bk0 & 3) << 2);  // N-major: source chunk of this thread (same for all i)
    // 16x16x32 form: a transposing read takes K rows r .. r + 3 in one lane group and r + 8 .. r + 11 in the next,
    // so rows 8-15 of every 16 are stored with their chunk pairs swapped: the source chunk then depends on i
    auto bcl_of = [&](int i) { return M16 ? bcl ^ ((((bk0 + i * (NT / NG)) >> 3) & 1) << 1) : bcl; };
    if constexpr (B_KMAJOR) {
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            const int n = n0 + r8 + i * (NT / 8);
            const int cl = cl0;
            boff[i] = n < N ? (uint32_t)n * ldb * 2u + cl * 16u : kOob;
        }
    } else {
        const bool on = col_on(bcl * 8);
        bstep = on ? 64u * ldb * 2u : 0u;
#pragma unroll
        for (int i = 0; i < NB; ++i)
            boff[i] = col_on(bcl_of(i) * 8) ? ((uint32_t)(bk0 + i * (NT / NG)) * ldb + src_col(bcl_of(i) * 8)) * 2u : kOob;
    }
    // byte offset of the tile that starts at K index k0 = 64 kc, for chunk i; tiles that reach
    // beyond K mask their tail (K-major) or run off the end of the buffer (N-major rows)
    auto a_src = [&](int i, int k0, bool full) -> uint32_t {
        const int cl = cl0;
        return (full || k0 + cl * 8 < K) ? aoff[i] + (uint32_t)k0 * 2u : kOob;
    };
    auto b_src = [&](int i, int k0, int kc, bool full) -> uint32_t {
        if constexpr (B_KMAJOR) {
            const int cl = cl0;
            return (full || k0 + cl * 8 < K) ? boff[i] + (uint32_t)k0 * 2u : kOob;
        } else {
            if constexpr (M16) return boff[i] == kOob ? kOob : boff[i] + (uint32_t)kc * bstep_u;
            return boff[i] + (uint32_t)kc * bstep;
        }
    };

    // chunk idx (row chunks first, then the second operand's) of the tile that starts
    // at K index 64 kc goes to `stage`; the wave's 64 lanes fill the KiB (i NT/64 + wave) of the tile
    const i32x4 ra_w = make_rsrc_words(a_base, a_bytes), rb_w = make_rsrc_words(b_base, b_bytes);
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint8_t *)smem;
    const uint32_t lds_wave = __builtin_amdgcn_readfirstlane(lds0 + wave * 1024);
    constexpr int ND = ACH + BCH;
    const int nk = (K + 63) >> 6;
    const bool k_even = (K & 63) == 0;
    // a tile beyond the last one gets a resource of size zero: every lane is out of range, nothing is
    // fetched and the stage it would have gone to is never read
    auto tile_rsrc = [&](i32x4 r, int kc) -> i32x4 {
        r.z = kc < nk ? r.z : 0;
        return r;
    };
    // even_c: K is a multiple of 64, so no lane of a tile below nk needs masking and the K offset of the
    // tile can travel as the instruction's scalar offset
    auto dma_chunk = [&](auto even_c, int idx, int stage, int kc, i32x4 ra_t, i32x4 rb_t) {
        constexpr bool even = decltype(even_c)::value;
        const int k0 = kc << 6;
        if (idx < ACH) {
            const uint32_t dst = lds_wave + (stage ? A_ST1 : 0) + idx * (NT / 64) * 1024;
            if constexpr (even) dma16s(ra_t, aoff[idx], (uint32_t)k0 * 2u, dst);
            else dma16(ra_t, a_src(idx, k0, false), dst);
        } else {
            const int i = idx - ACH;
            const uint32_t dst = lds_wave + (stage ? B_ST1 : B_ST0) + i * (NT / 64) * 1024;
            if constexpr (even) dma16s(rb_t, boff[i], B_KMAJOR ? (uint32_t)k0 * 2u : (uint32_t)kc * bstep_u, dst);
            else dma16(rb_t, b_src(i, k0, kc, false), dst);
        }
    };

    // ---- loads of the low-rank extension (used from the last tiles of the main loop on) ------
    // The extension steps after the main loop are taken four at a time (one 64-wide K tile); the operands of
    // such a batch travel global -> LDS like the tiles of the main loop and take the same places in a stage.
    const i32x4 rh_w = make_rsrc_words(p.hs, p.hs_bytes);
    const uint64_t zeros = reinterpret_cast<uint64_t>(p.zeros);
    // per-lane choice among the four steps of a batch
    auto pick = [](int j, uint32_t v0, uint32_t v1, uint32_t v2, uint32_t v3) { return j == 0 ? v0 : (j == 1 ? v1 : (j == 2 ? v2 : v3)); };
    // piece d of a batch: chunk d of the rows' operand (into the LDS area at byte a_base), or chunk d - ACH of
    // the tables' (area at b_base); called with d known after unrolling: the branches and the step index fold away.
    // once: the rows' operand is not that of the batch but rank indices 64 g .. 64 g + 63 of every row's own s h
    // (or dh), whatever its adapter: it is loaded once for the whole tile and masked per step when it is used.
    auto issue_piece = [&](uint32_t a_base, uint32_t b_base, const ExtBatch &bt, const int D, const bool once, const int g) {
        if (D < ACH && once) {
            const int i = D;
            const int r = r8 + i * (NT / 8);
            const int cl = cl0;
            const int k = 64 * g + cl * 8;
            const uint32_t off = k < p.hs_ld ? ((uint32_t)(m0 + r) * (uint32_t)p.hs_ld + (uint32_t)k) * 2u : kOob;
            dma16(rh_w, off, lds_wave + a_base + i * (NT / 64) * 1024);
        } else if (D < ACH) {
            // rows: position c8 of row r holds chunk cl; chunk cl belongs to step cl / 2, rank
            // indices koff + 8 (cl % 2) ..
            const int i = D;
            const int r = r8 + i * (NT / 8);
            const int cl = cl0;
            const int j = cl >> 1;
            const uint32_t kr = pick(j, bt.kr[0], bt.kr[1], bt.kr[2], bt.kr[3]);
            const uint32_t rows = pick(j, bt.rows[0], bt.rows[1], bt.rows[2], bt.rows[3]);
            // siblings: the columns after a sibling's own are the next sibling's, or were never written
            const bool in = r >= (int)(rows & 0xffffu) && r < (int)(rows >> 16) &&
                            (p.n_sib <= 1 || (kr & 0xffffu) + (cl & 1) * 8u < (kr >> 16));
            const uint32_t off = in ? ((uint32_t)(m0 + r) * (uint32_t)p.hs_ld + (uint32_t)sib * (kr >> 16) + (kr & 0xffffu) + (cl & 1) * 8u) * 2u : kOob;
            dma16(rh_w, off, lds_wave + a_base + i * (NT / 64) * 1024);
        } else if constexpr (!B_KMAJOR) {
            // table rows are rank indices: B_a[q][n]; tile row 16 j + i is rank index koff_j + i.
            // All lanes of a load belong to one step, whose table is the load's buffer: rank
            // indices beyond the rank lie beyond it.
            static_assert(16 % (NT / NG) == 0 || (NT / NG) % 16 == 0, "a direct load must not straddle two steps");
            const int i = D - ACH;
            const int j = (i * (NT / NG)) >> 4;
            const int k = bk0 + i * (NT / NG);
            uint32_t rk = bt.kr[j] >> 16, koff = bt.kr[j] & 0xffffu;
            bool mine = true;
            if constexpr (SWIGLU) {
                // the step belongs to the gate sibling (first half of the ranks) or the up sibling
                rk >>= 1;
                const bool up = koff >= rk;
                koff -= up ? rk : 0u;
                mine = (bcl * 8 >= BN / 2) == up;
            }
            const int bcl_i = bcl_of(i);
            const i32x4 rt = make_rsrc_words(reinterpret_cast<const void *>(bt.tab[j]), rk * (uint32_t)p.ext_ld * 2u);
            const uint32_t off = (mine && col_on(bcl_i * 8)) ? ((koff + (uint32_t)(k & 15)) * (uint32_t)p.ext_ld + (uint32_t)src_col(bcl_i * 8)) * 2u : kOob;
            dma16(rt, off, lds_wave + b_base + i * (NT / 64) * 1024);
        } else {
            // table rows are output columns: A_a[n][q], row length rank.  The four steps of a
            // batch may have four tables, so every lane forms its own 64-bit address.
            const int i = D - ACH;
            const bool all8 = (((bt.kr[0] | bt.kr[1] | bt.kr[2] | bt.kr[3]) >> 16) & 7u) == 0;
            const int r = r8 + i * (NT / 8);
            const int cl = cl0;
            const int j = cl >> 1;
            const uint32_t kr = pick(j, bt.kr[0], bt.kr[1], bt.kr[2], bt.kr[3]);
            const uint32_t tlo = pick(j, (uint32_t)bt.tab[0], (uint32_t)bt.tab[1], (uint32_t)bt.tab[2], (uint32_t)bt.tab[3]);
            const uint32_t thi = pick(j, (uint32_t)(bt.tab[0] >> 32), (uint32_t)(bt.tab[1] >> 32), (uint32_t)(bt.tab[2] >> 32), (uint32_t)(bt.tab[3] >> 32));
            if (all8) {
                const uint32_t rk = kr >> 16, q0 = (kr & 0xffffu) + (cl & 1) * 8u;
                const bool in = n0 + r < N && q0 < rk;
                const uint64_t addr = in ? (((uint64_t)thi << 32) | tlo) + ((uint64_t)(n0 + r) * rk + q0) * 2u : zeros;
                dma16g(addr, lds_wave + b_base + i * (NT / 64) * 1024);
            } else {
                // some rank is no multiple of 8: table rows are not 16-byte aligned; element by element
                uint8_t *tb = smem + b_base;
                const int rk = (int)(kr >> 16), q0 = (int)(kr & 0xffffu) + (cl & 1) * 8;
                uint16_t e[8];
#pragma unroll
                for (int q = 0; q < 8; ++q) e[q] = 0;
                if (n0 + r < N) {
                    const uint16_t *src = reinterpret_cast<const uint16_t *>(((uint64_t)thi << 32) | tlo) + (int64_t)(n0 + r) * rk + q0;
#pragma unroll
                    for (int q = 0; q < 8; ++q)
                        if (q0 + q < rk) e[q] = src[q];
                }
                uint4 v;
                v.x = e[0] | ((uint32_t)e[1] << 16);
                v.y = e[2] | ((uint32_t)e[3] << 16);
                v.z = e[4] | ((uint32_t)e[5] << 16);
                v.w = e[6] | ((uint32_t)e[7] << 16);
                *reinterpret_cast<uint4 *>(tb + (r8 + i * (NT / 8)) * 128 + c8 * 16) = v;
            }
        }
    };

    // The 256x256 tiles use what the main loop's two stages leave of the LDS (32 KiB of 160): the rows' area of the
    // extension lies behind them and is loaded before the main loop starts.
    constexpr bool ROWS_EARLY = !PARTIAL && !SIBS && BM * BN == 256 * 256;
    constexpr uint32_t XA_EARLY = 2 * STAGE;
    // The load of the step records is waited for behind the direct loads of the first tile (the records' chain of
    // two loads is longer than the one that leads to those loads, and nothing needs the records before the main
    // loop's last tiles).
    auto records_are_in = [&] { asm volatile("" : "+v"(rec.x), "+v"(rec.y), "+v"(rec.z), "+v"(rec.w)); };
    if constexpr (ROWS_EARLY) {
        if (e1 > e0) {
#pragma unroll
            for (int d = 0; d < ACH; ++d) issue_piece(XA_EARLY, 0u, ExtBatch{}, d, true, 0);
        }
    }
    // rank-wide pass: acc[ni][mi] holds the transposed 32x32 block: lane = row m, registers = columns n
    floatx16 acc[PARTIAL ? NI : 1][PARTIAL ? MI : 1];
    if constexpr (PARTIAL) {
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                for (int j = 0; j < 16; ++j) acc[ni][mi][j] = 0.f;
    }
    const int rl = lane & 31, kh = lane >> 5;
    bf16x8 af[2][PARTIAL ? MI : 1], bf[2][PARTIAL ? NI : 1];
    // 16x16x32 form: lane l supplies row (or column) l % 16 and K values 8 (l / 16) .. of a 32-wide K step; acc4[ni][mi]
    // holds the transposed 16x16 block: lane = row l % 16, registers = columns 4 (l / 16) .. + 3.  The row blocks of a
    // wave go in two halves of MH (a4, double-buffered by half); the second operand's fragments (b8) are single:
    // each is read again as soon as the last MFMA of the step that uses it has been issued.
    constexpr int MI16 = WM / 16, NI16 = WN / 16, MH = MI16 / 2, NM16 = NI16 * MH;
    floatx4 acc4[M16 ? NI16 : 1][M16 ? MI16 : 1];
    bf16x8 a4[2][M16 ? MH : 1], b8[M16 ? NI16 : 1];
    const int r16 = lane & 15, kq = lane >> 4;
    if constexpr (M16) {
#pragma unroll
        for (int ni = 0; ni < NI16; ++ni)
#pragma unroll
            for (int mi = 0; mi < MI16; ++mi) acc4[ni][mi] = floatx4{0.f, 0.f, 0.f, 0.f};
    }
    // phase ph of a K tile: K step ph / 2 (32 wide), row half ph % 2.  j-th fragment read for phase ph: the MH row
    // blocks of its half, then (first half of a step only) the NI16 blocks of the second operand
    // N-major second operand: byte offset of this lane's transposing reads for K step 0 (16 lanes fetch a 4 (K) x 16 (N)
    // block; lane group g takes K rows 8 g ..)
    uint32_t btr16[(M16 && !B_KMAJOR) ? NI16 : 1];
    if constexpr (M16 && !B_KMAJOR) {
        const int krow = kq * 8 + (r16 >> 2);
#pragma unroll
        for (int ni = 0; ni < NI16; ++ni) {
            const int col = wn * WN + ni * 16 + (r16 & 3) * 4;
            btr16[ni] = krow * BPITCH + ((((col >> 3) ^ ((krow & 3) << 2) ^ (((krow >> 3) & 1) << 1))) << 4) + (col & 7) * 2;
        }
    }
    // second-operand fragment ni of the 32-wide K step ks of the tile at tb
    auto read_b16 = [&](const uint8_t *tb, int ks, int ni) {
        if constexpr (B_KMAJOR) {
            b8[ni] = lds_frag(tb, wn * WN + ni * 16 + r16, ks * 4 + kq);
        } else {
            const uint8_t *src = tb + btr16[ni] + ks * 32 * BPITCH;
            const bf16x4 lo = lds_tr(src);
            const bf16x4 hi = lds_tr(src + 4 * BPITCH);
            b8[ni] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        }
    };
    auto read16 = [&](int stage, int ph, int j) {
        const uint8_t *ta = smem + (stage ? A_ST1 : 0);
        const uint8_t *tb = smem + (stage ? B_ST1 : B_ST0);
        if (j < MH) a4[ph & 1][j] = lds_frag(ta, wm * WM + ((ph & 1) * MH + j) * 16 + r16, (ph >> 1) * 4 + kq);
        else read_b16(tb, ph >> 1, j - MH);
    };
    auto mma16 = [&](int ph, int m) {
        const int ni = m / MH, mi = m % MH;
        mfma16(acc4[ni][(ph & 1) * MH + mi], b8[ni], a4[ph & 1][mi]);
    };
    // The reads for phase nph that ride behind MFMA m of the phase before it (`first`: the first MFMA they may
    // follow).  Only two or three other instructions fit behind a 16-cycle MFMA, so an MFMA carries at most one
    // memory instruction: the direct loads sit behind MFMAs 0, 4, 8, .. (DmaSlots), the row fragments behind
    // first + 2, + 6, .., the second operand's behind the last MFMA that uses the register (3, 7, ..: odd).
    auto reads16 = [&](int stage, int nph, int m, int first) {
#pragma unroll
        for (int i = 0; i < MH; ++i)
            if (m == (MH == 4 ? first + 2 + 4 * i : first + 2 * i)) read16(stage, nph, i);
        if ((nph & 1) == 0) {
#pragma unroll
            for (int ni = 0; ni < NI16; ++ni) {
                const int last_use = ni * MH + MH - 1, early = MH == 4 ? first + 1 + 2 * ni : first + ni;
                const int slot = last_use > early ? last_use : early;
                if (m == slot) read16(stage, nph, MH + ni);
            }
        }
    };
    static_assert(!M16 || (MH == 4 && NM16 / 4 + 2 + 4 * (MH - 1) < NM16) || (MH == 2 && NM16 == 8), "the read slots above are laid out for four (or two) row blocks per half");
    // N-major operand: byte offset of this lane's transposing read inside the tile for K step 0
    uint32_t btr[NI];
    {
        const int g = lane >> 4, i16 = lane & 15;
        const int krow = (g >> 1) * 8 + (i16 >> 2);  // (krow & 3) == i16 >> 2 also for rows + 4, + 16 ks
#pragma unroll
        for (int ni = 0; ni < NI; ++ni) {
            const int col = wn * WN + ni * 32 + (g & 1) * 16 + (i16 & 3) * 4;
            btr[ni] = krow * BPITCH + ((((col >> 3) ^ ((i16 >> 2) << 2))) << 4) + (col & 7) * 2;
        }
    }
    // ---- main K loop ----------------------------------------------------------------------
    if constexpr (PARTIAL) {
        // Rank-wide pass: bound by memory, not by the matrix pipe, so what counts is bytes in flight.  kWideStages LDS
        // stages of [rows tile | table tile]; the loads of kWideStages - 1 tiles are in flight while one is multiplied.
        // One barrier per tile: before it every wave has received its own loads of tile kc, after it all of the tile
        // is in LDS and every wave is done with tile kc - 1, whose stage the loads of tile kc + kWideStages - 1 may fill.
        constexpr int NS = wide_stages(B_KMAJOR);
        static_assert((NS - 2) * ND <= 63, "outstanding loads must fit the counter");
        auto issue_tile = [&](int kc) {
            const uint32_t base = lds_wave + (uint32_t)(kc % NS) * STAGE;
            const int k0 = kc << 6;
            const i32x4 ra_t = tile_rsrc(ra_w, kc), rb_t = tile_rsrc(rb_w, kc);
#pragma unroll
            for (int i = 0; i < ACH; ++i) dma16(ra_t, a_src(i, k0, false), base + i * (NT / 64) * 1024);
#pragma unroll
            for (int i = 0; i < BCH; ++i) dma16(rb_t, b_src(i, k0, kc, false), base + ATILE + i * (NT / 64) * 1024);
        };
        auto read_frags_at = [&](const uint8_t *ta, int ks, int buf) {
            const uint8_t *tb = ta + ATILE;
#pragma unroll
            for (int mi = 0; mi < MI; ++mi) af[buf][mi] = lds_frag(ta, wm * WM + mi * 32 + rl, ks * 2 + kh);
            if constexpr (B_KMAJOR) {
#pragma unroll
                for (int ni = 0; ni < NI; ++ni) bf[buf][ni] = lds_frag(tb, wn * WN + ni * 32 + rl, ks * 2 + kh);
            } else {
#pragma unroll
                for (int ni = 0; ni < NI; ++ni) {
                    const uint8_t *src = tb + btr[ni] + ks * 16 * BPITCH;
                    const bf16x4 lo = lds_tr(src);
                    const bf16x4 hi = lds_tr(src + 4 * BPITCH);
                    bf[buf][ni] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                }
            }
        };
#pragma unroll
        for (int t = 0; t < NS - 1; ++t) issue_tile(t);
        for (int kc = 0; kc < nk; ++kc) {
            wait_dma_but<(NS - 2) * ND>();
            __syncthreads();
            issue_tile(kc + NS - 1);
            const uint8_t *ta = smem + (kc % NS) * STAGE;
            read_frags_at(ta, 0, 0);
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                if (ks + 1 < 4) read_frags_at(ta, ks + 1, (ks + 1) & 1);
                // only the 32-column blocks the adapter's rank reaches
#pragma unroll
                for (int ni = 0; ni < NI; ++ni) {
                    if (n0 + wn * WN + ni * 32 < N) {
#pragma unroll
                        for (int mi = 0; mi < MI; ++mi)
                            acc[ni][mi] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bf[ks & 1][ni], af[ks & 1][mi], acc[ni][mi], 0, 0, 0);
                    }
                }
            }
        }
        wait_dma();  // loads of tiles beyond the last one (they fetch nothing)
    } else if (nk > 0) {
        {
            // One wave per SIMD (256x256) or two (128x128); tiles travel global -> LDS without touching registers.
            // A K tile is four phases of NM16 MFMAs of 16 cycles each.  Everything else a wave has to issue rides
            // behind single MFMAs, one instruction at a time, so that the matrix pipe never waits for the issue of a
            // load: the fragment reads of the next phase (see reads16) and the ND direct loads of the next tile,
            // spread over three phases (the MFMAs of phase 3 that follow the barrier, then phases 0 and 1, see
            // DmaSlots): issuing one takes a wave about as long as half an MFMA, and the CU accepts 1 KiB only
            // every 16-20 cycles; phases 2 and 3 give the last of them time to land.
            // One barrier per tile sits inside phase 3, after its first MFMAs: before it every wave has received
            // its own loads of tile kc+1 and all its fragments of tile kc, so after it the stage of tile kc may be
            // overwritten (tile kc+2) and tile kc+1 may be read.
            constexpr int PRE = NM16 / 4;  // (half of the phase before the barrier was 1 % slower on the 128x128 tile, an eighth level on the 256x256 one)
            // (split of the direct loads over the three phases: 3/8, 1/2, 1/8 on the 256x256 tile as in the other form -
            // 1/4, 1/2, 1/4 and 1/2, 1/2, 0 were 1-3 % slower there; 1/4, 1/2, 1/4 on the smaller tiles, 1 % faster)
            constexpr DmaSlots<NM16, PRE, ND, (BM * BN == 256 * 256 ? ND * 3 / 8 : ND / 4), ND / 2> SL{};
            constexpr int D3 = SL.n[0];
            static_assert(SL.placed() == ND, "not every direct load has a slot");
            auto pipeline = [&](auto even_c) {
            i32x4 ra_t = tile_rsrc(ra_w, 0), rb_t = tile_rsrc(rb_w, 0);
#pragma unroll
            for (int d = 0; d < ND; ++d) dma_chunk(even_c, d, 0, 0, ra_t, rb_t);
            ra_t = tile_rsrc(ra_w, 1);
            rb_t = tile_rsrc(rb_w, 1);
#pragma unroll
            for (int d = 0; d < D3; ++d) dma_chunk(even_c, d, 1, 1, ra_t, rb_t);
            records_are_in();  // (the compiler waits for all loads it knows of, which lets the direct loads land too)
            wait_dma_but<D3>();  // loads complete in order: tile 0 is in
            __builtin_amdgcn_s_barrier();
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int j = 0; j < MH + NI16; ++j) read16(0, 0, j);
            auto k_tile = [&](auto cur_c, int kc) {
                constexpr int cur = decltype(cur_c)::value, nxt = cur ^ 1;
#pragma unroll
                for (int ph = 0; ph < 3; ++ph) {
#pragma unroll
                    for (int m = 0; m < NM16; ++m) {
                        mma16(ph, m);
                        reads16(cur, ph + 1, m, 0);
                        if (ph < 2 && SL.slot[ph + 1][m] >= 0) dma_chunk(even_c, SL.slot[ph + 1][m], nxt, kc + 1, ra_t, rb_t);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
                // (the resources of the tile after the next are formed behind the MFMAs before the barrier: the
                // loads of the next tile, which used the old ones, were all issued in phases 0 and 1)
#pragma unroll
                for (int m = 0; m < PRE; ++m) {
                    mma16(3, m);
                    if (m == 0) ra_t = tile_rsrc(ra_w, kc + 2);
                    if (m == 1) rb_t = tile_rsrc(rb_w, kc + 2);
                    __builtin_amdgcn_sched_barrier(0);
                }
                drain_and_barrier();
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int m = PRE; m < NM16; ++m) {
                    mma16(3, m);
                    reads16(nxt, 0, m, PRE);
                    if (SL.slot[0][m] >= 0) dma_chunk(even_c, SL.slot[0][m], cur, kc + 2, ra_t, rb_t);
                    __builtin_amdgcn_sched_barrier(0);
                }
            };
            using I0 = std::integral_constant<int, 0>;
            using I1 = std::integral_constant<int, 1>;
            // Where paths meet the compiler may copy accumulators from one register to another, and it does not
            // know that the statements before are MFMAs whose results take time to land: every path that ends in
            // MFMAs and leads to such a place ends in mfma16_settle (the loop's own back edge needs no copies).
            int kc = 0;
            for (; kc + 1 < nk; kc += 2) {
                k_tile(I0{}, kc);
                k_tile(I1{}, kc + 1);
            }
            mfma16_settle();
            if (kc < nk) {
                k_tile(I0{}, kc++);
                mfma16_settle();
            }
            wait_dma();  // loads of tiles beyond the last one fetch nothing but still signal completion
            };
            if (k_even) pipeline(std::true_type{});
            else pipeline(std::false_type{});
        }
        __syncthreads();
    }


    // The epilogue needs the token of every row this lane stores: a load whose latency would stand at its start.
    // The 128x128 tiles issue it here, so that it lands while the extension runs (headline step -0.7 %); the 256x256
    // tiles have no registers to hold the tokens meanwhile (with them: spills, forward GEMM +2 %).
    constexpr bool TOK_EARLY = !PARTIAL && !SPLITK && BM * BN < 256 * 256;
    int etok[TOK_EARLY ? MI16 : 1];
    if constexpr (TOK_EARLY) {
#pragma unroll
        for (int mi = 0; mi < MI16; ++mi) etok[mi] = row_tok[m0 + wm * WM + mi * 16 + r16];
    }
    auto row_token16 = [&](int mi) -> int {
        if constexpr (TOK_EARLY) return etok[mi];
        else return row_tok[m0 + wm * WM + mi * 16 + r16];
    };

    // ---- low-rank extension: K-steps [s h | dh] x [B_a | A_a^T] of the tile's adapters ----
    // The steps are taken four at a time (one 64-wide K tile); the step records of a batch are fetched ahead of
    // its loads, those of the first batch before the main loop.  Rank indices beyond an adapter's rank and
    // columns beyond N are filled with zeros (out-of-range buffer offsets, or the zero block).
    // SIBS (sibling projections side by side): both operands of a batch travel global -> LDS like the tiles of
    // the main loop, into the stage the batch before it does not use, while that batch multiplies; rows of the
    // tile outside a step's row range are filled with zeros.
    if (SIBS && !PARTIAL && e1 > e0) {
        auto issue_batch = [&](int stage, const ExtBatch &bt) {
#pragma unroll
            for (int d = 0; d < ND; ++d) issue_piece(stage ? A_ST1 : 0, stage ? B_ST1 : B_ST0, bt, d, false, 0);
        };

        // A step touches only the rows of its adapter: a wave multiplies only those of its 16-row blocks that
        // the step's row range reaches (the others would add zeros).  `rows` = lo | hi << 16, uniform.
        const int wrow0 = __builtin_amdgcn_readfirstlane(wm * WM);
        ExtBatch cur_b = get_batch(e0);
        issue_batch(0, cur_b);
        ExtBatch nxt_b = get_batch(e0 + kExtBatch);
        int stage = 0;
        for (int eb = e0; eb < e1; eb += kExtBatch, stage ^= 1) {
            drain_and_barrier();  // this batch has landed; the stage of the batch before it is free
            const int nsteps = (e1 - eb) < kExtBatch ? (e1 - eb) : kExtBatch;
            {
                // 16x16x32 form: two steps per MFMA (K values 0-15 one step, 16-31 the next).  The rows' operand of the
                // batch holds zeros outside each step's row range already, so the fragments are used as they are; a
                // wave multiplies the 16-row blocks that either step reaches.
                const uint8_t *ta = smem + (stage ? A_ST1 : 0);
                const uint8_t *tb = smem + (stage ? B_ST1 : B_ST0);
                const bool more = eb + kExtBatch < e1;
#pragma unroll
                for (int q = 0; q < kExtBatch / 2; ++q) {
                    if (2 * q < nsteps) {
                        const uint32_t rows0 = cur_b.rows[2 * q], rows1 = cur_b.rows[2 * q + 1];
                        auto on16 = [&](int mi) {
                            const int r0 = wrow0 + mi * 16;
                            return ((int)(rows0 & 0xffffu) < r0 + 16 && (int)(rows0 >> 16) > r0) ||
                                   ((int)(rows1 & 0xffffu) < r0 + 16 && (int)(rows1 >> 16) > r0);
                        };
#pragma unroll
                        for (int ni = 0; ni < NI16; ++ni) read_b16(tb, q, ni);
#pragma unroll
                        for (int mi = 0; mi < MI16; ++mi)
                            if (on16(mi)) a4[mi / MH][mi % MH] = lds_frag(ta, wm * WM + mi * 16 + r16, q * 4 + kq);
#pragma unroll
                        for (int mi = 0; mi < MI16; ++mi) {
                            if (on16(mi)) {
#pragma unroll
                                for (int ni = 0; ni < NI16; ++ni) mfma16(acc4[ni][mi], b8[ni], a4[mi / MH][mi % MH]);
                                mfma16_settle();  // (a conditional block: paths meet behind it)
                            }
                        }
                    }
                    if (q == 0 && more) {
                        // the loads of the next batch, into the other stage
#pragma unroll
                        for (int d = 0; d < ND; ++d) issue_piece(stage ? 0 : A_ST1, stage ? B_ST0 : B_ST1, nxt_b, d, false, 0);
                    }
                }
                cur_b = nxt_b;
                nxt_b = get_batch(eb + 2 * kExtBatch);
            }
        }
        drain_and_barrier();  // every wave has its last fragments: LDS is free for the epilogue
    } else if (!SIBS && !PARTIAL && e1 > e0) {
        // One projection (or the SwiGLU pair, whose s h rows hold gate and up ranks side by side).  A batch of
        // the scheme above is bound by latency: its loads have only the batch before it to land.  Here the rows'
        // operand is loaded once for the tile: one LDS area holds rank indices 64 g .. 64 g + 63 of every row's
        // own s h (rows of different adapters side by side, what lies beyond a row's rank is never used), a step
        // reads its fragments at its own rank offset and clears the rows outside its row range in registers.
        // Only the tables stream: three areas, the loads of two batches in flight while one multiplies.
        static_assert(ATILE >= BTILE, "a table area must fit the place of a row area");
        const uint32_t xa = ROWS_EARLY ? XA_EARLY : 0;
        uint32_t t_cur = B_ST0, t_nxt = B_ST1, t_far = A_ST1;
        const int wrow0 = __builtin_amdgcn_readfirstlane(wm * WM);
        auto issue_rows = [&](int g) {
#pragma unroll
            for (int d = 0; d < ACH; ++d) issue_piece(xa, 0u, ExtBatch{}, d, true, g);
        };
        // true if every piece was one direct load (what the waits below count)
        auto issue_tab = [&](uint32_t base, const ExtBatch &bt) -> bool {
#pragma unroll
            for (int d = ACH; d < ND; ++d) issue_piece(0u, base, bt, d, false, 0);
            return !B_KMAJOR || (((bt.kr[0] | bt.kr[1] | bt.kr[2] | bt.kr[3]) >> 16) & 7u) == 0;
        };
        auto lds_done_and_barrier = [] { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); };

        ExtBatch cur_b = get_batch(e0);
        ExtBatch nxt_b = get_batch(e0 + kExtBatch);
        int g_cur = ROWS_EARLY ? 0 : (int)((cur_b.kr[0] & 0xffffu) >> 6);  // (what was loaded earlier: 0)
        if (!ROWS_EARLY) issue_rows(g_cur);
        issue_tab(t_cur, cur_b);
        bool nxt_direct = true;
        if (e0 + kExtBatch < e1) nxt_direct = issue_tab(t_nxt, nxt_b);
        for (int eb = e0; eb < e1; eb += kExtBatch) {
            const bool has1 = eb + kExtBatch < e1, has2 = eb + 2 * kExtBatch < e1;
            // this batch has landed (loads complete in order; those of the batch after it may still be on their way)
            if (has1 && nxt_direct) wait_dma_but<BCH>();
            else wait_dma();
            lds_done_and_barrier();  // ... in every wave, and the area of the batch before it is free
            const ExtBatch far_b = get_batch(eb + 2 * kExtBatch);
            bool far_direct = true;
            if (has2) far_direct = issue_tab(t_far, far_b);
            const int nsteps = (e1 - eb) < kExtBatch ? (e1 - eb) : kExtBatch;
            {
                // the steps of a batch lie inside one group of 64 rank indices (the planner sees to that); when the
                // group changes, the rows' area is loaded again (ranks above 64 only, once per tile and group)
                const int g = (int)((cur_b.kr[0] & 0xffffu) >> 6);
                if (g != g_cur) {
                    issue_rows(g);  // every wave is past the barrier above: none reads the old rows any more
                    wait_dma();
                    lds_done_and_barrier();
                    g_cur = g;
                }
            }
            {
                // Two steps per MFMA.  K values 0-15 of lane groups 0 and 1 belong to step 2 q, 16-31 of
                // groups 2 and 3 to step 2 q + 1: each lane takes the rank offset and the row range of its own step (a
                // step that does not exist has an empty row range, and its part of the table area holds zeros).
#pragma unroll
                for (int q = 0; q < kExtBatch / 2; ++q) {
                    if (2 * q < nsteps) {
                        const uint32_t rows0 = cur_b.rows[2 * q], rows1 = cur_b.rows[2 * q + 1];
                        const uint32_t kr_l = kq < 2 ? cur_b.kr[2 * q] : cur_b.kr[2 * q + 1];
                        const uint32_t rows_l = kq < 2 ? rows0 : rows1;
                        const int c0 = (int)((kr_l & 63u) >> 3) + (kq & 1);
                        const int lo = (int)(rows_l & 0xffffu), hi = (int)(rows_l >> 16);
                        auto on16 = [&](int mi) {
                            const int r0 = wrow0 + mi * 16;
                            return ((int)(rows0 & 0xffffu) < r0 + 16 && (int)(rows0 >> 16) > r0) ||
                                   ((int)(rows1 & 0xffffu) < r0 + 16 && (int)(rows1 >> 16) > r0);
                        };
#pragma unroll
                        for (int ni = 0; ni < NI16; ++ni) read_b16(smem + t_cur, q, ni);
#pragma unroll
                        for (int mi = 0; mi < MI16; ++mi) {
                            if (on16(mi)) {
                                const int row = wm * WM + mi * 16 + r16;
                                uint4 v = __builtin_bit_cast(uint4, lds_frag(smem + xa, row, c0));
                                const bool in = row >= lo && row < hi;
                                v.x = in ? v.x : 0u;
                                v.y = in ? v.y : 0u;
                                v.z = in ? v.z : 0u;
                                v.w = in ? v.w : 0u;
                                a4[mi / MH][mi % MH] = __builtin_bit_cast(bf16x8, v);
                            }
                        }
#pragma unroll
                        for (int mi = 0; mi < MI16; ++mi) {
                            if (on16(mi)) {
#pragma unroll
                                for (int ni = 0; ni < NI16; ++ni) mfma16(acc4[ni][mi], b8[ni], a4[mi / MH][mi % MH]);
                                mfma16_settle();  // (a conditional block: paths meet behind it)
                            }
                        }
                    }
                }
            }
            const uint32_t t = t_cur;
            t_cur = t_nxt;
            t_nxt = t_far;
            t_far = t;
            cur_b = nxt_b;
            nxt_b = far_b;
            nxt_direct = far_direct;
        }
        drain_and_barrier();  // every wave has its last fragments: LDS is free for the epilogue
    }

    // ---- epilogue: one rounding to bf16, rows scattered back to their tokens --------------
    // The accumulator layout gives a lane four consecutive columns of a row, and the 32 rows of a
    // block go to 32 different tokens: storing from there would touch 32 lines per instruction
    // with 8 bytes each.  Each wave instead writes its rounded tile to a private LDS area (row
    // pitch EP: the row, then its token index) and reads it back row by row, 16 bytes per lane,
    // so that a store instruction covers whole 128-byte lines of a few rows.
    if constexpr (PARTIAL || SPLITK) {
        // fp32 sums of the slice: a lane holds four consecutive (rank) columns of a row
        const int q_hi = SPLITK ? N : (N + 15) & ~15;
        if constexpr (SPLITK) rows_in = p.row_base + p.n_rows - m0;  // rows of the order beyond the last are padding
        float *__restrict__ part =
            p.part + ((int64_t)(SPLITK ? blockIdx.y : blockIdx.z) * p.part_rows + m0 - (SPLITK ? p.row_base : 0)) * p.part_ld;
        if constexpr (SPLITK) {
            mfma16_settle();
#pragma unroll
            for (int mi = 0; mi < MI16; ++mi) {
                const int r = wm * WM + mi * 16 + r16;
#pragma unroll
                for (int ni = 0; ni < NI16; ++ni) {
                    const int q = n0 + wn * WN + ni * 16 + kq * 4;
                    if (r < rows_in && q < q_hi) *reinterpret_cast<floatx4 *>(part + (int64_t)r * p.part_ld + q) = acc4[ni][mi];
                }
            }
        }
#pragma unroll
        for (int mi = 0; mi < (PARTIAL ? MI : 0); ++mi) {
            const int r = wm * WM + mi * 32 + rl;
#pragma unroll
            for (int ni = 0; ni < NI; ++ni) {
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int q = n0 + wn * WN + ni * 32 + g * 8 + kh * 4;
                    if (r < rows_in && q < q_hi)
                        *reinterpret_cast<floatx4 *>(part + (int64_t)r * p.part_ld + q) =
                            floatx4{acc[ni][mi][g * 4 + 0], acc[ni][mi][g * 4 + 1], acc[ni][mi][g * 4 + 2], acc[ni][mi][g * 4 + 3]};
                }
            }
        }
    } else {
        constexpr int EP = WN * 2 + 16;          // bytes per staged row
        constexpr int LPR = WN / 8, RPI = 64 / LPR;  // lanes per row, rows per store instruction
        uint8_t *ep = smem + wave * (WM * EP);
        if constexpr (SWIGLU) {
            // Each wave of a pair finishes half of the pair's rows: the gate wave the first half (it receives their
            // up values), the up wave the second half (it receives their gate values).  Accumulator layout: lane =
            // row l % 16 of a 16x16 block, registers = columns 4 (l / 16) ..: the two waves of a pair hold gate and
            // up of the same outputs lane for lane.  Area of the pair: [gate values of the second half | up values
            // of the first].  silu(g) u = g u / (1 + exp(-g)); the rounded rows are staged in the area just read and
            // stored as whole lines.
            mfma16_settle();
            if (p.pre_act) {
                uint16_t *__restrict__ Pre = reinterpret_cast<uint16_t *>(p.pre_act);
#pragma unroll
                for (int mi = 0; mi < MI16; ++mi) {
                    const int tok = row_token16(mi);
                    if (tok < 0 || !p.tok_train[tok]) continue;
#pragma unroll
                    for (int ni = 0; ni < NI16; ++ni) {
                        const int c = ni * 16 + kq * 4;
                        if (n0 + c >= N) continue;
                        uint2 v;
                        v.x = pack_bf16(acc4[ni][mi][0], acc4[ni][mi][1]);
                        v.y = pack_bf16(acc4[ni][mi][2], acc4[ni][mi][3]);
                        *reinterpret_cast<uint2 *>(Pre + (int64_t)tok * p.pre_ld + (wn ? p.act_col : 0) + n0 + c) = v;
                    }
                }
            }
            static_assert(MI16 % 2 == 0, "the rows of a wave pair are split in two");
            constexpr int MH2 = MI16 / 2;
            floatx4 *xg = reinterpret_cast<floatx4 *>(smem + wm * (WM * WN * 4));
            floatx4 *xu = xg + MH2 * NI16 * 64;
            auto send = [&](auto lo_c, floatx4 *dst) {
                constexpr int LO = decltype(lo_c)::value;
#pragma unroll
                for (int mh = 0; mh < MH2; ++mh)
#pragma unroll
                    for (int ni = 0; ni < NI16; ++ni) dst[(mh * NI16 + ni) * 64 + lane] = acc4[ni][LO + mh];
            };
            if (wn == 0) send(std::integral_constant<int, MH2>{}, xg);
            else send(std::integral_constant<int, 0>{}, xu);
            __syncthreads();
            auto finish = [&](auto lo_c, auto gate_c, const floatx4 *src) {
                constexpr int LO = decltype(lo_c)::value;
                constexpr bool OWN_GATE = decltype(gate_c)::value;
                uint8_t *area = reinterpret_cast<uint8_t *>(const_cast<floatx4 *>(src));
                uint2 out[MH2][NI16];
#pragma unroll
                for (int mh = 0; mh < MH2; ++mh) {
#pragma unroll
                    for (int ni = 0; ni < NI16; ++ni) {
                        const floatx4 o = src[(mh * NI16 + ni) * 64 + lane];
                        float r[4];
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const float own = acc4[ni][LO + mh][e];
                            const float gt = OWN_GATE ? own : o[e], up = OWN_GATE ? o[e] : own;
                            r[e] = gt * up * __builtin_amdgcn_rcpf(1.f + __expf(-gt));
                        }
                        out[mh][ni].x = pack_bf16(r[0], r[1]);
                        out[mh][ni].y = pack_bf16(r[2], r[3]);
                    }
                }
                __builtin_amdgcn_wave_barrier();  // every lane has read what it needs of the area
#pragma unroll
                for (int mh = 0; mh < MH2; ++mh) {
                    uint8_t *erow = area + (mh * 16 + r16) * EP;
                    if (kq == 0) *reinterpret_cast<int32_t *>(erow + WN * 2) = row_token16(LO + mh);
#pragma unroll
                    for (int ni = 0; ni < NI16; ++ni) *reinterpret_cast<uint2 *>(erow + (ni * 16 + kq * 4) * 2) = out[mh][ni];
                }
                __builtin_amdgcn_wave_barrier();
                uint16_t *__restrict__ Out = reinterpret_cast<uint16_t *>(p.out);
                const int rr = lane / LPR, cc = lane % LPR;
                const int n = n0 + cc * 8;
#pragma unroll 4
                for (int it = 0; it < (WM / 2) / RPI; ++it) {
                    const uint8_t *erow = area + (it * RPI + rr) * EP;
                    const uint4 v = *reinterpret_cast<const uint4 *>(erow + cc * 16);
                    const int tok = *reinterpret_cast<const int32_t *>(erow + WN * 2);
                    if (tok >= 0 && n < N) *reinterpret_cast<uint4 *>(Out + (int64_t)tok * p.ldo + n) = v;
                }
            };
            if (wn == 0) finish(std::integral_constant<int, 0>{}, std::true_type{}, xu);
            else finish(std::integral_constant<int, MH2>{}, std::false_type{}, xg);
            return;
        }
        {
            mfma16_settle();
#pragma unroll
            for (int mi = 0; mi < MI16; ++mi) {
                uint8_t *erow = ep + (mi * 16 + r16) * EP;
                if (kq == 0) *reinterpret_cast<int32_t *>(erow + WN * 2) = row_token16(mi);
#pragma unroll
                for (int ni = 0; ni < NI16; ++ni) {
                    uint2 v;
                    v.x = pack_bf16(acc4[ni][mi][0], acc4[ni][mi][1]);
                    v.y = pack_bf16(acc4[ni][mi][2], acc4[ni][mi][3]);
                    *reinterpret_cast<uint2 *>(erow + (ni * 16 + kq * 4) * 2) = v;
                }
            }
        }
        __builtin_amdgcn_wave_barrier();
        uint16_t *__restrict__ Out = reinterpret_cast<uint16_t *>(p.out);
        const int rr = lane / LPR, cc = lane % LPR;
        const int n = n0 + wn * WN + cc * 8;
#pragma unroll 4
        for (int it = 0; it < WM / RPI; ++it) {
            const uint8_t *erow = ep + (it * RPI + rr) * EP;
            const uint4 v = *reinterpret_cast<const uint4 *>(erow + cc * 16);
            const int tok = *reinterpret_cast<const int32_t *>(erow + WN * 2);
            if (tok >= 0 && n < N) *reinterpret_cast<uint4 *>(Out + (int64_t)tok * p.ldo + n) = v;
        }
    }
}

// =========================================================================================
// skinny: out[m][q] = sum_k in[tok(m)][k] * table_a(k, q)     (rank-wide output, HBM-bound)
//
// One block = one item (RT = 1 or 2 tiles of 16 rows of one adapter) x one of gridDim.y slices of K.
// Its KW waves split the slice; every wave runs 16x16x32 MFMAs on its own K range for all row
// tiles of the item, so a table fragment is fetched once per item and used RT times.  The
// streamed operand (rows of x or dy) goes from global memory straight into MFMA operand
// registers: lane l holds 8 consecutive K values of row l % 16.  The adapter table is either
// K-major ([rank][K], read the same way) or N-major ([K][rank]): then each wave copies its
// chunk as it lies in memory into a private LDS area and builds the operand with transposing
// reads.  Nothing in the K loop needs a block barrier.  The partial sums of the waves meet in
// LDS in wave order.  With more than one K slice the block writes its sums to a workspace and
// a second, small kernel adds the slices in slice order (fixed order, no float atomics, and no
// fences inside a kernel: on this GPU a device-wide fence writes back and invalidates the L2).
// =========================================================================================
// Results of four rank indices q .. q + 3 of row m of an item: the fp32 copy (token-indexed h_save
// or row-indexed workspace) and the scaled copy in the element type.
__device__ __forceinline__ void skinny_store(const SkinnyArgs &p, const SkinnyItem it, int m, int q, floatx4 sum)
{
    const int row = it.row_lo + m;
    const int tok = p.row_tok[row];
    float *f32_row = nullptr;
    if (p.f32_out) {
        if (p.f32_by_token) {
            if (p.tok_train[tok]) f32_row = p.f32_out + (int64_t)tok * p.f32_ld;
        } else {
            f32_row = p.f32_out + (int64_t)row * p.f32_ld;
        }
    }
    uint16_t *bf_row = p.bf_out ? reinterpret_cast<uint16_t *>(p.bf_out) + (int64_t)row * p.bf_ld : nullptr;
    if (p.n_sib > 1) {
        // one sibling's columns of the row (ranks are multiples of 8 here); the last sibling clears the rest
        const int rank = it.rank / p.n_sib, co = p.sib * rank;
        if (q < rank) {
            if (f32_row)
                *reinterpret_cast<floatx4 *>(f32_row + co + q) = sum * p.f32_mult;
            if (bf_row) {
                uint2 o;
                o.x = pack_bf16(sum[0] * p.bf_mult, sum[1] * p.bf_mult);
                o.y = pack_bf16(sum[2] * p.bf_mult, sum[3] * p.bf_mult);
                *reinterpret_cast<uint2 *>(bf_row + co + q) = o;
            }
        }
        if (q == 0 && p.sib == p.n_sib - 1) {
            if (f32_row)
                for (int z = it.rank; z < p.f32_cols; ++z) f32_row[z] = 0.f;
            if (bf_row)
                for (int z = it.rank; z < p.bf_ld; ++z) bf_row[z] = 0;
        }
        return;
    }
    const int rank = it.rank, rp = (rank + 15) & ~15;
    float v[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) v[e] = (q + e < rank) ? sum[e] : 0.f;
    if (f32_row) {
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (q + e < p.f32_cols) f32_row[q + e] = v[e] * p.f32_mult;
        // zero fill beyond the padded rank (h_save rows are max_rank wide)
        if (q + 4 == rp)
            for (int z = rp; z < p.f32_cols; ++z) f32_row[z] = 0.f;
    }
    if (bf_row) {
        uint2 o;
        o.x = pack_bf16(v[0] * p.bf_mult, v[1] * p.bf_mult);
        o.y = pack_bf16(v[2] * p.bf_mult, v[3] * p.bf_mult);
        *reinterpret_cast<uint2 *>(bf_row + q) = o;
    }
}

template <int RP>
struct SkinnyCfg {
    static constexpr int CHK = RP <= 64 ? 64 : 32;                    // K values per chunk
    static constexpr int STEPS = CHK / 32;
    static constexpr int KW = RP <= 32 ? 8 : 4;                       // waves per block
    static constexpr int NB = RP / 16;                                // 16-wide rank blocks
    static constexpr int RTMAX = RP <= 128 ? 2 : 1;                   // row tiles per item
    static constexpr int PITCH = RP * 2 + 16;                         // LDS row pitch of an N-major chunk
    static constexpr int STAGE_BYTES = CHK * PITCH;                   // per wave
    static constexpr int RED_LD = RP + 4;                             // floats
};

template <int RP, bool T_KMAJOR, int RT>
__global__ void __launch_bounds__(SkinnyCfg<RP>::KW * 64) skinny_kernel(SkinnyArgs p)
{
    using C = SkinnyCfg<RP>;
    constexpr int KW = C::KW, STEPS = C::STEPS, CHK = C::CHK, NB = C::NB;
    constexpr int ROWS = 16 * RT;
    constexpr int RED_BYTES = KW * ROWS * C::RED_LD * 4;
    extern __shared__ __align__(16) uint8_t smem[];
    float *red = reinterpret_cast<float *>(smem);
    uint8_t *stage = smem + RED_BYTES + (threadIdx.x >> 6) * C::STAGE_BYTES;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (blockIdx.x >= (unsigned)p.n_items) {
        // a warm-up block: its share of the next GEMM's weight, read once and dropped
        if (blockIdx.y == 0) warm_cache(p.warm_base, p.warm_bytes, blockIdx.x - p.n_items, p.warm_blocks, tid, KW * 64);
        return;
    }
    // (the item is the same for the whole block: kept in scalar registers)
    const SkinnyItem *ip = p.items + blockIdx.x;
    const SkinnyItem it = {__builtin_amdgcn_readfirstlane(ip->adapter), __builtin_amdgcn_readfirstlane(ip->row_lo),
                           __builtin_amdgcn_readfirstlane(ip->n_rows), __builtin_amdgcn_readfirstlane(ip->rank)};
    const int K = p.K, rank = p.n_sib > 1 ? it.rank / p.n_sib : it.rank;
    const int rp = (rank + 15) & ~15;
    const int l16 = lane & 15, kg = lane >> 4;
    const int n_rt = (it.n_rows + 15) >> 4;  // row tiles of this item
    const uint32_t tld = T_KMAJOR && p.tab_ld ? (uint32_t)p.tab_ld : (uint32_t)K, toff = T_KMAJOR ? (uint32_t)p.tab_off : 0u;

    // K range of this wave: the slices of the blocks, cut again into the ranges of their waves
    const int n_split = gridDim.y, split = blockIdx.y;
    const int per = (((K + n_split * KW - 1) / (n_split * KW)) + 31) & ~31;
    const int k_lo = (split * KW + wave) * per;
    const int k_hi = (k_lo + per) < K ? (k_lo + per) : K;

    const __amdgpu_buffer_rsrc_t rx = make_rsrc(p.in, p.in_bytes);
    const __amdgpu_buffer_rsrc_t rt = make_rsrc(reinterpret_cast<const void *>(p.tab[it.adapter]),
                                                T_KMAJOR ? (uint32_t)rank * tld * 2u : (uint32_t)rank * (uint32_t)K * 2u);
    uint32_t xoff[RT];
#pragma unroll
    for (int t = 0; t < RT; ++t) {
        xoff[t] = kOob;
        if (t * 16 + l16 < it.n_rows) {
            const int tok = p.row_tok[it.row_lo + t * 16 + l16];
            if (tok >= 0) xoff[t] = (uint32_t)tok * (uint32_t)p.ld_in * 2u + kg * 16u;
        }
    }

    // D chunks are in flight per wave (a ring of register sets): the pass is bound by memory latency.
    // Four where the registers of a chunk are few enough to keep four waves per SIMD, else two.
    constexpr int D = (RT * STEPS + STEPS * NB <= 8) ? 4 : 2;
    uint4 xreg[D][RT][STEPS];
    auto load_x = [&](int k0, int buf) {
#pragma unroll
        for (int t = 0; t < RT; ++t)
#pragma unroll
            for (int s = 0; s < STEPS; ++s) {
                const int k = k0 + s * 32;
                xreg[buf][t][s] = buf16(rx, (k + kg * 8 < k_hi) ? xoff[t] + (uint32_t)k * 2u : kOob);
            }
    };

    // K-major table: operand registers straight from memory
    uint4 treg[T_KMAJOR ? D : 1][T_KMAJOR ? STEPS * NB : 1];
    auto load_t_kmajor = [&](int k0, int buf) {
        if constexpr (T_KMAJOR) {
#pragma unroll
            for (int s = 0; s < STEPS; ++s) {
                const int k = k0 + s * 32 + kg * 8;
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) {
                    const int q = nb * 16 + l16;
                    treg[buf][s * NB + nb] =
                        buf16(rt, (q < rank && k < k_hi) ? ((uint32_t)q * tld + toff + (uint32_t)k) * 2u : kOob);
                }
            }
        }
    };
    // N-major table: the chunk [CHK][rank] is contiguous; copy it to LDS rows of PITCH bytes
    constexpr int NCP = T_KMAJOR ? 1 : (CHK * RP * 2 / 16 + 63) / 64;  // 16-byte pieces per lane
    uint4 creg[D][NCP];
    const bool fast_copy = (rank & 7) == 0;
    const int cpr = rank >> 3;  // 16-byte pieces per table row
    // piece c of the chunk is piece c % cpr of row c / cpr; the division is done once
    int crow[NCP], ccol[NCP];
    if constexpr (!T_KMAJOR) {
#pragma unroll
        for (int i = 0; i < NCP; ++i) {
            const int c = lane + i * 64;
            crow[i] = fast_copy ? c / cpr : 0;
            ccol[i] = fast_copy ? c - crow[i] * cpr : 0;
        }
    }
    auto load_t_nmajor = [&](int k0, int buf) {
        if constexpr (!T_KMAJOR) {
            // (issued for every rank, out of range where the slow copy below does the work: the number of loads
            // per chunk must not depend on a branch, or the compiler cannot count how many may still be in flight
            // and waits for more of them than the chunk it needs)
#pragma unroll
            for (int i = 0; i < NCP; ++i) {
                const int c = lane + i * 64;
                // rows beyond K lie beyond the table and read as zero
                creg[buf][i] = buf16(rt, (fast_copy && c < CHK * cpr) ? ((uint32_t)k0 * (uint32_t)rank) * 2u + (uint32_t)c * 16u : kOob);
            }
        }
    };
    // The loads of a chunk stay together and the chunks stay in order (the compiler may not move memory operations
    // across this): the wait before a chunk's first use then counts exactly the loads of the D - 1 chunks behind it.
    // Left to itself the compiler issues the first chunk's loads last in the prologue, and the loop then waits
    // for all loads at the top of every round.
    auto fence_chunk = [] { asm volatile("" ::: "memory"); };
    auto store_t_nmajor = [&](int k0, int buf) {
        if constexpr (!T_KMAJOR) {
            if (fast_copy) {
#pragma unroll
                for (int i = 0; i < NCP; ++i)
                    if (lane + i * 64 < CHK * cpr)
                        *reinterpret_cast<uint4 *>(stage + crow[i] * C::PITCH + ccol[i] * 16) = creg[buf][i];
            } else {
                // ranks that are no multiple of 8: element by element
                const uint16_t *tab = reinterpret_cast<const uint16_t *>(p.tab[it.adapter]);
                for (int e = lane; e < CHK * rank; e += 64) {
                    const int r = e / rank, q = e - r * rank;
                    const int k = k0 + r;
                    reinterpret_cast<uint16_t *>(stage + r * C::PITCH)[q] = k < K ? tab[(int64_t)k * rank + q] : (uint16_t)0;
                }
            }
        }
    };

    floatx4 acc[RT][NB];
#pragma unroll
    for (int t = 0; t < RT; ++t)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) acc[t][nb] = floatx4{0.f, 0.f, 0.f, 0.f};

    if (k_lo < k_hi) {
#pragma unroll
        for (int d = 0; d < D; ++d) {
            load_x(k_lo + d * CHK, d);
            load_t_kmajor(k_lo + d * CHK, d);
            load_t_nmajor(k_lo + d * CHK, d);
            fence_chunk();
        }
        for (int kb = k_lo; kb < k_hi; kb += D * CHK) {
#pragma unroll
            for (int d = 0; d < D; ++d) {
                const int k0 = kb + d * CHK;  // chunks beyond the wave's range were loaded as zeros
                store_t_nmajor(k0, d);
#pragma unroll
                for (int s = 0; s < STEPS; ++s) {
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb) {
                        if (nb * 16 < rp) {
                            bf16x8 tf;
                            if constexpr (T_KMAJOR) {
                                tf = __builtin_bit_cast(bf16x8, treg[d][s * NB + nb]);
                            } else {
                                const uint8_t *src = stage + (s * 32 + kg * 8 + (l16 >> 2)) * C::PITCH +
                                                     (nb * 16 + (l16 & 3) * 4) * 2;
                                const bf16x4 lo = lds_tr(src), hi = lds_tr(src + 4 * C::PITCH);
                                tf = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                            }
#pragma unroll
                            for (int t = 0; t < RT; ++t)
                                if (t < n_rt)
                                    acc[t][nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                                        tf, __builtin_bit_cast(bf16x8, xreg[d][t][s]), acc[t][nb], 0, 0, 0);
                        }
                    }
                }
                // refill this register set with the chunk D further on
                fence_chunk();
                load_x(k0 + D * CHK, d);
                load_t_kmajor(k0 + D * CHK, d);
                load_t_nmajor(k0 + D * CHK, d);
                fence_chunk();
            }
        }
    }

    // lane holds row m = 16 t + lane % 16, columns q = nb*16 + 4*(lane/16) + 0..3
    {
#pragma unroll
        for (int t = 0; t < RT; ++t) {
            float *mine = red + (wave * ROWS + t * 16 + l16) * C::RED_LD;
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
                *reinterpret_cast<floatx4 *>(mine + nb * 16 + kg * 4) = acc[t][nb];
        }
    }
    __syncthreads();

    // sum over the waves in wave order; with several K slices the sums go to the workspace and a
    // second kernel adds the slices
    const int n_quads = ROWS * (RP / 4);
    for (int idx = tid; idx < n_quads; idx += KW * 64) {
        const int m = idx % ROWS, q = (idx / ROWS) * 4;
        if (m >= it.n_rows || q >= rp) continue;
        floatx4 sum = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int w = 0; w < KW; ++w) sum += *reinterpret_cast<const floatx4 *>(red + (w * ROWS + m) * C::RED_LD + q);
        if (n_split > 1)
            *reinterpret_cast<floatx4 *>(p.part + ((int64_t)split * p.part_rows + it.row_lo + m) * p.part_ld + q) = sum;
        else
            skinny_store(p, it, m, q, sum);
    }
}

// Sum of n values that lie `stride` floats apart, added in index order; four loads are in flight at a time
// (the kernels that add K slices are bound by the latency of these loads, not by their bytes).
__device__ __forceinline__ floatx4 sum_slices(const float *first, int64_t stride, int n)
{
    floatx4 sum = floatx4{0.f, 0.f, 0.f, 0.f};
    int i = 0;
    for (; i + 4 <= n; i += 4) {
        const floatx4 v0 = *reinterpret_cast<const floatx4 *>(first + (i + 0) * stride);
        const floatx4 v1 = *reinterpret_cast<const floatx4 *>(first + (i + 1) * stride);
        const floatx4 v2 = *reinterpret_cast<const floatx4 *>(first + (i + 2) * stride);
        const floatx4 v3 = *reinterpret_cast<const floatx4 *>(first + (i + 3) * stride);
        sum += v0;
        sum += v1;
        sum += v2;
        sum += v3;
    }
    for (; i < n; ++i) sum += *reinterpret_cast<const floatx4 *>(first + i * stride);
    return sum;
}

// adds the K slices of every item in slice order and writes the results; block (i, j) takes rows
// 16 j .. 16 j + 15 of item i
__global__ void __launch_bounds__(256) skinny_finish_kernel(SkinnyArgs p, int n_split)
{
    const SkinnyItem it = p.items[blockIdx.x];
    const int rp = ((p.n_sib > 1 ? it.rank / p.n_sib : it.rank) + 15) & ~15;
    const int nq = rp >> 2;
    const int m_lo = blockIdx.y * 16, m_hi = it.n_rows < m_lo + 16 ? it.n_rows : m_lo + 16;
    for (int idx = threadIdx.x; idx < (m_hi - m_lo) * nq; idx += 256) {
        const int m = m_lo + idx / nq, q = (idx % nq) * 4;
        const floatx4 sum = sum_slices(p.part + (int64_t)(it.row_lo + m) * p.part_ld + q, (int64_t)p.part_rows * p.part_ld, n_split);
        skinny_store(p, it, m, q, sum);
    }
}

// =========================================================================================
// grad: out_a(q, n) = sum_t small[t][q] * big[tok(t)][n]   over the adapter's training rows t
// (dB_a: small = s h, big = dy;  dA_a^T: small = dh, big = x).
//
// One block = one trained adapter x 64 output columns (x one 128-wide slice of the rank).
// Its KW waves split the adapter's rows; each wave copies 32 rows of `big` (64 columns, as
// they lie in memory) and of `small` (converted to bf16) into a private LDS area and builds
// both 16x16x32 MFMA operands with transposing reads, since the contraction index (the
// token) is the slow index of both.  The partial sums of the waves meet in LDS in wave
// order: fixed order, no atomics, one writer per output element.
// =========================================================================================
template <int RP>
struct GradCfg {
    static constexpr int KW = RP <= 32 ? 8 : 4;
    static constexpr int CHT = 32;                 // rows per chunk = one MFMA K step
    static constexpr int MB = RP / 16;
    static constexpr int BPITCH = 64 * 2 + 32;     // bytes
    static constexpr int SPITCH = RP * 2 + 16;
    static constexpr int STAGE_BYTES = CHT * (BPITCH + SPITCH);  // per wave
    static constexpr int RED_LD = 65;              // floats
    static constexpr int RED_BYTES = KW * RP * RED_LD * 4;
    static constexpr int SMEM = (KW * STAGE_BYTES > RED_BYTES) ? KW * STAGE_BYTES : RED_BYTES;
    static constexpr int SV = CHT * RP / 4 / 64;   // float4 pieces of `small` per lane
    static constexpr int SROW = 64 * 4 / RP;       // rows advanced per piece index
};

template <int RP, bool SMALL_BF>
__global__ void __launch_bounds__(GradCfg<RP>::KW * 64) grad_kernel(GradArgs p)
{
    using C = GradCfg<RP>;
    constexpr int KW = C::KW, MB = C::MB, SV = SMALL_BF ? 1 : C::SV;
    constexpr int NP = RP / 16;   // 16-byte pieces of a bf16 `small` chunk per lane
    constexpr int PPR = RP / 8;   // pieces per row
    extern __shared__ __align__(16) uint8_t smem[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    uint8_t *stage_b = smem + wave * C::STAGE_BYTES;
    uint8_t *stage_s = stage_b + C::CHT * C::BPITCH;
    float *red = reinterpret_cast<float *>(smem);

    const int n0 = blockIdx.x * 64;
    const GradItem it = p.items[blockIdx.y];
    const int q0 = blockIdx.z * RP;
    const int rank = p.n_sib > 1 ? it.rank / p.n_sib : it.rank;
    const int N = p.N;
    const int l16 = lane & 15, kg = lane >> 4;

    const int n_rows = it.row_hi - it.row_lo;
    const int per = (((n_rows + KW - 1) / KW) + 31) & ~31;
    const int t_lo = it.row_lo + wave * per;
    const int t_hi = (t_lo + per) < it.row_hi ? (t_lo + per) : it.row_hi;

    const __amdgpu_buffer_rsrc_t rbig = make_rsrc(p.big, p.big_bytes);
    const int32_t *__restrict__ row_tok = p.row_tok;
    const float *__restrict__ Small = p.small_;
    const uint16_t *__restrict__ SmallB = reinterpret_cast<const uint16_t *>(p.small_bf);
    // the bf16 copy holds zeros from the rank up to the next multiple of 16; with siblings (ranks are multiples
    // of 8 then) the next sibling's columns follow at once
    const int rp_rank = p.n_sib > 1 ? rank : (rank + 15) & ~15;
    const int s_off = p.n_sib > 1 ? p.sib * rank : 0;

    // big: lane copies chunk column c = lane % 8 of rows lane / 8 + 8 i
    const int bc = lane & 7, br = lane >> 3;
    const uint32_t bcol = (n0 + bc * 8 < N) ? (uint32_t)(n0 + bc * 8) * 2u : kOob;
    // small: lane converts the float4 piece (row sr + SROW i, columns 4 sq ..)
    const int sq = lane % (RP / 4), sr = lane / (RP / 4);
    const bool small_vec = (p.ld_small & 3) == 0;

    int tokb[4], toks[SV];  // token of each row this lane touches in the next chunk (-1: none)
    auto load_toks = [&](int t0) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int t = t0 + br + i * 8;
            tokb[i] = t < t_hi ? row_tok[t] : -1;
        }
        if constexpr (!SMALL_BF) {
#pragma unroll
            for (int i = 0; i < SV; ++i) {
                const int t = t0 + sr + i * C::SROW;
                toks[i] = t < t_hi ? (p.small_by_token ? row_tok[t] : t) : -1;
            }
        }
    };
    uint4 breg[4];
    floatx4 sreg[SV];
    uint4 sbreg[SMALL_BF ? NP : 1];
    int t_next = t_lo;  // first row of the chunk the next load_data fetches
    auto load_data = [&]() {
#pragma unroll
        for (int i = 0; i < 4; ++i)
            breg[i] = buf16(rbig, (tokb[i] >= 0 && bcol != kOob) ? (uint32_t)tokb[i] * (uint32_t)p.ld_big * 2u + bcol : kOob);
        if constexpr (SMALL_BF) {
            // the bf16 copy is in row order and already scaled: 16-byte pieces as they lie in memory
#pragma unroll
            for (int i = 0; i < NP; ++i) {
                const int c = lane + i * 64;
                const int t = t_next + c / PPR, q = q0 + (c % PPR) * 8;
                uint4 v = make_uint4(0, 0, 0, 0);
                if (t < t_hi && q < rp_rank) v = ldg16(SmallB + (int64_t)t * p.ld_small_bf + s_off + q);
                sbreg[i] = v;
            }
            t_next += C::CHT;
            return;
        }
#pragma unroll
        for (int i = 0; i < SV; ++i) {
            floatx4 v = floatx4{0.f, 0.f, 0.f, 0.f};
            const int q = q0 + sq * 4;
            if (toks[i] >= 0 && q < rank) {
                const float *src = Small + (int64_t)toks[i] * p.ld_small + q;
                if (small_vec) {
                    v = *reinterpret_cast<const floatx4 *>(src);
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (q + e < rank) v[e] = src[e];
                }
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (q + e >= rank) v[e] = 0.f;
            }
            sreg[i] = v;
        }
    };
    auto store_data = [&]() {
#pragma unroll
        for (int i = 0; i < 4; ++i) *reinterpret_cast<uint4 *>(stage_b + (br + i * 8) * C::BPITCH + bc * 16) = breg[i];
        if constexpr (SMALL_BF) {
#pragma unroll
            for (int i = 0; i < NP; ++i) {
                const int c = lane + i * 64;
                *reinterpret_cast<uint4 *>(stage_s + (c / PPR) * C::SPITCH + (c % PPR) * 16) = sbreg[i];
            }
            return;
        }
#pragma unroll
        for (int i = 0; i < SV; ++i) {
            uint2 o;
            o.x = pack_bf16(sreg[i][0] * p.small_mult, sreg[i][1] * p.small_mult);
            o.y = pack_bf16(sreg[i][2] * p.small_mult, sreg[i][3] * p.small_mult);
            *reinterpret_cast<uint2 *>(stage_s + (sr + i * C::SROW) * C::SPITCH + sq * 8) = o;
        }
    };

    floatx4 acc[MB][4];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int nb = 0; nb < 4; ++nb) acc[mb][nb] = floatx4{0.f, 0.f, 0.f, 0.f};

    if (t_lo < t_hi) {
        load_toks(t_lo);
        load_data();
        load_toks(t_lo + C::CHT);
        for (int t0 = t_lo; t0 < t_hi; t0 += C::CHT) {
            store_data();
            load_data();                      // rows of the next chunk (tokens fetched one chunk ahead)
            load_toks(t0 + 2 * C::CHT);
            const int rrow = kg * 8 + (l16 >> 2), rcol = (l16 & 3) * 4;
            bf16x8 bf[4];
#pragma unroll
            for (int nb = 0; nb < 4; ++nb) {
                const uint8_t *src = stage_b + rrow * C::BPITCH + (nb * 16 + rcol) * 2;
                const bf16x4 lo = lds_tr(src), hi = lds_tr(src + 4 * C::BPITCH);
                bf[nb] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
            }
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) {
                if (q0 + mb * 16 < rank) {
                    const uint8_t *src = stage_s + rrow * C::SPITCH + (mb * 16 + rcol) * 2;
                    const bf16x4 lo = lds_tr(src), hi = lds_tr(src + 4 * C::SPITCH);
                    const bf16x8 sf = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
#pragma unroll
                    for (int nb = 0; nb < 4; ++nb)
                        acc[mb][nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(sf, bf[nb], acc[mb][nb], 0, 0, 0);
                }
            }
        }
    }

    __syncthreads();  // every wave is done with its staging area: the sums may reuse it
    // lane holds column n = nb*16 + lane%16, rows q = mb*16 + 4*(lane/16) + j
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int nb = 0; nb < 4; ++nb)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                red[(wave * RP + mb * 16 + kg * 4 + j) * C::RED_LD + nb * 16 + l16] = acc[mb][nb][j];
    __syncthreads();

    float *out = reinterpret_cast<float *>(p.out_tab[it.adapter]);
    const int qn = (rank - q0) < RP ? (rank - q0) : RP;  // rank indices of this slice
    if (qn <= 0) return;
    for (int idx = tid; idx < 64 * qn; idx += KW * 64) {
        int q, n;
        if (p.out_transposed) {
            n = idx / qn;
            q = idx - n * qn;
        } else {
            q = idx >> 6;
            n = idx & 63;
        }
        if (n0 + n >= N) continue;
        float sum = 0.f;
#pragma unroll
        for (int w = 0; w < KW; ++w) sum += red[(w * RP + q) * C::RED_LD + n];
        float *dst = p.out_transposed ? out + (int64_t)(n0 + n) * rank + q0 + q
                                      : out + (int64_t)(q0 + q) * (p.ld_out ? p.ld_out : (int64_t)N) + p.out_off + n0 + n;
        *dst = p.accumulate ? (*dst + sum) : sum;
    }
}

// =========================================================================================
// dy pass for narrow ranks (see DualArgs): one read of the training rows of dy gives dh and dB_a.
//
// One block = one piece of a trained adapter's rows (blockIdx.y) x one group of 512 columns (blockIdx.x).  Wave w owns
// the group's 64-column slab w for all rows of the piece, so dB_a needs no sum across waves; the rows go by in chunks
// of 32 (one MFMA K step of dB).  Per chunk a wave copies its 32 x 64 values of dy and the chunk's 32 x 16 of s h, as
// they lie in memory, into a private LDS area (from a ring of four chunks of loads in flight), builds both dB operands
// with transposing reads (the contraction index, the row, is the slow index of both), reads the same dy values again
// row by row as the dh operand (contraction over the slab's columns against B_a's, which the wave holds in registers)
// and leaves its 32 x 16 partial dh in LDS, where the eight waves' partials are added in wave order and written as the
// group's slice.  One barrier per chunk (the area of the partials is double-buffered).  The tokens of the piece's rows
// are read into LDS once, so that no load of the ring waits for another load; the sums of dh stay in LDS until the
// piece is done, so that the loop holds loads only (loads and stores complete out of order with respect to each other,
// and with both in flight the compiler has to wait for everything before it touches a loaded register).
// =========================================================================================
constexpr int kDualRing = 4;
struct DualCfg {
    static constexpr int BPITCH = 64 * 2 + 32, SPITCH = 16 * 2 + 16;  // bytes
    static constexpr int STAGE = 32 * (BPITCH + SPITCH);              // per wave
    static constexpr int RED_LD = 20;                                 // floats per row of a wave's partial dh
    static constexpr int RED = 8 * 32 * RED_LD * 4;                   // one buffer, all waves
    static constexpr int TOK = (kDualMaxPieceRows + kDualRing * 32) * 4;  // tokens of the piece's rows, then -1 for the ring's overrun
    static constexpr int DH = kDualMaxPieceRows * 16 * 4;             // the piece's dh sums of this column group
    static constexpr int SMEM = TOK + 8 * STAGE + 2 * RED + DH;
};
static_assert(kDualCols == 8 * 64 && kDualMaxPieceRows == 512, "eight waves of a 64-column slab; one token per thread");

__global__ void __launch_bounds__(512) dydual_kernel(DualArgs p)
{
    using C = DualCfg;
    extern __shared__ __align__(16) uint8_t smem[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n_item_rows = p.n_grad * p.max_pieces;
    if ((int)blockIdx.y >= n_item_rows) {
        // a row of blocks that fetch the next GEMM's weight: each reads its share once and drops it
        warm_cache(p.warm_base, p.warm_bytes, ((int)blockIdx.y - n_item_rows) * (int)gridDim.x + (int)blockIdx.x,
                   p.warm_rows * (int)gridDim.x, tid, 512);
        return;
    }
    const int g = blockIdx.y / p.max_pieces, piece = blockIdx.y - g * p.max_pieces;
    const GradItem it = p.items[g];
    const int n_pieces = (it.row_hi - it.row_lo + p.piece_rows - 1) / p.piece_rows;
    if (piece >= n_pieces) return;
    const int r_lo = it.row_lo + piece * p.piece_rows;
    const int r_hi = r_lo + p.piece_rows < it.row_hi ? r_lo + p.piece_rows : it.row_hi;
    const int n_rows = r_hi - r_lo, n_chunks = (n_rows + 31) >> 5;
    const int rank = it.rank, N = p.N;
    const int n0 = blockIdx.x * kDualCols + wave * 64;  // first column of this wave's slab
    const int l16 = lane & 15, kg = lane >> 4;

    int32_t *s_tok = reinterpret_cast<int32_t *>(smem);
    uint8_t *stage_b = smem + C::TOK + wave * C::STAGE;
    uint8_t *stage_s = stage_b + 32 * C::BPITCH;
    float *red = reinterpret_cast<float *>(smem + C::TOK + 8 * C::STAGE);
    float *s_dh = reinterpret_cast<float *>(smem + C::TOK + 8 * C::STAGE + 2 * C::RED);

    s_tok[tid] = tid < n_rows ? p.row_tok[r_lo + tid] : -1;
    if (tid < kDualRing * 32) s_tok[kDualMaxPieceRows + tid] = -1;
    // B_a's columns of the slab as the dh operand: lane = rank index l16, columns 8 kg .. of each 32-wide step
    // (through a buffer resource, like every other load here: the table's address is itself loaded from memory, and a
    // load through such a pointer is a flat one, which may complete out of order with the buffer loads - with one of
    // those pending the compiler waits for all loads wherever it has to wait for any)
    uint4 bfrag[2];
    {
        const __amdgpu_buffer_rsrc_t rtb = make_rsrc(reinterpret_cast<const void *>(p.tab_b[it.adapter]), (uint32_t)rank * (uint32_t)N * 2u);
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            const int col = n0 + ks * 32 + kg * 8;
            bfrag[ks] = buf16(rtb, (l16 < rank && col < N) ? ((uint32_t)l16 * (uint32_t)N + (uint32_t)col) * 2u : kOob);
        }
    }
    __syncthreads();

    // Every load of the loop goes through a buffer resource and happens whatever the data (rows beyond the piece get
    // an offset beyond the buffer and deliver zeros): the compiler counts the loads between a load and its use, and can
    // only do so when none of them sits behind a branch.
    const __amdgpu_buffer_rsrc_t rdy = make_rsrc(p.dy, p.dy_bytes);
    const __amdgpu_buffer_rsrc_t rhs = make_rsrc(p.hs, p.hs_bytes);
    const int bc = lane & 7, br = lane >> 3;  // dy: lane copies the 16-byte piece bc of rows br + 8 i
    const uint32_t bcol = (n0 + bc * 8 < N) ? (uint32_t)(n0 + bc * 8) * 2u : kOob;
    uint4 breg[kDualRing][4], sreg[kDualRing];
    auto load_chunk = [&](int ch, int buf) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int tok = s_tok[ch * 32 + br + 8 * i];  // (-1 beyond the piece: no branch, so the four reads go out together)
            breg[buf][i] = buf16(rdy, (tok >= 0 && bcol != kOob) ? (uint32_t)tok * (uint32_t)p.ld_dy * 2u + bcol : kOob);
        }
        // s h of the chunk: 32 rows x 16 values = 64 pieces of 16 bytes, one per lane
        const int m = ch * 32 + (lane >> 1);
        sreg[buf] = buf16(rhs, m < n_rows ? ((uint32_t)(r_lo + m) * (uint32_t)p.ld_hs + (lane & 1) * 8u) * 2u : kOob);
    };
    auto store_chunk = [&](int buf) {
#pragma unroll
        for (int i = 0; i < 4; ++i) *reinterpret_cast<uint4 *>(stage_b + (br + 8 * i) * C::BPITCH + bc * 16) = breg[buf][i];
        *reinterpret_cast<uint4 *>(stage_s + (lane >> 1) * C::SPITCH + (lane & 1) * 16) = sreg[buf];
    };
    // (the loads of a chunk stay together and the chunks in order, as in skinny_kernel)
    auto fence_chunk = [] { asm volatile("" ::: "memory"); };

    floatx4 acc_db[4];
#pragma unroll
    for (int nb = 0; nb < 4; ++nb) acc_db[nb] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int d = 0; d < kDualRing; ++d) {
        load_chunk(d, d);
        fence_chunk();
    }
    for (int c0 = 0; c0 < n_chunks; c0 += kDualRing) {
#pragma unroll
        for (int d = 0; d < kDualRing; ++d) {
            // (slots beyond the piece's last chunk hold zeros and are worked through like the others: a loop body
            // without branches is what lets the compiler count the loads in flight)
            const int ch = c0 + d;
            store_chunk(d);
            fence_chunk();
            load_chunk(ch + kDualRing, d);
            fence_chunk();
            {
                // dB: (s h)^T (rank index x rows) times dy (rows x columns), both by transposing reads
                const int rrow = kg * 8 + (l16 >> 2), rcol = (l16 & 3) * 4;
                bf16x8 sf;
                {
                    const uint8_t *src = stage_s + rrow * C::SPITCH + rcol * 2;
                    const bf16x4 lo = lds_tr(src), hi = lds_tr(src + 4 * C::SPITCH);
                    sf = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                }
#pragma unroll
                for (int nb = 0; nb < 4; ++nb) {
                    const uint8_t *src = stage_b + rrow * C::BPITCH + (nb * 16 + rcol) * 2;
                    const bf16x4 lo = lds_tr(src), hi = lds_tr(src + 4 * C::BPITCH);
                    const bf16x8 bf = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                    acc_db[nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(sf, bf, acc_db[nb], 0, 0, 0);
                }
                // dh: B_a (rank index x columns) times dy rows (columns x rows); lane = row l16 of a 16-row tile
                floatx4 acc_dh[2];
#pragma unroll
                for (int t = 0; t < 2; ++t) {
                    acc_dh[t] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int ks = 0; ks < 2; ++ks) {
                        const bf16x8 dyf = *reinterpret_cast<const bf16x8 *>(stage_b + (t * 16 + l16) * C::BPITCH + (ks * 32 + kg * 8) * 2);
                        acc_dh[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, bfrag[ks]), dyf, acc_dh[t], 0, 0, 0);
                    }
                }
                // lane holds row 16 t + l16 of the chunk, rank indices 4 kg + 0..3
                float *mine = red + (((ch & 1) * 8 + wave) * 32) * C::RED_LD;
#pragma unroll
                for (int t = 0; t < 2; ++t) *reinterpret_cast<floatx4 *>(mine + (t * 16 + l16) * C::RED_LD + kg * 4) = acc_dh[t];
                __syncthreads();
                const int m = tid >> 4, q = tid & 15;
                float sum = 0.f;
#pragma unroll
                for (int w = 0; w < 8; ++w) sum += red[((((ch & 1) * 8 + w) * 32) + m) * C::RED_LD + q];
                if (ch * 32 + m < kDualMaxPieceRows) s_dh[(ch * 32 + m) * 16 + q] = sum;
            }
        }
    }

    // this group's slice of dh for the piece's rows
    __syncthreads();
    for (int idx = tid; idx < n_rows * 16; idx += 512)
        p.part_dh[((int64_t)blockIdx.x * p.part_rows + r_lo + (idx >> 4)) * p.part_ld + (idx & 15)] = s_dh[idx];

    // dB: lane holds column nb*16 + l16 of the slab, rank indices 4 kg + j
    const bool direct = n_pieces == 1;
    float *base = direct ? reinterpret_cast<float *>(p.out_tab[it.adapter]) : p.part_dB + (int64_t)blockIdx.y * 16 * N;
#pragma unroll
    for (int nb = 0; nb < 4; ++nb) {
        const int n = n0 + nb * 16 + l16;
        if (n >= N) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int q = kg * 4 + j;
            if (q >= rank) continue;
            float *d = base + (int64_t)q * N + n;
            *d = (direct && p.accumulate) ? *d + acc_db[nb][j] : acc_db[nb][j];
        }
    }
}

// dB_a of the adapters whose rows were cut into several pieces: the pieces' sums added in piece order, four loads in
// flight at a time.  Block (x, q, item): 256 columns of rank index q.
__global__ void __launch_bounds__(256) dual_sum_kernel(DualArgs p)
{
    const GradItem it = p.items[blockIdx.z];
    const int n_pieces = (it.row_hi - it.row_lo + p.piece_rows - 1) / p.piece_rows;
    const int n = blockIdx.x * 256 + threadIdx.x, q = blockIdx.y;
    if (n_pieces <= 1 || n >= p.N || q >= it.rank) return;
    const float *part = p.part_dB + ((int64_t)blockIdx.z * p.max_pieces * 16 + q) * p.N + n;
    const int64_t stride = (int64_t)16 * p.N;
    float sum = 0.f;
    int pc = 0;
    for (; pc + 4 <= n_pieces; pc += 4) {
        const float v0 = part[(pc + 0) * stride], v1 = part[(pc + 1) * stride], v2 = part[(pc + 2) * stride],
                    v3 = part[(pc + 3) * stride];
        sum += v0;
        sum += v1;
        sum += v2;
        sum += v3;
    }
    for (; pc < n_pieces; ++pc) sum += part[pc * stride];
    float *d = reinterpret_cast<float *>(p.out_tab[it.adapter]) + (int64_t)q * p.N + n;
    *d = p.accumulate ? *d + sum : sum;
}

// =========================================================================================
// launchers
// =========================================================================================
// Row tiles per band of the tile order (see tile_coords): as many as keep a band's rows of the first operand
// (tile_rows x K elements of 2 bytes per row tile) within kBandBytes, in whole groups of 8; 0 = one band.
// Measured on 16384 rows, K = 8192 (268 MB of rows; 4.2 MB per row tile of 256), forward GEMM in us for N = 8192 / 28672:
// one band 1600 / 5687, bands of 8 row tiles 1530 / 5581, 16: 1484 / 5347, 32: 1474 / 5302, 40: 1550 / 5547 - beside a band's
// rows the cache also holds the column tiles the XCDs are at.  Where not even 16 row tiles fit (K = 28672: 14.7 MB per row
// tile) bands of 8 were 1 % slower than none: no bands there.
constexpr int64_t kBandBytes = (int64_t)140 << 20;
int gemm_band_rows(int tile_rows, int K, int tiles_m)
{
    const int64_t per_tile = (int64_t)tile_rows * K * 2;
    const int64_t band = (kBandBytes / (per_tile > 0 ? per_tile : 1)) & ~(int64_t)7;
    return (band < 16 || band >= tiles_m) ? 0 : (int)band;
}

void host_tile_order(int tiles_m, int tiles_n, int band, int32_t *tm, int32_t *tn)
{
    for (int pid = 0; pid < tiles_m * tiles_n; ++pid) {
        int m, n;
        tile_coords(pid, tiles_m, tiles_n, band, m, n);
        tm[pid] = m;
        tn[pid] = n;
    }
}

template <int BM, int BN, bool KM, bool SWIGLU = false, bool SIBS = false>
static hipError_t launch_gemm_t(const GemmArgs &a, hipStream_t st)
{
    // four waves, 2 x 2
    constexpr int NT = 256;
    // two stages; the 256x256 tiles keep the rows' area of the extension behind them
    constexpr int stage_bytes = 2 * (BM + BN) * 128 + ((!SIBS && BM * BN == 256 * 256) ? BM * 128 : 0);
    constexpr int epi_bytes = BM * BN * 2 + BM * 2 * 16;  // per wave (BM/2) rows of (BN/2) * 2 + 16 bytes
    constexpr int smem = stage_bytes > epi_bytes ? stage_bytes : epi_bytes;
    static_assert(!SWIGLU || smem >= BM * (BN / 2) * 4, "the up halves of all rows pass through LDS as fp32");
    auto kern = gemm_lora_kernel<BM, BN, 2, 2, KM, false, SWIGLU, false, SIBS>;
    static bool attr_done = false;
    if (!attr_done) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, smem);
        if (e != hipSuccess) return e;
        attr_done = true;
    }
    const int grid = a.tiles_m * a.tiles_n;
    if (grid <= 0) return hipSuccess;
    GemmArgs b = a;
    b.band_m = gemm_band_rows(BM, a.K, a.tiles_m);
    COLLM_LAUNCH(kern, dim3(grid), dim3(NT), smem, st, b);
    return hipGetLastError();
}

hipError_t launch_gemm(const GemmArgs &a, int tile_cfg, bool b_kmajor, hipStream_t st)
{
    if (a.n_sib > 1) {
        // sibling projections side by side (forward only, second operand [K][N]): the kernels whose extension
        // loads the rows' operand per batch, at the sibling's offset inside each adapter's ranks
        if (b_kmajor) return hipErrorInvalidValue;
        switch (tile_cfg) {
        case kTile256x256:
            return launch_gemm_t<256, 256, false, false, true>(a, st);
        case kTile128x128:
            return launch_gemm_t<128, 128, false, false, true>(a, st);
        default:
            return hipErrorInvalidValue;
        }
    }
    switch (tile_cfg) {
    case kTile256x256:
        return b_kmajor ? launch_gemm_t<256, 256, true>(a, st) : launch_gemm_t<256, 256, false>(a, st);
    case kTile128x128:
        return b_kmajor ? launch_gemm_t<128, 128, true>(a, st) : launch_gemm_t<128, 128, false>(a, st);
    default:
        return hipErrorInvalidValue;
    }
}

hipError_t launch_wide(const GemmArgs &a, int n_items, int rpad, int n_split, bool t_kmajor, hipStream_t st)
{
    static_assert(kWideRows == 128, "the rank-wide pass runs 128x128 tiles");
    if (n_items <= 0) return hipSuccess;
    if (n_split < 1 || !a.part || !a.items || !a.tab || a.k_per_split % 64 != 0) return hipErrorInvalidValue;
    const int smem = wide_stages(t_kmajor) * (128 + 128) * 128;
    GemmArgs b = a;
    b.n_items = n_items;
    if (!b.warm_base || b.warm_bytes < 16) b.warm_blocks = 0;
    const dim3 grid(n_items + b.warm_blocks, (rpad + 127) / 128, n_split);
    auto launch = [&](auto kern) -> hipError_t {
        static bool attr_done = false;
        if (!attr_done) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, smem);
            if (e != hipSuccess) return e;
            attr_done = true;
        }
        COLLM_LAUNCH(kern, grid, dim3(512), smem, st, b);
        return hipGetLastError();
    };
    // eight waves, 32 rows x 64 rank columns each (two per SIMD): the loop is bound by what a wave has to issue
    return t_kmajor ? launch(gemm_lora_kernel<128, 128, 4, 2, true, true>) : launch(gemm_lora_kernel<128, 128, 4, 2, false, true>);
}

hipError_t launch_skinny_finish(const SkinnyArgs &a, int n_items, int item_rows, int n_split, hipStream_t st)
{
    if (n_items <= 0) return hipSuccess;
    COLLM_LAUNCH(skinny_finish_kernel, dim3(n_items, (item_rows + 15) / 16), dim3(256), 0, st, a, n_split);
    return hipGetLastError();
}

// adds the K slices of a split GEMM in slice order, rounds once and writes the rows to their tokens;
// block x = row of the order, 4 columns per thread
__global__ void __launch_bounds__(256) gemm_finish_kernel(GemmArgs p, int n_split)
{
    const int r = blockIdx.x;  // row of the launch; row p.row_base + r of the order
    const int tok = p.row_tok[p.row_base + r];
    const int n = (blockIdx.y * 256 + threadIdx.x) * 4;
    if (tok < 0 || n >= p.N) return;
    const floatx4 sum = sum_slices(p.part + (int64_t)r * p.part_ld + n, (int64_t)p.part_rows * p.part_ld, n_split);
    uint2 v;
    v.x = pack_bf16(sum[0], sum[1]);
    v.y = pack_bf16(sum[2], sum[3]);
    *reinterpret_cast<uint2 *>(reinterpret_cast<uint16_t *>(p.out) + (int64_t)tok * p.ldo + n) = v;
}

hipError_t launch_gemm_splitk(const GemmArgs &a, int n_split, bool b_kmajor, hipStream_t st)
{
    if (n_split < 1 || !a.part || a.k_per_split % 64 != 0 || a.part_ld < a.N || a.part_ld % 4 != 0) return hipErrorInvalidValue;
    constexpr int smem = 2 * (128 + 128) * 128;
    const int tiles = a.tiles_m * a.tiles_n;
    if (tiles <= 0) return hipSuccess;
    auto launch = [&](auto kern) -> hipError_t {
        static bool attr_done = false;
        if (!attr_done) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, smem);
            if (e != hipSuccess) return e;
            attr_done = true;
        }
        COLLM_LAUNCH(kern, dim3(tiles, n_split), dim3(256), smem, st, a);
        return hipGetLastError();
    };
    if (a.n_sib > 1) return b_kmajor ? hipErrorInvalidValue : launch(gemm_lora_kernel<128, 128, 2, 2, false, false, false, true, true>);
    return b_kmajor ? launch(gemm_lora_kernel<128, 128, 2, 2, true, false, false, true>)
                    : launch(gemm_lora_kernel<128, 128, 2, 2, false, false, false, true>);
}

hipError_t launch_gemm_finish(const GemmArgs &a, int n_split, hipStream_t st)
{
    if (a.n_rows <= 0) return hipSuccess;
    COLLM_LAUNCH(gemm_finish_kernel, dim3(a.n_rows, (a.N / 4 + 255) / 256), dim3(256), 0, st, a, n_split);
    return hipGetLastError();
}

hipError_t launch_gemm_swiglu(const GemmArgs &a, int tile_cfg, hipStream_t st)
{
    switch (tile_cfg) {
    case kTile256x256:
        return launch_gemm_t<256, 256, false, true>(a, st);
    case kTile128x128:
        return launch_gemm_t<128, 128, false, true>(a, st);
    default:
        return hipErrorInvalidValue;
    }
}

int gemm_tile_rows(int tile_cfg) { return tile_cfg == kTile128x128 ? 128 : 256; }
int gemm_tile_cols(int tile_cfg) { return tile_cfg == kTile256x256 ? 256 : 128; }

template <int RP, bool KM, int RT>
static hipError_t launch_skinny_t(const SkinnyArgs &a, int n_items, int n_split, hipStream_t st)
{
    using C = SkinnyCfg<RP>;
    constexpr int smem = C::KW * 16 * RT * C::RED_LD * 4 + (KM ? 0 : C::KW * C::STAGE_BYTES);
    auto kern = skinny_kernel<RP, KM, RT>;
    static bool attr_done = false;
    if (!attr_done) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, smem);
        if (e != hipSuccess) return e;
        attr_done = true;
    }
    SkinnyArgs b = a;
    b.n_items = n_items;
    if (!b.warm_base || b.warm_bytes < 16) b.warm_blocks = 0;
    COLLM_LAUNCH(kern, dim3(n_items + b.warm_blocks, n_split), dim3(C::KW * 64), smem, st, b);
    if (n_split > 1) COLLM_LAUNCH(skinny_finish_kernel, dim3(n_items, RT), dim3(256), 0, st, a, n_split);
    return hipGetLastError();
}

template <int RP, bool KM>
static hipError_t launch_skinny_rt(const SkinnyArgs &a, int n_items, int row_tiles, int n_split, hipStream_t st)
{
    constexpr int RTMAX = SkinnyCfg<RP>::RTMAX;
    if (row_tiles > RTMAX) return hipErrorInvalidValue;
    if constexpr (RTMAX >= 2)
        if (row_tiles > 1) return launch_skinny_t<RP, KM, 2>(a, n_items, n_split, st);
    return launch_skinny_t<RP, KM, 1>(a, n_items, n_split, st);
}

int skinny_max_row_tiles(int rpad) { return rpad <= 128 ? 2 : 1; }
int skinny_waves(int rpad) { return rpad <= 32 ? 8 : 4; }
int skinny_chunk(int rpad) { return rpad <= 64 ? 64 : 32; }
int skinny_depth(int rpad, int row_tiles)
{
    // as in skinny_kernel: four chunks in flight where a chunk needs few registers, else two
    const int rp = rpad <= 16 ? 16 : (rpad <= 32 ? 32 : (rpad <= 64 ? 64 : (rpad <= 128 ? 128 : 256)));
    const int steps = skinny_chunk(rpad) / 32, nb = rp / 16;
    return (row_tiles * steps + steps * nb <= 8) ? 4 : 2;
}

hipError_t launch_skinny(const SkinnyArgs &a, int n_items, int rpad, int row_tiles, int n_split, bool t_kmajor,
                         hipStream_t st)
{
    if (n_items <= 0) return hipSuccess;
    if (n_split < 1 || (n_split > 1 && !a.part)) return hipErrorInvalidValue;
#define COLLM_SK(RP) \
    return t_kmajor ? launch_skinny_rt<RP, true>(a, n_items, row_tiles, n_split, st) \
                    : launch_skinny_rt<RP, false>(a, n_items, row_tiles, n_split, st)
    if (rpad <= 16) { COLLM_SK(16); }
    if (rpad <= 32) { COLLM_SK(32); }
    if (rpad <= 64) { COLLM_SK(64); }
    if (rpad <= 128) { COLLM_SK(128); }
    COLLM_SK(256);
#undef COLLM_SK
}

template <int RP, bool SMALL_BF>
static hipError_t launch_grad_t(const GradArgs &a, int n_grad, int rpad, hipStream_t st)
{
    using C = GradCfg<RP>;
    auto kern = grad_kernel<RP, SMALL_BF>;
    static bool attr_done = false;
    if (!attr_done) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, C::SMEM);
        if (e != hipSuccess) return e;
        attr_done = true;
    }
    const dim3 grid((a.N + 63) / 64, n_grad, (rpad + RP - 1) / RP);
    COLLM_LAUNCH(kern, grid, dim3(C::KW * 64), C::SMEM, st, a);
    return hipGetLastError();
}

hipError_t launch_dual(const DualArgs &a, hipStream_t st)
{
    if (a.n_grad <= 0) return hipSuccess;
    if (a.piece_rows < 32 || a.piece_rows % 32 || a.piece_rows > kDualMaxPieceRows || a.max_pieces < 1 || !a.part_dh ||
        !a.part_dB || a.part_ld < 16)
        return hipErrorInvalidValue;
    static bool attr_done = false;
    if (!attr_done) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(dydual_kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, DualCfg::SMEM);
        if (e != hipSuccess) return e;
        attr_done = true;
    }
    DualArgs b = a;
    if (!b.warm_base || b.warm_bytes < 16) b.warm_rows = 0;
    const dim3 grid((a.N + kDualCols - 1) / kDualCols, a.n_grad * a.max_pieces + b.warm_rows);
    COLLM_LAUNCH(dydual_kernel, grid, dim3(512), DualCfg::SMEM, st, b);
    return hipGetLastError();
}

hipError_t launch_dual_sum(const DualArgs &a, hipStream_t st)
{
    if (a.n_grad <= 0 || a.max_pieces <= 1) return hipSuccess;
    COLLM_LAUNCH(dual_sum_kernel, dim3((a.N + 255) / 256, 16, a.n_grad), dim3(256), 0, st, a);
    return hipGetLastError();
}

hipError_t launch_grad(const GradArgs &a, int n_grad, int rpad, hipStream_t st)
{
    if (n_grad <= 0 || a.N <= 0) return hipSuccess;
#define COLLM_GR(RP) return a.small_bf ? launch_grad_t<RP, true>(a, n_grad, rpad, st) : launch_grad_t<RP, false>(a, n_grad, rpad, st)
    if (rpad <= 16) { COLLM_GR(16); }
    if (rpad <= 32) { COLLM_GR(32); }
    if (rpad <= 64) { COLLM_GR(64); }
    COLLM_GR(128);  // larger ranks: 128-wide slices on grid.z
#undef COLLM_GR
}

// dst[t][q] = bf16(mult * src[tok(t)][q]) for the rows t of a row order; columns beyond src_cols are zero
__global__ void __launch_bounds__(256) pack_rows_kernel(const float *__restrict__ src, int64_t ld_src, int src_cols,
                                                        const int32_t *__restrict__ row_tok, int n_rows, float mult,
                                                        uint16_t *__restrict__ dst, int ld_dst)
{
    const int ppr = ld_dst / 8;
    const int64_t n = (int64_t)n_rows * ppr;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) {
        const int t = (int)(i / ppr), q = (int)(i % ppr) * 8;
        const int tok = row_tok[t];
        float v[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = (tok >= 0 && q + e < src_cols) ? src[(int64_t)tok * ld_src + q + e] * mult : 0.f;
        uint4 o;
        o.x = pack_bf16(v[0], v[1]);
        o.y = pack_bf16(v[2], v[3]);
        o.z = pack_bf16(v[4], v[5]);
        o.w = pack_bf16(v[6], v[7]);
        *reinterpret_cast<uint4 *>(dst + (int64_t)t * ld_dst + q) = o;
    }
}

hipError_t launch_pack_rows(const float *src, int64_t ld_src, int src_cols, const int32_t *row_tok, int n_rows,
                            float mult, void *dst, int ld_dst, hipStream_t st)
{
    if (n_rows <= 0) return hipSuccess;
    const int64_t n = (int64_t)n_rows * (ld_dst / 8);
    const int grid = (int)std::min<int64_t>((n + 255) / 256, 4096);
    COLLM_LAUNCH(pack_rows_kernel, dim3(grid), dim3(256), 0, st, src, ld_src, src_cols, row_tok, n_rows, mult,
                       reinterpret_cast<uint16_t *>(dst), ld_dst);
    return hipGetLastError();
}

}  // namespace collm
