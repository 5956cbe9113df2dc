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
// K offset 8 * (l / 16); result [4 * (l / 16) + j][l % 16].)
#include <hip/hip_runtime.h>
#include <stdint.h>

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

__device__ __forceinline__ int swz(int row) { return (row ^ (row >> 3)) & 7; }

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

// 8x8 transpose of 16-bit values held as 8 rows of 4 dwords: out[n] holds the 8 values of
// column n (row index ascending).
__device__ __forceinline__ void transpose8x8(const uint4 (&in)[8], uint4 (&out)[8])
{
    const uint32_t *v = reinterpret_cast<const uint32_t *>(in);
    uint32_t *o = reinterpret_cast<uint32_t *>(out);
#pragma unroll
    for (int p = 0; p < 4; ++p) {      // dword p holds columns 2p, 2p+1
#pragma unroll
        for (int kp = 0; kp < 4; ++kp) {  // row pair 2kp, 2kp+1
            const uint32_t a = v[(2 * kp) * 4 + p], b = v[(2 * kp + 1) * 4 + p];
            o[(2 * p) * 4 + kp] = (a & 0xffffu) | (b << 16);
            o[(2 * p + 1) * 4 + kp] = (a >> 16) | (b & 0xffff0000u);
        }
    }
}

// -----------------------------------------------------------------------------------------
// Tile movers.  "K-major" sources have the contraction index contiguous (rows of x, dy and,
// for the backward GEMM, rows of W): 16-byte chunks are copied as they are.  "N-major"
// sources ([K][N] matrices: W, B_a in the forward; dy, x in the gradient kernel) are read
// as 8x8 blocks, transposed in registers and written as chunks.
// -----------------------------------------------------------------------------------------
template <int ROWS, int NT>
struct KMajorMover {
    static constexpr int CH = (ROWS * 8 + NT - 1) / NT;
    uint4 reg[CH];

    // row_ptr(r) returns the address of element [r][0] of the source or nullptr
    template <class RowPtr>
    __device__ __forceinline__ void load(int tid, int k0, int K, RowPtr row_ptr)
    {
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            const int idx = tid + i * NT;
            const int r = idx >> 3, c = idx & 7;
            uint4 v = make_uint4(0, 0, 0, 0);
            if (ROWS * 8 % NT == 0 || idx < ROWS * 8) {
                const uint16_t *p = row_ptr(r);
                const int k = k0 + c * 8;
                if (p != nullptr && k < K) v = ldg16(p + k);
            }
            reg[i] = v;
        }
    }
    __device__ __forceinline__ void store(int tid, uint8_t *tile) const
    {
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            const int idx = tid + i * NT;
            const int r = idx >> 3, c = idx & 7;
            if (ROWS * 8 % NT == 0 || idx < ROWS * 8)
                *reinterpret_cast<uint4 *>(tile + tile_off(r, c)) = reg[i];
        }
    }
};

template <int COLS, int NT>
struct NMajorMover {
    static constexpr int NG = COLS / 8;                 // 8-column groups
    static constexpr int UN = (COLS + NT - 1) / NT;     // 8x8 units per thread (8 k-groups)
    uint4 reg[UN][8];

    // k_row_ptr(k) returns the address of source row k (tile-relative k in 0..63) at the
    // tile's first column, or nullptr; cols_left = number of valid columns from there.
    template <class KRowPtr>
    __device__ __forceinline__ void load(int tid, int cols_left, KRowPtr k_row_ptr)
    {
#pragma unroll
        for (int u = 0; u < UN; ++u) {
            const int idx = tid + u * NT;
            const int ng = idx % NG, kg = idx / NG;
            const bool on = (COLS % NT == 0 || idx < COLS) && (ng * 8 < cols_left);
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                uint4 v = make_uint4(0, 0, 0, 0);
                if (on) {
                    const uint16_t *p = k_row_ptr(kg * 8 + j);
                    if (p != nullptr) v = ldg16(p + ng * 8);
                }
                reg[u][j] = v;
            }
        }
    }
    __device__ __forceinline__ void store(int tid, uint8_t *tile) const
    {
#pragma unroll
        for (int u = 0; u < UN; ++u) {
            const int idx = tid + u * NT;
            const int ng = idx % NG, kg = idx / NG;
            if (COLS % NT == 0 || idx < COLS) {
                uint4 t[8];
                transpose8x8(reg[u], t);
#pragma unroll
                for (int j = 0; j < 8; ++j)
                    *reinterpret_cast<uint4 *>(tile + tile_off(ng * 8 + j, kg)) = t[j];
            }
        }
    }
};

// XCD-aware tile order: consecutive workgroup ids go round-robin to the 8 XCDs, each with
// its own L2.  Give every XCD one contiguous run of the logical tile order, and make that
// order walk groups of GM row tiles column by column so that concurrently running tiles of
// one XCD share rows of the first operand and columns of the second.
__device__ __forceinline__ void tile_coords(int pid, int tiles_m, int tiles_n, int &tm, int &tn)
{
    const int total = tiles_m * tiles_n;
    const int per = total >> 3, rem = total & 7;
    const int xcd = pid & 7, local = pid >> 3;
    const int logical = xcd * per + (xcd < rem ? xcd : rem) + local;
    constexpr int GM = 8;
    const int group = logical / (GM * tiles_n);
    const int first = group * GM;
    const int gsz = (tiles_m - first) < GM ? (tiles_m - first) : GM;
    const int in_group = logical - group * GM * tiles_n;
    tm = first + in_group % gsz;
    tn = in_group / gsz;
}

// =========================================================================================
// gemm_lora
//
// Block tile BM x BN, K step 64, WGM x WGN waves of (BM/WGM) x (BN/WGN) each.  Software
// pipeline, two LDS stages:
//   * the registers `areg`/`breg` always hold a tile in flight: the part of tile kc+1 that is
//     written to LDS during MFMA step s of tile kc is re-loaded at once with tile kc+2, so a
//     global load has a whole K step (64 MFMAs per wave) to arrive;
//   * operand fragments of MFMA step s+1 are read from LDS while step s multiplies.
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

// 4 rows x 8 columns of 16-bit values (4 x uint4) -> for each column the 4 row values (uint2)
__device__ __forceinline__ void transpose4x8(const uint4 (&in)[4], uint2 (&out)[8])
{
    const uint32_t *v = reinterpret_cast<const uint32_t *>(in);
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        const uint32_t r0 = v[0 * 4 + p], r1 = v[1 * 4 + p], r2 = v[2 * 4 + p], r3 = v[3 * 4 + p];
        out[2 * p].x = (r0 & 0xffffu) | (r1 << 16);
        out[2 * p].y = (r2 & 0xffffu) | (r3 << 16);
        out[2 * p + 1].x = (r0 >> 16) | (r1 & 0xffff0000u);
        out[2 * p + 1].y = (r2 >> 16) | (r3 & 0xffff0000u);
    }
}

template <int BM, int BN, int WGM, int WGN, bool B_KMAJOR>
__global__ void __launch_bounds__(WGM *WGN * 64) gemm_lora_kernel(GemmArgs p)
{
    constexpr int NT = WGM * WGN * 64;
    constexpr int WM = BM / WGM, WN = BN / WGN;
    constexpr int MI = WM / 32, NI = WN / 32;
    // second operand in LDS: K-major -> BN rows of 64 K values (swizzled chunks); N-major ->
    // 64 rows (K) of BN values as they lie in memory, row pitch padded by 64 bytes so that the
    // four rows a transposing read touches fall into different banks
    constexpr int BPITCH = BN * 2 + 64;
    constexpr int BTILE = B_KMAJOR ? BN * 128 : 64 * BPITCH;
    constexpr int STAGE = BM * 128 + BTILE;
    constexpr int ACH = BM * 8 / NT;   // 16-byte chunks of the row tile per thread
    constexpr int BCH = BN * 8 / NT;   // chunks of the second operand's tile per thread
    constexpr int NG = BN / 8;         // chunks per N-major row
    static_assert((BM * 8) % NT == 0 && (BN * 8) % NT == 0 && NT % NG == 0, "tile/thread mismatch");
    static_assert(ACH % 4 == 0 || ACH == 2, "row chunks are moved in four (or two) parts per K step");
    extern __shared__ __align__(16) uint8_t smem[];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave % WGM, wn = wave / WGM;
    int tile_m, tile_n;
    tile_coords(blockIdx.x, p.tiles_m, p.tiles_n, tile_m, tile_n);
    const int m0 = tile_m * BM, n0 = tile_n * BN;
    const int K = p.K, N = p.N;
    const int32_t *__restrict__ row_tok = p.row_tok;

    const __amdgpu_buffer_rsrc_t ra = make_rsrc(p.a, p.a_bytes);
    const __amdgpu_buffer_rsrc_t rb = make_rsrc(p.b, p.b_bytes);

    // ---- per-thread source offsets (bytes) and LDS destinations ---------------------------
    const int c8 = tid & 7;        // chunk column of this thread in K-major tiles
    const int r8 = tid >> 3;       // first row of this thread in K-major tiles
    uint32_t aoff[ACH];
#pragma unroll
    for (int i = 0; i < ACH; ++i) {
        const int tok = row_tok[m0 + r8 + i * (NT / 8)];
        aoff[i] = tok >= 0 ? (uint32_t)tok * (uint32_t)p.lda * 2u + c8 * 16u : kOob;
    }
    constexpr int NB = BCH;
    uint32_t boff[NB];
    uint32_t bstep = 0;  // N-major: advance of one K step, zero for columns beyond N
    const int bng = tid % NG, bk0 = tid / NG;  // N-major: chunk column and first K row of this thread
    if constexpr (B_KMAJOR) {
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            const int n = n0 + r8 + i * (NT / 8);
            boff[i] = n < N ? (uint32_t)n * (uint32_t)p.ldb * 2u + c8 * 16u : kOob;
        }
    } else {
        const bool on = n0 + bng * 8 < N;
        bstep = on ? 64u * (uint32_t)p.ldb * 2u : 0u;
#pragma unroll
        for (int i = 0; i < NB; ++i)
            boff[i] = on ? ((uint32_t)(bk0 + i * (NT / NG)) * (uint32_t)p.ldb + n0 + bng * 8) * 2u : kOob;
    }

    uint4 areg[ACH];
    uint4 breg[BCH];

    // loads part `part` of `parts` of the tile that starts at K index k0
    auto load_a = [&](int k0, int part, int parts) {
        const bool kin = k0 + c8 * 8 < K;
#pragma unroll
        for (int i = 0; i < ACH; ++i)
            if (i * parts / ACH == part) areg[i] = buf16(ra, kin ? aoff[i] + (uint32_t)k0 * 2u : kOob);
    };
    auto store_a = [&](int stage, int part, int parts) {
        uint8_t *ta = smem + stage * STAGE;
#pragma unroll
        for (int i = 0; i < ACH; ++i)
            if (i * parts / ACH == part)
                *reinterpret_cast<uint4 *>(ta + tile_off(r8 + i * (NT / 8), c8)) = areg[i];
    };
    auto load_b = [&](int k0, int kc, int part, int parts) {
        if constexpr (B_KMAJOR) {
            const bool kin = k0 + c8 * 8 < K;
#pragma unroll
            for (int i = 0; i < NB; ++i)
                if (i * parts / NB == part) breg[i] = buf16(rb, kin ? boff[i] + (uint32_t)k0 * 2u : kOob);
        } else {
#pragma unroll
            for (int i = 0; i < NB; ++i)  // rows beyond K lie beyond the buffer and read as zero
                if (i * parts / NB == part) breg[i] = buf16(rb, boff[i] + (uint32_t)kc * bstep);
        }
    };
    auto store_b = [&](int stage, int part, int parts) {
        uint8_t *tb = smem + stage * STAGE + BM * 128;
#pragma unroll
        for (int i = 0; i < NB; ++i)
            if (i * parts / NB == part) {
                if constexpr (B_KMAJOR)
                    *reinterpret_cast<uint4 *>(tb + tile_off(r8 + i * (NT / 8), c8)) = breg[i];
                else
                    *reinterpret_cast<uint4 *>(tb + (bk0 + i * (NT / NG)) * BPITCH + bng * 16) = breg[i];
            }
    };

    // acc[ni][mi] holds the transposed 32x32 block: lane = row m, registers = columns n
    floatx16 acc[NI][MI];
#pragma unroll
    for (int ni = 0; ni < NI; ++ni)
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
            for (int j = 0; j < 16; ++j) acc[ni][mi][j] = 0.f;

    const int rl = lane & 31, kh = lane >> 5;
    bf16x8 af[2][MI], bf[2][NI];
    auto read_frags = [&](int stage, int ks, int buf) {
        const uint8_t *ta = smem + stage * STAGE;
        const uint8_t *tb = ta + BM * 128;
#pragma unroll
        for (int mi = 0; mi < MI; ++mi) af[buf][mi] = lds_frag(ta, wm * WM + mi * 32 + rl, ks * 2 + kh);
        if constexpr (B_KMAJOR) {
#pragma unroll
            for (int ni = 0; ni < NI; ++ni) bf[buf][ni] = lds_frag(tb, wn * WN + ni * 32 + rl, ks * 2 + kh);
        } else {
            // transposing reads: 16 lanes fetch a 4 (K) x 16 (N) block, lane i of them reads 4
            // values of row i / 4 and receives the 4 K values of column i
            const int g = lane >> 4, i16 = lane & 15;
            const uint8_t *src = tb + (ks * 16 + (g >> 1) * 8 + (i16 >> 2)) * BPITCH +
                                 (wn * WN + (g & 1) * 16 + (i16 & 3) * 4) * 2;
#pragma unroll
            for (int ni = 0; ni < NI; ++ni) {
                const bf16x4 lo = lds_tr(src + ni * 64);
                const bf16x4 hi = lds_tr(src + ni * 64 + 4 * BPITCH);
                bf[buf][ni] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
            }
        }
    };
    auto mma = [&](int buf) {
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
                acc[ni][mi] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bf[buf][ni], af[buf][mi], acc[ni][mi], 0, 0, 0);
    };

    // ---- main K loop ----------------------------------------------------------------------
    const int nk = (K + 63) >> 6;
    if (nk > 0) {
        load_a(0, 0, 1);
        load_b(0, 0, 0, 1);
        store_a(0, 0, 1);
        store_b(0, 0, 1);
        load_a(64, 0, 1);      // tile 1 stays in flight in the registers
        load_b(64, 1, 0, 1);
        __syncthreads();
        read_frags(0, 0, 0);
        for (int kc = 0; kc < nk; ++kc) {
            const int cur = kc & 1, nxt = cur ^ 1;
            const int k2 = (kc + 2) << 6;
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                if (s < 3) read_frags(cur, s + 1, (s + 1) & 1);
                __builtin_amdgcn_sched_barrier(0);
                mma(s & 1);
                __builtin_amdgcn_sched_barrier(0);
                // move one quarter of tile kc+1 from registers to LDS, refill with tile kc+2
                store_a(nxt, s, 4);
                store_b(nxt, s, 4);
                load_a(k2, s, 4);
                load_b(k2, kc + 2, s, 4);
                __builtin_amdgcn_sched_barrier(0);
            }
            __syncthreads();
            if (kc + 1 < nk) read_frags(nxt, 0, 0);
        }
    }

    // ---- low-rank extension: K-steps [s h | dh] x [B_a | A_a^T] of the tile's adapters ----
    {
        const int e0 = p.ext_off[tile_m], e1 = p.ext_off[tile_m + 1];
        const uint16_t *__restrict__ Hs = reinterpret_cast<const uint16_t *>(p.hs);
        uint8_t *ta = smem;
        uint8_t *tb = smem + BM * 128;
        for (int eb = e0; eb < e1; eb += 4) {
            const int nsteps = (e1 - eb) < 4 ? (e1 - eb) : 4;
            ExtStep st[4];
            const uint16_t *tab[4];
            int rk[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if (j < nsteps) {
                    st[j] = p.ext[eb + j];
                    tab[j] = reinterpret_cast<const uint16_t *>(p.ext_tab[st[j].adapter]);
                    rk[j] = p.rank[st[j].adapter];
                } else {
                    st[j] = ExtStep{-1, 0, 0, 0};
                    tab[j] = nullptr;
                    rk[j] = 0;
                }
            }
            // rows: chunk c of row r belongs to step c / 2, rank indices koff + 8 (c % 2) ..
#pragma unroll
            for (int i = 0; i < ACH; ++i) {
                const int r = r8 + i * (NT / 8), c = c8;
                const int j = c >> 1;
                uint4 v = make_uint4(0, 0, 0, 0);
                if (j < nsteps && r >= st[j].row_lo && r < st[j].row_hi)
                    v = ldg16(Hs + (int64_t)(m0 + r) * p.hs_ld + st[j].koff + (c & 1) * 8);
                *reinterpret_cast<uint4 *>(ta + tile_off(r, c)) = v;
            }
            if constexpr (B_KMAJOR) {
                // table rows are output columns: A_a[n][q], row length rank
#pragma unroll
                for (int i = 0; i < BCH; ++i) {
                    const int r = r8 + i * (NT / 8), c = c8;
                    const int j = c >> 1;
                    uint4 v = make_uint4(0, 0, 0, 0);
                    if (j < nsteps && n0 + r < N) {
                        const int q0 = st[j].koff + (c & 1) * 8;
                        const uint16_t *src = tab[j] + (int64_t)(n0 + r) * rk[j] + q0;
                        if ((rk[j] & 7) == 0) {
                            if (q0 < rk[j]) v = ldg16(src);
                        } else {
                            uint16_t e[8];
#pragma unroll
                            for (int q = 0; q < 8; ++q) e[q] = (q0 + q < rk[j]) ? src[q] : (uint16_t)0;
                            v.x = e[0] | ((uint32_t)e[1] << 16);
                            v.y = e[2] | ((uint32_t)e[3] << 16);
                            v.z = e[4] | ((uint32_t)e[5] << 16);
                            v.w = e[6] | ((uint32_t)e[7] << 16);
                        }
                    }
                    *reinterpret_cast<uint4 *>(tb + tile_off(r, c)) = v;
                }
            } else {
                // table rows are rank indices: B_a[q][n], row length ext_ld; tile row 16 j + i
                // is rank index koff_j + i
#pragma unroll
                for (int i = 0; i < NB; ++i) {
                    const int k = bk0 + i * (NT / NG);
                    const int j = k >> 4;
                    uint4 v = make_uint4(0, 0, 0, 0);
                    if (j < nsteps && n0 + bng * 8 < N) {
                        const int q = st[j].koff + (k & 15);
                        if (q < rk[j]) v = ldg16(tab[j] + (int64_t)q * p.ext_ld + n0 + bng * 8);
                    }
                    *reinterpret_cast<uint4 *>(tb + k * BPITCH + bng * 16) = v;
                }
            }
            __syncthreads();
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                if (ks < nsteps) {
                    read_frags(0, ks, 0);
                    mma(0);
                }
            }
            __syncthreads();
        }
    }

    // ---- epilogue: one rounding to bf16, rows scattered back to their tokens --------------
    {
        uint16_t *__restrict__ Out = reinterpret_cast<uint16_t *>(p.out);
#pragma unroll
        for (int mi = 0; mi < MI; ++mi) {
            const int tok = row_tok[m0 + wm * WM + mi * 32 + rl];
            if (tok < 0) continue;
            uint16_t *orow = Out + (int64_t)tok * p.ldo;
#pragma unroll
            for (int ni = 0; ni < NI; ++ni) {
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int n = n0 + wn * WN + ni * 32 + g * 8 + kh * 4;
                    if (n < N) {
                        uint2 v;
                        v.x = pack_bf16(acc[ni][mi][g * 4 + 0], acc[ni][mi][g * 4 + 1]);
                        v.y = pack_bf16(acc[ni][mi][g * 4 + 2], acc[ni][mi][g * 4 + 3]);
                        *reinterpret_cast<uint2 *>(orow + n) = v;
                    }
                }
            }
        }
    }
}

// =========================================================================================
// skinny: out[m][q] = sum_k in[tok(m)][k] * table_a[k][q]     (rank-wide output)
// One block = one item (<= 64 rows of one adapter) x one K slice.  Four waves own 16 rows
// each (16x16x32 MFMA); the adapter table tile is staged in LDS for all of them.
// =========================================================================================
template <int RP, bool T_KMAJOR>
__global__ void __launch_bounds__(256) skinny_kernel(SkinnyArgs p)
{
    constexpr int NT = 256, BM = kSkinnyRows;
    constexpr int NI = RP / 16;
    constexpr int STAGE = (BM + RP) * 128;
    extern __shared__ __align__(16) uint8_t smem[];
    __shared__ int s_last;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const SkinnyItem it = p.items[blockIdx.x];
    const int ks = blockIdx.y;
    const int K = p.K;
    const int k_lo = ks * p.k_slice;
    const int k_hi = (k_lo + p.k_slice) < K ? (k_lo + p.k_slice) : K;
    const int rank = it.rank;
    const int rp = (rank + 15) & ~15;

    const uint16_t *__restrict__ In = reinterpret_cast<const uint16_t *>(p.in);
    const uint16_t *__restrict__ tab = reinterpret_cast<const uint16_t *>(p.tab[it.adapter]);
    const int32_t *__restrict__ row_tok = p.row_tok;

    KMajorMover<BM, NT> amov;
    KMajorMover<RP, NT> bmov_k;
    NMajorMover<RP, NT> bmov_n;

    auto a_row_ptr = [&](int r) -> const uint16_t * {
        if (r >= it.n_rows) return nullptr;
        const int tok = row_tok[it.row_lo + r];
        return tok >= 0 ? In + (int64_t)tok * p.ld_in : nullptr;
    };
    auto load_tiles = [&](int k0) {
        amov.load(tid, k0, k_hi, a_row_ptr);
        if constexpr (T_KMAJOR) {  // table [rank][K]
            bmov_k.load(tid, k0, k_hi, [&](int r) -> const uint16_t * {
                return r < rank ? tab + (int64_t)r * K : nullptr;
            });
        } else {  // table [K][rank]; rows of `rank` elements are only 16-byte loadable if rank % 8 == 0
            if ((rank & 7) == 0) {
                bmov_n.load(tid, rank, [&](int k) -> const uint16_t * {
                    return (k0 + k < k_hi) ? tab + (int64_t)(k0 + k) * rank : nullptr;
                });
            } else {
#pragma unroll
                for (int u = 0; u < bmov_n.UN; ++u) {
                    const int idx = tid + u * NT;
                    const int ng = idx % bmov_n.NG, kg = idx / bmov_n.NG;
#pragma unroll
                    for (int j = 0; j < 8; ++j) {
                        uint16_t e[8];
                        const int k = k0 + kg * 8 + j;
#pragma unroll
                        for (int q = 0; q < 8; ++q) {
                            const int col = ng * 8 + q;
                            e[q] = ((RP % NT == 0 || idx < RP) && k < k_hi && col < rank)
                                       ? tab[(int64_t)k * rank + col]
                                       : (uint16_t)0;
                        }
                        bmov_n.reg[u][j] = make_uint4(e[0] | ((uint32_t)e[1] << 16), e[2] | ((uint32_t)e[3] << 16),
                                                      e[4] | ((uint32_t)e[5] << 16), e[6] | ((uint32_t)e[7] << 16));
                    }
                }
            }
        }
    };
    auto store_tiles = [&](int stage) {
        uint8_t *ta = smem + stage * STAGE;
        uint8_t *tb = ta + BM * 128;
        amov.store(tid, ta);
        if constexpr (T_KMAJOR) bmov_k.store(tid, tb);
        else bmov_n.store(tid, tb);
    };

    floatx4 acc[NI];
#pragma unroll
    for (int ni = 0; ni < NI; ++ni) acc[ni] = floatx4{0.f, 0.f, 0.f, 0.f};

    const int nk = (k_hi - k_lo + 63) >> 6;
    if (nk > 0) {
        load_tiles(k_lo);
        store_tiles(0);
        __syncthreads();
        for (int kc = 0; kc < nk; ++kc) {
            const bool more = kc + 1 < nk;
            if (more) load_tiles(k_lo + ((kc + 1) << 6));
            {
                const uint8_t *ta = smem + (kc & 1) * STAGE;
                const uint8_t *tb = ta + BM * 128;
                const int rl = lane & 15, kq = lane >> 4;
#pragma unroll
                for (int s = 0; s < 2; ++s) {
                    const bf16x8 af = lds_frag(ta, wave * 16 + rl, s * 4 + kq);
#pragma unroll
                    for (int ni = 0; ni < NI; ++ni) {
                        if (ni * 16 < rp) {
                            const bf16x8 bf = lds_frag(tb, ni * 16 + rl, s * 4 + kq);
                            acc[ni] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(bf, af, acc[ni], 0, 0, 0);
                        }
                    }
                }
            }
            if (more) store_tiles((kc + 1) & 1);
            __syncthreads();
        }
    }

    // lane holds row m = wave*16 + lane%16, columns q = ni*16 + 4*(lane/16) + 0..3
    const int m = wave * 16 + (lane & 15);
    const int qb = 4 * (lane >> 4);
    const int n_split = gridDim.y;
    if (n_split > 1) {
        float *part = p.partial + ((int64_t)ks * p.rows_pad + it.row_lo) * p.rpad_ld;
        if (m < it.n_rows) {
#pragma unroll
            for (int ni = 0; ni < NI; ++ni)
                if (ni * 16 < rp)
                    *reinterpret_cast<floatx4 *>(part + (int64_t)m * p.rpad_ld + ni * 16 + qb) = acc[ni];
        }
        __threadfence();
        __syncthreads();
        if (tid == 0) {
            const int old = atomicAdd(p.counters + blockIdx.x, 1);
            s_last = (old == n_split - 1);
            if (s_last) p.counters[blockIdx.x] = 0;  // ready for the next launch
        }
        __syncthreads();
        if (!s_last) return;
        __threadfence();
        if (m < it.n_rows) {
#pragma unroll
            for (int ni = 0; ni < NI; ++ni) {
                if (ni * 16 < rp) {
                    floatx4 sum = floatx4{0.f, 0.f, 0.f, 0.f};
                    for (int s = 0; s < n_split; ++s) {
                        const float *ps = p.partial + ((int64_t)s * p.rows_pad + it.row_lo + m) * p.rpad_ld + ni * 16 + qb;
                        sum += *reinterpret_cast<const floatx4 *>(ps);
                    }
                    acc[ni] = sum;
                }
            }
        }
    }
    if (m >= it.n_rows) return;

    // finalize: fp32 copy (token-indexed h_save or row-indexed workspace) and scaled bf16 copy
    const int row = it.row_lo + m;
    const int tok = row_tok[row];
    float *f32_row = nullptr;
    if (p.f32_out) {
        if (p.f32_by_token) {
            if (p.tok_train[tok]) f32_row = p.f32_out + (int64_t)tok * p.f32_ld;
        } else {
            f32_row = p.f32_out + (int64_t)row * p.f32_ld;
        }
    }
    uint16_t *bf_row = p.bf_out ? reinterpret_cast<uint16_t *>(p.bf_out) + (int64_t)row * p.bf_ld : nullptr;
#pragma unroll
    for (int ni = 0; ni < NI; ++ni) {
        if (ni * 16 < rp) {
            const int q = ni * 16 + qb;
            float v[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] = (q + e < rank) ? acc[ni][e] : 0.f;
            if (f32_row) {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (q + e < p.f32_cols) f32_row[q + e] = v[e] * p.f32_mult;
            }
            if (bf_row) {
                uint2 o;
                o.x = pack_bf16(v[0] * p.bf_mult, v[1] * p.bf_mult);
                o.y = pack_bf16(v[2] * p.bf_mult, v[3] * p.bf_mult);
                *reinterpret_cast<uint2 *>(bf_row + q) = o;
            }
        }
    }
    // zero fill of the fp32 row beyond the padded rank (h_save is max_rank wide)
    if (f32_row) {
        for (int q = rp + qb; q < p.f32_cols; q += 16)
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (q + e < p.f32_cols) f32_row[q + e] = 0.f;
    }
}

// =========================================================================================
// grad: out_a[q][n] = mult * sum_t small[t][q] * big[tok(t)][n]   over the adapter's rows t
// (dB_a: small = h, big = dy;  dA_a^T: small = dh, big = x).  One block = one slice of one
// adapter's training rows x 128 output columns; 4 waves own 32 columns each.
// =========================================================================================
template <int RP>
__global__ void __launch_bounds__(256) grad_kernel(GradArgs p)
{
    constexpr int NT = 256, BN = 128;
    constexpr int MI = RP / 32;
    constexpr int STAGE = (RP + BN) * 128;
    extern __shared__ __align__(16) uint8_t smem[];
    __shared__ int s_last;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n0 = blockIdx.x * BN;
    const int gi = p.slices[2 * blockIdx.y], sl = p.slices[2 * blockIdx.y + 1];
    const GradItem it = p.items[gi];
    const int rank = it.rank;
    const int rp16 = (rank + 15) & ~15;
    const int t_lo = it.row_lo + sl * it.slice_rows;
    const int t_hi = (t_lo + it.slice_rows) < it.row_hi ? (t_lo + it.slice_rows) : it.row_hi;
    const int N = p.N;

    const uint16_t *__restrict__ Big = reinterpret_cast<const uint16_t *>(p.big);
    const int32_t *__restrict__ row_tok = p.row_tok;
    const float *__restrict__ Small = p.small_;

    NMajorMover<BN, NT> bmov;
    constexpr int SU = RP * 8 / NT;  // (q, chunk) units of the small operand per thread
    uint4 sreg[SU];

    auto load_tiles = [&](int t0) {
        bmov.load(tid, N - n0, [&](int k) -> const uint16_t * {
            const int t = t0 + k;
            if (t >= t_hi) return nullptr;
            return Big + (int64_t)row_tok[t] * p.ld_big + n0;
        });
#pragma unroll
        for (int u = 0; u < SU; ++u) {
            const int idx = tid + u * NT;
            const int q = idx % RP, c = idx / RP;
            float v[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int t = t0 + c * 8 + j;
                float x = 0.f;
                if (t < t_hi && q < rank) {
                    const int64_t r = p.small_by_token ? (int64_t)row_tok[t] : (int64_t)t;
                    x = Small[r * p.ld_small + q] * p.small_mult;
                }
                v[j] = x;
            }
            sreg[u] = make_uint4(pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3]), pack_bf16(v[4], v[5]),
                                 pack_bf16(v[6], v[7]));
        }
    };
    auto store_tiles = [&](int stage) {
        uint8_t *ts = smem + stage * STAGE;
        uint8_t *tb = ts + RP * 128;
#pragma unroll
        for (int u = 0; u < SU; ++u) {
            const int idx = tid + u * NT;
            const int q = idx % RP, c = idx / RP;
            *reinterpret_cast<uint4 *>(ts + tile_off(q, c)) = sreg[u];
        }
        bmov.store(tid, tb);
    };

    floatx16 acc[MI];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int j = 0; j < 16; ++j) acc[mi][j] = 0.f;

    const int nk = (t_hi - t_lo + 63) >> 6;
    if (nk > 0) {
        load_tiles(t_lo);
        store_tiles(0);
        __syncthreads();
        for (int kc = 0; kc < nk; ++kc) {
            const bool more = kc + 1 < nk;
            if (more) load_tiles(t_lo + ((kc + 1) << 6));
            {
                const uint8_t *ts = smem + (kc & 1) * STAGE;
                const uint8_t *tb = ts + RP * 128;
                const int rl = lane & 31, kh = lane >> 5;
#pragma unroll
                for (int s = 0; s < 4; ++s) {
                    const bf16x8 bf = lds_frag(tb, wave * 32 + rl, s * 2 + kh);
#pragma unroll
                    for (int mi = 0; mi < MI; ++mi) {
                        if (mi * 32 < rp16) {
                            const bf16x8 sf = lds_frag(ts, mi * 32 + rl, s * 2 + kh);
                            acc[mi] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(sf, bf, acc[mi], 0, 0, 0);
                        }
                    }
                }
            }
            if (more) store_tiles((kc + 1) & 1);
            __syncthreads();
        }
    }

    // lane holds column n, register j of block mi holds row q = mi*32 + 8*(j/4) + 4*(lane/32) + j%4
    const int n = n0 + wave * 32 + (lane & 31);
    const int kh = lane >> 5;
    if (it.ksplit > 1) {
        float *part = p.partial + ((int64_t)it.part_row + (int64_t)sl * rp16) * N;
        if (n < N) {
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                for (int j = 0; j < 16; ++j) {
                    const int q = mi * 32 + 8 * (j >> 2) + 4 * kh + (j & 3);
                    if (q < rp16) part[(int64_t)q * N + n] = acc[mi][j];
                }
        }
        __threadfence();
        __syncthreads();
        int *counter = p.counters + gi * gridDim.x + blockIdx.x;
        if (tid == 0) {
            const int old = atomicAdd(counter, 1);
            s_last = (old == it.ksplit - 1);
            if (s_last) *counter = 0;
        }
        __syncthreads();
        if (!s_last) return;
        __threadfence();
        if (n < N) {
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                for (int j = 0; j < 16; ++j) {
                    const int q = mi * 32 + 8 * (j >> 2) + 4 * kh + (j & 3);
                    float sum = 0.f;
                    if (q < rp16) {
                        const float *ps = p.partial + ((int64_t)it.part_row + q) * N + n;
                        for (int s = 0; s < it.ksplit; ++s) sum += ps[(int64_t)s * rp16 * N];
                    }
                    acc[mi][j] = sum;
                }
        }
    }
    if (n >= N) return;
    float *out = reinterpret_cast<float *>(p.out_tab[it.adapter]);
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const int q = mi * 32 + 8 * (j >> 2) + 4 * kh + (j & 3);
            if (q < rank) {
                float *dst = p.out_transposed ? out + (int64_t)n * rank + q : out + (int64_t)q * N + n;
                const float v = acc[mi][j];
                *dst = p.accumulate ? (*dst + v) : v;
            }
        }
}

// =========================================================================================
// launchers
// =========================================================================================
template <int BM, int BN, int WGM, int WGN, bool KM>
static hipError_t launch_gemm_t(const GemmArgs &a, hipStream_t st)
{
    constexpr int NT = WGM * WGN * 64;
    constexpr int smem = 2 * (BM * 128 + (KM ? BN * 128 : 64 * (BN * 2 + 64)));
    auto kern = gemm_lora_kernel<BM, BN, WGM, WGN, KM>;
    static bool attr_done = false;
    if (!attr_done) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, smem);
        if (e != hipSuccess) return e;
        attr_done = true;
    }
    const int grid = a.tiles_m * a.tiles_n;
    if (grid <= 0) return hipSuccess;
    hipLaunchKernelGGL(kern, dim3(grid), dim3(NT), smem, st, a);
    return hipGetLastError();
}

hipError_t launch_gemm(const GemmArgs &a, int tile_cfg, bool b_kmajor, hipStream_t st)
{
    switch (tile_cfg) {
    case kTile256x256:
        return b_kmajor ? launch_gemm_t<256, 256, 2, 2, true>(a, st) : launch_gemm_t<256, 256, 2, 2, false>(a, st);
    case kTile256x128:
        return b_kmajor ? launch_gemm_t<256, 128, 2, 2, true>(a, st) : launch_gemm_t<256, 128, 2, 2, false>(a, st);
    case kTile128x128:
        return b_kmajor ? launch_gemm_t<128, 128, 2, 2, true>(a, st) : launch_gemm_t<128, 128, 2, 2, false>(a, st);
    case kTile256x256w8:
        return b_kmajor ? launch_gemm_t<256, 256, 2, 4, true>(a, st) : launch_gemm_t<256, 256, 2, 4, false>(a, st);
    default:
        return hipErrorInvalidValue;
    }
}

int gemm_tile_rows(int tile_cfg) { return tile_cfg == kTile128x128 ? 128 : 256; }
int gemm_tile_cols(int tile_cfg) { return (tile_cfg == kTile256x256 || tile_cfg == kTile256x256w8) ? 256 : 128; }

template <int RP, bool KM>
static hipError_t launch_skinny_t(const SkinnyArgs &a, int n_items, int ksplit, hipStream_t st)
{
    constexpr int smem = 2 * (kSkinnyRows + RP) * 128;
    auto kern = skinny_kernel<RP, KM>;
    static bool attr_done = false;
    if (!attr_done) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, smem);
        if (e != hipSuccess) return e;
        attr_done = true;
    }
    hipLaunchKernelGGL(kern, dim3(n_items, ksplit), dim3(256), smem, st, a);
    return hipGetLastError();
}

hipError_t launch_skinny(const SkinnyArgs &a, int n_items, int ksplit, int rpad, bool t_kmajor, hipStream_t st)
{
    if (n_items <= 0) return hipSuccess;
#define COLLM_SK(RP)                                                                         \
    return t_kmajor ? launch_skinny_t<RP, true>(a, n_items, ksplit, st)                      \
                    : launch_skinny_t<RP, false>(a, n_items, ksplit, st)
    if (rpad <= 32) { COLLM_SK(32); }
    if (rpad <= 64) { COLLM_SK(64); }
    if (rpad <= 128) { COLLM_SK(128); }
    COLLM_SK(256);
#undef COLLM_SK
}

template <int RP>
static hipError_t launch_grad_t(const GradArgs &a, int n_tiles, int n_slices, hipStream_t st)
{
    constexpr int smem = 2 * (RP + 128) * 128;
    auto kern = grad_kernel<RP>;
    static bool attr_done = false;
    if (!attr_done) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, smem);
        if (e != hipSuccess) return e;
        attr_done = true;
    }
    hipLaunchKernelGGL(kern, dim3(n_tiles, n_slices), dim3(256), smem, st, a);
    return hipGetLastError();
}

hipError_t launch_grad(const GradArgs &a, int n_tiles, int n_slices, int rpad, hipStream_t st)
{
    if (n_tiles <= 0 || n_slices <= 0) return hipSuccess;
    if (rpad <= 32) return launch_grad_t<32>(a, n_tiles, n_slices, st);
    if (rpad <= 64) return launch_grad_t<64>(a, n_tiles, n_slices, st);
    if (rpad <= 128) return launch_grad_t<128>(a, n_tiles, n_slices, st);
    return launch_grad_t<256>(a, n_tiles, n_slices, st);
}

}  // namespace collm
