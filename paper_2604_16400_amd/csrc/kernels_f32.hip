// fp32 kernels of the mixed-batch LoRA linear layer: the same three passes as the bf16 path
// (GEMM with low-rank extension, skinny rank-wide pass, adapter gradients) with plain fp32
// fused multiply-add and ascending-index sums.  The fp32 element type exists for exactness
// checks on small layers, not for speed; the kernels are simple LDS-tiled loops.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <algorithm>
#include <cstring>

#include "kernels.h"

namespace collm {

constexpr int kF32Tile = 64;

// y[tok(m)][n] = sum_k a[tok(m)][k] b(k, n) + sum_q hs[m][q] table_a(q, n)
template <bool B_KMAJOR>
__global__ void __launch_bounds__(256) gemm_f32_kernel(GemmArgs p)
{
    __shared__ float As[16][kF32Tile + 1];
    __shared__ float Bs[16][kF32Tile + 1];
    const int tid = threadIdx.x;
    const int tx = tid & 15, ty = tid >> 4;
    const int n0 = blockIdx.x * kF32Tile, m0 = blockIdx.y * kF32Tile;
    const float *__restrict__ A = reinterpret_cast<const float *>(p.a);
    const float *__restrict__ B = reinterpret_cast<const float *>(p.b);
    const int K = p.K, N = p.N;

    float acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;

    const int lr = tid >> 2, lq = tid & 3;  // loader coordinates for K-contiguous sources
    const int a_tok = p.row_tok[m0 + lr];
    for (int k0 = 0; k0 < K; k0 += 16) {
        {
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            const int k = k0 + lq * 4;
            if (a_tok >= 0 && k < K) v = *reinterpret_cast<const float4 *>(A + (int64_t)a_tok * p.lda + k);
            As[lq * 4 + 0][lr] = v.x;
            As[lq * 4 + 1][lr] = v.y;
            As[lq * 4 + 2][lr] = v.z;
            As[lq * 4 + 3][lr] = v.w;
        }
        if constexpr (B_KMAJOR) {
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            const int k = k0 + lq * 4;
            if (n0 + lr < N && k < K) v = *reinterpret_cast<const float4 *>(B + (int64_t)(n0 + lr) * p.ldb + k);
            Bs[lq * 4 + 0][lr] = v.x;
            Bs[lq * 4 + 1][lr] = v.y;
            Bs[lq * 4 + 2][lr] = v.z;
            Bs[lq * 4 + 3][lr] = v.w;
        } else {
            const int kk = tid >> 4, nq = tid & 15;
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (k0 + kk < K && n0 + nq * 4 < N)
                v = *reinterpret_cast<const float4 *>(B + (int64_t)(k0 + kk) * p.ldb + n0 + nq * 4);
            Bs[kk][nq * 4 + 0] = v.x;
            Bs[kk][nq * 4 + 1] = v.y;
            Bs[kk][nq * 4 + 2] = v.z;
            Bs[kk][nq * 4 + 3] = v.w;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < 16; ++kk) {
            float a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) a[i] = As[kk][ty * 4 + i];
#pragma unroll
            for (int j = 0; j < 4; ++j) b[j] = Bs[kk][tx * 4 + j];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
        }
        __syncthreads();
    }

    // low-rank extension, straight from global memory (tables and activations are small)
    const float *__restrict__ Hs = reinterpret_cast<const float *>(p.hs);
    const int e0 = p.ext_off[blockIdx.y], e1 = p.ext_off[blockIdx.y + 1];
    for (int e = e0; e < e1; ++e) {
        const ExtStep st = p.ext[e];
        const int koff = (int)(st.koff_rank & 0xffffu), rk = (int)(st.koff_rank >> 16);
        const int row_lo = (int)(st.rows & 0xffffu), row_hi = (int)(st.rows >> 16);
        const float *__restrict__ tab = reinterpret_cast<const float *>(st.tab);
        const int q1 = (koff + kKStep) < rk ? (koff + kKStep) : rk;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int r = ty * 4 + i;
            if (r < row_lo || r >= row_hi) continue;
            for (int q = koff; q < q1; ++q) {
                const float hv = Hs[(int64_t)(m0 + r) * p.hs_ld + q];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int n = n0 + tx * 4 + j;
                    if (n < N) {
                        const float tv = B_KMAJOR ? tab[(int64_t)n * rk + q] : tab[(int64_t)q * p.ext_ld + n];
                        acc[i][j] = fmaf(hv, tv, acc[i][j]);
                    }
                }
            }
        }
    }

    float *__restrict__ Out = reinterpret_cast<float *>(p.out);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int tok = p.row_tok[m0 + ty * 4 + i];
        if (tok < 0) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int n = n0 + tx * 4 + j;
            if (n < N) Out[(int64_t)tok * p.ldo + n] = acc[i][j];
        }
    }
}

// out[m][q] = sum_k in[tok(m)][k] table_a(k, q), k ascending; one item per block
template <bool T_KMAJOR>
__global__ void __launch_bounds__(256) skinny_f32_kernel(SkinnyArgs p)
{
    const SkinnyItem it = p.items[blockIdx.x];
    const int rank = it.rank, K = p.K;
    const float *__restrict__ In = reinterpret_cast<const float *>(p.in);
    const float *__restrict__ tab = reinterpret_cast<const float *>(p.tab[it.adapter]);
    float *__restrict__ scaled = reinterpret_cast<float *>(p.bf_out);
    for (int idx = threadIdx.x; idx < it.n_rows * rank; idx += blockDim.x) {
        const int m = idx / rank, q = idx - m * rank;
        const int row = it.row_lo + m;
        const int tok = p.row_tok[row];
        const float *x = In + (int64_t)tok * p.ld_in;
        float acc = 0.f;
        for (int k = 0; k < K; ++k) {
            const float tv = T_KMAJOR ? tab[(int64_t)q * K + k] : tab[(int64_t)k * rank + q];
            acc = fmaf(x[k], tv, acc);
        }
        if (p.f32_out) {
            if (p.f32_by_token) {
                if (p.tok_train[tok]) p.f32_out[(int64_t)tok * p.f32_ld + q] = acc * p.f32_mult;
            } else {
                p.f32_out[(int64_t)row * p.f32_ld + q] = acc * p.f32_mult;
            }
        }
        if (scaled) scaled[(int64_t)row * p.bf_ld + q] = acc * p.bf_mult;
    }
    // zero fill beyond the rank
    for (int idx = threadIdx.x; idx < it.n_rows * 256; idx += blockDim.x) {
        const int m = idx >> 8, q = rank + (idx & 255);
        const int row = it.row_lo + m;
        const int tok = p.row_tok[row];
        if (p.f32_out && q < p.f32_cols) {
            if (p.f32_by_token) {
                if (p.tok_train[tok]) p.f32_out[(int64_t)tok * p.f32_ld + q] = 0.f;
            } else {
                p.f32_out[(int64_t)row * p.f32_ld + q] = 0.f;
            }
        }
        if (scaled && q < p.bf_ld) scaled[(int64_t)row * p.bf_ld + q] = 0.f;
    }
}

// out_a(q, n) = sum_t small[t][q] big[tok(t)][n], t ascending over the adapter's rows
__global__ void __launch_bounds__(256) grad_f32_kernel(GradArgs p)
{
    const GradItem it = p.items[blockIdx.y];
    const int n = blockIdx.x * 256 + threadIdx.x;
    const int N = p.N, rank = it.rank;
    if (n >= N) return;
    const float *__restrict__ Big = reinterpret_cast<const float *>(p.big);
    float *out = reinterpret_cast<float *>(p.out_tab[it.adapter]);
    for (int q0 = 0; q0 < rank; q0 += 8) {
        float acc[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] = 0.f;
        for (int t = it.row_lo; t < it.row_hi; ++t) {
            const int tok = p.row_tok[t];
            const float bv = Big[(int64_t)tok * p.ld_big + n];
            const float *s = p.small_ + (p.small_by_token ? (int64_t)tok : (int64_t)t) * p.ld_small;
#pragma unroll
            for (int e = 0; e < 8; ++e)
                if (q0 + e < rank) acc[e] = fmaf(s[q0 + e] * p.small_mult, bv, acc[e]);
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int q = q0 + e;
            if (q < rank) {
                float *dst = p.out_transposed ? out + (int64_t)n * rank + q : out + (int64_t)q * N + n;
                *dst = p.accumulate ? (*dst + acc[e]) : acc[e];
            }
        }
    }
}

// Plan upload: the host builds the plan in pinned, device-visible memory and this kernel
// copies it into device memory in stream order (a kernel launch costs the host far less than
// an asynchronous memcpy ordered against kernels on the same stream).  The block that
// finishes last publishes the upload's sequence number in a pinned word, which is how the
// host learns that the staging slot may be reused, without any event call.
__global__ void __launch_bounds__(256) plan_copy_kernel(const int4 *__restrict__ src, int4 *__restrict__ dst, int n16,
                                                        int *counter, volatile uint32_t *done_host, uint32_t seq)
{
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += gridDim.x * blockDim.x) dst[i] = src[i];
    __syncthreads();  // every load of this block has returned: its stores have been issued
    if (threadIdx.x == 0) {
        const int old = atomicAdd(counter, 1);
        if (old == (int)gridDim.x - 1) {
            *counter = 0;  // for the next upload (stream order)
            *done_host = seq;
            __threadfence_system();
        }
    }
}

hipError_t launch_plan_copy(const int32_t *src_pinned, int32_t *dst, size_t first_int, size_t n_ints, int *counter,
                            uint32_t *done_host_dev, uint32_t seq, hipStream_t st)
{
    // both ends are rounded outwards to 16 bytes; the plan block is padded accordingly
    const size_t lo = first_int & ~(size_t)3, hi = (first_int + n_ints + 3) & ~(size_t)3;
    const int n16 = (int)((hi - lo) / 4);
    const int blocks = std::max(1, std::min(256, (n16 + 255) / 256));
    COLLM_LAUNCH(plan_copy_kernel, dim3(blocks), dim3(256), 0, st,
                       reinterpret_cast<const int4 *>(src_pinned + lo), reinterpret_cast<int4 *>(dst + lo), n16, counter,
                       done_host_dev, seq);
    return hipGetLastError();
}

// Plan upload without a staging buffer: a chunk of the plan is an argument of the kernel (arguments are copied
// when the launch is enqueued, so the host block may change afterwards), and the kernel stores it.
constexpr int kPlanChunkInts = 896;  // 3.5 KiB of the 4 KiB a kernel's arguments may take
struct PlanChunk {
    int32_t v[kPlanChunkInts];
};
__global__ void __launch_bounds__(256) plan_words_kernel(PlanChunk c, int32_t *__restrict__ dst, int n)
{
    for (int i = threadIdx.x; i < n; i += 256) dst[i] = c.v[i];
}

hipError_t launch_plan_words(const int32_t *src_host, int32_t *dst, size_t n_ints, hipStream_t st)
{
    PlanChunk c;
    for (size_t lo = 0; lo < n_ints; lo += kPlanChunkInts) {
        const int n = (int)std::min<size_t>(kPlanChunkInts, n_ints - lo);
        std::memcpy(c.v, src_host + lo, (size_t)n * sizeof(int32_t));
        COLLM_LAUNCH(plan_words_kernel, dim3(1), dim3(256), 0, st, c, dst + lo, n);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

__global__ void __launch_bounds__(64) fill_zero_kernel(int4 *__restrict__ dst, int n16)
{
    for (int i = blockIdx.x * 64 + threadIdx.x; i < n16; i += gridDim.x * 64) dst[i] = make_int4(0, 0, 0, 0);
}

hipError_t launch_fill_zero(void *dst, size_t bytes, hipStream_t st)
{
    const int n16 = (int)(bytes / 16);
    if (n16 <= 0) return hipSuccess;
    COLLM_LAUNCH(fill_zero_kernel, dim3(std::min(256, (n16 + 63) / 64)), dim3(64), 0, st, reinterpret_cast<int4 *>(dst), n16);
    return hipGetLastError();
}

hipError_t launch_gemm_f32(const GemmArgs &a, bool b_kmajor, hipStream_t st)
{
    const dim3 grid((a.N + kF32Tile - 1) / kF32Tile, a.tiles_m);
    if (grid.x == 0 || grid.y == 0) return hipSuccess;
    if (b_kmajor) COLLM_LAUNCH(gemm_f32_kernel<true>, grid, dim3(256), 0, st, a);
    else COLLM_LAUNCH(gemm_f32_kernel<false>, grid, dim3(256), 0, st, a);
    return hipGetLastError();
}

hipError_t launch_skinny_f32(const SkinnyArgs &a, int n_items, bool t_kmajor, hipStream_t st)
{
    if (n_items <= 0) return hipSuccess;
    if (t_kmajor) COLLM_LAUNCH(skinny_f32_kernel<true>, dim3(n_items), dim3(256), 0, st, a);
    else COLLM_LAUNCH(skinny_f32_kernel<false>, dim3(n_items), dim3(256), 0, st, a);
    return hipGetLastError();
}

hipError_t launch_grad_f32(const GradArgs &a, int n_grad, hipStream_t st)
{
    if (n_grad <= 0 || a.N <= 0) return hipSuccess;
    COLLM_LAUNCH(grad_f32_kernel, dim3((a.N + 255) / 256, n_grad), dim3(256), 0, st, a);
    return hipGetLastError();
}

}  // namespace collm
