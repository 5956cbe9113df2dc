// Adapter update kernels: the step after the backward pass of the mixed-batch LoRA layer.
//   fedavg   dst = (1/K) sum_k src_k        aggregation of the replicas' adapter copies
//   adamw    one AdamW step on an adapter table from its fp32 gradient
//   swiglu_bwd  gradient of silu(gate) * up with respect to both pre-activations, training rows only
// All are element-wise and HBM-bound: 16-byte loads and stores, no shared memory.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kernels.h"

namespace collm {

namespace {

__device__ __forceinline__ float bf16_to_f32(uint16_t v) { return __uint_as_float((uint32_t)v << 16); }
__device__ __forceinline__ uint16_t f32_to_bf16(float f)
{
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    typedef float floatx2 __attribute__((ext_vector_type(2)));
    floatx2 v = {f, 0.f};
    return (uint16_t)(__builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2)) & 0xffffu);
}

// EPL elements per lane per trip: 8 bf16 or 4 fp32 (16 bytes)
template <bool BF16>
__global__ void __launch_bounds__(256) fedavg_kernel(FedAvgArgs p)
{
    constexpr int EPL = BF16 ? 8 : 4;
    const int64_t n_vec = p.n / EPL;
    const float inv = 1.0f / (float)p.n_copies;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n_vec; i += (int64_t)gridDim.x * 256) {
        float acc[EPL];
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[e] = 0.f;
        // copies are added in index order
        for (int k = 0; k < p.n_copies; ++k) {
            const uint4 v = reinterpret_cast<const uint4 *>(p.src[k])[i];
            const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int e = 0; e < EPL; ++e)
                acc[e] += BF16 ? bf16_to_f32((uint16_t)(w[e >> 1] >> ((e & 1) * 16))) : __uint_as_float(w[e]);
        }
        uint32_t o[4];
        if (BF16) {
#pragma unroll
            for (int e = 0; e < 4; ++e)
                o[e] = (uint32_t)f32_to_bf16(acc[2 * e] * inv) | ((uint32_t)f32_to_bf16(acc[2 * e + 1] * inv) << 16);
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) o[e] = __float_as_uint(acc[e] * inv);
        }
        reinterpret_cast<uint4 *>(p.dst)[i] = make_uint4(o[0], o[1], o[2], o[3]);
    }
    // tail (fewer than EPL elements): one thread
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        for (int64_t j = n_vec * EPL; j < p.n; ++j) {
            float acc = 0.f;
            for (int k = 0; k < p.n_copies; ++k)
                acc += BF16 ? bf16_to_f32(reinterpret_cast<const uint16_t *>(p.src[k])[j])
                            : reinterpret_cast<const float *>(p.src[k])[j];
            if (BF16) reinterpret_cast<uint16_t *>(p.dst)[j] = f32_to_bf16(acc * inv);
            else reinterpret_cast<float *>(p.dst)[j] = acc * inv;
        }
    }
}

template <bool BF16>
__global__ void __launch_bounds__(256) adamw_kernel(AdamWArgs p)
{
    const float c1 = p.lr / p.bias1;      // lr / (1 - beta1^t)
    const float rs2 = p.rsqrt_bias2;      // 1 / sqrt(1 - beta2^t)
    const float keep = 1.0f - p.lr * p.weight_decay;
    auto update = [&](float &w, float g, float &m, float &v) {
        m = p.beta1 * m + (1.0f - p.beta1) * g;
        v = p.beta2 * v + (1.0f - p.beta2) * g * g;
        w = w * keep - c1 * (m / (sqrtf(v) * rs2 + p.eps));
    };
    // four elements per lane per trip, every array moved with 16-byte (8-byte for bf16) accesses
    const int64_t n4 = p.n / 4;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n4; i += (int64_t)gridDim.x * 256) {
        const float4 g4 = reinterpret_cast<const float4 *>(p.grad)[i];
        float4 m4 = reinterpret_cast<const float4 *>(p.m)[i];
        float4 v4 = reinterpret_cast<const float4 *>(p.v)[i];
        float4 w4;
        if (p.master) {
            w4 = reinterpret_cast<const float4 *>(p.master)[i];
        } else if (BF16) {
            const uint2 b = reinterpret_cast<const uint2 *>(p.param)[i];
            w4 = make_float4(bf16_to_f32((uint16_t)b.x), bf16_to_f32((uint16_t)(b.x >> 16)), bf16_to_f32((uint16_t)b.y),
                             bf16_to_f32((uint16_t)(b.y >> 16)));
        } else {
            w4 = reinterpret_cast<const float4 *>(p.param)[i];
        }
        update(w4.x, g4.x, m4.x, v4.x);
        update(w4.y, g4.y, m4.y, v4.y);
        update(w4.z, g4.z, m4.z, v4.z);
        update(w4.w, g4.w, m4.w, v4.w);
        reinterpret_cast<float4 *>(p.m)[i] = m4;
        reinterpret_cast<float4 *>(p.v)[i] = v4;
        if (p.master) reinterpret_cast<float4 *>(p.master)[i] = w4;
        if (BF16) {
            uint2 b;
            b.x = (uint32_t)f32_to_bf16(w4.x) | ((uint32_t)f32_to_bf16(w4.y) << 16);
            b.y = (uint32_t)f32_to_bf16(w4.z) | ((uint32_t)f32_to_bf16(w4.w) << 16);
            reinterpret_cast<uint2 *>(p.param)[i] = b;
        } else {
            reinterpret_cast<float4 *>(p.param)[i] = w4;
        }
    }
    // tail (fewer than four elements): one thread
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        for (int64_t j = n4 * 4; j < p.n; ++j) {
            float w = p.master ? p.master[j]
                               : (BF16 ? bf16_to_f32(reinterpret_cast<const uint16_t *>(p.param)[j])
                                       : reinterpret_cast<const float *>(p.param)[j]);
            float m = p.m[j], v = p.v[j];
            update(w, p.grad[j], m, v);
            p.m[j] = m;
            p.v[j] = v;
            if (p.master) p.master[j] = w;
            if (BF16) reinterpret_cast<uint16_t *>(p.param)[j] = f32_to_bf16(w);
            else reinterpret_cast<float *>(p.param)[j] = w;
        }
    }
}

int grid_for(int64_t work_items)
{
    const int64_t blocks = (work_items + 255) / 256;
    return (int)(blocks < 1 ? 1 : (blocks > 256 * 16 ? 256 * 16 : blocks));  // at most 16 blocks per CU
}

// one block row = one training row, 8 columns per lane
__global__ void __launch_bounds__(256) swiglu_bwd_kernel(SwigluBwdArgs p)
{
    // rows on grid.x (no 65535 limit there), 2048-column slabs on grid.y
    int k = 0;
    while (k + 1 < p.n_seg && (int)blockIdx.x >= p.row0[k + 1]) ++k;
    const int64_t tok = p.tok0[k] + ((int)blockIdx.x - p.row0[k]);
    const int j = (blockIdx.y * 256 + threadIdx.x) * 8;
    if (j >= p.d_ff) return;
    const uint16_t *pre = reinterpret_cast<const uint16_t *>(p.pre) + tok * p.ld_pre;
    const uint4 gv = *reinterpret_cast<const uint4 *>(pre + j);
    const uint4 uv = *reinterpret_cast<const uint4 *>(pre + p.d_ff + j);
    const uint4 dv = *reinterpret_cast<const uint4 *>(reinterpret_cast<const uint16_t *>(p.dout) + tok * p.ld_dout + j);
    const uint32_t gw[4] = {gv.x, gv.y, gv.z, gv.w}, uw[4] = {uv.x, uv.y, uv.z, uv.w}, dw[4] = {dv.x, dv.y, dv.z, dv.w};
    uint32_t og[4], ou[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        uint16_t rg[2], ru[2];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const float g = bf16_to_f32((uint16_t)(gw[e] >> (16 * h)));
            const float u = bf16_to_f32((uint16_t)(uw[e] >> (16 * h)));
            const float d = bf16_to_f32((uint16_t)(dw[e] >> (16 * h)));
            const float sg = 1.f / (1.f + __expf(-g));
            rg[h] = f32_to_bf16(d * u * sg * (1.f + g * (1.f - sg)));
            ru[h] = f32_to_bf16(d * g * sg);
        }
        og[e] = (uint32_t)rg[0] | ((uint32_t)rg[1] << 16);
        ou[e] = (uint32_t)ru[0] | ((uint32_t)ru[1] << 16);
    }
    uint16_t *dy = reinterpret_cast<uint16_t *>(p.dy) + tok * p.ld_dy;
    *reinterpret_cast<uint4 *>(dy + j) = make_uint4(og[0], og[1], og[2], og[3]);
    *reinterpret_cast<uint4 *>(dy + p.d_ff + j) = make_uint4(ou[0], ou[1], ou[2], ou[3]);
}

}  // namespace

hipError_t launch_swiglu_bwd(const SwigluBwdArgs &a, hipStream_t st)
{
    const int rows = a.row0[a.n_seg];
    if (rows <= 0 || a.d_ff <= 0) return hipSuccess;
    COLLM_LAUNCH(swiglu_bwd_kernel, dim3(rows, (a.d_ff / 8 + 255) / 256), dim3(256), 0, st, a);
    return hipGetLastError();
}

hipError_t launch_fedavg(const FedAvgArgs &a, bool bf16, hipStream_t st)
{
    if (a.n <= 0) return hipSuccess;
    const int grid = grid_for(a.n / (bf16 ? 8 : 4));
    if (bf16) COLLM_LAUNCH(fedavg_kernel<true>, dim3(grid), dim3(256), 0, st, a);
    else COLLM_LAUNCH(fedavg_kernel<false>, dim3(grid), dim3(256), 0, st, a);
    return hipGetLastError();
}

hipError_t launch_adamw(const AdamWArgs &a, bool bf16, hipStream_t st)
{
    if (a.n <= 0) return hipSuccess;
    const int grid = grid_for((a.n + 3) / 4);
    if (bf16) COLLM_LAUNCH(adamw_kernel<true>, dim3(grid), dim3(256), 0, st, a);
    else COLLM_LAUNCH(adamw_kernel<false>, dim3(grid), dim3(256), 0, st, a);
    return hipGetLastError();
}

}  // namespace collm
