// LDS-tiled fp16 MFMA GEMM for prefill (large M) on gfx950.
//
// Function: the paper's large-M linear operator (Sec. III-B.2) -- out = x W^T
// with fp16 operands and fp32 accumulation (Sec. III-B.4) -- plus the same fused
// low-density operators as the decode path (Sec. III-C.1): RMSNorm in front
// (x*gamma applied while the activation tile is staged, sum x^2 on the side,
// 1/sqrt(mean+eps) applied to the accumulator) and SiLU(gate)*up behind.
// The paper's DDR->GSM->AM dataflow is specific to its scratchpad machine; here
// a workgroup owns a 128 x 128 output tile, stages 128 x 64 operand tiles in
// LDS (double buffered, XOR-swizzled 16-byte pieces so that both the staging
// writes and the MFMA operand reads are bank-conflict free) and runs
// v_mfma_f32_32x32x16_f16 on 64 x 64 wave tiles.
//
// Operand roles: the weight tile is the MFMA "A" operand (rows = output
// features n), the activation tile the "B" operand (columns = tokens m), so a
// lane ends up with 4 consecutive n of one token per register quad -- an 8-byte
// store -- and, for SwiGLU, with g and u of the same (token, j) in registers of
// the same lane (a tile interleaves 8 gate rows with the 8 matching up rows).
#include "thi_internal.h"

namespace thi {

namespace {

constexpr int GB = 128;        // tile extent along n (virtual weight rows) and along m
constexpr int GK = 64;         // k extent of a staged tile
constexpr int GPIECES = GK / 8;   // 16-byte pieces per tile row
constexpr int GTHREADS = 256;

__device__ __forceinline__ int swz(int row, int piece) { return row * GPIECES + (piece ^ ((row >> 1) & 7)); }

__device__ __forceinline__ uint16_t to_half_bits(float v) {
    _Float16 h = (_Float16)v;
    return __builtin_bit_cast(uint16_t, h);
}

template <int EPI>
__global__ __launch_bounds__(GTHREADS) void gemm_tile128(GemmArgs a, int tiles_n)
{
    __shared__ uintx4 Ws[2][GB * GPIECES];
    __shared__ uintx4 Xs[2][GB * GPIECES];
    __shared__ float s_r[GB];

    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int wn = wv & 1, wm = wv >> 1;
    const int tile_n = blockIdx.x % tiles_n, tile_m = blockIdx.x / tiles_n;
    const int K = a.K;
    const int ktiles = (K + GK - 1) / GK;

    // staging role: piece p of rows r0 + 32*i
    const int p = tid & 7, r0 = tid >> 3;
    const uint16_t* wrow[4];
    const uint16_t* xrow[4];
    bool xok[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int v = r0 + 32 * i;
        if (EPI == EPI_SWIGLU) {
            int j = tile_n * 64 + (v >> 4) * 8 + (v & 7);
            j = j < a.N ? j : a.N - 1;
            wrow[i] = (((v >> 3) & 1) ? a.w1 : a.w0) + (size_t)j * K;
        } else {
            int n = tile_n * GB + v;
            n = n < a.N ? n : a.N - 1;
            wrow[i] = a.w0 + (size_t)n * K;
        }
        const int m = tile_m * GB + v;
        xok[i] = m < a.M;
        xrow[i] = a.x + (size_t)(xok[i] ? m : 0) * K;
    }

    uintx4 wreg[4], xreg[4], greg;
    float ssq[4] = {0.f, 0.f, 0.f, 0.f};
    const uintx4 zero4 = {0u, 0u, 0u, 0u};

    auto fetch = [&](int kt) {
        const int k = kt * GK + p * 8;
        const bool kok = k < K;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            wreg[i] = kok ? *reinterpret_cast<const uintx4*>(wrow[i] + k) : zero4;
            xreg[i] = (kok && xok[i]) ? *reinterpret_cast<const uintx4*>(xrow[i] + k) : zero4;
        }
        if (EPI == EPI_RMSNORM) greg = kok ? *reinterpret_cast<const uintx4*>(a.gamma + k) : zero4;
    };
    auto stage = [&](int buf) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int v = r0 + 32 * i;
            uintx4 xv = xreg[i];
            if (EPI == EPI_RMSNORM) {
                half8 xh = __builtin_bit_cast(half8, xv);
                half8 gh = __builtin_bit_cast(half8, greg);
#pragma unroll
                for (int e = 0; e < 8; ++e) { float f = (float)xh[e]; ssq[i] = __builtin_fmaf(f, f, ssq[i]); }
                half8 pr = xh * gh;
                xv = __builtin_bit_cast(uintx4, pr);
            }
            Ws[buf][swz(v, p)] = wreg[i];
            Xs[buf][swz(v, p)] = xv;
        }
    };

    floatx16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    fetch(0);
    stage(0);
    __syncthreads();

    const int lr = lane & 31, lg = lane >> 5;
    for (int kt = 0; kt < ktiles; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < ktiles) fetch(kt + 1);
#pragma unroll
        for (int kk = 0; kk < GK / 16; ++kk) {
            half8 wa[2], xb[2];
#pragma unroll
            for (int tn = 0; tn < 2; ++tn)
                wa[tn] = __builtin_bit_cast(half8, Ws[buf][swz(wn * 64 + tn * 32 + lr, 2 * kk + lg)]);
#pragma unroll
            for (int tm = 0; tm < 2; ++tm)
                xb[tm] = __builtin_bit_cast(half8, Xs[buf][swz(wm * 64 + tm * 32 + lr, 2 * kk + lg)]);
#pragma unroll
            for (int tn = 0; tn < 2; ++tn)
#pragma unroll
                for (int tm = 0; tm < 2; ++tm)
                    acc[tn][tm] = __builtin_amdgcn_mfma_f32_32x32x16_f16(wa[tn], xb[tm], acc[tn][tm], 0, 0, 0);
        }
        if (kt + 1 < ktiles) stage(buf ^ 1);
        __syncthreads();
    }

    if (EPI == EPI_RMSNORM) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            float v = ssq[i];
            v += __shfl_xor(v, 1);
            v += __shfl_xor(v, 2);
            v += __shfl_xor(v, 4);
            if (p == 0) s_r[r0 + 32 * i] = 1.0f / __builtin_sqrtf(v / (float)K + a.eps);
        }
        __syncthreads();
    }

    // ---- epilogue ------------------------------------------------------------
#pragma unroll
    for (int tm = 0; tm < 2; ++tm) {
        const int ml = wm * 64 + tm * 32 + lr;
        const int m = tile_m * GB + ml;
        if (m >= a.M) continue;
        float scale = 1.0f;
        if (EPI == EPI_RMSNORM) scale = s_r[ml];
#pragma unroll
        for (int tn = 0; tn < 2; ++tn) {
            if (EPI == EPI_SWIGLU) {
#pragma unroll
                for (int aa = 0; aa < 4; aa += 2) {
                    const int v = wn * 64 + tn * 32 + 8 * aa;
                    const int j = tile_n * 64 + (v >> 4) * 8 + 4 * lg;
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        if (j + c < a.N) {
                            const float g = acc[tn][tm][4 * aa + c], u = acc[tn][tm][4 * (aa + 1) + c];
                            a.out[(size_t)m * a.ldo + j + c] = to_half_bits(g / (1.0f + __expf(-g)) * u);
                        }
                    }
                }
            } else {
#pragma unroll
                for (int aa = 0; aa < 4; ++aa) {
                    const int n = tile_n * GB + wn * 64 + tn * 32 + 8 * aa + 4 * lg;
                    if (n + 3 < a.N && (a.ldo & 3) == 0) {
                        half4 hv;
#pragma unroll
                        for (int c = 0; c < 4; ++c) hv[c] = (_Float16)(acc[tn][tm][4 * aa + c] * scale);
                        *reinterpret_cast<half4*>(a.out + (size_t)m * a.ldo + n) = hv;
                    } else {
#pragma unroll
                        for (int c = 0; c < 4; ++c)
                            if (n + c < a.N)
                                a.out[(size_t)m * a.ldo + n + c] = to_half_bits(acc[tn][tm][4 * aa + c] * scale);
                    }
                }
            }
        }
    }
}

}  // namespace

hipError_t launch_gemm(const GemmArgs& a, int epilogue, int num_cus, hipStream_t stream)
{
    (void)num_cus;
    const int vrows = (epilogue == EPI_SWIGLU) ? 2 * a.N : a.N;
    const int per_tile = (epilogue == EPI_SWIGLU) ? 64 : GB;
    const int tiles_n = (a.N + per_tile - 1) / per_tile;
    (void)vrows;
    const int tiles_m = (a.M + GB - 1) / GB;
    dim3 g((unsigned)((size_t)tiles_n * tiles_m)), b(GTHREADS);
    switch (epilogue) {
    case EPI_PLAIN: hipLaunchKernelGGL((gemm_tile128<EPI_PLAIN>), g, b, 0, stream, a, tiles_n); break;
    case EPI_RMSNORM: hipLaunchKernelGGL((gemm_tile128<EPI_RMSNORM>), g, b, 0, stream, a, tiles_n); break;
    default: hipLaunchKernelGGL((gemm_tile128<EPI_SWIGLU>), g, b, 0, stream, a, tiles_n); break;
    }
    return hipGetLastError();
}

}  // namespace thi
