// LDS-tiled fp16 MFMA GEMM for prefill (large M) on gfx950.
//
// Function: the paper's large-M linear operator (Sec. III-B.2) -- out = x W^T
// with fp16 operands and fp32 accumulation (Sec. III-B.4) -- plus the same fused
// low-density operators as the decode path (Sec. III-C.1): RMSNorm in front
// (x*gamma applied while the activation tile is staged, sum x^2 on the side,
// 1/sqrt(mean+eps) applied to the accumulator) and SiLU(gate)*up behind.
// The paper's DDR->GSM->AM dataflow is specific to its scratchpad machine; here
// a workgroup owns a BN x BM output tile (up to 256 x 256), stages BN x 64 and
// BM x 64 operand tiles in LDS (double buffered, XOR-swizzled 16-byte pieces so
// that both the staging writes and the MFMA operand reads are bank-conflict
// free) and runs v_mfma_f32_32x32x16_f16 on wave tiles of up to 64 x 128.
//
// Operand roles: the weight tile is the MFMA "A" operand (rows = output
// features n), the activation tile the "B" operand (columns = tokens m), so a
// lane ends up with 4 consecutive n of one token per register quad -- an 8-byte
// store -- and, for SwiGLU, with g and u of the same (token, j) in registers of
// the same lane (a tile interleaves 8 gate rows with the 8 matching up rows).
//
// Workgroups are numbered so that the eight XCDs (one L2 each; hardware deals
// consecutive workgroup ids round-robin to them) each walk a contiguous range
// of tiles, token-tile fastest, so the weight panel an XCD streams is shared by
// the workgroups running on it at that moment.
#include "thi_internal.h"
#include <cstdlib>

namespace thi {

namespace {

constexpr int GK = 64;            // k extent of a staged tile
constexpr int GPIECES = GK / 8;   // 16-byte pieces per tile row

// piece p of tile row `row` lives at 16-byte unit row*8 + (p ^ f(row)); f is a bijection on every
// aligned group of 8 rows and on the even and the odd rows of every aligned group of 16
__device__ __forceinline__ int swz(int row, int piece)
{
    return row * GPIECES + (piece ^ (((row >> 1) & 7) ^ ((row & 1) << 2)));
}

__device__ __forceinline__ uint16_t to_half_bits(float v)
{
    _Float16 h = (_Float16)v;
    return __builtin_bit_cast(uint16_t, h);
}

// One 16-byte piece per lane straight from global memory into LDS (no VGPR staging): lane L of the
// wave lands at lds_base + 16*L.  lds_base must be wave-uniform.
__device__ __forceinline__ void dma16(const uint16_t* src, uintx4* lds_base)
{
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src,
                                     (__attribute__((address_space(3))) void*)lds_base, 16, 0, 0);
}

// BN x BM output tile, WN x WM waves; wave tile (BN/WN) x (BM/WM) built from 32x32 MFMA tiles.
// KTAIL: K is not a multiple of 64 (pieces past K are zero-filled; operands then go through VGPRs).
template <int BN, int BM, int WN, int WM, int EPI, bool KTAIL>
__global__ __launch_bounds__(64 * WN * WM) void gemm_tile(GemmArgs a, int tiles_n, int tiles_m)
{
    constexpr int NWAVES = WN * WM;
    constexpr int THREADS = 64 * NWAVES;
    constexpr int ROWS_PER_PASS = THREADS / GPIECES;
    constexpr int WPASS = BN / ROWS_PER_PASS;   // per-thread pieces of the weight tile
    constexpr int XPASS = BM / ROWS_PER_PASS;
    constexpr int TN = BN / WN / 32;            // MFMA tiles per wave along n
    constexpr int TM = BM / WM / 32;
    constexpr int JPT = (EPI == EPI_SWIGLU) ? BN / 2 : BN;   // physical weight rows per tile
    constexpr bool W_DMA = !KTAIL;                           // weight tile: global -> LDS directly
    constexpr bool X_DMA = !KTAIL && EPI != EPI_RMSNORM;     // activation tile: same unless it is transformed
    constexpr int STAGE = (BN + BM) * GPIECES;   // 16-byte units per stage: weight tile, then activation tile
    static_assert(WPASS >= 1 && XPASS >= 1, "tile too small for the thread count");

    extern __shared__ uintx4 smem[];
    __shared__ float s_r[BM];

    const int tid = threadIdx.x, lane = tid & 63, wv = tid / 64;
    const int wn = wv % WN, wm = wv / WN;

    // XCD-aware numbering of the tiles
    int tile_id;
    {
        const int nwg = gridDim.x, bid = blockIdx.x;
        const int per = nwg / 8, rem = nwg % 8, xcd = bid % 8, local = bid / 8;
        tile_id = xcd * per + (xcd < rem ? xcd : rem) + local;
    }
    const int tile_m = tile_id % tiles_m, tile_n = tile_id / tiles_m;
    (void)tiles_n;
    const int K = a.K;
    const int ktiles = (K + GK - 1) / GK;

    // Staging role.  A wave instruction covers 8 tile rows x 8 pieces = 64 consecutive LDS units; lane L
    // owns unit L of it, i.e. row (8*block + L/8) and physical slot L%8, which holds logical piece
    // slot ^ f(row).  Pass i of this thread handles 8-row block (wv*PASS + i).
    const uint16_t* wsrc[WPASS];
    const uint16_t* xsrc[XPASS];
    int wunit[WPASS], xunit[XPASS];
    const int slot = lane & 7;
#pragma unroll
    for (int i = 0; i < WPASS; ++i) {
        const int v = (wv * WPASS + i) * 8 + (lane >> 3);
        const int piece = slot ^ (((v >> 1) & 7) ^ ((v & 1) << 2));
        wunit[i] = v * GPIECES + slot;
        if (EPI == EPI_SWIGLU) {
            int j = tile_n * JPT + (v >> 4) * 8 + (v & 7);
            j = j < a.N ? j : a.N - 1;
            wsrc[i] = (((v >> 3) & 1) ? a.w1 : a.w0) + (size_t)j * K + piece * 8;
        } else {
            int n = tile_n * BN + v;
            n = n < a.N ? n : a.N - 1;
            wsrc[i] = a.w0 + (size_t)n * K + piece * 8;
        }
    }
    int xpiece[XPASS];
#pragma unroll
    for (int i = 0; i < XPASS; ++i) {
        const int v = (wv * XPASS + i) * 8 + (lane >> 3);
        xpiece[i] = slot ^ (((v >> 1) & 7) ^ ((v & 1) << 2));
        xunit[i] = v * GPIECES + slot;
        int m = tile_m * BM + v;
        m = m < a.M ? m : a.M - 1;           // rows past M are loaded from a valid row and never stored
        xsrc[i] = a.x + (size_t)m * K + xpiece[i] * 8;
    }

    uintx4 wreg[W_DMA ? 1 : WPASS], xreg[X_DMA ? 1 : XPASS], greg[X_DMA ? 1 : XPASS];
    float ssq[XPASS];
#pragma unroll
    for (int i = 0; i < XPASS; ++i) ssq[i] = 0.f;
    const uintx4 zero4 = {0u, 0u, 0u, 0u};

    // K is a multiple of 8, so a 16-byte piece is entirely inside or outside [0,K); with KTAIL the
    // pieces past K are read from k = 0 (valid memory) and replaced by zeros.
    auto load_w = [&](int kt, int buf) {          // DMA: lands in stage buf; else: into wreg
#pragma unroll
        for (int i = 0; i < WPASS; ++i) {
            if (W_DMA) {
                dma16(wsrc[i] + kt * GK, smem + buf * STAGE + (wv * WPASS + i) * 64);
            } else {
                const int piece = (wunit[i] & 7) ^ ((((wunit[i] >> 3) >> 1) & 7) ^ (((wunit[i] >> 3) & 1) << 2));
                const bool kok = kt * GK + piece * 8 < K;
                uintx4 v = *reinterpret_cast<const uintx4*>(wsrc[i] + (kok ? kt * GK : -piece * 8));
                wreg[i] = kok ? v : zero4;
            }
        }
    };
    auto load_x = [&](int kt, int buf) {
#pragma unroll
        for (int i = 0; i < XPASS; ++i) {
            if (X_DMA) {
                dma16(xsrc[i] + kt * GK, smem + buf * STAGE + BN * GPIECES + (wv * XPASS + i) * 64);
            } else {
                const bool kok = !KTAIL || kt * GK + xpiece[i] * 8 < K;
                uintx4 v = *reinterpret_cast<const uintx4*>(xsrc[i] + (kok ? kt * GK : -xpiece[i] * 8));
                xreg[i] = kok ? v : zero4;
                if (EPI == EPI_RMSNORM) {
                    uintx4 g = *reinterpret_cast<const uintx4*>(a.gamma + (kok ? kt * GK + xpiece[i] * 8 : 0));
                    greg[i] = g;
                }
            }
        }
    };
    auto store_w = [&](int buf) {                 // VGPR path only
        if (!W_DMA) {
#pragma unroll
            for (int i = 0; i < WPASS; ++i) smem[buf * STAGE + wunit[i]] = wreg[i];
        }
    };
    auto store_x = [&](int buf) {
        if (!X_DMA) {
#pragma unroll
            for (int i = 0; i < XPASS; ++i) {
                uintx4 xv = xreg[i];
                if (EPI == EPI_RMSNORM) {
                    half8 xh = __builtin_bit_cast(half8, xv);
                    half8 gh = __builtin_bit_cast(half8, greg[i]);
#pragma unroll
                    for (int e = 0; e < 8; ++e) { float f = (float)xh[e]; ssq[i] = __builtin_fmaf(f, f, ssq[i]); }
                    half8 pr = xh * gh;
                    xv = __builtin_bit_cast(uintx4, pr);
                }
                smem[buf * STAGE + BN * GPIECES + xunit[i]] = xv;
            }
        }
    };

    floatx16 acc[TN][TM];
#pragma unroll
    for (int i = 0; i < TN; ++i)
#pragma unroll
        for (int j = 0; j < TM; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    const int lr = lane & 31, lg = lane >> 5;
    half8 wa[2][TN], xb[2][TM];
    auto frags = [&](int buf, int kk, int fs) {
#pragma unroll
        for (int tn = 0; tn < TN; ++tn)
            wa[fs][tn] = __builtin_bit_cast(half8, smem[buf * STAGE + swz(wn * (BN / WN) + tn * 32 + lr, 2 * kk + lg)]);
#pragma unroll
        for (int tm = 0; tm < TM; ++tm)
            xb[fs][tm] = __builtin_bit_cast(half8, smem[buf * STAGE + BN * GPIECES + swz(wm * (BM / WM) + tm * 32 + lr, 2 * kk + lg)]);
    };
    auto mfmas = [&](int fs) {
#pragma unroll
        for (int tn = 0; tn < TN; ++tn)
#pragma unroll
            for (int tm = 0; tm < TM; ++tm)
                acc[tn][tm] = __builtin_amdgcn_mfma_f32_32x32x16_f16(wa[fs][tn], xb[fs][tm], acc[tn][tm], 0, 0, 0);
    };
    // pair each LDS read of the next k-step with one MFMA of the current one
    auto interleave = [&]() {
#pragma unroll
        for (int i = 0; i < TN + TM; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
        __builtin_amdgcn_sched_group_barrier(0x008, TN * TM - (TN + TM), 0);
    };

    // ---- prologue: tiles 0 and 1 into stages 0 and 1; VGPR-path operands run one tile further ahead
    load_w(0, 0); load_x(0, 0);
    store_w(0); store_x(0);
    if (ktiles > 1) {
        load_w(1, 1); load_x(1, 1);
        store_w(1); store_x(1);
    }
    if (ktiles > 2) {
        if (!W_DMA) load_w(2, 0);
        if (!X_DMA) load_x(2, 0);
    }
    __syncthreads();
    frags(0, 0, 0);

    for (int kt = 0; kt < ktiles; ++kt) {
        const int buf = kt & 1;
#pragma unroll
        for (int kk = 0; kk < GK / 16 - 1; ++kk) {
            frags(buf, kk + 1, (kk + 1) & 1);
            mfmas(kk & 1);
            interleave();
        }
        // every read of stage buf has been issued; after the barrier the stage is free and tile kt+1
        // (other stage) is complete.  The direct-to-LDS loads of tile kt+1 were issued one iteration
        // ago; the compiler does not carry them across the loop edge, so wait for them here.
        if (W_DMA || X_DMA) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        if (kt + 2 < ktiles) {
            if (W_DMA) load_w(kt + 2, buf); else store_w(buf);
            if (X_DMA) load_x(kt + 2, buf); else store_x(buf);
            if (kt + 3 < ktiles) {
                if (!W_DMA) load_w(kt + 3, buf);
                if (!X_DMA) load_x(kt + 3, buf);
            }
        }
        if (kt + 1 < ktiles) frags(buf ^ 1, 0, 0);
        mfmas((GK / 16 - 1) & 1);
    }

    if (EPI == EPI_RMSNORM) {
#pragma unroll
        for (int i = 0; i < XPASS; ++i) {
            float v = ssq[i];
            v += __shfl_xor(v, 1);
            v += __shfl_xor(v, 2);
            v += __shfl_xor(v, 4);
            if (slot == 0) s_r[xunit[i] >> 3] = 1.0f / __builtin_sqrtf(v / (float)K + a.eps);
        }
        __syncthreads();
    }

    // ---- epilogue ------------------------------------------------------------
#pragma unroll
    for (int tm = 0; tm < TM; ++tm) {
        const int ml = wm * (BM / WM) + tm * 32 + lr;
        const int m = tile_m * BM + ml;
        if (m >= a.M) continue;
        float scale = 1.0f;
        if (EPI == EPI_RMSNORM) scale = s_r[ml];
#pragma unroll
        for (int tn = 0; tn < TN; ++tn) {
            if (EPI == EPI_SWIGLU) {
#pragma unroll
                for (int aa = 0; aa < 4; aa += 2) {
                    const int v = wn * (BN / WN) + tn * 32 + 8 * aa;
                    const int j = tile_n * JPT + (v >> 4) * 8 + 4 * lg;
                    half4 hv;
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        const float g = acc[tn][tm][4 * aa + c], u = acc[tn][tm][4 * (aa + 1) + c];
                        hv[c] = (_Float16)(g / (1.0f + __expf(-g)) * u);
                    }
                    if (j + 3 < a.N && (a.ldo & 3) == 0) {
                        *reinterpret_cast<half4*>(a.out + (size_t)m * a.ldo + j) = hv;
                    } else {
#pragma unroll
                        for (int c = 0; c < 4; ++c)
                            if (j + c < a.N) a.out[(size_t)m * a.ldo + j + c] = __builtin_bit_cast(uint16_t, hv[c]);
                    }
                }
            } else {
#pragma unroll
                for (int aa = 0; aa < 4; ++aa) {
                    const int n = tile_n * BN + wn * (BN / WN) + tn * 32 + 8 * aa + 4 * lg;
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

template <int BN, int BM, int WN, int WM>
hipError_t launch_cfg(const GemmArgs& a, int epilogue, hipStream_t stream)
{
    const int per_tile = (epilogue == EPI_SWIGLU) ? BN / 2 : BN;
    const int tiles_n = (a.N + per_tile - 1) / per_tile;
    const int tiles_m = (a.M + BM - 1) / BM;
    const size_t lds = (size_t)2 * (BN + BM) * GPIECES * sizeof(uintx4);
    dim3 g((unsigned)((size_t)tiles_n * tiles_m)), b(64 * WN * WM);
#define THI_LAUNCH_K(E, KT)                                                                                        \
    do {                                                                                                     \
        auto kern = gemm_tile<BN, BM, WN, WM, E, KT>;                                                            \
        static bool attr_set = false;                                                                        \
        if (!attr_set) {                                                                                     \
            (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kern),                                   \
                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);                 \
            attr_set = true;                                                                                 \
        }                                                                                                    \
        hipLaunchKernelGGL(kern, g, b, lds, stream, a, tiles_n, tiles_m);                                    \
    } while (0)
#define THI_LAUNCH(E)                                                                                        \
    do {                                                                                                     \
        if (a.K % GK) THI_LAUNCH_K(E, true);                                                                 \
        else THI_LAUNCH_K(E, false);                                                                         \
    } while (0)
    switch (epilogue) {
    case EPI_PLAIN: THI_LAUNCH(EPI_PLAIN); break;
    case EPI_RMSNORM: THI_LAUNCH(EPI_RMSNORM); break;
    default: THI_LAUNCH(EPI_SWIGLU); break;
    }
#undef THI_LAUNCH
#undef THI_LAUNCH_K
    return hipGetLastError();
}

}  // namespace

hipError_t launch_gemm(const GemmArgs& a, int epilogue, int num_cus, hipStream_t stream)
{
    static int dbg_cfg = getenv("THI_DBG_GEMM") ? atoi(getenv("THI_DBG_GEMM")) : 0;
    (void)num_cus;
    int cfg = dbg_cfg;
    if (cfg == 0) cfg = (a.M >= 512) ? 1 : 3;
    switch (cfg) {
    case 1: return launch_cfg<256, 256, 4, 2>(a, epilogue, stream);
    case 2: return launch_cfg<256, 256, 2, 4>(a, epilogue, stream);
    case 4: return launch_cfg<256, 128, 4, 2>(a, epilogue, stream);
    case 5: return launch_cfg<128, 256, 2, 4>(a, epilogue, stream);
    default: return launch_cfg<128, 128, 2, 2>(a, epilogue, stream);
    }
}

}  // namespace thi
