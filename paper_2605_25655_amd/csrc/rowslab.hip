// Row-slab decode kernel (M <= 32 tokens per launch) on gfx950: weight streaming with no
// workgroup-to-workgroup hand-over.
//
// The paper's small-M rule (Sec. III-B.2: broadcast X, split the work along N) taken literally:
// a workgroup owns a slab of 16 output features over the WHOLE reduction dimension, so nothing is
// shared between workgroups.  Inside the workgroup the k range is cut into eight contiguous pieces,
// one per wave; a wave streams its 16 rows x (K/8) k of weights in units of 256 k with fully
// coalesced 16-byte loads (one unit ahead of the arithmetic), passes them through a wave-private
// LDS buffer to reach the MFMA operand layout, and takes its slice of the activations from memory
// itself (they stay cache resident: every workgroup reads the same M x K block) -- in operand layout
// up to four tokens, like the weights from five tokens up (XT below).
// The eight partial tiles meet in LDS, are added in wave order (reproducible) and finished by the
// fused epilogue (Sec. III-C.1: RMSNorm scale, rotary embedding, SwiGLU).
//
// Chosen over the stream-K kernel when the slabs divide evenly enough among the compute units:
// there the hand-over between workgroups (several microseconds across the chip) is the larger loss.
#include "thi_internal.h"

#include <mutex>
#include <type_traits>

namespace thi {

namespace {

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef unsigned uintx2 __attribute__((ext_vector_type(2)));

// XT: the activations are loaded the way the weights are (16 lanes cover 256 contiguous bytes of a token
// row) and reach operand layout through the wave's LDS buffer.  From a handful of tokens up this is the
// cheaper way: loaded in operand layout, every lane asks for its own 16 bytes of a different row, which
// costs the vector cache several times the cycles per byte.  With very few tokens most lanes of an
// operand-layout load share an address and the direct load wins.
template <int MT, int EPI, bool XT>
__global__ __launch_bounds__(SK_THREADS) void skinny_rowslab(const uint16_t* x_, const uint16_t* w0_, const uint16_t* w1_,
                                                             const uint16_t* gamma_, int M_, int N_, int K_, int tiles_,
                                                             SkinnyArgs a)
{
    // The operands the first loads need come as leading scalar arguments: the hardware preloads those
    // into registers at wave launch, so the first weight request does not wait for an argument fetch.
    a.x = x_; a.w0 = w0_; a.w1 = w1_; a.gamma = gamma_; a.M = M_; a.N = N_; a.K = K_; a.tiles = tiles_;
    __shared__ uintx4 wt[SK_WAVES][WT_UNITS];          // wave-private transposition buffers
    __shared__ floatx4 s_part[SK_WAVES][MT * 64];      // the waves' partial tiles, a lane's four registers together
    __shared__ float s_red[SK_WAVES][32];
    __shared__ float s_ssq[32];
    extern __shared__ uintx4 s_gamma[];                // RMSNorm: each wave's slice of gamma

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int G = gridDim.x;
    const int K = a.K;

    // this wave's k range: whole groups of 128 k, so that every range starts on a 256-byte boundary of
    // its rows (K >= 1024: every wave has at least one group)
    const int S4 = (K + 127) >> 7;
    const int k_begin = ((wv * S4) >> 3) * 128;
    const int k_stop = (((wv + 1) * S4) >> 3) * 128;
    const int k_end = k_stop < K ? k_stop : K;
    const int nU = (k_end - k_begin + SK_KC - 1) / SK_KC;            // units of 256 k per slab
    const int n_slabs = (a.tiles - (int)blockIdx.x + G - 1) / G;     // slabs of this workgroup
    const int total = n_slabs * nU;

    const int g_pieces = (((S4 >> 3) + 1) * 128) >> 3;               // 16-byte pieces reserved per wave
    // weight-load role: load jj of a phase covers MFMA rows 4*jj + lane/16, piece lane%16
    const int ld_i = lane >> 4, ld_p = lane & 15;
    // operand role: token column c, k group kg
    const int c = lane & 15, kg = lane >> 4;
    const uintx4 zero4 = {0u, 0u, 0u, 0u};

    // row pointers of a slab for this lane's four load rows
    auto row_base = [&](int slab, int jj) -> const uint16_t* {
        const int v = 4 * jj + ld_i;                   // virtual row within the slab
        if (is_swiglu(EPI)) {
            int j = slab * 8 + (v & 7);
            j = j < a.N ? j : a.N - 1;
            return ((v >> 3) ? a.w1 : a.w0) + (size_t)j * K;
        }
        int n = slab * 16 + v;
        n = n < a.N ? n : a.N - 1;
        return a.w0 + (size_t)n * K;
    };
    // Every load is unconditional; one that would leave the wave's k range is redirected to the first
    // piece of the unit (same cache line as a neighbour's load) and zeroed when the unit is consumed.
    // A prefetch past the workgroup's last unit (valid = false) sends every lane to the start of the
    // activations (lines every compute unit has just read: the wait for these loads at the end of the
    // kernel is short): the code stays free of branches around loads, which keeps the hardware wait
    // counters exact.
    auto issue_w = [&](int slab, int uu, bool valid, uintx4 (&w)[8]) {
        const int k0 = k_begin + uu * SK_KC;
        const int k_lim = valid ? k_end : 0;
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
            const uint16_t* base = row_base(slab, jj);
#pragma unroll
            for (int ph = 0; ph < 2; ++ph) {
                const int k = k0 + ph * 128 + ld_p * 8;
                w[ph * 4 + jj] = ld_stream(valid ? base + (k < k_lim ? k : k0) : a.x);
            }
        }
    };

    floatx4 acc[MT];
    float ssq[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) { acc[mt] = floatx4{0.f, 0.f, 0.f, 0.f}; ssq[mt] = 0.f; }

    // one unit of weights is in flight ahead of the one being consumed (two register buffers in rotation;
    // a second unit ahead measured no faster)
    int slab = blockIdx.x, uu = 0;           // the unit being consumed
    int p_slab = blockIdx.x, p_uu = 0;       // the unit last requested
    int requested = 1;
    uintx4 wb0[8], wb1[8];
    // RMSNorm: this wave's slice of gamma goes to LDS once (wave-private: no workgroup barrier).  Its first
    // 64 pieces are requested before the first weights and stored behind them, so that the weights are in
    // flight while gamma arrives (all of gamma for K <= 4096).
    uintx4 g_first = zero4;
    if (is_rms(EPI)) g_first = ld_cached(a.gamma + k_begin + (lane * 8 < k_end - k_begin ? lane * 8 : 0));
    issue_w(p_slab, p_uu, true, wb0);
    if (is_rms(EPI)) {
        if (lane * 8 < k_end - k_begin) s_gamma[wv * g_pieces + lane] = g_first;
        for (int p = lane + 64; p * 8 < k_end - k_begin; p += 64)
            s_gamma[wv * g_pieces + p] = ld_cached(a.gamma + k_begin + p * 8);
        __builtin_amdgcn_wave_barrier();
    }

    auto step = [&](uintx4 (&cur)[8], uintx4 (&pre)[8]) {
        const int k0 = k_begin + uu * SK_KC;
        const bool first_slab = (slab == (int)blockIdx.x);

        // activations (and gamma) of this unit, in operand layout; issued before the prefetch so that
        // waiting for them leaves the prefetched weights in flight
        uintx4 xr[8][MT];
        uintx4 xl[XT ? MT : 1][8];
        if constexpr (XT) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int jj = 0; jj < 4; ++jj) {
                    const int m = mt * 16 + 4 * jj + ld_i;
                    const uint16_t* row = a.x + (size_t)(m < a.M ? m : a.M - 1) * K;
#pragma unroll
                    for (int ph = 0; ph < 2; ++ph) {
                        const int k = k0 + ph * 128 + ld_p * 8;
                        xl[mt][ph * 4 + jj] = ld_cached(row + (k < k_end ? k : k0));
                    }
                }
        } else {
#pragma unroll
            for (int s = 0; s < 8; ++s) {
                const int kx = k0 + s * 32 + kg * 8;
                const int kxc = kx < k_end ? kx : k0;
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) {
                    const int m = mt * 16 + c;
                    xr[s][mt] = ld_cached(a.x + (size_t)(m < a.M ? m : a.M - 1) * K + kxc);
                }
            }
        }
        if (++p_uu == nU) { p_uu = 0; p_slab += G; }
        issue_w(p_slab, p_uu, requested < total, pre);
        ++requested;
        if constexpr (XT) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int ph = 0; ph < 2; ++ph) {
                    __builtin_amdgcn_wave_barrier();
#pragma unroll
                    for (int jj = 0; jj < 4; ++jj) wt[wv][(4 * jj + ld_i) * WT_STRIDE + ld_p] = xl[mt][ph * 4 + jj];
                    __builtin_amdgcn_wave_barrier();
#pragma unroll
                    for (int s4 = 0; s4 < 4; ++s4) xr[ph * 4 + s4][mt] = wt[wv][c * WT_STRIDE + 4 * s4 + kg];
                }
        }

        // zero what came from a redirected address
        if (k0 + SK_KC > k_end) {
#pragma unroll
            for (int ph = 0; ph < 2; ++ph)
#pragma unroll
                for (int jj = 0; jj < 4; ++jj)
                    if (k0 + ph * 128 + ld_p * 8 >= k_end) cur[ph * 4 + jj] = zero4;
        }

#pragma unroll
        for (int ph = 0; ph < 2; ++ph) {
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) wt[wv][(4 * jj + ld_i) * WT_STRIDE + ld_p] = cur[ph * 4 + jj];
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int s4 = 0; s4 < 4; ++s4) {
                const int s = ph * 4 + s4;
                half8 wa = __builtin_bit_cast(half8, wt[wv][c * WT_STRIDE + 4 * s4 + kg]);
                const bool kok = k0 + s * 32 + kg * 8 < k_end;
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) {
                    uintx4 xv = (kok && mt * 16 + c < a.M) ? xr[s][mt] : zero4;
                    if (is_rms(EPI)) {
                        half8 xh = __builtin_bit_cast(half8, xv);
                        half8 gh = __builtin_bit_cast(half8, s_gamma[wv * g_pieces + (((kok ? k0 + s * 32 : k_begin) - k_begin) >> 3) + (kok ? kg : 0)]);
                        if (first_slab) {      // the same x serves every slab: its sum of squares is taken once
#pragma unroll
                            for (int e = 0; e < 8; e += 2) {
                                const half2_t h2 = {xh[e], xh[e + 1]};
                                ssq[mt] = __builtin_amdgcn_fdot2(h2, h2, ssq[mt], false);
                            }
                        }
                        half8 p = xh * gh;       // one rounding: the fp16 product of two fp16 values
                        xv = kok ? __builtin_bit_cast(uintx4, p) : zero4;
                    }
                    acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(wa, __builtin_bit_cast(half8, xv), acc[mt], 0, 0, 0);
                }
            }
        }

        const bool slab_ends = (uu + 1 == nU);
        const int this_slab = slab;
        if (++uu == nU) { uu = 0; slab += G; }
        if (!slab_ends) return;

        // ---- the eight partial tiles meet in LDS ---------------------------------------------------
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            s_part[wv][mt * 64 + lane] = acc[mt];
            if (is_rms(EPI) && first_slab) {
                float v = ssq[mt];
                v += __shfl_xor(v, 16);
                v += __shfl_xor(v, 32);
                if (kg == 0) s_red[wv][mt * 16 + c] = v;
            }
            acc[mt] = floatx4{0.f, 0.f, 0.f, 0.f};
        }
        if (is_rms(EPI) && first_slab && MT == 1 && kg == 0) s_red[wv][16 + c] = 0.f;
        __syncthreads();
        // The first MT waves add the eight partial tiles in wave order (fixed: reproducible) and finish what each of
        // their threads then holds -- four consecutive features of one token (two gate/up pairs after an exchange
        // between the wave's halves for SwiGLU) -- straight from registers.
        if (tid < MT * 64) {
            floatx4 v = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int w = 0; w < SK_WAVES; ++w) v += s_part[w][tid];
            const int l = tid & 63, quad = l >> 4, m = (tid >> 6) * 16 + (l & 15);
            float scale = 1.0f;
            if (is_rms(EPI)) {
                float q = 0.f;
                if (first_slab) {         // kept in s_ssq for the later slabs
#pragma unroll
                    for (int w = 0; w < SK_WAVES; ++w) q += s_red[w][m];
                    if (quad == 0) s_ssq[m] = q;
                } else {
                    q = s_ssq[m];
                }
                scale = 1.0f / __builtin_sqrtf(q / (float)K + a.eps);
            }
            if (is_swiglu(EPI)) {
                // rows 0..7 of a slab are gate rows, 8..15 the matching up rows: lane l holds rows 4*quad..+3, its
                // partner l ^ 32 the rows 8 further on
                floatx4 o;
#pragma unroll
                for (int i = 0; i < 4; ++i) o[i] = __shfl_xor(v[i], 32);
                if (quad < 2 && m < a.M) {
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const int j = this_slab * 8 + 4 * quad + i;
                        if (j < a.N) a.out[(size_t)m * a.ldo + j] = to_half_bits(silu_mul(v[i] * scale, o[i] * scale));
                    }
                }
            } else if (m < a.M) {
                const int n = this_slab * 16 + 4 * quad;
                float y[4];
#pragma unroll
                for (int i = 0; i < 4; i += 2) {      // pairs (n + i, n + i + 1)
                    y[i] = v[i] * scale;
                    y[i + 1] = v[i + 1] * scale;
                    if (EPI == EPI_RMSNORM_ROPE) rope_pair(a.rope, a.rope.pos[m], n + i, y[i], y[i + 1]);
                }
                uint16_t* const dst = a.out + (size_t)m * a.ldo + n;
                if (n + 3 < a.N && (a.ldo & 3) == 0) {
                    // the thread's four features as one 8-byte access (out and residual are 16-byte aligned)
                    if (a.residual) {
                        const uintx2 rv = *reinterpret_cast<const uintx2*>(a.residual + (size_t)m * a.ldo + n);
                        y[0] += half_bits_to_float((uint16_t)(rv[0] & 0xffffu));
                        y[1] += half_bits_to_float((uint16_t)(rv[0] >> 16));
                        y[2] += half_bits_to_float((uint16_t)(rv[1] & 0xffffu));
                        y[3] += half_bits_to_float((uint16_t)(rv[1] >> 16));
                    }
                    uintx2 ov;
                    ov[0] = (unsigned)to_half_bits(y[0]) | ((unsigned)to_half_bits(y[1]) << 16);
                    ov[1] = (unsigned)to_half_bits(y[2]) | ((unsigned)to_half_bits(y[3]) << 16);
                    *reinterpret_cast<uintx2*>(dst) = ov;
                } else {
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        if (n + i < a.N) {
                            float o = y[i];
                            if (a.residual) o += half_bits_to_float(a.residual[(size_t)m * a.ldo + n + i]);
                            dst[i] = to_half_bits(o);
                        }
                }
            }
        }
        // s_part / s_red are written again at the end of the workgroup's next slab: everybody must be done reading
        if (n_slabs > 1) __syncthreads();
    };

    for (int i = 0; i < total; i += 2) {
        step(wb0, wb1);
        if (i + 1 >= total) break;
        step(wb1, wb0);
    }
}

// 16-byte pieces of LDS per wave for its slice of gamma (same arithmetic as in the kernel)
int rowslab_gamma_pieces(int K) { return ((((K + 127) >> 7) >> 3) + 1) * 128 >> 3; }

template <int MT, bool XT>
hipError_t launch_mt(const SkinnyArgs& a, int epilogue, int grid, hipStream_t stream)
{
    dim3 g(grid), b(SK_THREADS);
    const size_t gamma_lds = (size_t)SK_WAVES * rowslab_gamma_pieces(a.K) * sizeof(uintx4);
    static std::once_flag attr_once;    // static + dynamic LDS can pass 64 KiB for large K
    std::call_once(attr_once, [] {
        const int most = (int)((size_t)SK_WAVES * rowslab_gamma_pieces(ROWSLAB_MAX_K) * sizeof(uintx4));
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(skinny_rowslab<MT, EPI_RMSNORM, XT>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, most);
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(skinny_rowslab<MT, EPI_RMSNORM_ROPE, XT>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, most);
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(skinny_rowslab<MT, EPI_RMSNORM_SWIGLU, XT>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, most);
    });
    switch (epilogue) {
    case EPI_PLAIN: hipLaunchKernelGGL((skinny_rowslab<MT, EPI_PLAIN, XT>), g, b, 0, stream, a.x, a.w0, a.w1, a.gamma, a.M, a.N, a.K, a.tiles, a); break;
    case EPI_RMSNORM: hipLaunchKernelGGL((skinny_rowslab<MT, EPI_RMSNORM, XT>), g, b, gamma_lds, stream, a.x, a.w0, a.w1, a.gamma, a.M, a.N, a.K, a.tiles, a); break;
    case EPI_RMSNORM_ROPE: hipLaunchKernelGGL((skinny_rowslab<MT, EPI_RMSNORM_ROPE, XT>), g, b, gamma_lds, stream, a.x, a.w0, a.w1, a.gamma, a.M, a.N, a.K, a.tiles, a); break;
    case EPI_RMSNORM_SWIGLU: hipLaunchKernelGGL((skinny_rowslab<MT, EPI_RMSNORM_SWIGLU, XT>), g, b, gamma_lds, stream, a.x, a.w0, a.w1, a.gamma, a.M, a.N, a.K, a.tiles, a); break;
    default: hipLaunchKernelGGL((skinny_rowslab<MT, EPI_SWIGLU, XT>), g, b, 0, stream, a.x, a.w0, a.w1, a.gamma, a.M, a.N, a.K, a.tiles, a); break;
    }
    return hipGetLastError();
}

}  // namespace

hipError_t launch_rowslab(const SkinnyArgs& a, int epilogue, int num_cus, hipStream_t stream)
{
    if (a.K < 1024 || a.K > ROWSLAB_MAX_K || a.tiles < 1) return hipErrorInvalidValue;
    int grid = num_cus < a.tiles ? num_cus : a.tiles;
    if (a.M <= 4) return launch_mt<1, false>(a, epilogue, grid, stream);
    if (a.M <= 16) return launch_mt<1, true>(a, epilogue, grid, stream);
    return launch_mt<2, true>(a, epilogue, grid, stream);
}

}  // namespace thi
