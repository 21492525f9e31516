// Weight-streaming skinny GEMM for decode (M <= 32 tokens per launch) on gfx950.
//
// The paper's small-M rule (Sec. III-B.2: broadcast X, split the work along N)
// is kept in spirit -- every workgroup sees the whole activation slice it needs
// and owns a slice of the weights -- but the partition is made for an HBM-bound
// GPU: the weight matrix is cut into work units of 128 rows x 256 k, the units
// are numbered tile-major and dealt out in equal contiguous shares to a fixed
// number of workgroups ("stream-K"), so every CU streams the same number of
// bytes whatever N and K are.  A tile whose k range is shared by several
// workgroups is finished by the one that owns its first k chunk; it adds the
// partial tiles of the others in workgroup order, so results are reproducible.
//
// Per unit and wave: 16 weight rows x 256 k are fetched with fully coalesced
// 16-byte loads (16 lanes cover 256 contiguous bytes of one row), passed through
// a wave-private LDS buffer to reach the MFMA operand layout, and multiplied
// against the activation slice that the workgroup staged in LDS already in
// operand order.  Products are fp16 x fp16 accumulated in fp32 by
// v_mfma_f32_16x16x32_f16 (Sec. III-B.4: fp16 storage, fp32 accumulation).
//
// Fused low-density operators (Sec. III-C.1):
//   RMSNorm  : x*gamma is formed while the slice is staged, sum x^2 is
//              accumulated on the side, the accumulator is scaled by
//              1/sqrt(mean + eps) before the store  (rmsnorm(x) W^T =
//              r * ((x*gamma) W^T));
//   SwiGLU   : a tile holds gate rows and the matching up rows so that one lane
//              ends up with g and u of the same (token, j); silu(g)*u is applied
//              to the fp32 accumulators before the fp16 store.
#include "thi_internal.h"

#include <type_traits>

namespace thi {

namespace {

// Device-scope (sc1) 16-byte accesses for the hand-over slots: write-through stores, loads that see
// other workgroups' stores.  They are not atomic as a whole (a reader can see a store half landed),
// so they are only used on data that a flag has announced.
__device__ __forceinline__ void store_device_x4(unsigned* p, uintx4 v) {
    asm volatile("global_store_dwordx4 %0, %1, off sc1" ::"v"(p), "v"(v) : "memory");
}
// Four (MT = 1) or eight (MT = 2) such loads and the wait for them in ONE statement: the registers
// are written asynchronously, so the compiler must not see them before the wait has passed.
// p0..p3: a lane's word group in four slots; with MT = 2 the second token tile lies 1024 bytes on.
template <int MT>
__device__ __forceinline__ void load_device_x4_batch(const unsigned* p0, const unsigned* p1, const unsigned* p2,
                                                     const unsigned* p3, uintx4 (&v)[4][MT])
{
    if constexpr (MT == 1) {
        asm volatile(
            "global_load_dwordx4 %0, %4, off sc1\n\t"
            "global_load_dwordx4 %1, %5, off sc1\n\t"
            "global_load_dwordx4 %2, %6, off sc1\n\t"
            "global_load_dwordx4 %3, %7, off sc1\n\t"
            "s_waitcnt vmcnt(0)"
            : "=&v"(v[0][0]), "=&v"(v[1][0]), "=&v"(v[2][0]), "=&v"(v[3][0])
            : "v"(p0), "v"(p1), "v"(p2), "v"(p3)
            : "memory");
    } else {
        asm volatile(
            "global_load_dwordx4 %0, %8, off sc1\n\t"
            "global_load_dwordx4 %1, %8, off offset:1024 sc1\n\t"
            "global_load_dwordx4 %2, %9, off sc1\n\t"
            "global_load_dwordx4 %3, %9, off offset:1024 sc1\n\t"
            "global_load_dwordx4 %4, %10, off sc1\n\t"
            "global_load_dwordx4 %5, %10, off offset:1024 sc1\n\t"
            "global_load_dwordx4 %6, %11, off sc1\n\t"
            "global_load_dwordx4 %7, %11, off offset:1024 sc1\n\t"
            "s_waitcnt vmcnt(0)"
            : "=&v"(v[0][0]), "=&v"(v[0][1]), "=&v"(v[1][0]), "=&v"(v[1][1]), "=&v"(v[2][0]), "=&v"(v[2][1]),
              "=&v"(v[3][0]), "=&v"(v[3][1])
            : "v"(p0), "v"(p1), "v"(p2), "v"(p3)
            : "memory");
    }
}

// U work units are dealt to G workgroups in contiguous shares: the first `rem`
// workgroups take q+1 units, the others q (q = U / G, rem = U % G).
struct Deal {
    int q, rem;
    __device__ __forceinline__ int begin(int w) const { return w * q + (w < rem ? w : rem); }
    __device__ __forceinline__ int owner(int u) const {
        const int edge = rem * (q + 1);
        return u < edge ? u / (q + 1) : rem + (u - edge) / q;
    }
};

template <int MT>
struct UnitRegs {
    uintx4 w[8];      // 16 rows x 256 k of weights: [phase*4 + jj]
    uintx4 x[MT];     // activation pieces this thread stages
    uintx4 g;         // gamma piece (RMSNorm only)
};

template <int MT, int EPI>
__global__ __launch_bounds__(SK_THREADS) void skinny_streamk(const uint16_t* x_, const uint16_t* w0_, const uint16_t* w1_,
                                                             int M_, int N_, int K_, int tiles_, int kchunks_, SkinnyArgs a)
{
    // The operands the first loads need come as leading scalar arguments: the hardware preloads those
    // into registers at wave launch, so the first weight request does not wait for an argument fetch.
    a.x = x_; a.w0 = w0_; a.w1 = w1_; a.M = M_; a.N = N_; a.K = K_; a.tiles = tiles_; a.kchunks = kchunks_;
    __shared__ uintx4 xs[2][8 * MT * 64];          // staged activations, MFMA B-operand order
    __shared__ uintx4 wt[SK_WAVES][WT_UNITS];      // wave-private transposition buffers
    constexpr int TOK = MT == 1 ? 32 : 16 * MT;    // token slots of the per-token sums (a single tile is padded to 32)
    __shared__ float s_red[SK_WAVES][TOK];
    __shared__ float s_ssq[TOK];
    __shared__ unsigned s_flag;
    static_assert(MT >= 1 && MT <= SK_MAX_MT, "token tiles per launch");

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wv = tid >> 6;
    const int G = gridDim.x;
    const int wg = blockIdx.x;
    const int kch = a.kchunks;
    const int U = a.tiles * kch;
    const Deal deal{U / G, U % G};
    const int u_begin = deal.begin(wg);
    const int u_end = deal.begin(wg + 1);
    if (u_begin >= u_end) return;

    const int K = a.K;
    // staging role: this wave stages k-step `wv` (32 k) of each unit; lane -> (token c, k-group g)
    const int st_c = lane >> 2, st_g = lane & 3;
    // weight-load role: load jj of a phase covers MFMA rows 4*jj + lane/16, piece lane%16
    const int ld_i = lane >> 4, ld_p = lane & 15;

    // ---- issue the global loads of one unit --------------------------------
    // Every load is unconditional (no control flow around it, so the hardware wait counters can be
    // reasoned about exactly): addresses that would fall outside the matrix are redirected to a valid
    // element of the same row and the value is replaced by zero when the unit is consumed.
    auto issue = [&](int u, UnitRegs<MT>& r) {
        const int t = u / kch;
        const int k0 = (u - t * kch) * SK_KC;
        // weights
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
            const uint16_t* base;
            if (is_swiglu(EPI)) {
                int j = t * 64 + wv * 8 + 2 * jj + (ld_i & 1);
                j = j < a.N ? j : a.N - 1;
                base = ((ld_i >> 1) ? a.w1 : a.w0) + (size_t)j * K;
            } else {
                int n = t * SK_ROWS + wv * 16 + 4 * jj + ld_i;
                n = n < a.N ? n : a.N - 1;
                base = a.w0 + (size_t)n * K;
            }
#pragma unroll
            for (int ph = 0; ph < 2; ++ph) {
                const int k = k0 + ph * 128 + ld_p * 8;
                r.w[ph * 4 + jj] = ld_stream(base + (k < K ? k : 0));
            }
        }
        // activations (+ gamma)
        const int kx = k0 + wv * 32 + st_g * 8;
        const int kxc = kx < K ? kx : 0;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            const int m = mt * 16 + st_c;
            r.x[mt] = ld_cached(a.x + (size_t)(m < a.M ? m : a.M - 1) * K + kxc);
        }
        if (is_rms(EPI)) r.g = ld_cached(a.gamma + kxc);
    };
    // zero what `issue` loaded from a redirected address
    auto mask_unit = [&](int u, UnitRegs<MT>& r) {
        const uintx4 zero4 = {0u, 0u, 0u, 0u};
        const int t = u / kch;
        const int k0 = (u - t * kch) * SK_KC;
        if (k0 + SK_KC > K) {
#pragma unroll
            for (int ph = 0; ph < 2; ++ph)
#pragma unroll
                for (int jj = 0; jj < 4; ++jj)
                    if (k0 + ph * 128 + ld_p * 8 >= K) r.w[ph * 4 + jj] = zero4;
        }
        const bool kok = k0 + wv * 32 + st_g * 8 < K;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
            if (!kok || mt * 16 + st_c >= a.M) r.x[mt] = zero4;
        if (is_rms(EPI) && !kok) r.g = zero4;
    };

    floatx4 acc[MT];
    float ssq[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) { acc[mt] = floatx4{0.f, 0.f, 0.f, 0.f}; ssq[mt] = 0.f; }

    UnitRegs<MT> nxt;
    issue(u_begin, nxt);
    int run_start = u_begin;         // first unit of the current tile run
    int buf = 0;

    // One unit.  HAS_NEXT is a compile-time fact so that the prefetch sits in straight-line code: the
    // wait for the current unit's loads then leaves exactly the prefetched unit's loads in flight.
    auto step = [&](int u, auto has_next) {
        UnitRegs<MT> cur = nxt;
        if constexpr (decltype(has_next)::value) issue(u + 1, nxt);
        mask_unit(u, cur);

        const int t = u / kch;
        // ---- stage activations (apply gamma, accumulate sum of squares) -----
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            uintx4 xv = cur.x[mt];
            if (is_rms(EPI)) {
                half8 xh = __builtin_bit_cast(half8, xv);
                half8 gh = __builtin_bit_cast(half8, cur.g);
#pragma unroll
                for (int e = 0; e < 8; ++e) { float f = (float)xh[e]; ssq[mt] = __builtin_fmaf(f, f, ssq[mt]); }
                half8 p = xh * gh;       // one rounding: the fp16 product of two fp16 values
                xv = __builtin_bit_cast(uintx4, p);
            }
            xs[buf][(wv * MT + mt) * 64 + st_g * 16 + st_c] = xv;
        }
        __syncthreads();

        // ---- weights: two phases of 16 rows x 128 k through the wave buffer --
#pragma unroll
        for (int ph = 0; ph < 2; ++ph) {
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int jj = 0; jj < 4; ++jj)
                wt[wv][(4 * jj + ld_i) * WT_STRIDE + ld_p] = cur.w[ph * 4 + jj];
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                half8 wa = __builtin_bit_cast(half8, wt[wv][(lane & 15) * WT_STRIDE + 4 * s + (lane >> 4)]);
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) {
                    half8 xb = __builtin_bit_cast(half8, xs[buf][((ph * 4 + s) * MT + mt) * 64 + lane]);
                    acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(wa, xb, acc[mt], 0, 0, 0);
                }
            }
        }
        buf ^= 1;

        // ---- end of this workgroup's run over tile t? ------------------------
        const bool run_ends = (u + 1 == u_end) || ((u + 1) % kch == 0);
        if (!run_ends) return;

        const int tile_begin = t * kch;
        const bool whole = ((run_start == tile_begin) && (u + 1 == tile_begin + kch));

        // sum of squares of this run, per token (fixed order: lanes, then waves)
        if (is_rms(EPI)) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                float v = ssq[mt];
                v += __shfl_xor(v, 1);
                v += __shfl_xor(v, 2);
                if (st_g == 0) s_red[wv][mt * 16 + st_c] = v;
            }
            if (MT == 1 && st_g == 0) s_red[wv][16 + st_c] = 0.f;
            __syncthreads();
            if (tid < TOK) {
                float v = 0.f;
#pragma unroll
                for (int i = 0; i < SK_WAVES; ++i) v += s_red[i][tid];
                s_ssq[tid] = v;
            }
            __syncthreads();
        }

        // ---- a tile shared by several workgroups ----------------------------------------------
        // Shares are contiguous, so the workgroup that owns the tile's first k chunk (w_first)
        // reaches the tile at the END of its share, every other contributor at the START of its
        // own.  The others hand in their partial tile -- device-scope stores into their hand-over
        // slot, then a flag once the stores are acknowledged -- and move on; w_first keeps its part
        // in registers, waits for the flags (normally long set) and adds the partials in workgroup
        // order.  A lane's four accumulator registers of a token tile travel as one 16-byte group:
        // the hand-over is bound by the number of device-scope memory instructions, not by bytes.
        // (The data is only read after the flag: a 16-byte access is not atomic as a whole.)
        bool finish = whole;
        if (!whole) {
            const int w_first = deal.owner(tile_begin);
            const int w_last = deal.owner(tile_begin + kch - 1);
            const bool lane_ssq = is_rms(EPI) && tid < TOK;
            const int own = (wv * SK_MAX_MT * 64 + lane) * 4;       // this lane's word group (token tile 0) in a slot
            if (wg != w_first) {
                unsigned* ps = a.handover + (size_t)wg * SK_SLOT_WORDS;
                // only the lanes that hold a real token (column c = lane % 16 of token tile mt) take part
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
                    if (mt * 16 + (lane & 15) < a.M)
                        store_device_x4(ps + own + mt * 256, __builtin_bit_cast(uintx4, acc[mt]));
                if (lane_ssq)
                    __hip_atomic_store(ps + SK_SLOT_SSQ + tid, __builtin_bit_cast(unsigned, s_ssq[tid]), __ATOMIC_RELAXED,
                                       __HIP_MEMORY_SCOPE_AGENT);
                // every thread waits until its write-through stores are acknowledged (a workgroup-scope
                // fence alone does not wait for that); only then may the flag go up
                asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
                __syncthreads();
                if (tid == 0 && !a.withhold_flags)
                    __hip_atomic_store(a.counters + wg, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            } else {
                if (wv == 0) {
                    // wave 0 polls the flags, one contributor per lane, so the round trips overlap
                    unsigned ok = 1u;
                    for (int wc0 = w_first + 1; wc0 <= w_last; wc0 += 64) {
                        const int wc = wc0 + lane;
                        const bool mine = wc <= w_last;
                        unsigned spins = 0;
                        bool seen = !mine;
                        while (true) {
                            if (!seen)
                                seen = __hip_atomic_load(a.counters + wc, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u;
                            if (__builtin_amdgcn_ballot_w64(!seen) == 0ull) break;
                            __builtin_amdgcn_s_sleep(1);
                            if (++spins > a.spin_limit) { ok = 0u; break; }      // bounded: every wave exits
                        }
                        if (mine && seen)
                            __hip_atomic_store(a.counters + wc, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    }
                    if (lane == 0) {
                        if (!ok) __hip_atomic_store(a.counters + (WS_MAX_COUNTERS - 1), 1u, __ATOMIC_RELAXED,
                                                    __HIP_MEMORY_SCOPE_AGENT);
                        s_flag = ok;
                    }
                }
                __syncthreads();
                finish = (s_flag != 0u);
                if (finish) {
                    float sq = lane_ssq ? s_ssq[tid] : 0.f;
                    // four contributors at a time so that the round trips overlap; every lane loads (from
                    // the last contributor's slot if there is no b-th one) and discards what is not its own
                    for (int wc0 = w_first + 1; wc0 <= w_last; wc0 += 4) {
                        uintx4 pv[4][MT];
                        unsigned ps4[4];
                        const unsigned* cs[4];
#pragma unroll
                        for (int b = 0; b < 4; ++b) {
                            const int wc = wc0 + b;
                            cs[b] = a.handover + (size_t)(wc <= w_last ? wc : w_last) * SK_SLOT_WORDS;
                            ps4[b] = (wc <= w_last && lane_ssq)
                                ? __hip_atomic_load(cs[b] + SK_SLOT_SSQ + tid, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)
                                : 0u;      // +0.0f
                        }
                        if constexpr (MT <= 2) {
                            load_device_x4_batch<MT>(cs[0] + own, cs[1] + own, cs[2] + own, cs[3] + own, pv);
                        } else {      // token tiles 0, 1, then the others: two batches
                            uintx4 lo[4][2], hi[4][MT - 2];
                            load_device_x4_batch<2>(cs[0] + own, cs[1] + own, cs[2] + own, cs[3] + own, lo);
                            load_device_x4_batch<MT - 2>(cs[0] + own + 512, cs[1] + own + 512, cs[2] + own + 512,
                                                         cs[3] + own + 512, hi);
#pragma unroll
                            for (int b = 0; b < 4; ++b)
#pragma unroll
                                for (int mt = 0; mt < MT; ++mt) pv[b][mt] = mt < 2 ? lo[b][mt < 2 ? mt : 0] : hi[b][mt >= 2 ? mt - 2 : 0];
                        }
#pragma unroll
                        for (int b = 0; b < 4; ++b) {
                            if (wc0 + b > w_last) continue;
#pragma unroll
                            for (int mt = 0; mt < MT; ++mt)
                                if (mt * 16 + (lane & 15) < a.M) {
#pragma unroll
                                    for (int i = 0; i < 4; ++i) {
                                        const unsigned word = pv[b][mt][i];      // (a bit_cast straight from a vector element miscompiles)
                                        acc[mt][i] += __builtin_bit_cast(float, word);
                                    }
                                }
                            if (lane_ssq) sq += __builtin_bit_cast(float, ps4[b]);
                        }
                    }
                    if (is_rms(EPI)) {
                        __syncthreads();
                        if (tid < TOK) s_ssq[tid] = sq;
                        __syncthreads();
                    }
                }
            }
        }

        if (finish) {
            const int q = lane >> 4, c = lane & 15;
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                const int m = mt * 16 + c;
                if (m >= a.M) continue;
                if (is_swiglu(EPI)) {
                    const int j = t * 64 + wv * 8 + 2 * q;
                    float scale = 1.0f;      // RMSNorm in front: gate and up both carry the 1/rms factor
                    if (is_rms(EPI)) scale = 1.0f / __builtin_sqrtf(s_ssq[m] / (float)K + a.eps);
#pragma unroll
                    for (int i = 0; i < 2; ++i)
                        if (j + i < a.N)
                            a.out[(size_t)m * a.ldo + j + i] =
                                to_half_bits(silu_mul(acc[mt][i] * scale, acc[mt][i + 2] * scale));
                } else {
                    float scale = 1.0f;
                    if (is_rms(EPI)) scale = 1.0f / __builtin_sqrtf(s_ssq[m] / (float)K + a.eps);
                    const int n = t * SK_ROWS + wv * 16 + 4 * q;
                    float v[4];
#pragma unroll
                    for (int i = 0; i < 4; ++i) v[i] = acc[mt][i] * scale;
                    if (EPI == EPI_RMSNORM_ROPE) {       // the lane holds two complete pairs of one token
                        const int mp = a.rope.pos[m];
                        rope_pair(a.rope, mp, n, v[0], v[1]);
                        rope_pair(a.rope, mp, n + 2, v[2], v[3]);
                    }
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        if (n + i < a.N) {
                            if (a.residual) v[i] += half_bits_to_float(a.residual[(size_t)m * a.ldo + n + i]);
                            a.out[(size_t)m * a.ldo + n + i] = to_half_bits(v[i]);
                        }
                }
            }
        }

        // start the next run
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) { acc[mt] = floatx4{0.f, 0.f, 0.f, 0.f}; ssq[mt] = 0.f; }
        run_start = u + 1;
        // s_red / s_ssq / s_flag are rewritten only after the next __syncthreads of the unit loop
    };
    for (int u = u_begin; u + 1 < u_end; ++u) step(u, std::true_type{});
    step(u_end - 1, std::false_type{});
}

template <int MT>
hipError_t launch_mt(const SkinnyArgs& a, int epilogue, int grid, hipStream_t stream)
{
    dim3 g(grid), b(SK_THREADS);
    switch (epilogue) {
    case EPI_PLAIN: hipLaunchKernelGGL((skinny_streamk<MT, EPI_PLAIN>), g, b, 0, stream, a.x, a.w0, a.w1, a.M, a.N, a.K, a.tiles, a.kchunks, a); break;
    case EPI_RMSNORM: hipLaunchKernelGGL((skinny_streamk<MT, EPI_RMSNORM>), g, b, 0, stream, a.x, a.w0, a.w1, a.M, a.N, a.K, a.tiles, a.kchunks, a); break;
    case EPI_RMSNORM_ROPE: hipLaunchKernelGGL((skinny_streamk<MT, EPI_RMSNORM_ROPE>), g, b, 0, stream, a.x, a.w0, a.w1, a.M, a.N, a.K, a.tiles, a.kchunks, a); break;
    case EPI_RMSNORM_SWIGLU: hipLaunchKernelGGL((skinny_streamk<MT, EPI_RMSNORM_SWIGLU>), g, b, 0, stream, a.x, a.w0, a.w1, a.M, a.N, a.K, a.tiles, a.kchunks, a); break;
    default: hipLaunchKernelGGL((skinny_streamk<MT, EPI_SWIGLU>), g, b, 0, stream, a.x, a.w0, a.w1, a.M, a.N, a.K, a.tiles, a.kchunks, a); break;
    }
    return hipGetLastError();
}

__global__ void fill_words_kernel(uint32_t* p, size_t words, uint32_t value)
{
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < words; i += stride) p[i] = value;
}

}  // namespace

hipError_t launch_skinny(const SkinnyArgs& a, int epilogue, int num_cus, hipStream_t stream)
{
    const long U = (long)a.tiles * a.kchunks;
    // one workgroup per CU: fewer, larger shares keep the number of workgroups that share a tile
    // (and so the partial-tile traffic) small; measured faster than two per CU on every shape
    long grid = num_cus;
    if (grid > SK_MAX_GRID) grid = SK_MAX_GRID;
    if (grid > U) grid = U;
    if (a.M <= 16) return launch_mt<1>(a, epilogue, (int)grid, stream);
    if (a.M <= 32) return launch_mt<2>(a, epilogue, (int)grid, stream);
    if (a.M <= 48) return launch_mt<3>(a, epilogue, (int)grid, stream);
    if (a.M <= 16 * SK_MAX_MT) return launch_mt<4>(a, epilogue, (int)grid, stream);
    return hipErrorInvalidValue;
}

hipError_t launch_fill_words(void* ptr, size_t bytes, uint32_t value, hipStream_t stream)
{
    const size_t words = bytes / 4;
    int blocks = (int)((words + 255) / 256);
    if (blocks > 1024) blocks = 1024;
    if (blocks < 1) blocks = 1;
    hipLaunchKernelGGL(fill_words_kernel, dim3(blocks), dim3(256), 0, stream, (uint32_t*)ptr, words, value);
    return hipGetLastError();
}

}  // namespace thi
