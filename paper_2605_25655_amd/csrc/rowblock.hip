// Row-block decode kernel (M <= 32 tokens per launch) on gfx950: the row-slab kernel's decomposition
// with several slabs in flight per workgroup.
//
// The paper's small-M rule (Sec. III-B.2: broadcast X, split the work along N): the output features
// are dealt to the workgroups in equal contiguous blocks (one workgroup per compute unit, so every
// compute unit streams the same number of weight bytes whatever N is), each block over the whole
// reduction dimension: nothing is handed from workgroup to workgroup.  A block is T tiles of 16 weight rows
// (rows past the block's end are masked).  Inside the workgroup the k range is cut into eight
// contiguous pieces, one per wave; per unit of 256 k a wave loads its slice of the activations ONCE
// (coalesced, then through its LDS buffer into MFMA operand layout) and uses it for all T tiles, so the
// activation traffic through the vector cache per weight byte is 1/T of the one-slab kernel's (what
// limits that kernel from M = 16 up).
// Weights stream as in the row-slab kernel: coalesced 16-byte loads one tile-step ahead of the
// arithmetic, a wave-private LDS buffer to reach operand layout.  The eight partial tiles meet in
// LDS, are added in wave order (reproducible) and finished by the fused epilogue (Sec. III-C.1:
// RMSNorm scale, rotary embedding, SwiGLU, residual).  T is the block's tile count when that is at most
// six; larger blocks take several passes over K with their tiles dealt evenly to the passes.
//
// Where N is so small that a block is a single tile (N = hidden size: the O and down projections), the
// activations would cost the vector cache twice the weights' bytes at 32 tokens.  The SPLIT variant (plain
// kind) then lets S workgroups share a block of S x as many rows, each over 1/S of K: a slice of x serves
// S x as many tiles.  The S sums of a block meet through hand-over slots in the workspace; the workgroup
// that arrives last (a counter per block, reset by that workgroup) adds them in share order, so the
// result does not depend on the order of arrival, and nobody waits for anybody.
#include "thi_internal.h"

#include <mutex>
#include <type_traits>

namespace thi {

namespace {

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef unsigned uintx2 __attribute__((ext_vector_type(2)));

// tiles per reduction round.  With RMSNorm in front a slice of gamma per wave lives in LDS as well (up to 66 KiB):
// all tiles in one round while the partial tiles fit 48 KiB (static LDS <= 85 KiB), else half a pass.
// Without gamma (plain and SwiGLU kinds) all tiles go in one round (up to 131 KiB of static LDS: one
// workgroup per compute unit either way).
template <int T, int MT, int EPI, bool SPLIT>
constexpr int reduction_tiles() { return (SPLIT || !is_rms(EPI)) ? T : (T * MT <= 6 && T <= 5) ? T : (T + 1) / 2; }

// The kernel's static LDS (one object per workgroup; the single-launch MLP overlays the objects of its two phases).
template <int T, int MT, int EPI, bool SPLIT>
struct RowBlockShared {
    uintx4 wt[SK_WAVES][WT_UNITS];                              // wave-private transposition buffers
    floatx4 s_part[SK_WAVES][reduction_tiles<T, MT, EPI, SPLIT>()][MT * 64]; // the waves' partial tiles, a lane's four registers together
    float s_red[SK_WAVES][32];
    float s_ssq[32];
    unsigned s_last;                                            // SPLIT: this workgroup closes its row block
};

// The whole kernel as a function of (block id, grid size), so that one launch can run two of them back to back.
// DEVOUT: the outputs are stored with device-scope (write-through) stores, for a consumer that reads them later in
// the SAME launch; pre(): called once, when the first weights have been requested and before the first activation
// load (the single-launch MLP waits there for the whole of h).
template <int T, int MT, int EPI, bool SPLIT, bool DEVOUT, typename Pre>
__device__ __forceinline__ void rowblock_body(SkinnyArgs a, const int per_wg, const int block_id, const int grid,
                                              RowBlockShared<T, MT, EPI, SPLIT>& sm, uintx4* s_gamma, Pre pre)
{
    static_assert(T >= 2 && T <= 6, "tiles in flight");
    constexpr int RT = reduction_tiles<T, MT, EPI, SPLIT>();
    constexpr int OUT_PER_TILE = is_swiglu(EPI) ? 8 : 16;
    auto& wt = sm.wt;
    auto& s_part = sm.s_part;
    auto& s_red = sm.s_red;
    auto& s_ssq = sm.s_ssq;
    unsigned& s_last = sm.s_last;
    static_assert(!SPLIT || EPI == EPI_PLAIN, "the reduction dimension is only shared for the plain kind");
    auto put = [&](uint16_t* p, uint16_t bits) __attribute__((always_inline)) {
        if constexpr (DEVOUT) __hip_atomic_store(p, bits, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        else *p = bits;
    };

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int K = a.K;

    // this workgroup's block of outputs (rows of W; gate/up row pairs for SwiGLU); SPLIT: S workgroups
    // share a block, each with 1/S of the reduction dimension (S travels in a.kchunks)
    const int S = SPLIT ? a.kchunks : 1;
    const int blocks = SPLIT ? grid / S : grid;
    const int rb = SPLIT ? block_id % blocks : block_id;
    const int ks = SPLIT ? block_id / blocks : 0;
    const int r0 = rb * per_wg;
    if (r0 >= a.N) return;
    const int r1 = r0 + per_wg < a.N ? r0 + per_wg : a.N;
    const int nT = (r1 - r0 + OUT_PER_TILE - 1) / OUT_PER_TILE;
    const int P = (nT + T - 1) / T;                    // passes over K

    // this wave's k range: whole groups of 128 k, so that every range starts on a 256-byte boundary of
    // its rows (K >= 1024: every wave has at least one group)
    const int S4 = (K + 127) >> 7;
    const int k_begin = SPLIT ? ((ks * 8 + wv) * S4 / (8 * S)) * 128 : ((wv * S4) >> 3) * 128;
    const int k_stop = SPLIT ? ((ks * 8 + wv + 1) * S4 / (8 * S)) * 128 : (((wv + 1) * S4) >> 3) * 128;
    const int k_end = k_stop < K ? k_stop : K;
    const int nU = (k_end - k_begin + SK_KC - 1) / SK_KC;            // units of 256 k per pass
    const int total = P * nU * T;                                    // tile-steps of this wave

    const int g_pieces = (((S4 >> 3) + 1) * 128) >> 3;               // 16-byte pieces reserved per wave
    // weight-load role: load jj of a phase covers MFMA rows 4*jj + lane/16, piece lane%16
    const int ld_i = lane >> 4, ld_p = lane & 15;
    // operand role: token column c, k group kg
    const int c = lane & 15, kg = lane >> 4;
    const uintx4 zero4 = {0u, 0u, 0u, 0u};

    // Every load is unconditional.  A row past the block's end is read from the block's last row (the
    // same lines a neighbouring lane asks for); a piece past the wave's k range from the first piece of
    // the unit; a whole tile past the block (or past the wave's last tile-step: valid = false) from the
    // start of the activations -- lines that every compute unit has just read, so that the wait for these
    // loads at the end of the kernel is short.  What such loads return is zeroed or never stored.
    auto issue_w = [&](int tile, int uu, bool valid, uintx4 (&w)[8]) __attribute__((always_inline)) {
        const int k0 = k_begin + uu * SK_KC;
        const bool whole = valid && tile < nT;
        const int k_lim = whole ? k_end : 0;
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
            const int v = 4 * jj + ld_i;                   // virtual row within the tile
            const uint16_t* base;
            if (is_swiglu(EPI)) {
                int j = r0 + tile * 8 + (v & 7);
                j = j < r1 ? j : r1 - 1;
                base = ((v >> 3) ? a.w1 : a.w0) + (size_t)j * K;
            } else {
                int n = r0 + tile * 16 + v;
                n = n < r1 ? n : r1 - 1;
                base = a.w0 + (size_t)n * K;
            }
#pragma unroll
            for (int ph = 0; ph < 2; ++ph) {
                const int k = k0 + ph * 128 + ld_p * 8;
                w[ph * 4 + jj] = ld_stream(whole ? base + (k < k_lim ? k : k0) : a.x);
            }
        }
    };

    floatx4 acc[T][MT];
    floatx4 ssq[MT];                         // RMSNorm: x x^T of this wave's k range, one 16x16 tile per token tile
#pragma unroll
    for (int t = 0; t < T; ++t)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) acc[t][mt] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) ssq[mt] = floatx4{0.f, 0.f, 0.f, 0.f};

    float ssq_first = 0.f;                   // RMSNorm: this thread's token's sum of squares (first pass)
    int pass = 0, uu = 0;                    // the unit being consumed
    int p_pass = 0, p_uu = 0;                // the unit of the tile-step last requested
    int requested = 1;
    uintx4 wb0[8], wb1[8];
    // RMSNorm: this wave's slice of gamma goes to LDS once (wave-private: no workgroup barrier).  Its first
    // 64 pieces are requested before the first weights and stored behind them, so that the weights are in
    // flight while gamma arrives (all of gamma for K <= 4096).
    uintx4 g_first = zero4;
    if (is_rms(EPI)) g_first = ld_cached(a.gamma + k_begin + (lane * 8 < k_end - k_begin ? lane * 8 : 0));
    issue_w(0, 0, true, wb0);
    if (is_rms(EPI)) {
        if (lane * 8 < k_end - k_begin) s_gamma[wv * g_pieces + lane] = g_first;
        for (int p = lane + 64; p * 8 < k_end - k_begin; p += 64)
            s_gamma[wv * g_pieces + p] = ld_cached(a.gamma + k_begin + p * 8);
        __builtin_amdgcn_wave_barrier();
    }

    pre();                                   // (the single-launch MLP: wait for the activations to be complete)

    uintx4 xr[8][MT];                        // the unit's activations, operand layout (x * gamma for RMSNorm)

    // One tile-step = request the next tile-step's weights (the next tile of this unit, or tile 0 of the
    // next unit), then multiply tile TI of the current pass by the unit's activations.
    auto request_next = [&](auto ti, uintx4 (&pre)[8]) __attribute__((always_inline)) {
        constexpr int TI = decltype(ti)::value;
        if constexpr (TI + 1 == T) {
            if (++p_uu == nU) { p_uu = 0; ++p_pass; }
            issue_w(p_pass * T, p_uu, requested < total, pre);
        } else {
            issue_w(p_pass * T + TI + 1, p_uu, requested < total, pre);
        }
        ++requested;
    };
    auto multiply = [&](auto ti, uintx4 (&cur)[8]) __attribute__((always_inline)) {
        constexpr int TI = decltype(ti)::value;
        const int k0 = k_begin + uu * SK_KC;
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
            // the second half of a unit that ends after 128 k holds nothing: skipped (wave-uniform)
            if (ph == 1 && k0 + 128 >= k_end) break;
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) wt[wv][(4 * jj + ld_i) * WT_STRIDE + ld_p] = cur[ph * 4 + jj];
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int s4 = 0; s4 < 4; ++s4) {
                const int s = ph * 4 + s4;
                const half8 wa = __builtin_bit_cast(half8, wt[wv][c * WT_STRIDE + 4 * s4 + kg]);
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) {
                    if constexpr (TI == 0) {
                        // first use of the unit's activations: mask them, and for RMSNorm multiply by gamma
                        // (the sum of squares of the first pass is the one used: every pass sees the same x);
                        // the later tiles of the unit reuse the result
                        const bool kok = k0 + s * 32 + kg * 8 < k_end;
                        uintx4 xv = (kok && mt * 16 + c < a.M) ? xr[s][mt] : zero4;
                        if (is_rms(EPI)) {
                            const half8 xh = __builtin_bit_cast(half8, xv);
                            const half8 gh = __builtin_bit_cast(half8, s_gamma[wv * g_pieces + (((kok ? k0 + s * 32 : k_begin) - k_begin) >> 3) + (kok ? kg : 0)]);
                            // sum of squares on the matrix pipe: x as both operands, the diagonal of x x^T
                            // (accumulated in every pass, branch-free; only the first pass's sum is used)
                            ssq[mt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(xh, xh, ssq[mt], 0, 0, 0);
                            const half8 p = xh * gh;       // one rounding: the fp16 product of two fp16 values
                            xv = kok ? __builtin_bit_cast(uintx4, p) : zero4;
                        }
                        xr[s][mt] = xv;
                    }
                    acc[TI][mt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(wa, __builtin_bit_cast(half8, xr[s][mt]),
                                                                         acc[TI][mt], 0, 0, 0);
                }
            }
        }
    };
    auto tile_step = [&](auto ti, uintx4 (&cur)[8], uintx4 (&pre)[8]) __attribute__((always_inline)) {
        request_next(ti, pre);
        multiply(ti, cur);
    };

    // SPLIT: the block's sums over this workgroup's share of K go to its hand-over slot, [tile][token][row]
    unsigned* const slot = a.handover + (size_t)block_id * SK_SLOT_WORDS;

    // One unit of 256 k for all T tiles of the pass.  Tile-steps alternate between the two register
    // buffers; PAR says which of them holds tile 0 of this unit (with an odd T it flips from unit to unit).
    auto run_unit = [&](auto par) __attribute__((always_inline)) {
        constexpr int PAR = decltype(par)::value;
        const int k0 = k_begin + uu * SK_KC;
        const bool first_pass = (pass == 0);

        // Activations of this unit, then the next tile-step's weights: waiting for the activations leaves
        // those weights in flight.  They are loaded the way the weights are -- 16 lanes cover 256
        // contiguous bytes of a token row -- and reach operand layout through the wave's LDS buffer:
        // loading them in operand layout (every lane its own 16 bytes of a different row) costs the
        // vector cache several times the cycles per byte.
        uintx4 xl[MT][8];
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
        request_next(std::integral_constant<int, 0>{}, PAR ? wb0 : wb1);
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
        multiply(std::integral_constant<int, 0>{}, PAR ? wb1 : wb0);
        tile_step(std::integral_constant<int, 1>{}, PAR ? wb0 : wb1, PAR ? wb1 : wb0);
        if constexpr (T > 2) tile_step(std::integral_constant<int, 2>{}, PAR ? wb1 : wb0, PAR ? wb0 : wb1);
        if constexpr (T > 3) tile_step(std::integral_constant<int, 3>{}, PAR ? wb0 : wb1, PAR ? wb1 : wb0);
        if constexpr (T > 4) tile_step(std::integral_constant<int, 4>{}, PAR ? wb1 : wb0, PAR ? wb0 : wb1);
        if constexpr (T > 5) tile_step(std::integral_constant<int, 5>{}, PAR ? wb0 : wb1, PAR ? wb1 : wb0);

        const bool pass_ends = (uu + 1 == nU);
        const int this_pass = pass;
        if (++uu == nU) { uu = 0; ++pass; }
        if (!pass_ends) return;

        // ---- the eight partial tiles of each of the pass's tiles meet in LDS, RT tiles per round -------
        if constexpr (SPLIT) {
            // One round, one barrier: every thread adds the eight partial values of (tile, lane, token tile)
            // in wave order and stores its four rows of one token -- 16 contiguous bytes of the slot -- with
            // a device-scope store.
#pragma unroll
            for (int tt = 0; tt < T; ++tt)
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) s_part[wv][tt][mt * 64 + lane] = acc[tt][mt];
            __syncthreads();
            for (int e = tid; e < T * MT * 64; e += SK_THREADS) {
                const int tt = e / (MT * 64), q = e % (MT * 64);
                floatx4 v = {0.f, 0.f, 0.f, 0.f};       // fixed order: waves 0..7
#pragma unroll
                for (int w = 0; w < SK_WAVES; ++w) v += s_part[w][tt][q];
                const int l = q & 63, m = (q >> 6) * 16 + (l & 15);
                if (tt < nT && m < a.M) {
                    unsigned* const dst = slot + (tt * 32 + m) * 16 + 4 * (l >> 4);
                    asm volatile("global_store_dwordx4 %0, %1, off sc1" ::"v"(dst), "v"(v) : "memory");
                }
            }
            return;
        }
        // Every thread adds the eight partial values of (tile, token tile, lane) in wave order and finishes what it
        // then holds -- four consecutive output features of one token (two gate/up pairs after an exchange between
        // the wave's halves for SwiGLU) -- straight from registers: one barrier per round.
        constexpr int ROUNDS = (T + RT - 1) / RT;
#pragma unroll
        for (int rr = 0; rr < ROUNDS; ++rr) {
#pragma unroll
            for (int tt = 0; tt < RT; ++tt)
                if (rr * RT + tt < T) {
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt) {
                        s_part[wv][tt][mt * 64 + lane] = acc[rr * RT + tt < T ? rr * RT + tt : 0][mt];
                        acc[rr * RT + tt < T ? rr * RT + tt : 0][mt] = floatx4{0.f, 0.f, 0.f, 0.f};
                    }
                }
            if (is_rms(EPI) && first_pass && rr == 0) {
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) {
                    // token c's sum of squares is element (c, c): row c = 4 * (lane / 16) + register index
                    const int i = c & 3;
                    const float v = i == 0 ? ssq[mt][0] : i == 1 ? ssq[mt][1] : i == 2 ? ssq[mt][2] : ssq[mt][3];
                    if (kg == (c >> 2)) s_red[wv][mt * 16 + c] = v;
                }
                if (MT == 1 && kg == 0) s_red[wv][16 + c] = 0.f;
            }
            __syncthreads();
            // this thread's token in every iteration below (512 is a multiple of MT * 64) and its RMSNorm factor:
            // the sum of squares of the first pass, added in wave order, kept in s_ssq for the later passes
            const int q = tid % (MT * 64), l = q & 63, m = (q >> 6) * 16 + (l & 15), quad = l >> 4;
            float scale = 1.0f;
            if (is_rms(EPI)) {
                float v = 0.f;
                if (first_pass) {
                    if (rr == 0) {
#pragma unroll
                        for (int w = 0; w < SK_WAVES; ++w) v += s_red[w][m];
                        if (tid < MT * 64 && quad == 0) s_ssq[m] = v;
                        ssq_first = v;
                    } else {
                        v = ssq_first;
                    }
                } else {
                    v = s_ssq[m];
                }
                scale = 1.0f / __builtin_sqrtf(v / (float)K + a.eps);
            }
            const int round_tiles = (rr + 1) * RT <= T ? RT : T - rr * RT;
            for (int e = tid; e < round_tiles * MT * 64; e += SK_THREADS) {
                const int tt = e / (MT * 64);
                floatx4 v = {0.f, 0.f, 0.f, 0.f};       // fixed order: waves 0..7
#pragma unroll
                for (int w = 0; w < SK_WAVES; ++w) v += s_part[w][tt][q];
                const int tile = this_pass * T + rr * RT + tt;
                if (is_swiglu(EPI)) {
                    // rows 0..7 of a tile are gate rows, 8..15 the matching up rows: lane l holds rows 4*quad..+3,
                    // its partner l ^ 32 the rows 8 further on
                    floatx4 o;
#pragma unroll
                    for (int i = 0; i < 4; ++i) o[i] = __shfl_xor(v[i], 32);
                    if (quad < 2 && tile < nT && m < a.M) {
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            const int j = r0 + tile * 8 + 4 * quad + i;
                            if (j < r1) put(a.out + (size_t)m * a.ldo + j, to_half_bits(silu_mul(v[i] * scale, o[i] * scale)));
                        }
                    }
                } else if (tile < nT && m < a.M) {
                    const int n = r0 + tile * 16 + 4 * quad;
                    float y[4];
#pragma unroll
                    for (int i = 0; i < 4; i += 2) {      // pairs (n + i, n + i + 1); blocks start on even rows
                        y[i] = v[i] * scale;
                        y[i + 1] = v[i + 1] * scale;
                        if (EPI == EPI_RMSNORM_ROPE) rope_pair(a.rope, a.rope.pos[m], n + i, y[i], y[i + 1]);
                    }
                    uint16_t* const dst = a.out + (size_t)m * a.ldo + n;
                    if (!DEVOUT && n + 3 < r1 && ((n | a.ldo) & 3) == 0) {
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
                            if (n + i < r1) {
                                float o = y[i];
                                if (a.residual) o += half_bits_to_float(a.residual[(size_t)m * a.ldo + n + i]);
                                put(dst + i, to_half_bits(o));
                            }
                    }
                }
            }
            // s_part (and s_red / s_ssq) are written again in the next round or pass: everybody must be done reading
            if (rr + 1 < ROUNDS || P > 1) __syncthreads();
        }
    };

    const int units = P * nU;
    if constexpr (T % 2 == 0) {
        for (int it = 0; it < units; ++it) run_unit(std::integral_constant<int, 0>{});
    } else {
        for (int it = 0; it < units; it += 2) {
            run_unit(std::integral_constant<int, 0>{});
            if (it + 1 >= units) break;
            run_unit(std::integral_constant<int, 1>{});
        }
    }

    if constexpr (SPLIT) {
        // The block's S workgroups have each handed in their sums (one pass: the host only splits K when
        // the block's tiles are all in flight).  Whoever arrives last adds the S contributions in share
        // order -- the same result whichever workgroup that is -- and writes the outputs.  Nobody waits:
        // the stores are device-scope and acknowledged before the arrival is counted.
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        if (tid == 0) {
            const unsigned before = __hip_atomic_fetch_add(a.counters + rb, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            const unsigned last = before + 1u == (unsigned)S;
            if (last) __hip_atomic_store(a.counters + rb, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // zero between calls
            s_last = last;
        }
        __syncthreads();
        if (s_last == 0u) return;
        const int r = tid & 15, m = tid >> 4;
        if (m >= a.M) return;
        const unsigned* const first = a.handover + (size_t)rb * SK_SLOT_WORDS + m * 16 + r;      // share 0's slot
        const size_t share_stride = (size_t)blocks * SK_SLOT_WORDS;
        float v[T];
#pragma unroll
        for (int t = 0; t < T; ++t) v[t] = 0.f;
        for (int s0 = 0; s0 < S; s0 += 4) {
            // the loads of four shares x T tiles are in flight together; a share or tile that does not
            // exist is read from one that does and not added
            unsigned pv[4][T];
#pragma unroll
            for (int b = 0; b < 4; ++b)
#pragma unroll
                for (int t = 0; t < T; ++t)
                    pv[b][t] = __hip_atomic_load(first + (size_t)(s0 + b < S ? s0 + b : S - 1) * share_stride + (t < nT ? t : 0) * 512,
                                                 __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
            for (int b = 0; b < 4; ++b)
#pragma unroll
                for (int t = 0; t < T; ++t)
                    if (s0 + b < S) v[t] += __builtin_bit_cast(float, pv[b][t]);
        }
#pragma unroll
        for (int t = 0; t < T; ++t) {
            const int n = r0 + t * 16 + r;
            if (t < nT && n < r1) {
                float o = v[t];
                if (a.residual) o += half_bits_to_float(a.residual[(size_t)m * a.ldo + n]);
                put(a.out + (size_t)m * a.ldo + n, to_half_bits(o));
            }
        }
    }
}

template <int T, int MT, int EPI, bool SPLIT = false>
__global__ __launch_bounds__(SK_THREADS) void skinny_rowblock(const uint16_t* x_, const uint16_t* w0_, const uint16_t* w1_,
                                                              const uint16_t* gamma_, int M_, int N_, int K_, int per_wg,
                                                              SkinnyArgs a)
{
    // The operands the first loads need come as leading scalar arguments: the hardware preloads those
    // into registers at wave launch, so the first weight request does not wait for an argument fetch.
    a.x = x_; a.w0 = w0_; a.w1 = w1_; a.gamma = gamma_; a.M = M_; a.N = N_; a.K = K_;
    __shared__ RowBlockShared<T, MT, EPI, SPLIT> sm;
    extern __shared__ uintx4 s_gamma[];                // RMSNorm: each wave's slice of gamma
    rowblock_body<T, MT, EPI, SPLIT, false>(a, per_wg, (int)blockIdx.x, (int)gridDim.x, sm, s_gamma, [] {});
}

// The SwiGLU MLP of a decode step as ONE launch (the paper's unified kernel scheduling, Sec. III-C.4: one launch per
// operator graph instead of one per operator): every workgroup first runs its row block of the gate/up projection
// (storing its part of h = silu(g)*u with device-scope stores), announces its arrival, requests the first weights of
// its row block of the down projection, and only then waits until the whole grid has arrived -- the wait for h
// overlaps the latency of those first weights, and neither the tail of the first phase nor a kernel boundary leaves
// the memory system idle.  All workgroups are resident at once (one per compute unit) and the wait is bounded
// (time-out marker as for the other hand-overs).  Both phases are the row-block kernel above; their static LDS
// objects are overlaid.
// The rendezvous avoids read-modify-write traffic on one word (256 device-scope atomic adds on one address take
// ~18 us): every workgroup stores a tag into its own status word and wave 0 of every waiting workgroup reads all of
// them (four words per lane) until they all carry the tag.  The tag is the launch's number on this workspace plus
// one, read from a status word at kernel entry and advanced by workgroup 0 once everybody has arrived -- nothing has
// to be reset, the launch can be replayed from a captured graph, and a freshly initialised workspace (all zero)
// never matches.  These words are the only status words that are not zero between calls.
// Reading h afterwards needs an agent-scope acquire: h was written through eight L2s, and a line of it may sit in
// this XCD's L2 with only this XCD's bytes current.  Executed by every workgroup the acquire (an L2 invalidate each)
// costs 13 us; the L2 is shared by the XCD, so ONE workgroup per XCD does it -- the one with the lowest number among
// those that report the same XCC id with their tag -- and announces it in a status word per XCD; the others wait for
// that word (bounded like every wait here) and only drop their own vector cache's lines.
template <int T1, int T2, int MT, int EPI1>
__global__ __launch_bounds__(SK_THREADS) void mlp_fused(const uint16_t* x_, const uint16_t* wg_, const uint16_t* wu_,
                                                        const uint16_t* gamma_, int M_, int I_, int H_, int per_wg1,
                                                        int per_wg2, int grid1, int grid2, SkinnyArgs a1, SkinnyArgs a2)
{
    a1.x = x_; a1.w0 = wg_; a1.w1 = wu_; a1.gamma = gamma_; a1.M = M_; a1.N = I_; a1.K = H_;
    a2.M = M_; a2.N = H_; a2.K = I_;
    union Shared {
        RowBlockShared<T1, MT, EPI1, false> up;
        RowBlockShared<T2, MT, EPI_PLAIN, true> down;
    };
    __shared__ Shared sm;
    extern __shared__ uintx4 s_gamma[];
    const int bid = (int)blockIdx.x;
    const int everybody = (int)gridDim.x;
    unsigned* const epoch = a2.counters + MLP_EPOCH_WORD;
    unsigned* const flags = a2.counters + MLP_FLAG_WORDS;
    // (every lane reads the same word: the value is wave-uniform)
    const unsigned launch_no = __hip_atomic_load(epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const unsigned tag = launch_no % 0x0ffffffeu + 1u;        // 28 bits, never the zero of a fresh workspace
    // the XCC this workgroup runs on (hardware register XCC_ID, bits 3:0), announced in the tag word's top four bits
    const unsigned xcc = (unsigned)__builtin_amdgcn_s_getreg(20 | (0 << 6) | (3 << 11)) & 15u;
    unsigned* const l2_done = flags + MLP_MAX_GRID;           // [16] per XCC: the tag of the last launch whose acquire is done

    if (bid < grid1) rowblock_body<T1, MT, EPI1, false, true>(a1, per_wg1, bid, grid1, sm.up, s_gamma, [] {});
    // this workgroup's part of h is acknowledged by the memory system before its arrival is announced
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (threadIdx.x == 0) __hip_atomic_store(flags + bid, tag | (xcc << 28), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (bid >= grid2) return;

    rowblock_body<T2, MT, EPI_PLAIN, true, false>(a2, per_wg2, bid, grid2, sm.down, s_gamma, [&] {
        if (threadIdx.x < 64) {
            const int lane = (int)threadIdx.x;
            unsigned spins = 0;
            bool ok = true;
            int first_here = 0x7fffffff;          // the lowest-numbered workgroup of the second phase on this XCC
            while (true) {
                bool all = true;
                first_here = 0x7fffffff;
#pragma unroll
                for (int q = 0; q < MLP_MAX_GRID / 64; ++q) {
                    const int w = q * 64 + lane;
                    const unsigned f = __hip_atomic_load(flags + (w < everybody ? w : 0), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    all = all && (w >= everybody || (f & 0x0fffffffu) == tag);
                    if (w < grid2 && (f >> 28) == xcc && w < first_here) first_here = w;
                }
                if (__builtin_amdgcn_ballot_w64(!all) == 0ull) break;
                __builtin_amdgcn_s_sleep(1);
                if (++spins > a2.spin_limit) { ok = false; break; }      // bounded: every wave exits
            }
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) {
                const int other = __shfl_xor(first_here, o);
                first_here = other < first_here ? other : first_here;
            }
            if (ok) {
                if (first_here == bid) {
                    // h was written through other L2s: this XCD's L2 (and this CU's vector cache) must forget it
                    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
                    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
                    if (lane == 0) __hip_atomic_store(l2_done + xcc, tag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                } else {
                    while (__hip_atomic_load(l2_done + xcc, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != tag) {
                        __builtin_amdgcn_s_sleep(1);
                        if (++spins > a2.spin_limit) { ok = false; break; }
                    }
                }
            }
            if (lane == 0) {
                if (!ok) __hip_atomic_store(a2.counters + (WS_MAX_COUNTERS - 1), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                // everybody has read the launch number (at entry, before arriving): it may advance
                if (bid == 0) __hip_atomic_store(epoch, launch_no + 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
        __syncthreads();
        // nothing of h may be served from this compute unit's vector cache either
        asm volatile("buffer_inv sc0" ::: "memory");
    });
}

// 16-byte pieces of LDS per wave for its slice of gamma (same arithmetic as in the kernel)
int gamma_pieces(int K) { return ((((K + 127) >> 7) >> 3) + 1) * 128 >> 3; }

// Opt a kernel in to more than 64 KiB of LDS: as much dynamic LDS as `want`, or as its static LDS leaves of a
// compute unit's 160 KiB.  Returns the dynamic bytes now allowed.
constexpr int CU_LDS_BYTES = 160 * 1024;
int allow_lds(const void* kernel, int want)
{
    hipFuncAttributes fa;
    if (hipFuncGetAttributes(&fa, kernel) != hipSuccess) return 0;
    int room = CU_LDS_BYTES - (int)fa.sharedSizeBytes;
    if (room < 0) room = 0;
    const int most = want < room ? want : room;
    if (hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, most) != hipSuccess) return 0;
    return most;
}

template <int T, int MT>
hipError_t launch_t_mt(const SkinnyArgs& a, int epilogue, const RowBlockPlan& p, hipStream_t stream)
{
    dim3 g(p.grid), b(SK_THREADS);
    const int per_wg = p.per_wg;
    const size_t gamma_lds = (size_t)SK_WAVES * gamma_pieces(a.K) * sizeof(uintx4);
    static std::once_flag attr_once;    // static (+ dynamic) LDS passes 64 KiB: every variant needs the opt-in
    std::call_once(attr_once, [] {
        // the kinds with gamma in LDS: static part <= 85 KiB, so the largest gamma slice stays inside the 160 KiB of a CU
        const int most = (int)((size_t)SK_WAVES * gamma_pieces(ROWSLAB_MAX_K) * sizeof(uintx4));
        (void)allow_lds(reinterpret_cast<const void*>(skinny_rowblock<T, MT, EPI_PLAIN>), 0);
        (void)allow_lds(reinterpret_cast<const void*>(skinny_rowblock<T, MT, EPI_PLAIN, true>), 0);
        (void)allow_lds(reinterpret_cast<const void*>(skinny_rowblock<T, MT, EPI_SWIGLU>), 0);
        (void)allow_lds(reinterpret_cast<const void*>(skinny_rowblock<T, MT, EPI_RMSNORM>), most);
        (void)allow_lds(reinterpret_cast<const void*>(skinny_rowblock<T, MT, EPI_RMSNORM_ROPE>), most);
        (void)allow_lds(reinterpret_cast<const void*>(skinny_rowblock<T, MT, EPI_RMSNORM_SWIGLU>), most);
    });
    if (p.ksplit > 1) {      // plain kind only (checked by the caller); the share count travels in kchunks
        SkinnyArgs s = a;
        s.kchunks = p.ksplit;
        hipLaunchKernelGGL((skinny_rowblock<T, MT, EPI_PLAIN, true>), g, b, 0, stream, s.x, s.w0, s.w1, s.gamma, s.M, s.N, s.K, per_wg, s);
        return hipGetLastError();
    }
    switch (epilogue) {
    case EPI_PLAIN: hipLaunchKernelGGL((skinny_rowblock<T, MT, EPI_PLAIN>), g, b, 0, stream, a.x, a.w0, a.w1, a.gamma, a.M, a.N, a.K, per_wg, a); break;
    case EPI_RMSNORM: hipLaunchKernelGGL((skinny_rowblock<T, MT, EPI_RMSNORM>), g, b, gamma_lds, stream, a.x, a.w0, a.w1, a.gamma, a.M, a.N, a.K, per_wg, a); break;
    case EPI_RMSNORM_ROPE: hipLaunchKernelGGL((skinny_rowblock<T, MT, EPI_RMSNORM_ROPE>), g, b, gamma_lds, stream, a.x, a.w0, a.w1, a.gamma, a.M, a.N, a.K, per_wg, a); break;
    case EPI_RMSNORM_SWIGLU: hipLaunchKernelGGL((skinny_rowblock<T, MT, EPI_RMSNORM_SWIGLU>), g, b, gamma_lds, stream, a.x, a.w0, a.w1, a.gamma, a.M, a.N, a.K, per_wg, a); break;
    default: hipLaunchKernelGGL((skinny_rowblock<T, MT, EPI_SWIGLU>), g, b, 0, stream, a.x, a.w0, a.w1, a.gamma, a.M, a.N, a.K, per_wg, a); break;
    }
    return hipGetLastError();
}

template <int T>
hipError_t launch_t(const SkinnyArgs& a, int epilogue, const RowBlockPlan& p, hipStream_t stream)
{
    if (a.M <= 16) return launch_t_mt<T, 1>(a, epilogue, p, stream);
    return launch_t_mt<T, 2>(a, epilogue, p, stream);
}

}  // namespace

hipError_t launch_mlp_fused(const SkinnyArgs& up, const SkinnyArgs& down, int epilogue_up, int num_cus, hipStream_t stream,
                            int ksplit_down)
{
    if (!mlp_fused_ok(up.M, up.K, up.N, epilogue_up, num_cus, ksplit_down)) return hipErrorInvalidValue;
    const RowBlockPlan p1 = plan_rowblock(up.N, epilogue_up, num_cus, 1), p2 = plan_rowblock(down.N, EPI_PLAIN, num_cus, ksplit_down);
    SkinnyArgs a2 = down;
    a2.kchunks = ksplit_down;
    const int grid = p1.grid > p2.grid ? p1.grid : p2.grid;
    const size_t gamma_lds = epilogue_up == EPI_RMSNORM_SWIGLU ? (size_t)SK_WAVES * gamma_pieces(up.K) * sizeof(uintx4) : 0;
    static std::once_flag attr_once;
    static int room_rms = 0;            // dynamic LDS the RMSNorm variant may use beside its static part
    std::call_once(attr_once, [] {
        const int most = (int)((size_t)SK_WAVES * gamma_pieces(ROWSLAB_MAX_K) * sizeof(uintx4));
        (void)allow_lds(reinterpret_cast<const void*>(mlp_fused<6, 4, 2, EPI_SWIGLU>), 0);
        room_rms = allow_lds(reinterpret_cast<const void*>(mlp_fused<6, 4, 2, EPI_RMSNORM_SWIGLU>), most);
    });
    if ((int)gamma_lds > room_rms) return hipErrorInvalidValue;      // gamma for this H does not fit beside the two phases' LDS
    if (epilogue_up == EPI_SWIGLU)
        hipLaunchKernelGGL((mlp_fused<6, 4, 2, EPI_SWIGLU>), dim3(grid), dim3(SK_THREADS), gamma_lds, stream, up.x, up.w0, up.w1, up.gamma,
                           up.M, up.N, up.K, p1.per_wg, p2.per_wg, p1.grid, p2.grid, up, a2);
    else
        hipLaunchKernelGGL((mlp_fused<6, 4, 2, EPI_RMSNORM_SWIGLU>), dim3(grid), dim3(SK_THREADS), gamma_lds, stream, up.x, up.w0, up.w1,
                           up.gamma, up.M, up.N, up.K, p1.per_wg, p2.per_wg, p1.grid, p2.grid, up, a2);
    return hipGetLastError();
}

hipError_t launch_rowblock(const SkinnyArgs& a, int epilogue, int num_cus, hipStream_t stream, int ksplit)
{
    if (a.K < 1024 || a.K > ROWSLAB_MAX_K || a.N < 1) return hipErrorInvalidValue;
    if (ksplit > 1 && !rowblock_split_ok(a.N, a.K, epilogue, num_cus, ksplit)) return hipErrorInvalidValue;
    const RowBlockPlan p = plan_rowblock(a.N, epilogue, num_cus, ksplit);
    switch (p.T) {
    case 2: return launch_t<2>(a, epilogue, p, stream);
    case 3: return launch_t<3>(a, epilogue, p, stream);
    case 4: return launch_t<4>(a, epilogue, p, stream);
    case 5: return launch_t<5>(a, epilogue, p, stream);
    default: return launch_t<6>(a, epilogue, p, stream);
    }
}

}  // namespace thi
